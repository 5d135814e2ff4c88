// Running softmax statistics shared by the bf16 forward sweeps.
#pragma once
#include <hip/hip_runtime.h>

namespace pard2 {

static constexpr float L2E = 1.4426950408889634f;

// Statistics over a set of logits: max, sum of exp(z - max), lowest index attaining the max.
struct RowStat {
  float m, s;
  int idx;
};
__device__ __forceinline__ RowStat merge(RowStat a, RowStat b) {
  RowStat o;
  o.m = fmaxf(a.m, b.m);
  const float ms = (o.m == -INFINITY) ? 0.f : o.m;  // both empty: keep s = 0 instead of NaN
  o.s = a.s * __builtin_amdgcn_exp2f((a.m - ms) * L2E) + b.s * __builtin_amdgcn_exp2f((b.m - ms) * L2E);
  o.idx = (a.m > b.m) ? a.idx : (b.m > a.m) ? b.idx : min(a.idx, b.idx);
  return o;
}

}  // namespace pard2
