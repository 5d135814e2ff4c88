// Bandwidth/latency-bound steps of the CAT loss: merging the per-range softmax
// statistics, the per-block prefix product of confidences (Eq.10), the weighted
// reduction of Eq.11 and the per-row gradient scale of the backward.
#include "kernels.h"

#include <limits.h>

namespace pard2 {

// ---------------------------------------------------------------- combine partial statistics
// One thread per token row: (max, sumexp, argmax) over all vocabulary ranges ->
// lse, log q_t(y_t) (log P of Eq.5/Eq.11), greedy prediction, confidence (Eq.9: given,
// or q_t(y_t) in the self-teacher instance).
__global__ __launch_bounds__(256) void combine_kernel(const float2* __restrict__ ms, const int32_t* __restrict__ idx,
                                                      const float* __restrict__ zy, int P,
                                                      const int32_t* __restrict__ y, const float* __restrict__ conf_in,
                                                      int T, int V, int ignore_index, float* __restrict__ lse,
                                                      float* __restrict__ logp_y, int32_t* __restrict__ argmax,
                                                      float* __restrict__ conf, int32_t* __restrict__ hit,
                                                      int32_t* __restrict__ dev_status) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= T) return;
  const float2* p = ms + (int64_t)t * P;
  const int32_t* pi = idx + (int64_t)t * P;
  float m = -INFINITY;
  int am = INT_MAX;
  for (int j = 0; j < P; ++j) {
    const float mj = p[j].x;
    if (mj > m) {  // ranges ascend in vocabulary id: the first range attaining the max has the lowest index
      m = mj;
      am = pi[j];
    }
  }
  float s = 0.f;
  for (int j = 0; j < P; ++j) s += p[j].y * expf(p[j].x - m);
  const float l = m + logf(s);
  const int yv = y[t];
  const bool ok = yv >= 0 && yv < V;
  if (!ok && yv != ignore_index && dev_status) *dev_status = 1;
  const float lp = ok ? zy[t] - l : 0.f;
  lse[t] = l;
  logp_y[t] = lp;
  if (argmax) argmax[t] = am;
  if (conf) conf[t] = conf_in ? conf_in[t] : (ok ? expf(lp) : 1.f);
  if (hit) hit[t] = ok && am == yv;
}

hipError_t launch_combine(StatsOut st, const int32_t* y, const float* conf_in, int T, int V, int ignore_index,
                          float* lse, float* logp_y, int32_t* argmax, float* conf, int32_t* hit,
                          int32_t* dev_status, hipStream_t s) {
  hipLaunchKernelGGL(combine_kernel, dim3((T + 255) / 256), dim3(256), 0, s, st.ms, st.idx, st.zy, st.P, y, conf_in,
                     T, V, ignore_index, lse, logp_y, argmax, conf, hit, dev_status);
  return hipGetLastError();
}

// ---------------------------------------------------------------- combine, two heads (Eq.12 with KD)
// One thread per token row.  Draft side as above.  Teacher side: lse_t, the teacher's p_t(y_t)
// (the confidence of Eq.9 unless one is given) and
//   KL(p_t || q_t) = sum_v p_t(v) (zT - zD)(v) - lse_t + lse = a / s - lse_t + lse.
// tok[t] = beta log q_t(y_t) - KL: minus the row's term beta CE + KD, in the place where the
// CE-only path hands log q_t(y_t) to the weighted reduction.
__global__ __launch_bounds__(256) void kd_combine_kernel(
    const float2* __restrict__ ms, const int32_t* __restrict__ idx, const float* __restrict__ zy,
    const float2* __restrict__ ms_t, const float* __restrict__ a_t, const float* __restrict__ zy_t, int P,
    const int32_t* __restrict__ y, const float* __restrict__ conf_in, int T, int V, int ignore_index, float beta,
    float* __restrict__ lse, float* __restrict__ lse_t, float* __restrict__ logp_y, float* __restrict__ kd,
    float* __restrict__ tok, int32_t* __restrict__ argmax, float* __restrict__ conf, int32_t* __restrict__ hit,
    int32_t* __restrict__ dev_status) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= T) return;
  const float2* p = ms + (int64_t)t * P;
  const int32_t* pi = idx + (int64_t)t * P;
  const float2* pt = ms_t + (int64_t)t * P;
  const float* pa = a_t + (int64_t)t * P;
  float m = -INFINITY, mt = -INFINITY;
  int am = INT_MAX;
  for (int j = 0; j < P; ++j) {
    const float mj = p[j].x;
    if (mj > m) {
      m = mj;
      am = pi[j];
    }
    mt = fmaxf(mt, pt[j].x);
  }
  float s = 0.f, st = 0.f, at = 0.f;
  for (int j = 0; j < P; ++j) {
    s += p[j].y * expf(p[j].x - m);
    const float e = expf(pt[j].x - mt);
    st += pt[j].y * e;
    at += pa[j] * e;
  }
  const float l = m + logf(s), lt = mt + logf(st);
  const float kl = at / st - lt + l;
  const int yv = y[t];
  const bool ok = yv >= 0 && yv < V;
  if (!ok && yv != ignore_index && dev_status) *dev_status = 1;
  const float lp = ok ? zy[t] - l : 0.f;
  lse[t] = l;
  lse_t[t] = lt;
  logp_y[t] = lp;
  if (kd) kd[t] = kl;
  tok[t] = ok ? beta * lp - kl : 0.f;
  if (argmax) argmax[t] = am;
  if (conf) conf[t] = conf_in ? conf_in[t] : (ok ? expf(zy_t[t] - lt) : 1.f);
  if (hit) hit[t] = ok && am == yv;
}

hipError_t launch_kd_combine(KdStatsOut st, const int32_t* y, const float* conf_in, int T, int V, int ignore_index,
                             float beta, float* lse, float* lse_t, float* logp_y, float* kd, float* tok,
                             int32_t* argmax, float* conf, int32_t* hit, int32_t* dev_status, hipStream_t s) {
  hipLaunchKernelGGL(kd_combine_kernel, dim3((T + 255) / 256), dim3(256), 0, s, st.draft.ms, st.draft.idx, st.draft.zy,
                     st.ms_t, st.a_t, st.zy_t, st.draft.P, y, conf_in, T, V, ignore_index, beta, lse, lse_t, logp_y,
                     kd, tok, argmax, conf, hit, dev_status);
  return hipGetLastError();
}

// ---------------------------------------------------------------- loss after the backward (two heads)
// The two-head dZ kernel leaves, per vocabulary tile, each row's sum_v p (zT - zD); summed over the
// tiles in a fixed order that is the cross term of KL(p || q) = sum - lse_t + lse.
__global__ __launch_bounds__(256) void kd_finish_kernel(const float* __restrict__ kd_part, int nparts,
                                                        const float* __restrict__ lse, const float* __restrict__ lse_t,
                                                        const float* __restrict__ logp_y, const int32_t* __restrict__ y,
                                                        float beta, int T, int V, float* __restrict__ kd,
                                                        float* __restrict__ tok) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= T) return;
  float a = 0.f;
  for (int j = 0; j < nparts; ++j) a += kd_part[(int64_t)j * T + t];
  const float kl = a - lse_t[t] + lse[t];
  if (kd) kd[t] = kl;
  const int yv = y[t];
  if (tok) tok[t] = (yv >= 0 && yv < V) ? beta * logp_y[t] - kl : 0.f;
}

hipError_t launch_kd_finish(const float* kd_part, int nparts, const float* lse, const float* lse_t,
                            const float* logp_y, const int32_t* y, float beta, int T, int V, float* kd, float* tok,
                            hipStream_t s) {
  hipLaunchKernelGGL(kd_finish_kernel, dim3((T + 255) / 256), dim3(256), 0, s, kd_part, nparts, lse, lse_t, logp_y, y,
                     beta, T, V, kd, tok);
  return hipGetLastError();
}

// loss = (1/N) sum_t w_t (-tok_t) over valid rows, one workgroup, fixed-order fp64 tree (reproducible).
__global__ __launch_bounds__(1024) void weighted_loss_kernel(const float* __restrict__ w, const float* __restrict__ tok,
                                                             const int32_t* __restrict__ y,
                                                             const int32_t* __restrict__ valid_len, int B, int K, int V,
                                                             int reduction, float* __restrict__ loss) {
  __shared__ double sh_sum[1024];
  __shared__ int sh_cnt[1024];
  const int64_t T = (int64_t)B * K;
  double sum = 0.0;
  int cnt = 0;
  for (int64_t t = threadIdx.x; t < T; t += blockDim.x) {
    const int b = (int)(t / K), k = (int)(t % K);
    const int Kb = valid_len ? valid_len[b] : K;
    const int yv = y[t];
    if (k < Kb && yv >= 0 && yv < V) {
      sum += (double)w[t] * (double)(-tok[t]);
      ++cnt;
    }
  }
  sh_sum[threadIdx.x] = sum;
  sh_cnt[threadIdx.x] = cnt;
  __syncthreads();
  for (int s = 512; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) {
      sh_sum[threadIdx.x] += sh_sum[threadIdx.x + s];
      sh_cnt[threadIdx.x] += sh_cnt[threadIdx.x + s];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const double l = reduction == 0 ? (sh_cnt[0] > 0 ? sh_sum[0] / sh_cnt[0] : 0.0) : sh_sum[0];
    *loss = (float)l;
  }
}

hipError_t launch_weighted_loss(const float* w, const float* tok, const int32_t* y, const int32_t* valid_len, int B,
                                int K, int V, int reduction, float* loss, hipStream_t s) {
  hipLaunchKernelGGL(weighted_loss_kernel, dim3(1), dim3(1024), 0, s, w, tok, y, valid_len, B, K, V, reduction, loss);
  return hipGetLastError();
}

// ---------------------------------------------------------------- per-block scan
// One thread per draft block walks its K slots left to right:
//   s_0 = 1, s_k = s_{k-1} * c_{k-1}   (Eq.10), or gamma^k / 1 for the comparators,
// masks invalid slots, and collects the block's diagnostics and its share of
// sum_t w_t * (-log q_t(y_t)).  Block shares are reduced in a fixed order (LDS tree per
// workgroup, then one workgroup over the group partials): the loss is reproducible.
constexpr int SCAN_THREADS = 256;
int scan_num_groups(int B) { return (B + SCAN_THREADS - 1) / SCAN_THREADS; }

__global__ __launch_bounds__(SCAN_THREADS) void scan_kernel(ScanArgs a) {
  __shared__ double sh_sum[SCAN_THREADS];
  __shared__ double sh_cnt[SCAN_THREADS];
  const int b = blockIdx.x * SCAN_THREADS + threadIdx.x;
  double lsum = 0.0, cnt = 0.0;
  if (b < a.B) {
    const int K = a.K;
    int Kb = a.valid_len ? a.valid_len[b] : K;
    Kb = max(0, min(Kb, K));
    int64_t pos = 0;
    if (a.conf_seq) {   // slots whose position lies past the sequence's end do not exist (Eq.12: n <= N - k)
      pos = a.anchor_pos[b];
      const int64_t end = min((int64_t)a.seq_end[b], a.n_pos);
      Kb = pos < 0 ? 0 : (int)max((int64_t)0, min((int64_t)Kb, end - pos));
      if (a.valid_len_out) a.valid_len_out[b] = Kb;
    }
    float run = 1.f, gpow = 1.f, el = 0.f;
    int al = 0;
    bool prefix = true;
    for (int k = 0; k < K; ++k) {
      const int64_t t = (int64_t)b * K + k;
      float c;
      if (a.conf_seq) {
        c = k < Kb ? a.conf_seq[pos + k] : 1.f;
        if (a.conf_out) a.conf_out[t] = c;
      } else {
        c = a.conf[t];
      }
      const float s = (a.weight_mode == 0) ? run : (a.weight_mode == 1) ? gpow : 1.f;
      bool has = true;
      if (a.y) {
        const int yv = a.y[t];
        has = yv >= 0 && yv < a.V;
      }
      const bool in = k < Kb;
      const bool valid = in && has;
      const float wv = valid ? s : 0.f;
      if (a.w) a.w[t] = wv;
      if (in) el += s * c;
      if (a.hit) {
        prefix = prefix && in && a.hit[t] != 0;
        al += prefix ? 1 : 0;
      }
      if (valid && a.logp_y) {
        lsum += (double)wv * (double)(-a.logp_y[t]);
        cnt += 1.0;
      }
      run *= c;
      gpow *= a.gamma;
    }
    if (a.exp_len) a.exp_len[b] = el;
    if (a.accept_len) a.accept_len[b] = al;
  }
  if (!a.loss) return;
  sh_sum[threadIdx.x] = lsum;
  sh_cnt[threadIdx.x] = cnt;
  __syncthreads();
  for (int s = SCAN_THREADS / 2; s > 0; s >>= 1) {
    if (threadIdx.x < s) {
      sh_sum[threadIdx.x] += sh_sum[threadIdx.x + s];
      sh_cnt[threadIdx.x] += sh_cnt[threadIdx.x + s];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    a.loss_partials[2 * blockIdx.x] = sh_sum[0];
    a.loss_partials[2 * blockIdx.x + 1] = sh_cnt[0];
  }
}

__global__ __launch_bounds__(64) void loss_finalize_kernel(const double* __restrict__ partials, int ngroups,
                                                           int reduction, float beta, float* __restrict__ loss) {
  if (threadIdx.x != 0) return;
  double sum = 0.0, cnt = 0.0;
  for (int i = 0; i < ngroups; ++i) {
    sum += partials[2 * i];
    cnt += partials[2 * i + 1];
  }
  double l;
  if (reduction == 0)
    l = cnt > 0.0 ? (double)beta * sum / cnt : 0.0;
  else
    l = (double)beta * sum;
  *loss = (float)l;
}

hipError_t launch_scan(const ScanArgs& a, hipStream_t s) {
  const int groups = scan_num_groups(a.B);
  hipLaunchKernelGGL(scan_kernel, dim3(groups), dim3(SCAN_THREADS), 0, s, a);
  if (a.loss)
    hipLaunchKernelGGL(loss_finalize_kernel, dim3(1), dim3(64), 0, s, a.loss_partials, groups, a.reduction, a.beta,
                       a.loss);
  return hipGetLastError();
}

// ---------------------------------------------------------------- backward row scale
// g_t = grad_loss * beta * w_t / N on valid rows (N = number of valid tokens for
// MEAN_VALID, 1 for SUM), 0 on invalid rows.  Single workgroup: T is at most a few 10^4.
__global__ __launch_bounds__(1024) void row_scale_kernel(const float* __restrict__ w, const int32_t* __restrict__ y,
                                                         const int32_t* __restrict__ valid_len,
                                                         const float* __restrict__ grad_loss, int B, int K, int V,
                                                         int reduction, float beta, float* __restrict__ g) {
  __shared__ int sh[1024];
  const int64_t T = (int64_t)B * K;
  auto valid = [&](int64_t t) {
    const int b = (int)(t / K), k = (int)(t % K);
    const int Kb = valid_len ? valid_len[b] : K;
    const int yv = y[t];
    return k < Kb && yv >= 0 && yv < V;
  };
  int cnt = 0;
  for (int64_t t = threadIdx.x; t < T; t += blockDim.x) cnt += valid(t) ? 1 : 0;
  sh[threadIdx.x] = cnt;
  __syncthreads();
  for (int s = 512; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) sh[threadIdx.x] += sh[threadIdx.x + s];
    __syncthreads();
  }
  const int n = sh[0];
  const float go = grad_loss ? *grad_loss : 1.f;
  float scale;
  if (reduction == 0)
    scale = n > 0 ? go * beta / (float)n : 0.f;
  else
    scale = go * beta;
  for (int64_t t = threadIdx.x; t < T; t += blockDim.x) g[t] = valid(t) ? scale * w[t] : 0.f;
}

hipError_t launch_row_scale(const float* w, const int32_t* y, const int32_t* valid_len, const float* grad_loss,
                            int B, int K, int V, int ignore_index, int reduction, float beta, float* g,
                            hipStream_t s) {
  (void)ignore_index;  // ignore_index is outside [0, V) by validation: the range test covers it
  hipLaunchKernelGGL(row_scale_kernel, dim3(1), dim3(1024), 0, s, w, y, valid_len, grad_loss, B, K, V, reduction,
                     beta, g);
  return hipGetLastError();
}

}  // namespace pard2
