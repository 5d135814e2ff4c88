// Internal launch interface between the C-ABI layer and the kernel translation units.
// Host functions only; every pointer below is a device pointer.
#pragma once
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pard2 {

inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

// Optional per-kernel timing (off by default): when switched on through
// pard2_cat_kernel_timing(), every launch of one of the contraction kernels carries a
// pair of HIP events.
enum KernelId { KT_FWD_STATS = 0, KT_DZ = 1, KT_DH = 2, KT_DW = 3, KT_KD_STATS = 4, KT_KD_DZ = 5,
                KT_INJECT_FWD = 6, KT_INJECT_DP = 7, KT_COUNT = 8 };
// false when timing is off or the stream is being captured into a graph; otherwise creates a start/stop pair, records it under `id` and hands it out
bool kt_events(int id, hipStream_t s, hipEvent_t* start, hipEvent_t* stop);

// Launch one of the timed kernels.  With timing on, the start/stop events ride on the kernel's own dispatch
// packet (hipExtLaunchKernelGGL), so no marker packets are queued between kernels and the launch-to-launch
// gaps stay what they are without timing.
template <class K, class... Args>
inline void launch_timed(int id, K kernel, dim3 grid, dim3 block, unsigned lds, hipStream_t s, Args... args) {
  hipEvent_t e0, e1;
  if (kt_events(id, s, &e0, &e1))
    hipExtLaunchKernelGGL(kernel, grid, block, lds, s, e0, e1, 0, args...);
  else
    hipLaunchKernelGGL(kernel, grid, block, lds, s, args...);
}

// Per-row, per-partial softmax statistics written by the forward sweep:
// ms[t*P + p] = (max, sum of exp(z - max)) over the p-th vocabulary range, idx = lowest
// index attaining that max; zy[t] = logit of the target id (written only for valid ids).
struct StatsOut {
  float2* ms;
  int32_t* idx;
  float* zy;
  int P;
};

// number of vocabulary partials per row the forward sweep produces
int fwd_num_partials_bf16(int T, int V);
int fwd_num_partials_f32(int T, int V);

hipError_t launch_fwd_stats_bf16(const void* H, int64_t ldH, const void* W, int64_t ldW, const int32_t* y,
                                 int T, int d, int V, StatsOut out, hipStream_t s);
hipError_t launch_fwd_stats_f32(const void* H, int64_t ldH, const void* W, int64_t ldW, const int32_t* y,
                                int T, int d, int V, StatsOut out, hipStream_t s);

// Merge partials: lse, log q(y), argmax, confidence; flags out-of-range targets.
hipError_t launch_combine(StatsOut st, const int32_t* y, const float* conf_in, int T, int V, int ignore_index,
                          float* lse, float* logp_y, int32_t* argmax, float* conf, int32_t* hit,
                          int32_t* dev_status, hipStream_t s);

// Per-block exclusive prefix product (Eq.10) + masks + optional diagnostics and loss partials.
struct ScanArgs {
  const float* conf;        // [T] confidences per (block, slot), or null when gathered (below)
  // gather mode (Sec.3.3 weights s_{n,k}): conf[b,k] = conf_seq[anchor_pos[b] + k] where that position
  // exists (below seq_end[b] and n_pos), 1 elsewhere; the block's valid length is cut accordingly
  const float* conf_seq;    // [n_pos] or null
  const int32_t* anchor_pos; // [B]
  const int32_t* seq_end;   // [B]
  int64_t n_pos;
  float* conf_out;          // [T] or null: the gathered confidences
  int32_t* valid_len_out;   // [B] or null: the resulting valid lengths
  const int32_t* y;         // [T] or null
  const int32_t* valid_len; // [B] or null
  const int32_t* hit;       // [T] or null
  const float* logp_y;      // [T] or null (needed for loss)
  float* w;                 // [T] or null
  float* exp_len;           // [B] or null
  int32_t* accept_len;      // [B] or null
  float* loss;              // [1] or null
  double* loss_partials;    // workspace [2 * scan_num_groups(B)] (needed for loss)
  int B, K, V, ignore_index, weight_mode, reduction;
  float beta, gamma;
};
int scan_num_groups(int B);
hipError_t launch_scan(const ScanArgs& a, hipStream_t s);

// g[t] = grad_loss * beta * w[t] / N on valid rows, 0 elsewhere (N from the masks).
hipError_t launch_row_scale(const float* w, const int32_t* y, const int32_t* valid_len, const float* grad_loss,
                            int B, int K, int V, int ignore_index, int reduction, float beta, float* g,
                            hipStream_t s);

// ---- backward, bf16 storage
struct BwdPlanBf16 {
  int64_t Vc;          // chunk width in vocabulary ids = row stride of the dZ scratch (elements)
  int nchunks;
  int kslices;         // k slices of the dH contraction (1 unless T x d has too few tiles)
  size_t off_g, off_dZ, off_dHacc, off_dHpart, total;
};
BwdPlanBf16 plan_bwd_bf16(int T, int d, int V);
// accumulate_dW: bit 0 = add to dW, bit 1 = dW is an fp32 [V, d] buffer (else bf16).
// The teacher side of the distillation term (Eq.12), when present: dZ then is
// g_t (beta (q - 1[v = y_t]) + q - p) with p the teacher head's softmax.
struct KdTeacher {
  const void* H;       // [T, d]
  const void* W;       // [V, d]
  int64_t ldH, ldW;
  int d;
  const float* lse;    // [T] logsumexp of the teacher's rows
  float beta;
  // backward only, or null: [row parts][T] per-row partial sums of p (zT - zD), one part per vocabulary
  // tile of the two-head dZ kernel (kd_num_row_parts_* parts), for a loss evaluated after the backward
  float* kd_part;
};
hipError_t launch_bwd_bf16(const BwdPlanBf16& p, const void* H, int64_t ldH, const void* W, int64_t ldW,
                           const int32_t* y, const float* lse, const float* g, int T, int d, int V,
                           void* dH, void* dW, int accumulate_dW, char* ws, hipStream_t s,
                           const KdTeacher* kd = nullptr);

// ---- two-head (draft + teacher) kernels of the distillation term, bf16 storage
// Forward sweep: the draft's statistics as in StatsOut plus, per row and vocabulary range, the
// teacher's (max, sum of exp) and a = sum_v exp(zT - max) (zT - zD); zy_t = teacher logit of the target.
struct KdStatsOut {
  StatsOut draft;
  float2* ms_t;
  float* a_t;
  float* zy_t;
};
int kd_num_partials_bf16(int T, int V);
hipError_t launch_kd_stats_f32(const void* H, int64_t ldH, const void* W, int64_t ldW, const KdTeacher& teacher,
                               const int32_t* y, int T, int d, int V, KdStatsOut out, hipStream_t s);
hipError_t launch_kd_stats_bf16(const void* H, int64_t ldH, const void* W, int64_t ldW, const KdTeacher& teacher,
                                const int32_t* y, int T, int d, int V, KdStatsOut out, hipStream_t s);
// Merge partials of both heads: lse, lse_t, log q(y), KL(p || q), argmax, confidence (given, or the
// teacher's p(y)), hit, and tok[t] = beta log q(y) - KL (minus the row's loss term; 0 on rows without target).
hipError_t launch_kd_combine(KdStatsOut st, const int32_t* y, const float* conf_in, int T, int V, int ignore_index,
                             float beta, float* lse, float* lse_t, float* logp_y, float* kd, float* tok,
                             int32_t* argmax, float* conf, int32_t* hit, int32_t* dev_status, hipStream_t s);
// dZ of one vocabulary chunk (tiles of kd_dz_tile() ids starting at id v0, Kc ids wide) into dZ[t][v - v0].
hipError_t launch_kd_dz_bf16(const void* H, int64_t ldH, const void* W, int64_t ldW, const KdTeacher& teacher,
                             const int32_t* y, const float* lse, const float* g, int T, int d, int V, int v0, int Kc,
                             void* dZ, int64_t ldz, float* kd_part, hipStream_t s);
int kd_num_row_parts_bf16(int V);
int kd_num_row_parts_f32(int V);
// kd[t] = sum over parts of kd_part[part][t] - lse_t[t] + lse[t]; tok[t] = beta log q(y) - kd (0 without target)
hipError_t launch_kd_finish(const float* kd_part, int nparts, const float* lse, const float* lse_t,
                            const float* logp_y, const int32_t* y, float beta, int T, int V, float* kd, float* tok,
                            hipStream_t s);
// loss = (1/N) sum over valid rows of w[t] * (-tok[t])  (N = valid rows, or 1 for the SUM reduction)
hipError_t launch_weighted_loss(const float* w, const float* tok, const int32_t* y, const int32_t* valid_len, int B,
                                int K, int V, int reduction, float* loss, hipStream_t s);

// ---- backward, fp32 storage
struct BwdPlanF32 {
  int64_t Vc;
  int nchunks;
  size_t off_g, off_dZ, total;
};
BwdPlanF32 plan_bwd_f32(int T, int d, int V);
hipError_t launch_bwd_f32(const BwdPlanF32& p, const void* H, int64_t ldH, const void* W, int64_t ldW,
                          const int32_t* y, const float* lse, const float* g, int T, int d, int V,
                          void* dH, void* dW, int accumulate_dW, char* ws, hipStream_t s,
                          const KdTeacher* kd = nullptr);

// ---- gated injection of target features into the draft's input embeddings (Sec.3.3), bf16
struct InjectFeats {
  const void* p[8];   // F feature tensors [T, dt], common row stride
};
hipError_t launch_inject_fwd(const void* E, const InjectFeats& feats, int64_t ldX, const void* P, const float* xi,
                             int T, int d, int dt, int F, void* Eout, hipStream_t s);
hipError_t launch_inject_bwd(const void* dEout, const InjectFeats& feats, int64_t ldX, const float* xi, int T, int d,
                             int dt, int F, void* dT, void* dP, int accumulate, hipStream_t s);

}  // namespace pard2
