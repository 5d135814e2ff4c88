// C ABI of the CAT-loss library: argument validation, workspace carving and the
// launch sequence.  No computation happens here.
#include "../../include/pard2_cat.h"

#include "kernels.h"

#include <math.h>
#include <string.h>

#include <mutex>
#include <vector>

using namespace pard2;

// ---- optional per-kernel event timing -------------------------------------------------
namespace pard2 {
namespace {
struct TimedLaunch {
  int id;
  hipEvent_t start, stop;
};
bool g_timing = false;
std::mutex g_timing_mu;
std::vector<TimedLaunch> g_launches;
}  // namespace

bool kt_events(int id, hipStream_t s, hipEvent_t* start, hipEvent_t* stop) {
  if (!g_timing) return false;
  hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(s, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone) return false;
  TimedLaunch t{id, nullptr, nullptr};
  if (hipEventCreate(&t.start) != hipSuccess) return false;
  if (hipEventCreate(&t.stop) != hipSuccess) {
    (void)hipEventDestroy(t.start);
    return false;
  }
  *start = t.start;
  *stop = t.stop;
  std::lock_guard<std::mutex> lk(g_timing_mu);
  g_launches.push_back(t);
  return true;
}
}  // namespace pard2

namespace {

struct FwdPlan {
  int P;
  size_t off_ms, off_idx, off_zy, off_conf, off_hit, off_partials, total;
};

size_t align256(size_t x) { return (x + 255) / 256 * 256; }

FwdPlan plan_fwd(const pard2_cat_desc* d) {
  FwdPlan p{};
  p.P = d->dtype == PARD2_BF16 ? fwd_num_partials_bf16(d->T, d->V) : fwd_num_partials_f32(d->T, d->V);
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o += align256(bytes); return at; };
  p.off_ms = take((size_t)d->T * p.P * sizeof(float2));
  p.off_idx = take((size_t)d->T * p.P * sizeof(int32_t));
  p.off_zy = take((size_t)d->T * 4);
  p.off_conf = take((size_t)d->T * 4);
  p.off_hit = take((size_t)d->T * 4);
  p.off_partials = take((size_t)scan_num_groups(d->B) * 2 * sizeof(double));
  p.total = o;
  return p;
}

size_t bwd_bytes(const pard2_cat_desc* d) {
  return d->dtype == PARD2_BF16 ? plan_bwd_bf16(d->T, d->d, d->V).total : plan_bwd_f32(d->T, d->d, d->V).total;
}

// workspace of the two-head forward: both heads' partial statistics, per-row scratch
struct KdFwdPlan {
  int P;    // vocabulary partials per row of the two-head sweep
  int P1;   // ... of a single-head sweep (the forward without the cross term runs two of those)
  size_t off_ms, off_idx, off_zy, off_ms_t, off_idx_t, off_a_t, off_zy_t, off_tok, off_conf, off_hit, off_partials,
      total;
};

// workspace of the two-head backward beyond the single-head plan: per-row cross-term partials and the
// per-row loss term, for a loss evaluated after the backward
struct KdBwdExtra {
  int nparts;
  size_t off_part, off_tok, total;
};

KdFwdPlan plan_kd_fwd(const pard2_cat_desc* d) {
  KdFwdPlan p{};
  p.P = d->dtype == PARD2_BF16 ? kd_num_partials_bf16(d->T, d->V) : fwd_num_partials_f32(d->T, d->V);
  p.P1 = d->dtype == PARD2_BF16 ? fwd_num_partials_bf16(d->T, d->V) : fwd_num_partials_f32(d->T, d->V);
  const int pm = p.P > p.P1 ? p.P : p.P1;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o += align256(bytes); return at; };
  p.off_ms = take((size_t)d->T * pm * sizeof(float2));
  p.off_idx = take((size_t)d->T * pm * sizeof(int32_t));
  p.off_zy = take((size_t)d->T * 4);
  p.off_ms_t = take((size_t)d->T * pm * sizeof(float2));
  p.off_idx_t = take((size_t)d->T * pm * sizeof(int32_t));
  p.off_a_t = take((size_t)d->T * pm * sizeof(float));
  p.off_zy_t = take((size_t)d->T * 4);
  p.off_tok = take((size_t)d->T * 4);
  p.off_conf = take((size_t)d->T * 4);
  p.off_hit = take((size_t)d->T * 4);
  p.off_partials = take((size_t)scan_num_groups(d->B) * 2 * sizeof(double));
  p.total = o;
  return p;
}

KdBwdExtra plan_kd_bwd_extra(const pard2_cat_desc* d) {
  KdBwdExtra x{};
  x.nparts = d->dtype == PARD2_BF16 ? kd_num_row_parts_bf16(d->V) : kd_num_row_parts_f32(d->V);
  size_t o = align256(bwd_bytes(d));
  x.off_part = o;
  o += align256((size_t)x.nparts * d->T * 4);
  x.off_tok = o;
  o += align256((size_t)d->T * 4);
  x.total = o;
  return x;
}

// descriptor + teacher checks shared by the two-head entry points (teacher pointers may be
// left out for the host-only size query)
int validate_kd(const pard2_cat_desc* d, int32_t dt, int64_t ldHt, int64_t ldWt) {
  int rc = pard2_cat_validate(d);
  if (rc != PARD2_OK) return rc;
  if (!(d->beta >= 0.f)) return PARD2_ERR_HYPER;
  if (dt <= 0 || ldHt < dt || ldWt < dt) return PARD2_ERR_SHAPE;
  if (d->dtype == PARD2_BF16 && ((dt & 7) || (ldHt & 7) || (ldWt & 7))) return PARD2_ERR_SHAPE;
  if (ldHt * 2 * 512 > 0x7fffffffLL || ldWt * 2 * 512 > 0x7fffffffLL) return PARD2_ERR_SHAPE;
  return PARD2_OK;
}

int check_arch() {
  static int cached[64];  // 0 unknown, 1 ok, 2 wrong
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return PARD2_ERR_ARCH;
  if (dev >= 0 && dev < 64 && cached[dev]) return cached[dev] == 1 ? PARD2_OK : PARD2_ERR_ARCH;
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return PARD2_ERR_ARCH;
  const bool ok = strncmp(prop.gcnArchName, "gfx950", 6) == 0;
  if (dev >= 0 && dev < 64) cached[dev] = ok ? 1 : 2;
  return ok ? PARD2_OK : PARD2_ERR_ARCH;
}

int check_workspace(const void* ws, size_t have, size_t need) {
  if (need == 0) return PARD2_OK;
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255) || have < need) return PARD2_ERR_WORKSPACE;
  return PARD2_OK;
}

bool misaligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) != 0; }

__global__ void set_i32_kernel(int32_t* p, int32_t v) { *p = v; }

}  // namespace

extern "C" {

int pard2_cat_abi_version(void) { return 1; }

int pard2_cat_kernel_timing(int enable) {
  std::lock_guard<std::mutex> lk(g_timing_mu);
  for (auto& t : g_launches) {
    (void)hipEventDestroy(t.start);
    (void)hipEventDestroy(t.stop);
  }
  g_launches.clear();
  g_timing = enable != 0;
  return PARD2_OK;
}

int pard2_cat_kernel_timing_read(int kernel, double* total_ms, int64_t* launches) {
  if (!total_ms || !launches) return PARD2_ERR_NULL;
  if (kernel < 0 || kernel >= KT_COUNT) return PARD2_ERR_SHAPE;
  std::lock_guard<std::mutex> lk(g_timing_mu);
  double sum = 0.0;
  int64_t n = 0;
  for (auto& t : g_launches) {
    if (t.id != kernel) continue;
    if (hipEventSynchronize(t.stop) != hipSuccess) return PARD2_ERR_LAUNCH;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, t.start, t.stop) != hipSuccess) return PARD2_ERR_LAUNCH;
    sum += ms;
    ++n;
  }
  *total_ms = sum;
  *launches = n;
  return PARD2_OK;
}

const char* pard2_status_string(int s) {
  switch (s) {
    case PARD2_OK: return "ok";
    case PARD2_ERR_NULL: return "required pointer is NULL";
    case PARD2_ERR_SHAPE: return "bad shape, stride or alignment";
    case PARD2_ERR_DTYPE: return "unknown dtype, weight_mode or reduction";
    case PARD2_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case PARD2_ERR_ARCH: return "device is not gfx950";
    case PARD2_ERR_HYPER: return "bad hyper-parameter";
    case PARD2_ERR_LAUNCH: return "HIP launch error";
    default: return "unknown status";
  }
}

int pard2_cat_validate(const pard2_cat_desc* d) {
  if (!d) return PARD2_ERR_NULL;
  if (d->dtype != PARD2_BF16 && d->dtype != PARD2_FP32) return PARD2_ERR_DTYPE;
  if (d->flags & ~PARD2_FLAG_DW_FP32) return PARD2_ERR_DTYPE;
  if (d->weight_mode < PARD2_W_CAT || d->weight_mode > PARD2_W_UNIFORM) return PARD2_ERR_DTYPE;
  if (d->reduction != PARD2_RED_MEAN_VALID && d->reduction != PARD2_RED_SUM) return PARD2_ERR_DTYPE;
  if (d->T <= 0 || d->d <= 0 || d->V <= 0 || d->B <= 0 || d->K <= 0) return PARD2_ERR_SHAPE;
  if ((int64_t)d->B * d->K != (int64_t)d->T) return PARD2_ERR_SHAPE;
  if (d->ldH < d->d || d->ldW < d->d) return PARD2_ERR_SHAPE;
  if (d->dtype == PARD2_BF16 && ((d->d & 7) || (d->ldH & 7) || (d->ldW & 7))) return PARD2_ERR_SHAPE;
  // tile-relative byte offsets inside the kernels are 32-bit
  if ((int64_t)d->ldH * 2 * 512 > 0x7fffffffLL || (int64_t)d->ldW * 2 * 512 > 0x7fffffffLL) return PARD2_ERR_SHAPE;
  if (d->ignore_index >= 0 && d->ignore_index < d->V) return PARD2_ERR_HYPER;
  if (!isfinite(d->beta)) return PARD2_ERR_HYPER;
  if (d->weight_mode == PARD2_W_DECAY && !(d->gamma > 0.f && d->gamma <= 1.f)) return PARD2_ERR_HYPER;
  return PARD2_OK;
}

size_t pard2_cat_workspace_bytes(const pard2_cat_desc* d) {
  if (pard2_cat_validate(d) != PARD2_OK) return 0;
  const size_t f = plan_fwd(d).total, b = bwd_bytes(d);
  return f > b ? f : b;
}

int pard2_cat_weights(const pard2_cat_desc* d, const float* conf, const int32_t* y, const int32_t* valid_len,
                      float* w, float* exp_len, void* stream) {
  int rc = pard2_cat_validate(d);
  if (rc != PARD2_OK) return rc;
  if (!conf || !w) return PARD2_ERR_NULL;
  if ((rc = check_arch()) != PARD2_OK) return rc;
  ScanArgs a{};
  a.conf = conf; a.y = y; a.valid_len = valid_len; a.w = w; a.exp_len = exp_len;
  a.B = d->B; a.K = d->K; a.V = d->V; a.ignore_index = d->ignore_index;
  a.weight_mode = d->weight_mode; a.reduction = d->reduction; a.beta = d->beta; a.gamma = d->gamma;
  return launch_scan(a, (hipStream_t)stream) == hipSuccess ? PARD2_OK : PARD2_ERR_LAUNCH;
}

int pard2_cat_weights_seq(const pard2_cat_desc* d, const float* conf_seq, int64_t n_pos, const int32_t* anchor_pos,
                          const int32_t* seq_end, const int32_t* y, float* w, float* conf, int32_t* valid_len,
                          float* exp_len, void* stream) {
  int rc = pard2_cat_validate(d);
  if (rc != PARD2_OK) return rc;
  if (!conf_seq || !anchor_pos || !seq_end || !w) return PARD2_ERR_NULL;
  if (n_pos <= 0) return PARD2_ERR_SHAPE;
  if ((rc = check_arch()) != PARD2_OK) return rc;
  ScanArgs a{};
  a.conf_seq = conf_seq; a.n_pos = n_pos; a.anchor_pos = anchor_pos; a.seq_end = seq_end;
  a.conf_out = conf; a.valid_len_out = valid_len;
  a.y = y; a.w = w; a.exp_len = exp_len;
  a.B = d->B; a.K = d->K; a.V = d->V; a.ignore_index = d->ignore_index;
  a.weight_mode = d->weight_mode; a.reduction = d->reduction; a.beta = d->beta; a.gamma = d->gamma;
  return launch_scan(a, (hipStream_t)stream) == hipSuccess ? PARD2_OK : PARD2_ERR_LAUNCH;
}

int pard2_cat_fwd(const pard2_cat_desc* d, const void* H, const void* W, const int32_t* y, const float* conf_in,
                  const int32_t* valid_len, float* loss, float* lse, float* logp_y, float* w, int32_t* argmax,
                  int32_t* accept_len, float* exp_len, int32_t* dev_status, void* workspace, size_t workspace_bytes,
                  void* stream) {
  int rc = pard2_cat_validate(d);
  if (rc != PARD2_OK) return rc;
  if (!H || !W || !y || !lse || !logp_y) return PARD2_ERR_NULL;
  if (d->dtype == PARD2_BF16 && (misaligned16(H) || misaligned16(W))) return PARD2_ERR_SHAPE;
  const FwdPlan p = plan_fwd(d);
  if ((rc = check_workspace(workspace, workspace_bytes, p.total)) != PARD2_OK) return rc;
  if ((rc = check_arch()) != PARD2_OK) return rc;
  hipStream_t s = (hipStream_t)stream;
  char* ws = (char*)workspace;
  StatsOut st{(float2*)(ws + p.off_ms), (int32_t*)(ws + p.off_idx), (float*)(ws + p.off_zy), p.P};
  float* conf = (float*)(ws + p.off_conf);
  int32_t* hit = (int32_t*)(ws + p.off_hit);

  if (dev_status) hipLaunchKernelGGL(set_i32_kernel, dim3(1), dim3(1), 0, s, dev_status, 0);
  hipError_t e = d->dtype == PARD2_BF16
                     ? launch_fwd_stats_bf16(H, d->ldH, W, d->ldW, y, d->T, d->d, d->V, st, s)
                     : launch_fwd_stats_f32(H, d->ldH, W, d->ldW, y, d->T, d->d, d->V, st, s);
  if (e != hipSuccess) return PARD2_ERR_LAUNCH;
  e = launch_combine(st, y, conf_in, d->T, d->V, d->ignore_index, lse, logp_y, argmax, conf, hit, dev_status, s);
  if (e != hipSuccess) return PARD2_ERR_LAUNCH;
  if (loss || w || accept_len || exp_len) {
    ScanArgs a{};
    a.conf = conf; a.y = y; a.valid_len = valid_len; a.hit = hit; a.logp_y = logp_y;
    a.w = w; a.exp_len = exp_len; a.accept_len = accept_len; a.loss = loss;
    a.loss_partials = (double*)(ws + p.off_partials);
    a.B = d->B; a.K = d->K; a.V = d->V; a.ignore_index = d->ignore_index;
    a.weight_mode = d->weight_mode; a.reduction = d->reduction; a.beta = d->beta; a.gamma = d->gamma;
    if (launch_scan(a, s) != hipSuccess) return PARD2_ERR_LAUNCH;
  }
  return PARD2_OK;
}

int pard2_cat_bwd(const pard2_cat_desc* d, const void* H, const void* W, const int32_t* y, const int32_t* valid_len,
                  const float* lse, const float* w, const float* grad_loss, void* dH, void* dW,
                  int32_t accumulate_dW, void* workspace, size_t workspace_bytes, void* stream) {
  int rc = pard2_cat_validate(d);
  if (rc != PARD2_OK) return rc;
  if (!H || !W || !y || !lse || !w || !dH || !dW) return PARD2_ERR_NULL;
  if (d->dtype == PARD2_BF16 && (misaligned16(H) || misaligned16(W) || misaligned16(dH) || misaligned16(dW)))
    return PARD2_ERR_SHAPE;
  if ((rc = check_workspace(workspace, workspace_bytes, bwd_bytes(d))) != PARD2_OK) return rc;
  if ((rc = check_arch()) != PARD2_OK) return rc;
  hipStream_t s = (hipStream_t)stream;
  char* ws = (char*)workspace;
  hipError_t e;
  if (d->dtype == PARD2_BF16) {
    const BwdPlanBf16 p = plan_bwd_bf16(d->T, d->d, d->V);
    float* g = (float*)(ws + p.off_g);
    e = launch_row_scale(w, y, valid_len, grad_loss, d->B, d->K, d->V, d->ignore_index, d->reduction, d->beta, g, s);
    if (e != hipSuccess) return PARD2_ERR_LAUNCH;
    e = launch_bwd_bf16(p, H, d->ldH, W, d->ldW, y, lse, g, d->T, d->d, d->V, dH, dW,
                        accumulate_dW | ((d->flags & PARD2_FLAG_DW_FP32) ? 2 : 0), ws, s);
  } else {
    const BwdPlanF32 p = plan_bwd_f32(d->T, d->d, d->V);
    float* g = (float*)(ws + p.off_g);
    e = launch_row_scale(w, y, valid_len, grad_loss, d->B, d->K, d->V, d->ignore_index, d->reduction, d->beta, g, s);
    if (e != hipSuccess) return PARD2_ERR_LAUNCH;
    e = launch_bwd_f32(p, H, d->ldH, W, d->ldW, y, lse, g, d->T, d->d, d->V, dH, dW, accumulate_dW, ws, s);
  }
  return e == hipSuccess ? PARD2_OK : PARD2_ERR_LAUNCH;
}

size_t pard2_cat_kd_workspace_bytes(const pard2_cat_desc* d, int32_t teacher_d) {
  if (validate_kd(d, teacher_d, teacher_d, teacher_d) != PARD2_OK) return 0;
  const size_t f = plan_kd_fwd(d).total, b = plan_kd_bwd_extra(d).total;
  return f > b ? f : b;
}

int pard2_cat_kd_fwd(const pard2_cat_desc* d, const void* H, const void* W, const pard2_kd_teacher* te,
                     const int32_t* y, const float* conf_in, const int32_t* valid_len, float* loss, float* lse,
                     float* lse_t, float* logp_y, float* kd, float* w, int32_t* argmax, int32_t* accept_len,
                     float* exp_len, int32_t* dev_status, void* workspace, size_t workspace_bytes, void* stream) {
  if (!d || !te) return PARD2_ERR_NULL;
  int rc = validate_kd(d, te->d, te->ldH, te->ldW);
  if (rc != PARD2_OK) return rc;
  if (!H || !W || !te->H || !te->W || !y || !lse || !lse_t || !logp_y) return PARD2_ERR_NULL;
  if (d->dtype == PARD2_BF16 && (misaligned16(H) || misaligned16(W) || misaligned16(te->H) || misaligned16(te->W)))
    return PARD2_ERR_SHAPE;
  const KdFwdPlan p = plan_kd_fwd(d);
  if ((rc = check_workspace(workspace, workspace_bytes, p.total)) != PARD2_OK) return rc;
  if ((rc = check_arch()) != PARD2_OK) return rc;
  hipStream_t s = (hipStream_t)stream;
  char* ws = (char*)workspace;
  KdStatsOut st{};
  st.draft = StatsOut{(float2*)(ws + p.off_ms), (int32_t*)(ws + p.off_idx), (float*)(ws + p.off_zy), p.P};
  st.ms_t = (float2*)(ws + p.off_ms_t);
  st.a_t = (float*)(ws + p.off_a_t);
  st.zy_t = (float*)(ws + p.off_zy_t);
  float* tok = (float*)(ws + p.off_tok);
  float* conf = (float*)(ws + p.off_conf);
  int32_t* hit = (int32_t*)(ws + p.off_hit);
  const KdTeacher kt{te->H, te->W, te->ldH, te->ldW, te->d, nullptr, d->beta, nullptr};

  if (dev_status) hipLaunchKernelGGL(set_i32_kernel, dim3(1), dim3(1), 0, s, dev_status, 0);
  if (!loss && !kd) {
    // Nothing asked for needs both heads' logits at the same (token, id): two single-head sweeps at the
    // single-head kernels' larger tile.  The cross term of the KL can be had from the backward instead.
    StatsOut sd{st.draft.ms, st.draft.idx, st.draft.zy, p.P1};
    StatsOut stt{st.ms_t, (int32_t*)(ws + p.off_idx_t), st.zy_t, p.P1};
    hipError_t e1, e2;
    if (d->dtype == PARD2_BF16) {
      e1 = launch_fwd_stats_bf16(te->H, te->ldH, te->W, te->ldW, y, d->T, te->d, d->V, stt, s);
      e2 = launch_fwd_stats_bf16(H, d->ldH, W, d->ldW, y, d->T, d->d, d->V, sd, s);
    } else {
      e1 = launch_fwd_stats_f32(te->H, te->ldH, te->W, te->ldW, y, d->T, te->d, d->V, stt, s);
      e2 = launch_fwd_stats_f32(H, d->ldH, W, d->ldW, y, d->T, d->d, d->V, sd, s);
    }
    if (e1 != hipSuccess || e2 != hipSuccess) return PARD2_ERR_LAUNCH;
    // teacher: lse_t and the confidence (given, or its own p(y), Eq.9); tok serves as scratch for log p(y)
    if (launch_combine(stt, y, conf_in, d->T, d->V, d->ignore_index, lse_t, tok, nullptr, conf, nullptr, dev_status,
                       s) != hipSuccess)
      return PARD2_ERR_LAUNCH;
    if (launch_combine(sd, y, nullptr, d->T, d->V, d->ignore_index, lse, logp_y, argmax, nullptr, hit, dev_status, s) !=
        hipSuccess)
      return PARD2_ERR_LAUNCH;
    if (w || accept_len || exp_len) {
      ScanArgs a{};
      a.conf = conf; a.y = y; a.valid_len = valid_len; a.hit = hit;
      a.w = w; a.exp_len = exp_len; a.accept_len = accept_len;
      a.B = d->B; a.K = d->K; a.V = d->V; a.ignore_index = d->ignore_index;
      a.weight_mode = d->weight_mode; a.reduction = d->reduction; a.beta = 1.f; a.gamma = d->gamma;
      if (launch_scan(a, s) != hipSuccess) return PARD2_ERR_LAUNCH;
    }
    return PARD2_OK;
  }
  const hipError_t e = d->dtype == PARD2_BF16 ? launch_kd_stats_bf16(H, d->ldH, W, d->ldW, kt, y, d->T, d->d, d->V, st, s)
                                              : launch_kd_stats_f32(H, d->ldH, W, d->ldW, kt, y, d->T, d->d, d->V, st, s);
  if (e != hipSuccess) return PARD2_ERR_LAUNCH;
  if (launch_kd_combine(st, y, conf_in, d->T, d->V, d->ignore_index, d->beta, lse, lse_t, logp_y, kd, tok, argmax, conf,
                        hit, dev_status, s) != hipSuccess)
    return PARD2_ERR_LAUNCH;
  if (loss || w || accept_len || exp_len) {
    ScanArgs a{};
    a.conf = conf; a.y = y; a.valid_len = valid_len; a.hit = hit;
    a.logp_y = tok;   // minus the row's (beta CE + KD): the reduction sums w * (-tok), with coefficient 1
    a.w = w; a.exp_len = exp_len; a.accept_len = accept_len; a.loss = loss;
    a.loss_partials = (double*)(ws + p.off_partials);
    a.B = d->B; a.K = d->K; a.V = d->V; a.ignore_index = d->ignore_index;
    a.weight_mode = d->weight_mode; a.reduction = d->reduction; a.beta = 1.f; a.gamma = d->gamma;
    if (launch_scan(a, s) != hipSuccess) return PARD2_ERR_LAUNCH;
  }
  return PARD2_OK;
}

int pard2_cat_kd_bwd(const pard2_cat_desc* d, const void* H, const void* W, const pard2_kd_teacher* te,
                     const int32_t* y, const int32_t* valid_len, const float* lse, const float* lse_t, const float* w,
                     const float* grad_loss, void* dH, void* dW, int32_t accumulate_dW, const float* logp_y,
                     float* kd, float* loss, void* workspace, size_t workspace_bytes, void* stream) {
  if (!d || !te) return PARD2_ERR_NULL;
  int rc = validate_kd(d, te->d, te->ldH, te->ldW);
  if (rc != PARD2_OK) return rc;
  if (!H || !W || !te->H || !te->W || !y || !lse || !lse_t || !w || !dH || !dW) return PARD2_ERR_NULL;
  if (loss && !logp_y) return PARD2_ERR_NULL;
  if (d->dtype == PARD2_BF16 && (misaligned16(H) || misaligned16(W) || misaligned16(te->H) || misaligned16(te->W) ||
                                 misaligned16(dH) || misaligned16(dW)))
    return PARD2_ERR_SHAPE;
  const KdBwdExtra x = plan_kd_bwd_extra(d);
  if ((rc = check_workspace(workspace, workspace_bytes, x.total)) != PARD2_OK) return rc;
  if ((rc = check_arch()) != PARD2_OK) return rc;
  hipStream_t s = (hipStream_t)stream;
  char* ws = (char*)workspace;
  float* kd_part = (kd || loss) ? (float*)(ws + x.off_part) : nullptr;
  const KdTeacher kt{te->H, te->W, te->ldH, te->ldW, te->d, lse_t, d->beta, kd_part};
  // g_t = grad_loss w_t / N: beta sits inside the bracket of Eq.12
  hipError_t e;
  if (d->dtype == PARD2_BF16) {
    const BwdPlanBf16 p = plan_bwd_bf16(d->T, d->d, d->V);
    float* g = (float*)(ws + p.off_g);
    e = launch_row_scale(w, y, valid_len, grad_loss, d->B, d->K, d->V, d->ignore_index, d->reduction, 1.f, g, s);
    if (e != hipSuccess) return PARD2_ERR_LAUNCH;
    e = launch_bwd_bf16(p, H, d->ldH, W, d->ldW, y, lse, g, d->T, d->d, d->V, dH, dW,
                        accumulate_dW | ((d->flags & PARD2_FLAG_DW_FP32) ? 2 : 0), ws, s, &kt);
  } else {
    const BwdPlanF32 p = plan_bwd_f32(d->T, d->d, d->V);
    float* g = (float*)(ws + p.off_g);
    e = launch_row_scale(w, y, valid_len, grad_loss, d->B, d->K, d->V, d->ignore_index, d->reduction, 1.f, g, s);
    if (e != hipSuccess) return PARD2_ERR_LAUNCH;
    e = launch_bwd_f32(p, H, d->ldH, W, d->ldW, y, lse, g, d->T, d->d, d->V, dH, dW, accumulate_dW, ws, s, &kt);
  }
  if (e != hipSuccess) return PARD2_ERR_LAUNCH;
  if (kd_part) {   // the loss of this step, evaluated from what the backward's recompute saw
    float* tok = (float*)(ws + x.off_tok);
    if (launch_kd_finish(kd_part, x.nparts, lse, lse_t, logp_y, y, d->beta, d->T, d->V, kd, loss ? tok : nullptr, s) !=
        hipSuccess)
      return PARD2_ERR_LAUNCH;
    if (loss && launch_weighted_loss(w, tok, y, valid_len, d->B, d->K, d->V, d->reduction, loss, s) != hipSuccess)
      return PARD2_ERR_LAUNCH;
  }
  return PARD2_OK;
}

static int validate_inject(int32_t T, int32_t d, int32_t dt, int32_t F, int64_t ldX) {
  if (T <= 0 || d <= 0 || dt <= 0 || F < 1 || F > 8) return PARD2_ERR_SHAPE;
  if ((d & 7) || (dt & 7) || (ldX & 7) || ldX < dt) return PARD2_ERR_SHAPE;
  // tile-relative byte offsets inside the kernels are 32-bit
  if ((int64_t)F * dt * 2 * 512 > 0x7fffffffLL || ldX * 2 * 512 > 0x7fffffffLL || (int64_t)d * 2 * 512 > 0x7fffffffLL)
    return PARD2_ERR_SHAPE;
  return PARD2_OK;
}

static int gather_feats(const void* const* feats, int F, InjectFeats* out) {
  for (int f = 0; f < 8; ++f) out->p[f] = nullptr;
  for (int f = 0; f < F; ++f) {
    if (!feats[f]) return PARD2_ERR_NULL;
    if (misaligned16(feats[f])) return PARD2_ERR_SHAPE;
    out->p[f] = feats[f];
  }
  return PARD2_OK;
}

int pard2_inject_fwd(int32_t T, int32_t d, int32_t dt, int32_t F, const void* E, const void* const* feats, int64_t ldX,
                     const void* P, const float* xi, void* Eout, void* stream) {
  int rc = validate_inject(T, d, dt, F, ldX);
  if (rc != PARD2_OK) return rc;
  if (!E || !feats || !P || !xi || !Eout) return PARD2_ERR_NULL;
  if (misaligned16(E) || misaligned16(P) || misaligned16(Eout)) return PARD2_ERR_SHAPE;
  InjectFeats fs;
  if ((rc = gather_feats(feats, F, &fs)) != PARD2_OK) return rc;
  if ((rc = check_arch()) != PARD2_OK) return rc;
  return launch_inject_fwd(E, fs, ldX, P, xi, T, d, dt, F, Eout, (hipStream_t)stream) == hipSuccess ? PARD2_OK
                                                                                                  : PARD2_ERR_LAUNCH;
}

int pard2_inject_bwd(int32_t T, int32_t d, int32_t dt, int32_t F, const void* dEout, const void* const* feats,
                     int64_t ldX, const float* xi, void* dT, void* dP, int32_t accumulate_dP, void* stream) {
  int rc = validate_inject(T, d, dt, F, ldX);
  if (rc != PARD2_OK) return rc;
  if (!dEout || !feats || !xi || !dT || !dP) return PARD2_ERR_NULL;
  if (misaligned16(dEout) || misaligned16(dT) || misaligned16(dP)) return PARD2_ERR_SHAPE;
  InjectFeats fs;
  if ((rc = gather_feats(feats, F, &fs)) != PARD2_OK) return rc;
  if ((rc = check_arch()) != PARD2_OK) return rc;
  return launch_inject_bwd(dEout, fs, ldX, xi, T, d, dt, F, dT, dP, accumulate_dP, (hipStream_t)stream) == hipSuccess
             ? PARD2_OK
             : PARD2_ERR_LAUNCH;
}

}  // extern "C"
