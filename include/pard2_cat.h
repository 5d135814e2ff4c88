/* pard2_cat.h — C ABI of the MI355X (gfx950) CAT-loss library for PARD-2 draft training.
 *
 * The library evaluates, for a parallel (mask-token) draft model's LM head, the
 * Confidence-Adaptive Token weighted cross-entropy and its gradients without ever
 * holding the T x V logits in memory:
 *
 *   logits       z[t,v] = sum_i H[t,i] W[v,i]                       head of Eq.4 / Eq.5
 *   log-softmax  log q_t(v) = z[t,v] - logsumexp_v z[t,v]           the log P of Eq.5 / Eq.11
 *   confidence   c_t = teacher probability of the true token        Eq.9
 *   weight       s[b,0] = 1,  s[b,k] = s[b,k-1] * c[b,k-1]          Eq.10 (per draft block)
 *   loss         (beta / N) * sum_t w_t * (-log q_t(y_t))           Eq.11, beta from Eq.12
 *   backward     dZ[t,v] = g_t (q_t(v) - 1[v = y_t]),  dH = dZ W,  dW = dZ^T H,
 *                g_t = grad_loss * beta * w_t / N; the weight is a constant
 *                (stop-gradient, Sec.3.2 text before Eq.11)
 *
 * Layout.  Token rows are block-major: row t = b*K + k is slot k of draft block
 * (anchor) b, T = B*K.  H is [T, d] with row stride ldH, W is [V, d] with row
 * stride ldW (elements); dH [T, d] and dW [V, d] are dense (row stride d).
 *
 * Pointers.  `desc` points to HOST memory.  Every other pointer is a DEVICE pointer
 * owned by the caller; the library never allocates, frees or keeps them.  Scratch
 * memory is the caller's `workspace` (device, 256-byte aligned, at least
 * pard2_cat_workspace_bytes(desc) bytes); its contents are undefined after a call.
 *
 * Execution.  All work is enqueued on `stream` (a hipStream_t passed as void*;
 * NULL = the default stream) and the calls return without synchronising.  Outputs
 * are fully overwritten (dW is added to when accumulate_dW != 0).  The device must
 * be gfx950: there is no fallback path.
 *
 * Errors.  Every entry point returns a pard2_status (0 = OK).  Host-detectable
 * problems (null pointer, bad shape/stride/dtype/hyper-parameter, workspace too
 * small, wrong device, failed launch) are returned before or instead of launching.
 * Data-dependent problems cannot be seen by the host: a target id outside [0, V)
 * that is not `ignore_index` sets *dev_status to a non-zero value on the device and
 * the row is treated as ignored.
 */
#ifndef PARD2_CAT_H
#define PARD2_CAT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  PARD2_OK = 0,
  PARD2_ERR_NULL = -1,      /* a required pointer is NULL                                  */
  PARD2_ERR_SHAPE = -2,     /* T != B*K, non-positive size, stride < d or misaligned       */
  PARD2_ERR_DTYPE = -3,     /* dtype / weight_mode / reduction not one of the enums below  */
  PARD2_ERR_WORKSPACE = -4, /* workspace NULL, misaligned or smaller than required         */
  PARD2_ERR_ARCH = -5,      /* current device is not gfx950                                */
  PARD2_ERR_HYPER = -6,     /* beta not finite, gamma outside (0, 1] in DECAY mode         */
  PARD2_ERR_LAUNCH = -7     /* HIP reported an error while enqueueing                      */
} pard2_status;

enum { PARD2_BF16 = 0, PARD2_FP32 = 1 };                  /* storage of H, W, dH, dW; sums are fp32 */
enum { PARD2_W_CAT = 0, PARD2_W_DECAY = 1, PARD2_W_UNIFORM = 2 };
enum { PARD2_RED_MEAN_VALID = 0, PARD2_RED_SUM = 1 };
/* descriptor flags.  PARD2_FLAG_DW_FP32: with bf16 storage, dW is an fp32 [V, d] buffer (written, or added to
 * when accumulate_dW != 0, without intermediate rounding: the main-gradient buffer of gradient accumulation,
 * Table 6's accumulation steps).  Ignored with fp32 storage, where dW is fp32 anyway. */
enum { PARD2_FLAG_DW_FP32 = 1 };

/* Problem descriptor (plain data, host memory). */
typedef struct {
  int32_t T, d, V;      /* token rows, hidden width, vocabulary size                         */
  int32_t B, K;         /* draft blocks (anchors) and slots per block; T must equal B*K      */
  int32_t dtype;        /* PARD2_BF16 or PARD2_FP32                                           */
  int32_t weight_mode;  /* PARD2_W_CAT: Eq.10.  PARD2_W_DECAY: gamma^k (fixed position decay,
                           the comparator of Table 3).  PARD2_W_UNIFORM: 1 (Eq.5).           */
  int32_t reduction;    /* PARD2_RED_MEAN_VALID: divide by the number of valid tokens (Eq.11's
                           1/K averaged over anchors when every block is full);
                           PARD2_RED_SUM: no division (Eq.12 as printed)                     */
  float beta;           /* coefficient of the CE term (Eq.12; 0.1 in Table 6, 1 gives Eq.11) */
  float gamma;          /* DECAY mode only, in (0, 1]                                        */
  int32_t ignore_index; /* a row whose target equals this carries no loss and no gradient    */
  int32_t flags;        /* 0, or PARD2_FLAG_DW_FP32                                           */
  int64_t ldH, ldW;     /* row strides of H and W in elements (>= d).  bf16: d, ldH, ldW must
                           be multiples of 8 and H, W 16-byte aligned                        */
} pard2_cat_desc;

/* Host-only helpers (no GPU needed). */
int pard2_cat_validate(const pard2_cat_desc* desc);            /* PARD2_OK or an error code       */
size_t pard2_cat_workspace_bytes(const pard2_cat_desc* desc);  /* 0 if the descriptor is invalid  */
const char* pard2_status_string(int status);
int pard2_cat_abi_version(void);

/* CAT weights of Eq.10 (or the DECAY / UNIFORM comparators) from given confidences.
 *   conf      [T]  confidences c[b,k] in [0,1] (Eq.9); not clamped.
 *   y         [T]  target ids or NULL; rows with y == ignore_index get w = 0 but the
 *                  product still runs through their conf.
 *   valid_len [B]  number of leading valid slots per block, or NULL = K everywhere;
 *                  slots k >= valid_len[b] get w = 0.
 *   w         [T]  out: s[b,k] on valid slots, 0 elsewhere.
 *   exp_len   [B]  out or NULL: estimated acceptance length sum_{k<valid_len} s_k c_k
 *                  (Eq.8 with the estimates of Eq.9/10).
 */
int pard2_cat_weights(const pard2_cat_desc* desc, const float* conf, const int32_t* y,
                      const int32_t* valid_len, float* w, float* exp_len, void* stream);

/* CAT weights gathered from ONE teacher pass over whole sequences (Sec.3.3: the weight of the
 * future token x_{n+k} given the prefix x_{<=n} depends on the anchor n as well as on k):
 *     conf[b,k] = c_seq[anchor_pos[b] + k],   s[b,k] = prod_{j<k} conf[b,j]      (Eq.10 per anchor)
 * so overlapping draft blocks of a sequence share the teacher's per-position confidences.
 *   c_seq      [n_pos] teacher probability of the token at each position of the concatenated
 *                      sequences (Eq.9, teacher-forced; e.g. exp(logp_y) of a stats-only forward).
 *   anchor_pos [B]     position of block b's slot-0 target token; negative = block absent.
 *   seq_end    [B]     one past the last position of the sequence holding block b: slots with
 *                      anchor_pos[b] + k >= min(seq_end[b], n_pos) do not exist (Eq.12 sums the
 *                      anchors n <= N - k only); they get w = 0 and conf = 1.
 *   y          [T]     or NULL, as in pard2_cat_weights.
 *   w          [T]     out.   conf [T] out or NULL (feed it to pard2_cat_fwd as conf_in).
 *   valid_len  [B]     out or NULL: existing slots per block (feed it to pard2_cat_fwd / _bwd).
 *   exp_len    [B]     out or NULL.
 */
int pard2_cat_weights_seq(const pard2_cat_desc* desc, const float* c_seq, int64_t n_pos,
                          const int32_t* anchor_pos, const int32_t* seq_end, const int32_t* y,
                          float* w, float* conf, int32_t* valid_len, float* exp_len, void* stream);

/* Forward: fused head contraction + online log-softmax + confidence + CAT weight + loss.
 *   H, W      storage type desc->dtype.
 *   y         [T]  int32 target ids.
 *   conf_in   [T]  teacher confidences (Eq.9), or NULL for the self-teacher instance in
 *                  which the head passed in also plays the teacher: c_t = q_t(y_t),
 *                  detached; ignored rows use c = 1.
 *   valid_len [B]  or NULL.
 *   loss      [1]  out, or NULL.  If loss and w are both NULL the call is "stats only"
 *                  (lse, logp_y, argmax): this is how teacher confidences
 *                  exp(logp_y) are extracted from a teacher head.
 *   lse       [T]  out: logsumexp of each row (needed by the backward).
 *   logp_y    [T]  out: log q_t(y_t) (0 on ignored rows).
 *   w         [T]  out or NULL: the CAT weight (0 on invalid slots).
 *   argmax    [T]  out or NULL: greedy prediction, lowest index on ties.
 *   accept_len[B]  out or NULL: number of leading slots whose greedy prediction equals
 *                  the target (the prefix a temperature-0 verifier would accept, Sec.2.1).
 *   exp_len   [B]  out or NULL: as in pard2_cat_weights.
 *   dev_status[1]  out or NULL: set to 0, then to 1 if any target id is out of range.
 */
int pard2_cat_fwd(const pard2_cat_desc* desc, const void* H, const void* W, const int32_t* y,
                  const float* conf_in, const int32_t* valid_len,
                  float* loss, float* lse, float* logp_y, float* w,
                  int32_t* argmax, int32_t* accept_len, float* exp_len, int32_t* dev_status,
                  void* workspace, size_t workspace_bytes, void* stream);

/* Backward of the forward's loss with the weight held constant.
 *   lse, w    [T]  as written by pard2_cat_fwd.
 *   grad_loss [1]  upstream gradient of the scalar loss, or NULL = 1.
 *   dH        [T,d] out, storage type desc->dtype; rows of invalid slots are zero.
 *   dW        [V,d] out (or += when accumulate_dW != 0), storage type desc->dtype, or fp32 when
 *                  desc->flags has PARD2_FLAG_DW_FP32.
 */
int pard2_cat_bwd(const pard2_cat_desc* desc, const void* H, const void* W, const int32_t* y,
                  const int32_t* valid_len, const float* lse, const float* w,
                  const float* grad_loss, void* dH, void* dW, int32_t accumulate_dW,
                  void* workspace, size_t workspace_bytes, void* stream);

/* ---- The full token loss of Eq.12: s_{n,k} (beta CE + KD) ------------------------------------
 *
 * Eq.12 adds a distillation term to the weighted cross-entropy without defining it.  The
 * reading built here: KD_t = KL(p_t || q_t) = sum_v p_t(v) (log p_t(v) - log q_t(v)) at
 * temperature 1, p_t = softmax of the TARGET model's head over its final hidden state for the
 * same token (teacher-forced: the distribution whose entry at the true token is the c of Eq.9),
 * q_t the draft's; the teacher receives no gradient.  Then
 *   loss = (1/N) sum_t w_t (beta (-log q_t(y_t)) + KD_t),      w = stop-gradient CAT weight,
 *   dZ[t,v] = g_t (beta (q_t(v) - 1[v = y_t]) + q_t(v) - p_t(v)),   g_t = grad_loss w_t / N.
 * Neither head's T x V logits are ever stored: each vocabulary tile of both heads is contracted
 * into registers side by side.
 *
 * The teacher (host struct, device pointers): H [T, d] hidden states gathered token-major by the
 * caller (row t = the target model's state that predicts token t), W [V, d] its LM head, both
 * of storage type desc->dtype (bf16: 16-byte aligned, d and the strides multiples of 8).  d may
 * differ from the draft's.
 */
typedef struct {
  const void* H;      /* [T, d]  row stride ldH (elements) */
  const void* W;      /* [V, d]  row stride ldW            */
  int64_t ldH, ldW;
  int32_t d;          /* teacher hidden width              */
  int32_t reserved;   /* set to 0                          */
} pard2_kd_teacher;

/* Host-only: workspace for pard2_cat_kd_fwd / _bwd (0 if the arguments are invalid). */
size_t pard2_cat_kd_workspace_bytes(const pard2_cat_desc* desc, int32_t teacher_d);

/* Forward of the Eq.12 token loss.  Arguments as pard2_cat_fwd, plus:
 *   conf_in   [T]  confidences, or NULL = the teacher head's own p_t(y_t) (Eq.9 as printed;
 *                  ignored rows use c = 1).
 *   lse_t     [T]  out: logsumexp of the teacher's rows (needed by the backward).
 *   kd        [T]  out or NULL: KL(p_t || q_t) per row.
 * If loss and kd are BOTH NULL nothing asked for needs the two heads' logits side by side, and the
 * call runs two single-head sweeps instead of the (slower per flop) two-head one: lse, lse_t, logp_y,
 * w, argmax, accept_len, exp_len as usual; the loss of the step can then be had from the backward.
 * desc->beta must be >= 0 (else PARD2_ERR_HYPER). */
int pard2_cat_kd_fwd(const pard2_cat_desc* desc, const void* H, const void* W,
                     const pard2_kd_teacher* teacher, const int32_t* y, const float* conf_in,
                     const int32_t* valid_len, float* loss, float* lse, float* lse_t, float* logp_y,
                     float* kd, float* w, int32_t* argmax, int32_t* accept_len, float* exp_len,
                     int32_t* dev_status, void* workspace, size_t workspace_bytes, void* stream);

/* Backward of pard2_cat_kd_fwd's loss into the draft's H and W (weight and teacher constant).
 *   lse, lse_t, w  [T] as written by pard2_cat_kd_fwd.   Other arguments as pard2_cat_bwd.
 *   kd        [T]  out or NULL, loss [1] out or NULL: the same values pard2_cat_kd_fwd returns,
 *                  evaluated from the logits this call recomputes anyway (the cross term of the KL
 *                  is summed per vocabulary tile and the tiles are added in a fixed order).
 *   logp_y    [T]  as written by pard2_cat_kd_fwd; needed only when loss is requested, else NULL. */
int pard2_cat_kd_bwd(const pard2_cat_desc* desc, const void* H, const void* W,
                     const pard2_kd_teacher* teacher, const int32_t* y, const int32_t* valid_len,
                     const float* lse, const float* lse_t, const float* w, const float* grad_loss,
                     void* dH, void* dW, int32_t accumulate_dW,
                     const float* logp_y, float* kd, float* loss,
                     void* workspace, size_t workspace_bytes, void* stream);

/* ---- Gated injection of target features into the draft's input embeddings (Sec.3.3) ---------
 *
 *   e'[t,:] = e[t,:] + xi_t * Proj([x_1[t,:]; ...; x_F[t,:]])
 * x_1..x_F are the target model's hidden states of F layers (the paper names low / middle / high
 * and trains with four), [.;.] concatenates along the feature axis, and xi ~ Bernoulli(1 - rho)
 * is drawn per training instance.  Reading (the paper only calls Proj "lightweight"): Proj is one
 * linear map without bias, P[d, F*dt] row-major, column block f multiplying x_f.  The gate is an
 * INPUT, xi[T] fp32, one value per token row (repeat an instance's draw over its rows; any real
 * value is accepted).  bf16 storage, fp32 accumulation; the concatenation is never formed.
 *
 *   T, d, dt, F   token rows, draft width, width of one feature, number of features (1..8);
 *                 d and dt multiples of 8.
 *   E     [T,d]   draft input embeddings, dense.      Eout [T,d] out (may alias E).
 *   feats [F]     HOST array of F device pointers, each [T,dt] with row stride ldX (elements,
 *                 a multiple of 8, >= dt); 16-byte aligned.
 *   P     [d,F*dt] dense.      xi [T] fp32.
 * Backward (the target model is frozen; the gradient of e is dEout itself):
 *   dEout [T,d]   upstream gradient.
 *   dT    [T,d]   out: xi * dEout, the gradient of the projected feature (also the kernel's
 *                 staging operand: required).
 *   dP    [d,F*dt] out (+= when accumulate_dP != 0).
 * Same pointer, stream and error conventions as above; no workspace. */
int pard2_inject_fwd(int32_t T, int32_t d, int32_t dt, int32_t F, const void* E,
                     const void* const* feats, int64_t ldX, const void* P, const float* xi,
                     void* Eout, void* stream);
int pard2_inject_bwd(int32_t T, int32_t d, int32_t dt, int32_t F, const void* dEout,
                     const void* const* feats, int64_t ldX, const float* xi, void* dT, void* dP,
                     int32_t accumulate_dP, void* stream);

/* Measurement aid (not part of the method).  pard2_cat_kernel_timing(1) makes every later
 * launch of the contraction kernels carry a pair of HIP events on its own dispatch;
 * pard2_cat_kernel_timing(0) switches it off; either call forgets earlier records.
 * pard2_cat_kernel_timing_read waits for the recorded launches of one kernel
 * (0 forward sweep, 1 dZ recompute, 2 dH, 3 dW, 4 two-head forward sweep, 5 two-head dZ,
 * 6 injection forward, 7 injection dP)
 * and returns their summed duration in milliseconds and their count.  Launches on a stream that is
 * being captured into a graph are not timed.  Host pointers.  Not
 * thread-safe against concurrent launches from other host threads. */
int pard2_cat_kernel_timing(int enable);
int pard2_cat_kernel_timing_read(int kernel, double* total_ms, int64_t* launches);

#ifdef __cplusplus
}
#endif
#endif /* PARD2_CAT_H */
