// fp32-storage path of the CAT loss (small / verification workloads): the same steps
// as the bf16 path with plain fp32 FMA contractions, so that results track the fp64
// definition to ~1e-6.  One LDS-tiled kernel serves all four contractions through
// element strides and an epilogue functor.
#include "kernels.h"

#include <limits.h>

namespace pard2 {

constexpr int FT = 64;   // output tile edge
constexpr int FK = 16;   // contraction step

// C[m][n] = sum_k A[m*sam + k*sak] * B[n*sbn + k*sbk]; 256 threads, 4x4 outputs each.
// After the k loop the tile is parked in LDS and handed to the epilogue.
template <class Epi>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ A, int64_t sam, int64_t sak,
                                                       const float* __restrict__ B, int64_t sbn, int64_t sbk, int M,
                                                       int N, int Kd, Epi epi) {
  __shared__ float As[FK][FT + 1];
  __shared__ float Bs[FK][FT + 1];
  __shared__ float Cs[FT][FT + 1];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int m0 = blockIdx.x * FT, n0 = blockIdx.y * FT;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < Kd; k0 += FK) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int e = tid + j * 256, r = e / FK, kk = e % FK;
      const int m = m0 + r, n = n0 + r, k = k0 + kk;
      As[kk][r] = (m < M && k < Kd) ? A[(int64_t)m * sam + (int64_t)k * sak] : 0.f;
      Bs[kk][r] = (n < N && k < Kd) ? B[(int64_t)n * sbn + (int64_t)k * sbk] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < FK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) Cs[ty * 4 + i][tx * 4 + j] = acc[i][j];
  __syncthreads();
  epi(m0, n0, M, N, Cs);
}

// Forward: m = token row, n = vocabulary id.  Per row of the tile: (max, sumexp, argmax)
// over the tile's 64 ids -> one partial per (row, column tile); target logit capture.
struct StatsEpi {
  const int32_t* y;
  float2* ms;
  int32_t* idx;
  float* zy;
  int P;
  __device__ void operator()(int m0, int n0, int M, int N, float (*Cs)[FT + 1]) const {
    const int r = threadIdx.x;
    if (r >= FT || m0 + r >= M) return;
    const int t = m0 + r;
    float m = -INFINITY;
    int am = INT_MAX;
    const int ncol = min(FT, N - n0);
    for (int j = 0; j < ncol; ++j)
      if (Cs[r][j] > m) {
        m = Cs[r][j];
        am = n0 + j;
      }
    float s = 0.f;
    for (int j = 0; j < ncol; ++j) s += expf(Cs[r][j] - m);
    ms[(int64_t)t * P + blockIdx.y] = make_float2(m, s);
    idx[(int64_t)t * P + blockIdx.y] = am;
    const int yv = y[t];
    if (yv >= n0 && yv < n0 + ncol) zy[t] = Cs[r][yv - n0];
  }
};

// Backward step 1: dZ[t][v - v0] = g_t (exp(z - lse_t) - 1[v = y_t]).
struct DzEpi {
  const int32_t* y;
  const float* lse;
  const float* g;
  float* dZ;
  int64_t ldz;
  int v0;
  __device__ void operator()(int m0, int n0, int M, int N, float (*Cs)[FT + 1]) const {
    for (int e = threadIdx.x; e < FT * FT; e += 256) {
      const int r = e / FT, j = e % FT;
      const int t = m0 + r, c = n0 + j;
      if (t >= M || c >= N) continue;
      const float q = expf(Cs[r][j] - lse[t]);
      dZ[(int64_t)t * ldz + c] = g[t] * (q - ((v0 + c == y[t]) ? 1.f : 0.f));
    }
  }
};

// Plain store / accumulate into a dense row-major output.
struct StoreEpi {
  float* C;
  int64_t ldc;
  int add;
  __device__ void operator()(int m0, int n0, int M, int N, float (*Cs)[FT + 1]) const {
    for (int e = threadIdx.x; e < FT * FT; e += 256) {
      const int r = e / FT, j = e % FT;
      const int m = m0 + r, n = n0 + j;
      if (m >= M || n >= N) continue;
      float* p = C + (int64_t)m * ldc + n;
      *p = add ? *p + Cs[r][j] : Cs[r][j];
    }
  }
};

// Two contractions over the same output tile, C1 = A1 B1^T (k extent K1) and C2 = A2 B2^T (K2), both
// k-contiguous row-major operands; the two tiles are parked in LDS and handed to the epilogue together.
// Serves the distillation term of Eq.12: tile 1 = teacher logits, tile 2 = draft logits.
template <class Epi>
__global__ __launch_bounds__(256) void gemm2_f32_kernel(const float* __restrict__ A1, int64_t lda1,
                                                        const float* __restrict__ B1, int64_t ldb1, int K1,
                                                        const float* __restrict__ A2, int64_t lda2,
                                                        const float* __restrict__ B2, int64_t ldb2, int K2, int M,
                                                        int N, Epi epi) {
  __shared__ float As[FK][FT + 1];
  __shared__ float Bs[FK][FT + 1];
  __shared__ float Cs[2][FT][FT + 1];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int m0 = blockIdx.x * FT, n0 = blockIdx.y * FT;
  for (int which = 0; which < 2; ++which) {
    const float* A = which ? A2 : A1;
    const float* B = which ? B2 : B1;
    const int64_t lda = which ? lda2 : lda1, ldb = which ? ldb2 : ldb1;
    const int Kd = which ? K2 : K1;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < Kd; k0 += FK) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int e = tid + j * 256, r = e / FK, kk = e % FK;
        const int m = m0 + r, n = n0 + r, k = k0 + kk;
        As[kk][r] = (m < M && k < Kd) ? A[(int64_t)m * lda + k] : 0.f;
        Bs[kk][r] = (n < N && k < Kd) ? B[(int64_t)n * ldb + k] : 0.f;
      }
      __syncthreads();
#pragma unroll
      for (int kk = 0; kk < FK; ++kk) {
        float a[4], b[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
        for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_fmaf(a[i], b[j], acc[i][j]);
      }
      __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) Cs[which][ty * 4 + i][tx * 4 + j] = acc[i][j];
  }
  __syncthreads();
  epi(m0, n0, M, N, Cs[0], Cs[1]);
}

// Two-head forward: m = token row, n = vocabulary id; ZT = teacher tile, ZD = draft tile.  Per row: the
// draft's (max, sumexp, argmax) and the teacher's (max, sumexp, sum e (zT - zD)) over the tile's ids.
struct KdStatsEpi {
  const int32_t* y;
  float2* ms;
  int32_t* idx;
  float* zy;
  float2* ms_t;
  float* a_t;
  float* zy_t;
  int P;
  __device__ void operator()(int m0, int n0, int M, int N, float (*ZT)[FT + 1], float (*ZD)[FT + 1]) const {
    const int r = threadIdx.x;
    if (r >= FT || m0 + r >= M) return;
    const int t = m0 + r;
    float m = -INFINITY, mt = -INFINITY;
    int am = INT_MAX;
    const int ncol = min(FT, N - n0);
    for (int j = 0; j < ncol; ++j) {
      if (ZD[r][j] > m) {
        m = ZD[r][j];
        am = n0 + j;
      }
      mt = fmaxf(mt, ZT[r][j]);
    }
    float s = 0.f, st = 0.f, at = 0.f;
    for (int j = 0; j < ncol; ++j) {
      s += expf(ZD[r][j] - m);
      const float e = expf(ZT[r][j] - mt);
      st += e;
      at += e * (ZT[r][j] - ZD[r][j]);
    }
    const int64_t o = (int64_t)t * P + blockIdx.y;
    ms[o] = make_float2(m, s);
    idx[o] = am;
    ms_t[o] = make_float2(mt, st);
    a_t[o] = at;
    const int yv = y[t];
    if (yv >= n0 && yv < n0 + ncol) {
      zy[t] = ZD[r][yv - n0];
      zy_t[t] = ZT[r][yv - n0];
    }
  }
};

// Two-head backward step 1: dZ[t][v - v0] = g_t ((1 + beta) q - p - beta 1[v = y_t]).
struct KdDzEpi {
  const int32_t* y;
  const float* lse;
  const float* lse_t;
  const float* g;
  float beta;
  float* dZ;
  int64_t ldz;
  int v0;
  float* kd_part;   // or null: [vocabulary tile][T] per-row sums of p (zT - zD)
  __device__ void operator()(int m0, int n0, int M, int N, float (*ZT)[FT + 1], float (*ZD)[FT + 1]) const {
    if (kd_part && threadIdx.x < FT && m0 + (int)threadIdx.x < M) {
      const int r = threadIdx.x, t = m0 + r;
      const int ncol = min(FT, N - n0);
      float a = 0.f;
      for (int j = 0; j < ncol; ++j) a += expf(ZT[r][j] - lse_t[t]) * (ZT[r][j] - ZD[r][j]);
      kd_part[(int64_t)(v0 / FT + blockIdx.y) * M + t] = a;
    }
    for (int e = threadIdx.x; e < FT * FT; e += 256) {
      const int r = e / FT, j = e % FT;
      const int t = m0 + r, c = n0 + j;
      if (t >= M || c >= N) continue;
      const float q = expf(ZD[r][j] - lse[t]), p = expf(ZT[r][j] - lse_t[t]);
      dZ[(int64_t)t * ldz + c] = g[t] * ((1.f + beta) * q - p - ((v0 + c == y[t]) ? beta : 0.f));
    }
  }
};

static int cdiv(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

int kd_num_row_parts_f32(int V) { return cdiv(V, FT); }

int fwd_num_partials_f32(int T, int V) {
  (void)T;
  return cdiv(V, FT);
}

hipError_t launch_fwd_stats_f32(const void* H, int64_t ldH, const void* W, int64_t ldW, const int32_t* y, int T,
                                int d, int V, StatsOut out, hipStream_t s) {
  StatsEpi epi{y, out.ms, out.idx, out.zy, out.P};
  hipLaunchKernelGGL(gemm_f32_kernel<StatsEpi>, dim3(cdiv(T, FT), cdiv(V, FT)), dim3(256), 0, s, (const float*)H, ldH,
                     (int64_t)1, (const float*)W, ldW, (int64_t)1, T, V, d, epi);
  return hipGetLastError();
}

hipError_t launch_kd_stats_f32(const void* H, int64_t ldH, const void* W, int64_t ldW, const KdTeacher& te,
                               const int32_t* y, int T, int d, int V, KdStatsOut out, hipStream_t s) {
  KdStatsEpi epi{y, out.draft.ms, out.draft.idx, out.draft.zy, out.ms_t, out.a_t, out.zy_t, out.draft.P};
  hipLaunchKernelGGL(gemm2_f32_kernel<KdStatsEpi>, dim3(cdiv(T, FT), cdiv(V, FT)), dim3(256), 0, s,
                     (const float*)te.H, te.ldH, (const float*)te.W, te.ldW, te.d, (const float*)H, ldH,
                     (const float*)W, ldW, d, T, V, epi);
  return hipGetLastError();
}

BwdPlanF32 plan_bwd_f32(int T, int d, int V) {
  (void)d;
  BwdPlanF32 p{};
  const int64_t maxc = 4096;
  p.nchunks = cdiv(V, maxc);
  p.Vc = round_up(cdiv(V, p.nchunks), FT);
  p.nchunks = cdiv(V, p.Vc);
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o += (bytes + 255) / 256 * 256; return at; };
  p.off_g = take((size_t)T * 4);
  p.off_dZ = take((size_t)T * p.Vc * 4);
  p.total = o;
  return p;
}

hipError_t launch_bwd_f32(const BwdPlanF32& p, const void* H_, int64_t ldH, const void* W_, int64_t ldW,
                          const int32_t* y, const float* lse, const float* g, int T, int d, int V, void* dH_,
                          void* dW_, int accumulate_dW, char* ws, hipStream_t s, const KdTeacher* kd) {
  const float* H = (const float*)H_;
  const float* W = (const float*)W_;
  float* dH = (float*)dH_;
  float* dW = (float*)dW_;
  float* dZ = (float*)(ws + p.off_dZ);
  for (int c = 0; c < p.nchunks; ++c) {
    const int v0 = (int)(c * p.Vc);
    const int nc = (int)((V - v0 < p.Vc) ? V - v0 : p.Vc);
    // dZ chunk [T][nc]: z = H W[v0..]^T
    if (kd) {
      KdDzEpi dz{y, lse, kd->lse, g, kd->beta, dZ, p.Vc, v0, kd->kd_part};
      hipLaunchKernelGGL(gemm2_f32_kernel<KdDzEpi>, dim3(cdiv(T, FT), cdiv(nc, FT)), dim3(256), 0, s,
                         (const float*)kd->H, kd->ldH, (const float*)kd->W + (int64_t)v0 * kd->ldW, kd->ldW, kd->d, H,
                         ldH, W + (int64_t)v0 * ldW, ldW, d, T, nc, dz);
    } else {
      DzEpi dz{y, lse, g, dZ, p.Vc, v0};
      hipLaunchKernelGGL(gemm_f32_kernel<DzEpi>, dim3(cdiv(T, FT), cdiv(nc, FT)), dim3(256), 0, s, H, ldH,
                         (int64_t)1, W + (int64_t)v0 * ldW, ldW, (int64_t)1, T, nc, d, dz);
    }
    // dH[t][i] (+)= sum_v dZ[t][v] W[v0+v][i]
    StoreEpi sh{dH, d, c > 0};
    hipLaunchKernelGGL(gemm_f32_kernel<StoreEpi>, dim3(cdiv(T, FT), cdiv(d, FT)), dim3(256), 0, s, dZ, p.Vc,
                       (int64_t)1, W + (int64_t)v0 * ldW, (int64_t)1, ldW, T, d, nc, sh);
    // dW[v0+v][i] = sum_t dZ[t][v] H[t][i]
    StoreEpi sw{dW + (int64_t)v0 * d, d, accumulate_dW};
    hipLaunchKernelGGL(gemm_f32_kernel<StoreEpi>, dim3(cdiv(nc, FT), cdiv(d, FT)), dim3(256), 0, s, dZ, (int64_t)1,
                       p.Vc, H, (int64_t)1, ldH, nc, d, T, sw);
  }
  return hipGetLastError();
}

}  // namespace pard2
