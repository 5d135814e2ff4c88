// Gated injection of target-model features into the draft's input embeddings (Sec.3.3):
//   e'[t,:] = e[t,:] + xi_t * Proj([x_1[t,:]; ...; x_F[t,:]]),   Proj = one linear map P[d, F*dt].
// The concatenation is never formed: the contraction walks the F feature tensors as F segments
// of its k range.  Backward: dT = xi * de' (the projected feature's gradient) and
// dP = dT^T . [x_1; ...; x_F], one contraction per feature with both operands read as they lie
// in memory (k = token row, k-major panels).  bf16 storage, fp32 accumulation, MFMA main loop
// shared with the loss kernels.
#include "gemm_nt_mfma.hpp"
#include "kernels.h"

namespace pard2 {

using ICfg = TileCfg<256, 256, 2, 4>;

// Forward.  M side = output feature i (rows of P, k-contiguous), N side = token t (rows of x_f).
template <class C>
__global__ __launch_bounds__(C::NTHREADS) void inject_fwd_kernel(const __bf16* E, InjectFeats feats, int64_t ldX,
                                                                 const __bf16* __restrict__ P,
                                                                 const float* __restrict__ xi, int T, int d, int dt,
                                                                 int F, int nIt, int nTt, __bf16* Eout) {
  // E and Eout may be the same buffer: every element is read and written by the same lane
  extern __shared__ __align__(16) char smem[];
  const WavePos<C> wp;
  int it, tt;
  banded_tile(xcd_contiguous_id(blockIdx.x, gridDim.x), nIt, nTt, 8, it, tt);
  const int m0 = it * C::BM, n0 = tt * C::BN;
  const int64_t ldP = (int64_t)F * dt;

  f32x16 acc[C::MI][C::NI];
  zero_acc<C>(acc);
  for (int f = 0; f < F; ++f)
    GemmNT<C>(P + (int64_t)f * dt, ldP, m0, d, dt, (const __bf16*)feats.p[f], ldX, n0, T, dt, smem).run(acc);

#pragma unroll
  for (int ni = 0; ni < C::NI; ++ni) {
    const int t = n0 + wp.n_of(ni);
    if (t >= T) continue;
    const float x = xi[t];
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        const int i = m0 + wp.m_of(mi, rq * 4);
        if (i >= d) continue;
        const bf16x4 e = *reinterpret_cast<const bf16x4*>(E + (int64_t)t * d + i);
        bf16x4 o;
#pragma unroll
        for (int j = 0; j < 4; ++j) o[j] = (__bf16)__builtin_fmaf(x, acc[mi][ni][rq * 4 + j], (float)e[j]);
        *reinterpret_cast<bf16x4*>(Eout + (int64_t)t * d + i) = o;
      }
  }
}

// dT[t,i] = xi_t * dEout[t,i], eight elements per thread (d is a multiple of 8).
__global__ __launch_bounds__(256) void inject_gate_kernel(const __bf16* __restrict__ dEout,
                                                          const float* __restrict__ xi, int64_t n8, int d8,
                                                          __bf16* __restrict__ dT) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n8) return;
  const float x = xi[i / d8];
  const bf16x8 v = reinterpret_cast<const bf16x8*>(dEout)[i];
  bf16x8 o;
#pragma unroll
  for (int j = 0; j < 8; ++j) o[j] = (__bf16)(x * (float)v[j]);
  reinterpret_cast<bf16x8*>(dT)[i] = o;
}

// dP[i, f*dt + c] (+)= sum_t dT[t,i] * x_f[t,c].  M side = feature column c (A = x_f, k-major),
// N side = output feature i (B = dT, k-major): a lane then holds four consecutive c of one row i
// of dP, an 8-byte store.
template <class C>
__global__ __launch_bounds__(C::NTHREADS) void inject_dp_kernel(InjectFeats feats, int64_t ldX,
                                                                const __bf16* __restrict__ dT, int T, int d, int dt,
                                                                int F, int nCt, int nIt, __bf16* __restrict__ dP,
                                                                int accumulate) {
  extern __shared__ __align__(16) char smem[];
  const WavePos<C> wp;
  const int id = xcd_contiguous_id(blockIdx.x, gridDim.x);
  const int per = nCt * nIt;
  const int f = id / per;
  int ct, it;
  banded_tile(id - f * per, nCt, nIt, 8, ct, it);
  const int m0 = ct * C::BM, n0 = it * C::BN;
  const int64_t ldP = (int64_t)F * dt;

  f32x16 acc[C::MI][C::NI];
  zero_acc<C>(acc);
  GemmNT<C, true, true>((const __bf16*)feats.p[f], ldX, m0, dt, T, dT, d, n0, d, T, smem).run(acc);

#pragma unroll
  for (int ni = 0; ni < C::NI; ++ni) {
    const int i = n0 + wp.n_of(ni);
    if (i >= d) continue;
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        const int c = m0 + wp.m_of(mi, rq * 4);
        if (c >= dt) continue;
        bf16x4* p = reinterpret_cast<bf16x4*>(dP + (int64_t)i * ldP + (int64_t)f * dt + c);
        f32x4 v = {acc[mi][ni][rq * 4], acc[mi][ni][rq * 4 + 1], acc[mi][ni][rq * 4 + 2], acc[mi][ni][rq * 4 + 3]};
        if (accumulate) {
          const bf16x4 old = *p;
          v[0] += (float)old[0]; v[1] += (float)old[1]; v[2] += (float)old[2]; v[3] += (float)old[3];
        }
        bf16x4 o = {(__bf16)v[0], (__bf16)v[1], (__bf16)v[2], (__bf16)v[3]};
        *p = o;
      }
  }
}

static int ceil_div(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

template <class K>
static hipError_t allow_lds(K kernel, int bytes) {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                             bytes);
}

hipError_t launch_inject_fwd(const void* E, const InjectFeats& feats, int64_t ldX, const void* P, const float* xi,
                             int T, int d, int dt, int F, void* Eout, hipStream_t s) {
  auto k = inject_fwd_kernel<ICfg>;
  hipError_t e = allow_lds(k, ICfg::LDS_BYTES);
  if (e != hipSuccess) return e;
  const int nIt = ceil_div(d, ICfg::BM), nTt = ceil_div(T, ICfg::BN);
  launch_timed(KT_INJECT_FWD, k, dim3(nIt * nTt), dim3(ICfg::NTHREADS), ICfg::LDS_BYTES, s, (const __bf16*)E, feats, ldX,
               (const __bf16*)P, xi, T, d, dt, F, nIt, nTt, (__bf16*)Eout);
  return hipGetLastError();
}

hipError_t launch_inject_bwd(const void* dEout, const InjectFeats& feats, int64_t ldX, const float* xi, int T, int d,
                             int dt, int F, void* dT, void* dP, int accumulate, hipStream_t s) {
  auto k = inject_dp_kernel<ICfg>;
  hipError_t e = allow_lds(k, ICfg::LDS_BYTES);
  if (e != hipSuccess) return e;
  const int64_t n8 = (int64_t)T * d / 8;
  hipLaunchKernelGGL(inject_gate_kernel, dim3((unsigned)((n8 + 255) / 256)), dim3(256), 0, s, (const __bf16*)dEout, xi,
                     n8, d / 8, (__bf16*)dT);
  const int nCt = ceil_div(dt, ICfg::BM), nIt = ceil_div(d, ICfg::BN);
  launch_timed(KT_INJECT_DP, k, dim3(nCt * nIt * F), dim3(ICfg::NTHREADS), ICfg::LDS_BYTES, s, feats, ldX, (const __bf16*)dT, T,
               d, dt, F, nCt, nIt, (__bf16*)dP, accumulate);
  return hipGetLastError();
}

}  // namespace pard2
