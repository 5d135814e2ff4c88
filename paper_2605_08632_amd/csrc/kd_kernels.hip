// Two-head bf16 kernels of the distillation term of Eq.12 on gfx950: for every vocabulary
// tile the teacher's logits zT = Ht . Wt^T and the draft's zD = H . W^T are contracted into two
// register accumulator sets of the same shape, so that everything that needs both at one
// (token, id) - the cross term of KL(p || q) in the forward, q - p in the backward - is formed
// in fp32 registers and neither head's T x V logits ever reach memory.
//
// Two accumulator sets halve the tile a wavefront can hold: the workgroup tile is 128 ids x
// 256 tokens (8 wavefronts of 64 x 64) instead of the single-head kernels' 256 x 256.
#include "gemm_nt_mfma.hpp"
#include "kernels.h"
#include "row_stats.hpp"

#include <limits.h>

namespace pard2 {

#ifndef PARD2_KD_TILE
#define PARD2_KD_TILE 128, 256, 2, 4
#endif
using KdCfg = TileCfg<PARD2_KD_TILE>;
// token tiles per band of the tile rasterisation
#ifndef PARD2_KD_BAND
#define PARD2_KD_BAND 8
#endif

// Teacher-side running statistics of a row over a set of ids: max, s = sum exp(zT - max) and
// a = sum exp(zT - max) (zT - zD); at the end  sum_v p(v) (zT - zD)(v) = a / s.
struct KdStat {
  float m, s, a;
};
__device__ __forceinline__ KdStat merge(KdStat x, KdStat y) {
  KdStat o;
  o.m = fmaxf(x.m, y.m);
  const float ms = (o.m == -INFINITY) ? 0.f : o.m;
  const float ex = __builtin_amdgcn_exp2f((x.m - ms) * L2E), ey = __builtin_amdgcn_exp2f((y.m - ms) * L2E);
  o.s = x.s * ex + y.s * ey;
  o.a = x.a * ex + y.a * ey;
  return o;
}

// ------------------------------------------------------------------------------------
// Forward sweep over both heads.  Work split as in the single-head sweep: a workgroup owns
// BN token rows and one of `nsplit` vocabulary ranges; a lane owns whole token rows, so all
// running statistics are lane-local until the end.  Per tile: teacher contraction (k = dt),
// then draft contraction (k = d), then one epilogue over both accumulator sets.
// ------------------------------------------------------------------------------------
template <class C>
__global__ __launch_bounds__(C::NTHREADS) void kd_stats_kernel(
    const __bf16* __restrict__ H, int64_t ldH, const __bf16* __restrict__ W, int64_t ldW,
    const __bf16* __restrict__ Ht, int64_t ldHt, const __bf16* __restrict__ Wt, int64_t ldWt,
    const int32_t* __restrict__ y, int T, int d, int dt, int V, int nTt, int nVt, int nsplit,
    float2* __restrict__ ms, int32_t* __restrict__ idx, float* __restrict__ zy, float2* __restrict__ ms_t,
    float* __restrict__ a_t, float* __restrict__ zy_t) {
  extern __shared__ __align__(16) char smem[];
  const WavePos<C> wp;
  int tt, sp;
  banded_tile(xcd_contiguous_id(blockIdx.x, gridDim.x), nTt, nsplit, PARD2_KD_BAND, tt, sp);
  const int n0 = tt * C::BN;
  const int vt_begin = (int)((int64_t)sp * nVt / nsplit), vt_end = (int)((int64_t)(sp + 1) * nVt / nsplit);

  RowStat run[C::NI];
  KdStat runT[C::NI];
  int yt[C::NI];
#pragma unroll
  for (int ni = 0; ni < C::NI; ++ni) {
    run[ni] = {-INFINITY, 0.f, INT_MAX};
    runT[ni] = {-INFINITY, 0.f, 0.f};
    const int t = n0 + wp.n_of(ni);
    yt[ni] = (t < T) ? y[t] : -1;
  }

  GemmNT<C> gT(Wt, ldWt, vt_begin * C::BM, V, dt, Ht, ldHt, n0, T, dt, smem);
  gT.prefetch();
  for (int vt = vt_begin; vt < vt_end; ++vt) {
    const int m0 = vt * C::BM;
    f32x16 accT[C::MI][C::NI], accD[C::MI][C::NI];
    zero_acc<C>(accT);
    gT.run(accT, true);
    const GemmNT<C> gD(W, ldW, m0, V, d, H, ldH, n0, T, d, smem);
    gD.prefetch();
    zero_acc<C>(accD);
    gD.run(accD, true);
    if (vt + 1 < vt_end) {   // the next tile's first loads fly under this tile's epilogue
      gT = GemmNT<C>(Wt, ldWt, m0 + C::BM, V, dt, Ht, ldHt, n0, T, dt, smem);
      gT.prefetch();
    }

    const int vw0 = m0 + wp.m_of(0, 0);
    const bool ragged = m0 + C::BM > V;
#pragma unroll
    for (int ni = 0; ni < C::NI; ++ni) {
      if (ragged) {
#pragma unroll
        for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if (m0 + wp.m_of(mi, r) >= V) {
              accD[mi][ni][r] = -INFINITY;
              accT[mi][ni][r] = -INFINITY;
            }
      }
      // both heads' logits of the target id: written by the one lane that holds (y_t, t)
      const int rel = yt[ni] - (m0 + wp.wm * C::WTM);
      if (rel >= 0 && rel < C::WTM) {
#pragma unroll
        for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if (m0 + wp.m_of(mi, r) == yt[ni]) {
              zy[n0 + wp.n_of(ni)] = accD[mi][ni][r];
              zy_t[n0 + wp.n_of(ni)] = accT[mi][ni][r];
            }
      }
      // draft: running (max, sum, argmax)
      {
        float tmax = -INFINITY;
#pragma unroll
        for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
          for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, accD[mi][ni][r]);
        if (tmax > run[ni].m) {  // strict: an earlier (lower) index keeps a tie
          int best = INT_MAX;
#pragma unroll
          for (int mi = C::MI - 1; mi >= 0; --mi)
#pragma unroll
            for (int r = 15; r >= 0; --r)
              if (accD[mi][ni][r] == tmax) best = vw0 + (wp.m_of(mi, r) - wp.m_of(0, 0));
          run[ni].idx = best;
        }
        const float mnew = fmaxf(run[ni].m, tmax);
        const float msafe = (mnew == -INFINITY) ? 0.f : mnew;
        const float nm = -msafe * L2E;
        float s = run[ni].s * __builtin_amdgcn_exp2f(__builtin_fmaf(run[ni].m, L2E, nm));
#pragma unroll
        for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
          for (int r = 0; r < 16; ++r) s += __builtin_amdgcn_exp2f(__builtin_fmaf(accD[mi][ni][r], L2E, nm));
        run[ni].m = mnew;
        run[ni].s = s;
      }
      // teacher: running (max, sum, sum of e (zT - zD))
      {
        float tmax = -INFINITY;
#pragma unroll
        for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
          for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, accT[mi][ni][r]);
        const float mnew = fmaxf(runT[ni].m, tmax);
        const float msafe = (mnew == -INFINITY) ? 0.f : mnew;
        const float nm = -msafe * L2E;
        const float resc = __builtin_amdgcn_exp2f(__builtin_fmaf(runT[ni].m, L2E, nm));
        float s = runT[ni].s * resc, a = runT[ni].a * resc;
#pragma unroll
        for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(accT[mi][ni][r], L2E, nm));
            s += e;
            // e == 0 covers ids past V (both logits -inf there: their difference is not a number)
            a += (e > 0.f) ? e * (accT[mi][ni][r] - accD[mi][ni][r]) : 0.f;
          }
        runT[ni].m = mnew;
        runT[ni].s = s;
        runT[ni].a = a;
      }
    }
  }

  // merge the two half-wavefronts (same rows, interleaved ids) ...
#pragma unroll
  for (int ni = 0; ni < C::NI; ++ni) {
    RowStat o;
    o.m = __shfl_xor(run[ni].m, 32);
    o.s = __shfl_xor(run[ni].s, 32);
    o.idx = __shfl_xor(run[ni].idx, 32);
    run[ni] = merge(run[ni], o);
    KdStat ot;
    ot.m = __shfl_xor(runT[ni].m, 32);
    ot.s = __shfl_xor(runT[ni].s, 32);
    ot.a = __shfl_xor(runT[ni].a, 32);
    runT[ni] = merge(runT[ni], ot);
  }
  // ... then the WGM wavefronts that share the rows, through LDS (free after the main loop)
  RowStat* sh = reinterpret_cast<RowStat*>(smem);                                        // [WGM][BN]
  KdStat* sht = reinterpret_cast<KdStat*>(smem + C::WGM * C::BN * sizeof(RowStat));      // [WGM][BN]
  if (wp.lane < 32) {
#pragma unroll
    for (int ni = 0; ni < C::NI; ++ni) {
      sh[wp.wm * C::BN + wp.n_of(ni)] = run[ni];
      sht[wp.wm * C::BN + wp.n_of(ni)] = runT[ni];
    }
  }
  __syncthreads();
  for (int n = threadIdx.x; n < C::BN; n += C::NTHREADS) {
    RowStat a = sh[n];
    KdStat b = sht[n];
    for (int w = 1; w < C::WGM; ++w) {
      a = merge(a, sh[w * C::BN + n]);
      b = merge(b, sht[w * C::BN + n]);
    }
    const int t = n0 + n;
    if (t < T) {
      ms[(int64_t)t * nsplit + sp] = make_float2(a.m, a.s);
      idx[(int64_t)t * nsplit + sp] = a.idx;
      ms_t[(int64_t)t * nsplit + sp] = make_float2(b.m, b.s);
      a_t[(int64_t)t * nsplit + sp] = b.a;
    }
  }
}

// ------------------------------------------------------------------------------------
// Backward step 1 with the distillation term, for one vocabulary chunk: recompute both
// heads' logits tile and form, in fp32 before the single rounding to bf16,
//   dZ[t,v] = g_t ((1 + beta) q_t(v) - p_t(v) - beta 1[v = y_t])
// (= g_t (beta (q - 1[v = y_t]) + q - p): gradient of beta CE + KL(p || q) with respect to the
// draft's logits, weight and teacher constant).  Written as dZ[t][v - chunk start] through an
// LDS tile so that every global store is a full 256-byte row segment.  A tile that lies
// entirely past V inside the chunk's padded width writes zeros.
// ------------------------------------------------------------------------------------
template <class C>
constexpr int kd_dz_pitch() {   // LDS bytes per staged row of BM bf16: 16-byte aligned, rows shift by 4 banks
  return C::BM * 2 + 16;
}
template <class C>
constexpr int kd_dz_lds_bytes() {
  return C::LDS_BYTES > C::BN * kd_dz_pitch<C>() ? C::LDS_BYTES : C::BN * kd_dz_pitch<C>();
}

template <class C>
__global__ __launch_bounds__(C::NTHREADS) void kd_dz_kernel(
    const __bf16* __restrict__ H, int64_t ldH, const __bf16* __restrict__ W, int64_t ldW,
    const __bf16* __restrict__ Ht, int64_t ldHt, const __bf16* __restrict__ Wt, int64_t ldWt,
    const int32_t* __restrict__ y, const float* __restrict__ lse, const float* __restrict__ lse_t,
    const float* __restrict__ g, float beta, int T, int d, int dt, int V, int nTt, int vt0, int nVtc,
    __bf16* __restrict__ dZ, int64_t ldz, float* __restrict__ kd_part) {
  extern __shared__ __align__(16) char smem[];
  constexpr int KD_DZ_PITCH = kd_dz_pitch<C>();
  static_assert(C::BN * KD_DZ_PITCH + C::WGM * C::BN * 4 <= kd_dz_lds_bytes<C>(), "row sums sit behind the staged tile");
  float* sh_a = reinterpret_cast<float*>(smem + C::BN * KD_DZ_PITCH);   // [WGM][BN] per-row sums of the tile
  const WavePos<C> wp;
  int tt, vtl;
  banded_tile(xcd_contiguous_id(blockIdx.x, gridDim.x), nTt, nVtc, PARD2_KD_BAND, tt, vtl);
  const int n0 = tt * C::BN, m0 = (vt0 + vtl) * C::BM, c0 = vtl * C::BM;
  const bool live = m0 < V;   // workgroup-uniform

  if (live) {
    f32x16 accT[C::MI][C::NI], accD[C::MI][C::NI];
    zero_acc<C>(accT);
    GemmNT<C>(Wt, ldWt, m0, V, dt, Ht, ldHt, n0, T, dt, smem).run(accT);
    const GemmNT<C> gD(W, ldW, m0, V, d, H, ldH, n0, T, d, smem);
    gD.prefetch();
    zero_acc<C>(accD);
    gD.run(accD, true);

    const bool ragged = m0 + C::BM > V;
#pragma unroll
    for (int ni = 0; ni < C::NI; ++ni) {
      const int tl = wp.n_of(ni);
      const int t = n0 + tl;
      const bool row = t < T;
      const float gt = row ? g[t] : 0.f;
      const float nlD = row ? -lse[t] * L2E : -INFINITY;     // rows past T: q = p = 0
      const float nlT = row ? -lse_t[t] * L2E : -INFINITY;
      const int yv = row ? y[t] : -1;
      const float gq = gt * (1.f + beta), gy = gt * beta;
      float arow = 0.f;
      if (ragged) {
#pragma unroll
        for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if (m0 + wp.m_of(mi, r) >= V) {   // ids past V: q = p = 0
              accD[mi][ni][r] = -INFINITY;
              accT[mi][ni][r] = -INFINITY;
            }
      }
#pragma unroll
      for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
          bf16x4 pk;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const float q = __builtin_amdgcn_exp2f(__builtin_fmaf(accD[mi][ni][rq * 4 + j], L2E, nlD));
            const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(accT[mi][ni][rq * 4 + j], L2E, nlT));
            pk[j] = (__bf16)(gq * q - gt * p);
            // cross term of KL(p || q): p (zT - zD); p == 0 covers ids past V and rows past T
            if (kd_part) arow += (p > 0.f) ? p * (accT[mi][ni][rq * 4 + j] - accD[mi][ni][rq * 4 + j]) : 0.f;
          }
          *reinterpret_cast<bf16x4*>(smem + tl * KD_DZ_PITCH + wp.m_of(mi, rq * 4) * 2) = pk;
        }
      if (kd_part) {   // the two half-wavefronts hold interleaved ids of the same rows
        arow += __shfl_xor(arow, 32);
        if (wp.lane < 32) sh_a[wp.wm * C::BN + tl] = arow;
      }
      // the target element carries the extra -beta g
      const int rel = yv - (m0 + wp.wm * C::WTM);
      if (rel >= 0 && rel < C::WTM) {
#pragma unroll
        for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if (m0 + wp.m_of(mi, r) == yv) {
              const float q = __builtin_amdgcn_exp2f(__builtin_fmaf(accD[mi][ni][r], L2E, nlD));
              const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(accT[mi][ni][r], L2E, nlT));
              *reinterpret_cast<__bf16*>(smem + tl * KD_DZ_PITCH + wp.m_of(mi, r) * 2) =
                  (__bf16)(gq * q - gt * p - gy);
            }
      }
    }
  }
  __syncthreads();
  // LDS -> global: BM / 8 lanes x 16 bytes cover one row of the tile
  constexpr int LANES_PER_ROW = C::BM / 8;
  constexpr int ROWS_PER_PASS = C::NTHREADS / LANES_PER_ROW;
  const int chunk = threadIdx.x % LANES_PER_ROW, r0 = threadIdx.x / LANES_PER_ROW;
#pragma unroll 4
  for (int r = r0; r < C::BN; r += ROWS_PER_PASS) {
    const int t = n0 + r;
    if (t < T) {
      u32x4 v = {0u, 0u, 0u, 0u};
      if (live) v = *reinterpret_cast<const u32x4*>(smem + r * KD_DZ_PITCH + chunk * 16);
      __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(dZ + (int64_t)t * ldz + c0 + chunk * 8));   // streamed out
    }
  }
  // per-row sum_v p (zT - zD) over this tile's ids -> kd_part[tile][t] (tiles past V write nothing)
  if (kd_part && live) {
    for (int n = threadIdx.x; n < C::BN; n += C::NTHREADS) {
      float a = sh_a[n];
      for (int w = 1; w < C::WGM; ++w) a += sh_a[w * C::BN + n];
      if (n0 + n < T) kd_part[(int64_t)(vt0 + vtl) * T + n0 + n] = a;
    }
  }
}

// ------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------
static int ceil_div(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

template <class K>
static hipError_t allow_lds(K kernel, int bytes) {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                             bytes);
}

int kd_num_row_parts_bf16(int V) { return ceil_div(V, KdCfg::BM); }

int kd_num_partials_bf16(int T, int V) {
  const int nTt = ceil_div(T, KdCfg::BN), nVt = ceil_div(V, KdCfg::BM);
  int ns = ceil_div(256, nTt);
  ns = ns < 1 ? 1 : ns;
  return ns > nVt ? nVt : ns;
}

hipError_t launch_kd_stats_bf16(const void* H, int64_t ldH, const void* W, int64_t ldW, const KdTeacher& te,
                                const int32_t* y, int T, int d, int V, KdStatsOut out, hipStream_t s) {
  const int nTt = ceil_div(T, KdCfg::BN), nVt = ceil_div(V, KdCfg::BM), ns = out.draft.P;
  auto k = kd_stats_kernel<KdCfg>;
  hipError_t e = allow_lds(k, KdCfg::LDS_BYTES);
  if (e != hipSuccess) return e;
  launch_timed(KT_KD_STATS, k, dim3(nTt * ns), dim3(KdCfg::NTHREADS), KdCfg::LDS_BYTES, s, (const __bf16*)H, ldH,
               (const __bf16*)W, ldW, (const __bf16*)te.H, te.ldH, (const __bf16*)te.W, te.ldW, y, T, d, te.d,
               V, nTt, nVt, ns, out.draft.ms, out.draft.idx, out.draft.zy, out.ms_t, out.a_t, out.zy_t);
  return hipGetLastError();
}

hipError_t launch_kd_dz_bf16(const void* H, int64_t ldH, const void* W, int64_t ldW, const KdTeacher& te,
                             const int32_t* y, const float* lse, const float* g, int T, int d, int V, int v0, int Kc,
                             void* dZ, int64_t ldz, float* kd_part, hipStream_t s) {
  if (v0 % KdCfg::BM != 0 || Kc % KdCfg::BM != 0 || v0 >= V) return hipErrorInvalidValue;
  constexpr int LDS = kd_dz_lds_bytes<KdCfg>();
  auto k = kd_dz_kernel<KdCfg>;
  hipError_t e = allow_lds(k, LDS);
  if (e != hipSuccess) return e;
  const int nTt = ceil_div(T, KdCfg::BN), nVtc = Kc / KdCfg::BM;
  launch_timed(KT_KD_DZ, k, dim3(nTt * nVtc), dim3(KdCfg::NTHREADS), LDS, s, (const __bf16*)H, ldH, (const __bf16*)W, ldW,
               (const __bf16*)te.H, te.ldH, (const __bf16*)te.W, te.ldW, y, lse, te.lse, g, te.beta, T, d, te.d,
               V, nTt, v0 / KdCfg::BM, nVtc, (__bf16*)dZ, ldz, kd_part);
  return hipGetLastError();
}

}  // namespace pard2
