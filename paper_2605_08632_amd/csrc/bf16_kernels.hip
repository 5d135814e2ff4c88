// bf16 kernels of the CAT loss on gfx950: the vocabulary-head sweep with online
// log-softmax statistics (forward), and the split-V backward (recompute + dZ, dH, dW).
// H, W and dZ are consumed exactly as they lie in memory (k-contiguous or k-major MFMA
// operand panels): the backward makes no transposed copies.
// All four contractions run on the matrix cores through GemmNT (gemm_nt_mfma.hpp).
#include "gemm_nt_mfma.hpp"
#include "kernels.h"
#include "row_stats.hpp"

#include <limits.h>

#include <utility>

namespace pard2 {

// Tile shape used by every bf16 contraction here.
#ifndef PARD2_TILE
#define PARD2_TILE 256, 256, 2, 4
#endif
using Cfg = TileCfg<PARD2_TILE>;
// token tiles per band of the tile rasterisation (how many token tiles share a vocabulary tile inside an XCD)
// vocabulary tiles (of 256 ids) per chunk of the split-V backward
#ifndef PARD2_CHUNK_TILES
#define PARD2_CHUNK_TILES 64
#endif
// workgroups the forward sweep aims for (token tiles x vocabulary ranges)
#ifndef PARD2_FWD_WGS
#define PARD2_FWD_WGS 256
#endif
#ifndef PARD2_BAND_FWD
#define PARD2_BAND_FWD 8
#endif
#ifndef PARD2_BAND_DZ
#define PARD2_BAND_DZ 8
#endif

// Measurement aid, compiled in only with -DPARD2_CLOCK_PROBE: one wavefront of workgroup 0 prints the
// shader clock its kernel ran at (cycle counter over the constant-rate wall counter).  The matrix cores
// are power-limited: the clock a kernel sustains depends on what it keeps busy and on the data.
#ifdef PARD2_CLOCK_PROBE
#define PARD2_PROBE_BEGIN const long long probe_c0 = clock64(), probe_w0 = wall_clock64();
#define PARD2_PROBE_END(name)                                                                      \
  if (blockIdx.x == 0 && threadIdx.x == 0)                                                         \
    printf("clock probe %s: %lld cycles / %lld wall ticks\n", name, (long long)(clock64() - probe_c0), \
           (long long)(wall_clock64() - probe_w0));
#else
#define PARD2_PROBE_BEGIN
#define PARD2_PROBE_END(name)
#endif

// ------------------------------------------------------------------------------------
// Forward sweep (head contraction of Eq.4/5 + online log-softmax of the log P in Eq.11).
// A workgroup owns BN token rows and one of `nsplit` vocabulary ranges; it walks the
// range tile by tile (BM vocabulary rows each), and after each tile folds the BM x BN
// logits held in registers into per-row running (max, sum, argmax).  The vocabulary is
// on the MFMA M side, so a lane owns whole token rows: the running statistics are
// lane-local and are merged across lanes / wavefronts only once, at the end.
// ------------------------------------------------------------------------------------
template <class C>
__global__ __launch_bounds__(C::NTHREADS) void fwd_stats_kernel(const __bf16* __restrict__ H, int64_t ldH,
                                                                const __bf16* __restrict__ W, int64_t ldW,
                                                                const int32_t* __restrict__ y, int T, int d, int V,
                                                                int nTt, int nVt, int nsplit, float2* __restrict__ ms,
                                                                int32_t* __restrict__ idx, float* __restrict__ zy) {
  extern __shared__ __align__(16) char smem[];
  PARD2_PROBE_BEGIN
  const WavePos<C> wp;
  int tt, sp;
  banded_tile(xcd_contiguous_id(blockIdx.x, gridDim.x), nTt, nsplit, PARD2_BAND_FWD, tt, sp);
  const int n0 = tt * C::BN;
  const int vt_begin = (int)((int64_t)sp * nVt / nsplit), vt_end = (int)((int64_t)(sp + 1) * nVt / nsplit);

  RowStat run[C::NI];
  int yt[C::NI];
#pragma unroll
  for (int ni = 0; ni < C::NI; ++ni) {
    run[ni] = {-INFINITY, 0.f, INT_MAX};
    const int t = n0 + wp.n_of(ni);
    yt[ni] = (t < T) ? y[t] : -1;
  }

  GemmNT<C> gemm(W, ldW, vt_begin * C::BM, V, d, H, ldH, n0, T, d, smem);
  gemm.prefetch();
  for (int vt = vt_begin; vt < vt_end; ++vt) {
    const int m0 = vt * C::BM;
    f32x16 acc[C::MI][C::NI];
    zero_acc<C>(acc);
    gemm.run(acc, true);
    if (vt + 1 < vt_end) {   // the next tile's first loads fly under this tile's epilogue
      gemm = GemmNT<C>(W, ldW, m0 + C::BM, V, d, H, ldH, n0, T, d, smem);
      gemm.prefetch();
    }

    const int vw0 = m0 + wp.m_of(0, 0);            // lowest vocabulary id this lane holds in the tile
    const bool ragged = m0 + C::BM > V;
#pragma unroll
    for (int ni = 0; ni < C::NI; ++ni) {
      if (ragged) {
#pragma unroll
        for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if (m0 + wp.m_of(mi, r) >= V) acc[mi][ni][r] = -INFINITY;
      }
      // target logit: the lane that holds (v = y_t, t) writes it (exactly one lane in the grid)
      const int rel = yt[ni] - (m0 + wp.wm * C::WTM);
      if (rel >= 0 && rel < C::WTM) {
#pragma unroll
        for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if (m0 + wp.m_of(mi, r) == yt[ni]) zy[n0 + wp.n_of(ni)] = acc[mi][ni][r];
      }
      float tmax = -INFINITY;
#pragma unroll
      for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
        for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, acc[mi][ni][r]);
      if (tmax > run[ni].m) {  // strict: an earlier (lower) index keeps a tie
        int best = INT_MAX;
#pragma unroll
        for (int mi = C::MI - 1; mi >= 0; --mi)
#pragma unroll
          for (int r = 15; r >= 0; --r)
            if (acc[mi][ni][r] == tmax) best = vw0 + (wp.m_of(mi, r) - wp.m_of(0, 0));
        run[ni].idx = best;
      }
      const float mnew = fmaxf(run[ni].m, tmax);
      const float msafe = (mnew == -INFINITY) ? 0.f : mnew;
      const float nm = -msafe * L2E;
      float s = run[ni].s * __builtin_amdgcn_exp2f(__builtin_fmaf(run[ni].m, L2E, nm));
#pragma unroll
      for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[mi][ni][r], L2E, nm));
      run[ni].m = mnew;
      run[ni].s = s;
    }
  }

  // merge the two half-wavefronts (same rows, interleaved vocabulary ids) ...
#pragma unroll
  for (int ni = 0; ni < C::NI; ++ni) {
    RowStat o;
    o.m = __shfl_xor(run[ni].m, 32);
    o.s = __shfl_xor(run[ni].s, 32);
    o.idx = __shfl_xor(run[ni].idx, 32);
    run[ni] = merge(run[ni], o);
  }
  // ... then the WGM wavefronts that share the rows, through LDS (free after the main loop)
  RowStat* sh = reinterpret_cast<RowStat*>(smem);  // [WGM][BN]
  if (wp.lane < 32) {
#pragma unroll
    for (int ni = 0; ni < C::NI; ++ni) sh[wp.wm * C::BN + wp.n_of(ni)] = run[ni];
  }
  __syncthreads();
  for (int n = threadIdx.x; n < C::BN; n += C::NTHREADS) {
    RowStat a = sh[n];
    for (int w = 1; w < C::WGM; ++w) a = merge(a, sh[w * C::BN + n]);
    const int t = n0 + n;
    if (t < T) {
      ms[(int64_t)t * nsplit + sp] = make_float2(a.m, a.s);
      idx[(int64_t)t * nsplit + sp] = a.idx;
    }
  }
  PARD2_PROBE_END("fwd_stats_kernel")
}

// ------------------------------------------------------------------------------------
// Backward step 1 for one vocabulary chunk: recompute the logits tile and form
//   dZ[t,v] = g_t * (exp(z[t,v] - lse_t) - 1[v = y_t])
// (softmax-CE gradient scaled by the constant CAT weight, Eq.11 with the stop-gradient),
// rounded to bf16 and written as dZ[t][v - chunk start].  The tile goes through LDS so
// that every global store is a full 512-byte row segment.
// ------------------------------------------------------------------------------------
constexpr int DZ_PITCH = 528;   // LDS bytes per staged row of 256 bf16: 16-byte aligned, rows shift by 4 banks
template <class C>
constexpr int dz_lds_bytes() {
  return C::LDS_BYTES > C::BN * DZ_PITCH ? C::LDS_BYTES : C::BN * DZ_PITCH;
}

template <class C>
__global__ __launch_bounds__(C::NTHREADS) void dz_kernel(const __bf16* __restrict__ H, int64_t ldH,
                                                         const __bf16* __restrict__ W, int64_t ldW,
                                                         const int32_t* __restrict__ y, const float* __restrict__ lse,
                                                         const float* __restrict__ g, int T, int d, int V, int nTt,
                                                         int vt0, int nVtc, __bf16* __restrict__ dZ, int64_t ldz) {
  extern __shared__ __align__(16) char smem[];
  const WavePos<C> wp;
  int tt, vtl;
  banded_tile(xcd_contiguous_id(blockIdx.x, gridDim.x), nTt, nVtc, PARD2_BAND_DZ, tt, vtl);
  const int n0 = tt * C::BN, m0 = (vt0 + vtl) * C::BM, c0 = vtl * C::BM;

  f32x16 acc[C::MI][C::NI];
  zero_acc<C>(acc);
  GemmNT<C>(W, ldW, m0, V, d, H, ldH, n0, T, d, smem).run(acc);

  // registers -> LDS tile [t][v] (a lane holds 4 consecutive v of one t: 8-byte writes).
  // g_t is folded into the exponent, g_t * exp(z - lse_t) = 2^(z*log2e - lse_t*log2e + log2 g_t):
  // one FMA, one v_exp and half a convert per logit.  The single (t, y_t) element of each row
  // is patched afterwards by the lane that holds it; vocabulary ids past V are masked only in
  // the ragged last tile, and a negative g (negative upstream gradient) takes the plain path.
  const bool ragged = m0 + C::BM > V;
#pragma unroll
  for (int ni = 0; ni < C::NI; ++ni) {
    const int tl = wp.n_of(ni);
    const int t = n0 + tl;
    const bool row = t < T;
    const float gt = row ? g[t] : 0.f;
    const float nl = row ? -lse[t] * L2E : -INFINITY;   // rows past T: q = 0
    const int yv = row ? y[t] : -1;
    if (ragged) {
#pragma unroll
      for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (m0 + wp.m_of(mi, r) >= V) acc[mi][ni][r] = -INFINITY;   // ids past V: dZ = 0
    }
    if (__any(gt < 0.f)) {
#pragma unroll
      for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
          bf16x4 pk;
#pragma unroll
          for (int j = 0; j < 4; ++j)
            pk[j] = (__bf16)(gt * __builtin_amdgcn_exp2f(__builtin_fmaf(acc[mi][ni][rq * 4 + j], L2E, nl)));
          *reinterpret_cast<bf16x4*>(smem + tl * DZ_PITCH + wp.m_of(mi, rq * 4) * 2) = pk;
        }
    } else {
      const float nlg = nl + __builtin_amdgcn_logf(gt);   // v_log_f32 = log2; log2(0) = -inf gives dZ = 0
#pragma unroll
      for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
          bf16x4 pk;
#pragma unroll
          for (int j = 0; j < 4; ++j)
            pk[j] = (__bf16)__builtin_amdgcn_exp2f(__builtin_fmaf(acc[mi][ni][rq * 4 + j], L2E, nlg));
          *reinterpret_cast<bf16x4*>(smem + tl * DZ_PITCH + wp.m_of(mi, rq * 4) * 2) = pk;
        }
    }
    // the target element: dZ = g (q - 1), computed in fp32 and rounded once
    const int rel = yv - (m0 + wp.wm * C::WTM);
    if (rel >= 0 && rel < C::WTM) {
#pragma unroll
      for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (m0 + wp.m_of(mi, r) == yv) {
            const float q = __builtin_amdgcn_exp2f(__builtin_fmaf(acc[mi][ni][r], L2E, nl));
            *reinterpret_cast<__bf16*>(smem + tl * DZ_PITCH + wp.m_of(mi, r) * 2) = (__bf16)(gt * (q - 1.f));
          }
    }
  }
  __syncthreads();
  // LDS -> global: 32 lanes x 16 bytes cover one row of the tile
  constexpr int ROWS_PER_PASS = C::NTHREADS / 32;
  const int chunk = threadIdx.x & 31, r0 = threadIdx.x >> 5;
#pragma unroll 4
  for (int r = r0; r < C::BN; r += ROWS_PER_PASS) {
    const int t = n0 + r;
    if (t < T) {
      const u32x4 v = *reinterpret_cast<const u32x4*>(smem + r * DZ_PITCH + chunk * 16);
      // streamed out: the chunk (hundreds of MB) is read back only by later kernels, keeping it out of
      // the L2 leaves the operand panels there (measured: dz 3.78 -> 3.67 ms per step)
      __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(dZ + (int64_t)t * ldz + c0 + chunk * 8));
    }
  }
}

// ------------------------------------------------------------------------------------
// Backward step 2: dH[t,i] (+)= sum_v dZ[t,v] * W[v,i] over the chunk's vocabulary ids.
// A = W rows of the chunk as they lie in memory (k-major: k = v, columns i), B = dZ
// (k-contiguous rows t).  The fp32 running sum across chunks lives in dHacc; the last
// chunk writes the bf16 result.
// With few token rows the T x d output has fewer tiles than the chip has compute units;
// then the chunk's k range is cut into `kslices` slices of Ks ids, each workgroup writes
// its slice's partial tile to dHpart[slice] and dh_reduce_kernel adds the slices in a
// fixed order (no atomics: reproducible).
// ------------------------------------------------------------------------------------
template <class C>
__global__ __launch_bounds__(C::NTHREADS) void dh_kernel(const __bf16* __restrict__ Wc, int64_t ldW,
                                                         const __bf16* __restrict__ dZ, int64_t ldz, int T, int d,
                                                         int nvalid, int Kc, int nIt, int nTt, int kslices, int Ks,
                                                         float* __restrict__ dHacc, float* __restrict__ dHpart,
                                                         __bf16* __restrict__ dH, int first, int last) {
  extern __shared__ __align__(16) char smem[];
  PARD2_PROBE_BEGIN
  const WavePos<C> wp;
  const int id = xcd_contiguous_id(blockIdx.x, gridDim.x);
  const int ntiles = nIt * nTt;
  const int slice = id / ntiles;
  int it, tt;
  banded_tile(id - slice * ntiles, nIt, nTt, 8, it, tt);
  const int m0 = it * C::BM, n0 = tt * C::BN;
  const int k0 = slice * Ks;
  const int KB = min(Ks, Kc - k0);               // dZ's columns up to Kc exist (zero past nvalid)
  const int KA = max(0, min(KB, nvalid - k0));   // W has nvalid rows in this chunk

  f32x16 acc[C::MI][C::NI];
  zero_acc<C>(acc);
  GemmNT<C, true, false>(Wc + (int64_t)k0 * ldW, ldW, m0, d, KA, dZ + k0, ldz, n0, T, KB, smem).run(acc);

#pragma unroll
  for (int ni = 0; ni < C::NI; ++ni) {
    const int t = n0 + wp.n_of(ni);
    if (t >= T) continue;
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        const int i = m0 + wp.m_of(mi, rq * 4);
        if (i >= d) continue;
        f32x4 v = {acc[mi][ni][rq * 4], acc[mi][ni][rq * 4 + 1], acc[mi][ni][rq * 4 + 2], acc[mi][ni][rq * 4 + 3]};
        if (kslices > 1) {
          *reinterpret_cast<f32x4*>(dHpart + ((int64_t)slice * T + t) * d + i) = v;
          continue;
        }
        f32x4* p = reinterpret_cast<f32x4*>(dHacc + (int64_t)t * d + i);
        if (!first) v += *p;
        if (last) {
          bf16x4 o = {(__bf16)v[0], (__bf16)v[1], (__bf16)v[2], (__bf16)v[3]};
          *reinterpret_cast<bf16x4*>(dH + (int64_t)t * d + i) = o;
        } else {
          *p = v;
        }
      }
  }
  PARD2_PROBE_END("dh_kernel")
}

// dHacc (+)= sum over slices of dHpart, in slice order; the last chunk writes bf16 dH instead.
// n4 = T*d/4 groups of four floats (d is a multiple of 8).
__global__ __launch_bounds__(256) void dh_reduce_kernel(const float* __restrict__ dHpart, int kslices, int64_t n4,
                                                        float* __restrict__ dHacc, __bf16* __restrict__ dH,
                                                        int first, int last) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n4) return;
  f32x4 v = {0.f, 0.f, 0.f, 0.f};
  if (!first) v = reinterpret_cast<const f32x4*>(dHacc)[i];
  for (int s = 0; s < kslices; ++s) v += reinterpret_cast<const f32x4*>(dHpart)[(int64_t)s * n4 + i];
  if (last) {
    bf16x4 o = {(__bf16)v[0], (__bf16)v[1], (__bf16)v[2], (__bf16)v[3]};
    reinterpret_cast<bf16x4*>(dH)[i] = o;
  } else {
    reinterpret_cast<f32x4*>(dHacc)[i] = v;
  }
}

// ------------------------------------------------------------------------------------
// Backward step 3: dW[v,i] = sum_t dZ[t,v] * H[t,i] for the chunk's vocabulary rows
// (complete per chunk: no accumulation across chunks).  Both operands are read as they
// lie in memory, k-major with k = t: A = H (columns i), B = dZ (columns v).
// ------------------------------------------------------------------------------------
template <class C>
__global__ __launch_bounds__(C::NTHREADS) void dw_kernel(const __bf16* __restrict__ H, int64_t ldH,
                                                         const __bf16* __restrict__ dZ, int64_t ldz, int T, int d,
                                                         int nvalid, int Kc, int nIt, int nVtc,
                                                         __bf16* __restrict__ dWc, int accumulate, int dw_f32) {
  extern __shared__ __align__(16) char smem[];
  const WavePos<C> wp;
  int it, vtl;
  banded_tile(xcd_contiguous_id(blockIdx.x, gridDim.x), nIt, nVtc, 8, it, vtl);
  const int m0 = it * C::BM, n0 = vtl * C::BN;

  f32x16 acc[C::MI][C::NI];
  zero_acc<C>(acc);
  GemmNT<C, true, true>(H, ldH, m0, d, T, dZ, ldz, n0, Kc, T, smem).run(acc);

#pragma unroll
  for (int ni = 0; ni < C::NI; ++ni) {
    const int vr = n0 + wp.n_of(ni);
    if (vr >= nvalid) continue;
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        const int i = m0 + wp.m_of(mi, rq * 4);
        if (i >= d) continue;
        f32x4 v = {acc[mi][ni][rq * 4], acc[mi][ni][rq * 4 + 1], acc[mi][ni][rq * 4 + 2], acc[mi][ni][rq * 4 + 3]};
        if (dw_f32) {   // fp32 gradient buffer: no rounding between accumulation steps
          f32x4* pf = reinterpret_cast<f32x4*>(reinterpret_cast<float*>(dWc) + (int64_t)vr * d + i);
          if (accumulate) v += *pf;
          *pf = v;
          continue;
        }
        bf16x4* p = reinterpret_cast<bf16x4*>(dWc + (int64_t)vr * d + i);
        if (accumulate) {
          const bf16x4 old = *p;
          v[0] += (float)old[0]; v[1] += (float)old[1]; v[2] += (float)old[2]; v[3] += (float)old[3];
        }
        bf16x4 o = {(__bf16)v[0], (__bf16)v[1], (__bf16)v[2], (__bf16)v[3]};
        *p = o;
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

int fwd_num_partials_bf16(int T, int V) {
  const int nTt = ceil_div(T, Cfg::BN), nVt = ceil_div(V, Cfg::BM);
  // enough vocabulary ranges to give every compute unit a workgroup, never more than tiles
  int ns = ceil_div(PARD2_FWD_WGS, nTt);
  ns = ns < 1 ? 1 : ns;
  return ns > nVt ? nVt : ns;
}

hipError_t launch_fwd_stats_bf16(const void* H, int64_t ldH, const void* W, int64_t ldW, const int32_t* y, int T,
                                 int d, int V, StatsOut out, hipStream_t s) {
  const int nTt = ceil_div(T, Cfg::BN), nVt = ceil_div(V, Cfg::BM), ns = out.P;
  auto k = fwd_stats_kernel<Cfg>;
  hipError_t e = allow_lds(k, Cfg::LDS_BYTES);
  if (e != hipSuccess) return e;
  launch_timed(KT_FWD_STATS, k, dim3(nTt * ns), dim3(Cfg::NTHREADS), Cfg::LDS_BYTES, s, (const __bf16*)H, ldH,
               (const __bf16*)W, ldW, y, T, d, V, nTt, nVt, ns, out.ms, out.idx, out.zy);
  return hipGetLastError();
}

// Slices of the dH contraction's k range for a chunk of Kc ids: (count, ids per slice).  One slice
// when the T x d output already fills the chip; otherwise enough slices for ~256 workgroups, each
// at least 16 stages of 64 ids long.
static std::pair<int, int> dh_k_slices(int T, int d, int Kc) {
  const int tiles = ceil_div(T, Cfg::BN) * ceil_div(d, Cfg::BM);
  if (tiles >= 192) return {1, Kc};
  int want = ceil_div(256, tiles);
  const int max_by_len = Kc / (16 * 64) > 1 ? Kc / (16 * 64) : 1;
  want = want > max_by_len ? max_by_len : want;
  want = want > 16 ? 16 : want;
  const int Ks = (int)round_up(ceil_div(Kc, want), 64);
  return {ceil_div(Kc, Ks), Ks};
}

BwdPlanBf16 plan_bwd_bf16(int T, int d, int V) {
  BwdPlanBf16 p{};
  const int nVt = ceil_div(V, Cfg::BM);
  const int max_tiles = PARD2_CHUNK_TILES;   // vocabulary tiles per chunk (Vc <= 16384 by default)
  p.nchunks = ceil_div(nVt, max_tiles);
  p.Vc = (int64_t)ceil_div(nVt, p.nchunks) * Cfg::BM;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o += (bytes + 255) / 256 * 256; return at; };
  p.off_g = take((size_t)T * 4);
  p.off_dZ = take((size_t)T * p.Vc * 2);
  p.off_dHacc = take((size_t)T * d * 4);
  p.kslices = dh_k_slices(T, d, (int)p.Vc).first;
  p.off_dHpart = take(p.kslices > 1 ? (size_t)p.kslices * T * d * 4 : 0);
  p.total = o;
  return p;
}

hipError_t launch_bwd_bf16(const BwdPlanBf16& p, const void* H, int64_t ldH, const void* W, int64_t ldW,
                           const int32_t* y, const float* lse, const float* g, int T, int d, int V, void* dH,
                           void* dW, int accumulate_dW, char* ws, hipStream_t s, const KdTeacher* kd) {
  __bf16* dZ = (__bf16*)(ws + p.off_dZ);
  float* dHacc = (float*)(ws + p.off_dHacc);
  float* dHpart = (float*)(ws + p.off_dHpart);
  constexpr int DZ_LDS = dz_lds_bytes<Cfg>();
  hipError_t e;
  if ((e = allow_lds(dz_kernel<Cfg>, DZ_LDS)) != hipSuccess) return e;
  if ((e = allow_lds(dh_kernel<Cfg>, Cfg::LDS_BYTES)) != hipSuccess) return e;
  if ((e = allow_lds(dw_kernel<Cfg>, Cfg::LDS_BYTES)) != hipSuccess) return e;

  const int nVt = ceil_div(V, Cfg::BM), nTt = ceil_div(T, Cfg::BN), nIt = ceil_div(d, Cfg::BM);
  const int dw_f32 = (accumulate_dW & 2) != 0;   // bit 1: dW is an fp32 buffer
  for (int c = 0; c < p.nchunks; ++c) {
    const int vt0 = (int)((int64_t)c * nVt / p.nchunks), vt1 = (int)((int64_t)(c + 1) * nVt / p.nchunks);
    const int nVtc = vt1 - vt0;
    const int v0 = vt0 * Cfg::BM;
    const int Kc = nVtc * Cfg::BM;                  // padded chunk width (dZ columns written)
    const int nvalid = (V - v0 < Kc) ? V - v0 : Kc; // vocabulary rows that exist in the chunk
    if (kd) {   // distillation term present: the two-head recompute forms dZ
      if ((e = launch_kd_dz_bf16(H, ldH, W, ldW, *kd, y, lse, g, T, d, V, v0, Kc, dZ, p.Vc, kd->kd_part, s)) != hipSuccess) return e;
    } else {
      launch_timed(KT_DZ, dz_kernel<Cfg>, dim3(nTt * nVtc), dim3(Cfg::NTHREADS), DZ_LDS, s, (const __bf16*)H, ldH,
                   (const __bf16*)W, ldW, y, lse, g, T, d, V, nTt, vt0, nVtc, dZ, p.Vc);
    }
    auto sl = dh_k_slices(T, d, Kc);
    if (sl.first > p.kslices) {              // never more slices than the workspace was planned for
      sl.second = (int)round_up(ceil_div(Kc, p.kslices), 64);
      sl.first = ceil_div(Kc, sl.second);
    }
    const int first = c == 0, last = c == p.nchunks - 1;
    launch_timed(KT_DH, dh_kernel<Cfg>, dim3(nIt * nTt * sl.first), dim3(Cfg::NTHREADS), Cfg::LDS_BYTES, s,
                 (const __bf16*)W + (int64_t)v0 * ldW, ldW, dZ, p.Vc, T, d, nvalid, Kc, nIt, nTt, sl.first,
                 sl.second, dHacc, dHpart, (__bf16*)dH, first, last);
    if (sl.first > 1) {
      const int64_t n4 = (int64_t)T * d / 4;
      hipLaunchKernelGGL(dh_reduce_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, s, dHpart, sl.first, n4,
                         dHacc, (__bf16*)dH, first, last);
    }
    launch_timed(KT_DW, dw_kernel<Cfg>, dim3(nIt * nVtc), dim3(Cfg::NTHREADS), Cfg::LDS_BYTES, s, (const __bf16*)H,
                 ldH, dZ, p.Vc, T, d, nvalid, Kc, nIt, nVtc,
                 dw_f32 ? (__bf16*)((float*)dW + (int64_t)v0 * d) : (__bf16*)dW + (int64_t)v0 * d,
                 accumulate_dW & 1, dw_f32);
  }
  return hipGetLastError();
}

}  // namespace pard2
