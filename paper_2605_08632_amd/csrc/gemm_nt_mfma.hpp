// bf16 "NT" contraction main loop for gfx950 (CDNA4) matrix cores.
//
//   acc[m][n] += sum_k A[m][k] * B[n][k]
//
// Both operands are row-major with the contraction index contiguous, which is the
// layout v_mfma_f32_32x32x16_bf16 wants in registers: lane l supplies 8 consecutive
// k values (k = 8*(l/32) .. +7) of row l%32 of A and of row l%32 of B, so one
// 16-byte LDS read fills an operand.  All four contractions of the CAT loss
// (logits, their recomputation, dH and dW) are brought to this form.
//
// Work split: a workgroup of WGM x WGN wavefronts (64 lanes each) owns a BM x BN
// output tile; each wavefront owns (BM/WGM) x (BN/WGN) of it as MI x NI MFMA
// sub-tiles of 32x32, fp32 accumulators living in registers for the whole k loop.
// Per k step of BK the tile's A and B panels are staged through LDS
// (global -> registers -> LDS, double buffered: the next panel's global loads are
// in flight while the current one feeds the matrix cores).
//
// Accumulator layout (hardware): element r (0..15) of sub-tile (mi, ni) held by
// lane l is
//     m = mi*32 + 8*(r/4) + 4*(l/32) + (r%4),     n = ni*32 + (l%32)
// relative to the wavefront's tile origin.  A lane therefore owns ONE n index per
// sub-tile column and 16*MI m indices: kernels put the index along which they
// reduce or store contiguously on the M side.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pard2 {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

template <int BM_, int BN_, int BK_, int WGM_, int WGN_>
struct TileCfg {
  static constexpr int BM = BM_, BN = BN_, BK = BK_, WGM = WGM_, WGN = WGN_;
  static constexpr int NWAVES = WGM * WGN;
  static constexpr int NTHREADS = 64 * NWAVES;
  static constexpr int WTM = BM / WGM, WTN = BN / WGN;  // wavefront tile
  static constexpr int MI = WTM / 32, NI = WTN / 32;    // 32x32 sub-tiles per wavefront
  static constexpr int CPR = BK / 8;                    // 16-byte chunks per panel row
  static constexpr int PITCH = BK * 2 + 16;             // LDS row pitch (bytes): +16 keeps 8
                                                        // consecutive rows on distinct banks
  static constexpr int A_LOADS = BM * CPR / NTHREADS;   // 16-byte loads per thread and panel
  static constexpr int B_LOADS = BN * CPR / NTHREADS;
  static constexpr int ROWS_PER_PASS = NTHREADS / CPR;
  static constexpr int STAGE_BYTES = (BM + BN) * PITCH;
  static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
  static_assert(BM % (32 * WGM) == 0 && BN % (32 * WGN) == 0, "wave tile must be 32-aligned");
  static_assert(BK % 16 == 0, "BK must hold whole MFMA k steps");
  static_assert((BM * CPR) % NTHREADS == 0 && (BN * CPR) % NTHREADS == 0, "loader split");
};

// Position of the calling wavefront/lane inside the workgroup tile.
template <class C>
struct WavePos {
  int lane, wm, wn;
  __device__ __forceinline__ WavePos() {
    const int wave = threadIdx.x >> 6;
    lane = threadIdx.x & 63;
    wm = wave % C::WGM;
    wn = wave / C::WGM;
  }
  // tile-relative m of accumulator element r of sub-tile row mi
  __device__ __forceinline__ int m_of(int mi, int r) const {
    return wm * C::WTM + mi * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
  }
  // tile-relative n of sub-tile column ni
  __device__ __forceinline__ int n_of(int ni) const { return wn * C::WTN + ni * 32 + (lane & 31); }
};

// One BM x BN x Kdim contraction.  Rows beyond M / N are clamped to the last valid
// row (their results are garbage the caller must mask); k beyond Kdim reads as zero.
// Kdim, lda, ldb must be multiples of 8 and the bases 16-byte aligned.
template <class C>
__device__ __forceinline__ void gemm_nt_mainloop(const __bf16* __restrict__ A, int64_t lda, int m0, int M,
                                                 const __bf16* __restrict__ B, int64_t ldb, int n0, int N,
                                                 int Kdim, char* smem, f32x16 (&acc)[C::MI][C::NI]) {
  const int tid = threadIdx.x;
  const WavePos<C> wp;
  const int lane = wp.lane;

  // ---- loader state: byte offsets from the tile's first row, one per 16-byte load
  const char* Abase = reinterpret_cast<const char*>(A + (int64_t)m0 * lda);
  const char* Bbase = reinterpret_cast<const char*>(B + (int64_t)n0 * ldb);
  const int kc = tid % C::CPR;  // which 16-byte chunk of the panel row this thread moves
  const int r0 = tid / C::CPR;
  uint32_t aoff[C::A_LOADS], boff[C::B_LOADS];
#pragma unroll
  for (int j = 0; j < C::A_LOADS; ++j) {
    int r = r0 + j * C::ROWS_PER_PASS;
    r = min(r, M - 1 - m0);
    aoff[j] = (uint32_t)((int64_t)r * lda * 2 + kc * 16);
  }
#pragma unroll
  for (int j = 0; j < C::B_LOADS; ++j) {
    int r = r0 + j * C::ROWS_PER_PASS;
    r = min(r, N - 1 - n0);
    boff[j] = (uint32_t)((int64_t)r * ldb * 2 + kc * 16);
  }
  const uint32_t st_off = (uint32_t)(r0 * C::PITCH + kc * 16);  // LDS store offset (pass 0)

  // ---- MFMA operand read offsets inside a stage
  const uint32_t a_rd = (uint32_t)((wp.wm * C::WTM + (lane & 31)) * C::PITCH + (lane >> 5) * 16);
  const uint32_t b_rd = (uint32_t)(C::BM * C::PITCH + (wp.wn * C::WTN + (lane & 31)) * C::PITCH + (lane >> 5) * 16);

  u32x4 areg[C::A_LOADS], breg[C::B_LOADS];
  const int nk = (Kdim + C::BK - 1) / C::BK;

  auto load_global = [&](int kt) {
    const int kbyte = kt * C::BK * 2;
    const bool full = (kt + 1) * C::BK <= Kdim;
    if (full) {
#pragma unroll
      for (int j = 0; j < C::A_LOADS; ++j) areg[j] = *reinterpret_cast<const u32x4*>(Abase + kbyte + aoff[j]);
#pragma unroll
      for (int j = 0; j < C::B_LOADS; ++j) breg[j] = *reinterpret_cast<const u32x4*>(Bbase + kbyte + boff[j]);
    } else {
      const bool in = kt * C::BK + kc * 8 < Kdim;
      const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
      for (int j = 0; j < C::A_LOADS; ++j)
        areg[j] = in ? *reinterpret_cast<const u32x4*>(Abase + kbyte + aoff[j]) : zero;
#pragma unroll
      for (int j = 0; j < C::B_LOADS; ++j)
        breg[j] = in ? *reinterpret_cast<const u32x4*>(Bbase + kbyte + boff[j]) : zero;
    }
  };
  auto store_lds = [&](int stage) {
    char* s = smem + stage * C::STAGE_BYTES + st_off;
#pragma unroll
    for (int j = 0; j < C::A_LOADS; ++j)
      *reinterpret_cast<u32x4*>(s + j * C::ROWS_PER_PASS * C::PITCH) = areg[j];
    s += C::BM * C::PITCH;
#pragma unroll
    for (int j = 0; j < C::B_LOADS; ++j)
      *reinterpret_cast<u32x4*>(s + j * C::ROWS_PER_PASS * C::PITCH) = breg[j];
  };

  load_global(0);
  store_lds(0);
  __syncthreads();

  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) load_global(kt + 1);
    const char* s = smem + cur * C::STAGE_BYTES;
#pragma unroll
    for (int kk = 0; kk < C::BK / 16; ++kk) {
      bf16x8 af[C::MI], bfr[C::NI];
#pragma unroll
      for (int mi = 0; mi < C::MI; ++mi)
        af[mi] = *reinterpret_cast<const bf16x8*>(s + a_rd + mi * 32 * C::PITCH + kk * 32);
#pragma unroll
      for (int ni = 0; ni < C::NI; ++ni)
        bfr[ni] = *reinterpret_cast<const bf16x8*>(s + b_rd + ni * 32 * C::PITCH + kk * 32);
#pragma unroll
      for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < C::NI; ++ni)
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mi], bfr[ni], acc[mi][ni], 0, 0, 0);
    }
    if (kt + 1 < nk) store_lds(cur ^ 1);
    __syncthreads();
  }
}

template <class C>
__device__ __forceinline__ void zero_acc(f32x16 (&acc)[C::MI][C::NI]) {
#pragma unroll
  for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < C::NI; ++ni)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;
}

// Workgroups are handed to the 8 XCDs round-robin (id % 8), and each XCD has its own
// L2.  This maps the hardware id to a logical id such that every XCD works on a
// contiguous range of logical ids (so neighbouring tiles share an L2).
__device__ __forceinline__ int xcd_contiguous_id(int bid, int nblocks) {
  constexpr int NXCD = 8;
  const int xcd = bid % NXCD, local = bid / NXCD;
  const int q = nblocks / NXCD, rem = nblocks % NXCD;
  // XCD x owns q (+1 if x < rem) ids
  const int start = xcd * q + min(xcd, rem);
  return start + local;
}

// Logical id -> (row tile, column tile): walk column tiles in bands of `band` rows so
// that ids close together reuse both operands' panels.
__device__ __forceinline__ void banded_tile(int id, int ntm, int ntn, int band, int& tm, int& tn) {
  const int per_band = band * ntn;
  const int b = id / per_band;
  const int first = b * band;
  const int rows = min(band, ntm - first);
  const int in = id - b * per_band;
  tm = first + in % rows;
  tn = in / rows;
}

}  // namespace pard2
