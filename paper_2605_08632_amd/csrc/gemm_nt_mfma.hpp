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
//
// Data movement: per k stage of BK = 64 the tile's A and B panels go global -> LDS
// directly (global_load_lds_dwordx4: no staging registers, asynchronous), into one of
// two LDS stages; the loads of stage s+1 are issued while stage s feeds the matrix
// cores, and one workgroup barrier per stage closes the hand-over.  LDS rows are
// 128 bytes, unpadded (a wave-level direct load fills 1 KB = 8 rows contiguously);
// bank conflicts are avoided by storing the 16-byte chunk c of row r at position
// c ^ ((r >> 1) & 7), which makes any 16 consecutive rows of one chunk column hit 16
// different 16-byte bank groups.  Operand fragments are double-buffered in registers
// across the four k steps of a stage so that LDS latency hides under MFMA issue.
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

template <int BM_, int BN_, int WGM_, int WGN_>
struct TileCfg {
  static constexpr int BM = BM_, BN = BN_, BK = 64, WGM = WGM_, WGN = WGN_;
  static constexpr int NWAVES = WGM * WGN;
  static constexpr int NTHREADS = 64 * NWAVES;
  static constexpr int WTM = BM / WGM, WTN = BN / WGN;  // wavefront tile
  static constexpr int MI = WTM / 32, NI = WTN / 32;    // 32x32 sub-tiles per wavefront
  static constexpr int ROWB = 128;                      // LDS row: BK bf16
  static constexpr int A_LOADS = BM / 8 / NWAVES;       // wave-level 1 KB direct loads per stage
  static constexpr int B_LOADS = BN / 8 / NWAVES;
  static constexpr int STAGE_BYTES = (BM + BN) * ROWB;
  static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
  static_assert(BM % (32 * WGM) == 0 && BN % (32 * WGN) == 0, "wave tile must be 32-aligned");
  static_assert(BM % (8 * NWAVES) == 0 && BN % (8 * NWAVES) == 0, "loader split");
  static_assert(A_LOADS % 2 == 0 && B_LOADS % 2 == 0, "loads are issued in two halves");
  static_assert(MI >= 2 && NI >= 2, "the split MFMA schedule needs a 2x2 sub-tile grid at least");
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

// 16 bytes of zeros: the source of direct loads whose k range lies past the operand's end
__device__ __attribute__((aligned(16))) static const uint32_t g_zero16[4] = {0, 0, 0, 0};

// Wait for all of this wavefront's direct loads and LDS reads, then meet the workgroup
// barrier.  (Kept as one asm block so that nothing is scheduled in between.)
__device__ __forceinline__ void wait_all_and_barrier() {
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n s_barrier" ::: "memory");
}

// One BM x BN x Kdim contraction.  Rows beyond M / N are clamped to the last valid
// row (their results are garbage the caller must mask); k beyond Kdim reads as zero.
// Kdim, lda, ldb must be multiples of 8 and the bases 16-byte aligned.  m0 < M, n0 < N.
//
// `prefetched`: the caller already issued stage 0 of THIS tile with gemm_nt_prefetch
// (used to overlap a tile's first loads with the previous tile's epilogue).
// On return every wavefront has passed a barrier after its last LDS read: LDS is free.
template <class C>
struct GemmNT {
  typedef __attribute__((address_space(3))) void* lds_ptr;
  typedef const __attribute__((address_space(1))) void* glb_ptr;

  const char* Abase;
  const char* Bbase;
  char* smem;
  uint32_t aoff[C::A_LOADS], boff[C::B_LOADS];
  int ach[C::A_LOADS], bch[C::B_LOADS];
  int Kdim, nk, wave;

  __device__ __forceinline__ GemmNT(const __bf16* __restrict__ A, int64_t lda, int m0, int M,
                                    const __bf16* __restrict__ B, int64_t ldb, int n0, int N, int Kdim_,
                                    char* smem_)
      : smem(smem_), Kdim(Kdim_) {
    const int lane = threadIdx.x & 63;
    wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int rin = lane >> 3, cpos = lane & 7;
    Abase = reinterpret_cast<const char*>(A + (int64_t)m0 * lda);
    Bbase = reinterpret_cast<const char*>(B + (int64_t)n0 * ldb);
#pragma unroll
    for (int j = 0; j < C::A_LOADS; ++j) {
      const int row = 8 * (wave + C::NWAVES * j) + rin;
      ach[j] = cpos ^ ((row >> 1) & 7);
      aoff[j] = (uint32_t)((int64_t)min(row, M - 1 - m0) * lda * 2 + ach[j] * 16);
    }
#pragma unroll
    for (int j = 0; j < C::B_LOADS; ++j) {
      const int row = 8 * (wave + C::NWAVES * j) + rin;
      bch[j] = cpos ^ ((row >> 1) & 7);
      boff[j] = (uint32_t)((int64_t)min(row, N - 1 - n0) * ldb * 2 + bch[j] * 16);
    }
    nk = (Kdim + 63) / 64;
  }

  // half h (0/1) of the direct loads of stage kt; full = every chunk lies below Kdim
  __device__ __forceinline__ void issue_half(int kt, int h, bool full) const {
    const int kbyte = kt * 128;
    char* sA = smem + (kt & 1) * C::STAGE_BYTES;
    char* sB = sA + C::BM * C::ROWB;
    const char* z = reinterpret_cast<const char*>(g_zero16);
#pragma unroll
    for (int j = 0; j < C::A_LOADS / 2; ++j) {
      const int jj = h * (C::A_LOADS / 2) + j;
      const char* src = Abase + kbyte + aoff[jj];
      if (!full && kt * 64 + ach[jj] * 8 >= Kdim) src = z;
      __builtin_amdgcn_global_load_lds((glb_ptr)src, (lds_ptr)(sA + (wave + C::NWAVES * jj) * 1024), 16, 0, 0);
    }
#pragma unroll
    for (int j = 0; j < C::B_LOADS / 2; ++j) {
      const int jj = h * (C::B_LOADS / 2) + j;
      const char* src = Bbase + kbyte + boff[jj];
      if (!full && kt * 64 + bch[jj] * 8 >= Kdim) src = z;
      __builtin_amdgcn_global_load_lds((glb_ptr)src, (lds_ptr)(sB + (wave + C::NWAVES * jj) * 1024), 16, 0, 0);
    }
  }

  // Issue stage 0 early (LDS must be free: all wavefronts past their last read).
  __device__ __forceinline__ void prefetch() const {
    issue_half(0, 0, false);
    issue_half(0, 1, false);
  }

  __device__ __forceinline__ void run(f32x16 (&acc)[C::MI][C::NI], bool prefetched = false) const {
    const int lane = threadIdx.x & 63;
    const int wm = wave % C::WGM, wn = wave / C::WGM;
    const int swz = ((lane & 31) >> 1) & 7;   // row-dependent part of the swizzle: sub-tile strides are
    uint32_t koff[4];                         // multiples of 32 rows, so it is a lane constant
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) koff[kk] = (uint32_t)(((kk * 2 + (lane >> 5)) ^ swz) * 16);
    const uint32_t a_row = (uint32_t)((wm * C::WTM + (lane & 31)) * C::ROWB);
    const uint32_t b_row = (uint32_t)(C::BM * C::ROWB + (wn * C::WTN + (lane & 31)) * C::ROWB);

    bf16x8 fa0[C::MI], fb0[C::NI], fa1[C::MI], fb1[C::NI];
    auto read_frags = [&](int kt, int kk, bf16x8 (&fa)[C::MI], bf16x8 (&fb)[C::NI]) {
      const char* s = smem + (kt & 1) * C::STAGE_BYTES;
#pragma unroll
      for (int mi = 0; mi < C::MI; ++mi)
        fa[mi] = *reinterpret_cast<const bf16x8*>(s + a_row + mi * 32 * C::ROWB + koff[kk]);
#pragma unroll
      for (int ni = 0; ni < C::NI; ++ni)
        fb[ni] = *reinterpret_cast<const bf16x8*>(s + b_row + ni * 32 * C::ROWB + koff[kk]);
    };
    // MFMAs number lo..hi-1 of the MI x NI grid (row-major numbering)
    auto mma_sel = [&](bf16x8 (&fa)[C::MI], bf16x8 (&fb)[C::NI], int lo, int hi) {
#pragma unroll
      for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < C::NI; ++ni)
          if (mi * C::NI + ni >= lo && mi * C::NI + ni < hi)
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[mi], fb[ni], acc[mi][ni], 0, 0, 0);
    };
    // the MFMAs with (mi + ni) of the given parity: parity 0 touches every fragment
    auto mma_par = [&](bf16x8 (&fa)[C::MI], bf16x8 (&fb)[C::NI], int parity) {
#pragma unroll
      for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < C::NI; ++ni)
          if (((mi + ni) & 1) == parity)
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[mi], fb[ni], acc[mi][ni], 0, 0, 0);
    };
    constexpr int NM = C::MI * C::NI;

    // One stage = four k steps.  The instruction order is pinned with scheduling barriers:
    //   first MFMA of a k step | (next stage's loads,) LDS reads of the next k step | its other MFMAs
    // so that every LDS read has a k step of MFMAs to land under.  In the last k step half of
    // the MFMAs run, then the barrier (next stage landed for everyone, this stage's buffer free),
    // then the first reads of the next stage under the remaining MFMAs.
#define PARD2_SB __builtin_amdgcn_sched_barrier(0)
#define PARD2_STAGE(ISSUE0, ISSUE1, HAS_NEXT)                                                             \
  mma_sel(fa0, fb0, 0, 1); PARD2_SB; ISSUE0; read_frags(kt, 1, fa1, fb1); PARD2_SB; mma_sel(fa0, fb0, 1, NM); PARD2_SB; \
  mma_sel(fa1, fb1, 0, 1); PARD2_SB; ISSUE1; read_frags(kt, 2, fa0, fb0); PARD2_SB; mma_sel(fa1, fb1, 1, NM); PARD2_SB; \
  mma_sel(fa0, fb0, 0, 1); PARD2_SB;         read_frags(kt, 3, fa1, fb1); PARD2_SB; mma_sel(fa0, fb0, 1, NM); PARD2_SB; \
  mma_par(fa1, fb1, 0); PARD2_SB; wait_all_and_barrier(); PARD2_SB;                                       \
  if (HAS_NEXT) read_frags(kt + 1, 0, fa0, fb0);                                                          \
  PARD2_SB; mma_par(fa1, fb1, 1); PARD2_SB;

    if (!prefetched) prefetch();
    wait_all_and_barrier();
    read_frags(0, 0, fa0, fb0);

    int kt = 0;
    for (; kt < nk - 2; ++kt) {
      PARD2_STAGE(issue_half(kt + 1, 0, true), issue_half(kt + 1, 1, true), true)
    }
    if (kt < nk - 1) {   // the last stage may be partial in k
      PARD2_STAGE(issue_half(kt + 1, 0, false), issue_half(kt + 1, 1, false), true)
      ++kt;
    }
    {
      PARD2_STAGE((void)0, (void)0, false)
    }
#undef PARD2_STAGE
#undef PARD2_SB
    // the barrier inside the last stage already separates every wavefront's last LDS read
    // from whatever the caller does with LDS next
  }
};

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
