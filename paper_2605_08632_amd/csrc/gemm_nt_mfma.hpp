// bf16 contraction main loop for gfx950 (CDNA4) matrix cores.
//
//   acc[m][n] += sum_k A(m,k) * B(n,k)
//
// Each operand is given in one of two memory layouts:
//   KC  "k-contiguous": row-major [rows][k]   (rows = m for A, n for B)
//   KM  "k-major":      row-major [k][rows]
// v_mfma_f32_32x32x16_bf16 wants, in registers, lane l to hold 8 consecutive k values
// (k = 8*(l/32) .. +7) of row l%32.  From a KC panel that is one 16-byte LDS read; from a
// KM panel it is two transposing LDS reads (ds_read_b64_tr_b16, which hands every lane of
// a 16-lane group one 16-bit column of a 4-row x 16-column block).  With both layouts on
// offer, all four contractions of the CAT loss (logits, their recomputation, dH, dW) read
// H, W and dZ exactly as they lie in memory: no transposed copies.
//
// Work split: a workgroup of WGM x WGN wavefronts (64 lanes each) owns a BM x BN
// output tile; each wavefront owns (BM/WGM) x (BN/WGN) of it as MI x NI MFMA
// sub-tiles of 32x32, fp32 accumulators living in registers for the whole k loop.
//
// Data movement: per k stage of BK = 64 the tile's A and B panels (32 KB each) go
// global -> LDS directly (global_load_lds_dwordx4: no staging registers, asynchronous),
// into one of two LDS stages; the loads of stage s+1 are issued while stage s feeds the
// matrix cores, and one workgroup barrier per stage closes the hand-over.  A wave-level
// direct load fills 1 KB of LDS contiguously, so panels are unpadded; bank conflicts are
// avoided by XOR-swizzling 16-byte chunks:
//   KC panel: 128-byte rows; chunk c of row r sits at c ^ ((r >> 1) & 7)
//   KM panel: 512-byte rows; chunk c of row k sits at c ^ ((k & 3) << 2)
// Operand fragments are double-buffered in registers across the four k steps of a stage
// so that LDS latency hides under MFMA issue.
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
typedef __attribute__((ext_vector_type(4))) short s16x4;

template <int BM_, int BN_, int WGM_, int WGN_>
struct TileCfg {
  static constexpr int BM = BM_, BN = BN_, BK = 64, WGM = WGM_, WGN = WGN_;
  static constexpr int NWAVES = WGM * WGN;
  static constexpr int NTHREADS = 64 * NWAVES;
  static constexpr int WTM = BM / WGM, WTN = BN / WGN;  // wavefront tile
  static constexpr int MI = WTM / 32, NI = WTN / 32;    // 32x32 sub-tiles per wavefront
  static constexpr int A_PANEL = BM * BK * 2, B_PANEL = BN * BK * 2;   // bytes per stage
  static constexpr int A_LOADS = A_PANEL / 1024 / NWAVES;              // wave-level 1 KB direct loads
  static constexpr int B_LOADS = B_PANEL / 1024 / NWAVES;
  static constexpr int STAGE_BYTES = A_PANEL + B_PANEL;
  static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
  static_assert(BM % (32 * WGM) == 0 && BN % (32 * WGN) == 0, "wave tile must be 32-aligned");
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

// One wave-level direct load: lane i's 16 bytes at `src` land at LDS byte address lds + 16*i
// (lds must be wavefront-uniform; it travels in M0).  Written as inline asm on purpose: the
// compiler's wait-count pass, when it knows of an outstanding direct load, puts a full
// vmcnt(0) wait before every transposing LDS read, which would serialise the pipeline.  All
// waits on these loads are explicit (wait_all_and_barrier).
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"   // M0 is reserved; naming it tells the compiler it changes
__device__ __forceinline__ void direct_load_16(const char* src, uint32_t lds) {
  asm volatile("s_mov_b32 m0, %1\n s_nop 0\n global_load_lds_dwordx4 %0, off" ::"v"(src), "s"(lds) : "memory", "m0");
}
#pragma clang diagnostic pop
__device__ __forceinline__ uint32_t lds_address(const char* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)p;
}

// One operand panel: where its direct loads come from and how its MFMA fragments are read.
//   KM = false: global [rows][k] with row stride ld; rows past `nrows` are clamped to the last one.
//   KM = true:  global [k][rows] with row stride ld; 8-column chunks past `nrows` are clamped
//               (nrows - r0 must be a multiple of 8).
// Either way k >= Kdim reads as zero and the caller masks results of clamped rows.
//   LOADS = wave-level loads per stage, NSUB = 32-row sub-tiles per wavefront, WT = wavefront
//   tile extent, wpos = the wavefront's index along this operand's rows.
template <bool KM, int LOADS, int NSUB, int WT, int NWAVES>
struct Panel {
  const char* base;      // first byte of the tile's (row r0, k 0) / (k 0, column r0)
  int64_t kstride;       // bytes per stage of 64 k
  int kdim;              // k extent of this operand (KC: a multiple of 8); k >= kdim reads as zero
  uint32_t off[LOADS];   // this lane's byte offset inside a stage, per load
  int kch[LOADS];        // KC: k chunk (0..7) the lane loads; KM: k row (0..63) the lane loads
  uint32_t rd_base;      // this lane's fragment read offset inside the panel
  uint32_t rd_sub[NSUB]; // KM only: swizzled column-chunk offset per sub-tile

  __device__ __forceinline__ void init(const __bf16* X, int64_t ld, int r0, int nrows, int kdim_, int wave,
                                       int wpos) {
    const int lane = threadIdx.x & 63;
    kdim = kdim_;
    if constexpr (!KM) {
      base = reinterpret_cast<const char*>(X + (int64_t)r0 * ld);
      kstride = 128;
      const int rin = lane >> 3, cpos = lane & 7;
#pragma unroll
      for (int j = 0; j < LOADS; ++j) {
        const int row = 8 * (wave + NWAVES * j) + rin;
        kch[j] = cpos ^ ((row >> 1) & 7);
        off[j] = (uint32_t)((int64_t)min(row, nrows - 1 - r0) * ld * 2 + kch[j] * 16);
      }
      // sub-tile strides are multiples of 32 rows, so the row part of the swizzle is a lane constant
      rd_base = (uint32_t)((wpos * WT + (lane & 31)) * 128);
    } else {
      base = reinterpret_cast<const char*>(X + r0);
      kstride = 64 * ld * 2;
      const int last = (nrows - r0) / 8 - 1;   // last valid 8-column chunk of this tile
#pragma unroll
      for (int j = 0; j < LOADS; ++j) {
        const int krow = 2 * (wave + NWAVES * j) + (lane >> 5);
        const int ch = (lane & 31) ^ ((krow & 3) << 2);
        kch[j] = krow;
        off[j] = (uint32_t)((int64_t)krow * ld * 2 + min(ch, last) * 16);
      }
      // lane j of a 16-lane group addresses row (k0 + j/4), columns 4*(j%4)..+3 of the group's
      // 16 columns; groups 0/1 take columns 0-15 / 16-31, groups 2/3 the next 8 k
      const int j = lane & 15, mhalf = (lane >> 4) & 1, khalf = lane >> 5;
      rd_base = (uint32_t)((khalf * 8 + (j >> 2)) * 512 + (j & 1) * 8);
#pragma unroll
      for (int s = 0; s < NSUB; ++s) {
        const int c = (wpos * WT + s * 32) / 8 + mhalf * 2 + ((j & 3) >> 1);
        rd_sub[s] = (uint32_t)((c ^ ((j >> 2) << 2)) * 16);
      }
    }
  }

  // half h (0/1) of the direct loads of stage kt into the LDS panel at `dst`
  __device__ __forceinline__ void issue_half(int kt, int h, bool full, char* dst, int wave) const {
    const char* src0 = base + (int64_t)kt * kstride;
    const char* z = reinterpret_cast<const char*>(g_zero16);
#pragma unroll
    for (int j = 0; j < LOADS / 2; ++j) {
      const int jj = h * (LOADS / 2) + j;
      const char* src = src0 + off[jj];
      if (!full) {
        const int k = KM ? kt * 64 + kch[jj] : kt * 64 + kch[jj] * 8;
        if (k >= kdim) src = z;
      }
      direct_load_16(src, __builtin_amdgcn_readfirstlane(lds_address(dst) + (wave + NWAVES * jj) * 1024));
    }
  }

  // fragment of sub-tile s for k step kk (16 k) of the stage whose panel starts at `p`
  __device__ __forceinline__ bf16x8 read_one(const char* p, int kk, int koff_kc, int s) const {
    if constexpr (!KM) {
      return *reinterpret_cast<const bf16x8*>(p + rd_base + s * 32 * 128 + koff_kc);
    } else {
      const char* q = p + rd_base + rd_sub[s] + kk * 16 * 512;
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(q));
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(q + 4 * 512));
      const __attribute__((ext_vector_type(8))) short v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
      return __builtin_bit_cast(bf16x8, v);
    }
  }
};

// One BM x BN contraction over k < max(KA, KB), where operand A is zero for k >= KA and B
// for k >= KB (normally KA == KB; they differ when one operand's buffer is zero-padded in k
// and the other's simply ends).  Strides must be multiples of 8 elements, the bases 16-byte
// aligned, m0 < M, n0 < N; for a k-contiguous operand its k extent must be a multiple of 8,
// for a k-major operand its row extent (M - m0 or N - n0).
//
// prefetch(): issue stage 0 early (LDS must be free: all wavefronts past their last read);
// run(acc, true) then skips it.  Used to overlap a tile's first loads with the previous
// tile's epilogue.  On return from run() every wavefront has passed a barrier after its
// last LDS read: LDS is free.
template <class C, bool AKM = false, bool BKM = false>
struct GemmNT {
  static_assert((!AKM || C::BM == 256) && (!BKM || C::BN == 256),
                "the k-major panel addressing assumes 512-byte panel rows");
  Panel<AKM, C::A_LOADS, C::MI, C::WTM, C::NWAVES> pa;
  Panel<BKM, C::B_LOADS, C::NI, C::WTN, C::NWAVES> pb;
  char* smem;
  int kfull, nk, wave;   // kfull: k below which both operands are plain data

  __device__ __forceinline__ GemmNT(const __bf16* __restrict__ A, int64_t lda, int m0, int M, int KA,
                                    const __bf16* __restrict__ B, int64_t ldb, int n0, int N, int KB,
                                    char* smem_)
      : smem(smem_) {
    wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    pa.init(A, lda, m0, M, KA, wave, wave % C::WGM);
    pb.init(B, ldb, n0, N, KB, wave, wave / C::WGM);
    kfull = min(KA, KB);
    nk = (max(KA, KB) + 63) / 64;
  }

  __device__ __forceinline__ void issue_half(int kt, int h, bool full) const {
    char* s = smem + (kt & 1) * C::STAGE_BYTES;
    pa.issue_half(kt, h, full, s, wave);
    pb.issue_half(kt, h, full, s + C::A_PANEL, wave);
  }

  __device__ __forceinline__ void prefetch() const {
    issue_half(0, 0, false);
    issue_half(0, 1, false);
  }

  __device__ __forceinline__ void run(f32x16 (&acc)[C::MI][C::NI], bool prefetched = false) const {
    const int lane = threadIdx.x & 63;
    const int swz = ((lane & 31) >> 1) & 7;
    int koff[4];   // k-contiguous panels: swizzled byte offset of the lane's k chunk per k step
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) koff[kk] = ((kk * 2 + (lane >> 5)) ^ swz) * 16;

    bf16x8 fa0[C::MI], fb0[C::NI], fa1[C::MI], fb1[C::NI];
    auto read_frags = [&](int kt, int kk, bf16x8 (&fa)[C::MI], bf16x8 (&fb)[C::NI]) {
      const char* s = smem + (kt & 1) * C::STAGE_BYTES;
      // in the order the MFMAs of the k step want them: column 0's B fragment, the A fragments, the other
      // B fragments (LDS reads return in order, so the first MFMA waits for two reads, not for all)
      fb[0] = pb.read_one(s + C::A_PANEL, kk, koff[kk], 0);
#pragma unroll
      for (int i = 0; i < C::MI; ++i) fa[i] = pa.read_one(s, kk, koff[kk], i);
#pragma unroll
      for (int i = 1; i < C::NI; ++i) fb[i] = pb.read_one(s + C::A_PANEL, kk, koff[kk], i);
    };
    // MFMAs number lo..hi-1 of the MI x NI grid, numbered column by column in a serpentine (down
    // column 0, up column 1, ...): consecutive MFMAs always share an operand register set, which
    // measured ~2 % faster than row-major issue on this power-limited part.
    auto mma_sel = [&](bf16x8 (&fa)[C::MI], bf16x8 (&fb)[C::NI], int lo, int hi) {
#pragma unroll
      for (int ni = 0; ni < C::NI; ++ni)
#pragma unroll
        for (int i = 0; i < C::MI; ++i) {
          const int mi = (ni & 1) ? C::MI - 1 - i : i;
          if (ni * C::MI + i >= lo && ni * C::MI + i < hi)
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[mi], fb[ni], acc[mi][ni], 0, 0, 0);
        }
    };
    constexpr int NM = C::MI * C::NI;

    // One stage = four k steps.  The instruction order is pinned with scheduling barriers:
    //   first MFMA of a k step | (next stage's loads,) LDS reads of the next k step interleaved with its
    //   other MFMAs
    // so that every LDS read has a k step of MFMAs to land under.  In the last k step most of
    // the MFMAs run, then the barrier (next stage landed for everyone, this stage's buffer free),
    // then the first reads of the next stage under the remaining MFMA(s).
#define PARD2_SB __builtin_amdgcn_sched_barrier(0)
// The last k step's MFMAs are split around the stage barrier: all but PARD2_AFTER_BARRIER of them are
// issued before it.  One MFMA after the barrier measured best (it covers the next stage's first LDS
// reads, and a late barrier leaves every wavefront's loads the longest time to land): 14.95 -> 14.76 ms
// per step against an even split, 15.05 ms with none.
#ifndef PARD2_AFTER_BARRIER
#define PARD2_AFTER_BARRIER 1
#endif
#ifndef PARD2_LEAD
#define PARD2_LEAD 1   /* MFMAs of a k step issued before the next k step's LDS reads */
#endif
// Inside a k step the LDS reads of the next k step are spread between this k step's MFMAs (one read,
// one MFMA, ...) instead of being issued in one burst: all eight wavefronts run the same phase of the
// loop at the same time, and a burst from each of them queues up at the LDS behind the direct loads'
// writes.  Spreading measured 14.83 -> 14.42 ms per step (dW, whose operands take two transposing reads
// per fragment, gains most).  PARD2_INTERLEAVE = LDS reads per MFMA in that pattern; 0 = burst.
#ifndef PARD2_INTERLEAVE
#define PARD2_INTERLEAVE 1
#endif
#if PARD2_INTERLEAVE > 0
#define PARD2_MIXSB
#define PARD2_G(mask, n) __builtin_amdgcn_sched_group_barrier(mask, n, 0)
#define PARD2_G1 PARD2_G(0x100, PARD2_INTERLEAVE); PARD2_G(0x008, 1)   /* DS reads, then one MFMA */
#define PARD2_MIX PARD2_G1; PARD2_G1; PARD2_G1; PARD2_G1; PARD2_G1; PARD2_G1; PARD2_G1; PARD2_G1   /* MI + NI <= 8 reads */
#else
#define PARD2_MIXSB PARD2_SB
#define PARD2_MIX
#endif
#define PARD2_LAST_A mma_sel(fa1, fb1, 0, NM - PARD2_AFTER_BARRIER)
#define PARD2_LAST_B mma_sel(fa1, fb1, NM - PARD2_AFTER_BARRIER, NM)
#define PARD2_STAGE(ISSUE0, ISSUE1, HAS_NEXT)                                                             \
  mma_sel(fa0, fb0, 0, PARD2_LEAD); PARD2_SB; ISSUE0; read_frags(kt, 1, fa1, fb1); PARD2_MIXSB; mma_sel(fa0, fb0, PARD2_LEAD, NM); PARD2_MIX; PARD2_SB; \
  mma_sel(fa1, fb1, 0, PARD2_LEAD); PARD2_SB; ISSUE1; read_frags(kt, 2, fa0, fb0); PARD2_MIXSB; mma_sel(fa1, fb1, PARD2_LEAD, NM); PARD2_MIX; PARD2_SB; \
  mma_sel(fa0, fb0, 0, PARD2_LEAD); PARD2_SB;         read_frags(kt, 3, fa1, fb1); PARD2_MIXSB; mma_sel(fa0, fb0, PARD2_LEAD, NM); PARD2_MIX; PARD2_SB; \
  PARD2_LAST_A; PARD2_SB; wait_all_and_barrier(); PARD2_SB;                                               \
  if (HAS_NEXT) read_frags(kt + 1, 0, fa0, fb0);                                                          \
  PARD2_SB; PARD2_LAST_B; PARD2_SB;

    if (!prefetched) prefetch();
    wait_all_and_barrier();
    read_frags(0, 0, fa0, fb0);

    int kt = 0;
    const int nfull = kfull / 64;   // stages 0 .. nfull-1 need no k checks
    for (; kt + 1 < nfull; ++kt) {
      PARD2_STAGE(issue_half(kt + 1, 0, true), issue_half(kt + 1, 1, true), true)
    }
    for (; kt < nk - 1; ++kt) {     // the last stage(s) may be partial in k
      PARD2_STAGE(issue_half(kt + 1, 0, false), issue_half(kt + 1, 1, false), true)
    }
    {
      PARD2_STAGE((void)0, (void)0, false)
    }
#undef PARD2_STAGE
#undef PARD2_MIX
#undef PARD2_MIXSB
#undef PARD2_G1
#undef PARD2_G
#undef PARD2_LAST_A
#undef PARD2_LAST_B
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
