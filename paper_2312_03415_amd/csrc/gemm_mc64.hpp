// Matrix-core kernel with a K tile of 64 for the large contractions of the LoRA layer (X W, dY W^T, X^T dY and
// their K-concatenated forms [X|T][W;B], [dY|Z1][W^T;A^T]; Eq. 1 / Eq. 3 and Algorithms 1-5 of arxiv 2312.03415)
// in bf16 / fp16 on gfx950.  Same contract as gemm_mc_kernel (gemm_mc.hpp), which it replaces wherever it applies.
//
// Why a second kernel.  Counters and a bare-MFMA probe name two costs of gemm_mc_kernel on this power-limited chip:
//  - back-to-back v_mfma_f32_16x16x32 (one wave per SIMD, operands in registers, N(0,1)-like data) sustain 1.8-1.9
//    PFLOP/s, v_mfma_f32_32x32x16 about a sixth less in the same loop (2.4 on zeros either way): the 16x16 form reads
//    and writes a quarter of the accumulator registers per instruction and adds 32 products into each, so it moves
//    fewer register bytes and does half as many fp32 accumulator updates per FLOP.
//  - With a K tile of 32 a row of a K-contiguous operand tile is 64 bytes: half a 128-byte cache line per request to
//    L2 (33.7 M requests for 8192 x 4096 x 4096 where the bytes need 16.8 M), and one workgroup barrier, one wait and
//    one step of the load cursor per 32 MFMAs' worth of work.
// Here a K tile is 64 (every row of a K-contiguous tile is one whole line) and the products are 16x16x32.
//
// Shape of the kernel
//  - 256x256 output tile per workgroup, 4 wavefronts (one per SIMD) with a 128x128 sub-tile each: 8 x 8 accumulator
//    blocks of 16x16 in 256 registers, operand fragments (8 + 8 per K step of 32) double-buffered in the other half
//    of the register file.
//  - LDS: two stages of 64 KB (A 256x64 + B 256x64), filled by 16-byte LDS-DMA loads (global memory straight to LDS),
//    and 32 KB behind them for the epilogue.  A K tile is two K steps of 64 MFMAs.  K step 0 is MFMAs and the
//    fragment reads of K step 1 only.  K step 1 carries everything else: behind its first MFMA the wave waits for its
//    own loads of the next tile (all of them: nothing younger is in flight), then the workgroup barrier (the next
//    tile has landed for everyone; everyone has read the last fragments of this tile, which were fetched during K
//    step 0); behind the following MFMAs come the next tile's first fragments and the 16 loads that refill this
//    tile's stage with the tile after the next, one load behind every fourth MFMA.  A load thus has about a K tile
//    (64 to 128 MFMAs) to land; cycle counters read in the kernel show no time lost in that wait or at the barrier.
//  - The load stream is continuous over everything a persistent workgroup does (one workgroup per compute unit
//    walks output tiles): the next output tile's first K tiles arrive while the current one is being stored.
//  - A partial K tile (K % 64 != 0, e.g. the rank-r segment) takes the same route: its out-of-range 16-byte chunks
//    are fetched from an in-range address of the same row and the fragment registers that hold k >= K are zeroed
//    on both operands after the LDS read.
//  - LDS-DMA writes lane l's 16 bytes at base + 16 l, so rows cannot be padded; bank conflicts are avoided by an
//    XOR swizzle applied on the global-address side:
//      K-contiguous tile [256 rows][8 chunks]     : chunk c of row q sits in slot c ^ ((q >> 1) & 7)
//      K-strided tile    [64 k-rows][32 chunks]   : chunk c of k-row q sits in slot c ^ (4 (q & 3))
//  - Epilogues: as in gemm_mc.hpp (rows staged through wave-private LDS so that whole 128-byte lines are stored),
//    with 8 KB of staging per wave.
#pragma once
#include <type_traits>
#include <utility>

#include "gemm_mc.hpp"

namespace rl {

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>): a loop whose index is a constant in every
// iteration whatever the optimiser's unrolling limits (register arrays must never be indexed by a run-time value)
template <int... Is, typename F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, Is...>, F&& f) {
  (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(std::make_integer_sequence<int, N>{}, static_cast<F&&>(f));
}

// acc[16 x 16] += rowop (16 rows x 32 k) * colop (32 k x 16 columns): lane l carries row / column l % 16 and the
// eight k 8 (l / 16) .. + 7; it receives column l % 16, rows 4 (l / 16) .. + 3
// Issued through inline assembly with the accumulator tied to the result: the 64 accumulator blocks fill the 256
// accumulation registers exactly, and the compiler, free to give the builtin's result a register tuple of its own,
// would need a 65th and starts copying blocks between the two register files around every MFMA.  Nothing the
// compiler generates reads an accumulator within the hazard window of an MFMA: the epilogue reads them in the order
// they were last written, 64 MFMAs apart.
template <typename T> struct Elem16;
template <> struct Elem16<__bf16> {
  static __device__ __forceinline__ void mma(f32x4& acc, i32x4 rowop, i32x4 colop) {
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(rowop), "v"(colop));
  }
};
template <> struct Elem16<_Float16> {
  static __device__ __forceinline__ void mma(f32x4& acc, i32x4 rowop, i32x4 colop) {
    asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+a"(acc) : "v"(rowop), "v"(colop));
  }
};

template <int AL, int BL>
struct Mc64Tile {
  static constexpr int BM = 256, BN = 256, BK = 64, NS = 2;
  static constexpr int NW = 4, NT = NW * 64;
  static constexpr bool A_STR = (AL == 1), B_STR = (BL == 0);
  static constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2;
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  static constexpr int LDS_BYTES = NS * STAGE_BYTES;
  static constexpr int STAGING_BYTES = 32 * 1024;    // epilogue: 8 KB per wave
  static constexpr int IPW = (A_BYTES / 1024) / NW;  // 1 KB LDS-DMA instructions per wave per operand tile (8)
  static constexpr int LPT = 2 * IPW;                // loads per K tile per wave
  static_assert(LDS_BYTES + STAGING_BYTES <= 160 * 1024, "LDS budget");
  static_assert(IPW == 8, "two groups of four loads per operand tile and wave, each group sharing one LDS base");
};

// PLAIN (decided on the host): M and N are multiples of the tile and
//   1: the launch has no addend, bias, scale, mask or split: every tile takes the short 16-bit epilogue;
//   2: the launch is a split contraction: every tile writes fp32 partials;
//   0: everything else (general epilogue).
template <typename T, int AL, int BL, int PLAIN>
__device__ __forceinline__ void gemm_mc64_body(const GemmArgs& g) {
  using P = Mc64Tile<AL, BL>;
  constexpr int BM = P::BM, BN = P::BN, BK = P::BK, IPW = P::IPW;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem_raw[];
  unsigned char* smem = smem_raw;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int s16 = lane & 15;

  // K tiles of one output tile: segment 0 then segment 1; the last tile of a segment may be partial
  const int nt0 = (g.K[0] + BK - 1) / BK, nt1 = (g.K[1] + BK - 1) / BK;
  const int ntk = nt0 + nt1;
  const int total = g.nbm * g.nbn;
  const int nwork = total * g.splits;  // work item w = split * total + tile sequence number

  // tile sequence number -> (m0, n0): each XCD (own L2) works on a contiguous run of tiles, walked in bands of 8
  // tile rows (see gemm_mc.hpp)
  auto tile_origin = [&](int seq, int& m0, int& n0) {
    int id;
    {
      const int x = seq & 7, slot = seq >> 3, q = total >> 3, rem = total & 7;
      id = x * q + (x < rem ? x : rem) + slot;
    }
    constexpr int BAND = 8;
    const int per_band = BAND * g.nbn;
    const int band = id / per_band, first_m = band * BAND;
    const int band_rows = (g.nbm - first_m) < BAND ? (g.nbm - first_m) : BAND;
    const int in_band = id - band * per_band;
    m0 = (first_m + in_band % band_rows) * BM;
    n0 = (in_band / band_rows) * BN;
  };
  auto split_range = [&](int w, int& tile_seq, int& split, int& u0, int& u1) {
    split = w / total;
    tile_seq = w - split * total;
    u0 = split * g.tiles_per_split;
    u1 = u0 + g.tiles_per_split;
    if (u1 > ntk) u1 = ntk;
  };

  // ---- load cursor: which K tile of which work item the next LDS-DMA batch fetches -----------------
  const int K0 = g.K[0], K1 = g.K[1];
  const T* const segA0 = static_cast<const T*>(g.A[0]);
  const T* const segA1 = static_cast<const T*>(g.A[1]);
  const T* const segB0 = static_cast<const T*>(g.B[0]);
  const T* const segB1 = static_cast<const T*>(g.B[1]);
  const uint32_t lda0 = (uint32_t)g.lda[0], lda1 = (uint32_t)g.lda[1];
  const uint32_t ldb0 = (uint32_t)g.ldb[0], ldb1 = (uint32_t)g.ldb[1];
  int cw = blockIdx.x, cu = 0, cu_end = 0, cm0 = 0, cn0 = 0, cnext = 0;
  bool clive = true;
  auto extent_bytes = [&](bool strided, int rows_or_cols, int K, uint32_t ld) -> uint32_t {
    if (K <= 0) return 0u;
    const uint64_t e = strided ? ((uint64_t)(K - 1) * ld + (uint64_t)rows_or_cols) : ((uint64_t)(rows_or_cols - 1) * ld + (uint64_t)K);
    return (uint32_t)(e * 2u);
  };
  // Four loads share one LDS base (M0) and differ in the instruction's immediate offset (0, 1, 2, 3 KB), which the
  // hardware adds to the LDS address and to the memory address alike.  The memory side is compensated in the
  // per-lane offsets; to keep those non-negative the descriptors start kBias bytes before the matrix (address
  // arithmetic only: every address actually formed lies inside the matrix).
  constexpr uint32_t kBias = 3 * 1024;
  auto make_rsrc = [&](const T* base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<unsigned char*>(const_cast<T*>(base)) - kBias, 0,
                                             bytes ? bytes + kBias : 0u, 0x00020000);
  };
  const __amdgpu_buffer_rsrc_t rsA0 = make_rsrc(segA0, extent_bytes(P::A_STR, g.M, K0, lda0));
  const __amdgpu_buffer_rsrc_t rsA1 = make_rsrc(segA1, extent_bytes(P::A_STR, g.M, K1, lda1));
  const __amdgpu_buffer_rsrc_t rsB0 = make_rsrc(segB0, extent_bytes(P::B_STR, g.N, K0, ldb0));
  const __amdgpu_buffer_rsrc_t rsB1 = make_rsrc(segB1, extent_bytes(P::B_STR, g.N, K1, ldb1));
  __amdgpu_buffer_rsrc_t rsA = rsA0, rsB = rsB0;  // descriptors of the cursor's segment
  uint32_t kA = 0, kB = 0;            // byte offset of the cursor's tile (k origin) in its segment (uniform)
  uint32_t stepA = 0, stepB = 0;      // bytes from one K tile to the next in the current segment
  uint32_t offA[IPW], offB[IPW];      // per-lane byte offsets, one per instruction

  // Rebuild the state for tile cu of work item cw (tile origin cm0, cn0).  Rows / columns beyond the matrix are
  // clamped: they only feed outputs that are never stored.  In a partial tile the chunks with k >= kvalid are
  // fetched from k = 0 of the same row / column (in range); the multiply zeroes them.
  auto cursor_setup = [&]() {
    const int seg = cu < nt0 ? 0 : 1;
    const int ts = cu - (seg ? nt0 : 0);
    const int kvalid = (seg ? K1 : K0) - ts * BK;
    const uint32_t lda = seg ? lda1 : lda0, ldb = seg ? ldb1 : ldb0;
    stepA = 2u * (P::A_STR ? (uint32_t)BK * lda : (uint32_t)BK);
    stepB = 2u * (P::B_STR ? (uint32_t)BK * ldb : (uint32_t)BK);
    rsA = seg ? rsA1 : rsA0;
    rsB = seg ? rsB1 : rsB0;
    kA = (uint32_t)ts * stepA;
    kB = (uint32_t)ts * stepB;
#pragma unroll
    for (int j = 0; j < IPW; ++j) {
      const int p = (wave * IPW + j) * 64 + lane;   // 16-byte slot of the operand tile this lane fills
      {
        const int row = P::A_STR ? (p >> 5) : (p >> 3);
        const int col = P::A_STR ? (((p & 31) ^ (4 * (row & 3))) << 3) : (((p & 7) ^ ((row >> 1) & 7)) << 3);
        if constexpr (!P::A_STR) {
          int gr = cm0 + row; gr = gr < g.M ? gr : g.M - 1;
          offA[j] = 2u * ((uint32_t)gr * lda + (uint32_t)(col < kvalid ? col : 0)) + (kBias - 1024u * (j & 3));
        } else {
          int gc = cm0 + col; gc = gc < g.M ? gc : g.M - 8;
          offA[j] = 2u * ((uint32_t)(row < kvalid ? row : 0) * lda + (uint32_t)gc) + (kBias - 1024u * (j & 3));
        }
      }
      {
        const int row = P::B_STR ? (p >> 5) : (p >> 3);
        const int col = P::B_STR ? (((p & 31) ^ (4 * (row & 3))) << 3) : (((p & 7) ^ ((row >> 1) & 7)) << 3);
        if constexpr (!P::B_STR) {
          int gr = cn0 + row; gr = gr < g.N ? gr : g.N - 1;
          offB[j] = 2u * ((uint32_t)gr * ldb + (uint32_t)(col < kvalid ? col : 0)) + (kBias - 1024u * (j & 3));
        } else {
          int gc = cn0 + col; gc = gc < g.N ? gc : g.N - 8;
          offB[j] = 2u * ((uint32_t)(row < kvalid ? row : 0) * ldb + (uint32_t)gc) + (kBias - 1024u * (j & 3));
        }
      }
    }
    // the next tile index at which the state must be rebuilt again
    if (kvalid < BK) {
      cnext = cu + 1;  // offsets of a partial tile are its own
    } else {
      cnext = cu_end;
      if (cu < nt0 && nt0 < cnext) cnext = nt0;                                 // segment switch
      if ((K0 % BK) != 0 && cu < nt0 - 1 && nt0 - 1 < cnext) cnext = nt0 - 1;  // partial tail of segment 0
      if ((K1 % BK) != 0 && ntk - 1 < cnext) cnext = ntk - 1;                  // partial tail of segment 1
    }
  };
  auto cursor_open = [&]() {  // start loading work item cw
    int seq, split;
    split_range(cw, seq, split, cu, cu_end);
    tile_origin(seq, cm0, cn0);
    cursor_setup();
  };
  cursor_open();

  // Load j (0..15) of the cursor's K tile into stage `st`: 0..7 the A half, 8..15 the B half.  j must be a
  // constant after unrolling: it selects the immediate offset.
  auto issue_load = [&](int st, auto j_c) {
    constexpr int j = decltype(j_c)::value;
    constexpr bool isB = j >= IPW;
    constexpr int jj = j & (IPW - 1);
    unsigned char* dst = smem + st * P::STAGE_BYTES + (isB ? P::A_BYTES : 0) + wave * (IPW * 1024) + (jj >> 2) * 4096;
    const uint32_t uk = __builtin_amdgcn_readfirstlane(isB ? kB : kA);  // wave-uniform: keeps the load free of a per-lane loop
    const __amdgpu_buffer_rsrc_t rs = isB ? rsB : rsA;
    const uint32_t off = isB ? offB[jj] : offA[jj];
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (mc_lds_void_t*)dst, 16, off, uk, (jj & 3) * 1024, 0);
  };
  // Move the cursor on.  Past the last work item it stays on the last tile, which is then fetched again (into a
  // stage nobody reads): the loop below issues the same loads in every K tile.
  auto cursor_event = [&]() {  // cu has just reached cnext: next work item, the end of all work, or a rebuild
    if (cu == cu_end) {
      if (cw + (int)gridDim.x < nwork) {
        cw += gridDim.x;
        cursor_open();
      } else {
        clive = false;
        --cu;
        kA -= stepA;  // stay on the last tile
        kB -= stepB;
      }
      return;
    }
    cursor_setup();
  };
  auto cursor_advance = [&]() {
    const bool live = clive;
    cu += live ? 1 : 0;
    kA += live ? stepA : 0u;
    kB += live ? stepB : 0u;
    if (__builtin_expect(live && cu == cnext, 0)) cursor_event();
  };

  // ---- fragment addresses (bytes inside a stage, stage 0) -------------------------------------------
  // MFMA 16x16x32: lane l carries row (or column) l % 16 of its 16-wide block and the eight k 8 (l / 16) .. + 7 of the
  // K step.  grp = l / 16.
  // K-contiguous tile: row q is 128 bytes; the 16 bytes at k = 32 ks + 8 grp live in slot (4 ks + grp) ^ ((q >> 1) & 7);
  //   block b of the wave's 128 rows is 16 rows = 2048 bytes further on (immediate offset).
  // K-strided tile: transposing 8-byte LDS load: within its 16-lane group lane s points at k-row 32 ks + 8 grp + s / 4
  //   (+ 4 for the second load), columns c0 + 4 (s % 4) .. + 3, and receives column c0 + s for four consecutive k.
  //   Block b of the wave's 128 columns: 16-byte chunk (16 w + 2 b + (s % 4) / 2) ^ 4 (s / 4), one address per block.
  const int grp = lane >> 4;
  uint32_t fragA[8], fragB[8];
  {
    const int sw = (s16 >> 1) & 7;
    if constexpr (!P::A_STR) {
      const uint32_t rowb = (uint32_t)(wm * 128 + s16) * 128u;
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) fragA[ks] = rowb + (uint32_t)(((4 * ks + grp) ^ sw) << 4);
    } else {
      const int k = s16 >> 2;
#pragma unroll
      for (int b = 0; b < 8; ++b)
        fragA[b] = (uint32_t)((8 * grp + k) * 512 + ((wm * 16 + 2 * b + ((s16 & 3) >> 1)) ^ (4 * k)) * 16 + 8 * (s16 & 1));
    }
    if constexpr (!P::B_STR) {
      const uint32_t rowb = (uint32_t)(wn * 128 + s16) * 128u;
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) fragB[ks] = P::A_BYTES + rowb + (uint32_t)(((4 * ks + grp) ^ sw) << 4);
    } else {
      const int k = s16 >> 2;
#pragma unroll
      for (int b = 0; b < 8; ++b)
        fragB[b] = P::A_BYTES +
                   (uint32_t)((8 * grp + k) * 512 + ((wn * 16 + 2 * b + ((s16 & 3) >> 1)) ^ (4 * k)) * 16 + 8 * (s16 & 1));
    }
  }
  const uint32_t lds_base = (uint32_t)(uintptr_t)((mc_lds_void_t*)smem);

  // MFMA q uses A fragment q / 8 and B fragment q % 8, so A fragment i is dead behind MFMA 8 i + 7 and the next K
  // step's fragment i is read into the same registers right there: A fragments 0..6 are single-buffered.  Fragment 7,
  // which would be fetched behind the very last MFMA, and the B fragments, all live until the last MFMA, are
  // double-buffered; every read of a K step is then issued at least 8 MFMAs before the step ends.
  i32x4 fa[2][8], fb[2][8];  // (of fa[1] only fragment 7 is used)
#define FA(buf, i) fa[(i) == 7 ? (buf) : 0][i]
  // One 16-wide operand fragment of K step KSR from the stage at byte offset `soff` (all reads through inline
  // assembly: the compiler makes every LDS read it tracks wait for all outstanding LDS-DMA loads, which would
  // serialise the ring; reads it cannot see are waited for by hand, below).
  auto read_frag_op = [&](bool strided, const uint32_t (&fr)[8], uint32_t soff, auto blk_c, auto ksr_c) -> i32x4 {
    constexpr int KSR = decltype(ksr_c)::value, blk = decltype(blk_c)::value;
    if (!strided) {
      const uint32_t addr = lds_base + soff + fr[KSR];
      i32x4 out;  // 16 rows of 128 bytes per block
      asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(out) : "v"(addr), "i"(blk * 2048));
      return out;
    } else {
      const uint32_t addr = lds_base + soff + fr[blk];
      i32x2 lo, hi2;
      asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(lo) : "v"(addr), "i"(KSR * 16384));
      asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(hi2) : "v"(addr), "i"(KSR * 16384 + 2048));
      i32x4 out = {lo[0], lo[1], hi2[0], hi2[1]};
      return out;
    }
  };
  // everything the hand-issued LDS reads fetched for the K step that multiplies out of buffer `buf` has arrived
  auto wait_frags = [&](int buf) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(FA(buf, 0)), "+v"(FA(buf, 1)), "+v"(FA(buf, 2)), "+v"(FA(buf, 3)), "+v"(FA(buf, 4)), "+v"(FA(buf, 5)), "+v"(FA(buf, 6)), "+v"(FA(buf, 7)),
                   "+v"(fb[buf][0]), "+v"(fb[buf][1]), "+v"(fb[buf][2]), "+v"(fb[buf][3]), "+v"(fb[buf][4]), "+v"(fb[buf][5]),
                   "+v"(fb[buf][6]), "+v"(fb[buf][7]));
  };
  // zero the fragment registers of K step ks that hold k >= kvalid (this lane's 8 k start at 32 ks + 8 grp)
  auto mask_frags = [&](int buf, int ks, int kvalid) {
    if (ks * 32 + 8 * grp >= kvalid) {
#pragma unroll
      for (int a = 0; a < 8; ++a) FA(buf, a) = i32x4{0, 0, 0, 0};
#pragma unroll
      for (int b = 0; b < 8; ++b) fb[buf][b] = i32x4{0, 0, 0, 0};
    }
  };

  f32x4 acc[8][8];  // [row block][column block]; lane l: row l % 16, columns 4 (l / 16) .. + 3 of the block

#define MC_FENCE() __builtin_amdgcn_sched_barrier(0)
  // One K step of 32, in exactly this instruction order (a scheduling fence after every piece): 64 MFMAs out of the
  // A fragments and buffer `bufc` of the B fragments.  The next K step's fragments (K step KSR of the stage at
  // `soff`) are fetched behind them: A fragment i < 7 behind MFMA 8 i + 7, B fragments 0..7 behind MFMAs 8..15, A
  // fragment 7 behind MFMA 16.  An MFMA occupies the matrix core for 16 cycles and a wave issues at most one
  // instruction per 4, so up to three other instructions fit behind each.
  // SYNC: the wait for this wave's loads and LDS reads and the workgroup barrier run behind the first MFMA (the stage
  // the reads address is safe only after the barrier); `behind(q)` is called behind every MFMA (the loads that
  // refill the stage just released, the cursor's step).
  auto kstep = [&](auto ksr_c, auto sync_c, int bufc, int bufr, uint32_t soff, auto behind) {
    constexpr bool SYNC = decltype(sync_c)::value;
    wait_frags(bufc);
    MC_FENCE();
    static_for<64>([&](auto qc) {
      constexpr int q = decltype(qc)::value;
      Elem16<T>::mma(acc[q >> 3][q & 7], fb[bufc][q & 7], FA(bufc, q >> 3));
      MC_FENCE();
      if constexpr (SYNC && q == 0) {
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(mc_wait_imm(0, true));
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        MC_FENCE();
      }
      if constexpr ((q & 7) == 7 && q < 56) {
        fa[0][q >> 3] = read_frag_op(P::A_STR, fragA, soff, std::integral_constant<int, (q >> 3)>{}, ksr_c);
        MC_FENCE();
      }
      if constexpr (q >= 8 && q < 16) {
        fb[bufr][q - 8] = read_frag_op(P::B_STR, fragB, soff, std::integral_constant<int, q - 8>{}, ksr_c);
        MC_FENCE();
      }
      if constexpr (q == 16) {
        fa[bufr][7] = read_frag_op(P::A_STR, fragA, soff, std::integral_constant<int, 7>{}, ksr_c);
        MC_FENCE();
      }
      behind(qc);
    });
  };
  auto nothing = [](auto) {};

  // ---- prologue: both stages filled, the first tile landed for everyone, its first fragments in registers
  static_for<P::LPT>([&](auto j) { issue_load(0, j); });
  cursor_advance();
  static_for<P::LPT>([&](auto j) { issue_load(1, j); });
  cursor_advance();
  MC_FENCE();
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(mc_wait_imm(P::LPT, true));  // loads return in order: the older tile is in
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  MC_FENCE();
  {
    using K0c = std::integral_constant<int, 0>;
    static_for<8>([&](auto b) { fb[0][decltype(b)::value] = read_frag_op(P::B_STR, fragB, 0u, b, K0c{}); });
    static_for<8>([&](auto a) { fa[0][decltype(a)::value] = read_frag_op(P::A_STR, fragA, 0u, a, K0c{}); });
  }
  // the only K tiles that can be partial: the last one of each segment
  const int pu0 = (K0 % BK) != 0 ? nt0 - 1 : -1, pu1 = (K1 % BK) != 0 ? ntk - 1 : -1;
  int st = 0;  // stage of the tile being multiplied; runs on across work items

  for (int w = blockIdx.x; w < nwork; w += gridDim.x) {
    int seq, split, u0, u1, m0, n0;
    split_range(w, seq, split, u0, u1);
    tile_origin(seq, m0, n0);
    static_for<64>([&](auto e) { acc[decltype(e)::value >> 3][decltype(e)::value & 7] = f32x4{0.f, 0.f, 0.f, 0.f}; });

    for (int u = u0; u < u1; ++u) {
      const bool partial = (u == pu0) | (u == pu1);  // wave-uniform, rare
      const uint32_t soff = (uint32_t)(st * P::STAGE_BYTES), soffn = (uint32_t)((st ^ 1) * P::STAGE_BYTES);
      int kvalid = BK;
      if (__builtin_expect(partial, 0)) kvalid = u < nt0 ? K0 - u * BK : K1 - (u - nt0) * BK;
      auto mask = [&](int buf, int ks) {
        if (__builtin_expect(partial, 0)) {  // zero what lies beyond K
          MC_FENCE();
          wait_frags(buf);
          mask_frags(buf, ks, kvalid);
          MC_FENCE();
          asm volatile("s_nop 7");  // (the MFMAs that read the registers just written are not the compiler's to guard)
          MC_FENCE();
        }
      };
      mask(0, 0);
      kstep(std::integral_constant<int, 1>{}, std::false_type{}, 0, 1, soff, nothing);
      mask(1, 1);
      // K step 1: the next tile has landed and this tile's stage is free behind the barrier; the next tile's first
      // fragments, and the refill of this stage with the cursor's tile, one load behind every fourth MFMA of the whole K
      // step (the compute unit's address path takes about as long for the four waves' 64 loads as the waves take for a
      // K step: bunched more closely, the loads hold up the MFMAs behind them); the cursor moves on behind the last load
      kstep(std::integral_constant<int, 0>{}, std::true_type{}, 1, 0, soffn, [&](auto qc) {
        constexpr int q = decltype(qc)::value;
        if constexpr (q >= 2 && (q - 2) % 4 == 0) {
          issue_load(st, std::integral_constant<int, (q - 2) / 4>{});
          MC_FENCE();
        }
        if constexpr (q == 63) { cursor_advance(); MC_FENCE(); }
      });
      st ^= 1;
    }

    // ---- epilogue (the next work item's first tiles keep arriving meanwhile)
    asm volatile("s_nop 7\n\ts_nop 7");  // the last MFMAs' results, read by hand below
    if constexpr (PLAIN == 1) {
      // Row-contiguous stores: two row blocks (32 rows x 128 columns of this wave) at a time go through a private
      // 8 KB LDS area, row r at r * 256 bytes: 8-byte pieces in the accumulator layout in (a lane holds columns
      // 16 b + 4 grp .. + 3 of its row: piece 4 b + grp of 32; pairs of pieces are rotated by the row against bank
      // conflicts), 16-byte pieces of 4 rows x 256 bytes out, so that every store instruction writes whole lines.
      unsigned char* const stg = smem + P::LDS_BYTES + wave * 8192;
      const uint32_t stg_base = (uint32_t)(uintptr_t)((mc_lds_void_t*)stg);
      const int rr = lane >> 4, rc = lane & 15;              // read side: row within a group of 4, 16-byte chunk
      T* gp = static_cast<T*>(g.C) + (int64_t)(m0 + wm * 128 + rr) * g.ldc + (n0 + wn * 128 + rc * 8);
      typedef float f32x2_t __attribute__((ext_vector_type(2)));
      typedef T tx2_t __attribute__((ext_vector_type(2)));
      static_for<4>([&](auto a2c) {
        constexpr int a2 = decltype(a2c)::value;
        static_for<16>([&](auto ec) {
          constexpr int ah = decltype(ec)::value >> 3, b = decltype(ec)::value & 7, a = 2 * a2 + ah;
          const uint32_t row = (uint32_t)(16 * ah + s16);
          const uint32_t wr = stg_base + row * 256u;
          const uint32_t wsw = 2u * (row & 15u);
          float x0, x1, x2, x3;  // explicit reads at the point of use (see gemm_mc.hpp)
          asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x0) : "a"(acc[a][b][0]));
          asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x1) : "a"(acc[a][b][1]));
          asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x2) : "a"(acc[a][b][2]));
          asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x3) : "a"(acc[a][b][3]));
          const f32x2_t lo = {x0, x1}, hi2 = {x2, x3};
          i32x2 v = {(int)__builtin_bit_cast(unsigned, __builtin_convertvector(lo, tx2_t)),
                     (int)__builtin_bit_cast(unsigned, __builtin_convertvector(hi2, tx2_t))};
          const uint32_t slot = ((uint32_t)(4 * b + (grp & 2)) ^ wsw) + (uint32_t)(grp & 1);
          asm volatile("ds_write_b64 %0, %1" : : "v"(wr + slot * 8u), "v"(v) : "memory");
          __builtin_amdgcn_sched_barrier(0);
        });
        __builtin_amdgcn_sched_barrier(0);
        i32x4 o[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const int row = 4 * k + rr;
          const uint32_t addr = stg_base + (uint32_t)row * 256u + (((uint32_t)(2 * rc) ^ (2u * (uint32_t)(row & 15))) * 8u);
          asm volatile("ds_read_b128 %0, %1" : "=v"(o[k]) : "v"(addr) : "memory");
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          mc_wait_piece(k, o);
          *reinterpret_cast<i32x4*>(gp + (int64_t)(a2 * 32 + 4 * k) * g.ldc) = o[k];
          __builtin_amdgcn_sched_barrier(0);
        }
      });
    } else {
      // fp32 partials of a split contraction (PLAIN == 2), or the general epilogue (ragged tiles, addend, bias, scale,
      // mask, partials of a ragged split).  One row block (16 rows x 128 fp32 columns of this wave = 8 KB) at a time
      // passes through the wave's LDS area, row r at r * 512 bytes: 16-byte pieces in the accumulator layout in (piece
      // 4 b + grp of 32, rotated by the row against bank conflicts), two rows x 512 bytes per instruction out, so that
      // a lane owns four consecutive columns of one row: the unit of every option (one mask group, 8 bytes of
      // addend / bias / output, 16 bytes of partials), and a store instruction covers 2 rows x 256 bytes (512 of
      // partials).  Arithmetic and its order are store_block's: alpha, mask, + addend, + bias, one rounding.
      const Epilogue ep{g.C, g.ldc, g.D, g.ldd, g.partial, g.M, g.N, split, g.alpha, g.bias, g.drop_thr, g.drop_key, g.drop_cpr};
      unsigned char* const stg = smem + P::LDS_BYTES + wave * 8192;
      const uint32_t stg_base = (uint32_t)(uintptr_t)((mc_lds_void_t*)stg);
      const uint32_t wr = stg_base + (uint32_t)s16 * 512u;
      const int rr = lane >> 5, rc = lane & 31;
      const int n = n0 + wn * 128 + rc * 4;   // this lane's four columns (N is a multiple of 8: valid together)
      const bool n_ok = n < g.N;
      [[maybe_unused]] f32x4 bias4 = {0.f, 0.f, 0.f, 0.f};
      if constexpr (PLAIN == 0) {
        if (g.bias != nullptr && g.partial == nullptr && n_ok) {
          T b4[4];
          *reinterpret_cast<i32x2*>(b4) = *reinterpret_cast<const i32x2*>(static_cast<const T*>(g.bias) + n);
#pragma unroll
          for (int e = 0; e < 4; ++e) bias4[e] = (float)b4[e];
        }
      }
      static_for<8>([&](auto ac) {
        constexpr int a = decltype(ac)::value;
        static_for<8>([&](auto bc) {
          constexpr int b = decltype(bc)::value;
          float x0, x1, x2, x3;
          asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x0) : "a"(acc[a][b][0]));
          asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x1) : "a"(acc[a][b][1]));
          asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x2) : "a"(acc[a][b][2]));
          asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x3) : "a"(acc[a][b][3]));
          const f32x4 v = {x0, x1, x2, x3};
          const uint32_t slot = (uint32_t)(4 * b + grp) ^ (uint32_t)s16;
          asm volatile("ds_write_b128 %0, %1" : : "v"(wr + slot * 16u), "v"(v) : "memory");
          __builtin_amdgcn_sched_barrier(0);
        });
        f32x4 o[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const int row = 2 * k + rr;
          const uint32_t addr = stg_base + (uint32_t)row * 512u + (((uint32_t)rc ^ (uint32_t)row) * 16u);
          asm volatile("ds_read_b128 %0, %1" : "=v"(o[k]) : "v"(addr) : "memory");
        }
        // the addend's eight pieces are requested together, ahead of their use (one at a time, every piece would
        // wait out a trip to memory)
        [[maybe_unused]] i32x2 dq[8];
        if constexpr (PLAIN == 0) {
          if (g.D != nullptr && g.partial == nullptr) {
#pragma unroll
            for (int k = 0; k < 8; ++k) {
              const int m = m0 + wm * 128 + a * 16 + 2 * k + rr;
              dq[k] = (m < g.M && n_ok) ? *reinterpret_cast<const i32x2*>(static_cast<const T*>(g.D) + (int64_t)m * g.ldd + n) : i32x2{0, 0};
            }
          }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          mc_wait_piece(k, o);
          const int m = m0 + wm * 128 + a * 16 + 2 * k + rr;
          if constexpr (PLAIN == 2) {
            *reinterpret_cast<f32x4*>(g.partial + ((int64_t)split * g.M + m) * g.N + n) = o[k];
          } else {
            if (m < g.M && n_ok) {
              if (g.partial != nullptr) {
                *reinterpret_cast<f32x4*>(g.partial + ((int64_t)split * g.M + m) * g.N + n) = o[k];
              } else {
                f32x4 v = epilogue_scale(ep, o[k], m, n);
                if (g.D != nullptr) {
                  T d4[4];
                  *reinterpret_cast<i32x2*>(d4) = dq[k];
#pragma unroll
                  for (int e = 0; e < 4; ++e) v[e] += (float)d4[e];
                }
                if (g.bias != nullptr) v += bias4;
                T o4[4] = {from_f32<T>(v[0]), from_f32<T>(v[1]), from_f32<T>(v[2]), from_f32<T>(v[3])};
                *reinterpret_cast<i32x2*>(static_cast<T*>(g.C) + (int64_t)m * g.ldc + n) = *reinterpret_cast<const i32x2*>(o4);
              }
            }
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      });
    }
  }
  // the LDS-DMA writes still in flight target this workgroup's LDS: let them land before it is released
  __builtin_amdgcn_s_waitcnt(mc_wait_imm(0, true));
#undef MC_FENCE
#undef FA
}

template <typename T, int AL, int BL, int PLAIN>
__global__ __launch_bounds__(256, 1) void gemm_mc64_kernel(GemmArgs g) {
  gemm_mc64_body<T, AL, BL, PLAIN>(g);
}

}  // namespace rl
