// Matrix-core kernel for the large contractions of the LoRA layer (X W, dY W^T, X^T dY and their
// K-concatenated forms [X|T][W;B], [dY|Z1][W^T;A^T]; Eq. 1 / Eq. 3 and Algorithms 1-5 of arxiv
// 2312.03415) in bf16 / fp16 on gfx950.  Same contract as gemm_kernel (gemm_engine.hpp).
// Dense products run on its successor with a K tile of 64 (gemm_mc64.hpp), which includes this file for the helpers
// they share; this kernel remains the route of an int4 frozen weight (BQ) and tile id 6 of runlora_gemm.
//
// Shape of the kernel
//  - 256x256 output tile per workgroup, 4 wavefronts (one per SIMD), each owning a 128x128 sub-tile:
//    16 accumulator blocks of 32x32 = 256 accumulator registers, which leaves the other half of
//    the 512-entry register file for double-buffered operand fragments.  A K step (16) is
//    16 MFMAs fed by 8 LDS reads of 16 bytes: half the LDS traffic per MFMA of a 128x64 sub-tile.
//  - K tile = 32.  LDS is a ring of NS = 3 stages of 32 KB (A 256x32 + B 256x32; 4 and 5 stages measured the
//    same, and the LDS behind three stages holds the epilogue's staging area); global memory goes straight to
//    LDS (16-byte LDS-DMA loads, no register staging).  While one K tile is multiplied the next one has landed
//    and the one after it is in flight, so a load has ~2000 MFMA cycles to land.
//  - The load stream is continuous over everything a persistent workgroup does: when the K tiles
//    of one output tile are exhausted it goes on with the next output tile, so the first tiles of
//    the next output tile arrive while the current one is being stored.
//  - One s_barrier per K tile, placed behind the first MFMA of the tile's second K step.  It orders
//    "everyone has read stage s" before "stage s is refilled" and "my loads of tile t+1 have
//    landed" (s_waitcnt vmcnt(8 (NS-2)): the eight loads of a K tile per wave return in order, so at most one
//    tile's worth outstanding means tile t+1 is in) before "anyone reads tile t+1".
//  - A partial K tile (K % 32 != 0, e.g. the rank-r segment with r = 8 or 16) takes the same route:
//    its out-of-range 16-byte chunks are fetched from an in-range address of the same row and the
//    fragment registers that hold k >= K are zeroed on both operands after the LDS read.
//  - LDS-DMA writes lane l's 16 bytes at base + 16 l, so rows cannot be padded; bank conflicts are
//    avoided by an XOR swizzle applied on the global-address side:
//      K-contiguous tile [256 rows][4 chunks]     : chunk c of row q sits in slot c ^ ((q >> 2) & 3)
//      K-strided tile    [32 k-rows][32 chunks]   : chunk c of k-row q sits in slot c ^ (4 (q & 3))
#pragma once
#include <type_traits>

#include "gemm_engine.hpp"

namespace rl {

typedef __attribute__((address_space(3))) void mc_lds_void_t;
typedef __attribute__((address_space(1))) const void mc_global_cvoid_t;

template <int AL, int BL, int NS_>
struct McTile {
  static constexpr int BM = 256, BN = 256, BK = 32, NS = NS_;
  static constexpr int NW = 4, NT = NW * 64;
  static constexpr int WTM = 128, WTN = 128, TM = 4, TN = 4;
  static constexpr bool A_STR = (AL == 1), B_STR = (BL == 0);
  static constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2;
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  static constexpr int LDS_BYTES = NS * STAGE_BYTES;
  static constexpr int IPW = (A_BYTES / 1024) / NW;  // 1 KB LDS-DMA instructions per wave per operand tile (4)
  static constexpr int LPT = 2 * IPW;                // loads per K tile per wave
  static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
  static_assert(IPW == 4, "four loads per operand tile and wave share one LDS base");
};

// s_waitcnt immediate: at most `vm` vector-memory operations outstanding; lgkm_zero = also wait for
// every LDS / scalar-memory operation; the export counter is left alone
constexpr int mc_wait_imm(int vm, bool lgkm_zero) {
  return (vm & 15) | (7 << 4) | ((lgkm_zero ? 0 : 15) << 8) | ((vm >> 4) << 14);
}

// Piece k of eight LDS reads issued back to back has arrived (LDS operations return in order; the count of
// s_waitcnt is an immediate, hence the switch, which unrolling resolves).
template <typename V>
__device__ __forceinline__ void mc_wait_piece(int k, V (&o)[8]) {
  switch (k) {
    case 0: asm volatile("s_waitcnt lgkmcnt(7)" : "+v"(o[0])); break;
    case 1: asm volatile("s_waitcnt lgkmcnt(6)" : "+v"(o[1])); break;
    case 2: asm volatile("s_waitcnt lgkmcnt(5)" : "+v"(o[2])); break;
    case 3: asm volatile("s_waitcnt lgkmcnt(4)" : "+v"(o[3])); break;
    case 4: asm volatile("s_waitcnt lgkmcnt(3)" : "+v"(o[4])); break;
    case 5: asm volatile("s_waitcnt lgkmcnt(2)" : "+v"(o[5])); break;
    case 6: asm volatile("s_waitcnt lgkmcnt(1)" : "+v"(o[6])); break;
    default: asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(o[7])); break;
  }
}

// The kernel body is a device function (the buffer-descriptor builtins exist only in device code).
// BQ: B of segment 0 is int4 with fp16 group scales (GemmArgs::Bscale).  The B half of a K tile then
// does not go to LDS by LDS-DMA: every lane fetches, for each of its four 16-byte LDS slots, the eight
// 4-bit weights (one dword) and their eight scales (16 bytes) into registers, and one K tile later
// writes the dequantised 16 bytes to the very slot the LDS-DMA load of a dense B would have filled, in
// time for the tile after that.  The dequantisation runs one value behind each MFMA (sign-extending
// bit-field extract, int -> float, mixed-precision FMA with the fp16 scale, packed conversion), two
// slots per K step.  Everything downstream (swizzle, fragment reads, MFMAs) is unchanged.  The dense
// second segment of a K-concatenated product takes the same route with its 16 bytes passed through,
// so that every K tile issues the same number of loads (the waits count them).
// PLAIN (decided on the host: two epilogues in one kernel cost registers): M and N are multiples of the tile and
//   1: the launch has no addend, bias, scale, mask or split: every tile takes the short 16-bit epilogue, which
//      needs 32 KB of LDS behind the ring (8 KB per wave);
//   2: the launch is a split contraction: every tile writes fp32 partials, 64 KB of LDS behind the ring;
//   0: everything else (general epilogue), 64 KB behind the ring as well.
// All three store whole row segments (see the epilogue).
template <typename T, int AL, int BL, int NS, bool BQ = false, int PLAIN = 0>
__device__ __forceinline__ void gemm_mc_body(const GemmArgs& g) {
  using P = McTile<AL, BL, NS>;
  static_assert(!BQ || (NS == 3 && AL == 0), "int4 B: 3-stage ring, A stored [M,K]");
  constexpr int BM = P::BM, BN = P::BN, BK = P::BK, IPW = P::IPW;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem_raw[];
  unsigned char* smem = smem_raw;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int l31 = lane & 31, hi = lane >> 5, s16 = lane & 15;

  // K tiles of one output tile: segment 0 then segment 1; the last tile of a segment may be partial
  const int nt0 = (g.K[0] + BK - 1) / BK, nt1 = (g.K[1] + BK - 1) / BK;
  const int ntk = nt0 + nt1;
  const int total = g.nbm * g.nbn;
  const int nwork = total * g.splits;  // work item w = split * total + tile sequence number

  // tile sequence number -> (m0, n0).  Consecutive workgroups sit on different XCDs (8, each with its
  // own L2): renumber so that each XCD works on a contiguous run of tiles, then walk the tile grid in
  // bands of 8 tile rows (a run shares A rows and B columns in its L2).
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
  // Everything the fetch itself needs is kept ready in registers (two uniform pointers to the tile's
  // k origin and one per-lane offset per instruction), so that the eight loads are straight-line code
  // that the scheduler can spread between the MFMAs.  Moving on to the next tile is a pointer bump,
  // except at an "event" (partial tile, segment switch, next work item), where the state is rebuilt.
  const int K0 = g.K[0], K1 = g.K[1];
  const T* const segA0 = static_cast<const T*>(g.A[0]);
  const T* const segA1 = static_cast<const T*>(g.A[1]);
  const T* const segB0 = static_cast<const T*>(g.B[0]);
  const T* const segB1 = static_cast<const T*>(g.B[1]);
  const uint32_t lda0 = (uint32_t)g.lda[0], lda1 = (uint32_t)g.lda[1];
  const uint32_t ldb0 = (uint32_t)g.ldb[0], ldb1 = (uint32_t)g.ldb[1];
  int cw = blockIdx.x, cu = 0, cu_end = 0, cm0 = 0, cn0 = 0, cnext = 0;
  bool clive = true;
  // Loads go through buffer descriptors: a uniform descriptor per operand and segment, a uniform
  // byte offset for the K tile (scalar register) and one 32-bit per-lane byte offset per instruction.
  auto extent_bytes = [&](bool strided, int rows_or_cols, int K, uint32_t ld) -> uint32_t {
    // [rows, K] with K contiguous, or [K, cols] strided; 0 for an absent segment
    if (K <= 0) return 0u;
    const uint64_t e = strided ? ((uint64_t)(K - 1) * ld + (uint64_t)rows_or_cols) : ((uint64_t)(rows_or_cols - 1) * ld + (uint64_t)K);
    return (uint32_t)(e * 2u);
  };
  // The four loads of an operand tile share one LDS base (M0) and differ in the instruction's
  // immediate offset (0, 1, 2, 3 KB), which the hardware adds to the LDS address and to the memory
  // address alike.  The memory side is compensated in the per-lane offsets; to keep those
  // non-negative the descriptors start kBias bytes before the matrix (address arithmetic only:
  // every address actually formed lies inside the matrix).
  constexpr uint32_t kBias = (IPW - 1) * 1024;
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
  // BQ: register route of the B half.  rsQ / offBq / kBq address the dword of eight 4-bit weights of
  // each slot, rsS / offBs / kBs its eight fp16 scales; in the dense second segment both address the
  // slot's 16 bytes of B itself.
  auto plain_rsrc = [&](const void* base, uint64_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (uint32_t)bytes, 0x00020000);
  };
  const uint32_t ldbs2 = 2u * (uint32_t)g.ldbs;
  __amdgpu_buffer_rsrc_t rsQ0 = rsB0, rsS0 = rsB0, rsD1 = rsB0, rsQ = rsB0, rsS = rsB0;
  if constexpr (BQ) {
    // W as the kernel sees it: [N, K0] with K contiguous (dY W^T) or [K0, N] (X W)
    const uint64_t w_rows = P::B_STR ? (uint64_t)K0 : (uint64_t)g.N, w_cols = P::B_STR ? (uint64_t)g.N : (uint64_t)K0;
    rsQ0 = plain_rsrc(g.B[0], ((w_rows - 1) * ldb0 + w_cols + 1) / 2);
    rsS0 = plain_rsrc(g.Bscale, (((w_rows + 63) / 64 - 1) * (uint64_t)g.ldbs + w_cols) * 2);
    rsD1 = plain_rsrc(g.B[1], extent_bytes(P::B_STR, g.N, K1, ldb1));
    rsQ = rsQ0;
    rsS = rsS0;
  }
  uint32_t kBq = 0, kBs = 0, stepBq = 0;
  uint32_t offBq[IPW], offBs[IPW];
  int cts = 0;       // K tile index of the cursor inside its segment
  bool cq = false;   // the cursor's segment is the int4 one

  // Rebuild the state for tile cu of work item cw (tile origin cm0, cn0).  Rows / columns beyond the
  // matrix are clamped: they only feed outputs that are never stored.  In a partial tile the chunks
  // with k >= kvalid are fetched from k = 0 of the same row / column (in range); the multiply
  // zeroes them.
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
      const int p = (wave * IPW + j) * 64 + lane;
      {
        const int row = P::A_STR ? (p >> 5) : (p >> 2);
        const int col = P::A_STR ? (((p & 31) ^ (4 * (row & 3))) << 3) : (((p & 3) ^ ((row >> 2) & 3)) << 3);
        if constexpr (!P::A_STR) {
          int gr = cm0 + row; gr = gr < g.M ? gr : g.M - 1;
          offA[j] = 2u * ((uint32_t)gr * lda + (uint32_t)(col < kvalid ? col : 0)) + (kBias - 1024u * j);
        } else {
          int gc = cm0 + col; gc = gc < g.M ? gc : g.M - 8;
          offA[j] = 2u * ((uint32_t)(row < kvalid ? row : 0) * lda + (uint32_t)gc) + (kBias - 1024u * j);
        }
      }
      {
        const int row = P::B_STR ? (p >> 5) : (p >> 2);
        const int col = P::B_STR ? (((p & 31) ^ (4 * (row & 3))) << 3) : (((p & 3) ^ ((row >> 2) & 3)) << 3);
        uint32_t elem, sc;  // element offset of the slot's first value in B; byte offset of its scales
        if constexpr (!P::B_STR) {
          int gr = cn0 + row; gr = gr < g.N ? gr : g.N - 1;
          const uint32_t c = (uint32_t)(col < kvalid ? col : 0);
          elem = (uint32_t)gr * ldb + c;
          sc = (uint32_t)(gr >> 6) * ldbs2 + 2u * c;
        } else {
          int gc = cn0 + col; gc = gc < g.N ? gc : g.N - 8;
          elem = (uint32_t)(row < kvalid ? row : 0) * ldb + (uint32_t)gc;
          sc = 2u * (uint32_t)gc;
        }
        offB[j] = 2u * elem + (kBias - 1024u * j);
        if constexpr (BQ) {
          offBq[j] = seg == 0 ? elem / 2u : 2u * elem;
          offBs[j] = seg == 0 ? sc : 2u * elem;
        }
      }
    }
    if constexpr (BQ) {
      cq = seg == 0;
      cts = ts;
      rsQ = cq ? rsQ0 : rsD1;
      rsS = cq ? rsS0 : rsD1;
      // (wave-uniform by construction; said explicitly so that they stay in scalar registers)
      stepBq = __builtin_amdgcn_readfirstlane(cq ? stepB / 4u : stepB);
      kBq = __builtin_amdgcn_readfirstlane((uint32_t)ts * stepBq);
      kBs = __builtin_amdgcn_readfirstlane(cq ? (P::B_STR ? (uint32_t)(ts >> 1) * ldbs2 : (uint32_t)ts * (2u * BK)) : kBq);
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

  // Fetch the A half / the B half of the cursor's K tile into LDS stage `st`: four loads each, no
  // branches.  The two halves are issued in different K steps so that the loads are spread evenly
  // over the MFMAs (a burst of loads from all four waves backs up the address unit and stalls issue).
  auto issue_A1 = [&](int st, int j) {  // j must be a constant after unrolling: it is the immediate offset
    unsigned char* sA = smem + st * P::STAGE_BYTES + wave * (IPW * 1024);
    const uint32_t ukA = __builtin_amdgcn_readfirstlane(kA);  // wave-uniform: keeps the load free of a per-lane loop
    switch (j) {
      case 0: __builtin_amdgcn_raw_ptr_buffer_load_lds(rsA, (mc_lds_void_t*)sA, 16, offA[0], ukA, 0, 0); break;
      case 1: __builtin_amdgcn_raw_ptr_buffer_load_lds(rsA, (mc_lds_void_t*)sA, 16, offA[1], ukA, 1024, 0); break;
      case 2: __builtin_amdgcn_raw_ptr_buffer_load_lds(rsA, (mc_lds_void_t*)sA, 16, offA[2], ukA, 2048, 0); break;
      default: __builtin_amdgcn_raw_ptr_buffer_load_lds(rsA, (mc_lds_void_t*)sA, 16, offA[3], ukA, 3072, 0); break;
    }
  };
  auto issue_B1 = [&](int st, int j) {
    unsigned char* sB = smem + st * P::STAGE_BYTES + P::A_BYTES + wave * (IPW * 1024);
    const uint32_t ukB = __builtin_amdgcn_readfirstlane(kB);
    switch (j) {
      case 0: __builtin_amdgcn_raw_ptr_buffer_load_lds(rsB, (mc_lds_void_t*)sB, 16, offB[0], ukB, 0, 0); break;
      case 1: __builtin_amdgcn_raw_ptr_buffer_load_lds(rsB, (mc_lds_void_t*)sB, 16, offB[1], ukB, 1024, 0); break;
      case 2: __builtin_amdgcn_raw_ptr_buffer_load_lds(rsB, (mc_lds_void_t*)sB, 16, offB[2], ukB, 2048, 0); break;
      default: __builtin_amdgcn_raw_ptr_buffer_load_lds(rsB, (mc_lds_void_t*)sB, 16, offB[3], ukB, 3072, 0); break;
    }
  };
  auto issue_A = [&](int st) {
#pragma unroll
    for (int j = 0; j < IPW; ++j) issue_A1(st, j);
  };
  auto issue_B = [&](int st) {
#pragma unroll
    for (int j = 0; j < IPW; ++j) issue_B1(st, j);
  };
  // BQ: slot j of the B half of the cursor's K tile into registers, and one value of a slot on its
  // way to LDS.  Slots 0,1 are refilled in K step 1 and slots 2,3 in the following K step 0 (the cursor
  // does not move in between); one K tile later they are dequantised in the same two K steps, one
  // value behind each MFMA, and stored to the stage of the tile that is multiplied next.
  uint32_t rw[IPW];   // eight 4-bit weights per slot
  i32x4 rsc[IPW];     // their eight fp16 scales (or, in the dense segment, the slot's 16 bytes of B)
  bool q01 = false, q23 = false;  // slots 0,1 / 2,3 hold int4 weights (wave-uniform)
  auto load_B = [&](int j) {
    if constexpr (BQ) {
      // (the scalar offsets are wave-uniform; saying so keeps the loads free of per-lane loops)
      rw[j] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(rsQ, offBq[j], __builtin_amdgcn_readfirstlane(kBq), 0);
      rsc[j] = __builtin_bit_cast(i32x4, __builtin_amdgcn_raw_buffer_load_b128(rsS, offBs[j], __builtin_amdgcn_readfirstlane(kBs), 0));
    }
  };
  uint32_t dq[IPW];
  float dq_even = 0.f;
  uint32_t dq_x = 0;
  auto commit_B = [&](int stage, int j, int e, bool isq) {  // value e (0..7) of slot j
    if constexpr (BQ) {
      typedef float f32x2_t __attribute__((ext_vector_type(2)));
      typedef T tx2_t __attribute__((ext_vector_type(2)));
      const uint32_t scp = (uint32_t)rsc[j][e >> 1];
      if (e == 0) dq_x = rw[j] ^ 0x88888888u;  // offset-binary nibbles -> two's complement, once per slot
      const uint32_t x = dq_x;
      const int qv = (int)(x << (28 - 4 * e)) >> 28;
      const _Float16 sv = __builtin_bit_cast(_Float16, (unsigned short)((e & 1) ? (scp >> 16) : (scp & 0xFFFFu)));
      // q * scale is exact in fp32 (4 bits x 11 bits); written as a fused multiply-add with +0 so that
      // the fp16 scale feeds the mixed-precision FMA directly; one rounding to T, two values at a time
      const float f = __builtin_fmaf((float)qv, (float)sv, 0.f);
      if ((e & 1) == 0) {
        dq_even = f;
      } else {
        const f32x2_t f2 = {dq_even, f};
        const uint32_t packed = __builtin_bit_cast(uint32_t, __builtin_convertvector(f2, tx2_t));
        dq[e >> 1] = isq ? packed : scp;
      }
      if (e == 7) {
        i32x4 v = {(int)dq[0], (int)dq[1], (int)dq[2], (int)dq[3]};
        *reinterpret_cast<i32x4*>(smem + stage * P::STAGE_BYTES + P::A_BYTES + (wave * IPW + j) * 1024 + lane * 16) = v;
      }
    }
  };
  // Move the cursor on.  Past the last work item it stays on the last tile, which is then fetched
  // again (into a stage nobody reads), so that the number of loads in flight, which the waits below
  // count, never changes.
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
    if constexpr (!BQ) {
      // straight-line in the common case (next tile of the same run, or nothing left to fetch): the
      // pointers are bumped unconditionally, an event rebuilds them
      const bool live = clive;
      cu += live ? 1 : 0;
      kA += live ? stepA : 0u;
      kB += live ? stepB : 0u;
      if (__builtin_expect(live && cu == cnext, 0)) cursor_event();
    } else {
      if (!clive) return;
      ++cu;
      if (cu != cnext) {
        kA += stepA;
        kB += stepB;
        ++cts;
        kBq = __builtin_amdgcn_readfirstlane(kBq + stepBq);
        kBs = __builtin_amdgcn_readfirstlane(cq ? (P::B_STR ? (uint32_t)(cts >> 1) * ldbs2 : (uint32_t)cts * (2u * BK)) : kBq);
        return;
      }
      kA += stepA;  // (cursor_event undoes this where it matters)
      kB += stepB;
      cursor_event();
    }
  };

  // ---- fragment addresses (bytes inside a stage, stage 0) -------------------------------------------
  // K-contiguous tile: row q, the 16 bytes at k = 16 ks + 8 hi live in slot (2 ks + hi) ^ ((q >> 2) & 3)
  // K-strided tile: transposing 8-byte LDS load; within a 16-lane group lane s points at k-row
  // 16 ks + 8 hi + s/4 (+4 for the second load), columns c0 + 4 (s%4) .. +3, and receives column c0 + s
  // for four consecutive k.  Block b of the wave's 128 columns: chunk slot (16 w + 4 b + ...) ^ 4 (s/4).
  uint32_t fragA[4], fragB[4];
  {
    const int sw = (l31 >> 2) & 3;
    if constexpr (!P::A_STR) {
      const uint32_t rowb = (uint32_t)(wm * 128 + l31) * 64u;
      fragA[0] = rowb + (uint32_t)((hi ^ sw) << 4);
      fragA[1] = rowb + (uint32_t)(((2 + hi) ^ sw) << 4);
      fragA[2] = fragA[3] = 0;
    } else {
      const int k = s16 >> 2;
#pragma unroll
      for (int b = 0; b < 4; ++b)
        fragA[b] = (uint32_t)((8 * hi + k) * 512 + (wm * 16 + ((b ^ k) << 2) + 2 * ((lane >> 4) & 1) + ((s16 & 3) >> 1)) * 16 +
                              ((4 * (s16 & 3)) & 7) * 2);
    }
    if constexpr (!P::B_STR) {
      const uint32_t rowb = (uint32_t)(wn * 128 + l31) * 64u;
      fragB[0] = P::A_BYTES + rowb + (uint32_t)((hi ^ sw) << 4);
      fragB[1] = P::A_BYTES + rowb + (uint32_t)(((2 + hi) ^ sw) << 4);
      fragB[2] = fragB[3] = 0;
    } else {
      const int k = s16 >> 2;
#pragma unroll
      for (int b = 0; b < 4; ++b)
        fragB[b] = P::A_BYTES +
                   (uint32_t)((8 * hi + k) * 512 + (wn * 16 + ((b ^ k) << 2) + 2 * ((lane >> 4) & 1) + ((s16 & 3) >> 1)) * 16 +
                              ((4 * (s16 & 3)) & 7) * 2);
    }
  }
  // LDS byte address of the ring (dynamic LDS need not start at 0)
  const uint32_t lds_base = (uint32_t)(uintptr_t)((mc_lds_void_t*)smem);

  i32x4 fa[2][4], fb[2][4];
  // One 32-wide operand fragment of K step KSR from the stage at byte offset `soff`.
  //  K-contiguous operand: one 16-byte LDS load.
  //  K-strided operand: two transposing 8-byte LDS loads, issued through inline assembly: the
  //  compiler makes every LDS read it knows about wait for all outstanding LDS-DMA loads
  //  (s_waitcnt vmcnt(0)), which would serialise the ring; reads it cannot see are waited for by
  //  hand (wait_tr below).
  auto read_frag_op = [&](bool strided, const uint32_t (&fr)[4], uint32_t soff, int blk, auto ksr_c) -> i32x4 {
    constexpr int KSR = decltype(ksr_c)::value;
    if (!strided) {
      return *reinterpret_cast<const i32x4*>(smem + soff + fr[KSR] + blk * 2048);
    } else {
      const uint32_t addr = lds_base + soff + fr[blk];
      i32x2 lo, hi2;
      asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(lo) : "v"(addr), "i"(KSR * 8192));
      asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(hi2) : "v"(addr), "i"(KSR * 8192 + 2048));
      i32x4 out = {lo[0], lo[1], hi2[0], hi2[1]};
      return out;
    }
  };
  // everything the hand-issued LDS reads fetched into buffer `buf` has arrived
  auto wait_tr = [&](int buf) {
    if constexpr (P::A_STR && P::B_STR)
      asm volatile("s_waitcnt lgkmcnt(0)"
                   : "+v"(fa[buf][0]), "+v"(fa[buf][1]), "+v"(fa[buf][2]), "+v"(fa[buf][3]), "+v"(fb[buf][0]),
                     "+v"(fb[buf][1]), "+v"(fb[buf][2]), "+v"(fb[buf][3]));
    else if constexpr (P::A_STR)
      asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(fa[buf][0]), "+v"(fa[buf][1]), "+v"(fa[buf][2]), "+v"(fa[buf][3]));
    else if constexpr (P::B_STR)
      asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(fb[buf][0]), "+v"(fb[buf][1]), "+v"(fb[buf][2]), "+v"(fb[buf][3]));
  };
  // zero the fragment registers of K step ks that hold k >= kvalid (this lane's 8 k start at 16 ks + 8 hi)
  auto mask_frags = [&](int buf, int ks, int kvalid) {
    if (ks * 16 + 8 * hi >= kvalid) {
#pragma unroll
      for (int a = 0; a < 4; ++a) fa[buf][a] = i32x4{0, 0, 0, 0};
#pragma unroll
      for (int b = 0; b < 4; ++b) fb[buf][b] = i32x4{0, 0, 0, 0};
    }
  };

  f32x16 acc[4][4];

#define MC_VMEM_AT(q) (((q) & 3) == 3)
#define MC_VMEM_EARLY(q) ((q) == 2 || (q) == 5 || (q) == 8 || (q) == 11)
#define MC_FENCE() __builtin_amdgcn_sched_barrier(0)
  // One K step, in exactly this instruction order (a scheduling fence after every piece): 16 MFMAs out
  // of fragment buffer `bufc`; behind each of the first 8, one fragment of K step KSR of the stage at
  // `soff` goes to buffer `bufr`; behind every fourth, one of the 4 LDS-DMA loads `issue_one(j)`.
  // A wave issues at most one instruction per 4 cycles and an MFMA occupies the matrix core for 32, so
  // up to ~7 other instructions fit behind each MFMA; spreading them keeps the matrix core fed, and
  // spreading the loads keeps the four waves from flooding the address unit at the same moment.
  // sync_c: -1 = none; otherwise MC_SYNC(sync_c) runs behind the first MFMA and the fragment reads follow
  // from the second on (the stage they read, and the stage the loads refill, are safe only after it).
  // early_c: loads behind MFMAs 2, 5, 8, 11 instead of 3, 7, 11, 15 (leaves the tail of the step free).
  auto kstep = [&](auto ksr_c, auto sync_c, auto early_c, int bufc, int bufr, uint32_t soff, auto issue_one, auto behind) {
    constexpr int SYNC = decltype(sync_c)::value;
    constexpr bool EARLY = decltype(early_c)::value;
    constexpr int R0 = SYNC >= 0 ? 1 : 0;
    wait_tr(bufc);
    MC_FENCE();
    int j = 0;
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      Elem<T>::mma(acc[q >> 2][q & 3], fb[bufc][q & 3], fa[bufc][q >> 2]);
      MC_FENCE();
      if constexpr (SYNC >= 0) {
        if (q == 0) {
          asm volatile("" ::: "memory");
          __builtin_amdgcn_s_waitcnt(mc_wait_imm(SYNC, true));
          __builtin_amdgcn_s_barrier();
          asm volatile("" ::: "memory");
          MC_FENCE();
        }
      }
      if (q >= R0 && q < R0 + 4) {
        fa[bufr][q - R0] = read_frag_op(P::A_STR, fragA, soff, q - R0, ksr_c);
        MC_FENCE();
      } else if (q >= R0 + 4 && q < R0 + 8) {
        fb[bufr][q - R0 - 4] = read_frag_op(P::B_STR, fragB, soff, q - R0 - 4, ksr_c);
        MC_FENCE();
      }
      behind(q);  // further work placed behind MFMA q (the int4 route's dequantisation, the cursor's step)
      if (EARLY ? MC_VMEM_EARLY(q) : MC_VMEM_AT(q)) {
        issue_one(j++);
        MC_FENCE();
      }
    }
  };
  auto nothing = [](int) {};
  // all of this wave's LDS reads are complete and at most `vm` of its loads are in flight; then
  // the workgroup barrier.  The empty asm statements keep the compiler from moving memory
  // accesses across it.
#define MC_SYNC(vm)                                                         \
  do {                                                                      \
    MC_FENCE();                                                             \
    asm volatile("" ::: "memory");                                          \
    __builtin_amdgcn_s_waitcnt(mc_wait_imm((vm), true));                    \
    __builtin_amdgcn_s_barrier();                                           \
    asm volatile("" ::: "memory");                                          \
    MC_FENCE();                                                             \
  } while (0)

  // ---- prologue: fill the ring (the last tile only by its A half: the loop issues B halves in K
  // step 0 and A halves in K step 1), wait for the first tile
  if constexpr (!BQ) {
#pragma unroll
    for (int s = 0; s < NS - 1; ++s) {
      issue_A(s);
      issue_B(s);
      cursor_advance();
    }
    issue_A(NS - 1);
    MC_SYNC((NS - 2) * P::LPT + IPW);
  } else {
    // B of tile 0 goes to LDS at once; then the steady state is set up: slots 0,1 of tile 1 in LDS
    // and refilled with tile 2, slots 2,3 of tile 1 still in the registers
    issue_A(0);
#pragma unroll
    for (int j = 0; j < IPW; ++j) load_B(j);
    q01 = q23 = cq;
    cursor_advance();
#pragma unroll
    for (int j = 0; j < IPW; ++j)
#pragma unroll
      for (int e = 0; e < 8; ++e) commit_B(0, j, e, q01);
    issue_A(1);
#pragma unroll
    for (int j = 0; j < IPW; ++j) load_B(j);
    q01 = q23 = cq;
    cursor_advance();
    issue_A(2);
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 8; ++e) commit_B(1, j, e, q01);
    load_B(0);
    load_B(1);
    q01 = cq;
    // A of tile 0 is older than everything else issued here (8 + 4 + 8 + 4 + 4 loads)
    MC_SYNC(28);
  }
  {
    using K0c = std::integral_constant<int, 0>;
#pragma unroll
    for (int a = 0; a < 4; ++a) fa[0][a] = read_frag_op(P::A_STR, fragA, 0u, a, K0c{});
#pragma unroll
    for (int b = 0; b < 4; ++b) fb[0][b] = read_frag_op(P::B_STR, fragB, 0u, b, K0c{});
  }
  // the only K tiles that can be partial: the last one of each segment
  const int pu0 = (K0 % BK) != 0 ? nt0 - 1 : -1, pu1 = (K1 % BK) != 0 ? ntk - 1 : -1;
  int stp = NS - 1;  // stage of the previous tile = where the tile being fetched goes
  int st = 0;  // stage of the tile being multiplied; runs on across work items

  for (int w = blockIdx.x; w < nwork; w += gridDim.x) {
    int seq, split, u0, u1, m0, n0;
    split_range(w, seq, split, u0, u1);
    tile_origin(seq, m0, n0);
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    for (int u = u0; u < u1; ++u) {
      const bool partial = (u == pu0) | (u == pu1);  // wave-uniform, rare
      const int stn = (st + 1 == NS) ? 0 : st + 1;
      int kvalid = BK;
      if (__builtin_expect(partial, 0)) {  // zero what lies beyond K
        kvalid = u < nt0 ? K0 - u * BK : K1 - (u - nt0) * BK;
        MC_FENCE();
        wait_tr(0);
        mask_frags(0, 0, kvalid);
      }
      // K step 0 out of buffer 0; K step 1's fragments go to buffer 1; second half of the fetch
      // that the previous K step began
      using NoSync = std::integral_constant<int, -1>;
      if constexpr (!BQ) {
        // the cursor moves on behind MFMA 12, after the last of this step's loads (which belong to its tile)
        kstep(std::integral_constant<int, 1>{}, NoSync{}, std::true_type{}, 0, 1, (uint32_t)(st * P::STAGE_BYTES),
              [&](int j) { issue_B1(stp, j); }, [&](int q) { if (q == 12) { cursor_advance(); MC_FENCE(); } });
      } else {
        // int4 route: behind MFMA q, value q % 8 of slot 2 + q / 8 of the next tile's B (fetched during
        // the previous tile) is dequantised; a completed slot goes to the next tile's stage and its
        // registers are refilled with the B half of the cursor's tile.
        kstep(std::integral_constant<int, 1>{}, NoSync{}, std::false_type{}, 0, 1, (uint32_t)(st * P::STAGE_BYTES),
              [&](int j) { if (j & 1) load_B(2 + (j >> 1)); },
              [&](int q) { commit_B(stn, 2 + (q >> 3), q & 7, q23); MC_FENCE(); });
        q23 = cq;
        cursor_advance();
      }
      // Tile u+1 must have landed (own loads, then everyone's: loads return in order, so "at most
      // (NS-2) tiles' worth outstanding" means tile u+1 is in), and everyone must be done reading
      // stage st before it is refilled.  (Int4 route: the loads issued after the last A load of tile
      // u+1 are 2 + 4 + 8 + 4: see K step 1 below.)
      // The wait and the barrier run behind the first MFMA of K step 1 (which only needs registers).
      if (__builtin_expect(partial, 0)) {
        MC_FENCE();
        wait_tr(1);
        mask_frags(1, 1, kvalid);
        MC_FENCE();
      }
      // K step 1 out of buffer 1, with the next tile's first fragments and the first half of the
      // refill of stage st
      if constexpr (!BQ) {
        kstep(std::integral_constant<int, 0>{}, std::integral_constant<int, (NS - 2) * P::LPT>{}, std::false_type{}, 1, 0,
              (uint32_t)(stn * P::STAGE_BYTES), [&](int j) { issue_A1(st, j); }, nothing);
      } else {
        // int4 route: slots 0,1 of the tile after the next one (the cursor has moved on) likewise; their
        // loads follow the A loads at MFMA 7 and 15
        kstep(std::integral_constant<int, 0>{}, std::integral_constant<int, 18>{}, std::false_type{}, 1, 0,
              (uint32_t)(stn * P::STAGE_BYTES), [&](int j) { issue_A1(st, j); if (j & 1) load_B(j >> 1); },
              [&](int q) { commit_B(stp, q >> 3, q & 7, q01); MC_FENCE(); });
        q01 = cq;
      }
      stp = st;
      st = stn;
    }

    // ---- epilogue (the next work item's first tiles keep arriving meanwhile)
    if constexpr (PLAIN == 1) {
      // Row-contiguous stores: a wave store instruction that covers whole 128-byte lines costs a quarter of one
      // that writes 32 bytes to each of 32 rows.  Each block row (32 rows x 128 columns of this wave) goes through
      // a private 8 KB LDS area: 8-byte pieces in the accumulator layout in, 16-byte pieces of 4 rows x 256 bytes out.
      unsigned char* const stg = smem + P::LDS_BYTES + wave * 8192;
      const uint32_t stg_base = (uint32_t)(uintptr_t)((mc_lds_void_t*)stg);
      const uint32_t wr = stg_base + (uint32_t)l31 * 256u;   // this lane's row in the area
      const uint32_t wsw = 2u * (uint32_t)(l31 & 15);        // its rotation of the 8-byte slots (even: pairs stay together)
      const int rr = lane >> 4, rc = lane & 15;              // read side: row within a group of 4, 16-byte chunk
      T* gp = static_cast<T*>(g.C) + (int64_t)(m0 + wm * 128 + rr) * g.ldc + (n0 + wn * 128 + rc * 8);
      typedef float f32x2_t __attribute__((ext_vector_type(2)));
      typedef T tx2_t __attribute__((ext_vector_type(2)));
#pragma unroll
      for (int a = 0; a < 4; ++a) {
#pragma unroll
        for (int b = 0; b < 4; ++b) {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            // explicit reads at the point of use: left to itself the compiler copies all 256 accumulator
            // registers to vector registers ahead of the epilogue and runs out of registers
            float x0, x1, x2, x3;
            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x0) : "a"(acc[a][b][4 * q + 0]));
            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x1) : "a"(acc[a][b][4 * q + 1]));
            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x2) : "a"(acc[a][b][4 * q + 2]));
            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x3) : "a"(acc[a][b][4 * q + 3]));
            const f32x2_t lo = {x0, x1}, hi2 = {x2, x3};
            i32x2 v = {(int)__builtin_bit_cast(unsigned, __builtin_convertvector(lo, tx2_t)),
                       (int)__builtin_bit_cast(unsigned, __builtin_convertvector(hi2, tx2_t))};
            const uint32_t slot = ((uint32_t)(8 * b + 2 * q) ^ wsw) + (uint32_t)hi;  // columns 32 b + 8 q + 4 hi .. + 3
            asm volatile("ds_write_b64 %0, %1" : : "v"(wr + slot * 8u), "v"(v) : "memory");
            __builtin_amdgcn_sched_barrier(0);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
        // all eight reads first, then each store as soon as its piece has arrived (LDS operations return in order)
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
          *reinterpret_cast<i32x4*>(gp + (int64_t)(a * 32 + 4 * k) * g.ldc) = o[k];
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    } else if constexpr (PLAIN == 2) {
      // fp32 partials of a split contraction, row-contiguous like the 16-bit case: each block row (32 rows x 128
      // fp32 columns of this wave = 16 KB) passes through LDS; 16-byte pieces in the accumulator layout in, two
      // rows x 512 bytes per store instruction out.
      unsigned char* const stg = smem + P::LDS_BYTES + wave * 16384;
      const uint32_t stg_base = (uint32_t)(uintptr_t)((mc_lds_void_t*)stg);
      const uint32_t wr = stg_base + (uint32_t)l31 * 512u;
      const uint32_t wsw = (uint32_t)l31;                   // rotation of the 16-byte slots of this lane's row
      const int rr = lane >> 5, rc = lane & 31;              // read side: row within a pair, 16-byte chunk
      float* gp = g.partial + ((int64_t)split * g.M + (m0 + wm * 128 + rr)) * g.N + (n0 + wn * 128 + rc * 4);
#pragma unroll
      for (int a = 0; a < 4; ++a) {
#pragma unroll
        for (int b = 0; b < 4; ++b) {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            float x0, x1, x2, x3;  // explicit reads at the point of use, as above
            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x0) : "a"(acc[a][b][4 * q + 0]));
            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x1) : "a"(acc[a][b][4 * q + 1]));
            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x2) : "a"(acc[a][b][4 * q + 2]));
            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x3) : "a"(acc[a][b][4 * q + 3]));
            const f32x4 v = {x0, x1, x2, x3};
            const uint32_t slot = (uint32_t)(8 * b + 2 * q + hi) ^ wsw;  // columns 32 b + 8 q + 4 hi .. + 3
            asm volatile("ds_write_b128 %0, %1" : : "v"(wr + slot * 16u), "v"(v) : "memory");
            __builtin_amdgcn_sched_barrier(0);
          }
        }
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          f32x4 o[8];
#pragma unroll
          for (int k = 0; k < 8; ++k) {
            const int row = 2 * (8 * half + k) + rr;
            const uint32_t addr = stg_base + (uint32_t)row * 512u + (((uint32_t)rc ^ (uint32_t)(row & 31)) * 16u);
            asm volatile("ds_read_b128 %0, %1" : "=v"(o[k]) : "v"(addr) : "memory");
          }
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int k = 0; k < 8; ++k) {
            mc_wait_piece(k, o);
            *reinterpret_cast<f32x4*>(gp + (int64_t)(a * 32 + 2 * (8 * half + k)) * g.N) = o[k];
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      }
    } else {
      // General epilogue (ragged tiles, addend, bias, scale, mask, or partials of a ragged split): the fp32 block row
      // passes through the same 16 KB LDS area as above and comes back as rows; a lane then owns four consecutive
      // columns of one row, which is the unit of every option (one mask group, 8 bytes of addend / bias / output),
      // and a store instruction covers 2 rows x 256 bytes (512 of partials).  Arithmetic and its order are
      // store_block's: alpha, mask, + addend, + bias, one rounding.
      const Epilogue ep{g.C, g.ldc, g.D, g.ldd, g.partial, g.M, g.N, split, g.alpha, g.bias, g.drop_thr, g.drop_key, g.drop_cpr};
      unsigned char* const stg = smem + P::LDS_BYTES + wave * 16384;
      const uint32_t stg_base = (uint32_t)(uintptr_t)((mc_lds_void_t*)stg);
      const uint32_t wr = stg_base + (uint32_t)l31 * 512u;
      const uint32_t wsw = (uint32_t)l31;
      const int rr = lane >> 5, rc = lane & 31;
      const int n = n0 + wn * 128 + rc * 4;   // this lane's four columns (N is a multiple of 8: valid together)
      const bool n_ok = n < g.N;
      f32x4 bias4 = {0.f, 0.f, 0.f, 0.f};
      if (g.bias != nullptr && g.partial == nullptr && n_ok) {
        T b4[4];
        *reinterpret_cast<i32x2*>(b4) = *reinterpret_cast<const i32x2*>(static_cast<const T*>(g.bias) + n);
#pragma unroll
        for (int e = 0; e < 4; ++e) bias4[e] = (float)b4[e];
      }
#pragma unroll
      for (int a = 0; a < 4; ++a) {
#pragma unroll
        for (int b = 0; b < 4; ++b) {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            float x0, x1, x2, x3;
            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x0) : "a"(acc[a][b][4 * q + 0]));
            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x1) : "a"(acc[a][b][4 * q + 1]));
            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x2) : "a"(acc[a][b][4 * q + 2]));
            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x3) : "a"(acc[a][b][4 * q + 3]));
            const f32x4 v = {x0, x1, x2, x3};
            const uint32_t slot = (uint32_t)(8 * b + 2 * q + hi) ^ wsw;
            asm volatile("ds_write_b128 %0, %1" : : "v"(wr + slot * 16u), "v"(v) : "memory");
            __builtin_amdgcn_sched_barrier(0);
          }
        }
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          f32x4 o[8];
#pragma unroll
          for (int k = 0; k < 8; ++k) {
            const int row = 2 * (8 * half + k) + rr;
            const uint32_t addr = stg_base + (uint32_t)row * 512u + (((uint32_t)rc ^ (uint32_t)(row & 31)) * 16u);
            asm volatile("ds_read_b128 %0, %1" : "=v"(o[k]) : "v"(addr) : "memory");
          }
          // the addend's eight pieces of this half are requested together, ahead of their use (one at a time, every
          // piece would wait out a trip to memory)
          i32x2 dq[8];
          if (g.D != nullptr && g.partial == nullptr) {
#pragma unroll
            for (int k = 0; k < 8; ++k) {
              const int m = m0 + wm * 128 + a * 32 + 2 * (8 * half + k) + rr;
              dq[k] = (m < g.M && n_ok) ? *reinterpret_cast<const i32x2*>(static_cast<const T*>(g.D) + (int64_t)m * g.ldd + n) : i32x2{0, 0};
            }
          }
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int k = 0; k < 8; ++k) {
            mc_wait_piece(k, o);
            const int m = m0 + wm * 128 + a * 32 + 2 * (8 * half + k) + rr;
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
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      }
    }
  }
  // the LDS-DMA writes still in flight target this workgroup's LDS: let them land before it is released
  __builtin_amdgcn_s_waitcnt(mc_wait_imm(0, true));
#undef MC_SYNC
#undef MC_VMEM_AT
#undef MC_FENCE
}

template <typename T, int AL, int BL, int NS, bool BQ = false, int PLAIN = 0>
__global__ __launch_bounds__(256, 1) void gemm_mc_kernel(GemmArgs g) {
  gemm_mc_body<T, AL, BL, NS, BQ, PLAIN>(g);
}

}  // namespace rl
