// Software-pipelined tile GEMM for the large contractions (X W, dY W^T, X^T dY and their
// K-concatenated forms) in bf16 / fp16 on gfx950.  Same contract as gemm_kernel (gemm_engine.hpp).
//
// What differs from the generic engine:
//  - global memory -> LDS directly (16-byte LDS-DMA loads: no register staging, no LDS store
//    instructions).  An LDS-DMA load places lane l's 16 bytes at base + 16*l, so rows cannot be
//    padded; bank conflicts are avoided by an XOR swizzle applied on the global-address side:
//      K-contiguous tile  [rows][BK/8 chunks of 16 B] : chunk kc of row q sits in slot
//                         kc ^ ((q >> SH) & (BK/8-1)), SH = log2(rows per 256 bytes)
//      K-strided tile     [BK k-rows][cols/8 chunks]  : chunk c of k-row q sits in slot c ^ (4*(q&3))
//    Partial K tiles (the tail of a segment, and the short rank-r segment) are zero-filled through
//    registers into the same swizzled layout.
//  - the K loop is pipelined by hand: tile t+2 is requested while tile t is multiplied, and the
//    operand fragments of K step s+1 are read from LDS while the MFMAs of step s issue; one
//    workgroup barrier per K tile.
//  - tile shapes: 256x256x64 with 8 wavefronts (one workgroup per compute unit), and 256x128x32
//    with 4 wavefronts, two workgroups per compute unit, so that one workgroup's barrier, load
//    issue and epilogue overlap the other's MFMAs.
#pragma once
#include "gemm_engine.hpp"

namespace rl {

typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(1))) const void global_cvoid_t;

template <typename T, int AL, int BL, int BM_, int BN_, int BK_, int WM, int WN>
struct PipeTile {
  static constexpr int BM = BM_, BN = BN_, BK = BK_;
  static constexpr int NW = WM * WN, NT = NW * 64;
  static constexpr int WTM = BM / WM, WTN = BN / WN, TM = WTM / 32, TN = WTN / 32;
  static constexpr bool A_STR = (AL == 1), B_STR = (BL == 0);
  static constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2;
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
  static constexpr int A_IPW = (A_BYTES / 1024) / NW;  // 1 KB LDS-DMA instructions per wave per tile
  static constexpr int B_IPW = (B_BYTES / 1024) / NW;
  static constexpr int KSN = BK / 16;  // MFMA K steps per tile
  static_assert(sizeof(T) == 2, "16-bit element types only");
  static_assert((A_BYTES / 1024) % NW == 0 && (B_BYTES / 1024) % NW == 0, "wave count");
  static_assert(BK == 64 || BK == 32, "BK");
  static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile");
};

// Where the 16-byte chunk at chunk position p of an operand tile comes from: (row, col) in
// elements within the tile.  STRIDED = tile rows are k and columns are m/n; ROWLEN = elements per
// tile row (BK for a K-contiguous tile, BM or BN for a strided one).
template <bool STRIDED, int ROWLEN>
__device__ __forceinline__ void chunk_coords(int p, int& row, int& col) {
  constexpr int CPR = ROWLEN / 8;  // chunks per row
  row = p / CPR;
  const int slot = p % CPR;
  if constexpr (!STRIDED) {
    constexpr int SH = (ROWLEN == 64) ? 1 : 2;
    col = (slot ^ ((row >> SH) & (CPR - 1))) << 3;
  } else {
    col = (slot ^ (4 * (row & 3))) << 3;
  }
}

template <typename T, int AL, int BL, int BM, int BN, int BK, int WM, int WN, int MIN_WG>
__global__ __launch_bounds__(WM* WN * 64, MIN_WG) void gemm_pipe_kernel(GemmArgs g) {
  using P = PipeTile<T, AL, BL, BM, BN, BK, WM, WN>;
  constexpr int A_IPW = P::A_IPW, B_IPW = P::B_IPW, KSN = P::KSN;
  constexpr int A_ROWLEN = P::A_STR ? BM : BK, B_ROWLEN = P::B_STR ? BN : BK;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem_raw[];
  unsigned char* smem = smem_raw;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, lives in a scalar register
  const int wm = wave / WN, wn = wave % WN;

  const int nt0 = (g.K[0] + BK - 1) / BK, nt1 = (g.K[1] + BK - 1) / BK;
  const int full0 = g.K[0] / BK;  // tiles of segment 0 that are complete: the fast path
  const int t_begin = blockIdx.y * g.tiles_per_split;
  int t_end = t_begin + g.tiles_per_split;
  if (t_end > nt0 + nt1) t_end = nt0 + nt1;
  const T* A0 = static_cast<const T*>(g.A[0]);
  const T* B0 = static_cast<const T*>(g.B[0]);
  const size_t stepA = P::A_STR ? (size_t)BK * (size_t)g.lda[0] : (size_t)BK;
  const size_t stepB = P::B_STR ? (size_t)BK * (size_t)g.ldb[0] : (size_t)BK;
  const int l31 = lane & 31, hi = lane >> 5, s16 = lane & 15;

  // Persistent workgroups: each walks the output tiles seq = blockIdx.x, blockIdx.x + gridDim.x, ...
  // so that the stores of one tile drain while the next tile's K loop already runs (a fresh
  // workgroup per tile would expose every tile's write burst).
  const int total = g.nbm * g.nbn;
  for (int seq = blockIdx.x; seq < total; seq += gridDim.x) {
  // tile sequence -> tile: consecutive sequence numbers go to different XCDs (8 of them, each with
  // its own L2), so renumber such that each XCD works on a contiguous run of tiles, then walk the
  // tile grid in bands of 8 tile rows (a run shares A rows and B columns in its L2)
  int id = seq;
  {
    const int x = id & 7, slot = id >> 3, q = total >> 3, rem = total & 7;
    id = x * q + (x < rem ? x : rem) + slot;
  }
  constexpr int BAND = 8;
  const int per_band = BAND * g.nbn;
  const int band = id / per_band, first_m = band * BAND;
  const int band_rows = (g.nbm - first_m) < BAND ? (g.nbm - first_m) : BAND;
  const int in_band = id - band * per_band;
  const int tile_m = first_m + in_band % band_rows, tile_n = in_band / band_rows;
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  if (seq != (int)blockIdx.x) __syncthreads();  // the previous tile's last LDS reads are done

  // ---- fast-path source offsets (segment 0), one per LDS-DMA instruction of this lane.  Rows and
  // columns beyond the matrix are clamped: they only feed outputs that are never stored.
  uint32_t offA[A_IPW], offB[B_IPW];
#pragma unroll
  for (int j = 0; j < A_IPW; ++j) {
    const int p = (wave * A_IPW + j) * 64 + lane;
    int row, col;
    chunk_coords<P::A_STR, A_ROWLEN>(p, row, col);
    if constexpr (!P::A_STR) {
      int gr = m0 + row; gr = gr < g.M ? gr : g.M - 1;
      offA[j] = (uint32_t)gr * (uint32_t)g.lda[0] + (uint32_t)col;
    } else {
      int gc = m0 + col; gc = gc < g.M ? gc : g.M - 8;
      offA[j] = (uint32_t)row * (uint32_t)g.lda[0] + (uint32_t)gc;
    }
  }
#pragma unroll
  for (int j = 0; j < B_IPW; ++j) {
    const int p = (wave * B_IPW + j) * 64 + lane;
    int row, col;
    chunk_coords<P::B_STR, B_ROWLEN>(p, row, col);
    if constexpr (!P::B_STR) {
      int gr = n0 + row; gr = gr < g.N ? gr : g.N - 1;
      offB[j] = (uint32_t)gr * (uint32_t)g.ldb[0] + (uint32_t)col;
    } else {
      int gc = n0 + col; gc = gc < g.N ? gc : g.N - 8;
      offB[j] = (uint32_t)row * (uint32_t)g.ldb[0] + (uint32_t)gc;
    }
  }
  // Request K tile t into LDS stage `st`.
  auto issue_tile = [&](int t, int st) {
    unsigned char* sA = smem + st * P::STAGE_BYTES;
    unsigned char* sB = sA + P::A_BYTES;
    if (t < full0) {
      // uniform base advanced in scalar registers + per-lane offsets that never change
      const T* At = A0 + (size_t)t * stepA;
      const T* Bt = B0 + (size_t)t * stepB;
#pragma unroll
      for (int j = 0; j < A_IPW; ++j)
        __builtin_amdgcn_global_load_lds((global_cvoid_t*)(At + offA[j]),
                                         (lds_void_t*)(sA + (wave * A_IPW + j) * 1024), 16, 0, 0);
#pragma unroll
      for (int j = 0; j < B_IPW; ++j)
        __builtin_amdgcn_global_load_lds((global_cvoid_t*)(Bt + offB[j]),
                                         (lds_void_t*)(sB + (wave * B_IPW + j) * 1024), 16, 0, 0);
    } else {
      // partial tile or second segment: predicated loads, zero fill, same swizzled layout
      const int s = t < nt0 ? 0 : 1;
      const int k0 = (t - (s ? nt0 : 0)) * BK;
      const int Ks = g.K[s];
      const T* Ap = static_cast<const T*>(g.A[s]);
      const T* Bp = static_cast<const T*>(g.B[s]);
      const int64_t lda = g.lda[s], ldb = g.ldb[s];
      i32x4 va[A_IPW];
#pragma unroll
      for (int j = 0; j < A_IPW; ++j) {
        const int p = (wave * A_IPW + j) * 64 + lane;
        int row, col;
        chunk_coords<P::A_STR, A_ROWLEN>(p, row, col);
        i32x4 v = {0, 0, 0, 0};
        if constexpr (!P::A_STR) {
          if (m0 + row < g.M && k0 + col < Ks)
            v = *reinterpret_cast<const i32x4*>(Ap + (int64_t)(m0 + row) * lda + k0 + col);
        } else {
          if (k0 + row < Ks && m0 + col < g.M)
            v = *reinterpret_cast<const i32x4*>(Ap + (int64_t)(k0 + row) * lda + m0 + col);
        }
        va[j] = v;
      }
#pragma unroll
      for (int j = 0; j < A_IPW; ++j)
        *reinterpret_cast<i32x4*>(sA + ((wave * A_IPW + j) * 64 + lane) * 16) = va[j];
      i32x4 vb[B_IPW];
#pragma unroll
      for (int j = 0; j < B_IPW; ++j) {
        const int p = (wave * B_IPW + j) * 64 + lane;
        int row, col;
        chunk_coords<P::B_STR, B_ROWLEN>(p, row, col);
        i32x4 w = {0, 0, 0, 0};
        if constexpr (!P::B_STR) {
          if (n0 + row < g.N && k0 + col < Ks)
            w = *reinterpret_cast<const i32x4*>(Bp + (int64_t)(n0 + row) * ldb + k0 + col);
        } else {
          if (k0 + row < Ks && n0 + col < g.N)
            w = *reinterpret_cast<const i32x4*>(Bp + (int64_t)(k0 + row) * ldb + n0 + col);
        }
        vb[j] = w;
      }
#pragma unroll
      for (int j = 0; j < B_IPW; ++j)
        *reinterpret_cast<i32x4*>(sB + ((wave * B_IPW + j) * 64 + lane) * 16) = vb[j];
    }
  };

  // ---- fragment reads (one 32-wide block of an operand for K step ks) ---------------------------
  // K-contiguous tile: row q, 16 bytes at k = 16*ks + 8*hi
  auto read_kc = [&](const unsigned char* tile, int idx0, int ks) -> i32x4 {
    constexpr int CPR = BK / 8, SH = (BK == 64) ? 1 : 2;
    const int q = idx0 + l31;
    const int slot = ((2 * ks + hi) ^ ((q >> SH) & (CPR - 1)));
    return *reinterpret_cast<const i32x4*>(tile + q * (BK * 2) + (slot << 4));
  };
  // K-strided tile (rows are k, ROWLEN columns): transposing LDS load.  Within a 16-lane block lane
  // s points at k-row k + s/4, columns c0 + 4*(s%4) .. +3, and receives column c0 + s for four
  // consecutive k.
  auto read_str = [&](const unsigned char* tile, int rowlen, int idx0, int ks) -> i32x4 {
    const int krow = ks * 16 + 8 * hi + (s16 >> 2);
    const int col = idx0 + 16 * ((lane >> 4) & 1) + 4 * (s16 & 3);
    const int slot = (col >> 3) ^ (4 * (krow & 3));
    const unsigned char* p = tile + krow * (rowlen * 2) + (slot << 4) + ((col & 7) << 1);
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
    s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * (rowlen * 2)));
    i32x2 l2 = __builtin_bit_cast(i32x2, lo), h2 = __builtin_bit_cast(i32x2, hi4);
    i32x4 out = {l2[0], l2[1], h2[0], h2[1]};
    return out;
  };

  i32x4 fa[2][P::TM], fb[2][P::TN];
  auto read_frags = [&](int buf, int st, int ks) {
    const unsigned char* sA = smem + st * P::STAGE_BYTES;
    const unsigned char* sB = sA + P::A_BYTES;
#pragma unroll
    for (int a = 0; a < P::TM; ++a) {
      const int idx = wm * P::WTM + a * 32;
      fa[buf][a] = P::A_STR ? read_str(sA, BM, idx, ks) : read_kc(sA, idx, ks);
    }
#pragma unroll
    for (int b = 0; b < P::TN; ++b) {
      const int idx = wn * P::WTN + b * 32;
      fb[buf][b] = P::B_STR ? read_str(sB, BN, idx, ks) : read_kc(sB, idx, ks);
    }
  };

  f32x16 acc[P::TM][P::TN];
#pragma unroll
  for (int a = 0; a < P::TM; ++a)
#pragma unroll
    for (int b = 0; b < P::TN; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  // MFMAs i0..i1-1 of one K step (index = a*TN + b)
  auto mma_range = [&](int buf, int i0, int i1) {
#pragma unroll
    for (int i = i0; i < i1; ++i) Elem<T>::mma(acc[i / P::TN][i % P::TN], fb[buf][i % P::TN], fa[buf][i / P::TN]);
  };
  constexpr int NM = P::TM * P::TN;
  constexpr int NR = (P::A_STR ? 2 : 1) * P::TM + (P::B_STR ? 2 : 1) * P::TN;  // LDS reads per K step

  if (t_begin < t_end) {
    issue_tile(t_begin, 0);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (t_begin + 1 < t_end) issue_tile(t_begin + 1, 1);
    read_frags(0, 0, 0);

    // Each K step issues its MFMAs and the LDS requests for the next step as one scheduling
    // region; sched_group_barrier asks for "MFMA, two LDS reads, MFMA, two LDS reads, ..." so that
    // every request is issued in the shadow of a running MFMA and has the rest of the step to
    // complete before the next step's first MFMA waits for it.
#define RL_FENCE() __builtin_amdgcn_sched_barrier(0)
#define RL_INTERLEAVE()                                                    \
  do {                                                                     \
    _Pragma("unroll") for (int q_ = 0; q_ < NR / 2; ++q_) {                \
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                   \
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);                   \
    }                                                                      \
    __builtin_amdgcn_sched_group_barrier(0x008, NM - NR / 2, 0);           \
  } while (0)
    for (int t = t_begin; t < t_end; ++t) {
      const int st = (t - t_begin) & 1;
#pragma unroll
      for (int ks = 0; ks < KSN - 1; ++ks) {
        RL_FENCE();
        mma_range(ks & 1, 0, NM);
        read_frags((ks + 1) & 1, st, ks + 1);
        RL_INTERLEAVE();
      }
      // last K step of the tile (fragments in buffer 1); the next tile's first fragments go to 0
      RL_FENCE();
      mma_range(1, 0, 1);
      RL_FENCE();
      if (t + 1 < t_end) {
        // tile t+1 must have landed (own requests done, then everyone's), and every wave must be
        // done reading stage st before it is refilled with tile t+2
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        if (t + 2 < t_end) issue_tile(t + 2, st);
        RL_FENCE();
        read_frags(0, st ^ 1, 0);
      }
      RL_FENCE();
      mma_range(1, 1, NM);
    }
#undef RL_INTERLEAVE
#undef RL_FENCE
  }

  // ---- epilogue
  Epilogue ep{g.C, g.ldc, g.D, g.ldd, g.partial, g.M, g.N, (int)blockIdx.y};
#pragma unroll
  for (int a = 0; a < P::TM; ++a)
#pragma unroll
    for (int b = 0; b < P::TN; ++b)
      store_block<T>(ep, acc[a][b], m0 + wm * P::WTM + a * 32 + (lane & 31), n0 + wn * P::WTN + b * 32, lane);
  }  // persistent tile loop
}

}  // namespace rl
