// Tile GEMM engine for gfx950 (CDNA4): C[M,N] = sum over segments of op(A_s)[M,K_s] * op(B_s)[K_s,N]
// (+ D), fp32 accumulation on the matrix cores, one rounding to the output type.
//
// Every product of the LoRA layer (Eq. 1 and Eq. 3 of arxiv 2312.03415, and the intermediates of
// Algorithms 1-5) is an instance of this kernel: operand layouts select X W (row x row), dY W^T
// (row x col) and X^T dY (col x row); a second K segment gives [X|T][W;B] and [dY|Z1][W^T;A^T];
// the addend D gives W + AB and the "+=" steps of the default chain; gridDim.y > 1 splits the
// contraction over workgroups, each writing an fp32 partial that a second kernel sums in a fixed
// order (no atomics, run-to-run identical).
//
// Execution model: one workgroup owns a BM x BN output tile; WM x WN wavefronts (64 lanes) each own
// a (BM/WM) x (BN/WN) sub-tile made of 32x32 MFMA blocks.  Global memory -> registers -> LDS with
// the next K tile in flight while the current one is multiplied (two LDS stages, one barrier per
// K tile).  LDS keeps each operand in its global orientation; rows are padded so that the
// fragment reads are bank-conflict free.  K-contiguous operands are read with 16-byte LDS loads,
// K-strided 16-bit operands with the transposing 64-bit LDS load.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rl {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 f16x8;
typedef __attribute__((__vector_size__(4 * sizeof(_Float16)))) _Float16 f16x4;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(int)))) int i32x4;
typedef __attribute__((__vector_size__(2 * sizeof(int)))) int i32x2;

struct GemmArgs {
  const void* A[2];   // segment s: A stored [M,K_s] (AL=0) or [K_s,M] (AL=1)
  const void* B[2];   // segment s: B stored [K_s,N] (BL=0) or [N,K_s] (BL=1)
  int64_t lda[2], ldb[2];
  int K[2];           // K[1] = 0 when there is one segment
  void* C;            // [M,N] output in T (or unused when partial != nullptr)
  int64_t ldc;
  const void* D;      // optional addend [M,N] in T
  int64_t ldd;
  float* partial;     // split-K: fp32 [gridDim.y][M][N], dense
  int M, N;
  int tiles_per_split;  // K tiles per gridDim.y slice
  int nbm, nbn;         // tile grid
  int splits;           // number of K slices (gemm_mc_kernel: folded into blockIdx.x)
  // B of segment 0 stored as symmetric int4 with group scales (the frozen W of a quantised layer):
  // element (row, col) of the stored matrix is nibble (row * ldb + col) of B[0] (low nibble first),
  // value (nibble - 8) * scale[(row / 64) * ldbs + col], scales in fp16.  Bscale == nullptr: dense B.
  const void* Bscale;
  int64_t ldbs;
  // C = alpha * (sum of the products) + D + bias: alpha scales the products only; bias is a row
  // vector [N] in T added to every row (nullptr = none)
  float alpha;
  const void* bias;
  // drop_thr != 0: output element (m, n) of alpha * (the products) is zeroed where the dropout mask
  // drops element (m, n) of X (the adapter's share of dX); drop_cpr = groups of four columns per row
  uint32_t drop_thr, drop_key, drop_cpr;
  // One-pass LoRA forward (gemm_kernel's FUSE build, Y = X W + (s X A) B of Section 2's forward 1 in one kernel):
  // LA = the adapter's A [K[0], R] row-major (R <= 32), t_alpha = s.  The kernel then forms T = t_alpha * A[0] LA
  // for its own rows next to the main product, rounds it to T's type and contracts it with B[1] ([R, N]) as one more
  // K tile; A[1] is not read.  nullptr = an ordinary launch.
  const void* LA;
  int64_t ldla;
  int R;
  float t_alpha;
};

// ---- per-type pieces --------------------------------------------------------------------------

template <typename T> struct Elem;
template <> struct Elem<__bf16> {
  static __device__ __forceinline__ void mma(f32x16& acc, i32x4 rowop, i32x4 colop) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, rowop),
                                                  __builtin_bit_cast(bf16x8, colop), acc, 0, 0, 0);
  }
};
template <> struct Elem<_Float16> {
  static __device__ __forceinline__ void mma(f32x16& acc, i32x4 rowop, i32x4 colop) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, rowop),
                                                 __builtin_bit_cast(f16x8, colop), acc, 0, 0, 0);
  }
};
template <> struct Elem<float> {
  // a lane carries 4 consecutive k; four K=2 MFMAs each take one of them (same k order on both
  // operands, so the pairing is consistent)
  static __device__ __forceinline__ void mma(f32x16& acc, i32x4 rowop, i32x4 colop) {
    f32x4 a = __builtin_bit_cast(f32x4, rowop), b = __builtin_bit_cast(f32x4, colop);
#pragma unroll
    for (int j = 0; j < 4; ++j) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[j], b[j], acc, 0, 0, 0);
  }
};

template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ __bf16 from_f32<__bf16>(float v) { return (__bf16)v; }
template <> __device__ __forceinline__ _Float16 from_f32<_Float16>(float v) { return (_Float16)v; }

// ---- LoRA dropout mask (an option beyond the paper's layer, whose experiments run with dropout 0) ----
// Element (t, c) of X [n, i] is kept iff byte (c & 3) of H(t * (i / 4) + (c >> 2)) is >= thr, where
// H(x) = mix(x ^ key), mix = the 32-bit hash below, key = mix(seed ^ 0x9E3779B9) (computed on the host)
// and thr = round(256 p): a counter-based generator, so that forward and backward, and the CPU oracle,
// see the same mask without storing it.  One hash serves four consecutive columns.
__device__ __forceinline__ uint32_t drop_mix(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}
// bit 7 of byte k of the result is set iff byte k of h is >= thr (1 <= thr <= 255), all four bytes at once:
// the low seven bits are compared by an addition that carries into bit 7 (0x7F + 0x80 at most: no carry between
// bytes), the top bits decide the rest.  thr is uniform, so its part is scalar arithmetic.
__device__ __forceinline__ uint32_t drop_ge_bytes(uint32_t h, uint32_t thr) {
  const uint32_t lo = (h & 0x7F7F7F7Fu) + (0x80u - (thr & 0x7Fu)) * 0x01010101u;
  const uint32_t ge = (thr & 0x80u) ? (h & lo) : (h | lo);
  return ge & 0x80808080u;
}
// keep-masks of the four columns of group g: 0xFFFFFFFF / 0 per column
__device__ __forceinline__ void drop_keep4(uint32_t g, uint32_t key, uint32_t thr, uint32_t (&keep)[4]) {
  const uint32_t f = drop_ge_bytes(drop_mix(g ^ key), thr);
#pragma unroll
  for (int k = 0; k < 4; ++k) keep[k] = (uint32_t)((int32_t)(f << (24 - 8 * k)) >> 31);
}
// a 16-byte chunk of X whose first column belongs to group g (8 columns = groups g, g+1 for 16-bit
// types; 4 columns = group g for fp32) with the dropped elements zeroed
template <typename T>
__device__ __forceinline__ i32x4 drop_chunk(i32x4 v, uint32_t g, uint32_t key, uint32_t thr) {
  if constexpr (sizeof(T) == 4) {
    uint32_t k0[4];
    drop_keep4(g, key, thr, k0);
    return i32x4{(int)((uint32_t)v[0] & k0[0]), (int)((uint32_t)v[1] & k0[1]), (int)((uint32_t)v[2] & k0[2]), (int)((uint32_t)v[3] & k0[3])};
  } else {
    // per hash: flags -> 0xFF / 0x00 per byte -> each byte doubled into a 16-bit lane mask (byte permute)
    const uint32_t f0 = drop_ge_bytes(drop_mix(g ^ key), thr), f1 = drop_ge_bytes(drop_mix((g + 1) ^ key), thr);
    const uint32_t m0 = (f0 - (f0 >> 7)) | f0, m1 = (f1 - (f1 >> 7)) | f1;
    return i32x4{(int)((uint32_t)v[0] & __builtin_amdgcn_perm(m0, m0, 0x01010000u)),
                 (int)((uint32_t)v[1] & __builtin_amdgcn_perm(m0, m0, 0x03030202u)),
                 (int)((uint32_t)v[2] & __builtin_amdgcn_perm(m1, m1, 0x01010000u)),
                 (int)((uint32_t)v[3] & __builtin_amdgcn_perm(m1, m1, 0x03030202u))};
  }
}

// ---- epilogue of one 32x32 accumulator block ------------------------------------------------------
// With the MFMA operands swapped, lane l holds row m = l%32 and, for q = 0..3, the four consecutive
// columns 8q + 4(l/32) + {0..3}.  For 16-bit outputs the two half-waves exchange their halves of
// column groups (q, q+1) (v_permlane32_swap): lanes 0-31 then own columns 8q..8q+7 and lanes 32-63
// columns 8(q+1)..8(q+1)+7 of their row, so each lane stores 16 bytes and the pair (l, l+32)
// fills a 32-byte sector per store instead of half of one.
struct Epilogue {
  void* C;
  int64_t ldc;
  const void* D;
  int64_t ldd;
  float* partial;  // [splits][M][N] or nullptr
  int M, N, split;
  float alpha;       // scales the accumulated products (not D, not bias); partials stay unscaled
  const void* bias;  // [N] in T, or nullptr
  uint32_t drop_thr, drop_key, drop_cpr;  // see GemmArgs
};
// alpha * acc of four consecutive columns n .. n+3 (n a multiple of 4) of row m, dropout mask applied
__device__ __forceinline__ f32x4 epilogue_scale(const Epilogue& ep, f32x4 v, int m, int n) {
  if (ep.alpha != 1.f) v *= ep.alpha;
  if (ep.drop_thr != 0u) {
    uint32_t keep[4];
    drop_keep4((uint32_t)m * ep.drop_cpr + (uint32_t)(n >> 2), ep.drop_key, ep.drop_thr, keep);
#pragma unroll
    for (int k = 0; k < 4; ++k) v[k] = keep[k] ? v[k] : 0.f;
  }
  return v;
}

template <typename T>
__device__ __forceinline__ void store_block(const Epilogue& ep, const f32x16& acc, int m, int nbase, int lane) {
  if (m >= ep.M) return;
  const int h = lane >> 5;
  if (ep.partial) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int n = nbase + 8 * q + 4 * h;
      if (n >= ep.N) continue;
      f32x4 v = {acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
      *reinterpret_cast<f32x4*>(ep.partial + ((int64_t)ep.split * ep.M + m) * ep.N + n) = v;
    }
    return;
  }
  if constexpr (sizeof(T) == 4) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int n = nbase + 8 * q + 4 * h;
      if (n >= ep.N) continue;
      f32x4 v = {acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
      v = epilogue_scale(ep, v, m, n);
      if (ep.D) v += *reinterpret_cast<const f32x4*>(static_cast<const float*>(ep.D) + (int64_t)m * ep.ldd + n);
      if (ep.bias) v += *reinterpret_cast<const f32x4*>(static_cast<const float*>(ep.bias) + n);
      *reinterpret_cast<f32x4*>(static_cast<float*>(ep.C) + (int64_t)m * ep.ldc + n) = v;
    }
  } else {
#pragma unroll
    for (int qp = 0; qp < 2; ++qp) {  // column groups (2qp, 2qp+1)
      unsigned pa[2], pb[2];          // packed 16-bit pairs of group 2qp and 2qp+1
#pragma unroll
      for (int w = 0; w < 2; ++w) {
        const int q = 2 * qp + w;
        f32x4 v = {acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
        v = epilogue_scale(ep, v, m, nbase + 8 * q + 4 * h);
        if (ep.D || ep.bias) {
          const int n = nbase + 8 * q + 4 * h;
          if (n < ep.N) {
            T d4[4];
            if (ep.D) {
              *reinterpret_cast<i32x2*>(d4) =
                  *reinterpret_cast<const i32x2*>(static_cast<const T*>(ep.D) + (int64_t)m * ep.ldd + n);
#pragma unroll
              for (int e = 0; e < 4; ++e) v[e] += (float)d4[e];
            }
            if (ep.bias) {
              *reinterpret_cast<i32x2*>(d4) = *reinterpret_cast<const i32x2*>(static_cast<const T*>(ep.bias) + n);
#pragma unroll
              for (int e = 0; e < 4; ++e) v[e] += (float)d4[e];
            }
          }
        }
        T o4[4] = {from_f32<T>(v[0]), from_f32<T>(v[1]), from_f32<T>(v[2]), from_f32<T>(v[3])};
        unsigned* dst = w == 0 ? pa : pb;
        dst[0] = reinterpret_cast<unsigned*>(o4)[0];
        dst[1] = reinterpret_cast<unsigned*>(o4)[1];
      }
      // after the swap: lanes 0-31 hold (pa of h=0, pa of h=1), lanes 32-63 hold (pb of h=0, pb of h=1)
      auto s0 = __builtin_amdgcn_permlane32_swap(pa[0], pb[0], false, false);
      auto s1 = __builtin_amdgcn_permlane32_swap(pa[1], pb[1], false, false);
      const int n = nbase + 8 * (2 * qp + h);
      if (n < ep.N) {  // N is a multiple of 8 for 16-bit types: the 8 columns are valid together
        i32x4 out = {(int)s0[0], (int)s1[0], (int)s0[1], (int)s1[1]};
        *reinterpret_cast<i32x4*>(static_cast<T*>(ep.C) + (int64_t)m * ep.ldc + n) = out;
      }
    }
  }
}

// LDS row length (elements) for a tile whose rows hold `cols` elements.
//  K-contiguous tile: +16 bytes, so 16 consecutive rows read by 16-byte loads hit distinct banks.
//  K-strided tile   : row stride = 64 bytes mod 128 (16-bit, transposing loads) / +8 floats (fp32).
template <typename T, bool STRIDED, int COLS> struct LdsLd {
  static constexpr int VE = 16 / sizeof(T);
  static constexpr int value =
      !STRIDED ? COLS + VE
               : (sizeof(T) == 2 ? (((COLS * 2) % 128 == 64) ? COLS : COLS + 32) : COLS + 8);
};

// One 32-wide operand fragment for K step `ks` out of an LDS tile.
// Returns 16 bytes: the VE consecutive k values this lane feeds to the MFMA(s).
template <typename T, bool STRIDED, int LD>
__device__ __forceinline__ i32x4 read_frag(const T* tile, int idx0, int ks, int lane) {
  constexpr int VE = 16 / sizeof(T);
  if constexpr (!STRIDED) {
    const T* p = tile + (idx0 + (lane & 31)) * LD + ks * (2 * VE) + VE * (lane >> 5);
    return *reinterpret_cast<const i32x4*>(p);
  } else if constexpr (sizeof(T) == 2) {
    // transposing load: within a 16-lane block, lane s points at [k0 + s/4][c0 + 4*(s%4) .. +3]
    // and receives column c0 + s for k0..k0+3.
    const int s = lane & 15;
    const int c0 = idx0 + 16 * ((lane >> 4) & 1);
    const int k0 = ks * 16 + 8 * (lane >> 5);
    const T* p = tile + (k0 + (s >> 2)) * LD + c0 + 4 * (s & 3);
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * LD));
    i32x2 l2 = __builtin_bit_cast(i32x2, lo), h2 = __builtin_bit_cast(i32x2, hi);
    i32x4 out = {l2[0], l2[1], h2[0], h2[1]};
    return out;
  } else {
    const T* p = tile + (ks * 8 + 4 * (lane >> 5)) * LD + idx0 + (lane & 31);
    f32x4 v = {p[0], p[LD], p[2 * LD], p[3 * LD]};
    return __builtin_bit_cast(i32x4, v);
  }
}

// Eight int4 weights (one 32-bit word, low nibble first) times their eight fp16 scales -> eight T.
template <typename T>
__device__ __forceinline__ i32x4 dequant_chunk(uint32_t w, i32x4 sc) {
  const _Float16* s8 = reinterpret_cast<const _Float16*>(&sc);
  T o8[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int q = (int)((w >> (4 * j)) & 15u) - 8;
    o8[j] = from_f32<T>((float)q * (float)s8[j]);
  }
  return *reinterpret_cast<i32x4*>(o8);
}

// ---- the kernel ---------------------------------------------------------------------------------
// AL: 0 = A stored [M,K] (K contiguous), 1 = A stored [K,M].   BL: 0 = B stored [K,N], 1 = [N,K].
template <typename T, int AL, int BL, int BM, int BN, int BK, int WM, int WN>
struct GemmTile {
  static constexpr int NT = WM * WN * 64;
  static constexpr int VE = 16 / sizeof(T);
  static constexpr int KS = 2 * VE;
  static constexpr int WTM = BM / WM, WTN = BN / WN, TM = WTM / 32, TN = WTN / 32;
  static constexpr bool A_STR = (AL == 1), B_STR = (BL == 0);
  static constexpr int A_ROWS = A_STR ? BK : BM, A_COLS = A_STR ? BM : BK;
  static constexpr int B_ROWS = B_STR ? BK : BN, B_COLS = B_STR ? BN : BK;
  static constexpr int A_LD = LdsLd<T, A_STR, A_COLS>::value;
  static constexpr int B_LD = LdsLd<T, B_STR, B_COLS>::value;
  static constexpr int A_ELEMS = A_ROWS * A_LD, B_ELEMS = B_ROWS * B_LD;
  static constexpr int STAGE_ELEMS = A_ELEMS + B_ELEMS;
  static constexpr int LDS_BYTES = 2 * STAGE_ELEMS * (int)sizeof(T);
  static constexpr int A_CPR = A_COLS / VE, B_CPR = B_COLS / VE;  // 16-byte chunks per tile row
  static constexpr int A_CHUNKS = A_ROWS * A_CPR, B_CHUNKS = B_ROWS * B_CPR;
  static constexpr int A_PER = (A_CHUNKS + NT - 1) / NT, B_PER = (B_CHUNKS + NT - 1) / NT;
  // FUSE build: a [BK][RP] slice of the adapter's A per stage, K-strided like W; the 32-row blocks of T = X A of
  // a row of waves are dealt round-robin to its WN waves
  static constexpr int RP = 32;
  static constexpr int L_LD = LdsLd<T, true, RP>::value;
  static constexpr int L_ELEMS = BK * L_LD;
  static constexpr int L_CPR = RP / VE, L_CHUNKS = BK * L_CPR, L_PER = (L_CHUNKS + NT - 1) / NT;
  static constexpr int TT = (TM + WN - 1) / WN;
  static constexpr int FUSE_STAGE_ELEMS = STAGE_ELEMS + L_ELEMS;
  static constexpr int FUSE_LDS_BYTES = 2 * FUSE_STAGE_ELEMS * (int)sizeof(T);
  static_assert(WTM % 32 == 0 && WTN % 32 == 0 && BK % KS == 0, "tile shape");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
};

// BQ: B of segment 0 is int4 with group scales (see GemmArgs); it is dequantised on its way from
// the load registers to LDS, so the matrix cores see ordinary T operands.
// FUSE: the one-pass LoRA forward (see GemmArgs::LA): X stored [M,K], W stored [K,N], no K split.  Next to the main
// product every wave accumulates its share of T = X LA (one more 32-column block per 32 rows, fed from the X
// fragments already in registers and a [BK][32] slice of LA staged like W); behind the last K tile of segment 0
// the workgroup writes alpha-scaled, rounded T into the A half of the free LDS stage, where the K tile of segment 1
// (B[1], rows >= R zero) finds it as its A operand.
template <typename T, int AL, int BL, int BM, int BN, int BK, int WM, int WN, bool BQ = false, bool FUSE = false>
__global__ __launch_bounds__(WM* WN * 64) void gemm_kernel(GemmArgs g) {
  using G = GemmTile<T, AL, BL, BM, BN, BK, WM, WN>;
  constexpr int NT = G::NT, VE = G::VE;
  constexpr int STAGE_ELEMS = FUSE ? G::FUSE_STAGE_ELEMS : G::STAGE_ELEMS;
  static_assert(!FUSE || (AL == 0 && BL == 0 && !BQ && BK >= G::RP), "the one-pass forward: X [M,K], W [K,N], dense");
  static_assert(!FUSE || G::FUSE_LDS_BYTES <= 160 * 1024, "LDS budget");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  T* smem = reinterpret_cast<T*>(smem_raw);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;

  // ---- workgroup -> tile.  Consecutive workgroup ids go to different XCDs (8 of them, each with
  // its own L2), so first renumber such that each XCD gets a contiguous run of tiles, then walk
  // the tile grid in bands of 8 tile rows so that a run shares B columns and A rows in its L2.
  const int total = g.nbm * g.nbn;
  int id = blockIdx.x;
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

  // ---- K tiles of this workgroup (over both segments; gridDim.y slices them)
  const int nt0 = (g.K[0] + BK - 1) / BK, nt1 = (g.K[1] + BK - 1) / BK;
  const int t_begin = blockIdx.y * g.tiles_per_split;
  int t_end = t_begin + g.tiles_per_split;
  if (t_end > nt0 + nt1) t_end = nt0 + nt1;

  f32x16 acc[G::TM][G::TN];
#pragma unroll
  for (int a = 0; a < G::TM; ++a)
#pragma unroll
    for (int b = 0; b < G::TN; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  i32x4 ra[G::A_PER], rb[G::B_PER];
  uint32_t rq[BQ ? G::B_PER : 1];  // packed int4 words of the tile in flight (BQ, segment 0)
  bool quant_tile = false;         // the tile in flight is one of the int4 segment
  [[maybe_unused]] i32x4 rl[FUSE ? G::L_PER : 1];    // slice of LA of the tile in flight
  [[maybe_unused]] f32x16 tacc[FUSE ? G::TT : 1];    // T blocks of this wave: row blocks a with a % WN == wn
  if constexpr (FUSE) {
#pragma unroll
    for (int a = 0; a < G::TT; ++a)
#pragma unroll
      for (int v = 0; v < 16; ++v) tacc[a][v] = 0.f;
  }

  auto load_global = [&](int t) {
    const int s = t < nt0 ? 0 : 1;
    const int k0 = (t - (s ? nt0 : 0)) * BK;
    const int Ks = g.K[s];
    const T* Ap = static_cast<const T*>(g.A[s]);
    const T* Bp = static_cast<const T*>(g.B[s]);
    const int64_t lda = g.lda[s], ldb = g.ldb[s];
    if constexpr (FUSE) {
      if (s == 0) {
#pragma unroll
        for (int j = 0; j < G::L_PER; ++j) {
          const int c = tid + j * NT;
          const int row = c / G::L_CPR, col = (c % G::L_CPR) * VE;
          i32x4 v = {0, 0, 0, 0};
          if ((G::L_CHUNKS % NT == 0 || c < G::L_CHUNKS) && k0 + row < Ks && col < g.R)
            v = *reinterpret_cast<const i32x4*>(static_cast<const T*>(g.LA) + (int64_t)(k0 + row) * g.ldla + col);
          rl[j] = v;
        }
      }
    }
#pragma unroll
    for (int j = 0; j < G::A_PER; ++j) {
      if (FUSE && s == 1) break;  // the A operand of segment 1 is T, formed in the kernel
      const int c = tid + j * NT;
      const int row = c / G::A_CPR, col = (c % G::A_CPR) * VE;
      i32x4 v = {0, 0, 0, 0};
      if (G::A_CHUNKS % NT == 0 || c < G::A_CHUNKS) {
        if constexpr (!G::A_STR) {  // row = m, col = k
          if (m0 + row < g.M && k0 + col < Ks)
            v = *reinterpret_cast<const i32x4*>(Ap + (int64_t)(m0 + row) * lda + k0 + col);
        } else {  // row = k, col = m
          if (k0 + row < Ks && m0 + col < g.M)
            v = *reinterpret_cast<const i32x4*>(Ap + (int64_t)(k0 + row) * lda + m0 + col);
        }
      }
      ra[j] = v;
    }
    if constexpr (BQ) quant_tile = (s == 0);
#pragma unroll
    for (int j = 0; j < G::B_PER; ++j) {
      const int c = tid + j * NT;
      const int row = c / G::B_CPR, col = (c % G::B_CPR) * VE;
      i32x4 v = {0, 0, 0, 0};
      uint32_t w = 0x88888888u;  // eight zeros in the int4 encoding
      if (G::B_CHUNKS % NT == 0 || c < G::B_CHUNKS) {
        // (sr, sc) = position in the stored matrix
        const int sr = G::B_STR ? k0 + row : n0 + row, sc = G::B_STR ? n0 + col : k0 + col;
        const bool ok = G::B_STR ? (k0 + row < Ks && n0 + col < g.N) : (n0 + row < g.N && k0 + col < Ks);
        if (ok) {
          if (BQ && s == 0) {
            w = *reinterpret_cast<const uint32_t*>(static_cast<const unsigned char*>(g.B[0]) + (((int64_t)sr * ldb + sc) >> 1));
            v = *reinterpret_cast<const i32x4*>(static_cast<const _Float16*>(g.Bscale) + (int64_t)(sr >> 6) * g.ldbs + sc);
          } else {
            v = *reinterpret_cast<const i32x4*>(Bp + (int64_t)sr * ldb + sc);
          }
        }
      }
      rb[j] = v;
      if constexpr (BQ) rq[j] = w;
    }
  };

  // t_tile (FUSE): the tile being stored is the one of segment 1: its A half is T out of the accumulators
  auto store_lds = [&](int stage, [[maybe_unused]] bool t_tile) {
    T* sA = smem + stage * STAGE_ELEMS;
    T* sB = sA + G::A_ELEMS;
    if (FUSE && t_tile) {
      if constexpr (FUSE) {
        // lane l of a 32x32 block holds row l % 32 and, for q = 0..3, columns 8 q + 4 (l / 32) + {0..3}
#pragma unroll
        for (int a = 0; a < G::TM; ++a) {
          if (a % WN != wn) continue;
          T* row = sA + (wm * G::WTM + a * 32 + (lane & 31)) * G::A_LD + 4 * (lane >> 5);
#pragma unroll
          for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int e = 0; e < 4; ++e) row[8 * q + e] = from_f32<T>(g.t_alpha * tacc[a / WN][4 * q + e]);
        }
      }
    } else {
#pragma unroll
      for (int j = 0; j < G::A_PER; ++j) {
        const int c = tid + j * NT;
        if (G::A_CHUNKS % NT == 0 || c < G::A_CHUNKS)
          *reinterpret_cast<i32x4*>(sA + (c / G::A_CPR) * G::A_LD + (c % G::A_CPR) * VE) = ra[j];
      }
      if constexpr (FUSE) {
        T* sL = sB + G::B_ELEMS;
#pragma unroll
        for (int j = 0; j < G::L_PER; ++j) {
          const int c = tid + j * NT;
          if (G::L_CHUNKS % NT == 0 || c < G::L_CHUNKS)
            *reinterpret_cast<i32x4*>(sL + (c / G::L_CPR) * G::L_LD + (c % G::L_CPR) * VE) = rl[j];
        }
      }
    }
#pragma unroll
    for (int j = 0; j < G::B_PER; ++j) {
      const int c = tid + j * NT;
      if (G::B_CHUNKS % NT == 0 || c < G::B_CHUNKS) {
        i32x4 v = rb[j];
        if constexpr (BQ) {
          if (quant_tile) v = dequant_chunk<T>(rq[j], rb[j]);
        }
        *reinterpret_cast<i32x4*>(sB + (c / G::B_CPR) * G::B_LD + (c % G::B_CPR) * VE) = v;
      }
    }
  };

  if (t_begin < t_end) {
    load_global(t_begin);
    store_lds(0, false);  // (a FUSE launch has K[0] >= 1: its first tile is never the T tile)
  }
  __syncthreads();

  int stage = 0;
  for (int t = t_begin; t < t_end; ++t) {
    const bool more = (t + 1 < t_end);
    if (more) load_global(t + 1);
    const T* sA = smem + stage * STAGE_ELEMS;
    const T* sB = sA + G::A_ELEMS;
    [[maybe_unused]] const bool main_tile = t < nt0;
#pragma unroll
    for (int ks = 0; ks < BK / G::KS; ++ks) {
      if (FUSE && !main_tile && ks >= G::RP / G::KS) break;  // T is RP wide: the rest of the A half is not its
      i32x4 fa[G::TM], fb[G::TN];
#pragma unroll
      for (int a = 0; a < G::TM; ++a)
        fa[a] = read_frag<T, G::A_STR, G::A_LD>(sA, wm * G::WTM + a * 32, ks, lane);
#pragma unroll
      for (int b = 0; b < G::TN; ++b)
        fb[b] = read_frag<T, G::B_STR, G::B_LD>(sB, wn * G::WTN + b * 32, ks, lane);
#pragma unroll
      for (int a = 0; a < G::TM; ++a)
#pragma unroll
        for (int b = 0; b < G::TN; ++b) Elem<T>::mma(acc[a][b], fb[b], fa[a]);  // rows of the MFMA = n
      if constexpr (FUSE) {
        if (main_tile) {
          const i32x4 fl = read_frag<T, true, G::L_LD>(sB + G::B_ELEMS, 0, ks, lane);
#pragma unroll
          for (int a = 0; a < G::TM; ++a)
            if (a % WN == wn) Elem<T>::mma(tacc[a / WN], fl, fa[a]);
        }
      }
    }
    if (more) store_lds(stage ^ 1, FUSE && t + 1 >= nt0);
    __syncthreads();
    stage ^= 1;
  }

  // ---- epilogue
  Epilogue ep{g.C, g.ldc, g.D, g.ldd, g.partial, g.M, g.N, (int)blockIdx.y, g.alpha, g.bias, g.drop_thr, g.drop_key, g.drop_cpr};
#pragma unroll
  for (int a = 0; a < G::TM; ++a)
#pragma unroll
    for (int b = 0; b < G::TN; ++b)
      store_block<T>(ep, acc[a][b], m0 + wm * G::WTM + a * 32 + (lane & 31), n0 + wn * G::WTN + b * 32, lane);
}

// Sum the split-K partials in slice order and round once: C = alpha * sum_z partial[z] (+ D) (+ bias).
template <typename T>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ partial, int splits,
                                                            int M, int N, T* __restrict__ C, int64_t ldc,
                                                            const T* __restrict__ D, int64_t ldd, float alpha,
                                                            const T* __restrict__ bias, uint32_t drop_thr,
                                                            uint32_t drop_key, uint32_t drop_cpr) {
  const int64_t quads = (int64_t)M * N / 4;  // N is a multiple of 4
  for (int64_t qd = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; qd < quads;
       qd += (int64_t)gridDim.x * blockDim.x) {
    const int64_t e = qd * 4;
    const int m = (int)(e / N), n = (int)(e % N);
    f32x4 s = *reinterpret_cast<const f32x4*>(partial + e);
    for (int z = 1; z < splits; ++z) {
      f32x4 p = *reinterpret_cast<const f32x4*>(partial + (int64_t)z * M * N + e);
      s += p;
    }
    if (alpha != 1.f) s *= alpha;
    if (drop_thr != 0u) {
      uint32_t keep[4];
      drop_keep4((uint32_t)m * drop_cpr + (uint32_t)(n >> 2), drop_key, drop_thr, keep);
#pragma unroll
      for (int k = 0; k < 4; ++k) s[k] = keep[k] ? s[k] : 0.f;
    }
    if (D) {
#pragma unroll
      for (int k = 0; k < 4; ++k) s[k] += (float)D[(int64_t)m * ldd + n + k];
    }
    if (bias) {
#pragma unroll
      for (int k = 0; k < 4; ++k) s[k] += (float)bias[n + k];
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) C[(int64_t)m * ldc + n + k] = from_f32<T>(s[k]);
  }
}

}  // namespace rl
