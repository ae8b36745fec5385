// Streaming kernel for the rank-r products of the LoRA layer (arxiv 2312.03415, Algorithms 1-5):
//   T = X A, Z1 = dY B^T            (long rows in, r columns out)
//   dA = X^T Z1, dB = T^T dY        (reduction over the tokens, r columns out)
//   dA = Z2 B^T, dB = A^T Z2        (Algorithms 2-4)
// All have the shape C[M, N<=128] = op(A)[M,K] op(B)[K,N] with M and K large: each byte of the big
// operand is used for only ~r FLOPs, so the kernel is HBM-bandwidth bound and is built for bytes in
// flight rather than for MFMA occupancy.
//
//  - One workgroup = NWV (4) wavefronts that share a block of 32 * MR output rows and split the
//    workgroup's K range between them.  MR = 2 (64 rows) is used by paired launches whose A operands are
//    stored [K,M] (N <= 64, no LoRA dropout mask: a masked problem is bound by its waves' mask arithmetic): a block's rows are then columns of A, a 32-column strip is 64 bytes per
//    row of A, half a 128-byte line, and the other half has to come from the neighbouring workgroup's
//    fetch staying in L2; with 128-byte strips the paired dA / dB launch runs 20 % faster (OPT shapes:
//    25.6 -> 20.5 us).  Single launches keep 32 rows: halving their workgroup count costs more than the
//    strips gain (dB of OPT fc1 alone: 18.8 -> 23.4 us).  (The workgroup's K range is split between the waves as wave w taking K tiles w, w+NWV, ...; 8 or 16 wavefronts per
//    workgroup measured slower.)  Every wavefront runs its own
//    global -> register -> LDS -> MFMA pipeline on a private LDS region: no workgroup barrier in the
//    loop, the next tile's loads are in flight while the current one is multiplied.
//  - The waves' partial accumulators are summed through LDS in wave order and written once.  A grid
//    that also splits K over workgroups (gridDim.y) writes fp32 partials that a second kernel sums
//    in slice order.  No atomics: results are identical from run to run.
//  - One launch can carry two independent problems (e.g. Z1 and T, or dA and dB): blockIdx.x
//    ranges select the problem, so the pair costs one launch and fills the chip together.
//  - trans_out stores C^T (used for dB, computed as (dY^T T)^T so that its long dimension is M).
#pragma once
#include "gemm_engine.hpp"

namespace rl {

struct SkinnyProblem {
  const void* A;  // a_strided = 0: [M,K] row-major; 1: [K,M]
  const void* B;  // b_kcontig = 0: [K,N] row-major; 1: [N,K]
  void* C;        // [M,N] (trans_out = 0) or [N,M] (trans_out = 1), element type T
  float* partial; // gridDim.y > 1: fp32 [gridDim.y][M][N]
  int64_t lda, ldb, ldc;
  int M, N, K;
  int a_strided, b_kcontig, trans_out;
  int row_blocks;       // ceil(M / (32 * mr))
  int a_bytes, b_bytes; // extent of A and B in bytes (< 2 GiB): the range the loads are checked against
  int tiles_per_split;  // K tiles of this problem per gridDim.y slice
  float alpha;          // C = alpha * op(A) op(B) (the LoRA scale, applied where a rank-r factor is formed)
  // drop_thr != 0: A is the layer input X and its dropped elements (drop_chunk, gemm_engine.hpp) are
  // zeroed on their way to LDS; drop_cpr = groups of four columns per row of X
  uint32_t drop_thr, drop_key, drop_cpr;
};

struct SkinnyArgs {
  SkinnyProblem p[2];
  int nprob;
  int mr;  // 32-row blocks per workgroup (1 or 2): selects the build
};

template <typename T, int RT, int NWV, int MR>
struct SkinnyTile {
  static constexpr int VE = 16 / sizeof(T);
  static constexpr int MB = 32 * MR;  // output rows per workgroup
  static constexpr int BK = 8 * VE;  // 64 (16-bit) or 32 (fp32): 128 bytes of K per row
  static constexpr int KS = 2 * VE;
  static constexpr int NB = 32 * RT;
  // per-wave LDS (elements): the larger of the two orientations of each operand
  static constexpr int A_LD0 = LdsLd<T, false, BK>::value, A_LD1 = LdsLd<T, true, MB>::value;
  static constexpr int B_LD0 = LdsLd<T, true, NB>::value, B_LD1 = LdsLd<T, false, BK>::value;
  static constexpr int A_ELEMS = (32 * A_LD0 > BK * A_LD1) ? 32 * A_LD0 : BK * A_LD1;
  static constexpr int B_ELEMS = (BK * B_LD0 > NB * B_LD1) ? BK * B_LD0 : NB * B_LD1;
  static constexpr int WAVE_ELEMS = A_ELEMS + B_ELEMS;
  static constexpr int STAGE_BYTES = NWV * WAVE_ELEMS * (int)sizeof(T);
  static constexpr int REDUCE_BYTES = NWV * (MB / 32) * RT * 1024 * 4;  // NWV waves x blocks of 32x32 fp32
  static constexpr int LDS_BYTES = STAGE_BYTES > REDUCE_BYTES ? STAGE_BYTES : REDUCE_BYTES;
};

// One problem's work for this workgroup.  AL / BL are the operand layouts (compile time, so that
// the load and fragment paths are straight-line code): AL = 1: A stored [K,M]; BL = 1: B stored [N,K].
// DROP: this problem's A is the layer input X under LoRA dropout and is masked on its way to LDS (a compile-time
// property of the problem's slot in the launch: a run-time test in the loop cost the whole launch a factor of two,
// masked problem or not); the plain build carries none of it.
template <typename T, int RT, int NWV, int AL, int BL, bool DROP, int MR>
__device__ __forceinline__ void skinny_body(const SkinnyProblem& P, int bx, unsigned char* smem_raw) {
  using S = SkinnyTile<T, RT, NWV, MR>;
  constexpr int VE = S::VE, BK = S::BK;
  constexpr bool a_str = AL != 0, b_kc = BL != 0;
  static_assert(MR == 1 || (AL != 0 && RT <= 2), "64-row blocks exist for the [K,M] orientation only");
  constexpr int MB = 32 * MR;  // output rows of this workgroup
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int m0 = bx * MB;
  const int M = P.M, N = P.N, K = P.K;
  const T* Ap = static_cast<const T*>(P.A);
  const T* Bp = static_cast<const T*>(P.B);
  const int64_t lda = P.lda, ldb = P.ldb;

  const int ktiles = (K + BK - 1) / BK;
  const int t_begin = blockIdx.y * P.tiles_per_split;
  int t_end = t_begin + P.tiles_per_split;
  if (t_end > ktiles) t_end = ktiles;

  T* sA = reinterpret_cast<T*>(smem_raw) + wave * S::WAVE_ELEMS;
  T* sB = sA + S::A_ELEMS;

  f32x16 acc[MR][RT];
#pragma unroll
  for (int a = 0; a < MR; ++a)
#pragma unroll
    for (int b = 0; b < RT; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  constexpr int A_PER = 4 * MR;  // 32 x 8 chunks (or BK x MB/VE) over 64 lanes
  constexpr int B_PER = 4 * RT;  // BK x NB/VE... = 256*RT chunks over 64 lanes
  // register stages: the loads of DEPTH tiles are in flight per wave (a streaming kernel lives on
  // bytes in flight, not on occupancy)
  constexpr int DEPTH = MR * RT == 1 ? 4 : (MR * RT == 2 ? 3 : 2);  // (6 stages at RT = 1 measured 7-28 % slower)
  i32x4 ra[DEPTH][A_PER], rb[DEPTH][B_PER];

  // Loads go through buffer descriptors: a lane whose chunk lies outside the matrix (or whose tile
  // lies beyond this wave's share) uses an offset past the end of the buffer and receives zeros
  // from the hardware's range check.  No branch and no select around the loads, so every path
  // issues the same number of them and the waits can count how many are still in flight.
  const __amdgpu_buffer_rsrc_t rsrcA = __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(Ap), 0, P.a_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrcB = __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(Bp), 0, P.b_bytes, 0x00020000);
  constexpr uint32_t OOB = 0x80000000u;  // buffers are < 2 GiB (checked on the host)
  const uint32_t ulda = (uint32_t)lda, uldb = (uint32_t)ldb;
  // Workgroups walk their K range from different starting tiles (a rotation by the row-block
  // index): at any instant the workgroups then read different columns of the big operand, which
  // spreads the requests over the memory channels instead of all hitting the same column offset.
  const int span = t_end - t_begin;
  const int rot = span > 0 ? (bx * 5) % span : 0;
  int kst[DEPTH];  // k origin of the tile in each register stage (for the dropout mask)
  auto load_global = [&](int d, int q) {  // q = position in this workgroup's tile sequence
    const bool live = q < span;
    int tq = q + rot;
    if (tq >= span) tq -= span;
    const int k0 = (t_begin + tq) * BK;
    if constexpr (DROP) kst[d] = k0;
#pragma unroll
    for (int j = 0; j < A_PER; ++j) {
      const int c = lane + 64 * j;
      bool ok;
      uint32_t off;
      if constexpr (!a_str) {  // tile [32 m][BK k]: 8 chunks per row
        const int row = c >> 3, col = (c & 7) * VE;
        ok = live && m0 + row < M && k0 + col < K;
        off = (uint32_t)(m0 + row) * ulda + (uint32_t)(k0 + col);
      } else {  // tile [BK k][MB m]: MB/VE chunks per row
        constexpr int CPR = MB / VE;
        const int row = c / CPR, col = (c % CPR) * VE;
        ok = live && k0 + row < K && m0 + col < M;
        off = (uint32_t)(k0 + row) * ulda + (uint32_t)(m0 + col);
      }
      ra[d][j] = __builtin_amdgcn_raw_buffer_load_b128(rsrcA, ok ? off * (uint32_t)sizeof(T) : OOB, 0, 0);
    }
#pragma unroll
    for (int j = 0; j < B_PER; ++j) {
      const int c = lane + 64 * j;
      bool ok;
      uint32_t off;
      if constexpr (!b_kc) {  // tile [BK k][NB n]
        constexpr int CPR = S::NB / VE;
        const int row = c / CPR, col = (c % CPR) * VE;
        ok = live && k0 + row < K && col < N;
        off = (uint32_t)(k0 + row) * uldb + (uint32_t)col;
      } else {  // tile [NB n][BK k]: 8 chunks per row
        const int row = c >> 3, col = (c & 7) * VE;
        ok = live && row < N && k0 + col < K;
        off = (uint32_t)row * uldb + (uint32_t)(k0 + col);
      }
      rb[d][j] = __builtin_amdgcn_raw_buffer_load_b128(rsrcB, ok ? off * (uint32_t)sizeof(T) : OOB, 0, 0);
    }
  };

  auto store_lds = [&](int d) {
    if constexpr (DROP) {  // A is X under LoRA dropout
#pragma unroll
      for (int j = 0; j < A_PER; ++j) {
        const int c = lane + 64 * j;
        uint32_t t, col;  // token (row of X) and first column of X of this chunk
        if constexpr (!a_str) {
          t = (uint32_t)(m0 + (c >> 3));
          col = (uint32_t)(kst[d] + (c & 7) * VE);
        } else {
          constexpr int CPR = MB / VE;
          t = (uint32_t)(kst[d] + c / CPR);
          col = (uint32_t)(m0 + (c % CPR) * VE);
        }
        ra[d][j] = drop_chunk<T>(ra[d][j], t * P.drop_cpr + (col >> 2), P.drop_key, P.drop_thr);
      }
    }
#pragma unroll
    for (int j = 0; j < A_PER; ++j) {
      const int c = lane + 64 * j;
      if constexpr (!a_str) {
        *reinterpret_cast<i32x4*>(sA + (c >> 3) * S::A_LD0 + (c & 7) * VE) = ra[d][j];
      } else {
        constexpr int CPR = MB / VE;
        *reinterpret_cast<i32x4*>(sA + (c / CPR) * S::A_LD1 + (c % CPR) * VE) = ra[d][j];
      }
    }
#pragma unroll
    for (int j = 0; j < B_PER; ++j) {
      const int c = lane + 64 * j;
      if constexpr (!b_kc) {
        constexpr int CPR = S::NB / VE;
        *reinterpret_cast<i32x4*>(sB + (c / CPR) * S::B_LD0 + (c % CPR) * VE) = rb[d][j];
      } else {
        *reinterpret_cast<i32x4*>(sB + (c >> 3) * S::B_LD1 + (c & 7) * VE) = rb[d][j];
      }
    }
  };

  // wave w owns tiles t_begin + w + NWV*j, j = 0 .. J-1 (the same J for every wave; tiles past
  // t_end load zeros), walked DEPTH at a time with all loop bounds uniform
  const int J = (t_end - t_begin + NWV - 1) / NWV;
  const int t0 = wave;
#pragma unroll
  for (int d = 0; d < DEPTH; ++d) load_global(d, t0 + NWV * d);
  for (int j0 = 0; j0 < J; j0 += DEPTH) {
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
      store_lds(d);  // same wave wrote/reads this region: LDS operations of one wave stay in order
      load_global(d, t0 + NWV * (j0 + d + DEPTH));
#pragma unroll
      for (int ks = 0; ks < BK / S::KS; ++ks) {
        i32x4 fa[MR];
#pragma unroll
        for (int a = 0; a < MR; ++a)
          fa[a] = a_str ? read_frag<T, true, S::A_LD1>(sA, a * 32, ks, lane) : read_frag<T, false, S::A_LD0>(sA, a * 32, ks, lane);
#pragma unroll
        for (int b = 0; b < RT; ++b) {
          i32x4 fb = b_kc ? read_frag<T, false, S::B_LD1>(sB, b * 32, ks, lane)
                          : read_frag<T, true, S::B_LD0>(sB, b * 32, ks, lane);
#pragma unroll
          for (int a = 0; a < MR; ++a) Elem<T>::mma(acc[a][b], fb, fa[a]);  // MFMA rows = n, columns = m
        }
      }
    }
  }

  // ---- sum the waves' accumulators in wave order through LDS ------------------------------
  __syncthreads();  // every wave is done with its staging region
  float* red = reinterpret_cast<float*>(smem_raw);
  {
    // lane holds row m = l%32, columns n = 8q + 4(l/32) + e of each 32x32 block; red is [wave][n block][m of MB][32 n]
    const int m = lane & 31, nsub = 4 * (lane >> 5);
#pragma unroll
    for (int a = 0; a < MR; ++a)
#pragma unroll
      for (int b = 0; b < RT; ++b)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          f32x4 v = {acc[a][b][4 * q], acc[a][b][4 * q + 1], acc[a][b][4 * q + 2], acc[a][b][4 * q + 3]};
          *reinterpret_cast<f32x4*>(red + ((wave * RT + b) * MB + a * 32 + m) * 32 + 8 * q + nsub) = v;
        }
  }
  __syncthreads();
  // MR*RT*1024 outputs over NWV*64 threads; consecutive threads walk n (row-major store) or m (transposed)
  const bool trans = P.trans_out != 0;
#pragma unroll
  for (int j = 0; j < (16 * MR * RT) / NWV; ++j) {
    const int e = tid + NWV * 64 * j;
    int m, n;
    if (!trans) { n = e % S::NB; m = e / S::NB; } else { m = e % MB; n = e / MB; }
    const int b = n >> 5, nn = n & 31;
    float s = red[((0 * RT + b) * MB + m) * 32 + nn];
#pragma unroll
    for (int w = 1; w < NWV; ++w) s += red[((w * RT + b) * MB + m) * 32 + nn];
    if (m0 + m < M && n < N) {
      if (P.partial) {
        P.partial[((int64_t)blockIdx.y * M + (m0 + m)) * N + n] = s;  // unscaled: the reduce applies alpha
        continue;
      }
      s *= P.alpha;
      if (!trans) {
        static_cast<T*>(P.C)[(int64_t)(m0 + m) * P.ldc + n] = from_f32<T>(s);
      } else {
        static_cast<T*>(P.C)[(int64_t)n * P.ldc + (m0 + m)] = from_f32<T>(s);
      }
    }
  }
}

// AL is common to both problems of a paired launch; BL0 / BL1 are their B layouts.
// DROPM: bit w set = problem w of the launch is masked (see skinny_body)
template <typename T, int RT, int NWV, int AL, int BL0, int BL1, int DROPM = 0, int MR = 1>
__global__ __launch_bounds__(NWV * 64) void skinny_kernel(SkinnyArgs g) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  // Consecutive workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2 and its own
  // path to memory.  Renumber so that (a) neighbouring row blocks of a problem run on the same XCD: a
  // [K,M] operand is read in 64-byte column strips, and the two strips that share a 128-byte line
  // should be fetched through one L2; and (b) each problem of a paired launch is spread over all
  // eight XCDs in proportion: XCD x takes the x-th eighth of problem 0's row blocks, then the x-th
  // eighth of problem 1's.  (Dealing the ids out problem after problem would put a long problem on
  // half of the XCDs and leave the other half idle once the short one is done.)  The grid holds
  // 8 * (ceil(R0/8) + ceil(R1/8)) workgroups; the few without a row block leave at once.
  const int x = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int R0 = g.p[0].row_blocks, R1 = g.nprob > 1 ? g.p[1].row_blocks : 0;
  const int n0 = R0 / 8 + (x < (R0 & 7) ? 1 : 0), s0 = x * (R0 / 8) + (x < (R0 & 7) ? x : (R0 & 7));
  if (slot < n0) {
    skinny_body<T, RT, NWV, AL, BL0, (DROPM & 1) != 0, MR>(g.p[0], s0 + slot, smem_raw);
    return;
  }
  const int n1 = R1 / 8 + (x < (R1 & 7) ? 1 : 0), s1 = x * (R1 / 8) + (x < (R1 & 7) ? x : (R1 & 7));
  if (slot - n0 < n1) skinny_body<T, RT, NWV, AL, BL1, (DROPM & 2) != 0, MR>(g.p[1], s1 + (slot - n0), smem_raw);
}

// Second stage for a K split over workgroups: C = sum over slices (in slice order) of the fp32
// partials, rounded once; both problems of a paired launch in one go.
template <typename T>
__global__ __launch_bounds__(256) void skinny_reduce_kernel(SkinnyArgs g, int splits) {
  for (int w = 0; w < g.nprob; ++w) {
    const SkinnyProblem& P = g.p[w];
    const int64_t total = (int64_t)P.M * P.N;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
      // walk the output in its storage order so that stores coalesce
      int m, n;
      if (!P.trans_out) { m = (int)(e / P.N); n = (int)(e % P.N); } else { n = (int)(e / P.M); m = (int)(e % P.M); }
      const float* src = P.partial + (int64_t)m * P.N + n;
      float s = src[0];
      for (int z = 1; z < splits; ++z) s += src[(int64_t)z * total];
      s *= P.alpha;
      if (!P.trans_out) static_cast<T*>(P.C)[(int64_t)m * P.ldc + n] = from_f32<T>(s);
      else static_cast<T*>(P.C)[(int64_t)n * P.ldc + m] = from_f32<T>(s);
    }
  }
}

}  // namespace rl
