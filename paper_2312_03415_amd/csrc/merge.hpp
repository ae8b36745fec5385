// M = W + alpha A B for the merged-weight graphs (forward2, Eq. 2; Z1 / Z3 of Algorithms 4 and 5 of arxiv
// 2312.03415): [i,o] = [i,o] + [i,r][r,o] with r <= 128, bf16 / fp16.  The default chain's rank-r updates
// (Y += T B, dX += Z1 A^T: the same operation on [n,o] / [n,i], in place) run here as well, and so do the two
// passes DoRA adds: the squared column norms of W + alpha A B (nothing stored) and W diag(g) + alpha A B.
//
// The product is tiny (2 i o r FLOPs); the kernel reads W once and writes M once, so it is bound by
// HBM bandwidth (2 i o e bytes) and is organised around coalesced 16-byte accesses with many of
// them in flight:
//  - a workgroup (4 wavefronts) owns a strip of columns (each wave 32*CB of them) and walks a
//    range of 32-row blocks.  The B fragments of its columns are read once (through LDS, with the
//    transposing LDS load) and stay in registers for the whole walk.
//  - per row block: the A fragment (32 rows x r) comes straight from global memory, r/16 MFMAs per
//    32x32 block give A B in fp32, the wave passes it through its private LDS region to turn the
//    MFMA's register layout into rows, adds W (prefetched one row block ahead, 16 bytes per lane,
//    whole 128/256-byte row segments per wave instruction), rounds once and stores 16 bytes per lane.
//    W is read with non-temporal loads: nothing reads it again soon, while M is read by the next kernel.
#pragma once
#include "gemm_engine.hpp"

namespace rl {

struct MergeArgs {
  const void *W, *A, *B;
  void* M;
  int64_t ldw, lda, ldb, ldm;
  int I, O, R;
  int blocks_per_wg;  // 32-row blocks each workgroup walks (gridDim.y covers ceil(I/32) of them)
  float alpha;        // the layer's LoRA scale (1 for the paper's layer)
  int b_trans;        // 1: B is stored [O, R] (the r values of a column contiguous), as A^T of dX += Z1 A^T is
  const float* wcol;  // optional [O]: M = W diag(wcol) + alpha A B (the column-scaled frozen weight of DoRA)
  // optional [gridDim.y][O]: nothing is stored to M; each workgroup writes, per column, the sum over its
  // rows of (W + alpha A B)^2 in fp32 (the squared column norms, summed over gridDim.y by the caller)
  float* sq_partial;
  // drop_thr != 0: the product is masked before it is added, M = W + mask o (alpha A B), with the LoRA dropout
  // keep-mask of element (row, column) of M (drop_keep4, gemm_engine.hpp; drop_cpr = groups of four columns per row)
  uint32_t drop_thr, drop_key, drop_cpr;
};

template <int KSTEPS, int CB>
struct MergeTile {
  static constexpr int COLS = 32 * CB;        // columns per wave
  static constexpr int LD = COLS + 4;         // fp32 row length of the transposition buffer
  static constexpr int RED_BYTES = 32 * LD * 4, STAGE_BYTES = 16 * KSTEPS * COLS * 2;
  static constexpr int WAVE_BYTES = RED_BYTES > STAGE_BYTES ? RED_BYTES : STAGE_BYTES;
  static constexpr int LDS_BYTES = 4 * WAVE_BYTES;
  static constexpr int LPR = COLS / 8;        // lanes per output row (8 columns each)
  static constexpr int RPP = 64 / LPR;        // rows per pass
  static constexpr int PASSES = 32 / RPP;
};

template <typename T, int KSTEPS, int CB>
__global__ __launch_bounds__(256) void merge_kernel(MergeArgs g) {
  using MT = MergeTile<KSTEPS, CB>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l31 = lane & 31, hi = lane >> 5;
  unsigned char* wsm = smem_raw + wave * MT::WAVE_BYTES;  // this wave's LDS region
  const int n0 = (blockIdx.x * 4 + wave) * MT::COLS;      // first column of this wave
  const T* Wp = static_cast<const T*>(g.W);
  const T* Ap = static_cast<const T*>(g.A);
  const T* Bp = static_cast<const T*>(g.B);
  T* Mp = static_cast<T*>(g.M);

  // ---- B fragments of this wave's columns: stage B[0:16*KSTEPS, n0:n0+COLS] (zero beyond r / o) in
  // LDS as [k][COLS], read with the transposing load, keep in registers
  constexpr int BLD = MT::COLS;  // read once per workgroup: bank conflicts do not matter here
  T* sB = reinterpret_cast<T*>(wsm);
  for (int c = lane; c < 16 * KSTEPS * (MT::COLS / 8); c += 64) {
    const int k = c / (MT::COLS / 8), col = (c % (MT::COLS / 8)) * 8;
    i32x4 v = {0, 0, 0, 0};
    if (!g.b_trans && k < g.R && n0 + col < g.O) v = *reinterpret_cast<const i32x4*>(Bp + (int64_t)k * g.ldb + n0 + col);
    *reinterpret_cast<i32x4*>(sB + k * BLD + col) = v;
  }
  if (g.b_trans) {  // B stored [O, R]: 16 bytes = eight k of one column, scattered into the [k][COLS] tile (once per workgroup)
    __builtin_amdgcn_s_waitcnt(0xc07f);
    for (int c = lane; c < MT::COLS * (2 * KSTEPS); c += 64) {
      const int col = c / (2 * KSTEPS), k8 = (c % (2 * KSTEPS)) * 8;
      if (n0 + col < g.O && k8 < g.R) {
        const i32x4 v = *reinterpret_cast<const i32x4*>(Bp + (int64_t)(n0 + col) * g.ldb + k8);
        const T* e8 = reinterpret_cast<const T*>(&v);
#pragma unroll
        for (int e = 0; e < 8; ++e) sB[(k8 + e) * BLD + col] = e8[e];
      }
    }
  }
  __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): the wave's own LDS writes are done (same wave reads them)
  i32x4 fb[CB][KSTEPS];
#pragma unroll
  for (int b = 0; b < CB; ++b)
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) fb[b][ks] = read_frag<T, true, BLD>(sB, b * 32, ks, lane);

  // ---- walk the row blocks
  const int nblocks = (g.I + 31) / 32;
  const int rb0 = blockIdx.y * g.blocks_per_wg;
  int rb1 = rb0 + g.blocks_per_wg;
  if (rb1 > nblocks) rb1 = nblocks;
  const int prow = lane / MT::LPR, pcol = (lane % MT::LPR) * 8;  // this lane's (row in pass, column) for W / M
  const bool col_ok = n0 + pcol < g.O;
  float gs[8], sq[8];  // W's column scale (1 without one) and the running squared column sums of this lane's 8 columns
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    gs[e] = (g.wcol != nullptr && col_ok) ? g.wcol[n0 + pcol + e] : 1.f;
    sq[e] = 0.f;
  }
  // W rows and the A fragment of a row block are fetched one block ahead, so that no global-memory
  // latency sits between two blocks
  i32x4 wreg[MT::PASSES], fnext[KSTEPS];
  auto prefetch = [&](int rb) {
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {  // A fragment: row m = 32 rb + l%32, the 8 k at 16 ks + 8 (l/32)
      const int arow = rb * 32 + l31, k = 16 * ks + 8 * hi;
      i32x4 v = {0, 0, 0, 0};
      if (arow < g.I && k < g.R) v = *reinterpret_cast<const i32x4*>(Ap + (int64_t)arow * g.lda + k);
      fnext[ks] = v;
    }
#pragma unroll
    for (int p = 0; p < MT::PASSES; ++p) {
      const int row = rb * 32 + p * MT::RPP + prow;
      i32x4 v = {0, 0, 0, 0};
      if (col_ok && row < g.I) v = __builtin_nontemporal_load(reinterpret_cast<const i32x4*>(Wp + (int64_t)row * g.ldw + n0 + pcol));
      wreg[p] = v;
    }
  };
  if (rb0 < rb1) prefetch(rb0);
  float* red = reinterpret_cast<float*>(wsm);
  for (int rb = rb0; rb < rb1; ++rb) {
    i32x4 fa[KSTEPS], wcur[MT::PASSES];
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) fa[ks] = fnext[ks];
#pragma unroll
    for (int p = 0; p < MT::PASSES; ++p) wcur[p] = wreg[p];
    if (rb + 1 < rb1) prefetch(rb + 1);
    f32x16 acc[CB];
#pragma unroll
    for (int b = 0; b < CB; ++b) {
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[b][v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KSTEPS; ++ks) Elem<T>::mma(acc[b], fb[b][ks], fa[ks]);
    }
    // register layout (row l%32; columns 8q + 4(l/32) + 0..3 of each block) -> rows in LDS
#pragma unroll
    for (int b = 0; b < CB; ++b)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        f32x4 v = {acc[b][4 * q], acc[b][4 * q + 1], acc[b][4 * q + 2], acc[b][4 * q + 3]};
        *reinterpret_cast<f32x4*>(red + l31 * MT::LD + b * 32 + 8 * q + 4 * hi) = v;
      }
#pragma unroll
    for (int p = 0; p < MT::PASSES; ++p) {
      const int rloc = p * MT::RPP + prow, row = rb * 32 + rloc;
      f32x4 s0 = *reinterpret_cast<const f32x4*>(red + rloc * MT::LD + pcol);
      f32x4 s1 = *reinterpret_cast<const f32x4*>(red + rloc * MT::LD + pcol + 4);
      if (g.drop_thr != 0u) {  // uniform
        uint32_t k0[4], k1[4];
        const uint32_t grp = (uint32_t)row * g.drop_cpr + (uint32_t)((n0 + pcol) >> 2);
        drop_keep4(grp, g.drop_key, g.drop_thr, k0);
        drop_keep4(grp + 1, g.drop_key, g.drop_thr, k1);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          s0[e] = k0[e] ? s0[e] : 0.f;
          s1[e] = k1[e] ? s1[e] : 0.f;
        }
      }
      const T* w8 = reinterpret_cast<const T*>(&wcur[p]);
      if (g.sq_partial != nullptr) {  // uniform: rows and columns outside the matrix contribute zeros
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float v0 = (float)w8[e] + g.alpha * s0[e], v1 = (float)w8[4 + e] + g.alpha * s1[e];
          sq[e] += v0 * v0;
          sq[4 + e] += v1 * v1;
        }
        continue;
      }
      T o8[8];
#pragma unroll
      for (int e = 0; e < 4; ++e) {  // the scaled W is rounded on its own (times 1 is exact), then the sum as before
        o8[e] = from_f32<T>(__fmul_rn((float)w8[e], gs[e]) + g.alpha * s0[e]);
        o8[4 + e] = from_f32<T>(__fmul_rn((float)w8[4 + e], gs[4 + e]) + g.alpha * s1[e]);
      }
      if (col_ok && row < g.I) *reinterpret_cast<i32x4*>(Mp + (int64_t)row * g.ldm + n0 + pcol) = *reinterpret_cast<i32x4*>(o8);
    }
  }
  if (g.sq_partial != nullptr) {
    // the RPP lanes that share a column group add up in a fixed order through the wave's LDS region
    *reinterpret_cast<f32x4*>(red + prow * MT::COLS + pcol) = f32x4{sq[0], sq[1], sq[2], sq[3]};
    *reinterpret_cast<f32x4*>(red + prow * MT::COLS + pcol + 4) = f32x4{sq[4], sq[5], sq[6], sq[7]};
    for (int c = lane; c < MT::COLS; c += 64) {
      float t = 0.f;
      for (int p = 0; p < MT::RPP; ++p) t += red[p * MT::COLS + c];
      if (n0 + c < g.O) g.sq_partial[(int64_t)blockIdx.y * g.O + n0 + c] = t;
    }
  }
}

}  // namespace rl
