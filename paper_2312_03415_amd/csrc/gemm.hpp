// Host-side interface of the tile GEMM engine (gemm_engine.hpp): problem description, launch plan
// (tile shape + split of the contraction) and launch.  Internal to the library.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stddef.h>
#include <stdint.h>

namespace rl {

enum { DT_F32 = 0, DT_F16 = 1, DT_BF16 = 2 };

// C[M,N] (dtype) = sum_s op(A_s) op(B_s) (+ D).
struct GemmDesc {
  int dtype = DT_BF16;
  int a_strided = 0;  // 0: A_s stored [M,K_s] row-major; 1: A_s stored [K_s,M]
  int b_kcontig = 0;  // 0: B_s stored [K_s,N] row-major; 1: B_s stored [N,K_s]
  int64_t M = 0, N = 0;
  int nseg = 1;
  const void* A[2] = {nullptr, nullptr};
  const void* B[2] = {nullptr, nullptr};
  int64_t lda[2] = {0, 0}, ldb[2] = {0, 0}, K[2] = {0, 0};
  void* C = nullptr;
  int64_t ldc = 0;
  const void* D = nullptr;  // optional addend, same dtype as C (may alias C)
  int64_t ldd = 0;
  bool has_addend = false;  // an addend is part of the product (also set when only shapes are modelled and D is null)
  // B[0] is symmetric int4 (packed nibbles, ldb[0] in elements) with fp16 group scales
  // [rows/64, ldbs]; nullptr = dense.  16-bit types, A stored [M,K].
  const void* Bscale = nullptr;
  int64_t ldbs = 0;
  bool b_int4 = false;  // B[0] is int4 (set together with Bscale; also when only shapes are modelled)
  // C = alpha * (sum of the products) + D + bias;  bias: row vector [N] of the dtype, or nullptr
  float alpha = 1.f;
  const void* bias = nullptr;
  // LoRA dropout (drop_thr != 0): zero output element (m, n) of alpha * (the products) where the mask
  // drops element (m, n) of X; key and threshold as in gemm_engine.hpp, drop_cpr = columns of X / 4
  uint32_t drop_thr = 0, drop_key = 0, drop_cpr = 0;
  // One-pass LoRA forward, C = A[0] B[0] + round(t_alpha A[0] LA) B[1] in one kernel: nseg = 2, A[1] unused,
  // K[1] = R <= kFuseMaxR, LA stored [K[0], R] row-major; A [M,K], B [K,N], dense B, no addend, no K split
  // (plan with gemm_plan_fused).  fuse_t is also set when only shapes are modelled and LA is null.
  const void* LA = nullptr;
  int64_t ldla = 0;
  float t_alpha = 1.f;
  bool fuse_t = false;
};
constexpr int64_t kFuseMaxR = 32;

enum TileCfg {
  CFG_BIG = 0, CFG_MID, CFG_TALL32, CFG_TALL64, CFG_WIDE32, CFG_WIDE64,
  CFG_MC3,  // matrix-core kernel (gemm_mc.hpp, 16-bit types): 256x256x32, 4 waves, 3-stage LDS ring, 32x32x16 products
            // (the int4 route of the frozen weight runs here)
  CFG_MC4,  // matrix-core kernel (gemm_mc64.hpp, 16-bit types): 256x256x64, 4 waves, 2 LDS stages, 16x16x32 products
            // (the id the heuristics pick for dense B)
  CFG_COUNT
};

struct GemmPlan {
  int cfg = CFG_MID;
  int bm = 128, bn = 128, bk = 64;
  int nbm = 1, nbn = 1;
  int splits = 1;            // > 1: fp32 partials + fixed-order reduce
  int tiles_per_split = 1;
  size_t partial_bytes = 0;  // scratch needed when splits > 1 (or by the tail launch)
  // > 0: the output columns [tail_n0, N) are a launch of their own, planned by gemm_plan on that
  // sub-problem (a few tiles with the contraction split), so that the main launch is whole rounds of
  // one tile per compute unit instead of ending on a mostly idle round
  int64_t tail_n0 = 0;
};

// Tile shape and K split for a problem; depends on shapes and dtype only (never on pointers), so
// the same plan sizes the workspace and drives the launch.  force_cfg / force_splits (>= 0 / > 0)
// override the heuristics (used by the tuning sweeps and tests).
GemmPlan gemm_plan(int dtype, int64_t M, int64_t N, int64_t K0, int64_t K1, int force_cfg = -1,
                   int force_splits = 0, bool b_int4 = false);

// Plan for the one-pass LoRA forward (GemmDesc::fuse_t): a tile shape of the generic engine, the contraction whole.
GemmPlan gemm_plan_fused(int dtype, int64_t M, int64_t N, int64_t K0, int64_t R);

// Plan of the launch that computes the columns [main.tail_n0, N) cut off from `main`.
GemmPlan gemm_tail_plan(const GemmPlan& main, int dtype, int64_t M, int64_t N, int64_t K0, int64_t K1);

// Plan for a product whose B[0] is int4 (GemmDesc::Bscale): matrix-core kernel or the generic
// engine's 128x128 tile.
GemmPlan gemm_plan_int4(int dtype, int64_t M, int64_t N, int64_t K0, int64_t K1);

// Enqueue the product.  `scratch` must hold plan.partial_bytes when plan.splits > 1.
hipError_t gemm_run(const GemmDesc& d, const GemmPlan& plan, float* scratch, hipStream_t stream);

// ---- streaming kernel for the rank-r products (skinny.hpp) --------------------------------------
// C[M,N<=128] = op(A)[M,K] op(B)[K,N], optionally stored transposed; up to two problems per launch.
struct SkinnyDesc {
  const void* A = nullptr;
  const void* B = nullptr;
  void* C = nullptr;
  int64_t lda = 0, ldb = 0, ldc = 0;
  int64_t M = 0, N = 0, K = 0;
  int a_strided = 0, b_kcontig = 0, trans_out = 0;
  float alpha = 1.f;  // C = alpha * op(A) op(B)
  uint32_t drop_thr = 0, drop_key = 0, drop_cpr = 0;  // != 0: A is X, masked by LoRA dropout on load
};
struct SkinnyPlan {
  int rt = 1;      // 32-column blocks per row block: N <= 32*rt
  int splits = 1;  // K split over workgroups (fp32 partials + ordered reduce)
  int mr = 1;      // 32-row blocks per workgroup: 2 for paired launches in the [K,M] orientation with N <= 64
  size_t partial_bytes = 0;
};
inline bool skinny_ok(int64_t N) { return N <= 128; }
SkinnyPlan skinny_plan(int dtype, int nprob, const SkinnyDesc* d);
hipError_t skinny_run(int dtype, int nprob, const SkinnyDesc* d, const SkinnyPlan& plan, float* scratch,
                      hipStream_t stream);
struct SkinnyArgs;
hipError_t skinny_launch_bf16(int rt, const SkinnyArgs& a, dim3 grid, int splits, hipStream_t s);
hipError_t skinny_launch_f16(int rt, const SkinnyArgs& a, dim3 grid, int splits, hipStream_t s);
hipError_t skinny_launch_f32(int rt, const SkinnyArgs& a, dim3 grid, int splits, hipStream_t s);

// ---- timing of a step's kernels ----------------------------------------------------------------------
// While event pairs are set here (per host thread), every kernel of the step launched from this thread (the tile
// GEMM, a cut-off tail launch, the streaming kernel, the merge kernel and the reduce kernels behind them) is
// launched with the next unused pair bound to its own dispatch, so that the pair's difference is that kernel's
// duration alone, as a kernel trace reports it.  Pair 0 is the step's first (main) kernel.
struct KernelEvents {
  static constexpr int kMax = 4;
  hipEvent_t start[kMax] = {nullptr, nullptr, nullptr, nullptr}, stop[kMax] = {nullptr, nullptr, nullptr, nullptr};
  int avail = 0, used = 0;
};
extern thread_local KernelEvents g_kernel_events;
template <typename Kern, typename... Args>
inline void launch_timed(Kern kern, dim3 grid, dim3 block, unsigned lds, hipStream_t s, Args... args) {
  KernelEvents& ke = g_kernel_events;
  if (ke.used < ke.avail) {
    hipExtLaunchKernelGGL(kern, grid, block, lds, s, ke.start[ke.used], ke.stop[ke.used], 0, args...);
    ++ke.used;
  } else {
    hipLaunchKernelGGL(kern, grid, block, lds, s, args...);
  }
}

// ---- M = W + A B (merge.hpp): 16-bit types, r <= 128 --------------------------------------------
struct MergeDesc {
  const void *W = nullptr, *A = nullptr, *B = nullptr;
  void* M = nullptr;
  int64_t ldw = 0, lda = 0, ldb = 0, ldm = 0;
  int64_t I = 0, O = 0, R = 0;
  float alpha = 1.f;  // M = W + alpha A B
  int b_trans = 0;    // B stored [O, R]
  const float* wcol = nullptr;  // optional [O]: M = W diag(wcol) + alpha A B
  // optional: store nothing to M; write the squared column sums of W + alpha A B, one row of O floats per
  // row slice of the launch (merge_grid's gy rows; the caller adds them up)
  float* sq_partial = nullptr;
  // drop_thr != 0: M = W + mask o (alpha A B) with the LoRA dropout keep-mask over M's elements (gemm_engine.hpp)
  uint32_t drop_thr = 0, drop_key = 0, drop_cpr = 0;
};
inline bool merge_ok(int dtype, int64_t r) { return dtype != DT_F32 && r <= 128; }
// the merge kernel's launch shape: gx workgroups of `cols` columns, gy row slices of bpw 32-row blocks each
// (about two workgroups per compute unit, each walking several row blocks)
inline void merge_grid(int64_t I, int64_t O, int64_t R, int* gx, int* gy, int* bpw) {
  const int cols = R <= 64 ? 512 : 256;
  *gx = (int)((O + cols - 1) / cols);
  const int nb = (int)((I + 31) / 32);
  int y = 512 / *gx;
  if (y < 1) y = 1;
  if (y > nb) y = nb;
  *bpw = (nb + y - 1) / y;
  *gy = (nb + *bpw - 1) / *bpw;
}
hipError_t merge_run(int dtype, const MergeDesc& d, hipStream_t stream);
struct MergeArgs;
hipError_t merge_launch_bf16(const MergeArgs& a, hipStream_t s);
hipError_t merge_launch_f16(const MergeArgs& a, hipStream_t s);

// per-dtype launchers (one translation unit each)
struct GemmArgs;
hipError_t gemm_launch_bf16(int cfg, int al, int bl, const GemmArgs& a, dim3 grid, hipStream_t s);
hipError_t gemm_launch_f16(int cfg, int al, int bl, const GemmArgs& a, dim3 grid, hipStream_t s);
hipError_t gemm_launch_f32(int cfg, int al, int bl, const GemmArgs& a, dim3 grid, hipStream_t s);
struct DropMask { uint32_t thr = 0, key = 0, cpr = 0; };
hipError_t splitk_reduce_launch(int dtype, const float* partial, int splits, int M, int N, void* C,
                                int64_t ldc, const void* D, int64_t ldd, float alpha, const void* bias,
                                DropMask drop, hipStream_t s);

}  // namespace rl
