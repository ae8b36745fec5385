// Launch planning and dispatch for the tile GEMM engine.
#include "gemm.hpp"
#include "gemm_engine.hpp"
#include "skinny.hpp"
#include "merge.hpp"

namespace rl {

thread_local KernelEvents g_kernel_events;

static const int kTileBM[CFG_COUNT] = {256, 128, 128, 128, 32, 64, 256, 256};
static const int kTileBN[CFG_COUNT] = {256, 128, 32, 64, 128, 128, 256, 256};
static const int kTileBK16[CFG_COUNT] = {64, 64, 64, 64, 64, 64, 32, 64};  // K tile, 16-bit types

// Slices of a contraction of length K for `tiles` output tiles of the matrix-core kernel (one 256x256 workgroup per
// compute unit).  In units of a whole tile's time (0.024 us per k): s slices take ceil(tiles * s / 256) rounds of 1 / s
// each; the reduce pass reads s fp32 partials per output at ~5.5 TB/s (2 tiles s / K) and is a launch of ~5 us (200 / K).
// 96 tiles at K = 4096 run best in two slices (192 work items, one round of half tiles), not in the three that fill 256
// slots and spill 32 items into a second round.
static int pick_splits(int64_t tiles, int64_t K, int smin) {
  int best = smin;
  double best_cost = 1e30;
  const double k = (double)(K > 0 ? K : 1);
  for (int s = smin; s <= 8; ++s) {
    const double rounds = (double)((tiles * s + 255) / 256);
    const double cost = rounds / s + (s > 1 ? 2.0 * (double)tiles * s / k + 200.0 / k : 0.0);
    if (cost < best_cost - 1e-9) { best_cost = cost; best = s; }
  }
  return best;
}

GemmPlan gemm_plan(int dtype, int64_t M, int64_t N, int64_t K0, int64_t K1, int force_cfg,
                   int force_splits, bool b_int4) {
  GemmPlan p;
  int cfg;
  if (b_int4 && force_cfg < 0) {
    // an int4 B runs on the matrix-core kernel (3-stage ring) when its 256x256 tiles fill the chip,
    // else on the generic engine's 128x128 tiles
    const int64_t big_tiles = ((M + 255) / 256) * ((N + 255) / 256);
    cfg = (big_tiles >= 160 || (big_tiles >= 80 && K0 + K1 >= 2048)) ? CFG_MC3 : CFG_MID;
  } else if (force_cfg >= 0 && force_cfg < CFG_COUNT) {
    cfg = force_cfg;
    if ((cfg == CFG_MC3 || cfg == CFG_MC4) && dtype == DT_F32) cfg = CFG_BIG;  // 16-bit only
  } else if (M <= 32) {
    cfg = CFG_WIDE32;
  } else if (M <= 64) {
    cfg = CFG_WIDE64;
  } else if (N <= 32) {
    cfg = CFG_TALL32;
  } else if (N <= 64) {
    cfg = CFG_TALL64;
  } else {
    // the 256x256 tile needs enough tiles to occupy the 256 compute units; a grid between half
    // and full is filled by splitting the contraction in two
    const int64_t big_tiles = ((M + 255) / 256) * ((N + 255) / 256);
    const bool pipe_ok = dtype != DT_F32;
    if (big_tiles >= 160 || (big_tiles >= 80 && K0 + K1 >= 2048))
      cfg = pipe_ok ? CFG_MC4 : CFG_BIG;
    else
      cfg = CFG_MID;
  }
  p.cfg = cfg;
  p.bk = (dtype == DT_F32) ? 32 : kTileBK16[cfg];
  p.bm = kTileBM[cfg];
  p.bn = kTileBN[cfg];
  p.nbm = (int)((M + p.bm - 1) / p.bm);
  p.nbn = (int)((N + p.bn - 1) / p.bn);
  const int64_t tiles = (int64_t)p.nbm * p.nbn;
  const int ktiles = (int)((K0 + p.bk - 1) / p.bk + (K1 + p.bk - 1) / p.bk);
  int splits = 1;
  if (force_splits > 0) {
    splits = force_splits;
  } else if (cfg == CFG_MC3 || cfg == CFG_MC4 || cfg == CFG_BIG) {
    if (tiles < 160 && (int64_t)ktiles * p.bk >= 1024) splits = pick_splits(tiles, (int64_t)ktiles * p.bk, 1);
  } else if (tiles < 256 && ktiles >= 8) {
    // fill the chip (aim at ~512 workgroups) but keep >= 4 K tiles per slice
    int64_t want = (512 + tiles - 1) / tiles;
    int64_t cap = ktiles / 4;
    splits = (int)(want < cap ? want : cap);
    if (splits > 64) splits = 64;
    if (splits < 1) splits = 1;
  }
  if (splits > ktiles) splits = ktiles > 0 ? ktiles : 1;
  p.tiles_per_split = (ktiles + splits - 1) / splits;
  if (p.tiles_per_split < 1) p.tiles_per_split = 1;
  p.splits = (ktiles + p.tiles_per_split - 1) / p.tiles_per_split;  // no empty slice
  if (p.splits < 1) p.splits = 1;
  p.partial_bytes = p.splits > 1 ? (size_t)p.splits * (size_t)M * (size_t)N * sizeof(float) : 0;
  // Tile quantisation: with one 256x256 tile per compute unit and round, a grid of e.g. 32 x 43 tiles
  // ends on a round that is 3/8 full.  If whole tile columns can be cut off such that the rest is an
  // exact number of rounds and the cut-off part is small enough to be split along K, run that part
  // as a launch of its own (half a round with the contraction in two, plus its reduce).
  if (force_cfg < 0 && force_splits <= 0 && (p.cfg == CFG_MC4 || (b_int4 && p.cfg == CFG_MC3)) && p.splits == 1 &&
      tiles > 256 && (int64_t)ktiles * p.bk >= 2048) {
    for (int t = p.nbn - 1; t >= 1 && t >= p.nbn - 16; --t) {
      const int64_t main_tiles = (int64_t)p.nbm * t, tail_tiles = (int64_t)p.nbm * (p.nbn - t);
      if (tail_tiles > 128) break;
      if (main_tiles % 256 != 0 || tail_tiles < 32) continue;
      p.tail_n0 = (int64_t)t * p.bn;
      p.nbn = t;
      p.partial_bytes = gemm_tail_plan(p, dtype, M, N, K0, K1).partial_bytes;
      break;
    }
  }
  return p;
}

GemmPlan gemm_tail_plan(const GemmPlan& main, int dtype, int64_t M, int64_t N, int64_t K0, int64_t K1) {
  // same kernel as the main launch with the contraction split (pick_splits)
  const int64_t nt = N - main.tail_n0;
  const int64_t tiles = (int64_t)main.nbm * ((nt + main.bn - 1) / main.bn);
  const int best = pick_splits(tiles, K0 + K1, 2);
  return gemm_plan(dtype, M, nt, K0, K1, main.cfg, best);
}

GemmPlan gemm_plan_int4(int dtype, int64_t M, int64_t N, int64_t K0, int64_t K1) {
  return gemm_plan(dtype, M, N, K0, K1, -1, 0, true);
}

GemmPlan gemm_plan_fused(int dtype, int64_t M, int64_t N, int64_t K0, int64_t R) {
  // the shape rules of gemm_plan with the generic engine's 256x256 tile where the matrix-core kernel would run;
  // the workgroup that owns an output tile needs the whole contraction of its rows of T: no split
  int cfg = gemm_plan(dtype, M, N, K0, R).cfg;
  if (cfg == CFG_MC3 || cfg == CFG_MC4) cfg = CFG_BIG;
  return gemm_plan(dtype, M, N, K0, R, cfg, 1);
}

hipError_t gemm_run(const GemmDesc& d, const GemmPlan& plan, float* scratch, hipStream_t stream) {
  if (d.M <= 0 || d.N <= 0) return hipErrorInvalidValue;
  if (plan.tail_n0 > 0) {
    // columns [0, tail_n0) with this plan, columns [tail_n0, N) as their own problem
    if (plan.tail_n0 >= d.N) return hipErrorInvalidValue;
    if (d.drop_thr != 0) return hipErrorInvalidValue;  // the mask is indexed by the full product's columns (K = r: never cut)
    const size_t esz = d.dtype == DT_F32 ? 4 : 2;
    GemmDesc dm = d, dt = d;
    GemmPlan pm = plan;
    pm.tail_n0 = 0;
    pm.partial_bytes = 0;
    dm.N = plan.tail_n0;
    dt.N = d.N - plan.tail_n0;
    for (int s = 0; s < d.nseg; ++s) {
      const int64_t off = d.b_kcontig ? plan.tail_n0 * d.ldb[s] : plan.tail_n0;
      if (s == 0 && d.Bscale != nullptr) {
        // int4: two weights per byte; the scales of columns (B stored [K,N]) or of row groups
        // (B stored [N,K]; tail_n0 is a multiple of 64) move along
        dt.B[0] = static_cast<const char*>(d.B[0]) + (size_t)off / 2;
        const int64_t soff = d.b_kcontig ? (plan.tail_n0 / 64) * d.ldbs : plan.tail_n0;
        dt.Bscale = static_cast<const char*>(d.Bscale) + (size_t)soff * 2;
      } else {
        dt.B[s] = static_cast<const char*>(d.B[s]) + (size_t)off * esz;
      }
    }
    dt.C = static_cast<char*>(d.C) + (size_t)plan.tail_n0 * esz;
    if (d.D) dt.D = static_cast<const char*>(d.D) + (size_t)plan.tail_n0 * esz;
    if (d.bias) dt.bias = static_cast<const char*>(d.bias) + (size_t)plan.tail_n0 * esz;
    hipError_t e = gemm_run(dm, pm, nullptr, stream);
    if (e != hipSuccess) return e;
    const GemmPlan pt = gemm_tail_plan(plan, d.dtype, d.M, d.N, d.K[0], d.nseg > 1 ? d.K[1] : 0);
    if (pt.tail_n0 > 0 || pt.partial_bytes > plan.partial_bytes) return hipErrorInvalidValue;
    return gemm_run(dt, pt, scratch, stream);
  }
  if (plan.splits > 1 && scratch == nullptr) return hipErrorInvalidValue;
  if (d.fuse_t) {
    const bool ok = d.LA != nullptr && d.nseg == 2 && d.K[1] >= 1 && d.K[1] <= kFuseMaxR && d.K[0] >= 1 && !d.a_strided &&
                    !d.b_kcontig && plan.splits == 1 && d.D == nullptr && d.Bscale == nullptr && d.drop_thr == 0 &&
                    plan.cfg != CFG_MC3 && plan.cfg != CFG_MC4;
    if (!ok) return hipErrorInvalidValue;
  }
  int cfg = plan.cfg;
  if (d.Bscale != nullptr && cfg != CFG_BIG && cfg != CFG_MID && cfg != CFG_MC3) return hipErrorInvalidValue;  // see gemm_plan_int4
  if (d.Bscale != nullptr && d.a_strided) return hipErrorInvalidValue;
  if (cfg == CFG_MC3 || cfg == CFG_MC4) {
    // the matrix-core kernel addresses each operand with 32-bit byte offsets into a buffer descriptor whose
    // extent is the operand's bytes plus 3 KB (gemm_mc.hpp, kBias): the 16-bit elements of an operand, rows x ld,
    // must stay below 2^31 - 2048 so that neither wraps; it also clamps a strided operand's last columns to
    // [dim-8, dim) and wants every K slice to hold at least one K tile
    bool ok = d.dtype != DT_F32 && plan.bk == (cfg == CFG_MC4 ? 64 : 32);
    constexpr int64_t kMaxElems = (1LL << 31) - 2048;
    for (int s = 0; s < d.nseg; ++s) {
      const int64_t a_rows = d.a_strided ? d.K[s] : d.M, b_rows = d.b_kcontig ? d.N : d.K[s];
      if (a_rows * d.lda[s] >= kMaxElems || b_rows * d.ldb[s] >= kMaxElems) ok = false;
    }
    if ((d.a_strided && d.M < 8) || (!d.b_kcontig && d.N < 8)) ok = false;
    if (!ok) cfg = CFG_BIG;
  }
  GemmArgs a{};
  for (int s = 0; s < 2; ++s) {
    const bool on = s < d.nseg;
    a.A[s] = on ? d.A[s] : nullptr;
    a.B[s] = on ? d.B[s] : nullptr;
    a.lda[s] = on ? d.lda[s] : 0;
    a.ldb[s] = on ? d.ldb[s] : 0;
    a.K[s] = on ? (int)d.K[s] : 0;
  }
  a.C = d.C;
  a.ldc = d.ldc;
  a.D = plan.splits > 1 ? nullptr : d.D;
  a.ldd = d.ldd;
  a.partial = plan.splits > 1 ? scratch : nullptr;
  a.M = (int)d.M;
  a.N = (int)d.N;
  a.tiles_per_split = plan.splits > 1 ? plan.tiles_per_split : (1 << 30);
  a.nbm = plan.nbm;
  a.nbn = plan.nbn;
  a.splits = plan.splits;
  a.Bscale = d.Bscale;
  a.ldbs = d.ldbs;
  a.alpha = d.alpha;
  a.bias = plan.splits > 1 ? nullptr : d.bias;
  a.drop_thr = d.drop_thr;
  a.drop_key = d.drop_key;
  a.drop_cpr = d.drop_cpr;
  a.LA = d.fuse_t ? d.LA : nullptr;
  a.ldla = d.ldla;
  a.R = d.fuse_t ? (int)d.K[1] : 0;
  a.t_alpha = d.t_alpha;
  dim3 grid((unsigned)(plan.nbm * plan.nbn), (unsigned)plan.splits, 1);
  const int al = d.a_strided ? 1 : 0, bl = d.b_kcontig ? 1 : 0;
  hipError_t e;
  switch (d.dtype) {
    case DT_BF16: e = gemm_launch_bf16(cfg, al, bl, a, grid, stream); break;
    case DT_F16: e = gemm_launch_f16(cfg, al, bl, a, grid, stream); break;
    case DT_F32: e = gemm_launch_f32(cfg, al, bl, a, grid, stream); break;
    default: return hipErrorInvalidValue;
  }
  if (e != hipSuccess) return e;
  if (plan.splits > 1)
    e = splitk_reduce_launch(d.dtype, scratch, plan.splits, (int)d.M, (int)d.N, d.C, d.ldc, d.D, d.ldd, d.alpha,
                             d.bias, DropMask{d.drop_thr, d.drop_key, d.drop_cpr}, stream);
  return e;
}

hipError_t splitk_reduce_launch(int dtype, const float* partial, int splits, int M, int N, void* C,
                                int64_t ldc, const void* D, int64_t ldd, float alpha, const void* bias,
                                DropMask drop, hipStream_t s) {
  const int64_t quads = (int64_t)M * N / 4;
  int blocks = (int)((quads + 255) / 256);
  if (blocks > 4096) blocks = 4096;
  if (blocks < 1) blocks = 1;
  switch (dtype) {
    case DT_BF16:
      launch_timed(splitk_reduce_kernel<__bf16>, dim3(blocks), dim3(256), 0, s, partial, splits, M, N,
                         static_cast<__bf16*>(C), ldc, static_cast<const __bf16*>(D), ldd, alpha,
                         static_cast<const __bf16*>(bias), drop.thr, drop.key, drop.cpr);
      break;
    case DT_F16:
      launch_timed(splitk_reduce_kernel<_Float16>, dim3(blocks), dim3(256), 0, s, partial, splits, M, N,
                         static_cast<_Float16*>(C), ldc, static_cast<const _Float16*>(D), ldd, alpha,
                         static_cast<const _Float16*>(bias), drop.thr, drop.key, drop.cpr);
      break;
    case DT_F32:
      launch_timed(splitk_reduce_kernel<float>, dim3(blocks), dim3(256), 0, s, partial, splits, M, N,
                         static_cast<float*>(C), ldc, static_cast<const float*>(D), ldd, alpha,
                         static_cast<const float*>(bias), drop.thr, drop.key, drop.cpr);
      break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// ---- streaming kernel for the rank-r products -----------------------------------------------------

SkinnyPlan skinny_plan(int dtype, int nprob, const SkinnyDesc* d) {
  SkinnyPlan p;
  const int bk = dtype == DT_F32 ? 32 : 64;
  int64_t blocks = 0, min_ktiles = 1 << 30, outs = 0, maxn = 0;
  for (int w = 0; w < nprob; ++w)
    if (d[w].N > maxn) maxn = d[w].N;
  p.rt = maxn <= 32 ? 1 : (maxn <= 64 ? 2 : 4);
  // see skinny.hpp; a masked problem (LoRA dropout) is bound by its waves' mask arithmetic, which 32-row workgroups
  // spread over twice as many waves
  const bool masked = d[0].drop_thr != 0 || (nprob == 2 && d[1].drop_thr != 0);
  p.mr = (nprob == 2 && d[0].a_strided && d[1].a_strided && p.rt <= 2 && !masked) ? 2 : 1;
  const int mb = 32 * p.mr;
  for (int w = 0; w < nprob; ++w) {
    blocks += (d[w].M + mb - 1) / mb;
    const int64_t kt = (d[w].K + bk - 1) / bk;
    if (kt < min_ktiles) min_ktiles = kt;
    outs += d[w].M * d[w].N;
  }
  // split K over workgroups only when there are fewer workgroups than compute units, and keep >= 8 K tiles
  // per wave and slice.  (64-row workgroups: 128-160 of them without a split beat twice as many plus the
  // reduce pass, measured on the paired dA / dB launches.)
  int64_t splits = 1;
  if (blocks < (p.mr == 2 ? 128 : 224)) {
    splits = (256 + blocks - 1) / blocks;
    int64_t cap = min_ktiles / 32;
    if (cap < 1) cap = 1;
    if (splits > cap) splits = cap;
    if (splits > 16) splits = 16;
  }
  p.splits = (int)splits;
  p.partial_bytes = splits > 1 ? (size_t)splits * (size_t)outs * sizeof(float) : 0;
  return p;
}

hipError_t skinny_run(int dtype, int nprob, const SkinnyDesc* d, const SkinnyPlan& plan, float* scratch,
                      hipStream_t stream) {
  if (nprob < 1 || nprob > 2) return hipErrorInvalidValue;
  if (plan.splits > 1 && scratch == nullptr) return hipErrorInvalidValue;
  const int bk = dtype == DT_F32 ? 32 : 64;
  SkinnyArgs a{};
  a.nprob = nprob;
  a.mr = plan.mr;
  if (plan.mr != 1 && !(plan.mr == 2 && nprob == 2 && d[0].a_strided && d[1].a_strided && plan.rt <= 2)) return hipErrorInvalidValue;
  float* part = scratch;
  for (int w = 0; w < nprob; ++w) {
    SkinnyProblem& P = a.p[w];
    if (d[w].N > 32 * plan.rt || d[w].M < 1 || d[w].K < 1) return hipErrorInvalidValue;
    P.A = d[w].A; P.B = d[w].B; P.C = d[w].C;
    P.lda = d[w].lda; P.ldb = d[w].ldb; P.ldc = d[w].ldc;
    P.M = (int)d[w].M; P.N = (int)d[w].N; P.K = (int)d[w].K;
    P.a_strided = d[w].a_strided; P.b_kcontig = d[w].b_kcontig; P.trans_out = d[w].trans_out;
    P.alpha = d[w].alpha;
    P.drop_thr = d[w].drop_thr; P.drop_key = d[w].drop_key; P.drop_cpr = d[w].drop_cpr;
    const int mb = 32 * plan.mr;
    P.row_blocks = (int)((d[w].M + mb - 1) / mb);
    {
      const int64_t esz = dtype == DT_F32 ? 4 : 2;
      const int64_t a_rows = d[w].a_strided ? d[w].K : d[w].M, a_cols = d[w].a_strided ? d[w].M : d[w].K;
      const int64_t b_rows = d[w].b_kcontig ? d[w].N : d[w].K, b_cols = d[w].b_kcontig ? d[w].K : d[w].N;
      const int64_t ab = ((a_rows - 1) * d[w].lda + a_cols) * esz, bb = ((b_rows - 1) * d[w].ldb + b_cols) * esz;
      if (ab >= (1LL << 31) || bb >= (1LL << 31)) return hipErrorInvalidValue;  // callers check skinny_fits()
      P.a_bytes = (int)ab;
      P.b_bytes = (int)bb;
    }
    const int64_t kt = (d[w].K + bk - 1) / bk;
    P.tiles_per_split = (int)((kt + plan.splits - 1) / plan.splits);
    P.partial = nullptr;
    if (plan.splits > 1) {
      P.partial = part;
      part += (size_t)plan.splits * (size_t)d[w].M * (size_t)d[w].N;
    }
  }
  // one slot list per XCD: ceil(R0/8) + ceil(R1/8) workgroups on each (see skinny_kernel)
  int64_t per_xcd = 0;
  for (int w = 0; w < nprob; ++w) per_xcd += (a.p[w].row_blocks + 7) / 8;
  dim3 grid((unsigned)(8 * per_xcd), (unsigned)plan.splits, 1);
  switch (dtype) {
    case DT_BF16: return skinny_launch_bf16(plan.rt, a, grid, plan.splits, stream);
    case DT_F16: return skinny_launch_f16(plan.rt, a, grid, plan.splits, stream);
    case DT_F32: return skinny_launch_f32(plan.rt, a, grid, plan.splits, stream);
    default: return hipErrorInvalidValue;
  }
}

// ---- M = W + A B ------------------------------------------------------------------------------------

hipError_t merge_run(int dtype, const MergeDesc& d, hipStream_t stream) {
  if (!merge_ok(dtype, d.R) || d.I < 1 || d.O < 1 || d.R < 1) return hipErrorInvalidValue;
  MergeArgs a{};
  a.W = d.W; a.A = d.A; a.B = d.B; a.M = d.M;
  a.ldw = d.ldw; a.lda = d.lda; a.ldb = d.ldb; a.ldm = d.ldm;
  a.I = (int)d.I; a.O = (int)d.O; a.R = (int)d.R;
  a.blocks_per_wg = 1;
  a.alpha = d.alpha;
  a.b_trans = d.b_trans;
  a.wcol = d.wcol;
  a.sq_partial = d.sq_partial;
  a.drop_thr = d.drop_thr; a.drop_key = d.drop_key; a.drop_cpr = d.drop_cpr;
  return dtype == DT_BF16 ? merge_launch_bf16(a, stream) : merge_launch_f16(a, stream);
}

}  // namespace rl
