// Selector: Table 1 FLOP counts, a per-kernel time model for MI355X, and the choice of the
// (forward, backward) pair of computation graphs by operation count or by estimated time (the
// selection step named in the abstract of arxiv 2312.03415).  Pure host code, no HIP call.
#include <cstdlib>
#include <cstring>

#include "../../include/runlora.h"
#include "model_constants.hpp"
#include "schedule.hpp"

namespace rl {

// Table 1.  The default chain has forward1's products; its backward is backward1 without the
// recomputation of XA.  backward6 follows the recount of item 6 (+2ior; the table prints +4ior).
int64_t table1_flops(int is_bwd, int v, int64_t n, int64_t i, int64_t o, int64_t r) {
  if (!is_bwd) {
    switch (v) {
      case 0:
      case 1:
      case 3: return 2 * n * (i * o + r * i + o * r);  // (3: forward1's graph; its kernel's repeated X A is not counted)
      case 2: return 2 * (i * o * r + n * o * i);
      default: return -1;
    }
  }
  switch (v) {
    case 0: return 2 * n * (2 * o * r + 2 * i * r + o * i);
    case 1: return 2 * n * (2 * o * r + 3 * i * r + o * i);
    case 2: return 2 * n * (o * r + 2 * i * r + 2 * i * o) + 2 * i * o * r;
    case 3: return 2 * n * (2 * i * o + o * r + i * r) + 4 * i * r * o;
    case 4: return 2 * (2 * n * i * o + 3 * i * o * r);
    case 5: return 2 * n * (2 * o * r + 2 * i * r + o * i) + 2 * i * o * r;
    case 6: return 2 * n * (2 * o * r + 2 * i * r + 2 * o * i) + 2 * i * o * r;
    case 7:
    case 8: return 2 * n * (o * r + i * r + 2 * o * i) + 4 * i * o * r;
    default: return -1;
  }
}

// Tile GEMM: workgroups run in rounds of (compute units x resident workgroups); a round costs
// (K tiles x measured time per K tile) + a fixed prologue/epilogue; a split contraction adds the
// write and re-read of the fp32 partials and the reduce launch; a plan with cut-off tail columns is
// two launches.
static double gemm_time_us(const GemmDesc& d, const GemmPlan& p) {
  const ModelConstants& mc = model_constants();
  const double e = (double)dtype_size(d.dtype);
  if (p.tail_n0 > 0) {
    GemmDesc dm = d, dt = d;
    GemmPlan pm = p;
    pm.tail_n0 = 0;
    dm.N = p.tail_n0;
    dt.N = d.N - p.tail_n0;
    return gemm_time_us(dm, pm) + gemm_time_us(dt, gemm_tail_plan(p, d.dtype, d.M, d.N, d.K[0], d.nseg > 1 ? d.K[1] : 0));
  }
  const TileModel& tm = mc.tile[d.dtype == DT_F32 ? 1 : 0][p.cfg];
  const int lay = d.a_strided ? 2 : (d.b_kcontig ? 1 : 0);
  const double wgs = (double)p.nbm * p.nbn * p.splits;
  const double slots = 256.0 * tm.wg_per_cu;
  double rounds = wgs / slots;
  // a grid that does not fill the resident slots leaves each workgroup more of its compute unit
  double share = 1.0;
  if (rounds < 1.0) {
    share = rounds > 1.0 / tm.wg_per_cu ? rounds : 1.0 / tm.wg_per_cu;
    rounds = 1.0;
  } else {
    rounds = (double)(int64_t)(rounds + 0.999);
  }
  const int64_t kt0 = (d.K[0] + p.bk - 1) / p.bk, kt1 = d.nseg > 1 ? (d.K[1] + p.bk - 1) / p.bk : 0;
  double ktiles = (double)(kt0 + kt1);
  if (p.splits > 1) ktiles = (double)p.tiles_per_split;
  // (partial and second-segment K tiles run at the speed of any other)
  const bool has_d = d.has_addend || d.D != nullptr;
  const bool addend = has_d && p.splits == 1;
  // int4 B on the matrix-core kernel: the dequantisation behind the MFMAs costs ~20 % per K tile
  // (measured on the 5120 x 13824 layer)
  double q = (d.b_int4 && p.cfg == CFG_MC3) ? 1.2 : 1.0;
  if (d.fuse_t) {
    // one-pass forward: next to its TM x TN blocks of 32 x 32 per K step a wave multiplies ceil(TM / WN) blocks of
    // T = X A (+1/8 of the MFMA work on the 256x256 tile, +1/4 on 128x128, +1/2 on 128x64 and 64x128) and stages a
    // slice of A per K tile.  Measured against the K-concatenated launch on the same tile with the contraction
    // whole: 1.25-1.35 (256x256), 1.35-1.63 (128x128), 1.64 (128x64, 64x128); the 32-wide tiles (T as wide as the
    // output) are taken at 2.
    static const double ratio[6] = {1.32, 1.62, 2.0, 1.66, 2.0, 1.66};
    if (p.cfg >= 0 && p.cfg < 6) q *= ratio[p.cfg];
  }
  double us = rounds * (ktiles * tm.tk_us[lay] * share * q + (addend ? tm.tfix_d_us : tm.tfix_us));
  if (p.splits > 1)
    us += (double)d.M * d.N * (4.0 * (p.splits + 1) + (has_d ? e : 0.0) + e) / (mc.reduce_tbps * 1e12) * 1e6 + mc.reduce_fix_us + mc.launch_us;
  return us;
}

// Time of one launch.
//  Streaming kernel: bytes / measured streaming rate + a fixed cost (+ the partials' round trip
//  and the reduce launch when the contraction is also split over workgroups).
//  Tile GEMM: workgroups run in rounds of (compute units x resident workgroups); a round costs
//  (K tiles x measured time per K tile) + a fixed prologue/epilogue; a split contraction adds the
//  write and re-read of the fp32 partials and the reduce launch.
static double step_time_us(const Step& s) {
  const ModelConstants& mc = model_constants();
  const double e = (double)dtype_size(s.d.dtype);
  if (s.is_merge)
    return e * 2.0 * (double)s.mg.I * (double)s.mg.O / (mc.merge_tbps * 1e12) * 1e6 + mc.merge_fix_us;
  if (s.nsk > 0) {
    double us = mc.stream_fix_us;  // the measured intercepts already hold the cost of the launch itself
    double outs = 0;
    for (int w = 0; w < s.nsk; ++w) {
      const SkinnyDesc& k = s.sk[w];
      const double bytes = e * ((double)k.M * k.K + (double)k.K * k.N + (double)k.M * k.N);
      us += bytes / (mc.stream_tbps[k.a_strided ? 1 : 0] * 1e12) * 1e6;
      outs += (double)k.M * k.N;
    }
    if (s.skplan.splits > 1) us += 4.0 * outs * (s.skplan.splits + 1) / (mc.reduce_tbps * 1e12) * 1e6 + mc.stream_fix_us + mc.launch_us;
    return us;
  }
  return gemm_time_us(s.d, s.plan);
}

// have_M: the backward finds W + AB kept by forward2 and does not form it again; have_T: it finds T = XA kept by
// forward1 (keep_T on the forward side changes nothing: the same launch writes T elsewhere)
double model_time_us(int is_bwd, int variant, const LayerDims& L, bool have_M = false, bool have_T = false) {
  Schedule sch;
  bool ok;
  if (!is_bwd) {
    FwdOperands op;
    ok = build_forward(variant, L, op, nullptr, &sch);
  } else {
    BwdOperands op;
    op.have_M = have_M;
    op.have_T = have_T;
    ok = build_backward(variant, L, op, nullptr, &sch);
  }
  if (!ok) return -1.0;
  double us = 0;
  for (const Step& s : sch.steps) us += step_time_us(s);
  return us;
}

}  // namespace rl

using namespace rl;

static int to_internal_dtype(int dtype) {
  switch (dtype) {
    case RL_F32: return DT_F32;
    case RL_F16: return DT_F16;
    case RL_BF16: return DT_BF16;
    case RL_INT4_G64: return DT_BF16;
    default: return -1;
  }
}

extern "C" int64_t runlora_flops(int is_bwd, int variant, int64_t n, int64_t i, int64_t o, int64_t r) {
  return table1_flops(is_bwd, variant, n, i, o, r);
}

extern "C" double runlora_model_time_us(int is_bwd, int variant, int64_t n, int64_t i, int64_t o, int64_t r,
                                        int dtype) {
  int dt = to_internal_dtype(dtype);
  if (dt < 0 || n < 1 || i < 1 || o < 1 || r < 1) return -1.0;
  if (variant < 0 || variant > (is_bwd ? 8 : 3)) return -1.0;
  LayerDims L{n, i, o, r, dt};
  L.w_int4 = dtype == RL_INT4_G64;  // priced with the int4 route's plans; merged graphs then return -1
  return model_time_us(is_bwd, variant, L);
}

extern "C" int runlora_select_by(int criterion, int64_t n, int64_t i, int64_t o, int64_t r, int dtype,
                                 int* fwd, int* bwd) {
  if (!fwd || !bwd) return RL_ERR_NULL;
  if (n < 1 || i < 1 || o < 1 || r < 1) return RL_ERR_SHAPE;
  int dt = to_internal_dtype(dtype);
  if (dt < 0) return RL_ERR_DTYPE;
  if (criterion < 0 || criterion > 3) return RL_ERR_VARIANT;
  const bool int4 = (dtype == RL_INT4_G64);
  // an int4 W has no dense buffer to merge AB into: forward1 and backward1..3 only
  // (forward 3 is forward1's graph in one kernel: a candidate under the time criteria only, where it applies)
  const int fmax = int4 ? 1 : (criterion == 0 ? 2 : 3), bmax = int4 ? 3 : 5;
  LayerDims L{n, i, o, r, dt};
  L.w_int4 = int4;
  int bf = 1, bb = 1;
  double cf = 0, cb = 0;
  for (int v = 1; v <= fmax; ++v) {
    double c = criterion == 0 ? (double)table1_flops(0, v, n, i, o, r) : model_time_us(0, v, L);
    if (v == 1 || c < cf) { cf = c; bf = v; }  // strict '<': ties go to the lower id
  }
  for (int v = 1; v <= bmax; ++v) {
    double c = criterion == 0 ? (double)table1_flops(1, v, n, i, o, r) : model_time_us(1, v, L);
    if (v == 1 || c < cb) { cb = c; bb = v; }
  }
  // The default chain (keeps XA, no fusion) is a legal pair too; under the time criterion it is
  // returned when the model says it beats the best RunLoRA pair (large r at few tokens, where the
  // recomputation of XA in Algorithms 1 and 5 is not free).  Table 1 does not list it, so the FLOP
  // criterion never returns it.
  if (criterion >= 1) {
    // With W + AB kept by forward2 the search is no longer separable: forward2 paired with
    // backward4 / 5 saves the second merge pass, which may beat the separately best pair.
    if (criterion == 2 && !int4) {
      const double f2 = model_time_us(0, 2, L);
      for (int v = 4; v <= 5; ++v) {
        const double c = f2 + model_time_us(1, v, L, true);
        if (c < cf + cb) { cf = f2; cb = c - f2; bf = 2; bb = v; }
      }
    }
    // Criterion 3, for callers that let forward1 keep T = XA (n r elements): forward1 paired with the backwards that
    // would form X A again (Algorithms 1 and 5) is priced without that pass; forward2 computes no T, so its pairs stay
    if (criterion == 3) {
      const double f1 = model_time_us(0, 1, L);
      for (int v = 1; v <= bmax; v += 4) {  // Algorithms 1 and 5
        const double c = f1 + model_time_us(1, v, L, false, true);
        if (c < cf + cb) { cf = f1; cb = c - f1; bf = 1; bb = v; }
      }
    }
    const double c0 = model_time_us(0, 0, L) + model_time_us(1, 0, L);
    if (c0 < cf + cb) { bf = 0; bb = 0; }
  }
  *fwd = bf;
  *bwd = bb;
  return RL_OK;
}

// value of a debugging override (a small non-negative integer in the environment), or -1
static int env_variant(const char* name, int max_id) {
  const char* v = std::getenv(name);
  if (!v || !*v) return -1;
  char* end = nullptr;
  const long id = std::strtol(v, &end, 10);
  return (end && *end == '\0' && id >= 0 && id <= max_id) ? (int)id : -2;  // -2: set but not a variant id
}

extern "C" int runlora_select(int64_t n, int64_t i, int64_t o, int64_t r, int dtype, int* fwd, int* bwd) {
  const char* env = std::getenv("RUNLORA_CRITERION");
  int criterion = (env && std::strcmp(env, "flops") == 0) ? 0 : 1;
  int rc = runlora_select_by(criterion, n, i, o, r, dtype, fwd, bwd);
  if (rc != RL_OK) return rc;
  // RUNLORA_FORCE_FWD / RUNLORA_FORCE_BWD pin one side of the pair (debugging: run a whole model in one graph)
  const int ff = env_variant("RUNLORA_FORCE_FWD", RL_FWD3), fb = env_variant("RUNLORA_FORCE_BWD", RL_BWD8);
  if (ff == -2 || fb == -2) return RL_ERR_VARIANT;
  if (ff >= 0) *fwd = ff;
  if (fb >= 0) *bwd = fb;
  if (ff >= 0 || fb >= 0) {
    if (*bwd == RL_BWD_DEFAULT && *fwd != RL_FWD_DEFAULT) {
      if (fb >= 0 && ff >= 0) return RL_ERR_VARIANT;  // the default backward needs the default forward's XA
      if (fb >= 0) *fwd = RL_FWD_DEFAULT; else *bwd = RL_BWD1;
    }
    const bool merged = *fwd == RL_FWD2 || *bwd == RL_BWD4 || *bwd == RL_BWD5 || *bwd == RL_BWD7 || *bwd == RL_BWD8;
    if (dtype == RL_INT4_G64 && merged) return RL_ERR_UNSUPPORTED;
  }
  return RL_OK;
}
