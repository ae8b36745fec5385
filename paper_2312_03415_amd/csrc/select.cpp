// Selector: Table 1 FLOP counts, a per-kernel time model for MI355X, and the choice of the
// (forward, backward) pair ("choosing best forward and backward computation graph based on FLOPs
// and time estimations", abstract of arxiv 2312.03415).  Pure host code, no HIP call.
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
      case 1: return 2 * n * (i * o + r * i + o * r);
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

// Time of one GEMM launch: the slower of its arithmetic at the tile shape's measured rate and its
// memory traffic at the measured streaming rate, plus a fixed launch cost; a split contraction
// adds the write and re-read of the fp32 partials and the reduce launch.
static double step_time_us(const Step& s) {
  const ModelConstants& mc = model_constants();
  if (s.nsk > 0) {
    // streaming kernel: one read of each operand, one write of the (small) output
    const double e = (double)dtype_size(s.d.dtype);
    double bytes = 0, outs = 0;
    for (int w = 0; w < s.nsk; ++w) {
      const SkinnyDesc& k = s.sk[w];
      bytes += e * ((double)k.M * k.K + (double)k.K * k.N + (double)k.M * k.N);
      outs += (double)k.M * k.N;
    }
    double us = bytes / (mc.stream_tbps * 1e12) * 1e6 + mc.launch_us;
    if (s.skplan.splits > 1) us += 2.0 * 4.0 * outs * s.skplan.splits / (mc.stream_tbps * 1e12) * 1e6 + mc.launch_us;
    return us;
  }
  const GemmDesc& d = s.d;
  const GemmPlan& p = s.plan;
  const double e = (double)dtype_size(d.dtype);
  const double K = (double)(d.K[0] + (d.nseg > 1 ? d.K[1] : 0));
  // the engine multiplies whole tiles: count the padded problem
  const double Mp = (double)p.nbm * p.bm, Np = (double)p.nbn * p.bn;
  const double flops = 2.0 * Mp * Np * K;
  const ModelConstants& c = mc;
  const int fam = d.dtype == DT_F32 ? 1 : 0;
  double rate = c.tile_tflops[fam][p.cfg] * 1e12;
  // few workgroups leave compute units idle
  const double wgs = (double)p.nbm * p.nbn * p.splits;
  const double fill = wgs >= 256.0 ? 1.0 : wgs / 256.0;
  rate *= fill;
  // operand traffic: each A row-band is read once per pass over the column tiles that do not share
  // an L2, modelled as one read of each operand plus the output (and addend)
  double bytes = e * ((double)d.M * K + K * (double)d.N + (double)d.M * d.N * (d.D ? 2.0 : 1.0));
  double t = flops / rate;
  double tm = bytes / (c.stream_tbps * 1e12);
  double us = (t > tm ? t : tm) * 1e6 + c.launch_us;
  if (p.splits > 1) {
    const double pb = (double)p.partial_bytes;
    us += 2.0 * pb / (c.stream_tbps * 1e12) * 1e6 + c.launch_us;
  }
  return us;
}

double model_time_us(int is_bwd, int variant, const LayerDims& L) {
  Schedule sch;
  bool ok;
  if (!is_bwd) {
    FwdOperands op;
    ok = build_forward(variant, L, op, nullptr, &sch);
  } else {
    BwdOperands op;
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
  if (variant < 0 || variant > (is_bwd ? 5 : 2)) return -1.0;
  LayerDims L{n, i, o, r, dt};
  return model_time_us(is_bwd, variant, L);
}

extern "C" int runlora_select_by(int criterion, int64_t n, int64_t i, int64_t o, int64_t r, int dtype,
                                 int* fwd, int* bwd) {
  if (!fwd || !bwd) return RL_ERR_NULL;
  if (n < 1 || i < 1 || o < 1 || r < 1) return RL_ERR_SHAPE;
  int dt = to_internal_dtype(dtype);
  if (dt < 0) return RL_ERR_DTYPE;
  if (criterion != 0 && criterion != 1) return RL_ERR_VARIANT;
  const bool int4 = (dtype == RL_INT4_G64);
  // an int4 W has no dense buffer to merge AB into: forward1 and backward1..3 only
  const int fmax = int4 ? 1 : 2, bmax = int4 ? 3 : 5;
  LayerDims L{n, i, o, r, dt};
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
  *fwd = bf;
  *bwd = bb;
  return RL_OK;
}

extern "C" int runlora_select(int64_t n, int64_t i, int64_t o, int64_t r, int dtype, int* fwd, int* bwd) {
  const char* env = std::getenv("RUNLORA_CRITERION");
  int criterion = (env && std::strcmp(env, "flops") == 0) ? 0 : 1;
  return runlora_select_by(criterion, n, i, o, r, dtype, fwd, bwd);
}
