// C ABI of the library (include/runlora.h): argument checks, variant schedules -> launches.
#include <cstdio>
#include <cstring>
#include <mutex>
#include <vector>

#include "../../include/runlora.h"
#include "schedule.hpp"
#include "dora.hpp"
#include "vera.hpp"

using namespace rl;

// Scratch of runlora_forward_static: a fixed array in this library's device image instead of a caller-provided
// workspace (each GPU the library runs on holds its own copy until the process ends).  In host code the name is a
// stand-in, not a device address: the address is looked up once per device (static_scratch below) and that
// pointer is what the host hands to the kernels.
constexpr size_t kStaticScratchBytes = (size_t)RL_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

thread_local char g_hip_error[256] = "";

int set_hip_error(hipError_t e, const char* what) {
  std::snprintf(g_hip_error, sizeof(g_hip_error), "%s: %s", what, hipGetErrorString(e));
  return RL_ERR_HIP;
}

int internal_dtype(int dtype) {
  switch (dtype) {
    case RL_F32: return DT_F32;
    case RL_F16: return DT_F16;
    case RL_BF16: return DT_BF16;
    default: return -1;
  }
}

// shape / dtype / alignment rules of one dense tensor
int check_tensor(const rl_tensor_t* t, int64_t rows, int64_t cols, int dtype) {
  if (!t || !t->data) return RL_ERR_NULL;
  if (t->dtype != dtype) return RL_ERR_DTYPE;
  if (t->rows != rows || t->cols != cols || t->ld < t->cols) return RL_ERR_SHAPE;
  const int64_t q = dtype == RL_F32 ? 4 : 8;
  if ((reinterpret_cast<uintptr_t>(t->data) & 15) != 0 || t->ld % q != 0) return RL_ERR_ALIGN;
  return RL_OK;
}

int check_dims(int64_t n, int64_t i, int64_t o, int64_t r, int dtype) {
  if (n < 1 || i < 1 || o < 1 || r < 1) return RL_ERR_SHAPE;
  if (n > (1LL << 30) || i > (1LL << 30) || o > (1LL << 30) || r > (1LL << 30)) return RL_ERR_SHAPE;
  const int64_t q = dtype == RL_F32 ? 4 : 8;
  if (i % q || o % q || r % q) return RL_ERR_ALIGN;
  return RL_OK;
}

struct Range {
  const char* lo;
  const char* hi;
};
Range range_of(const void* p, int64_t rows, int64_t ld, int64_t cols, size_t esz) {
  const char* lo = static_cast<const char*>(p);
  return {lo, lo + ((size_t)(rows - 1) * (size_t)ld + (size_t)cols) * esz};
}
bool overlap(Range a, Range b) { return a.lo < b.hi && b.lo < a.hi; }

Mat mat(const rl_tensor_t* t) {
  Mat m;
  m.ptr = t->data;
  m.ld = t->ld;
  return m;
}

// the frozen W: dense in the layer dtype, or int4 with group scales (16-bit activations only)
int check_weight(const rl_tensor_t* W, int64_t i, int64_t o, int dtype, bool* int4) {
  *int4 = false;
  if (!W || !W->data) return RL_ERR_NULL;
  if (W->dtype != RL_INT4_G64) return check_tensor(W, i, o, dtype);
  if (dtype == RL_F32) return RL_ERR_DTYPE;
  if (!W->scales) return RL_ERR_NULL;
  if (W->group != 64) return RL_ERR_UNSUPPORTED;
  if (W->rows != i || W->cols != o || W->ld < W->cols) return RL_ERR_SHAPE;
  if ((reinterpret_cast<uintptr_t>(W->data) & 15) != 0 || (reinterpret_cast<uintptr_t>(W->scales) & 15) != 0 ||
      W->ld % 8 != 0)
    return RL_ERR_ALIGN;
  *int4 = true;
  return RL_OK;
}

Range weight_range(const rl_tensor_t* W, int64_t i, int64_t o, size_t esz, bool int4) {
  if (!int4) return range_of(W->data, i, W->ld, o, esz);
  const char* lo = static_cast<const char*>(W->data);
  return {lo, lo + ((size_t)(i - 1) * (size_t)W->ld + (size_t)o + 1) / 2};
}

Mat weight_mat(const rl_tensor_t* W, int64_t o, bool int4) {
  Mat m = mat(W);
  if (int4) {
    m.scales = W->scales;
    m.lds = o;  // scales are dense [ceil(i/64), o]
  }
  return m;
}


// optional per-step event timing (runlora_profile_*), one recorder per host thread
struct Profiler {
  bool on = false;
  std::vector<hipEvent_t> start, stop;    // around the whole step
  std::vector<hipEvent_t> kstart, kstop;  // KernelEvents::kMax pairs per step, bound to its kernels (launch_timed, gemm.hpp)
  std::vector<char> kbound;               // how many of a step's pairs its launches consumed
  bool kernel_events = false;             // runlora_profile_kernel_times
  std::vector<rl_step_time_t> rec;
  size_t used = 0;
};
thread_local Profiler g_prof;

void describe_step(const Step& s, rl_step_time_t* r) {
  if (s.is_merge) {
    const double e = (double)dtype_size(s.d.dtype);
    r->what = s.what;
    r->us = 0.0;
    r->kernel_us = 0.0;
    r->main_us = 0.0;
    r->kernels = 0;
    r->flops = 2.0 * (double)s.mg.I * (double)s.mg.O * (double)s.mg.R;
    r->bytes = e * (2.0 * (double)s.mg.I * (double)s.mg.O + (double)s.mg.R * (double)(s.mg.I + s.mg.O));
    r->M = s.mg.I; r->N = s.mg.O; r->K = s.mg.R;
    r->tile_cfg = CFG_COUNT + 3;
    r->splits = 1;
    r->a_strided = 0; r->b_kcontig = 0;
    return;
  }
  if (s.nsk > 0) {
    const double e = (double)dtype_size(s.d.dtype);
    r->what = s.what;
    r->us = 0.0;
    r->kernel_us = 0.0;
    r->main_us = 0.0;
    r->kernels = 0;
    r->flops = 0.0;
    r->bytes = 0.0;
    for (int w = 0; w < s.nsk; ++w) {
      const SkinnyDesc& k = s.sk[w];
      r->flops += 2.0 * (double)k.M * (double)k.N * (double)k.K;
      r->bytes += e * ((double)k.M * k.K + (double)k.K * k.N + (double)k.M * k.N);
    }
    r->M = s.sk[0].M; r->N = s.sk[0].N; r->K = s.sk[0].K;
    r->tile_cfg = CFG_COUNT + (s.skplan.rt == 1 ? 0 : (s.skplan.rt == 2 ? 1 : 2));
    r->splits = s.skplan.splits;
    r->a_strided = s.sk[0].a_strided; r->b_kcontig = s.sk[0].b_kcontig;
    return;
  }
  const GemmDesc& d = s.d;
  const double K = (double)(d.K[0] + (d.nseg > 1 ? d.K[1] : 0));
  const double e = (double)dtype_size(d.dtype);
  r->what = s.what;
  r->us = 0.0;
  r->kernel_us = 0.0;
  r->main_us = 0.0;
  r->kernels = 0;
  r->flops = 2.0 * (double)d.M * (double)d.N * K;
  r->bytes = e * ((double)d.M * K + K * (double)d.N + (double)d.M * (double)d.N * (d.D ? 2.0 : 1.0));
  r->M = d.M; r->N = d.N; r->K = (int64_t)K;
  r->tile_cfg = s.plan.cfg; r->splits = s.plan.splits;
  r->a_strided = d.a_strided; r->b_kcontig = d.b_kcontig;
}

// set by the DoRA entry points around their inner layer call: the frozen weight is W diag(g_wcol)
thread_local const float* g_wcol = nullptr;
struct WCol {
  explicit WCol(const float* g) { g_wcol = g; }
  ~WCol() { g_wcol = nullptr; }
};
// While set, the layer calls check their arguments and build their schedule but enqueue nothing: an
// entry point built on top of them validates everything this way before its own first launch.
thread_local bool g_dry_run = false;
struct DryRun {
  DryRun() { g_dry_run = true; }
  ~DryRun() { g_dry_run = false; }
};

int run_schedule(const Schedule& sch, char* ws, hipStream_t stream) {
  if (g_dry_run) return RL_OK;
  float* partial = ws ? reinterpret_cast<float*>(ws + sch.partial_offset) : nullptr;
  for (const Step& s : sch.steps) {
    const bool timed = g_prof.on && g_prof.used < g_prof.start.size();
    if (timed) {
      hipError_t e = hipEventRecord(g_prof.start[g_prof.used], stream);
      if (e != hipSuccess) return set_hip_error(e, "profile event");
      if (g_prof.kernel_events) {
        KernelEvents ke;
        for (int k = 0; k < KernelEvents::kMax; ++k) {
          ke.start[k] = g_prof.kstart[g_prof.used * KernelEvents::kMax + k];
          ke.stop[k] = g_prof.kstop[g_prof.used * KernelEvents::kMax + k];
        }
        ke.avail = KernelEvents::kMax;
        g_kernel_events = ke;
      }
    }
    hipError_t e = s.is_merge ? merge_run(s.d.dtype, s.mg, stream)
                   : s.nsk > 0 ? skinny_run(s.d.dtype, s.nsk, s.sk, s.skplan, partial, stream)
                               : gemm_run(s.d, s.plan, partial, stream);
    const int kbound = (timed && g_prof.kernel_events) ? g_kernel_events.used : 0;  // pairs the step's launches consumed
    g_kernel_events = KernelEvents{};
    if (e != hipSuccess) return set_hip_error(e, s.what);
    if (timed) {
      g_prof.kbound[g_prof.used] = (char)kbound;
      e = hipEventRecord(g_prof.stop[g_prof.used], stream);
      if (e != hipSuccess) return set_hip_error(e, "profile event");
      describe_step(s, &g_prof.rec[g_prof.used]);
      ++g_prof.used;
    }
  }
  return RL_OK;
}

// key of the dropout mask (see drop_mix in gemm_engine.hpp; the same hash on the host)
uint32_t drop_key_of(uint32_t seed) {
  uint32_t x = seed ^ 0x9E3779B9u;
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// address of this device's copy of `scratch` (device = the calling thread's current device)
int static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return set_hip_error(e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) return RL_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return set_hip_error(e, "hipGetSymbolAddress(scratch)");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return RL_OK;
}

int check_workspace(const Schedule& sch, const rl_opts_t* opts) {
  if (sch.workspace_bytes == 0) return RL_OK;
  if (!opts || !opts->workspace || opts->workspace_bytes < sch.workspace_bytes) {
    std::snprintf(g_hip_error, sizeof(g_hip_error), "this call needs a workspace of %zu bytes", sch.workspace_bytes);
    return RL_ERR_WORKSPACE;
  }
  if ((reinterpret_cast<uintptr_t>(opts->workspace) & 255) != 0) return RL_ERR_ALIGN;
  return RL_OK;
}

}  // namespace

namespace {
// use_static: the scratch is this device's copy of the library's fixed array instead of opts->workspace
int forward_impl(int variant, const rl_tensor_t* X, const rl_tensor_t* W, const rl_tensor_t* A, const rl_tensor_t* B,
                 rl_tensor_t* Y, rl_saved_t* saved, const rl_opts_t* opts, bool use_static) {
  if (!X || !W || !A || !B || !Y || !saved) return RL_ERR_NULL;
  if (variant < RL_FWD_DEFAULT || variant > RL_FWD3) return RL_ERR_VARIANT;
  const int dtype = X->dtype;
  const int dt = internal_dtype(dtype);
  if (dt < 0) return RL_ERR_DTYPE;
  const int64_t n = X->rows, i = X->cols, o = W->cols, r = A->cols;
  int rc;
  bool w_int4 = false;
  if ((rc = check_dims(n, i, o, r, dtype)) != RL_OK) return rc;
  if ((rc = check_tensor(X, n, i, dtype)) != RL_OK) return rc;
  if ((rc = check_weight(W, i, o, dtype, &w_int4)) != RL_OK) return rc;
  if (w_int4 && variant == RL_FWD2) return RL_ERR_UNSUPPORTED;  // no dense W to merge AB into
  if ((rc = check_tensor(A, i, r, dtype)) != RL_OK) return rc;
  if ((rc = check_tensor(B, r, o, dtype)) != RL_OK) return rc;
  if ((rc = check_tensor(Y, n, o, dtype)) != RL_OK) return rc;
  const size_t esz = dtype_size(dt);
  Range ry = range_of(Y->data, n, Y->ld, o, esz);
  if (overlap(ry, range_of(X->data, n, X->ld, i, esz)) || overlap(ry, weight_range(W, i, o, esz, w_int4)) ||
      overlap(ry, range_of(A->data, i, A->ld, r, esz)) || overlap(ry, range_of(B->data, r, B->ld, o, esz)))
    return RL_ERR_ALIAS;

  const float scale = (opts && opts->scale != 0.f) ? opts->scale : 1.f;
  LayerDims L{n, i, o, r, dt, w_int4, scale};
  L.wcol = g_wcol;
  if (opts && opts->dropout_p != 0.f) {
    if (!(opts->dropout_p > 0.f && opts->dropout_p < 1.f)) return RL_ERR_SHAPE;
    if (variant == RL_FWD2 || r > 128 || n * X->ld >= (1LL << 30)) return RL_ERR_UNSUPPORTED;
    int thr = (int)(opts->dropout_p * 256.f + 0.5f);
    thr = thr < 1 ? 1 : (thr > 255 ? 255 : thr);
    L.drop_thr = (uint32_t)thr;
    L.drop_key = drop_key_of(opts->dropout_seed);
  }
  FwdOperands op;
  op.X = mat(X); op.W = weight_mat(W, o, w_int4); op.A = mat(A); op.B = mat(B); op.Y = mat(Y);
  if (opts && opts->bias) {
    if ((reinterpret_cast<uintptr_t>(opts->bias) & 15) != 0) return RL_ERR_ALIGN;
    if (overlap(ry, range_of(opts->bias, 1, o, o, esz))) return RL_ERR_ALIAS;
    op.bias = opts->bias;
  }
  if (variant == RL_FWD2 && saved->M) {  // keep W + s AB for the backward in the caller's buffer
    const int64_t q = dtype == RL_F32 ? 4 : 8;
    if (saved->ldm < o) return RL_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(saved->M) & 15) != 0 || saved->ldm % q != 0) return RL_ERR_ALIGN;
    Range rm = range_of(saved->M, i, saved->ldm, o, esz);
    if (overlap(rm, ry) || overlap(rm, range_of(X->data, n, X->ld, i, esz)) ||
        overlap(rm, weight_range(W, i, o, esz, w_int4)) || overlap(rm, range_of(A->data, i, A->ld, r, esz)) ||
        overlap(rm, range_of(B->data, r, B->ld, o, esz)))
      return RL_ERR_ALIAS;
    op.M.ptr = saved->M;
    op.M.ld = saved->ldm;
    op.keep_M = true;
  }
  // forward1 (also asked for as forward 3) keeps T = s XA for the backward when the caller hands it a buffer
  const bool keep_T = (variant == RL_FWD1 || variant == RL_FWD3) && saved->T != nullptr;
  if (variant == RL_FWD_DEFAULT || keep_T) {
    if (!saved->T) return RL_ERR_NULL;
    const int64_t q = dtype == RL_F32 ? 4 : 8;
    if (saved->ldt < r) return RL_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(saved->T) & 15) != 0 || saved->ldt % q != 0) return RL_ERR_ALIGN;
    Range rt = range_of(saved->T, n, saved->ldt, r, esz);
    if (overlap(rt, ry) || overlap(rt, range_of(X->data, n, X->ld, i, esz)) || overlap(rt, weight_range(W, i, o, esz, w_int4)) ||
        overlap(rt, range_of(A->data, i, A->ld, r, esz)) || overlap(rt, range_of(B->data, r, B->ld, o, esz)))
      return RL_ERR_ALIAS;
    op.T.ptr = saved->T;
    op.T.ld = saved->ldt;
    op.keep_T = keep_T;
  }
  Schedule sch;
  char* ws = opts ? static_cast<char*>(opts->workspace) : nullptr;
  if (use_static) {
    // size the schedule first (no HIP call yet), then lay it out in the fixed array
    if (!build_forward(variant, L, op, nullptr, &sch)) return RL_ERR_VARIANT;
    if (sch.workspace_bytes > kStaticScratchBytes) {
      std::snprintf(g_hip_error, sizeof(g_hip_error), "runlora_forward_static: this call needs %zu bytes of scratch, the fixed array holds %zu",
                    sch.workspace_bytes, kStaticScratchBytes);
      return RL_ERR_WORKSPACE;
    }
    void* p = nullptr;
    ws = nullptr;
    if (!g_dry_run && sch.workspace_bytes > 0) {
      if ((rc = static_scratch(&p)) != RL_OK) return rc;
      ws = static_cast<char*>(p);
    }
    if (!build_forward(variant, L, op, ws, &sch)) return RL_ERR_VARIANT;
  } else {
    if (!build_forward(variant, L, op, ws, &sch)) return RL_ERR_VARIANT;
    if ((rc = check_workspace(sch, opts)) != RL_OK) return rc;
  }

  hipStream_t stream = opts ? static_cast<hipStream_t>(opts->stream) : nullptr;
  rc = run_schedule(sch, ws, stream);
  if (rc != RL_OK) return rc;

  saved->fwd_variant = variant;
  saved->dtype = dtype;
  saved->n = n; saved->i = i; saved->o = o; saved->r = r;
  saved->X = X->data;
  saved->ldx = X->ld;
  saved->scale = scale;
  saved->dropout_thr = L.drop_thr;
  saved->dropout_seed = L.drop_thr ? opts->dropout_seed : 0u;
  if (variant != RL_FWD_DEFAULT && !keep_T) { saved->T = nullptr; saved->ldt = 0; }
  if (variant != RL_FWD2) { saved->M = nullptr; saved->ldm = 0; }
  return RL_OK;
}
}  // namespace

extern "C" int runlora_forward(int variant, const rl_tensor_t* X, const rl_tensor_t* W, const rl_tensor_t* A,
                               const rl_tensor_t* B, rl_tensor_t* Y, rl_saved_t* saved, const rl_opts_t* opts) {
  return forward_impl(variant, X, W, A, B, Y, saved, opts, false);
}

extern "C" int runlora_forward_static(int variant, const rl_tensor_t* X, const rl_tensor_t* W, const rl_tensor_t* A,
                                      const rl_tensor_t* B, rl_tensor_t* Y, rl_saved_t* saved, const rl_opts_t* opts) {
  return forward_impl(variant, X, W, A, B, Y, saved, opts, true);
}

extern "C" int runlora_backward(int variant, const rl_tensor_t* dY, const rl_saved_t* saved, const rl_tensor_t* W,
                                const rl_tensor_t* A, const rl_tensor_t* B, rl_tensor_t* dX, rl_tensor_t* dA,
                                rl_tensor_t* dB, const rl_opts_t* opts) {
  if (!dY || !saved || !W || !A || !B) return RL_ERR_NULL;
  if (variant < RL_BWD_DEFAULT || variant > RL_BWD8) return RL_ERR_VARIANT;
  const int dtype = dY->dtype;
  const int dt = internal_dtype(dtype);
  if (dt < 0) return RL_ERR_DTYPE;
  const int64_t n = dY->rows, o = dY->cols, i = W->rows, r = A->cols;
  int rc;
  bool w_int4 = false;
  if ((rc = check_dims(n, i, o, r, dtype)) != RL_OK) return rc;
  if ((rc = check_tensor(dY, n, o, dtype)) != RL_OK) return rc;
  if ((rc = check_weight(W, i, o, dtype, &w_int4)) != RL_OK) return rc;
  if (w_int4 && (variant == RL_BWD4 || variant == RL_BWD5 || variant == RL_BWD7 || variant == RL_BWD8))
    return RL_ERR_UNSUPPORTED;
  if ((rc = check_tensor(A, i, r, dtype)) != RL_OK) return rc;
  if ((rc = check_tensor(B, r, o, dtype)) != RL_OK) return rc;
  if (dX && (rc = check_tensor(dX, n, i, dtype)) != RL_OK) return rc;
  if (dA && (rc = check_tensor(dA, i, r, dtype)) != RL_OK) return rc;
  if (dB && (rc = check_tensor(dB, r, o, dtype)) != RL_OK) return rc;
  // the forward's record must describe this very layer
  if (saved->fwd_variant < RL_FWD_DEFAULT || saved->fwd_variant > RL_FWD3) return RL_ERR_SAVED_MISMATCH;
  if (saved->dtype != dtype || saved->n != n || saved->i != i || saved->o != o || saved->r != r)
    return RL_ERR_SAVED_MISMATCH;
  if (!saved->X) return RL_ERR_NULL;
  const int64_t q = dtype == RL_F32 ? 4 : 8;
  if (saved->ldx < i) return RL_ERR_SAVED_MISMATCH;
  if ((reinterpret_cast<uintptr_t>(saved->X) & 15) != 0 || saved->ldx % q != 0) return RL_ERR_ALIGN;
  if (variant == RL_BWD_DEFAULT) {
    if (saved->fwd_variant != RL_FWD_DEFAULT || !saved->T || saved->ldt < r) return RL_ERR_SAVED_MISMATCH;
    if ((reinterpret_cast<uintptr_t>(saved->T) & 15) != 0 || saved->ldt % q != 0) return RL_ERR_ALIGN;
  }
  // T = s XA kept by the default chain's forward or by forward1 serves the graphs that would form X A again
  const bool use_T = (variant == RL_BWD1 || variant == RL_BWD5 || variant == RL_BWD6 || variant == RL_BWD7) && saved->T != nullptr &&
                     (saved->fwd_variant == RL_FWD_DEFAULT || saved->fwd_variant == RL_FWD1 || saved->fwd_variant == RL_FWD3);
  if (use_T) {
    if (saved->ldt < r) return RL_ERR_SAVED_MISMATCH;
    if ((reinterpret_cast<uintptr_t>(saved->T) & 15) != 0 || saved->ldt % q != 0) return RL_ERR_ALIGN;
  }
  // W + s AB kept by forward2 serves the graphs that would form it again
  const bool merged_bwd = variant == RL_BWD4 || variant == RL_BWD5 || variant == RL_BWD7 || variant == RL_BWD8;
  const bool use_M = merged_bwd && saved->fwd_variant == RL_FWD2 && saved->M != nullptr;
  if (use_M) {
    if (saved->ldm < o) return RL_ERR_SAVED_MISMATCH;
    if ((reinterpret_cast<uintptr_t>(saved->M) & 15) != 0 || saved->ldm % q != 0) return RL_ERR_ALIGN;
  }
  const size_t esz = dtype_size(dt);
  Range in[7] = {range_of(dY->data, n, dY->ld, o, esz), range_of(saved->X, n, saved->ldx, i, esz),
                 weight_range(W, i, o, esz, w_int4), range_of(A->data, i, A->ld, r, esz),
                 range_of(B->data, r, B->ld, o, esz),
                 (variant == RL_BWD_DEFAULT || use_T) ? range_of(saved->T, n, saved->ldt, r, esz) : Range{nullptr, nullptr},
                 use_M ? range_of(saved->M, i, saved->ldm, o, esz) : Range{nullptr, nullptr}};
  Range outr[3];
  int nout = 0;
  if (dX) outr[nout++] = range_of(dX->data, n, dX->ld, i, esz);
  if (dA) outr[nout++] = range_of(dA->data, i, dA->ld, r, esz);
  if (dB) outr[nout++] = range_of(dB->data, r, dB->ld, o, esz);
  for (int a = 0; a < nout; ++a) {
    for (int b = 0; b < 7; ++b)
      if (in[b].lo && overlap(outr[a], in[b])) return RL_ERR_ALIAS;
    for (int b = a + 1; b < nout; ++b)
      if (overlap(outr[a], outr[b])) return RL_ERR_ALIAS;
  }

  LayerDims L{n, i, o, r, dt, w_int4, saved->scale != 0.f ? saved->scale : 1.f};
  L.wcol = g_wcol;
  if (saved->dropout_thr != 0u) {
    if (saved->dropout_thr > 255u) return RL_ERR_SAVED_MISMATCH;
    if (variant > RL_BWD1 || r > 128 || n * saved->ldx >= (1LL << 30)) return RL_ERR_UNSUPPORTED;
    L.drop_thr = saved->dropout_thr;
    L.drop_key = drop_key_of(saved->dropout_seed);
  }
  BwdOperands op;
  if (use_M) { op.M.ptr = saved->M; op.M.ld = saved->ldm; op.have_M = true; }
  op.have_T = use_T;
  op.dY = mat(dY); op.W = weight_mat(W, o, w_int4); op.A = mat(A); op.B = mat(B);
  op.X.ptr = saved->X; op.X.ld = saved->ldx;
  op.T.ptr = saved->T; op.T.ld = saved->ldt;
  op.want_dX = dX != nullptr; op.want_dA = dA != nullptr; op.want_dB = dB != nullptr;
  if (dX) op.dX = mat(dX);
  if (dA) op.dA = mat(dA);
  if (dB) op.dB = mat(dB);
  Schedule sch;
  char* ws = opts ? static_cast<char*>(opts->workspace) : nullptr;
  if (!build_backward(variant, L, op, ws, &sch)) return RL_ERR_VARIANT;
  if ((rc = check_workspace(sch, opts)) != RL_OK) return rc;
  hipStream_t stream = opts ? static_cast<hipStream_t>(opts->stream) : nullptr;
  return run_schedule(sch, ws, stream);
}

// ---- VeRA: the LoRA graphs on (A, B~ = diag(d) B diag(b)), see vera.hpp ------------------------------------

namespace {

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// workspace layout of the VeRA calls: [B~ r x o][dB~ r x o][the LoRA call's own workspace]
struct VeraLayout {
  size_t factor_bytes = 0;  // one r x o matrix in the layer dtype, rounded up to 256
  rl_tensor_t Bt{}, dBt{};
  rl_opts_t inner{};
};

int vera_layout(const rl_tensor_t* B, const void* d, const void* b, const rl_opts_t* opts, VeraLayout* v) {
  if (!B || !d || !b) return RL_ERR_NULL;
  const int dt = internal_dtype(B->dtype);
  if (dt < 0) return RL_ERR_DTYPE;
  if (B->rows < 1 || B->cols < 1 || B->rows > (1LL << 30) || B->cols > (1LL << 30)) return RL_ERR_SHAPE;
  if (((reinterpret_cast<uintptr_t>(d) | reinterpret_cast<uintptr_t>(b)) & 15) != 0) return RL_ERR_ALIGN;
  v->factor_bytes = align256((size_t)B->rows * (size_t)B->cols * dtype_size(dt));
  if (!opts || !opts->workspace || opts->workspace_bytes < 2 * v->factor_bytes) return RL_ERR_WORKSPACE;
  if ((reinterpret_cast<uintptr_t>(opts->workspace) & 255) != 0) return RL_ERR_ALIGN;
  char* ws = static_cast<char*>(opts->workspace);
  v->Bt = rl_tensor_t{ws, B->rows, B->cols, B->cols, B->dtype, nullptr, 0};
  v->dBt = rl_tensor_t{ws + v->factor_bytes, B->rows, B->cols, B->cols, B->dtype, nullptr, 0};
  v->inner = *opts;
  v->inner.workspace = ws + 2 * v->factor_bytes;
  v->inner.workspace_bytes = opts->workspace_bytes - 2 * v->factor_bytes;
  return RL_OK;
}

}  // namespace

extern "C" int runlora_vera_forward(int variant, const rl_tensor_t* X, const rl_tensor_t* W, const rl_tensor_t* A,
                                    const rl_tensor_t* B, const void* d, const void* b, rl_tensor_t* Y,
                                    rl_saved_t* saved, const rl_opts_t* opts) {
  if (!X || !W || !A || !B || !Y || !saved) return RL_ERR_NULL;
  VeraLayout v;
  int rc = vera_layout(B, d, b, opts, &v);
  if (rc != RL_OK) return rc;
  if (B->dtype != X->dtype) return RL_ERR_DTYPE;
  if ((rc = check_tensor(B, A->cols, W->cols, X->dtype)) != RL_OK) return rc;
  const size_t esz = dtype_size(internal_dtype(B->dtype));
  if (Y->data && Y->rows >= 1 && Y->ld >= Y->cols && Y->cols == B->cols) {
    Range ry = range_of(Y->data, Y->rows, Y->ld, Y->cols, esz);
    if (overlap(ry, range_of(d, 1, B->rows, B->rows, esz)) || overlap(ry, range_of(b, 1, B->cols, B->cols, esz)) ||
        overlap(ry, range_of(B->data, B->rows, B->ld, B->cols, esz)))
      return RL_ERR_ALIAS;
  }
  {
    DryRun dry;  // every check of the layer call, before the first launch
    rl_saved_t probe = *saved;
    if ((rc = runlora_forward(variant, X, W, A, &v.Bt, Y, &probe, &v.inner)) != RL_OK) return rc;
  }
  hipStream_t stream = static_cast<hipStream_t>(opts->stream);
  hipError_t e = vera_scale_run(internal_dtype(B->dtype), B->data, B->ld, d, b, v.Bt.data, v.Bt.ld, B->rows, B->cols, stream);
  if (e != hipSuccess) return set_hip_error(e, "B~ = diag(d) B diag(b)");
  return runlora_forward(variant, X, W, A, &v.Bt, Y, saved, &v.inner);
}

extern "C" int runlora_vera_backward(int variant, const rl_tensor_t* dY, const rl_saved_t* saved, const rl_tensor_t* W,
                                     const rl_tensor_t* A, const rl_tensor_t* B, const void* d, const void* b,
                                     rl_tensor_t* dX, void* dd, void* db, const rl_opts_t* opts) {
  if (!dY || !saved || !W || !A || !B) return RL_ERR_NULL;
  VeraLayout v;
  int rc = vera_layout(B, d, b, opts, &v);
  if (rc != RL_OK) return rc;
  if (B->dtype != dY->dtype) return RL_ERR_DTYPE;
  if ((rc = check_tensor(B, A->cols, dY->cols, dY->dtype)) != RL_OK) return rc;
  if (((reinterpret_cast<uintptr_t>(dd) | reinterpret_cast<uintptr_t>(db)) & 15) != 0) return RL_ERR_ALIGN;
  const size_t esz = dtype_size(internal_dtype(B->dtype));
  const int64_t r = B->rows, o = B->cols;
  {  // the vector gradients must not overlap anything the call reads or its other outputs
    Range outs[2] = {dd ? range_of(dd, 1, r, r, esz) : Range{nullptr, nullptr}, db ? range_of(db, 1, o, o, esz) : Range{nullptr, nullptr}};
    std::vector<Range> others = {range_of(d, 1, r, r, esz), range_of(b, 1, o, o, esz), range_of(B->data, r, B->ld, o, esz)};
    if (dY->data && dY->rows >= 1 && dY->ld >= dY->cols) others.push_back(range_of(dY->data, dY->rows, dY->ld, dY->cols, esz));
    if (A->data && A->rows >= 1 && A->ld >= A->cols) others.push_back(range_of(A->data, A->rows, A->ld, A->cols, esz));
    if (saved->X && saved->n >= 1 && saved->ldx >= saved->i && saved->i >= 1) others.push_back(range_of(saved->X, saved->n, saved->ldx, saved->i, esz));
    if (dX && dX->data && dX->rows >= 1 && dX->ld >= dX->cols) others.push_back(range_of(dX->data, dX->rows, dX->ld, dX->cols, esz));
    if (W->data && W->rows >= 1 && W->ld >= W->cols) others.push_back(range_of(W->data, W->rows, W->ld, W->cols, W->dtype == RL_INT4_G64 ? 1 : esz));
    for (const Range& out : outs) {
      if (!out.lo) continue;
      for (const Range& in : others)
        if (overlap(out, in)) return RL_ERR_ALIAS;
    }
    if (outs[0].lo && outs[1].lo && overlap(outs[0], outs[1])) return RL_ERR_ALIAS;
  }
  rl_tensor_t* dBt = (dd || db) ? &v.dBt : nullptr;
  {
    DryRun dry;
    if ((rc = runlora_backward(variant, dY, saved, W, A, &v.Bt, dX, nullptr, dBt, &v.inner)) != RL_OK) return rc;
  }
  const int dt = internal_dtype(B->dtype);
  hipStream_t stream = static_cast<hipStream_t>(opts->stream);
  hipError_t e = vera_scale_run(dt, B->data, B->ld, d, b, v.Bt.data, v.Bt.ld, r, o, stream);
  if (e != hipSuccess) return set_hip_error(e, "B~ = diag(d) B diag(b)");
  if ((rc = runlora_backward(variant, dY, saved, W, A, &v.Bt, dX, nullptr, dBt, &v.inner)) != RL_OK) return rc;
  if (dBt) {
    e = vera_grad_run(dt, v.dBt.data, v.dBt.ld, B->data, B->ld, d, b, dd, db, r, o, stream);
    if (e != hipSuccess) return set_hip_error(e, "dd, db from dB~");
  }
  return RL_OK;
}

extern "C" size_t runlora_vera_workspace_bytes(int fwd, int bwd, int64_t n, int64_t i, int64_t o, int64_t r, int dtype) {
  const int dt = internal_dtype(dtype);
  if (dt < 0 || n < 1 || i < 1 || o < 1 || r < 1) return 0;
  if (fwd > RL_FWD3 || bwd > RL_BWD8 || (fwd < 0 && bwd < 0)) return 0;
  return 2 * align256((size_t)r * (size_t)o * dtype_size(dt)) + runlora_workspace_bytes(fwd, bwd, n, i, o, r, dtype);
}

// ---- DoRA: the merged-weight graphs on (W diag(g), A, B diag(g)), g = m / c, see dora.hpp ----------------

namespace {

// workspace layout of the DoRA calls: [g: o floats][B~ r x o][dB~ r x o][partial sums: rows x o floats][the layer call's own]
struct DoraLayout {
  float* g = nullptr;
  rl_tensor_t Bt{}, dBt{};
  float* partial = nullptr;
  int norm_rows = 0, dm_rows = 0;
  size_t head_bytes = 0;
  rl_opts_t inner{};
};

size_t dora_head_bytes(int64_t n, int64_t i, int64_t o, int64_t r, int dt, int* norm_rows, int* dm_rows) {
  int gx = 0, gy = 0, bpw = 0;
  merge_grid(i, o, r, &gx, &gy, &bpw);
  const int dmr = dora_dm_slices(n, o);
  if (norm_rows) *norm_rows = gy;
  if (dm_rows) *dm_rows = dmr;
  const size_t rows = (size_t)(gy > dmr ? gy : dmr);
  return align256((size_t)o * 4) + 2 * align256((size_t)r * (size_t)o * dtype_size(dt)) + align256(rows * (size_t)o * 4);
}

int dora_layout(const rl_tensor_t* W, const rl_tensor_t* A, const rl_tensor_t* B, const void* m, int64_t n,
                const rl_opts_t* opts, DoraLayout* v) {
  if (!m) return RL_ERR_NULL;
  const int dt = internal_dtype(B->dtype);
  if (dt < 0) return RL_ERR_DTYPE;
  if (W->dtype != B->dtype || A->dtype != B->dtype) return RL_ERR_DTYPE;
  const int64_t i = W->rows, o = W->cols, r = A->cols;
  if (n < 1 || i < 1 || o < 1 || r < 1 || i > (1LL << 30) || o > (1LL << 30) || B->rows != r || B->cols != o || A->rows != i)
    return RL_ERR_SHAPE;
  if (dt == DT_F32 || r > 128) return RL_ERR_UNSUPPORTED;
  if ((reinterpret_cast<uintptr_t>(m) & 15) != 0) return RL_ERR_ALIGN;
  v->head_bytes = dora_head_bytes(n, i, o, r, dt, &v->norm_rows, &v->dm_rows);
  if (!opts || !opts->workspace || opts->workspace_bytes < v->head_bytes) return RL_ERR_WORKSPACE;
  if ((reinterpret_cast<uintptr_t>(opts->workspace) & 255) != 0) return RL_ERR_ALIGN;
  char* ws = static_cast<char*>(opts->workspace);
  const size_t fb = align256((size_t)r * (size_t)o * dtype_size(dt));
  v->g = reinterpret_cast<float*>(ws);
  ws += align256((size_t)o * 4);
  v->Bt = rl_tensor_t{ws, r, o, o, B->dtype, nullptr, 0};
  v->dBt = rl_tensor_t{ws + fb, r, o, o, B->dtype, nullptr, 0};
  v->partial = reinterpret_cast<float*>(ws + 2 * fb);
  v->inner = *opts;
  v->inner.workspace = static_cast<char*>(opts->workspace) + v->head_bytes;
  v->inner.workspace_bytes = opts->workspace_bytes - v->head_bytes;
  return RL_OK;
}

}  // namespace

extern "C" int runlora_dora_forward(int variant, const rl_tensor_t* X, const rl_tensor_t* W, const rl_tensor_t* A,
                                    const rl_tensor_t* B, const void* m, rl_tensor_t* Y, rl_saved_t* saved, float* c,
                                    const rl_opts_t* opts) {
  if (!X || !W || !A || !B || !Y || !saved || !c) return RL_ERR_NULL;
  if (variant != RL_FWD2) return variant < RL_FWD_DEFAULT || variant > RL_FWD3 ? RL_ERR_VARIANT : RL_ERR_UNSUPPORTED;
  DoraLayout v;
  int rc = dora_layout(W, A, B, m, X->rows, opts, &v);
  if (rc != RL_OK) return rc;
  if (opts->dropout_p != 0.f) return RL_ERR_UNSUPPORTED;
  if ((reinterpret_cast<uintptr_t>(c) & 15) != 0) return RL_ERR_ALIGN;
  const int dt = internal_dtype(B->dtype);
  const size_t esz = dtype_size(dt);
  const int64_t i = W->rows, o = W->cols, r = A->cols;
  if ((rc = check_tensor(B, r, o, X->dtype)) != RL_OK) return rc;
  {  // c is written before Y is: it may overlap no operand and not Y; Y may not overlap m
    Range rc_ = range_of(c, 1, o, o, 4), rm = range_of(m, 1, o, o, esz);
    std::vector<Range> others = {rm, range_of(B->data, r, B->ld, o, esz)};
    if (W->data && W->ld >= o) others.push_back(range_of(W->data, i, W->ld, o, esz));
    if (A->data && A->ld >= r) others.push_back(range_of(A->data, i, A->ld, r, esz));
    if (X->data && X->rows >= 1 && X->ld >= X->cols) others.push_back(range_of(X->data, X->rows, X->ld, X->cols, esz));
    if (opts->bias) others.push_back(range_of(opts->bias, 1, o, o, esz));
    if (saved->M && saved->ldm >= o) others.push_back(range_of(saved->M, i, saved->ldm, o, esz));
    if (Y->data && Y->rows >= 1 && Y->ld >= Y->cols && Y->cols == o) {
      Range ry = range_of(Y->data, Y->rows, Y->ld, o, esz);
      if (overlap(ry, rm)) return RL_ERR_ALIAS;
      others.push_back(ry);
    }
    for (const Range& in : others)
      if (overlap(rc_, in)) return RL_ERR_ALIAS;
  }
  WCol hook(v.g);
  {
    DryRun dry;  // every check of the layer call, before the first launch
    rl_saved_t probe = *saved;
    if ((rc = runlora_forward(variant, X, W, A, &v.Bt, Y, &probe, &v.inner)) != RL_OK) return rc;
  }
  hipStream_t stream = static_cast<hipStream_t>(opts->stream);
  MergeDesc nd;
  nd.W = W->data; nd.A = A->data; nd.B = B->data; nd.M = nullptr;
  nd.ldw = W->ld; nd.lda = A->ld; nd.ldb = B->ld; nd.ldm = 0;
  nd.I = i; nd.O = o; nd.R = r;
  nd.alpha = opts->scale != 0.f ? opts->scale : 1.f;
  nd.sq_partial = v.partial;
  hipError_t e = merge_run(dt, nd, stream);
  if (e != hipSuccess) return set_hip_error(e, "column sums of (W + s A B)^2");
  if ((e = dora_norm_finish_run(dt, v.partial, v.norm_rows, m, c, v.g, o, stream)) != hipSuccess)
    return set_hip_error(e, "c, g = m / c");
  if ((e = dora_colscale_run(dt, B->data, B->ld, v.g, v.Bt.data, v.Bt.ld, r, o, stream)) != hipSuccess)
    return set_hip_error(e, "B~ = B diag(g)");
  return runlora_forward(variant, X, W, A, &v.Bt, Y, saved, &v.inner);
}

extern "C" int runlora_dora_backward(int variant, const rl_tensor_t* dY, const rl_saved_t* saved, const rl_tensor_t* W,
                                     const rl_tensor_t* A, const rl_tensor_t* B, const void* m, const float* c,
                                     const rl_tensor_t* Y, rl_tensor_t* dX, rl_tensor_t* dA, rl_tensor_t* dB, void* dm,
                                     const rl_opts_t* opts) {
  if (!dY || !saved || !W || !A || !B || !c) return RL_ERR_NULL;
  if (variant < RL_BWD_DEFAULT || variant > RL_BWD8) return RL_ERR_VARIANT;
  if (variant != RL_BWD4 && variant != RL_BWD5 && variant != RL_BWD7 && variant != RL_BWD8) return RL_ERR_UNSUPPORTED;
  DoraLayout v;
  int rc = dora_layout(W, A, B, m, dY->rows, opts, &v);
  if (rc != RL_OK) return rc;
  if (saved->dropout_thr != 0u) return RL_ERR_UNSUPPORTED;
  if (dm && !Y) return RL_ERR_NULL;
  if (((reinterpret_cast<uintptr_t>(c) | reinterpret_cast<uintptr_t>(dm)) & 15) != 0) return RL_ERR_ALIGN;
  const int dt = internal_dtype(B->dtype);
  const size_t esz = dtype_size(dt);
  const int64_t n = dY->rows, i = W->rows, o = W->cols, r = A->cols;
  if ((rc = check_tensor(B, r, o, dY->dtype)) != RL_OK) return rc;
  if (dB && (rc = check_tensor(dB, r, o, dY->dtype)) != RL_OK) return rc;
  if (dm) {
    if ((rc = check_tensor(Y, n, o, dY->dtype)) != RL_OK) return rc;
    if (opts->bias && (reinterpret_cast<uintptr_t>(opts->bias) & 15) != 0) return RL_ERR_ALIGN;
  }
  {  // dm and dB are written here: they may overlap nothing the call reads and none of its other outputs
    std::vector<Range> outs, others = {range_of(m, 1, o, o, esz), range_of(c, 1, o, o, 4), range_of(B->data, r, B->ld, o, esz)};
    if (dm) outs.push_back(range_of(dm, 1, o, o, esz));
    if (dB) outs.push_back(range_of(dB->data, r, dB->ld, o, esz));
    if (dY->data && dY->rows >= 1 && dY->ld >= dY->cols) others.push_back(range_of(dY->data, n, dY->ld, dY->cols, esz));
    if (Y && Y->data && Y->ld >= o) others.push_back(range_of(Y->data, n, Y->ld, o, esz));
    if (opts->bias) others.push_back(range_of(opts->bias, 1, o, o, esz));
    if (W->data && W->ld >= o) others.push_back(range_of(W->data, i, W->ld, o, esz));
    if (A->data && A->ld >= r) others.push_back(range_of(A->data, i, A->ld, r, esz));
    if (saved->X && saved->n >= 1 && saved->ldx >= saved->i && saved->i >= 1) others.push_back(range_of(saved->X, saved->n, saved->ldx, saved->i, esz));
    if (saved->M && saved->ldm >= o) others.push_back(range_of(saved->M, i, saved->ldm, o, esz));
    if (dX && dX->data && dX->rows >= 1 && dX->ld >= dX->cols) others.push_back(range_of(dX->data, dX->rows, dX->ld, dX->cols, esz));
    if (dA && dA->data && dA->rows >= 1 && dA->ld >= dA->cols) others.push_back(range_of(dA->data, dA->rows, dA->ld, dA->cols, esz));
    for (const Range& out : outs)
      for (const Range& in : others)
        if (overlap(out, in)) return RL_ERR_ALIAS;
    if (outs.size() == 2 && overlap(outs[0], outs[1])) return RL_ERR_ALIAS;
    if (Y && Y->data && Y->ld >= o) {  // the forward's output is read after dX and dA are written
      Range ry = range_of(Y->data, n, Y->ld, o, esz);
      if (dX && dX->data && dX->rows >= 1 && dX->ld >= dX->cols && overlap(ry, range_of(dX->data, dX->rows, dX->ld, dX->cols, esz))) return RL_ERR_ALIAS;
      if (dA && dA->data && dA->rows >= 1 && dA->ld >= dA->cols && overlap(ry, range_of(dA->data, dA->rows, dA->ld, dA->cols, esz))) return RL_ERR_ALIAS;
    }
  }
  rl_tensor_t* dBt = dB ? &v.dBt : nullptr;
  WCol hook(v.g);
  {
    DryRun dry;
    if ((rc = runlora_backward(variant, dY, saved, W, A, &v.Bt, dX, dA, dBt, &v.inner)) != RL_OK) return rc;
  }
  hipStream_t stream = static_cast<hipStream_t>(opts->stream);
  hipError_t e = dora_g_run(dt, m, c, v.g, o, stream);
  if (e != hipSuccess) return set_hip_error(e, "g = m / c");
  if ((e = dora_colscale_run(dt, B->data, B->ld, v.g, v.Bt.data, v.Bt.ld, r, o, stream)) != hipSuccess)
    return set_hip_error(e, "B~ = B diag(g)");
  if ((rc = runlora_backward(variant, dY, saved, W, A, &v.Bt, dX, dA, dBt, &v.inner)) != RL_OK) return rc;
  if (dB && (e = dora_colscale_run(dt, v.dBt.data, v.dBt.ld, v.g, dB->data, dB->ld, r, o, stream)) != hipSuccess)
    return set_hip_error(e, "dB = dB~ diag(g)");
  if (dm && (e = dora_dm_run(dt, dY->data, dY->ld, Y->data, Y->ld, opts->bias, m, v.partial, dm, n, o, stream)) != hipSuccess)
    return set_hip_error(e, "dm");
  return RL_OK;
}

extern "C" size_t runlora_dora_workspace_bytes(int fwd, int bwd, int64_t n, int64_t i, int64_t o, int64_t r, int dtype) {
  const int dt = internal_dtype(dtype);
  if (dt < 0 || dt == DT_F32 || n < 1 || i < 1 || o < 1 || r < 1 || r > 128) return 0;
  if (fwd > RL_FWD3 || bwd > RL_BWD8 || (fwd < 0 && bwd < 0)) return 0;
  return dora_head_bytes(n, i, o, r, dt, nullptr, nullptr) + runlora_workspace_bytes(fwd, bwd, n, i, o, r, dtype);
}

extern "C" size_t runlora_saved_bytes(int fwd, int64_t n, int64_t i, int64_t o, int64_t r, int dtype, int keep_merged) {
  const int dt = internal_dtype(dtype);
  if (dt < 0 || n < 1 || i < 1 || o < 1 || r < 1) return 0;
  const size_t e = dtype_size(dt);
  switch (fwd) {
    case RL_FWD_DEFAULT: return (size_t)n * (size_t)r * e;  // T = XA
    case RL_FWD1:
    case RL_FWD3: return (keep_merged & 2) ? (size_t)n * (size_t)r * e : 0;  // T = XA kept on request
    case RL_FWD2: return (keep_merged & 1) ? (size_t)i * (size_t)o * e : 0;
    default: return 0;
  }
}

extern "C" size_t runlora_workspace_bytes(int fwd, int bwd, int64_t n, int64_t i, int64_t o, int64_t r, int dtype) {
  return runlora_workspace_bytes_w(fwd, bwd, n, i, o, r, dtype, dtype);
}

extern "C" size_t runlora_workspace_bytes_w(int fwd, int bwd, int64_t n, int64_t i, int64_t o, int64_t r, int dtype,
                                            int w_dtype) {
  const int dt = internal_dtype(dtype);
  if (dt < 0 || n < 1 || i < 1 || o < 1 || r < 1) return 0;
  if (w_dtype != dtype && w_dtype != RL_INT4_G64) return 0;
  LayerDims L{n, i, o, r, dt, w_dtype == RL_INT4_G64};
  size_t need = 0;
  Schedule sch;
  // dense rows (ld = columns): which kernel a rank-r product runs on, and with it the scratch, depends on the
  // operands' extents; a call on tensors with padded rows may need more and says how much (RL_ERR_WORKSPACE)
  if (fwd >= 0) {
    FwdOperands op;
    op.X.ld = i; op.W.ld = o; op.A.ld = r; op.B.ld = o; op.Y.ld = o; op.T.ld = r; op.M.ld = o;
    if (build_forward(fwd, L, op, nullptr, &sch) && sch.workspace_bytes > need) need = sch.workspace_bytes;
  }
  if (bwd >= 0) {
    BwdOperands op;
    op.dY.ld = o; op.X.ld = i; op.W.ld = o; op.A.ld = r; op.B.ld = o; op.T.ld = r; op.dX.ld = i; op.dA.ld = r; op.dB.ld = o;
    op.M.ld = o;
    if (build_backward(bwd, L, op, nullptr, &sch) && sch.workspace_bytes > need) need = sch.workspace_bytes;
  }
  return need;
}

extern "C" const char* runlora_strerror(int code) {
  switch (code) {
    case RL_OK: return "ok";
    case RL_ERR_NULL: return "a required pointer is NULL";
    case RL_ERR_SHAPE: return "tensor dimensions do not fit together";
    case RL_ERR_DTYPE: return "unknown dtype or mixed dtypes in one call";
    case RL_ERR_VARIANT: return "unknown variant id";
    case RL_ERR_SAVED_MISMATCH: return "saved context does not match this backward";
    case RL_ERR_ALIGN: return "pointer, leading dimension or dimension violates the alignment rules";
    case RL_ERR_ALIAS: return "an output buffer overlaps an input buffer";
    case RL_ERR_WORKSPACE: return "workspace missing or too small";
    case RL_ERR_UNSUPPORTED: return "request not supported by this build";
    case RL_ERR_HIP: return "HIP launch failed";
    default: return "unknown status";
  }
}

extern "C" const char* runlora_last_hip_error(void) { return g_hip_error; }
extern "C" int runlora_version(void) { return 100; }

// ---- the tile GEMM as a call of its own ---------------------------------------------------------

static int check_gemm(const rl_gemm_t* g, GemmDesc* d, GemmPlan* plan) {
  if (!g || !g->A || !g->B || !g->C) return RL_ERR_NULL;
  const int dt = internal_dtype(g->dtype);
  if (dt < 0) return RL_ERR_DTYPE;
  if (g->a_strided && g->b_kcontig) return RL_ERR_UNSUPPORTED;
  if (g->M < 1 || g->N < 1 || g->K < 1 || g->K2 < 0) return RL_ERR_SHAPE;
  if (g->M > (1LL << 30) || g->N > (1LL << 30) || g->K > (1LL << 30) || g->K2 > (1LL << 30)) return RL_ERR_SHAPE;
  if (g->K2 > 0 && (!g->A2 || !g->B2)) return RL_ERR_NULL;
  if (g->tile_cfg < -1 || g->tile_cfg > CFG_COUNT || g->splits < 0) return RL_ERR_VARIANT;
  if (g->trans_out != 0 && g->trans_out != 1) return RL_ERR_VARIANT;
  if (g->tile_cfg == CFG_COUNT) {  // the streaming kernel
    if (g->N > 128 || g->K2 > 0 || g->D) return RL_ERR_UNSUPPORTED;
    const int64_t esz = g->dtype == RL_F32 ? 4 : 2;
    const int64_t a_rows = g->a_strided ? g->K : g->M, b_rows = g->b_kcontig ? g->N : g->K;
    if (a_rows * g->lda * esz >= (1LL << 31) || b_rows * g->ldb * esz >= (1LL << 31)) return RL_ERR_UNSUPPORTED;
  } else if (g->trans_out) {
    return RL_ERR_UNSUPPORTED;
  }
  const int64_t q = dt == DT_F32 ? 4 : 8;
  if (g->N % q || g->K % q || g->K2 % q || (g->a_strided && g->M % q)) return RL_ERR_ALIGN;
  const int64_t a_cols = g->a_strided ? g->M : g->K, a2_cols = g->a_strided ? g->M : g->K2;
  const int64_t b_cols = g->b_kcontig ? g->K : g->N, b2_cols = g->b_kcontig ? g->K2 : g->N;
  if (g->lda < a_cols || g->ldb < b_cols || g->ldc < (g->trans_out ? g->M : g->N)) return RL_ERR_SHAPE;
  if (g->K2 > 0 && (g->lda2 < a2_cols || g->ldb2 < b2_cols)) return RL_ERR_SHAPE;
  if (g->D && g->ldd < g->N) return RL_ERR_SHAPE;
  const void* ptrs[6] = {g->A, g->B, g->A2, g->B2, g->D, g->C};
  for (const void* p : ptrs)
    if (p && (reinterpret_cast<uintptr_t>(p) & 15) != 0) return RL_ERR_ALIGN;
  if (g->lda % q || g->ldb % q || g->ldc % q || (g->K2 > 0 && (g->lda2 % q || g->ldb2 % q)) || (g->D && g->ldd % q))
    return RL_ERR_ALIGN;
  d->dtype = dt;
  d->a_strided = g->a_strided;
  d->b_kcontig = g->b_kcontig;
  d->M = g->M; d->N = g->N;
  d->nseg = g->K2 > 0 ? 2 : 1;
  d->A[0] = g->A; d->B[0] = g->B; d->lda[0] = g->lda; d->ldb[0] = g->ldb; d->K[0] = g->K;
  d->A[1] = g->A2; d->B[1] = g->B2; d->lda[1] = g->lda2; d->ldb[1] = g->ldb2; d->K[1] = g->K2;
  d->C = g->C; d->ldc = g->ldc; d->D = g->D; d->ldd = g->ldd;
  d->alpha = g->alpha != 0.f ? g->alpha : 1.f;
  if (g->bias) {
    if ((reinterpret_cast<uintptr_t>(g->bias) & 15) != 0) return RL_ERR_ALIGN;
    if (g->tile_cfg == CFG_COUNT) return RL_ERR_UNSUPPORTED;  // the streaming kernel has no bias path
    d->bias = g->bias;
  }
  if (g->tile_cfg != CFG_COUNT) *plan = gemm_plan(dt, g->M, g->N, g->K, g->K2, g->tile_cfg, g->splits);
  return RL_OK;
}

static void gemm_as_skinny(const rl_gemm_t* g, SkinnyDesc* k, SkinnyPlan* plan) {
  k->A = g->A; k->B = g->B; k->C = g->C;
  k->lda = g->lda; k->ldb = g->ldb; k->ldc = g->ldc;
  k->M = g->M; k->N = g->N; k->K = g->K;
  k->a_strided = g->a_strided; k->b_kcontig = g->b_kcontig; k->trans_out = g->trans_out;
  k->alpha = g->alpha != 0.f ? g->alpha : 1.f;
  *plan = skinny_plan(internal_dtype(g->dtype), 1, k);
  if (g->splits > 0) {
    plan->splits = g->splits;
    plan->partial_bytes = g->splits > 1 ? (size_t)g->splits * (size_t)g->M * (size_t)g->N * sizeof(float) : 0;
  }
}

extern "C" size_t runlora_gemm_workspace_bytes(const rl_gemm_t* g) {
  GemmDesc d;
  GemmPlan plan;
  if (check_gemm(g, &d, &plan) != RL_OK) return 0;
  if (g->tile_cfg == CFG_COUNT) {
    SkinnyDesc k;
    SkinnyPlan sp;
    gemm_as_skinny(g, &k, &sp);
    return sp.partial_bytes;
  }
  return plan.partial_bytes;
}

extern "C" int runlora_gemm(const rl_gemm_t* g, const rl_opts_t* opts) {
  GemmDesc d;
  GemmPlan plan;
  int rc = check_gemm(g, &d, &plan);
  if (rc != RL_OK) return rc;
  SkinnyDesc k;
  SkinnyPlan sp;
  const bool streaming = g->tile_cfg == CFG_COUNT;
  if (streaming) {
    gemm_as_skinny(g, &k, &sp);
    plan.partial_bytes = sp.partial_bytes;
  }
  float* scratch = nullptr;
  if (plan.partial_bytes > 0) {
    if (!opts || !opts->workspace || opts->workspace_bytes < plan.partial_bytes) return RL_ERR_WORKSPACE;
    if ((reinterpret_cast<uintptr_t>(opts->workspace) & 255) != 0) return RL_ERR_ALIGN;
    scratch = static_cast<float*>(opts->workspace);
  }
  hipStream_t stream = opts ? static_cast<hipStream_t>(opts->stream) : nullptr;
  hipError_t e = streaming ? skinny_run(d.dtype, 1, &k, sp, scratch, stream) : gemm_run(d, plan, scratch, stream);
  if (e != hipSuccess) return set_hip_error(e, "runlora_gemm");
  return RL_OK;
}

// ---- per-step timing ------------------------------------------------------------------------------

extern "C" int runlora_profile_disable(void) {
  for (hipEvent_t e : g_prof.start) if (e) (void)hipEventDestroy(e);
  for (hipEvent_t e : g_prof.stop) if (e) (void)hipEventDestroy(e);
  for (hipEvent_t e : g_prof.kstart) if (e) (void)hipEventDestroy(e);
  for (hipEvent_t e : g_prof.kstop) if (e) (void)hipEventDestroy(e);
  g_prof.start.clear();
  g_prof.stop.clear();
  g_prof.kstart.clear();
  g_prof.kstop.clear();
  g_prof.kbound.clear();
  g_prof.rec.clear();
  g_prof.used = 0;
  g_prof.on = false;
  return RL_OK;
}

extern "C" int runlora_profile_enable(int max_steps) {
  if (max_steps < 1 || max_steps > (1 << 20)) return RL_ERR_SHAPE;
  runlora_profile_disable();
  g_prof.start.resize(max_steps);
  g_prof.stop.resize(max_steps);
  g_prof.rec.resize(max_steps);
  constexpr int KM = KernelEvents::kMax;
  g_prof.start.assign(max_steps, nullptr);
  g_prof.stop.assign(max_steps, nullptr);
  g_prof.kstart.assign((size_t)max_steps * KM, nullptr);
  g_prof.kstop.assign((size_t)max_steps * KM, nullptr);
  g_prof.kbound.assign(max_steps, 0);
  for (int k = 0; k < max_steps; ++k) {
    hipError_t e = hipEventCreate(&g_prof.start[k]);
    if (e == hipSuccess) e = hipEventCreate(&g_prof.stop[k]);
    for (int q = 0; q < KM && e == hipSuccess; ++q) {
      e = hipEventCreate(&g_prof.kstart[(size_t)k * KM + q]);
      if (e == hipSuccess) e = hipEventCreate(&g_prof.kstop[(size_t)k * KM + q]);
    }
    if (e != hipSuccess) {
      runlora_profile_disable();  // destroys what was created (the rest is still null)
      return set_hip_error(e, "hipEventCreate");
    }
  }
  g_prof.on = true;
  return RL_OK;
}

extern "C" int runlora_profile_kernel_times(int on) {
  g_prof.kernel_events = on != 0;
  return RL_OK;
}

extern "C" int runlora_profile_collect(rl_step_time_t* out, int cap) {
  if (!out && cap > 0) return RL_ERR_NULL;
  if (!g_prof.on) return 0;
  int written = 0;
  for (size_t k = 0; k < g_prof.used; ++k) {
    hipError_t e = hipEventSynchronize(g_prof.stop[k]);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, g_prof.start[k], g_prof.stop[k]);
    float kms = ms, main_ms = ms;
    const int nk = g_prof.kbound[k];
    if (nk > 0) kms = 0.f;
    for (int q = 0; q < nk && e == hipSuccess; ++q) {
      float one = 0.f;
      e = hipEventElapsedTime(&one, g_prof.kstart[k * KernelEvents::kMax + q], g_prof.kstop[k * KernelEvents::kMax + q]);
      kms += one;
      if (q == 0) main_ms = one;
    }
    if (e != hipSuccess) {
      g_prof.used = 0;
      return set_hip_error(e, "profile collect");
    }
    if (written < cap) {
      out[written] = g_prof.rec[k];
      out[written].us = (double)ms * 1e3;
      out[written].kernel_us = (double)kms * 1e3;
      out[written].main_us = (double)main_ms * 1e3;
      out[written].kernels = nk;
      ++written;
    }
  }
  g_prof.used = 0;
  return written;
}
