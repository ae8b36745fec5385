// Variant schedules: each computation graph of the LoRA layer (Section 2 of arxiv 2312.03415:
// forward variants 1-2, Algorithms 1-5, and the default chain) written as the ordered list of
// GEMM launches that realises it, together with its scratch layout.  The same list drives the
// launches (api.hip), the workspace size and the selector's time model (select.cpp), so the three
// cannot drift apart.  Internal to the library.
#pragma once
#include <vector>

#include "gemm.hpp"

namespace rl {

struct Mat {  // device matrix view; ptr may be null when only shapes are needed
  const void* ptr = nullptr;
  int64_t ld = 0;
  // frozen W stored as int4 with group scales (see GemmDesc::Bscale): ptr = packed nibbles
  const void* scales = nullptr;
  int64_t lds = 0;
};

struct LayerDims {
  int64_t n = 0, i = 0, o = 0, r = 0;
  int dtype = DT_BF16;
  bool w_int4 = false;  // W is int4: its products run on the generic engine, merged graphs do not exist
  // LoRA scale s of Y = XW + s (XA) B.  It is applied where a rank-r factor or the merged weight is
  // formed (T = s XA, Z1 = s dY B^T, M = W + s AB, dA = s Z2 B^T, dB = s A^T Z2), so that every later
  // product of the graph is the paper's, unchanged.
  float scale = 1.f;
  // LoRA dropout on the adapter's input (drop_thr = round(256 p), 0 = none): Y = XW + s' ((X o m) A) B with
  // the keep-mask m of gemm_engine.hpp and s' = scale / (1 - drop_thr / 256) in place of scale.  Only the
  // graphs that never merge AB into W and never form X^T dY exist with it: forward 0/1, backward 0/1, the
  // latter with dX = dY W^T followed by dX += m o (Z1 A^T) instead of the concatenated contraction.
  uint32_t drop_thr = 0, drop_key = 0;
  // DoRA: the frozen weight is W diag(wcol) (device, o floats).  It is never formed: only the graphs in which
  // W enters through M = W + s AB alone exist with it (forward2, backward 4 / 5 / 7 / 8), where the merge kernel
  // scales W's columns on the way; 16-bit types, r <= 128.
  const float* wcol = nullptr;
};

struct Step {
  bool is_merge = false;  // M = W + A B on the merge kernel (mg); otherwise see nsk
  MergeDesc mg;
  int nsk = 0;  // 0: one tile-GEMM launch (d, plan); 1 or 2: streaming-kernel launch of sk[0..nsk-1]
  GemmDesc d;
  GemmPlan plan;
  SkinnyDesc sk[2];
  SkinnyPlan skplan;
  const char* what = "";  // the product(s) in the paper's notation, e.g. "Z1 = dY B^T"
};

struct Schedule {
  std::vector<Step> steps;
  size_t workspace_bytes = 0;  // intermediates + split-K partials
  size_t partial_offset = 0;   // where the shared split-K scratch starts
};

struct FwdOperands {
  Mat X, W, A, B, Y, T;  // T: caller's buffer for the default chain (kept for the backward)
  bool keep_T = false;   // forward1: write T = s XA into T (caller's buffer) and leave it for the backward
  const void* bias = nullptr;  // frozen bias of the base layer [o], added by the GEMM that writes Y
  Mat M;                       // forward2 with keep_M: W + s AB goes here (caller's buffer) and stays
  bool keep_M = false;
};
struct BwdOperands {
  Mat dY, X, W, A, B, T, dX, dA, dB;
  bool want_dX = true, want_dA = true, want_dB = true;
  Mat M;                // have_M: W + s AB as forward2 left it; the merged graphs read it instead of
  bool have_M = false;  // forming it again
  bool have_T = false;  // T = s XA as the default chain's forward or forward1 left it: the graphs that would form
                        // X A again (Z2 of Algorithms 1 and 5, T of items 6 and 7) read it instead
};

// ws_base may be null (sizing / modelling).  Returns false for an unknown variant.
bool build_forward(int variant, const LayerDims& L, const FwdOperands& op, void* ws_base, Schedule* out);
bool build_backward(int variant, const LayerDims& L, const BwdOperands& op, void* ws_base, Schedule* out);

inline size_t dtype_size(int dtype) { return dtype == DT_F32 ? 4 : 2; }

}  // namespace rl
