// Variant schedules (see schedule.hpp).  Host code only.
#include "schedule.hpp"

namespace rl {
namespace {

constexpr size_t kAlign = 256;

struct Builder {
  const LayerDims& L;
  char* base;
  size_t used = 0;
  size_t max_partial = 0;
  Schedule* out;
  bool failed = false;  // a step this build cannot run (masking X inside the tile GEMM)

  Builder(const LayerDims& l, void* ws, Schedule* o) : L(l), base(static_cast<char*>(ws)), out(o) {}

  // the LoRA scale as the kernels apply it: under dropout the kept inputs are scaled by 1 / (1 - p)
  float scale() const { return L.drop_thr ? L.scale * 256.f / (256.f - (float)L.drop_thr) : L.scale; }
  uint32_t drop_cpr() const { return (uint32_t)(L.i / 4); }

  // dense [rows, cols] scratch matrix in the layer dtype
  Mat scratch(int64_t rows, int64_t cols) {
    Mat m;
    m.ptr = base ? base + used : nullptr;
    m.ld = cols;
    size_t bytes = (size_t)rows * (size_t)cols * dtype_size(L.dtype);
    used += (bytes + kAlign - 1) / kAlign * kAlign;
    return m;
  }

  // C[M,N] = op(A)[M,K] op(B)[K,N] (+ second segment) (+ D)
  // b_is_w: B is the layer's frozen W (int4 when L.w_int4)
  void gemm(const char* what, int a_strided, int b_kcontig, int64_t M, int64_t N, int64_t K, Mat A, Mat B,
            Mat C, const Mat* D = nullptr, int64_t K2 = 0, const Mat* A2 = nullptr, const Mat* B2 = nullptr,
            bool b_is_w = false, float alpha = 1.f, const void* bias = nullptr, bool mask_out = false) {
    // A rank-r update of a large matrix (Y += T B, dX += Z1 A^T of the default chain) is the merge kernel's
    // operation, M = W + alpha A B, on other operands: one pass over the matrix at streaming speed instead of
    // a tile GEMM whose contraction is a fraction of a K tile.  Under LoRA dropout the update of dX is masked
    // (dX += m o (Z1 A^T)): the kernel masks the product before it adds.
    if (D && K2 == 0 && !a_strided && !bias && !(b_is_w && L.w_int4) && merge_ok(L.dtype, K)) {
      Step m;
      m.what = what;
      m.is_merge = true;
      m.d.dtype = L.dtype;
      m.mg.W = D->ptr; m.mg.A = A.ptr; m.mg.B = B.ptr; m.mg.M = const_cast<void*>(C.ptr);
      m.mg.ldw = D->ld; m.mg.lda = A.ld; m.mg.ldb = B.ld; m.mg.ldm = C.ld;
      m.mg.I = M; m.mg.O = N; m.mg.R = K;
      m.mg.alpha = alpha;
      m.mg.b_trans = b_kcontig;
      if (mask_out && L.drop_thr) { m.mg.drop_thr = L.drop_thr; m.mg.drop_key = L.drop_key; m.mg.drop_cpr = drop_cpr(); }
      out->steps.push_back(m);
      return;
    }
    Step s;
    s.what = what;
    GemmDesc& d = s.d;
    d.dtype = L.dtype;
    d.alpha = alpha;
    d.bias = bias;
    if (mask_out && L.drop_thr) { d.drop_thr = L.drop_thr; d.drop_key = L.drop_key; d.drop_cpr = drop_cpr(); }
    d.a_strided = a_strided;
    d.b_kcontig = b_kcontig;
    d.M = M;
    d.N = N;
    d.nseg = K2 > 0 ? 2 : 1;
    d.A[0] = A.ptr; d.lda[0] = A.ld; d.B[0] = B.ptr; d.ldb[0] = B.ld; d.K[0] = K;
    if (K2 > 0) { d.A[1] = A2->ptr; d.lda[1] = A2->ld; d.B[1] = B2->ptr; d.ldb[1] = B2->ld; d.K[1] = K2; }
    d.C = const_cast<void*>(C.ptr);
    d.ldc = C.ld;
    if (D) { d.D = D->ptr; d.ldd = D->ld; d.has_addend = true; }
    if (b_is_w && L.w_int4) {
      d.b_int4 = true;
      d.Bscale = B.scales;
      d.ldbs = B.lds;
      s.plan = gemm_plan_int4(L.dtype, M, N, K, K2);
    } else {
      s.plan = gemm_plan(L.dtype, M, N, K, K2);
    }
    if (s.plan.partial_bytes > max_partial) max_partial = s.plan.partial_bytes;
    out->steps.push_back(s);
  }

  // Y = X W + (s X A) B (+ bias) in one launch of the tile GEMM's one-pass build: X is read once, T = s X A lives
  // in the kernel only
  void fused_forward(const char* what, Mat X, Mat W, Mat A, Mat B, Mat Y, const void* bias) {
    Step s;
    s.what = what;
    GemmDesc& d = s.d;
    d.dtype = L.dtype;
    d.bias = bias;
    d.M = L.n;
    d.N = L.o;
    d.nseg = 2;
    d.A[0] = X.ptr; d.lda[0] = X.ld; d.B[0] = W.ptr; d.ldb[0] = W.ld; d.K[0] = L.i;
    d.A[1] = nullptr; d.lda[1] = 0; d.B[1] = B.ptr; d.ldb[1] = B.ld; d.K[1] = L.r;
    d.C = const_cast<void*>(Y.ptr);
    d.ldc = Y.ld;
    d.LA = A.ptr;
    d.ldla = A.ld;
    d.t_alpha = scale();
    d.fuse_t = true;
    s.plan = gemm_plan_fused(L.dtype, L.n, L.o, L.i, L.r);
    out->steps.push_back(s);
  }

  // M = W + A B: the bandwidth-bound merge kernel when it applies (16-bit, r <= 128), else the tile
  // GEMM with W as the addend
  void merge(const char* what, Mat A, Mat B, Mat W, Mat M) {
    if (!merge_ok(L.dtype, L.r)) {
      gemm(what, 0, 0, L.i, L.o, L.r, A, B, M, &W, 0, nullptr, nullptr, false, scale());
      return;
    }
    Step s;
    s.what = what;
    s.is_merge = true;
    s.d.dtype = L.dtype;
    s.mg.W = W.ptr; s.mg.A = A.ptr; s.mg.B = B.ptr; s.mg.M = const_cast<void*>(M.ptr);
    s.mg.ldw = W.ld; s.mg.lda = A.ld; s.mg.ldb = B.ld; s.mg.ldm = M.ld;
    s.mg.I = L.i; s.mg.O = L.o; s.mg.R = L.r;
    s.mg.alpha = scale();
    s.mg.wcol = L.wcol;
    out->steps.push_back(s);
  }

  // Rank-r product C[M,N] = op(A) op(B) (N = r, or M = r with the output stored transposed) on the
  // streaming kernel; falls back to the tile GEMM when r is too large for it.
  struct Sk {
    int a_strided, b_kcontig;
    int64_t M, N, K;
    Mat A, B, C;
    bool scaled = false;  // this product carries the layer's LoRA scale
    bool mask_x = false;  // A is the layer input X: masked under LoRA dropout
  };
  SkinnyDesc to_skinny(const Sk& g) const {
    SkinnyDesc d;
    d.alpha = g.scaled ? scale() : 1.f;
    if (g.mask_x && L.drop_thr) { d.drop_thr = L.drop_thr; d.drop_key = L.drop_key; d.drop_cpr = drop_cpr(); }
    if (g.N <= g.M || g.a_strided == 0) {
      d.A = g.A.ptr; d.lda = g.A.ld; d.B = g.B.ptr; d.ldb = g.B.ld; d.C = const_cast<void*>(g.C.ptr); d.ldc = g.C.ld;
      d.M = g.M; d.N = g.N; d.K = g.K; d.a_strided = g.a_strided; d.b_kcontig = g.b_kcontig; d.trans_out = 0;
    } else {
      // short M (= r), long N, both operands stored [K, .]: compute C^T = op(B)^T op(A)
      d.A = g.B.ptr; d.lda = g.B.ld; d.B = g.A.ptr; d.ldb = g.A.ld; d.C = const_cast<void*>(g.C.ptr); d.ldc = g.C.ld;
      d.M = g.N; d.N = g.M; d.K = g.K; d.a_strided = 1; d.b_kcontig = 0; d.trans_out = 1;
    }
    return d;
  }
  bool sk_ok(const Sk& g) const {
    // operands are addressed with 31-bit byte offsets
    const int64_t esz = (int64_t)dtype_size(L.dtype);
    const int64_t a_rows = g.a_strided ? g.K : g.M, b_rows = g.b_kcontig ? g.N : g.K;
    if (a_rows * g.A.ld * esz >= (1LL << 31) || b_rows * g.B.ld * esz >= (1LL << 31)) return false;
    return sk_shape_ok(g);
  }
  static bool sk_shape_ok(const Sk& g) {
    const int64_t shortdim = (g.N <= g.M || g.a_strided == 0) ? g.N : g.M;
    // the transposed form needs both operands stored [K, .]
    if (!(g.N <= g.M || g.a_strided == 0) && g.b_kcontig) return false;
    return skinny_ok(shortdim);
  }
  void skinny(const char* what, const Sk& g) {
    if (!sk_ok(g)) {
      if (g.mask_x && L.drop_thr) { failed = true; return; }  // only the streaming kernel masks its A operand
      gemm(what, g.a_strided, g.b_kcontig, g.M, g.N, g.K, g.A, g.B, g.C, nullptr, 0, nullptr, nullptr, false,
           g.scaled ? scale() : 1.f);
      return;
    }
    Step s;
    s.what = what;
    s.nsk = 1;
    s.d.dtype = L.dtype;
    s.sk[0] = to_skinny(g);
    s.skplan = skinny_plan(L.dtype, 1, s.sk);
    if (s.skplan.partial_bytes > max_partial) max_partial = s.skplan.partial_bytes;
    out->steps.push_back(s);
  }
  void skinny2(const char* what, const char* what1, const Sk& g1, const char* what2, const Sk& g2) {
    bool pair = sk_ok(g1) && sk_ok(g2);
    SkinnyDesc d1, d2;
    if (pair) {
      d1 = to_skinny(g1);
      d2 = to_skinny(g2);
      // one launch serves both only if they stream the same way: same A layout, and the B layouts
      // in an order the kernel is built for ([N,K] first when they differ)
      if (d1.a_strided != d2.a_strided) pair = false;
      else if (d1.b_kcontig == 0 && d2.b_kcontig == 1) { SkinnyDesc t = d1; d1 = d2; d2 = t; }
      if (pair && d1.a_strided == 1 && (d1.b_kcontig || d2.b_kcontig)) pair = false;
    }
    if (!pair) {
      skinny(what1, g1);
      skinny(what2, g2);
      return;
    }
    Step s;
    s.what = what;
    s.nsk = 2;
    s.d.dtype = L.dtype;
    s.sk[0] = d1;
    s.sk[1] = d2;
    s.skplan = skinny_plan(L.dtype, 2, s.sk);
    if (s.skplan.partial_bytes > max_partial) max_partial = s.skplan.partial_bytes;
    out->steps.push_back(s);
  }

  void finish() {
    out->partial_offset = used;
    out->workspace_bytes = used + (max_partial + kAlign - 1) / kAlign * kAlign;
  }
};

// Z1 = dY B^T and Z2 = X A in one launch, then dA = X^T Z1 and dB = Z2^T dY in one launch
// (Algorithms 1 and 5 share these four statements).
void rank_r_pass(Builder& b, const BwdOperands& op, int64_t n, int64_t i, int64_t o, int64_t r, Mat Z1, Mat Z2,
                 bool need_Z1, bool need_Z2, bool dA, bool dB) {
  const Builder::Sk z1{0, 1, n, r, o, op.dY, op.B, Z1, true}, z2{0, 0, n, r, i, op.X, op.A, Z2, true, true};
  if (need_Z1 && need_Z2) b.skinny2("Z1 = dY B^T ; Z2 = X A", "Z1 = dY B^T", z1, "Z2 = X A", z2);
  else if (need_Z1) b.skinny("Z1 = dY B^T", z1);
  else if (need_Z2) b.skinny("Z2 = X A", z2);
  const Builder::Sk ga{1, 0, i, r, n, op.X, Z1, op.dA, false, true}, gb{1, 0, r, o, n, Z2, op.dY, op.dB};
  if (dA && dB) b.skinny2("dA = X^T Z1 ; dB = Z2^T dY", "dA = X^T Z1", ga, "dB = Z2^T dY", gb);
  else if (dA) b.skinny("dA = X^T Z1", ga);
  else if (dB) b.skinny("dB = Z2^T dY", gb);
}

// dA = Z2 B^T and dB = A^T Z2 (Algorithms 3 and 4), one launch when both are wanted
void z2_grads(Builder& b, const BwdOperands& op, int64_t i, int64_t o, int64_t r, Mat Z2, bool dA, bool dB) {
  const Builder::Sk ga{0, 1, i, r, o, Z2, op.B, op.dA, true}, gb{1, 0, r, o, i, op.A, Z2, op.dB, true};
  if (dA && dB) b.skinny2("dA = Z2 B^T ; dB = A^T Z2", "dA = Z2 B^T", ga, "dB = A^T Z2", gb);
  else if (dA) b.skinny("dA = Z2 B^T", ga);
  else if (dB) b.skinny("dB = A^T Z2", gb);
}

}  // namespace

bool build_forward(int variant, const LayerDims& L, const FwdOperands& op, void* ws_base, Schedule* out) {
  out->steps.clear();
  Builder b(L, ws_base, out);
  const int64_t n = L.n, i = L.i, o = L.o, r = L.r;
  if (L.wcol && (variant != 2 || !merge_ok(L.dtype, r) || L.w_int4 || L.drop_thr)) return false;  // see LayerDims::wcol
  switch (variant) {
    case 0: {  // default chain: T kept, one kernel per product
      b.skinny("T = X A", {0, 0, n, r, i, op.X, op.A, op.T, true, true});
      b.gemm("Y = X W", 0, 0, n, o, i, op.X, op.W, op.Y, nullptr, 0, nullptr, nullptr, true, 1.f, op.bias);
      b.gemm("Y += T B", 0, 0, n, o, r, op.T, op.B, op.Y, &op.Y);
      break;
    }
    case 3:  // forward1 in one pass over X; where that build does not apply, forward1's two launches
      if (r <= kFuseMaxR && !L.w_int4 && !L.drop_thr && !op.keep_T) {
        b.fused_forward("Y = X [W|A] ; Y += T B", op.X, op.W, op.A, op.B, op.Y, op.bias);
        break;
      }
      [[fallthrough]];
    case 1: {  // forward1: (XW) + ((XA)B), the sum folded into one contraction over [X|T]
      Mat T = op.keep_T ? op.T : b.scratch(n, r);
      b.skinny("T = X A", {0, 0, n, r, i, op.X, op.A, T, true, true});
      b.gemm("Y = [X|T] [W;B]", 0, 0, n, o, i, op.X, op.W, op.Y, nullptr, r, &T, &op.B, true, 1.f, op.bias);
      break;
    }
    case 2: {  // forward2: X (W + AB)
      if (L.w_int4 || L.drop_thr) return false;  // no dense buffer to merge AB into / no merged weight under dropout
      Mat M = op.keep_M ? op.M : b.scratch(i, o);
      b.merge("M = W + A B", op.A, op.B, op.W, M);
      b.gemm("Y = X M", 0, 0, n, o, i, op.X, M, op.Y, nullptr, 0, nullptr, nullptr, false, 1.f, op.bias);
      break;
    }
    default:
      return false;
  }
  b.finish();
  return !b.failed;
}

bool build_backward(int variant, const LayerDims& L, const BwdOperands& op, void* ws_base, Schedule* out) {
  out->steps.clear();
  Builder b(L, ws_base, out);
  const int64_t n = L.n, i = L.i, o = L.o, r = L.r;
  const bool dX = op.want_dX, dA = op.want_dA, dB = op.want_dB;
  if (L.drop_thr && variant > 1) return false;  // see LayerDims::drop_thr
  if (L.wcol && ((variant != 4 && variant != 5 && variant != 7 && variant != 8) || !merge_ok(L.dtype, r) || L.drop_thr))
    return false;  // see LayerDims::wcol
  switch (variant) {
    case 0: {  // backward of the default chain (uses the kept T = XA)
      Mat Z1 = b.scratch(n, r);
      // one kernel per product, as autograd would run them
      if (dA || dX) b.skinny("Z1 = dY B^T", {0, 1, n, r, o, op.dY, op.B, Z1, true});
      if (dB) b.skinny("dB = T^T dY", {1, 0, r, o, n, op.T, op.dY, op.dB});
      if (dA) b.skinny("dA = X^T Z1", {1, 0, i, r, n, op.X, Z1, op.dA, false, true});
      if (dX) {
        b.gemm("dX = dY W^T", 0, 1, n, i, o, op.dY, op.W, op.dX, nullptr, 0, nullptr, nullptr, true);
        b.gemm("dX += Z1 A^T", 0, 1, n, i, r, Z1, op.A, op.dX, &op.dX, 0, nullptr, nullptr, false, 1.f, nullptr, true);
      }
      break;
    }
    case 1: {  // Algorithm 1
      Mat Z1 = b.scratch(n, r), Z2 = op.have_T ? op.T : b.scratch(n, r);
      rank_r_pass(b, op, n, i, o, r, Z1, Z2, dA || dX, dB && !op.have_T, dA, dB);
      if (dX && L.drop_thr) {  // the mask sits between the two products: no concatenated contraction
        b.gemm("dX = dY W^T", 0, 1, n, i, o, op.dY, op.W, op.dX, nullptr, 0, nullptr, nullptr, true);
        b.gemm("dX += Z1 A^T", 0, 1, n, i, r, Z1, op.A, op.dX, &op.dX, 0, nullptr, nullptr, false, 1.f, nullptr, true);
      } else if (dX) {
        b.gemm("dX = [dY|Z1] [W^T;A^T]", 0, 1, n, i, o, op.dY, op.W, op.dX, nullptr, r, &Z1, &op.A, true);
      }
      break;
    }
    case 2: {  // Algorithm 2
      Mat Z1 = b.scratch(n, r), Z2 = b.scratch(i, o);
      if (dA || dX) b.skinny("Z1 = dY B^T", {0, 1, n, r, o, op.dY, op.B, Z1, true});
      if (dB) b.gemm("Z2 = X^T dY", 1, 0, i, o, n, op.X, op.dY, Z2);
      if (dA && dB)
        b.skinny2("dA = X^T Z1 ; dB = A^T Z2", "dA = X^T Z1", {1, 0, i, r, n, op.X, Z1, op.dA}, "dB = A^T Z2",
                  {1, 0, r, o, i, op.A, Z2, op.dB, true});
      else if (dA) b.skinny("dA = X^T Z1", {1, 0, i, r, n, op.X, Z1, op.dA});
      else if (dB) b.skinny("dB = A^T Z2", {1, 0, r, o, i, op.A, Z2, op.dB, true});
      if (dX) b.gemm("dX = [dY|Z1] [W^T;A^T]", 0, 1, n, i, o, op.dY, op.W, op.dX, nullptr, r, &Z1, &op.A, true);
      break;
    }
    case 3: {  // Algorithm 3
      Mat Z1 = b.scratch(n, r), Z2 = b.scratch(i, o);
      if (dX) b.skinny("Z1 = dY B^T", {0, 1, n, r, o, op.dY, op.B, Z1, true});
      if (dA || dB) b.gemm("Z2 = X^T dY", 1, 0, i, o, n, op.X, op.dY, Z2);
      z2_grads(b, op, i, o, r, Z2, dA, dB);
      if (dX) b.gemm("dX = [dY|Z1] [W^T;A^T]", 0, 1, n, i, o, op.dY, op.W, op.dX, nullptr, r, &Z1, &op.A, true);
      break;
    }
    case 4: {  // Algorithm 4
      if (L.w_int4) return false;
      Mat Z1 = op.have_M ? op.M : b.scratch(i, o), Z2 = b.scratch(i, o);
      if (dX && !op.have_M) b.merge("Z1 = W + A B", op.A, op.B, op.W, Z1);
      if (dA || dB) b.gemm("Z2 = X^T dY", 1, 0, i, o, n, op.X, op.dY, Z2);
      z2_grads(b, op, i, o, r, Z2, dA, dB);
      if (dX) b.gemm("dX = dY Z1^T", 0, 1, n, i, o, op.dY, Z1, op.dX);
      break;
    }
    case 5: {  // Algorithm 5
      if (L.w_int4) return false;
      Mat Z1 = b.scratch(n, r), Z2 = op.have_T ? op.T : b.scratch(n, r), Z3 = op.have_M ? op.M : b.scratch(i, o);
      if (dX && !op.have_M) b.merge("Z3 = W + A B", op.A, op.B, op.W, Z3);
      rank_r_pass(b, op, n, i, o, r, Z1, Z2, dA, dB && !op.have_T, dA, dB);
      if (dX) b.gemm("dX = dY Z3^T", 0, 1, n, i, o, op.dY, Z3, op.dX);
      break;
    }
    // Items 6-8 of the list of eight bracketings in Section 2 (the paper drops them because Table 1
    // never ranks them first; they are built from the same launches as Algorithms 1-5)
    case 6: {  // dA = (X^T dY) B^T, dB = (A^T X^T) dY, dX = dY W^T + (dY B^T) A^T
      Mat Z1 = b.scratch(n, r), T = op.have_T ? op.T : b.scratch(n, r), Z2 = b.scratch(i, o);
      const Builder::Sk z1{0, 1, n, r, o, op.dY, op.B, Z1, true}, t{0, 0, n, r, i, op.X, op.A, T, true};
      const bool need_T = dB && !op.have_T;
      if (dX && need_T) b.skinny2("Z1 = dY B^T ; T = X A", "Z1 = dY B^T", z1, "T = X A", t);
      else if (dX) b.skinny("Z1 = dY B^T", z1);
      else if (need_T) b.skinny("T = X A", t);
      if (dA) b.gemm("Z2 = X^T dY", 1, 0, i, o, n, op.X, op.dY, Z2);
      if (dA) b.skinny("dA = Z2 B^T", {0, 1, i, r, o, Z2, op.B, op.dA, true});
      if (dB) b.skinny("dB = T^T dY", {1, 0, r, o, n, T, op.dY, op.dB});
      if (dX) b.gemm("dX = [dY|Z1] [W^T;A^T]", 0, 1, n, i, o, op.dY, op.W, op.dX, nullptr, r, &Z1, &op.A, true);
      break;
    }
    case 7: {  // dA = (X^T dY) B^T, dB = (A^T X^T) dY, dX = dY (W^T + B^T A^T)
      if (L.w_int4) return false;
      Mat T = op.have_T ? op.T : b.scratch(n, r), Z2 = b.scratch(i, o), M = op.have_M ? op.M : b.scratch(i, o);
      if (dX && !op.have_M) b.merge("M = W + A B", op.A, op.B, op.W, M);
      if (dB && !op.have_T) b.skinny("T = X A", {0, 0, n, r, i, op.X, op.A, T, true});
      if (dA) b.gemm("Z2 = X^T dY", 1, 0, i, o, n, op.X, op.dY, Z2);
      if (dA) b.skinny("dA = Z2 B^T", {0, 1, i, r, o, Z2, op.B, op.dA, true});
      if (dB) b.skinny("dB = T^T dY", {1, 0, r, o, n, T, op.dY, op.dB});
      if (dX) b.gemm("dX = dY M^T", 0, 1, n, i, o, op.dY, M, op.dX);
      break;
    }
    case 8: {  // dA = X^T (dY B^T), dB = A^T (X^T dY), dX = dY (W^T + B^T A^T)
      if (L.w_int4) return false;
      Mat Z1 = b.scratch(n, r), Z2 = b.scratch(i, o), M = op.have_M ? op.M : b.scratch(i, o);
      if (dX && !op.have_M) b.merge("M = W + A B", op.A, op.B, op.W, M);
      if (dA) b.skinny("Z1 = dY B^T", {0, 1, n, r, o, op.dY, op.B, Z1, true});
      if (dB) b.gemm("Z2 = X^T dY", 1, 0, i, o, n, op.X, op.dY, Z2);
      if (dA && dB)
        b.skinny2("dA = X^T Z1 ; dB = A^T Z2", "dA = X^T Z1", {1, 0, i, r, n, op.X, Z1, op.dA}, "dB = A^T Z2",
                  {1, 0, r, o, i, op.A, Z2, op.dB, true});
      else if (dA) b.skinny("dA = X^T Z1", {1, 0, i, r, n, op.X, Z1, op.dA});
      else if (dB) b.skinny("dB = A^T Z2", {1, 0, r, o, i, op.A, Z2, op.dB, true});
      if (dX) b.gemm("dX = dY M^T", 0, 1, n, i, o, op.dY, M, op.dX);
      break;
    }
    default:
      return false;
  }
  b.finish();
  return !b.failed;
}

}  // namespace rl
