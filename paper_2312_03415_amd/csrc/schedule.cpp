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

  Builder(const LayerDims& l, void* ws, Schedule* o) : L(l), base(static_cast<char*>(ws)), out(o) {}

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
  void gemm(const char* what, int a_strided, int b_kcontig, int64_t M, int64_t N, int64_t K, Mat A, Mat B,
            Mat C, const Mat* D = nullptr, int64_t K2 = 0, const Mat* A2 = nullptr, const Mat* B2 = nullptr) {
    Step s;
    s.what = what;
    GemmDesc& d = s.d;
    d.dtype = L.dtype;
    d.a_strided = a_strided;
    d.b_kcontig = b_kcontig;
    d.M = M;
    d.N = N;
    d.nseg = K2 > 0 ? 2 : 1;
    d.A[0] = A.ptr; d.lda[0] = A.ld; d.B[0] = B.ptr; d.ldb[0] = B.ld; d.K[0] = K;
    if (K2 > 0) { d.A[1] = A2->ptr; d.lda[1] = A2->ld; d.B[1] = B2->ptr; d.ldb[1] = B2->ld; d.K[1] = K2; }
    d.C = const_cast<void*>(C.ptr);
    d.ldc = C.ld;
    if (D) { d.D = D->ptr; d.ldd = D->ld; }
    s.plan = gemm_plan(L.dtype, M, N, K, K2);
    if (s.plan.partial_bytes > max_partial) max_partial = s.plan.partial_bytes;
    out->steps.push_back(s);
  }

  void finish() {
    out->partial_offset = used;
    out->workspace_bytes = used + (max_partial + kAlign - 1) / kAlign * kAlign;
  }
};

}  // namespace

bool build_forward(int variant, const LayerDims& L, const FwdOperands& op, void* ws_base, Schedule* out) {
  out->steps.clear();
  Builder b(L, ws_base, out);
  const int64_t n = L.n, i = L.i, o = L.o, r = L.r;
  switch (variant) {
    case 0: {  // default chain: T kept, one kernel per product
      b.gemm("T = X A", 0, 0, n, r, i, op.X, op.A, op.T);
      b.gemm("Y = X W", 0, 0, n, o, i, op.X, op.W, op.Y);
      b.gemm("Y += T B", 0, 0, n, o, r, op.T, op.B, op.Y, &op.Y);
      break;
    }
    case 1: {  // forward1: (XW) + ((XA)B), the sum folded into one contraction over [X|T]
      Mat T = b.scratch(n, r);
      b.gemm("T = X A", 0, 0, n, r, i, op.X, op.A, T);
      b.gemm("Y = [X|T] [W;B]", 0, 0, n, o, i, op.X, op.W, op.Y, nullptr, r, &T, &op.B);
      break;
    }
    case 2: {  // forward2: X (W + AB)
      Mat M = b.scratch(i, o);
      b.gemm("M = W + A B", 0, 0, i, o, r, op.A, op.B, M, &op.W);
      b.gemm("Y = X M", 0, 0, n, o, i, op.X, M, op.Y);
      break;
    }
    default:
      return false;
  }
  b.finish();
  return true;
}

bool build_backward(int variant, const LayerDims& L, const BwdOperands& op, void* ws_base, Schedule* out) {
  out->steps.clear();
  Builder b(L, ws_base, out);
  const int64_t n = L.n, i = L.i, o = L.o, r = L.r;
  const bool dX = op.want_dX, dA = op.want_dA, dB = op.want_dB;
  switch (variant) {
    case 0: {  // backward of the default chain (uses the kept T = XA)
      Mat Z1 = b.scratch(n, r);
      if (dA || dX) b.gemm("Z1 = dY B^T", 0, 1, n, r, o, op.dY, op.B, Z1);
      if (dB) b.gemm("dB = T^T dY", 1, 0, r, o, n, op.T, op.dY, op.dB);
      if (dA) b.gemm("dA = X^T Z1", 1, 0, i, r, n, op.X, Z1, op.dA);
      if (dX) {
        b.gemm("dX = dY W^T", 0, 1, n, i, o, op.dY, op.W, op.dX);
        b.gemm("dX += Z1 A^T", 0, 1, n, i, r, Z1, op.A, op.dX, &op.dX);
      }
      break;
    }
    case 1: {  // Algorithm 1
      Mat Z1 = b.scratch(n, r), Z2 = b.scratch(n, r);
      if (dA || dX) b.gemm("Z1 = dY B^T", 0, 1, n, r, o, op.dY, op.B, Z1);
      if (dB) b.gemm("Z2 = X A", 0, 0, n, r, i, op.X, op.A, Z2);
      if (dA) b.gemm("dA = X^T Z1", 1, 0, i, r, n, op.X, Z1, op.dA);
      if (dB) b.gemm("dB = Z2^T dY", 1, 0, r, o, n, Z2, op.dY, op.dB);
      if (dX) b.gemm("dX = [dY|Z1] [W^T;A^T]", 0, 1, n, i, o, op.dY, op.W, op.dX, nullptr, r, &Z1, &op.A);
      break;
    }
    case 2: {  // Algorithm 2
      Mat Z1 = b.scratch(n, r), Z2 = b.scratch(i, o);
      if (dA || dX) b.gemm("Z1 = dY B^T", 0, 1, n, r, o, op.dY, op.B, Z1);
      if (dB) b.gemm("Z2 = X^T dY", 1, 0, i, o, n, op.X, op.dY, Z2);
      if (dA) b.gemm("dA = X^T Z1", 1, 0, i, r, n, op.X, Z1, op.dA);
      if (dB) b.gemm("dB = A^T Z2", 1, 0, r, o, i, op.A, Z2, op.dB);
      if (dX) b.gemm("dX = [dY|Z1] [W^T;A^T]", 0, 1, n, i, o, op.dY, op.W, op.dX, nullptr, r, &Z1, &op.A);
      break;
    }
    case 3: {  // Algorithm 3
      Mat Z1 = b.scratch(n, r), Z2 = b.scratch(i, o);
      if (dX) b.gemm("Z1 = dY B^T", 0, 1, n, r, o, op.dY, op.B, Z1);
      if (dA || dB) b.gemm("Z2 = X^T dY", 1, 0, i, o, n, op.X, op.dY, Z2);
      if (dA) b.gemm("dA = Z2 B^T", 0, 1, i, r, o, Z2, op.B, op.dA);
      if (dB) b.gemm("dB = A^T Z2", 1, 0, r, o, i, op.A, Z2, op.dB);
      if (dX) b.gemm("dX = [dY|Z1] [W^T;A^T]", 0, 1, n, i, o, op.dY, op.W, op.dX, nullptr, r, &Z1, &op.A);
      break;
    }
    case 4: {  // Algorithm 4
      Mat Z1 = b.scratch(i, o), Z2 = b.scratch(i, o);
      if (dX) b.gemm("Z1 = W + A B", 0, 0, i, o, r, op.A, op.B, Z1, &op.W);
      if (dA || dB) b.gemm("Z2 = X^T dY", 1, 0, i, o, n, op.X, op.dY, Z2);
      if (dA) b.gemm("dA = Z2 B^T", 0, 1, i, r, o, Z2, op.B, op.dA);
      if (dB) b.gemm("dB = A^T Z2", 1, 0, r, o, i, op.A, Z2, op.dB);
      if (dX) b.gemm("dX = dY Z1^T", 0, 1, n, i, o, op.dY, Z1, op.dX);
      break;
    }
    case 5: {  // Algorithm 5
      Mat Z1 = b.scratch(n, r), Z2 = b.scratch(n, r), Z3 = b.scratch(i, o);
      if (dA) b.gemm("Z1 = dY B^T", 0, 1, n, r, o, op.dY, op.B, Z1);
      if (dB) b.gemm("Z2 = X A", 0, 0, n, r, i, op.X, op.A, Z2);
      if (dX) b.gemm("Z3 = W + A B", 0, 0, i, o, r, op.A, op.B, Z3, &op.W);
      if (dA) b.gemm("dA = X^T Z1", 1, 0, i, r, n, op.X, Z1, op.dA);
      if (dB) b.gemm("dB = Z2^T dY", 1, 0, r, o, n, Z2, op.dY, op.dB);
      if (dX) b.gemm("dX = dY Z3^T", 0, 1, n, i, o, op.dY, Z3, op.dX);
      break;
    }
    default:
      return false;
  }
  b.finish();
  return true;
}

}  // namespace rl
