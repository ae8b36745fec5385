/*
 * fp64 CPU oracle for the LoRA-augmented linear layer of RunLoRA (arxiv 2312.03415).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the checker the GPU library is compared against.
 * Nothing in the product path may include, link or call it; it shares no code, header, table
 * or helper with the HIP kernels.  Only tests, the smoke check and the bench's cpu_baseline
 * leg load it.
 *
 * Notation follows the paper (Section 2, Table 1 caption): n = b*s tokens, i = d_in,
 * o = d_out, r = LoRA rank.  All matrices are dense row-major fp64:
 *   X [n,i]  W [i,o]  A [i,r]  B [r,o]  Y,dY [n,o]  dX [n,i]  dA [i,r]  dB [r,o].
 * W is frozen: no dW is produced (Eq. 3 lists dA, dB, dX only).
 *
 * Two kinds of function live here:
 *   - orc_reference_*: the plain definitions, Eq. 1 and Eq. 3, written out.
 *   - orc_forward / orc_backward: every computation graph the paper lists, step by step in
 *     the paper's order (forward variants 1-2 of Section 2; the eight backward bracketings of
 *     Section 2; Algorithms 1-5 give the step order of backward1..5), plus the "default chain"
 *     (forward of Eq. 1 that keeps XA for the backward, and the backward autograd derives
 *     from it).
 *
 * Every matrix product goes through one naive routine, orc_matmul, which adds 2*m*k*n to a
 * counter so that the per-variant totals can be checked against Table 1.  Element-wise
 * additions are not counted (Table 1 counts none: forward1 carries no n*o term).
 * Intermediates are never rounded.
 *
 * Pins (tests/test_oracle_pins.py): Table 1 closed forms, agreement of all variants,
 * central finite differences, B=0 / A=0 special cases, the dense layer W' = W+AB computed by a
 * library matmul, linearity, int4 group dequantisation against a Kronecker-product layout.
 */
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static long long g_flops = 0;

void orc_flops_reset(void) { g_flops = 0; }
long long orc_flops_get(void) { return g_flops; }
int orc_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/*
 * C[m,n] = op(P) * op(Q)  (+ C if accumulate), fp64, naive.
 * op(P) is m x k: P is stored [m,k] (ta=0) or [k,m] (ta=1); op(Q) is k x n: Q stored [k,n]
 * (tb=0) or [n,k] (tb=1).  Leading dimensions are the stored row lengths.
 * Loop order row / contraction / column; rows are shared out over the host threads.
 */
void orc_matmul(int ta, int tb, int64_t m, int64_t n, int64_t k, const double* P, int64_t ldp,
                const double* Q, int64_t ldq, double* C, int64_t ldc, int accumulate) {
  g_flops += 2LL * m * n * k;
#pragma omp parallel for schedule(static)
  for (int64_t a = 0; a < m; ++a) {
    double* crow = C + a * ldc;
    if (!accumulate)
      for (int64_t c = 0; c < n; ++c) crow[c] = 0.0;
    for (int64_t q = 0; q < k; ++q) {
      const double p = ta ? P[q * ldp + a] : P[a * ldp + q];
      if (!tb) {
        const double* qrow = Q + q * ldq;
        for (int64_t c = 0; c < n; ++c) crow[c] += p * qrow[c];
      } else {
        for (int64_t c = 0; c < n; ++c) crow[c] += p * Q[c * ldq + q];
      }
    }
  }
}

static double* alloc_mat(int64_t rows, int64_t cols) {
  size_t cnt = (size_t)(rows > 0 ? rows : 1) * (size_t)(cols > 0 ? cols : 1);
  return (double*)malloc(cnt * sizeof(double));
}

/* dst[rows,cols] = P + Q (element-wise; not counted, as in Table 1). */
static void add_mat(int64_t rows, int64_t cols, const double* P, const double* Q, double* dst) {
#pragma omp parallel for schedule(static)
  for (int64_t a = 0; a < rows; ++a)
    for (int64_t c = 0; c < cols; ++c) dst[a * cols + c] = P[a * cols + c] + Q[a * cols + c];
}

/* ---- the plain definitions ------------------------------------------------------------ */

/* Eq. 1:  Y = X W + (X A) B. */
void orc_reference_forward(int64_t n, int64_t i, int64_t o, int64_t r, const double* X,
                           const double* W, const double* A, const double* B, double* Y) {
  double* XA = alloc_mat(n, r);
  orc_matmul(0, 0, n, o, i, X, i, W, o, Y, o, 0);
  orc_matmul(0, 0, n, r, i, X, i, A, r, XA, r, 0);
  orc_matmul(0, 0, n, o, r, XA, r, B, o, Y, o, 1);
  free(XA);
}

/* Eq. 3:  dA = X^T dY B^T,  dB = A^T X^T dY,  dX = dY W^T + dY B^T A^T  (left to right). */
void orc_reference_backward(int64_t n, int64_t i, int64_t o, int64_t r, const double* X,
                            const double* W, const double* A, const double* B, const double* dY,
                            double* dX, double* dA, double* dB) {
  double* XtdY = alloc_mat(i, o);
  double* dYBt = alloc_mat(n, r);
  orc_matmul(1, 0, i, o, n, X, i, dY, o, XtdY, o, 0);   /* X^T dY            */
  orc_matmul(0, 1, i, r, o, XtdY, o, B, o, dA, r, 0);    /* (X^T dY) B^T      */
  orc_matmul(1, 0, r, o, i, A, r, XtdY, o, dB, o, 0);    /* A^T (X^T dY)      */
  orc_matmul(0, 1, n, i, o, dY, o, W, o, dX, i, 0);      /* dY W^T            */
  orc_matmul(0, 1, n, r, o, dY, o, B, o, dYBt, r, 0);    /* dY B^T            */
  orc_matmul(0, 1, n, i, r, dYBt, r, A, r, dX, i, 1);    /* + (dY B^T) A^T    */
  free(XtdY);
  free(dYBt);
}

/* ---- forward computation graphs ------------------------------------------------------- */

/*
 * variant 0: default chain.  T = XA is kept for the backward (T_saved [n,r] must be given),
 *            Y = XW, then Y += T B.  Same products as forward1.
 * variant 1: forward1, Y = (XW) + ((XA)B); XA is not kept (Section 2).
 * variant 2: forward2, Y = X (W + AB)  (Eq. 2).
 * Returns 0, or -1 for an unknown variant / missing T_saved.
 */
int orc_forward(int variant, int64_t n, int64_t i, int64_t o, int64_t r, const double* X,
                const double* W, const double* A, const double* B, double* Y, double* T_saved) {
  if (variant == 0) {
    if (!T_saved) return -1;
    orc_matmul(0, 0, n, r, i, X, i, A, r, T_saved, r, 0);
    orc_matmul(0, 0, n, o, i, X, i, W, o, Y, o, 0);
    orc_matmul(0, 0, n, o, r, T_saved, r, B, o, Y, o, 1);
    return 0;
  }
  if (variant == 1) {
    double* XA = alloc_mat(n, r);
    double* XAB = alloc_mat(n, o);
    double* XW = alloc_mat(n, o);
    orc_matmul(0, 0, n, o, i, X, i, W, o, XW, o, 0);
    orc_matmul(0, 0, n, r, i, X, i, A, r, XA, r, 0);
    orc_matmul(0, 0, n, o, r, XA, r, B, o, XAB, o, 0);
    add_mat(n, o, XW, XAB, Y);
    free(XA);
    free(XAB);
    free(XW);
    return 0;
  }
  if (variant == 2) {
    double* AB = alloc_mat(i, o);
    double* M = alloc_mat(i, o);
    orc_matmul(0, 0, i, o, r, A, r, B, o, AB, o, 0);
    add_mat(i, o, W, AB, M);
    orc_matmul(0, 0, n, o, i, X, i, M, o, Y, o, 0);
    free(AB);
    free(M);
    return 0;
  }
  return -1;
}

/* ---- backward computation graphs ------------------------------------------------------ */

/* the three ways each gradient is bracketed in Section 2's list of eight */
static void dA_outer(int64_t n, int64_t i, int64_t o, int64_t r, const double* X, const double* dY,
                     const double* B, double* dA) { /* X^T (dY B^T) */
  double* Z = alloc_mat(n, r);
  orc_matmul(0, 1, n, r, o, dY, o, B, o, Z, r, 0);
  orc_matmul(1, 0, i, r, n, X, i, Z, r, dA, r, 0);
  free(Z);
}
static void dA_inner(int64_t n, int64_t i, int64_t o, int64_t r, const double* X, const double* dY,
                     const double* B, double* dA) { /* (X^T dY) B^T */
  double* Z = alloc_mat(i, o);
  orc_matmul(1, 0, i, o, n, X, i, dY, o, Z, o, 0);
  orc_matmul(0, 1, i, r, o, Z, o, B, o, dA, r, 0);
  free(Z);
}
static void dB_outer(int64_t n, int64_t i, int64_t o, int64_t r, const double* X, const double* dY,
                     const double* A, double* dB) { /* (A^T X^T) dY */
  double* Z = alloc_mat(r, n);
  orc_matmul(1, 1, r, n, i, A, r, X, i, Z, n, 0);
  orc_matmul(0, 0, r, o, n, Z, n, dY, o, dB, o, 0);
  free(Z);
}
static void dB_inner(int64_t n, int64_t i, int64_t o, int64_t r, const double* X, const double* dY,
                     const double* A, double* dB) { /* A^T (X^T dY) */
  double* Z = alloc_mat(i, o);
  orc_matmul(1, 0, i, o, n, X, i, dY, o, Z, o, 0);
  orc_matmul(1, 0, r, o, i, A, r, Z, o, dB, o, 0);
  free(Z);
}
static void dX_split(int64_t n, int64_t i, int64_t o, int64_t r, const double* dY, const double* W,
                     const double* A, const double* B, double* dX) { /* dY W^T + (dY B^T) A^T */
  double* Z = alloc_mat(n, r);
  orc_matmul(0, 1, n, i, o, dY, o, W, o, dX, i, 0);
  orc_matmul(0, 1, n, r, o, dY, o, B, o, Z, r, 0);
  orc_matmul(0, 1, n, i, r, Z, r, A, r, dX, i, 1);
  free(Z);
}
static void dX_merged(int64_t n, int64_t i, int64_t o, int64_t r, const double* dY, const double* W,
                      const double* A, const double* B, double* dX) { /* dY (W^T + B^T A^T) */
  double* AB = alloc_mat(i, o);
  double* M = alloc_mat(i, o);
  orc_matmul(0, 0, i, o, r, A, r, B, o, AB, o, 0);
  add_mat(i, o, W, AB, M);
  orc_matmul(0, 1, n, i, o, dY, o, M, o, dX, i, 0);
  free(AB);
  free(M);
}

/*
 * variant 0   : backward of the default chain.  Needs T_saved = XA from forward variant 0.
 *               Z1 = dY B^T; dB = T^T dY; dA = X^T Z1; dX = dY W^T; dX += Z1 A^T.
 * variant 1..5: Algorithms 1-5, statement by statement (shared intermediates computed once,
 *               as the algorithms do).
 * variant 6..8: items 6-8 of the list of eight bracketings (no algorithm is printed for them;
 *               each gradient is evaluated on its own, in the bracketing the item shows).
 * Returns 0, or -1 for an unknown variant / missing T_saved.
 */
int orc_backward(int variant, int64_t n, int64_t i, int64_t o, int64_t r, const double* X,
                 const double* W, const double* A, const double* B, const double* dY,
                 const double* T_saved, double* dX, double* dA, double* dB) {
  switch (variant) {
    case 0: {
      if (!T_saved) return -1;
      double* Z1 = alloc_mat(n, r);
      orc_matmul(0, 1, n, r, o, dY, o, B, o, Z1, r, 0);
      orc_matmul(1, 0, r, o, n, T_saved, r, dY, o, dB, o, 0);
      orc_matmul(1, 0, i, r, n, X, i, Z1, r, dA, r, 0);
      orc_matmul(0, 1, n, i, o, dY, o, W, o, dX, i, 0);
      orc_matmul(0, 1, n, i, r, Z1, r, A, r, dX, i, 1);
      free(Z1);
      return 0;
    }
    case 1: { /* Algorithm 1 */
      double* Z1 = alloc_mat(n, r);
      double* Z2 = alloc_mat(n, r);
      orc_matmul(0, 1, n, r, o, dY, o, B, o, Z1, r, 0);  /* Z1 = dY B^T          */
      orc_matmul(0, 0, n, r, i, X, i, A, r, Z2, r, 0);   /* Z2 = X A             */
      orc_matmul(1, 0, i, r, n, X, i, Z1, r, dA, r, 0);  /* dA = X^T Z1          */
      orc_matmul(1, 0, r, o, n, Z2, r, dY, o, dB, o, 0); /* dB = Z2^T dY         */
      orc_matmul(0, 1, n, i, o, dY, o, W, o, dX, i, 0);  /* dX = dY W^T          */
      orc_matmul(0, 1, n, i, r, Z1, r, A, r, dX, i, 1);  /*      + Z1 A^T        */
      free(Z1);
      free(Z2);
      return 0;
    }
    case 2: { /* Algorithm 2 */
      double* Z1 = alloc_mat(n, r);
      double* Z2 = alloc_mat(i, o);
      orc_matmul(0, 1, n, r, o, dY, o, B, o, Z1, r, 0);  /* Z1 = dY B^T          */
      orc_matmul(1, 0, i, o, n, X, i, dY, o, Z2, o, 0);  /* Z2 = X^T dY          */
      orc_matmul(1, 0, i, r, n, X, i, Z1, r, dA, r, 0);  /* dA = X^T Z1          */
      orc_matmul(1, 0, r, o, i, A, r, Z2, o, dB, o, 0);  /* dB = A^T Z2          */
      orc_matmul(0, 1, n, i, o, dY, o, W, o, dX, i, 0);
      orc_matmul(0, 1, n, i, r, Z1, r, A, r, dX, i, 1);  /* dX = dY W^T + Z1 A^T */
      free(Z1);
      free(Z2);
      return 0;
    }
    case 3: { /* Algorithm 3 */
      double* Z1 = alloc_mat(n, r);
      double* Z2 = alloc_mat(i, o);
      orc_matmul(0, 1, n, r, o, dY, o, B, o, Z1, r, 0);  /* Z1 = dY B^T          */
      orc_matmul(1, 0, i, o, n, X, i, dY, o, Z2, o, 0);  /* Z2 = X^T dY          */
      orc_matmul(0, 1, i, r, o, Z2, o, B, o, dA, r, 0);  /* dA = Z2 B^T          */
      orc_matmul(1, 0, r, o, i, A, r, Z2, o, dB, o, 0);  /* dB = A^T Z2          */
      orc_matmul(0, 1, n, i, o, dY, o, W, o, dX, i, 0);
      orc_matmul(0, 1, n, i, r, Z1, r, A, r, dX, i, 1);  /* dX = dY W^T + Z1 A^T */
      free(Z1);
      free(Z2);
      return 0;
    }
    case 4: { /* Algorithm 4 */
      double* AB = alloc_mat(i, o);
      double* Z1 = alloc_mat(i, o);
      double* Z2 = alloc_mat(i, o);
      orc_matmul(0, 0, i, o, r, A, r, B, o, AB, o, 0);
      add_mat(i, o, W, AB, Z1);                           /* Z1 = W + A B         */
      orc_matmul(1, 0, i, o, n, X, i, dY, o, Z2, o, 0);   /* Z2 = X^T dY          */
      orc_matmul(0, 1, i, r, o, Z2, o, B, o, dA, r, 0);   /* dA = Z2 B^T          */
      orc_matmul(1, 0, r, o, i, A, r, Z2, o, dB, o, 0);   /* dB = A^T Z2          */
      orc_matmul(0, 1, n, i, o, dY, o, Z1, o, dX, i, 0);  /* dX = dY Z1^T         */
      free(AB);
      free(Z1);
      free(Z2);
      return 0;
    }
    case 5: { /* Algorithm 5 */
      double* Z1 = alloc_mat(n, r);
      double* Z2 = alloc_mat(n, r);
      double* AB = alloc_mat(i, o);
      double* Z3 = alloc_mat(i, o);
      orc_matmul(0, 1, n, r, o, dY, o, B, o, Z1, r, 0);   /* Z1 = dY B^T          */
      orc_matmul(0, 0, n, r, i, X, i, A, r, Z2, r, 0);    /* Z2 = X A             */
      orc_matmul(0, 0, i, o, r, A, r, B, o, AB, o, 0);
      add_mat(i, o, W, AB, Z3);                           /* Z3 = W + A B         */
      orc_matmul(1, 0, i, r, n, X, i, Z1, r, dA, r, 0);   /* dA = X^T Z1          */
      orc_matmul(1, 0, r, o, n, Z2, r, dY, o, dB, o, 0);  /* dB = Z2^T dY         */
      orc_matmul(0, 1, n, i, o, dY, o, Z3, o, dX, i, 0);  /* dX = dY Z3^T         */
      free(Z1);
      free(Z2);
      free(AB);
      free(Z3);
      return 0;
    }
    case 6: /* item 6: dA=(X^T dY)B^T, dB=(A^T X^T)dY, dX=dY W^T+(dY B^T)A^T */
      dA_inner(n, i, o, r, X, dY, B, dA);
      dB_outer(n, i, o, r, X, dY, A, dB);
      dX_split(n, i, o, r, dY, W, A, B, dX);
      return 0;
    case 7: /* item 7: dA=(X^T dY)B^T, dB=(A^T X^T)dY, dX=dY(W^T+B^T A^T) */
      dA_inner(n, i, o, r, X, dY, B, dA);
      dB_outer(n, i, o, r, X, dY, A, dB);
      dX_merged(n, i, o, r, dY, W, A, B, dX);
      return 0;
    case 8: /* item 8: dA=X^T(dY B^T), dB=A^T(X^T dY), dX=dY(W^T+B^T A^T) */
      dA_outer(n, i, o, r, X, dY, B, dA);
      dB_inner(n, i, o, r, X, dY, A, dB);
      dX_merged(n, i, o, r, dY, W, A, B, dX);
      return 0;
    default:
      return -1;
  }
}

/*
 * Frozen weight held as symmetric 4-bit integers (QLoRA-style use mentioned in Section 1; the
 * format itself is this workload's: groups of `group` consecutive rows of W along d_in share
 * one scale per column).  W[k,j] = q[k,j] * scale[k / group, j], q in [-7,7] given unpacked,
 * scale [ceil(i/group), o] given as the fp64 value of the stored half-precision number.
 */
void orc_dequant_int4(int64_t i, int64_t o, int64_t group, const int8_t* q, const double* scale,
                      double* W) {
#pragma omp parallel for schedule(static)
  for (int64_t k = 0; k < i; ++k)
    for (int64_t j = 0; j < o; ++j) W[k * o + j] = (double)q[k * o + j] * scale[(k / group) * o + j];
}

/* Rows [row0, row0+rows) of Y and dX only (rows of X and dY are independent in Eq. 1 and in the
 * dX line of Eq. 3): used to check sampled rows of layers too large to run in full. */
void orc_reference_rows(int64_t rows, int64_t i, int64_t o, int64_t r, const double* Xrows,
                        const double* dYrows, const double* W, const double* A, const double* B,
                        double* Yrows, double* dXrows) {
  double* XA = alloc_mat(rows, r);
  double* dYBt = alloc_mat(rows, r);
  orc_matmul(0, 0, rows, o, i, Xrows, i, W, o, Yrows, o, 0);
  orc_matmul(0, 0, rows, r, i, Xrows, i, A, r, XA, r, 0);
  orc_matmul(0, 0, rows, o, r, XA, r, B, o, Yrows, o, 1);
  orc_matmul(0, 1, rows, i, o, dYrows, o, W, o, dXrows, i, 0);
  orc_matmul(0, 1, rows, r, o, dYrows, o, B, o, dYBt, r, 0);
  orc_matmul(0, 1, rows, i, r, dYBt, r, A, r, dXrows, i, 1);
  free(XA);
  free(dYBt);
}
