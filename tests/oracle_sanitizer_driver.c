/*
 * Driver for a sanitizer build of the CPU oracle (tests/test_oracle_sanitizers.py compiles this file together with
 * oracle/runlora_oracle.c under -fsanitize=address,undefined and runs it).  Every buffer is a heap block of exactly
 * the size its matrix needs, so an out-of-range index inside the oracle is an AddressSanitizer report; shapes are
 * ragged and small.  Two pins run through the instrumented code: a hand-worked 2 x 2 layer (Eq. 1 of arxiv
 * 2312.03415) and the agreement of every forward / backward computation graph of Section 2 with the plain definitions
 * (Eq. 1, Eq. 3).  Exit status 0 and a last line "ok" mean no report and no mismatch.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

void orc_reference_forward(int64_t n, int64_t i, int64_t o, int64_t r, const double* X, const double* W, const double* A,
                           const double* B, double* Y);
void orc_reference_backward(int64_t n, int64_t i, int64_t o, int64_t r, const double* X, const double* W, const double* A,
                            const double* B, const double* dY, double* dX, double* dA, double* dB);
int orc_forward(int variant, int64_t n, int64_t i, int64_t o, int64_t r, const double* X, const double* W, const double* A,
                const double* B, double* Y, double* T_saved);
int orc_backward(int variant, int64_t n, int64_t i, int64_t o, int64_t r, const double* X, const double* W, const double* A,
                 const double* B, const double* dY, const double* T_saved, double* dX, double* dA, double* dB);
void orc_reference_rows(int64_t rows, int64_t i, int64_t o, int64_t r, const double* Xrows, const double* dYrows,
                        const double* W, const double* A, const double* B, double* Yrows, double* dXrows);
void orc_dequant_int4(int64_t i, int64_t o, int64_t group, const int8_t* q, const double* scale, double* W);

static uint64_t g_state = 88172645463325252ull;
static double next_value(void) { /* xorshift64, mapped to (-1, 1) */
  g_state ^= g_state << 13;
  g_state ^= g_state >> 7;
  g_state ^= g_state << 17;
  return (double)(g_state >> 11) / 9007199254740992.0 * 2.0 - 1.0;
}
static double* filled(int64_t count) {
  double* p = (double*)malloc((size_t)count * sizeof(double));
  for (int64_t k = 0; k < count; ++k) p[k] = next_value();
  return p;
}
static double* blank(int64_t count) { return (double*)malloc((size_t)count * sizeof(double)); }
static double max_diff(const double* a, const double* b, int64_t count) {
  double m = 0.0;
  for (int64_t k = 0; k < count; ++k) m = fmax(m, fabs(a[k] - b[k]));
  return m;
}

int main(void) {
  int bad = 0;
  { /* hand-worked layer: X = [1 2; 3 4], W = identity, A = [1; 1], B = [1 -1]  =>  Y = X + (XA)B = [4 -1; 10 -3] */
    double *X = blank(4), *W = blank(4), *A = blank(2), *B = blank(2), *Y = blank(4);
    X[0] = 1; X[1] = 2; X[2] = 3; X[3] = 4;
    W[0] = 1; W[1] = 0; W[2] = 0; W[3] = 1;
    A[0] = 1; A[1] = 1;
    B[0] = 1; B[1] = -1;
    const double want[4] = {4, -1, 10, -3};
    for (int v = 1; v <= 2; ++v) {
      if (orc_forward(v, 2, 2, 2, 1, X, W, A, B, Y, NULL) != 0 || max_diff(Y, want, 4) != 0.0) { printf("hand-worked layer: forward%d wrong\n", v); bad = 1; }
    }
    orc_reference_forward(2, 2, 2, 1, X, W, A, B, Y);
    if (max_diff(Y, want, 4) != 0.0) { printf("hand-worked layer: Eq. 1 wrong\n"); bad = 1; }
    free(X); free(W); free(A); free(B); free(Y);
  }
  const int64_t shapes[3][4] = {{7, 5, 6, 3}, {1, 9, 2, 4}, {12, 3, 11, 1}};
  for (int s = 0; s < 3; ++s) {
    const int64_t n = shapes[s][0], i = shapes[s][1], o = shapes[s][2], r = shapes[s][3];
    double *X = filled(n * i), *W = filled(i * o), *A = filled(i * r), *B = filled(r * o), *dY = filled(n * o);
    double *Y0 = blank(n * o), *dX0 = blank(n * i), *dA0 = blank(i * r), *dB0 = blank(r * o);
    double *Y = blank(n * o), *dX = blank(n * i), *dA = blank(i * r), *dB = blank(r * o), *T = blank(n * r);
    orc_reference_forward(n, i, o, r, X, W, A, B, Y0);
    orc_reference_backward(n, i, o, r, X, W, A, B, dY, dX0, dA0, dB0);
    for (int v = 0; v <= 2; ++v) {
      if (orc_forward(v, n, i, o, r, X, W, A, B, Y, v == 0 ? T : NULL) != 0 || max_diff(Y, Y0, n * o) > 1e-12) {
        printf("shape %d: forward %d disagrees with Eq. 1\n", s, v);
        bad = 1;
      }
    }
    for (int v = 0; v <= 8; ++v) {
      if (orc_backward(v, n, i, o, r, X, W, A, B, dY, v == 0 ? T : NULL, dX, dA, dB) != 0 || max_diff(dX, dX0, n * i) > 1e-12 ||
          max_diff(dA, dA0, i * r) > 1e-12 || max_diff(dB, dB0, r * o) > 1e-12) {
        printf("shape %d: backward %d disagrees with Eq. 3\n", s, v);
        bad = 1;
      }
    }
    if (orc_forward(3, n, i, o, r, X, W, A, B, Y, NULL) != -1 || orc_backward(9, n, i, o, r, X, W, A, B, dY, NULL, dX, dA, dB) != -1) {
      printf("shape %d: unknown variant accepted\n", s);
      bad = 1;
    }
    if (n >= 3) { /* rows 1..2 on their own */
      double *Yr = blank(2 * o), *dXr = blank(2 * i);
      orc_reference_rows(2, i, o, r, X + i, dY + o, W, A, B, Yr, dXr);
      if (max_diff(Yr, Y0 + o, 2 * o) > 1e-12 || max_diff(dXr, dX0 + i, 2 * i) > 1e-12) { printf("shape %d: row sample wrong\n", s); bad = 1; }
      free(Yr); free(dXr);
    }
    free(X); free(W); free(A); free(B); free(dY); free(Y0); free(dX0); free(dA0); free(dB0);
    free(Y); free(dX); free(dA); free(dB); free(T);
  }
  { /* group dequantisation with a ragged last group: 70 rows in groups of 64 */
    const int64_t i = 70, o = 3, group = 64, groups = 2;
    int8_t* q = (int8_t*)malloc((size_t)(i * o));
    double *scale = filled(groups * o), *W = blank(i * o);
    for (int64_t k = 0; k < i * o; ++k) q[k] = (int8_t)((k * 5) % 15 - 7);
    orc_dequant_int4(i, o, group, q, scale, W);
    for (int64_t k = 0; k < i; ++k)
      for (int64_t j = 0; j < o; ++j)
        if (W[k * o + j] != (double)q[k * o + j] * scale[(k / group) * o + j]) bad = 1;
    free(q); free(scale); free(W);
  }
  printf(bad ? "mismatch\n" : "ok\n");
  return bad;
}
