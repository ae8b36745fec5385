"""fp64 CPU oracle for the RunLoRA layer (arxiv 2312.03415): TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the bench's cpu_baseline leg may import this package.  It
shares nothing with the HIP path and never imports it.  The arithmetic lives in
runlora_oracle.c (plain C, naive loops); this module marshals numpy arrays into it (the scaled
layer at the end reduces to the paper's layer by a substitution, written out there).

Shapes (paper's notation, Section 2): X [n,i], W [i,o], A [i,r], B [r,o], Y/dY [n,o],
dX [n,i], dA [i,r], dB [r,o]; everything float64, C-contiguous.
"""
import ctypes
import os

import numpy as np

from . import build as _build

FWD_DEFAULT, FWD1, FWD2 = 0, 1, 2
BWD_DEFAULT = 0  # 1..5 = Algorithms 1-5, 6..8 = remaining bracketings of Section 2

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB
        if (not os.path.exists(path)) or os.path.getmtime(path) < os.path.getmtime(_build.SRC):
            path = _build.build()
        L = ctypes.CDLL(path)
        i64, dp, ci = ctypes.c_int64, ctypes.POINTER(ctypes.c_double), ctypes.c_int
        L.orc_flops_reset.restype = None
        L.orc_flops_get.restype = ctypes.c_longlong
        L.orc_num_threads.restype = ci
        L.orc_matmul.argtypes = [ci, ci, i64, i64, i64, dp, i64, dp, i64, dp, i64, ci]
        L.orc_matmul.restype = None
        L.orc_reference_forward.argtypes = [i64] * 4 + [dp] * 5
        L.orc_reference_forward.restype = None
        L.orc_reference_backward.argtypes = [i64] * 4 + [dp] * 8
        L.orc_reference_backward.restype = None
        L.orc_forward.argtypes = [ci] + [i64] * 4 + [dp] * 6
        L.orc_forward.restype = ci
        L.orc_backward.argtypes = [ci] + [i64] * 4 + [dp] * 9
        L.orc_backward.restype = ci
        L.orc_dequant_int4.argtypes = [i64, i64, i64, ctypes.POINTER(ctypes.c_int8), dp, dp]
        L.orc_dequant_int4.restype = None
        L.orc_reference_rows.argtypes = [i64] * 4 + [dp] * 7
        L.orc_reference_rows.restype = None
        _lib = L
    return _lib


def _p(a):
    if a is None:
        return None
    assert a.dtype == np.float64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _dims(X, W, A, B):
    n, i = X.shape
    i2, o = W.shape
    i3, r = A.shape
    r2, o2 = B.shape
    assert i == i2 == i3 and o == o2 and r == r2, "shape mismatch"
    return n, i, o, r


def flops_reset():
    lib().orc_flops_reset()


def flops_get() -> int:
    return int(lib().orc_flops_get())


def num_threads() -> int:
    return int(lib().orc_num_threads())


def matmul(P, Q, ta=False, tb=False):
    """op(P) @ op(Q) through the oracle's own naive routine."""
    P, Q = _f64(P), _f64(Q)
    m, k = (P.shape[1], P.shape[0]) if ta else P.shape
    k2, n = (Q.shape[1], Q.shape[0]) if tb else Q.shape
    assert k == k2
    C = np.empty((m, n), dtype=np.float64)
    lib().orc_matmul(int(ta), int(tb), m, n, k, _p(P), P.shape[1], _p(Q), Q.shape[1], _p(C), n, 0)
    return C


def reference_forward(X, W, A, B):
    """Eq. 1 written out."""
    X, W, A, B = map(_f64, (X, W, A, B))
    n, i, o, r = _dims(X, W, A, B)
    Y = np.empty((n, o))
    lib().orc_reference_forward(n, i, o, r, _p(X), _p(W), _p(A), _p(B), _p(Y))
    return Y


def reference_backward(X, W, A, B, dY):
    """Eq. 3 written out -> (dX, dA, dB)."""
    X, W, A, B, dY = map(_f64, (X, W, A, B, dY))
    n, i, o, r = _dims(X, W, A, B)
    assert dY.shape == (n, o)
    dX, dA, dB = np.empty((n, i)), np.empty((i, r)), np.empty((r, o))
    lib().orc_reference_backward(n, i, o, r, _p(X), _p(W), _p(A), _p(B), _p(dY), _p(dX), _p(dA), _p(dB))
    return dX, dA, dB


def forward(variant, X, W, A, B):
    """One forward graph -> (Y, T) with T = XA for the default chain (variant 0), else None."""
    X, W, A, B = map(_f64, (X, W, A, B))
    n, i, o, r = _dims(X, W, A, B)
    Y = np.empty((n, o))
    T = np.empty((n, r)) if variant == FWD_DEFAULT else None
    rc = lib().orc_forward(variant, n, i, o, r, _p(X), _p(W), _p(A), _p(B), _p(Y), _p(T))
    if rc != 0:
        raise ValueError(f"oracle forward: bad variant {variant}")
    return Y, T


def backward(variant, X, W, A, B, dY, T=None):
    """One backward graph -> (dX, dA, dB).  Variant 0 needs T = XA kept by forward variant 0."""
    X, W, A, B, dY = map(_f64, (X, W, A, B, dY))
    n, i, o, r = _dims(X, W, A, B)
    assert dY.shape == (n, o)
    if T is not None:
        T = _f64(T)
        assert T.shape == (n, r)
    dX, dA, dB = np.empty((n, i)), np.empty((i, r)), np.empty((r, o))
    rc = lib().orc_backward(variant, n, i, o, r, _p(X), _p(W), _p(A), _p(B), _p(dY), _p(T), _p(dX), _p(dA), _p(dB))
    if rc != 0:
        raise ValueError(f"oracle backward: bad variant {variant} (or missing T)")
    return dX, dA, dB


def dequant_int4(q, scale, group=64):
    """W[k,j] = q[k,j] * scale[k // group, j]; q int8 in [-7,7] unpacked, scale float64."""
    q = np.ascontiguousarray(q, dtype=np.int8)
    scale = _f64(scale)
    i, o = q.shape
    assert scale.shape == ((i + group - 1) // group, o)
    W = np.empty((i, o))
    lib().orc_dequant_int4(i, o, group, q.ctypes.data_as(ctypes.POINTER(ctypes.c_int8)), _p(scale), _p(W))
    return W


def reference_rows(Xrows, dYrows, W, A, B):
    """Y and dX for a subset of token rows (rows are independent in Eq. 1 / Eq. 3's dX)."""
    Xrows, dYrows, W, A, B = map(_f64, (Xrows, dYrows, W, A, B))
    rows, i = Xrows.shape
    o, r = W.shape[1], A.shape[1]
    Y, dX = np.empty((rows, o)), np.empty((rows, i))
    lib().orc_reference_rows(rows, i, o, r, _p(Xrows), _p(dYrows), _p(W), _p(A), _p(B), _p(Y), _p(dX))
    return Y, dX


# ---- the layer with a LoRA scale and a frozen bias (not in the paper, which has s = 1, no bias) ----
# Y = XW + 1 b^T + s (XA) B is Eq. 1 evaluated on B' = sB, plus the bias row.  Eq. 3 on B' then gives
# dX and dA of the scaled layer as they are, and dB = s dB' by the chain rule through B' = sB; the
# bias is frozen like W and has no gradient.

def scaled_forward(X, W, A, B, scale=1.0, bias=None):
    Y = reference_forward(X, W, A, float(scale) * _f64(B))
    if bias is not None:
        Y = Y + _f64(bias).reshape(1, -1)
    return Y


def scaled_backward(X, W, A, B, dY, scale=1.0):
    dX, dA, dBp = reference_backward(X, W, A, float(scale) * _f64(B), dY)
    return dX, dA, float(scale) * dBp


def scaled_rows(Xrows, dYrows, W, A, B, scale=1.0, bias=None):
    """Y and dX of the scaled layer on a subset of token rows."""
    Y, dX = reference_rows(Xrows, dYrows, W, A, float(scale) * _f64(B))
    if bias is not None:
        Y = Y + _f64(bias).reshape(1, -1)
    return Y, dX


# ---- LoRA dropout on the adapter's input (not in the paper's experiments, which run with dropout 0) ----
# The keep-mask is defined by a counter-based generator (stated in include/runlora.h), which both sides
# implement on their own; everything after the mask is the plain definition
#     Y  = XW + 1 b^T + s' ((X o m) A) B,      s' = s / (1 - p_q),  p_q = round(256 p) / 256
#     dA = s' (X o m)^T dY B^T,   dB = s' ((X o m) A)^T dY,   dX = dY W^T + s' m o (dY B^T A^T).

def _mix32(x):
    x = np.asarray(x, dtype=np.uint32).copy()
    x ^= x >> np.uint32(16)
    x *= np.uint32(0x7FEB352D)
    x ^= x >> np.uint32(15)
    x *= np.uint32(0x846CA68B)
    x ^= x >> np.uint32(16)
    return x


def dropout_mask(n, i, p, seed):
    """(keep-mask [n, i] of 0.0 / 1.0, p_q): element (t, c) is kept iff byte c % 4 of
    mix(group ^ mix(seed ^ 0x9E3779B9)), group = t * (i / 4) + c // 4, is >= round(256 p)."""
    assert i % 4 == 0 and n * i < 2 ** 34
    thr = min(max(int(p * 256.0 + 0.5), 1), 255)
    with np.errstate(over="ignore"):
        key = _mix32(np.uint32((int(seed) & 0xFFFFFFFF) ^ 0x9E3779B9))
        groups = np.arange(n * (i // 4), dtype=np.uint64).astype(np.uint32)
        h = _mix32(groups ^ key)
    by = np.stack([(h >> np.uint32(8 * k)) & np.uint32(255) for k in range(4)], axis=1)   # [groups, 4]
    return (by >= thr).astype(np.float64).reshape(n, i), thr / 256.0


def dropout_forward(X, W, A, B, mask, p_q, scale=1.0, bias=None):
    X, W, A, B, mask = map(_f64, (X, W, A, B, mask))
    s = float(scale) / (1.0 - p_q)
    Y = matmul(X, W) + s * matmul(matmul(X * mask, A), B)
    if bias is not None:
        Y = Y + _f64(bias).reshape(1, -1)
    return Y


def dropout_backward(X, W, A, B, dY, mask, p_q, scale=1.0):
    X, W, A, B, dY, mask = map(_f64, (X, W, A, B, dY, mask))
    s = float(scale) / (1.0 - p_q)
    Xm = X * mask
    Z1 = matmul(dY, B, tb=True)
    dA = s * matmul(Xm, Z1, ta=True)
    dB = s * matmul(matmul(Xm, A), dY, ta=True)
    dX = matmul(dY, W, tb=True) + s * mask * matmul(Z1, A, tb=True)
    return dX, dA, dB



# ---- VeRA: frozen A and B, trainable scaling vectors (named in the paper's conclusion as an adapter ----
# the method carries over to; the paper gives no formulas, the definition below is the published one
# written in this file's orientation, Y = XW):
#     Y = XW + 1 bias^T + s (((X A) diag(d)) B) diag(b),      d in R^r, b in R^o trainable, A, B, W frozen
# Gradients by the chain rule, step by step through T = XA, U = T diag(d), V = U B, Y = .. + s V diag(b):
#     dV = s dY diag(b);  db[j] = s sum_t dY[t,j] V[t,j];  dU = dV B^T;  dd[k] = sum_t T[t,k] dU[t,k];
#     dX = dY W^T + (dU diag(d)) A^T.

def vera_forward(X, W, A, B, d, b, scale=1.0, bias=None):
    X, W, A, B, d, b = map(_f64, (X, W, A, B, d, b))
    T = matmul(X, A)
    V = matmul(T * d.reshape(1, -1), B)
    Y = matmul(X, W) + float(scale) * V * b.reshape(1, -1)
    if bias is not None:
        Y = Y + _f64(bias).reshape(1, -1)
    return Y


def vera_backward(X, W, A, B, d, b, dY, scale=1.0):
    """(dX [n,i], dd [r], db [o])."""
    X, W, A, B, d, b, dY = map(_f64, (X, W, A, B, d, b, dY))
    s = float(scale)
    T = matmul(X, A)
    V = matmul(T * d.reshape(1, -1), B)
    db = s * np.sum(dY * V, axis=0)
    dU = matmul(s * dY * b.reshape(1, -1), B, tb=True)
    dd = np.sum(T * dU, axis=0)
    dX = matmul(dY, W, tb=True) + matmul(dU * d.reshape(1, -1), A, tb=True)
    return dX, dd, db


# ---- DoRA: magnitude / direction decomposition of the adapted weight (named in the paper's conclusion ----
# as an adapter the method carries over to; the paper gives no formulas, the definition below is the
# published one written in this file's orientation, Y = XW, output feature j = column j):
#     V = W + s A B,   c[j] = || V[:, j] ||_2,   Y = X (V diag(m / c)) + 1 bias^T,     m in R^o trainable
# The published method back-propagates with c held constant (it is detached from the graph), and so do
# the gradients here.  Step by step through U = X V, Y = U diag(g) + bias, g = m / c:
#     dm[j] = sum_t dY[t,j] U[t,j] / c[j];   dU = dY diag(g);   dX = dU V^T;
#     dA = s X^T (dU B^T);   dB = s (X A)^T dU.

def dora_norm(W, A, B, scale=1.0):
    """c [o]: the column norms of W + s A B."""
    W, A, B = map(_f64, (W, A, B))
    V = W + float(scale) * matmul(A, B)
    return np.sqrt(np.sum(V * V, axis=0))


def dora_forward(X, W, A, B, m, scale=1.0, bias=None):
    X, W, A, B, m = map(_f64, (X, W, A, B, m))
    V = W + float(scale) * matmul(A, B)
    c = np.sqrt(np.sum(V * V, axis=0))
    Y = matmul(X, V) * (m / c).reshape(1, -1)
    if bias is not None:
        Y = Y + _f64(bias).reshape(1, -1)
    return Y


def dora_backward(X, W, A, B, m, dY, scale=1.0):
    """(dX [n,i], dA [i,r], dB [r,o], dm [o]) with the column norm treated as a constant."""
    X, W, A, B, m, dY = map(_f64, (X, W, A, B, m, dY))
    s = float(scale)
    V = W + s * matmul(A, B)
    c = np.sqrt(np.sum(V * V, axis=0))
    U = matmul(X, V)
    dm = np.sum(dY * U, axis=0) / c
    dU = dY * (m / c).reshape(1, -1)
    dX = matmul(dU, V, tb=True)
    dA = s * matmul(X, matmul(dU, B, tb=True), ta=True)
    dB = s * matmul(matmul(X, A), dU, ta=True)
    return dX, dA, dB, dm
