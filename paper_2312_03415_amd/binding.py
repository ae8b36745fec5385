"""ctypes binding of librunlora.so (include/runlora.h): argument marshalling only.

Every step of the layer runs inside the HIP library; torch is used for device memory and for the
current stream.  There is no fallback: if the library is missing, loading raises.

    runlora_forward(variant, X, W, A, B, Y, saved, workspace=None, stream=None)
    runlora_backward(variant, dY, saved, W, A, B, dX, dA, dB, workspace=None, stream=None)
    runlora_select(n_tokens, d_in, d_out, r, dtype) -> (fwd, bwd)

Tensors are 2-D torch tensors on the GPU (row-major, last dimension contiguous):
X [n,i], W [i,o], A [i,r], B [r,o], Y/dY [n,o], dX [n,i], dA [i,r], dB [r,o]  (Section 2 of
arxiv 2312.03415: Y = XW + (XA)B, W frozen).
"""
import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "librunlora.so")

RL_F32, RL_F16, RL_BF16, RL_INT4_G64 = 0, 1, 2, 3
FWD_DEFAULT, FWD1, FWD2, FWD3 = 0, 1, 2, 3
BWD_DEFAULT, BWD1, BWD2, BWD3, BWD4, BWD5, BWD6, BWD7, BWD8 = 0, 1, 2, 3, 4, 5, 6, 7, 8
FWD_VARIANTS = (FWD_DEFAULT, FWD1, FWD2, FWD3)
BWD_VARIANTS = (BWD_DEFAULT, BWD1, BWD2, BWD3, BWD4, BWD5, BWD6, BWD7, BWD8)
BWD_MERGED = (BWD4, BWD5, BWD7, BWD8)  # the graphs that read W + AB as a matrix

RL_OK = 0
RL_ERR_NULL, RL_ERR_SHAPE, RL_ERR_DTYPE, RL_ERR_VARIANT, RL_ERR_SAVED_MISMATCH = -1, -2, -3, -4, -5
RL_ERR_ALIGN, RL_ERR_ALIAS, RL_ERR_WORKSPACE, RL_ERR_UNSUPPORTED, RL_ERR_HIP = -6, -7, -8, -9, -10

EXPORTS = (
    "runlora_forward", "runlora_forward_static", "runlora_backward", "runlora_select", "runlora_select_by", "runlora_flops",
    "runlora_model_time_us", "runlora_workspace_bytes", "runlora_workspace_bytes_w", "runlora_saved_bytes",
    "runlora_strerror", "runlora_last_hip_error",
    "runlora_version", "runlora_gemm", "runlora_gemm_workspace_bytes",
    "runlora_profile_enable", "runlora_profile_collect", "runlora_profile_disable", "runlora_profile_kernel_times",
    "runlora_probe_mfma",
    "runlora_vera_forward", "runlora_vera_backward", "runlora_vera_workspace_bytes",
    "runlora_dora_forward", "runlora_dora_backward", "runlora_dora_workspace_bytes",
)


class rl_tensor_t(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("rows", ctypes.c_int64), ("cols", ctypes.c_int64),
                ("ld", ctypes.c_int64), ("dtype", ctypes.c_int32), ("scales", ctypes.c_void_p),
                ("group", ctypes.c_int32)]


class rl_saved_t(ctypes.Structure):
    _fields_ = [("fwd_variant", ctypes.c_int32), ("dtype", ctypes.c_int32), ("n", ctypes.c_int64),
                ("i", ctypes.c_int64), ("o", ctypes.c_int64), ("r", ctypes.c_int64),
                ("X", ctypes.c_void_p), ("ldx", ctypes.c_int64), ("T", ctypes.c_void_p),
                ("ldt", ctypes.c_int64), ("M", ctypes.c_void_p), ("ldm", ctypes.c_int64),
                ("scale", ctypes.c_float), ("dropout_thr", ctypes.c_uint32), ("dropout_seed", ctypes.c_uint32)]


class rl_opts_t(ctypes.Structure):
    _fields_ = [("stream", ctypes.c_void_p), ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
                ("scale", ctypes.c_float), ("bias", ctypes.c_void_p), ("dropout_p", ctypes.c_float),
                ("dropout_seed", ctypes.c_uint32)]


class rl_gemm_t(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("a_strided", ctypes.c_int32), ("b_kcontig", ctypes.c_int32),
                ("tile_cfg", ctypes.c_int32), ("splits", ctypes.c_int32),
                ("M", ctypes.c_int64), ("N", ctypes.c_int64), ("K", ctypes.c_int64), ("K2", ctypes.c_int64),
                ("A", ctypes.c_void_p), ("B", ctypes.c_void_p), ("A2", ctypes.c_void_p), ("B2", ctypes.c_void_p),
                ("D", ctypes.c_void_p), ("C", ctypes.c_void_p),
                ("lda", ctypes.c_int64), ("ldb", ctypes.c_int64), ("lda2", ctypes.c_int64), ("ldb2", ctypes.c_int64),
                ("ldc", ctypes.c_int64), ("ldd", ctypes.c_int64), ("trans_out", ctypes.c_int32),
                ("alpha", ctypes.c_float), ("bias", ctypes.c_void_p)]


class rl_step_time_t(ctypes.Structure):
    _fields_ = [("what", ctypes.c_char_p), ("us", ctypes.c_double), ("flops", ctypes.c_double),
                ("bytes", ctypes.c_double), ("M", ctypes.c_int64), ("N", ctypes.c_int64), ("K", ctypes.c_int64),
                ("tile_cfg", ctypes.c_int32), ("splits", ctypes.c_int32), ("a_strided", ctypes.c_int32),
                ("b_kcontig", ctypes.c_int32), ("kernel_us", ctypes.c_double), ("main_us", ctypes.c_double),
                ("kernels", ctypes.c_int32)]


class RunLoRAError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"runlora error {code}: {text}")
        self.code = code


_lib = None


def lib():
    """Load librunlora.so (built by `python -m paper_2312_03415_amd.build`).  Raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} not found: build it with `python -m paper_2312_03415_amd.build` (no CPU fallback exists)")
    # torch ships its own copy of the HIP runtime; importing it first makes the library's dependency
    # resolve to that copy, so that both sides share one runtime (and one view of the device) whatever
    # the caller's import order
    import torch  # noqa: F401
    L = ctypes.CDLL(LIB_PATH)
    tp, sp, op = ctypes.POINTER(rl_tensor_t), ctypes.POINTER(rl_saved_t), ctypes.POINTER(rl_opts_t)
    i64, ci, ip = ctypes.c_int64, ctypes.c_int, ctypes.POINTER(ctypes.c_int)
    L.runlora_forward.argtypes = [ci, tp, tp, tp, tp, tp, sp, op]
    L.runlora_forward.restype = ci
    L.runlora_forward_static.argtypes = [ci, tp, tp, tp, tp, tp, sp, op]
    L.runlora_forward_static.restype = ci
    L.runlora_backward.argtypes = [ci, tp, sp, tp, tp, tp, tp, tp, tp, op]
    L.runlora_backward.restype = ci
    vp = ctypes.c_void_p
    L.runlora_vera_forward.argtypes = [ci, tp, tp, tp, tp, vp, vp, tp, sp, op]
    L.runlora_vera_forward.restype = ci
    L.runlora_vera_backward.argtypes = [ci, tp, sp, tp, tp, tp, vp, vp, tp, vp, vp, op]
    L.runlora_vera_backward.restype = ci
    L.runlora_vera_workspace_bytes.argtypes = [ci, ci, i64, i64, i64, i64, ci]
    L.runlora_vera_workspace_bytes.restype = ctypes.c_size_t
    L.runlora_dora_forward.argtypes = [ci, tp, tp, tp, tp, vp, tp, sp, vp, op]
    L.runlora_dora_forward.restype = ci
    L.runlora_dora_backward.argtypes = [ci, tp, sp, tp, tp, tp, vp, vp, tp, tp, tp, tp, vp, op]
    L.runlora_dora_backward.restype = ci
    L.runlora_dora_workspace_bytes.argtypes = [ci, ci, i64, i64, i64, i64, ci]
    L.runlora_dora_workspace_bytes.restype = ctypes.c_size_t
    L.runlora_select.argtypes = [i64, i64, i64, i64, ci, ip, ip]
    L.runlora_select.restype = ci
    L.runlora_select_by.argtypes = [ci, i64, i64, i64, i64, ci, ip, ip]
    L.runlora_select_by.restype = ci
    L.runlora_flops.argtypes = [ci, ci, i64, i64, i64, i64]
    L.runlora_flops.restype = i64
    L.runlora_model_time_us.argtypes = [ci, ci, i64, i64, i64, i64, ci]
    L.runlora_model_time_us.restype = ctypes.c_double
    L.runlora_workspace_bytes.argtypes = [ci, ci, i64, i64, i64, i64, ci]
    L.runlora_workspace_bytes.restype = ctypes.c_size_t
    L.runlora_workspace_bytes_w.argtypes = [ci, ci, i64, i64, i64, i64, ci, ci]
    L.runlora_workspace_bytes_w.restype = ctypes.c_size_t
    L.runlora_saved_bytes.argtypes = [ci, i64, i64, i64, i64, ci, ci]
    L.runlora_saved_bytes.restype = ctypes.c_size_t
    L.runlora_strerror.argtypes = [ci]
    L.runlora_strerror.restype = ctypes.c_char_p
    L.runlora_last_hip_error.argtypes = []
    L.runlora_last_hip_error.restype = ctypes.c_char_p
    L.runlora_version.argtypes = []
    L.runlora_version.restype = ci
    L.runlora_gemm.argtypes = [ctypes.POINTER(rl_gemm_t), op]
    L.runlora_gemm.restype = ci
    L.runlora_gemm_workspace_bytes.argtypes = [ctypes.POINTER(rl_gemm_t)]
    L.runlora_gemm_workspace_bytes.restype = ctypes.c_size_t
    L.runlora_profile_enable.argtypes = [ci]
    L.runlora_profile_enable.restype = ci
    L.runlora_profile_collect.argtypes = [ctypes.POINTER(rl_step_time_t), ci]
    L.runlora_profile_collect.restype = ci
    L.runlora_probe_mfma.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ci, ctypes.c_void_p, ctypes.POINTER(ctypes.c_double)]
    L.runlora_probe_mfma.restype = ci
    L.runlora_profile_kernel_times.argtypes = [ci]
    L.runlora_profile_kernel_times.restype = ci
    L.runlora_profile_disable.argtypes = []
    L.runlora_profile_disable.restype = ci
    _lib = L
    return L


def _check(code):
    if code != RL_OK:
        L = lib()
        text = L.runlora_strerror(code).decode()
        if code in (RL_ERR_HIP, RL_ERR_WORKSPACE) and L.runlora_last_hip_error():
            text += " (" + L.runlora_last_hip_error().decode() + ")"
        raise RunLoRAError(code, text)


def dtype_code(torch_dtype):
    import torch
    return {torch.float32: RL_F32, torch.float16: RL_F16, torch.bfloat16: RL_BF16}[torch_dtype]


def dtype_from_name(name):
    return {"f32": RL_F32, "f16": RL_F16, "bf16": RL_BF16, "int4": RL_INT4_G64}[name]


class Int4Weight:
    """A frozen W [rows, cols] stored as symmetric int4 with one fp16 scale per 64 rows per column
    (RL_INT4_G64): `packed` is a uint8 device tensor [rows, ld/2] (element (k,j) in the low nibble of
    byte j/2 of row k for even j, high nibble for odd j; value = nibble - 8), `scales` an fp16 device
    tensor [ceil(rows/64), cols]."""

    def __init__(self, packed, scales, rows, cols):
        assert packed.dim() == 2 and packed.stride(1) == 1 and packed.shape[0] == rows
        assert scales.dim() == 2 and scales.is_contiguous() and scales.shape == ((rows + 63) // 64, cols)
        self.packed, self.scales, self.rows, self.cols = packed, scales, rows, cols
        self.ld = packed.stride(0) * 2

    @staticmethod
    def from_host(q, scale, device="cuda"):
        """q: int8 numpy [rows, cols] with values in [-7,7] (cols even); scale: float16 numpy."""
        import numpy as np
        import torch
        rows, cols = q.shape
        u = (q.astype(np.int16) + 8).astype(np.uint8)
        packed = (u[:, 0::2] | (u[:, 1::2] << 4)).astype(np.uint8)
        return Int4Weight(torch.from_numpy(np.ascontiguousarray(packed)).to(device),
                          torch.from_numpy(np.ascontiguousarray(scale)).to(device), rows, cols)


def tensor_desc(t):
    """rl_tensor_t view of a 2-D torch tensor or an Int4Weight (None -> NULL pointer argument)."""
    if t is None:
        return None
    if isinstance(t, Int4Weight):
        return rl_tensor_t(t.packed.data_ptr(), t.rows, t.cols, t.ld, RL_INT4_G64, t.scales.data_ptr(), 64)
    if t.dim() != 2 or t.stride(1) != 1:
        raise ValueError("expected a 2-D tensor with contiguous rows")
    return rl_tensor_t(t.data_ptr(), t.shape[0], t.shape[1], t.stride(0), dtype_code(t.dtype), None, 0)


def _opts(workspace, stream, scale=None, bias=None, dropout_p=None, dropout_seed=0):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    if bias is not None and (bias.dim() != 1 or bias.stride(0) != 1):
        raise ValueError("bias must be a contiguous 1-D tensor")
    return rl_opts_t(stream, ws_ptr, ws_bytes, 0.0 if scale is None else float(scale),
                     bias.data_ptr() if bias is not None else None, 0.0 if not dropout_p else float(dropout_p),
                     int(dropout_seed) & 0xFFFFFFFF)


def _ref(desc):
    return ctypes.byref(desc) if desc is not None else None


def runlora_forward(variant, X, W, A, B, Y, saved, workspace=None, stream=None, scale=None, bias=None,
                    dropout_p=None, dropout_seed=0):
    """Y = XW (+ bias) + scale (XA)B in forward graph `variant`; fills `saved` (rl_saved_t).  For
    FWD_DEFAULT set saved.T / saved.ldt to an [n,r] buffer first, for FWD2 optionally saved.M /
    saved.ldm to an [i,o] buffer that keeps W + scale AB for the backward (see new_saved).
    scale None = 1 (the paper's layer); bias: 1-D tensor [o] of the activation dtype or None;
    dropout_p / dropout_seed: LoRA dropout on the adapter's input (mask defined in runlora.h), None = off."""
    if bias is not None and (bias.dtype != X.dtype or bias.numel() != Y.shape[1]):
        raise ValueError("bias must have d_out elements of the activation dtype")
    dx, dw, da, db, dy = (tensor_desc(t) for t in (X, W, A, B, Y))
    o = _opts(workspace, stream, scale, bias, dropout_p, dropout_seed)
    _check(lib().runlora_forward(variant, _ref(dx), _ref(dw), _ref(da), _ref(db), _ref(dy), ctypes.byref(saved),
                                 ctypes.byref(o)))
    return Y


STATIC_SCRATCH_BYTES = 16 << 20  # RL_STATIC_SCRATCH_BYTES of runlora.h


def runlora_forward_static(variant, X, W, A, B, Y, saved, stream=None, scale=None, bias=None, dropout_p=None,
                           dropout_seed=0):
    """runlora_forward with the variant's scratch in the library's fixed device array (no workspace argument, no
    device allocation); raises RL_ERR_WORKSPACE if the call needs more than STATIC_SCRATCH_BYTES."""
    if bias is not None and (bias.dtype != X.dtype or bias.numel() != Y.shape[1]):
        raise ValueError("bias must have d_out elements of the activation dtype")
    dx, dw, da, db, dy = (tensor_desc(t) for t in (X, W, A, B, Y))
    o = _opts(None, stream, scale, bias, dropout_p, dropout_seed)
    _check(lib().runlora_forward_static(variant, _ref(dx), _ref(dw), _ref(da), _ref(db), _ref(dy), ctypes.byref(saved),
                                        ctypes.byref(o)))
    return Y


def runlora_backward(variant, dY, saved, W, A, B, dX, dA, dB, workspace=None, stream=None):
    """Gradients of Eq. 3 in backward graph `variant`; any of dX/dA/dB may be None (skipped)."""
    ddy, dw, da, db = (tensor_desc(t) for t in (dY, W, A, B))
    gx, ga, gb = tensor_desc(dX), tensor_desc(dA), tensor_desc(dB)
    o = _opts(workspace, stream)
    _check(lib().runlora_backward(variant, _ref(ddy), ctypes.byref(saved), _ref(dw), _ref(da), _ref(db), _ref(gx),
                                  _ref(ga), _ref(gb), ctypes.byref(o)))
    return dX, dA, dB


def _vec(t, count, dtype, name):
    """Device pointer of a 1-D vector argument (None -> NULL)."""
    if t is None:
        return None
    if t.dim() != 1 or t.numel() != count or t.dtype != dtype or t.stride(0) != 1:
        raise ValueError(f"{name} must be a dense vector of {count} elements of the activation dtype")
    return t.data_ptr()


def runlora_vera_forward(variant, X, W, A, B, d, b, Y, saved, workspace, stream=None, scale=None, bias=None,
                         dropout_p=None, dropout_seed=0):
    """VeRA forward, Y = XW (+ bias) + scale ((XA) diag(d)) B diag(b), in forward graph `variant`; the
    workspace (runlora_vera_workspace_bytes) is required.  Other arguments as runlora_forward."""
    if bias is not None and (bias.dtype != X.dtype or bias.numel() != Y.shape[1]):
        raise ValueError("bias must have d_out elements of the activation dtype")
    dx, dw, da, db, dy = (tensor_desc(t) for t in (X, W, A, B, Y))
    o = _opts(workspace, stream, scale, bias, dropout_p, dropout_seed)
    _check(lib().runlora_vera_forward(variant, _ref(dx), _ref(dw), _ref(da), _ref(db), _vec(d, B.shape[0], X.dtype, "d"),
                                      _vec(b, B.shape[1], X.dtype, "b"), _ref(dy), ctypes.byref(saved), ctypes.byref(o)))
    return Y


def runlora_vera_backward(variant, dY, saved, W, A, B, d, b, dX, dd, db, workspace, stream=None):
    """VeRA gradients for X, d and b in backward graph `variant`; any of dX / dd / db may be None."""
    ddy, dw, da, dbm = (tensor_desc(t) for t in (dY, W, A, B))
    gx = tensor_desc(dX)
    o = _opts(workspace, stream)
    r, oo = B.shape
    _check(lib().runlora_vera_backward(variant, _ref(ddy), ctypes.byref(saved), _ref(dw), _ref(da), _ref(dbm),
                                       _vec(d, r, dY.dtype, "d"), _vec(b, oo, dY.dtype, "b"), _ref(gx),
                                       _vec(dd, r, dY.dtype, "dd"), _vec(db, oo, dY.dtype, "db"), ctypes.byref(o)))
    return dX, dd, db


def runlora_vera_workspace_bytes(fwd, bwd, n, i, o, r, dtype):
    return int(lib().runlora_vera_workspace_bytes(fwd, bwd, n, i, o, r, dtype))


def runlora_dora_forward(variant, X, W, A, B, m, Y, saved, c, workspace, stream=None, scale=None, bias=None):
    """DoRA forward, Y = X ((W + scale A B) diag(m / c)) (+ bias), c = column norms of W + scale A B (written to
    the fp32 vector c); variant must be RL_FWD2; the workspace (runlora_dora_workspace_bytes) is required."""
    import torch
    if bias is not None and (bias.dtype != X.dtype or bias.numel() != Y.shape[1]):
        raise ValueError("bias must have d_out elements of the activation dtype")
    dx, dw, da, db, dy = (tensor_desc(t) for t in (X, W, A, B, Y))
    o = _opts(workspace, stream, scale, bias)
    _check(lib().runlora_dora_forward(variant, _ref(dx), _ref(dw), _ref(da), _ref(db), _vec(m, B.shape[1], X.dtype, "m"),
                                      _ref(dy), ctypes.byref(saved), _vec(c, B.shape[1], torch.float32, "c"), ctypes.byref(o)))
    return Y


def runlora_dora_backward(variant, dY, saved, W, A, B, m, c, Y, dX, dA, dB, dm, workspace, stream=None, bias=None):
    """DoRA gradients for X, A, B and m (column norm held constant) in backward graph `variant` (RL_BWD4 / 5 / 7 /
    8); any of dX / dA / dB / dm may be None; Y (the forward's output) and the forward's bias are needed for dm."""
    import torch
    ddy, dw, da, dbm = (tensor_desc(t) for t in (dY, W, A, B))
    gy = tensor_desc(Y)
    gx, ga, gb = (tensor_desc(t) for t in (dX, dA, dB))
    o = _opts(workspace, stream, None, bias)
    oo = B.shape[1]
    _check(lib().runlora_dora_backward(variant, _ref(ddy), ctypes.byref(saved), _ref(dw), _ref(da), _ref(dbm),
                                       _vec(m, oo, dY.dtype, "m"), _vec(c, oo, torch.float32, "c"), _ref(gy), _ref(gx),
                                       _ref(ga), _ref(gb), _vec(dm, oo, dY.dtype, "dm"), ctypes.byref(o)))
    return dX, dA, dB, dm


def runlora_dora_workspace_bytes(fwd, bwd, n, i, o, r, dtype):
    return int(lib().runlora_dora_workspace_bytes(fwd, bwd, n, i, o, r, dtype))


def runlora_select(n_tokens, d_in, d_out, r, dtype, criterion=None):
    """(fwd, bwd) for a layer shape.  criterion None = library default (time model unless
    RUNLORA_CRITERION=flops), 0 = Table 1 FLOPs, 1 = time model, 2 = time model when forward2 keeps
    W + AB for the backward."""
    f, b = ctypes.c_int(-1), ctypes.c_int(-1)
    if criterion is None:
        _check(lib().runlora_select(n_tokens, d_in, d_out, r, dtype, ctypes.byref(f), ctypes.byref(b)))
    else:
        _check(lib().runlora_select_by(criterion, n_tokens, d_in, d_out, r, dtype, ctypes.byref(f), ctypes.byref(b)))
    return f.value, b.value


def runlora_flops(is_bwd, variant, n, i, o, r):
    return int(lib().runlora_flops(int(is_bwd), variant, n, i, o, r))


def runlora_model_time_us(is_bwd, variant, n, i, o, r, dtype):
    return float(lib().runlora_model_time_us(int(is_bwd), variant, n, i, o, r, dtype))


def runlora_workspace_bytes(fwd, bwd, n, i, o, r, dtype, w_dtype=None):
    if w_dtype is None:
        return int(lib().runlora_workspace_bytes(fwd, bwd, n, i, o, r, dtype))
    return int(lib().runlora_workspace_bytes_w(fwd, bwd, n, i, o, r, dtype, w_dtype))


def runlora_saved_bytes(fwd, n, i, o, r, dtype, keep_merged=False, keep_t=False):
    """Bytes forward graph `fwd` keeps for the backward besides X."""
    return int(lib().runlora_saved_bytes(fwd, n, i, o, r, dtype, int(bool(keep_merged)) | (2 if keep_t else 0)))


def runlora_gemm(A, B, C, a_strided=False, b_kcontig=False, A2=None, B2=None, D=None, tile_cfg=-1, splits=0,
                 workspace=None, stream=None, trans_out=False, alpha=None, bias=None):
    """C = alpha (op(A) op(B) (+ op(A2) op(B2))) (+ D) (+ bias) through the library's tile GEMM (see
    runlora.h)."""
    import torch
    M = A.shape[1] if a_strided else A.shape[0]
    K = A.shape[0] if a_strided else A.shape[1]
    N = B.shape[0] if b_kcontig else B.shape[1]
    K2 = 0
    if A2 is not None:
        K2 = A2.shape[0] if a_strided else A2.shape[1]
    g = rl_gemm_t(dtype_code(A.dtype), int(a_strided), int(b_kcontig), tile_cfg, splits, M, N, K, K2,
                  A.data_ptr(), B.data_ptr(), A2.data_ptr() if A2 is not None else None,
                  B2.data_ptr() if B2 is not None else None, D.data_ptr() if D is not None else None, C.data_ptr(),
                  A.stride(0), B.stride(0), A2.stride(0) if A2 is not None else 0,
                  B2.stride(0) if B2 is not None else 0, C.stride(0), D.stride(0) if D is not None else 0, int(trans_out),
                  0.0 if alpha is None else float(alpha), bias.data_ptr() if bias is not None else None)
    need = int(lib().runlora_gemm_workspace_bytes(ctypes.byref(g)))
    if need and (workspace is None or workspace.numel() * workspace.element_size() < need):
        workspace = torch.empty(need, dtype=torch.uint8, device=C.device)
    o = _opts(workspace, stream)
    _check(lib().runlora_gemm(ctypes.byref(g), ctypes.byref(o)))
    return C


def runlora_profile_enable(max_steps):
    _check(lib().runlora_profile_enable(max_steps))


def runlora_profile_collect(cap=4096):
    """Per-step timings of the layer calls since enable / the last collect, as a list of dicts."""
    buf = (rl_step_time_t * cap)()
    k = lib().runlora_profile_collect(buf, cap)
    if k < 0:
        _check(k)
    keys = ("us", "kernel_us", "main_us", "kernels", "flops", "bytes", "M", "N", "K", "tile_cfg", "splits", "a_strided", "b_kcontig")
    return [dict(what=buf[j].what.decode(), **{f: getattr(buf[j], f) for f in keys}) for j in range(k)]


def runlora_profile_kernel_times(on=True):
    """Also time each of a step's kernels alone (rl_step_time_t.kernel_us / main_us) in the profile passes of this thread."""
    _check(lib().runlora_profile_kernel_times(1 if on else 0))


def runlora_profile_disable():
    _check(lib().runlora_profile_disable())


def runlora_probe_mfma(random_data, device="cuda"):
    """Sustained bf16 MFMA TFLOP/s of this GPU on zeros (False) or random operands (True)."""
    import torch
    scratch = torch.empty(1 << 20, dtype=torch.uint8, device=device)
    out = ctypes.c_double(0.0)
    _check(lib().runlora_probe_mfma(scratch.data_ptr(), scratch.numel(), int(bool(random_data)),
                                    torch.cuda.current_stream().cuda_stream, ctypes.byref(out)))
    return out.value


# ---- conveniences on top of the ABI (device memory only) --------------------------------------

def new_saved(T=None, M=None):
    """A zeroed rl_saved_t; T: [n,r] buffer for FWD_DEFAULT's XA; M: [i,o] buffer in which FWD2 keeps
    W + AB for the backward."""
    s = rl_saved_t()
    if T is not None:
        s.T = T.data_ptr()
        s.ldt = T.stride(0)
    if M is not None:
        s.M = M.data_ptr()
        s.ldm = M.stride(0)
    return s


def new_workspace(fwd, bwd, n, i, o, r, dtype, device="cuda", w_dtype=None):
    import torch
    nbytes = runlora_workspace_bytes(fwd, bwd, n, i, o, r, dtype, w_dtype)
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
