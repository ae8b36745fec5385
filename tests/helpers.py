"""Shared by the GPU parity tests: moving seeded inputs to the device and comparing with the oracle."""
import numpy as np

from paper_2312_03415_amd import synth

# relative Frobenius error allowed per output tensor against the fp64 oracle
TOL = {"f32": 1e-5, "f16": 2e-3, "bf16": 1e-2}


def torch_dtype(name):
    import torch
    return {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[name]


def to_device(stored, dtype, device="cuda"):
    """numpy array produced by synth.store -> torch tensor of the matching dtype on the GPU."""
    import torch
    if dtype == "bf16":
        return torch.from_numpy(stored.view(np.int16)).view(torch.bfloat16).to(device)
    return torch.from_numpy(stored).to(device)


def to_f64(t):
    """device tensor -> exact float64 numpy values."""
    import torch
    return t.detach().to("cpu").to(torch.float64).numpy()


# Per-element bound beside the Frobenius one: |got - want| <= REL |want| + ABS rms(want), rms taken over the row (or
# the whole matrix for the small gradients), REL = (1 + roundings) u, ABS = 6 u, u = the storage type's unit roundoff
# (2^-9 bf16, 2^-11 fp16).  Each rounding of the output to the storage type costs at most u |want| (one rounding in
# RunLoRA's graphs; two in the default chain, whose Y = XW and dX = dY W^T are stored before the rank-r term is added);
# fp32 accumulation over K terms adds ~ sqrt(K) 2^-24 rms; an operand that was itself rounded to the storage type on
# the way (T = XA, Z1 = dY B^T, W + AB, X^T dY) adds a random relative error of at most u per term, ~ u / sqrt(3) rms
# per output, whose largest value over 10^5..10^8 outputs stays below 6 u rms (measured: no element of any graph
# beyond 0.75 of this bound).  A single 16-byte fragment (8 of K terms) lost or doubled shifts every element of its
# row by ~ sqrt(8 / K) rms = 0.027..0.06 rms at K = 11008..2048: outside the bound for the 16-bit types, where the
# Frobenius figure alone (1e-2 / 2e-3 of the whole tensor) would let it pass.  fp32 (true fp32 products, fp32
# accumulation, no rounded intermediates of note): 2e-6 |want| + 2e-5 rms.
UNIT_ROUNDOFF = {"bf16": 2.0 ** -9, "f16": 2.0 ** -11}


def elem_excess(got, want, dtype, per_row=True, roundings=1):
    """max over elements of |got - want| / (REL |want| + ABS rms): <= 1 means every element is within the bound."""
    if dtype == "f32":
        rel, ab = 2e-6, 2e-5
    else:
        rel, ab = (1 + roundings) * UNIT_ROUNDOFF[dtype], 6 * UNIT_ROUNDOFF[dtype]
    want = np.asarray(want, dtype=np.float64)
    if per_row and want.ndim == 2:
        rms = np.sqrt(np.mean(want * want, axis=1, keepdims=True))
    else:
        rms = np.sqrt(np.mean(want * want))
    bound = rel * np.abs(want) + ab * rms
    if not np.all(bound > 0):      # an all-zero reference row: the result must be zero there
        bound = np.where(bound > 0, bound, np.finfo(np.float64).tiny)
    return float(np.max(np.abs(got - want) / bound))


def relerr(got, want):
    den = np.linalg.norm(want)
    if den == 0.0:
        return float(np.linalg.norm(got))
    return float(np.linalg.norm(got - want) / den)


def layer_on_device(L, b_variance=None):
    """(stored-on-device tensors, float64 host copies of the same rounded values)."""
    st = synth.layer_inputs(L, b_variance=b_variance)
    dev = {k: to_device(v, L.dtype) for k, v in st.items()}
    host = {k: synth.widen(v, L.dtype) for k, v in st.items()}
    return dev, host
