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
