"""GPU: runlora_forward_static (the entry point for callers that cannot allocate: its scratch is a fixed array in the
library's device image) against runlora_forward on the same inputs, bit for bit, on two calls in a row, the second with
a smaller input; and its refusal of a call that needs more scratch than the array holds.  Collected last (file name)."""
import numpy as np
import pytest

import oracle
from helpers import TOL, layer_on_device, relerr, to_f64, torch_dtype
from paper_2312_03415_amd import binding as rl
from paper_2312_03415_amd import synth

pytestmark = pytest.mark.gpu


def forward_both(L, fwd, dev):
    import torch
    td = torch_dtype(L.dtype)
    code = rl.dtype_from_name(L.dtype)
    nan = float("nan")
    Y0 = torch.full((L.n, L.o), nan, dtype=td, device="cuda")
    Y1 = torch.full((L.n, L.o), nan, dtype=td, device="cuda")
    ws = rl.new_workspace(fwd, -1, L.n, L.i, L.o, L.r, code)
    s0, s1 = rl.new_saved(), rl.new_saved()
    rl.runlora_forward(fwd, dev["X"], dev["W"], dev["A"], dev["B"], Y0, s0, workspace=ws)
    rl.runlora_forward_static(fwd, dev["X"], dev["W"], dev["A"], dev["B"], Y1, s1)
    torch.cuda.synchronize()
    assert s1.fwd_variant == fwd and s1.n == L.n and s1.X == dev["X"].data_ptr()
    return Y0, Y1


@pytest.mark.parametrize("fwd", [1, 2])
def test_static_scratch_forward_matches_workspace_forward(fwd):
    import torch
    # first a shape whose scratch spans megabytes (T = XA, or W + AB), then a smaller, ragged one with split-K partials:
    # the array still holds the first call's contents when the second one runs
    shapes = [synth.Layer("static_big", 4096, 1024, 2048, 64, "bf16", 21), synth.Layer("static_small", 600, 520, 392, 24, "bf16", 22)]
    for L in shapes:
        print(f"case static fwd={fwd} layer={L}", flush=True)
        assert 0 < rl.runlora_workspace_bytes(fwd, -1, L.n, L.i, L.o, L.r, rl.RL_BF16) <= rl.STATIC_SCRATCH_BYTES
        dev, host = layer_on_device(L)
        Y0, Y1 = forward_both(L, fwd, dev)
        assert not torch.isnan(Y1).any()
        assert torch.equal(Y0, Y1)
        want = oracle.reference_forward(host["X"], host["W"], host["A"], host["B"])
        assert relerr(to_f64(Y1), want) < TOL[L.dtype]


def test_static_scratch_refuses_what_does_not_fit():
    import torch
    L = synth.Layer("static_too_big", 512, 4096, 4096, 16, "bf16", 23)   # forward2's W + AB is 32 MiB
    assert rl.runlora_workspace_bytes(2, -1, L.n, L.i, L.o, L.r, rl.RL_BF16) > rl.STATIC_SCRATCH_BYTES
    g = torch.Generator(device="cuda").manual_seed(1)
    mk = lambda *s: torch.randn(*s, device="cuda", generator=g).to(torch.bfloat16)
    X, W, A, B = mk(L.n, L.i), mk(L.i, L.o), mk(L.i, L.r), mk(L.r, L.o)
    Y = torch.zeros(L.n, L.o, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(rl.RunLoRAError) as e:
        rl.runlora_forward_static(2, X, W, A, B, Y, rl.new_saved())
    assert e.value.code == rl.RL_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert not Y.any()   # nothing was enqueued
