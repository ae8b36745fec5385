"""GPU parity: every forward x backward computation graph of the layer, through the C ABI, against
the fp64 CPU oracle on the same seeded inputs (relative Frobenius error per output tensor)."""
import itertools

import numpy as np
import pytest

import oracle
from helpers import TOL, layer_on_device, relerr, to_device, to_f64, torch_dtype
from paper_2312_03415_amd import binding as rl
from paper_2312_03415_amd import synth

pytestmark = pytest.mark.gpu


def run_pair(L, dev, fwd, bwd, want_grads=(True, True, True)):
    """One forward + backward through the library; returns float64 host copies."""
    import torch
    td = torch_dtype(L.dtype)
    code = rl.dtype_from_name(L.dtype)
    nan = float("nan")
    Y = torch.full((L.n, L.o), nan, dtype=td, device="cuda")
    T = torch.full((L.n, L.r), nan, dtype=td, device="cuda") if fwd == rl.FWD_DEFAULT else None
    saved = rl.new_saved(T)
    ws = rl.new_workspace(fwd, bwd, L.n, L.i, L.o, L.r, code)
    rl.runlora_forward(fwd, dev["X"], dev["W"], dev["A"], dev["B"], Y, saved, workspace=ws)
    dX = torch.full((L.n, L.i), nan, dtype=td, device="cuda") if want_grads[0] else None
    dA = torch.full((L.i, L.r), nan, dtype=td, device="cuda") if want_grads[1] else None
    dB = torch.full((L.r, L.o), nan, dtype=td, device="cuda") if want_grads[2] else None
    rl.runlora_backward(bwd, dev["dY"], saved, dev["W"], dev["A"], dev["B"], dX, dA, dB, workspace=ws)
    torch.cuda.synchronize()
    out = {"Y": to_f64(Y)}
    for k, v in (("dX", dX), ("dA", dA), ("dB", dB)):
        if v is not None:
            out[k] = to_f64(v)
    return out


def reference(host):
    Y = oracle.reference_forward(host["X"], host["W"], host["A"], host["B"])
    dX, dA, dB = oracle.reference_backward(host["X"], host["W"], host["A"], host["B"], host["dY"])
    return {"Y": Y, "dX": dX, "dA": dA, "dB": dB}


def legal_pairs():
    for f, b in itertools.product(rl.FWD_VARIANTS, rl.BWD_VARIANTS):
        if b == rl.BWD_DEFAULT and f != rl.FWD_DEFAULT:
            continue
        yield f, b


def check(L, pairs, b_variance=None):
    dev, host = layer_on_device(L, b_variance)
    want = reference(host)
    for f, b in pairs:
        print(f"case layer={L} fwd={f} bwd={b}", flush=True)
        got = run_pair(L, dev, f, b)
        for k in ("Y", "dX", "dA", "dB"):
            err = relerr(got[k], want[k])
            assert err < TOL[L.dtype], (f, b, k, err)


def test_tiny_fp32_all_pairs():
    """BASELINE config 1: n=256 (2x128), i=o=768, r=8, fp32; every legal forward x backward pair."""
    check(synth.config_tiny_f32()[0], list(legal_pairs()))


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
def test_ragged_shapes_all_pairs(dtype):
    """Token count not a multiple of any tile, d_in != d_out, several tiles in every direction."""
    L = synth.Layer("ragged", 333, 264, 392, 24, dtype, 3)
    check(L, list(legal_pairs()))


@pytest.mark.parametrize("shape", [(1, 8, 8, 8), (7, 16, 8, 8), (130, 8, 264, 8), (129, 520, 8, 16), (64, 72, 72, 64)])
def test_degenerate_shapes(shape):
    """One token, smallest legal dims, rank equal to a dimension."""
    n, i, o, r = shape
    L = synth.Layer("degenerate", n, i, o, r, "bf16", 5)
    check(L, [(1, 1), (2, 5), (0, 0), (1, 4), (2, 3), (1, 2), (3, 1)])


def test_zero_B_gives_zero_dA_and_plain_linear():
    """B = 0: Y = XW, dA = 0 exactly (the standard LoRA initialisation)."""
    import torch
    L = synth.Layer("zeroB", 200, 136, 264, 16, "bf16", 6)
    dev, host = layer_on_device(L)
    dev["B"].zero_()
    host["B"][:] = 0.0
    want = reference(host)
    for f, b in [(1, 1), (2, 5), (0, 0), (1, 3)]:
        got = run_pair(L, dev, f, b)
        assert np.all(got["dA"] == 0.0)
        for k in ("Y", "dX", "dB"):
            assert relerr(got[k], want[k]) < TOL["bf16"], (f, b, k)


def test_skipped_gradients_leave_buffers_alone():
    L = synth.Layer("skip", 150, 72, 136, 8, "f16", 7)
    dev, host = layer_on_device(L)
    want = reference(host)
    for b in (1, 3, 5):
        got = run_pair(L, dev, 1, b, want_grads=(False, True, True))
        assert "dX" not in got
        assert relerr(got["dA"], want["dA"]) < TOL["f16"] and relerr(got["dB"], want["dB"]) < TOL["f16"]
        got = run_pair(L, dev, 1, b, want_grads=(True, False, False))
        assert relerr(got["dX"], want["dX"]) < TOL["f16"]


def test_exact_on_small_integers():
    """Integer-valued inputs small enough that every intermediate is exact in bf16: all graphs must
    return the oracle's values bit for bit."""
    import torch
    rng = np.random.default_rng(2)
    n, i, o, r = 96, 40, 48, 8
    L = synth.Layer("ints", n, i, o, r, "bf16", 0)
    host = {"X": rng.integers(-1, 2, size=(n, i)), "W": rng.integers(-1, 2, size=(i, o)),
            "A": (rng.random((i, r)) < 0.15).astype(np.int64), "B": rng.integers(-1, 2, size=(r, o)),
            "dY": (rng.random((n, o)) < 0.1).astype(np.int64) * rng.integers(-1, 2, size=(n, o))}
    host = {k: v.astype(np.float64) for k, v in host.items()}
    dev = {k: to_device(synth.store(v, "bf16"), "bf16") for k, v in host.items()}
    want = reference(host)
    for k, v in want.items():
        assert np.abs(v).max() <= 256, k
    T = host["X"] @ host["A"]
    Z2 = host["X"].T @ host["dY"]
    assert max(np.abs(T).max(), np.abs(host["dY"] @ host["B"].T).max(), np.abs(Z2).max(),
               np.abs(host["W"] + host["A"] @ host["B"]).max()) <= 256
    for f, b in legal_pairs():
        got = run_pair(L, dev, f, b)
        for k in ("Y", "dX", "dA", "dB"):
            assert np.array_equal(got[k], want[k]), (f, b, k)


@pytest.mark.parametrize("shape,pair", [((1000, 264, 392, 16), (1, 1)), ((1000, 264, 392, 16), (2, 4)),
                                        ((4096, 2048, 2048, 16), (1, 1)), ((4096, 2048, 2048, 16), (2, 3))])
def test_run_to_run_identical(shape, pair):
    """No atomics anywhere: repeated runs give identical bits (token reductions and split contractions are summed
    in a fixed order).  The second shape has 16 x 8 tiles of 256 x 256 at K >= 2048: its Y and dX products run on the
    matrix-core kernel with the contraction split in two, X^T dY on the 128 x 128 tile GEMM with a split, and its
    token reductions split K over workgroups."""
    n, i, o, r = shape
    L = synth.Layer("determinism", n, i, o, r, "bf16", 8)
    dev, _ = layer_on_device(L)
    first = run_pair(L, dev, *pair)
    for _ in range(10):
        again = run_pair(L, dev, *pair)
        for k in first:
            assert np.array_equal(first[k], again[k]), k
