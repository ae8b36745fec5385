"""GPU parity of the one-pass forward (RL_FWD3: forward 1 of Section 2, Y = XW + (XA)B, in a single kernel that
reads X once and never stores XA) against the fp64 oracle: every tile shape its kernel is built in, all three
dtypes, ranks up to its limit of 32, scale and bias, the hand-over to forward 1's two launches beyond the limit,
exactness on small integers, and sampled rows at a full-size layer."""
import numpy as np
import pytest

import oracle
from helpers import TOL, elem_excess, layer_on_device, relerr, to_device, to_f64, torch_dtype
from paper_2312_03415_amd import binding as rl
from paper_2312_03415_amd import synth

pytestmark = pytest.mark.gpu

# (n, i, o, r): the tile shape follows from (n, o): <= 32 / <= 64 rows, <= 32 / <= 64 columns, 128 x 128, and
# 256 x 256 for >= 80 large tiles at d_in >= 2048; ragged in every direction, several K tiles, K tails
SHAPES = [
    (1, 8, 8, 8), (29, 200, 392, 16),        # 32 x 128 tiles
    (64, 72, 264, 32), (50, 136, 136, 8),    # 64 x 128
    (333, 264, 24, 24), (200, 72, 32, 8),    # 128 x 32
    (260, 136, 56, 16), (129, 520, 64, 32),  # 128 x 64
    (333, 264, 392, 24), (130, 8, 264, 8),   # 128 x 128
]


def forward3(L, dev, scale=1.0, bias=None):
    import torch
    td = torch_dtype(L.dtype)
    code = rl.dtype_from_name(L.dtype)
    Y = torch.full((L.n, L.o), float("nan"), dtype=td, device="cuda")
    saved = rl.new_saved()
    ws = rl.new_workspace(rl.FWD3, 1, L.n, L.i, L.o, L.r, code)
    rl.runlora_forward(rl.FWD3, dev["X"], dev["W"], dev["A"], dev["B"], Y, saved, workspace=ws, scale=scale, bias=bias)
    torch.cuda.synchronize()
    return Y, saved, ws


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("shape", SHAPES)
def test_matches_oracle_in_every_tile_shape(shape, dtype):
    n, i, o, r = shape
    if dtype == "f32" and (i % 4 or o % 4 or r % 4):
        pytest.skip("dimension rule")
    L = synth.Layer("onepass", n, i, o, r, dtype, 21)
    print(f"case one-pass forward dtype={dtype} n={n} i={i} o={o} r={r}", flush=True)
    dev, host = layer_on_device(L)
    want = oracle.forward(1, host["X"], host["W"], host["A"], host["B"])[0]
    Y, _, _ = forward3(L, dev)
    got = to_f64(Y)
    assert relerr(got, want) < TOL[dtype]
    assert elem_excess(got, want, dtype) <= 1.0


def test_needs_no_workspace_and_feeds_every_backward():
    """T never reaches memory: the forward needs no scratch; any backward that does not want the kept XA follows."""
    import torch
    L = synth.Layer("onepass", 333, 264, 392, 24, "bf16", 22)
    assert rl.runlora_workspace_bytes(rl.FWD3, -1, L.n, L.i, L.o, L.r, rl.RL_BF16) == 0
    assert rl.runlora_workspace_bytes(rl.FWD1, -1, L.n, L.i, L.o, L.r, rl.RL_BF16) > 0
    dev, host = layer_on_device(L)
    dXw, dAw, dBw = oracle.reference_backward(host["X"], host["W"], host["A"], host["B"], host["dY"])
    for bwd in rl.BWD_VARIANTS:
        if bwd == rl.BWD_DEFAULT:
            continue
        td = torch_dtype(L.dtype)
        Y = torch.empty((L.n, L.o), dtype=td, device="cuda")
        gX, gA, gB = (torch.full(s, float("nan"), dtype=td, device="cuda") for s in ((L.n, L.i), (L.i, L.r), (L.r, L.o)))
        ws = rl.new_workspace(rl.FWD3, bwd, L.n, L.i, L.o, L.r, rl.RL_BF16)
        saved = rl.new_saved()
        rl.runlora_forward(rl.FWD3, dev["X"], dev["W"], dev["A"], dev["B"], Y, saved, workspace=ws)
        rl.runlora_backward(bwd, dev["dY"], saved, dev["W"], dev["A"], dev["B"], gX, gA, gB, workspace=ws)
        torch.cuda.synchronize()
        for got, want in ((gX, dXw), (gA, dAw), (gB, dBw)):
            assert relerr(to_f64(got), want) < TOL["bf16"], bwd


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_scale_and_bias(dtype):
    L = synth.Layer("onepass", 300, 136, 264, 16, dtype, 23)
    dev, host = layer_on_device(L)
    bst = synth.store(synth.normal(synth.BASE_SEED, 98, (L.o,)), dtype)
    bias_dev, bias64 = to_device(bst, dtype), synth.widen(bst, dtype)
    scale = 0.375
    want = oracle.forward(1, host["X"], host["W"], scale * host["A"], host["B"])[0] + bias64[None, :]
    Y, _, _ = forward3(L, dev, scale=scale, bias=bias_dev)
    assert relerr(to_f64(Y), want) < TOL[dtype]
    assert elem_excess(to_f64(Y), want, dtype) <= 1.0


def test_rank_beyond_the_limit_runs_as_forward1():
    """r = 64: the call is served by forward 1's two launches, bit for bit."""
    import torch
    L = synth.Layer("onepass", 260, 136, 264, 64, "bf16", 24)
    dev, host = layer_on_device(L)
    assert rl.runlora_workspace_bytes(rl.FWD3, -1, L.n, L.i, L.o, L.r, rl.RL_BF16) == \
        rl.runlora_workspace_bytes(rl.FWD1, -1, L.n, L.i, L.o, L.r, rl.RL_BF16) > 0
    Y3, _, _ = forward3(L, dev)
    Y1 = torch.empty_like(Y3)
    ws = rl.new_workspace(rl.FWD1, 1, L.n, L.i, L.o, L.r, rl.RL_BF16)
    rl.runlora_forward(rl.FWD1, dev["X"], dev["W"], dev["A"], dev["B"], Y1, rl.new_saved(), workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(Y1, Y3)
    want = oracle.forward(1, host["X"], host["W"], host["A"], host["B"])[0]
    assert relerr(to_f64(Y3), want) < TOL["bf16"]


@pytest.mark.parametrize("shape", [(96, 40, 48, 8), (300, 200, 392, 32), (520, 2048, 520, 24)])
def test_exact_on_small_integers(shape):
    """Integer-valued inputs whose every intermediate (XA included) is exact in bf16: the oracle's values bit for bit."""
    n, i, o, r = shape
    rng = np.random.default_rng(5)
    L = synth.Layer("ints", n, i, o, r, "bf16", 0)
    host = {"X": rng.integers(-1, 2, size=(n, i)) * (rng.random((n, i)) < 0.2), "W": rng.integers(-1, 2, size=(i, o)) * (rng.random((i, o)) < 0.2),
            "A": rng.integers(-1, 2, size=(i, r)) * (rng.random((i, r)) < 0.1), "B": rng.integers(-1, 2, size=(r, o))}
    host = {k: v.astype(np.float64) for k, v in host.items()}
    T = host["X"] @ host["A"]
    want = oracle.forward(1, host["X"], host["W"], host["A"], host["B"])[0]
    assert np.abs(T).max() <= 256 and np.abs(want).max() <= 256 and np.abs(T).max() > 0
    dev = {k: to_device(synth.store(v, "bf16"), "bf16") for k, v in host.items()}
    Y, _, _ = forward3(L, dev)
    assert np.array_equal(to_f64(Y), want)


@pytest.mark.parametrize("r", [8, 32])
def test_llama7b_q_rows(r):
    """n 8192, 4096 -> 4096 (the 256 x 256 tile of the kernel), sampled rows against the oracle."""
    import torch
    L = [x for x in synth.config_llama7b(r, "bf16") if x.name == "q"][0]
    print(f"case one-pass forward full size n={L.n} i={L.i} o={L.o} r={L.r}", flush=True)
    dev, host = layer_on_device(L)
    rows = np.unique(np.concatenate([np.arange(0, L.n, 256), np.arange(255, L.n, 256), np.random.default_rng(3).integers(0, L.n, 32)]))
    want = oracle.reference_rows(host["X"][rows], host["dY"][rows], host["W"], host["A"], host["B"])[0]
    Y, _, _ = forward3(L, dev)
    assert not torch.isnan(Y).any()
    got = to_f64(Y[torch.from_numpy(rows).to("cuda")])
    assert relerr(got, want) < TOL["bf16"]
    assert elem_excess(got, want, "bf16") <= 1.0


@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_large_tile_with_ragged_edges(dtype):
    """9 x 10 tiles of 256 x 256 (the last column of tiles 96 wide) over 32 / 64 K tiles, sampled rows."""
    import torch
    L = synth.Layer("onepass", 2304, 2048, 2400, 16, dtype, 25)
    print(f"case one-pass forward large tile dtype={dtype}", flush=True)
    dev, host = layer_on_device(L)
    rows = np.unique(np.concatenate([np.arange(0, L.n, 256), np.arange(255, L.n, 256), np.random.default_rng(4).integers(0, L.n, 16)]))
    want = oracle.reference_rows(host["X"][rows], host["dY"][rows], host["W"], host["A"], host["B"])[0]
    Y, _, _ = forward3(L, dev)
    assert not torch.isnan(Y).any()
    got = to_f64(Y[torch.from_numpy(rows).to("cuda")])
    assert relerr(got, want) < TOL[dtype]
    assert elem_excess(got, want, dtype) <= 1.0
