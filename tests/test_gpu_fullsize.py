"""GPU parity at the full sizes the bench times (and in the launch configuration it uses: the pair
runlora_select picks, the library's own tile and split heuristics): Y and dX on sampled token rows
that the oracle computes one by one (rows of Eq. 1 and of dX in Eq. 3 are independent), dA and dB
in full (they cost only 2n(i+o)r)."""
import numpy as np
import pytest

import oracle
from helpers import TOL, layer_on_device, relerr, to_f64, torch_dtype
from paper_2312_03415_amd import binding as rl
from paper_2312_03415_amd import synth

pytestmark = pytest.mark.gpu


def check_layer(L, pairs):
    import torch
    dev, host = layer_on_device(L)
    code = rl.dtype_from_name(L.dtype)
    td = torch_dtype(L.dtype)
    # first and last row of every 256-row tile, plus random rows
    rows = np.unique(np.concatenate([np.arange(0, L.n, 256), np.arange(255, L.n, 256),
                                     np.random.default_rng(11).integers(0, L.n, 32)]))
    Yr, dXr = oracle.reference_rows(host["X"][rows], host["dY"][rows], host["W"], host["A"], host["B"])
    dA = oracle.matmul(host["X"], oracle.matmul(host["dY"], host["B"], tb=True), ta=True)
    dB = oracle.matmul(oracle.matmul(host["X"], host["A"]), host["dY"], ta=True)
    for fwd, bwd in pairs:
        print(f"case full-size layer={L.name} n={L.n} i={L.i} o={L.o} r={L.r} fwd={fwd} bwd={bwd}", flush=True)
        nan = float("nan")
        Y = torch.full((L.n, L.o), nan, dtype=td, device="cuda")
        T = torch.full((L.n, L.r), nan, dtype=td, device="cuda") if fwd == 0 else None
        gX = torch.full((L.n, L.i), nan, dtype=td, device="cuda")
        gA = torch.full((L.i, L.r), nan, dtype=td, device="cuda")
        gB = torch.full((L.r, L.o), nan, dtype=td, device="cuda")
        ws = rl.new_workspace(fwd, bwd, L.n, L.i, L.o, L.r, code)
        saved = rl.new_saved(T)
        rl.runlora_forward(fwd, dev["X"], dev["W"], dev["A"], dev["B"], Y, saved, workspace=ws)
        rl.runlora_backward(bwd, dev["dY"], saved, dev["W"], dev["A"], dev["B"], gX, gA, gB, workspace=ws)
        torch.cuda.synchronize()
        idx = torch.from_numpy(rows).to("cuda")
        assert relerr(to_f64(Y[idx]), Yr) < TOL[L.dtype], (fwd, bwd, "Y")
        assert relerr(to_f64(gX[idx]), dXr) < TOL[L.dtype], (fwd, bwd, "dX")
        assert relerr(to_f64(gA), dA) < TOL[L.dtype], (fwd, bwd, "dA")
        assert relerr(to_f64(gB), dB) < TOL[L.dtype], (fwd, bwd, "dB")
        assert not torch.isnan(Y).any() and not torch.isnan(gX).any()   # every tile was written


@pytest.mark.parametrize("which", [0, 1])
def test_opt13b_mlp_layer(which):
    """bench.py's default workload: the selected pair, the default chain, and both merged graphs."""
    L = synth.config_opt13b_mlp("bf16")[which]
    sel = rl.runlora_select(L.n, L.i, L.o, L.r, rl.RL_BF16)
    check_layer(L, sorted({sel, (0, 0), (2, 5), (1, 1)}))


@pytest.mark.parametrize("name", ["q", "gate", "down"])
def test_llama7b_layer(name):
    L = [x for x in synth.config_llama7b(32, "bf16") if x.name == name][0]
    sel = rl.runlora_select(L.n, L.i, L.o, L.r, rl.RL_BF16)
    check_layer(L, sorted({sel, (0, 0)}))


@pytest.mark.parametrize("r", [8, 128])
def test_llama7b_q_other_ranks(r):
    """The smallest and the largest rank of the Llama-7B configuration: r = 8 is a quarter of a K tile
    in the concatenated contraction, r = 128 the widest rank-r product of the streaming kernel."""
    L = [x for x in synth.config_llama7b(r, "bf16") if x.name == "q"][0]
    sel = rl.runlora_select(L.n, L.i, L.o, L.r, rl.RL_BF16)
    check_layer(L, sorted({sel, (1, 1), (2, 5)}))


def test_llama7b_gate_with_scale_and_bias():
    """The 4096 -> 11008 layer (its Y GEMM is cut into a main launch and a split-K tail launch) with a
    LoRA scale and a frozen bias: the bias must reach both launches and the tail's reduce."""
    import torch
    from helpers import to_device
    L = [x for x in synth.config_llama7b(32, "bf16") if x.name == "gate"][0]
    dev, host = layer_on_device(L)
    bst = synth.store(synth.normal(synth.BASE_SEED, 99, (L.o,)), L.dtype)
    bias_dev, bias64 = to_device(bst, L.dtype), synth.widen(bst, L.dtype)
    scale = 0.25
    rows = np.unique(np.concatenate([np.arange(0, L.n, 256), np.arange(255, L.n, 256),
                                     np.random.default_rng(12).integers(0, L.n, 32)]))
    Yr, dXr = oracle.scaled_rows(host["X"][rows], host["dY"][rows], host["W"], host["A"], host["B"], scale, bias64)
    td = torch_dtype(L.dtype)
    code = rl.dtype_from_name(L.dtype)
    for fwd, bwd in [(1, 1), (2, 5)]:
        Y = torch.full((L.n, L.o), float("nan"), dtype=td, device="cuda")
        gX = torch.full((L.n, L.i), float("nan"), dtype=td, device="cuda")
        ws = rl.new_workspace(fwd, bwd, L.n, L.i, L.o, L.r, code)
        saved = rl.new_saved()
        rl.runlora_forward(fwd, dev["X"], dev["W"], dev["A"], dev["B"], Y, saved, workspace=ws, scale=scale, bias=bias_dev)
        rl.runlora_backward(bwd, dev["dY"], saved, dev["W"], dev["A"], dev["B"], gX, None, None, workspace=ws)
        torch.cuda.synchronize()
        idx = torch.from_numpy(rows).to("cuda")
        assert relerr(to_f64(Y[idx]), Yr) < TOL[L.dtype], (fwd, bwd)
        assert relerr(to_f64(gX[idx]), dXr) < TOL[L.dtype], (fwd, bwd)
        assert not torch.isnan(Y).any() and not torch.isnan(gX).any()
