"""GPU parity at the full sizes the bench times (and in the launch configuration it uses: the pair
runlora_select picks, the library's own tile and split heuristics): Y and dX on sampled token rows
that the oracle computes one by one (rows of Eq. 1 and of dX in Eq. 3 are independent), dA and dB
in full where that costs the oracle seconds (2n(i+o)r operations), else on sampled columns of dA and
sampled rows of dB (each is X^T (dY b) or (X a)^T dY for one column b of B^T / a of A).  Every compared
tensor must meet the relative Frobenius tolerance and the per-element bound of helpers.elem_excess."""
import numpy as np
import pytest

import oracle
from helpers import TOL, elem_excess, layer_on_device, relerr, to_device, to_f64, torch_dtype
from paper_2312_03415_amd import binding as rl
from paper_2312_03415_amd import synth

pytestmark = pytest.mark.gpu

FULL_GRAD_OPS = 2.5e10   # dA and dB in full up to this many oracle operations (~10 s), sampled beyond


def sample_rows(n, extra, seed):
    """first and last row of every 256-row tile, plus random rows"""
    return np.unique(np.concatenate([np.arange(0, n, 256), np.arange(255, n, 256),
                                     np.random.default_rng(seed).integers(0, n, extra)]))


def grad_reference(L, host):
    """(dA reference, its column index or None), (dB reference, its row index or None)."""
    if 4.0 * L.n * (L.i + L.o) * L.r <= FULL_GRAD_OPS:
        dA = oracle.matmul(host["X"], oracle.matmul(host["dY"], host["B"], tb=True), ta=True)
        dB = oracle.matmul(oracle.matmul(host["X"], host["A"]), host["dY"], ta=True)
        return (dA, None), (dB, None)
    k = np.unique(np.concatenate([[0, L.r - 1], np.random.default_rng(13).integers(0, L.r, 6)]))
    Bk, Ak = np.ascontiguousarray(host["B"][k]), np.ascontiguousarray(host["A"][:, k])
    dA = oracle.matmul(host["X"], oracle.matmul(host["dY"], Bk, tb=True), ta=True)     # columns k of dA
    dB = oracle.matmul(oracle.matmul(host["X"], Ak), host["dY"], ta=True)              # rows k of dB
    return (dA, k), (dB, k)


def compare(tag, got, want, dtype, per_row=True, roundings=1):
    err, exc = relerr(got, want), elem_excess(got, want, dtype, per_row, roundings)
    print(f"   {tag}: rel. Frobenius {err:.2e} (tol {TOL[dtype]:.0e}), worst element at {exc:.2f} of its bound", flush=True)
    assert err < TOL[dtype], (tag, err)
    assert exc <= 1.0, (tag, exc)


def check_layer(L, pairs, extra_rows=32):
    import torch
    dev, host = layer_on_device(L)
    code = rl.dtype_from_name(L.dtype)
    td = torch_dtype(L.dtype)
    rows = sample_rows(L.n, extra_rows, 11)
    Yr, dXr = oracle.reference_rows(host["X"][rows], host["dY"][rows], host["W"], host["A"], host["B"])
    (dA, ka), (dB, kb) = grad_reference(L, host)
    for fwd, bwd in pairs:
        print(f"case full-size layer={L.name} dtype={L.dtype} n={L.n} i={L.i} o={L.o} r={L.r} fwd={fwd} bwd={bwd}", flush=True)
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
        # the default chain stores Y = XW and dX = dY W^T before it adds the rank-r term: two roundings
        compare(f"({fwd},{bwd}) Y", to_f64(Y[idx]), Yr, L.dtype, roundings=2 if fwd == 0 else 1)
        compare(f"({fwd},{bwd}) dX", to_f64(gX[idx]), dXr, L.dtype, roundings=2 if bwd == 0 else 1)
        compare(f"({fwd},{bwd}) dA", to_f64(gA) if ka is None else to_f64(gA)[:, ka], dA, L.dtype, per_row=False)
        compare(f"({fwd},{bwd}) dB", to_f64(gB) if kb is None else to_f64(gB)[kb], dB, L.dtype, per_row=False)
        # every tile was written
        assert not torch.isnan(Y).any() and not torch.isnan(gX).any() and not torch.isnan(gA).any() and not torch.isnan(gB).any()


@pytest.mark.parametrize("which", [0, 1])
def test_opt13b_mlp_layer(which):
    """bench.py --workload opt13b: the selected pair, the default chain, and both merged graphs."""
    L = synth.config_opt13b_mlp("bf16")[which]
    sel = rl.runlora_select(L.n, L.i, L.o, L.r, rl.RL_BF16)
    check_layer(L, sorted({sel, (0, 0), (2, 5), (1, 1)}))


@pytest.mark.parametrize("name", ["q", "gate", "down"])
def test_llama7b_layer(name):
    """bench.py's default workload (rank 32): the selected pair and the default chain."""
    L = [x for x in synth.config_llama7b(32, "bf16") if x.name == name][0]
    sel = rl.runlora_select(L.n, L.i, L.o, L.r, rl.RL_BF16)
    check_layer(L, sorted({sel, (0, 0)}))


@pytest.mark.parametrize("name", ["q", "gate", "down"])
@pytest.mark.parametrize("r", [8, 128])
def test_llama7b_other_ranks(name, r):
    """The smallest and the largest rank of the Llama-7B configuration on each of its three layer shapes: r = 8
    is a quarter of a K tile in the concatenated contraction, r = 128 the widest rank-r product of the
    streaming kernel."""
    L = [x for x in synth.config_llama7b(r, "bf16") if x.name == name][0]
    sel = rl.runlora_select(L.n, L.i, L.o, L.r, rl.RL_BF16)
    check_layer(L, sorted({sel, (1, 1), (2, 5)}) if name == "q" else sorted({sel, (1, 1)}), extra_rows=0 if name != "q" else 32)


@pytest.mark.parametrize("n,r", [(16384, 256), (16384, 1024), (128, 1024), (1024, 64)])
def test_selector_sweep_shapes(n, r):
    """Shapes of the fp16 crossover sweep (d_in = d_out = 4096) that the selector test only times: the most
    tokens, and ranks beyond the streaming kernel's 128 columns (rank-r products on the 128x128 tile GEMM,
    W + AB through the tile GEMM's addend path).  The selected pair, forward2 with Algorithm 4 (X^T dY at full
    size) and forward1 with Algorithm 3."""
    L = [x for x in synth.config_selector_sweep("f16") if x.n == n and x.r == r][0]
    sel = rl.runlora_select(L.n, L.i, L.o, L.r, rl.RL_F16)
    check_layer(L, sorted({sel, (2, 4), (1, 3)}), extra_rows=8)


def test_llama7b_gate_with_scale_and_bias():
    """The 4096 -> 11008 layer (its Y GEMM is cut into a main launch and a split-K tail launch) with a
    LoRA scale and a frozen bias: the bias must reach both launches and the tail's reduce."""
    import torch
    L = [x for x in synth.config_llama7b(32, "bf16") if x.name == "gate"][0]
    dev, host = layer_on_device(L)
    bst = synth.store(synth.normal(synth.BASE_SEED, 99, (L.o,)), L.dtype)
    bias_dev, bias64 = to_device(bst, L.dtype), synth.widen(bst, L.dtype)
    scale = 0.25
    rows = sample_rows(L.n, 32, 12)
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
        compare(f"({fwd},{bwd}) Y", to_f64(Y[idx]), Yr, L.dtype)
        compare(f"({fwd},{bwd}) dX", to_f64(gX[idx]), dXr, L.dtype)
        assert not torch.isnan(Y).any() and not torch.isnan(gX).any()


def test_llama7b_gate_exact_on_small_integers():
    """Bit-exact check at a bench size, in the bench's launch configuration.  Inputs are small integers, sparse
    enough that every intermediate the graphs store in bf16 (T = XA, Z1 = dY B^T, W + AB, X^T dY) is an integer of
    at most 256 in magnitude, hence exact; every fp32 partial sum is an integer below 2^24, hence exact in any
    order; so each output must equal the oracle's exact value rounded once to bf16, bit for bit.  The 4096 -> 11008
    shape with r = 8 runs the short-epilogue build of the matrix-core kernel over several tiles per workgroup, the
    cut-off tile columns with their split contraction and its reduce, the concatenated contraction with a second
    segment of 8, X^T dY at full size, and the 64-row build of the streaming kernel; one wrong 16-byte fragment
    anywhere changes an integer."""
    import torch
    rng = np.random.default_rng(5)
    n, i, o, r = 8192, 4096, 11008, 8
    L = synth.Layer("gate_ints", n, i, o, r, "bf16", 0)

    def sparse(shape, p):
        return ((rng.random(shape) < p) * rng.choice([-1.0, 1.0], size=shape)).astype(np.float64)

    host = {"X": sparse((n, i), 0.5), "W": sparse((i, o), 0.25), "A": sparse((i, r), 0.02), "B": sparse((r, o), 0.5),
            "dY": sparse((n, o), 0.02)}
    dev = {k: to_device(synth.store(v, "bf16"), "bf16") for k, v in host.items()}
    rows = np.unique(np.concatenate([[0, 255, 256, n - 256, n - 1], rng.integers(0, n, 19)]))
    Yr, dXr = oracle.reference_rows(host["X"][rows], host["dY"][rows], host["W"], host["A"], host["B"])
    T = oracle.matmul(host["X"], host["A"])
    Z1 = oracle.matmul(host["dY"], host["B"], tb=True)
    dA = oracle.matmul(host["X"], Z1, ta=True)
    dB = oracle.matmul(T, host["dY"], ta=True)
    M = host["W"] + oracle.matmul(host["A"], host["B"])
    # intermediates kept in bf16 must be exact there; X^T dY is checked on a sample of its rows (its entries are
    # sums of n products of which ~1 % are non-zero: |.| stays far below 256)
    z2rows = rng.integers(0, i, 16)
    Z2s = oracle.matmul(np.ascontiguousarray(host["X"][:, z2rows]), host["dY"], ta=True)
    assert max(np.abs(T).max(), np.abs(Z1).max(), np.abs(M).max(), np.abs(Z2s).max()) <= 256
    assert max(np.abs(dA).max(), np.abs(dB).max(), np.abs(Yr).max(), np.abs(dXr).max()) < 2 ** 24

    def rounded(a):  # the oracle's exact value, rounded once to bf16
        return synth.widen(synth.store(a, "bf16"), "bf16")

    td = torch.bfloat16
    for fwd, bwd in [(1, 1), (2, 5), (2, 4), (0, 0), (1, 3)]:
        print(f"case exact-integers gate shape fwd={fwd} bwd={bwd}", flush=True)
        Y = torch.full((n, o), float("nan"), dtype=td, device="cuda")
        Tb = torch.full((n, r), float("nan"), dtype=td, device="cuda") if fwd == 0 else None
        gX = torch.full((n, i), float("nan"), dtype=td, device="cuda")
        gA = torch.full((i, r), float("nan"), dtype=td, device="cuda")
        gB = torch.full((r, o), float("nan"), dtype=td, device="cuda")
        ws = rl.new_workspace(fwd, bwd, n, i, o, r, rl.RL_BF16)
        saved = rl.new_saved(Tb)
        rl.runlora_forward(fwd, dev["X"], dev["W"], dev["A"], dev["B"], Y, saved, workspace=ws)
        rl.runlora_backward(bwd, dev["dY"], saved, dev["W"], dev["A"], dev["B"], gX, gA, gB, workspace=ws)
        torch.cuda.synchronize()
        idx = torch.from_numpy(rows).to("cuda")
        assert np.array_equal(to_f64(Y[idx]), rounded(Yr)), (fwd, bwd, "Y")
        assert np.array_equal(to_f64(gX[idx]), rounded(dXr)), (fwd, bwd, "dX")
        assert np.array_equal(to_f64(gA), rounded(dA)), (fwd, bwd, "dA")
        assert np.array_equal(to_f64(gB), rounded(dB)), (fwd, bwd, "dB")
        assert not torch.isnan(Y).any() and not torch.isnan(gX).any()
