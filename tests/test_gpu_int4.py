"""GPU parity for a frozen W stored as symmetric int4 with group-of-64 fp16 scales (the quantised
configuration of the task; the paper mentions quantised weights in one sentence of Section 1):
every graph that does not need W + AB as a matrix, through the C ABI, against the fp64 oracle
evaluated on the dequantised W = q * scale."""
import numpy as np
import pytest

import oracle
from helpers import TOL, relerr, to_device, to_f64, torch_dtype
from paper_2312_03415_amd import binding as rl
from paper_2312_03415_amd import synth

pytestmark = pytest.mark.gpu

PAIRS = [(0, 0), (1, 1), (1, 2), (1, 3), (0, 0), (1, 1)]


def make_layer(L, q=None, scale=None):
    st = synth.layer_inputs(L)
    if q is None:
        q, scale = synth.int4_weight(L)
    dev = {k: to_device(v, L.dtype) for k, v in st.items() if k != "W"}
    host = {k: synth.widen(v, L.dtype) for k, v in st.items() if k != "W"}
    dev["W"] = rl.Int4Weight.from_host(q, scale)
    host["W"] = oracle.dequant_int4(q, scale.astype(np.float64))
    return dev, host


def run_pair(L, dev, fwd, bwd):
    import torch
    td = torch_dtype(L.dtype)
    code = rl.dtype_from_name(L.dtype)
    nan = float("nan")
    Y = torch.full((L.n, L.o), nan, dtype=td, device="cuda")
    T = torch.full((L.n, L.r), nan, dtype=td, device="cuda") if fwd == 0 else None
    saved = rl.new_saved(T)
    ws = rl.new_workspace(fwd, bwd, L.n, L.i, L.o, L.r, code, w_dtype=rl.RL_INT4_G64)
    rl.runlora_forward(fwd, dev["X"], dev["W"], dev["A"], dev["B"], Y, saved, workspace=ws)
    dX = torch.full((L.n, L.i), nan, dtype=td, device="cuda")
    dA = torch.full((L.i, L.r), nan, dtype=td, device="cuda")
    dB = torch.full((L.r, L.o), nan, dtype=td, device="cuda")
    rl.runlora_backward(bwd, dev["dY"], saved, dev["W"], dev["A"], dev["B"], dX, dA, dB, workspace=ws)
    torch.cuda.synchronize()
    return {"Y": to_f64(Y), "dX": to_f64(dX), "dA": to_f64(dA), "dB": to_f64(dB)}


def reference(host):
    Y = oracle.reference_forward(host["X"], host["W"], host["A"], host["B"])
    dX, dA, dB = oracle.reference_backward(host["X"], host["W"], host["A"], host["B"], host["dY"])
    return {"Y": Y, "dX": dX, "dA": dA, "dB": dB}


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("shape", [(333, 264, 392, 24), (70, 72, 136, 8), (600, 520, 328, 16)])
def test_int4_weight_all_supported_pairs(shape, dtype):
    """Ragged shapes: d_in not a multiple of the group (a partial last group), several tiles."""
    n, i, o, r = shape
    L = synth.Layer("int4", n, i, o, r, dtype, 9)
    dev, host = make_layer(L)
    want = reference(host)
    for f, b in [(0, 0), (1, 1), (1, 2), (1, 3)]:
        print(f"case int4 shape={shape} dtype={dtype} fwd={f} bwd={b}", flush=True)
        got = run_pair(L, dev, f, b)
        for k in ("Y", "dX", "dA", "dB"):
            assert relerr(got[k], want[k]) < TOL[dtype], (f, b, k, relerr(got[k], want[k]))


def test_int4_merged_graphs_are_refused():
    L = synth.Layer("int4", 64, 64, 64, 8, "bf16", 9)
    dev, _ = make_layer(L)
    import torch
    Y = torch.empty((L.n, L.o), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    with pytest.raises(rl.RunLoRAError) as e:
        rl.runlora_forward(2, dev["X"], dev["W"], dev["A"], dev["B"], Y, rl.new_saved(), workspace=ws)
    assert e.value.code == rl.RL_ERR_UNSUPPORTED
    saved = rl.new_saved()
    rl.runlora_forward(1, dev["X"], dev["W"], dev["A"], dev["B"], Y, saved, workspace=ws)
    dX = torch.empty((L.n, L.i), dtype=torch.bfloat16, device="cuda")
    for bwd in (4, 5):
        with pytest.raises(rl.RunLoRAError) as e:
            rl.runlora_backward(bwd, dev["dY"], saved, dev["W"], dev["A"], dev["B"], dX, None, None, workspace=ws)
        assert e.value.code == rl.RL_ERR_UNSUPPORTED


def test_int4_exact_with_unit_scales():
    """scales = 1 and small integer inputs: every product is an exact integer, so the GPU must
    return the oracle's values bit for bit (the integer GEMM check of the quantised path)."""
    rng = np.random.default_rng(4)
    n, i, o, r = 96, 136, 72, 8
    L = synth.Layer("int4ints", n, i, o, r, "bf16", 0)
    q = rng.integers(-7, 8, size=(i, o)).astype(np.int8)
    scale = np.ones(((i + 63) // 64, o), dtype=np.float16)
    host = {"X": (rng.random((n, i)) < 0.1) * rng.integers(-1, 2, size=(n, i)),
            "A": (rng.random((i, r)) < 0.1).astype(np.int64), "B": rng.integers(-1, 2, size=(r, o)),
            "dY": (rng.random((n, o)) < 0.08) * rng.integers(-1, 2, size=(n, o))}
    host = {k: v.astype(np.float64) for k, v in host.items()}
    dev = {k: to_device(synth.store(v, "bf16"), "bf16") for k, v in host.items()}
    dev["W"] = rl.Int4Weight.from_host(q, scale)
    host["W"] = oracle.dequant_int4(q, scale.astype(np.float64))
    want = reference(host)
    for v in want.values():
        assert np.abs(v).max() <= 256
    for f, b in [(0, 0), (1, 1), (1, 3)]:
        got = run_pair(L, dev, f, b)
        for k in ("Y", "dX", "dA", "dB"):
            assert np.array_equal(got[k], want[k]), (f, b, k)


def test_int4_config_shape_sampled_rows():
    """The quantised configuration at its full size (n 4096, 5120 -> 13824, r 64, bf16): Y and dX on
    sampled token rows (rows are independent), dA and dB in full."""
    L = synth.config_qlora()[0]
    dev, host = make_layer(L)
    rows = np.unique(np.concatenate([np.arange(0, L.n, 256), np.arange(255, L.n, 256),
                                     np.random.default_rng(5).integers(0, L.n, 32)]))
    got = run_pair(L, dev, 1, 1)
    Yr, dXr = oracle.reference_rows(host["X"][rows], host["dY"][rows], host["W"], host["A"], host["B"])
    assert relerr(got["Y"][rows], Yr) < TOL["bf16"]
    assert relerr(got["dX"][rows], dXr) < TOL["bf16"]
    Z1 = oracle.matmul(host["dY"], host["B"], tb=True)
    assert relerr(got["dA"], oracle.matmul(host["X"], Z1, ta=True)) < TOL["bf16"]
    Tm = oracle.matmul(host["X"], host["A"])
    assert relerr(got["dB"], oracle.matmul(Tm, host["dY"], ta=True)) < TOL["bf16"]


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_int4_matrix_core_route_ragged(dtype):
    """Large enough for the matrix-core kernel's int4 route (>= 160 tiles of 256x256) and ragged in
    every direction: n not a multiple of the tile, d_in = 32*64 + 8 (a partial last K tile and a
    partial last scale group for X W), d_out = 32*112 + 8 (the same for dY W^T), r = 24 (a partial K
    tile in the dense second segment).  Y and dX on sampled rows (first and last row of every tile
    row, plus random ones), dA and dB in full; also the default chain, whose dX GEMM has no second
    segment."""
    L = synth.Layer("int4mc", 3001, 2056, 3592, 24, dtype, 12)
    dev, host = make_layer(L)
    rows = np.unique(np.concatenate([np.arange(0, L.n, 256), np.arange(255, L.n, 256), [L.n - 1],
                                     np.random.default_rng(6).integers(0, L.n, 24)]))
    Yr, dXr = oracle.reference_rows(host["X"][rows], host["dY"][rows], host["W"], host["A"], host["B"])
    dA = oracle.matmul(host["X"], oracle.matmul(host["dY"], host["B"], tb=True), ta=True)
    dB = oracle.matmul(oracle.matmul(host["X"], host["A"]), host["dY"], ta=True)
    for f, b in [(1, 1), (0, 0)]:
        print(f"case int4 matrix-core dtype={dtype} fwd={f} bwd={b}", flush=True)
        got = run_pair(L, dev, f, b)
        assert not np.isnan(got["Y"]).any() and not np.isnan(got["dX"]).any()
        assert relerr(got["Y"][rows], Yr) < TOL[dtype], (f, b)
        assert relerr(got["dX"][rows], dXr) < TOL[dtype], (f, b)
        assert relerr(got["dA"], dA) < TOL[dtype] and relerr(got["dB"], dB) < TOL[dtype]


def test_int4_matrix_core_route_with_scale_and_bias():
    """The int4 route's epilogue and the dense second segment with a LoRA scale and a bias."""
    import torch
    L = synth.Layer("int4mcs", 3001, 2056, 3592, 24, "bf16", 13)
    dev, host = make_layer(L)
    bst = synth.store(synth.normal(synth.BASE_SEED, 98, (L.o,)), L.dtype)
    bias_dev, bias64 = to_device(bst, L.dtype), synth.widen(bst, L.dtype)
    scale = 0.5
    rows = np.unique(np.concatenate([np.arange(0, L.n, 256), [L.n - 1], np.random.default_rng(7).integers(0, L.n, 24)]))
    Yr, dXr = oracle.scaled_rows(host["X"][rows], host["dY"][rows], host["W"], host["A"], host["B"], scale, bias64)
    code = rl.dtype_from_name(L.dtype)
    Y = torch.full((L.n, L.o), float("nan"), dtype=torch.bfloat16, device="cuda")
    gX = torch.full((L.n, L.i), float("nan"), dtype=torch.bfloat16, device="cuda")
    gA = torch.full((L.i, L.r), float("nan"), dtype=torch.bfloat16, device="cuda")
    gB = torch.full((L.r, L.o), float("nan"), dtype=torch.bfloat16, device="cuda")
    ws = rl.new_workspace(1, 1, L.n, L.i, L.o, L.r, code, w_dtype=rl.RL_INT4_G64)
    saved = rl.new_saved()
    rl.runlora_forward(1, dev["X"], dev["W"], dev["A"], dev["B"], Y, saved, workspace=ws, scale=scale, bias=bias_dev)
    rl.runlora_backward(1, dev["dY"], saved, dev["W"], dev["A"], dev["B"], gX, gA, gB, workspace=ws)
    torch.cuda.synchronize()
    assert relerr(to_f64(Y)[rows], Yr) < TOL["bf16"] and relerr(to_f64(gX)[rows], dXr) < TOL["bf16"]
    Z1 = scale * oracle.matmul(host["dY"], host["B"], tb=True)
    assert relerr(to_f64(gA), oracle.matmul(host["X"], Z1, ta=True)) < TOL["bf16"]
    Tm = scale * oracle.matmul(host["X"], host["A"])
    assert relerr(to_f64(gB), oracle.matmul(Tm, host["dY"], ta=True)) < TOL["bf16"]

