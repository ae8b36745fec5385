"""GPU: the tile GEMM behind every step, each tile shape x operand layout x dtype, on ragged shapes
that span several tiles, against the oracle's naive fp64 matmul (through the C ABI)."""
import numpy as np
import pytest

import oracle
from helpers import elem_excess, TOL, relerr, to_device, to_f64, torch_dtype
from paper_2312_03415_amd import binding as rl
from paper_2312_03415_amd import synth

pytestmark = pytest.mark.gpu

LAYOUTS = {"NN": (False, False), "NT": (False, True), "TN": (True, False)}
# (M, N, K) per tile config: more than one tile each way, ragged last tile, ragged last K tile
SHAPES = {
    0: (600, 520, 328),   # 256x256
    1: (300, 264, 200),   # 128x128
    2: (300, 24, 200),    # 128x32
    3: (300, 56, 200),    # 128x64
    4: (24, 264, 456),    # 32x128
    5: (56, 264, 456),    # 64x128
    6: (600, 520, 328),   # 256x256, matrix-core kernel (fp32 falls back to config 0)
    7: (600, 520, 328),   # 256x256, matrix-core kernel, shorter epilogue where the call allows it
}


def make(seed, stream, shape, dtype, var=1.0):
    st = synth.store(synth.normal(seed, stream, shape, var), dtype)
    return to_device(st, dtype), synth.widen(st, dtype)


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("layout", list(LAYOUTS))
@pytest.mark.parametrize("cfg", list(SHAPES))
def test_gemm_tile_configs(cfg, layout, dtype):
    import torch
    a_str, b_kc = LAYOUTS[layout]
    M, N, K = SHAPES[cfg]
    if a_str:
        M = (M + 7) // 8 * 8   # a [K,M] operand needs M to be a multiple of 8
    print(f"case cfg={cfg} layout={layout} dtype={dtype} M={M} N={N} K={K}", flush=True)
    A, Ah = make(3, 1, (K, M) if a_str else (M, K), dtype)
    B, Bh = make(3, 2, (N, K) if b_kc else (K, N), dtype, 1.0 / K)
    want = oracle.matmul(Ah, Bh, ta=a_str, tb=b_kc)
    C = torch.full((M, N), float("nan"), dtype=torch_dtype(dtype), device="cuda")
    rl.runlora_gemm(A, B, C, a_strided=a_str, b_kcontig=b_kc, tile_cfg=cfg, splits=1)
    torch.cuda.synchronize()
    assert relerr(to_f64(C), want) < TOL[dtype]
    # split contraction (fp32 partials + ordered reduce) and an addend
    D, Dh = make(3, 3, (M, N), dtype)
    C2 = torch.full((M, N), float("nan"), dtype=torch_dtype(dtype), device="cuda")
    rl.runlora_gemm(A, B, C2, a_strided=a_str, b_kcontig=b_kc, D=D, tile_cfg=cfg, splits=3)
    torch.cuda.synchronize()
    assert relerr(to_f64(C2), want + Dh) < TOL[dtype]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("layout", ["NN", "NT"])
def test_gemm_two_segments_and_heuristic_plan(layout, dtype):
    """[A|A2][B;B2] with a short second segment (the K-concatenated LoRA term), plan left to the library."""
    import torch
    a_str, b_kc = LAYOUTS[layout]
    M, N, K, K2 = 333, 264, 200, 24
    print(f"case two-seg layout={layout} dtype={dtype}", flush=True)
    A, Ah = make(5, 1, (M, K), dtype)
    A2, A2h = make(5, 2, (M, K2), dtype)
    B, Bh = make(5, 3, (N, K) if b_kc else (K, N), dtype, 1.0 / K)
    B2, B2h = make(5, 4, (N, K2) if b_kc else (K2, N), dtype, 1.0 / K2)
    want = oracle.matmul(Ah, Bh, tb=b_kc) + oracle.matmul(A2h, B2h, tb=b_kc)
    for cfg in (-1, 0, 1, 6, 7):
        C = torch.full((M, N), float("nan"), dtype=torch_dtype(dtype), device="cuda")
        rl.runlora_gemm(A, B, C, b_kcontig=b_kc, A2=A2, B2=B2, tile_cfg=cfg)
        torch.cuda.synchronize()
        assert relerr(to_f64(C), want) < TOL[dtype], cfg
        # contraction split across both segments
        C = torch.full((M, N), float("nan"), dtype=torch_dtype(dtype), device="cuda")
        rl.runlora_gemm(A, B, C, b_kcontig=b_kc, A2=A2, B2=B2, tile_cfg=cfg, splits=2)
        torch.cuda.synchronize()
        assert relerr(to_f64(C), want) < TOL[dtype], (cfg, "split")


def test_gemm_exact_on_small_integers():
    """Integer-valued inputs are exact in every dtype and every accumulation order: bit-exact result."""
    import torch
    rng = np.random.default_rng(0)
    M, N, K = 130, 72, 96
    for dtype in ("bf16", "f16", "f32"):
        Ah = rng.integers(-3, 4, size=(M, K)).astype(np.float64)
        Bh = rng.integers(-3, 4, size=(K, N)).astype(np.float64)
        A = to_device(synth.store(Ah, dtype), dtype)
        B = to_device(synth.store(Bh, dtype), dtype)
        want = oracle.matmul(Ah, Bh)
        assert np.abs(want).max() < 256          # representable in bf16's 8-bit significand
        for cfg in (0, 1, 2, 3, 6, 7):
            C = torch.empty((M, N), dtype=torch_dtype(dtype), device="cuda")
            rl.runlora_gemm(A, B, C, tile_cfg=cfg, splits=2)
            torch.cuda.synchronize()
            assert np.array_equal(to_f64(C), want), (dtype, cfg)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("layout", list(LAYOUTS))
def test_matrix_core_builds_exact_on_small_integers(layout, dtype):
    """Every build of the matrix-core kernel on integer-valued inputs, bit for bit against the oracle: 512 x 768
    outputs (2 x 3 whole tiles: the short epilogue; with the contraction split in two: the fp32-partials epilogue;
    with a bias of zeros: the general epilogue), 520 x 776 (ragged tiles), K = 32 * 8 + 8 (a partial last K
    tile) and a second segment of 8."""
    import torch
    a_str, b_kc = LAYOUTS[layout]
    rng = np.random.default_rng(4)
    K, K2 = 264, 8
    td = torch_dtype(dtype)
    for M, N in ((512, 768), (520, 776)):
        Ah = rng.integers(-2, 3, size=(K, M) if a_str else (M, K)).astype(np.float64)
        Bh = rng.integers(-2, 3, size=(N, K) if b_kc else (K, N)).astype(np.float64)
        A2h = rng.integers(-2, 3, size=(K2, M) if a_str else (M, K2)).astype(np.float64)
        B2h = rng.integers(-2, 3, size=(N, K2) if b_kc else (K2, N)).astype(np.float64)
        A, B, A2, B2 = (to_device(synth.store(v, dtype), dtype) for v in (Ah, Bh, A2h, B2h))
        want = oracle.matmul(Ah, Bh, ta=a_str, tb=b_kc) + oracle.matmul(A2h, B2h, ta=a_str, tb=b_kc)
        assert np.abs(want).max() <= 256   # exact in bf16's 8-bit significand
        zero_bias = torch.zeros(N, dtype=td, device="cuda")
        for cfg in (6, 7):   # K tile 32 / K tile 64 where that kernel has the build (else it runs as 6)
            for splits, bias in ((1, None), (2, None), (1, zero_bias), (3, zero_bias)):
                print(f"case mc-exact layout={layout} dtype={dtype} M={M} N={N} cfg={cfg} splits={splits} bias={bias is not None}", flush=True)
                C = torch.full((M, N), float("nan"), dtype=td, device="cuda")
                rl.runlora_gemm(A, B, C, a_strided=a_str, b_kcontig=b_kc, A2=A2, B2=B2, tile_cfg=cfg, splits=splits, bias=bias)
                torch.cuda.synchronize()
                assert np.array_equal(to_f64(C), want), (M, N, cfg, splits, bias is not None)


def test_gemm_strided_rows_and_aliased_addend():
    """Leading dimensions larger than the row length; D aliasing C (the '+=' of the default chain)."""
    import torch
    dtype = "bf16"
    M, N, K = 200, 136, 72
    Abuf, Abh = make(9, 1, (M, K + 24), dtype)
    Bbuf, Bbh = make(9, 2, (K, N + 8), dtype, 1.0 / K)
    Cbuf, Cbh = make(9, 3, (M, N + 16), dtype)
    A, B, C = Abuf[:, :K], Bbuf[:, :N], Cbuf[:, :N]
    want = oracle.matmul(Abh[:, :K].copy(), Bbh[:, :N].copy()) + Cbh[:, :N]
    rl.runlora_gemm(A, B, C, D=C)
    torch.cuda.synchronize()
    assert relerr(to_f64(C), want) < TOL[dtype]
    assert np.array_equal(to_f64(Cbuf[:, N:]), Cbh[:, N:])      # padding columns untouched


@pytest.mark.parametrize("cfg", [6, 7])
@pytest.mark.parametrize("layout", list(LAYOUTS))
def test_matrix_core_kernels_with_padded_leading_dimensions(layout, cfg):
    """Every operand a view into a wider buffer (row length < leading dimension, each padded differently), two K
    segments, ragged M / N and K tails: the kernels' address arithmetic must use the strides, and the padding
    columns of the output must stay untouched.  Whole-tile shape as well (the builds with the short epilogues)."""
    import torch
    dtype = "bf16"
    a_str, b_kc = LAYOUTS[layout]
    for M, N, K, K2 in ((520, 392, 200, 24), (512, 256, 192, 0)):
        print(f"case padded ld cfg={cfg} layout={layout} M={M} N={N} K={K} K2={K2}", flush=True)
        Abuf, Abh = make(11, 1, (K, M + 40) if a_str else (M, K + 24), dtype)
        Bbuf, Bbh = make(11, 2, (N, K + 8) if b_kc else (K, N + 16), dtype, 1.0 / K)
        A, Ah = (Abuf[:, :M], Abh[:, :M].copy()) if a_str else (Abuf[:, :K], Abh[:, :K].copy())
        B, Bh = (Bbuf[:, :K], Bbh[:, :K].copy()) if b_kc else (Bbuf[:, :N], Bbh[:, :N].copy())
        want = oracle.matmul(Ah, Bh, ta=a_str, tb=b_kc)
        A2 = B2 = None
        if K2 and not a_str:
            A2buf, A2h = make(11, 4, (M, K2 + 8), dtype)
            B2buf, B2h = make(11, 5, (N, K2 + 16) if b_kc else (K2, N + 8), dtype, 1.0 / K2)
            A2 = A2buf[:, :K2]
            B2, B2hv = (B2buf[:, :K2], B2h[:, :K2].copy()) if b_kc else (B2buf[:, :N], B2h[:, :N].copy())
            want = want + oracle.matmul(A2h[:, :K2].copy(), B2hv, tb=b_kc)
        Cbuf = torch.full((M, N + 32), 3.0, dtype=torch_dtype(dtype), device="cuda")
        C = Cbuf[:, :N]
        for splits in (1, 2):
            C.fill_(float("nan"))
            rl.runlora_gemm(A, B, C, a_strided=a_str, b_kcontig=b_kc, A2=A2, B2=B2, tile_cfg=cfg, splits=splits)
            torch.cuda.synchronize()
            assert relerr(to_f64(C), want) < TOL[dtype], (M, N, splits)
            assert elem_excess(to_f64(C), want, dtype) <= 1.0, (M, N, splits)
            assert torch.all(Cbuf[:, N:] == 3.0)


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("layout", list(LAYOUTS))
@pytest.mark.parametrize("N", [8, 24, 56, 120])
def test_streaming_kernel(N, layout, dtype):
    """The rank-r streaming kernel (tile_cfg 8): every operand layout, ragged M and K, K split over
    workgroups or not, plain and transposed store."""
    import torch
    a_str, b_kc = LAYOUTS[layout]
    M, K = (264, 1000) if a_str else (333, 520)
    print(f"case streaming N={N} layout={layout} dtype={dtype}", flush=True)
    A, Ah = make(7, 1, (K, M) if a_str else (M, K), dtype)
    B, Bh = make(7, 2, (N, K) if b_kc else (K, N), dtype, 1.0 / K)
    want = oracle.matmul(Ah, Bh, ta=a_str, tb=b_kc)
    for splits in (1, 3):
        C = torch.full((M, N), float("nan"), dtype=torch_dtype(dtype), device="cuda")
        rl.runlora_gemm(A, B, C, a_strided=a_str, b_kcontig=b_kc, tile_cfg=8, splits=splits)
        Ct = torch.full((N, (M + 7) // 8 * 8), float("nan"), dtype=torch_dtype(dtype), device="cuda")[:, :M]
        rl.runlora_gemm(A, B, Ct, a_strided=a_str, b_kcontig=b_kc, tile_cfg=8, splits=splits, trans_out=True)
        torch.cuda.synchronize()
        assert relerr(to_f64(C), want) < TOL[dtype], splits
        assert relerr(to_f64(Ct), want.T) < TOL[dtype], splits
    # heuristic split
    C = torch.full((M, N), float("nan"), dtype=torch_dtype(dtype), device="cuda")
    rl.runlora_gemm(A, B, C, a_strided=a_str, b_kcontig=b_kc, tile_cfg=8)
    torch.cuda.synchronize()
    assert relerr(to_f64(C), want) < TOL[dtype]


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("layout", list(LAYOUTS))
def test_short_epilogue_build_equals_the_general_one(layout, dtype):
    """When a launch of the matrix-core kernel (tile_cfg 7) has only whole 256x256 tiles and nothing but rounding
    in its epilogue, a build with a short epilogue runs.  Its output must be bit for bit that of the general
    build, which an all-zero bias selects (adding +0 changes no value that is not -0), and match the oracle;
    two tiles per workgroup row and column, several K tiles, ragged last K tile, second segment."""
    import torch
    a_str, b_kc = LAYOUTS[layout]
    M, N, K, K2 = 512, 768, 1048, 24
    A, Ah = make(5, 1, (K, M) if a_str else (M, K), dtype)
    B, Bh = make(5, 2, (N, K) if b_kc else (K, N), dtype, 1.0 / K)
    A2, A2h = make(5, 3, (K2, M) if a_str else (M, K2), dtype)
    B2, B2h = make(5, 4, (N, K2) if b_kc else (K2, N), dtype, 1.0 / K2)
    want = oracle.matmul(Ah, Bh, ta=a_str, tb=b_kc) + oracle.matmul(A2h, B2h, ta=a_str, tb=b_kc)
    td = torch_dtype(dtype)
    C = torch.full((M, N), float("nan"), dtype=td, device="cuda")
    Cg = torch.full((M, N), float("nan"), dtype=td, device="cuda")
    zero_bias = torch.zeros(N, dtype=td, device="cuda")
    rl.runlora_gemm(A, B, C, a_strided=a_str, b_kcontig=b_kc, A2=A2, B2=B2, tile_cfg=7, splits=1)
    rl.runlora_gemm(A, B, Cg, a_strided=a_str, b_kcontig=b_kc, A2=A2, B2=B2, tile_cfg=7, splits=1, bias=zero_bias)
    torch.cuda.synchronize()
    assert relerr(to_f64(C), want) < TOL[dtype]
    assert torch.equal(C.view(torch.int16), Cg.view(torch.int16))


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("layout", list(LAYOUTS))
def test_split_contraction_over_whole_tiles(layout, dtype):
    """A split contraction whose M and N are multiples of 256 runs the build of the matrix-core kernel that
    stores its fp32 partials row by row; 2 and 3 slices (the last one shorter and ending in a partial K tile),
    with and without an addend, scale and bias in the reduce."""
    import torch
    a_str, b_kc = LAYOUTS[layout]
    M, N, K = 512, 768, 2096
    A, Ah = make(7, 1, (K, M) if a_str else (M, K), dtype)
    B, Bh = make(7, 2, (N, K) if b_kc else (K, N), dtype, 1.0 / K)
    D, Dh = make(7, 3, (M, N), dtype)
    bias, biash = make(7, 4, (N,), dtype)
    want = oracle.matmul(Ah, Bh, ta=a_str, tb=b_kc)
    td = torch_dtype(dtype)
    for splits in (2, 3):
        C = torch.full((M, N), float("nan"), dtype=td, device="cuda")
        rl.runlora_gemm(A, B, C, a_strided=a_str, b_kcontig=b_kc, tile_cfg=7, splits=splits)
        torch.cuda.synchronize()
        assert relerr(to_f64(C), want) < TOL[dtype], splits
        C2 = torch.full((M, N), float("nan"), dtype=td, device="cuda")
        rl.runlora_gemm(A, B, C2, a_strided=a_str, b_kcontig=b_kc, D=D, tile_cfg=7, splits=splits, alpha=0.5, bias=bias)
        torch.cuda.synchronize()
        assert relerr(to_f64(C2), 0.5 * want + Dh + biash[None, :]) < TOL[dtype], splits
