"""Host-side checks of the C-ABI library that need no GPU: it loads, exports what the header
declares, its Table 1 closed forms and FLOP-criterion selector agree with the paper, and every
argument error is reported before any HIP call."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2312_03415_amd import binding as rl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "runlora.h")).read()
    declared = set(re.findall(r"\b(runlora_\w+)\s*\(", header))
    assert declared, "no declarations found"
    L = rl.lib()
    for name in declared:
        assert hasattr(L, name), f"{name} declared in runlora.h but not exported"
    assert declared == set(rl.EXPORTS)
    assert L.runlora_version() >= 100
    assert L.runlora_strerror(rl.RL_ERR_ALIGN).decode()


def test_flops_match_table1(table1):
    rng = np.random.default_rng(0)
    for _ in range(50):
        n, i, o, r = (int(v) for v in rng.integers(1, 20000, size=4))
        assert rl.runlora_flops(0, 1, n, i, o, r) == table1["forward1"](n, i, o, r)
        assert rl.runlora_flops(0, 2, n, i, o, r) == table1["forward2"](n, i, o, r)
        for v in range(1, 9):
            assert rl.runlora_flops(1, v, n, i, o, r) == table1[f"backward{v}"](n, i, o, r)
        assert rl.runlora_flops(0, 0, n, i, o, r) == table1["forward1"](n, i, o, r)
        assert rl.runlora_flops(0, 3, n, i, o, r) == table1["forward1"](n, i, o, r)   # forward1's graph in one kernel
        assert rl.runlora_flops(1, 0, n, i, o, r) == table1["backward1"](n, i, o, r) - 2 * n * i * r
    assert rl.runlora_flops(0, 4, 1, 1, 1, 1) == -1 and rl.runlora_flops(1, 9, 1, 1, 1, 1) == -1


def test_flop_criterion_closed_forms(table1):
    """Consequences of Table 1: forward2 wins iff n > io/(i+o) (independent of r); backward5 beats
    backward1 iff n > o; backward2/3 never win under r(i+o) < io (Section 2)."""
    rng = np.random.default_rng(1)
    for _ in range(400):
        n, i, o, r = (int(v) for v in rng.integers(1, 6000, size=4))
        f, b = rl.runlora_select(n, i, o, r, rl.RL_BF16, criterion=0)
        ff = {v: table1[f"forward{v}"](n, i, o, r) for v in (1, 2)}
        bf = {v: table1[f"backward{v}"](n, i, o, r) for v in range(1, 6)}
        assert ff[f] == min(ff.values()) and bf[b] == min(bf.values())
        assert f == (2 if n * (i + o) > i * o else 1)
        if r * (i + o) < i * o:
            assert b in (1, 4, 5)
            if b != 4:
                assert b == (5 if n > o else 1)


def test_flop_criterion_on_llama_mlp_setting():
    """The setting of the paper's batch/sequence figure: i=4096, o=11008, r=128 satisfies Eq. 5;
    forward2 from n = 2986 tokens on, backward5 beyond n = 11008, backward1 below."""
    i, o, r = 4096, 11008, 128
    assert r * (i + o) < i * o
    assert rl.runlora_select(2985, i, o, r, rl.RL_BF16, 0)[0] == 1
    assert rl.runlora_select(2986, i, o, r, rl.RL_BF16, 0)[0] == 2
    assert rl.runlora_select(11008, i, o, r, rl.RL_BF16, 0)[1] == 1
    assert rl.runlora_select(11009, i, o, r, rl.RL_BF16, 0)[1] == 5
    # int4 W: merged graphs are unavailable
    assert rl.runlora_select(4096, 5120, 13824, 64, rl.RL_INT4_G64, 0) == (1, 1)


def test_select_time_model_returns_legal_pairs():
    for n in (128, 1024, 8192, 16384):
        for r in (8, 64, 256):
            f, b = rl.runlora_select(n, 4096, 4096, r, rl.RL_F16)
            assert (f in (1, 2, 3) and b in (1, 2, 3, 4, 5)) or (f, b) == (0, 0)
            assert rl.runlora_model_time_us(0, f, n, 4096, 4096, r, rl.RL_F16) > 0
    assert rl.runlora_model_time_us(0, 7, 128, 64, 64, 8, rl.RL_F16) < 0
    assert rl.runlora_model_time_us(1, 8, 128, 64, 64, 8, rl.RL_F16) > 0      # items 6-8 are modelled too
    assert rl.runlora_model_time_us(1, 9, 128, 64, 64, 8, rl.RL_F16) < 0
    f, b = ctypes.c_int(), ctypes.c_int()
    assert rl.lib().runlora_select(0, 8, 8, 8, rl.RL_F16, ctypes.byref(f), ctypes.byref(b)) == rl.RL_ERR_SHAPE
    assert rl.lib().runlora_select(8, 8, 8, 8, 77, ctypes.byref(f), ctypes.byref(b)) == rl.RL_ERR_DTYPE
    assert rl.lib().runlora_select(8, 8, 8, 8, rl.RL_F16, None, ctypes.byref(b)) == rl.RL_ERR_NULL


def test_select_honours_the_debugging_overrides(monkeypatch):
    n, i, o, r = 8192, 4096, 4096, 32
    free = rl.runlora_select(n, i, o, r, rl.RL_BF16)
    monkeypatch.setenv("RUNLORA_FORCE_FWD", "2")
    assert rl.runlora_select(n, i, o, r, rl.RL_BF16) == (2, free[1] if free[1] != 0 else 1)
    monkeypatch.setenv("RUNLORA_FORCE_BWD", "4")
    assert rl.runlora_select(n, i, o, r, rl.RL_BF16) == (2, 4)
    assert rl.runlora_select(n, i, o, r, rl.RL_BF16, criterion=1) == free        # runlora_select_by ignores them
    f, b = ctypes.c_int(), ctypes.c_int()
    assert rl.lib().runlora_select(n, i, o, r, rl.RL_INT4_G64, ctypes.byref(f), ctypes.byref(b)) == rl.RL_ERR_UNSUPPORTED
    monkeypatch.setenv("RUNLORA_FORCE_BWD", "0")
    assert rl.lib().runlora_select(n, i, o, r, rl.RL_BF16, ctypes.byref(f), ctypes.byref(b)) == rl.RL_ERR_VARIANT   # (2, 0) is illegal
    monkeypatch.delenv("RUNLORA_FORCE_FWD")
    assert rl.runlora_select(n, i, o, r, rl.RL_BF16) == (0, 0)                    # the default backward brings its forward
    monkeypatch.setenv("RUNLORA_FORCE_BWD", "nine")
    assert rl.lib().runlora_select(n, i, o, r, rl.RL_BF16, ctypes.byref(f), ctypes.byref(b)) == rl.RL_ERR_VARIANT
    monkeypatch.delenv("RUNLORA_FORCE_BWD")
    assert rl.runlora_select(n, i, o, r, rl.RL_BF16) == free


def test_select_with_kept_merged_weight():
    """Criterion 2 prices forward2 + backward4/5 without the second W + AB pass: it may only move the
    choice towards such a pair, never to a slower one under the plain model."""
    for n in (128, 1024, 4096, 16384):
        for i, o, r in ((4096, 4096, 64), (8192, 2048, 16), (4096, 11008, 128), (4096, 4096, 1024)):
            f1, b1 = rl.runlora_select(n, i, o, r, rl.RL_BF16, criterion=1)
            f2, b2 = rl.runlora_select(n, i, o, r, rl.RL_BF16, criterion=2)
            assert (f2, b2) == (f1, b1) or (f2 == 2 and b2 in (4, 5)), (n, i, o, r)
    f, b = ctypes.c_int(), ctypes.c_int()
    assert rl.lib().runlora_select_by(4, 8, 8, 8, 8, rl.RL_F16, ctypes.byref(f), ctypes.byref(b)) == rl.RL_ERR_VARIANT
    # an int4 W has no merged graphs whatever the criterion
    f2, b2 = rl.runlora_select(16384, 4096, 4096, 64, rl.RL_INT4_G64, criterion=2)
    assert f2 in (0, 1) and b2 in (0, 1, 2, 3)


def test_select_with_kept_T():
    """Criterion 3 prices forward1 + backward1/5 without the second X A pass: it may only move the choice towards
    such a pair, and the model must see the saving."""
    for n in (128, 1024, 8192, 16384):
        for i, o, r in ((4096, 4096, 32), (4096, 11008, 32), (11008, 4096, 128), (4096, 4096, 1024)):
            p1 = rl.runlora_select(n, i, o, r, rl.RL_BF16, criterion=1)
            p3 = rl.runlora_select(n, i, o, r, rl.RL_BF16, criterion=3)
            assert p3 == p1 or (p3[0] == 1 and p3[1] in (1, 5)), (n, i, o, r)
    # at the Llama shapes the kept T decides between forward1 and forward2, which the plain model prices alike
    assert rl.runlora_select(8192, 4096, 4096, 32, rl.RL_BF16, criterion=3) == (1, 1)
    assert rl.runlora_select(8192, 11008, 4096, 32, rl.RL_BF16, criterion=3) == (1, 1)
    assert rl.runlora_select(4096, 5120, 13824, 64, rl.RL_INT4_G64, criterion=3) == (1, 1)


def test_saved_bytes_is_the_memory_claim_of_section2():
    """The default chain keeps XA (n r elements) for its backward, RunLoRA's forwards keep nothing
    besides X (Section 2); forward2 asked to keep W + AB holds i o elements."""
    n, i, o, r = 8192, 4096, 11008, 128
    assert rl.runlora_saved_bytes(0, n, i, o, r, rl.RL_BF16) == n * r * 2
    assert rl.runlora_saved_bytes(0, n, i, o, r, rl.RL_F32) == n * r * 4
    assert rl.runlora_saved_bytes(1, n, i, o, r, rl.RL_BF16) == 0
    assert rl.runlora_saved_bytes(2, n, i, o, r, rl.RL_BF16) == 0
    assert rl.runlora_saved_bytes(2, n, i, o, r, rl.RL_BF16, keep_merged=True) == i * o * 2
    assert rl.runlora_saved_bytes(1, n, i, o, r, rl.RL_BF16, keep_merged=True) == 0
    assert rl.runlora_saved_bytes(5, n, i, o, r, rl.RL_BF16) == 0
    # forward1 (also as forward 3) asked to keep XA holds what the default chain holds
    assert rl.runlora_saved_bytes(1, n, i, o, r, rl.RL_BF16, keep_t=True) == n * r * 2
    assert rl.runlora_saved_bytes(3, n, i, o, r, rl.RL_BF16, keep_t=True) == n * r * 2
    assert rl.runlora_saved_bytes(2, n, i, o, r, rl.RL_BF16, keep_t=True) == 0
    assert rl.runlora_saved_bytes(2, n, i, o, r, rl.RL_BF16, keep_merged=True, keep_t=True) == i * o * 2


def test_workspace_bytes_cover_intermediates():
    n, i, o, r = 8192, 4096, 4096, 32
    e = 2
    assert rl.runlora_workspace_bytes(1, -1, n, i, o, r, rl.RL_BF16) >= n * r * e              # T
    assert rl.runlora_workspace_bytes(2, -1, n, i, o, r, rl.RL_BF16) >= i * o * e              # M
    assert rl.runlora_workspace_bytes(-1, 4, n, i, o, r, rl.RL_BF16) >= 2 * i * o * e          # M, Z2
    assert rl.runlora_workspace_bytes(-1, 5, n, i, o, r, rl.RL_BF16) >= 2 * n * r * e + i * o * e
    both = rl.runlora_workspace_bytes(2, 5, n, i, o, r, rl.RL_BF16)
    assert both == max(rl.runlora_workspace_bytes(2, -1, n, i, o, r, rl.RL_BF16),
                       rl.runlora_workspace_bytes(-1, 5, n, i, o, r, rl.RL_BF16))


# ---- argument validation: fake (never dereferenced) device addresses ----------------------------

def test_split_contractions_are_sized_by_whole_rounds():
    """The fp32 partials in the workspace tell how a large product is split.  4096 -> 11008 at 8192 tokens: 32 x 43
    tiles of 256 x 256; 40 tile columns are five whole rounds of 256 compute units, the 96 tiles of the last three
    columns run in two K slices (192 work items in one round; three slices would spill into a second round).
    8192 -> 2048 at 4096 tokens: 128 tiles, the contraction in two."""
    n, i, o, r = 8192, 4096, 11008, 32
    assert rl.runlora_workspace_bytes(1, -1, n, i, o, r, rl.RL_BF16) == n * r * 2 + 2 * n * 768 * 4
    n, i, o, r = 4096, 8192, 2048, 16
    assert rl.runlora_workspace_bytes(1, -1, n, i, o, r, rl.RL_BF16) == n * r * 2 + 2 * n * o * 4
    # a contraction too short to pay for the partials' round trip stays whole
    assert rl.runlora_workspace_bytes(1, -1, 4096, 512, 2048, 16, rl.RL_BF16) == 4096 * 16 * 2


def T(ptr, rows, cols, dtype=rl.RL_BF16, ld=None):
    return rl.rl_tensor_t(ptr, rows, cols, cols if ld is None else ld, dtype, None, 0)


def fwd_args(n=64, i=32, o=48, r=8, dtype=rl.RL_BF16):
    base = 0x10000000
    step = 0x1000000
    return dict(X=T(base, n, i, dtype), W=T(base + step, i, o, dtype), A=T(base + 2 * step, i, r, dtype),
                B=T(base + 3 * step, r, o, dtype), Y=T(base + 4 * step, n, o, dtype))


def call_fwd(variant, a, saved=None, opts=None):
    saved = saved if saved is not None else rl.rl_saved_t()
    ref = lambda x: ctypes.byref(x) if x is not None else None
    return rl.lib().runlora_forward(variant, ref(a["X"]), ref(a["W"]), ref(a["A"]), ref(a["B"]), ref(a["Y"]),
                                    ctypes.byref(saved), ref(opts))


def test_forward_rejects_bad_arguments_before_touching_the_gpu():
    a = fwd_args()
    assert call_fwd(9, a) == rl.RL_ERR_VARIANT
    assert call_fwd(-1, a) == rl.RL_ERR_VARIANT
    b = fwd_args(); b["W"] = None
    assert call_fwd(1, b) == rl.RL_ERR_NULL
    b = fwd_args(); b["W"].data = None
    assert call_fwd(1, b) == rl.RL_ERR_NULL
    b = fwd_args(); b["W"].rows = 40
    assert call_fwd(1, b) == rl.RL_ERR_SHAPE
    b = fwd_args(); b["B"].cols = 56
    assert call_fwd(1, b) == rl.RL_ERR_SHAPE
    b = fwd_args(); b["A"].dtype = rl.RL_F16
    assert call_fwd(1, b) == rl.RL_ERR_DTYPE
    b = fwd_args(); b["X"].dtype = 42
    assert call_fwd(1, b) == rl.RL_ERR_DTYPE
    b = fwd_args(); b["X"].data += 2
    assert call_fwd(1, b) == rl.RL_ERR_ALIGN
    b = fwd_args(); b["X"].ld = 36
    assert call_fwd(1, b) == rl.RL_ERR_ALIGN
    b = fwd_args(r=4)
    assert call_fwd(1, b) == rl.RL_ERR_ALIGN          # r must be a multiple of 8 for 16-bit types
    b = fwd_args(); b["Y"].data = b["X"].data
    assert call_fwd(1, b) == rl.RL_ERR_ALIAS
    # LoRA dropout: probability in (0, 1); no merged forward, r <= 128
    assert call_fwd(1, a, opts=rl.rl_opts_t(None, 0x70000000, 1 << 30, 0.0, None, 1.5, 1)) == rl.RL_ERR_SHAPE
    assert call_fwd(2, a, opts=rl.rl_opts_t(None, 0x70000000, 1 << 30, 0.0, None, 0.1, 1)) == rl.RL_ERR_UNSUPPORTED
    # needs workspace, none given / too small / misaligned
    assert call_fwd(1, a) == rl.RL_ERR_WORKSPACE
    assert call_fwd(1, a, opts=rl.rl_opts_t(None, 0x70000000, 16)) == rl.RL_ERR_WORKSPACE
    need = rl.runlora_workspace_bytes(1, -1, 64, 32, 48, 8, rl.RL_BF16)
    assert call_fwd(1, a, opts=rl.rl_opts_t(None, 0x70000010, need)) == rl.RL_ERR_ALIGN
    # default chain needs the caller's T buffer
    assert call_fwd(0, a) == rl.RL_ERR_NULL
    # int4 W: needs scales and group 64; the merged forward does not exist for it; fp32 activations are refused
    b = fwd_args(); b["W"].dtype = rl.RL_INT4_G64
    assert call_fwd(1, b) == rl.RL_ERR_NULL
    b["W"].scales = 0x50000000
    assert call_fwd(1, b) == rl.RL_ERR_UNSUPPORTED          # group != 64
    b["W"].group = 64
    assert call_fwd(2, b) == rl.RL_ERR_UNSUPPORTED          # X (W + AB) needs a dense W
    b["W"].scales = 0x50000004
    assert call_fwd(1, b) == rl.RL_ERR_ALIGN


def test_workspace_size_holds_for_operands_beyond_two_gib():
    """An X (or dY) whose extent reaches 2 GiB leaves the streaming kernel (31-bit byte offsets) for the tile GEMM,
    whose split contraction needs fp32 partials: the size the library reports must be the size the call then asks
    for.  Checked through the text of RL_ERR_WORKSPACE, which names the need (nothing is launched)."""
    n, i, o, r = 1 << 19, 4096, 256, 16          # n * i * 2 bytes = 4 GiB
    L = rl.lib()
    br = ctypes.byref
    base, step = 0x10000000000, 0x1000000000
    small = rl.rl_opts_t(None, 0x70000000, 256)

    def told():
        return int(re.search(r"(\d+) bytes", L.runlora_last_hip_error().decode()).group(1))

    a = fwd_args(n, i, o, r)
    for k, name in enumerate(("X", "W", "A", "B", "Y")):
        a[name].data = base + k * step
    need = rl.runlora_workspace_bytes(1, -1, n, i, o, r, rl.RL_BF16)
    assert need >= n * r * 2
    assert call_fwd(1, a, opts=small) == rl.RL_ERR_WORKSPACE and told() == need
    # backward1: dA = X^T Z1 over 2^19 tokens falls to the tile GEMM with its contraction split over workgroups
    dY, W, A, B = T(base, n, o), T(base + step, i, o), T(base + 2 * step, i, r), T(base + 3 * step, r, o)
    dX, dA, dB = T(base + 4 * step, n, i), T(base + 5 * step, i, r), T(base + 6 * step, r, o)
    saved = rl.rl_saved_t(1, rl.RL_BF16, n, i, o, r, base + 7 * step, i, None, 0)
    need = rl.runlora_workspace_bytes(-1, 1, n, i, o, r, rl.RL_BF16)
    assert need > 2 * n * r * 2                  # Z1, Z2 and fp32 partials
    assert L.runlora_backward(1, br(dY), br(saved), br(W), br(A), br(B), br(dX), br(dA), br(dB), br(small)) == rl.RL_ERR_WORKSPACE
    assert told() == need
    # under LoRA dropout the masked products exist on the streaming kernel only: such an X is refused outright
    assert call_fwd(1, a, opts=rl.rl_opts_t(None, 0x70000000, 1 << 40, 0.0, None, 0.1, 1)) == rl.RL_ERR_UNSUPPORTED


def test_default_forward_checks_its_T_buffer_against_every_input():
    a = fwd_args()
    ws = rl.rl_opts_t(None, 0x70000000, 1 << 30)
    for name in ("X", "W", "A", "B", "Y"):
        saved = rl.rl_saved_t()
        saved.T, saved.ldt = a[name].data, 8
        assert call_fwd(0, a, saved, ws) == rl.RL_ERR_ALIAS, name


def test_static_scratch_forward_checks_arguments_and_size_before_touching_the_gpu():
    """runlora_forward_static: the same argument checks as runlora_forward, and a call that needs more scratch than
    the library's fixed array is refused with both figures in the error text; no workspace argument is needed."""
    L = rl.lib()
    ref = lambda x: ctypes.byref(x) if x is not None else None

    def call(variant, a):
        return L.runlora_forward_static(variant, ref(a["X"]), ref(a["W"]), ref(a["A"]), ref(a["B"]), ref(a["Y"]),
                                        ctypes.byref(rl.rl_saved_t()), None)

    a = fwd_args()
    assert call(9, a) == rl.RL_ERR_VARIANT
    b = fwd_args(); b["W"].rows = 40
    assert call(1, b) == rl.RL_ERR_SHAPE
    b = fwd_args(); b["Y"].data = b["X"].data
    assert call(1, b) == rl.RL_ERR_ALIAS
    assert call(0, a) == rl.RL_ERR_NULL                      # the default chain still needs the caller's T buffer
    big = fwd_args(512, 4096, 4096, 16)                      # forward2 would form W + AB: 32 MiB
    assert rl.runlora_workspace_bytes(2, -1, 512, 4096, 4096, 16, rl.RL_BF16) > rl.STATIC_SCRATCH_BYTES
    assert call(2, big) == rl.RL_ERR_WORKSPACE
    text = L.runlora_last_hip_error().decode()
    assert str(rl.STATIC_SCRATCH_BYTES) in text and str(rl.runlora_workspace_bytes(2, -1, 512, 4096, 4096, 16, rl.RL_BF16)) in text
    header = open(os.path.join(ROOT, "include", "runlora.h")).read()
    m = re.search(r"#define RL_STATIC_SCRATCH_BYTES \((\d+)u << (\d+)\)", header)
    assert m and int(m.group(1)) << int(m.group(2)) == rl.STATIC_SCRATCH_BYTES


def test_backward_rejects_bad_arguments_before_touching_the_gpu():
    n, i, o, r = 64, 32, 48, 8
    base, step = 0x10000000, 0x1000000
    dt = rl.RL_BF16
    dY, W, A, B = T(base, n, o), T(base + step, i, o), T(base + 2 * step, i, r), T(base + 3 * step, r, o)
    dX, dA, dB = T(base + 4 * step, n, i), T(base + 5 * step, i, r), T(base + 6 * step, r, o)
    saved = rl.rl_saved_t(1, dt, n, i, o, r, base + 7 * step, i, None, 0)
    L = rl.lib()
    br = ctypes.byref

    def call(variant, saved=saved, dY=dY, dX=dX, opts=None):
        return L.runlora_backward(variant, br(dY), br(saved), br(W), br(A), br(B), br(dX) if dX else None, br(dA),
                                  br(dB), br(opts) if opts else None)

    assert call(9) == rl.RL_ERR_VARIANT
    assert call(-1) == rl.RL_ERR_VARIANT
    assert call(6) == rl.RL_ERR_WORKSPACE                 # items 6-8 of Section 2's list are legal graphs
    assert call(0) == rl.RL_ERR_SAVED_MISMATCH            # default backward needs the default forward's T
    s2 = rl.rl_saved_t(1, dt, n + 1, i, o, r, base + 7 * step, i, None, 0)
    assert call(1, saved=s2) == rl.RL_ERR_SAVED_MISMATCH
    s3 = rl.rl_saved_t(1, rl.RL_F16, n, i, o, r, base + 7 * step, i, None, 0)
    assert call(1, saved=s3) == rl.RL_ERR_SAVED_MISMATCH
    s4 = rl.rl_saved_t(1, dt, n, i, o, r, None, i, None, 0)
    assert call(1, saved=s4) == rl.RL_ERR_NULL
    assert call(1, dY=T(base, n, o + 8)) == rl.RL_ERR_SHAPE
    assert call(1, dX=T(base, n, i)) == rl.RL_ERR_ALIAS    # dX on top of dY
    assert call(1) == rl.RL_ERR_WORKSPACE
    assert call(1, dX=None) == rl.RL_ERR_WORKSPACE          # skipping dX is legal; still needs scratch


def test_vera_calls_reject_bad_arguments_before_touching_the_gpu():
    """The VeRA entry points check their own arguments and, through a dry run of the layer call they are
    built on, everything that call checks, before the first launch."""
    n, i, o, r = 64, 32, 48, 8
    dt = rl.RL_BF16
    L = rl.lib()
    br = ctypes.byref
    a = fwd_args(n, i, o, r)
    d, b = 0x20000000, 0x20001000
    need = rl.runlora_vera_workspace_bytes(1, 1, n, i, o, r, dt)
    assert need == 2 * ((r * o * 2 + 255) // 256 * 256) + rl.runlora_workspace_bytes(1, 1, n, i, o, r, dt)
    assert rl.runlora_vera_workspace_bytes(4, 1, n, i, o, r, dt) == 0 and rl.runlora_vera_workspace_bytes(-1, -1, n, i, o, r, dt) == 0
    ws = rl.rl_opts_t(None, 0x70000000, need)

    def fwd(variant, a=a, d=d, b=b, opts=ws):
        return L.runlora_vera_forward(variant, br(a["X"]), br(a["W"]), br(a["A"]), br(a["B"]), d, b, br(a["Y"]),
                                      br(rl.rl_saved_t()), br(opts) if opts else None)

    assert fwd(1, d=None) == rl.RL_ERR_NULL
    assert fwd(1, b=b + 4) == rl.RL_ERR_ALIGN
    assert fwd(1, opts=None) == rl.RL_ERR_WORKSPACE
    assert fwd(1, opts=rl.rl_opts_t(None, 0x70000000, 2 * 768)) == rl.RL_ERR_WORKSPACE      # room for B~ and dB~ only
    assert fwd(5) == rl.RL_ERR_VARIANT
    assert fwd(1, d=a["Y"].data) == rl.RL_ERR_ALIAS
    c = fwd_args(n, i, o, r); c["X"].ld = 36
    assert fwd(1, a=c) == rl.RL_ERR_ALIGN                                                   # found by the dry run
    c = fwd_args(n, i, o, r); c["B"].rows = 16
    assert fwd(1, a=c) == rl.RL_ERR_SHAPE
    assert fwd(0) == rl.RL_ERR_NULL                                                         # default chain: no T buffer given

    base, step = 0x10000000, 0x1000000
    dY, W, A, B, dX = T(base, n, o), T(base + step, i, o), T(base + 2 * step, i, r), T(base + 3 * step, r, o), T(base + 4 * step, n, i)
    saved = rl.rl_saved_t(1, dt, n, i, o, r, base + 7 * step, i, None, 0)
    dd, db = 0x20002000, 0x20003000

    def bwd(variant, saved=saved, d=d, b=b, dd=dd, db=db, opts=ws):
        return L.runlora_vera_backward(variant, br(dY), br(saved), br(W), br(A), br(B), d, b, br(dX), dd, db,
                                       br(opts) if opts else None)

    assert bwd(9) == rl.RL_ERR_VARIANT
    assert bwd(1, b=None) == rl.RL_ERR_NULL
    assert bwd(1, dd=dd + 8) == rl.RL_ERR_ALIGN
    assert bwd(1, dd=d) == rl.RL_ERR_ALIAS
    assert bwd(1, db=dY.data) == rl.RL_ERR_ALIAS
    assert bwd(1, dd=db) == rl.RL_ERR_ALIAS
    assert bwd(0) == rl.RL_ERR_SAVED_MISMATCH
    assert bwd(1, opts=rl.rl_opts_t(None, 0x70000000, 2 * 768)) == rl.RL_ERR_WORKSPACE
    assert bwd(1, saved=rl.rl_saved_t(1, dt, n + 1, i, o, r, base + 7 * step, i, None, 0)) == rl.RL_ERR_SAVED_MISMATCH


def test_dora_calls_reject_bad_arguments_before_touching_the_gpu():
    """The DoRA entry points refuse the graphs that read W outside W + sAB, fp32, r > 128 and dropout, check their own
    vectors, and run every check of the layer call they are built on before the first launch."""
    n, i, o, r = 64, 32, 48, 8
    dt = rl.RL_BF16
    L = rl.lib()
    br = ctypes.byref
    a = fwd_args(n, i, o, r)
    m, c = 0x20000000, 0x20001000
    need = rl.runlora_dora_workspace_bytes(2, 5, n, i, o, r, dt)
    assert need > rl.runlora_workspace_bytes(2, 5, n, i, o, r, dt) + 2 * r * o * 2 + o * 4
    assert rl.runlora_dora_workspace_bytes(2, 5, n, i, o, r, rl.RL_F32) == 0
    assert rl.runlora_dora_workspace_bytes(2, 5, n, i, o, 136, dt) == 0
    assert rl.runlora_dora_workspace_bytes(-1, -1, n, i, o, r, dt) == 0
    ws = rl.rl_opts_t(None, 0x70000000, need)

    def fwd(variant, a=a, m=m, c=c, opts=ws):
        return L.runlora_dora_forward(variant, br(a["X"]), br(a["W"]), br(a["A"]), br(a["B"]), m, br(a["Y"]),
                                      br(rl.rl_saved_t()), c, br(opts) if opts else None)

    assert fwd(0) == rl.RL_ERR_UNSUPPORTED and fwd(1) == rl.RL_ERR_UNSUPPORTED
    assert fwd(3) == rl.RL_ERR_UNSUPPORTED and fwd(4) == rl.RL_ERR_VARIANT
    assert fwd(2, m=None) == rl.RL_ERR_NULL and fwd(2, c=None) == rl.RL_ERR_NULL
    assert fwd(2, m=m + 4) == rl.RL_ERR_ALIGN and fwd(2, c=c + 4) == rl.RL_ERR_ALIGN
    assert fwd(2, opts=None) == rl.RL_ERR_WORKSPACE
    assert fwd(2, opts=rl.rl_opts_t(None, 0x70000000, 4096)) == rl.RL_ERR_WORKSPACE
    assert fwd(2, c=a["Y"].data) == rl.RL_ERR_ALIAS and fwd(2, c=m) == rl.RL_ERR_ALIAS and fwd(2, m=a["Y"].data) == rl.RL_ERR_ALIAS
    drop = rl.rl_opts_t(None, 0x70000000, need, 0.0, None, 0.1, 3)
    assert fwd(2, opts=drop) == rl.RL_ERR_UNSUPPORTED
    f32 = fwd_args(n, i, o, r, rl.RL_F32)
    assert fwd(2, a=f32) == rl.RL_ERR_UNSUPPORTED
    big = fwd_args(n, 256, o, 136)
    assert fwd(2, a=big) == rl.RL_ERR_UNSUPPORTED
    e = fwd_args(n, i, o, r); e["X"].ld = 36
    assert fwd(2, a=e) == rl.RL_ERR_ALIGN                                                   # found by the dry run

    base, step = 0x10000000, 0x1000000
    dY, W, A, B, dX = T(base, n, o), T(base + step, i, o), T(base + 2 * step, i, r), T(base + 3 * step, r, o), T(base + 4 * step, n, i)
    dA, dB, Y = T(base + 5 * step, i, r), T(base + 6 * step, r, o), T(base + 8 * step, n, o)
    saved = rl.rl_saved_t(2, dt, n, i, o, r, base + 7 * step, i, None, 0)
    dm = 0x20002000

    def bwd(variant, saved=saved, m=m, c=c, Y=Y, dm=dm, dB=dB, opts=ws):
        return L.runlora_dora_backward(variant, br(dY), br(saved), br(W), br(A), br(B), m, c, br(Y) if Y else None, br(dX),
                                       br(dA), br(dB) if dB else None, dm, br(opts) if opts else None)

    assert bwd(9) == rl.RL_ERR_VARIANT
    for v in (0, 1, 2, 3, 6):
        assert bwd(v) == rl.RL_ERR_UNSUPPORTED
    assert bwd(5, c=None) == rl.RL_ERR_NULL and bwd(5, m=None) == rl.RL_ERR_NULL
    assert bwd(5, Y=None) == rl.RL_ERR_NULL              # dm needs the forward's output
    assert bwd(5, dm=dm + 8) == rl.RL_ERR_ALIGN
    assert bwd(5, dm=m) == rl.RL_ERR_ALIAS and bwd(5, dm=dY.data) == rl.RL_ERR_ALIAS and bwd(5, dm=Y.data) == rl.RL_ERR_ALIAS
    assert bwd(5, dB=T(base + 3 * step, r, o)) == rl.RL_ERR_ALIAS                           # dB on top of B
    assert bwd(5, Y=T(base + 4 * step, n, o)) == rl.RL_ERR_ALIAS                            # Y is read after dX is written
    assert bwd(5, opts=rl.rl_opts_t(None, 0x70000000, 4096)) == rl.RL_ERR_WORKSPACE
    assert bwd(5, saved=rl.rl_saved_t(2, dt, n + 1, i, o, r, base + 7 * step, i, None, 0)) == rl.RL_ERR_SAVED_MISMATCH


def test_gemm_call_rejects_bad_arguments():
    g = rl.rl_gemm_t(rl.RL_BF16, 1, 1, -1, 0, 64, 64, 64, 0, 0x1000, 0x2000, None, None, None, 0x3000, 64, 64, 0, 0, 64, 0)
    L = rl.lib()
    assert L.runlora_gemm(ctypes.byref(g), None) == rl.RL_ERR_UNSUPPORTED
    g.b_kcontig = 0
    g.N = 60
    assert L.runlora_gemm(ctypes.byref(g), None) == rl.RL_ERR_ALIGN
    g.N = 64
    g.tile_cfg = 17
    assert L.runlora_gemm(ctypes.byref(g), None) == rl.RL_ERR_VARIANT
    g.tile_cfg = 8          # streaming kernel: N <= 128 only
    g.N = 136
    assert L.runlora_gemm(ctypes.byref(g), None) == rl.RL_ERR_UNSUPPORTED
    g.N = 64
    g.tile_cfg = 1
    g.trans_out = 1         # transposed store exists in the streaming kernel only
    assert L.runlora_gemm(ctypes.byref(g), None) == rl.RL_ERR_UNSUPPORTED
    g.trans_out = 0
    g.tile_cfg = -1
    g.C = None
    assert L.runlora_gemm(ctypes.byref(g), None) == rl.RL_ERR_NULL
