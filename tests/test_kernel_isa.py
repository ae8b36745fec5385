"""Static checks of the matrix-core kernel's machine code (no GPU needed: hipcc cross-compiles).

The kernel's speed rests on three properties of its K loop that a harmless-looking source change can
silently break, with results staying correct: (1) no full wait for outstanding loads (`s_waitcnt
vmcnt(0)`) inside a K step, which would serialise the LDS ring; (2) no per-lane loop around a load (the
compiler wraps a load whose scalar offset it cannot prove uniform in a `s_cbranch_execnz` loop);
(3) no register spills.  Both the dense and the int4 route are checked, in the NN and NT layouts.
"""
import os
import re
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "..", "paper_2312_03415_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


@pytest.fixture(scope="module")
def asm(tmp_path_factory):
    out = tmp_path_factory.mktemp("isa") / "gemm_bf16.s"
    p = subprocess.run([HIPCC, *FLAGS, "-S", "--cuda-device-only", os.path.join(CSRC, "gemm_bf16.hip"), "-o", str(out)],
                       capture_output=True, text=True)
    assert p.returncode == 0, p.stderr[-2000:]
    return out.read_text()


def kernel_text(asm, al, bl, ns, bq, plain=0):
    name = f"_ZN2rl14gemm_mc_kernelIDF16bLi{al}ELi{bl}ELi{ns}ELb{bq}ELi{plain}EEEvNS_8GemmArgsE"
    start = asm.index("\n" + name + ":")
    return name, asm[start:asm.index("s_endpgm", start)]


def blocks(text):
    cur, out = [], []
    for line in text.split("\n"):
        if re.match(r"^\.LBB\d+_\d+:", line):
            out.append(cur)
            cur = []
        elif line.startswith("\t") and not line.strip().startswith((";", ".")):
            cur.append(line.strip())
    out.append(cur)
    return out


@pytest.mark.parametrize("al,bl,ns,bq,plain", [(0, 0, 3, 0, 0), (0, 1, 3, 0, 0), (1, 0, 3, 0, 0), (0, 0, 3, 1, 0), (0, 1, 3, 1, 0),
                                                (0, 0, 3, 0, 1), (0, 1, 3, 0, 1), (1, 0, 3, 0, 1), (0, 1, 3, 0, 2), (0, 0, 3, 1, 1)])
def test_k_loop_of_the_matrix_core_kernel(asm, al, bl, ns, bq, plain):
    name, text = kernel_text(asm, al, bl, ns, bq, plain)
    meta = asm[asm.index(".name:           " + name):]
    meta = meta[:meta.index(".wavefront_size")]
    assert re.search(r"\.vgpr_spill_count:\s+0\b", meta), "the kernel spills vector registers"
    # the two K steps of a tile: straight-line runs of MFMAs (the cursor's rare-event branch may cut one in two)
    ksteps = [b for b in blocks(text) if sum(i.startswith("v_mfma") for i in b) >= 3]
    assert sum(sum(i.startswith("v_mfma") for i in b) for b in ksteps) >= 32, "expected the 32 MFMAs of a K tile in a few straight-line blocks"
    assert len(ksteps) <= 4 * (2 if bq else 1), "the K steps are cut into many blocks: branches between the MFMAs"
    for b in ksteps:
        first = next(k for k, i in enumerate(b) if i.startswith("v_mfma"))
        last = max(k for k, i in enumerate(b) if i.startswith("v_mfma"))
        body = b[first:last + 1]
        assert not any(re.match(r"s_waitcnt\s+vmcnt\(0\)", i) for i in body), "full load wait inside a K step"
        assert not any(i.startswith("scratch_") for i in body), "spill traffic inside a K step"
    for b in blocks(text):
        if b and b[-1].startswith("s_cbranch_execnz"):
            assert not any(i.startswith(("buffer_load", "global_load")) for i in b), "a load sits in a per-lane (waterfall) loop"


@pytest.mark.parametrize("al,bl,plain", [(0, 0, 1), (0, 1, 1), (1, 0, 1), (0, 0, 0), (0, 1, 0), (0, 1, 2), (0, 0, 2)])
def test_k_loop_of_the_matrix_core_kernel_with_k_tile_64(asm, al, bl, plain):
    """gemm_mc64_kernel: a K tile is two straight-line K steps of 64 MFMAs (16x16x32) with tied accumulators and nothing
    between them but the fragment reads, the 16 refill loads and, in the second, one wait + barrier; no spills, no
    accumulator traffic between the two register files, no load in a per-lane loop."""
    name = f"_ZN2rl16gemm_mc64_kernelIDF16bLi{al}ELi{bl}ELi{plain}EEEvNS_8GemmArgsE"
    start = asm.index("\n" + name + ":")
    text = asm[start:asm.index("s_endpgm", start)]
    meta = asm[asm.index(".name:           " + name):]
    meta = meta[:meta.index(".wavefront_size")]
    assert re.search(r"\.vgpr_spill_count:\s+0\b", meta), "the kernel spills vector registers"
    ksteps = [b for b in blocks(text) if sum(i.startswith("v_mfma_f32_16x16x32") for i in b) >= 64]
    assert len(ksteps) == 2, "expected the two K steps of a tile as two straight-line blocks of 64 MFMAs"
    syncs = 0
    for b in ksteps:
        first = next(k for k, i in enumerate(b) if i.startswith("v_mfma"))
        last = max(k for k, i in enumerate(b) if i.startswith("v_mfma"))
        body = b[first:last + 1]
        assert sum(i.startswith("v_mfma") for i in body) == 64
        assert not any(i.startswith(("scratch_", "v_accvgpr")) for i in body), "spill or accumulator copies inside a K step"
        for i in body:
            m = re.match(r"v_mfma_f32_16x16x32_\w+\s+(a\[\d+:\d+\]), \S+, \S+, (a\[\d+:\d+\])", i)
            if i.startswith("v_mfma"):
                assert m and m.group(1) == m.group(2), "accumulator not tied: " + i
        waits = [i for i in body if re.match(r"s_waitcnt\s+vmcnt\(0\)", i)]
        assert len(waits) <= 1
        syncs += len(waits)
        n_loads = sum(i.startswith("buffer_load") for i in body)
        assert n_loads in (0, 16)
        assert len(body) <= 64 + 90, "too many instructions between the MFMAs of a K step"
    assert syncs == 1, "exactly one of the two K steps waits for the loads"
    for b in blocks(text):
        if b and b[-1].startswith("s_cbranch_execnz"):
            assert not any(i.startswith(("buffer_load", "global_load")) for i in b), "a load sits in a per-lane (waterfall) loop"
