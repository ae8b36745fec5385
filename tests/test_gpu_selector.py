"""GPU: the selector against exhaustive timing: every legal (forward, backward) pair is timed and
runlora_select's choice must be within 5 % of the best one, and no slower than the default chain.  On the
crossover sweep (fp16, d_in = d_out = 4096, tokens in {128, 1024, 16384}, rank in {8, 64, 256, 1024}), on the
bf16 layer shapes the bench times (the two MLP layers of the OPT-1.3B-shaped block at rank 16; the attention,
gate and down projections of the Llama-7B-shaped block at ranks 8, 32 and 128) and on the int4-weight layer
(5120 -> 13824, rank 64), whose candidate set has no merged-weight graph.

What is timed is GPU time: the library records a pair of HIP events around every launch of a call
(runlora_profile_*), and a pair's time is the sum over its launches, median over repetitions.  Host
launch overhead is left out on purpose: it depends on the caller, not on the computation graph.
All non-default backward graphs need only X from the forward, so pair time = t_fwd + t_bwd and the
exhaustive search over pairs is a search over forwards plus a search over backwards.
"""
import numpy as np
import pytest

from helpers import torch_dtype
from paper_2312_03415_amd import binding as rl
from paper_2312_03415_amd import synth

pytestmark = pytest.mark.gpu

REPS = 7


def time_layer(L, int4=False):
    """{('fwd', v): us, ('bwd', v): us} of every variant (int4: of those that exist for an int4 W), GPU time per
    call (median of REPS)."""
    import torch
    td = torch_dtype(L.dtype)
    code = rl.dtype_from_name(L.dtype)
    g = torch.Generator(device="cuda").manual_seed(L.index)
    mk = lambda *s, scale=1.0: (torch.randn(*s, device="cuda", generator=g) * scale).to(td)
    X, dY = mk(L.n, L.i), mk(L.n, L.o)
    A, B = mk(L.i, L.r, scale=L.i ** -0.5), mk(L.r, L.o, scale=(0.1 / L.r) ** 0.5)
    if int4:
        q, scale = synth.int4_weight(L)
        W = rl.Int4Weight.from_host(q, scale)
        fwds, bwds, wd = (0, 1), (0, 1, 2, 3), rl.RL_INT4_G64
    else:
        W = mk(L.i, L.o, scale=L.i ** -0.5)
        fwds, bwds, wd = rl.FWD_VARIANTS, rl.BWD_VARIANTS, None
    Y, T = torch.empty(L.n, L.o, device="cuda", dtype=td), torch.empty(L.n, L.r, device="cuda", dtype=td)
    dX, dA, dB = (torch.empty(s, device="cuda", dtype=td) for s in ((L.n, L.i), (L.i, L.r), (L.r, L.o)))
    need = max(rl.runlora_workspace_bytes(f, b, L.n, L.i, L.o, L.r, code, wd) for f in fwds for b in bwds)
    ws = torch.empty(need + 256, dtype=torch.uint8, device="cuda")
    out = {}

    def measure(call):
        call()  # warm-up (also the first-launch attribute calls)
        torch.cuda.synchronize()
        times = []
        for _ in range(REPS):
            rl.runlora_profile_enable(64)
            call()
            torch.cuda.synchronize()
            times.append(sum(r["us"] for r in rl.runlora_profile_collect(64)))
            rl.runlora_profile_disable()
        return float(np.median(times))

    saved = {}
    for f in fwds:
        sv = rl.new_saved(T if f == rl.FWD_DEFAULT else None)
        out[("fwd", f)] = measure(lambda: rl.runlora_forward(f, X, W, A, B, Y, sv, workspace=ws))
        saved[f] = sv
    for b in bwds:
        sv = saved[rl.FWD_DEFAULT] if b == rl.BWD_DEFAULT else saved[rl.FWD1]
        if b == rl.BWD_DEFAULT:   # T must hold XA of this X again (other forwards reused the workspace, not T)
            rl.runlora_forward(rl.FWD_DEFAULT, X, W, A, B, Y, sv, workspace=ws)
        out[("bwd", b)] = measure(lambda: rl.runlora_backward(b, dY, sv, W, A, B, dX, dA, dB, workspace=ws))
    return out


def check_selection(L, int4=False):
    t = time_layer(L, int4)
    code = rl.RL_INT4_G64 if int4 else rl.dtype_from_name(L.dtype)
    fwd, bwd = rl.runlora_select(L.n, L.i, L.o, L.r, code)
    t_sel = t[("fwd", fwd)] + t[("bwd", bwd)]
    best_f = min((1,) if int4 else (1, 2, 3), key=lambda v: t[("fwd", v)])
    best_b = min((1, 2, 3) if int4 else (1, 2, 3, 4, 5), key=lambda v: t[("bwd", v)])
    t_best = t[("fwd", best_f)] + t[("bwd", best_b)]
    t_def = t[("fwd", 0)] + t[("bwd", 0)]
    if t_def < t_best:   # the default chain is a legal pair as well
        t_best, best_f, best_b = t_def, 0, 0
    model = {k: rl.runlora_model_time_us(k[0] == "bwd", k[1], L.n, L.i, L.o, L.r, code) for k in t}
    print(f"selector {L.name} {'int4 W ' if int4 else ''}{L.dtype} n={L.n} {L.i}->{L.o} r={L.r}: selected ({fwd},{bwd}) {t_sel:.1f} us; "
          f"best ({best_f},{best_b}) {t_best:.1f} us; default chain {t_def:.1f} us", flush=True)
    print("   measured " + " ".join(f"{k[0][0]}{k[1]}={v:.1f}" for k, v in sorted(t.items())), flush=True)
    print("   model    " + " ".join(f"{k[0][0]}{k[1]}={v:.1f}" for k, v in sorted(model.items())), flush=True)
    assert t_sel <= 1.05 * t_best, (L.name, (fwd, bwd), (best_f, best_b), t_sel, t_best)


@pytest.mark.parametrize("L", synth.config_selector_sweep("f16"), ids=lambda L: L.name)
def test_selected_pair_within_5_percent_of_best(L):
    check_selection(L)


BF16_LAYERS = synth.config_opt13b_mlp("bf16") + [x for r in (8, 32, 128) for x in synth.config_llama7b(r, "bf16") if x.name in ("q", "gate", "down")]


@pytest.mark.parametrize("L", BF16_LAYERS, ids=lambda L: f"{L.name}_{L.i}x{L.o}_r{L.r}")
def test_selected_pair_on_the_bench_layers(L):
    check_selection(L)


def test_selected_pair_on_the_int4_layer():
    check_selection(synth.config_qlora()[0], int4=True)
