"""Forward+backward time of one transformer decoder block whose linear layers carry LoRA adapters, in
the shape of the whole-model comparisons of arxiv 2312.03415 (Section 3, Tables 2-8: same network, LoRA
on every attention and MLP linear, only the way the adapter layers are computed differs).

    python -m paper_2312_03415_amd.block_timing --model llama7b --batch 4 --seq 2048 --rank 32

Two ways to run the same block on the same synthetic weights and inputs:
  runlora   every linear is a RunLoRALinear with the pair runlora_select picks for its shape
  default   the same modules pinned to the default chain (pair (0, 0)): this library's kernels, one launch
            per product, XA kept for the backward

Attention, normalisation and activation are torch's own operators in both; weights are N(0, 1/d_in),
inputs N(0, 1), the upstream gradient N(0, 1); no dataset or checkpoint is involved.  Prints one JSON line.
"""
import argparse
import json
import math

import torch
import torch.nn.functional as F
from torch import nn

from .module import RunLoRALinear

MODELS = {
    # hidden, heads, mlp width, gated MLP (SwiGLU) or fc1-ReLU-fc2, bias on the linears, RMSNorm or LayerNorm
    "llama7b": dict(d=4096, heads=32, ffn=11008, gated=True, bias=False, rms=True),
    "llama13b": dict(d=5120, heads=40, ffn=13824, gated=True, bias=False, rms=True),
    "opt1.3b": dict(d=2048, heads=32, ffn=8192, gated=False, bias=True, rms=False),
    "opt6.7b": dict(d=4096, heads=32, ffn=16384, gated=False, bias=True, rms=False),
}


class RMSNorm(nn.Module):
    def __init__(self, d, dtype, device):
        super().__init__()
        self.weight = nn.Parameter(torch.ones(d, dtype=dtype, device=device), requires_grad=False)

    def forward(self, x):
        v = x.float()
        return (v * torch.rsqrt(v.pow(2).mean(-1, keepdim=True) + 1e-6)).to(x.dtype) * self.weight


class Block(nn.Module):
    """Pre-norm decoder block: x + attn(norm(x)), then x + mlp(norm(x)); causal attention."""

    def __init__(self, cfg, make_linear, dtype, device):
        super().__init__()
        d, ffn = cfg["d"], cfg["ffn"]
        self.heads = cfg["heads"]
        self.gated = cfg["gated"]
        norm = (lambda: RMSNorm(d, dtype, device)) if cfg["rms"] else (lambda: nn.LayerNorm(d, dtype=dtype, device=device))
        self.norm1, self.norm2 = norm(), norm()
        for p in list(self.norm1.parameters()) + list(self.norm2.parameters()):
            p.requires_grad_(False)
        self.q_proj, self.k_proj, self.v_proj, self.o_proj = (make_linear(name, d, d) for name in ("q", "k", "v", "o"))
        if self.gated:
            self.gate_proj, self.up_proj, self.down_proj = make_linear("gate", d, ffn), make_linear("up", d, ffn), make_linear("down", ffn, d)
        else:
            self.fc1, self.fc2 = make_linear("fc1", d, ffn), make_linear("fc2", ffn, d)

    def forward(self, x):
        b, s, d = x.shape
        h = self.norm1(x)
        split = lambda t: t.view(b, s, self.heads, d // self.heads).transpose(1, 2)
        a = F.scaled_dot_product_attention(split(self.q_proj(h)), split(self.k_proj(h)), split(self.v_proj(h)), is_causal=True)
        x = x + self.o_proj(a.transpose(1, 2).reshape(b, s, d))
        h = self.norm2(x)
        if self.gated:
            return x + self.down_proj(F.silu(self.gate_proj(h)) * self.up_proj(h))
        return x + self.fc2(F.relu(self.fc1(h)))


def build_block(cfg, kind, r, alpha, dtype, device, seed):
    """Same frozen weights and adapters for every kind (the generator is reseeded per linear)."""

    def make_linear(name, d_in, d_out):
        g = torch.Generator(device="cpu").manual_seed(seed + sum(map(ord, name)))
        w = (torch.randn(d_in, d_out, generator=g) / math.sqrt(d_in)).to(dtype).to(device)
        bias = (torch.randn(d_out, generator=g) * 0.02).to(dtype).to(device) if cfg["bias"] else None
        A = (torch.randn(d_in, r, generator=g) / math.sqrt(d_in)).to(dtype).to(device)
        B = (torch.randn(r, d_out, generator=g) * math.sqrt(0.1 / r)).to(dtype).to(device)
        lin = RunLoRALinear(w, r, alpha, bias, pair=(0, 0) if kind == "default" else None)
        with torch.no_grad():
            lin.lora_A.copy_(A)
            lin.lora_B.copy_(B)
        return lin

    return Block(cfg, make_linear, dtype, device)


def time_block(block, x, dy, iters, warmup):
    """Median milliseconds of forward + backward (gradients for x, every A and every B)."""
    times = []
    for it in range(warmup + iters):
        for p in block.parameters():
            p.grad = None
        x.grad = None
        t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0.record()
        y = block(x)
        y.backward(dy)
        t1.record()
        t1.synchronize()
        if it >= warmup:
            times.append(t0.elapsed_time(t1))
    times.sort()
    return times[len(times) // 2], y.detach()


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--model", choices=sorted(MODELS), default="llama7b")
    ap.add_argument("--batch", type=int, default=4)
    ap.add_argument("--seq", type=int, default=2048)
    ap.add_argument("--rank", type=int, default=32)
    ap.add_argument("--alpha", type=float, default=None, help="LoRA alpha (default: 2 r)")
    ap.add_argument("--dtype", choices=("bf16", "f16"), default="bf16")
    ap.add_argument("--iters", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--kinds", default="runlora,default")
    args = ap.parse_args(argv)

    if not torch.cuda.is_available():
        raise SystemExit("block_timing needs a GPU")
    device = torch.device("cuda:0")
    dtype = torch.bfloat16 if args.dtype == "bf16" else torch.float16
    cfg = MODELS[args.model]
    alpha = args.alpha if args.alpha is not None else 2.0 * args.rank
    g = torch.Generator(device="cpu").manual_seed(20231203)
    x0 = torch.randn(args.batch, args.seq, cfg["d"], generator=g).to(dtype).to(device)
    dy = torch.randn(args.batch, args.seq, cfg["d"], generator=g).to(dtype).to(device)

    out = {"model": args.model, "batch": args.batch, "seq": args.seq, "tokens": args.batch * args.seq, "rank": args.rank,
           "dtype": args.dtype, "data": "synthetic", "iters": args.iters, "ms_fwd_bwd": {}}
    ys = {}
    for kind in args.kinds.split(","):
        if kind not in ("runlora", "default"):
            raise SystemExit(f"unknown kind {kind!r}")
        block = build_block(cfg, kind, args.rank, alpha, dtype, device, seed=7)
        x = x0.clone().requires_grad_(True)
        ms, ys[kind] = time_block(block, x, dy, args.iters, args.warmup)
        out["ms_fwd_bwd"][kind] = round(ms, 4)
        if kind == "runlora":
            out["pairs"] = {name: list(m.pair_for(args.batch * args.seq)) for name, m in block.named_children()
                            if isinstance(m, RunLoRALinear)}
        del block, x
        torch.cuda.empty_cache()
    t = out["ms_fwd_bwd"]
    if "runlora" in t:
        if "default" in t:
            out["speedup_vs_default"] = round(t["default"] / t["runlora"], 4)
            out["saving_vs_default_pct"] = round(100.0 * (t["default"] - t["runlora"]) / t["default"], 2)
            # both blocks compute the same function: report how far the outputs are apart
            d = (ys["runlora"].double() - ys["default"].double()).norm() / ys["default"].double().norm()
            out["rel_diff_vs_default"] = float(f"{d.item():.3e}")
    print(json.dumps(out))
    return out


if __name__ == "__main__":
    main()
