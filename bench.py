#!/usr/bin/env python3
"""Benchmark of the LoRA-linear hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload opt13b|llama7b] [--rank R]

A step = forward + backward of every layer of the workload, each in the (forward, backward) pair
that runlora_select picks, on seeded synthetic inputs already resident in HBM.  The default
workload is the OPT-1.3B-shaped MLP pair (tokens 8x512 = 4096, fc1 2048->8192, fc2 8192->2048,
rank 16, bf16).  Input/output sets are rotated so that the 256 MB Infinity Cache cannot serve
them between steps.  The same steps are also timed in the default chain (same kernels, one per
product, XA kept) for the speedup figure.

Prints ONE JSON line: the headline value is useful TFLOP/s = (fewest FLOPs any legal pair needs,
Table 1 of arxiv 2312.03415 plus the default chain) / measured time; `roofline` describes the
dominant kernel from per-launch HIP-event timings of an identical pass; `cpu_baseline` is the fp64
CPU oracle's default chain on a bounded token sample, on this machine's host cores.
"""
import argparse
import json
import sys
import time

import numpy as np

MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f16": 2500.0, "f32": 157.3}
HBM_PEAK_GBPS = 8000.0
TILE_NAMES = ["256x256", "128x128", "128x32", "128x64", "32x128", "64x128", "256x256mc3", "256x256mc", "stream32", "stream64", "stream128", "merge"]

# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
# (profiles/), scaled by what the same counters read for a copy kernel of known size; None until
# measured for the workload.
TRAFFIC_BYTES = {
    # profiles/bench_opt13b_hbm_traffic.txt: (FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0) KiB per launch, all
    # launches of the matrix-core kernel of that layout together (all of its builds)
    ("opt13b", "gemm_kernel<bf16,NN,256x256mc>"): int((133129 * 2.0 + 65536) * 1024),
    ("opt13b", "gemm_kernel<bf16,NT,256x256mc>"): int((132490 * 2.0 + 65536) * 1024),
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="opt13b", choices=["opt13b", "llama7b", "qlora"])
    ap.add_argument("--rank", type=int, default=None, help="LoRA rank override (llama7b: 8/32/128)")
    ap.add_argument("--sets", type=int, default=4, help="rotating input/output sets (together beyond the 256 MB Infinity Cache)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--keep-merged", action="store_true",
                    help="let forward2 keep W + AB for backward4/5 (i*o elements held per layer; pairs chosen for that)")
    ap.add_argument("--dropout", type=float, default=0.0,
                    help="LoRA dropout probability (0 = the paper's setting); pairs are then (1,1), the only RunLoRA graphs that exist with it")
    ap.add_argument("--dora", action="store_true",
                    help="run the layers as DoRA (trainable magnitudes m on top of A, B) through runlora_dora_*: forward2 + a merged "
                         "backward (5, or the second number of --pair); the default-chain leg is then the LoRA layer's")
    ap.add_argument("--vera", action="store_true",
                    help="run the layers as VeRA (frozen A, B, trainable vectors d and b; use with --rank 256 or so) through runlora_vera_*")
    ap.add_argument("--pair", default=None, help="force one 'fwd,bwd' pair on every layer instead of runlora_select")
    ap.add_argument("--copy-probe", action="store_true",
                    help="only run a 1 GiB device copy five times (reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU (no collectives, no sharding); use --gpus 1")

    import torch

    from paper_2312_03415_amd import binding as rl
    from paper_2312_03415_amd import synth

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    rl.lib()  # fail loudly if the HIP library is missing
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.copy_probe:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)   # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_bytes_read": src.numel() * 4, "copy_probe_bytes_written": src.numel() * 4, "copies": 5}))
        return

    if args.workload == "opt13b":
        layers = synth.config_opt13b_mlp("bf16")
        if args.rank:
            layers = [synth.Layer(L.name, L.n, L.i, L.o, args.rank, L.dtype, L.index) for L in layers]
        wl_name = "OPT-1.3B-shaped MLP pair, tokens 8x512=4096, fc1 2048x8192 + fc2 8192x2048, r=%d" % layers[0].r
    elif args.workload == "llama7b":
        layers = synth.config_llama7b(args.rank or 32, "bf16")
        wl_name = "Llama-7B-shaped block, tokens 4x2048=8192, q/k/v/o + gate/up + down, r=%d" % layers[0].r
    else:
        layers = synth.config_qlora()
        if args.rank:
            layers = [synth.Layer(L.name, L.n, L.i, L.o, args.rank, L.dtype, L.index) for L in layers]
        wl_name = "frozen W 5120x13824 as int4 (groups of 64, fp16 scales), tokens 4096, r=%d, bf16 activations" % layers[0].r
    int4 = args.workload == "qlora"
    dtype = layers[0].dtype
    code = rl.dtype_from_name(dtype)
    tdt = {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}[dtype]

    def to_dev(stored):
        if dtype == "bf16":
            return torch.from_numpy(stored.view(np.int16)).view(torch.bfloat16).to(dev)
        return torch.from_numpy(stored).to(dev)

    # ---- inputs (seeded, synthetic), `sets` device copies per layer --------------------------
    host_inputs = []
    state = []
    for L in layers:
        st = synth.layer_inputs(L)
        host_inputs.append(st)
        base = {k: to_dev(v) for k, v in st.items()}
        if int4:  # the frozen weight in its 4-bit form; the dense copy is only the CPU baseline's
            q, scale = synth.int4_weight(L)
            base["W"] = rl.Int4Weight.from_host(q, scale)
            st["W"] = synth.store(q.astype(np.float64) * np.repeat(scale.astype(np.float64), 64, axis=0)[:L.i], dtype)
        sets = []
        for s in range(args.sets):
            t = {k: (v if (s == 0 or k == "W" and int4) else v.clone()) for k, v in base.items()}
            t["Y"] = torch.empty((L.n, L.o), dtype=tdt, device=dev)
            t["T"] = torch.empty((L.n, L.r), dtype=tdt, device=dev)
            t["dX"] = torch.empty((L.n, L.i), dtype=tdt, device=dev)
            t["dA"] = torch.empty((L.i, L.r), dtype=tdt, device=dev)
            t["dB"] = torch.empty((L.r, L.o), dtype=tdt, device=dev)
            t["M"] = torch.empty((L.i, L.o), dtype=tdt, device=dev) if args.keep_merged else None
            if args.dora:
                t["m"] = to_dev(synth.store(0.5 + np.abs(synth.normal(synth.BASE_SEED + L.index, 10, (L.o,))), dtype))
                t["c"] = torch.empty((L.o,), dtype=torch.float32, device=dev)
                t["dm"] = torch.empty((L.o,), dtype=tdt, device=dev)
            if args.vera:
                t["d"] = to_dev(synth.store(synth.normal(synth.BASE_SEED + L.index, 10, (L.r,)), dtype))
                t["b"] = to_dev(synth.store(synth.normal(synth.BASE_SEED + L.index, 11, (L.o,)), dtype))
                t["dd"] = torch.empty((L.r,), dtype=tdt, device=dev)
                t["db"] = torch.empty((L.o,), dtype=tdt, device=dev)
            sets.append(t)
        if args.dora:
            fwd, bwd = 2, (int(args.pair.split(",")[1]) if args.pair else 5)
        elif args.dropout > 0.0:
            fwd, bwd = 1, 1
        elif args.pair:
            fwd, bwd = (int(v) for v in args.pair.split(","))
        else:
            fwd, bwd = rl.runlora_select(L.n, L.i, L.o, L.r, rl.RL_INT4_G64 if int4 else code,
                                         criterion=2 if args.keep_merged else None)
        wd = rl.RL_INT4_G64 if int4 else None
        ws_bytes = max(rl.runlora_workspace_bytes(fwd, bwd, L.n, L.i, L.o, L.r, code, wd),
                       rl.runlora_workspace_bytes(0, 0, L.n, L.i, L.o, L.r, code, wd))
        if args.vera:
            ws_bytes = max(rl.runlora_vera_workspace_bytes(fwd, bwd, L.n, L.i, L.o, L.r, code),
                           rl.runlora_vera_workspace_bytes(0, 0, L.n, L.i, L.o, L.r, code))
        if args.dora:
            ws_bytes = max(ws_bytes, rl.runlora_dora_workspace_bytes(fwd, bwd, L.n, L.i, L.o, L.r, code))
        ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)
        state.append(dict(L=L, sets=sets, pair=(fwd, bwd), ws=ws))

    def step(k, default_chain, only=None):
        for st in (state if only is None else [only]):
            t = st["sets"][k % args.sets]
            fwd, bwd = (0, 0) if default_chain else st["pair"]
            saved = rl.new_saved(t["T"] if fwd == 0 else None, t["M"] if fwd == 2 and bwd in rl.BWD_MERGED else None)
            if args.dora and not default_chain:
                rl.runlora_dora_forward(fwd, t["X"], t["W"], t["A"], t["B"], t["m"], t["Y"], saved, t["c"], st["ws"])
                rl.runlora_dora_backward(bwd, t["dY"], saved, t["W"], t["A"], t["B"], t["m"], t["c"], t["Y"], t["dX"], t["dA"],
                                         t["dB"], t["dm"], st["ws"])
                continue
            if args.vera:
                rl.runlora_vera_forward(fwd, t["X"], t["W"], t["A"], t["B"], t["d"], t["b"], t["Y"], saved, st["ws"])
                rl.runlora_vera_backward(bwd, t["dY"], saved, t["W"], t["A"], t["B"], t["d"], t["b"], t["dX"], t["dd"],
                                         t["db"], st["ws"])
                continue
            rl.runlora_forward(fwd, t["X"], t["W"], t["A"], t["B"], t["Y"], saved, workspace=st["ws"],
                               dropout_p=args.dropout or None, dropout_seed=k)
            rl.runlora_backward(bwd, t["dY"], saved, t["W"], t["A"], t["B"], t["dX"], t["dA"], t["dB"],
                                workspace=st["ws"])

    def timed(default_chain):
        for k in range(args.warmup):
            step(k, default_chain)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(args.steps):
            step(k, default_chain)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / args.steps

    sec_sel = timed(False)
    sec_def = timed(True)

    # ---- useful FLOPs: the fewest any legal pair needs ---------------------------------------
    def useful_flops(L):
        best = None
        for f in ((0, 1) if int4 else (0, 1, 2)):          # an int4 W has no merged-weight graphs
            for b in ((0, 1, 2, 3) if int4 else (0, 1, 2, 3, 4, 5)):
                if b == 0 and f != 0:
                    continue
                fl = rl.runlora_flops(0, f, L.n, L.i, L.o, L.r) + rl.runlora_flops(1, b, L.n, L.i, L.o, L.r)
                best = fl if best is None else min(best, fl)
        if args.vera:  # no gradient for A: its product, X^T (dY B^T) or (X^T dY) B^T, is not part of the layer
            best -= 2 * L.r * L.i * min(L.n, L.o)
        return best

    f_useful = sum(useful_flops(L) for L in layers)
    value = f_useful / sec_sel / 1e12

    # ---- per layer: forward + backward of the selected pair and of the default chain, median of
    # `steps` iterations, HIP events on the launch stream around each iteration
    def layer_ms(st, default_chain):
        for k in range(args.warmup):
            step(k, default_chain, st)
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
        for k, (e0, e1) in enumerate(ev):
            e0.record()
            step(k, default_chain, st)
            e1.record()
        torch.cuda.synchronize()
        ts = sorted(e0.elapsed_time(e1) for e0, e1 in ev)
        return ts[len(ts) // 2]

    per_layer = []
    for st in state:
        L = st["L"]
        ms_sel, ms_def = layer_ms(st, False), layer_ms(st, True)
        per_layer.append(dict(name=L.name, pair=list(st["pair"]), ms=round(ms_sel, 4), ms_default_chain=round(ms_def, 4),
                              speedup=round(ms_def / ms_sel, 4), useful_tflops=round(useful_flops(L) / ms_sel / 1e9, 1)))

    # ---- per-kernel timings of an identical pass (HIP events the library binds, on the launch stream, to the
    # dispatch of every step's main kernel: the kernel's own duration) -> roofline of the dominant kernel
    rl.runlora_profile_kernel_times(True)
    rl.runlora_profile_enable(args.steps * len(layers) * 16)
    for k in range(args.steps):
        step(k, False)
    torch.cuda.synchronize()
    recs = rl.runlora_profile_collect(args.steps * len(layers) * 16)
    rl.runlora_profile_disable()
    rl.runlora_profile_kernel_times(False)
    groups = {}
    ridge = MFMA_PEAK_TFLOPS[dtype] * 1e12 / (HBM_PEAK_GBPS * 1e9)
    for r in recs:
        lay = "NN" if not r["a_strided"] and not r["b_kcontig"] else ("NT" if r["b_kcontig"] else "TN")
        # the same kernel serves compute-bound contractions and memory-bound ones (W + AB has K = r)
        key = (lay, TILE_NAMES[r["tile_cfg"]] + ("" if r["flops"] / r["bytes"] >= ridge else "/mem"))
        # the kernel's own duration (what a kernel trace reports for it); the reduce pass behind a split contraction
        # is a kernel of its own and is not in these figures
        g = groups.setdefault(key, dict(us=0.0, flops=0.0, bytes=0.0, launches=0, what=set()))
        g["us"] += r["kernel_us"]; g["flops"] += r["flops"]; g["bytes"] += r["bytes"]; g["launches"] += 1
        g["what"].add(r["what"])
    dom_key = max(groups, key=lambda k: groups[k]["us"])
    dom = groups[dom_key]
    total_kernel_us = sum(g["us"] for g in groups.values())
    intensity = dom["flops"] / dom["bytes"]
    kname = "gemm_kernel<%s,%s,%s>" % (dtype, dom_key[0], dom_key[1])
    if intensity >= ridge:
        ach = dom["flops"] / dom["us"] / 1e6
        roofline = dict(bound="mfma", achieved=round(ach, 1), peak=MFMA_PEAK_TFLOPS[dtype], unit="TFLOP/s",
                        frac=round(ach / MFMA_PEAK_TFLOPS[dtype], 4))
    else:
        ach = dom["bytes"] / dom["us"] / 1e3
        roofline = dict(bound="hbm", achieved=round(ach, 1), peak=HBM_PEAK_GBPS, unit="GB/s",
                        frac=round(ach / HBM_PEAK_GBPS, 4))
    if roofline["bound"] == "mfma":
        # what a bare MFMA loop sustains on this (power-limited) GPU: on zeros, and on random operands
        roofline["mfma_probe_tflops"] = {"zeros": round(rl.runlora_probe_mfma(False), 1),
                                         "random": round(rl.runlora_probe_mfma(True), 1)}
        roofline["frac_of_random_data_probe"] = round(ach / roofline["mfma_probe_tflops"]["random"], 4)
    roofline.update(traffic=TRAFFIC_BYTES.get((args.workload, kname)), kernel=kname,
                    products=sorted(dom["what"]), launches_per_step=dom["launches"] / args.steps,
                    avg_launch_us=round(dom["us"] / dom["launches"], 2),
                    share_of_kernel_time=round(dom["us"] / total_kernel_us, 3))
    per_kernel = {"%s/%s" % k: dict(us_per_step=round(g["us"] / args.steps, 1),
                                    tflops=round(g["flops"] / g["us"] / 1e6, 1),
                                    alg_gbps=round(g["bytes"] / g["us"] / 1e3, 1)) for k, g in groups.items()}

    # ---- CPU baseline: the oracle's default chain on a bounded token sample ---------------------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        sample = 512
        t_cpu, fl_cpu = 0.0, 0
        for L, st in zip(layers, host_inputs):
            h = {k: synth.widen(v, dtype) for k, v in st.items()}
            X, dY = h["X"][:sample].copy(), h["dY"][:sample].copy()
            t0 = time.perf_counter()
            _, T = oracle.forward(0, X, h["W"], h["A"], h["B"])
            oracle.backward(0, X, h["W"], h["A"], h["B"], dY, T)
            t_cpu += time.perf_counter() - t0
            fl_cpu += rl.runlora_flops(0, 0, sample, L.i, L.o, L.r) + rl.runlora_flops(1, 0, sample, L.i, L.o, L.r)
        cpu = dict(value=round(fl_cpu / t_cpu / 1e12, 5), unit="TFLOP/s", cores=oracle.num_threads(), kind="oracle",
                   sample="default chain fwd+bwd, fp64, first %d of %d tokens of each layer, full weights; %.1f s"
                          % (sample, layers[0].n, t_cpu))

    out = {
        "metric": "LoRA-linear fwd+bwd useful TFLOP/s + speedup over default chain, bf16",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec_sel * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dtype, "data": "synthetic",
        "config": {"workload": wl_name, "layers": [dict(name=L.name, n=L.n, d_in=L.i, d_out=L.o, r=L.r) for L in layers],
                   "pairs": {st["L"].name: list(st["pair"]) for st in state}, "input_sets": args.sets,
                   "keep_merged": bool(args.keep_merged), "lora_dropout": args.dropout,
                   "adapter": "vera" if args.vera else ("dora" if args.dora else "lora")},
        "ms_per_step_default_chain": round(sec_def * 1e3, 4),
        "speedup_over_default_chain": round(sec_def / sec_sel, 4),
        "time_reduction_pct": round(100.0 * (sec_def - sec_sel) / sec_def, 2),
        "useful_gflop_per_step": round(f_useful / 1e9, 2),
        "per_layer": per_layer, "roofline": roofline, "kernels": per_kernel, "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
