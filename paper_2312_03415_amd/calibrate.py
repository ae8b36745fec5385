"""Measure the constants of the selector's time model on the GPU this runs on and write
csrc/model_constants.hpp (then rebuild the library):

    python -m paper_2312_03415_amd.calibrate [--out PATH]

Everything is timed through the library's own C ABI (runlora_gemm), the way a caller sees it: HIP
events around a batch of calls on one stream, rotating operand sets so that the 256 MB Infinity
Cache does not serve them, on problems long enough that the GPU and not the caller's launch rate
sets the time.  Per tile shape and operand layout two contraction lengths give the
time per K tile and the fixed cost of a round of workgroups; a third run with an addend gives the
fixed cost with D; the streaming kernel is timed on both orientations of the big operand; the
W + AB kernel on two sizes through the merged forward's own step timing; a tiny problem gives the
launch cost.
"""
import argparse
import os

import torch

from . import binding as rl

HERE = os.path.dirname(os.path.abspath(__file__))
TILE_BM = [256, 128, 128, 128, 32, 64, 256, 256]
TILE_BN = [256, 128, 32, 64, 128, 128, 256, 256]
TILE_BK16 = [64, 64, 64, 64, 64, 64, 32, 64]
WG_PER_CU = [1, 2, 3, 2, 3, 3, 1, 1]
NAMES = ["256x256", "128x128", "128x32", "128x64", "32x128", "64x128", "256x256x32 matrix-core (id 6)", "256x256x64 matrix-core (id 7)"]
LAYOUTS = {"NN": (0, 0), "NT": (0, 1), "TN": (1, 0)}
LAYOUT_ID = {"NN": 0, "NT": 1, "TN": 2}


def timeit(fn, iters=8, warm=2):
    for k in range(warm):
        fn(k)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for k in range(iters):
        fn(k)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters * 1e3


def gemm_time(dt, layout, M, N, K, cfg, K2=0, addend=False, splits=1, sets=3, trans=False):
    a_str, b_kc = LAYOUTS[layout]
    As = [torch.randn((K, M) if a_str else (M, K), device="cuda").to(dt) for _ in range(sets)]
    Bs = [(torch.randn((N, K) if b_kc else (K, N), device="cuda") / K ** 0.5).to(dt) for _ in range(sets)]
    C = torch.empty((N, M) if trans else (M, N), device="cuda", dtype=dt)
    D = torch.randn((M, N), device="cuda").to(dt) if addend else None
    A2 = torch.randn((M, K2), device="cuda").to(dt) if K2 else None
    B2 = torch.randn((N, K2) if b_kc else (K2, N), device="cuda").to(dt) if K2 else None
    ws = torch.empty(512 << 20, dtype=torch.uint8, device="cuda")
    return timeit(lambda k: rl.runlora_gemm(As[k % sets], Bs[k % sets], C, a_strided=a_str, b_kcontig=b_kc, A2=A2, B2=B2,
                                            D=D, tile_cfg=cfg, splits=splits, workspace=ws, trans_out=trans))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--out", default=os.path.join(HERE, "csrc", "model_constants.hpp"))
    args = ap.parse_args()
    rl.lib()
    bf, f32 = torch.bfloat16, torch.float32

    # cost of a launch on the GPU's side (dispatch + a kernel that does next to nothing): HIP events
    # recorded by the library around each step of a tiny layer
    n, i, o, r = 64, 64, 64, 8
    X, W = torch.randn(n, i, device="cuda").to(bf), torch.randn(i, o, device="cuda").to(bf)
    A, B = torch.randn(i, r, device="cuda").to(bf), torch.randn(r, o, device="cuda").to(bf)
    Y, T = torch.empty(n, o, device="cuda", dtype=bf), torch.empty(n, r, device="cuda", dtype=bf)
    ws = rl.new_workspace(0, 0, n, i, o, r, rl.RL_BF16)
    rl.runlora_profile_enable(4096)
    for _ in range(50):
        rl.runlora_forward(0, X, W, A, B, Y, rl.new_saved(T), workspace=ws)
    torch.cuda.synchronize()
    recs = rl.runlora_profile_collect(4096)
    rl.runlora_profile_disable()
    us = sorted(rec["us"] for rec in recs[30:])
    launch = us[len(us) // 2]
    print("launch_us", round(launch, 2), flush=True)

    tiles = {0: {}, 1: {}}
    for fam, dt in ((0, bf), (1, f32)):
        for cfg in range(8):
            if fam == 1 and cfg >= 6:
                tiles[fam][cfg] = dict(tiles[fam][0])   # fp32 falls back to the generic 256x256 tile
                continue
            bm, bn = TILE_BM[cfg], TILE_BN[cfg]
            bk = 32 if fam == 1 else TILE_BK16[cfg]
            slots = 256 * WG_PER_CU[cfg]
            # two full rounds of workgroups: 32 tile rows x (2*slots/32) tile columns
            M, N = bm * 32, bn * (2 * slots // 32)
            k_long, k_short = (2048, 256) if fam == 1 else (4096, 512)
            tk, fix = [], []
            for layout in ("NN", "NT", "TN"):
                t_long = gemm_time(dt, layout, M, N, k_long, cfg)
                t_short = gemm_time(dt, layout, M, N, k_short, cfg)
                per_tile = (t_long - t_short) / 2.0 / ((k_long - k_short) / bk)
                tk.append(max(per_tile, 1e-3))
                fix.append(max(t_short / 2.0 - (k_short / bk) * per_tile, 0.5))
            t_d = gemm_time(dt, "NN", M, N, k_short, cfg, addend=True)
            fix_d = max(t_d / 2.0 - (k_short / bk) * tk[0], fix[0])
            tiles[fam][cfg] = dict(tk=tk, fix=sum(fix) / 3.0, fix_d=fix_d)
            print(fam, NAMES[cfg], [round(v, 3) for v in tk], round(tiles[fam][cfg]["fix"], 2), round(fix_d, 2), flush=True)

    # W + AB kernel: per-step event times of the merged forward on two sizes -> rate and fixed cost
    def merge_time(i, o, r=32, n=256, sets=4):
        X = torch.randn(n, i, device="cuda").to(bf)
        As = [torch.randn(i, r, device="cuda").to(bf) for _ in range(sets)]
        Bs = [torch.randn(r, o, device="cuda").to(bf) for _ in range(sets)]
        Ws = [torch.randn(i, o, device="cuda").to(bf) for _ in range(sets)]
        Yb = torch.empty(n, o, device="cuda", dtype=bf)
        wss = [rl.new_workspace(2, -1, n, i, o, r, rl.RL_BF16) for _ in range(sets)]
        rl.runlora_profile_enable(4096)
        for k in range(20):
            rl.runlora_forward(2, X, Ws[k % sets], As[k % sets], Bs[k % sets], Yb, rl.new_saved(), workspace=wss[k % sets])
        torch.cuda.synchronize()
        rec = rl.runlora_profile_collect(4096)
        rl.runlora_profile_disable()
        m = sorted(x["us"] for x in rec[8:] if "W + A B" in x["what"])
        return m[len(m) // 2]
    tm_b, tm_s = merge_time(8192, 8192), merge_time(4096, 4096)
    merge_tbps = 2.0 * 2.0 * (8192.0 * 8192 - 4096.0 * 4096) / (tm_b - tm_s) / 1e6
    merge_fix = max(tm_s - 2.0 * 2.0 * 4096 * 4096 / merge_tbps / 1e6 - launch, 0.0)
    print("merge_tbps", round(merge_tbps, 2), "fix", round(merge_fix, 2), flush=True)

    # streaming kernel: two sizes per orientation -> rate and fixed cost
    def stream(layout, M, K, sets):
        return gemm_time(bf, layout, M, 32, K, 8, sets=sets)
    rates, fixes = [], []
    # both sizes rotate over > 512 MB of operands, beyond the 256 MB Infinity Cache
    # (and both run long enough that the GPU, not the caller's launch rate, sets the time)
    for layout, (Mb, Kb), (Ms, Ks) in (("NN", (16384, 8192), (8192, 8192)), ("TN", (8192, 16384), (8192, 8192))):
        tb, ts = stream(layout, Mb, Kb, 3), stream(layout, Ms, Ks, 5)
        bytes_b, bytes_s = 2.0 * Mb * Kb, 2.0 * Ms * Ks
        rate = (bytes_b - bytes_s) / (tb - ts) / 1e6          # TB/s
        rates.append(rate)
        fixes.append(max(ts - bytes_s / rate / 1e6, 0.0))
    print("stream_tbps", [round(v, 2) for v in rates], "fix", [round(v, 2) for v in fixes], flush=True)

    # second stage of a split contraction (partials written, read back and summed by the reduce kernel): what two split
    # launches take beyond their one-round model, a large output split in two on the matrix-core kernel and a small
    # one split sixteen ways on the 128x128 tile, gives a rate over the partials' bytes and a fixed cost
    def split_extra(layout, M, N, K, cfg, splits):
        t = gemm_time(bf, layout, M, N, K, cfg, splits=splits)
        kt = K // TILE_BK16[cfg] // splits
        return max(t - (kt * tiles[0][cfg]["tk"][LAYOUT_ID[layout]] + tiles[0][cfg]["fix"]), 1.0)
    x_big, b_big = split_extra("NT", 4096, 2048, 8192, 7, 2), 4096.0 * 2048 * (4 * 3 + 2)
    x_small, b_small = split_extra("NN", 128, 4096, 4096, 1, 16), 128.0 * 4096 * (4 * 17 + 2)
    reduce_tbps = (b_big - b_small) / max(x_big - x_small, 1.0) / 1e6
    reduce_fix = max(x_small - b_small / reduce_tbps / 1e6 - launch, 0.0)
    print("reduce_tbps", round(reduce_tbps, 2), "fix", round(reduce_fix, 2), "(extras", round(x_big, 1), round(x_small, 1), ")", flush=True)

    def row(t):
        return "{{%.3f, %.3f, %.3f}, %.2f, %.2f, %d}" % (t["tk"][0], t["tk"][1], t["tk"][2], t["fix"], t["fix_d"], t["wg"])

    lines = []
    for fam in (0, 1):
        rows = []
        for cfg in range(8):
            t = dict(tiles[fam][cfg], wg=WG_PER_CU[cfg])
            rows.append("           %s,  // %s" % (row(t), NAMES[cfg]))
        lines.append("       {\n" + "\n".join(rows) + "\n       }")
    body = ",\n".join(lines)
    text = open(os.path.join(HERE, "csrc", "model_constants.hpp")).read()  # keep the struct definitions
    head = text[:text.index("inline const ModelConstants& model_constants()")]
    out = head + """inline const ModelConstants& model_constants() {
  static const ModelConstants c = {
      {
%s},
      {%.2f, %.2f},
      %.2f,
      %.2f,
      %.2f,
      %.2f,
      %.2f,
      %.2f,
  };
  return c;
}

}  // namespace rl
""" % (body, rates[0], rates[1], sum(fixes) / 2.0, reduce_tbps, reduce_fix, launch, merge_tbps, merge_fix)
    with open(args.out, "w") as fh:
        fh.write(out)
    print("wrote", args.out)


if __name__ == "__main__":
    main()
