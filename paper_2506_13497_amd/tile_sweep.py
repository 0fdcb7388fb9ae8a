"""Tuning aid for the linear's tile choice: times every compiled output tile on the model's
linears over a range of token counts and (optionally) refits the launcher's cost model.

    python -m paper_2506_13497_amd.tile_sweep                  # table: model's pick against every forced tile
    python -m paper_2506_13497_amd.tile_sweep --fit            # also least-squares constants for the model
    python -m paper_2506_13497_amd.tile_sweep --tokens 2304,3680

Needs a GPU.  Not on the hot path: it only calls ddit_linear_fwd_tile / ddit_linear_tile_choice.
The model (see the tile-choice comment in csrc/gemm_bf16.hip): with tiles = ceil(N/rows) ceil(n/cols),
q = ceil(tiles / CUs),
    t = (a k/1152 + e[epilogue]) q / gain[min(q, workgroups per CU)] (1 + load min(1, tiles/CUs)) + launch.
"""
from __future__ import annotations

import argparse
import math
import sys

import torch

from . import binding as b

# name, epilogue, out-features n, in-features k  (hidden 1152, MLP 4608)
LINEARS = [("qkv", 0, 3456, 1152), ("attn_out", 2, 1152, 1152), ("fc1", 1, 4608, 1152), ("fc2", 2, 1152, 4608),
           ("cross_q", 0, 1152, 1152), ("cross_kv", 0, 2304, 1152)]
TOKENS = [288, 576, 920, 1215, 1840, 2304, 2880, 3240, 3680, 4320, 4860, 5760, 6480, 7360, 8640, 9720, 11520, 12960,
          14400, 19440, 24300, 36000, 48600]


def time_linear(tile, epi, N, n, k, bufs, iters=20):
    u, W, bias, out, resid, tab, c6 = bufs

    def call():
        b.ddit_linear_fwd_tile(tile, epi, u, k, W, bias, N, n, k, None if epi == 2 else out, n,
                               resid=resid if epi == 2 else None, ada_table=tab if epi == 2 else None,
                               c6=c6 if epi == 2 else None, gate_row=2 if epi == 2 else -1, tokens_per_sample=N)
    for _ in range(3):
        call()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        call()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters * 1000.0


def sweep(tokens):
    count = b.ddit_linear_tile_count()
    tiles = [b.ddit_linear_tile_info(t) for t in range(count)]
    print("tiles: " + "  ".join("%d=%dx%d" % (i, t["rows"], t["cols"]) for i, t in enumerate(tiles)))
    print("%-9s %6s %5s %8s | " % ("linear", "N", "pick", "pick_us") + " ".join("%7s" % ("t%d_us" % i) for i in range(count))
          + " | pick/best")
    torch.manual_seed(0)
    data = []
    tab = torch.randn(6, 1152, device="cuda")
    c6 = torch.randn(1, 6 * 1152, device="cuda")
    for N in tokens:
        for name, epi, n, k in LINEARS:
            bufs = ((torch.randn(N, k, device="cuda") * 0.5).bfloat16(), (torch.randn(n, k, device="cuda") * 0.03).bfloat16(),
                    torch.randn(n, device="cuda").bfloat16(), torch.empty(N, n, device="cuda", dtype=torch.bfloat16),
                    torch.zeros(N, n, device="cuda") if epi == 2 else None, tab, c6)
            us = [time_linear(t, epi, N, n, k, bufs) for t in range(count)]
            pick = b.ddit_linear_tile_choice(epi, N, n, k)[0]
            pick_us = time_linear(-1, epi, N, n, k, bufs)
            print("%-9s %6d %5d %8.1f | " % (name, N, pick, pick_us) + " ".join("%7.1f" % x for x in us)
                  + " | %.2f" % (pick_us / min(us)), flush=True)
            data.append((epi, N, n, k, us))
    return tiles, data


def fit(tiles, data, cus):
    import numpy as np
    from scipy.optimize import least_squares
    count = len(tiles)

    def model(x, t, epi, N, n, k):
        a, e = x[4 * t], x[4 * t + 1 + epi]
        gain = (1.0, x[4 * count], x[4 * count + 1])
        load, launch = x[4 * count + 2], x[4 * count + 3]
        nt = math.ceil(N / tiles[t]["rows"]) * math.ceil(n / tiles[t]["cols"])
        q = math.ceil(nt / cus)
        return (a * k / 1152 + e) * q / gain[min(q, tiles[t]["workgroups_per_cu"]) - 1] * (1 + load * min(1.0, nt / cus)) + launch

    def resid(x):
        return np.array([math.log(max(model(x, t, epi, N, n, k), 1e-3) / us[t])
                         for epi, N, n, k, us in data for t in range(count)])
    x0 = []
    for t in tiles:
        area = t["rows"] * t["cols"] / (128.0 * 128.0)
        x0 += [8.0 * area ** 0.75, 1.0, 2.0, 4.0]
    x0 += [1.2, 1.3, 0.3, 1.0]
    lo = [0.0] * (4 * count) + [1.0, 1.0, 0.0, 0.0]      # times are not negative, sharing a CU does not cost
    sol = least_squares(resid, np.array(x0), loss="soft_l1", f_scale=0.1, bounds=(lo, np.inf))
    x = sol.x
    print("\nfitted constants (microseconds): rows x cols: a, e[bf16], e[GELU], e[residual]")
    for t in range(count):
        print("  %3d x %3d: %6.2f  %5.2f %5.2f %5.2f" % (tiles[t]["rows"], tiles[t]["cols"], *x[4 * t:4 * t + 4]))
    print("  gain for 2, 3 resident workgroups: %.2f %.2f   full-chip slow-down: %.2f   launch: %.2f"
          % tuple(x[4 * count:4 * count + 4]))
    r = resid(x)
    best = sum(min(us) for _, _, _, _, us in data)
    picked = sum(us[min(range(count), key=lambda t: model(x, t, epi, N, n, k))] for epi, N, n, k, us in data)
    print("  rms log error %.3f; total time of the fitted model's picks / of the best tiles: %.4f" %
          (float(np.sqrt((r ** 2).mean())), picked / best))


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--tokens", default=None, help="comma-separated token counts (default: 23 counts, 288..48600)")
    ap.add_argument("--fit", action="store_true", help="refit the cost model's constants to this sweep")
    args = ap.parse_args(argv)
    if not torch.cuda.is_available():
        sys.exit("tile_sweep needs a GPU")
    tokens = [int(v) for v in args.tokens.split(",")] if args.tokens else TOKENS
    tiles, data = sweep(tokens)
    if args.fit:
        fit(tiles, data, torch.cuda.get_device_properties(0).multi_processor_count)


if __name__ == "__main__":
    main()
