#!/usr/bin/env python3
"""Benchmark of the STDiT denoising step on one MI355X.

A step = one full pass of the hot path (timestep conditioning + 28 blocks = 56 layers) over one
synthetic batch.  The default run times the 480p workload (B=1, T=30, 30x54 tokens per frame,
L=48600, hidden 1152, 16 heads x 72, MLP 4608, 300 text tokens with a seeded padding mask: `value`)
and then the 720p share of a 4-way head split (L=108000, 4 of 16 heads), and reports both in ONE
JSON line, each with its per-kernel table.  Inputs and weights are resident in HBM before the timed
regions.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C4|C5|C3|C2] [--no-cpu]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E, published

WORKLOAD_NAMES = {"C2": "144p", "C3": "240p-b2", "C4": "480p", "C5": "720p-share-4of16-heads"}

# kernel groups of a step: key -> (kernel template in the rocprofv3 trace, bound, profile file with the measured HBM traffic)
KERNEL_GROUPS = {
    "gemm_residual": ("k_gemm_bf16<..., EPI=2> (fc2, attention and cross-attention out-projections: gated fp32 residual update)", "mfma"),
    "gemm_gelu": ("k_gemm_bf16<..., EPI=1> (MLP fc1 + GELU)", "mfma"),
    "gemm_bf16": ("k_gemm_bf16<..., EPI=0> (q|k|v and cross-attention q projections)", "mfma"),
    "spatial_attention": ("k_flash_attn (streaming form: spatial self-attention)", "mfma"),
    "cross_attention": ("k_flash_attn (resident form: cross-attention)", "mfma"),
    "temporal_attention": ("k_temporal_attn", "hbm"),
    "modulated_layernorm": ("k_modulated_layernorm", "hbm"),
}


def step_flops(sh, valid):
    """Algorithmic FLOPs of one step: 2*m*n*k per linear, 4*Lq*Lk*dh per attention head (head dim 72,
    not the padded width; cross-attention counted at the actual valid text length)."""
    N, D, A, M, S, T, L, Ly = sh.N, sh.D, sh.A, sh.M, sh.S, sh.T, sh.L, sh.Ly
    lin = lambda rows, n, k: 2.0 * rows * n * k
    per_layer_common = lin(N, 3 * A, D) + lin(N, D, A) + lin(N, A, D) + lin(sh.B * Ly, 2 * A, D) + lin(N, D, A) \
        + lin(N, M, D) + lin(N, D, M)
    cross = sum(4.0 * L * int(v) * A for v in valid)
    spatial = 4.0 * N * S * A
    temporal = 4.0 * N * T * A
    per_block = 2 * per_layer_common + 2 * cross + spatial + temporal
    return {"step": sh.n_blocks * per_block, "gemm_layer": per_layer_common, "spatial": spatial,
            "temporal": temporal, "cross": cross, "fc1": lin(N, M, D)}


def measured_traffic(group, workload):
    """HBM bytes per launch of a kernel group as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (two
    runs, scaled by what the same counters read for a plain copy kernel of known size); the figure is kept,
    with the commands that produced it, in profiles/.  None if not measured for this workload."""
    path = os.path.join(ROOT, "profiles", "%s_%s_hbm_traffic.txt" % (group, WORKLOAD_NAMES[workload].split("-")[0]))
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return int(float(line.split(":", 1)[1]))
    except OSError:
        pass
    return None


# per-step time of one rank at degree of parallelism p (section 4.2.3): latent shapes by resolution
DOP_RESOLUTIONS = [("144p", 16, 9, 16), ("240p", 16, 15, 27), ("360p", 16, 23, 40), ("480p", 30, 30, 54),
                   ("720p", 30, 45, 80)]
XGMI_GBS_PER_PEER = 60.0   # assumed one-direction payload rate of one xGMI link (published 153.6 GB/s both ways)


def dop_table(m, syn, torch, steps):
    """DiT_step_time(parallel size p, resolution r) on this GPU for one rank of a dynamic-sequence-
    parallel run, and the change rate z = 1 - t(p)/t(p/2) the paper's greedy scheduler derives its
    per-resolution GPU count B from (section 4.2.3).  One rank's share: ceil(T/p) frames of the
    request (spatial layers are sharded by frame; the temporal layers' share, S/p locations over all
    frames, has the same token count, and every other stage is token-wise).  The two all-to-alls per
    block are NOT run (one GPU per box): their time is modelled from the bytes and an assumed link
    rate, and reported beside the measured compute."""
    base_sh = syn.CONFIGS["C4"]["shape"]
    gen = torch.Generator(device="cuda")
    gen.manual_seed(77)
    draw = lambda shape_, std, dt=torch.bfloat16: (torch.randn(shape_, generator=gen, device="cuda") * std).to(torch.bfloat16).to(dt)
    sw = {k: draw(s_, 0.02) for k, s_ in syn.step_shapes(base_sh).items()}
    blocks = [{kind: {n: draw(s_, 0.02, torch.float32 if n == "ada_table" else torch.bfloat16)
                      for n, s_ in syn.layer_shapes(base_sh).items()} for kind in ("spatial", "temporal")}
              for _ in range(base_sh.n_blocks)]
    st = m.step_struct(sw, blocks)
    rows = []
    for name, T, Hp, Wp in DOP_RESOLUTIONS:
        t_ms, comm_ms = {}, {}
        for p in (1, 2, 4, 8):
            Tp = -(-T // p)
            sh = syn.small_variant(base_sh, T=Tp, Hp=Hp, Wp=Wp)
            shape = m.make_shape(sh.B, sh.T, sh.Hp, sh.Wp, sh.D, sh.H, sh.dh, sh.M, sh.Ly, sh.n_blocks)
            ws = m.alloc_workspace(shape)
            x_in, y = draw((sh.B, sh.T, sh.S, sh.D), 1.0), draw((sh.B, sh.Ly, sh.D), 1.0)
            x_out = torch.empty_like(x_in)
            run = lambda: m.ddit_denoise_step(shape, st, x_in, y, None, [500.0], None, x_out, ws)
            run()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                run()
            torch.cuda.synchronize()
            t_ms[p] = (time.perf_counter() - t0) * 1e3 / steps
            # per block two all-to-alls; a rank sends N_rank*D*2 bytes, (p-1)/p of it to p-1 peers in parallel
            per_peer = sh.N * sh.D * 2.0 / p if p > 1 else 0.0
            comm_ms[p] = 2 * sh.n_blocks * per_peer / (XGMI_GBS_PER_PEER * 1e9) * 1e3
            del ws, x_in, x_out
        z = {p: 1.0 - t_ms[p] / t_ms[p // 2] for p in (2, 4, 8)}
        zc = {p: 1.0 - (t_ms[p] + comm_ms[p]) / (t_ms[p // 2] + comm_ms[p // 2]) for p in (2, 4, 8)}
        rows.append({"resolution": name, "T": T, "Hp": Hp, "Wp": Wp,
                     "step_ms": {str(p): round(v, 3) for p, v in t_ms.items()},
                     "modelled_exchange_ms": {str(p): round(v, 3) for p, v in comm_ms.items()},
                     "z_compute": {str(p): round(v, 4) for p, v in z.items()},
                     "z_with_exchange": {str(p): round(v, 4) for p, v in zc.items()},
                     "B_argmax_z_with_exchange": max(zc, key=zc.get)})
        print("[bench] %s: %s" % (name, json.dumps(rows[-1])), file=sys.stderr, flush=True)
    return rows


# the model's linears (hidden 1152, MLP 4608): name, epilogue, out-features, in-features
SWEEP_LINEARS = [("qkv", 0, 3456, 1152), ("attn_out", 2, 1152, 1152), ("fc1", 1, 4608, 1152), ("fc2", 2, 1152, 4608),
                 ("cross_q", 0, 1152, 1152), ("cross_kv", 0, 2304, 1152)]
SWEEP_TOKENS = [288, 576, 920, 1215, 1840, 2304, 2880, 3240, 3680, 4320, 4860, 5760, 6480, 7360, 8640, 9720, 11520, 12960,
                14400, 19440, 24300, 36000, 48600]


def tile_sweep(m, torch, tokens):
    """Every compiled output tile of the linear forced in turn (ddit_linear_fwd_tile) on the model's linears over a
    range of token counts, beside the launcher's own pick: the table the launcher's cost model was fitted to."""
    count = m.ddit_linear_tile_count()
    tiles = [m.ddit_linear_tile_info(t) for t in range(count)]
    print("tiles: " + "  ".join("%d=%dx%d" % (i, t["rows"], t["cols"]) for i, t in enumerate(tiles)))
    print("%-9s %6s %5s %8s | " % ("linear", "N", "pick", "pick_us") + " ".join("%7s" % ("t%d_us" % i) for i in range(count))
          + " | pick/best")
    torch.manual_seed(0)
    tab, c6 = torch.randn(6, 1152, device="cuda"), torch.randn(1, 6 * 1152, device="cuda")
    ratios = []
    for N in tokens:
        for name, epi, n, k in SWEEP_LINEARS:
            u, W = (torch.randn(N, k, device="cuda") * 0.5).bfloat16(), (torch.randn(n, k, device="cuda") * 0.03).bfloat16()
            bias, out = torch.randn(n, device="cuda").bfloat16(), torch.empty(N, n, device="cuda", dtype=torch.bfloat16)
            resid = torch.zeros(N, n, device="cuda") if epi == 2 else None

            def timed(tile):
                call = lambda: m.ddit_linear_fwd_tile(tile, epi, u, k, W, bias, N, n, k, None if epi == 2 else out, n, resid=resid,
                                                      ada_table=tab if epi == 2 else None, c6=c6 if epi == 2 else None,
                                                      gate_row=2 if epi == 2 else -1, tokens_per_sample=N)
                for _ in range(3):
                    call()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(20):
                    call()
                e1.record()
                e1.synchronize()
                return e0.elapsed_time(e1) / 20 * 1000.0
            us = [timed(t) for t in range(count)]
            pick, pick_us = m.ddit_linear_tile_choice(epi, N, n, k)[0], timed(-1)
            ratios.append(pick_us / min(us))
            print("%-9s %6d %5d %8.1f | " % (name, N, pick, pick_us) + " ".join("%7.1f" % x for x in us)
                  + " | %.2f" % ratios[-1], flush=True)
    print("rows %d; pick / best: mean %.3f, worst %.2f" % (len(ratios), sum(ratios) / len(ratios), max(ratios)))


class Workload:
    """One configuration resident on the device: weights, inputs, workspace, the step call."""

    def __init__(self, m, syn, torch, name):
        self.m, self.torch, self.name = m, torch, name
        cfg = syn.CONFIGS[name]
        self.sh, self.base = sh, base = cfg["shape"], cfg["base"]
        t0 = time.time()
        # Weights are drawn on the device (seeded torch generator, same N(0, 0.02^2) distribution and
        # shapes as ddit_synth, which the parity tests use): 1.2 G numpy draws would take minutes.
        gen = torch.Generator(device="cuda")
        gen.manual_seed(1000 + base)

        def draw(shape_, std, dtype=torch.bfloat16):
            t = torch.randn(shape_, generator=gen, device="cuda", dtype=torch.float32) * std
            return t.to(torch.bfloat16).to(dtype)   # fp32 tensors hold bf16-representable values
        self.draw = draw
        self.sw = {k: draw(s_, 0.02) for k, s_ in syn.step_shapes(sh).items()}
        self.blocks = []
        for _ in range(sh.n_blocks):
            self.blocks.append({kind: {n: draw(s_, 0.02, torch.float32 if n == "ada_table" else torch.bfloat16)
                                       for n, s_ in syn.layer_shapes(sh).items()} for kind in ("spatial", "temporal")})
        for wb in self.blocks:   # scales of the optional q/k normalisation (read only by the variant timed after the step)
            for lw_ in wb.values():
                lw_["g_q"] = (1.0 + draw((sh.dh,), 0.2, torch.float32)).to(torch.bfloat16)
                lw_["g_k"] = (1.0 + draw((sh.dh,), 0.2, torch.float32)).to(torch.bfloat16)
        self.x_in, self.y = draw((sh.B, sh.T, sh.S, sh.D), 1.0), draw((sh.B, sh.Ly, sh.D), 1.0)
        self.valid = [int(v) for v in syn.make_valid_len(sh, base, cfg["valid"])]
        self.tsteps = [float(t) for t in syn.make_timesteps(sh, base, cfg["t"])]
        self.shape = m.make_shape(sh.B, sh.T, sh.Hp, sh.Wp, sh.D, sh.H, sh.dh, sh.M, sh.Ly, sh.n_blocks)
        self.ws = m.alloc_workspace(self.shape)
        self.st = m.step_struct(self.sw, self.blocks)
        self.x_out = torch.empty_like(self.x_in)
        self.fl = step_flops(sh, self.valid)
        torch.cuda.synchronize()
        print("[bench] %s: inputs+weights resident after %.1fs (workspace %.2f GB)" %
              (name, time.time() - t0, self.ws.numel() / 1e9), file=sys.stderr, flush=True)

    def one_step(self):
        self.m.ddit_denoise_step(self.shape, self.st, self.x_in, self.y, self.valid, self.tsteps, None, self.x_out, self.ws)

    def time_steps(self, steps, warmup):
        torch = self.torch
        for _ in range(warmup):
            self.one_step()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(steps):
            self.one_step()
        torch.cuda.synchronize()
        ms = max((time.perf_counter() - t1) * 1e3 / max(steps, 1), 1e-9)
        # outside the timed region: the step's output must be finite everywhere
        assert bool(torch.isfinite(self.x_out.float()).all()), "%s: non-finite values in the step's output" % self.name
        return ms

    def describe(self):
        sh = self.sh
        return "%s (%s): B=%d T=%d S=%d L=%d D=%d heads=%dx%d M=%d Ly=%d valid=%s blocks=%d" % (
            self.name, WORKLOAD_NAMES[self.name], sh.B, sh.T, sh.S, sh.L, sh.D, sh.H, sh.dh, sh.M, sh.Ly, self.valid, sh.n_blocks)

    def kernel_table(self, reps):
        """Every kernel of a block timed where it runs in the step: the launches of a spatial and a temporal layer
        issued in the step's order through the single-stage entry points (the same kernels on the same shapes,
        each reading what the launch before it wrote), one HIP event pair per launch on the stream the kernels run
        on, averaged over `reps` passes with a different block's weights each.  Returns the per-group table
        (launches per step, average duration, share of the step, achieved rate against its roofline)."""
        m, torch, sh = self.m, self.torch, self.sh
        N, D, A, M, L = sh.N, sh.D, sh.A, sh.M, sh.L
        dev = "cuda"
        x32 = torch.randn(N, D, device=dev)
        c6 = (torch.randn(sh.B, 6 * D, device=dev) * 0.5)
        xh = torch.empty(N, D, dtype=torch.bfloat16, device=dev)
        qkv = torch.empty(N, 3 * A, dtype=torch.bfloat16, device=dev)
        o = torch.empty(N, A, dtype=torch.bfloat16, device=dev)
        kvc = torch.randn(sh.B * sh.Ly, 2 * A, device=dev).to(torch.bfloat16)
        h = torch.empty(N, M, dtype=torch.bfloat16, device=dev)
        ev = lambda: torch.cuda.Event(enable_timing=True)
        records = []   # (group, e0, e1, algorithmic flops, algorithmic bytes)
        fl = self.fl

        def timed(group, fn, flops=0.0, nbytes=0.0):
            e0, e1 = ev(), ev()
            e0.record()
            fn()
            e1.record()
            records.append((group, e0, e1, flops, nbytes, (kind_now[0], len(records) - layer_start[0])))

        lin = lambda n, k: 2.0 * N * n * k

        kind_now, layer_start = [None], [0]

        def layer(kind, lw, keep):
            start = len(records)
            kind_now[0], layer_start[0] = kind, start
            timed("modulated_layernorm", lambda: m.ddit_modulated_layernorm_fwd(x32, lw["ada_table"], c6, 0, L, 1e-6, xh),
                  nbytes=6.0 * N * D)
            timed("gemm_bf16", lambda: m.ddit_linear_fwd(m.DDIT_EPI_BF16, xh, D, lw["w_qkv"], lw["b_qkv"], N, 3 * A, D, qkv, 3 * A),
                  lin(3 * A, D))
            if kind == "spatial":
                timed("spatial_attention", lambda: m.ddit_attn_fwd(m.DDIT_ATTN_SPATIAL, self.shape, qkv[:, :A], qkv[:, A:2 * A],
                                                                   qkv[:, 2 * A:], 3 * A, 3 * A, None, o, A), fl["spatial"])
            else:
                timed("temporal_attention", lambda: m.ddit_attn_fwd(m.DDIT_ATTN_TEMPORAL, self.shape, qkv[:, :A], qkv[:, A:2 * A],
                                                                    qkv[:, 2 * A:], 3 * A, 3 * A, None, o, A), fl["temporal"],
                      8.0 * N * A)
            timed("gemm_residual", lambda: m.ddit_linear_fwd(m.DDIT_EPI_RESIDUAL_F32, o, A, lw["w_o"], lw["b_o"], N, D, A, xh, D,
                                                             resid=x32, ada_table=lw["ada_table"], c6=c6, gate_row=2,
                                                             tokens_per_sample=L), lin(D, A))
            timed("gemm_bf16", lambda: m.ddit_linear_fwd(m.DDIT_EPI_BF16, xh, D, lw["w_cq"], lw["b_cq"], N, A, D, qkv, 3 * A),
                  lin(A, D))
            timed("cross_attention", lambda: m.ddit_attn_fwd(m.DDIT_ATTN_CROSS, self.shape, qkv[:, :A], kvc[:, :A], kvc[:, A:],
                                                             3 * A, 2 * A, self.valid, o, A), fl["cross"])
            timed("gemm_residual", lambda: m.ddit_linear_fwd(m.DDIT_EPI_RESIDUAL_F32, o, A, lw["w_co"], lw["b_co"], N, D, A, None, 0,
                                                             resid=x32, tokens_per_sample=L), lin(D, A))
            timed("modulated_layernorm", lambda: m.ddit_modulated_layernorm_fwd(x32, lw["ada_table"], c6, 1, L, 1e-6, xh),
                  nbytes=6.0 * N * D)
            timed("gemm_gelu", lambda: m.ddit_linear_fwd(m.DDIT_EPI_GELU_BF16, xh, D, lw["w_fc1"], lw["b_fc1"], N, M, D, h, M),
                  lin(M, D))
            timed("gemm_residual", lambda: m.ddit_linear_fwd(m.DDIT_EPI_RESIDUAL_F32, h, M, lw["w_fc2"], lw["b_fc2"], N, D, M, None, 0,
                                                             resid=x32, ada_table=lw["ada_table"], c6=c6, gate_row=5,
                                                             tokens_per_sample=L), lin(D, M))
            if not keep:
                del records[start:]

        for r in range(reps + 1):
            wb = self.blocks[r % len(self.blocks)]
            for kind in ("spatial", "temporal"):
                layer(kind, wb[kind], keep=r > 0)   # the first pass warms up
            if r % 4 == 3:   # keep the stream's values bounded over many passes (outside every event pair)
                x32.normal_()
        torch.cuda.synchronize()
        # a launch that took more than three times the median of its own place in the layer is a hiccup of the machine
        # (seen once in dozens of runs: one launch of 68 ms among 15-us ones), not the kernel: it counts as the median
        by_place = {}
        for group, e0, e1, flops, nbytes, place in records:
            by_place.setdefault(place, []).append(e0.elapsed_time(e1))
        med = {place: sorted(v)[len(v) // 2] for place, v in by_place.items()}
        groups, self.hiccups = {}, 0
        for group, e0, e1, flops, nbytes, place in records:
            g = groups.setdefault(group, {"n": 0, "ms": 0.0, "flops": 0.0, "bytes": 0.0})
            g["n"] += 1
            ms_ = e0.elapsed_time(e1)
            if ms_ > 3.0 * med[place]:
                ms_, self.hiccups = med[place], self.hiccups + 1
            g["ms"] += ms_
            g["flops"] += flops
            g["bytes"] += nbytes
        per_block = {k: g["n"] / reps for k, g in groups.items()}
        total_ms = sum(g["ms"] for g in groups.values()) / reps * sh.n_blocks
        table = []
        for key, g in groups.items():
            avg_ms = g["ms"] / g["n"]
            name, bound = KERNEL_GROUPS[key]
            row = {"group": key, "kernel": name, "launches_per_step": int(round(per_block[key] * sh.n_blocks)),
                   "avg_ms": round(avg_ms, 4), "share_of_step": round(g["ms"] / reps * sh.n_blocks / total_ms, 4), "bound": bound}
            if bound == "mfma":
                tf = g["flops"] / (g["ms"] * 1e-3) / 1e12
                row.update({"achieved": round(tf, 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(tf / PEAK_BF16_TFLOPS, 4),
                            "algorithmic_gflop_per_launch": round(g["flops"] / g["n"] / 1e9, 2)})
            else:
                gbs = g["bytes"] / (g["ms"] * 1e-3) / 1e9
                row.update({"achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(gbs / PEAK_HBM_GBS, 4),
                            "algorithmic_mb_per_launch": round(g["bytes"] / g["n"] / 1e6, 2)})
            table.append(row)
        table.sort(key=lambda r: -r["share_of_step"])
        del x32, xh, qkv, o, kvc, h
        return table, total_ms

    def gemm_tiles(self):
        """The output tile the launcher's model takes for each linear of this workload (rows x cols)."""
        m, sh = self.m, self.sh
        out = {}
        for name, epi, n, k in (("qkv", m.DDIT_EPI_BF16, 3 * sh.A, sh.D), ("attn_out", m.DDIT_EPI_RESIDUAL_F32, sh.D, sh.A),
                                ("cross_q", m.DDIT_EPI_BF16, sh.A, sh.D), ("fc1", m.DDIT_EPI_GELU_BF16, sh.M, sh.D),
                                ("fc2", m.DDIT_EPI_RESIDUAL_F32, sh.D, sh.M)):
            tile, _ = m.ddit_linear_tile_choice(epi, sh.N, n, k)
            info = m.ddit_linear_tile_info(tile)
            out[name] = "%dx%d" % (info["rows"], info["cols"])
        return out


def roofline_of(table, workload, tiles):
    """The roofline object of the kernel group with the largest share of the step."""
    top = table[0]
    r = {"kernel": top["kernel"], "group": top["group"], "bound": top["bound"], "achieved": top["achieved"], "peak": top["peak"],
         "unit": top["unit"], "frac": top["frac"], "ms_per_launch": top["avg_ms"], "share_of_step": top["share_of_step"],
         "launches_per_step": top["launches_per_step"], "traffic": measured_traffic(top["group"], workload)}
    if top["group"].startswith("gemm"):
        r["tiles"] = tiles
    return r


def probes(m, torch, sh):
    """The denominators, measured on this machine: a register-resident MFMA loop (constant and random operand data), a
    streaming copy, and the memory traffic of an out-projection's residual epilogue without its matrix work."""
    out = {}
    ev = lambda: torch.cuda.Event(enable_timing=True)

    def timed(fn, reps=5):
        fn()
        e0, e1 = ev(), ev()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) / reps
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    sink = torch.empty(512 * cus, device="cuda")
    for label, data in (("ones", torch.ones(32768, device="cuda").to(torch.bfloat16)),
                        ("random", torch.randn(32768, device="cuda").to(torch.bfloat16))):
        flops = [0.0]

        def run():
            flops[0] = m.ddit_probe_mfma_bf16(data, sink, 20000)
        ms = timed(run, 3)
        out["mfma_bf16_loop_%s_tflops" % label] = round(flops[0] / (ms * 1e-3) / 1e12, 1)
    nbytes = 1 << 30
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda").random_(0, 255)
    dst = torch.empty_like(src)
    ms = timed(lambda: m.ddit_probe_stream_copy(src, dst, nbytes))
    out["stream_copy_GBps"] = round(2.0 * nbytes / (ms * 1e-3) / 1e9, 1)
    sink_r = torch.empty(4096 * cus, device="cuda")
    ms = timed(lambda: m.ddit_probe_stream_read(src, nbytes, sink_r))
    out["stream_read_GBps"] = round(nbytes / (ms * 1e-3) / 1e9, 1)
    del src, dst, sink_r
    N, D, A = sh.N, sh.D, sh.A
    x = torch.randn(N, D, device="cuda")
    xh = torch.empty(N, D, dtype=torch.bfloat16, device="cuda")
    o = torch.randn(N, A, device="cuda").to(torch.bfloat16)
    gate = torch.randn(D, device="cuda") * 0.01
    ms = timed(lambda: m.ddit_probe_residual_stream(x, xh, o, gate, N, D, A))
    traffic = N * (8.0 * D + 2.0 * D + 2.0 * A)
    out["residual_stream_floor"] = {"ms": round(ms, 4), "GBps": round(traffic / (ms * 1e-3) / 1e9, 1),
                                    "bytes": int(traffic),
                                    "what": "x fp32 [N,D] read and written, bf16 copy written, o bf16 [N,A] read: the traffic of an "
                                            "out-projection's residual epilogue and operand rows, no matrix work"}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=None, choices=sorted(WORKLOAD_NAMES),
                    help="time this workload only (default: C4 = 480p as the headline value, then C5 = 720p share)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-stages", action="store_true", help="skip the per-kernel timings")
    ap.add_argument("--only-stage", default=None,
                    help="time only this entry of 'stages' (for counter runs of one kernel), e.g. spatial_attention")
    ap.add_argument("--tile-sweep", action="store_true",
                    help="instead of the benchmark line: every compiled tile of the linear forced in turn, beside the launcher's pick")
    ap.add_argument("--dop-table", action="store_true",
                    help="instead of the benchmark line: per-rank step time by resolution and degree of parallelism")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (one rank's share of the step); --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import ddit_synth as syn
    import paper_2506_13497_amd as m   # raises if the HIP library is not built

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.tile_sweep:
        tile_sweep(m, torch, SWEEP_TOKENS)
        return
    if args.dop_table:
        rows = dop_table(m, syn, torch, max(args.steps // 3, 2))
        print(json.dumps({"metric": "DiT step time (ms) of one rank by resolution and degree of parallelism", "unit": "ms",
                          "n_gpus": 1, "dtype": "bf16", "data": "synthetic",
                          "assumed_xgmi_GBps_per_peer": XGMI_GBS_PER_PEER, "table": rows}), flush=True)
        return
    primary = args.workload or "C4"
    w = Workload(m, syn, torch, primary)
    sh, base, shape, blocks, valid, fl = w.sh, w.base, w.shape, w.blocks, w.valid, w.fl
    x_in, y = w.x_in, w.y

    if args.only_stage:
        args.warmup, args.no_cpu = 0, True
    n_steps = 0 if args.only_stage else args.steps
    ms_per_step = w.time_steps(n_steps, args.warmup) if n_steps else 1e-9
    step_tflops = fl["step"] / (ms_per_step * 1e-3) / 1e12
    print("[bench] %s step %.2f ms, %.1f TFLOP/s algorithmic" % (primary, ms_per_step, step_tflops), file=sys.stderr, flush=True)

    # the same step with per-head q/k normalisation and temporal rotary embedding switched on (the two
    # options of the released model that the paper does not mention): reported beside the metric, not as it
    variant_ms = None
    if not args.only_stage and not args.no_stages:
        shape_v = m.make_shape(sh.B, sh.T, sh.Hp, sh.Wp, sh.D, sh.H, sh.dh, sh.M, sh.Ly, sh.n_blocks,
                               m.DDIT_FLAG_QK_NORM | m.DDIT_FLAG_ROPE_TEMPORAL)
        ws_v = m.alloc_workspace(shape_v)
        x_v = torch.empty_like(x_in)
        step_v = lambda: m.ddit_denoise_step(shape_v, w.st, x_in, y, valid, w.tsteps, None, x_v, ws_v)
        step_v()
        torch.cuda.synchronize()
        tv = time.perf_counter()
        for _ in range(3):
            step_v()
        torch.cuda.synchronize()
        variant_ms = (time.perf_counter() - tv) * 1e3 / 3
        del ws_v, x_v
        print("[bench] step with q/k normalisation + rotary embedding: %.2f ms" % variant_ms, file=sys.stderr, flush=True)

    # ---- per-kernel timings with HIP events on the stream the kernels run on
    def time_call(fn, reps):
        fn(); fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) / reps   # ms

    kernels, roofline, denominators = None, None, None
    reps = max(args.steps, 5)
    if not args.no_stages and not args.only_stage:
        kernels, table_ms = w.kernel_table(reps)
        roofline = roofline_of(kernels, primary, w.gemm_tiles())
        roofline["sum_of_kernels_ms"] = round(table_ms, 2)
        roofline["launches_taken_as_median"] = w.hiccups
        print("[bench] %s kernels (sum %.1f ms): %s" % (primary, table_ms, json.dumps(kernels)), file=sys.stderr, flush=True)
        denominators = probes(m, torch, sh)
        print("[bench] denominators: %s" % json.dumps(denominators), file=sys.stderr, flush=True)

    def attention_stages(wk, want):
        """The attention kernels back to back on cache-warm operands (the kernel table has them in the step's context)."""
        s_, shp = wk.sh, wk.shape
        N, A = s_.N, s_.A
        out = {}
        qkv = torch.randn(N, 3 * A, device="cuda").to(torch.bfloat16)
        o = torch.empty(N, A, dtype=torch.bfloat16, device="cuda")
        for name, kind, flops in (("spatial_attention", m.DDIT_ATTN_SPATIAL, wk.fl["spatial"]),
                                  ("temporal_attention", m.DDIT_ATTN_TEMPORAL, wk.fl["temporal"])):
            if not want(name):
                continue
            ms = time_call(lambda: m.ddit_attn_fwd(kind, shp, qkv[:, :A], qkv[:, A:2 * A], qkv[:, 2 * A:], 3 * A, 3 * A,
                                                   None, o, A), reps)
            tf = flops / (ms * 1e-3) / 1e12
            gbs = 8.0 * N * A / (ms * 1e-3) / 1e9     # q,k,v read + o written once, bf16
            out[name] = {"ms": round(ms, 4), "tflops": round(tf, 1), "frac_mfma": round(tf / PEAK_BF16_TFLOPS, 4),
                         "GBps": round(gbs, 1), "frac_hbm": round(gbs / PEAK_HBM_GBS, 4)}
        kvc = torch.randn(s_.B * s_.Ly, 2 * A, device="cuda").to(torch.bfloat16)
        if want("cross_attention"):
            ms = time_call(lambda: m.ddit_attn_fwd(m.DDIT_ATTN_CROSS, shp, qkv[:, :A], kvc[:, :A], kvc[:, A:], 3 * A,
                                                   2 * A, wk.valid, o, A), reps)
            tf = wk.fl["cross"] / (ms * 1e-3) / 1e12
            out["cross_attention"] = {"ms": round(ms, 4), "tflops": round(tf, 1),
                                      "frac_mfma": round(tf / PEAK_BF16_TFLOPS, 4), "valid_len": wk.valid}
        del qkv, o, kvc
        return out

    stages = {}
    want = lambda name: not args.only_stage or args.only_stage == name
    if not args.no_stages:
        N, D, A, M = sh.N, sh.D, sh.A, sh.M
        lw = blocks[0]["spatial"]
        stages.update(attention_stages(w, want))
        xh = torch.randn(N, D, device="cuda").to(torch.bfloat16)
        x32 = torch.randn(N, D, device="cuda")
        c6 = torch.randn(sh.B, 6 * D, device="cuda")
        if want("modulated_layernorm"):
            ms = time_call(lambda: m.ddit_modulated_layernorm_fwd(x32, lw["ada_table"], c6, 0, sh.L, 1e-6, xh), reps)
            gbs = 6.0 * N * D / (ms * 1e-3) / 1e9
            stages["modulated_layernorm"] = {"ms": round(ms, 4), "GBps": round(gbs, 1), "frac_hbm": round(gbs / PEAK_HBM_GBS, 4)}
        for name, epi, n_, k_, gate in (("fc1_gelu", m.DDIT_EPI_GELU_BF16, M, D, -1), ("attn_out_residual", m.DDIT_EPI_RESIDUAL_F32, D, A, 2),
                                        ("fc2_residual", m.DDIT_EPI_RESIDUAL_F32, D, M, 5)):
            if args.only_stage != name:      # counter runs of one GEMM launch shape; the kernel table times them in context
                continue
            u_ = torch.randn(N, k_, device="cuda").to(torch.bfloat16)
            w_ = (torch.randn(n_, k_, device="cuda") * 0.02).to(torch.bfloat16)
            out_ = torch.empty(N, n_, dtype=torch.bfloat16, device="cuda")
            if epi == m.DDIT_EPI_RESIDUAL_F32:
                fn = lambda: m.ddit_linear_fwd(epi, u_, k_, w_, None, N, n_, k_, out_, n_, resid=x32, ada_table=lw["ada_table"], c6=c6,
                                               gate_row=gate, tokens_per_sample=sh.L)
            else:
                fn = lambda: m.ddit_linear_fwd(epi, u_, k_, w_, None, N, n_, k_, out_, n_)
            ms = time_call(fn, reps)
            tf = 2.0 * N * n_ * k_ / (ms * 1e-3) / 1e12
            stages[name] = {"ms": round(ms, 4), "tflops": round(tf, 1), "frac_mfma": round(tf / PEAK_BF16_TFLOPS, 4)}
        if want("qk_norm_rope"):
            qk_buf = torch.randn(N, 3 * A, device="cuda").to(torch.bfloat16)
            tab = torch.empty(sh.T * sh.dh, dtype=torch.float32, device="cuda")
            ms = time_call(lambda: m.ddit_qk_norm_rope_fwd(qk_buf, 3 * A, N, sh.H, sh.dh, lw["g_q"], lw["g_k"], 1e-6, sh.S,
                                                           sh.T, tab), reps)
            gbs = 8.0 * N * A / (ms * 1e-3) / 1e9        # q and k read and written once, bf16
            stages["qk_norm_rope"] = {"ms": round(ms, 4), "GBps": round(gbs, 1), "frac_hbm": round(gbs / PEAK_HBM_GBS, 4)}
            del qk_buf
        # the layers around the step and the solver (latent with 4 channels, text width 4096)
        C_lat, C_text = 4, 4096
        io_w = {k: w.draw(s_, 0.02, torch.float32 if k == "final_table" else torch.bfloat16)
                for k, s_ in syn.io_shapes(sh, C_lat, C_text, C_lat).items()}
        io = m.io_struct(io_w, C_lat, C_lat, C_text)
        ws_io = torch.empty(m.ddit_io_workspace_bytes(shape, io), dtype=torch.uint8, device="cuda")
        z = torch.randn(sh.B, C_lat, sh.T, 2 * sh.Hp, 2 * sh.Wp, device="cuda")
        eps = torch.empty_like(z)
        temb = torch.randn(sh.B, D, device="cuda")
        c_text = torch.randn(sh.B, sh.Ly, C_text, device="cuda").to(torch.bfloat16)
        y_e = torch.empty(sh.B, sh.Ly, D, dtype=torch.bfloat16, device="cuda")
        io_bytes = 2.0 * N * D + 4.0 * z.numel()
        for name, fn, nbytes in (
                ("embed_latent", lambda: m.ddit_embed_latent(shape, io, z, xh, ws_io), io_bytes),
                ("output_head", lambda: m.ddit_output_head(shape, io, xh, temb, eps), io_bytes),
                ("embed_caption", lambda: m.ddit_embed_caption(shape, io, c_text, y_e, ws_io), None),
                ("solver_step", lambda: m.ddit_solver_step(z, eps, eps, 1.0, [500.0] * sh.B, [500.0] * sh.B,
                                                           z.numel() // sh.B), None)):
            if not want(name):
                continue
            ms = time_call(fn, reps)
            stages[name] = {"ms": round(ms, 4)}
            if nbytes:
                gbs = nbytes / (ms * 1e-3) / 1e9
                stages[name].update({"GBps": round(gbs, 1), "frac_hbm": round(gbs / PEAK_HBM_GBS, 4)})
        del xh, x32, ws_io
        print("[bench] stages: %s" % json.dumps(stages), file=sys.stderr, flush=True)

    # ---- CPU oracle on a bounded sample of the same workload
    cpu = None
    if not args.no_cpu:
        from oracle import stdit_oracle as ora
        f64 = lambda a: syn.bits_to_f64(a) if a.dtype == np.uint16 else a.astype(np.float64)
        # a third of the frames through a spatial layer and a third of the locations through a temporal
        # layer (same token count): every stage is linear in frames resp. locations, so each scales to its layer
        Ts = max(1, sh.T // 3)
        Ss = max(1, sh.S // 3)
        wl_s = {k: v.double().cpu().numpy() for k, v in blocks[0]["spatial"].items()}
        wl_t = {k: v.double().cpu().numpy() for k, v in blocks[0]["temporal"].items()}
        xs_s = x_in[:, :Ts].contiguous().double().cpu().numpy()
        xs_t = x_in[:, :, :Ss].contiguous().double().cpu().numpy()
        ys = y.double().cpu().numpy()
        c6s = f64(syn.make_c6(sh, base, 0.5))
        tc = time.perf_counter()
        ora.layer_fwd("spatial", xs_s, ys, np.array(valid), c6s, wl_s, sh.H, sh.dh)
        dt_s = time.perf_counter() - tc
        tc = time.perf_counter()
        ora.layer_fwd("temporal", xs_t, ys, np.array(valid), c6s, wl_t, sh.H, sh.dh)
        dt_t = time.perf_counter() - tc
        est_ms = (dt_s * sh.T / Ts + dt_t * sh.S / Ss) * sh.n_blocks * 1e3
        try:
            from threadpoolctl import threadpool_info
            nthr = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            nthr = os.cpu_count()
        cpu = {"value": round(est_ms, 1), "unit": "ms", "cores": int(nthr), "kind": "oracle",
               "sample": "fp64 numpy oracle: one spatial layer on %d of %d frames (%.1f s) and one temporal layer on %d of "
                         "%d locations (%.1f s), %d tokens each; scaled to whole layers x%d blocks = a full step"
                         % (Ts, sh.T, dt_s, Ss, sh.S, dt_t, sh.B * Ts * sh.S, sh.n_blocks)}
        del wl_s, wl_t, xs_s, xs_t

    # ---- the other half of the metric: the 720p share, same measurements, same line
    workloads = {primary: {"workload": w.describe(), "ms_per_step": round(ms_per_step, 3), "step_tflops": round(step_tflops, 1),
                           "step_frac_mfma_peak": round(step_tflops / PEAK_BF16_TFLOPS, 4),
                           "step_algorithmic_tflop": round(fl["step"] / 1e12, 2), "kernels": kernels,
                           "attention_stages": {k: v for k, v in stages.items() if k.endswith("attention")}}}
    second = None
    if args.workload is None and not args.only_stage:
        del w.ws, w.x_out
        w.blocks = w.st = None
        blocks = None
        torch.cuda.empty_cache()
        w5 = Workload(m, syn, torch, "C5")
        ms5 = w5.time_steps(args.steps, args.warmup)
        tf5 = w5.fl["step"] / (ms5 * 1e-3) / 1e12
        print("[bench] C5 step %.2f ms, %.1f TFLOP/s algorithmic" % (ms5, tf5), file=sys.stderr, flush=True)
        second = {"workload": w5.describe(), "ms_per_step": round(ms5, 3), "step_tflops": round(tf5, 1),
                  "step_frac_mfma_peak": round(tf5 / PEAK_BF16_TFLOPS, 4), "step_algorithmic_tflop": round(w5.fl["step"] / 1e12, 2)}
        if not args.no_stages:
            k5, t5 = w5.kernel_table(max(reps // 2, 3))
            second["kernels"] = k5
            second["roofline"] = roofline_of(k5, "C5", w5.gemm_tiles())
            second["roofline"]["sum_of_kernels_ms"] = round(t5, 2)
            second["roofline"]["launches_taken_as_median"] = w5.hiccups
            second["attention_stages"] = attention_stages(w5, lambda name: True)
            print("[bench] C5 kernels (sum %.1f ms): %s" % (t5, json.dumps(k5)), file=sys.stderr, flush=True)
            print("[bench] C5 attention: %s" % json.dumps(second["attention_stages"]), file=sys.stderr, flush=True)
        workloads["C5"] = second

    out = {
        "metric": "DiT denoise-step latency (ms) at %s-shaped latents%s; attention TFLOP/s in 'stages' and 'workloads'" %
                  (WORKLOAD_NAMES[primary].split("-")[0], " (value) and at the 720p share (c5_step_ms)" if second else ""),
        "value": round(ms_per_step, 3), "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.describe()},
        "step_tflops": round(step_tflops, 1), "step_frac_mfma_peak": round(step_tflops / PEAK_BF16_TFLOPS, 4),
        "step_algorithmic_tflop": round(fl["step"] / 1e12, 2),
        "roofline": roofline, "kernels": kernels, "stages": stages, "cpu_baseline": cpu,
        "c5_step_ms": None if not second else second["ms_per_step"],
        "c5_step_frac_mfma_peak": None if not second else second["step_frac_mfma_peak"],
        "workloads": workloads, "measured_denominators": denominators,
        "step_ms_with_qk_norm_and_rotary": None if variant_ms is None else round(variant_ms, 3),
        "paper_context": "paper reports only 'several seconds to tens of seconds' of DiT time per 30-step request on "
                         "H800 at 144p-360p (section 6.3); no per-step figure to compare with",
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
