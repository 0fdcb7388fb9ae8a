#!/usr/bin/env python3
"""Benchmark of the STDiT denoising step on one MI355X.

A step = one full pass of the hot path (timestep conditioning + 28 blocks = 56 layers) over
one synthetic 480p-shaped batch (B=1, T=30, 30x54 tokens per frame, L=48600, hidden 1152,
16 heads x 72, MLP 4608, 300 text tokens with a seeded padding mask).  Inputs and weights
are resident in HBM before the timed region.  Prints ONE JSON line.

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


def measured_traffic(workload):
    """HBM bytes per launch of the fc1 GEMM as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (two
    runs, scaled by what the same counters read for the step's own streaming cast kernels of known
    size); the figure is kept, with the commands that produced it, in profiles/.  None if not measured
    for this workload."""
    path = os.path.join(ROOT, "profiles", "gemm_fc1_gelu_%s_hbm_traffic.txt" % WORKLOAD_NAMES[workload])
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C4", choices=sorted(WORKLOAD_NAMES))
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-stages", action="store_true", help="skip the per-kernel timings")
    ap.add_argument("--only-stage", default=None,
                    help="time only this entry of 'stages' (for counter runs of one kernel), e.g. spatial_attention")
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
    if args.dop_table:
        rows = dop_table(m, syn, torch, max(args.steps // 3, 2))
        print(json.dumps({"metric": "DiT step time (ms) of one rank by resolution and degree of parallelism", "unit": "ms",
                          "n_gpus": 1, "dtype": "bf16", "data": "synthetic",
                          "assumed_xgmi_GBps_per_peer": XGMI_GBS_PER_PEER, "table": rows}), flush=True)
        return
    cfg = syn.CONFIGS[args.workload]
    sh, base = cfg["shape"], cfg["base"]

    t0 = time.time()
    # Weights are drawn on the device (seeded torch generator, same N(0, 0.02^2) distribution and
    # shapes as ddit_synth, which the parity tests use): 1.2 G numpy draws would take minutes.
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1000 + base)

    def draw(shape_, std, dtype=torch.bfloat16):
        t = torch.randn(shape_, generator=gen, device="cuda", dtype=torch.float32) * std
        return t.to(torch.bfloat16).to(dtype)   # fp32 tensors hold bf16-representable values

    sw = {k: draw(s_, 0.02) for k, s_ in syn.step_shapes(sh).items()}
    blocks = []
    for i in range(sh.n_blocks):
        blocks.append({kind: {n: draw(s_, 0.02, torch.float32 if n == "ada_table" else torch.bfloat16)
                              for n, s_ in syn.layer_shapes(sh).items()} for kind in ("spatial", "temporal")})
    for wb in blocks:   # scales of the optional q/k normalisation (read only by the variant timed after the step)
        for lw_ in wb.values():
            lw_["g_q"] = (1.0 + draw((sh.dh,), 0.2, torch.float32)).to(torch.bfloat16)
            lw_["g_k"] = (1.0 + draw((sh.dh,), 0.2, torch.float32)).to(torch.bfloat16)
    x_in, y = draw((sh.B, sh.T, sh.S, sh.D), 1.0), draw((sh.B, sh.Ly, sh.D), 1.0)
    valid = [int(v) for v in syn.make_valid_len(sh, base, cfg["valid"])]
    tsteps = [float(t) for t in syn.make_timesteps(sh, base, cfg["t"])]
    shape = m.make_shape(sh.B, sh.T, sh.Hp, sh.Wp, sh.D, sh.H, sh.dh, sh.M, sh.Ly, sh.n_blocks)
    ws = m.alloc_workspace(shape)
    st = m.step_struct(sw, blocks)
    x_out = torch.empty_like(x_in)
    torch.cuda.synchronize()
    print("[bench] %s: inputs+weights resident after %.1fs (workspace %.2f GB)" %
          (args.workload, time.time() - t0, ws.numel() / 1e9), file=sys.stderr, flush=True)

    def one_step():
        m.ddit_denoise_step(shape, st, x_in, y, valid, tsteps, None, x_out, ws)

    if args.only_stage:
        args.warmup, args.no_cpu = 0, True
    n_steps = 0 if args.only_stage else args.steps
    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(n_steps):
        one_step()
    torch.cuda.synchronize()
    ms_per_step = max((time.perf_counter() - t1) * 1e3 / max(n_steps, 1), 1e-9)
    fl = step_flops(sh, valid)
    step_tflops = fl["step"] / (ms_per_step * 1e-3) / 1e12
    print("[bench] step %.2f ms, %.1f TFLOP/s algorithmic" % (ms_per_step, step_tflops), file=sys.stderr, flush=True)

    # the same step with per-head q/k normalisation and temporal rotary embedding switched on (the two
    # options of the released model that the paper does not mention): reported beside the metric, not as it
    variant_ms = None
    if not args.only_stage and not args.no_stages:
        shape_v = m.make_shape(sh.B, sh.T, sh.Hp, sh.Wp, sh.D, sh.H, sh.dh, sh.M, sh.Ly, sh.n_blocks,
                               m.DDIT_FLAG_QK_NORM | m.DDIT_FLAG_ROPE_TEMPORAL)
        ws_v = m.alloc_workspace(shape_v)
        x_v = torch.empty_like(x_in)
        step_v = lambda: m.ddit_denoise_step(shape_v, st, x_in, y, valid, tsteps, None, x_v, ws_v)
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

    stages, roofline = {}, None
    want = lambda name: not args.only_stage or args.only_stage == name
    if not args.no_stages:
        N, D, A, M = sh.N, sh.D, sh.A, sh.M
        lw = blocks[0]["spatial"]
        xh = torch.randn(N, D, device="cuda").to(torch.bfloat16)
        h = torch.empty(N, M, dtype=torch.bfloat16, device="cuda")
        reps = max(args.steps, 5)
        # The roofline kernel is timed where it runs in the step: between the LayerNorm that produces its input
        # and the fc2 GEMM that consumes its output (their traffic leaves the caches in the state the step
        # leaves them in), with one event pair per launch on the stream the kernels run on.
        def fc1_in_context(reps_):
            x32_ = torch.randn(N, D, device="cuda")
            c6_ = torch.randn(sh.B, 6 * D, device="cuda")
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps_ + 2)]
            for e0, e1 in ev:
                m.ddit_modulated_layernorm_fwd(x32_, lw["ada_table"], c6_, 1, sh.L, 1e-6, xh)
                e0.record()
                m.ddit_linear_fwd(m.DDIT_EPI_GELU_BF16, xh, D, lw["w_fc1"], lw["b_fc1"], N, M, D, h, M)
                e1.record()
                m.ddit_linear_fwd(m.DDIT_EPI_RESIDUAL_F32, h, M, lw["w_fc2"], lw["b_fc2"], N, D, M, None, 0, resid=x32_,
                                  ada_table=lw["ada_table"], c6=c6_, gate_row=5, tokens_per_sample=sh.L)
            torch.cuda.synchronize()
            t = [e0.elapsed_time(e1) for e0, e1 in ev[2:]]
            return sum(t) / len(t)
        ms = fc1_in_context(reps) if want("fc1_gelu") else float("nan")
        tf = fl["fc1"] / (ms * 1e-3) / 1e12
        roofline = {"kernel": "k_gemm_bf16<2,4,3,3,4,1> = 192x384 tiles, GELU epilogue (MLP fc1, %dx%dx%d)" % (N, M, D),
                    "bound": "mfma", "achieved": round(tf, 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(tf / PEAK_BF16_TFLOPS, 4), "ms_per_launch": round(ms, 4),
                    "traffic": measured_traffic(args.workload)}
        if want("fc1_gelu"):
            stages["fc1_gelu"] = {"ms": round(ms, 4), "tflops": round(tf, 1), "frac_mfma": round(tf / PEAK_BF16_TFLOPS, 4)}
        else:
            roofline = None
        qkv = torch.randn(N, 3 * A, device="cuda").to(torch.bfloat16)
        o = torch.empty(N, A, dtype=torch.bfloat16, device="cuda")
        for name, kind, flops in (("spatial_attention", m.DDIT_ATTN_SPATIAL, fl["spatial"]),
                                  ("temporal_attention", m.DDIT_ATTN_TEMPORAL, fl["temporal"])):
            if not want(name):
                continue
            ms = time_call(lambda: m.ddit_attn_fwd(kind, shape, qkv[:, :A], qkv[:, A:2 * A], qkv[:, 2 * A:], 3 * A, 3 * A,
                                                   None, o, A), reps)
            tf = flops / (ms * 1e-3) / 1e12
            gbs = 8.0 * N * A / (ms * 1e-3) / 1e9     # q,k,v read + o written once, bf16
            stages[name] = {"ms": round(ms, 4), "tflops": round(tf, 1), "frac_mfma": round(tf / PEAK_BF16_TFLOPS, 4),
                            "GBps": round(gbs, 1), "frac_hbm": round(gbs / PEAK_HBM_GBS, 4)}
        kvc = torch.randn(sh.B * sh.Ly, 2 * A, device="cuda").to(torch.bfloat16)
        if want("cross_attention"):
            ms = time_call(lambda: m.ddit_attn_fwd(m.DDIT_ATTN_CROSS, shape, qkv[:, :A], kvc[:, :A], kvc[:, A:], 3 * A,
                                                   2 * A, valid, o, A), reps)
            tf = fl["cross"] / (ms * 1e-3) / 1e12
            stages["cross_attention"] = {"ms": round(ms, 4), "tflops": round(tf, 1),
                                         "frac_mfma": round(tf / PEAK_BF16_TFLOPS, 4), "valid_len": valid}
        x32 = torch.randn(N, D, device="cuda")
        c6 = torch.randn(sh.B, 6 * D, device="cuda")
        if want("modulated_layernorm"):
            ms = time_call(lambda: m.ddit_modulated_layernorm_fwd(x32, lw["ada_table"], c6, 0, sh.L, 1e-6, xh), reps)
            gbs = 6.0 * N * D / (ms * 1e-3) / 1e9
            stages["modulated_layernorm"] = {"ms": round(ms, 4), "GBps": round(gbs, 1), "frac_hbm": round(gbs / PEAK_HBM_GBS, 4)}
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
        io_w = {k: draw(s_, 0.02, torch.float32 if k == "final_table" else torch.bfloat16)
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
        del xh, h, qkv, o, kvc, x32, ws_io
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

    out = {
        "metric": "DiT denoise-step latency (ms) at %s-shaped latents; attention TFLOP/s in 'stages'" %
                  WORKLOAD_NAMES[args.workload].split("-")[0],
        "value": round(ms_per_step, 3), "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s (%s): B=%d T=%d S=%d L=%d D=%d heads=%dx%d M=%d Ly=%d valid=%s blocks=%d" %
                   (args.workload, WORKLOAD_NAMES[args.workload], sh.B, sh.T, sh.S, sh.L, sh.D, sh.H, sh.dh, sh.M, sh.Ly,
                    valid, sh.n_blocks)},
        "step_tflops": round(step_tflops, 1), "step_frac_mfma_peak": round(step_tflops / PEAK_BF16_TFLOPS, 4),
        "step_algorithmic_tflop": round(fl["step"] / 1e12, 2),
        "roofline": roofline, "stages": stages, "cpu_baseline": cpu,
        "step_ms_with_qk_norm_and_rotary": None if variant_ms is None else round(variant_ms, 3),
        "paper_context": "paper reports only 'several seconds to tens of seconds' of DiT time per 30-step request on "
                         "H800 at 144p-360p (section 6.3); no per-step figure to compare with",
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
