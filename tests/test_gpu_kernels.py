"""Kernel-level parity on the GPU: each stage of the path, called through the C ABI,
against the matching function of the CPU oracle on the same seeded inputs.

Bar (written out in helpers.assert_parity): per element |gpu-ora| <= 2e-2 (1+|ora|) and
relative Frobenius error <= 5e-3.  For the attention outputs |O| is small, so the
Frobenius bound is the binding one."""
import math

import numpy as np
import pytest
import torch

import ddit_synth as syn
from helpers import assert_parity, dev_to_f64, rel_fro, to_dev, to_f64
from oracle import stdit_oracle as ora

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lib():
    import paper_2506_13497_amd as m
    assert torch.cuda.is_available()
    return m


def _shape(lib, sh, flags=0):
    return lib.make_shape(sh.B, sh.T, sh.Hp, sh.Wp, sh.D, sh.H, sh.dh, sh.M, sh.Ly, sh.n_blocks, flags)


# ----------------------------------------------------------------------------- adaLN + LN
@pytest.mark.parametrize("N,tps,D", [(256, 256, 256), (37, 19, 1152), (2 * 405, 405, 1152), (9, 9, 4096), (5, 5, 8)])
def test_modulated_layernorm(lib, N, tps, D):
    B = (N + tps - 1) // tps
    rng = np.random.default_rng(N + D)
    x = (rng.standard_normal((N, D)) * 1.5 + 0.3).astype(np.float32)
    tab = rng.standard_normal((6, D)).astype(np.float32) * 0.5
    c6 = rng.standard_normal((B, 6 * D)).astype(np.float32) * 0.5
    out = torch.empty(N, D, dtype=torch.bfloat16, device="cuda")
    for which in (0, 1):
        lib.ddit_modulated_layernorm_fwd(to_dev(x), to_dev(tab), to_dev(c6), which, tps, 1e-6, out)
        torch.cuda.synchronize()
        xn = ora.layer_norm(x.astype(np.float64))
        ref = np.empty((N, D))
        for n in range(N):
            m = ora.split_modulation(tab.astype(np.float64), c6[n // tps].astype(np.float64), D)
            sfx = "msa" if which == 0 else "mlp"
            ref[n] = ora.modulate(xn[n], m["shift_" + sfx], m["scale_" + sfx])
        assert_parity(dev_to_f64(out), ref, "modulated LN which=%d" % which)


# ----------------------------------------------------------------------------- q/k normalisation, rotary embedding
@pytest.mark.parametrize("N,H,dh,S,T,extra", [(37, 16, 72, 5, 3, 0), (1000, 4, 72, 7, 30, 16), (130, 2, 64, 1, 130, 8),
                                              (3 * 40 * 11, 16, 72, 11, 40, 0), (1, 1, 64, 1, 1, 0)])
@pytest.mark.parametrize("norm,rope", [(True, False), (False, True), (True, True)], ids=["norm", "rope", "norm+rope"])
def test_qk_norm_rope(lib, N, H, dh, S, T, extra, norm, rope):
    """In place on the q | k columns of a fused q|k|v buffer; v and any padding columns stay bit for bit."""
    A = H * dh
    ld = 3 * A + extra
    buf = syn.normal_bits((31, N, H, dh), (N, ld), 1.5)
    gq = syn.f32_to_bf16_bits((1 + 0.2 * np.random.default_rng(1).standard_normal(dh)).astype(np.float32))
    gk = syn.f32_to_bf16_bits((1 + 0.2 * np.random.default_rng(2).standard_normal(dh)).astype(np.float32))
    d = to_dev(buf)
    tab = torch.empty(T * dh, dtype=torch.float32, device="cuda") if rope else None
    lib.ddit_qk_norm_rope_fwd(d, ld, N, H, dh, to_dev(gq) if norm else None, to_dev(gk) if norm else None, 1e-6, S, T, tab)
    torch.cuda.synchronize()
    got = dev_to_f64(d)
    x = to_f64(buf)
    frame = ((np.arange(N) // S) % T).astype(np.float64)[:, None]
    for i, g in enumerate((gq, gk)):
        u = x[:, i * A:(i + 1) * A].reshape(N, H, dh)
        if norm:
            u = ora.rms_norm(u, to_f64(g), 1e-6)
        if rope:
            u = ora.rotary(u, frame)
        assert_parity(got[:, i * A:(i + 1) * A], u.reshape(N, A), "q/k part %d" % i)
    assert np.array_equal(got[:, 2 * A:], x[:, 2 * A:]), "v or padding columns were touched"
    if rope:   # the table the call leaves behind: (cos, sin) of t * 10000^(-2i/dh)
        tt = dev_to_f64(tab).reshape(T, dh // 2, 2)
        ang = np.arange(T)[:, None] * 10000.0 ** (-2.0 * np.arange(dh // 2) / dh)
        assert np.abs(tt[..., 0] - np.cos(ang)).max() < 2e-5 and np.abs(tt[..., 1] - np.sin(ang)).max() < 2e-5


def test_qk_norm_rope_480p_shape_sampled_rows(lib):
    """The benchmark's shape (48600 tokens, 16 x 72, 30 frames of 1620): sampled token rows against the oracle."""
    N, H, dh, S, T = 48600, 16, 72, 1620, 30
    A = H * dh
    g = torch.Generator(device="cuda"); g.manual_seed(5)
    d = (torch.randn(N, 3 * A, generator=g, device="cuda") * 1.5).to(torch.bfloat16)
    before = d.clone()
    gq = syn.f32_to_bf16_bits((1 + 0.2 * np.random.default_rng(3).standard_normal(dh)).astype(np.float32))
    gk = syn.f32_to_bf16_bits((1 + 0.2 * np.random.default_rng(4).standard_normal(dh)).astype(np.float32))
    tab = torch.empty(T * dh, dtype=torch.float32, device="cuda")
    lib.ddit_qk_norm_rope_fwd(d, 3 * A, N, H, dh, to_dev(gq), to_dev(gk), 1e-6, S, T, tab)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([[0, 1, S - 1, S, N - S - 1, N - 1], np.random.default_rng(6).integers(0, N, 500)]))
    ridx = torch.from_numpy(rows).cuda()
    got, x = dev_to_f64(d[ridx]), dev_to_f64(before[ridx])
    frame = ((rows // S) % T).astype(np.float64)[:, None]
    for i, gg in enumerate((gq, gk)):
        u = ora.rotary(ora.rms_norm(x[:, i * A:(i + 1) * A].reshape(-1, H, dh), to_f64(gg), 1e-6), frame)
        assert_parity(got[:, i * A:(i + 1) * A], u.reshape(-1, A), "q/k part %d, sampled rows" % i)
    assert torch.equal(d[:, 2 * A:], before[:, 2 * A:])


def test_qk_norm_rope_empty_and_identity(lib):
    buf = syn.normal_bits((32,), (64, 3 * 144), 1.0)
    d = to_dev(buf)
    lib.ddit_qk_norm_rope_fwd(d, 3 * 144, 0, 2, 72, None, None, 1e-6, 4, 4, None)      # no rows
    lib.ddit_qk_norm_rope_fwd(d, 3 * 144, 64, 2, 72, None, None, 1e-6, 4, 4, None)     # neither option: nothing to do
    # T = 1: every token is in frame 0, the rotation is the identity
    tab = torch.empty(72, dtype=torch.float32, device="cuda")
    lib.ddit_qk_norm_rope_fwd(d, 3 * 144, 64, 2, 72, None, None, 1e-6, 64, 1, tab)
    torch.cuda.synchronize()
    assert torch.equal(d, to_dev(buf))


# ----------------------------------------------------------------------------- linear + epilogues
LIN_CASES = [
    # N, n, k
    (256, 768, 256),      # C1 qkv
    (300, 2304, 1152),    # text k|v projection
    (1000, 1152, 288),    # k not a multiple of 64 (narrow attention width), ragged N
    (777, 4608, 1152),    # fc1 shape, ragged token tail, several tiles
    (515, 1152, 4608),    # fc2 shape
    (130, 864, 1152),     # n not a multiple of the tile
    (130, 864, 1160),     # k tail (k % 32 == 8) on the small tile
    (1, 8, 8),            # a single partial k-step
    (40, 64, 72),         # two full k-steps and a tail: fewer steps than the pipeline is deep
    # the 192 x 288 tile (six wavefronts; out-features a multiple of 288 but not of 384) needs >= 200 tiles:
    (13001, 864, 1160),   # q|k|v width of a 4-head share, ragged token tail, k tail
    (40000, 288, 1152),   # one tile wide
    # the large tile (192 x 384, eight wavefronts) needs >= 200 tiles:
    (12900, 1152, 288),   # narrow attention width as k, ragged token tail, tiles over two samples
    (5000, 4608, 1160),   # k tail on the large tile
    (5600, 2440, 512),    # n not a multiple of 384: ragged last out-feature tile
    # per-rank shapes of the step-time table, where the launcher picks the mid-size forms:
    (7360, 3456, 1152),   # 360p at parallel size 2, q|k|v: 192 x 192, two workgroups per CU, several rounds
    (24300, 1152, 1152),  # 480p at parallel size 2, out-projection: the same form with the residual epilogue
    (3680, 1152, 4608),   # 360p at parallel size 4, fc2: 128 x 192 with the CU to itself, long k
]


@pytest.mark.parametrize("N,n,k", LIN_CASES)
@pytest.mark.parametrize("epi", [0, 1, 2])
def test_linear(lib, N, n, k, epi):
    _check_linear(lib, N, n, k, epi, -1)


N_TILES = 9   # forms of the kernel compiled into the library (parametrisation needs it before the library loads)
TILE_CASES = [
    (403, 872, 1160),     # ragged in rows and columns for every tile shape, k tail
    (1, 8, 8),            # one partial tile, one partial k-step
    (700, 1152, 288),     # narrow k, several row tiles
    (26000, 864, 296),    # more tiles than resident workgroups for every form (680 of 192 x 192 on 512 slots, 2856 of
                          # 64 x 128 on 768): the persistent loop's later rounds, fetching the next tile under the epilogue
]


def test_tile_list_matches(lib):
    assert lib.ddit_linear_tile_count() == N_TILES


@pytest.mark.parametrize("N,n,k", TILE_CASES)
@pytest.mark.parametrize("epi", [0, 1, 2])
@pytest.mark.parametrize("tile", range(N_TILES))
def test_linear_every_tile(lib, tile, epi, N, n, k):
    """Every compiled output tile computes the same function on shapes its grid does not divide."""
    _check_linear(lib, N, n, k, epi, tile)


@pytest.mark.parametrize("tile", range(N_TILES))
@pytest.mark.parametrize("N,tps", [(50, 7), (7, 7), (1, 1), (200, 3)])
def test_linear_residual_tile_over_many_samples(lib, tile, N, tps):
    """Samples much shorter than a tile: every row looks up its own sample's gate; the rows of the tile
    past the end of the problem must not name a sample that does not exist."""
    n, k = 264, 96
    B = (N + tps - 1) // tps
    u = syn.normal_bits((41, N, tps), (N, k), 1.0)
    W = syn.normal_bits((42, N, tps), (n, k), 1.0 / math.sqrt(k))
    b = syn.normal_bits((43, N, tps), (n,), 0.5)
    rng = np.random.default_rng(N + tps)
    resid = rng.standard_normal((N, n)).astype(np.float32)
    tab = rng.standard_normal((6, n)).astype(np.float32)
    c6 = rng.standard_normal((B, 6 * n)).astype(np.float32)
    dres = to_dev(resid)
    lib.ddit_linear_fwd_tile(tile, 2, to_dev(u), k, to_dev(W), to_dev(b), N, n, k, None, 0, resid=dres, ada_table=to_dev(tab),
                             c6=to_dev(c6), gate_row=5, tokens_per_sample=tps)
    torch.cuda.synchronize()
    lin = ora.linear(to_f64(u), to_f64(W), to_f64(b))
    ref = resid.astype(np.float64)
    for r in range(N):
        ref[r] += (tab[5] + c6[r // tps].reshape(6, n)[5]).astype(np.float64) * lin[r]
    assert_parity(dev_to_f64(dres), ref, "residual linear, %d samples in a tile" % B)


def _check_linear(lib, N, n, k, epi, tile):
    u = syn.normal_bits((11, N, n, k), (N, k), 1.0)
    W = syn.normal_bits((12, N, n, k), (n, k), 1.0 / math.sqrt(k))
    b = syn.normal_bits((13, N, n, k), (n,), 0.5)
    lin = ora.linear(to_f64(u), to_f64(W), to_f64(b))
    du, dW, db = to_dev(u), to_dev(W), to_dev(b)
    if epi in (0, 1):
        out = torch.full((N, n), float("nan"), dtype=torch.bfloat16, device="cuda")
        lib.ddit_linear_fwd_tile(tile, epi, du, k, dW, db, N, n, k, out, n)
        torch.cuda.synchronize()
        ref = lin if epi == 0 else ora.gelu_tanh(lin)
        assert_parity(dev_to_f64(out), ref, "linear epi=%d" % epi)
    else:
        tps = max(1, (N + 1) // 2)   # two samples
        B = (N + tps - 1) // tps
        rng = np.random.default_rng(5)
        resid = rng.standard_normal((N, n)).astype(np.float32)
        tab = rng.standard_normal((6, n)).astype(np.float32)
        c6 = rng.standard_normal((B, 6 * n)).astype(np.float32)
        for gate_row in (2, 5, -1):
            dres = to_dev(resid)
            out = torch.full((N, n), float("nan"), dtype=torch.bfloat16, device="cuda")
            lib.ddit_linear_fwd_tile(tile, 2, du, k, dW, db, N, n, k, out, n, resid=dres, ada_table=to_dev(tab),
                                     c6=to_dev(c6), gate_row=gate_row, tokens_per_sample=tps)
            torch.cuda.synchronize()
            ref = resid.astype(np.float64).copy()
            for r in range(N):
                gate = 1.0 if gate_row < 0 else (tab[gate_row] + c6[r // tps].reshape(6, n)[gate_row]).astype(np.float64)
                ref[r] += gate * lin[r]
            assert_parity(dev_to_f64(dres), ref, "linear residual gate_row=%d" % gate_row)
            assert torch.equal(out, dres.to(torch.bfloat16)), "bf16 copy of the stream differs"
        # without the bf16 copy
        dres = to_dev(resid)
        lib.ddit_linear_fwd_tile(tile, 2, du, k, dW, None, N, n, k, None, 0, resid=dres)
        torch.cuda.synchronize()
        assert_parity(dev_to_f64(dres), resid + ora.linear(to_f64(u), to_f64(W)), "linear residual, no bias/gate/copy")


def test_linear_strided_in_out(lib):
    """u read with a row stride larger than k, out written as a column slice (fused qkv buffer use)."""
    N, n, k, ld_u, ld_out = 200, 128, 192, 320, 384
    ubuf = syn.normal_bits((21,), (N, ld_u), 1.0)
    W = syn.normal_bits((22,), (n, k), 0.1)
    outbuf = torch.full((N, ld_out), 7.0, dtype=torch.bfloat16, device="cuda")
    lib.ddit_linear_fwd(0, to_dev(ubuf), ld_u, to_dev(W), None, N, n, k, outbuf, ld_out)
    torch.cuda.synchronize()
    ref = ora.linear(to_f64(ubuf)[:, :k], to_f64(W))
    assert_parity(dev_to_f64(outbuf[:, :n]), ref, "strided linear")
    assert torch.all(outbuf[:, n:] == 7.0), "wrote outside its column slice"


# ----------------------------------------------------------------------------- attention
def _attn_case(lib, kind, sh, q_scale=1.0, valid=None, seed=0, Lq=None, fused=False):
    d = syn.make_attn_inputs(kind, sh, 50 + seed, q_scale=q_scale, Lq=Lq)
    q, k, v = (to_f64(d[n]) for n in "qkv")
    A = sh.A
    if kind == "cross":
        o_ref, lse_ref = ora.cross_attention(q, k, v, valid)
        kid = lib.DDIT_ATTN_CROSS
        shape = _shape(lib, syn.small_variant(sh, T=1, Hp=1, Wp=q.shape[1]))
    else:
        fn = ora.spatial_attention if kind == "spatial" else ora.temporal_attention
        o_ref, lse_ref = fn(q, k, v)
        kid = lib.DDIT_ATTN_SPATIAL if kind == "spatial" else lib.DDIT_ATTN_TEMPORAL
        shape = _shape(lib, sh)
    dq, dk, dv = (to_dev(d[n]) for n in "qkv")
    ld_q = ld_kv = A
    if fused and kind != "cross":   # q|k|v as column slices of one [tokens, 3A] buffer
        buf = torch.cat([dq.reshape(-1, A), dk.reshape(-1, A), dv.reshape(-1, A)], dim=1).contiguous()
        dq, dk, dv = buf[:, :A], buf[:, A:2 * A], buf[:, 2 * A:]
        ld_q = ld_kv = 3 * A
    o = torch.full(q.shape, float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.full(lse_ref.shape, float("nan"), dtype=torch.float32, device="cuda")
    lib.ddit_attn_fwd(kid, shape, dq, dk, dv, ld_q, ld_kv, None if valid is None else list(valid), o, A, lse)
    torch.cuda.synchronize()
    ev, fv = assert_parity(dev_to_f64(o), o_ref, "%s attention O" % kind)
    assert np.max(np.abs(dev_to_f64(lse) - lse_ref)) < 2e-2, "lse"
    return ev, fv


SELF_SHAPES = [
    syn.Shape(1, 4, 8, 8, 256, 4, 64, 1024, 16, 1),       # C1: one key tile, dh 64
    syn.Shape(1, 3, 9, 16, 1152, 2, 72, 4608, 300, 1),    # 144p frame: S=144, three key tiles, ragged
    syn.Shape(2, 2, 15, 27, 1152, 3, 72, 4608, 300, 1),   # 240p frame: S=405, ragged query and key tails
    syn.Shape(1, 1, 30, 54, 1152, 1, 72, 4608, 300, 1),   # 480p frame: S=1620
    syn.Shape(1, 5, 1, 1, 64, 1, 64, 64, 8, 1),           # S=1
    syn.Shape(1, 2, 13, 5, 128, 2, 64, 64, 8, 1),         # S=65: one key past a tile
]


@pytest.mark.parametrize("sh", SELF_SHAPES, ids=lambda s: "T%dS%dH%ddh%d" % (s.T, s.S, s.H, s.dh))
@pytest.mark.parametrize("q_scale", [1.0, 4.0])
def test_spatial_attention(lib, sh, q_scale):
    _attn_case(lib, "spatial", sh, q_scale=q_scale)


def test_spatial_attention_fused_buffer(lib):
    _attn_case(lib, "spatial", SELF_SHAPES[1], fused=True)


TEMPORAL_SHAPES = [
    syn.Shape(1, 4, 8, 8, 256, 4, 64, 1024, 16, 1),
    syn.Shape(1, 16, 5, 7, 1152, 16, 72, 4608, 300, 1),
    syn.Shape(2, 30, 3, 11, 1152, 4, 72, 4608, 300, 1),
    syn.Shape(1, 1, 4, 4, 1152, 2, 72, 4608, 300, 1),     # T=1: O = V
    syn.Shape(1, 32, 2, 3, 1152, 1, 72, 4608, 300, 1),
    syn.Shape(1, 45, 2, 3, 1152, 2, 72, 4608, 300, 1),    # T above the short-sequence kernel's limit
]


@pytest.mark.parametrize("sh", TEMPORAL_SHAPES, ids=lambda s: "T%dS%dH%ddh%d" % (s.T, s.S, s.H, s.dh))
@pytest.mark.parametrize("q_scale", [1.0, 4.0])
def test_temporal_attention(lib, sh, q_scale):
    _attn_case(lib, "temporal", sh, q_scale=q_scale)


def test_temporal_attention_fused_buffer(lib):
    _attn_case(lib, "temporal", TEMPORAL_SHAPES[1], fused=True)


@pytest.mark.parametrize("Lq,Ly,H,dh,valid", [
    (256, 16, 4, 64, None), (256, 16, 4, 64, [5]), (1000, 300, 3, 72, [300]), (1000, 300, 3, 72, [32]),
    (333, 300, 2, 72, [166]), (70, 300, 2, 72, [1]), (129, 65, 1, 72, [64]),
])
def test_cross_attention(lib, Lq, Ly, H, dh, valid):
    sh = syn.Shape(1, 1, 1, Lq, H * dh, H, dh, 64, Ly, 1)
    _attn_case(lib, "cross", sh, valid=valid, Lq=Lq)
    _attn_case(lib, "cross", sh, valid=valid, Lq=Lq, q_scale=4.0, seed=1)


def test_cross_attention_batch2_masks(lib):
    sh = syn.Shape(2, 1, 1, 200, 144, 2, 72, 64, 300, 1)
    _attn_case(lib, "cross", sh, valid=[45, 290], Lq=200)


# ---- self-attention with q/k normalisation and rotary embedding folded into the attention kernels
OPT_SHAPES = [
    syn.Shape(1, 4, 8, 8, 256, 4, 64, 1024, 16, 1),       # one key tile, dh 64
    syn.Shape(2, 3, 15, 27, 1152, 3, 72, 4608, 300, 1),   # S = 405 ragged, three heads (a partial head group), batch 2
    syn.Shape(1, 30, 9, 16, 1152, 16, 72, 4608, 300, 1),  # T = 30 frames, 16 heads
    syn.Shape(1, 40, 3, 5, 144, 2, 72, 64, 8, 1),         # T = 40: beyond the dedicated temporal kernel
]


@pytest.mark.parametrize("sh", OPT_SHAPES, ids=lambda s: "B%dT%dS%dH%ddh%d" % (s.B, s.T, s.S, s.H, s.dh))
@pytest.mark.parametrize("kind", ["spatial", "temporal"])
@pytest.mark.parametrize("norm,rope", [(True, False), (False, True), (True, True)], ids=["norm", "rope", "norm+rope"])
@pytest.mark.parametrize("fuse,one_buffer", [(True, True), (True, False), (False, True), (False, False)],
                         ids=["fused-qkvbuf", "fused-separate", "passes-qkvbuf", "passes-separate"])
def test_self_attention_with_options(lib, sh, kind, norm, rope, fuse, one_buffer):
    if kind == "spatial" and sh.S > 200 and sh.T > 8:
        pytest.skip("covered by the smaller frames")
    d = syn.make_attn_inputs(kind, sh, 70, q_scale=1.0)
    q, k, v = (to_f64(d[n]) for n in "qkv")                       # [B,T,S,H,dh]
    A, dh = sh.A, sh.dh
    gq = syn.f32_to_bf16_bits((1 + 0.2 * np.random.default_rng(11).standard_normal(dh)).astype(np.float32))
    gk = syn.f32_to_bf16_bits((1 + 0.2 * np.random.default_rng(12).standard_normal(dh)).astype(np.float32))
    qq, kk = q, k
    if norm:
        qq, kk = ora.rms_norm(qq, to_f64(gq)), ora.rms_norm(kk, to_f64(gk))
    if rope and kind == "temporal":
        frame = np.arange(sh.T, dtype=np.float64)[None, :, None, None]
        qq, kk = ora.rotary(qq, frame), ora.rotary(kk, frame)
    o_ref, lse_ref = (ora.spatial_attention if kind == "spatial" else ora.temporal_attention)(qq, kk, v)
    dq, dk, dv = (to_dev(d[n]).reshape(-1, A) for n in "qkv")
    ld = A
    if one_buffer:
        buf = torch.cat([dq, dk, dv], dim=1).contiguous()
        dq, dk, dv = buf[:, :A], buf[:, A:2 * A], buf[:, 2 * A:]
        ld = 3 * A
    v_before = dv.clone()
    o = torch.full((sh.N, A), float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.full(lse_ref.shape, float("nan"), dtype=torch.float32, device="cuda")
    tab = torch.empty(sh.T * dh, dtype=torch.float32, device="cuda") if rope else None
    kid = lib.DDIT_ATTN_SPATIAL if kind == "spatial" else lib.DDIT_ATTN_TEMPORAL
    lib.ddit_self_attn_fwd(kid, _shape(lib, sh), dq, dk, dv, ld, ld, to_dev(gq) if norm else None, to_dev(gk) if norm else None,
                           tab, fuse, o, A, lse)
    torch.cuda.synchronize()
    assert_parity(dev_to_f64(o).reshape(o_ref.shape), o_ref, "%s attention with options" % kind)
    assert np.max(np.abs(dev_to_f64(lse) - lse_ref)) < 3e-2, "lse"
    assert torch.equal(dv, v_before), "v was written"


# Short text sequences shared by many queries take the resident form of the kernel (all K/V tiles of a
# (sample, head) unit fetched once, the workgroup walking over a run of query tiles): it is chosen when a
# unit has at least four 256-query tiles per workgroup, at one workgroup per CU.  These shapes reach it on
# a 256-CU device (and are valid cases for the streaming form on any other).
@pytest.mark.parametrize("B,Lq,Ly,H,dh,valid,q_scale", [
    (64, 1000, 100, 4, 64, "mixed", 1.0),       # 256 units, one workgroup each, four query tiles, ragged last one
    (2, 8200, 300, 16, 72, [287, 33], 1.0),     # 32 units x 7 workgroups with runs of 5 (last: 3) query tiles
    (2, 8200, 300, 16, 72, [300, 1], 4.0),      # peaked scores; a single valid key
    (64, 1024, 320, 4, 72, None, 1.0),          # five full key tiles: the longest resident sequence
    (64, 1024, 321, 4, 72, None, 1.0),          # one key more: streaming form
], ids=["b64-dh64", "b2-h16", "b2-h16-peaked", "ly320", "ly321"])
def test_cross_attention_many_queries(lib, B, Lq, Ly, H, dh, valid, q_scale):
    sh = syn.Shape(B, 1, 1, Lq, H * dh, H, dh, 64, Ly, 1)
    if valid == "mixed":
        valid = [1 + (37 * b) % Ly for b in range(B)]
    _attn_case(lib, "cross", sh, valid=valid, Lq=Lq, q_scale=q_scale, seed=3)


# ---- closed forms and invariances, on the GPU
def test_values_of_ones_give_ones(lib):
    sh = SELF_SHAPES[2]
    d = syn.make_attn_inputs("spatial", sh, 3)
    ones = torch.ones((sh.B, sh.T, sh.S, sh.H, sh.dh), dtype=torch.bfloat16, device="cuda")
    for kid in (lib.DDIT_ATTN_SPATIAL, lib.DDIT_ATTN_TEMPORAL):
        o = torch.zeros_like(ones)
        lib.ddit_attn_fwd(kid, _shape(lib, sh), to_dev(d["q"]), to_dev(d["k"]), ones, sh.A, sh.A, None, o, sh.A)
        torch.cuda.synchronize()
        assert torch.max(torch.abs(o.float() - 1.0)).item() <= 2 ** -7   # a couple of bf16 ulps at 1.0


def test_zero_keys_give_mean_of_values(lib):
    sh = SELF_SHAPES[1]
    d = syn.make_attn_inputs("spatial", sh, 4)
    zk = torch.zeros((sh.B, sh.T, sh.S, sh.H, sh.dh), dtype=torch.bfloat16, device="cuda")
    o = torch.zeros_like(zk)
    lse = torch.zeros((sh.B, sh.T, sh.S, sh.H), dtype=torch.float32, device="cuda")
    lib.ddit_attn_fwd(lib.DDIT_ATTN_SPATIAL, _shape(lib, sh), to_dev(d["q"]), zk, to_dev(d["v"]), sh.A, sh.A, None, o, sh.A, lse)
    torch.cuda.synchronize()
    v = to_f64(d["v"])
    ref = np.broadcast_to(v.mean(axis=2, keepdims=True), v.shape)
    assert np.max(np.abs(dev_to_f64(o) - ref)) < 3e-3
    assert np.max(np.abs(dev_to_f64(lse) - math.log(sh.S))) < 1e-3


def test_large_common_logit_offset(lib):
    """Adding one large vector to every key moves each query's logits by a per-row constant far
    beyond what exp() of a raw logit could take (|offset| up to ~200); the result must stay
    finite and match the oracle evaluated on the same (bf16-rounded) shifted keys."""
    sh = SELF_SHAPES[1]
    d = syn.make_attn_inputs("spatial", sh, 5)
    u = (np.random.default_rng(0).standard_normal(sh.dh) * 64.0).astype(np.float32)
    kshift = syn.f32_to_bf16_bits(syn.bits_to_f32(d["k"]) + u)
    o = torch.zeros((sh.B, sh.T, sh.S, sh.H, sh.dh), dtype=torch.bfloat16, device="cuda")
    lib.ddit_attn_fwd(lib.DDIT_ATTN_SPATIAL, _shape(lib, sh), to_dev(d["q"]), to_dev(kshift), to_dev(d["v"]),
                      sh.A, sh.A, None, o, sh.A)
    torch.cuda.synchronize()
    ref = ora.spatial_attention(to_f64(d["q"]), to_f64(kshift), to_f64(d["v"]))[0]
    assert_parity(dev_to_f64(o), ref, "shifted keys")


def test_attention_is_deterministic(lib):
    sh = SELF_SHAPES[2]
    d = syn.make_attn_inputs("spatial", sh, 6)
    outs = []
    for _ in range(2):
        o = torch.zeros((sh.B, sh.T, sh.S, sh.H, sh.dh), dtype=torch.bfloat16, device="cuda")
        lib.ddit_attn_fwd(lib.DDIT_ATTN_SPATIAL, _shape(lib, sh), to_dev(d["q"]), to_dev(d["k"]), to_dev(d["v"]), sh.A, sh.A, None, o, sh.A)
        outs.append(o)
    torch.cuda.synchronize()
    assert torch.equal(outs[0], outs[1])


# ----------------------------------------------------------------------------- timestep conditioning
def test_timestep_conditioning(lib):
    sh = syn.Shape(2, 2, 2, 2, 1152, 16, 72, 4608, 8, 0)
    sw = syn.make_step_weights(sh, 9, w_std=0.05)
    dsw = {k: to_dev(v) for k, v in sw.items()}
    st = lib.step_struct(dsw, [])
    t = [3.25, 987.5]
    c6 = torch.empty(sh.B, 6 * sh.D, dtype=torch.float32, device="cuda")
    scratch = torch.empty(sh.B * (256 + 2 * sh.D), dtype=torch.float32, device="cuda")
    lib.ddit_timestep_conditioning(_shape(lib, sh), st, t, None, c6, scratch)
    torch.cuda.synchronize()
    sw64 = {k: to_f64(v) for k, v in sw.items()}
    ref = ora.conditioning(ora.timestep_embedding(np.array(t), sw64), sw64)
    assert rel_fro(dev_to_f64(c6), ref) < 1e-4
    # the sinusoidal features themselves (first 256 floats per sample of the scratch)
    feat = dev_to_f64(scratch[:sh.B * 256].reshape(sh.B, 256))
    assert np.max(np.abs(feat - ora.timestep_features(np.array(t)))) < 1e-6
    # a given temb bypasses the embedder
    temb = syn.make_temb(sh, 9)
    lib.ddit_timestep_conditioning(_shape(lib, sh), st, None, to_dev(temb), c6, None)
    torch.cuda.synchronize()
    assert rel_fro(dev_to_f64(c6), ora.conditioning(temb.astype(np.float64), sw64)) < 1e-4
