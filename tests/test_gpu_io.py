"""Parity on the GPU of the layers around the token-space step (patch embedding + position code,
caption embedder, output head), of the whole model on a latent, and of the sampling loop of
eq. 1 (Euler solver, guidance, resumable step ranges, replay from a captured HIP graph), all
through the C ABI against the CPU oracle on the same seeded inputs.

The latent-sized results are compared under the usual bar; the solver's own arithmetic (one
multiply-add per element in fp32) is compared to 1e-6."""
import numpy as np
import pytest
import torch

import ddit_synth as syn
from helpers import assert_parity, dev_to_f64, dict_dev, dict_f64, to_dev, to_f64
from oracle import latent_io_oracle as lio
from oracle import stdit_oracle as ora

pytestmark = pytest.mark.gpu

# (shape, latent channels, text width): a small one with ragged token counts, and one with the
# paper model's hidden size and head shape
IO_CASES = [
    (syn.Shape(B=2, T=3, Hp=5, Wp=7, D=256, H=4, dh=64, M=512, Ly=16, n_blocks=1), 4, 64),
    (syn.Shape(B=1, T=2, Hp=6, Wp=9, D=1152, H=16, dh=72, M=1536, Ly=24, n_blocks=1), 4, 128),
]
IDS = ["D256", "D1152"]


@pytest.fixture(scope="module")
def lib():
    import paper_2506_13497_amd as m
    assert torch.cuda.is_available()
    return m


def _shape(lib, sh, flags=0):
    return lib.make_shape(sh.B, sh.T, sh.Hp, sh.Wp, sh.D, sh.H, sh.dh, sh.M, sh.Ly, sh.n_blocks, flags)


class Setup:
    def __init__(self, lib, sh, C, C_text, base=31, options=False):
        self.sh, self.C, self.C_text, self.options = sh, C, C_text, options
        self.shape = _shape(lib, sh, (lib.DDIT_FLAG_QK_NORM | lib.DDIT_FLAG_ROPE_TEMPORAL) if options else 0)
        self.io_w = syn.make_io_weights(sh, base, C, C_text, C)
        self.sw = syn.make_step_weights(sh, base)
        self.blocks = [syn.make_block_weights(sh, base, i, qk_norm=options, table_std=0.3) for i in range(sh.n_blocks)]
        self.z = syn.make_latent(sh, base, C)
        self.c_text = syn.make_caption(sh, base, C_text)
        self.c_unc = syn.make_caption(sh, base, C_text, which=1)
        self.d_io, self.d_sw = dict_dev(self.io_w), dict_dev(self.sw)
        self.d_blocks = [dict_dev(b) for b in self.blocks]
        self.io = lib.io_struct(self.d_io, C, C, C_text)
        self.step = lib.step_struct(self.d_sw, self.d_blocks)
        self.ws = torch.empty(lib.ddit_io_workspace_bytes(self.shape, self.io), dtype=torch.uint8, device="cuda")
        self.f_io, self.f_sw = dict_f64(self.io_w), dict_f64(self.sw)
        self.f_blocks = [dict_f64(b) for b in self.blocks]

    def caption_dev(self, lib, c_bits):
        y = torch.full((self.sh.B, self.sh.Ly, self.sh.D), float("nan"), dtype=torch.bfloat16, device="cuda")
        lib.ddit_embed_caption(self.shape, self.io, to_dev(c_bits), y, self.ws)
        return y

    def oracle_model(self, c_bits, valid):
        c = to_f64(c_bits)
        return lambda z, t: lio.eps_theta(z, c, valid, t, self.f_io, self.f_sw, self.f_blocks, self.sh.H, self.sh.dh,
                                          rope_temporal=self.options)


@pytest.mark.parametrize("case", IO_CASES, ids=IDS)
def test_embed_latent(lib, case):
    st = Setup(lib, *case)
    sh = st.sh
    x = torch.full((sh.B, sh.T, sh.S, sh.D), float("nan"), dtype=torch.bfloat16, device="cuda")
    lib.ddit_embed_latent(st.shape, st.io, to_dev(st.z), x, st.ws)
    torch.cuda.synchronize()
    ref = lio.embed_latent(st.z.astype(np.float64), st.f_io["w_patch"], st.f_io["b_patch"], sh.D)
    assert_parity(dev_to_f64(x), ref, "patch embedding")


@pytest.mark.parametrize("case", IO_CASES, ids=IDS)
def test_embed_caption(lib, case):
    st = Setup(lib, *case)
    y = st.caption_dev(lib, st.c_text)
    torch.cuda.synchronize()
    w = st.f_io
    ref = lio.embed_caption(to_f64(st.c_text), w["w_y1"], w["b_y1"], w["w_y2"], w["b_y2"])
    assert_parity(dev_to_f64(y), ref, "caption embedder")


@pytest.mark.parametrize("case", IO_CASES, ids=IDS)
def test_output_head(lib, case):
    st = Setup(lib, *case)
    sh = st.sh
    x = syn.normal_bits((77, 1), (sh.B, sh.T, sh.S, sh.D), 1.5)
    temb = syn.make_temb(sh, 78)
    out = torch.full((sh.B, st.C, sh.T, 2 * sh.Hp, 2 * sh.Wp), float("nan"), dtype=torch.float32, device="cuda")
    lib.ddit_output_head(st.shape, st.io, to_dev(x), to_dev(temb), out)
    torch.cuda.synchronize()
    w = st.f_io
    ref = lio.output_head(to_f64(x), temb.astype(np.float64), w["final_table"], w["w_final"], w["b_final"], sh.Hp, sh.Wp, st.C)
    assert_parity(dev_to_f64(out), ref, "output head")


@pytest.mark.parametrize("case", IO_CASES, ids=IDS)
def test_eps_theta(lib, case):
    st = Setup(lib, *case)
    sh = st.sh
    valid = [sh.Ly - 3 * b for b in range(sh.B)]
    t = [250.0 + 500.0 * b for b in range(sh.B)]
    y = st.caption_dev(lib, st.c_text)
    out = torch.full((sh.B, st.C, sh.T, 2 * sh.Hp, 2 * sh.Wp), float("nan"), dtype=torch.float32, device="cuda")
    lib.ddit_eps_theta(st.shape, st.step, st.io, to_dev(st.z), y, valid, t, out, st.ws)
    torch.cuda.synchronize()
    ref = st.oracle_model(st.c_text, np.array(valid))(st.z.astype(np.float64), np.array(t))
    assert_parity(dev_to_f64(out), ref, "eps_theta on a latent")


def test_eps_theta_with_qk_norm_and_rotary(lib):
    """Latent in, prediction out with both self-attention options on (the folded paths of the step)."""
    st = Setup(lib, *IO_CASES[0], options=True)
    sh = st.sh
    valid = [sh.Ly - 3 * b for b in range(sh.B)]
    t = [100.0 + 700.0 * b for b in range(sh.B)]
    y = st.caption_dev(lib, st.c_text)
    out = torch.full((sh.B, st.C, sh.T, 2 * sh.Hp, 2 * sh.Wp), float("nan"), dtype=torch.float32, device="cuda")
    lib.ddit_eps_theta(st.shape, st.step, st.io, to_dev(st.z), y, valid, t, out, st.ws)
    torch.cuda.synchronize()
    ref = st.oracle_model(st.c_text, np.array(valid))(st.z.astype(np.float64), np.array(t))
    assert_parity(dev_to_f64(out), ref, "eps_theta with q/k normalisation and rotary embedding")


def test_solver_step(lib):
    B, per = 3, 1000
    g = np.random.default_rng(5)
    z, ec, eu = (g.standard_normal((B, per)).astype(np.float32) for _ in range(3))
    t, tn = [900.0, 500.0, 100.0], [800.0, 250.0, 0.0]
    for guidance, with_u in ((1.0, False), (7.5, True), (0.0, True)):
        dz = to_dev(z.copy())
        lib.ddit_solver_step(dz, to_dev(ec), to_dev(eu) if with_u else None, guidance, t, tn, per)
        torch.cuda.synchronize()
        e = lio.guide(ec.astype(np.float64), eu.astype(np.float64), guidance) if with_u else ec.astype(np.float64)
        ref = lio.solver_step(z.astype(np.float64), e, np.array(t), np.array(tn))
        assert np.max(np.abs(dev_to_f64(dz) - ref)) < 1e-5, (guidance, with_u)


def _run_sample(lib, st, z0, y, valid, y_u, guidance, n, first, last):
    sh = st.sh
    z = z0.clone()
    scratch = torch.empty(2 * z.numel(), dtype=torch.float32, device="cuda")
    lib.ddit_sample(st.shape, st.step, st.io, z, y, valid, y_u, guidance, n, first, last, scratch, st.ws)
    return z


def test_sampling_loop_with_guidance(lib):
    st = Setup(lib, *IO_CASES[0])
    sh = st.sh
    valid = [sh.Ly, sh.Ly - 5]
    n, guidance = 4, 3.0
    y, y_u = st.caption_dev(lib, st.c_text), st.caption_dev(lib, st.c_unc)
    z0 = to_dev(st.z)
    z = _run_sample(lib, st, z0, y, valid, y_u, guidance, n, 0, 3)
    torch.cuda.synchronize()
    mc, mu = st.oracle_model(st.c_text, np.array(valid)), st.oracle_model(st.c_unc, None)
    ref = lio.sample(st.z.astype(np.float64), lambda zz, t: lio.guide(mc(zz, t), mu(zz, t), guidance), n, 0, 3)
    assert_parity(dev_to_f64(z), ref, "latent after 3 of 4 guided steps")
    # the prediction matters: without the steps the latent is far from the result
    assert np.abs(st.z - ref).max() > 0.05
    # a run split at a step boundary is the same run
    part = _run_sample(lib, st, _run_sample(lib, st, z0, y, valid, y_u, guidance, n, 0, 2), y, valid, y_u, guidance, n, 2, 3)
    torch.cuda.synchronize()
    assert torch.equal(part, z)


def test_sampling_loop_without_guidance(lib):
    st = Setup(lib, *IO_CASES[1])
    n = 5
    y = st.caption_dev(lib, st.c_text)
    z = _run_sample(lib, st, to_dev(st.z), y, None, None, 1.0, n, 1, 3)
    torch.cuda.synchronize()
    ref = lio.sample(st.z.astype(np.float64), st.oracle_model(st.c_text, None), n, 1, 3)
    assert_parity(dev_to_f64(z), ref, "latent after steps 1..2 of 5")


def test_step_replays_from_a_captured_graph(lib):
    """One sampling step captured into a HIP graph gives, on every replay, what the eager call gives
    (the library allocates nothing, synchronises nothing and clears no memory behind the caller's back)."""
    st = Setup(lib, *IO_CASES[0])
    sh = st.sh
    y, y_u = st.caption_dev(lib, st.c_text), st.caption_dev(lib, st.c_unc)
    z0 = to_dev(st.z)
    eager = _run_sample(lib, st, z0, y, None, y_u, 2.0, 4, 1, 2)
    torch.cuda.synchronize()
    z = z0.clone()
    scratch = torch.empty(2 * z.numel(), dtype=torch.float32, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            lib.ddit_sample(st.shape, st.step, st.io, z, y, None, y_u, 2.0, 4, 1, 2, scratch, st.ws)
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        z.copy_(z0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(z, eager), "replay %d differs from the eager step" % rep
        # eager work of the program between replays
        again = _run_sample(lib, st, z0, y, None, y_u, 2.0, 4, 1, 2)
        torch.cuda.synchronize()
        assert torch.equal(again, eager)


def test_io_argument_errors(lib):
    st = Setup(lib, *IO_CASES[0])
    sh = st.sh
    small = torch.empty(1024, dtype=torch.uint8, device="cuda")
    x = torch.empty((sh.B, sh.T, sh.S, sh.D), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(lib.DditError) as e:
        lib.ddit_embed_latent(st.shape, st.io, to_dev(st.z), x, small)
    assert e.value.status == lib.DDIT_ERR_WORKSPACE
    bad = lib.io_struct(st.d_io, st.C, st.C, st.C_text + 4)
    with pytest.raises(lib.DditError) as e:
        lib.ddit_io_workspace_bytes(st.shape, bad)
    assert e.value.status == lib.DDIT_ERR_UNSUPPORTED
    z = to_dev(st.z)
    scratch = torch.empty(2 * z.numel(), dtype=torch.float32, device="cuda")
    y = torch.zeros((sh.B, sh.Ly, sh.D), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(lib.DditError) as e:
        lib.ddit_sample(st.shape, st.step, st.io, z, y, None, None, 1.0, 4, 3, 5, scratch, st.ws)
    assert e.value.status == lib.DDIT_ERR_INVALID_ARG
    assert torch.equal(z, to_dev(st.z)), "nothing may run on an argument error"


def test_cross_attention_cache(lib):
    """The per-request cache of cross-attention keys/values: its contents against the oracle's
    projection, and a step (and a guided sampling run) reading it against the same call projecting
    the text itself: bit-identical, the kernels and their inputs being the same."""
    sh = syn.small_variant(IO_CASES[0][0], n_blocks=2)
    st = Setup(lib, sh, IO_CASES[0][1], IO_CASES[0][2])
    y, y_u = st.caption_dev(lib, st.c_text), st.caption_dev(lib, st.c_unc)
    nbytes = lib.ddit_cross_kv_bytes(st.shape)
    assert nbytes == 2 * sh.n_blocks * sh.B * sh.Ly * 2 * sh.A * 2
    kv = torch.full((nbytes // 2,), float("nan"), dtype=torch.bfloat16, device="cuda")
    kv_u = torch.empty_like(kv)
    lib.ddit_cross_kv_precompute(st.shape, st.step, y, kv)
    lib.ddit_cross_kv_precompute(st.shape, st.step, y_u, kv_u)
    torch.cuda.synchronize()
    got = dev_to_f64(kv).reshape(2 * sh.n_blocks, sh.B, sh.Ly, 2 * sh.A)
    yf = dev_to_f64(y)
    for layer, (blk, kind) in enumerate([(0, "spatial"), (0, "temporal"), (1, "spatial"), (1, "temporal")]):
        w = st.f_blocks[blk][kind]
        assert_parity(got[layer], ora.linear(yf, w["w_ckv"], w["b_ckv"]), "cached k|v of layer %d" % layer)
    # one token-space step
    x = to_dev(syn.make_activations(sh, 41)["x"])
    valid = [sh.Ly - 2, sh.Ly]
    outs = []
    for cache in (None, kv):
        o = torch.full((sh.B, sh.T, sh.S, sh.D), float("nan"), dtype=torch.bfloat16, device="cuda")
        lib.ddit_denoise_step_cached(st.shape, st.step, x, None if cache is not None else y, cache, valid, [300.0, 600.0],
                                     None, o, st.ws)
        outs.append(o)
    torch.cuda.synchronize()
    assert torch.isfinite(outs[0].float()).all() and torch.equal(outs[0], outs[1])
    # a guided sampling run
    z0 = to_dev(st.z)
    scratch = torch.empty(2 * z0.numel(), dtype=torch.float32, device="cuda")
    runs = []
    for caches in ((None, None), (kv, kv_u)):
        z = z0.clone()
        lib.ddit_sample(st.shape, st.step, st.io, z, y, valid, y_u, 2.5, 4, 0, 2, scratch, st.ws, caches[0], caches[1])
        runs.append(z)
    torch.cuda.synchronize()
    assert torch.equal(runs[0], runs[1])
    with pytest.raises(lib.DditError) as e:
        lib.ddit_sample(st.shape, st.step, st.io, z0.clone(), y, valid, y_u, 2.5, 4, 0, 1, scratch, st.ws, kv, None)
    assert e.value.status == lib.DDIT_ERR_INVALID_ARG


@pytest.mark.parametrize("D,H,dh,Ly,B,n_blocks,drop_bias", [
    (1152, 16, 72, 300, 2, 3, False),     # 2A = 2304: every output tile divides it; six layers in one launch
    (1152, 4, 72, 77, 1, 2, True),        # one rank's share of the heads (2A = 576), ragged text length, a layer without bias
    (144, 1, 72, 40, 2, 2, False),        # 2A = 144: no tile divides it, the layers are projected one by one
], ids=["full-width", "head-share-no-bias", "one-by-one"])
def test_text_kv_of_all_layers(lib, D, H, dh, Ly, B, n_blocks, drop_bias):
    """The text k|v projections of all layers (one grouped launch where the shape allows) against the oracle."""
    sh = syn.Shape(B, 2, 2, 2, D, H, dh, 64, Ly, n_blocks)
    sw = syn.make_step_weights(sh, 61)
    blocks = [syn.make_block_weights(sh, 61, i) for i in range(n_blocks)]
    if drop_bias:
        blocks[1]["spatial"] = {k: v for k, v in blocks[1]["spatial"].items() if k != "b_ckv"}
    y = syn.make_activations(sh, 61)["y"]
    shape = _shape(lib, sh)
    d_sw, d_blocks = {k: to_dev(v) for k, v in sw.items()}, [dict_dev(b) for b in blocks]   # kept alive: the struct holds pointers
    step = lib.step_struct(d_sw, d_blocks)
    kv = torch.full((lib.ddit_cross_kv_bytes(shape) // 2,), float("nan"), dtype=torch.bfloat16, device="cuda")
    lib.ddit_cross_kv_precompute(shape, step, to_dev(y), kv)
    torch.cuda.synchronize()
    got = dev_to_f64(kv).reshape(2 * n_blocks, B * Ly, 2 * sh.A)
    yf = to_f64(y).reshape(B * Ly, D)
    for layer in range(2 * n_blocks):
        w = dict_f64(blocks[layer // 2]["temporal" if layer & 1 else "spatial"])
        assert_parity(got[layer], ora.linear(yf, w["w_ckv"], w.get("b_ckv")), "text k|v of layer %d" % layer)
