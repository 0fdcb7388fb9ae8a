"""Pins of the CPU oracle against things other than itself.

The paper prints no activation value for the STDiT step, so the oracle is pinned by:
brute-force loop implementations at tiny sizes, library routines of another package
(torch CPU, fp64), closed forms, invariances that follow from section 2.2's statement
of which tokens each attention kind relates, and the parameter count of Table 1.
The last test class plants mistakes in the oracle and checks the pins notice."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import brute_force as bf
import ddit_synth as syn
from helpers import dict_f64, rel_fro, to_f64
from oracle import stdit_oracle as ora

TINY = syn.Shape(B=2, T=3, Hp=2, Wp=2, D=16, H=2, dh=4, M=24, Ly=5, n_blocks=2)


def _paper_values():
    """The few numbers the paper itself prints (tests/golden/paper_printed_values.txt)."""
    import os
    out = {}
    for line in open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "paper_printed_values.txt")):
        line = line.split("#", 1)[0].strip()
        if line:
            k, v = (t.strip() for t in line.split("=", 1))
            out[k] = float(v)
    return out


def _rand(shape, seed, scale=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * scale


def _tiny_layer(seed=0, sh=TINY, std=0.3, table_std=0.5):
    w = dict_f64(syn.make_layer_weights(sh, 77 + seed, 0, "spatial", w_std=std, table_std=table_std))
    x = _rand((sh.B, sh.T, sh.S, sh.D), seed + 1)
    y = _rand((sh.B, sh.Ly, sh.D), seed + 2)
    c6 = _rand((sh.B, 6 * sh.D), seed + 3, 0.5)
    return w, x, y, c6


# --------------------------------------------------------------------------- P1
class TestBruteForce:
    def test_spatial_temporal_cross_vs_loops(self):
        B, T, S, H, dh, Ly = 2, 3, 5, 2, 8, 4
        q, k, v = (_rand((B, T, S, H, dh), i) for i in range(3))
        o, _ = ora.spatial_attention(q, k, v)
        np.testing.assert_allclose(o, np.array(bf.spatial(q.tolist(), k.tolist(), v.tolist())), rtol=0, atol=1e-12)
        o, _ = ora.temporal_attention(q, k, v)
        np.testing.assert_allclose(o, np.array(bf.temporal(q.tolist(), k.tolist(), v.tolist())), rtol=0, atol=1e-12)
        qc = _rand((B, 7, H, dh), 5)
        kc, vc = _rand((B, Ly, H, dh), 6), _rand((B, Ly, H, dh), 7)
        for vl in (None, [4, 2], [1, 3]):
            o, _ = ora.cross_attention(qc, kc, vc, vl)
            ref = np.array(bf.cross(qc.tolist(), kc.tolist(), vc.tolist(), vl))
            np.testing.assert_allclose(o, ref, rtol=0, atol=1e-12)

    def test_spatial_and_temporal_differ(self):
        q, k, v = (_rand((1, 3, 4, 1, 4), i) for i in range(3))
        assert rel_fro(ora.spatial_attention(q, k, v)[0], ora.temporal_attention(q, k, v)[0]) > 0.1

    def test_layer_norm_and_linear_vs_loops(self):
        u = _rand((6, 16), 3) * 3 + 1.5
        got = ora.layer_norm(u)
        for r in range(6):
            np.testing.assert_allclose(got[r], bf.layer_norm_row(u[r].tolist(), 1e-6), atol=1e-12)
        W, b = _rand((5, 16), 4), _rand((5,), 5)
        got = ora.linear(u, W, b)
        for r in range(6):
            np.testing.assert_allclose(got[r], bf.linear_row(u[r].tolist(), W.tolist(), b.tolist()), atol=1e-12)


# ------------------------------------------------------- library routines (torch, fp64)
class TestLibraryRoutines:
    def test_sdpa_vs_torch(self):
        q, k, v = (_rand((3, 2, 9, 8), i) for i in range(3))
        o, lse = ora.sdpa(q, k, v)
        t = F.scaled_dot_product_attention(*(torch.from_numpy(a) for a in (q, k, v)))
        np.testing.assert_allclose(o, t.numpy(), atol=1e-12)
        s = torch.from_numpy(q) @ torch.from_numpy(k).transpose(-1, -2) / math.sqrt(8)
        np.testing.assert_allclose(lse, torch.logsumexp(s, -1).numpy(), atol=1e-12)

    def test_masked_sdpa_vs_torch(self):
        q, k, v = _rand((2, 6, 8), 0), _rand((2, 7, 8), 1), _rand((2, 7, 8), 2)
        mask = torch.zeros(6, 7, dtype=torch.bool)
        mask[:, :3] = True
        t = F.scaled_dot_product_attention(*(torch.from_numpy(a) for a in (q, k, v)), attn_mask=mask)
        np.testing.assert_allclose(ora.sdpa(q, k, v, n_valid=3)[0], t.numpy(), atol=1e-12)

    def test_layer_norm_vs_torch(self):
        u = _rand((4, 5, 32), 1) * 2 - 0.7
        t = F.layer_norm(torch.from_numpy(u), (32,), eps=1e-6)
        np.testing.assert_allclose(ora.layer_norm(u), t.numpy(), atol=1e-12)

    def test_gelu_silu_vs_torch(self):
        u = np.linspace(-6, 6, 241)
        np.testing.assert_allclose(ora.gelu_tanh(u), F.gelu(torch.from_numpy(u), approximate="tanh").numpy(), atol=1e-14)
        np.testing.assert_allclose(ora.silu(u), F.silu(torch.from_numpy(u)).numpy(), atol=1e-14)

    def test_gelu_tanh_close_to_exact_gelu(self):
        # exact GELU is u * Phi(u); the tanh form stays within 1e-3 of it everywhere
        u = np.linspace(-8, 8, 3201)
        exact = np.array([a * 0.5 * (1 + math.erf(a / math.sqrt(2))) for a in u])
        gap = np.max(np.abs(ora.gelu_tanh(u) - exact))
        assert 1e-5 < gap < 1e-3
        assert ora.gelu_tanh(np.array([0.0]))[0] == 0.0
        # large |u|: identity / zero
        np.testing.assert_allclose(ora.gelu_tanh(np.array([10.0, -10.0])), [10.0, 0.0], atol=1e-12)

    def test_linear_vs_torch(self):
        u, W, b = _rand((3, 4, 8), 0), _rand((5, 8), 1), _rand((5,), 2)
        t = F.linear(torch.from_numpy(u), torch.from_numpy(W), torch.from_numpy(b))
        np.testing.assert_allclose(ora.linear(u, W, b), t.numpy(), atol=1e-12)


# --------------------------------------------------------------- closed forms, invariants
class TestAttentionClosedForms:
    def test_rows_sum_to_one(self):  # P2
        q, k, v = (_rand((2, 6, 8), i) for i in range(3))
        _, _, p = ora.sdpa(q, k, v, return_probs=True)
        np.testing.assert_allclose(p.sum(-1), 1.0, atol=1e-14)
        _, _, p = ora.sdpa(q, k, v, n_valid=2, return_probs=True)
        np.testing.assert_allclose(p.sum(-1), 1.0, atol=1e-14)
        assert np.all(p[..., 2:] == 0.0)
        # V := 1 gives O = 1 for all three kinds
        qq, kk = _rand((1, 3, 4, 2, 4), 0), _rand((1, 3, 4, 2, 4), 1)
        ones = np.ones_like(qq)
        np.testing.assert_allclose(ora.spatial_attention(qq, kk, ones)[0], 1.0, atol=1e-14)
        np.testing.assert_allclose(ora.temporal_attention(qq, kk, ones)[0], 1.0, atol=1e-14)

    def test_zero_keys_give_mean_of_values(self):  # P3
        B, T, S, H, dh = 1, 3, 5, 2, 4
        q, v = _rand((B, T, S, H, dh), 0), _rand((B, T, S, H, dh), 1)
        k = np.zeros_like(q)
        o, lse = ora.spatial_attention(q, k, v)
        np.testing.assert_allclose(o, np.broadcast_to(v.mean(axis=2, keepdims=True), v.shape), atol=1e-14)
        np.testing.assert_allclose(lse, math.log(S), atol=1e-14)
        o, lse = ora.temporal_attention(q, k, v)
        np.testing.assert_allclose(o, np.broadcast_to(v.mean(axis=1, keepdims=True), v.shape), atol=1e-14)
        np.testing.assert_allclose(lse, math.log(T), atol=1e-14)
        qc, kc, vc = _rand((2, 6, H, dh), 2), np.zeros((2, 7, H, dh)), _rand((2, 7, H, dh), 3)
        o, lse = ora.cross_attention(qc, kc, vc, [3, 7])
        np.testing.assert_allclose(o[0], np.broadcast_to(vc[0, :3].mean(0), o[0].shape), atol=1e-14)
        np.testing.assert_allclose(o[1], np.broadcast_to(vc[1].mean(0), o[1].shape), atol=1e-14)
        np.testing.assert_allclose(lse[0], math.log(3), atol=1e-14)

    def test_dominant_key_selects_its_value(self):  # P4
        dh = 4
        q = np.zeros((1, 1, 6, 1, dh)); q[..., 0] = 1.0
        k = np.zeros_like(q); v = _rand(q.shape, 1)
        k[0, 0, 2, 0, 0] = 50.0 * math.sqrt(dh)  # logit +50 above the others
        o, _ = ora.spatial_attention(q, k, v)
        np.testing.assert_allclose(o[0, 0, :, 0], np.broadcast_to(v[0, 0, 2, 0], (6, dh)), atol=1e-20 + 6 * math.exp(-50) * 5)

    def test_two_key_closed_form(self):
        # two keys: weights are a logistic function of the logit difference
        dh = 4
        q = np.array([[1.0, 2.0, -1.0, 0.5]]); k = _rand((2, dh), 3); v = _rand((2, dh), 4)
        d = (q @ (k[0] - k[1])) / math.sqrt(dh)
        w0 = 1.0 / (1.0 + math.exp(-d[0]))
        np.testing.assert_allclose(ora.sdpa(q, k, v)[0][0], w0 * v[0] + (1 - w0) * v[1], atol=1e-14)

    def test_key_shift_invariance(self):  # P14
        q, k, v = (_rand((2, 3, 5, 2, 8), i) for i in range(3))
        u = _rand((8,), 9) * 300.0  # large enough to overflow a naive exp
        for fn in (ora.spatial_attention, ora.temporal_attention):
            np.testing.assert_allclose(fn(q, k + u, v)[0], fn(q, k, v)[0], atol=1e-9)

    def test_scale_is_inverse_sqrt_dh(self):
        # lse of a single query against keys with known dot products
        dh = 16
        q = np.ones((1, dh)); k = np.stack([np.ones(dh) * a for a in (0.0, 1.0, 2.0)]); v = np.eye(3, dh)
        _, lse = ora.sdpa(q, k, v)
        want = math.log(sum(math.exp(a * dh / 4.0) for a in (0.0, 1.0, 2.0)))
        assert abs(lse[0] - want) < 1e-12


class TestLayerInvariants:
    def test_frame_permutation_equivariance_spatial(self):  # P5
        w, x, y, c6 = _tiny_layer()
        perm = np.array([2, 0, 1])
        a = ora.layer_fwd("spatial", x[:, perm], y, None, c6, w, TINY.H, TINY.dh)
        b = ora.layer_fwd("spatial", x, y, None, c6, w, TINY.H, TINY.dh)[:, perm]
        np.testing.assert_allclose(a, b, atol=1e-12)

    def test_location_permutation_equivariance_temporal(self):
        w, x, y, c6 = _tiny_layer()
        perm = np.array([3, 1, 0, 2])
        a = ora.layer_fwd("temporal", x[:, :, perm], y, None, c6, w, TINY.H, TINY.dh)
        b = ora.layer_fwd("temporal", x, y, None, c6, w, TINY.H, TINY.dh)[:, :, perm]
        np.testing.assert_allclose(a, b, atol=1e-12)

    def test_locality_per_axis(self):  # P5b: which axis each kind mixes
        w, x, y, c6 = _tiny_layer()
        x2 = x.copy(); x2[:, 1] += _rand(x2[:, 1].shape, 50)   # change frame 1 only (not a constant: LN removes those)
        a = ora.layer_fwd("spatial", x, y, None, c6, w, TINY.H, TINY.dh)
        b = ora.layer_fwd("spatial", x2, y, None, c6, w, TINY.H, TINY.dh)
        assert np.array_equal(a[:, [0, 2]], b[:, [0, 2]]) and not np.allclose(a[:, 1], b[:, 1])
        a = ora.layer_fwd("temporal", x, y, None, c6, w, TINY.H, TINY.dh)
        b = ora.layer_fwd("temporal", x2, y, None, c6, w, TINY.H, TINY.dh)
        assert not np.allclose(a[:, 0], b[:, 0])   # temporal mixes across frames
        x3 = x.copy(); x3[:, :, 2] -= _rand(x3[:, :, 2].shape, 51)   # change location 2 only
        b = ora.layer_fwd("temporal", x3, y, None, c6, w, TINY.H, TINY.dh)
        assert np.array_equal(a[:, :, [0, 1, 3]], b[:, :, [0, 1, 3]]) and not np.allclose(a[:, :, 2], b[:, :, 2])
        a = ora.layer_fwd("spatial", x, y, None, c6, w, TINY.H, TINY.dh)
        b = ora.layer_fwd("spatial", x3, y, None, c6, w, TINY.H, TINY.dh)
        assert not np.allclose(a[:, :, 0], b[:, :, 0])

    def test_single_frame_temporal_is_value_projection(self):  # P6
        sh = syn.small_variant(TINY, T=1)
        w, x, y, c6 = _tiny_layer(sh=sh)
        taps = {}
        ora.layer_fwd("temporal", x, y, None, c6, w, sh.H, sh.dh, taps)
        v_flat = taps["v"].reshape(sh.B, 1, sh.S, sh.A)
        np.testing.assert_allclose(taps["attn_branch"], v_flat @ w["w_o"].T + w["b_o"], atol=1e-13)
        # and v itself is the third slice of the qkv projection of the modulated norm
        np.testing.assert_allclose(v_flat, (taps["xh_msa"] @ w["w_qkv"].T + w["b_qkv"])[..., 2 * sh.A:], atol=1e-13)

    def test_zero_gates(self):  # P7
        w, x, y, c6 = _tiny_layer()
        D = TINY.D
        w = dict(w); tab = w["ada_table"].copy(); w["ada_table"] = tab
        c6 = c6.copy()
        # gates are rows 2 and 5 of table + c6: zero both
        tab[2] = 0; tab[5] = 0
        c6.reshape(TINY.B, 6, D)[:, [2, 5]] = 0
        taps = {}
        out = ora.layer_fwd("spatial", x, y, None, c6, w, TINY.H, TINY.dh, taps)
        np.testing.assert_allclose(out, x + taps["cross_branch"], atol=1e-14)
        assert np.abs(taps["cross_branch"]).max() > 1e-3
        # cross-attention of the *unmodified* stream (it does not see norm or modulation)
        qc = (x @ w["w_cq"].T + w["b_cq"]).reshape(TINY.B, TINY.L, TINY.H, TINY.dh)
        np.testing.assert_allclose(taps["qc"], qc, atol=1e-14)
        w["w_co"] = np.zeros_like(w["w_co"]); w["b_co"] = np.zeros_like(w["b_co"])
        out = ora.layer_fwd("spatial", x, y, None, c6, w, TINY.H, TINY.dh)
        assert np.array_equal(out, x)

    def test_layer_norm_moments_and_scale_minus_one(self):  # P8
        u = _rand((7, 64), 0) * 0.01 + 3.0
        n = ora.layer_norm(u)
        np.testing.assert_allclose(n.mean(-1), 0.0, atol=1e-12)
        var = u.var(-1)
        np.testing.assert_allclose(n.var(-1), var / (var + 1e-6), rtol=1e-10)
        w, x, y, c6 = _tiny_layer()
        D = TINY.D
        w = dict(w); w["ada_table"] = w["ada_table"].copy()
        c6 = c6.copy()
        w["ada_table"][1] = -1.0; c6.reshape(TINY.B, 6, D)[:, 1] = 0.0   # scale_msa = -1
        taps = {}
        ora.layer_fwd("spatial", x, y, None, c6, w, TINY.H, TINY.dh, taps)
        shift = w["ada_table"][0] + c6.reshape(TINY.B, 6, D)[:, 0]
        np.testing.assert_allclose(taps["xh_msa"], np.broadcast_to(shift[:, None, None, :], x.shape), atol=1e-14)

    def test_modulation_chunk_order(self):
        D = 8
        table = np.arange(6 * D, dtype=np.float64).reshape(6, D)
        m = ora.split_modulation(table, np.zeros(6 * D), D)
        for i, n in enumerate(["shift_msa", "scale_msa", "gate_msa", "shift_mlp", "scale_mlp", "gate_mlp"]):
            assert np.array_equal(m[n], table[i])
        np.testing.assert_allclose(ora.modulate(np.full(3, 2.0), 0.5, 0.25), 2.0 * 1.25 + 0.5)

    def test_masked_text_positions_do_not_matter(self):  # P9
        w, x, y, c6 = _tiny_layer()
        vl = np.array([2, 4])
        y2 = y.copy(); y2[0, 2:] += 5.0; y2[1, 4:] -= 3.0
        a = ora.layer_fwd("spatial", x, y, vl, c6, w, TINY.H, TINY.dh)
        b = ora.layer_fwd("spatial", x, y2, vl, c6, w, TINY.H, TINY.dh)
        assert np.array_equal(a, b)
        c = ora.layer_fwd("spatial", x, y2, None, c6, w, TINY.H, TINY.dh)
        assert not np.allclose(a, c)
        with pytest.raises(ValueError):
            ora.layer_fwd("spatial", x, y, np.array([0, 4]), c6, w, TINY.H, TINY.dh)

    def test_identity_linear(self):  # P10
        u = _rand((3, 6), 0)
        assert np.array_equal(ora.linear(u, np.eye(6), np.zeros(6)), u)
        assert np.array_equal(ora.linear(u, np.eye(6)), u)
        W = np.zeros((2, 6)); W[1, 4] = 1.0   # out index is the FIRST axis of W
        np.testing.assert_array_equal(ora.linear(u, W)[:, 1], u[:, 4])

    def test_batch_independence(self):  # P11
        w, x, y, c6 = _tiny_layer()
        x2, y2, c62 = x.copy(), y.copy(), c6.copy()
        x2[1] += _rand(x2[1].shape, 52); y2[1] -= 1; c62[1] *= 2
        vl, vl2 = np.array([3, 5]), np.array([3, 2])
        for kind in ("spatial", "temporal"):
            a = ora.layer_fwd(kind, x, y, vl, c6, w, TINY.H, TINY.dh)
            b = ora.layer_fwd(kind, x2, y2, vl2, c62, w, TINY.H, TINY.dh)
            assert np.array_equal(a[0], b[0]) and not np.allclose(a[1], b[1])

    def test_head_split_layout(self):
        # head h owns columns h*dh..(h+1)*dh of each of the q|k|v row groups of W_qkv
        w, x, y, c6 = _tiny_layer()
        taps = {}
        ora.layer_fwd("spatial", x, y, None, c6, w, TINY.H, TINY.dh, taps)
        A, dh = TINY.A, TINY.dh
        full = taps["xh_msa"] @ w["w_qkv"].T + w["b_qkv"]
        for h in range(TINY.H):
            np.testing.assert_array_equal(taps["q"][..., h, :], full[..., h * dh:(h + 1) * dh])
            np.testing.assert_array_equal(taps["k"][..., h, :], full[..., A + h * dh:A + (h + 1) * dh])
            np.testing.assert_array_equal(taps["v"][..., h, :], full[..., 2 * A + h * dh:2 * A + (h + 1) * dh])
        # zeroing head 1's value rows leaves head 0's attention output unchanged
        w2 = dict(w); w2["w_qkv"] = w["w_qkv"].copy(); w2["b_qkv"] = w["b_qkv"].copy()
        w2["w_qkv"][2 * A + dh:2 * A + 2 * dh] = 0; w2["b_qkv"][2 * A + dh:2 * A + 2 * dh] = 0
        taps2 = {}
        ora.layer_fwd("spatial", x, y, None, c6, w2, TINY.H, TINY.dh, taps2)
        assert np.array_equal(taps["o"][..., 0, :], taps2["o"][..., 0, :])
        assert np.all(taps2["o"][..., 1, :] == 0)

    def test_narrow_attention_width(self):
        # A = H*dh < D (one rank's share of a head split) runs and keeps the shape
        sh = syn.small_variant(TINY, H=1)
        assert sh.A < sh.D
        w, x, y, c6 = _tiny_layer(sh=sh)
        out = ora.layer_fwd("spatial", x, y, None, c6, w, sh.H, sh.dh)
        assert out.shape == x.shape and np.isfinite(out).all()


class TestStep:
    def test_timestep_features(self):
        e = ora.timestep_features(np.array([0.0, 1.0, 777.25]))
        assert e.shape == (3, 256)
        np.testing.assert_array_equal(e[0, :128], 1.0); np.testing.assert_array_equal(e[0, 128:], 0.0)
        assert abs(e[1, 0] - math.cos(1.0)) < 1e-15 and abs(e[1, 128] - math.sin(1.0)) < 1e-15
        np.testing.assert_allclose(e[:, :128] ** 2 + e[:, 128:] ** 2, 1.0, atol=1e-12)
        # frequency i is 10000^(-i/128): check i = 64 (1/100) and i = 127
        assert abs(e[2, 64] - math.cos(777.25 / 100.0)) < 1e-12
        assert abs(e[2, 128 + 127] - math.sin(777.25 * 10000.0 ** (-127 / 128))) < 1e-12

    def test_conditioning_chain_vs_torch(self):
        sh = TINY
        sw = dict_f64(syn.make_step_weights(sh, 5, w_std=0.3))
        t = np.array([3.0, 912.5])
        e = torch.from_numpy(ora.timestep_features(t))
        tw = {k: torch.from_numpy(v) for k, v in sw.items()}
        temb = F.linear(F.silu(F.linear(e, tw["w_t1"], tw["b_t1"])), tw["w_t2"], tw["b_t2"])
        c6 = F.linear(F.silu(temb), tw["w_ada"], tw["b_ada"])
        np.testing.assert_allclose(ora.timestep_embedding(t, sw), temb.numpy(), atol=1e-12)
        np.testing.assert_allclose(ora.conditioning(ora.timestep_embedding(t, sw), sw), c6.numpy(), atol=1e-12)

    def test_step_is_layers_composed(self):  # P13
        sh = TINY
        sw = dict_f64(syn.make_step_weights(sh, 5, w_std=0.3))
        blocks = [dict_f64(syn.make_block_weights(sh, 6, i, w_std=0.3, table_std=0.5)) for i in range(2)]
        x, y = _rand((sh.B, sh.T, sh.S, sh.D), 1), _rand((sh.B, sh.Ly, sh.D), 2)
        t = np.array([10.0, 500.0]); vl = np.array([5, 2])
        got = ora.denoise_step(x, y, vl, t, sw, blocks, sh.H, sh.dh)
        c6 = ora.conditioning(ora.timestep_embedding(t, sw), sw)
        z = x
        for i in range(2):
            for kind in ("spatial", "temporal"):
                z = ora.layer_fwd(kind, z, y, vl, c6, blocks[i][kind], sh.H, sh.dh)
        assert np.array_equal(got, z)
        # layer order matters and is spatial first
        z2 = ora.layer_fwd("temporal", x, y, vl, c6, blocks[0]["spatial"], sh.H, sh.dh)
        assert not np.allclose(z2, ora.layer_fwd("spatial", x, y, vl, c6, blocks[0]["spatial"], sh.H, sh.dh))

    def test_full_layer_vs_torch_modules(self):
        """The whole layer rebuilt from torch library calls (fp64) in the stated order."""
        sh = TINY
        w, x, y, c6 = _tiny_layer()
        vl = np.array([4, 2])
        tw = {k: torch.from_numpy(v) for k, v in w.items()}
        X, Y, C = torch.from_numpy(x), torch.from_numpy(y), torch.from_numpy(c6)
        B, T, S, D, H, dh, A = sh.B, sh.T, sh.S, sh.D, sh.H, sh.dh, sh.A
        for kind in ("spatial", "temporal"):
            m = (tw["ada_table"][None] + C.reshape(B, 6, D))[:, :, None, None, :]   # [B,6,1,1,D]
            xh = F.layer_norm(X, (D,), eps=1e-6) * (1 + m[:, 1]) + m[:, 0]
            qkv = F.linear(xh, tw["w_qkv"], tw["b_qkv"]).reshape(B, T, S, 3, H, dh)
            q, k, v = qkv[:, :, :, 0], qkv[:, :, :, 1], qkv[:, :, :, 2]
            if kind == "spatial":   # sequences over S: [B,T,H,S,dh]
                o = F.scaled_dot_product_attention(q.permute(0, 1, 3, 2, 4), k.permute(0, 1, 3, 2, 4),
                                                   v.permute(0, 1, 3, 2, 4)).permute(0, 1, 3, 2, 4)
            else:                   # sequences over T: [B,S,H,T,dh]
                o = F.scaled_dot_product_attention(q.permute(0, 2, 3, 1, 4), k.permute(0, 2, 3, 1, 4),
                                                   v.permute(0, 2, 3, 1, 4)).permute(0, 3, 1, 2, 4)
            z = X + m[:, 2] * F.linear(o.reshape(B, T, S, A), tw["w_o"], tw["b_o"])
            qc = F.linear(z, tw["w_cq"], tw["b_cq"]).reshape(B, T * S, H, dh).transpose(1, 2)
            kv = F.linear(Y, tw["w_ckv"], tw["b_ckv"]).reshape(B, sh.Ly, 2, H, dh)
            kc, vc = kv[:, :, 0].transpose(1, 2), kv[:, :, 1].transpose(1, 2)
            mask = torch.arange(sh.Ly)[None, :] < torch.from_numpy(vl)[:, None]      # [B,Ly]
            oc = F.scaled_dot_product_attention(qc, kc, vc, attn_mask=mask[:, None, None, :])
            z = z + F.linear(oc.transpose(1, 2).reshape(B, T, S, A), tw["w_co"], tw["b_co"])
            xh2 = F.layer_norm(z, (D,), eps=1e-6) * (1 + m[:, 4]) + m[:, 3]
            z = z + m[:, 5] * F.linear(F.gelu(F.linear(xh2, tw["w_fc1"], tw["b_fc1"]), approximate="tanh"),
                                       tw["w_fc2"], tw["b_fc2"])
            got = ora.layer_fwd(kind, x, y, vl, c6, w, H, dh)
            np.testing.assert_allclose(got, z.numpy(), atol=1e-11)

    def test_parameter_count_matches_table_1(self):  # P12
        n = ora.parameter_count(1152, 1152, 4608, 28)
        assert abs(n - 1.19e9) < 0.01e9           # 1.19 B for this structure
        printed = _paper_values()["stdit3_parameters_billion"] * 1e9      # Table 1: STDiT3, 1.1 B
        assert printed == 1.1e9 and abs(n / printed - 1.0) < 0.10
        # the alternative reading (one cross-attention and one MLP per block) is far from what the table prints
        D, A, M = 1152, 1152, 4608
        cross = (A * D + A) + (2 * A * D + 2 * A) + (D * A + D)
        mlp = (M * D + M) + (D * M + D)
        one_per_block = n - 28 * (cross + mlp)
        assert abs(one_per_block - 0.75e9) < 0.01e9 and abs(one_per_block / printed - 1.0) > 0.25
        # count equals the number of elements the generator actually makes
        sh = syn.CONFIGS["C2"]["shape"]
        per_layer = sum(int(np.prod(s)) for s in syn.layer_shapes(sh).values())
        step = sum(int(np.prod(s)) for s in syn.step_shapes(sh).values())
        assert n == 56 * per_layer + step

    def test_fp32_run_bounds_oracle_rounding(self):  # P15
        sh = syn.small_variant(TINY, D=64, M=128, Hp=4, Wp=4)
        w, x, y, c6 = _tiny_layer(sh=sh, std=0.1)
        ref = ora.layer_fwd("spatial", x, y, None, c6, w, sh.H, sh.dh)
        w32 = {k: v.astype(np.float32) for k, v in w.items()}
        got = ora.layer_fwd("spatial", x.astype(np.float32), y.astype(np.float32), None,
                            c6.astype(np.float32), w32, sh.H, sh.dh)
        assert got.dtype == np.float32
        assert rel_fro(got, ref) < 1e-5


# --------------------------------------------------------------- planted mistakes
class TestQkNormRotary:
    """The two optional pieces: per-head RMS normalisation of q and k, and the rotary
    embedding of the temporal layer's q and k."""

    def test_rms_norm_vs_torch_and_loops(self):
        u, g = _rand((5, 3, 8), 1) * 2 + 0.3, _rand((8,), 2) * 0.2 + 1
        got = ora.rms_norm(u, g, 1e-6)
        ref = F.rms_norm(torch.from_numpy(u), (8,), torch.from_numpy(g), 1e-6).numpy()
        np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(got[2, 1], bf.rms_norm_row(u[2, 1].tolist(), g.tolist(), 1e-6), atol=1e-12)

    def test_rms_norm_closed_forms(self):
        # (3, 4): mean square 12.5
        np.testing.assert_allclose(ora.rms_norm(np.array([3.0, 4.0]), np.ones(2), 0.0), np.array([3.0, 4.0]) / math.sqrt(12.5))
        u = _rand((7, 12), 3) + 0.7                                  # non-zero mean: not a LayerNorm
        n = ora.rms_norm(u, np.ones(12), 0.0)
        np.testing.assert_allclose((n ** 2).mean(-1), 1.0, atol=1e-12)
        np.testing.assert_allclose(ora.rms_norm(5.0 * u, np.ones(12), 0.0), n, atol=1e-12)     # scale invariant
        assert abs(n.mean(-1)).max() > 0.1                                                     # mean is kept
        # eps enters under the root, added to the mean square
        np.testing.assert_allclose(ora.rms_norm(np.array([2.0, 0.0]), np.ones(2), 2.0), np.array([1.0, 0.0]))

    def test_rotary_is_complex_multiplication(self):
        u = _rand((4, 6, 10), 4)
        pos = np.arange(6, dtype=np.float64)[None, :] * np.ones((4, 1))
        got = ora.rotary(u, pos)
        w = 10000.0 ** (-2.0 * np.arange(5) / 10)
        z = (u[..., 0::2] + 1j * u[..., 1::2]) * np.exp(1j * pos[..., None] * w)
        np.testing.assert_allclose(got[..., 0::2], z.real, atol=1e-12)
        np.testing.assert_allclose(got[..., 1::2], z.imag, atol=1e-12)
        for b, t in ((0, 0), (1, 3), (3, 5)):
            np.testing.assert_allclose(got[b, t], bf.rotary_row(u[b, t].tolist(), float(t)), atol=1e-12)

    def test_rotary_quarter_turn_and_frequency_ladder(self):
        # d = 4: pair 0 turns by pos, pair 1 by pos / 100
        e0 = np.array([1.0, 0.0, 0.0, 0.0])
        np.testing.assert_allclose(ora.rotary(e0, math.pi / 2), [0.0, 1.0, 0.0, 0.0], atol=1e-15)
        e2 = np.array([0.0, 0.0, 1.0, 0.0])
        np.testing.assert_allclose(ora.rotary(e2, 100 * math.pi / 2), [0.0, 0.0, 0.0, 1.0], atol=1e-12)
        np.testing.assert_allclose(ora.rotary(e2, math.pi / 2), [0, 0, math.cos(math.pi / 200), math.sin(math.pi / 200)], atol=1e-15)

    def test_rotary_identity_norm_and_relative_position(self):
        q, k = _rand((9, 8), 5), _rand((9, 8), 6)
        np.testing.assert_allclose(ora.rotary(q, np.zeros(9)), q, atol=0)
        pos = np.arange(9.0)
        rq, rk = ora.rotary(q, pos), ora.rotary(k, pos)
        np.testing.assert_allclose((rq ** 2).sum(-1), (q ** 2).sum(-1), rtol=1e-12)
        # scores depend on the positions only through their difference
        s0 = rq @ rk.T
        s1 = ora.rotary(q, pos + 37.0) @ ora.rotary(k, pos + 37.0).T
        np.testing.assert_allclose(s0, s1, atol=1e-10)
        assert rel_fro(s0, q @ k.T) > 0.05                      # and it does something

    def test_temporal_layer_with_both_options_vs_loops(self):
        sh = TINY
        w, x, y, c6 = _tiny_layer(3)
        w = dict(w, g_q=_rand((sh.dh,), 11) * 0.3 + 1, g_k=_rand((sh.dh,), 12) * 0.3 + 1)
        taps = {}
        out = ora.layer_fwd("temporal", x, y, None, c6, w, sh.H, sh.dh, taps, rope_temporal=True)
        plain = {}
        ora.layer_fwd("temporal", x, y, None, c6, {n: v for n, v in w.items() if n not in ("g_q", "g_k")}, sh.H, sh.dh, plain)
        # q, k of the taps = loops over the untouched projections: norm first, rotation second
        for name, g in (("q", w["g_q"]), ("k", w["g_k"])):
            for b in range(sh.B):
                for t in range(sh.T):
                    for s_ in range(sh.S):
                        for h in range(sh.H):
                            ref = bf.rotary_row(bf.rms_norm_row(plain[name][b, t, s_, h].tolist(), g.tolist(), 1e-6), float(t))
                            np.testing.assert_allclose(taps[name][b, t, s_, h], ref, atol=1e-12)
        np.testing.assert_allclose(taps["v"], plain["v"], atol=0)
        o = np.array(bf.temporal(taps["q"].tolist(), taps["k"].tolist(), taps["v"].tolist()))
        np.testing.assert_allclose(taps["o"], o, atol=1e-12)
        # cross-attention keeps its plain projections of the stream and the text
        np.testing.assert_allclose(taps["qc"].reshape(sh.B, sh.T, sh.S, -1), ora.linear(taps["x_after_attn"], w["w_cq"], w["b_cq"]), atol=1e-12)
        np.testing.assert_allclose(taps["kc"].reshape(sh.B, sh.Ly, -1), ora.linear(y, w["w_ckv"], w["b_ckv"])[..., :sh.A], atol=1e-12)
        assert rel_fro(out, ora.layer_fwd("temporal", x, y, None, c6, w, sh.H, sh.dh)) > 1e-4   # rotation matters

    def test_spatial_layer_normalises_but_never_rotates(self):
        sh = TINY
        w, x, y, c6 = _tiny_layer(4)
        wn = dict(w, g_q=_rand((sh.dh,), 13) * 0.3 + 1, g_k=_rand((sh.dh,), 14) * 0.3 + 1)
        a = ora.layer_fwd("spatial", x, y, None, c6, wn, sh.H, sh.dh, rope_temporal=True)
        b = ora.layer_fwd("spatial", x, y, None, c6, wn, sh.H, sh.dh, rope_temporal=False)
        np.testing.assert_allclose(a, b, atol=0)
        assert rel_fro(a, ora.layer_fwd("spatial", x, y, None, c6, w, sh.H, sh.dh)) > 1e-4
        # block and step hand the option down
        wb = {"spatial": wn, "temporal": wn}
        c = ora.block_fwd(x, y, None, c6, wb, sh.H, sh.dh, rope_temporal=True)
        d = ora.layer_fwd("temporal", ora.layer_fwd("spatial", x, y, None, c6, wn, sh.H, sh.dh), y, None, c6, wn, sh.H, sh.dh,
                          rope_temporal=True)
        np.testing.assert_allclose(c, d, atol=0)


class TestPinsCatchMistakes:
    """Each case plants one plausible mistake in the oracle (on the CPU) and checks that
    at least one of the pins above fails."""

    def _pins_fail(self, monkeypatch, name, wrong):
        monkeypatch.setattr(ora, name, wrong)
        failed = 0
        suites = [TestBruteForce(), TestLibraryRoutines(), TestAttentionClosedForms(), TestLayerInvariants(), TestStep(),
                  TestQkNormRotary()]
        for s in suites:
            for attr in dir(s):
                if attr.startswith("test_"):
                    try:
                        getattr(s, attr)()
                    except AssertionError:
                        failed += 1
                    except Exception:
                        failed += 1
        return failed

    def test_missing_softmax_scale(self, monkeypatch):
        good = ora.sdpa
        def wrong(q, k, v, n_valid=None, return_probs=False):
            return good(q * math.sqrt(q.shape[-1]), k, v, n_valid, return_probs)
        assert self._pins_fail(monkeypatch, "sdpa", wrong) > 0

    def test_unbiased_variance(self, monkeypatch):
        def wrong(u, eps=1e-6):
            mu = u.mean(-1, keepdims=True)
            return (u - mu) / np.sqrt(u.var(-1, ddof=1, keepdims=True) + eps)
        assert self._pins_fail(monkeypatch, "layer_norm", wrong) > 0

    def test_modulate_without_plus_one(self, monkeypatch):
        assert self._pins_fail(monkeypatch, "modulate", lambda u, sh, sc: u * sc + sh) > 0

    def test_swapped_shift_scale(self, monkeypatch):
        good = ora.split_modulation
        def wrong(table, c, D):
            m = good(table, c, D)
            m["shift_msa"], m["scale_msa"] = m["scale_msa"], m["shift_msa"]
            return m
        assert self._pins_fail(monkeypatch, "split_modulation", wrong) > 0

    def test_transposed_weight(self, monkeypatch):
        def wrong(u, W, b=None):
            out = u @ (W if W.shape[0] == W.shape[1] else W.T)
            return out if b is None else out + b
        assert self._pins_fail(monkeypatch, "linear", wrong) > 0

    def test_erf_gelu_instead_of_tanh(self, monkeypatch):
        from scipy.special import erf
        assert self._pins_fail(monkeypatch, "gelu_tanh", lambda u: 0.5 * u * (1 + erf(u / np.sqrt(2)))) > 0

    def test_sin_first_features(self, monkeypatch):
        good = ora.timestep_features
        def wrong(t):
            e = good(t)
            return np.concatenate([e[:, 128:], e[:, :128]], -1)
        assert self._pins_fail(monkeypatch, "timestep_features", wrong) > 0

    def test_spatial_temporal_swapped(self, monkeypatch):
        good_t = ora.temporal_attention
        assert self._pins_fail(monkeypatch, "spatial_attention", good_t) > 0

    def test_rotary_turning_the_other_way(self, monkeypatch):
        good = ora.rotary
        assert self._pins_fail(monkeypatch, "rotary", lambda u, pos, theta=10000.0: good(u, -np.asarray(pos, dtype=np.float64), theta)) > 0

    def test_rotary_pairing_first_half_with_second_half(self, monkeypatch):
        def wrong(u, pos, theta=10000.0):
            d = u.shape[-1]
            w = theta ** (-2.0 * np.arange(d // 2) / d)
            ang = np.asarray(pos, dtype=np.float64)[..., None] * w
            a, b = u[..., :d // 2], u[..., d // 2:]
            return np.concatenate([a * np.cos(ang) - b * np.sin(ang), b * np.cos(ang) + a * np.sin(ang)], -1)
        assert self._pins_fail(monkeypatch, "rotary", wrong) > 0

    def test_rotary_frequency_exponent_without_the_two(self, monkeypatch):
        good = ora.rotary
        assert self._pins_fail(monkeypatch, "rotary", lambda u, pos, theta=10000.0: good(u, pos, math.sqrt(theta))) > 0

    def test_rms_norm_that_centres(self, monkeypatch):
        def wrong(u, g, eps=1e-6):
            c = u - u.mean(-1, keepdims=True)
            return c / np.sqrt((c ** 2).mean(-1, keepdims=True) + eps) * g
        assert self._pins_fail(monkeypatch, "rms_norm", wrong) > 0

    def test_rms_norm_eps_outside_the_root(self, monkeypatch):
        def wrong(u, g, eps=1e-6):
            return u / (np.sqrt((u ** 2).mean(-1, keepdims=True)) + eps) * g
        assert self._pins_fail(monkeypatch, "rms_norm", wrong) > 0
