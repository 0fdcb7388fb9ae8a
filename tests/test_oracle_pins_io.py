"""Pins of the latent-in / latent-out oracle and of the sampling loop against things other than
themselves: routines of other packages (torch convolution, layer norm and GELU in fp64; einops
pixel rearrangement), brute-force loops, closed forms of the position code, the exact solution of
a linear flow under explicit Euler, guidance at s = 0 and s = 1, and composition."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F
from einops import rearrange

import ddit_synth as syn
from helpers import dict_f64
from oracle import latent_io_oracle as lio
from oracle import stdit_oracle as ora

TINY = syn.Shape(B=2, T=3, Hp=2, Wp=3, D=16, H=2, dh=4, M=24, Ly=5, n_blocks=1)
C, C_TEXT, C_OUT = 3, 10, 3


def _rand(shape, seed, scale=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * scale


def _io(sh=TINY):
    return dict_f64(syn.make_io_weights(sh, 11, C, C_TEXT, C_OUT, w_std=0.3, patch_std=0.3, final_std=0.3))


class TestPatches:
    def test_patchify_vs_loops_and_einops(self):
        z = _rand((2, C, 3, 4, 6), 0)
        p = lio.patchify(z)
        assert p.shape == (2, 3, 6, 4 * C)
        for b, t, i, j, c, di, dj in [(0, 0, 0, 0, 0, 0, 0), (1, 2, 1, 2, 2, 1, 0), (0, 1, 1, 0, 1, 0, 1), (1, 0, 0, 1, 2, 1, 1)]:
            assert p[b, t, i * 3 + j, (c * 2 + di) * 2 + dj] == z[b, c, t, 2 * i + di, 2 * j + dj]
        np.testing.assert_array_equal(p, rearrange(z, "b c t (h p) (w q) -> b t (h w) (c p q)", p=2, q=2))

    def test_unpatchify_vs_einops_and_round_trip(self):
        tok = _rand((2, 3, 6, 4 * C_OUT), 1)
        z = lio.unpatchify(tok, 2, 3, C_OUT)
        np.testing.assert_array_equal(z, rearrange(tok, "b t (h w) (p q c) -> b c t (h p) (w q)", h=2, w=3, p=2, q=2))
        # patchify orders (c, di, dj), the head orders (di, dj, c): with that reordering the two are inverse
        zz = _rand((2, C, 3, 4, 6), 2)
        p = lio.patchify(zz).reshape(2, 3, 6, C, 2, 2)
        back = lio.unpatchify(np.transpose(p, (0, 1, 2, 4, 5, 3)).reshape(2, 3, 6, 4 * C), 2, 3, C)
        np.testing.assert_array_equal(back, zz)

    def test_odd_latent_rejected(self):
        with pytest.raises(ValueError):
            lio.patchify(np.zeros((1, 2, 1, 3, 4)))


class TestPositionCode:
    def test_origin_and_norm(self):
        D = 24
        pc = lio.position_code(3, 5, D)
        assert pc.shape == (15, D)
        Q = D // 4
        np.testing.assert_allclose(pc[0], np.concatenate([np.zeros(Q), np.ones(Q), np.zeros(Q), np.ones(Q)]), atol=0)
        np.testing.assert_allclose((pc ** 2).sum(axis=1), D / 2, rtol=1e-13)   # sin^2 + cos^2 per frequency, two axes

    def test_first_frequency_and_axes(self):
        D, Hp, Wp = 16, 4, 3
        pc = lio.position_code(Hp, Wp, D).reshape(Hp, Wp, D)
        Q = D // 4
        # frequency 0 is 1 rad per step; the last is 10000^(-(Q-1)/Q)
        assert pc[2, 1, 0] == pytest.approx(math.sin(1.0), rel=1e-14)
        assert pc[2, 1, 2 * Q] == pytest.approx(math.sin(2.0), rel=1e-14)
        assert pc[3, 2, 2 * Q - 1] == pytest.approx(math.cos(2.0 * 10000.0 ** (-(Q - 1) / Q)), rel=1e-13)
        # the column half does not depend on the row and vice versa
        np.testing.assert_array_equal(pc[0, :, :2 * Q], pc[3, :, :2 * Q])
        np.testing.assert_array_equal(pc[:, 0, 2 * Q:], pc[:, 2, 2 * Q:])

    def test_inner_product_depends_on_offset_only(self):
        pc = lio.position_code(5, 6, 32).reshape(5, 6, 32)
        a = pc[0, 1] @ pc[2, 4]
        b = pc[2, 2] @ pc[4, 5]
        assert a == pytest.approx(b, rel=1e-12)


class TestEmbedders:
    def test_patch_embedding_is_a_strided_convolution(self):
        sh = TINY
        w = _io()
        z = _rand((sh.B, C, sh.T, 2 * sh.Hp, 2 * sh.Wp), 3)
        x = lio.embed_latent(z, w["w_patch"], w["b_patch"], sh.D)
        conv = F.conv3d(torch.from_numpy(z), torch.from_numpy(w["w_patch"].reshape(sh.D, C, 1, 2, 2)),
                        torch.from_numpy(w["b_patch"]), stride=(1, 2, 2))          # [B,D,T,Hp,Wp]
        ref = conv.permute(0, 2, 3, 4, 1).reshape(sh.B, sh.T, sh.S, sh.D).numpy() + lio.position_code(sh.Hp, sh.Wp, sh.D)
        np.testing.assert_allclose(x, ref, rtol=1e-12, atol=1e-12)

    def test_caption_embedder_vs_torch(self):
        w = _io()
        c = _rand((2, 5, C_TEXT), 4)
        y = lio.embed_caption(c, w["w_y1"], w["b_y1"], w["w_y2"], w["b_y2"])
        t = lambda a: torch.from_numpy(a)
        ref = F.linear(F.gelu(F.linear(t(c), t(w["w_y1"]), t(w["b_y1"])), approximate="tanh"), t(w["w_y2"]), t(w["b_y2"]))
        np.testing.assert_allclose(y, ref.numpy(), rtol=1e-12, atol=1e-12)

    def test_output_head_vs_torch(self):
        sh = TINY
        w = _io()
        x = _rand((sh.B, sh.T, sh.S, sh.D), 5, 2.0) + 0.7
        temb = _rand((sh.B, sh.D), 6, 0.5)
        out = lio.output_head(x, temb, w["final_table"], w["w_final"], w["b_final"], sh.Hp, sh.Wp, C_OUT)
        t = lambda a: torch.from_numpy(a)
        ln = F.layer_norm(t(x), (sh.D,), eps=1e-6)
        shift = t(w["final_table"][0] + temb)[:, None, None, :]
        scale = t(w["final_table"][1] + temb)[:, None, None, :]
        tok = F.linear(ln * (1 + scale) + shift, t(w["w_final"]), t(w["b_final"])).numpy()
        ref = rearrange(tok, "b t (h w) (p q c) -> b c t (h p) (w q)", h=sh.Hp, w=sh.Wp, p=2, q=2)
        np.testing.assert_allclose(out, ref, rtol=1e-11, atol=1e-11)

    def test_output_head_selects_normalised_features(self):
        """With zero modulation and a selection matrix as the Linear, the latent holds LayerNorm values."""
        sh = TINY
        x = _rand((1, 1, sh.S, sh.D), 7)
        sel = np.zeros((4 * C_OUT, sh.D))
        for r in range(4 * C_OUT):
            sel[r, r] = 1.0
        out = lio.output_head(x, np.zeros((1, sh.D)), np.zeros((2, sh.D)), sel, np.zeros(4 * C_OUT), sh.Hp, sh.Wp, C_OUT)
        ln = (x - x.mean(-1, keepdims=True)) / np.sqrt(x.var(-1, keepdims=True) + 1e-6)
        # token s = 1*Wp + 2 -> (i, j) = (1, 2); feature r = (di*2 + dj)*C_out + c
        s, di, dj, c = 1 * sh.Wp + 2, 1, 0, 2
        assert out[0, c, 0, 2 * 1 + di, 2 * 2 + dj] == pytest.approx(ln[0, 0, s, (di * 2 + dj) * C_OUT + c], rel=1e-12)


class TestModel:
    def _setup(self, n_blocks=1):
        sh = syn.small_variant(TINY, n_blocks=n_blocks)
        io_w = _io(sh)
        sw = dict_f64(syn.make_step_weights(sh, 12, w_std=0.2))
        blocks = [dict_f64(syn.make_block_weights(sh, 12, i, w_std=0.2, table_std=0.3)) for i in range(n_blocks)]
        z = _rand((sh.B, C, sh.T, 2 * sh.Hp, 2 * sh.Wp), 8)
        c = _rand((sh.B, sh.Ly, C_TEXT), 9)
        return sh, io_w, sw, blocks, z, c

    def test_without_blocks_is_embed_then_head(self):
        sh, io_w, sw, _, z, c = self._setup(0)
        t = np.array([300.0, 700.0])
        out = lio.eps_theta(z, c, None, t, io_w, sw, [], sh.H, sh.dh)
        x = lio.embed_latent(z, io_w["w_patch"], io_w["b_patch"], sh.D)
        ref = lio.output_head(x, ora.timestep_embedding(t, sw), io_w["final_table"], io_w["w_final"], io_w["b_final"],
                              sh.Hp, sh.Wp, C_OUT)
        np.testing.assert_allclose(out, ref, rtol=1e-13)

    def test_samples_are_independent_and_padding_is_ignored(self):
        sh, io_w, sw, blocks, z, c = self._setup(1)
        t = np.array([300.0, 700.0])
        vl = np.array([3, 5])
        out = lio.eps_theta(z, c, vl, t, io_w, sw, blocks, sh.H, sh.dh)
        c2 = c.copy()
        c2[0, 3:] = 99.0                        # padded text of sample 0
        z2 = z.copy()
        z2[1] += 1.0                            # another latent for sample 1
        out2 = lio.eps_theta(z2, c2, vl, t, io_w, sw, blocks, sh.H, sh.dh)
        np.testing.assert_allclose(out2[0], out[0], rtol=1e-12, atol=1e-12)
        assert np.abs(out2[1] - out[1]).max() > 1e-3

    def test_timestep_reaches_the_head(self):
        sh, io_w, sw, blocks, z, c = self._setup(1)
        a = lio.eps_theta(z, c, None, np.array([100.0, 100.0]), io_w, sw, blocks, sh.H, sh.dh)
        b = lio.eps_theta(z, c, None, np.array([100.0, 900.0]), io_w, sw, blocks, sh.H, sh.dh)
        np.testing.assert_allclose(a[0], b[0], rtol=1e-12, atol=1e-12)
        assert np.abs(a[1] - b[1]).max() > 1e-4


class TestSolver:
    def test_schedule(self):
        ts = lio.step_schedule(30)
        assert ts[0] == 1000.0 and ts[-1] == 0.0 and len(ts) == 31
        np.testing.assert_allclose(np.diff(ts), -1000.0 / 30, rtol=1e-12)

    def test_constant_prediction(self):
        z0 = _rand((2, 3, 2, 4, 4), 10)
        v = _rand((2, 3, 2, 4, 4), 11)
        out = lio.sample(z0, lambda z, t: v, 7)
        np.testing.assert_allclose(out, z0 - v, rtol=1e-12, atol=1e-12)     # the step variable runs from 1000 to 0

    def test_linear_flow_closed_form(self):
        """eps = a z under explicit Euler with n equal steps of -1/n: z_n = z_0 (1 - a/n)^n."""
        z0 = _rand((1, 2, 1, 2, 2), 12)
        a, n = 0.8, 13
        out = lio.sample(z0, lambda z, t: a * z, n)
        np.testing.assert_allclose(out, z0 * (1.0 - a / n) ** n, rtol=1e-12)

    def test_per_sample_times_and_resume(self):
        z = _rand((2, 1, 1, 2, 2), 13)
        e = _rand((2, 1, 1, 2, 2), 14)
        out = lio.solver_step(z, e, np.array([800.0, 500.0]), np.array([700.0, 100.0]))
        np.testing.assert_allclose(out[0], z[0] - 0.1 * e[0], rtol=1e-13)
        np.testing.assert_allclose(out[1], z[1] - 0.4 * e[1], rtol=1e-13)
        model = lambda zz, t: np.sin(zz) * (t / 1000.0).reshape(-1, 1, 1, 1, 1)
        full = lio.sample(z, model, 9)
        part = lio.sample(lio.sample(z, model, 9, 0, 4), model, 9, 4, 9)
        np.testing.assert_array_equal(full, part)

    def test_guidance(self):
        ec, eu = _rand((2, 3), 15), _rand((2, 3), 16)
        np.testing.assert_array_equal(lio.guide(ec, eu, 1.0), eu + (ec - eu))
        np.testing.assert_allclose(lio.guide(ec, eu, 1.0), ec, rtol=1e-14, atol=1e-15)
        np.testing.assert_array_equal(lio.guide(ec, eu, 0.0), eu)
        np.testing.assert_allclose(lio.guide(ec, eu, 7.5), 7.5 * ec - 6.5 * eu, rtol=1e-13, atol=1e-13)


class TestPlantedMistakes:
    """Each plausible slip in the oracle must trip at least one pin above."""

    def test_swapped_patch_axes_is_caught(self):
        z = _rand((1, C, 1, 4, 6), 20)
        wrong = rearrange(z, "b c t (h p) (w q) -> b t (h w) (c q p)", p=2, q=2)
        assert np.abs(wrong - lio.patchify(z)).max() > 0.1

    def test_wrong_solver_sign_is_caught(self):
        z0, v = _rand((1, 1, 1, 2, 2), 21), _rand((1, 1, 1, 2, 2), 22)
        wrong = z0 + v
        assert np.abs(wrong - lio.sample(z0, lambda z, t: v, 5)).max() > 0.1

    def test_unbiased_variance_in_head_is_caught(self):
        sh = TINY
        x = _rand((1, 1, sh.S, sh.D), 23)
        sel = np.eye(4 * C_OUT, sh.D)
        out = lio.output_head(x, np.zeros((1, sh.D)), np.zeros((2, sh.D)), sel, np.zeros(4 * C_OUT), sh.Hp, sh.Wp, C_OUT)
        wrong = (x - x.mean(-1, keepdims=True)) / np.sqrt(x.var(-1, ddof=1, keepdims=True) + 1e-6)
        assert abs(out[0, 0, 0, 0, 0] - wrong[0, 0, 0, 0]) > 1e-3 * abs(out[0, 0, 0, 0, 0])
