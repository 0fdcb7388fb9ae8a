"""Seeded random valid shapes through the C ABI against the CPU oracle: the linear on every output
tile with every epilogue (token counts around the tile edges, out-feature and contraction counts that
are any multiple of 8, strided operands, samples shorter than a tile), and the three attention kinds
(ragged sequence lengths, partial head groups, both head dims, masked text, the resident form).
The shapes are drawn here, in the test, from a fixed seed; the values come from the shared input
generator."""
import math
import random

import numpy as np
import pytest
import torch

import ddit_synth as syn
from helpers import assert_parity, dev_to_f64, to_dev, to_f64
from oracle import stdit_oracle as ora

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lib():
    import paper_2506_13497_amd as m
    assert torch.cuda.is_available()
    return m


def _linear_cases(seed, count):
    rng = random.Random(seed)
    out = []
    for i in range(count):
        N = rng.choice([1, 7, 63, 64, 65, 191, 192, 193, 383, 500, 1000])
        c = dict(i=i, tile=rng.randrange(-1, 7), epi=rng.randrange(3), N=N, n=8 * rng.randrange(1, 130),
                 k=8 * rng.randrange(1, 90), bias=rng.random() < 0.8)
        c["ld_u"] = c["k"] + 8 * rng.randrange(0, 3)
        c["ld_out"] = c["n"] + 8 * rng.randrange(0, 3)
        tps = rng.choice([N, max(1, N // 2), max(1, N // 3), max(1, N // 9)])
        if (N + tps - 1) // tps > 64:
            tps = N
        c.update(tps=tps, gate_row=rng.choice([-1, 2, 5]), copy=rng.random() < 0.5)
        out.append(c)
    return out


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_linear_random_shapes(lib, seed):
    for c in _linear_cases(seed, 40):
        N, n, k, epi, tile = c["N"], c["n"], c["k"], c["epi"], c["tile"]
        key = (900 + seed, c["i"])
        ubuf = syn.normal_bits(key + (1,), (N, c["ld_u"]), 0.7)
        W = syn.normal_bits(key + (2,), (n, k), 1.0 / math.sqrt(k))
        b = syn.normal_bits(key + (3,), (n,), 0.3) if c["bias"] else None
        lin = ora.linear(to_f64(ubuf)[:, :k], to_f64(W), None if b is None else to_f64(b))
        what = "seed %d case %s" % (seed, c)
        if epi < 2:
            out = torch.full((N, c["ld_out"]), 3.0, dtype=torch.bfloat16, device="cuda")
            lib.ddit_linear_fwd_tile(tile, epi, to_dev(ubuf), c["ld_u"], to_dev(W), None if b is None else to_dev(b), N, n, k, out,
                                     c["ld_out"])
            torch.cuda.synchronize()
            assert_parity(dev_to_f64(out[:, :n]), lin if epi == 0 else ora.gelu_tanh(lin), what)
            assert torch.all(out[:, n:] == 3.0), "wrote past its columns: " + what
        else:
            tps, gr = c["tps"], c["gate_row"]
            B = (N + tps - 1) // tps
            g = np.random.default_rng(seed * 1000 + c["i"])
            resid = g.standard_normal((N, n)).astype(np.float32)
            tab = g.standard_normal((6, n)).astype(np.float32)
            c6 = g.standard_normal((B, 6 * n)).astype(np.float32)
            dres = to_dev(resid)
            out = torch.full((N, n), 3.0, dtype=torch.bfloat16, device="cuda") if c["copy"] else None
            lib.ddit_linear_fwd_tile(tile, 2, to_dev(ubuf), c["ld_u"], to_dev(W), None if b is None else to_dev(b), N, n, k, out, n,
                                     resid=dres, ada_table=to_dev(tab), c6=to_dev(c6), gate_row=gr, tokens_per_sample=tps)
            torch.cuda.synchronize()
            ref = resid.astype(np.float64)
            for r in range(N):
                gate = 1.0 if gr < 0 else (tab[gr] + c6[r // tps].reshape(6, n)[gr]).astype(np.float64)
                ref[r] += gate * lin[r]
            # the branch that was added, not the O(1) stream it was added to, carries the comparison
            assert_parity(dev_to_f64(dres) - resid.astype(np.float64), ref - resid.astype(np.float64), what, elem=2e-2, fro=5e-3)
            if out is not None:
                assert torch.equal(out, dres.to(torch.bfloat16)), "bf16 copy differs: " + what


def _attn_cases(seed, count):
    rng = random.Random(seed)
    out = []
    for i in range(count):
        kind = rng.choice(["spatial", "temporal", "cross", "cross"])
        c = dict(i=i, kind=kind, dh=rng.choice([64, 72]))
        if kind == "cross":
            c.update(B=rng.randrange(1, 4), H=rng.randrange(1, 6), T=1, S=rng.randrange(1, 700), Ly=rng.randrange(1, 400))
        else:
            c.update(B=rng.randrange(1, 3), H=rng.randrange(1, 6), T=rng.randrange(1, 45), S=rng.randrange(1, 200), Ly=8)
        c["valid"] = [rng.randrange(1, c["Ly"] + 1) for _ in range(c["B"])] if kind == "cross" else None
        out.append(c)
    # two cases that take the resident form (256 units: one workgroup each, four or five query tiles)
    for i, (dh, Lq, Ly) in enumerate([(72, 769 + rng.randrange(200), rng.randrange(200, 321)), (64, 1024 + rng.randrange(200), rng.randrange(1, 200))]):
        out.append(dict(i=count + i, kind="cross", dh=dh, B=64, H=4, T=1, S=Lq, Ly=Ly, valid=[rng.randrange(1, Ly + 1) for _ in range(64)]))
    return out


@pytest.mark.parametrize("seed", [0, 1])
def test_attention_random_shapes(lib, seed):
    for c in _attn_cases(seed, 14):
        kind, B, T, S, H, dh, Ly = c["kind"], c["B"], c["T"], c["S"], c["H"], c["dh"], c["Ly"]
        A = H * dh
        sh = syn.Shape(B, T, 1, S, A, H, dh, 64, Ly, 1)
        d = syn.make_attn_inputs(kind, sh, 300 + 10 * seed + c["i"], Lq=S if kind == "cross" else None)
        q, k, v = (to_f64(d[n]) for n in "qkv")
        if kind == "cross":
            ref, _ = ora.cross_attention(q, k, v, c["valid"])
            kid = lib.DDIT_ATTN_CROSS
        else:
            ref, _ = (ora.spatial_attention if kind == "spatial" else ora.temporal_attention)(q, k, v)
            kid = lib.DDIT_ATTN_SPATIAL if kind == "spatial" else lib.DDIT_ATTN_TEMPORAL
        shape = lib.make_shape(B, T, 1, S, A, H, dh, 64, Ly, 1)
        o = torch.full(q.shape, float("nan"), dtype=torch.bfloat16, device="cuda")
        lib.ddit_attn_fwd(kid, shape, to_dev(d["q"]), to_dev(d["k"]), to_dev(d["v"]), A, A, c["valid"], o, A)
        torch.cuda.synchronize()
        assert_parity(dev_to_f64(o), ref, "seed %d case %s" % (seed, {n: c[n] for n in c if n != "valid"}))


@pytest.mark.parametrize("seed", [0, 1])
def test_layernorm_and_qk_treatment_random_shapes(lib, seed):
    rng = random.Random(50 + seed)
    for i in range(16):          # modulated LayerNorm: any hidden size that is a multiple of 8, samples of any length
        N, D = rng.choice([1, 3, 4, 5, 17, 64, 255, 1000]), 8 * rng.randrange(1, 513)
        tps = rng.choice([N, max(1, N // 2), max(1, N // 7)])
        B = (N + tps - 1) // tps
        g = np.random.default_rng(seed * 100 + i)
        x = (g.standard_normal((N, D)) * 1.5 + 0.3).astype(np.float32)
        tab = (g.standard_normal((6, D)) * 0.5).astype(np.float32)
        c6 = (g.standard_normal((B, 6 * D)) * 0.5).astype(np.float32)
        which = rng.randrange(2)
        out = torch.full((N, D), float("nan"), dtype=torch.bfloat16, device="cuda")
        lib.ddit_modulated_layernorm_fwd(to_dev(x), to_dev(tab), to_dev(c6), which, tps, 1e-6, out)
        torch.cuda.synchronize()
        xn = ora.layer_norm(x.astype(np.float64))
        ref = np.empty((N, D))
        sfx = "msa" if which == 0 else "mlp"
        for r in range(N):
            m = ora.split_modulation(tab.astype(np.float64), c6[r // tps].astype(np.float64), D)
            ref[r] = ora.modulate(xn[r], m["shift_" + sfx], m["scale_" + sfx])
        assert_parity(dev_to_f64(out), ref, "LayerNorm N=%d D=%d tps=%d which=%d" % (N, D, tps, which))
    for i in range(16):          # q | k treatment in place: any head count, both head dims, padded rows
        N, H, dh = rng.choice([1, 2, 9, 63, 64, 65, 577, 1000]), rng.randrange(1, 17), rng.choice([64, 72])
        S, T = rng.randrange(1, 40), rng.randrange(1, 50)
        A = H * dh
        ld = 3 * A + 8 * rng.randrange(0, 3)
        norm, rope = rng.choice([(True, False), (False, True), (True, True)])
        buf = syn.normal_bits((70 + seed, i), (N, ld), 1.5)
        gq = syn.f32_to_bf16_bits((1 + 0.2 * np.random.default_rng(i).standard_normal(dh)).astype(np.float32))
        gk = syn.f32_to_bf16_bits((1 + 0.2 * np.random.default_rng(100 + i).standard_normal(dh)).astype(np.float32))
        d = to_dev(buf)
        tab = torch.empty(T * dh, dtype=torch.float32, device="cuda") if rope else None
        lib.ddit_qk_norm_rope_fwd(d, ld, N, H, dh, to_dev(gq) if norm else None, to_dev(gk) if norm else None, 1e-6, S, T, tab)
        torch.cuda.synchronize()
        got, x = dev_to_f64(d), to_f64(buf)
        frame = ((np.arange(N) // S) % T).astype(np.float64)[:, None]
        for j, gg in enumerate((gq, gk)):
            u = x[:, j * A:(j + 1) * A].reshape(N, H, dh)
            if norm:
                u = ora.rms_norm(u, to_f64(gg), 1e-6)
            if rope:
                u = ora.rotary(u, frame)
            assert_parity(got[:, j * A:(j + 1) * A], u.reshape(N, A), "q/k treatment N=%d H=%d dh=%d S=%d T=%d" % (N, H, dh, S, T))
        assert np.array_equal(got[:, 2 * A:], x[:, 2 * A:]), "columns past q | k were touched"
