"""CPU oracle of the STDiT denoising step  eps_theta(x_t, t, c)  (paper eq. 1).

THIS IS TEST INFRASTRUCTURE, not a product path: only the tests, the smoke check and
the benchmark's cpu_baseline leg may import it.  It shares no code with the HIP
library and imports nothing from it.

What it computes.  The paper's section 2.2 says the DiT denoises with three kinds
of Transformer blocks: *spatial* blocks relate tokens that share a temporal index,
*temporal* blocks relate tokens across time, and *cross-attention* brings in the
conditioning (text) input.  Table 1 names the model (STDiT-v3, 1.1 B parameters) and
the related-work section says attention is computed by Flash Attention, i.e. it is
exact softmax attention.  Every kernel on the HIP path (tiled attention with online
softmax, GEMMs with fused epilogues) reaches the plain mathematical result up to
rounding order, so this oracle is the plain definition written out in fp64 with full
score matrices and no intermediate rounding, blocking or fusion.

Where the paper is silent (it never writes the block down), the readings are:
  * a *layer* = self-attention (spatial or temporal) -> cross-attention -> MLP, each
    added to the residual stream; a *block* = spatial layer then temporal layer;
    "28 blocks" = 56 layers (this structure counts 1.19 B parameters, matching
    Table 1's 1.1 B; the alternative with one cross-attention and one MLP per block
    counts 0.75 B);
  * adaLN-single: one conditioning vector c6 = W_ada SiLU(temb) + b_ada per sample,
    shared by all layers, plus a learned per-layer table [6,D]; their sum splits into
    (shift_msa, scale_msa, gate_msa, shift_mlp, scale_mlp, gate_mlp);
    modulate(u) = u (1 + scale) + shift;
  * LayerNorm has no affine parameters, eps 1e-6, biased variance;
  * cross-attention reads the residual stream itself (no norm, no modulation) and its
    output is added without a gate;
  * GELU is the tanh form; softmax scale is 1/sqrt(d_h);
  * text padding is a prefix mask: keys j < valid_len[b] take part, the rest get
    weight exactly 0;
  * the timestep feature is [cos(t f_i), sin(t f_i)], f_i = 10000^(-i/128), i < 128,
    followed by Linear(256->D), SiLU, Linear(D->D);
  * the attention width A = H d_h may be smaller than D (one rank's share of a
    head-split run): W_qkv is [3A, D], W_o is [D, A];
  * two options the released model of Table 1 has and the paper does not mention, both
    off unless asked for: (i) per-head RMS normalisation of the self-attention queries
    and keys, u / sqrt(mean(u^2) + eps) * g over the d_h elements of a head with learned
    g_q, g_k in R^{d_h} per layer (eps = the LayerNorm's), not applied in
    cross-attention; (ii) rotary position embedding of the TEMPORAL self-attention's
    queries and keys (after the normalisation), position = frame index, element pairs
    (2i, 2i+1) rotated by the angle  t * 10000^(-2i/d_h).

Tensors: x [B,T,S,D] with token index ((b T + t) S + s); y [B,Ly,D]; weights [out,in]
so that linear(u) = u W^T + b.  All arguments and results are float64 numpy arrays.

Pins (tests/test_oracle_pins.py): brute-force loop attention on tiny inputs, library
routines of another package for attention / LayerNorm / GELU / SiLU, closed forms
(uniform keys, one dominant key, T = 1, zero gates), invariances (key shift, frame
permutation, locality per axis, mask independence, batch independence), composition,
and the parameter count against Table 1.  The paper prints no activation value, so
absolute values are pinned only by those.  The two options: another package's RMS norm,
unit mean square and scale invariance; rotation written as complex multiplication, the
relative-position property of the scores, norm preservation, identity at position 0,
and a brute-force temporal layer.
"""
from __future__ import annotations

import math

import numpy as np

LN_EPS = 1e-6
T_FREQ = 256
ADA_NAMES = ("shift_msa", "scale_msa", "gate_msa", "shift_mlp", "scale_mlp", "gate_mlp")


# ---------------------------------------------------------------------------
# elementary pieces
# ---------------------------------------------------------------------------
def linear(u, W, b=None):
    """u W^T + b over the last axis; W is [out, in]."""
    out = u @ W.T
    if b is not None:
        out = out + b
    return out


def layer_norm(u, eps=LN_EPS):
    """(u - mean) / sqrt(var + eps) over the last axis, biased variance, no affine."""
    mu = u.mean(axis=-1, keepdims=True)
    var = ((u - mu) ** 2).mean(axis=-1, keepdims=True)
    return (u - mu) / np.sqrt(var + eps)


def modulate(u, shift, scale):
    return u * (1.0 + scale) + shift


def gelu_tanh(u):
    return 0.5 * u * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (u + 0.044715 * u ** 3)))


def silu(u):
    return u / (1.0 + np.exp(-u))


def rms_norm(u, g, eps=LN_EPS):
    """u / sqrt(mean(u^2) + eps) * g over the last axis."""
    return u / np.sqrt((u ** 2).mean(axis=-1, keepdims=True) + eps) * g


def rotary(u, pos, theta=10000.0):
    """Rotary position embedding over the last axis (even length d): the pair
    (u[2i], u[2i+1]) is rotated by the angle pos * theta^(-2i/d).
    pos: array broadcastable to u.shape[:-1]."""
    d = u.shape[-1]
    if d % 2:
        raise ValueError("rotary embedding needs an even width")
    w = theta ** (-2.0 * np.arange(d // 2, dtype=np.float64) / d)
    ang = np.asarray(pos, dtype=np.float64)[..., None] * w
    c, s = np.cos(ang), np.sin(ang)
    a, b = u[..., 0::2], u[..., 1::2]
    out = np.empty(np.broadcast_shapes(u.shape, c.shape[:-1] + (d,)), dtype=np.float64)
    out[..., 0::2] = a * c - b * s
    out[..., 1::2] = b * c + a * s
    return out


def softmax_rows(s):
    """Softmax over the last axis; -inf entries get weight exactly 0."""
    m = s.max(axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / e.sum(axis=-1, keepdims=True)


def sdpa(q, k, v, n_valid=None, return_probs=False):
    """softmax(q k^T / sqrt(d_h)) v over the last two axes.

    q [..., Lq, dh], k and v [..., Lk, dh].  If n_valid is given, key columns
    j >= n_valid are excluded (score -inf).  Also returns the log-sum-exp of the
    scaled scores per query row."""
    dh = q.shape[-1]
    s = (q @ np.swapaxes(k, -1, -2)) / math.sqrt(float(dh))
    if n_valid is not None:
        s = s.copy()
        s[..., int(n_valid):] = -np.inf
    p = softmax_rows(s)
    m = s.max(axis=-1)
    lse = m + np.log(np.exp(s - m[..., None]).sum(axis=-1))
    o = p @ v
    if return_probs:
        return o, lse, p
    return o, lse


# ---------------------------------------------------------------------------
# the three attention kinds (section 2.2)
# ---------------------------------------------------------------------------
def spatial_attention(q, k, v):
    """q,k,v [B,T,S,H,dh]: for every (b,t,h) attend over the S tokens of frame t.
    Returns o [B,T,S,H,dh] and lse [B,T,S,H]."""
    B, T, S, H, dh = q.shape
    o = np.empty_like(q)
    lse = np.empty((B, T, S, H))
    for b in range(B):
        for t in range(T):
            # [H,S,dh] slices of this frame
            qq, kk, vv = (np.transpose(a[b, t], (1, 0, 2)) for a in (q, k, v))
            oo, ll = sdpa(qq, kk, vv)
            o[b, t] = np.transpose(oo, (1, 0, 2))
            lse[b, t] = ll.T
    return o, lse


def temporal_attention(q, k, v):
    """q,k,v [B,T,S,H,dh]: for every (b,s,h) attend over the T frames at location s."""
    B, T, S, H, dh = q.shape
    o = np.empty_like(q)
    lse = np.empty((B, T, S, H))
    for b in range(B):
        # [S,H,T,dh]
        qq, kk, vv = (np.transpose(a[b], (1, 2, 0, 3)) for a in (q, k, v))
        oo, ll = sdpa(qq, kk, vv)
        o[b] = np.transpose(oo, (2, 0, 1, 3))
        lse[b] = np.transpose(ll, (2, 0, 1))
    return o, lse


def cross_attention(q, k, v, valid_len=None):
    """q [B,L,H,dh], k,v [B,Ly,H,dh]; keys j >= valid_len[b] are masked out.
    Returns o [B,L,H,dh], lse [B,L,H]."""
    B, L, H, dh = q.shape
    o = np.empty_like(q)
    lse = np.empty((B, L, H))
    for b in range(B):
        nv = None if valid_len is None else int(valid_len[b])
        if nv is not None and not (1 <= nv <= k.shape[1]):
            raise ValueError("valid_len must be in [1, Ly]")
        qq, kk, vv = (np.transpose(a[b], (1, 0, 2)) for a in (q, k, v))
        oo, ll = sdpa(qq, kk, vv, n_valid=nv)
        o[b] = np.transpose(oo, (1, 0, 2))
        lse[b] = ll.T
    return o, lse


# ---------------------------------------------------------------------------
# layer, block, step
# ---------------------------------------------------------------------------
def split_modulation(table, c6_b, D):
    """(table [6,D] + c6_b [6D]) -> dict of six [D] vectors."""
    m = table + c6_b.reshape(6, D)
    return {n: m[i] for i, n in enumerate(ADA_NAMES)}


def layer_fwd(kind, x, y, valid_len, c6, w, H, dh, taps=None, rope_temporal=False):
    """One layer of kind 'spatial' or 'temporal'.  If w holds 'g_q' and 'g_k' ([dh]) the
    self-attention's q and k are RMS-normalised per head; with rope_temporal the temporal
    layer's q and k get the rotary embedding of their frame index.

    x [B,T,S,D], y [B,Ly,D], valid_len [B] or None, c6 [B,6D], w: dict of fp64 arrays
    (w_qkv,b_qkv,w_o,b_o,w_cq,b_cq,w_ckv,b_ckv,w_co,b_co,w_fc1,b_fc1,w_fc2,b_fc2,
    ada_table).  Returns the new x.  If taps is a dict it receives every intermediate."""
    B, T, S, D = x.shape
    A = H * dh
    Ly = y.shape[1]
    x = x.copy()
    tp = {} if taps is None else taps
    mods = [split_modulation(w["ada_table"], c6[b], D) for b in range(B)]

    def per_sample(name):
        return np.stack([mods[b][name] for b in range(B)])[:, None, None, :]  # [B,1,1,D]

    # --- self-attention branch
    xh = modulate(layer_norm(x), per_sample("shift_msa"), per_sample("scale_msa"))
    qkv = linear(xh, w["w_qkv"], w["b_qkv"])                      # [B,T,S,3A]
    q, k, v = (qkv[..., i * A:(i + 1) * A].reshape(B, T, S, H, dh) for i in range(3))
    if "g_q" in w:
        q, k = rms_norm(q, w["g_q"]), rms_norm(k, w["g_k"])
    if rope_temporal and kind == "temporal":
        frame = np.arange(T, dtype=np.float64)[None, :, None, None]          # [1,T,1,1]
        q, k = rotary(q, frame), rotary(k, frame)
    if kind == "spatial":
        o, lse = spatial_attention(q, k, v)
    elif kind == "temporal":
        o, lse = temporal_attention(q, k, v)
    else:
        raise ValueError(kind)
    attn_out = linear(o.reshape(B, T, S, A), w["w_o"], w["b_o"])
    x = x + per_sample("gate_msa") * attn_out
    tp.update(xh_msa=xh, q=q, k=k, v=v, o=o, lse=lse, attn_branch=attn_out, x_after_attn=x.copy())

    # --- cross-attention branch: reads the stream itself, ungated
    qc = linear(x, w["w_cq"], w["b_cq"]).reshape(B, T * S, H, dh)
    kvc = linear(y, w["w_ckv"], w["b_ckv"])                        # [B,Ly,2A]
    kc = kvc[..., :A].reshape(B, Ly, H, dh)
    vc = kvc[..., A:].reshape(B, Ly, H, dh)
    oc, lse_c = cross_attention(qc, kc, vc, valid_len)
    cross_out = linear(oc.reshape(B, T, S, A), w["w_co"], w["b_co"])
    x = x + cross_out
    tp.update(qc=qc, kc=kc, vc=vc, oc=oc, cross_branch=cross_out, x_after_cross=x.copy())

    # --- MLP branch
    xh2 = modulate(layer_norm(x), per_sample("shift_mlp"), per_sample("scale_mlp"))
    h = gelu_tanh(linear(xh2, w["w_fc1"], w["b_fc1"]))
    mlp_out = linear(h, w["w_fc2"], w["b_fc2"])
    x = x + per_sample("gate_mlp") * mlp_out
    tp.update(xh_mlp=xh2, h=h, mlp_branch=mlp_out)
    return x


def block_fwd(x, y, valid_len, c6, wblock, H, dh, taps=None, rope_temporal=False):
    """A block = spatial layer followed by temporal layer.  wblock = {'spatial':..,'temporal':..}."""
    ts = None if taps is None else taps.setdefault("spatial", {})
    tt = None if taps is None else taps.setdefault("temporal", {})
    x = layer_fwd("spatial", x, y, valid_len, c6, wblock["spatial"], H, dh, ts, rope_temporal=rope_temporal)
    x = layer_fwd("temporal", x, y, valid_len, c6, wblock["temporal"], H, dh, tt, rope_temporal=rope_temporal)
    return x


def timestep_features(t):
    """[cos(t f_i) for i<128] followed by [sin(t f_i)], f_i = 10000^(-i/128).  t [B] -> [B,256]."""
    half = T_FREQ // 2
    f = np.exp(-np.log(10000.0) * np.arange(half, dtype=np.float64) / half)
    arg = np.asarray(t, dtype=np.float64)[:, None] * f[None, :]
    return np.concatenate([np.cos(arg), np.sin(arg)], axis=-1)


def timestep_embedding(t, sw):
    """temb = W_t2 SiLU(W_t1 e + b_t1) + b_t2, e = timestep_features(t)."""
    return linear(silu(linear(timestep_features(t), sw["w_t1"], sw["b_t1"])), sw["w_t2"], sw["b_t2"])


def conditioning(temb, sw):
    """c6 = W_ada SiLU(temb) + b_ada : [B,D] -> [B,6D]."""
    return linear(silu(temb), sw["w_ada"], sw["b_ada"])


def denoise_step(x, y, valid_len, t, sw, blocks, H, dh, temb=None, rope_temporal=False):
    """One denoising step in token space: conditioning from the timestep (or from a given
    temb [B,D]), then the blocks in order.  blocks: list of {'spatial':..,'temporal':..}."""
    if temb is None:
        temb = timestep_embedding(t, sw)
    c6 = conditioning(temb, sw)
    for wb in blocks:
        x = block_fwd(x, y, valid_len, c6, wb, H, dh, rope_temporal=rope_temporal)
    return x


def parameter_count(D, A, M, n_blocks, t_freq=T_FREQ):
    """Closed-form number of parameters of the structure above (for the Table 1 pin)."""
    per_layer = (3 * A * D + 3 * A) + (D * A + D) + (A * D + A) + (2 * A * D + 2 * A) \
        + (D * A + D) + (M * D + M) + (D * M + D) + 6 * D
    step = (D * t_freq + D) + (D * D + D) + (6 * D * D + 6 * D)
    return 2 * n_blocks * per_layer + step
