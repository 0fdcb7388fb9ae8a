"""CPU oracle of what surrounds the token-space denoising step: latent in, latent out, and the
sampling loop  x_{t-1} = Phi(x_t, t, eps_t)  of the paper's eq. 1.

THIS IS TEST INFRASTRUCTURE, not a product path: only the tests, the smoke check and the
benchmark's cpu_baseline leg may import it.  It shares no code with the HIP library.

The paper's section 2.1 states the reverse process (start from Gaussian noise, T steps, each a
call of eps_theta on (x_t, t, c) followed by a solver Phi) and section 2.2 the pipeline (text
encoder -> DiT on a latent video -> VAE), but writes neither the embedding of the latent into
tokens, nor the output head, nor Phi.  The readings taken here (all plain definitions, fp64):

  * latent z [B, C, T, 2 Hp, 2 Wp]; a token is one 1x2x2 patch: token (b, t, i, j) sees
    z[b, :, t, 2i:2i+2, 2j:2j+2] flattened in the order (c, di, dj) and is embedded by one
    Linear(4C -> D); tokens are ordered s = i Wp + j inside frame t;
  * a fixed 2-D sine/cosine position code is added to every frame's tokens: with Q = D/4 and
    w_m = 10000^(-m/Q), the four quarters of the D-vector of location (i, j) are
    sin(j w_m), cos(j w_m), sin(i w_m), cos(i w_m), m < Q;
  * the text condition c [B, Ly, C_text] enters through Linear(C_text -> D), GELU (tanh form),
    Linear(D -> D);
  * the output head is LayerNorm (no affine, eps 1e-6, biased variance) modulated by
    (shift, scale) = final_table[2, D] + temb_b, temb the D-vector timestep embedding, then
    Linear(D -> 4 C_out) whose outputs are ordered (di, dj, c), put back to
    [B, C_out, T, 2 Hp, 2 Wp];
  * Phi is the explicit Euler step of a rectified flow in the step variable: with the training
    range T_TRAIN = 1000,  z_next = z + (t_next - t) / T_TRAIN * eps,  and a sampling run
    visits t_i = T_TRAIN (1 - i/n), i = 0..n-1, ending at t_n = 0;
  * with guidance scale s and an unconditional text input, eps = eps_u + s (eps_c - eps_u);
    s = 1 is the conditional prediction alone.

Pins (tests/test_oracle_pins_io.py): convolution, layer norm, GELU and pixel rearrangement
routines of other packages; brute-force loops; closed forms of the position code; the exact
solution of a linear flow; guidance at s = 0 and s = 1; composition of the pieces.
"""
from __future__ import annotations

import numpy as np

from . import stdit_oracle as so

T_TRAIN = 1000.0


# ---------------------------------------------------------------------------
# latent <-> tokens
# ---------------------------------------------------------------------------
def patchify(z):
    """z [B,C,T,2Hp,2Wp] -> patches [B,T,Hp*Wp,4C], last axis ordered (c, di, dj)."""
    B, C, T, Hl, Wl = z.shape
    if Hl % 2 or Wl % 2:
        raise ValueError("latent height and width must be even")
    Hp, Wp = Hl // 2, Wl // 2
    out = np.empty((B, T, Hp * Wp, 4 * C), dtype=z.dtype)
    for i in range(Hp):
        for j in range(Wp):
            blk = z[:, :, :, 2 * i:2 * i + 2, 2 * j:2 * j + 2]          # [B,C,T,2,2]
            out[:, :, i * Wp + j, :] = np.transpose(blk, (0, 2, 1, 3, 4)).reshape(B, T, 4 * C)
    return out


def unpatchify(tok, Hp, Wp, C_out):
    """tok [B,T,Hp*Wp,4*C_out], last axis ordered (di, dj, c) -> z [B,C_out,T,2Hp,2Wp]."""
    B, T, S, F = tok.shape
    if S != Hp * Wp or F != 4 * C_out:
        raise ValueError("token tensor does not match the grid")
    z = np.empty((B, C_out, T, 2 * Hp, 2 * Wp), dtype=tok.dtype)
    for i in range(Hp):
        for j in range(Wp):
            v = tok[:, :, i * Wp + j, :].reshape(B, T, 2, 2, C_out)      # (di, dj, c)
            z[:, :, :, 2 * i:2 * i + 2, 2 * j:2 * j + 2] = np.transpose(v, (0, 4, 1, 2, 3))
    return z


def position_code(Hp, Wp, D):
    """[Hp*Wp, D] fixed 2-D sine/cosine code; quarters: sin(j w), cos(j w), sin(i w), cos(i w)."""
    if D % 4:
        raise ValueError("D must be a multiple of 4")
    Q = D // 4
    w = np.exp(-np.log(10000.0) * np.arange(Q, dtype=np.float64) / Q)
    ii, jj = np.meshgrid(np.arange(Hp, dtype=np.float64), np.arange(Wp, dtype=np.float64), indexing="ij")
    ii, jj = ii.reshape(-1, 1), jj.reshape(-1, 1)
    return np.concatenate([np.sin(jj * w), np.cos(jj * w), np.sin(ii * w), np.cos(ii * w)], axis=1)


def embed_latent(z, w_patch, b_patch, D):
    """Tokens x [B,T,S,D] = Linear(patches) + position code."""
    B, C, T, Hl, Wl = z.shape
    x = so.linear(patchify(z), w_patch, b_patch)
    return x + position_code(Hl // 2, Wl // 2, D)[None, None]


def embed_caption(c_text, w_y1, b_y1, w_y2, b_y2):
    """y [B,Ly,D] = W_y2 GELU_tanh(W_y1 c + b_y1) + b_y2."""
    return so.linear(so.gelu_tanh(so.linear(c_text, w_y1, b_y1)), w_y2, b_y2)


def output_head(x, temb, final_table, w_final, b_final, Hp, Wp, C_out):
    """x [B,T,S,D], temb [B,D], final_table [2,D] (shift, scale) -> latent [B,C_out,T,2Hp,2Wp]."""
    m = final_table[None] + temb[:, None, :]                               # [B,2,D]
    xh = so.modulate(so.layer_norm(x), m[:, 0][:, None, None, :], m[:, 1][:, None, None, :])
    return unpatchify(so.linear(xh, w_final, b_final), Hp, Wp, C_out)


def eps_theta(z, c_text, valid_len, t, io_w, sw, blocks, H, dh, rope_temporal=False):
    """The whole model: latent z [B,C,T,2Hp,2Wp], text c_text [B,Ly,C_text], timesteps t [B]
    -> prediction with the latent's shape.  io_w: dict w_patch,b_patch,w_y1,b_y1,w_y2,b_y2,
    final_table,w_final,b_final; sw, blocks and the two self-attention options as in
    stdit_oracle.denoise_step."""
    D = io_w["w_patch"].shape[0]
    B, C, T, Hl, Wl = z.shape
    x = embed_latent(z, io_w["w_patch"], io_w["b_patch"], D)
    y = embed_caption(c_text, io_w["w_y1"], io_w["b_y1"], io_w["w_y2"], io_w["b_y2"])
    temb = so.timestep_embedding(t, sw)
    x = so.denoise_step(x, y, valid_len, t, sw, blocks, H, dh, temb=temb, rope_temporal=rope_temporal)
    C_out = io_w["w_final"].shape[0] // 4
    return output_head(x, temb, io_w["final_table"], io_w["w_final"], io_w["b_final"], Hl // 2, Wl // 2, C_out)


# ---------------------------------------------------------------------------
# solver and sampling loop (eq. 1)
# ---------------------------------------------------------------------------
def guide(eps_c, eps_u, s):
    """eps_u + s (eps_c - eps_u)."""
    return eps_u + s * (eps_c - eps_u)


def solver_step(z, eps, t, t_next):
    """Phi: z + (t_next - t) / T_TRAIN * eps  (t, t_next scalars or [B])."""
    dt = (np.asarray(t_next, dtype=np.float64) - np.asarray(t, dtype=np.float64)) / T_TRAIN
    return z + dt.reshape(dt.shape + (1,) * (z.ndim - dt.ndim)) * eps


def step_schedule(n_steps):
    """t_0..t_n with t_i = T_TRAIN (1 - i/n)."""
    return T_TRAIN * (1.0 - np.arange(n_steps + 1, dtype=np.float64) / n_steps)


def sample(z, model, n_steps, first_step=0, last_step=None):
    """Runs steps first_step..last_step-1 of an n_steps schedule from latent z.
    model(z, t [B]) -> eps with z's shape.  Returns the latent after the last step run."""
    ts = step_schedule(n_steps)
    last_step = n_steps if last_step is None else last_step
    B = z.shape[0]
    for i in range(first_step, last_step):
        t = np.full(B, ts[i])
        z = solver_step(z, model(z, t), ts[i], ts[i + 1])
    return z
