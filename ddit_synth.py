"""Seeded synthetic inputs for the STDiT denoising step.

This module only *draws numbers*: shapes, seeds, normal/uniform draws and the
rounding of each draw to a bf16 bit pattern.  It contains none of the method's
arithmetic (no LayerNorm, attention, linear, GELU ...) and is the only module the
CPU oracle's tests and the HIP path's tests/bench both use, so that the two sides
see bit-identical inputs.

Every tensor is generated as fp32 from ``numpy.random.Generator(PCG64(SeedSequence
([base, block, tensor_id])))``, rounded to nearest-even bf16, and returned as a
``uint16`` array holding the bf16 bit pattern.  ``bits_to_f64`` widens it exactly.
Tensors that are fp32 at the library boundary (the adaLN table, the conditioning
vector) are returned as fp32 arrays that already hold bf16-representable values,
so the fp64 oracle and the fp32 device buffers agree exactly.

The workloads follow the shapes of OpenSora-style video latents (the paper
evaluates 51-frame requests at 144p/240p/360p, section 6.1; the larger ones extend
that list): tokens per frame S = Hp*Wp, T latent frames, 300 text tokens, hidden
1152 = 16 heads x 72, MLP 4608, 28 blocks.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional

import numpy as np


@dataclass(frozen=True)
class Shape:
    B: int
    T: int
    Hp: int
    Wp: int
    D: int
    H: int
    dh: int
    M: int
    Ly: int
    n_blocks: int

    @property
    def S(self) -> int:
        return self.Hp * self.Wp

    @property
    def L(self) -> int:
        return self.T * self.S

    @property
    def N(self) -> int:
        return self.B * self.L

    @property
    def A(self) -> int:
        return self.H * self.dh


# name -> (shape, base seed, text valid-length rule, timestep rule)
CONFIGS: Dict[str, dict] = {
    # one small block the CPU oracle finishes in well under a second
    "C1": dict(shape=Shape(1, 4, 8, 8, 256, 4, 64, 1024, 16, 1), base=1, valid="full", t="given_temb"),
    # 144p-shaped 28-block stack
    "C2": dict(shape=Shape(1, 16, 9, 16, 1152, 16, 72, 4608, 300, 28), base=2, valid="full", t="fixed500"),
    # 240p-shaped, batch 2, per-sample timesteps
    "C3": dict(shape=Shape(2, 16, 15, 27, 1152, 16, 72, 4608, 300, 28), base=3, valid="full", t="uniform"),
    # 480p-shaped, random text padding
    "C4": dict(shape=Shape(1, 30, 30, 54, 1152, 16, 72, 4608, 300, 28), base=4, valid="uniform32", t="uniform"),
    # 720p-shaped, one rank's share of a 4-way head split: 4 of 16 heads in attention
    "C5": dict(shape=Shape(1, 30, 45, 80, 1152, 4, 72, 4608, 300, 28), base=5, valid="full", t="uniform"),
}

# tensor ids inside one layer (stable: changing them changes every golden value)
_LAYER_TENSORS = ["w_qkv", "b_qkv", "w_o", "b_o", "w_cq", "b_cq", "w_ckv", "b_ckv",
                  "w_co", "b_co", "w_fc1", "b_fc1", "w_fc2", "b_fc2", "ada_table"]
_STEP_TENSORS = ["w_t1", "b_t1", "w_t2", "b_t2", "w_ada", "b_ada"]
_KIND_ID = {"spatial": 0, "temporal": 1}
T_FREQ = 256  # width of the sinusoidal timestep feature vector


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to the nearest bf16 (ties to even); returns the uint16 pattern."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return bits_to_f32(bits).astype(np.float64)


def _rng(*key: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence(list(key))))


def normal_bits(key, shape, std: float = 1.0) -> np.ndarray:
    """bf16 bit pattern of N(0, std^2) draws."""
    g = _rng(*key)
    return f32_to_bf16_bits((g.standard_normal(size=shape, dtype=np.float32) * np.float32(std)))


def layer_shapes(sh: Shape) -> Dict[str, tuple]:
    D, A, M = sh.D, sh.A, sh.M
    return {
        "w_qkv": (3 * A, D), "b_qkv": (3 * A,),
        "w_o": (D, A), "b_o": (D,),
        "w_cq": (A, D), "b_cq": (A,),
        "w_ckv": (2 * A, D), "b_ckv": (2 * A,),
        "w_co": (D, A), "b_co": (D,),
        "w_fc1": (M, D), "b_fc1": (M,),
        "w_fc2": (D, M), "b_fc2": (D,),
        "ada_table": (6, D),
    }


def step_shapes(sh: Shape) -> Dict[str, tuple]:
    D = sh.D
    return {"w_t1": (D, T_FREQ), "b_t1": (D,), "w_t2": (D, D), "b_t2": (D,),
            "w_ada": (6 * D, D), "b_ada": (6 * D,)}


def make_layer_weights(sh: Shape, base: int, block: int, kind: str,
                       w_std: float = 0.02, table_std: float = 0.02) -> Dict[str, np.ndarray]:
    """Weights of one layer: bf16 bit patterns (uint16); ``ada_table`` as fp32 holding
    bf16-representable values."""
    out = {}
    for tid, name in enumerate(_LAYER_TENSORS):
        shape = layer_shapes(sh)[name]
        key = (base, block, 10 + 100 * _KIND_ID[kind] + tid)
        if name == "ada_table":
            out[name] = bits_to_f32(normal_bits(key, shape, table_std))
        else:
            out[name] = normal_bits(key, shape, w_std)
    return out


def make_qk_norm_scales(sh: Shape, base: int, block: int, kind: str, spread: float = 0.2) -> Dict[str, np.ndarray]:
    """Per-head RMS-norm scales g_q, g_k [dh] of one layer's self-attention: bf16 bit patterns of
    1 + spread * N(0,1) draws (a trained norm's scales sit around one)."""
    out = {}
    for tid, name in enumerate(("g_q", "g_k")):
        g = _rng(base, block, 70 + 100 * _KIND_ID[kind] + tid)
        out[name] = f32_to_bf16_bits((1.0 + spread * g.standard_normal(size=(sh.dh,), dtype=np.float32)).astype(np.float32))
    return out


def make_block_weights(sh: Shape, base: int, block: int, qk_norm: bool = False, **kw) -> Dict[str, Dict[str, np.ndarray]]:
    out = {k: make_layer_weights(sh, base, block, k, **kw) for k in ("spatial", "temporal")}
    if qk_norm:
        for k in out:
            out[k].update(make_qk_norm_scales(sh, base, block, k))
    return out


def make_step_weights(sh: Shape, base: int, w_std: float = 0.02) -> Dict[str, np.ndarray]:
    out = {}
    for tid, name in enumerate(_STEP_TENSORS):
        out[name] = normal_bits((base, 9000, tid), step_shapes(sh)[name], w_std)
    return out


def make_activations(sh: Shape, base: int) -> Dict[str, np.ndarray]:
    """x [B,T,S,D] and y [B,Ly,D] as bf16 bit patterns, N(0,1)."""
    return {"x": normal_bits((base, 9100, 0), (sh.B, sh.T, sh.S, sh.D), 1.0),
            "y": normal_bits((base, 9100, 1), (sh.B, sh.Ly, sh.D), 1.0)}


def make_c6(sh: Shape, base: int, std: float = 1.0) -> np.ndarray:
    """A conditioning vector c6 [B,6D] given directly (fp32 holding bf16-representable
    values), for block-level calls that bypass the timestep embedder."""
    return bits_to_f32(normal_bits((base, 9100, 2), (sh.B, 6 * sh.D), std))


def make_temb(sh: Shape, base: int) -> np.ndarray:
    """A 'random timestep embedding' [B,D] ~ N(0,1), fp32 holding bf16-representable values."""
    return bits_to_f32(normal_bits((base, 9100, 3), (sh.B, sh.D), 1.0))


def make_timesteps(sh: Shape, base: int, rule: str) -> np.ndarray:
    g = _rng(base, 999, 0)
    if rule == "fixed500":
        return np.full((sh.B,), 500.0, dtype=np.float32)
    # uniform in [0, 1000)
    return g.uniform(0.0, 1000.0, size=(sh.B,)).astype(np.float32)


def make_valid_len(sh: Shape, base: int, rule: str) -> np.ndarray:
    g = _rng(base, 999, 1)
    if rule == "full":
        return np.full((sh.B,), sh.Ly, dtype=np.int32)
    lo = min(32, sh.Ly)
    return g.integers(lo, sh.Ly + 1, size=(sh.B,)).astype(np.int32)


def make_attn_inputs(kind: str, sh: Shape, base: int, q_scale: float = 1.0,
                     Lq: Optional[int] = None) -> Dict[str, np.ndarray]:
    """q,k,v ~ N(0,1) (q optionally scaled: the 'peaked' variant) for attention-only
    calls.  self kinds: each [B,T,S,H,dh]; cross: q [B,L,H,dh], k,v [B,Ly,H,dh]."""
    if kind == "cross":
        qs = (sh.B, sh.L if Lq is None else Lq, sh.H, sh.dh)
        ks = (sh.B, sh.Ly, sh.H, sh.dh)
    else:
        qs = ks = (sh.B, sh.T, sh.S, sh.H, sh.dh)
    g = _rng(base + 100, 9200, 0)
    q = g.standard_normal(size=qs, dtype=np.float32) * np.float32(q_scale)
    return {"q": f32_to_bf16_bits(q),
            "k": normal_bits((base + 100, 9200, 1), ks, 1.0),
            "v": normal_bits((base + 100, 9200, 2), ks, 1.0)}


# ---- latent-in / latent-out layers and the sampling loop -------------------------------------
_IO_TENSORS = ["w_patch", "b_patch", "w_y1", "b_y1", "w_y2", "b_y2", "final_table", "w_final", "b_final"]


def io_shapes(sh: Shape, C: int, C_text: int, C_out: int) -> Dict[str, tuple]:
    D = sh.D
    return {"w_patch": (D, 4 * C), "b_patch": (D,), "w_y1": (D, C_text), "b_y1": (D,),
            "w_y2": (D, D), "b_y2": (D,), "final_table": (2, D), "w_final": (4 * C_out, D),
            "b_final": (4 * C_out,)}


def make_io_weights(sh: Shape, base: int, C: int, C_text: int, C_out: int, w_std: float = 0.02,
                    patch_std: float = 0.25, final_std: float = 0.05) -> Dict[str, np.ndarray]:
    """Weights of the patch embedder, the caption embedder and the output head: bf16 bit patterns;
    ``final_table`` as fp32 holding bf16-representable values."""
    out = {}
    shapes = io_shapes(sh, C, C_text, C_out)
    for tid, name in enumerate(_IO_TENSORS):
        key = (base, 9300, tid)
        std = patch_std if name == "w_patch" else final_std if name == "w_final" else w_std
        if name == "final_table":
            out[name] = bits_to_f32(normal_bits(key, shapes[name], 0.5))
        else:
            out[name] = normal_bits(key, shapes[name], std)
    return out


def make_latent(sh: Shape, base: int, C: int) -> np.ndarray:
    """Latent video z [B,C,T,2Hp,2Wp] ~ N(0,1) (the start of the reverse process), fp32 holding
    bf16-representable values."""
    return bits_to_f32(normal_bits((base, 9400, 0), (sh.B, C, sh.T, 2 * sh.Hp, 2 * sh.Wp), 1.0))


def make_caption(sh: Shape, base: int, C_text: int, which: int = 0) -> np.ndarray:
    """Text-encoder output c [B,Ly,C_text] ~ N(0,1) as bf16 bit patterns (which = 1: a second,
    'unconditional' input)."""
    return normal_bits((base, 9400, 1 + which), (sh.B, sh.Ly, C_text), 1.0)


def small_variant(sh: Shape, **kw) -> Shape:
    return replace(sh, **kw)
