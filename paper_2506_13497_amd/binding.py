"""ctypes binding of libddit_hot: one Python function per C entry point, same names.

Argument marshalling only (tensor -> pointer, dataclass -> struct); every step of the
path runs inside the library's HIP kernels.  There is no fallback: if the shared
library is missing or fails to load, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libddit_hot.so")

DDIT_OK = 0
DDIT_ERR_INVALID_ARG, DDIT_ERR_UNSUPPORTED, DDIT_ERR_WORKSPACE, DDIT_ERR_ALIGNMENT, DDIT_ERR_HIP = -1, -2, -3, -4, -5
DDIT_ATTN_SPATIAL, DDIT_ATTN_TEMPORAL, DDIT_ATTN_CROSS = 0, 1, 2
DDIT_EPI_BF16, DDIT_EPI_GELU_BF16, DDIT_EPI_RESIDUAL_F32 = 0, 1, 2
DDIT_FLAG_TAPS, DDIT_FLAG_QK_NORM, DDIT_FLAG_ROPE_TEMPORAL = 1, 2, 4
TAP_NAMES = ["xh_msa", "qkv", "o", "x_after_attn", "qc", "kvc", "oc", "x_after_cross", "xh_mlp", "h", "x_out"]
_TAP_DTYPE = {"x_after_attn": torch.float32, "x_after_cross": torch.float32, "x_out": torch.float32}

EXPORTS = ["ddit_abi_version", "ddit_status_string", "ddit_last_error", "ddit_workspace_bytes", "ddit_tap_region",
           "ddit_attn_fwd", "ddit_stdit_block_fwd", "ddit_stdit_block_fwd_static", "ddit_denoise_step", "ddit_modulated_layernorm_fwd",
           "ddit_linear_fwd", "ddit_timestep_conditioning", "ddit_io_workspace_bytes", "ddit_embed_latent",
           "ddit_embed_caption", "ddit_output_head", "ddit_eps_theta", "ddit_solver_step", "ddit_sample",
           "ddit_cross_kv_bytes", "ddit_cross_kv_precompute", "ddit_denoise_step_cached", "ddit_linear_tile_count",
           "ddit_linear_tile_info", "ddit_linear_tile_choice", "ddit_linear_fwd_tile", "ddit_qk_norm_rope_fwd", "ddit_self_attn_fwd", "ddit_optimal_dop",
           "ddit_buddy_create", "ddit_buddy_alloc", "ddit_buddy_release", "ddit_buddy_free_gpus", "ddit_buddy_destroy",
           "ddit_sched_simulate", "ddit_probe_mfma_bf16", "ddit_probe_stream_copy", "ddit_probe_stream_read", "ddit_probe_residual_stream"]


class ddit_shape(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("flags", C.c_uint32),
                ("B", C.c_int32), ("T", C.c_int32), ("Hp", C.c_int32), ("Wp", C.c_int32),
                ("D", C.c_int32), ("H", C.c_int32), ("dh", C.c_int32), ("M", C.c_int32),
                ("Ly", C.c_int32), ("n_blocks", C.c_int32), ("ln_eps", C.c_float)]


_LAYER_FIELDS = ["w_qkv", "b_qkv", "w_o", "b_o", "w_cq", "b_cq", "w_ckv", "b_ckv", "w_co", "b_co",
                 "w_fc1", "b_fc1", "w_fc2", "b_fc2", "ada_table", "g_q", "g_k"]


class ddit_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _LAYER_FIELDS]


class ddit_block_weights(C.Structure):
    _fields_ = [("spatial", ddit_layer_weights), ("temporal", ddit_layer_weights)]


class ddit_step_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("w_t1", "b_t1", "w_t2", "b_t2", "w_ada", "b_ada")] + \
               [("blocks", C.POINTER(ddit_block_weights))]


_IO_FIELDS = ["w_patch", "b_patch", "w_y1", "b_y1", "w_y2", "b_y2", "final_table", "w_final", "b_final"]


class ddit_io_weights(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("C_in", C.c_int32), ("C_out", C.c_int32), ("C_text", C.c_int32)] + \
               [(n, C.c_void_p) for n in _IO_FIELDS]


class ddit_sched_config(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("n_gpus", C.c_int32), ("n_steps", C.c_int32), ("n_resolutions", C.c_int32),
                ("n_dop", C.c_int32), ("vae_gpus", C.c_int32), ("step_us", C.POINTER(C.c_int64)),
                ("opt_dop", C.POINTER(C.c_int32)), ("vae_us", C.POINTER(C.c_int64))]


class ddit_sched_request(C.Structure):
    _fields_ = [("arrival_us", C.c_int64), ("resolution", C.c_int32), ("reserved", C.c_int32)]


class ddit_sched_record(C.Structure):
    _fields_ = [("start_us", C.c_int64), ("dit_end_us", C.c_int64), ("end_us", C.c_int64), ("starvation", C.c_int64),
                ("first_dop", C.c_int32), ("final_dop", C.c_int32), ("promotions", C.c_int32), ("reserved", C.c_int32)]


class ddit_sched_event(C.Structure):
    _fields_ = [("time_us", C.c_int64), ("kind", C.c_int32), ("request", C.c_int32), ("gpu_start", C.c_int32),
                ("gpu_count", C.c_int32)]


class ddit_sched_totals(C.Structure):
    _fields_ = [("occupancy_gpu_us", C.c_int64), ("makespan_us", C.c_int64)]


SCHED_EVENT_NAMES = ["start", "promote", "dit_done", "release"]


class DditError(RuntimeError):
    def __init__(self, status: int, detail: str):
        super().__init__("libddit_hot status %d: %s" % (status, detail))
        self.status = status


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError("libddit_hot.so is not built (%s): run `python -m paper_2506_13497_amd.build` or "
                          "__graft_entry__.build(); there is no fallback path" % LIB_PATH)
    lib = C.CDLL(LIB_PATH)
    lib.ddit_abi_version.restype = C.c_uint32
    lib.ddit_status_string.restype = C.c_char_p
    lib.ddit_status_string.argtypes = [C.c_int]
    lib.ddit_last_error.restype = C.c_char_p
    lib.ddit_workspace_bytes.argtypes = [C.POINTER(ddit_shape), C.POINTER(C.c_size_t)]
    lib.ddit_tap_region.argtypes = [C.POINTER(ddit_shape), C.c_int, C.c_int, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
    lib.ddit_attn_fwd.argtypes = [C.c_int, C.POINTER(ddit_shape), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64,
                                  C.c_int64, C.POINTER(C.c_int32), C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                                  C.c_size_t, C.c_void_p]
    lib.ddit_stdit_block_fwd.argtypes = [C.POINTER(ddit_shape), C.POINTER(ddit_block_weights), C.c_void_p, C.c_void_p,
                                         C.POINTER(C.c_int32), C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
                                         C.c_void_p]
    lib.ddit_stdit_block_fwd_static.argtypes = [C.POINTER(ddit_shape), C.POINTER(ddit_block_weights), C.c_void_p,
                                                C.c_void_p, C.POINTER(C.c_int32), C.c_void_p, C.c_void_p, C.c_void_p]
    lib.ddit_denoise_step.argtypes = [C.POINTER(ddit_shape), C.POINTER(ddit_step_weights), C.c_void_p, C.c_void_p,
                                      C.POINTER(C.c_int32), C.POINTER(C.c_float), C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.c_size_t, C.c_void_p]
    lib.ddit_modulated_layernorm_fwd.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int64, C.c_int64,
                                                 C.c_int32, C.c_float, C.c_void_p, C.c_void_p]
    lib.ddit_linear_fwd.argtypes = [C.c_int, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_int64, C.c_int32,
                                    C.c_int32, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                                    C.c_int64, C.c_void_p]
    lib.ddit_qk_norm_rope_fwd.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                          C.c_float, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p]
    lib.ddit_optimal_dop.argtypes = [C.POINTER(C.c_int64), C.c_int32, C.c_int64, C.c_int64, C.POINTER(C.c_int32)]
    lib.ddit_buddy_create.argtypes = [C.c_int32, C.POINTER(C.c_void_p)]
    lib.ddit_buddy_alloc.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_int32)]
    lib.ddit_buddy_release.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
    lib.ddit_buddy_free_gpus.argtypes = [C.c_void_p, C.POINTER(C.c_int32)]
    lib.ddit_buddy_destroy.argtypes = [C.c_void_p]
    lib.ddit_sched_simulate.argtypes = [C.POINTER(ddit_sched_config), C.POINTER(ddit_sched_request), C.c_int32,
                                        C.POINTER(ddit_sched_record), C.POINTER(ddit_sched_event), C.c_int64,
                                        C.POINTER(C.c_int64), C.POINTER(ddit_sched_totals)]
    lib.ddit_self_attn_fwd.argtypes = [C.c_int, C.POINTER(ddit_shape), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64,
                                       C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_int64,
                                       C.c_void_p, C.c_void_p]
    lib.ddit_linear_fwd_tile.argtypes = [C.c_int] + list(lib.ddit_linear_fwd.argtypes)
    lib.ddit_linear_tile_count.argtypes = []
    lib.ddit_linear_tile_info.argtypes = [C.c_int] + [C.POINTER(C.c_int32)] * 4
    lib.ddit_linear_tile_choice.argtypes = [C.c_int, C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_int32),
                                            C.POINTER(C.c_float)]
    lib.ddit_timestep_conditioning.argtypes = [C.POINTER(ddit_shape), C.POINTER(ddit_step_weights),
                                               C.POINTER(C.c_float), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    SP, WP, IP, VP, FP = C.POINTER(ddit_shape), C.POINTER(ddit_step_weights), C.POINTER(ddit_io_weights), C.c_void_p, \
        C.POINTER(C.c_float)
    lib.ddit_io_workspace_bytes.argtypes = [SP, IP, C.POINTER(C.c_size_t)]
    lib.ddit_embed_latent.argtypes = [SP, IP, VP, VP, VP, C.c_size_t, VP]
    lib.ddit_embed_caption.argtypes = [SP, IP, VP, VP, VP, C.c_size_t, VP]
    lib.ddit_output_head.argtypes = [SP, IP, VP, VP, VP, VP]
    lib.ddit_eps_theta.argtypes = [SP, WP, IP, VP, VP, VP, C.POINTER(C.c_int32), FP, VP, VP, C.c_size_t, VP]
    lib.ddit_cross_kv_bytes.argtypes = [SP, C.POINTER(C.c_size_t)]
    lib.ddit_cross_kv_precompute.argtypes = [SP, WP, VP, VP, VP]
    lib.ddit_denoise_step_cached.argtypes = [SP, WP, VP, VP, VP, C.POINTER(C.c_int32), FP, VP, VP, VP, C.c_size_t, VP]
    lib.ddit_solver_step.argtypes = [VP, VP, VP, C.c_float, FP, FP, C.c_int32, C.c_int64, VP]
    lib.ddit_sample.argtypes = [SP, WP, IP, VP, VP, C.POINTER(C.c_int32), VP, VP, VP, C.c_float, C.c_int32, C.c_int32,
                                C.c_int32, VP, VP, C.c_size_t, VP]
    lib.ddit_probe_mfma_bf16.argtypes = [VP, VP, C.c_int32, C.POINTER(C.c_double), VP]
    lib.ddit_probe_stream_copy.argtypes = [VP, VP, C.c_int64, VP]
    lib.ddit_probe_stream_read.argtypes = [VP, C.c_int64, VP, VP]
    lib.ddit_probe_residual_stream.argtypes = [VP, VP, VP, VP, C.c_int64, C.c_int32, C.c_int32, VP]
    for n in EXPORTS:
        if n not in ("ddit_abi_version", "ddit_status_string", "ddit_last_error", "ddit_linear_tile_count"):
            getattr(lib, n).restype = C.c_int
    return lib


_lib = _load()


def _check(rc: int) -> None:
    if rc != DDIT_OK:
        raise DditError(rc, (_lib.ddit_last_error() or b"").decode())


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def make_shape(B, T, Hp, Wp, D, H, dh, M, Ly, n_blocks, flags=0, ln_eps=1e-6) -> ddit_shape:
    return ddit_shape(C.sizeof(ddit_shape), flags, B, T, Hp, Wp, D, H, dh, M, Ly, n_blocks, ln_eps)


def _i32(vals: Optional[Sequence[int]]):
    if vals is None:
        return None
    return (C.c_int32 * len(vals))(*[int(v) for v in vals])


def layer_struct(w: Dict[str, torch.Tensor]) -> ddit_layer_weights:
    s = ddit_layer_weights()
    for n in _LAYER_FIELDS:
        t = w.get(n)
        setattr(s, n, None if t is None else t.data_ptr())
    return s


def block_struct(wb: Dict[str, Dict[str, torch.Tensor]]) -> ddit_block_weights:
    return ddit_block_weights(layer_struct(wb["spatial"]), layer_struct(wb["temporal"]))


def step_struct(sw: Dict[str, torch.Tensor], blocks: List[Dict[str, Dict[str, torch.Tensor]]]):
    arr = (ddit_block_weights * max(len(blocks), 1))()
    for i, wb in enumerate(blocks):
        arr[i] = block_struct(wb)
    s = ddit_step_weights()
    for n in ("w_t1", "b_t1", "w_t2", "b_t2", "w_ada", "b_ada"):
        t = sw.get(n)
        setattr(s, n, None if t is None else t.data_ptr())
    s.blocks = C.cast(arr, C.POINTER(ddit_block_weights))
    s._keep = arr  # keep the host array alive with the struct
    return s


# ----------------------------------------------------------------------------- entry points
def ddit_abi_version() -> int:
    return int(_lib.ddit_abi_version())


def ddit_status_string(status: int) -> str:
    return _lib.ddit_status_string(status).decode()


def ddit_last_error() -> str:
    return (_lib.ddit_last_error() or b"").decode()


def ddit_workspace_bytes(shape: ddit_shape) -> int:
    n = C.c_size_t(0)
    _check(_lib.ddit_workspace_bytes(C.byref(shape), C.byref(n)))
    return int(n.value)


def ddit_tap_region(shape: ddit_shape, layer: int, tap: int):
    off, nb = C.c_size_t(0), C.c_size_t(0)
    _check(_lib.ddit_tap_region(C.byref(shape), layer, tap, C.byref(off), C.byref(nb)))
    return int(off.value), int(nb.value)


def ddit_attn_fwd(kind: int, shape: ddit_shape, q, k, v, ld_q: int, ld_kv: int, kv_valid_len, o, ld_o: int,
                  lse=None, workspace=None) -> None:
    _check(_lib.ddit_attn_fwd(kind, C.byref(shape), _ptr(q), _ptr(k), _ptr(v), ld_q, ld_kv, _i32(kv_valid_len),
                              _ptr(o), ld_o, _ptr(lse), _ptr(workspace),
                              0 if workspace is None else workspace.numel() * workspace.element_size(), _stream()))


def ddit_stdit_block_fwd(shape: ddit_shape, weights: ddit_block_weights, x_in, y, y_valid_len, c6, x_out,
                         workspace) -> None:
    _check(_lib.ddit_stdit_block_fwd(C.byref(shape), C.byref(weights), _ptr(x_in), _ptr(y), _i32(y_valid_len),
                                     _ptr(c6), _ptr(x_out), _ptr(workspace),
                                     workspace.numel() * workspace.element_size(), _stream()))


DDIT_STATIC_SCRATCH_BYTES = 64 << 20


def ddit_stdit_block_fwd_static(shape: ddit_shape, weights: ddit_block_weights, x_in, y, y_valid_len, c6, x_out) -> None:
    _check(_lib.ddit_stdit_block_fwd_static(C.byref(shape), C.byref(weights), _ptr(x_in), _ptr(y), _i32(y_valid_len),
                                            _ptr(c6), _ptr(x_out), _stream()))


def ddit_denoise_step(shape: ddit_shape, weights: ddit_step_weights, x_in, y, y_valid_len, timesteps, temb, x_out,
                      workspace) -> None:
    ts = None if timesteps is None else (C.c_float * len(timesteps))(*[float(t) for t in timesteps])
    _check(_lib.ddit_denoise_step(C.byref(shape), C.byref(weights), _ptr(x_in), _ptr(y), _i32(y_valid_len), ts,
                                  _ptr(temb), _ptr(x_out), _ptr(workspace),
                                  workspace.numel() * workspace.element_size(), _stream()))


def ddit_modulated_layernorm_fwd(x, ada_table, c6, which: int, tokens_per_sample: int, eps: float, out) -> None:
    N, D = x.shape[0], x.shape[1]
    _check(_lib.ddit_modulated_layernorm_fwd(_ptr(x), _ptr(ada_table), _ptr(c6), which, N, tokens_per_sample, D, eps,
                                             _ptr(out), _stream()))


def ddit_linear_fwd(epilogue: int, u, ld_u: int, W, bias, N: int, n: int, k: int, out, ld_out: int, resid=None,
                    ada_table=None, c6=None, gate_row: int = -1, tokens_per_sample: int = 1) -> None:
    _check(_lib.ddit_linear_fwd(epilogue, _ptr(u), ld_u, _ptr(W), _ptr(bias), N, n, k, _ptr(out), ld_out,
                                _ptr(resid), _ptr(ada_table), _ptr(c6), gate_row, tokens_per_sample, _stream()))


def ddit_qk_norm_rope_fwd(qk, ld: int, N: int, H: int, dh: int, g_q, g_k, eps: float, S: int, T: int,
                          rope_table=None) -> None:
    _check(_lib.ddit_qk_norm_rope_fwd(_ptr(qk), ld, N, H, dh, _ptr(g_q), _ptr(g_k), eps, S, T, _ptr(rope_table), _stream()))


def ddit_optimal_dop(step_us_row: Sequence[int], z_min_num: int = 0, z_min_den: int = 1) -> int:
    row = (C.c_int64 * len(step_us_row))(*[int(v) for v in step_us_row])
    out = C.c_int32()
    _check(_lib.ddit_optimal_dop(row, len(step_us_row), z_min_num, z_min_den, C.byref(out)))
    return out.value


def ddit_buddy_create(n_gpus: int):
    h = C.c_void_p()
    _check(_lib.ddit_buddy_create(n_gpus, C.byref(h)))
    return h


def ddit_buddy_alloc(pool, size: int) -> int:
    """-> start of the block, or -1 when nothing fits."""
    out = C.c_int32()
    _check(_lib.ddit_buddy_alloc(pool, size, C.byref(out)))
    return out.value


def ddit_buddy_release(pool, start: int, size: int) -> None:
    _check(_lib.ddit_buddy_release(pool, start, size))


def ddit_buddy_free_gpus(pool) -> int:
    out = C.c_int32()
    _check(_lib.ddit_buddy_free_gpus(pool, C.byref(out)))
    return out.value


def ddit_buddy_destroy(pool) -> None:
    _check(_lib.ddit_buddy_destroy(pool))


def ddit_sched_simulate(n_gpus: int, n_steps: int, step_us: Sequence[Sequence[int]], opt_dop: Sequence[int],
                        requests: Sequence[Sequence[int]], vae_us: Optional[Sequence[int]] = None, vae_gpus: int = 1,
                        max_events: Optional[int] = None):
    """requests: (arrival_us, resolution) pairs -> (records, events, totals) as plain dicts / tuples."""
    R, K = len(step_us), len(step_us[0])
    flat = (C.c_int64 * (R * K))(*[int(v) for row in step_us for v in row])
    bb = (C.c_int32 * R)(*[int(v) for v in opt_dop])
    vv = None if vae_us is None else (C.c_int64 * R)(*[int(v) for v in vae_us])
    cfg = ddit_sched_config(C.sizeof(ddit_sched_config), n_gpus, n_steps, R, K, vae_gpus, flat, bb, vv)
    n = len(requests)
    rq = (ddit_sched_request * max(n, 1))()
    for i, (a, r) in enumerate(requests):
        rq[i].arrival_us, rq[i].resolution = int(a), int(r)
    recs = (ddit_sched_record * max(n, 1))()
    cap = max_events if max_events is not None else n * (4 + 3 * max(K, 1) + 2 * n_gpus.bit_length()) + 8
    ev = (ddit_sched_event * max(cap, 1))()
    n_ev = C.c_int64()
    tot = ddit_sched_totals()
    _check(_lib.ddit_sched_simulate(C.byref(cfg), rq, n, recs, ev if cap > 0 else None, cap, C.byref(n_ev), C.byref(tot)))
    if max_events is None and n_ev.value > cap:          # the estimate was short: run again with the exact size
        cap = n_ev.value
        ev = (ddit_sched_event * cap)()
        _check(_lib.ddit_sched_simulate(C.byref(cfg), rq, n, recs, ev, cap, C.byref(n_ev), C.byref(tot)))
    names = ("start_us", "dit_end_us", "end_us", "first_dop", "final_dop", "promotions", "starvation")
    records = [{k: getattr(recs[i], k) for k in names} for i in range(n)]
    events = [(ev[i].time_us, SCHED_EVENT_NAMES[ev[i].kind], ev[i].request, ev[i].gpu_start, ev[i].gpu_count)
              for i in range(min(n_ev.value, cap))]
    return records, events, {"occupancy_gpu_us": tot.occupancy_gpu_us, "makespan_us": tot.makespan_us,
                             "n_events": n_ev.value}


def ddit_self_attn_fwd(kind: int, shape: ddit_shape, q, k, v, ld_q: int, ld_kv: int, g_q, g_k, rope_table, fuse: bool, o,
                       ld_o: int, lse=None) -> None:
    _check(_lib.ddit_self_attn_fwd(kind, C.byref(shape), _ptr(q), _ptr(k), _ptr(v), ld_q, ld_kv, _ptr(g_q), _ptr(g_k),
                                   _ptr(rope_table), 1 if fuse else 0, _ptr(o), ld_o, _ptr(lse), _stream()))


def ddit_linear_tile_count() -> int:
    return int(_lib.ddit_linear_tile_count())


def ddit_linear_tile_info(tile: int) -> Dict[str, int]:
    v = [C.c_int32() for _ in range(4)]
    _check(_lib.ddit_linear_tile_info(tile, *[C.byref(x) for x in v]))
    return dict(zip(("rows", "cols", "wavefronts", "workgroups_per_cu"), (x.value for x in v)))


def ddit_linear_tile_choice(epilogue: int, N: int, n: int, k: int, compute_units: int = 0):
    """-> (tile, [predicted microseconds of every tile])."""
    tile = C.c_int32()
    us = (C.c_float * ddit_linear_tile_count())()
    _check(_lib.ddit_linear_tile_choice(epilogue, N, n, k, compute_units, C.byref(tile), us))
    return tile.value, list(us)


def ddit_linear_fwd_tile(tile: int, epilogue: int, u, ld_u: int, W, bias, N: int, n: int, k: int, out, ld_out: int,
                         resid=None, ada_table=None, c6=None, gate_row: int = -1, tokens_per_sample: int = 1) -> None:
    _check(_lib.ddit_linear_fwd_tile(tile, epilogue, _ptr(u), ld_u, _ptr(W), _ptr(bias), N, n, k, _ptr(out), ld_out,
                                     _ptr(resid), _ptr(ada_table), _ptr(c6), gate_row, tokens_per_sample, _stream()))


def ddit_timestep_conditioning(shape: ddit_shape, weights: ddit_step_weights, timesteps, temb, c6_out, scratch) -> None:
    ts = None if timesteps is None else (C.c_float * len(timesteps))(*[float(t) for t in timesteps])
    _check(_lib.ddit_timestep_conditioning(C.byref(shape), C.byref(weights), ts, _ptr(temb), _ptr(c6_out),
                                           _ptr(scratch), _stream()))


def io_struct(w: Dict[str, torch.Tensor], C_in: int, C_out: int, C_text: int) -> ddit_io_weights:
    s = ddit_io_weights()
    s.struct_size = C.sizeof(ddit_io_weights)
    s.C_in, s.C_out, s.C_text = C_in, C_out, C_text
    for n in _IO_FIELDS:
        t = w.get(n)
        setattr(s, n, None if t is None else t.data_ptr())
    return s


def _floats(vals):
    return None if vals is None else (C.c_float * len(vals))(*[float(v) for v in vals])


def _nbytes(t: Optional[torch.Tensor]) -> int:
    return 0 if t is None else t.numel() * t.element_size()


def ddit_io_workspace_bytes(shape: ddit_shape, io: ddit_io_weights) -> int:
    n = C.c_size_t(0)
    _check(_lib.ddit_io_workspace_bytes(C.byref(shape), C.byref(io), C.byref(n)))
    return int(n.value)


def ddit_embed_latent(shape: ddit_shape, io: ddit_io_weights, z, x_out, workspace) -> None:
    _check(_lib.ddit_embed_latent(C.byref(shape), C.byref(io), _ptr(z), _ptr(x_out), _ptr(workspace),
                                  _nbytes(workspace), _stream()))


def ddit_embed_caption(shape: ddit_shape, io: ddit_io_weights, c_text, y_out, workspace) -> None:
    _check(_lib.ddit_embed_caption(C.byref(shape), C.byref(io), _ptr(c_text), _ptr(y_out), _ptr(workspace),
                                   _nbytes(workspace), _stream()))


def ddit_output_head(shape: ddit_shape, io: ddit_io_weights, x, temb, eps_out) -> None:
    _check(_lib.ddit_output_head(C.byref(shape), C.byref(io), _ptr(x), _ptr(temb), _ptr(eps_out), _stream()))


def ddit_eps_theta(shape: ddit_shape, weights: ddit_step_weights, io: ddit_io_weights, z, y, y_valid_len, timesteps,
                   eps_out, workspace, cross_kv=None) -> None:
    _check(_lib.ddit_eps_theta(C.byref(shape), C.byref(weights), C.byref(io), _ptr(z), _ptr(y), _ptr(cross_kv),
                               _i32(y_valid_len), _floats(timesteps), _ptr(eps_out), _ptr(workspace),
                               _nbytes(workspace), _stream()))


def ddit_cross_kv_bytes(shape: ddit_shape) -> int:
    n = C.c_size_t(0)
    _check(_lib.ddit_cross_kv_bytes(C.byref(shape), C.byref(n)))
    return int(n.value)


def ddit_cross_kv_precompute(shape: ddit_shape, weights: ddit_step_weights, y, cross_kv_out) -> None:
    _check(_lib.ddit_cross_kv_precompute(C.byref(shape), C.byref(weights), _ptr(y), _ptr(cross_kv_out), _stream()))


def ddit_denoise_step_cached(shape: ddit_shape, weights: ddit_step_weights, x_in, y, cross_kv, y_valid_len, timesteps,
                             temb, x_out, workspace) -> None:
    _check(_lib.ddit_denoise_step_cached(C.byref(shape), C.byref(weights), _ptr(x_in), _ptr(y), _ptr(cross_kv),
                                         _i32(y_valid_len), _floats(timesteps), _ptr(temb), _ptr(x_out),
                                         _ptr(workspace), _nbytes(workspace), _stream()))


def ddit_solver_step(z, eps_c, eps_u, guidance: float, t, t_next, per_sample: int) -> None:
    _check(_lib.ddit_solver_step(_ptr(z), _ptr(eps_c), _ptr(eps_u), guidance, _floats(t), _floats(t_next), len(t),
                                 per_sample, _stream()))


def ddit_sample(shape: ddit_shape, weights: ddit_step_weights, io: ddit_io_weights, z, y, y_valid_len, y_uncond,
                guidance: float, n_steps: int, first_step: int, last_step: int, eps_scratch, workspace,
                cross_kv=None, cross_kv_uncond=None) -> None:
    _check(_lib.ddit_sample(C.byref(shape), C.byref(weights), C.byref(io), _ptr(z), _ptr(y), _i32(y_valid_len),
                            _ptr(y_uncond), _ptr(cross_kv), _ptr(cross_kv_uncond), guidance, n_steps, first_step,
                            last_step, _ptr(eps_scratch), _ptr(workspace), _nbytes(workspace), _stream()))


def ddit_probe_mfma_bf16(operands, sink, iters: int) -> float:
    """-> floating-point operations of the launch."""
    fl = C.c_double(0.0)
    _check(_lib.ddit_probe_mfma_bf16(_ptr(operands), _ptr(sink), iters, C.byref(fl), _stream()))
    return fl.value


def ddit_probe_stream_copy(src, dst, nbytes: int) -> None:
    _check(_lib.ddit_probe_stream_copy(_ptr(src), _ptr(dst), nbytes, _stream()))


def ddit_probe_stream_read(src, nbytes: int, sink) -> None:
    _check(_lib.ddit_probe_stream_read(_ptr(src), nbytes, _ptr(sink), _stream()))


def ddit_probe_residual_stream(x, xh_out, o, gate, N: int, D: int, A: int) -> None:
    _check(_lib.ddit_probe_residual_stream(_ptr(x), _ptr(xh_out), _ptr(o), _ptr(gate), N, D, A, _stream()))


# ----------------------------------------------------------------------------- helpers (no arithmetic)
def alloc_workspace(shape: ddit_shape, device="cuda") -> torch.Tensor:
    return torch.empty(ddit_workspace_bytes(shape), dtype=torch.uint8, device=device)


def read_tap(shape: ddit_shape, workspace: torch.Tensor, layer: int, name: str) -> torch.Tensor:
    """View of one tap region of the workspace as a flat tensor of its dtype."""
    off, nb = ddit_tap_region(shape, layer, TAP_NAMES.index(name))
    raw = workspace[off:off + nb]
    return raw.view(_TAP_DTYPE.get(name, torch.bfloat16))
