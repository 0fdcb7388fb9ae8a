"""Shared test helpers: widen the seeded bf16 bit patterns for the fp64 oracle."""
import numpy as np

import ddit_synth as syn


def to_f64(a):
    if a.dtype == np.uint16:
        return syn.bits_to_f64(a)
    return a.astype(np.float64)


def dict_f64(d):
    return {k: (dict_f64(v) if isinstance(v, dict) else to_f64(v)) for k, v in d.items()}


def rel_fro(a, b):
    """||a-b||_F / ||b||_F in fp64."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def elem_violation(gpu, ora, atol_rel=2e-2):
    """max over elements of |gpu-ora| / (1+|ora|), to compare with 2e-2."""
    gpu = np.asarray(gpu, dtype=np.float64)
    ora = np.asarray(ora, dtype=np.float64)
    return float(np.max(np.abs(gpu - ora) / (1.0 + np.abs(ora))))


# ---- GPU-side marshalling (no arithmetic) -------------------------------------------------
def to_dev(a):
    """Seeded array -> device tensor: uint16 bf16 patterns become torch.bfloat16, fp32 stays."""
    import torch
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16).copy()).view(torch.bfloat16).cuda()
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def dict_dev(d):
    return {k: (dict_dev(v) if isinstance(v, dict) else to_dev(v)) for k, v in d.items()}


def dev_to_f64(t):
    return t.detach().double().cpu().numpy()


def assert_parity(gpu, ora, what="", elem=2e-2, fro=5e-3):
    """The parity bar: per element |gpu-ora| <= 2e-2 (1+|ora|) and relative Frobenius error <= 5e-3."""
    ev, fv = elem_violation(gpu, ora), rel_fro(gpu, ora)
    assert np.isfinite(np.asarray(gpu, dtype=np.float64)).all(), what + ": non-finite GPU output"
    assert ev <= elem, "%s: max |gpu-ora|/(1+|ora|) = %.3e > %.1e" % (what, ev, elem)
    assert fv <= fro, "%s: relative Frobenius error %.3e > %.1e" % (what, fv, fro)
    return ev, fv
