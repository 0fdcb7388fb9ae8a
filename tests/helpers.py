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
