"""The entry point that allocates nothing: ddit_stdit_block_fwd_static keeps the block's workspace
in a device array built into the library.  Checked through the C ABI against ddit_stdit_block_fwd
(caller-owned workspace; same kernels, so the two outputs must be bit-identical) and against the
CPU oracle at the parity bar, on two calls in a row, the second on a smaller input: the built-in
array then still holds the first call's contents."""
import numpy as np
import pytest
import torch

import ddit_synth as syn
from helpers import assert_parity, dev_to_f64, dict_dev, dict_f64, to_dev, to_f64
from oracle import stdit_oracle as ora

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lib():
    import paper_2506_13497_amd as m
    assert torch.cuda.is_available()
    return m


def _shape(lib, sh, flags=0):
    return lib.make_shape(sh.B, sh.T, sh.Hp, sh.Wp, sh.D, sh.H, sh.dh, sh.M, sh.Ly, sh.n_blocks, flags)


def _both(lib, sh, base, valid):
    """-> (output of the static entry point, output of the workspace entry point, oracle), same inputs."""
    wb = syn.make_block_weights(sh, base, 0)
    act = syn.make_activations(sh, base)
    c6 = syn.make_c6(sh, base, std=0.5)
    shape = _shape(lib, sh)
    assert lib.ddit_workspace_bytes(shape) <= lib.DDIT_STATIC_SCRATCH_BYTES
    dwb = dict_dev(wb)
    st = lib.block_struct(dwb)
    x, y, c6d = to_dev(act["x"]), to_dev(act["y"]), to_dev(c6)
    vl = None if valid is None else list(valid)
    out_static = torch.full((sh.B, sh.T, sh.S, sh.D), float("nan"), dtype=torch.bfloat16, device="cuda")
    lib.ddit_stdit_block_fwd_static(shape, st, x, y, vl, c6d, out_static)
    torch.cuda.synchronize()
    ws = lib.alloc_workspace(shape)
    out_ws = torch.full_like(out_static, float("nan"))
    lib.ddit_stdit_block_fwd(shape, st, x, y, vl, c6d, out_ws, ws)
    torch.cuda.synchronize()
    ref = ora.block_fwd(to_f64(act["x"]), to_f64(act["y"]), valid, c6.astype(np.float64), dict_f64(wb), sh.H, sh.dh)
    return out_static, out_ws, ref


def test_static_scratch_block_twice_second_smaller(lib):
    # first call: ragged batch-2 shape at the model's width (S = 35, T = 3), masked text
    big = syn.Shape(2, 3, 5, 7, 1152, 16, 72, 4608, 300, 1)
    a, b, ref = _both(lib, big, 31, [45, 300])
    assert torch.equal(a.view(torch.int16), b.view(torch.int16)), "static-scratch block differs from the workspace block"
    assert_parity(dev_to_f64(a), ref, "static-scratch block, first call")
    # second call: a smaller input (fewer frames and locations, shorter text) on the same GPU's array
    small = syn.Shape(1, 2, 3, 5, 1152, 16, 72, 4608, 64, 1)
    a2, b2, ref2 = _both(lib, small, 32, [17])
    assert torch.equal(a2.view(torch.int16), b2.view(torch.int16)), "second (smaller) call differs"
    assert_parity(dev_to_f64(a2), ref2, "static-scratch block, second call")


def test_static_scratch_limit_and_flags_are_refused(lib):
    too_big = syn.Shape(1, 30, 30, 54, 1152, 16, 72, 4608, 300, 1)   # 480p: 1.3 GB of workspace
    shape = _shape(lib, too_big)
    assert lib.ddit_workspace_bytes(shape) > lib.DDIT_STATIC_SCRATCH_BYTES
    dummy = torch.zeros(64, dtype=torch.bfloat16, device="cuda")
    wb = dict_dev(syn.make_block_weights(syn.CONFIGS["C1"]["shape"], 1, 0))
    st = lib.block_struct(wb)
    with pytest.raises(lib.binding.DditError) as e:
        lib.ddit_stdit_block_fwd_static(shape, st, dummy, dummy, None, dummy.float(), dummy)
    assert e.value.status == lib.DDIT_ERR_WORKSPACE and "holds" in str(e.value)
    c1 = syn.CONFIGS["C1"]["shape"]
    with pytest.raises(lib.binding.DditError) as e:
        lib.ddit_stdit_block_fwd_static(_shape(lib, c1, lib.DDIT_FLAG_TAPS), st, dummy, dummy, None, dummy.float(), dummy)
    assert e.value.status == lib.DDIT_ERR_UNSUPPORTED
