"""Host-side tests of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments with the documented status codes before anything is
enqueued (so no HIP call happens on these paths)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2506_13497_amd", "libddit_hot.so")
HEADER = os.path.join(ROOT, "include", "ddit_hot.h")



@pytest.fixture(scope="module", autouse=True)
def _library_is_built():
    # a missing library is a failure of the build, not a reason to skip: nothing below can be trusted without it
    assert os.path.exists(LIB), "libddit_hot.so is not built: run __graft_entry__.build() (or python -m paper_2506_13497_amd.build)"


@pytest.fixture(scope="module")
def m():
    import paper_2506_13497_amd as mod
    return mod


def _declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(ddit_[a-z_0-9]+)\s*\(", src)))


def test_library_exports_every_declared_symbol(m):
    lib = C.CDLL(LIB)
    names = _declared_functions()
    assert {"ddit_attn_fwd", "ddit_stdit_block_fwd", "ddit_denoise_step"} <= set(names)
    for n in names:
        assert hasattr(lib, n), "missing export " + n
    assert sorted(m.binding.EXPORTS) == names
    assert m.ddit_abi_version() == 7


def test_status_strings(m):
    assert m.ddit_status_string(0) == "ok"
    for code in (-1, -2, -3, -4, -5):
        assert m.ddit_status_string(code) not in ("ok", "unknown status")
    assert m.ddit_status_string(-99) == "unknown status"


def _shape(m, **kw):
    d = dict(B=1, T=4, Hp=8, Wp=8, D=256, H=4, dh=64, M=1024, Ly=16, n_blocks=1)
    d.update(kw)
    return m.make_shape(**d)


def test_workspace_bytes_and_layout_monotone(m):
    small = m.ddit_workspace_bytes(_shape(m))
    big = m.ddit_workspace_bytes(_shape(m, T=8))
    taps = m.ddit_workspace_bytes(_shape(m, flags=m.DDIT_FLAG_TAPS))
    assert 0 < small < big and taps > small
    # the fixed part: x fp32 + xh + qkv + o + kvc + h (+ conditioning), each 256-byte aligned
    N, D, A, M_, Ly = 256, 256, 256, 1024, 16
    lower = N * D * 4 + N * D * 2 + N * 3 * A * 2 + N * A * 2 + Ly * 2 * A * 2 + N * M_ * 2
    assert lower <= small <= lower + 64 * 1024
    off, nb = m.ddit_tap_region(_shape(m, flags=m.DDIT_FLAG_TAPS), 1, m.TAP_NAMES.index("h"))
    assert nb == N * M_ * 2 and off % 256 == 0 and off + nb <= taps


@pytest.mark.parametrize("kw,code", [
    (dict(dh=80), -2), (dict(H=8, dh=64), -2), (dict(D=250), -2), (dict(B=0), -1), (dict(Ly=0), -1),
    (dict(B=65), -2), (dict(D=8192, H=4), -2),
    # 5 samples of the 720p shape: 540000 tokens x 4608 passes 2^31, which the linears' 31-bit indices cannot hold;
    # refused here, before any layer's kernels are enqueued
    (dict(B=5, T=30, Hp=45, Wp=80, D=1152, H=16, dh=72, M=4608, Ly=300, n_blocks=28), -2),
    (dict(B=64, T=30, Hp=45, Wp=80, D=1152, H=4, dh=72, M=4608, Ly=300), -2),
    (dict(M=1 << 24), -2),
])
def test_bad_shapes_are_rejected(m, kw, code):
    with pytest.raises(m.binding.DditError) as e:
        m.ddit_workspace_bytes(_shape(m, **kw))
    assert e.value.status == code and len(str(e.value)) > 20


def test_struct_size_versions_the_shape(m):
    sh = _shape(m)
    sh.struct_size = 12
    with pytest.raises(m.binding.DditError) as e:
        m.ddit_workspace_bytes(sh)
    assert e.value.status == -1 and "struct_size" in str(e.value)


def test_tap_region_needs_flag(m):
    with pytest.raises(m.binding.DditError) as e:
        m.ddit_tap_region(_shape(m), 0, 0)
    assert e.value.status == -1


class _FakeTensor:
    """Stands in for a device tensor on the validation-only paths: just an address and a size."""
    def __init__(self, addr, nbytes=1 << 20):
        self._a, self._n = addr, nbytes

    def data_ptr(self):
        return self._a

    def numel(self):
        return self._n

    def element_size(self):
        return 1


def _call_attn(m, q=0x10000, k=0x20000, v=0x30000, o=0x40000, ld=256, valid=None, kind=0, shape=None):
    lib = m.binding._lib
    sh = shape or _shape(m)
    vl = None if valid is None else (C.c_int32 * len(valid))(*valid)
    return lib.ddit_attn_fwd(kind, C.byref(sh), C.c_void_p(q), C.c_void_p(k), C.c_void_p(v), ld, ld, vl,
                             C.c_void_p(o), ld, None, None, 0, None)


def test_attn_argument_validation_happens_before_any_launch(m):
    assert _call_attn(m, q=0) == -1                       # NULL pointer
    assert _call_attn(m, q=0x10008) == -4                 # misaligned
    assert _call_attn(m, ld=128) == -1                    # leading dimension below H*dh
    assert _call_attn(m, ld=260) == -4                    # not a multiple of 8
    assert _call_attn(m, kind=7) == -1
    assert _call_attn(m, kind=2, valid=[0]) == -1         # valid_len below 1
    assert _call_attn(m, kind=2, valid=[17]) == -1        # above Ly
    assert "valid_len" in m.ddit_last_error()


def test_block_and_step_validation(m):
    lib = m.binding._lib
    sh = _shape(m)
    need = m.ddit_workspace_bytes(sh)
    wb = m.binding.ddit_block_weights()
    P = C.c_void_p
    # NULL weights / c6
    assert lib.ddit_stdit_block_fwd(C.byref(sh), None, P(0x1000), P(0x2000), None, P(0x3000), P(0x4000), P(0x100000), need, None) == -1
    # workspace too small: message carries the required size
    assert lib.ddit_stdit_block_fwd(C.byref(sh), C.byref(wb), P(0x1000), P(0x2000), None, P(0x3000), P(0x4000), P(0x100000), need - 1, None) == -3
    assert str(need) in m.ddit_last_error()
    # NULL workspace
    assert lib.ddit_stdit_block_fwd(C.byref(sh), C.byref(wb), P(0x1000), P(0x2000), None, P(0x3000), P(0x4000), None, 0, None) == -3
    # workspace fine, but the (all-NULL) layer weights are rejected by name
    assert lib.ddit_stdit_block_fwd(C.byref(sh), C.byref(wb), P(0x1000), P(0x2000), None, P(0x3000), P(0x4000), P(0x100000), need, None) == -1
    assert "w_qkv" in m.ddit_last_error()
    # misaligned x_in
    assert lib.ddit_stdit_block_fwd(C.byref(sh), C.byref(wb), P(0x1004), P(0x2000), None, P(0x3000), P(0x4000), P(0x100000), need, None) == -4
    # step: NULL weights struct
    assert lib.ddit_denoise_step(C.byref(sh), None, P(0x1000), P(0x2000), None, None, None, P(0x4000), P(0x100000), need, None) == -1


def test_linear_and_layernorm_validation(m):
    lib = m.binding._lib
    P = C.c_void_p
    assert lib.ddit_linear_fwd(0, P(0x1000), 64, P(0x2000), None, 16, 64, 64, None, 64, None, None, None, -1, 1, None) == -1   # no out
    assert lib.ddit_linear_fwd(0, P(0x1000), 60, P(0x2000), None, 16, 64, 64, P(0x3000), 64, None, None, None, -1, 1, None) == -1  # ld_u < k
    assert lib.ddit_linear_fwd(0, P(0x1000), 64, P(0x2000), None, 16, 60, 64, P(0x3000), 64, None, None, None, -1, 1, None) == -2  # n % 8
    assert lib.ddit_linear_fwd(2, P(0x1000), 64, P(0x2000), None, 16, 64, 64, None, 0, None, None, None, -1, 1, None) == -1      # no resid
    assert lib.ddit_linear_fwd(2, P(0x1000), 64, P(0x2000), None, 16, 64, 64, None, 0, P(0x5000), None, None, 2, 1, None) == -1  # gate w/o table
    assert lib.ddit_linear_fwd(9, P(0x1000), 64, P(0x2000), None, 16, 64, 64, P(0x3000), 64, None, None, None, -1, 1, None) == -1
    assert lib.ddit_modulated_layernorm_fwd(P(0x1000), P(0x2000), P(0x3000), 2, 4, 4, 64, 1e-6, P(0x4000), None) == -1  # which
    assert lib.ddit_modulated_layernorm_fwd(P(0x1000), P(0x2000), P(0x3000), 0, 4, 4, 60, 1e-6, P(0x4000), None) == -2  # D % 8
    assert lib.ddit_modulated_layernorm_fwd(None, P(0x2000), P(0x3000), 0, 4, 4, 64, 1e-6, P(0x4000), None) == -1


def test_qk_norm_rope_validation_and_workspace(m):
    lib = m.binding._lib
    P = C.c_void_p
    ok = (P(0x1000), 3 * 144, 10, 2, 72, P(0x2000), P(0x3000), 1e-6, 5, 2, None, None)
    def call(**kw):
        names = ("qk", "ld", "N", "H", "dh", "g_q", "g_k", "eps", "S", "T", "tab", "stream")
        a = dict(zip(names, ok)); a.update(kw)
        return lib.ddit_qk_norm_rope_fwd(*[a[n] for n in names])
    assert call(qk=None) == -1
    assert call(dh=80) == -2
    assert call(ld=280) == -1                    # narrower than q | k
    assert call(g_k=None) == -1                  # scales come in pairs
    assert call(eps=0.0) == -1
    assert call(qk=P(0x1004)) == -4
    assert call(tab=P(0x4004)) == -4
    assert call(T=0) == -1
    # the rotary table lives in the workspace only when asked for
    plain = m.ddit_workspace_bytes(_shape(m))
    assert m.ddit_workspace_bytes(_shape(m, flags=m.DDIT_FLAG_ROPE_TEMPORAL)) > plain
    assert m.ddit_workspace_bytes(_shape(m, flags=m.DDIT_FLAG_QK_NORM)) == plain


def test_zero_tokens_is_a_successful_no_op(m):
    """The degenerate size: a stage called on zero token rows validates its arguments, enqueues nothing
    and returns OK (so it needs no GPU); bad arguments are still refused first."""
    lib = m.binding._lib
    P = C.c_void_p
    lin = lambda N, ld_u=64: lib.ddit_linear_fwd(0, P(0x1000), ld_u, P(0x2000), None, N, 64, 64, P(0x3000), 64,
                                                 None, None, None, -1, 1, None)
    assert lin(0) == 0
    assert lin(0, ld_u=60) == -1                  # a row stride shorter than k
    assert lin(-1) == -1
    ln = lambda N, x=0x1000: lib.ddit_modulated_layernorm_fwd(P(x), P(0x2000), P(0x3000), 0, N, 1, 64,
                                                              C.c_float(1e-6), P(0x4000), None)
    assert ln(0) == 0
    assert ln(0, x=0x1004) == -4                  # alignment is checked before the size
    assert ln(-1) == -1
    qk = lambda N: lib.ddit_qk_norm_rope_fwd(P(0x1000), 3456, N, 16, 72, P(0x2000), P(0x3000), C.c_float(1e-6), 1, 1,
                                             None, None)
    assert qk(0) == 0
    assert qk(-1) == -1


def test_linear_tile_list_and_cost_model(m):
    """Host side of the tile choice: the list is consistent, bad indices are refused before any
    launch, and the model's pick is the cheapest of its own prices and behaves sensibly at the
    two ends (one tile's worth of tokens -> the smallest tile; a full 480p fc1 -> the largest)."""
    lib = m.binding._lib
    P = C.c_void_p
    count = m.ddit_linear_tile_count()
    assert count >= 2
    areas, forms = [], set()
    for t in range(count):
        info = m.ddit_linear_tile_info(t)
        assert info["rows"] % 64 == 0 and info["cols"] % 32 == 0
        assert info["wavefronts"] in (4, 6, 8) and 1 <= info["workgroups_per_cu"] <= 3
        areas.append(info["rows"] * info["cols"])
        forms.add((info["rows"], info["cols"], info["workgroups_per_cu"]))
    # largest first; a tile may come in two forms that differ in how many workgroups share a CU
    assert areas == sorted(areas, reverse=True) and len(forms) == count
    for bad in (-1, count):
        with pytest.raises(m.DditError) as e:
            m.ddit_linear_tile_info(bad)
        assert e.value.status == -1
    assert lib.ddit_linear_tile_info(0, None, None, None, None) == 0           # every output is optional
    # a forced tile past the list is refused; arguments are still validated first
    args = (0, P(0x1000), 64, P(0x2000), None, 16, 64, 64, P(0x3000), 64, None, None, None, -1, 1, None)
    assert lib.ddit_linear_fwd_tile(count, *args) == -1
    assert "no tile" in m.ddit_last_error()
    assert lib.ddit_linear_fwd_tile(0, 0, P(0x1000), 60, P(0x2000), None, 16, 64, 64, P(0x3000), 64, None, None, None, -1, 1, None) == -1
    # choice
    tile = C.c_int32(-7)
    assert lib.ddit_linear_tile_choice(3, 100, 64, 64, 256, C.byref(tile), None) == -1
    assert lib.ddit_linear_tile_choice(0, 100, 0, 64, 256, C.byref(tile), None) == -1
    assert lib.ddit_linear_tile_choice(0, 100, 64, 64, 256, None, None) == -1
    for epi in (0, 1, 2):
        for N, n, k in [(1, 8, 8), (64, 128, 1152), (2304, 1152, 4608), (3680, 3456, 1152), (48600, 4608, 1152),
                        (13001, 864, 1160)]:
            t, us = m.ddit_linear_tile_choice(epi, N, n, k, 256)
            assert 0 <= t < count and len(us) == count and all(x > 0 for x in us)
            assert us[t] == min(us)
        assert m.ddit_linear_tile_choice(epi, 64, 128, 1152, 256)[0] == count - 1
        assert m.ddit_linear_tile_choice(epi, 48600, 4608, 1152, 256)[0] == 0
        # more tokens never cost less, whatever the tile
        prev = [0.0] * count
        for N in (1, 100, 1000, 3000, 9000, 27000, 81000):
            us = m.ddit_linear_tile_choice(epi, N, 1152, 1152, 256)[1]
            assert all(a >= b for a, b in zip(us, prev))
            prev = us
    # fewer CUs: the same problem spreads over more rounds, so no tile gets cheaper
    a = m.ddit_linear_tile_choice(0, 20000, 1152, 1152, 256)[1]
    b = m.ddit_linear_tile_choice(0, 20000, 1152, 1152, 64)[1]
    assert all(y >= x for x, y in zip(a, b))


def _io(m, **kw):
    d = dict(C_in=4, C_out=4, C_text=64)
    d.update(kw)
    io = m.binding.ddit_io_weights()
    io.struct_size = C.sizeof(m.binding.ddit_io_weights)
    io.C_in, io.C_out, io.C_text = d["C_in"], d["C_out"], d["C_text"]
    return io


def test_io_workspace_and_cache_sizes(m):
    sh = _shape(m)
    step = m.ddit_workspace_bytes(sh)
    total = m.ddit_io_workspace_bytes(sh, _io(m))
    N, D, S, Ly = 256, 256, 64, 16
    extra = S * D * 4 + 2 * N * D * 2 + Ly * D * 2
    assert step + extra <= total <= step + extra + 64 * 1024
    assert m.ddit_cross_kv_bytes(_shape(m, n_blocks=3)) == 2 * 3 * Ly * 2 * 256 * 2


@pytest.mark.parametrize("kw,code", [(dict(C_in=17), -2), (dict(C_out=0), -1), (dict(C_text=60), -2)])
def test_bad_io_weights_are_rejected(m, kw, code):
    with pytest.raises(m.binding.DditError) as e:
        m.ddit_io_workspace_bytes(_shape(m), _io(m, **kw))
    assert e.value.status == code


def test_io_struct_size_and_sample_ranges(m):
    lib = m.binding._lib
    sh = _shape(m)
    io = _io(m)
    io.struct_size = 8
    n = C.c_size_t(0)
    assert lib.ddit_io_workspace_bytes(C.byref(sh), C.byref(io), C.byref(n)) == -1
    assert "struct_size" in m.ddit_last_error()
    io = _io(m)
    sw = m.binding.ddit_step_weights()
    P = C.c_void_p
    args = lambda n_steps, first, last, z=0x1000: (C.byref(sh), C.byref(sw), C.byref(io), P(z), P(0x2000), None, None, None, None,
                                                   C.c_float(1.0), n_steps, first, last, P(0x3000), P(0x100000), 1 << 30, None)
    assert lib.ddit_sample(*args(0, 0, 0)) == -1          # no steps
    assert lib.ddit_sample(*args(4, 3, 2)) == -1          # range reversed
    assert lib.ddit_sample(*args(4, 0, 5)) == -1          # past the end
    assert lib.ddit_sample(*args(4, 0, 1, z=0)) == -1     # NULL latent
    assert lib.ddit_sample(*args(4, 2, 2)) == 0           # an empty range does nothing
    # solver step: B outside 1..64, NULL pointers
    assert lib.ddit_solver_step(P(0x1000), P(0x2000), None, C.c_float(1.0), (C.c_float * 1)(1.0), (C.c_float * 1)(0.0), 0, 10, None) == -1
    assert lib.ddit_solver_step(None, P(0x2000), None, C.c_float(1.0), (C.c_float * 1)(1.0), (C.c_float * 1)(0.0), 1, 10, None) == -1
    # cache precompute: NULL y
    assert lib.ddit_cross_kv_precompute(C.byref(sh), C.byref(sw), None, P(0x1000), None) == -1


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in r.stderr
