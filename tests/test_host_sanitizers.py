"""The library's host code under AddressSanitizer and UndefinedBehaviorSanitizer, on the CPU.

Every source of the library is compiled again with the two sanitizers on its HOST code only (the device
code is untouched; sanitizers never run on the GPU) and linked with a small driver
(tests/host_checks_main.cpp) into one executable.  The driver is fed seeded scheduler workloads, allocator
operation sequences, rows of step times, shapes and linear problems; it calls the host-only entry points and
the validation paths of the GPU entry points, none of which makes a HIP call.  A sanitizer report aborts the
run (and fails the test); what the driver prints must equal the oracle's results (scheduler, allocator,
optimal parallel size) and the ordinary build's answers (sizes, tap regions, statuses, tile prices).
No GPU needed."""
import os
import random
import subprocess
import sys

import pytest

from oracle import sched_oracle as so
from test_oracle_pins_sched import random_case

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2506_13497_amd")
SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
       "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]


def _load_build():
    import importlib.util
    spec = importlib.util.spec_from_file_location("_ddit_build_for_san", os.path.join(PKG, "build.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


@pytest.fixture(scope="module")
def exe(tmp_path_factory):
    b = _load_build()
    out = os.path.join(PKG, "_build", "san")
    os.makedirs(out, exist_ok=True)
    path = os.path.join(out, "host_checks")
    hipcc = b._hipcc()
    from concurrent.futures import ThreadPoolExecutor

    def compile_one(src):
        obj = os.path.join(out, src.replace(".hip", ".o"))
        cmd = [hipcc, *b.FLAGS, *SAN, "-c", os.path.join(b.CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, "sanitizer build of %s failed:\n%s" % (src, r.stderr[-3000:])
        return obj
    with ThreadPoolExecutor(max_workers=min(8, len(b.SOURCES))) as ex:
        objs = list(ex.map(compile_one, b.SOURCES))
    main_obj = os.path.join(out, "host_checks_main.o")
    main_cmd = [hipcc, "-fno-gpu-sanitize", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-O1", "-g", "-std=c++17", "-x", "c++"]
    r = subprocess.run(main_cmd + ["-c", os.path.join(ROOT, "tests", "host_checks_main.cpp"), "-o", main_obj], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    link_cmd = [hipcc, "-fno-gpu-sanitize", "-fsanitize=address,undefined", "--offload-arch=gfx950", "-o", path, main_obj, *objs]
    r = subprocess.run(link_cmd, capture_output=True, text=True)
    assert r.returncode == 0, "link failed:\n" + r.stderr[-3000:]
    return path


def _run(exe, text, tmp_path):
    cmds = tmp_path / "commands.txt"
    cmds.write_text(text)
    supp = tmp_path / "lsan.supp"
    # the HIP runtime keeps process-lifetime allocations of its own; leaks of this library's code are still reported
    supp.write_text("leak:libamdhip64\nleak:libhsa-runtime64\nleak:libamd_comgr\nleak:librocprofiler\nleak:libdrm\n")
    env = dict(os.environ, ASAN_OPTIONS="abort_on_error=0:halt_on_error=1:detect_leaks=1:exitcode=99",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1", LSAN_OPTIONS="suppressions=%s:print_suppressions=0" % supp)
    r = subprocess.run([exe, str(cmds)], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0, "exit %d\nstdout tail:\n%s\nstderr tail:\n%s" % (r.returncode, r.stdout[-1500:], r.stderr[-4000:])
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-4000:]
    lines = r.stdout.strip().splitlines()
    assert lines[-1] == "done"
    return lines[1:-1]


def _sched_text(case, max_events):
    R, K = len(case["step_us"]), len(case["step_us"][0])
    vae = case.get("vae_us")
    t = ["SCHED %d %d %d %d %d %d %d" % (case["n_gpus"], case["n_steps"], R, K, case.get("vae_gpus", 1), 1 if vae else 0, max_events)]
    t.append(" ".join(str(int(v)) for row in case["step_us"] for v in row))
    t.append(" ".join(str(int(v)) for v in case["opt_dop"]))
    if vae:
        t.append(" ".join(str(int(v)) for v in vae))
    t.append(str(len(case["requests"])))
    t += ["%d %d" % (a, r) for a, r in case["requests"]]
    return "\n".join(t) + "\n"


def test_scheduler_allocator_and_dop_under_sanitizers_equal_the_oracle(exe, tmp_path):
    cases, text = [], ""
    for seed in range(24):
        case = random_case(3000 + seed, n_gpus=[1, 2, 4, 8, 16, 64][seed % 6], n=[0, 1, 9, 70, 150][seed % 5])
        rec, ev, tot = so.simulate(**case)
        cap = len(ev) if seed % 3 else max(len(ev) // 2, 0)   # every third case: an event array shorter than the log
        cases.append((case, rec, ev, tot, cap))
        text += _sched_text(case, cap)
    rng = random.Random(11)
    buddy_expect = []
    for n in (1, 8, 64, 4096):
        ref, held, ops, exp = so.Buddy(n), [], [], ["buddy create 0"]
        for _ in range(400):
            roll = rng.random()
            if held and roll < 0.4:
                st, s = held.pop(rng.randrange(len(held)))
                ref.release(st, s)
                ops.append("r %d %d" % (st, s)); exp.append("r 0")
            elif roll < 0.5:
                ops.append("f"); exp.append("f 0 %d" % ref.free_gpus())
            elif roll < 0.55:
                ops.append("r %d %d" % (rng.randrange(-2, n + 2), 3)); exp.append("r -1")   # not a block: refused
            else:
                s = 1 << rng.randrange(n.bit_length())
                got = ref.alloc(s)
                ops.append("a %d" % s); exp.append("a 0 %d" % (-1 if got is None else got))
                if got is not None:
                    held.append((got, s))
        exp.append("buddy destroy 0")
        text += "BUDDY %d %d\n%s\n" % (n, len(ops), "\n".join(ops))
        buddy_expect.append(exp)
    dop_rows = []
    for _ in range(200):
        k = rng.randrange(1, 8)
        row = [rng.randrange(1, 10 ** 9) for _ in range(k)]
        dop_rows.append(row)
        text += "DOP %d 0 1 %s\n" % (k, " ".join(map(str, row)))
    dop_rows.append([1 << 40, (1 << 40) - 1, (1 << 39) + 1, 1])
    text += "DOP 4 0 1 %s\n" % " ".join(map(str, dop_rows[-1]))
    out = _run(exe, text, tmp_path)
    i = 0
    for case, rec, ev, tot, cap in cases:
        assert out[i] == "sched rc 0"; i += 1
        for r in rec:
            assert out[i] == "rec %d %d %d %d %d %d %d" % (r["start_us"], r["dit_end_us"], r["end_us"], r["first_dop"], r["final_dop"],
                                                           r["promotions"], r["starvation"]), (i, out[i], r)
            i += 1
        kinds = {"start": 0, "promote": 1, "dit_done": 2, "release": 3}
        for e in ev[:cap]:
            assert out[i] == "ev %d %d %d %d %d" % (e[0], kinds[e[1]], e[2], e[3], e[4]); i += 1
        assert out[i] == "tot %d %d %d" % (tot["occupancy_gpu_us"], tot["makespan_us"], len(ev)); i += 1
    for exp in buddy_expect:
        assert out[i:i + len(exp)] == exp
        i += len(exp)
    for row in dop_rows:
        assert out[i] == "dop 0 %d" % so.optimal_dop(row); i += 1
    assert i == len(out)


def test_validation_and_layout_under_sanitizers_equal_the_ordinary_build(exe, tmp_path):
    import ctypes as C
    import paper_2506_13497_amd as m
    shapes = [  # flags B T Hp Wp D H dh M Ly n_blocks
        (0, 1, 4, 8, 8, 256, 4, 64, 1024, 16, 1), (1, 1, 4, 8, 8, 256, 4, 64, 1024, 16, 1), (5, 2, 3, 5, 7, 1152, 16, 72, 4608, 300, 1),
        (0, 1, 30, 30, 54, 1152, 16, 72, 4608, 300, 28), (1, 1, 30, 45, 80, 1152, 4, 72, 4608, 300, 28),
        (0, 64, 1, 1, 1, 8, 0, 64, 8, 1, 0), (0, 1, 1, 1, 1, 64, 1, 64, 8, 1, 0), (0, 1, 4, 8, 8, 256, 4, 80, 1024, 16, 1),
        (0, 5, 30, 45, 80, 1152, 16, 72, 4608, 300, 28), (0, 65, 1, 1, 1, 64, 1, 64, 8, 1, 1), (0, 1, 1, 1, 1, 4104, 1, 64, 8, 1, 1),
        (0, 1, 1, 1, 1, 64, 1, 64, 1 << 24, 1, 1), (0, 1, 32768, 32768, 2, 64, 1, 64, 8, 1, 1),
    ]
    linears = [(e, N, n, k, cu) for e in (0, 1, 2) for N, n, k in ((48600, 1152, 1152), (2304, 4608, 1152), (300, 2304, 1152), (0, 8, 8),
                                                                       (108000, 864, 1152)) for cu in (256, 0, 304)]
    text = "".join("SHAPE %s\n" % " ".join(map(str, s)) for s in shapes) + "".join("LINEAR %d %d %d %d %d\n" % l for l in linears)
    out = _run(exe, text, tmp_path)
    # the same questions to the ordinary build, through ctypes
    lib = m.binding._lib
    i = 0
    for s in shapes:
        shp = m.make_shape(*s[1:], flags=s[0])
        n = C.c_size_t(0)
        rc = lib.ddit_workspace_bytes(C.byref(shp), C.byref(n))
        assert out[i] == "shape ws %d %d" % (rc, n.value if rc == 0 else 0), (s, out[i]); i += 1
        rc = lib.ddit_cross_kv_bytes(C.byref(shp), C.byref(n))
        assert out[i] == "shape kv %d %d" % (rc, n.value if rc == 0 else 0); i += 1
        if s[0] & 1:
            for layer in range(2):
                for t in range(len(m.TAP_NAMES)):
                    off, nb = C.c_size_t(0), C.c_size_t(0)
                    rc = lib.ddit_tap_region(C.byref(shp), layer, t, C.byref(off), C.byref(nb))
                    assert out[i] == "tap %d %d %d %d %d" % (layer, t, rc, off.value if rc == 0 else 0, nb.value if rc == 0 else 0); i += 1
        assert out[i].startswith("shape io "); i += 1
        statuses = {}
        while i < len(out) and out[i].startswith("v "):
            _, name, rc = out[i].split(); statuses[name] = int(rc); i += 1
        ok = lib.ddit_workspace_bytes(C.byref(shp), C.byref(n)) == 0
        assert len(statuses) == 13 and all(v < 0 for v in statuses.values()), statuses   # every call is refused ...
        if ok:                                                                          # ... for the reason it was built to be
            assert statuses["block_null"] == -1 and statuses["block_ws"] == -3 and statuses["attn_null"] == -1
            assert statuses["attn_len"] == -1 and statuses["attn_kind"] == -1 and statuses["eps_ws"] == -3
            assert statuses["sample_steps"] == -1 and statuses["kv_null"] == -1
        else:
            assert len(set(statuses.values()) - {statuses["block_null"]}) <= 1
    for e, N, n_, k, cu in linears:
        tile, us = m.ddit_linear_tile_choice(e, N, n_, k, cu)
        got = out[i].split(); i += 1
        assert got[:3] == ["tile", "0", str(tile)]
        assert [float(v) for v in got[3:]] == pytest.approx(us, rel=1e-4)
        assert out[i:i + 4] == ["v linear_null -1", "v linear_dims -2", "v linear_align -4", "v linear_zero_rows 0"]; i += 4
    assert i == len(out)
