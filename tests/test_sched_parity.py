"""The library's host-side scheduling calls against the oracle (oracle/sched_oracle.py): exact
agreement (integer microseconds) of the optimal degree of parallelism, the buddy allocator and
the whole event simulation, on hand cases, seeded random workloads and a table of step times
measured for this library.  No GPU needed: these entry points make no HIP call."""
import ctypes as C
import os
import random
from fractions import Fraction

import pytest

from oracle import sched_oracle as so
from test_oracle_pins_sched import check_invariants, random_case

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2506_13497_amd", "libddit_hot.so")

@pytest.fixture(scope="module", autouse=True)
def _library_is_built():
    assert os.path.exists(LIB), "libddit_hot.so is not built: run __graft_entry__.build()"



@pytest.fixture(scope="module")
def m():
    import paper_2506_13497_amd as mod
    return mod


def run_both(m, case):
    rec, ev, tot = so.simulate(**case)
    grec, gev, gtot = m.ddit_sched_simulate(case["n_gpus"], case["n_steps"], case["step_us"], case["opt_dop"],
                                            case["requests"], case.get("vae_us"), case.get("vae_gpus", 1))
    assert gtot.pop("n_events") == len(ev)
    return (rec, ev, tot), (grec, gev, gtot)


@pytest.mark.parametrize("seed", range(40))
def test_simulation_equals_oracle_on_random_workloads(m, seed):
    case = random_case(1000 + seed, n_gpus=[1, 2, 4, 8, 8, 16, 64][seed % 7], n=[0, 1, 7, 60, 200][seed % 5])
    ora, got = run_both(m, case)
    assert got[0] == ora[0], "records differ"
    assert got[1] == ora[1], "event logs differ"
    assert got[2] == ora[2]
    if case["requests"]:
        check_invariants(case, *got)


# step times (microseconds) of this library on one MI355X by resolution (144p, 240p, 360p, 480p, 720p)
# and parallel size 1, 2, 4, 8: compute plus the modelled exchange of the all-to-alls
MEASURED_US = [[13680, 11820, 10240, 9730], [24360, 18720, 12250, 10590], [46660, 34240, 19750, 13890],
               [146090, 103650, 51940, 28510], [362990, 247950, 118340, 59290]]


def test_paper_style_workload_on_the_measured_table(m):
    """Eight GPUs, 30 steps, exponential arrivals, a mix of resolutions (the shape of the paper's
    section 6.1 workload), B from the table itself."""
    B = [so.optimal_dop(row) for row in MEASURED_US]
    assert B == [m.ddit_optimal_dop(row) for row in MEASURED_US]
    rng = random.Random(7)
    for rate_per_s in (0.25, 1.0, 4.0):
        t, reqs = 0.0, []
        for _ in range(120):
            t += rng.expovariate(rate_per_s) * 1e6
            reqs.append((int(t), rng.choices([0, 1, 2], weights=[5, 3, 2])[0]))
        case = dict(n_gpus=8, n_steps=30, step_us=MEASURED_US, opt_dop=B, requests=reqs, vae_us=[40000, 90000, 200000, 0, 0], vae_gpus=1)
        ora, got = run_both(m, case)
        assert got == ora
        check_invariants(case, *got)
    burst = dict(n_gpus=8, n_steps=30, step_us=MEASURED_US, opt_dop=B, requests=[(0, i % 3) for i in range(50)])
    ora, got = run_both(m, burst)
    assert got == ora


def test_event_log_truncation(m):
    case = random_case(5, n=30)
    rec, ev, tot = so.simulate(**case)
    grec, gev, gtot = m.ddit_sched_simulate(case["n_gpus"], case["n_steps"], case["step_us"], case["opt_dop"], case["requests"],
                                            case["vae_us"], case["vae_gpus"], max_events=10)
    assert gev == ev[:10] and gtot["n_events"] == len(ev) and grec == rec
    grec, gev, gtot = m.ddit_sched_simulate(case["n_gpus"], case["n_steps"], case["step_us"], case["opt_dop"], case["requests"],
                                            case["vae_us"], case["vae_gpus"], max_events=0)
    assert gev == [] and grec == rec and gtot["occupancy_gpu_us"] == tot["occupancy_gpu_us"]


def test_optimal_dop_equals_oracle(m):
    rng = random.Random(3)
    for _ in range(500):
        k = rng.randrange(1, 6)
        row = [rng.randrange(1, 50) if rng.random() < 0.3 else rng.randrange(1, 10 ** 9) for _ in range(k)]
        num, den = rng.choice([(0, 1), (1, 4), (1, 3), (9, 10), (rng.randrange(0, 100), 100)])
        assert m.ddit_optimal_dop(row, num, den) == so.optimal_dop(row, Fraction(num, den)), (row, num, den)
    big = [1 << 40, (1 << 40) - 1, (1 << 39) + 1, 1]          # products that need more than 64 bits
    assert m.ddit_optimal_dop(big) == so.optimal_dop(big)


@pytest.mark.parametrize("n,seed", [(1, 0), (8, 1), (16, 2), (256, 3)])
def test_buddy_pool_equals_oracle(m, n, seed):
    rng = random.Random(seed)
    pool, ref, held = m.ddit_buddy_create(n), so.Buddy(n), []
    try:
        for _ in range(800):
            if held and rng.random() < 0.45:
                st, s = held.pop(rng.randrange(len(held)))
                m.ddit_buddy_release(pool, st, s)
                ref.release(st, s)
            else:
                s = 1 << rng.randrange(n.bit_length())
                want = ref.alloc(s)
                got = m.ddit_buddy_alloc(pool, s)
                assert got == (-1 if want is None else want)
                if want is not None:
                    held.append((want, s))
            assert m.ddit_buddy_free_gpus(pool) == ref.free_gpus()
    finally:
        m.ddit_buddy_destroy(pool)


def test_argument_validation(m):
    lib = m.binding._lib
    pool = m.ddit_buddy_create(8)
    try:
        assert m.ddit_buddy_alloc(pool, 4) == 0
        for start, size in ((0, 3), (1, 2), (8, 1), (-1, 1), (0, 16)):
            with pytest.raises(m.DditError):
                m.ddit_buddy_release(pool, start, size)           # not an aligned block of the pool
        with pytest.raises(m.DditError):
            m.ddit_buddy_release(pool, 4, 4)                      # free already
        with pytest.raises(m.DditError):
            m.ddit_buddy_release(pool, 0, 8)                      # only half of it is allocated
        with pytest.raises(m.DditError):
            m.ddit_buddy_alloc(pool, 3)
        m.ddit_buddy_release(pool, 0, 4)
        assert m.ddit_buddy_free_gpus(pool) == 8
    finally:
        m.ddit_buddy_destroy(pool)
    with pytest.raises(m.DditError):
        m.ddit_buddy_create(12)
    ok = dict(n_gpus=4, n_steps=2, step_us=[[9, 6, 4]], opt_dop=[2], requests=[(0, 0), (3, 0)])
    m.ddit_sched_simulate(**ok)
    for bad in (dict(n_gpus=6), dict(n_steps=0), dict(opt_dop=[3]), dict(opt_dop=[8]), dict(step_us=[[9, 0, 4]]),
                dict(requests=[(5, 0), (3, 0)]), dict(requests=[(0, 1)]), dict(requests=[(-1, 0)]), dict(vae_gpus=3),
                dict(n_gpus=2), dict(vae_us=[-1])):
        with pytest.raises(m.DditError) as e:
            m.ddit_sched_simulate(**dict(ok, **bad))
        assert e.value.status == m.DDIT_ERR_INVALID_ARG, bad
    cfg = m.binding.ddit_sched_config()
    cfg.struct_size = 4
    assert lib.ddit_sched_simulate(C.byref(cfg), None, 0, None, None, 0, None, None) == -1
    assert lib.ddit_sched_simulate(None, None, 0, None, None, 0, None, None) == -1
    assert lib.ddit_optimal_dop(None, 1, 0, 1, None) == -1
    with pytest.raises(m.DditError):
        m.ddit_optimal_dop([5, 4], 1, 0)
    with pytest.raises(m.DditError):
        m.ddit_optimal_dop([5, 0])


def test_request_count_is_bounded(m):
    """More requests than the documented bound are refused up front (status, not an exception or an
    unbounded host allocation)."""
    lib = m.binding._lib
    step = (C.c_int64 * 1)(5)
    opt = (C.c_int32 * 1)(1)
    cfg = m.binding.ddit_sched_config(C.sizeof(m.binding.ddit_sched_config), 1, 1, 1, 1, 1, step, opt, None)
    assert lib.ddit_sched_simulate(C.byref(cfg), None, (1 << 22) + 1, None, None, 0, None, None) == m.DDIT_ERR_UNSUPPORTED
    assert "at most" in m.ddit_last_error()


def _paper_printed():
    """key -> value of tests/golden/paper_printed_values.txt (the few numbers the paper prints)."""
    out = {}
    for line in open(os.path.join(ROOT, "tests", "golden", "paper_printed_values.txt")):
        line = line.split("#", 1)[0].strip()
        if line:
            k, v = line.split("=")
            out[k.strip()] = float(v)
    return out


def test_paper_printed_B_and_step_count_on_the_measured_table(m):
    """The paper prints B = 1, 2, 4 for 144p, 240p, 360p (section 4.2.3) and 30 denoising steps (section 6.1), found
    on its own hardware.  On this library's measured table the same rule (largest change rate z) gives 2, 4, 4: one
    MI355X is further from saturation at the low resolutions than the paper's GPU, so a doubling still pays where the
    paper's no longer did.  Both sets of B drive the same scheduler: the library must agree with the oracle event for
    event under either, and the paper's smaller groups must occupy no more GPU time per request."""
    pv = _paper_printed()
    paper_B = [int(pv["optimal_dop_144p"]), int(pv["optimal_dop_240p"]), int(pv["optimal_dop_360p"])]
    steps = int(pv["denoising_steps"])
    assert paper_B == [1, 2, 4] and steps == 30
    ours_B = [so.optimal_dop(row) for row in MEASURED_US[:3]]
    assert ours_B == [m.ddit_optimal_dop(row) for row in MEASURED_US[:3]] == [2, 4, 4]
    assert all(p <= o for p, o in zip(paper_B, ours_B))
    rng = random.Random(30)
    t, reqs = 0.0, []
    for _ in range(90):
        t += rng.expovariate(2.0) * 1e6
        reqs.append((int(t), rng.randrange(3)))
    occ = {}
    for name, B in (("paper", paper_B), ("ours", ours_B)):
        case = dict(n_gpus=8, n_steps=steps, step_us=MEASURED_US[:3], opt_dop=B, requests=reqs, vae_us=[0, 0, 0], vae_gpus=1)
        ora, got = run_both(m, case)
        assert got == ora, name
        check_invariants(case, *got)
        occ[name] = got[2]["occupancy_gpu_us"]
    assert occ["paper"] <= occ["ours"]      # smaller groups: less GPU time in total (Amdahl), at longer latency
