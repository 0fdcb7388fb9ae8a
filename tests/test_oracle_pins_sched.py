"""Pins of the scheduling oracle (oracle/sched_oracle.py) against things other than itself:
hand-worked schedules, a brute-force bitmap model of the GPU pool, invariants every schedule
must satisfy, closed forms for the uncontended and the serial case, and planted mistakes.
All CPU; the paper prints no schedule, so there is no golden trace to compare with."""
from fractions import Fraction
import random

import pytest

from oracle import sched_oracle as so


# --------------------------------------------------------------------------- optimal degree of parallelism
class TestOptimalDop:
    def test_hand_examples(self):
        assert so.change_rate([100, 60, 40, 35], 2) == Fraction(2, 5)
        assert so.change_rate([100, 60, 40, 35], 4) == Fraction(1, 3)
        assert so.change_rate([100, 60, 40, 35], 8) == Fraction(1, 8)
        assert so.optimal_dop([100, 60, 40, 35]) == 2
        assert so.optimal_dop([100, 90, 50, 45]) == 4
        assert so.optimal_dop([100, 95, 90, 45]) == 8

    def test_no_gain_means_one_and_threshold(self):
        assert so.optimal_dop([100, 100, 100, 101]) == 1          # nothing gains
        assert so.optimal_dop([100, 80, 70, 65]) == 2
        assert so.optimal_dop([100, 80, 70, 65], Fraction(1, 4)) == 1   # best z = 0.2 is under the bar
        assert so.optimal_dop([100, 80, 70, 65], Fraction(1, 5)) == 1   # "exceeds" is strict

    def test_ties_go_to_the_smaller_size_and_ideal_scaling(self):
        assert so.optimal_dop([80, 40, 20, 10]) == 2              # z = 1/2 everywhere
        assert so.optimal_dop([7]) == 1                           # a table with one column

    def test_bad_sizes(self):
        for i in (0, 1, 3, 16):
            with pytest.raises(ValueError):
                so.change_rate([4, 3, 2, 1], i)


# --------------------------------------------------------------------------- buddy allocator
class Bitmap:
    """Brute-force model of the pool: one flag per GPU."""
    def __init__(self, n):
        self.busy = [False] * n

    def has_aligned_free_range(self, size):
        return any(not any(self.busy[s:s + size]) for s in range(0, len(self.busy), size))

    def mark(self, start, size, value):
        for g in range(start, start + size):
            assert self.busy[g] != value, "GPU %d %s twice" % (g, "taken" if value else "released")
            self.busy[g] = value


class TestBuddy:
    def test_hand_sequence(self):
        b = so.Buddy(8)
        assert [b.alloc(1), b.alloc(1), b.alloc(2), b.alloc(4)] == [0, 1, 2, 4]
        assert b.alloc(1) is None and b.free_gpus() == 0
        b.release(1, 1)
        assert b.alloc(2) is None                   # one free GPU is not a pair
        b.release(0, 1)                             # merges with GPU 1
        assert b.alloc(2) == 0

    def test_smallest_sufficient_block_not_lowest_address(self):
        b = so.Buddy(8)
        assert b.alloc(4) == 0
        assert b.alloc(1) == 4                      # splits (4,4): free (5,1), (6,2)
        b.release(0, 4)                             # free (0,4), (5,1), (6,2)
        assert b.alloc(2) == 6                      # the pair, not the lower half of (0,4)
        assert b.alloc(1) == 5
        assert b.alloc(4) == 0

    def test_everything_merges_back(self):
        b = so.Buddy(16)
        blocks = [(b.alloc(s), s) for s in (1, 2, 1, 4, 8)]
        assert all(st is not None for st, _ in blocks) and b.free_gpus() == 0
        for st, s in reversed(blocks):
            b.release(st, s)
        assert b.free == [[], [], [], [], [0]]

    @pytest.mark.parametrize("n,seed", [(8, 1), (8, 2), (16, 3), (64, 4), (1, 5), (2, 6)])
    def test_against_bitmap_model(self, n, seed):
        """alloc succeeds exactly when the bitmap has an aligned free range of that size; blocks are
        aligned, inside the pool and never overlap."""
        rng = random.Random(seed)
        b, bm, held = so.Buddy(n), Bitmap(n), []
        sizes = [1 << k for k in range(n.bit_length())]
        for _ in range(600):
            if held and rng.random() < 0.45:
                st, s = held.pop(rng.randrange(len(held)))
                b.release(st, s)
                bm.mark(st, s, False)
            else:
                s = rng.choice(sizes)
                possible = bm.has_aligned_free_range(s)
                st = b.alloc(s)
                assert (st is not None) == possible
                if st is not None:
                    assert st % s == 0 and 0 <= st and st + s <= n
                    bm.mark(st, s, True)
                    held.append((st, s))
            assert b.free_gpus() == bm.busy.count(False)
        for st, s in held:
            b.release(st, s)
        assert b.free_gpus() == n and b.free[-1] == [0]

    def test_bad_arguments(self):
        with pytest.raises(ValueError):
            so.Buddy(6)
        with pytest.raises(ValueError):
            so.Buddy(8).alloc(3)


# --------------------------------------------------------------------------- schedules worked by hand
class TestHandSchedules:
    def test_one_request(self):
        rec, ev, tot = so.simulate(8, 3, [[40, 25, 10, 9]], [4], [(5, 0)])
        assert rec == [dict(start_us=5, dit_end_us=35, end_us=35, first_dop=4, final_dop=4, promotions=0, starvation=0)]
        assert ev == [(5, "start", 0, 0, 4), (35, "dit_done", 0, 0, 4), (35, "release", 0, 0, 4)]
        assert tot == dict(occupancy_gpu_us=4 * 30, makespan_us=35)

    def test_two_requests_one_pair_first_come_first_served(self):
        rec, ev, tot = so.simulate(2, 2, [[100, 60]], [2], [(0, 0), (0, 0)])
        assert [r["start_us"] for r in rec] == [0, 120] and [r["end_us"] for r in rec] == [120, 240]
        assert tot == dict(occupancy_gpu_us=480, makespan_us=240)

    def test_hungry_request_is_promoted_between_steps(self):
        # GPU 0: request 0 (B = 1, 4 steps of 50).  Request 1 (B = 2, steps of 100 on one GPU, 60 on two)
        # arrives at 10, starts hungry on GPU 1: steps end at 110, 210; GPU 0 comes free at 200: one step
        # done -> starvation 1 x (100 - 60); the step in flight ends at 210 at the old rate, the
        # last two take 60 each.
        rec, ev, tot = so.simulate(2, 4, [[50, 50], [100, 60]], [1, 2], [(0, 0), (10, 1)])
        assert rec[1] == dict(start_us=10, dit_end_us=330, end_us=330, first_dop=1, final_dop=2, promotions=1, starvation=40)
        assert (200, "promote", 1, 0, 1) in ev
        assert tot["occupancy_gpu_us"] == 200 + 190 + 2 * 130

    def _priority_case(self):
        # resolutions: 0 ends after 300, 1 after 2000, 2 after 10000 (all B = 1); 3 and 4 want four GPUs
        # and differ in what running on two costs them (220 - 190 against 220 - 120 per step)
        step = [[30] * 4, [200] * 4, [1000] * 4, [400, 220, 190, 180], [400, 220, 120, 70]]
        B = [1, 1, 1, 4, 4]
        reqs = [(0, 1), (0, 1), (0, 2), (0, 2), (0, 0), (0, 3), (0, 4), (1000, 0)]
        return so.simulate(8, 10, step, B, reqs)

    def test_starvation_decides_who_is_promoted_and_waiting_comes_last(self):
        rec, ev, _ = self._priority_case()
        # requests 0-4 take GPUs 0-4; request 5 gets the pair (6,2), request 6 the single GPU 5
        assert [e for e in ev if e[0] == 0 and e[1] == "start"] == [
            (0, "start", 0, 0, 1), (0, "start", 1, 1, 1), (0, "start", 2, 2, 1), (0, "start", 3, 3, 1),
            (0, "start", 4, 4, 1), (0, "start", 5, 6, 2), (0, "start", 6, 5, 1)]
        # 300: GPU 4 comes free; request 5 (starvation 30 after one step) is asked first but needs a pair;
        # request 6 (no step done yet) takes the single
        assert [e for e in ev if e[0] == 300] == [(300, "dit_done", 4, 4, 1), (300, "release", 4, 4, 1), (300, "promote", 6, 4, 1)]
        # 2000: GPUs 0 and 1 merge into a pair.  Request 5 has 9 steps done: 9 x 30 = 270; request 6 has
        # 8 (one at 400, then every 220): 8 x 100 = 800 -> the later request is served first, and the
        # waiting request 7 (arrived at 1000) gets nothing
        at = [e for e in ev if e[0] == 2000]
        assert (2000, "promote", 6, 0, 2) in at and not any(e[1] == "promote" and e[2] == 5 for e in at)
        assert not any(e[1] == "start" for e in at)
        assert rec[5]["starvation"] == 270 and rec[6]["starvation"] == 800
        assert rec[6]["final_dop"] == 4 and rec[5]["final_dop"] == 2 and rec[5]["dit_end_us"] == 2200
        assert rec[7]["start_us"] > 2000

    def test_scale_down_for_the_decoder(self):
        # two steps of 10 on four GPUs, then 7 on the lowest GPU; a second request (B = 2) waiting since 5
        # gets the pair (2,2) the moment the first one scales down
        rec, ev, tot = so.simulate(4, 2, [[40, 20, 10], [50, 30, 20]], [4, 2], [(0, 0), (5, 1)], vae_us=[7, 0], vae_gpus=1)
        assert ev[:6] == [(0, "start", 0, 0, 4), (20, "dit_done", 0, 0, 4), (20, "release", 0, 2, 2), (20, "release", 0, 1, 1),
                          (20, "start", 1, 2, 2), (27, "release", 0, 0, 1)]
        assert rec[0]["dit_end_us"] == 20 and rec[0]["end_us"] == 27
        assert rec[1]["start_us"] == 20 and rec[1]["end_us"] == 80
        assert tot["occupancy_gpu_us"] == 4 * 20 + 7 + 2 * 60

    def test_simultaneous_events_step_ends_before_arrivals(self):
        # the GPU that comes free at 100 serves the request that arrives at 100
        rec, _, _ = so.simulate(1, 1, [[100]], [1], [(0, 0), (100, 0)])
        assert rec[1]["start_us"] == 100


# --------------------------------------------------------------------------- invariants and closed forms
def random_case(seed, n_gpus=8, n=40):
    rng = random.Random(seed)
    R = 3
    K = n_gpus.bit_length()
    step = []
    for _ in range(R):
        a, c = rng.randrange(200, 5000), rng.randrange(20, 400)
        step.append([a // (1 << k) + c for k in range(K)])
    B = [rng.choice([1 << k for k in range(K)]) for _ in range(R)]
    t, reqs = 0, []
    for _ in range(n):
        t += rng.choice([0, 0, rng.randrange(1, 4000)])
        reqs.append((t, rng.randrange(R)))
    vae = [rng.choice([0, rng.randrange(1, 900)]) for _ in range(R)]
    return dict(n_gpus=n_gpus, n_steps=rng.choice([1, 3, 30]), step_us=step, opt_dop=B, requests=reqs, vae_us=vae,
                vae_gpus=rng.choice([1, 2]))


def check_invariants(case, rec, ev, tot):
    G, S = case["n_gpus"], case["n_steps"]
    step, B, reqs, vae = case["step_us"], case["opt_dop"], case["requests"], case["vae_us"]
    busy = [None] * G
    held = {}
    last_t = 0
    occ = 0
    for t, kind, i, start, count in ev:
        assert t >= last_t
        occ += sum(x is not None for x in busy) * (t - last_t)
        last_t = t
        if kind in ("start", "promote"):
            assert start % count == 0 and start + count <= G
            for g in range(start, start + count):
                assert busy[g] is None, "GPU %d given twice" % g
                busy[g] = i
            held[i] = held.get(i, 0) + count
            assert held[i] & (held[i] - 1) == 0 and held[i] <= B[reqs[i][1]]
        elif kind == "release":
            for g in range(start, start + count):
                assert busy[g] == i
                busy[g] = None
            held[i] -= count
    assert all(x is None for x in busy)
    assert occ == tot["occupancy_gpu_us"]
    starts = [r["start_us"] for r in rec]
    assert starts == sorted(starts)                                   # first come, first served
    for i, r in enumerate(rec):
        a, res = reqs[i]
        assert r["start_us"] >= a and 1 <= r["first_dop"] <= r["final_dop"] <= B[res]
        # between S steps at the rate of B and S steps at the rate of the first grant
        assert S * step[res][B[res].bit_length() - 1] <= r["dit_end_us"] - r["start_us"] <= S * step[res][r["first_dop"].bit_length() - 1] \
            or step[res] != sorted(step[res], reverse=True)
        assert r["end_us"] == r["dit_end_us"] + vae[res]
        assert (r["promotions"] == 0) == (r["first_dop"] == r["final_dop"]) or r["promotions"] > 0
    assert tot["makespan_us"] == max(r["end_us"] for r in rec)


class TestInvariants:
    @pytest.mark.parametrize("seed", range(12))
    def test_random_workloads(self, seed):
        case = random_case(seed, n_gpus=[8, 8, 4, 16][seed % 4])
        check_invariants(case, *so.simulate(**case))

    def test_no_contention_everyone_runs_at_B_from_the_start(self):
        step, B = [[900, 500, 300, 200], [400, 250, 200, 190]], [4, 2]
        reqs = [(0, 0), (10_000, 1), (20_000, 0), (30_000, 1)]        # far apart
        rec, _, tot = so.simulate(8, 30, step, B, reqs)
        for (a, r), x in zip(reqs, rec):
            assert x["start_us"] == a and x["first_dop"] == B[r] and x["promotions"] == 0
            assert x["end_us"] == a + 30 * step[r][B[r].bit_length() - 1]
        assert tot["occupancy_gpu_us"] == 2 * 4 * 30 * 300 + 2 * 2 * 30 * 250

    def test_one_gpu_is_a_serial_queue(self):
        step, reqs = [[70], [110]], [(0, 0), (0, 1), (0, 1), (5, 0)]
        rec, _, tot = so.simulate(1, 5, step, [1, 1], reqs)
        assert [r["end_us"] for r in rec] == [350, 900, 1450, 1800]
        assert tot["occupancy_gpu_us"] == 1800

    def test_burst_of_equal_requests_on_a_full_pool(self):
        # 4 requests with B = 2 on 8 GPUs all start at once; 8 of them run in two rounds
        rec, _, _ = so.simulate(8, 10, [[100, 60, 50, 45]], [2], [(0, 0)] * 8)
        assert sorted(r["end_us"] for r in rec) == [600] * 4 + [1200] * 4


# --------------------------------------------------------------------------- planted mistakes
class TestPinsCatchMistakes:
    def _fails(self, suites):
        failed = 0
        for s in suites:
            for name in dir(s):
                if name.startswith("test_"):
                    fn = getattr(s, name)
                    if getattr(fn, "pytestmark", None):
                        continue                      # parametrised ones are run by pytest itself
                    try:
                        fn()
                    except (Exception, pytest.fail.Exception):
                        failed += 1
        return failed

    def test_first_fit_allocator(self, monkeypatch):
        def alloc(self, size):
            k = size.bit_length() - 1
            best = None
            for j in range(k, self.levels):
                for st in self.free[j]:
                    if best is None or st < best[0]:
                        best = (st, j)
            if best is None:
                return None
            st, j = best
            self.free[j].remove(st)
            while j > k:
                j -= 1
                self.free[j].append(st + (1 << j))
            return st
        monkeypatch.setattr(so.Buddy, "alloc", alloc)
        assert self._fails([TestBuddy()]) > 0

    def test_release_that_never_merges(self, monkeypatch):
        monkeypatch.setattr(so.Buddy, "release", lambda self, st, s: self.free[s.bit_length() - 1].append(st))
        assert self._fails([TestBuddy()]) > 0

    def test_least_starved_first(self, monkeypatch):
        real = sorted
        def wrong(it, key=None, **kw):
            it = list(it)
            if key is not None and it and isinstance(key(it[0]), tuple):
                return real(it, key=lambda j: (-key(j)[0], key(j)[1]))     # ascending starvation
            return real(it, key=key, **kw)
        monkeypatch.setattr(so, "sorted", wrong, raising=False)
        assert self._fails([TestHandSchedules()]) > 0

    def test_change_rate_upside_down(self, monkeypatch):
        monkeypatch.setattr(so, "change_rate", lambda row, i: 1 - Fraction(row[i.bit_length() - 2], row[i.bit_length() - 1]))
        assert self._fails([TestOptimalDop()]) > 0
