"""CPU oracle of the paper's greedy, step-granular scheduling of DiT requests over a pool of GPUs
(section 4.2.3 and the greedy scheduling algorithm of the appendix) on top of a buddy allocator of
GPUs (section 5), driven by a table of per-step times DiT_step_time(parallel size, resolution).

THIS IS TEST INFRASTRUCTURE, not a product path: only the tests may import it.  It shares no code
with the library.  Plain Python lists and loops, integer arithmetic only: all times are integer
microseconds, so the library's event simulation must agree with it exactly.

What the paper fixes
  * every resolution r has an optimal degree of parallelism B(r): the parallel size i at which
    z(i) = 1 - step_time(i, r) / step_time(i/2, r) is largest (eq. of section 4.2.3);
  * requests are served first come, first served; an arriving request asks for B GPUs and, if
    fewer are free, starts on what it can get ("hungry"); whenever GPUs are released, hungry
    requests are promoted towards B, the one with the largest starvation time first, where
        starv += (cur_step - last_step) * (cur_step_time - opt_step_time)
    is brought up to date at every such event; promotion takes effect between two denoising
    steps; hungry requests are served before waiting ones;
  * the allocator keeps the GPUs in multi-level lists as a buddy system that splits and merges
    pairs; an allocation for a waiting request starts from B and goes down until it succeeds.

Readings taken where the paper is silent (each is also stated in the library's header)
  S1 group sizes are powers of two; a request holds a list of aligned blocks of the buddy system
     (one block at its start, one more per doubling);
  S2 the allocator takes the SMALLEST free block that is large enough, the lowest-numbered one of
     that size, and splits it keeping the lower half each time; a freed block merges with its
     buddy as long as that is free;
  S3 a promotion from p to 2p GPUs asks the allocator for one more block of p GPUs (any block: the
     paper's engine forms groups from arbitrary GPU ids), and repeats until B is reached or the
     allocator has no such block ("try best");
  S4 the GPUs of a promotion are held from the moment they are granted, the step in flight ends
     at the old rate, every later step runs at the new one;
  S5 events at the same microsecond: step ends first (by request index), then arrivals (by
     index), then ONE scheduling pass; a pass promotes only if GPUs were released since the last
     promotion round; ties of starvation go to the earlier arrival;
  S6 B = 1 when no doubling gains more than z_min (the paper reports B = 1 for its lowest
     resolution although its argmax ranges over 2, 4, 8); z compares integer step times exactly;
  S7 after its last denoising step a request keeps the `vae_gpus` lowest-numbered GPUs of its
     lowest-numbered block (at most that block) for vae_us[r] microseconds (the paper's scale-down
     for the decoder, masters = lowest ids) and releases the rest at once, upper halves first;
     vae_us[r] = 0 releases everything, block by block in the order they were granted.
"""
from __future__ import annotations

from fractions import Fraction


# ---------------------------------------------------------------------------
# optimal degree of parallelism (section 4.2.3)
# ---------------------------------------------------------------------------
def change_rate(step_us_row, i):
    """z for parallel size i (a power of two >= 2): 1 - t(i) / t(i/2), as an exact fraction.
    step_us_row[k] is the step time at parallel size 2^k."""
    k = i.bit_length() - 1
    if i < 2 or (1 << k) != i or k >= len(step_us_row):
        raise ValueError("parallel size must be a power of two inside the table")
    return 1 - Fraction(step_us_row[k], step_us_row[k - 1])


def optimal_dop(step_us_row, z_min=Fraction(0)):
    """B: the parallel size with the largest z (the smaller size on ties), or 1 if no z exceeds z_min."""
    best_i, best_z = 1, Fraction(z_min)
    for k in range(1, len(step_us_row)):
        z = change_rate(step_us_row, 1 << k)
        if z > best_z:
            best_i, best_z = 1 << k, z
    return best_i


# ---------------------------------------------------------------------------
# buddy allocator over GPUs 0 .. n-1 (n a power of two)
# ---------------------------------------------------------------------------
class Buddy:
    def __init__(self, n_gpus):
        if n_gpus < 1 or n_gpus & (n_gpus - 1):
            raise ValueError("the number of GPUs must be a power of two")
        self.n = n_gpus
        self.levels = n_gpus.bit_length()                 # level k holds free blocks of 2^k GPUs
        self.free = [[] for _ in range(self.levels)]
        self.free[self.levels - 1].append(0)

    def alloc(self, size):
        """Start of an aligned block of `size` GPUs, or None."""
        k = size.bit_length() - 1
        if size < 1 or (1 << k) != size:
            raise ValueError("block sizes are powers of two")
        j = k
        while j < self.levels and not self.free[j]:
            j += 1
        if j >= self.levels:
            return None
        start = min(self.free[j])
        self.free[j].remove(start)
        while j > k:                                      # split, keep the lower half
            j -= 1
            self.free[j].append(start + (1 << j))
        return start

    def release(self, start, size):
        k = size.bit_length() - 1
        while k < self.levels - 1 and (start ^ (1 << k)) in self.free[k]:
            self.free[k].remove(start ^ (1 << k))
            start = min(start, start ^ (1 << k))
            k += 1
        self.free[k].append(start)

    def free_gpus(self):
        return sum(len(f) << k for k, f in enumerate(self.free))


# ---------------------------------------------------------------------------
# the scheduler as a discrete-event simulation
# ---------------------------------------------------------------------------
def simulate(n_gpus, n_steps, step_us, opt_dop, requests, vae_us=None, vae_gpus=1):
    """step_us[r][k]: microseconds of one denoising step of resolution r on 2^k GPUs;
    opt_dop[r]: B(r); requests: list of (arrival_us, r) in arrival order.
    Returns (per-request records, event log, totals).
      record: dict(start_us, dit_end_us, end_us, first_dop, final_dop, promotions, starvation)
      event : (time_us, kind, request, gpu_start, gpu_count) with kind in
              'start', 'promote' (one per block granted), 'dit_done' (gpu_count = the DoP reached),
              'release' (one per block given back), in the order they happen
      totals: dict(occupancy_gpu_us, makespan_us)"""
    R = len(step_us)
    vae_us = [0] * R if vae_us is None else list(vae_us)
    if n_steps < 1:
        raise ValueError("a request has at least one denoising step")
    for a, b in zip(requests, requests[1:]):
        if b[0] < a[0]:
            raise ValueError("requests must be ordered by arrival time")
    bud = Buddy(n_gpus)
    n = len(requests)
    rec = [dict(start_us=-1, dit_end_us=-1, end_us=-1, first_dop=0, final_dop=0, promotions=0, starvation=0)
           for _ in range(n)]
    st = [None] * n                     # running state per request
    events = []
    waiting = []                        # indices, arrival order
    hungry = []                         # indices
    step_end = {}                       # request -> time of the end of its step in flight
    vae_end = {}                        # request -> time its decoder phase ends
    next_arrival = 0
    released = False                    # GPUs were released since the last promotion round
    occupancy = 0
    now = 0

    def t_step(r, p):
        return step_us[r][p.bit_length() - 1]

    def hold(i, t):                     # account the GPUs request i has held since its last change
        nonlocal occupancy
        s = st[i]
        occupancy += s["p"] * (t - s["since"])
        s["since"] = t

    def give_back(i, start, size):
        bud.release(start, size)
        events.append((now, "release", i, start, size))

    while next_arrival < n or step_end or vae_end:
        cands = []
        if next_arrival < n:
            cands.append(requests[next_arrival][0])
        cands += list(step_end.values()) + list(vae_end.values())
        now = min(cands)
        # ---- step ends and decoder ends at this microsecond, by request index
        for i in sorted(k for k, t in list(step_end.items()) + list(vae_end.items()) if t == now):
            s = st[i]
            r = requests[i][1]
            if i in vae_end:
                del vae_end[i]
                hold(i, now)
                give_back(i, *s["blocks"][0])
                rec[i]["end_us"] = now
                st[i] = None
                released = True
                continue
            s["step"] += 1
            if s["step"] < n_steps:
                step_end[i] = now + t_step(r, s["p"])      # the group may have grown meanwhile (S4)
                continue
            del step_end[i]
            rec[i]["dit_end_us"] = now
            rec[i]["final_dop"] = s["p"]
            if i in hungry:
                hungry.remove(i)
            events.append((now, "dit_done", i, min(b[0] for b in s["blocks"]), s["p"]))
            hold(i, now)
            if vae_us[r] == 0:
                for b in s["blocks"]:
                    give_back(i, *b)
                rec[i]["end_us"] = now
                st[i] = None
            else:
                low = min(s["blocks"])
                for b in s["blocks"]:
                    if b != low:
                        give_back(i, *b)
                start, size = low
                keep = min(vae_gpus, size)
                while size > keep:                        # split off the upper half
                    size //= 2
                    give_back(i, start + size, size)
                s["blocks"] = [(start, size)]
                s["p"] = size
                vae_end[i] = now + vae_us[r]
            released = True
        # ---- arrivals at this microsecond
        while next_arrival < n and requests[next_arrival][0] == now:
            waiting.append(next_arrival)
            next_arrival += 1
        # ---- one scheduling pass: promotions (only after a release), then the waiting queue
        if released:
            for i in hungry:
                s = st[i]
                r = requests[i][1]
                s["starv"] += (s["step"] - s["last_step"]) * (t_step(r, s["p"]) - t_step(r, opt_dop[r]))
                s["last_step"] = s["step"]
                rec[i]["starvation"] = s["starv"]
            for i in sorted(hungry, key=lambda j: (-st[j]["starv"], j)):
                s = st[i]
                r = requests[i][1]
                grown = False
                while s["p"] < opt_dop[r]:
                    start = bud.alloc(s["p"])
                    if start is None:
                        break
                    if not grown:
                        hold(i, now)
                        grown = True
                    s["blocks"].append((start, s["p"]))
                    events.append((now, "promote", i, start, s["p"]))
                    s["p"] *= 2
                if grown:
                    rec[i]["promotions"] += 1
                    if s["p"] == opt_dop[r]:
                        hungry.remove(i)
            released = False
        still = []
        for i in waiting:
            r = requests[i][1]
            p = opt_dop[r]
            start = None
            while p >= 1:
                start = bud.alloc(p)
                if start is not None:
                    break
                p //= 2
            if start is None:
                still.append(i)
                continue
            st[i] = dict(blocks=[(start, p)], p=p, step=0, last_step=0, starv=0, since=now)
            rec[i]["start_us"] = now
            rec[i]["first_dop"] = p
            step_end[i] = now + t_step(r, p)
            events.append((now, "start", i, start, p))
            if p < opt_dop[r]:
                hungry.append(i)
        waiting = still
    return rec, events, dict(occupancy_gpu_us=occupancy, makespan_us=now)
