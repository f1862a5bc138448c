"""Host side of the persistent decode kernel: the work partition, and a threaded model of its grid barrier.

The kernel keeps one workgroup per compute unit resident and lets them meet after every phase.  Two things
about it can be checked without a GPU: that the partition gives every work unit to exactly one workgroup and
keeps a workgroup's rows within its reduction buffer, and that the barrier protocol (arrival counters,
generation targets, bounded waits that give up for good) always lets every participant finish.
"""
import itertools
import threading
import time

import numpy as np
import pytest

import paper_2501_07139_amd as fq

ROWS = {2: 32, 3: 64, 4: 16, 8: 16}
PHASES = {0: (0, 3), 1: (3, 1), 2: (4, 2), 3: (6, 1)}   # first matrix, number of matrices


@pytest.mark.parametrize("hidden,ffn", [(4096, 11008), (5120, 13824), (256, 640), (8192, 16384)])
@pytest.mark.parametrize("grid", [256, 248, 8])
def test_partition_gives_every_unit_to_exactly_one_workgroup(hidden, ffn, grid):
    rng = np.random.default_rng(hidden)
    patterns = [rng.choice([2, 3, 4, 8], size=7) for _ in range(6)] + [np.full(7, b) for b in (2, 3, 4, 8)]
    for bits7 in patterns:
        for ph, (first, count) in PHASES.items():
            N = ffn if ph == 2 else hidden
            units = [((N + 63) // 64 * 64) // ROWS[int(bits7[first + j])] for j in range(count)]
            seen = [np.zeros(u, dtype=np.int32) for u in units]
            worst_rows = 0
            for wg in range(grid):
                part = fq.fq_decode_partition(bits7, ph, N, wg, grid)
                rows = 0
                for j in range(3):
                    a, b = part[j]
                    if j >= count:
                        assert (a, b) == (0, 0)
                        continue
                    assert 0 <= a <= b <= units[j]
                    # every matrix is split evenly: a workgroup's run is within one unit of the mean
                    assert units[j] // grid <= b - a <= -(-units[j] // grid)
                    seen[j][a:b] += 1
                    rows += (b - a) * ROWS[int(bits7[first + j])]
                worst_rows = max(worst_rows, rows)
            for j in range(count):
                assert np.all(seen[j] == 1), (bits7, ph, j)
            if grid == 256:
                assert worst_rows <= 384   # the kernel's reduction buffer


def test_partition_balances_bytes():
    """Workgroups that take the longer runs of one matrix take the shorter runs of the next (reverse order), so
    the bytes of a workgroup stay within one unit per matrix of the mean."""
    bits7 = np.array([2, 4, 8, 2, 4, 4, 2], dtype=np.uint8)
    grid = 256
    cost = {2: 32 * (2 / 8 + 1 / 32), 3: 64 * (3 / 8 + 1 / 32), 4: 16 * (4 / 8 + 1 / 32), 8: 16 * (1 + 1 / 32)}
    for ph, N in ((0, 4096), (2, 11008)):
        first, count = PHASES[ph]
        loads = []
        for wg in range(grid):
            part = fq.fq_decode_partition(bits7, ph, N, wg, grid)
            loads.append(sum((b - a) * cost[int(bits7[first + j])] for j, (a, b) in enumerate(part[:count])))
        assert max(loads) <= np.mean(loads) + sum(cost[int(bits7[first + j])] for j in range(count)) + 1e-9


def test_partition_rejects_bad_arguments():
    ok = np.array([2, 3, 4, 8, 2, 3, 4], dtype=np.uint8)
    with pytest.raises(fq.FqError):
        fq.fq_decode_partition(ok, 4, 4096, 0, 256)
    with pytest.raises(fq.FqError):
        fq.fq_decode_partition(ok, 0, 4096, 256, 256)
    with pytest.raises(fq.FqError):
        fq.fq_decode_partition(np.array([2, 3, 4, 8, 2, 3, 5], dtype=np.uint8), 0, 4096, 0, 256)


# ------------------------------------------------------------------ the barrier protocol, modelled with threads
class BarrierModel:
    """Eight arrival counters; arrive(wg) bumps counter wg % 8; wait(k) polls until all eight have reached
    (gen0 + k) * per.  A wait that exceeds `limit` seconds, or sees the error word, gives up: it raises the
    error word and the participant never waits again.  The same steps as the kernel's exchange wavefront."""

    def __init__(self, grid, limit, gen0=0):
        assert grid % 8 == 0
        self.counters = [0] * 8
        self.lock = threading.Lock()
        self.err = 0
        self.per, self.limit, self.gen0 = grid // 8, limit, gen0

    def arrive(self, wg):
        with self.lock:                      # an atomic add
            self.counters[wg % 8] += 1

    def wait(self, k, state):
        if state["dead"]:
            return
        target = (self.gen0 + k) * self.per
        t0 = time.monotonic()
        while True:
            snapshot = list(self.counters)   # eight independent loads, each possibly stale but never ahead
            if all(v >= target for v in snapshot):
                return
            if self.err or time.monotonic() - t0 > self.limit:
                state["dead"] = True
                self.err = 1
                return
            time.sleep(0)


def run_model(grid, phases, limit, absent=(), gen0=0):
    bar = BarrierModel(grid, limit, gen0)
    log = [[] for _ in range(grid)]
    produced = [[None] * grid for _ in range(phases)]
    stale = []

    def workgroup(wg):
        state = {"dead": False}
        for p in range(phases):
            if p > 0:
                bar.wait(p, state)
                if not state["dead"] and any(v is None for v in produced[p - 1]):
                    stale.append((wg, p))            # passed the barrier before everybody had published
            if wg in absent and p == 1:
                return                               # a workgroup that never arrives again
            produced[p][wg] = p                      # publish, then arrive
            bar.arrive(wg)
            log[wg].append(p)
        bar.wait(phases, state)
        log[wg].append("end" if not state["dead"] else "gave up")

    threads = [threading.Thread(target=workgroup, args=(w,)) for w in range(grid)]
    t0 = time.monotonic()
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=30)
    assert not any(t.is_alive() for t in threads), "a participant is stuck"
    return bar, log, stale, time.monotonic() - t0


@pytest.mark.parametrize("gen0", [0, 64])
def test_barrier_model_orders_every_phase(gen0):
    grid, phases = 32, 12
    if gen0:   # a later launch of the same call: the counters carry on from the earlier launches
        bar, log, stale, _ = run_model(grid, phases, limit=20.0, gen0=0)
        assert not stale
    bar = BarrierModel(grid, 20.0, gen0)
    bar.counters = [gen0 * bar.per] * 8
    _, log, stale, _ = run_model(grid, phases, limit=20.0)
    assert not stale and bar.err == 0
    assert all(l == list(range(phases)) + ["end"] for l in log)


def test_barrier_model_gives_up_when_a_participant_never_arrives():
    grid, phases = 32, 6
    bar, log, stale, took = run_model(grid, phases, limit=0.2, absent={5})
    # Once somebody has given up the error word is up and the results are void: the others keep arriving
    # without waiting, so a late waiter may even see its count reached.  What must hold is that the error is
    # raised, that nobody is stuck, and that the waiting was bounded (about one bound, not one per phase).
    assert bar.err == 1
    assert took < 10.0
    assert any(l[-1] == "gave up" for l in log)
    for wg, l in enumerate(log):
        if wg == 5:
            assert l == [0]
        else:
            assert l[-1] in ("gave up", "end") and l[:-1] == list(range(phases))   # everybody runs to the end


def test_barrier_model_with_a_zero_bound_never_blocks():
    bar, log, stale, took = run_model(32, 5, limit=0.0)
    assert took < 10.0 and all(len(l) == 6 for l in log)
