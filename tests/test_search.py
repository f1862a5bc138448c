"""Host logic of the ensemble tree search (Algorithm 1): the library's driver against the plain reference
under one deterministic metric, and the properties the paper states (one-way transitions, one module per
step, termination at QM(n_low), candidate counts)."""
import hashlib
import importlib.util
import os

import numpy as np
import pytest

from oracle import search_ref

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _load_search():
    # by path: the package itself needs the built library, this module does not
    spec = importlib.util.spec_from_file_location("fq_search", os.path.join(ROOT, "paper_2501_07139_amd", "search.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


search = _load_search()
LEVELS = (2, 3, 4, 8)


def synthetic_problem(seed, entries):
    rng = np.random.default_rng(seed)
    shapes = [(int(rng.integers(1, 5)) * 64, int(rng.integers(1, 4)) * 128) for _ in range(entries)]
    weight = rng.uniform(0.5, 2.0, entries)
    penalty = {8: 0.0, 4: 0.05, 3: 0.2, 2: 1.0}
    sens = {(e, b): float(weight[e] * penalty[b] * rng.uniform(0.8, 1.25)) for e in range(entries) for b in (2, 3, 4)}

    def ppl(bits):
        # separable part plus a deterministic interaction term that depends on the whole vector
        h = int.from_bytes(hashlib.sha256(bytes(bits)).digest()[:4], "little") / 2 ** 32
        return float(5.0 + sum(weight[e] * penalty[b] for e, b in enumerate(bits)) + 0.01 * h)

    return shapes, sens, ppl


def run_driver(start, levels, sens, ppl, shapes, stems, branches):
    """The library's driver: (paths as [(bitvec, ppl)], vectors scored per iteration in scoring order)."""
    calls, trace = [], []

    def evaluate(bits, parent, entry):
        calls.append(bits)
        if parent is not None:  # the driver tells which single entry changed
            assert sum(a != b for a, b in zip(bits, parent.bitvec)) == 1 and bits[entry] != parent.bitvec[entry]
        return ppl(bits), None

    paths = search.tree_search(start, levels, sens, evaluate, shapes, stems, branches, trace=trace)
    pools, at = [], 1
    for it in trace:
        pools.append(calls[at:at + len(it)])
        at += len(it)
    assert at == len(calls) and calls[0] == tuple(start)
    return [[(n.bitvec, n.ppl) for n in p] for p in paths], pools


def run_reference(start, levels, sens, ppl, shapes, stems, branches):
    """The plain reference: (paths as [(bitvec, ppl)], vectors scored per iteration)."""
    calls, pools = [], []

    def evaluate(bits):
        calls.append(bits)
        return ppl(bits)

    paths = search_ref.tree_search_ref(start, levels, sens, evaluate, shapes, stems, branches, pools=pools)
    assert calls[0] == tuple(start) and sorted(calls[1:]) == sorted(c for p in pools for c in p)
    at, in_order = 1, []
    for p in pools:  # in scoring order, like the driver's
        in_order.append(calls[at:at + len(p)])
        assert sorted(in_order[-1]) == sorted(p)
        at += len(p)
    return [[(b, v) for b, v in p] for p in paths], in_order


def is_successor(parent, child):
    diff = [(a, b) for a, b in zip(parent, child) if a != b]
    return len(diff) == 1 and diff[0][1] < diff[0][0]


IMPLEMENTATIONS = {"driver": run_driver, "reference": run_reference}


@pytest.mark.parametrize("entries,stems,branches", [(5, 1, 1), (6, 2, 3), (7, 3, 2), (4, 4, 8), (9, 2, 4)])
def test_driver_follows_the_reference_exactly(entries, stems, branches):
    shapes, sens, ppl = synthetic_problem(entries * 100 + stems * 10 + branches, entries)
    start = (8,) * entries
    got, got_pools = run_driver(start, LEVELS, sens, ppl, shapes, stems, branches)
    want, want_pools = run_reference(start, LEVELS, sens, ppl, shapes, stems, branches)
    assert got == want
    assert [sorted(p) for p in got_pools] == [sorted(p) for p in want_pools]


@pytest.mark.parametrize("impl", sorted(IMPLEMENTATIONS))
@pytest.mark.parametrize("stems,branches", [(1, 2), (3, 3), (2, 12)])
def test_paths_are_one_way_one_module_per_step_and_end_at_the_lowest_model(impl, stems, branches):
    """Section "Efficient Design Space Navigation": only transitions to a lower bit-width, one module per
    step, every stem ends at QM(n_low); checked on the driver and on the reference alike."""
    entries = 6
    shapes, sens, ppl = synthetic_problem(7, entries)
    paths, pools = IMPLEMENTATIONS[impl]((8,) * entries, LEVELS, sens, ppl, shapes, stems, branches)
    assert 1 <= len(paths) <= stems
    for path in paths:
        assert path[0][0] == (8,) * entries and path[-1][0] == (2,) * entries
        # a matrix goes down in one to three steps
        assert 1 + entries <= len(path) <= 1 + (len(LEVELS) - 1) * entries
        for (a, _), (b, vb) in zip(path, path[1:]):
            assert is_successor(a, b)
            assert set(b) <= set(LEVELS) and vb == ppl(b)
            assert search_ref.footprint(b, shapes) < search_ref.footprint(a, shapes)
    means = [np.mean([v for _, v in p]) for p in paths]
    assert means == sorted(means)
    for pool in pools:
        assert len(pool) == len(set(pool))            # a configuration is scored once per iteration
        assert len(pool) <= stems * branches          # the analysis filter bounds the pool


@pytest.mark.parametrize("impl", sorted(IMPLEMENTATIONS))
def test_candidate_counts_match_the_papers_complexity(impl):
    """Below QM(n_up) there are (m + 1) * #module options, m the number of stored models between n_low and
    n_up: 66 for the two-model ensemble of a 66-module network, three times that with two models in between
    (Section "Efficient Design Space Navigation")."""
    for levels, m in (((2, 8), 0), ((2, 4, 8), 1), (LEVELS, 2)):
        entries = 66
        shapes, sens, ppl = synthetic_problem(3, entries)
        table = {(e, b): sens.get((e, b), 1.0 + e) for e in range(entries) for b in levels[:-1]}
        # an unfiltered first iteration scores every option below the root
        _, pools = IMPLEMENTATIONS[impl]((8,) * entries, levels, table, ppl, shapes, 1, 10 ** 6)
        assert len(pools[0]) == (m + 1) * entries
        assert all(is_successor((8,) * entries, c) for c in pools[0])
    # with two stored models every step has one option per module still at n_up, so the stem has #module steps
    paths, pools = IMPLEMENTATIONS[impl]((8,) * 11, (2, 8), {(e, 2): float(e) for e in range(11)},
                                         synthetic_problem(3, 11)[2], synthetic_problem(3, 11)[0], 1, 11)
    assert len(paths[0]) - 1 == 11 and [len(p) for p in pools] == list(range(11, 0, -1))


def test_successors_of_the_driver():
    entries = 11
    vec = (8,) * entries
    assert len(search.successors(vec, (2, 8))) == entries
    assert len(search.successors(vec, LEVELS)) == 3 * entries
    assert search.successors((2,) * entries, LEVELS) == []
    mixed = (8, 2, 4, 3)
    assert sorted((e, b) for e, b, _ in search.successors(mixed, LEVELS)) == [(0, 2), (0, 3), (0, 4), (2, 2), (2, 3), (3, 2)]
    for e, b, v in search.successors(mixed, LEVELS):
        assert v[e] == b and all(v[i] == mixed[i] for i in range(4) if i != e)


@pytest.mark.parametrize("impl", sorted(IMPLEMENTATIONS))
def test_greedy_choice_with_an_unfiltered_pool_and_a_separable_metric(impl):
    """One stem, every successor scored: each step takes the candidate with the smallest perplexity, which
    for a separable metric is the cheapest single move, and equal perplexities go to the smaller model."""
    entries = 5
    shapes, sens, _ = synthetic_problem(11, entries)
    cost = {8: 0.0, 4: 0.1, 3: 0.35, 2: 1.0}
    w = [1.0, 0.3, 2.0, 0.7, 1.5]
    ppl = lambda bits: 3.0 + sum(w[e] * cost[b] for e, b in enumerate(bits))
    path = IMPLEMENTATIONS[impl]((8,) * entries, LEVELS, sens, ppl, shapes, 1, 10 ** 6)[0][0]
    for (a, _), (b, vb) in zip(path, path[1:]):
        options = [tuple(a[:e]) + (nb,) + tuple(a[e + 1:]) for e in range(entries) for nb in LEVELS if nb < a[e]]
        assert vb == min(ppl(v) for v in options)
    # ties: a constant metric leaves the footprint to decide, so every step takes the largest saving
    flat = IMPLEMENTATIONS[impl]((8,) * entries, LEVELS, sens, lambda bits: 7.0, shapes, 1, 10 ** 6)[0][0]
    for (a, _), (b, _) in zip(flat, flat[1:]):
        options = [tuple(a[:e]) + (nb,) + tuple(a[e + 1:]) for e in range(entries) for nb in LEVELS if nb < a[e]]
        assert search_ref.footprint(b, shapes) == min(search_ref.footprint(v, shapes) for v in options)


@pytest.mark.parametrize("impl", sorted(IMPLEMENTATIONS))
def test_the_papers_example_two_stems_three_branches(impl):
    """The worked example of Section "Efficient Design Space Navigation" (two stems, three branches): at the
    start of the second iteration the last models of the two ensembles are EQM_1,0 and EQM_1,1; the
    sensitivity table leaves three successors of each, EQM_2,0 .. EQM_2,5, for the calibration set, and the
    two best of those, EQM_2,2 and EQM_2,5, become the new last models.  Every number below is written by
    hand: a perplexity exists only for the vectors the example scores, so scoring anything else fails."""
    levels = (2, 4, 8)
    shapes = [(64, 128)] * 4
    sens = {(0, 4): 1.0, (0, 2): 2.0, (1, 4): 3.0, (2, 4): 4.0, (3, 4): 5.0, (1, 2): 6.0, (2, 2): 7.0, (3, 2): 8.0}
    root = (8, 8, 8, 8)
    eqm1 = [(4, 8, 8, 8), (2, 8, 8, 8), (8, 4, 8, 8)]            # the three least sensitive moves below the root
    eqm2 = [(2, 8, 8, 8), (4, 4, 8, 8), (4, 8, 4, 8),            # successors of EQM_1,0 = (4,8,8,8)
            (2, 4, 8, 8), (2, 8, 4, 8), (2, 8, 8, 4)]            # successors of EQM_1,1 = (2,8,8,8)
    table = {root: 5.00, eqm1[0]: 5.10, eqm1[1]: 5.20, eqm1[2]: 5.90,
             eqm2[0]: 5.20, eqm2[1]: 5.60, eqm2[2]: 5.15, eqm2[3]: 5.70, eqm2[4]: 5.80, eqm2[5]: 5.18}
    stop = {"after": 1 + 3 + 6}
    scored = []

    class Done(Exception):
        pass

    def ppl(bits):
        if len(scored) == stop["after"]:
            raise Done()
        scored.append(bits)
        return table[bits]            # KeyError: a vector the example does not score

    with pytest.raises(Done):
        IMPLEMENTATIONS[impl](root, levels, sens, ppl, shapes, 2, 3)
    assert scored[0] == root
    assert sorted(scored[1:4]) == sorted(eqm1)
    assert sorted(scored[4:10]) == sorted(eqm2) and len(set(scored[4:10])) == 6
    # the third iteration starts from EQM_2,2 and EQM_2,5: run it to see which models were kept
    more = {}

    def ppl3(bits):
        if bits in table:
            return table[bits]
        more.setdefault(bits, 6.0 + 0.01 * len(more))
        return more[bits]

    paths, pools = IMPLEMENTATIONS[impl](root, levels, sens, ppl3, shapes, 2, 3)
    assert sorted(pools[1]) == sorted(eqm2)
    kept = {eqm2[2], eqm2[5]}
    assert all(any(is_successor(k, c) for k in kept) for c in pools[2])
    assert all(any(is_successor(k, c) for c in pools[2]) for k in kept)
    # and the stems that led there are the example's: EQM_1,0 -> EQM_2,2 and EQM_1,1 -> EQM_2,5
    second = {p[2][0]: p[1][0] for p in paths}
    for p in paths:
        assert p[1][0] in (eqm1[0], eqm1[1]) and p[2][0] in kept
    assert all(second[c] == (eqm1[0] if c == eqm2[2] else eqm1[1]) for c in second)


@pytest.mark.parametrize("impl", ["driver", "reference"])
def test_pruning_counts_use_and_breaks_ties_by_footprint(impl):
    """Section "EQM Pruning Strategy" on a hand-made ensemble: rank by the number of member models that use a
    mid-level packing; similar use is ordered by use at lower footprints; unused packings come last."""
    prune = search.prune_ensemble if impl == "driver" else search_ref.prune_ref
    shapes = [(64, 128), (128, 128), (64, 256)]
    levels = (2, 4, 8)
    ensemble = [(8, 8, 8), (4, 8, 8), (4, 4, 8), (2, 4, 8), (2, 4, 4), (2, 2, 4), (2, 2, 2)]
    # use counts by hand: (0,4) in 2 models, (1,4) in 3, (2,4) in 2; (2,4) is used by the smaller models
    ranking, dropped, kept, stored = prune(ensemble, levels, shapes, 1 / 3)
    assert ranking == [(1, 4), (2, 4), (0, 4)]
    assert dropped == {(0, 4)}
    assert kept == [m for m in ensemble if m[0] != 4]
    per = lambda e, b: shapes[e][0] * shapes[e][1] * b // 8 + 4 * shapes[e][0] * (shapes[e][1] // 128)
    assert stored == sum(per(e, b) for e in range(3) for b in levels) - per(0, 4)
    # rate 0 keeps everything, rate 1 only the end points' packings
    assert prune(ensemble, levels, shapes, 0.0)[1] == set()
    r1 = prune(ensemble, levels, shapes, 1.0)
    assert r1[1] == {(0, 4), (1, 4), (2, 4)} and r1[3] == sum(per(e, b) for e in range(3) for b in (2, 8))
    assert r1[2] == [m for m in ensemble if 4 not in m]


def test_footprint_accounting():
    shapes = [(4096, 4096)] * 4 + [(11008, 4096)] * 2 + [(4096, 11008)]
    weights = sum(n * k for n, k in shapes)
    for b in LEVELS:
        f = search.footprint_bytes((b,) * 7, shapes)
        assert f == weights * b // 8 + 4 * weights // 128
        assert f == search_ref.footprint((b,) * 7, shapes)
    # one MLP matrix from 8 to 2 bits: 45.1 M weights * 6 bits = 33.8 MB, inside the ~100 MB granularity target
    d = search.footprint_bytes((8,) * 7, shapes) - search.footprint_bytes((8, 8, 8, 8, 2, 8, 8), shapes)
    assert d == 11008 * 4096 * 6 // 8


@pytest.mark.parametrize("rate", [0.0, 0.25, 0.5, 0.75, 1.0])
def test_pruning_follows_the_reference_and_the_papers_storage_arithmetic(rate):
    entries = 8
    shapes, sens, ppl = synthetic_problem(21, entries)
    path = search.tree_search((8,) * entries, LEVELS, sens, lambda b, p, e: (ppl(b), None), shapes, 1, 3)[0]
    ensemble = [n.bitvec for n in path]
    got = search.prune_ensemble(ensemble, LEVELS, shapes, rate)
    want = search_ref.prune_ref(ensemble, LEVELS, shapes, rate)
    assert got[0] == want[0] and got[1] == want[1] and got[2] == want[2] and got[3] == want[3]
    ranking, dropped, kept, stored = got
    assert len(ranking) == entries * 2 and len(dropped) == int(rate * entries * 2)
    # the end points never depend on a mid-level packing
    assert ensemble[0] in kept and ensemble[-1] in kept
    # storage: all four packings at rate 0, only n_low and n_up at rate 1, linear in the dropped bytes
    full = sum(search.footprint_bytes((b,) * entries, shapes) for b in LEVELS)
    ends = sum(search.footprint_bytes((b,) * entries, shapes) for b in (2, 8))
    assert stored == full - sum(search.footprint_bytes((b,), [shapes[e]]) for e, b in dropped)
    if rate == 0.0:
        assert stored == full and kept == ensemble
    if rate == 1.0:
        assert stored == ends and all(set(m) <= {2, 8} for m in kept)
    # what is dropped is used by no more models than anything that is kept
    count = lambda k: sum(m[k[0]] == k[1] for m in ensemble)
    if dropped and len(dropped) < len(ranking):
        assert max(count(k) for k in dropped) <= min(count(k) for k in ranking if k not in dropped)


def test_pruning_tie_break_prefers_use_at_low_footprints():
    shapes = [(64, 128)] * 3
    # matrices 0 and 1 are each used once at 4 bits; matrix 1's use happens in the smaller model
    ensemble = [(8, 8, 8), (4, 8, 8), (2, 8, 8), (2, 4, 8), (2, 2, 8), (2, 2, 2)]
    ranking, dropped, kept, _ = search.prune_ensemble(ensemble, (2, 4, 8), shapes, 1 / 3)
    assert ranking == [(1, 4), (0, 4), (2, 4)]       # equal counts: lower footprint first; unused last
    assert dropped == {(2, 4)} and kept == ensemble

