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


@pytest.mark.parametrize("entries,stems,branches", [(5, 1, 1), (6, 2, 3), (7, 3, 2), (4, 4, 8), (9, 2, 4)])
def test_driver_follows_the_reference_exactly(entries, stems, branches):
    shapes, sens, ppl = synthetic_problem(entries * 100 + stems * 10 + branches, entries)
    start = (8,) * entries
    calls = []

    def evaluate(bits, parent, entry):
        calls.append(bits)
        if parent is not None:  # the driver tells which single entry changed
            assert sum(a != b for a, b in zip(bits, parent.bitvec)) == 1 and bits[entry] != parent.bitvec[entry]
        return ppl(bits), None

    got = search.tree_search(start, LEVELS, sens, evaluate, shapes, stems, branches)
    want = search_ref.tree_search_ref(start, LEVELS, sens, ppl, shapes, stems, branches)
    assert [[(n.bitvec, n.ppl) for n in p] for p in got] == [[(b, v) for b, v in p] for p in want]
    assert len(calls) == len(set(calls))  # duplicates in the pool are scored once


@pytest.mark.parametrize("stems,branches", [(1, 2), (3, 3)])
def test_paths_are_one_way_one_module_per_step_and_end_at_the_lowest_model(stems, branches):
    entries = 6
    shapes, sens, ppl = synthetic_problem(7, entries)
    paths = search.tree_search((8,) * entries, LEVELS, sens, lambda b, p, e: (ppl(b), None), shapes, stems, branches)
    assert 1 <= len(paths) <= stems
    order = sorted(LEVELS)
    for path in paths:
        assert path[0].bitvec == (8,) * entries and path[-1].bitvec == (2,) * entries
        # every stored level of every matrix is passed once: (levels - 1) * entries steps
        assert len(path) == 1 + (len(LEVELS) - 1) * entries
        for a, b in zip(path, path[1:]):
            changed = [e for e in range(entries) if a.bitvec[e] != b.bitvec[e]]
            assert len(changed) == 1
            e = changed[0]
            assert order.index(b.bitvec[e]) == order.index(a.bitvec[e]) - 1  # one level down, never up
            assert search.footprint_bytes(b.bitvec, shapes) < search.footprint_bytes(a.bitvec, shapes)
    means = [np.mean([n.ppl for n in p]) for p in paths]
    assert means == sorted(means)


def test_candidate_counts_match_the_papers_complexity():
    """With two stored models every module has one possible move: the first step has #module candidates and
    the whole search (m + 1) * #module steps, m the number of models between n_low and n_up."""
    entries = 11
    vec = (8,) * entries
    assert len(search.successors(vec, (2, 8))) == entries
    assert len(search.successors(vec, LEVELS)) == entries
    assert search.successors((2,) * entries, LEVELS) == []
    mixed = (8, 2, 4, 3)
    assert sorted((e, b) for e, b, _ in search.successors(mixed, LEVELS)) == [(0, 4), (2, 3), (3, 2)]
    shapes, sens, ppl = synthetic_problem(3, entries)
    sens2 = {(e, 2): sens[(e, 2)] for e in range(entries)}
    path = search.tree_search(vec, (2, 8), sens2, lambda b, p, e: (ppl(b), None), shapes, 1, entries)[0]
    assert len(path) - 1 == (0 + 1) * entries


def test_greedy_choice_with_an_unfiltered_pool_and_a_separable_metric():
    """One stem, every successor scored: each step takes the candidate with the smallest perplexity."""
    entries = 5
    shapes, sens, _ = synthetic_problem(11, entries)
    cost = {8: 0.0, 4: 0.1, 3: 0.35, 2: 1.0}
    w = [1.0, 0.3, 2.0, 0.7, 1.5]
    ppl = lambda bits: 3.0 + sum(w[e] * cost[b] for e, b in enumerate(bits))
    path = search.tree_search((8,) * entries, LEVELS, sens, lambda b, p, e: (ppl(b), None), shapes, 1, entries)[0]
    for a, b in zip(path, path[1:]):
        best = min(ppl(v) for _, _, v in search.successors(a.bitvec, LEVELS))
        assert b.ppl == best


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

