"""Elastic hosting run time (FlexQuant, arXiv 2501.07139, Sections "Transition Granularity" and "FlexQuant
Framework"): member selection under a budget and the swap plan on the CPU; the resident model against a
fully resident stack on the GPU (bit-exact: same kernels, same packings, other addresses)."""
import numpy as np
import pytest

import fq_synth


def make_path(entries, levels, seed):
    """A one-way path from all-n_up to all-n_low, one entry lowered by one level per step."""
    rng = np.random.default_rng(seed)
    order = sorted(levels)
    cur = [order[-1]] * entries
    path = [tuple(cur)]
    while any(b != order[0] for b in cur):
        e = int(rng.choice([i for i, b in enumerate(cur) if b != order[0]]))
        cur[e] = order[order.index(cur[e]) - 1]
        path.append(tuple(cur))
    return path


def test_fit_picks_the_largest_member_that_fits():
    from paper_2501_07139_amd import elastic

    fp = [1000, 900, 900, 650, 400]
    assert elastic.fit(fp, 10 ** 9) == 0
    assert elastic.fit(fp, 1000) == 0 and elastic.fit(fp, 999) == 1
    assert elastic.fit(fp, 899) == 3 and elastic.fit(fp, 400) == 4
    with pytest.raises(MemoryError):
        elastic.fit(fp, 399)
    with pytest.raises(ValueError):
        elastic.fit([5, 7], 6)


def test_plan_walks_the_ensemble_member_by_member():
    from paper_2501_07139_amd import elastic, search

    shapes = fq_synth.block_matrix_shapes(256, 512) * 2
    path = make_path(14, (2, 4, 8), 3)
    assert len(path) == 14 * 2 + 1
    fps = [search.footprint_bytes(v, shapes) for v in path]
    assert all(a > b for a, b in zip(fps, fps[1:]))               # one-way moves only shrink the model
    down = elastic.plan(path, 0, len(path) - 1)
    assert len(down) == 28 and all(nb < ob for _, ob, nb in down)
    up = elastic.plan(path, len(path) - 1, 0)
    assert [(e, nb, ob) for e, ob, nb in reversed(up)] == down    # the way back undoes the same swaps
    assert elastic.plan(path, 5, 5) == []
    # replaying a plan on the start vector gives the target vector
    cur = list(path[3])
    for e, ob, nb in elastic.plan(path, 3, 17):
        assert cur[e] == ob
        cur[e] = nb
    assert tuple(cur) == path[17]
    # transitional memory: the largest packing loaded by any swap of the plan
    big = max(search.footprint_bytes((nb,), [shapes[e]]) for e, _, nb in down)
    assert elastic.transitional_bytes(down, shapes) == big
    assert elastic.transitional_bytes([], shapes) == 0
    # granularity of the ensemble: the largest footprint step equals the largest single-matrix saving
    gaps = [a - b for a, b in zip(fps, fps[1:])]
    assert max(gaps) == max(search.footprint_bytes((ob,), [shapes[e]]) - search.footprint_bytes((nb,), [shapes[e]])
                            for e, ob, nb in down)


@pytest.mark.gpu
def test_resident_model_follows_the_budget_and_matches_a_fully_resident_stack():
    import torch

    import oracle
    import paper_2501_07139_amd as fq
    from paper_2501_07139_amd import elastic, search

    levels = (2, 3, 4, 8)
    sh = fq_synth.MODEL_SHAPES["tiny"]
    L = sh["layers"]
    shapes = fq_synth.block_matrix_shapes(sh["hidden"], sh["ffn"]) * L
    quantized, layers = [], []
    for l in range(L):
        qrow, drow = [], []
        for j, (N, K) in enumerate(shapes[:7]):
            W = fq_synth.weights(700, N, K, 0.02, l, j)
            by = {b: oracle.quantize_rtn(W, b) for b in levels}
            qrow.append(by)
            drow.append({b: fq.PackedMatrix.from_host(*by[b], b) for b in levels})
        quantized.append(qrow)
        layers.append(drow)
    full = fq.Stack(layers)                       # every packing resident: the reference
    store = elastic.HostStore(quantized)
    path = make_path(7 * L, levels, 11)
    model = elastic.ElasticModel(store, path)
    assert store.stored_bytes() == sum(search.footprint_bytes((b,), [s]) for s in shapes for b in levels)

    def same(i, M):
        x = torch.from_numpy(fq_synth.activations(701 + M, M, sh["hidden"]).view(np.int16)).cuda().view(torch.float16)
        got = model.forward(x)
        want = fq.fq_stack_forward(full, np.asarray(path[i], dtype=np.uint8), x)
        return torch.equal(got.view(torch.int16), want.view(torch.int16))

    deq = {}

    def oracle_agrees(i, M):
        """The hosted member against the oracle's stack of that member's stored widths (Section "Transition
        Granularity": after the replacements the model IS member i), at the stack tolerance."""
        xh = fq_synth.activations(801 + M, M, sh["hidden"])
        mats = []
        for l in range(L):
            row = []
            for j in range(7):
                b = path[i][7 * l + j]
                if (l, j, b) not in deq:
                    deq[(l, j, b)] = oracle.dequant(*quantized[l][j][b])
                row.append(deq[(l, j, b)])
            mats.append(row)
        want = oracle.stack_forward(xh, mats).astype(np.float64)
        got = model.forward(torch.from_numpy(xh.view(np.int16)).cuda().view(torch.float16))
        got = got.cpu().view(torch.int16).numpy().view(np.float16).astype(np.float64)
        d = np.abs(got - want)
        return d.max() <= 2e-2 and d.mean() <= 2e-3

    assert model.resident_bytes() == model.footprints[0] and same(0, 1) and same(0, 40)
    assert oracle_agrees(0, 1) and oracle_agrees(0, 24)
    # shrink the budget step by step: the hosted member is always the largest that fits
    for budget in (model.footprints[5], model.footprints[20] + 1, model.footprints[-1]):
        i = model.set_budget(budget)
        assert i == elastic.fit(model.footprints, budget) and model.index == i
        assert model.resident_bytes() == model.footprints[i] <= budget
        assert tuple(int(b) for b in model.bitvec) == path[i]
        assert same(i, 1) and same(i, 40)
        assert oracle_agrees(i, 1) and oracle_agrees(i, 24)
    # swap by swap the transitional memory is one packing
    assert model.peak_extra_bytes <= max(search.footprint_bytes((b,), [s]) for s in shapes for b in levels)
    # memory comes back: grow again
    i = model.set_budget(model.footprints[7])
    assert i == 7 and model.resident_bytes() == model.footprints[7] and same(7, 1) and same(7, 40)
    # a queued move does not disturb serving until it is committed
    moves = model.begin_move(12)
    assert len(moves) == 5 and model.index == 7 and same(7, 1) and same(7, 40)
    with pytest.raises(RuntimeError):
        model.begin_move(13)
    model.commit()
    assert model.index == 12 and model.resident_bytes() == model.footprints[12] and same(12, 1) and same(12, 40)
    assert oracle_agrees(12, 1) and oracle_agrees(12, 24)
    # a non-resident width is refused by the library, not silently served
    bad = np.asarray(path[0], dtype=np.uint8)
    x = torch.zeros((1, sh["hidden"]), dtype=torch.float16, device="cuda")
    with pytest.raises(fq.FqError):
        fq.fq_stack_forward(model.stack, bad, x)
    torch.cuda.synchronize()
