"""Plain reference of the ensemble tree search (FlexQuant, arXiv 2501.07139, Algorithm 1 and the prose of
Section "Efficient Design Space Navigation").  Test infrastructure: slow, no caching, no GPU; only the tests use it.

Steps, in the paper's order and names, for a beam of #stem paths (the prose's reading of the single list of
the listing):
  EQM_last        the last model of every path
  candidateGenerator   every model obtained from an EQM_last by moving ONE matrix to one of its lower stored
                       bit-widths (one-way: never up); below QM(n_up) these are the (m+1) * #module options
                       the section counts
  analysisFilter  per EQM_last, the #branch candidates whose (matrix, new bits) has the smallest value in the
                  pre-built sensitivity table
  calibrationEval the perplexity of a candidate, from the caller's function
  rank            the pooled candidates (duplicates once, attributed to the first path that produced them)
                  by perplexity; ties by smaller footprint, then by the bit vector
  the first #stem become the new EQM_last of their parents' paths
until no EQM_last has a successor, i.e. all have reached QM(n_low).  Result: the paths, by mean perplexity.
"""
import numpy as np


def footprint(bits, shapes, group=128):
    return sum(n * k * int(b) // 8 + 2 * 2 * n * (k // group) for b, (n, k) in zip(bits, shapes))


def tree_search_ref(start, levels, sensitivity, calibration_eval, shapes, stems, branches, pools=None):
    """pools, if a list, receives the candidates scored by every iteration, in rank order."""
    levels = sorted(levels)
    start = tuple(int(b) for b in start)
    paths = [[(start, calibration_eval(start))]]
    while True:
        pooled = []  # (candidate, index of the parent path)
        seen = set()
        for pi, path in enumerate(paths):
            last = path[-1][0]
            cands = []
            for entry in range(len(last)):
                for lower in levels:
                    if lower >= last[entry]:
                        continue  # one-way: only lower stored widths
                    cand = list(last)
                    cand[entry] = lower
                    cands.append((sensitivity[(entry, lower)], entry, lower, tuple(cand)))
            cands.sort()
            for _, _, _, cand in cands[:branches]:
                if cand not in seen:
                    seen.add(cand)
                    pooled.append((cand, pi))
        if not pooled:
            break
        ranked = sorted((calibration_eval(c), footprint(c, shapes), c, pi) for c, pi in pooled)
        if pools is not None:
            pools.append([c for _, _, c, _ in ranked])
        paths = [paths[pi] + [(c, ppl)] for ppl, _, c, pi in ranked[:stems]]
    return sorted(paths, key=lambda p: (float(np.mean([ppl for _, ppl in p])), p[-1][0]))


def prune_ref(ensemble, levels, shapes, rate):
    """Section "EQM Pruning Strategy", written out plainly: count, per stored mid-level packing
    (matrix, bits), the models of the ensemble that use it; rank by count (more first), equal counts by the
    mean footprint of the using models (lower first), never-used packings last; drop the bottom `rate`
    share; what stays stored is every n_low and n_up packing plus the kept mid-level ones."""
    levels = sorted(levels)
    mids = levels[1:-1]
    rows = []
    for entry in range(len(shapes)):
        for bits in mids:
            users = [footprint(m, shapes) for m in ensemble if m[entry] == bits]
            mean_fp = sum(users) / len(users) if users else float("inf")
            rows.append((-len(users), mean_fp, entry, bits))
    rows.sort()
    ranking = [(entry, bits) for _, _, entry, bits in rows]
    ndrop = int(rate * len(ranking) + 1e-9)
    dropped = set(ranking[len(ranking) - ndrop:]) if ndrop else set()
    kept = [m for m in ensemble if all((e, b) not in dropped for e, b in enumerate(m))]
    stored = 0
    for entry, shape in enumerate(shapes):
        for bits in levels:
            if (entry, bits) not in dropped:
                stored += footprint((bits,), [shape])
    return ranking, dropped, kept, stored

