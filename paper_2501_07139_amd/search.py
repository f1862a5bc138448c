"""Tree search for the ensemble of hybrid models (FlexQuant, arXiv 2501.07139, Algorithm 1), as a driver
over the library's entry points.

An EQM is a bit vector: one stored bit-width per matrix.  From QM(n_up) the search lowers one matrix per step
to any of its lower stored bit-widths (transitions are one-way; Section "Efficient Design Space Navigation"
counts (m+1) * #module options below the root, m the number of models between n_low and n_up) until
QM(n_low) is reached; every step generates the successors of the current models, keeps the #branch least sensitive ones per model (analysis filter, from
the pre-built table of `sweep.sensitivity_table`), scores those on the calibration rows (perplexity) and
keeps the #stem best as the new current models.

Readings of the text (Algorithm 1 keeps one list where the prose keeps #stem of them): the search is a beam
of #stem paths; the candidates of all current models form one pool, duplicates are scored once, the pool is
ranked by perplexity (ties: smaller footprint, then the bit vector itself) and its first #stem members
become the current models, each remembering its parent.  A candidate may coincide with a model another
path reached earlier (one path lowers a matrix in two steps, another in one): it is scored again and, if
kept, the two paths continue as separate ensembles.  A current model already at QM(n_low) generates
nothing; the search ends when the pool is empty.  The output is every surviving path, best first by mean
perplexity of its members.

All arithmetic of the evaluation runs in the library's kernels (`fq_stack_forward`, `fq_head_nll`); a candidate differs from its parent in one block, so it is run from that block onwards over
the parent's cached block inputs.
"""
from __future__ import annotations

from typing import Callable, Dict, List, Optional, Sequence, Tuple

import numpy as np

BitVec = Tuple[int, ...]


def footprint_bytes(bitvec: Sequence[int], shapes: Sequence[Tuple[int, int]], group: int = 128) -> int:
    """Packed bytes of a hybrid model: codes plus one fp16 scale and zero per group."""
    total = 0
    for b, (n, k) in zip(bitvec, shapes):
        total += n * k * int(b) // 8 + 4 * n * (k // group)
    return total


def successors(bitvec: BitVec, levels: Sequence[int]) -> List[Tuple[int, int, BitVec]]:
    """(entry, new bits, new vector) for every entry lowered to each stored level below its own: from
    QM(n_up) these are the (m+1) * #module options of Section "Efficient Design Space Navigation"."""
    order = sorted(levels)
    out = []
    for e, b in enumerate(bitvec):
        for nb in order[:order.index(b)]:
            out.append((e, nb, bitvec[:e] + (nb,) + bitvec[e + 1:]))
    return out


class Node:
    __slots__ = ("bitvec", "ppl", "parent", "state")

    def __init__(self, bitvec: BitVec, ppl: float, parent: Optional["Node"], state=None):
        self.bitvec, self.ppl, self.parent, self.state = bitvec, ppl, parent, state

    def path(self) -> List["Node"]:
        n, out = self, []
        while n is not None:
            out.append(n)
            n = n.parent
        return out[::-1]


def tree_search(start: Sequence[int], levels: Sequence[int], sensitivity: Dict[Tuple[int, int], float],
                evaluate: Callable[[BitVec, Optional[Node], Optional[int]], Tuple[float, object]],
                shapes: Sequence[Tuple[int, int]], stems: int, branches: int,
                trace: Optional[list] = None) -> List[List[Node]]:
    """Algorithm 1.  `evaluate(bitvec, parent, entry)` returns (perplexity, state kept with the node); parent
    and the changed entry let it reuse the parent's work.  Returns the surviving paths, best first.  If
    `trace` is a list, every iteration appends its scored pool as [(bitvec, perplexity), ...] in rank order."""
    start = tuple(int(b) for b in start)
    ppl0, st0 = evaluate(start, None, None)
    current = [Node(start, ppl0, None, st0)]
    while True:
        pool: Dict[BitVec, Tuple[Node, int]] = {}
        for node in current:
            cands = successors(node.bitvec, levels)
            cands.sort(key=lambda c: (sensitivity[(c[0], c[1])], c[0], c[1]))  # analysis filter
            for e, nb, vec in cands[:branches]:
                pool.setdefault(vec, (node, e))  # a duplicate keeps its first parent
        if not pool:
            break
        scored = []
        for vec, (parent, e) in pool.items():
            ppl, st = evaluate(vec, parent, e)
            scored.append(Node(vec, ppl, parent, st))
        scored.sort(key=lambda n: (n.ppl, footprint_bytes(n.bitvec, shapes), n.bitvec))
        if trace is not None:
            trace.append([(n.bitvec, n.ppl) for n in scored])
        for n in scored[stems:]:
            n.state = None
        for n in current:
            n.state = None  # the parents' cached inputs are no longer needed
        current = scored[:stems]
    paths = [n.path() for n in current]
    paths.sort(key=lambda p: (float(np.mean([n.ppl for n in p])), p[-1].bitvec))
    return paths


def prune_ensemble(ensemble: Sequence[BitVec], levels: Sequence[int], shapes: Sequence[Tuple[int, int]],
                   rate: float):
    """Pruning of the stored mid-level packings (Section "EQM Pruning Strategy").

    Every packing (matrix, bits) with bits strictly between n_low and n_up is ranked by the number of models
    of the ensemble that use it; equal counts are ordered by the footprint at which they are used (mean over
    the using models, lower footprints first, since perplexity is most sensitive there); unused packings
    come last.  The lowest `rate` share of that ranking is dropped.  Returns (ranking best first, dropped
    set, models of the ensemble that need no dropped packing, stored bytes after pruning)."""
    order = sorted(levels)
    mids = order[1:-1]
    entries = len(shapes)
    use: Dict[Tuple[int, int], List[int]] = {(e, b): [] for e in range(entries) for b in mids}
    for vec in ensemble:
        f = footprint_bytes(vec, shapes)
        for e, b in enumerate(vec):
            if b in mids:
                use[(e, int(b))].append(f)
    def key(item):
        (e, b), fs = item
        return (-len(fs), float(np.mean(fs)) if fs else float("inf"), e, b)
    ranking = [k for k, _ in sorted(use.items(), key=key)]
    ndrop = int(np.floor(rate * len(ranking) + 1e-9))
    dropped = set(ranking[len(ranking) - ndrop:]) if ndrop else set()
    kept_models = [vec for vec in ensemble if not any((e, int(b)) in dropped for e, b in enumerate(vec))]
    stored = 0
    for e, (n, k) in enumerate(shapes):
        for b in order:
            if (e, b) not in dropped:
                stored += footprint_bytes((b,), [(n, k)])
    return ranking, dropped, kept_models, stored


class CalibrationEval:
    """calibrationEval of Algorithm 1 on the GPU: perplexity of a hybrid model over the calibration rows,
    exp(mean token NLL).  Keeps the input of every block with the node so that a successor restarts at the
    block it changes."""

    def __init__(self, stack, head, x, labels, real_blocks: bool = False):
        """real_blocks: run the blocks as real decoder blocks (rotary embedding, causal attention) with the
        calibration rows as ONE sequence at positions 0..M-1, instead of the attention-free stack."""
        import torch

        from . import (Stack, fq_head_nll_workspace_bytes, fq_prefill_workspace_bytes, fq_stack_workspace_bytes,
                       rope_table)

        self.stack, self.head, self.x, self.labels = stack, head, x, labels
        self.L = stack.L
        self.one = [Stack([stack.layers[l]]) for l in range(self.L)]
        M = x.shape[0]
        self.real = real_blocks
        if real_blocks:
            self.ws = torch.empty(fq_prefill_workspace_bytes(M, stack.hidden, stack.ffn), dtype=torch.uint8, device=x.device)
            self.rope = rope_table(M, device=x.device)
            self.kc = torch.empty((1, stack.hidden // 128, M, 128), dtype=torch.float16, device=x.device)
            self.vc = torch.empty_like(self.kc)
        else:
            self.ws = torch.empty(fq_stack_workspace_bytes(M, stack.hidden, stack.ffn), dtype=torch.uint8, device=x.device)
        self.ws_head = torch.empty(fq_head_nll_workspace_bytes(M, head.shape[0]), dtype=torch.uint8, device=x.device)
        self.evaluations = 0
        self.blocks_run = 0

    def __call__(self, bitvec: BitVec, parent: Optional[Node], entry: Optional[int]):
        from . import fq_head_nll, fq_prefill_forward, fq_stack_forward

        bv = np.asarray(bitvec, dtype=np.uint8)
        first = 0 if parent is None or parent.state is None else entry // 7
        inputs = [self.x] if first == 0 else list(parent.state[:first + 1])
        for l in range(first, self.L):
            if self.real:  # the caches are scratch here: every block of a sequence forward fills its own
                inputs.append(fq_prefill_forward(self.one[l], bv[7 * l:7 * l + 7], inputs[l], self.kc, self.vc,
                                                 self.rope, workspace=self.ws))
            else:
                inputs.append(fq_stack_forward(self.one[l], bv[7 * l:7 * l + 7], inputs[l], workspace=self.ws))
        nll = fq_head_nll(inputs[self.L], self.head, self.labels, workspace=self.ws_head)
        nll = nll.cpu().numpy().astype(np.float64)
        self.evaluations += 1
        self.blocks_run += self.L - first
        return float(np.exp(nll.mean())), inputs
