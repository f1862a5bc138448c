"""Sensitivity analysis of the ensemble search, as a driver over the library's entry points.

FlexQuant (arXiv 2501.07139, Section "Efficient Design Space Navigation") ranks the candidates of every search step with a
table built once: take QM(n_up), lower one module at a time to each lower bit-width, and record the
Euclidean distance between the logits of that hybrid model and those of QM(n_up) on the calibration
batch.  The smaller the distance, the earlier the module is lowered.

A candidate differs from QM(n_up) in one matrix of one block, so everything below that block is shared:
the driver keeps the input of every block under QM(n_up) and runs a candidate from its block onwards
(half the blocks on average).  All arithmetic happens in the library's kernels (`fq_stack_forward`,
`fq_dense_f16`, `fq_logit_l2`); this module only sequences the calls and sums the per-row results.
"""
from __future__ import annotations

from typing import Dict, Iterable, List, Optional, Sequence, Tuple

import numpy as np

from . import BIT_WIDTHS, Stack, fq_dense_f16, fq_logit_l2, fq_stack_forward, fq_stack_workspace_bytes


def sensitivity_table(stack: Stack, head, bitvec_up, x, lower_bits: Optional[Sequence[int]] = None,
                      entries: Optional[Iterable[int]] = None) -> Dict[Tuple[int, int], float]:
    """Distance between the logits of QM(n_up) with one matrix lowered and those of QM(n_up).

    stack      the stored packings (every bit-width a candidate may select must be present)
    head       fp16 [V, hidden] device tensor, the unquantized vocabulary head
    bitvec_up  uint8 [7 L], the bit-width of every matrix in QM(n_up)
    x          fp16 [M, hidden] device tensor, the calibration rows entering block 0
    lower_bits bit-widths to try below a matrix's own (default: all stored ones that are lower)
    entries    indices into bitvec_up to analyse (default: all)

    Returns {(entry, bits): distance}, the distance taken over the whole batch:
    sqrt(sum over rows and vocabulary of the squared logit difference).
    """
    import torch

    bitvec_up = np.asarray(bitvec_up, dtype=np.uint8)
    L = stack.L
    if bitvec_up.size != 7 * L:
        raise ValueError("bitvec_up needs 7 entries per block")
    M = x.shape[0]
    ws = torch.empty(fq_stack_workspace_bytes(M, stack.hidden, stack.ffn), dtype=torch.uint8, device=x.device)
    subs = [Stack(stack.layers[l:]) for l in range(L)]  # tables of the blocks l.. for a run from block l

    # inputs of every block under QM(n_up), and its logits
    inputs = [x]
    one = [Stack([stack.layers[l]]) for l in range(L)]
    for l in range(L):
        inputs.append(fq_stack_forward(one[l], bitvec_up[7 * l:7 * l + 7], inputs[l], workspace=ws))
    ref_logits = fq_dense_f16(inputs[L], head)

    table: Dict[Tuple[int, int], float] = {}
    hidden_out = torch.empty_like(x)
    logits = torch.empty_like(ref_logits)
    dist = torch.empty(M, dtype=torch.float32, device=x.device)
    for e in (range(7 * L) if entries is None else entries):
        l = e // 7
        own = int(bitvec_up[e])
        stored = [b for b in BIT_WIDTHS if b in stack.layers[l][e % 7]]
        for b in (lower_bits if lower_bits is not None else stored):
            if b >= own or b not in stored:
                continue
            cand = bitvec_up[7 * l:].copy()
            cand[e - 7 * l] = b
            fq_stack_forward(subs[l], cand, inputs[l], out=hidden_out, workspace=ws)
            fq_dense_f16(hidden_out, head, out=logits)
            fq_logit_l2(logits, ref_logits, out=dist)
            table[(e, b)] = float(np.sqrt(np.sum(dist.cpu().numpy().astype(np.float64) ** 2)))  # host: M values
    return table


def analysis_filter(table: Dict[Tuple[int, int], float], candidates: Sequence[Tuple[int, int]], branch: int
                    ) -> List[Tuple[int, int]]:
    """The #branch candidates (entry, bits) with the smallest recorded distance, smallest first."""
    ranked = sorted(candidates, key=lambda c: (table[c], c))
    return ranked[:branch]
