"""Run-time side of elastic hosting: keep ONE hybrid model resident and move it along the ensemble as the
memory budget changes (FlexQuant, arXiv 2501.07139, Sections "Transition Granularity" and "FlexQuant
Framework").

The ensemble is the search's output: bit vectors ordered from QM(n_up) down to QM(n_low), consecutive ones
differing in few matrices (one, when it is a path of the tree search).  Every stored packing lives in pinned
host memory (the device's "storage"); only the packings the current model selects are in HBM.  A move to
another member swaps matrix by matrix, the way the paper prescribes for a replacement: the new packing is
loaded next to the current model, the model's table entry is flipped, then the old packing is released, so
the transitional memory is one matrix's packing.  Uploads run on a copy stream; the model keeps serving with
its old table until `commit()`.

All arithmetic is `fq_stack_forward`; this module only moves bytes and flips pointers.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from . import BIT_WIDTHS, PackedMatrix, Stack, fq_pack_groups, fq_stack_forward, fq_stack_workspace_bytes
from .search import footprint_bytes

BitVec = Tuple[int, ...]
Move = Tuple[int, int, int]  # (entry, bits now, bits after)


def fit(footprints: Sequence[int], budget: int) -> int:
    """Index of the member to host under `budget` bytes: the largest footprint that fits (the paper's
    "fits in the available memory yet maximizes performance").  footprints must be non-increasing."""
    if any(b > a for a, b in zip(footprints, footprints[1:])):
        raise ValueError("ensemble must be ordered by non-increasing footprint")
    for i, f in enumerate(footprints):
        if f <= budget:
            return i
    raise MemoryError("no member of the ensemble fits in %d bytes (smallest needs %d)" % (budget, footprints[-1]))


def plan(ensemble: Sequence[BitVec], cur: int, target: int) -> List[Move]:
    """The swaps that take member `cur` to member `target`, walking the ensemble member by member so that
    every intermediate state is itself a member.  Entries are flat indices 7*block + matrix."""
    moves: List[Move] = []
    step = 1 if target > cur else -1
    for i in range(cur, target, step):
        a, b = ensemble[i], ensemble[i + step]
        for e, (x, y) in enumerate(zip(a, b)):
            if x != y:
                moves.append((e, int(x), int(y)))
    return moves


def transitional_bytes(moves: Sequence[Move], shapes: Sequence[Tuple[int, int]]) -> int:
    """Largest packing loaded next to the model during `moves`: the transitional memory cost."""
    return max((footprint_bytes((nb,), [shapes[e]]) for e, _, nb in moves), default=0)


class HostStore:
    """Every stored packing of every matrix, in pinned host memory in the device format."""

    def __init__(self, quantized: Sequence[Sequence[Dict[int, tuple]]]):
        # quantized[l][j][bits] = (codes u8 [N,K], scales fp16 [N,K/128], zeros fp16 [N,K/128])
        import torch

        self.L = len(quantized)
        self.shapes: List[Tuple[int, int]] = []
        self.blobs: List[Dict[int, tuple]] = []
        for mats in quantized:
            if len(mats) != 7:
                raise ValueError("a block has seven matrices")
            for by_bits in mats:
                N, K = next(iter(by_bits.values()))[0].shape
                self.shapes.append((N, K))
                entry = {}
                for bits, (codes, scales, zeros) in by_bits.items():
                    p, s, z = fq_pack_groups(codes, scales, zeros, bits)
                    entry[int(bits)] = tuple(torch.from_numpy(a).pin_memory()
                                             for a in (p, s.view(np.int16), z.view(np.int16)))
                self.blobs.append(entry)

    def stored_bytes(self) -> int:
        return sum(footprint_bytes((b,), [self.shapes[e]]) for e, by in enumerate(self.blobs) for b in by)

    def upload(self, entry: int, bits: int, device) -> PackedMatrix:
        """Queue the copies of one packing on the current stream; returns its device tensors."""
        import torch

        p, s, z = self.blobs[entry][bits]
        N, K = self.shapes[entry]
        dp, ds, dz = (torch.empty_like(t, device=device) for t in (p, s, z))
        for d, h in ((dp, p), (ds, s), (dz, z)):
            d.copy_(h, non_blocking=True)
        return PackedMatrix(dp, ds.view(torch.float16), dz.view(torch.float16), N, K, bits)


class ElasticModel:
    """One resident member of an ensemble, movable along it."""

    def __init__(self, store: HostStore, ensemble: Sequence[Sequence[int]], start: int = 0, device="cuda"):
        import torch

        self.store, self.device = store, torch.device(device)
        self.ensemble: List[BitVec] = [tuple(int(b) for b in v) for v in ensemble]
        if any(len(v) != 7 * store.L for v in self.ensemble):
            raise ValueError("bit vectors need 7 entries per block")
        self.footprints = [footprint_bytes(v, store.shapes) for v in self.ensemble]
        fit(self.footprints, self.footprints[0])  # checks the order
        self.index = start
        self.copy_stream = torch.cuda.Stream(device=self.device)  # default priority
        self.resident: List[PackedMatrix] = [store.upload(e, b, self.device) for e, b in enumerate(self.ensemble[start])]
        torch.cuda.current_stream(self.device).synchronize()
        layers = [[{w.bits: w} for w in self.resident[7 * l:7 * l + 7]] for l in range(store.L)]
        self.stack = Stack(layers)
        self.bitvec = np.asarray(self.ensemble[start], dtype=np.uint8)
        self._pending: Optional[tuple] = None
        self._ws = None
        self.peak_extra_bytes = 0
        self.bytes_loaded = 0

    # ------------------------------------------------------------------ state
    def resident_bytes(self) -> int:
        return sum(w.nbytes for w in self.resident)

    def forward(self, x, out=None):
        import torch

        M = x.shape[0]
        need = fq_stack_workspace_bytes(M, self.stack.hidden, self.stack.ffn)
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        return fq_stack_forward(self.stack, self.bitvec, x, out=out, workspace=self._ws)

    # ------------------------------------------------------------ transitions
    def begin_move(self, target: int) -> List[Move]:
        """Queue the uploads for the move to member `target` on the copy stream.  The model keeps its table:
        forward() serves the current member until commit().  All new packings of the move are loaded before
        any old one is released, so the transitional memory is their sum; move_to() goes one swap at a time
        and keeps it at one packing."""
        import torch

        if self._pending is not None:
            raise RuntimeError("a move is already pending")
        moves = plan(self.ensemble, self.index, target)
        final: Dict[int, int] = {}
        for e, _, nb in moves:
            final[e] = nb
        new: Dict[int, PackedMatrix] = {}
        main = torch.cuda.current_stream(self.device)
        self.copy_stream.wait_stream(main)  # memory handed out below may still be in use by queued kernels
        with torch.cuda.stream(self.copy_stream):
            for e, nb in final.items():
                if nb != self.resident[e].bits:
                    new[e] = self.store.upload(e, nb, self.device)
        done = torch.cuda.Event()
        done.record(self.copy_stream)
        extra = sum(w.nbytes for w in new.values())
        self.peak_extra_bytes = max(self.peak_extra_bytes, extra)
        self.bytes_loaded += extra
        self._pending = (target, new, done)
        return moves

    def commit(self) -> None:
        """Make the compute stream wait for the uploads, flip the table entries, release the old packings."""
        import torch

        if self._pending is None:
            return
        target, new, done = self._pending
        main = torch.cuda.current_stream(self.device)
        main.wait_event(done)
        for e, w in new.items():
            l, j = divmod(e, 7)
            old = self.resident[e]
            for t in (w.packed, w.scales, w.zeros):
                t.record_stream(main)  # allocated under the copy stream, used (and later freed) under this one
            self._flip(l, j, old.bits, w)
            self.resident[e] = w
            self.stack.layers[l][j] = {w.bits: w}
        self.index = target
        self.bitvec = np.asarray(self.ensemble[target], dtype=np.uint8)
        self._pending = None

    def move_to(self, target: int) -> List[Move]:
        """Move member by member, swap by swap: load one packing, flip, release the old one."""
        done: List[Move] = []
        step = 1 if target > self.index else -1
        while self.index != target:
            done += self.begin_move(self.index + step)
            self.commit()
        return done

    def set_budget(self, budget_bytes: int) -> int:
        """Host the best member that fits; returns its index."""
        target = fit(self.footprints, budget_bytes)
        self.move_to(target)
        return target

    def _flip(self, l: int, j: int, old_bits: int, w: PackedMatrix) -> None:
        entry = self.stack.table[l].m[j]
        i_old, i_new = BIT_WIDTHS.index(old_bits), BIT_WIDTHS.index(w.bits)
        entry.packed[i_old] = entry.scales[i_old] = entry.zeros[i_old] = None
        entry.packed[i_new], entry.scales[i_new], entry.zeros[i_new] = (w.packed.data_ptr(), w.scales.data_ptr(),
                                                                        w.zeros.data_ptr())
