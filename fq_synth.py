"""Seeded synthetic inputs for the mixed-bit quantized-linear path.

This module only draws random numbers and names shapes.  It holds none of the
method's arithmetic (no quantization, packing, matmul or loss code), so that the
CPU oracle and the GPU library can both be fed from it without sharing anything
else.

The shapes stand in for the Llama-family models the paper evaluates
(Section "Experiment"): Llama-2 7B (hidden 4096, FFN 11008, 32 layers) and
13B (hidden 5120, FFN 13824, 40 layers), a 32000-entry vocabulary and
2048/4096-token calibration rows.  Weights are N(0, 0.02^2) in fp32 (the usual
random initialisation), activations N(0, 1) rounded to fp16, labels uniform.
"""
from __future__ import annotations

import numpy as np

BIT_WIDTHS = (2, 3, 4, 8)
GROUP = 128
VOCAB = 32000
MATRIX_NAMES = ("q", "k", "v", "o", "gate", "up", "down")

MODEL_SHAPES = {
    "7b": {"hidden": 4096, "ffn": 11008, "layers": 32},
    "13b": {"hidden": 5120, "ffn": 13824, "layers": 40},
    # small stand-in with the same structure, for tests the oracle finishes quickly
    "tiny": {"hidden": 256, "ffn": 640, "layers": 3},
}


def block_matrix_shapes(hidden: int, ffn: int):
    """(N_out, K_in) of the seven linears of one decoder block, in MATRIX_NAMES order."""
    return [
        (hidden, hidden),
        (hidden, hidden),
        (hidden, hidden),
        (hidden, hidden),
        (ffn, hidden),
        (ffn, hidden),
        (hidden, ffn),
    ]


def _rng(seed, *stream):
    key = np.array([int(seed) & 0xFFFFFFFFFFFFFFFF, _fold(stream)], dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=key))


def _fold(stream) -> int:
    h = 0x9E3779B97F4A7C15
    for s in stream:
        h = (h * 0x100000001B3 + int(s) + 0x632BE59BD9B4E019) & 0xFFFFFFFFFFFFFFFF
    return h


def weights(seed: int, n: int, k: int, std: float = 0.02, *stream) -> np.ndarray:
    """fp32 [n, k] ~ N(0, std^2)."""
    g = _rng(seed, 1, *stream)
    w = g.standard_normal((n, k), dtype=np.float32)
    w *= np.float32(std)
    return w


def activations(seed: int, m: int, k: int, *stream) -> np.ndarray:
    """fp16 [m, k] ~ N(0, 1), drawn in fp32 and rounded once."""
    g = _rng(seed, 2, *stream)
    return g.standard_normal((m, k), dtype=np.float32).astype(np.float16)


def labels(seed: int, m: int, vocab: int = VOCAB, *stream) -> np.ndarray:
    """int32 [m] uniform in [0, vocab)."""
    g = _rng(seed, 3, *stream)
    return g.integers(0, vocab, size=m, dtype=np.int64).astype(np.int32)


def logits(seed: int, m: int, vocab: int = VOCAB, std: float = 1.28, *stream) -> np.ndarray:
    """fp16 [m, vocab] ~ N(0, std^2): the spread a random-init 4096-wide head gives."""
    g = _rng(seed, 4, *stream)
    x = g.standard_normal((m, vocab), dtype=np.float32)
    x *= np.float32(std)
    return x.astype(np.float16)


def bit_vector(seed: int, count: int, probs=None) -> np.ndarray:
    """uint8 [count]: one bit-width per matrix, iid with P over BIT_WIDTHS.

    The default (.30, .30, .30, .10) averages 3.5 bits.
    """
    if probs is None:
        probs = (0.30, 0.30, 0.30, 0.10)
    g = _rng(seed, 5)
    idx = g.choice(len(BIT_WIDTHS), size=count, p=np.asarray(probs, dtype=np.float64))
    return np.asarray(BIT_WIDTHS, dtype=np.uint8)[idx]


def codes(seed: int, n: int, k: int, bits: int, *stream) -> np.ndarray:
    """uint8 [n, k] uniform in [0, 2^bits)."""
    g = _rng(seed, 6, *stream)
    return g.integers(0, 1 << bits, size=(n, k), dtype=np.uint8)
