"""Pins of the real-decoder-block reference (oracle/decoder_ref.py) to what the published definitions fix:
closed forms of the rotary embedding and of softmax attention, invariants, brute force on tiny inputs, and
the equivalence of token-by-token decoding with the masked whole-sequence product (two routes, one result).
CPU only."""
import math

import numpy as np
import pytest

import fq_synth
import oracle
from oracle import decoder_ref as ref


def f16(a):
    return np.asarray(a, dtype=np.float64).astype(np.float16)


# ------------------------------------------------------------------------ rope
def test_rope_closed_forms():
    d = 128
    x = np.zeros(d)
    x[64] = 1.0                               # first element of pair i = 32: theta = 10000^(-64/128) = 0.01
    y = ref.rope(x, 100, 1)
    assert abs(y[64] - math.cos(1.0)) < 1e-15 and abs(y[65] - math.sin(1.0)) < 1e-15
    assert np.count_nonzero(y) == 2
    x = np.zeros(d)
    x[1] = 1.0                                # second element of pair 0: theta = 1
    y = ref.rope(x, 2, 1)
    assert abs(y[0] + math.sin(2.0)) < 1e-15 and abs(y[1] - math.cos(2.0)) < 1e-15
    x = np.zeros(d)
    x[126] = 3.0                              # last pair: theta = 10000^(-126/128)
    th = 10000.0 ** (-126.0 / 128.0)
    y = ref.rope(x, 4000, 1)
    assert abs(y[126] - 3 * math.cos(4000 * th)) < 1e-12 and abs(y[127] - 3 * math.sin(4000 * th)) < 1e-12


def test_rope_invariants():
    rng = np.random.default_rng(0)
    H, nh = 256, 4
    q, k = rng.normal(size=H), rng.normal(size=H)
    assert np.array_equal(ref.rope(q, 0, nh), q)                       # position 0 is the identity
    r = ref.rope(q, 37, nh).reshape(-1, 2)
    assert np.allclose((r ** 2).sum(1), (q.reshape(-1, 2) ** 2).sum(1), rtol=1e-13)   # every pair keeps its norm
    # the product of two rotated vectors depends on the distance of their positions only, head by head
    for m, n in ((50, 20), (7, 7), (3, 90)):
        a = (ref.rope(q, m, nh) * ref.rope(k, n, nh)).reshape(nh, -1).sum(1)
        b = (ref.rope(q, m - n + 100, nh) * ref.rope(k, 100, nh)).reshape(nh, -1).sum(1)
        assert np.allclose(a, b, rtol=1e-10, atol=1e-12)
    # heads are rotated alike: a head's result does not depend on which head it is
    one = ref.rope(q[:64], 11, 1)
    assert np.array_equal(ref.rope(np.tile(q[:64], 4), 11, 4), np.tile(one, 4))
    # rotations compose: position m then n more = position m + n
    assert np.allclose(ref.rope(ref.rope(q, 5, nh), 9, nh), ref.rope(q, 14, nh), rtol=1e-12, atol=1e-14)


# ------------------------------------------------------------------- attention
def test_attention_closed_forms():
    rng = np.random.default_rng(1)
    H, nh = 32, 2
    q = rng.normal(size=H)
    V = rng.normal(size=(5, H))
    K = rng.normal(size=(5, H))
    assert np.allclose(ref.attention(q, K[:1], V[:1], nh), V[0], rtol=1e-15)         # one position: its value
    same = np.tile(K[0], (5, 1))
    assert np.allclose(ref.attention(q, same, V, nh), V.mean(0), rtol=1e-12)          # equal keys: the mean
    big = K.copy()
    big[3] = 1e3 * q                                                                  # one key dominates
    assert np.allclose(ref.attention(q, big, V, nh), V[3], rtol=1e-12)
    perm = rng.permutation(5)
    assert np.allclose(ref.attention(q, K[perm], V[perm], nh), ref.attention(q, K, V, nh), rtol=1e-12)
    # the 1/sqrt(d) scale: d = 4, q.k = (2, 0) -> scores (1, 0) -> weights e/(1+e), 1/(1+e)
    q4 = np.array([2.0, 0, 0, 0])
    K4 = np.array([[1.0, 0, 0, 0], [0, 1.0, 0, 0]])
    V4 = np.array([[1.0, 0, 0, 0], [0, 0, 0, 1.0]])
    out = ref.attention(q4, K4, V4, 1)
    e = math.e
    assert np.allclose(out, [e / (1 + e), 0, 0, 1 / (1 + e)], rtol=1e-14)
    # heads do not mix: head 1's output is untouched by head 0's inputs
    q2, K2, V2 = q.copy(), K.copy(), V.copy()
    q2[:16] += 5.0
    K2[:, :16] *= -2.0
    V2[:, :16] += 1.0
    assert np.array_equal(ref.attention(q2, K2, V2, nh)[16:], ref.attention(q, K, V, nh)[16:])


def test_attention_brute_force():
    rng = np.random.default_rng(2)
    T, nh, d = 3, 2, 4
    q, K, V = rng.normal(size=nh * d), rng.normal(size=(T, nh * d)), rng.normal(size=(T, nh * d))
    want = []
    for h in range(nh):
        s = [sum(q[h * d + i] * K[t][h * d + i] for i in range(d)) / math.sqrt(d) for t in range(T)]
        z = sum(math.exp(v) for v in s)
        for i in range(d):
            want.append(sum(math.exp(s[t]) / z * V[t][h * d + i] for t in range(T)))
    assert np.allclose(ref.attention(q, K, V, nh), want, rtol=1e-13)


# ----------------------------------------------------------------------- block
def small_mats(seed, H, F, zero=()):
    mats = []
    for j, (N, K) in enumerate(fq_synth.block_matrix_shapes(H, F)):
        W = fq_synth.weights(seed, N, K, 0.05, 0, j)
        mats.append(np.zeros_like(W) if j in zero else W)
    return mats


def test_block_is_the_identity_when_o_and_down_are_zero():
    H, F, nh = 128, 256, 2
    x = fq_synth.activations(1, 1, H)
    kc, vc = np.zeros((4, H), np.float16), np.zeros((4, H), np.float16)
    t = ref.decode_block(x, small_mats(3, H, F, zero=(3, 6)), kc, vc, 2, nh)
    assert np.array_equal(t["x_next"], x) and np.array_equal(t["x1"], x)              # two residual adds, no norm after
    # the cache row of this position: the rotated key and the plain value; other rows untouched
    assert np.array_equal(kc[2], t["kr"][0]) and np.array_equal(vc[2], t["v"][0])
    assert not kc[[0, 1, 3]].any() and not vc[[0, 1, 3]].any()
    assert np.array_equal(t["kr"][0], oracle.round_f16(ref.rope(t["k"][0], 2, nh)))
    assert not np.array_equal(t["kr"], t["k"])


def test_block_with_identity_matrices_reduces_to_the_formula():
    """H = F = 128, every matrix the identity, position 0 with an empty cache: attention returns v = u, so
    x1 = x + u, and the MLP adds silu(u2)^2-like term with no normalisation of its own."""
    H, nh = 128, 1
    eye = np.eye(H, dtype=np.float32)
    x = fq_synth.activations(5, 1, H)
    kc, vc = np.zeros((1, H), np.float16), np.zeros((1, H), np.float16)
    t = ref.decode_block(x, [eye] * 7, kc, vc, 0, nh)
    xf = x.astype(np.float64)
    u = f16(xf / np.sqrt((xf ** 2).mean() + 1e-5))
    x1 = f16(xf + u.astype(np.float64))
    x1f = x1.astype(np.float64)
    u2 = f16(x1f / np.sqrt((x1f ** 2).mean() + 1e-5)).astype(np.float64)
    m = f16(u2 / (1 + np.exp(-u2)) * u2)
    want = f16(x1f + m.astype(np.float64))
    assert np.array_equal(t["a"], u) and np.array_equal(t["x1"], x1)
    assert np.array_equal(t["m"], m) and np.array_equal(t["x_next"], want)


def test_token_by_token_decoding_equals_the_masked_sequence_product():
    H, F, nh, T = 128, 256, 2, 6
    mats = small_mats(7, H, F)
    X = fq_synth.activations(8, T, H)
    kc, vc = np.zeros((T, H), np.float16), np.zeros((T, H), np.float16)
    rows = [ref.decode_block(X[t:t + 1], mats, kc, vc, t, nh)["x_next"][0] for t in range(T)]
    got = np.stack(rows).astype(np.float64)
    want = ref.sequence_block(X, mats, nh).astype(np.float64)
    # same roundings, different summation routes: a few fp16 ulps at most, and most entries identical
    assert np.max(np.abs(got - want)) <= 4e-3 * np.max(np.abs(want))
    assert np.mean(got == want) > 0.97
    # causality: changing a later token leaves earlier outputs alone
    X2 = X.copy()
    X2[4] = fq_synth.activations(9, 1, H)[0]
    kc2, vc2 = np.zeros((T, H), np.float16), np.zeros((T, H), np.float16)
    rows2 = [ref.decode_block(X2[t:t + 1], mats, kc2, vc2, t, nh)["x_next"][0] for t in range(T)]
    assert all(np.array_equal(rows[t], rows2[t]) for t in range(4)) and not np.array_equal(rows[5], rows2[5])


def test_sequence_attention_rows_are_the_decode_attention():
    rng = np.random.default_rng(4)
    T, nh = 9, 2
    H = 128 * nh
    q, k, v = (rng.normal(size=(T, H)).astype(np.float16) for _ in range(3))
    a, kr = ref.sequence_attention(q, k, v, nh)
    for t in range(T):
        assert np.array_equal(kr[t], oracle.round_f16(ref.rope(k[t], t, nh)))
        row = ref.attention(oracle.round_f16(ref.rope(q[t], t, nh)), kr[:t + 1], v[:t + 1], nh)
        assert np.max(np.abs(a[t].astype(np.float64) - row)) <= 1e-3 * max(1.0, np.abs(row).max())
    # the sequence route fills the caches the way decoding does
    H2, F2 = 128, 256
    mats = small_mats(7, H2, F2)
    X = fq_synth.activations(8, 5, H2)
    kc, vc = np.zeros((6, H2), np.float16), np.zeros((6, H2), np.float16)
    ref.sequence_block(X, mats, 1, kc, vc)
    kd, vd = np.zeros((6, H2), np.float16), np.zeros((6, H2), np.float16)
    for t in range(5):
        ref.decode_block(X[t:t + 1], mats, kd, vd, t, 1)
    assert np.array_equal(kc, kd) and np.array_equal(vc, vd) and not kc[5].any()


def test_decode_step_runs_the_blocks_in_order():
    H, F, nh, L = 128, 256, 2, 3
    layers = [small_mats(20 + l, H, F) for l in range(L)]
    x = fq_synth.activations(30, 1, H)
    kcs, vcs = np.zeros((L, 2, H), np.float16), np.zeros((L, 2, H), np.float16)
    got = ref.decode_step(x, layers, kcs, vcs, 0, nh)
    y = x
    for l in range(L):
        y = ref.decode_block(y, layers[l], np.zeros((2, H), np.float16), np.zeros((2, H), np.float16), 0, nh)["x_next"]
    assert np.array_equal(got, y) and kcs[:, 0].any() and not kcs[:, 1].any()
