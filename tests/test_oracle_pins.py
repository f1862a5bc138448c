"""Pins for the CPU oracle: each checks it against something other than itself.

Closed forms, exact rational arithmetic (fractions), numpy's own IEEE half
conversion and float64 matmul, hand-derived bit positions, and the invariants
the paper states (nesting by truncation, an n-bit layer approximating its FP16
counterpart ever better as n grows).
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import fq_synth
import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
BITS = (2, 3, 4, 8)


# ----------------------------------------------------------------------- fp16
def test_half_to_double_matches_ieee_for_every_bit_pattern():
    pats = np.arange(65536, dtype=np.uint16)
    want = pats.view(np.float16).astype(np.float64)
    got = np.array([oracle.h2d(int(p)) for p in pats])
    both_nan = np.isnan(want) & np.isnan(got)
    assert np.all((got == want) | both_nan)
    assert np.all(np.signbit(got[~both_nan]) == np.signbit(want[~both_nan]))


def test_double_to_half_is_round_half_even_everywhere():
    rng = np.random.default_rng(7)
    vals = [0.0, -0.0, 1.0, -1.0, 65504.0, 65519.99, 65520.0, 7e4, -7e4, 2.0 ** -24, 2.0 ** -25,
            2.0 ** -25 * 1.0000001, 3 * 2.0 ** -25, 2.0 ** -14, 2.0 ** -14 - 2.0 ** -25, 1e-9, float("inf"),
            1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 1.0 + 2.0 ** -11 + 2.0 ** -30, 2047.5, 2048.5, 2049.0]
    # every halfway point between neighbouring halves, and just beside it
    pats = rng.integers(0, 0x7BFF, size=3000).astype(np.uint16)
    lo = pats.view(np.float16).astype(np.float64)
    hi = (pats + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    mid = (lo + hi) / 2
    vals += list(mid) + list(np.nextafter(mid, np.inf)) + list(np.nextafter(mid, -np.inf)) + list(-mid)
    vals += list(rng.standard_normal(5000) * np.exp(rng.uniform(-20, 12, size=5000)))
    vals = np.array(vals, dtype=np.float64)
    with np.errstate(over="ignore"):
        want = vals.astype(np.float16).view(np.uint16)
    got = np.array([oracle.d2h(float(v)) for v in vals], dtype=np.uint16)
    assert np.array_equal(got, want)
    assert np.array_equal(oracle.round_f16(vals).view(np.uint16), want)
    assert oracle.d2h(float("nan")) & 0x7C00 == 0x7C00 and oracle.d2h(float("nan")) & 0x3FF


# ------------------------------------------------------------------- quantize
def _on_grid(rng, N, K, bits, group=128):
    """Weights that sit exactly on a quantization grid, with 0 and maxq hit in every group."""
    maxq = (1 << bits) - 1
    G = K // group
    # any fp16 scale in a sane range, any integer zero
    s = (rng.uniform(1e-4, 1e-2, size=(N, G))).astype(np.float16)
    z = rng.integers(0, maxq + 1, size=(N, G)).astype(np.float16)
    q = rng.integers(0, maxq + 1, size=(N, K), dtype=np.uint8)
    q = q.reshape(N, G, group)
    q[:, :, 0] = 0
    q[:, :, 1] = maxq
    q = q.reshape(N, K)
    sf = np.repeat(s.astype(np.float32), group, axis=1)
    zf = np.repeat(z.astype(np.float32), group, axis=1)
    W = sf * (q.astype(np.float32) - zf)  # exact in fp32: <=9 bits times 11 bits
    return W, q, s, z


@pytest.mark.parametrize("bits", BITS)
def test_quantize_of_on_grid_weights_returns_the_grid(bits):
    rng = np.random.default_rng(100 + bits)
    W, q, s, z = _on_grid(rng, 24, 512, bits)
    cq, cs, cz = oracle.quantize_rtn(W, bits)
    assert np.array_equal(cs.view(np.uint16), s.view(np.uint16))
    assert np.array_equal(cz.view(np.uint16), z.view(np.uint16))
    assert np.array_equal(cq, q)
    assert np.array_equal(oracle.dequant(cq, cs, cz).view(np.uint32), W.view(np.uint32))


@pytest.mark.parametrize("bits", BITS)
def test_quantize_against_exact_rational_arithmetic(bits):
    """Scale, zero and every code agree with the definition evaluated in fractions."""
    W = fq_synth.weights(11, 6, 256)
    W[0, :128] = 0.0  # a degenerate all-zero group
    W[1, :128] = np.abs(W[1, :128])  # one-sided: range must still contain 0
    W[2, 128:] = -np.abs(W[2, 128:])
    codes, scales, zeros = oracle.quantize_rtn(W, bits)
    maxq = (1 << bits) - 1
    for n in range(W.shape[0]):
        for g in range(2):
            w = [Fraction(float(v)) for v in W[n, g * 128:(g + 1) * 128]]
            lo, hi = min(min(w), 0), max(max(w), 0)
            s = Fraction(float(scales[n, g]))
            z = Fraction(float(zeros[n, g]))
            if hi == lo:
                assert s == 1 and z == 0 and not codes[n, g * 128:(g + 1) * 128].any()
                continue
            exact_scale = float(np.float32(float(hi - lo)) / np.float32(maxq))  # fp32 quotient
            assert float(s) == float(np.float16(exact_scale))
            assert z.denominator == 1 and 0 <= z <= maxq
            assert abs(z - min(max(-lo / s, 0), maxq)) <= Fraction(1, 2) + Fraction(1, 10 ** 4)
            for i, wi in enumerate(w):
                ideal = min(max(wi / s + z, 0), maxq)
                assert abs(int(codes[n, g * 128 + i]) - ideal) <= Fraction(1, 2) + Fraction(1, 10 ** 4)


@pytest.mark.parametrize("bits", BITS)
def test_reconstruction_error_bound(bits):
    """|w - s(q-z)| <= 0.5 s + maxq |s - s32| <= 0.625 s inside the range."""
    W = fq_synth.weights(3, 32, 1024)
    q, s, z = oracle.quantize_rtn(W, bits)
    What = oracle.dequant(q, s, z)
    sf = np.repeat(s.astype(np.float64), 128, axis=1)
    assert np.all(np.abs(W.astype(np.float64) - What) <= 0.625 * sf + 1e-12)


def test_quantize_ties_round_to_even_and_codes_use_the_fp16_scale():
    # lo = 0, hi = 15 -> s = 1, z = 0; 0.5 -> 0, 1.5 -> 2, 2.5 -> 2, 3.5 -> 4
    w = np.zeros((1, 128), dtype=np.float32)
    w[0, :6] = [15.0, 0.5, 1.5, 2.5, 3.5, 14.5]
    q, s, z = oracle.quantize_rtn(w, 4)
    assert float(s[0, 0]) == 1.0 and float(z[0, 0]) == 0.0
    assert list(q[0, :6]) == [15, 0, 2, 2, 4, 14]
    # negative side: lo = -8 -> z = 8 for s = 1 (hi = 7)
    w[0, :6] = [7.0, -8.0, -0.5, -1.5, 0.0, 3.0]
    q, s, z = oracle.quantize_rtn(w, 4)
    assert float(s[0, 0]) == 1.0 and float(z[0, 0]) == 8.0
    assert list(q[0, :6]) == [15, 0, 8, 6, 8, 11]


# --------------------------------------------------------------------- unpack
def _golden_positions():
    rows = []
    with open(os.path.join(GOLDEN, "packed_positions.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            tok = line.split()
            bits, N, K, n, k = map(int, tok[:5])
            pos = [tuple(map(int, t.split(":"))) for t in tok[5:]]
            rows.append((bits, N, K, n, k, pos))
    return rows


@pytest.mark.parametrize("row", _golden_positions(), ids=lambda r: "b%d_n%d_k%d" % (r[0], r[3], r[4]))
def test_unpack_reads_hand_derived_bit_positions(row):
    bits, N, K, n, k, pos = row
    assert len(pos) == bits
    for i, (byte, bit) in enumerate(pos):
        buf = np.zeros(oracle.packed_bytes(N, K, bits), dtype=np.uint8)
        buf[byte] = 1 << bit
        codes = oracle.unpack(buf, N, K, bits)
        want = np.zeros((N, K), dtype=np.uint8)
        want[n, k] = 1 << i
        assert np.array_equal(codes, want)


@pytest.mark.parametrize("bits", BITS)
def test_unpack_is_a_bijection_on_bits(bits):
    """Every bit of the buffer feeds exactly one bit of exactly one code, none twice."""
    N, K = 64, 256
    nbytes = oracle.packed_bytes(N, K, bits)
    assert nbytes == N * K * bits // 8
    seen = np.zeros((N, K), dtype=np.uint16)
    for bit in range(8):
        # set bit `bit` of every 7th byte family in turn: 8*7 calls cover each bit once
        for phase in range(7):
            buf = np.zeros(nbytes, dtype=np.uint8)
            buf[phase::7] = 1 << bit
            codes = oracle.unpack(buf, N, K, bits).astype(np.uint16)
            assert not np.any(seen & codes)
            seen |= codes
    assert np.all(seen == (1 << bits) - 1)
    # and the count of set code bits equals the count of set buffer bits
    rng = np.random.default_rng(5)
    buf = rng.integers(0, 256, size=nbytes, dtype=np.uint8)
    codes = oracle.unpack(buf, N, K, bits)
    assert int(np.unpackbits(codes).sum()) == int(np.unpackbits(buf).sum())


def _pack_by_the_text(codes, bits):
    """The packed format written out once more, as a scatter, in plain Python ints."""
    N, K = codes.shape
    R = {2: 32, 3: 64, 4: 16, 8: 16}[bits]
    G = K // 128
    words = np.zeros(oracle.packed_bytes(N, K, bits) // 4, dtype=np.uint64)
    for n in range(N):
        for k in range(K):
            q = int(codes[n, k])
            u, r = divmod(n % R, 16)
            s, rem = divmod(k % 128, 32)
            c, e = divmod(rem, 8)
            t = 8 * s + e
            lane = 16 * c + r
            base = ((n // R) * G + k // 128) * (R * 16 * bits // 4)

            def word(i):
                j = bits * u + i
                return base + (j // 4) * 256 + 4 * lane + j % 4

            if bits == 4:
                words[word(s)] |= q << (16 * (e % 2) + 4 * (e // 2))
            elif bits == 8:
                words[word(2 * s + e // 4)] |= q << (16 * (e % 2) + 8 * ((e % 4) // 2))
            elif bits == 2:
                words[word(s // 2)] |= q << (16 * (e % 2) + 2 * (4 * (s % 2) + e // 2))
            elif t < 30:
                words[word(t // 10)] |= q << (16 * (t % 2) + 3 * ((t % 10) // 2))
            else:
                for i in range(3):
                    words[word(i)] |= ((q >> i) & 1) << (15 if t == 30 else 31)
    return words.astype("<u4").view(np.uint8)


@pytest.mark.parametrize("bits", BITS)
def test_unpack_inverts_a_scatter_written_from_the_text(bits):
    N, K = 70, 256  # ragged: 70 rows live in 128 padded rows
    for kind in ("random", "k_index", "n_index", "all_max"):
        if kind == "random":
            codes = fq_synth.codes(9, N, K, bits)
        elif kind == "k_index":
            codes = np.tile((np.arange(K) % (1 << bits)).astype(np.uint8), (N, 1))
        elif kind == "n_index":
            codes = np.tile((np.arange(N) % (1 << bits)).astype(np.uint8)[:, None], (1, K))
        else:
            codes = np.full((N, K), (1 << bits) - 1, dtype=np.uint8)
        packed = _pack_by_the_text(codes, bits)
        assert packed.size == 128 * K * bits // 8
        assert np.array_equal(oracle.unpack(packed, N, K, bits), codes)


def test_untile_meta_positions():
    N, G = 40, 3
    tiled = np.zeros(64 * G, dtype=np.uint16)
    # entry (n=17, g=2) lives at (17//16)*G*16 + 2*16 + 17%16
    tiled[1 * G * 16 + 2 * 16 + 1] = 0x3C00
    out = oracle.untile_meta(tiled, N, G)
    want = np.zeros((N, G), dtype=np.float16)
    want[17, 2] = 1.0
    assert np.array_equal(out, want)


# ------------------------------------------------------------------- dequant
def test_dequant_hand_values_and_exactness():
    codes = np.zeros((2, 128), dtype=np.uint8)
    codes[0, :4] = [0, 5, 15, 9]
    codes[1, :3] = [255, 0, 128]
    s = np.array([[0.5], [0.001953125]], dtype=np.float16)
    z = np.array([[9.0], [100.0]], dtype=np.float16)
    W = oracle.dequant(codes, s, z)
    assert list(W[0, :4]) == [-4.5, -2.0, 3.0, 0.0]
    assert list(W[1, :3]) == [155 * 0.001953125, -100 * 0.001953125, 28 * 0.001953125]
    # arbitrary fp16 scales: the fp32 result equals the exact rational product
    rng = np.random.default_rng(2)
    codes = rng.integers(0, 256, size=(8, 256), dtype=np.uint8)
    s = rng.uniform(1e-4, 1e-2, size=(8, 2)).astype(np.float16)
    z = rng.integers(0, 256, size=(8, 2)).astype(np.float16)
    W = oracle.dequant(codes, s, z)
    for n in range(8):
        for k in range(0, 256, 17):
            exact = Fraction(float(s[n, k // 128])) * (int(codes[n, k]) - Fraction(float(z[n, k // 128])))
            assert Fraction(float(W[n, k])) == exact


@pytest.mark.parametrize("bits", (2, 3, 4))
@pytest.mark.parametrize("midpoint", (False, True))
def test_truncated_codes_reconstruct_the_masked_high_precision_weights(bits, midpoint):
    """Section "Elastic Serving": dropping code bits yields the lower-precision layer."""
    W = fq_synth.weights(21, 16, 512)
    q8, s8, z8 = oracle.quantize_rtn(W, 8)
    d = 8 - bits
    q, s, z = oracle.truncate(q8, s8, z8, d, midpoint=midpoint)
    assert q.max() <= (1 << bits) - 1 and np.array_equal(q, q8 >> d)
    assert np.array_equal(s.astype(np.float64), s8.astype(np.float64) * 2 ** d)
    low = oracle.dequant(q, s, z).astype(np.float64)
    masked = oracle.dequant(q8 & ~np.uint8((1 << d) - 1), s8, z8).astype(np.float64)
    if midpoint:
        masked = masked + np.repeat(s8.astype(np.float64), 128, axis=1) * 2 ** (d - 1)
    assert np.array_equal(low, masked)


# -------------------------------------------------------------------- qlinear
def test_qlinear_against_exact_fractions_on_a_tiny_case():
    X = fq_synth.activations(4, 3, 256)
    W = fq_synth.weights(4, 5, 256)
    q, s, z = oracle.quantize_rtn(W, 3)
    W32 = oracle.dequant(q, s, z)
    Y = oracle.qlinear(X, W32)
    assert Y.shape == (3, 5)
    for m in range(3):
        for n in range(5):
            exact = sum(Fraction(float(X[m, k])) * Fraction(float(W32[n, k])) for k in range(256))
            assert abs(Y[m, n] - float(exact)) <= 1e-13 * max(1.0, abs(float(exact)))


def test_qlinear_and_dense_match_float64_matmul():
    X = fq_synth.activations(5, 7, 384)
    W32 = fq_synth.weights(5, 13, 384)
    want = X.astype(np.float64) @ W32.astype(np.float64).T
    assert np.allclose(oracle.qlinear(X, W32), want, rtol=1e-12, atol=1e-12)
    Wh = W32.astype(np.float16)
    want = X.astype(np.float64) @ Wh.astype(np.float64).T
    assert np.allclose(oracle.dense_f16(X, Wh), want, rtol=1e-12, atol=1e-12)


def test_qlinear_integer_case_is_exact():
    rng = np.random.default_rng(8)
    X = rng.integers(-4, 5, size=(4, 256)).astype(np.float16)
    codes = rng.integers(0, 16, size=(6, 256), dtype=np.uint8)
    s = np.full((6, 2), 0.25, dtype=np.float16)
    z = np.full((6, 2), 8.0, dtype=np.float16)
    Y = oracle.qlinear(X, oracle.dequant(codes, s, z))
    want = (X.astype(np.int64) @ (codes.astype(np.int64) - 8).T) * 0.25
    assert np.array_equal(Y, want.astype(np.float64))


def test_more_bits_approximate_the_unquantized_layer_better():
    """Section "FlexQuant Framework": an n-bit layer approximates its FP16 counterpart.

    Rounding noise of variance s^2/12 with a 128-sample Gaussian range of about
    5.2 sigma gives rms(Y_b - Y)/rms(Y) ~ 5.2 / ((2^b - 1) sqrt(12)).
    """
    X = fq_synth.activations(6, 16, 1024)
    W = fq_synth.weights(6, 96, 1024)
    Y = oracle.qlinear(X, W)
    err = {}
    for bits in BITS:
        q, s, z = oracle.quantize_rtn(W, bits)
        Yb = oracle.qlinear(X, oracle.dequant(q, s, z))
        err[bits] = np.sqrt(np.mean((Yb - Y) ** 2) / np.mean(Y ** 2))
    assert err[2] > err[3] > err[4] > err[8]
    assert err[8] < 1e-2
    for bits in BITS:
        model = 5.2 / (((1 << bits) - 1) * math.sqrt(12))
        assert 0.75 * model < err[bits] < 1.3 * model, (bits, err[bits], model)
    W32_8 = oracle.dequant(*oracle.quantize_rtn(W, 8))
    s8 = np.repeat(oracle.quantize_rtn(W, 8)[1].astype(np.float64), 128, axis=1)
    assert np.all(np.abs(W32_8 - W) <= 0.625 * s8)


# ----------------------------------------------------------------------- glue
def test_rms_and_silu_closed_forms():
    t = np.array([[3.0, -3.0, 3.0, -3.0], [0.0, 0.0, 0.0, 8.0]])
    out = oracle.rms_rows(t, eps=0.0).astype(np.float64)
    assert np.array_equal(out, [[1, -1, 1, -1], [0, 0, 0, 2]])
    out = oracle.rms_rows(np.full((1, 64), 2.0), eps=12.0).astype(np.float64)  # 2/sqrt(4+12)
    assert np.array_equal(out, np.full((1, 64), 0.5))
    g = np.array([0.0, 1.0, -1.0, 20.0, -20.0], dtype=np.float16)
    p = np.array([7.0, 2.0, 2.0, 1.0, 1.0], dtype=np.float16)
    got = oracle.silu_mul(g, p)
    want = [0.0, 2 * 0.7310585786300049, -2 * 0.2689414213699951, 20 / (1 + math.exp(-20)), -20 / (1 + math.exp(20))]
    assert np.allclose(got, want, rtol=1e-14, atol=0)


def test_block_forward_dataflow_on_a_case_with_a_known_answer():
    """Identity-like matrices make every intermediate of the block computable by hand."""
    H, F = 128, 256
    eye = np.eye(H, dtype=np.float32)
    zero_hh = np.zeros((H, H), dtype=np.float32)
    up = np.zeros((F, H), dtype=np.float32)
    up[:H] = eye
    down = np.zeros((H, F), dtype=np.float32)
    down[:, :H] = eye
    x = np.zeros((2, H), dtype=np.float16)
    x[0, 0] = 4.0
    x[1, 5] = -2.0
    t = oracle.block_forward(x, [eye, eye, zero_hh, 2 * eye, up, up, down])
    r = math.sqrt(H)  # rms of a one-hot row of value v is |v|/sqrt(H): normalised value sign(v) sqrt(H)
    u0 = float(np.float16(4.0 / math.sqrt(16.0 / H + 1e-5)))
    assert abs(u0 - r) < 0.01 and float(t["u"][0, 0]) == u0 and float(t["u"][1, 5]) < 0
    assert float(t["q"][0, 0]) == u0 and float(t["k"][0, 0]) == u0 and not t["v"].any()
    a0 = float(np.float16(2 * u0 / math.sqrt((2 * u0) ** 2 / H + 1e-5)))
    assert float(t["a"][0, 0]) == a0
    assert float(t["o"][0, 0]) == float(np.float16(2 * a0))
    x1 = float(np.float16(4.0 + float(np.float16(2 * a0))))
    assert float(t["x1"][0, 0]) == x1
    u2 = float(np.float16(x1 / math.sqrt(x1 * x1 / H + 1e-5)))
    assert float(t["u2"][0, 0]) == u2 and float(t["g"][0, 0]) == u2 and float(t["p"][0, 0]) == u2
    sm = u2 / (1 + math.exp(-u2)) * u2
    m0 = float(np.float16(sm / math.sqrt(sm * sm / F + 1e-5)))
    assert float(t["m"][0, 0]) == m0 and t["m"].shape == (2, F)
    assert float(t["d"][0, 0]) == m0
    xn = x1 + m0
    assert float(t["x_next"][0, 0]) == float(np.float16(xn / math.sqrt(xn * xn / H + 1e-5)))
    assert np.count_nonzero(t["x_next"][0]) == 1 and np.count_nonzero(t["x_next"][1]) == 1


# ------------------------------------------------------------------------ NLL
def test_token_nll_closed_forms():
    V = 32000
    z = np.zeros((3, V), dtype=np.float16)
    lab = np.array([0, 31999, 12345], dtype=np.int32)
    assert np.allclose(oracle.token_nll(z, lab), math.log(V), rtol=0, atol=1e-12)
    assert abs(math.log(V) - 10.373491181781864) < 1e-12
    # shift invariance, also at the edge of the fp16 range
    for c in (7.0, -65504.0, 65504.0):
        assert np.allclose(oracle.token_nll(z + np.float16(c), lab), math.log(V), rtol=0, atol=1e-12)
    # one dominant logit
    x = np.zeros((2, V), dtype=np.float16)
    x[:, 17] = 60.0
    got = oracle.token_nll(x, np.array([17, 18], dtype=np.int32))
    assert abs(got[0] - math.log1p((V - 1) * math.exp(-60.0))) < 1e-15
    assert abs(got[1] - (60.0 + math.log1p((V - 1) * math.exp(-60.0)))) < 1e-12
    # two-valued row: logsumexp known in closed form
    x = np.zeros((1, 10), dtype=np.float16)
    x[0, :4] = 2.0
    got = oracle.token_nll(x, np.array([1], dtype=np.int32))
    assert abs(got[0] - (math.log(4 * math.exp(2.0) + 6) - 2.0)) < 1e-14
    # ignored position
    assert oracle.token_nll(x, np.array([-1], dtype=np.int32))[0] == 0.0


def test_token_nll_against_float64_logsumexp_and_perplexity():
    L = fq_synth.logits(12, 64, 1000)
    lab = fq_synth.labels(12, 64, 1000)
    x = L.astype(np.float64)
    want = np.log(np.exp(x - x.max(1, keepdims=True)).sum(1)) + x.max(1) - x[np.arange(64), lab]
    got = oracle.token_nll(L, lab)
    assert np.allclose(got, want, rtol=0, atol=1e-12)
    # Gaussian logits: E[nll] ~ ln V + sigma^2/2
    assert abs(got.mean() - (math.log(1000) + 1.28 ** 2 / 2)) < 0.25
    assert abs(oracle.perplexity(got) - math.exp(want.mean())) < 1e-9 * math.exp(want.mean())


# ------------------------------------------------------------- logit distance
def test_logit_l2_closed_forms_and_metric_properties():
    V = 1000
    a = fq_synth.logits(30, 6, V)
    # identical logits: distance 0; a single changed entry: its absolute change
    assert np.all(oracle.logit_l2(a, a) == 0.0)
    b = a.copy()
    b[2, 17] = np.float16(float(a[2, 17]) + 3.0)
    d = oracle.logit_l2(a, b)
    want = abs(float(b[2, 17]) - float(a[2, 17]))
    assert d[2] == want and np.all(np.delete(d, 2) == 0.0)
    # a 3-4-5 triangle spread over two entries, and k equal offsets: |c| sqrt(k)
    z = np.zeros((2, V), dtype=np.float16)
    y = z.copy()
    y[0, 5], y[0, 900] = 3.0, -4.0
    y[1, :64] = 0.5
    got = oracle.logit_l2(y, z)
    assert got[0] == 5.0 and got[1] == 0.5 * 8.0
    # symmetry, and the triangle inequality against a third point
    c = fq_synth.logits(31, 6, V)
    e = fq_synth.logits(32, 6, V)
    dac, dca = oracle.logit_l2(a, c), oracle.logit_l2(c, a)
    assert np.array_equal(dac, dca)
    assert np.all(dac <= oracle.logit_l2(a, e) + oracle.logit_l2(e, c) + 1e-12)
    # brute force in Python floats on a tiny case
    small_a, small_c = a[:2, :7], c[:2, :7]
    for m in range(2):
        ss = 0.0
        for v in range(7):
            ss += (float(small_a[m, v]) - float(small_c[m, v])) ** 2
        assert abs(oracle.logit_l2(small_a, small_c)[m] - math.sqrt(ss)) < 1e-13
    # independent N(0, s^2) logits: distance ~ s sqrt(2V)
    assert np.all(np.abs(dac / (1.28 * math.sqrt(2 * V)) - 1) < 0.1)


# ------------------------------------------------------------- paper arithmetic
def test_numbers_the_paper_prints():
    vals = {}
    with open(os.path.join(GOLDEN, "paper_arithmetic.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                tok = line.split()
                vals[tok[0]] = tok[1:]
    modules = int(vals["modules_7b"][0])
    assert abs(2 ** modules / float(vals["design_space_two_models_7b"][0]) - 1) < 5e-3
    # footprint of the synthetic 7B stack at the four stored bit rates
    shapes = fq_synth.block_matrix_shapes(4096, 11008)
    params = 32 * sum(n * k for n, k in shapes)
    total_gb = sum(b / 8 * params for b in (2.5, 4.0, 5.0, 7.5)) / 1e9
    assert abs(total_gb - float(vals["storage_gb_four_qms"][0])) < 2.0
    mid_gb = (4.0 + 5.0) / 8 * params / 1e9
    for rate, want in zip((0.25, 0.5, 0.75), map(float, vals["storage_gb_pruned_25_50_75"][:3])):
        assert abs((total_gb - rate * mid_gb) - want) < 2.0
