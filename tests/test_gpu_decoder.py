"""Real decoder blocks, one decode step (attention over a key/value cache, rotary embedding, residual SwiGLU
block) through the C-ABI against oracle/decoder_ref.py.  Floating point: outputs within 2e-3 of the row's
scale like the linears; cache rows of the rotated key within one fp16 ulp (fp32 rotation with an fp32 table
against fp64), value rows and untouched rows bit-exact."""
import numpy as np
import pytest

import fq_synth
import oracle
from oracle import decoder_ref as ref

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch():
    import torch

    return torch


@pytest.fixture(scope="module")
def fq():
    import paper_2501_07139_amd as fq

    return fq


def dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda().view(torch.float16)


def host16(t):
    return t.cpu().view(__import__("torch").int16).numpy().view(np.float16)


def to_heads(a, n_heads):
    """[..., T, H] position-major (the reference's) -> [..., n_heads, T, 128] head-major (the library's)."""
    a = np.asarray(a)
    return np.ascontiguousarray(np.swapaxes(a.reshape(a.shape[:-1] + (n_heads, 128)), -3, -2))


def from_heads(a):
    a = np.swapaxes(np.asarray(a), -3, -2)
    return np.ascontiguousarray(a).reshape(a.shape[:-2] + (-1,))


def ulps(a, b):
    """Distance in fp16 steps between two fp16 arrays (same sign assumed where it matters)."""
    ia = a.view(np.int16).astype(np.int32)
    ib = b.view(np.int16).astype(np.int32)
    ia = np.where(ia < 0, -(ia & 0x7FFF), ia)
    ib = np.where(ib < 0, -(ib & 0x7FFF), ib)
    return np.abs(ia - ib)


def rel_err(y, r):
    """max |y - r| / max(|r|, rms of r's row): the element-wise relative error, with the row's scale as the
    floor where r is near zero (the same reading as for the linears)."""
    y, r = np.atleast_2d(y.astype(np.float64)), np.atleast_2d(r.astype(np.float64))
    rms = np.sqrt(np.mean(r * r, axis=1, keepdims=True))
    return float(np.max(np.abs(y - r) / np.maximum(np.maximum(np.abs(r), rms), 1e-30)))


@pytest.mark.parametrize("case", [(4, 300, (0, 1, 15, 16, 127, 128, 129, 255, 256, 299)), (32, 2048, (2047,)),
                                  (40, 4096, (4095, 1000))], ids=str)
def test_attn_decode_against_oracle(fq, torch, case):
    n_heads, Tmax, positions = case
    H = 128 * n_heads
    rng = np.random.default_rng(5)
    K = (rng.normal(size=(Tmax, H)) * 0.8).astype(np.float16)
    V = rng.normal(size=(Tmax, H)).astype(np.float16)
    rope = fq.rope_table(Tmax)
    for pos in positions:
        q = (rng.normal(size=H) * 1.5).astype(np.float16)
        k = rng.normal(size=H).astype(np.float16)
        v = rng.normal(size=H).astype(np.float16)
        dK, dV = dev(torch, to_heads(K, n_heads)), dev(torch, to_heads(V, n_heads))
        got = host16(fq.fq_attn_decode(dev(torch, q), dev(torch, k), dev(torch, v), dK, dV, pos, rope))
        qr = oracle.round_f16(ref.rope(q, pos, n_heads))
        kr = oracle.round_f16(ref.rope(k, pos, n_heads))
        Kw, Vw = K.copy(), V.copy()
        Kw[pos], Vw[pos] = kr, v
        want = ref.attention(qr, Kw[:pos + 1], Vw[:pos + 1], n_heads)
        assert rel_err(got, want) <= 2e-3, pos
        gK, gV = from_heads(host16(dK)), from_heads(host16(dV))
        assert np.array_equal(gV.view(np.uint16), Vw.view(np.uint16)), pos            # value row stored as is
        keep = np.arange(Tmax) != pos
        assert np.array_equal(gK[keep].view(np.uint16), K[keep].view(np.uint16)), pos  # other rows untouched
        d = ulps(gK[pos], kr)
        assert d.max() <= 1 and np.mean(d == 0) > 0.98, pos


def test_attn_decode_closed_forms(fq, torch):
    n_heads, Tmax = 2, 260
    H = 256
    rope = fq.rope_table(Tmax)
    rng = np.random.default_rng(6)
    V = rng.normal(size=(Tmax, H)).astype(np.float16)
    q = rng.normal(size=H).astype(np.float16)
    zero = np.zeros(H, np.float16)
    # all keys zero: uniform weights -> the mean of the values, over one split and over three
    for pos in (0, 99, 259):
        Kc, Vc = dev(torch, np.zeros((n_heads, Tmax, 128), np.float16)), dev(torch, to_heads(V, n_heads))
        got = host16(fq.fq_attn_decode(dev(torch, q), dev(torch, zero), dev(torch, V[pos]), Kc, Vc, pos, rope))
        want = V[:pos + 1].astype(np.float64).mean(0)
        assert np.max(np.abs(got.astype(np.float64) - want)) <= 1e-3 * max(1.0, np.abs(want).max()) + 5e-4, pos
    # position 0 leaves q and k unrotated: the stored key row is k itself
    k = rng.normal(size=H).astype(np.float16)
    Kc, Vc = (dev(torch, np.zeros((n_heads, Tmax, 128), np.float16)) for _ in range(2))
    out = host16(fq.fq_attn_decode(dev(torch, q), dev(torch, k), dev(torch, V[7]), Kc, Vc, 0, rope))
    assert np.array_equal(from_heads(host16(Kc))[0].view(np.uint16), k.view(np.uint16))
    assert np.array_equal(out.view(np.uint16), V[7].view(np.uint16))                   # one position: its value


def build_real_stack(fq, seed, levels=(2, 3, 4, 8)):
    sh = fq_synth.MODEL_SHAPES["tiny"]
    layers, host = [], []
    for l in range(sh["layers"]):
        mats, hm = [], []
        for j, (N, K) in enumerate(fq_synth.block_matrix_shapes(sh["hidden"], sh["ffn"])):
            W = fq_synth.weights(seed, N, K, 0.06, l, j)
            by, hby = {}, {}
            for b in levels:
                codes, s, z = oracle.quantize_rtn(W, b)
                by[b] = fq.PackedMatrix.from_host(codes, s, z, b)
                hby[b] = oracle.dequant(codes, s, z)
            mats.append(by)
            hm.append(hby)
        layers.append(mats)
        host.append(hm)
    return fq.Stack(layers), host, sh


def test_decode_step_against_oracle(fq, torch):
    stack, host, sh = build_real_stack(fq, 800)
    L, H, nh, Tmax, T = sh["layers"], sh["hidden"], sh["hidden"] // 128, 140, 134
    bitvec = fq_synth.bit_vector(801, 7 * L, probs=(0.25, 0.25, 0.25, 0.25))
    mats = [[host[l][j][int(bitvec[7 * l + j])] for j in range(7)] for l in range(L)]
    rope = fq.rope_table(Tmax)
    kc = torch.zeros((L, nh, Tmax, 128), dtype=torch.float16, device="cuda")
    vc = torch.zeros_like(kc)
    okc, ovc = np.zeros((L, Tmax, H), np.float16), np.zeros((L, Tmax, H), np.float16)
    X = fq_synth.activations(802, T, H)
    worst, mean = 0.0, 0.0
    for pos in range(T):
        got = host16(fq.fq_decode_step(stack, bitvec, dev(torch, X[pos]), kc, vc, pos, rope))
        if pos in (0, 1, 2, 17, 127, 128, 133):  # the oracle follows on a sample of positions, from the GPU's caches
            okc[:], ovc[:] = from_heads(host16(kc)), from_heads(host16(vc))
            want = ref.decode_step(X[pos:pos + 1], mats, okc, ovc, pos, nh)[0]
            diff = np.abs(got.astype(np.float64) - want.astype(np.float64))
            scale = np.sqrt(np.mean(want.astype(np.float64) ** 2))
            worst, mean = max(worst, diff.max() / scale), max(mean, diff.mean() / scale)
            # the rows this step appended, against the oracle's
            assert np.max(np.abs(from_heads(host16(kc))[:, pos].astype(np.float64) - okc[:, pos].astype(np.float64))) <= 2e-2
            assert np.max(np.abs(from_heads(host16(vc))[:, pos].astype(np.float64) - ovc[:, pos].astype(np.float64))) <= 2e-2
    # end to end over three blocks: fp16 re-rounding between steps lets single ulps flip
    assert worst <= 2e-2 and mean <= 2e-3, (worst, mean)


def test_decode_block_teacher_forced(fq, torch):
    """One block at a time from identical inputs and caches: every stored tensor of the block is a few fp16
    ulps from the oracle's at most."""
    stack, host, sh = build_real_stack(fq, 810, levels=(3, 4))
    H, nh, Tmax = sh["hidden"], sh["hidden"] // 128, 150
    rng = np.random.default_rng(3)
    rope = fq.rope_table(Tmax)
    for l, pos, bits in ((0, 0, 4), (1, 64, 3), (2, 149, 4)):
        sub = fq.Stack([stack.layers[l]])
        bv = np.full(7, bits, dtype=np.uint8)
        K0 = (rng.normal(size=(1, Tmax, H)) * 0.7).astype(np.float16)
        V0 = rng.normal(size=(1, Tmax, H)).astype(np.float16)
        x = fq_synth.activations(811 + l, 1, H)
        kc, vc = dev(torch, to_heads(K0, nh)), dev(torch, to_heads(V0, nh))
        got = host16(fq.fq_decode_step(sub, bv, dev(torch, x[0]), kc, vc, pos, rope))
        t = ref.decode_block(x, [host[l][j][bits] for j in range(7)], K0[0], V0[0], pos, nh)
        want = t["x_next"][0].astype(np.float64)
        assert np.max(np.abs(got.astype(np.float64) - want)) <= 1e-2 * max(1.0, np.abs(want).max()), (l, pos)
        assert np.mean(np.abs(got.astype(np.float64) - want)) <= 1e-3


def test_decode_step_refuses_bad_arguments(fq, torch):
    stack, host, sh = build_real_stack(fq, 820, levels=(4,))
    L, H = sh["layers"], sh["hidden"]
    bv = np.full(7 * L, 4, dtype=np.uint8)
    rope = fq.rope_table(16)
    kc = torch.zeros((L, H // 128, 16, 128), dtype=torch.float16, device="cuda")
    x = torch.zeros(H, dtype=torch.float16, device="cuda")
    with pytest.raises(fq.FqError):
        fq.fq_decode_step(stack, bv, x, kc, kc.clone(), 16, rope)        # pos == Tmax
    with pytest.raises(fq.FqError):
        fq.fq_decode_step(stack, bv, x, kc, kc.clone(), -1, rope)
    with pytest.raises(fq.FqError):
        fq.fq_decode_step(stack, bv, x, kc, kc.clone(), 0, rope, workspace=torch.empty(64, dtype=torch.uint8, device="cuda"))
    bad = bv.copy()
    bad[3] = 8                                                           # not stored
    with pytest.raises(fq.FqError):
        fq.fq_decode_step(stack, bad, x, kc, kc.clone(), 0, rope)
    torch.cuda.synchronize()


# --------------------------------------------------------------------- prefill
@pytest.mark.parametrize("case", [(2, 1, 8), (2, 63, 64), (2, 64, 64), (2, 65, 200), (4, 200, 256), (32, 2048, 2048)], ids=str)
def test_attn_prefill_against_oracle(fq, torch, case):
    """Causal attention over a whole sequence against the masked T x T product of the oracle (full sequence
    for short ones, a sample of rows through the decode form for the long one); caches as after decoding."""
    n_heads, T, Tmax = case
    H = 128 * n_heads
    rng = np.random.default_rng(9)
    q = (rng.normal(size=(T, H)) * 1.5).astype(np.float16)
    k = rng.normal(size=(T, H)).astype(np.float16)
    v = rng.normal(size=(T, H)).astype(np.float16)
    rope = fq.rope_table(Tmax)
    kc = torch.full((n_heads, Tmax, 128), float("nan"), dtype=torch.float16, device="cuda")
    vc = torch.full_like(kc, float("nan"))
    got = host16(fq.fq_attn_prefill(dev(torch, q), dev(torch, k), dev(torch, v), kc, vc, rope))
    gK, gV = from_heads(host16(kc)), from_heads(host16(vc))
    assert np.array_equal(gV[:T].view(np.uint16), v.view(np.uint16))
    assert np.isnan(gK[T:].astype(np.float32)).all() and np.isnan(gV[T:].astype(np.float32)).all()  # rows past T untouched
    if T <= 256:
        want, kr = ref.sequence_attention(q, k, v, n_heads)
        assert rel_err(got, want) <= 2e-3
        d = ulps(gK[:T], kr)
        assert d.max() <= 1 and np.mean(d == 0) > 0.98
    else:
        rows = [0, 1, 63, 64, 65, 1000, 1023, 1024, T - 2, T - 1]
        kr = oracle.round_f16(np.stack([ref.rope(k[t], t, n_heads) for t in range(T)]))
        # one fp16 step of the result, or (where the rotation cancels to almost nothing) of the fp32 terms
        dk = np.abs(gK[:T].astype(np.float64) - kr.astype(np.float64))
        assert np.all(dk <= 1e-3 * np.abs(kr.astype(np.float64)) + 2e-6)
        for t in rows:
            want = ref.attention(oracle.round_f16(ref.rope(q[t], t, n_heads)), kr[:t + 1], v[:t + 1], n_heads)
            assert rel_err(got[t], want) <= 2e-3, t


def test_prefill_forward_against_oracle_and_decode_continues_from_it(fq, torch):
    stack, host, sh = build_real_stack(fq, 830)
    L, H, nh, Tmax, T = sh["layers"], sh["hidden"], sh["hidden"] // 128, 160, 150
    bitvec = fq_synth.bit_vector(831, 7 * L, probs=(0.25, 0.25, 0.25, 0.25))
    mats = [[host[l][j][int(bitvec[7 * l + j])] for j in range(7)] for l in range(L)]
    rope = fq.rope_table(Tmax)
    X = fq_synth.activations(832, T + 1, H)
    kc = torch.zeros((L, nh, Tmax, 128), dtype=torch.float16, device="cuda")
    vc = torch.zeros_like(kc)
    got = host16(fq.fq_prefill_forward(stack, bitvec, dev(torch, X[:T]), kc, vc, rope))
    okc, ovc = np.zeros((L, Tmax, H), np.float16), np.zeros((L, Tmax, H), np.float16)
    want = ref.sequence_stack(X[:T], mats, nh, okc, ovc).astype(np.float64)
    diff = np.abs(got.astype(np.float64) - want)
    scale = np.sqrt(np.mean(want ** 2))
    assert diff.max() / scale <= 2e-2 and diff.mean() / scale <= 2e-3
    assert np.max(np.abs(from_heads(host16(kc)).astype(np.float64) - okc.astype(np.float64))) <= 3e-2
    assert np.max(np.abs(from_heads(host16(vc)).astype(np.float64) - ovc.astype(np.float64))) <= 3e-2
    # the next token decodes from the prefilled caches like from caches filled token by token
    nxt = host16(fq.fq_decode_step(stack, bitvec, dev(torch, X[T]), kc, vc, T, rope))
    kc2, vc2 = torch.zeros_like(kc), torch.zeros_like(vc)
    for pos in range(T + 1):
        step = host16(fq.fq_decode_step(stack, bitvec, dev(torch, X[pos]), kc2, vc2, pos, rope))
    d2 = np.abs(nxt.astype(np.float64) - step.astype(np.float64))
    assert d2.max() <= 2e-2 * max(1.0, np.abs(step.astype(np.float64)).max()) and d2.mean() <= 2e-3
    # a short sequence (at most 16 rows) takes the small-M linears
    short = host16(fq.fq_prefill_forward(stack, bitvec, dev(torch, X[:5]), torch.zeros_like(kc), torch.zeros_like(vc), rope))
    w5 = ref.sequence_stack(X[:5], mats, nh).astype(np.float64)
    assert np.max(np.abs(short.astype(np.float64) - w5)) / np.sqrt(np.mean(w5 ** 2)) <= 2e-2


def test_glue_silu_mul_without_norm(fq, torch):
    g = fq_synth.activations(840, 3, 640)
    p = fq_synth.activations(841, 3, 640)
    got = host16(fq.fq_glue(5, dev(torch, g), dev(torch, p)))
    want = oracle.round_f16(oracle.silu_mul(g, p))
    assert ulps(got, want).max() <= 1 and np.mean(got.view(np.uint16) == want.view(np.uint16)) > 0.98


def test_calibration_eval_on_real_blocks_matches_the_oracle_perplexity(fq, torch):
    """calibrationEval of Algorithm 1 with the blocks run as real decoder blocks: perplexity of a hybrid model
    over one calibration sequence, restarted from a changed block, against the oracle's chain."""
    from paper_2501_07139_amd import search

    stack, host, sh = build_real_stack(fq, 850, levels=(2, 4, 8))
    L, H, nh, M, V = sh["layers"], sh["hidden"], sh["hidden"] // 128, 96, 1000
    x = fq_synth.activations(851, M, H)
    head = fq_synth.weights(852, V, H, 0.05).astype(np.float16)
    labels = fq_synth.labels(853, M, V)
    ev = search.CalibrationEval(stack, dev(torch, head), dev(torch, x), torch.from_numpy(labels).cuda(), real_blocks=True)

    def oracle_ppl(bits):
        mats = [[host[l][j][bits[7 * l + j]] for j in range(7)] for l in range(L)]
        logits = oracle.round_f16(oracle.dense_f16(ref.sequence_stack(x, mats, nh), head))
        return oracle.perplexity(oracle.token_nll(logits, labels))

    up = (8,) * (7 * L)
    ppl_up, state = ev(up, None, None)
    assert abs(ppl_up / oracle_ppl(up) - 1) <= 2e-3
    parent = search.Node(up, ppl_up, None, state)
    child = up[:9] + (2,) + up[10:]              # block 1, matrix 2 lowered: restart at block 1
    ppl_c, _ = ev(child, parent, 9)
    assert ev.blocks_run == L + (L - 1)
    assert abs(ppl_c / oracle_ppl(child) - 1) <= 2e-3


def test_decode_step_and_prefill_replay_from_captured_graphs(fq, torch):
    """The launches of a decode step and of a prefill forward can be captured and replayed (the library queues
    kernels only: no memsets, no allocations): every replay, with eager work in between, reproduces the eager
    result bit for bit."""
    stack, host, sh = build_real_stack(fq, 860, levels=(3, 8))
    L, H, nh, Tmax, T = sh["layers"], sh["hidden"], sh["hidden"] // 128, 200, 140
    bitvec = np.tile(np.array([3, 8, 3, 8, 3, 8, 3], dtype=np.uint8), L)
    rope = fq.rope_table(Tmax)
    X = dev(torch, fq_synth.activations(861, T + 1, H))
    kc = torch.zeros((L, nh, Tmax, 128), dtype=torch.float16, device="cuda")
    vc = torch.zeros_like(kc)
    ws_p = torch.empty(fq.fq_prefill_workspace_bytes(T, H, sh["ffn"]), dtype=torch.uint8, device="cuda")
    ws_d = torch.empty(fq.fq_decode_workspace_bytes(H, sh["ffn"], Tmax), dtype=torch.uint8, device="cuda")
    out_p = torch.empty((T, H), dtype=torch.float16, device="cuda")
    out_d = torch.empty(H, dtype=torch.float16, device="cuda")
    xs, xt = X[:T].contiguous(), X[T].contiguous()
    fq.fq_prefill_forward(stack, bitvec, xs, kc, vc, rope, out=out_p, workspace=ws_p)   # eager, also the warm-up
    fq.fq_decode_step(stack, bitvec, xt, kc, vc, T, rope, out=out_d, workspace=ws_d)
    torch.cuda.synchronize()
    want_p, want_d, want_k = out_p.clone(), out_d.clone(), kc.clone()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        fq.fq_prefill_forward(stack, bitvec, xs, kc, vc, rope, out=out_p, workspace=ws_p)
        fq.fq_decode_step(stack, bitvec, xt, kc, vc, T, rope, out=out_d, workspace=ws_d)
    for r in range(3):
        out_p.fill_(float("nan"))
        out_d.fill_(float("nan"))
        kc.zero_()
        vc.zero_()
        ws_p.random_(0, 255)
        ws_d.random_(0, 255)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_p.view(torch.int16), want_p.view(torch.int16)), r
        assert torch.equal(out_d.view(torch.int16), want_d.view(torch.int16)), r
        assert torch.equal(kc.view(torch.int16), want_k.view(torch.int16)), r
