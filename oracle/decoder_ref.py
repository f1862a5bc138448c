"""Plain reference of one decode step through real decoder blocks (test infrastructure: only tests, the smoke
check and the benchmark's CPU leg use it; it imports nothing from the GPU package).

FlexQuant (arXiv 2501.07139, Section "Experiment") hosts Llama models; the block here is that architecture
written out from its published definitions, around the quantized linears of the hybrid model:
  u  = rms(x)                      pre-norm, eps 1e-5; the norm's gain is folded into the following linears
  q, k, v = Lq(u), Lk(u), Lv(u)
  q', k' = rope(q, pos), rope(k, pos)      rotary embedding (RoFormer): in every head the adjacent pair
                                   (x[2i], x[2i+1]) is rotated by the angle pos * base^(-2i/d), base 10000
  cache: K[pos] = k', V[pos] = v
  a  = softmax_t(q' . K[t] / sqrt(d)) . V   per head, over the positions t <= pos (multi-head, n_kv = n_heads)
  o  = Lo(a);  x1 = x + o
  u2 = rms(x1);  g, p = Lgate(u2), Lup(u2);  m = silu(g) * p;  d = Ldown(m)
  x_next = x1 + d
Every named tensor is rounded to fp16 where the GPU stores it; arithmetic in between is fp64.
"""
import numpy as np

import oracle

ROPE_BASE = 10000.0


def _f64(a):
    return np.asarray(a).astype(np.float64)


def rope(x, pos, n_heads, base=ROPE_BASE):
    """Rotate a [H] vector (H = n_heads * d) to position `pos`; fp64 in and out, no rounding."""
    x = _f64(x).reshape(n_heads, -1, 2)
    d = 2 * x.shape[1]
    ang = pos * base ** (-2.0 * np.arange(d // 2) / d)
    c, s = np.cos(ang), np.sin(ang)
    out = np.empty_like(x)
    out[:, :, 0] = x[:, :, 0] * c - x[:, :, 1] * s
    out[:, :, 1] = x[:, :, 0] * s + x[:, :, 1] * c
    return out.reshape(-1)


def attention(q, K, V, n_heads):
    """q [H], K and V [T,H] (the T cached positions): per head softmax(q . K[t] / sqrt(d)) . V, fp64."""
    q, K, V = _f64(q), _f64(K), _f64(V)
    T, H = K.shape
    d = H // n_heads
    out = np.empty(H)
    for h in range(n_heads):
        sl = slice(h * d, (h + 1) * d)
        s = K[:, sl] @ q[sl] / np.sqrt(d)
        w = np.exp(s - s.max())
        out[sl] = (w / w.sum()) @ V[:, sl]
    return out


def decode_block(x, mats, k_cache, v_cache, pos, n_heads):
    """One block for the token at position `pos`.  x fp16 [1,H]; mats the seven dequantized fp32 matrices
    (q, k, v, o, gate, up, down); k_cache, v_cache fp16 [Tmax,H], rows < pos filled, row pos written here.
    Returns the dict of intermediates; 'x_next' feeds the next block."""
    wq, wk, wv, wo, wg, wu, wd = mats
    r16 = oracle.round_f16
    t = {}
    t["u"] = oracle.rms_rows(_f64(x))
    t["q"] = r16(oracle.qlinear(t["u"], wq))
    t["k"] = r16(oracle.qlinear(t["u"], wk))
    t["v"] = r16(oracle.qlinear(t["u"], wv))
    t["qr"] = r16(rope(t["q"][0], pos, n_heads))[None, :]
    t["kr"] = r16(rope(t["k"][0], pos, n_heads))[None, :]
    k_cache[pos] = t["kr"][0]
    v_cache[pos] = t["v"][0]
    t["a"] = r16(attention(t["qr"][0], k_cache[:pos + 1], v_cache[:pos + 1], n_heads))[None, :]
    t["o"] = r16(oracle.qlinear(t["a"], wo))
    t["x1"] = r16(_f64(x) + _f64(t["o"]))
    t["u2"] = oracle.rms_rows(_f64(t["x1"]))
    t["g"] = r16(oracle.qlinear(t["u2"], wg))
    t["p"] = r16(oracle.qlinear(t["u2"], wu))
    t["m"] = r16(oracle.silu_mul(t["g"], t["p"]))
    t["d"] = r16(oracle.qlinear(t["m"], wd))
    t["x_next"] = r16(_f64(t["x1"]) + _f64(t["d"]))
    return t


def decode_step(x, layer_mats, k_caches, v_caches, pos, n_heads):
    """x fp16 [1,H] through all blocks at position pos; k_caches, v_caches fp16 [L,Tmax,H], updated in place."""
    for l, mats in enumerate(layer_mats):
        x = decode_block(x, mats, k_caches[l], v_caches[l], pos, n_heads)["x_next"]
    return x


def sequence_attention(q, k, v, n_heads):
    """Causal attention over a whole sequence: q, k, v fp16 [T,H], row t at position t.  Returns
    (a fp16 [T,H], rotated keys fp16 [T,H]); the values enter the cache as they are.  The masked T x T
    product: another route to what T calls of attention() on a growing cache give."""
    r16 = oracle.round_f16
    T, H = q.shape
    d = H // n_heads
    qr = r16(np.stack([rope(q[t], t, n_heads) for t in range(T)]))
    kr = r16(np.stack([rope(k[t], t, n_heads) for t in range(T)]))
    a = np.empty((T, H))
    mask = np.triu(np.ones((T, T), dtype=bool), 1)
    for h in range(n_heads):
        sl = slice(h * d, (h + 1) * d)
        s = _f64(qr[:, sl]) @ _f64(kr[:, sl]).T / np.sqrt(d)
        s[mask] = -np.inf
        w = np.exp(s - s.max(axis=1, keepdims=True))
        a[:, sl] = (w / w.sum(axis=1, keepdims=True)) @ _f64(v[:, sl])
    return r16(a), kr


def sequence_block(X, mats, n_heads, k_cache=None, v_cache=None):
    """The block over a whole sequence at once, X fp16 [T,H] (row t at position t); fills rows 0..T-1 of the
    caches (fp16 [Tmax,H]) when given.  Used to pin token-by-token decoding and as the prefill reference."""
    wq, wk, wv, wo, wg, wu, wd = mats
    r16 = oracle.round_f16
    T = X.shape[0]
    u = oracle.rms_rows(_f64(X))
    q, k, v = (r16(oracle.qlinear(u, w)) for w in (wq, wk, wv))
    a, kr = sequence_attention(q, k, v, n_heads)
    if k_cache is not None:
        k_cache[:T] = kr
        v_cache[:T] = v
    o = r16(oracle.qlinear(a, wo))
    x1 = r16(_f64(X) + _f64(o))
    u2 = oracle.rms_rows(_f64(x1))
    g, p = r16(oracle.qlinear(u2, wg)), r16(oracle.qlinear(u2, wu))
    m = r16(oracle.silu_mul(g, p))
    dd = r16(oracle.qlinear(m, wd))
    return r16(_f64(x1) + _f64(dd))


def sequence_stack(X, layer_mats, n_heads, k_caches=None, v_caches=None):
    for l, mats in enumerate(layer_mats):
        X = sequence_block(X, mats, n_heads, None if k_caches is None else k_caches[l],
                           None if v_caches is None else v_caches[l])
    return X
