"""CPU oracle (test infrastructure only).

A thin numpy front for ``fq_oracle.c`` plus the few lines that string its steps
into the synthetic decoder stack.  Nothing here is used by the product path:
only tests, the smoke check and the benchmark's CPU-baseline leg import it, and
it imports nothing from the GPU package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fq_oracle.c")
_LIB = os.path.join(_HERE, "libfq_oracle.so")
_lib = None

RMS_EPS = 1e-5


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fused multiply-add, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-shared", "-fPIC",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.ora_h2d.restype = ctypes.c_double
        _lib.ora_h2d.argtypes = [ctypes.c_uint16]
        _lib.ora_d2h.restype = ctypes.c_uint16
        _lib.ora_d2h.argtypes = [ctypes.c_double]
        _lib.ora_packed_bytes.restype = ctypes.c_size_t
        _lib.ora_packed_bytes.argtypes = [ctypes.c_int] * 3
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a)
    if a.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {a.dtype}")
    return a


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what} failed with code {rc}")


def threads() -> int:
    """Number of OpenMP threads the C loops run on."""
    n = os.environ.get("OMP_NUM_THREADS")
    return int(n) if n else (os.cpu_count() or 1)


# ---------------------------------------------------------------- fp16 helpers
def h2d(bits: int) -> float:
    return _load().ora_h2d(int(bits))


def d2h(v: float) -> int:
    return _load().ora_d2h(float(v))


def round_f16(a) -> np.ndarray:
    a = _c(np.asarray(a, dtype=np.float64), np.float64)
    out = np.empty(a.shape, dtype=np.uint16)
    _load().ora_round_f16(_p(a), ctypes.c_size_t(a.size), _p(out))
    return out.view(np.float16)


# -------------------------------------------------------------------- quantize
def quantize_rtn(W, bits: int, group: int = 128):
    """fp32 [N,K] -> (codes u8 [N,K], scales f16 [N,G], zeros f16 [N,G])."""
    W = _c(W, np.float32)
    N, K = W.shape
    G = K // group
    codes = np.empty((N, K), dtype=np.uint8)
    scales = np.empty((N, G), dtype=np.uint16)
    zeros = np.empty((N, G), dtype=np.uint16)
    _check(_load().ora_quantize_rtn(_p(W), N, K, bits, group, _p(codes), _p(scales), _p(zeros)), "quantize_rtn")
    return codes, scales.view(np.float16), zeros.view(np.float16)


def packed_bytes(N: int, K: int, bits: int) -> int:
    return _load().ora_packed_bytes(N, K, bits)


def unpack(packed, N: int, K: int, bits: int) -> np.ndarray:
    packed = _c(np.asarray(packed).view(np.uint8).reshape(-1), np.uint8)
    if packed.size < packed_bytes(N, K, bits):
        raise ValueError("packed buffer too small")
    codes = np.empty((N, K), dtype=np.uint8)
    _check(_load().ora_unpack(_p(packed), N, K, bits, _p(codes)), "unpack")
    return codes


def untile_meta(tiled, N: int, G: int) -> np.ndarray:
    tiled = _c(np.asarray(tiled).view(np.uint16).reshape(-1), np.uint16)
    if tiled.size < (N + 63) // 64 * 64 * G:
        raise ValueError("tiled meta buffer too small")
    out = np.empty((N, G), dtype=np.uint16)
    _check(_load().ora_untile_meta(_p(tiled), N, G, _p(out)), "untile_meta")
    return out.view(np.float16)


def dequant(codes, scales, zeros, group: int = 128) -> np.ndarray:
    codes = _c(codes, np.uint8)
    N, K = codes.shape
    s = _c(np.asarray(scales).view(np.uint16), np.uint16)
    z = _c(np.asarray(zeros).view(np.uint16), np.uint16)
    W32 = np.empty((N, K), dtype=np.float32)
    _check(_load().ora_dequant(_p(codes), _p(s), _p(z), N, K, group, _p(W32)), "dequant")
    return W32


def truncate(codes, scales, zeros, drop: int, group: int = 128, midpoint: bool = False):
    """Drop the `drop` low bits of every code; returns (codes', scales', zeros')."""
    codes = _c(codes, np.uint8)
    N, K = codes.shape
    s = _c(np.asarray(scales).view(np.uint16), np.uint16)
    z = _c(np.asarray(zeros).view(np.uint16), np.uint16)
    co = np.empty_like(codes)
    so = np.empty_like(s)
    zo = np.empty_like(z)
    _check(_load().ora_truncate(_p(codes), _p(s), _p(z), N, K, group, drop, int(midpoint),
                                _p(co), _p(so), _p(zo)), "truncate")
    return co, so.view(np.float16), zo.view(np.float16)


# --------------------------------------------------------------------- linears
def qlinear(X, W32) -> np.ndarray:
    """fp16 [M,K] x fp32 [N,K] -> fp64 [M,N], ascending-k fp64 accumulation."""
    X = _c(np.asarray(X).view(np.uint16), np.uint16)
    W32 = _c(W32, np.float32)
    M, K = X.shape
    N, K2 = W32.shape
    if K != K2:
        raise ValueError("inner dimensions differ")
    Y = np.empty((M, N), dtype=np.float64)
    _check(_load().ora_qlinear(_p(X), M, _p(W32), N, K, _p(Y)), "qlinear")
    return Y


def dense_f16(X, W) -> np.ndarray:
    X = _c(np.asarray(X).view(np.uint16), np.uint16)
    W = _c(np.asarray(W).view(np.uint16), np.uint16)
    M, K = X.shape
    N, K2 = W.shape
    if K != K2:
        raise ValueError("inner dimensions differ")
    Y = np.empty((M, N), dtype=np.float64)
    _check(_load().ora_dense_f16(_p(X), M, _p(W), N, K, _p(Y)), "dense_f16")
    return Y


# ------------------------------------------------------------------------ glue
def rms_rows(t, eps: float = RMS_EPS) -> np.ndarray:
    t = _c(np.asarray(t, dtype=np.float64), np.float64)
    M, H = t.shape
    out = np.empty((M, H), dtype=np.uint16)
    _load().ora_rms_rows(_p(t), M, H, ctypes.c_double(eps), _p(out))
    return out.view(np.float16)


def silu_mul(g, p) -> np.ndarray:
    g = _c(np.asarray(g).view(np.uint16), np.uint16)
    p = _c(np.asarray(p).view(np.uint16), np.uint16)
    out = np.empty(g.shape, dtype=np.float64)
    _load().ora_silu_mul(_p(g), _p(p), ctypes.c_size_t(g.size), _p(out))
    return out


def _f64(a) -> np.ndarray:
    return np.asarray(a).astype(np.float64)  # fp16 -> fp64 is exact


def block_forward(x, mats):
    """One block of the synthetic stack.

    `x` fp16 [M,H]; `mats` the seven dequantized fp32 matrices in the order
    q, k, v, o, gate, up, down.  Every named tensor is rounded to fp16 where
    the GPU stores it.  Returns a dict of all intermediates; 'x_next' feeds the
    next block.  Rows are independent.
    """
    wq, wk, wv, wo, wg, wu, wd = mats
    t = {}
    t["u"] = rms_rows(_f64(x))
    t["q"] = round_f16(qlinear(t["u"], wq))
    t["k"] = round_f16(qlinear(t["u"], wk))
    t["v"] = round_f16(qlinear(t["u"], wv))
    t["a"] = rms_rows(_f64(t["q"]) + _f64(t["k"]) + _f64(t["v"]))
    t["o"] = round_f16(qlinear(t["a"], wo))
    t["x1"] = round_f16(_f64(x) + _f64(t["o"]))
    t["u2"] = rms_rows(_f64(t["x1"]))
    t["g"] = round_f16(qlinear(t["u2"], wg))
    t["p"] = round_f16(qlinear(t["u2"], wu))
    t["m"] = rms_rows(silu_mul(t["g"], t["p"]))
    t["d"] = round_f16(qlinear(t["m"], wd))
    t["x_next"] = rms_rows(_f64(t["x1"]) + _f64(t["d"]))
    return t


def stack_forward(x, layer_mats):
    """Run fp16 [M,H] through a list of blocks (each a 7-list of fp32 matrices)."""
    for mats in layer_mats:
        x = block_forward(x, mats)["x_next"]
    return x


# ------------------------------------------------------------------------- NLL
def token_nll(logits, labels) -> np.ndarray:
    logits = _c(np.asarray(logits).view(np.uint16), np.uint16)
    labels = _c(labels, np.int32)
    M, V = logits.shape
    out = np.empty(M, dtype=np.float64)
    _check(_load().ora_token_nll(_p(logits), _p(labels), M, V, _p(out)), "token_nll")
    return out


def logit_l2(a, b) -> np.ndarray:
    """Row-wise Euclidean distance between two fp16 logit arrays [M,V] (the sensitivity value of the
    search's analysis filter is this distance between a hybrid model's logits and QM(n_up)'s)."""
    a, b = np.asarray(a), np.asarray(b)
    if a.dtype != np.float16 or b.dtype != np.float16:
        raise TypeError("logit_l2 takes fp16 logits (round fp64 ones with round_f16 first)")
    a = _c(a.view(np.uint16), np.uint16)
    b = _c(b.view(np.uint16), np.uint16)
    assert a.shape == b.shape and a.ndim == 2
    M, V = a.shape
    out = np.empty(M, dtype=np.float64)
    _check(_load().ora_logit_l2(_p(a), _p(b), M, V, _p(out)), "logit_l2")
    return out


def perplexity(nll) -> float:
    """exp(mean token NLL) of one sequence."""
    return float(np.exp(np.mean(np.asarray(nll, dtype=np.float64))))
