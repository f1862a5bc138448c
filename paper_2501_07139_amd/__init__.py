"""Python binding of libfq (argument marshalling only).

Every function has the name and meaning of the C entry point declared in
``include/fq.h``; all arithmetic happens inside the library's HIP kernels (or,
for the one-off quantize/pack preparation, its host code).  PyTorch is used for
device memory and streams, numpy for host buffers.  There is no fallback: if the
built library is missing the import fails.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libfq.so")

BIT_WIDTHS = (2, 3, 4, 8)
GROUP = 128

FQ_OK = 0
ERROR_NAMES = {-1: "FQ_ERR_NULL", -2: "FQ_ERR_SHAPE", -3: "FQ_ERR_BITS", -4: "FQ_ERR_GROUP",
               -5: "FQ_ERR_ALIGN", -6: "FQ_ERR_WORKSPACE", -7: "FQ_ERR_HIP"}


class FqError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"{ERROR_NAMES.get(code, code)}: {message}")
        self.code = code


class fq_matrix(ctypes.Structure):
    _fields_ = [("packed", ctypes.c_void_p * 4), ("scales", ctypes.c_void_p * 4), ("zeros", ctypes.c_void_p * 4),
                ("N", ctypes.c_int), ("K", ctypes.c_int)]


class fq_layer(ctypes.Structure):
    _fields_ = [("m", fq_matrix * 7)]


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built; run `python paper_2501_07139_amd/build.py`")
    # PyTorch ships its own HIP runtime (same soname).  Import it first so that libfq binds to
    # that one copy; two runtimes in one process do not both see the device.
    import torch  # noqa: F401

    lib = ctypes.CDLL(LIB_PATH)
    vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    sig = {
        "fq_last_error": (ctypes.c_char_p, []),
        "fq_version": (ctypes.c_char_p, []),
        "fq_quantize_rtn": (ci, [vp, ci, ci, ci, ci, vp, vp, vp]),
        "fq_packed_bytes": (sz, [ci, ci, ci]),
        "fq_meta_count": (sz, [ci, ci, ci]),
        "fq_pack_groups": (ci, [vp, vp, vp, ci, ci, ci, ci, vp, vp, vp]),
        "fq_dequant": (ci, [vp, vp, vp, ci, ci, ci, ci, vp, ci, vp]),
        "fq_qlinear": (ci, [vp, ci, vp, vp, vp, ci, ci, ci, ci, vp, vp]),
        "fq_qlinear_tile": (ci, [vp, ci, vp, vp, vp, ci, ci, ci, ci, vp, ci, vp]),
        "fq_stream_read": (ci, [vp, ctypes.c_size_t, vp, vp]),
        "fq_qlinear_mixed": (ci, [vp, ci, vp, ci, ci, ci, vp, vp]),
        "fq_stack_workspace_bytes": (sz, [ci, ci, ci]),
        "fq_stack_forward": (ci, [ctypes.POINTER(fq_layer), ci, vp, vp, ci, vp, vp, sz, vp]),
        "fq_stack_forward_noalloc": (ci, [ctypes.POINTER(fq_layer), ci, vp, vp, ci, vp, vp]),
        "fq_set_decode_mode": (ci, [ci]),
        "fq_decode_give_up_ticks": (ctypes.c_ulonglong, [ctypes.c_ulonglong]),
        "fq_async_error": (ci, []),
        "fq_decode_persistent": (ci, [ci, ci]),
        "fq_decode_persistent_launches": (ctypes.c_ulonglong, []),
        "fq_decode_partition": (ci, [vp, ci, ci, ci, ci, vp]),
        "fq_clear_async_error": (None, []),
        "fq_glue": (ci, [ci, vp, vp, vp, ci, ci, vp, vp]),
        "fq_init": (ci, []),
        "fq_dense_f16": (ci, [vp, ci, vp, ci, ci, vp, vp]),
        "fq_dense_f16_tile": (ci, [vp, ci, vp, ci, ci, vp, ci, vp]),
        "fq_rope_table": (ci, [ci, ci, ctypes.c_double, vp]),
        "fq_token_nll": (ci, [vp, vp, ci, ci, vp, vp]),
        "fq_logit_l2": (ci, [vp, vp, ci, ci, vp, vp]),
        "fq_head_nll_workspace_bytes": (sz, [ci, ci]),
        "fq_head_nll": (ci, [vp, ci, vp, ci, ci, vp, vp, vp, sz, vp]),
        "fq_attn_workspace_bytes": (sz, [ci, ci]),
        "fq_decode_workspace_bytes": (sz, [ci, ci, ci]),
        "fq_attn_decode": (ci, [vp, vp, vp, vp, vp, ci, ci, ci, vp, vp, vp, sz, vp]),
        "fq_decode_step": (ci, [ctypes.POINTER(fq_layer), ci, vp, vp, vp, vp, vp, ci, ci, vp, vp, sz, vp]),
        "fq_attn_prefill_workspace_bytes": (sz, [ci, ci]),
        "fq_prefill_workspace_bytes": (sz, [ci, ci, ci]),
        "fq_attn_prefill": (ci, [vp, vp, vp, ci, vp, vp, ci, ci, vp, vp, vp, sz, vp]),
        "fq_prefill_forward": (ci, [ctypes.POINTER(fq_layer), ci, vp, vp, ci, vp, vp, vp, ci, vp, vp, sz, vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    return lib


_lib = _load()
EXPORTS = ("fq_last_error", "fq_version", "fq_quantize_rtn", "fq_packed_bytes", "fq_meta_count", "fq_pack_groups",
           "fq_dequant", "fq_qlinear", "fq_qlinear_tile", "fq_qlinear_mixed", "fq_stream_read", "fq_stack_workspace_bytes", "fq_stack_forward", "fq_glue", "fq_dense_f16",
           "fq_token_nll", "fq_logit_l2", "fq_head_nll_workspace_bytes", "fq_head_nll",
           "fq_attn_workspace_bytes", "fq_decode_workspace_bytes", "fq_attn_decode", "fq_decode_step",
           "fq_attn_prefill_workspace_bytes", "fq_prefill_workspace_bytes", "fq_attn_prefill", "fq_prefill_forward",
           "fq_init", "fq_dense_f16_tile", "fq_rope_table", "fq_stack_forward_noalloc", "fq_set_decode_mode",
           "fq_decode_give_up_ticks", "fq_async_error", "fq_clear_async_error", "fq_decode_partition", "fq_decode_persistent",
           "fq_decode_persistent_launches")


def _check(rc: int) -> None:
    if rc != FQ_OK:
        raise FqError(rc, _lib.fq_last_error().decode())


def fq_last_error() -> str:
    return _lib.fq_last_error().decode()


def fq_version() -> str:
    return _lib.fq_version().decode()


def fq_init() -> None:
    """Prepare the library's kernels on the current device (needed before capturing calls into a graph)."""
    _check(_lib.fq_init())


# ------------------------------------------------------------------ host side
def _np(a, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != dtype:
        raise TypeError(f"expected {np.dtype(dtype)}, got {a.dtype}")
    return a


def _hp(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def fq_quantize_rtn(W, bits: int, group: int = GROUP):
    """fp32 [N,K] -> (codes u8 [N,K], scales fp16 [N,K/128], zeros fp16 [N,K/128]), all host."""
    W = _np(W, np.float32)
    N, K = W.shape
    G = max(K // 128, 1)
    codes = np.empty((N, K), dtype=np.uint8)
    scales = np.empty((N, G), dtype=np.float16)
    zeros = np.empty((N, G), dtype=np.float16)
    _check(_lib.fq_quantize_rtn(_hp(W), N, K, bits, group, _hp(codes), _hp(scales), _hp(zeros)))
    return codes, scales, zeros


def fq_packed_bytes(N: int, K: int, bits: int) -> int:
    return _lib.fq_packed_bytes(N, K, bits)


def fq_meta_count(N: int, K: int, group: int = GROUP) -> int:
    return _lib.fq_meta_count(N, K, group)


def fq_pack_groups(codes, scales, zeros, bits: int, group: int = GROUP):
    """Host codes/scales/zeros -> (packed u8, tiled scales fp16, tiled zeros fp16) in the device format."""
    codes = _np(codes, np.uint8)
    N, K = codes.shape
    scales = _np(np.asarray(scales).view(np.float16), np.float16)
    zeros = _np(np.asarray(zeros).view(np.float16), np.float16)
    nbytes, nmeta = fq_packed_bytes(N, K, bits), fq_meta_count(N, K, group)
    packed = np.empty(max(nbytes, 1), dtype=np.uint8)
    st = np.empty(max(nmeta, 1), dtype=np.float16)
    zt = np.empty(max(nmeta, 1), dtype=np.float16)
    _check(_lib.fq_pack_groups(_hp(codes), _hp(scales), _hp(zeros), N, K, bits, group, _hp(packed), _hp(st), _hp(zt)))
    return packed, st, zt


# ---------------------------------------------------------------- device side
def _torch():
    import torch

    return torch


def _dp(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        return _torch().cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _dev(t, dtype, what: str):
    torch = _torch()
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{what} must be a device tensor")
    if t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"{what} must be contiguous {dtype}, got {t.dtype}")
    return t


class PackedMatrix:
    """Device copies of one matrix in one bit-width (packed codes, tiled scales, tiled zeros)."""

    def __init__(self, packed, scales, zeros, N: int, K: int, bits: int):
        self.packed, self.scales, self.zeros = packed, scales, zeros
        self.N, self.K, self.bits = N, K, bits

    @classmethod
    def from_host(cls, codes, scales, zeros, bits: int, device="cuda"):
        torch = _torch()
        N, K = codes.shape
        p, s, z = fq_pack_groups(codes, scales, zeros, bits)
        return cls(torch.from_numpy(p).to(device), torch.from_numpy(s.view(np.int16)).to(device).view(torch.float16),
                   torch.from_numpy(z.view(np.int16)).to(device).view(torch.float16), N, K, bits)

    @property
    def nbytes(self) -> int:
        """Algorithmic bytes of this matrix: packed codes + fp16 scales + fp16 zeros."""
        return self.N * self.K * self.bits // 8 + 2 * 2 * self.N * (self.K // 128)


def fq_dequant(w: PackedMatrix, fp16: bool = False, stream=None):
    torch = _torch()
    out = torch.empty((w.N, w.K), dtype=torch.float16 if fp16 else torch.float32, device=w.packed.device)
    _check(_lib.fq_dequant(_dp(w.packed), _dp(w.scales), _dp(w.zeros), w.N, w.K, w.bits, GROUP, _dp(out), int(fp16),
                           _stream(stream)))
    return out


def fq_qlinear(x, w: PackedMatrix, out=None, stream=None, group: int = GROUP, tile_rows: int = 0):
    torch = _torch()
    x = _dev(x, torch.float16, "x")
    M, K = x.shape
    if K != w.K:
        raise FqError(-2, f"x has K={K}, weights have K={w.K}")
    if out is None:
        out = torch.empty((M, w.N), dtype=torch.float16, device=x.device)
    _dev(out, torch.float16, "out")
    _check(_lib.fq_qlinear_tile(_dp(x), M, _dp(w.packed), _dp(w.scales), _dp(w.zeros), w.N, w.K, w.bits, group,
                                _dp(out), tile_rows, _stream(stream)))
    return out


MAX_SEGMENTS = 8


class _Segment(ctypes.Structure):
    _fields_ = [("packed", ctypes.c_void_p), ("scales", ctypes.c_void_p), ("zeros", ctypes.c_void_p),
                ("N", ctypes.c_int), ("bits", ctypes.c_int)]


def fq_qlinear_mixed(x, segments, out=None, stream=None, group: int = GROUP):
    """One matrix stored as runs of output rows, each a PackedMatrix of its own bit-width over the same K."""
    torch = _torch()
    x = _dev(x, torch.float16, "x")
    M, K = x.shape
    if not 1 <= len(segments) <= MAX_SEGMENTS:
        raise FqError(-2, f"{len(segments)} segments (1..{MAX_SEGMENTS})")
    if any(w.K != K for w in segments):
        raise FqError(-2, "every segment must have the K of x")
    arr = (_Segment * len(segments))(*[_Segment(_dp(w.packed), _dp(w.scales), _dp(w.zeros), w.N, w.bits) for w in segments])
    if out is None:
        out = torch.empty((M, sum(w.N for w in segments)), dtype=torch.float16, device=x.device)
    _dev(out, torch.float16, "out")
    _check(_lib.fq_qlinear_mixed(_dp(x), M, ctypes.cast(arr, ctypes.c_void_p), len(segments), K, group, _dp(out),
                                 _stream(stream)))
    return out


STREAM_READ_WORDS = 2048


def fq_stream_read(src, sink=None, stream=None):
    """Plain read of a device buffer (a measurement aid); returns the checksum words."""
    torch = _torch()
    if sink is None:
        sink = torch.empty(STREAM_READ_WORDS, dtype=torch.int32, device=src.device)
    _check(_lib.fq_stream_read(_dp(src), src.numel() * src.element_size(), _dp(sink), _stream(stream)))
    return sink


class Stack:
    """Host table of device pointers for L blocks x 7 matrices x the stored bit-widths."""

    def __init__(self, layers: Sequence[Sequence[dict]]):
        # layers[l][j] maps bits -> PackedMatrix
        self.layers = layers
        self.L = len(layers)
        self.table = (fq_layer * self.L)()
        for l, mats in enumerate(layers):
            if len(mats) != 7:
                raise ValueError("a block has seven matrices")
            for j, by_bits in enumerate(mats):
                any_w = next(iter(by_bits.values()))
                entry = self.table[l].m[j]
                entry.N, entry.K = any_w.N, any_w.K
                for i, b in enumerate(BIT_WIDTHS):
                    w = by_bits.get(b)
                    entry.packed[i] = _dp(w.packed) if w else None
                    entry.scales[i] = _dp(w.scales) if w else None
                    entry.zeros[i] = _dp(w.zeros) if w else None
        self.hidden = layers[0][0][next(iter(layers[0][0]))].K
        self.ffn = layers[0][4][next(iter(layers[0][4]))].N


def fq_stack_workspace_bytes(M: int, hidden: int, ffn: int) -> int:
    return _lib.fq_stack_workspace_bytes(M, hidden, ffn)


def fq_stack_forward(stack: Stack, bitvec, x, out=None, workspace=None, stream=None):
    torch = _torch()
    x = _dev(x, torch.float16, "x")
    M = x.shape[0]
    bitvec = _np(np.asarray(bitvec, dtype=np.uint8), np.uint8)
    if bitvec.size != 7 * stack.L:
        raise FqError(-2, f"bitvec has {bitvec.size} entries, stack needs {7 * stack.L}")
    if out is None:
        out = torch.empty_like(x)
    if workspace is None:
        workspace = torch.empty(fq_stack_workspace_bytes(M, stack.hidden, stack.ffn), dtype=torch.uint8, device=x.device)
    _check(_lib.fq_stack_forward(stack.table, stack.L, _hp(bitvec), _dp(x), M, _dp(out), _dp(workspace),
                                 workspace.numel(), _stream(stream)))
    return out


def fq_set_decode_mode(mode: int) -> int:
    """0: per-phase launches (default); 1: the persistent kernel for M == 1 where it applies.  Returns the previous mode."""
    return _lib.fq_set_decode_mode(mode)


def fq_decode_give_up_ticks(ticks: int) -> int:
    return _lib.fq_decode_give_up_ticks(ticks)


def fq_decode_partition(bits7, phase: int, N: int, wg: int, grid: int):
    """[(first, end)] of workgroup wg's work units in each matrix of the phase (see fq.h)."""
    bits7 = _np(np.asarray(bits7, dtype=np.uint8), np.uint8)
    out = np.zeros(6, dtype=np.int32)
    _check(_lib.fq_decode_partition(_hp(bits7), phase, N, wg, grid, _hp(out)))
    return [(int(out[2 * j]), int(out[2 * j + 1])) for j in range(3)]


def fq_decode_persistent(hidden: int, ffn: int) -> int:
    return _lib.fq_decode_persistent(hidden, ffn)


def fq_decode_persistent_launches() -> int:
    return _lib.fq_decode_persistent_launches()


def fq_async_error() -> int:
    return _lib.fq_async_error()


def fq_clear_async_error() -> None:
    _lib.fq_clear_async_error()


def fq_stack_forward_noalloc(stack: Stack, bitvec, x, out, stream=None):
    """fq_stack_forward on the library's own static scratch (M <= 16); `out` is the caller's."""
    torch = _torch()
    x = _dev(x, torch.float16, "x")
    out = _dev(out, torch.float16, "out")
    bitvec = _np(np.asarray(bitvec, dtype=np.uint8), np.uint8)
    if bitvec.size != 7 * stack.L:
        raise FqError(-2, f"bitvec has {bitvec.size} entries, stack needs {7 * stack.L}")
    _check(_lib.fq_stack_forward_noalloc(stack.table, stack.L, _hp(bitvec), _dp(x), x.shape[0], _dp(out),
                                         _stream(stream)))
    return out


def fq_glue(op: int, a, b=None, c=None, out=None, stream=None):
    torch = _torch()
    a = _dev(a, torch.float16, "a")
    M, H = a.shape
    if out is None:
        out = torch.empty_like(a)
    _check(_lib.fq_glue(op, _dp(a), _dp(b), _dp(c), M, H, _dp(out), _stream(stream)))
    return out


def fq_dense_f16(x, W, out=None, stream=None, tile_rows: int = 0):
    """tile_rows = 128 or 256 pins one of the two kernels (fq_dense_f16_tile); 0 lets the library choose."""
    torch = _torch()
    x = _dev(x, torch.float16, "x")
    W = _dev(W, torch.float16, "W")
    M, K = x.shape
    N = W.shape[0]
    if W.shape[1] != K:
        raise FqError(-2, f"x has K={K}, W has K={W.shape[1]}")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=x.device)
    if tile_rows:
        _check(_lib.fq_dense_f16_tile(_dp(x), M, _dp(W), N, K, _dp(out), tile_rows, _stream(stream)))
    else:
        _check(_lib.fq_dense_f16(_dp(x), M, _dp(W), N, K, _dp(out), _stream(stream)))
    return out


def fq_logit_l2(a, b, out=None, stream=None):
    torch = _torch()
    a = _dev(a, torch.float16, "a")
    b = _dev(b, torch.float16, "b")
    if a.shape != b.shape or a.dim() != 2:
        raise ValueError("fq_logit_l2: a and b must be [M,V] arrays of one shape")
    M, V = a.shape
    if out is None:
        out = torch.empty(M, dtype=torch.float32, device=a.device)
    _check(_lib.fq_logit_l2(_dp(a), _dp(b), M, V, _dp(out), _stream(stream)))
    return out


def fq_head_nll_workspace_bytes(M: int, V: int) -> int:
    return _lib.fq_head_nll_workspace_bytes(M, V)


def fq_head_nll(x, W, labels, out=None, workspace=None, stream=None):
    torch = _torch()
    x = _dev(x, torch.float16, "x")
    W = _dev(W, torch.float16, "W")
    labels = _dev(labels, torch.int32, "labels")
    M, K = x.shape
    V = W.shape[0]
    if W.shape[1] != K or labels.numel() != M:
        raise ValueError("fq_head_nll: x [M,K], W [V,K], labels [M]")
    if out is None:
        out = torch.empty(M, dtype=torch.float32, device=x.device)
    if workspace is None:
        workspace = torch.empty(fq_head_nll_workspace_bytes(M, V), dtype=torch.uint8, device=x.device)
    _check(_lib.fq_head_nll(_dp(x), M, _dp(W), V, K, _dp(labels), _dp(out), _dp(workspace), workspace.numel(),
                            _stream(stream)))
    return out


def fq_token_nll(logits, labels, out=None, stream=None):
    torch = _torch()
    logits = _dev(logits, torch.float16, "logits")
    labels = _dev(labels, torch.int32, "labels")
    M, V = logits.shape
    if out is None:
        out = torch.empty(M, dtype=torch.float32, device=logits.device)
    _check(_lib.fq_token_nll(_dp(logits), _dp(labels), M, V, _dp(out), _stream(stream)))
    return out


# ------------------------------------------------------------ real decoder blocks
def rope_table(Tmax: int, head_dim: int = 128, base: float = 10000.0, device="cuda"):
    """(cos, sin) of pos * base^(-2i/head_dim) as fp32 [Tmax, head_dim/2, 2] on the device: the library's
    host routine fq_rope_table fills it, this only uploads."""
    torch = _torch()
    table = np.empty((Tmax, head_dim // 2, 2), dtype=np.float32)
    _check(_lib.fq_rope_table(Tmax, head_dim, float(base), _hp(table)))
    return torch.from_numpy(table).to(device)


def fq_attn_workspace_bytes(Tmax: int, n_heads: int) -> int:
    return _lib.fq_attn_workspace_bytes(Tmax, n_heads)


def fq_decode_workspace_bytes(hidden: int, ffn: int, Tmax: int) -> int:
    return _lib.fq_decode_workspace_bytes(hidden, ffn, Tmax)


def fq_attn_decode(q, k, v, k_cache, v_cache, pos: int, rope, out=None, workspace=None, stream=None):
    torch = _torch()
    q, k, v = (_dev(t, torch.float16, n) for t, n in ((q, "q"), (k, "k"), (v, "v")))
    k_cache, v_cache = _dev(k_cache, torch.float16, "k_cache"), _dev(v_cache, torch.float16, "v_cache")
    rope = _dev(rope, torch.float32, "rope")
    if k_cache.dim() != 3 or k_cache.shape[2] != 128 or v_cache.shape != k_cache.shape:
        raise ValueError("fq_attn_decode: caches [n_heads, Tmax, 128]")
    n_heads, Tmax, _ = k_cache.shape
    H = 128 * n_heads
    if q.numel() != H or k.numel() != H or v.numel() != H:
        raise ValueError("fq_attn_decode: q, k, v [128 n_heads]")
    if rope.shape[0] < Tmax or tuple(rope.shape[1:]) != (64, 2):
        raise ValueError("fq_attn_decode: rope must be [>=Tmax, 64, 2]")
    if out is None:
        out = torch.empty_like(q)
    if workspace is None:
        workspace = torch.empty(fq_attn_workspace_bytes(Tmax, H // 128), dtype=torch.uint8, device=q.device)
    _check(_lib.fq_attn_decode(_dp(q), _dp(k), _dp(v), _dp(k_cache), _dp(v_cache), pos, Tmax, H // 128, _dp(rope),
                               _dp(out), _dp(workspace), workspace.numel(), _stream(stream)))
    return out


def fq_decode_step(stack: Stack, bitvec, x, k_cache, v_cache, pos: int, rope, out=None, workspace=None, stream=None):
    """One token through the stack's blocks as real decoder blocks; caches fp16 [L, n_heads, Tmax, 128]."""
    torch = _torch()
    x = _dev(x, torch.float16, "x")
    k_cache, v_cache = _dev(k_cache, torch.float16, "k_cache"), _dev(v_cache, torch.float16, "v_cache")
    rope = _dev(rope, torch.float32, "rope")
    bitvec = np.ascontiguousarray(bitvec, dtype=np.uint8)
    if bitvec.size != 7 * stack.L:
        raise ValueError("bitvec needs 7 entries per block")
    if k_cache.dim() != 4 or k_cache.shape[3] != 128 or v_cache.shape != k_cache.shape:
        raise ValueError("fq_decode_step: caches [L, n_heads, Tmax, 128]")
    L, n_heads, Tmax, _ = k_cache.shape
    H = 128 * n_heads
    if L != stack.L or H != stack.hidden or x.numel() != H:
        raise ValueError("fq_decode_step: x [hidden], caches [L, hidden/128, Tmax, 128]")
    if rope.shape[0] < Tmax or tuple(rope.shape[1:]) != (64, 2):
        raise ValueError("fq_decode_step: rope must be [>=Tmax, 64, 2]")
    if out is None:
        out = torch.empty_like(x)
    if workspace is None:
        workspace = torch.empty(fq_decode_workspace_bytes(H, stack.ffn, Tmax), dtype=torch.uint8, device=x.device)
    _check(_lib.fq_decode_step(stack.table, stack.L, _hp(bitvec), _dp(x), _dp(out), _dp(k_cache), _dp(v_cache), pos,
                               Tmax, _dp(rope), _dp(workspace), workspace.numel(), _stream(stream)))
    return out


def fq_attn_prefill_workspace_bytes(T: int, n_heads: int) -> int:
    return _lib.fq_attn_prefill_workspace_bytes(T, n_heads)


def fq_prefill_workspace_bytes(T: int, hidden: int, ffn: int) -> int:
    return _lib.fq_prefill_workspace_bytes(T, hidden, ffn)


def fq_attn_prefill(q, k, v, k_cache, v_cache, rope, out=None, workspace=None, stream=None):
    """Causal attention over rows 0..T-1 (positions 0..T-1); q, k, v fp16 [T, 128 n_heads]; fills the caches."""
    torch = _torch()
    q, k, v = (_dev(t, torch.float16, n) for t, n in ((q, "q"), (k, "k"), (v, "v")))
    k_cache, v_cache = _dev(k_cache, torch.float16, "k_cache"), _dev(v_cache, torch.float16, "v_cache")
    rope = _dev(rope, torch.float32, "rope")
    if k_cache.dim() != 3 or k_cache.shape[2] != 128 or v_cache.shape != k_cache.shape:
        raise ValueError("fq_attn_prefill: caches [n_heads, Tmax, 128]")
    n_heads, Tmax, _ = k_cache.shape
    T, H = q.shape
    if H != 128 * n_heads or k.shape != q.shape or v.shape != q.shape:
        raise ValueError("fq_attn_prefill: q, k, v [T, 128 n_heads]")
    if rope.shape[0] < Tmax or tuple(rope.shape[1:]) != (64, 2):
        raise ValueError("fq_attn_prefill: rope must be [>=Tmax, 64, 2]")
    if out is None:
        out = torch.empty_like(q)
    if workspace is None:
        workspace = torch.empty(fq_attn_prefill_workspace_bytes(T, n_heads), dtype=torch.uint8, device=q.device)
    _check(_lib.fq_attn_prefill(_dp(q), _dp(k), _dp(v), T, _dp(k_cache), _dp(v_cache), Tmax, n_heads, _dp(rope),
                                _dp(out), _dp(workspace), workspace.numel(), _stream(stream)))
    return out


def fq_prefill_forward(stack: Stack, bitvec, x, k_cache, v_cache, rope, out=None, workspace=None, stream=None):
    """A whole sequence x [T, hidden] through the stack's blocks as real decoder blocks; caches
    fp16 [L, n_heads, Tmax, 128], positions 0..T-1 filled."""
    torch = _torch()
    x = _dev(x, torch.float16, "x")
    k_cache, v_cache = _dev(k_cache, torch.float16, "k_cache"), _dev(v_cache, torch.float16, "v_cache")
    rope = _dev(rope, torch.float32, "rope")
    bitvec = np.ascontiguousarray(bitvec, dtype=np.uint8)
    if bitvec.size != 7 * stack.L:
        raise ValueError("bitvec needs 7 entries per block")
    if k_cache.dim() != 4 or k_cache.shape[3] != 128 or v_cache.shape != k_cache.shape:
        raise ValueError("fq_prefill_forward: caches [L, n_heads, Tmax, 128]")
    L, n_heads, Tmax, _ = k_cache.shape
    T, H = x.shape
    if L != stack.L or H != stack.hidden or H != 128 * n_heads:
        raise ValueError("fq_prefill_forward: x [T, hidden], caches [L, hidden/128, Tmax, 128]")
    if rope.shape[0] < Tmax or tuple(rope.shape[1:]) != (64, 2):
        raise ValueError("fq_prefill_forward: rope must be [>=Tmax, 64, 2]")
    if out is None:
        out = torch.empty_like(x)
    if workspace is None:
        workspace = torch.empty(fq_prefill_workspace_bytes(T, H, stack.ffn), dtype=torch.uint8, device=x.device)
    _check(_lib.fq_prefill_forward(stack.table, stack.L, _hp(bitvec), _dp(x), T, _dp(out), _dp(k_cache), _dp(v_cache),
                                   Tmax, _dp(rope), _dp(workspace), workspace.numel(), _stream(stream)))
    return out
