"""Host logic of libfq against the oracle, and the shape of the C-ABI (no GPU needed)."""
import ctypes
import os
import re

import numpy as np
import pytest

import fq_synth
import oracle
import paper_2501_07139_amd as fq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BITS = (2, 3, 4, 8)


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "fq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(fq_[a-z0-9_]+)\s*\(", text))
    assert declared == set(fq.EXPORTS)
    lib = ctypes.CDLL(fq.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name
    assert "gfx950" in fq.fq_version()


@pytest.mark.parametrize("bits", BITS)
def test_quantizer_matches_oracle_bit_for_bit(bits):
    W = fq_synth.weights(40 + bits, 130, 640)
    W[3, :128] = 0.0
    W[4, 128:256] = np.abs(W[4, 128:256])
    W[5, :] *= 1e-7  # scales below the fp16 normal range
    W[6, :] *= 3e3   # large values
    got = fq.fq_quantize_rtn(W, bits)
    want = oracle.quantize_rtn(W, bits)
    for g, w in zip(got, want):
        assert np.array_equal(np.asarray(g).view(np.uint8), np.asarray(w).view(np.uint8))


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("shape", [(1, 128), (70, 256), (64, 1024), (200, 384)])
def test_packer_against_oracle_unpack(bits, shape):
    N, K = shape
    G = K // 128
    for kind in range(4):
        if kind == 0:
            codes = fq_synth.codes(bits, N, K, bits, kind)
        elif kind == 1:
            codes = np.tile((np.arange(K) % (1 << bits)).astype(np.uint8), (N, 1))
        elif kind == 2:
            codes = np.tile((np.arange(N) % (1 << bits)).astype(np.uint8)[:, None], (1, K))
        else:
            codes = np.full((N, K), (1 << bits) - 1, dtype=np.uint8)
        s = fq_synth.activations(1, N, G).astype(np.float16)
        z = fq_synth.activations(2, N, G).astype(np.float16)
        packed, st, zt = fq.fq_pack_groups(codes, s, z, bits)
        assert packed.size == fq.fq_packed_bytes(N, K, bits) == oracle.packed_bytes(N, K, bits)
        assert packed.size == (N + 63) // 64 * 64 * K * bits // 8
        assert st.size == zt.size == fq.fq_meta_count(N, K) == (N + 63) // 64 * 64 * G
        assert np.array_equal(oracle.unpack(packed, N, K, bits), codes)
        assert np.array_equal(oracle.untile_meta(st, N, G).view(np.uint16), s.view(np.uint16))
        assert np.array_equal(oracle.untile_meta(zt, N, G).view(np.uint16), z.view(np.uint16))
    # pad rows are zero codes with zero scale
    Np = (N + 63) // 64 * 64
    if Np > N:
        full = oracle.unpack(packed, Np, K, bits)
        assert not full[N:].any()
        assert not oracle.untile_meta(st, Np, G)[N:].any()


def test_walking_one_code():
    N, K, bits = 64, 128, 3
    s = np.ones((N, 1), dtype=np.float16)
    z = np.zeros((N, 1), dtype=np.float16)
    for n, k in [(0, 0), (63, 127), (17, 102), (33, 103), (5, 19)]:
        codes = np.zeros((N, K), dtype=np.uint8)
        codes[n, k] = 5
        packed, _, _ = fq.fq_pack_groups(codes, s, z, bits)
        assert int(np.unpackbits(packed).sum()) == 2
        assert np.array_equal(oracle.unpack(packed, N, K, bits), codes)


def test_error_codes_without_launching_anything():
    W = np.zeros((4, 128), dtype=np.float32)
    with pytest.raises(fq.FqError) as e:
        fq.fq_quantize_rtn(W, 5)
    assert e.value.code == -3
    with pytest.raises(fq.FqError) as e:
        fq.fq_quantize_rtn(W, 4, group=64)
    assert e.value.code == -4
    with pytest.raises(fq.FqError) as e:
        fq.fq_quantize_rtn(np.zeros((4, 100), dtype=np.float32), 4)
    assert e.value.code == -2
    codes = np.full((4, 128), 9, dtype=np.uint8)
    with pytest.raises(fq.FqError) as e:
        fq.fq_pack_groups(codes, np.ones((4, 1), np.float16), np.zeros((4, 1), np.float16), 3)
    assert e.value.code == -3 and "fit" in str(e.value)
    assert fq.fq_packed_bytes(4, 100, 4) == 0 and fq.fq_packed_bytes(4, 128, 5) == 0
    lib = fq._lib
    assert lib.fq_qlinear(None, 1, None, None, None, 1, 128, 4, 128, None, None) == -1
    assert "NULL" in fq.fq_last_error()
    assert lib.fq_qlinear(16, 1, 16, 16, 16, 1, 128, 7, 128, 16, None) == -3
    assert lib.fq_qlinear(16, 1, 16, 16, 16, 1, 128, 4, 64, 16, None) == -4
    assert lib.fq_qlinear(16, 1, 16, 16, 16, 1, 100, 4, 128, 16, None) == -2
    assert lib.fq_qlinear(16, 1, 24, 16, 16, 1, 128, 4, 128, 16, None) == -5
    assert lib.fq_qlinear(16, 0, 16, 16, 16, 1, 128, 4, 128, 16, None) == -2
    assert lib.fq_token_nll(None, None, 1, 1, None, None) == -1
    assert lib.fq_logit_l2(None, 16, 1, 1, 16, None) == -1
    assert lib.fq_logit_l2(16, 16, 0, 8, 16, None) == -2
    assert lib.fq_logit_l2(16, 24, 1, 8, 16, None) == -5
    assert lib.fq_head_nll(None, 1, 16, 8, 128, 16, 16, 16, 1 << 20, None) == -1
    assert lib.fq_head_nll(16, 1, 16, 8, 100, 16, 16, 16, 1 << 20, None) == -2
    assert lib.fq_head_nll(16, 4, 16, 70, 128, 16, 16, 16, 8, None) == -6 and "need" in fq.fq_last_error()
    assert lib.fq_head_nll(16, 4, 16, 70, 128, 16, 16, None, 1 << 20, None) == -6
    assert lib.fq_head_nll(16, 4, 24, 70, 128, 16, 16, 16, 1 << 20, None) == -5
    assert fq.fq_head_nll_workspace_bytes(4, 70) == 4 * 2 * 8 + 4 * 4 and fq.fq_head_nll_workspace_bytes(0, 70) == 0
    assert fq.fq_head_nll_workspace_bytes(3, 64) % 16 == 0
    assert lib.fq_attn_decode(None, 16, 16, 16, 16, 0, 8, 2, 16, 16, 16, 1 << 20, None) == -1
    assert lib.fq_attn_decode(16, 16, 16, 16, 16, 8, 8, 2, 16, 16, 16, 1 << 20, None) == -2     # pos == Tmax
    assert lib.fq_attn_decode(16, 16, 16, 16, 16, 0, 8, 2, 16, 16, 16, 8, None) == -6
    assert lib.fq_attn_decode(16, 16, 24, 16, 16, 0, 8, 2, 16, 16, 16, 1 << 20, None) == -5
    assert fq.fq_attn_workspace_bytes(128, 2) >= 2 * 1 * 130 * 4 and fq.fq_attn_workspace_bytes(129, 2) >= 2 * 2 * 130 * 4
    assert fq.fq_decode_workspace_bytes(256, 640, 128) >= 8 * 512 + 2 * 1280 + fq.fq_attn_workspace_bytes(128, 2)
    assert fq.fq_decode_workspace_bytes(200, 640, 128) == 0
    assert lib.fq_attn_prefill(None, 16, 16, 4, 16, 16, 8, 2, 16, 16, 16, 1 << 24, None) == -1
    assert lib.fq_attn_prefill(16, 16, 16, 9, 16, 16, 8, 2, 16, 16, 16, 1 << 24, None) == -2     # T > Tmax
    assert lib.fq_attn_prefill(16, 16, 16, 4, 16, 16, 8, 2, 16, 16, 16, 8, None) == -6
    assert fq.fq_attn_prefill_workspace_bytes(65, 2) >= 65 * 256 * 2 + 256 * 128 * 2
    assert fq.fq_prefill_workspace_bytes(0, 256, 640) == 0 and fq.fq_prefill_workspace_bytes(4, 200, 640) == 0
    assert lib.fq_glue(9, 16, 16, 16, 1, 128, 16, None) == -2
    assert lib.fq_dense_f16(16, 1, 16, 1, 100, 16, None) == -2
    # the matrix-core kernels address their arrays through 32-bit offsets: 4 GiB of activations is refused
    assert lib.fq_qlinear(16, 1 << 20, 16, 16, 16, 128, 4096, 4, 128, 16, None) == -2
    assert "4 GiB" in fq.fq_last_error()
    assert lib.fq_dense_f16(16, 1 << 20, 16, 128, 4096, 16, None) == -2
    assert fq.fq_stack_workspace_bytes(0, 128, 128) == 0


def test_stack_forward_rejects_a_missing_packing_before_launching():
    layer = fq.fq_layer()
    for j in range(7):
        layer.m[j].N = 256 if j in (4, 5) else 128
        layer.m[j].K = 256 if j == 6 else 128
        for i in range(4):
            layer.m[j].packed[i] = 4096
            layer.m[j].scales[i] = 4096
            layer.m[j].zeros[i] = 4096
    layer.m[3].packed[1] = None  # no 3-bit packing for matrix o
    table = (fq.fq_layer * 1)(layer)
    bitvec = np.array([4, 4, 4, 3, 4, 4, 4], dtype=np.uint8)
    rc = fq._lib.fq_stack_forward(table, 1, bitvec.ctypes.data_as(ctypes.c_void_p), 4096, 4, 4096, 4096, 1 << 30, None)
    assert rc == -1 and "3-bit" in fq.fq_last_error()
    bitvec[3] = 5
    rc = fq._lib.fq_stack_forward(table, 1, bitvec.ctypes.data_as(ctypes.c_void_p), 4096, 4, 4096, 4096, 1 << 30, None)
    assert rc == -3
    bitvec[3] = 4
    rc = fq._lib.fq_stack_forward(table, 1, bitvec.ctypes.data_as(ctypes.c_void_p), 4096, 4, 4096, 4096, 16, None)
    assert rc == -6


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU only: asked for more it says so and exits without touching a device."""
    import subprocess
    import sys

    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "one GPU" in (r.stdout + r.stderr)


def test_rope_table_against_the_closed_form():
    """fq_rope_table: (cos, sin) of pos * base^(-2i/d), fp64 rounded once to fp32."""
    Tmax, d = 300, 128
    table = np.empty((Tmax, d // 2, 2), dtype=np.float32)
    rc = fq._lib.fq_rope_table(Tmax, d, 10000.0, table.ctypes.data_as(ctypes.c_void_p))
    assert rc == 0
    ang = np.arange(Tmax, dtype=np.float64)[:, None] * 10000.0 ** (-2.0 * np.arange(d // 2, dtype=np.float64) / d)
    # pow and ** may differ in the last place of the fp64 angle: one fp32 ulp of slack, exact almost everywhere
    assert np.max(np.abs(table[..., 0] - np.cos(ang))) <= 2.0 ** -23
    assert np.max(np.abs(table[..., 1] - np.sin(ang))) <= 2.0 ** -23
    assert np.array_equal(table[0, :, 0], np.ones(d // 2, dtype=np.float32)) and not table[0, :, 1].any()
    assert np.allclose(table[..., 0].astype(np.float64) ** 2 + table[..., 1].astype(np.float64) ** 2, 1.0, atol=3e-7)
    assert fq._lib.fq_rope_table(0, d, 10000.0, table.ctypes.data_as(ctypes.c_void_p)) == -2
    assert fq._lib.fq_rope_table(4, 7, 10000.0, table.ctypes.data_as(ctypes.c_void_p)) == -2
    assert fq._lib.fq_rope_table(4, d, 10000.0, None) == -1


def test_dense_tile_argument_is_validated_on_the_host():
    one = ctypes.c_void_p(16)
    assert fq._lib.fq_dense_f16_tile(one, 4, one, 4, 128, one, 64, None) == -2
    assert "tile_rows" in fq.fq_last_error()


def test_new_entry_points_validate_their_arguments_on_the_host():
    """fq_qlinear_tile, fq_qlinear_mixed and fq_stream_read refuse bad arguments before anything is launched."""
    import ctypes

    lib = fq._lib
    assert lib.fq_qlinear_tile(16, 32, 16, 16, 16, 64, 128, 4, 128, 16, 64, None) == -2 and "tile_rows" in fq.fq_last_error()
    assert lib.fq_qlinear_tile(None, 32, 16, 16, 16, 64, 128, 4, 128, 16, 256, None) == -1
    seg = (fq._Segment * 2)(fq._Segment(16, 16, 16, 64, 4), fq._Segment(16, 16, 16, 64, 5))
    p = ctypes.cast(seg, ctypes.c_void_p)
    assert lib.fq_qlinear_mixed(16, 1, p, 0, 128, 128, 16, None) == -2
    assert lib.fq_qlinear_mixed(16, 1, p, fq.MAX_SEGMENTS + 1, 128, 128, 16, None) == -2
    assert lib.fq_qlinear_mixed(16, 1, None, 1, 128, 128, 16, None) == -1
    assert lib.fq_qlinear_mixed(16, 1, p, 2, 128, 128, 16, None) == -3          # the second run's width
    assert lib.fq_qlinear_mixed(16, 1, p, 1, 100, 128, 16, None) == -2          # K
    assert lib.fq_qlinear_mixed(24, 1, p, 1, 128, 128, 16, None) == -5          # alignment of x
    assert lib.fq_qlinear_mixed(16, 0, p, 1, 128, 128, 16, None) == -2
    assert lib.fq_stream_read(None, 64, 16, None) == -1
    assert lib.fq_stream_read(16, 40, 16, None) == -2 and lib.fq_stream_read(16, 0, 16, None) == -2
    assert lib.fq_stream_read(24, 64, 16, None) == -5
    assert fq.fq_set_decode_mode(0) in (0, 1)
