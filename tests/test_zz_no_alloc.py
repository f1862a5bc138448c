"""The entry point that allocates nothing, through the C-ABI, against fq_stack_forward.

fq_stack_forward_noalloc runs the kernels of fq_stack_forward on an array inside the library's device code
instead of a caller's workspace, so its output must equal fq_stack_forward's bit for bit.  Two calls in a
row, the second with fewer rows and a shorter stack, show that nothing left in the array by one call
disturbs the next.
"""
import ctypes

import numpy as np
import pytest

import fq_synth
import oracle

pytestmark = pytest.mark.gpu


def test_no_alloc_stack_forward_matches_the_workspace_entry_point_twice_in_a_row():
    import torch

    import paper_2501_07139_amd as fq

    sh = fq_synth.MODEL_SHAPES["tiny"]
    L = sh["layers"]
    layers = []
    for l in range(L):
        mats = []
        for j, (N, K) in enumerate(fq_synth.block_matrix_shapes(sh["hidden"], sh["ffn"])):
            W = fq_synth.weights(880, N, K, 0.02, l, j)
            mats.append({b: fq.PackedMatrix.from_host(*oracle.quantize_rtn(W, b), b) for b in (2, 3, 4, 8)})
        layers.append(mats)
    stack = fq.Stack(layers)
    short = fq.Stack(layers[:1])
    fq.fq_init()
    stream = torch.cuda.current_stream().cuda_stream or None

    def call(st, M, seed):
        bitvec = fq_synth.bit_vector(seed, 7 * st.L, probs=(0.25, 0.25, 0.25, 0.25))
        x = torch.from_numpy(fq_synth.activations(seed, M, sh["hidden"]).view(np.int16)).cuda().view(torch.float16)
        want = fq.fq_stack_forward(st, bitvec, x)
        got = torch.full_like(x, float("nan"))
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        rc = fq._lib.fq_stack_forward_noalloc(st.table, st.L, bitvec.ctypes.data_as(ctypes.c_void_p), x.data_ptr(), M,
                                              got.data_ptr(), stream)
        assert rc == 0, fq.fq_last_error()
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(got.view(torch.int16), want.view(torch.int16)), (st.L, M)

    call(stack, 16, 881)     # the most rows the entry point takes
    call(short, 3, 882)      # then a smaller input: fewer rows, fewer blocks
    call(stack, 1, 883)      # and the single-token decode shape
    # beyond its limits it refuses instead of overrunning its array
    x = torch.zeros((17, sh["hidden"]), dtype=torch.float16, device="cuda")
    bitvec = np.full(7 * L, 4, dtype=np.uint8)
    rc = fq._lib.fq_stack_forward_noalloc(stack.table, L, bitvec.ctypes.data_as(ctypes.c_void_p), x.data_ptr(), 17,
                                          x.data_ptr(), stream)
    assert rc == -2 and "exceeds" in fq.fq_last_error()
    torch.cuda.synchronize()
