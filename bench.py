#!/usr/bin/env python3
"""Benchmark of the mixed-bit quantized-linear hot path on one MI355X.

Workload ("llama2-7b-block"): the seven linears of one Llama-2-7B-shaped decoder
block (q/k/v/o 4096x4096, gate/up 4096->11008, down 11008->4096), group 128,
per-matrix bit-widths drawn (seeded) from {2,3,4,8}, random-init weights,
synthetic activations.  One step is one pass of the whole path:

  leg A (calibration forward, M=2048): block forward through fq_stack_forward,
        fp16 head 4096->32000, fused token NLL;
  leg B (decode, M=1): the block's GEMVs through fq_stack_forward over DECODE_LAYERS
        distinct copies of the block, so that every pass streams more packed bytes
        than the 256 MB last-level cache holds (cold weights, launch gaps included).

Prints ONE JSON line.  `value` is the dequant-GEMM rate at M=2048 (algorithmic flops of
the block's seven launches over the sum of their median durations); the decode rate
(packed bytes per second over the cold 8-block stack) is in `roofline_gemv`; `legs`
holds the step's other parts and the legs beyond the step: the 13B-shaped block at
M=4096 and M=1, the ensemble sweep (64 bit vectors x 4 sequences over a 32-block
stack), single decode launches rotating over more than 512 MB, a plain streaming
read of the decode footprint as the practical ceiling.  Kernel durations are taken
with events on the launch stream, 50 repetitions, median and minimum reported.
`roofline` is for the kernel the step spends most of its time in (the dequant-GEMM);
`cpu_baseline` times the CPU oracle on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

HIDDEN, FFN, VOCAB = 4096, 11008, 32000
M_FWD = 2048
DECODE_LAYERS = 8
REPS = 50                      # repetitions behind every median / minimum
ROTATE_BYTES = 512 << 20       # single decode launches rotate over at least this much packed data
HIDDEN_13B, FFN_13B, M_13B = 5120, 13824, 4096
SWEEP_VECTORS, SWEEP_SEQUENCES = 64, 4
PEAK_MFMA_F16_TFLOPS = 2516.6  # 256 CU x 4096 flop/clk x 2.4 GHz
PEAK_HBM_GBPS = 8000.0
SEED = 1

# HBM traffic of the seven dequant-GEMM launches of leg A, from two `rocprofv3 --pmc` runs (FETCH_SIZE, then
# WRITE_SIZE, KiB per dispatch) scaled by what the same counters read for a 64 MiB device copy (FETCH_SIZE
# reads 0.500 of the true bytes on this machine, WRITE_SIZE 1.000).  Valid only for the kernel sources whose
# digest is recorded with it; bench.py reports null once they have changed.
GEMM_TRAFFIC = {"kernel_digest": "efcd1fc7f8bd8b14", "fetch_bytes": 820.1e6, "write_bytes": 174.1e6}  # profiles/qgemm_gemv_llama2-7b-block_hbm_traffic.txt


SWAP_ENTRY = 4  # the matrix (gate) the transition leg swaps


def kernel_digest() -> str:
    import hashlib

    h = hashlib.sha256()
    for name in ("fq_gemm.hip", "fq_device.h"):
        with open(os.path.join(ROOT, "paper_2501_07139_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing (profiling runs)")
    ap.add_argument("--cpu-rows", type=int, default=96, help="rows of leg A the oracle is timed on")
    ap.add_argument("--single-launches", action="store_true",
                    help="for counter runs: a 64 MiB device copy, then one launch of each linear at M=2048 and M=1 and one of the head with fused loss, no timing")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch

    import fq_synth
    import paper_2501_07139_amd as fq

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    fq.fq_init()  # kernel attributes and occupancy figures, once: every later call only enqueues work

    def to_dev(a):
        if a.dtype == np.float16:
            return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.float16)
        return torch.from_numpy(a).to(dev)

    # ---------------------------------------------------------------- inputs
    shapes = fq_synth.block_matrix_shapes(HIDDEN, FFN)
    bitvec = fq_synth.bit_vector(SEED, 7, probs=(0.25, 0.25, 0.25, 0.25))
    host_q = []   # per matrix: (codes, scales, zeros) at the selected bit-width (for the oracle leg)
    block = []    # per matrix: {bits: PackedMatrix}
    for j, (N, K) in enumerate(shapes):
        W = fq_synth.weights(SEED, N, K, 0.02, 0, j)
        b = int(bitvec[j])
        codes, s, z = fq.fq_quantize_rtn(W, b)
        host_q.append((codes, s, z))
        block.append({b: fq.PackedMatrix.from_host(codes, s, z, b)})
        if j == SWAP_ENTRY:  # a second stored width of one matrix, for the transition leg
            swap_bits = 2 if b != 2 else 4
            swap_q = fq.fq_quantize_rtn(W, swap_bits)
        del W
    # decode leg: DECODE_LAYERS distinct device copies of the block
    dec_layers = [block]
    for _ in range(DECODE_LAYERS - 1):
        dec_layers.append([{b: fq.PackedMatrix(w.packed.clone(), w.scales.clone(), w.zeros.clone(), w.N, w.K, b)
                            for b, w in m.items()} for m in block])
    stack_fwd = fq.Stack([block])
    stack_dec = fq.Stack(dec_layers)
    bitvec_dec = np.tile(bitvec, DECODE_LAYERS)

    x_fwd_h = fq_synth.activations(SEED, M_FWD, HIDDEN)
    x_fwd = to_dev(x_fwd_h)
    x_dec = to_dev(fq_synth.activations(SEED + 1, 1, HIDDEN))
    head_h = fq_synth.weights(SEED, VOCAB, HIDDEN, 0.02, 99).astype(np.float16)
    head = to_dev(head_h)
    labels_h = fq_synth.labels(SEED, M_FWD, VOCAB)
    labels = to_dev(labels_h)

    ws_fwd = torch.empty(fq.fq_stack_workspace_bytes(M_FWD, HIDDEN, FFN), dtype=torch.uint8, device=dev)
    ws_dec = torch.empty(fq.fq_stack_workspace_bytes(1, HIDDEN, FFN), dtype=torch.uint8, device=dev)
    h_out = torch.empty_like(x_fwd)
    d_out = torch.empty_like(x_dec)
    logits = torch.empty((M_FWD, VOCAB), dtype=torch.float16, device=dev)
    nll = torch.empty(M_FWD, dtype=torch.float32, device=dev)

    ws_head = torch.empty(fq.fq_head_nll_workspace_bytes(M_FWD, VOCAB), dtype=torch.uint8, device=dev)

    def leg_a():
        # block forward, then head GEMM and token loss in one call (the logits are never stored)
        fq.fq_stack_forward(stack_fwd, bitvec, x_fwd, out=h_out, workspace=ws_fwd)
        fq.fq_head_nll(h_out, head, labels, out=nll, workspace=ws_head)

    def leg_b():
        fq.fq_stack_forward(stack_dec, bitvec_dec, x_dec, out=d_out, workspace=ws_dec)

    def step():
        leg_a()
        leg_b()

    if args.single_launches:
        src = torch.empty(64 << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)  # reference dispatch: reads 64 MiB, writes 64 MiB
        torch.cuda.synchronize()
        u = fq.fq_glue(0, x_fwd)
        mm = torch.empty((M_FWD, FFN), dtype=torch.float16, device=dev).normal_()
        for j, (N, K) in enumerate(shapes):
            w = block[j][int(bitvec[j])]
            fq.fq_qlinear(mm if K == FFN else u, w)
            torch.cuda.synchronize()
            fq.fq_qlinear((mm if K == FFN else u)[:1].contiguous(), w)
            torch.cuda.synchronize()
        fq.fq_head_nll(u, head, labels, out=nll, workspace=ws_head)
        torch.cuda.synchronize()
        print("single launches done: copy, then (M=2048, M=1) for " + ", ".join(
            "%s %d-bit" % (fq_synth.MATRIX_NAMES[j], int(bitvec[j])) for j in range(7)) + ", then head with fused loss")
        return

    # ------------------------------------------------------- algorithmic work
    gemm_flops = sum(2.0 * M_FWD * N * K for N, K in shapes)
    head_flops = 2.0 * M_FWD * VOCAB * HIDDEN
    gemv_flops = DECODE_LAYERS * sum(2.0 * N * K for N, K in shapes)
    block_bytes = sum(block[j][int(bitvec[j])].nbytes + 2 * K + 2 * N for j, (N, K) in enumerate(shapes))
    gemv_bytes = DECODE_LAYERS * block_bytes
    nll_bytes = 2.0 * M_FWD * VOCAB
    step_flops = gemm_flops + head_flops + gemv_flops

    # ------------------------------------------------------------ timed steps
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    # per-leg and per-kernel durations with events on the launch stream: one pair of events per repetition,
    # all queued before the first wait, so the device never idles between them
    def durations(fn, reps=REPS):
        fn()
        torch.cuda.synchronize()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for a, b in ev:
            a.record()
            fn()
            b.record()
        torch.cuda.synchronize()
        return np.array([a.elapsed_time(b) for a, b in ev])  # ms

    def timed(fn, reps=REPS):
        return float(np.median(durations(fn, reps)))

    def med_min(fn, reps=REPS, per=1):
        d = durations(fn, reps) / per
        return float(np.median(d)), float(d.min())

    reps = REPS
    ms_fwd_block = timed(lambda: fq.fq_stack_forward(stack_fwd, bitvec, x_fwd, out=h_out, workspace=ws_fwd), reps)
    ms_head_nll = timed(lambda: fq.fq_head_nll(h_out, head, labels, out=nll, workspace=ws_head), reps)
    # the same two steps as separate calls (not part of the step): head GEMM storing its logits, loss reading them
    nll_two = torch.empty_like(nll)
    ms_head = timed(lambda: fq.fq_dense_f16(h_out, head, out=logits), reps)
    ms_nll = timed(lambda: fq.fq_token_nll(logits, labels, out=nll_two), reps)
    ms_dec, ms_dec_min = med_min(leg_b)
    # beyond the step: the logit distance of the search's sensitivity analysis (reads two logit arrays once)
    logits_b = torch.empty_like(logits).normal_(0.0, 1.28)
    l2 = torch.empty(M_FWD, dtype=torch.float32, device=dev)
    ms_l2 = timed(lambda: fq.fq_logit_l2(logits, logits_b, out=l2), reps)

    # the dominant kernel: dequant-GEMM launches of leg A, one by one
    kernels = []
    u = fq.fq_glue(0, x_fwd)
    mm = torch.empty((M_FWD, FFN), dtype=torch.float16, device=dev).normal_()
    gemm_ms_total = 0.0
    for j, (N, K) in enumerate(shapes):
        w = block[j][int(bitvec[j])]
        xin = mm if K == FFN else u
        out = torch.empty((M_FWD, N), dtype=torch.float16, device=dev)
        ms, ms_min = med_min(lambda: fq.fq_qlinear(xin, w, out=out))
        gemm_ms_total += ms
        kernels.append({"matrix": fq_synth.MATRIX_NAMES[j], "N": N, "K": K, "bits": int(bitvec[j]),
                        "ms": round(ms, 4), "ms_min": round(ms_min, 4), "tflops": round(2.0 * M_FWD * N * K / ms / 1e9, 1)})
    gemm_tflops = gemm_flops / gemm_ms_total / 1e9

    # GEMV kernels of leg B, rotating over the distinct copies (cold).  The launches are replayed from a
    # captured HIP graph: issued one by one from Python they would be bound by the host's call rate.
    gemv_ms_total = 0.0
    gemv_kernels = []
    for j, (N, K) in enumerate(shapes):
        w0 = block[j][int(bitvec[j])]
        copies = -(-ROTATE_BYTES // w0.nbytes)  # enough distinct copies to pass 512 MB, twice the last-level cache
        ws = [w0] + [fq.PackedMatrix(w0.packed.clone(), w0.scales.clone(), w0.zeros.clone(), w0.N, w0.K, w0.bits)
                     for _ in range(copies - 1)]
        xin = torch.empty((1, K), dtype=torch.float16, device=dev).normal_()
        out = torch.empty((1, N), dtype=torch.float16, device=dev)

        def rot():
            for w in ws:
                fq.fq_qlinear(xin, w, out=out)

        rot()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            rot()
        ms, ms_min = med_min(graph.replay, per=copies)
        gemv_ms_total += ms
        nbytes = w0.nbytes + 2 * K + 2 * N
        gemv_kernels.append({"matrix": fq_synth.MATRIX_NAMES[j], "N": N, "K": K, "bits": int(bitvec[j]), "copies": copies,
                             "us": round(ms * 1e3, 2), "us_min": round(ms_min * 1e3, 2),
                             "GBps": round(nbytes / ms / 1e6, 1)})
        del ws, graph

    # ---------------------------------------------------------- legs beyond the step
    # Each runs on its own and reports {"error": ...} if it fails: the step's figures above do not depend on them.
    def optional(fn):
        try:
            return fn()
        except Exception as e:  # noqa: BLE001 - the reason is reported in the JSON line
            torch.cuda.synchronize()
            return {"error": "%s: %s" % (type(e).__name__, e)}

    T_CTX = 2048

    def leg_real_blocks():
        """The 8 block copies as real decoder blocks: one token over a key/value cache of 2048 positions, and
        the block over a whole sequence of 2048 positions (causal attention)."""
        rope = fq.rope_table(T_CTX)
        kc = torch.empty((DECODE_LAYERS, HIDDEN // 128, T_CTX, 128), dtype=torch.float16, device=dev).normal_()
        vc = torch.empty_like(kc).normal_()
        ws_real = torch.empty(fq.fq_decode_workspace_bytes(HIDDEN, FFN, T_CTX), dtype=torch.uint8, device=dev)
        x_tok = x_dec.view(-1)
        y_tok = torch.empty_like(x_tok)
        ms_real = timed(lambda: fq.fq_decode_step(stack_dec, bitvec_dec, x_tok, kc, vc, T_CTX - 1, rope, out=y_tok,
                                                  workspace=ws_real), reps)
        q1 = torch.empty(HIDDEN, dtype=torch.float16, device=dev).normal_()
        a1 = torch.empty_like(q1)

        def attn_rot():  # one call per layer's cache: cold reads
            for l in range(DECODE_LAYERS):
                fq.fq_attn_decode(q1, q1, q1, kc[l], vc[l], T_CTX - 1, rope, out=a1, workspace=ws_real)

        attn_rot()
        torch.cuda.synchronize()
        attn_graph = torch.cuda.CUDAGraph()  # replayed from a graph: issued from Python the calls are host-bound
        with torch.cuda.graph(attn_graph):
            attn_rot()
        ms_attn = timed(attn_graph.replay, reps) / DECODE_LAYERS
        kv_bytes = 2.0 * T_CTX * HIDDEN * 2
        ws_pre = torch.empty(fq.fq_prefill_workspace_bytes(M_FWD, HIDDEN, FFN), dtype=torch.uint8, device=dev)
        pre_out = torch.empty_like(x_fwd)
        ms_prefill = timed(lambda: fq.fq_prefill_forward(stack_fwd, bitvec, x_fwd, kc[:1], vc[:1], rope, out=pre_out,
                                                         workspace=ws_pre), reps)
        qkv_rows = [torch.empty((M_FWD, HIDDEN), dtype=torch.float16, device=dev).normal_() for _ in range(3)]
        a_rows = torch.empty_like(qkv_rows[0])
        ms_attn_pre = timed(lambda: fq.fq_attn_prefill(qkv_rows[0], qkv_rows[1], qkv_rows[2], kc[0], vc[0], rope,
                                                       out=a_rows, workspace=ws_pre), reps)
        attn_flops = 2 * 2.0 * (HIDDEN // 128) * 128 * (M_FWD * (M_FWD + 1) / 2)  # causal: QK^T and PV
        return {"decode": {"context": T_CTX, "layers": DECODE_LAYERS, "ms": round(ms_real, 4),
                           "us_per_block": round(ms_real * 1e3 / DECODE_LAYERS, 2),
                           "GBps_weights_and_cache": round((gemv_bytes + DECODE_LAYERS * kv_bytes) / ms_real / 1e6, 1),
                           "attention_us": round(ms_attn * 1e3, 2),
                           "attention_GBps": round(kv_bytes / ms_attn / 1e6, 1),
                           "attention_frac_hbm_peak": round(kv_bytes / ms_attn / 1e6 / PEAK_HBM_GBPS, 4)},
                "prefill": {"positions": M_FWD, "ms_block": round(ms_prefill, 4),
                            "tflops_block": round((gemm_flops + attn_flops) / ms_prefill / 1e9, 1),
                            "attention_ms": round(ms_attn_pre, 4),
                            "attention_tflops": round(attn_flops / ms_attn_pre / 1e9, 1)}}

    def leg_transition():
        """A run-time transition: one matrix swapped for its other stored width and back.  The new packing comes
        from pinned host memory, so this is a PCIe figure."""
        from paper_2501_07139_amd import elastic

        store = elastic.HostStore([[{int(bitvec[j]): host_q[j], **({swap_bits: swap_q} if j == SWAP_ENTRY else {})}
                                    for j in range(7)]])
        members = [tuple(int(b) for b in bitvec),
                   tuple(swap_bits if j == SWAP_ENTRY else int(b) for j, b in enumerate(bitvec))]
        members.sort(key=lambda v: -v[SWAP_ENTRY])
        hosted = elastic.ElasticModel(store, members)
        for _ in range(2):  # first use: allocations
            hosted.move_to(1)
            hosted.move_to(0)
        torch.cuda.synchronize()
        loaded0, t0 = hosted.bytes_loaded, time.perf_counter()
        for _ in range(5):
            hosted.move_to(1)
            hosted.move_to(0)
        torch.cuda.synchronize()
        swap_s = (time.perf_counter() - t0) / 10
        swap_bytes = (hosted.bytes_loaded - loaded0) / 10
        ms_dec_hosted = timed(lambda: hosted.forward(x_dec), reps)
        return {"matrix": fq_synth.MATRIX_NAMES[SWAP_ENTRY], "widths": [int(bitvec[SWAP_ENTRY]), swap_bits],
                "ms_per_swap": round(swap_s * 1e3, 3), "MB_loaded_per_swap": round(swap_bytes / 1e6, 2),
                "GBps_host_to_device": round(swap_bytes / swap_s / 1e9, 1),
                "ms_block_decode_of_hosted_model": round(ms_dec_hosted, 4)}

    def leg_gemv_large():
        """The decode kernel on a 70B-shaped matrix (8192 -> 28672), where the fixed cost of a launch no longer
        dominates: packed bytes are random, scales and zeros constants (no quantizer run), 4 cold copies."""
        big = []
        BN, BK = 28672, 8192
        for bb in (2, 4, 8):
            nb, nm = fq.fq_packed_bytes(BN, BK, bb), fq.fq_meta_count(BN, BK)
            ws_big = [fq.PackedMatrix(torch.randint(0, 255, (nb,), dtype=torch.uint8, device=dev),
                                      torch.full((nm,), 0.01, dtype=torch.float16, device=dev),
                                      torch.full((nm,), 1.0, dtype=torch.float16, device=dev), BN, BK, bb) for _ in range(4)]
            xb = torch.empty((1, BK), dtype=torch.float16, device=dev).normal_()
            ob = torch.empty((1, BN), dtype=torch.float16, device=dev)

            def rot_big():
                for w in ws_big:
                    fq.fq_qlinear(xb, w, out=ob)

            rot_big()
            torch.cuda.synchronize()
            gb = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gb):
                rot_big()
            msb = timed(gb.replay, reps) / 4
            big.append({"N": BN, "K": BK, "bits": bb, "MB": round(ws_big[0].nbytes / 1e6, 1), "us": round(msb * 1e3, 2),
                        "GBps": round(ws_big[0].nbytes / msb / 1e6, 1),
                        "frac_hbm_peak": round(ws_big[0].nbytes / msb / 1e6 / PEAK_HBM_GBPS, 4)})
            del ws_big, gb
        return big

    def leg_full_stack():
        """The ensemble sweep: the whole 32-block 7B-shaped stack with all four widths of every matrix resident
        (random packed bytes, constant scales and zeros: no quantizer run), scored for 64 seeded bit vectors
        averaging about 3.5 bits on 4 calibration sequences of 2048 tokens each (one forward of 8192 rows per
        vector through the stack, the head and the loss)."""
        L_FULL, CANDS, SEQS = 32, SWEEP_VECTORS, SWEEP_SEQUENCES
        layers = []
        resident = 0
        for _ in range(L_FULL):
            mats = []
            for (N, K) in shapes:
                by = {}
                for bb in (2, 3, 4, 8):
                    nb, nm = fq.fq_packed_bytes(N, K, bb), fq.fq_meta_count(N, K)
                    by[bb] = fq.PackedMatrix(torch.randint(0, 255, (nb,), dtype=torch.uint8, device=dev),
                                             torch.full((nm,), 0.01, dtype=torch.float16, device=dev),
                                             torch.full((nm,), float((1 << bb) // 2), dtype=torch.float16, device=dev),
                                             N, K, bb)
                    resident += by[bb].nbytes
                mats.append(by)
            layers.append(mats)
        full = fq.Stack(layers)
        vecs = [fq_synth.bit_vector(SEED + 10 + c, 7 * L_FULL, probs=(0.3, 0.3, 0.3, 0.1)) for c in range(CANDS)]
        rows = SEQS * M_FWD
        x_seq = x_fwd.repeat(SEQS, 1) * torch.linspace(0.9, 1.1, SEQS, device=dev, dtype=torch.float16).repeat_interleave(M_FWD)[:, None]
        lab_seq = labels.repeat(SEQS)
        hid = torch.empty_like(x_seq)
        losses = torch.empty(rows, dtype=torch.float32, device=dev)
        ws_seq = torch.empty(fq.fq_stack_workspace_bytes(rows, HIDDEN, FFN), dtype=torch.uint8, device=dev)
        ws_head_seq = torch.empty(fq.fq_head_nll_workspace_bytes(rows, VOCAB), dtype=torch.uint8, device=dev)

        def score(c):
            fq.fq_stack_forward(full, vecs[c], x_seq, out=hid, workspace=ws_seq)
            fq.fq_head_nll(hid, head, lab_seq, out=losses, workspace=ws_head_seq)

        score(0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for c in range(CANDS):
            score(c)
        torch.cuda.synchronize()
        per = (time.perf_counter() - t0) / CANDS
        flops = SEQS * (L_FULL * gemm_flops + head_flops)
        return {"blocks": L_FULL, "resident_GB": round(resident / 1e9, 2), "bit_vectors": CANDS, "sequences": SEQS,
                "tokens_per_sequence": M_FWD, "mean_bits": round(float(np.mean(np.concatenate(vecs))), 2),
                "s_whole_sweep": round(per * CANDS, 3), "ms_per_bit_vector": round(per * 1e3, 3),
                "tokens_per_s": round(rows / per, 1), "tflops": round(flops / per / 1e12, 1),
                "finite": bool(torch.isfinite(losses).all().item())}

    def random_matrix(N, K, bb):
        """A packed matrix of random bytes with constant scales and zeros (no quantizer run)."""
        nb, nm = fq.fq_packed_bytes(N, K, bb), fq.fq_meta_count(N, K)
        return fq.PackedMatrix(torch.randint(0, 255, (nb,), dtype=torch.uint8, device=dev),
                               torch.full((nm,), 0.01, dtype=torch.float16, device=dev),
                               torch.full((nm,), float((1 << bb) // 2), dtype=torch.float16, device=dev), N, K, bb)

    def leg_13b():
        """A Llama-2-13B-shaped block (hidden 5120, FFN 13824) with bit-widths drawn 60/30/10 % from 2/3/4:
        the seven dequant-GEMM launches and the block forward at M=4096, and decode at M=1 over 8 distinct
        copies of the block (cold weights, more than the 256 MB last-level cache)."""
        shapes13 = fq_synth.block_matrix_shapes(HIDDEN_13B, FFN_13B)
        bv = fq_synth.bit_vector(SEED + 4, 7, probs=(0.6, 0.3, 0.1, 0.0))
        copies = [[{int(bv[j]): random_matrix(N, K, int(bv[j]))} for j, (N, K) in enumerate(shapes13)]
                  for _ in range(DECODE_LAYERS)]
        flops13 = sum(2.0 * M_13B * N * K for N, K in shapes13)
        bytes13 = sum(copies[0][j][int(bv[j])].nbytes + 2 * K + 2 * N for j, (N, K) in enumerate(shapes13))
        xm = torch.empty((M_13B, HIDDEN_13B), dtype=torch.float16, device=dev).normal_()
        xf = torch.empty((M_13B, FFN_13B), dtype=torch.float16, device=dev).normal_()
        per_kernel, total = [], 0.0
        for j, (N, K) in enumerate(shapes13):
            w = copies[0][j][int(bv[j])]
            o = torch.empty((M_13B, N), dtype=torch.float16, device=dev)
            ms, ms_min = med_min(lambda: fq.fq_qlinear(xf if K == FFN_13B else xm, w, out=o))
            total += ms
            per_kernel.append({"matrix": fq_synth.MATRIX_NAMES[j], "N": N, "K": K, "bits": int(bv[j]), "ms": round(ms, 4),
                               "ms_min": round(ms_min, 4), "tflops": round(2.0 * M_13B * N * K / ms / 1e9, 1)})
        one = fq.Stack([copies[0]])
        ws13 = torch.empty(fq.fq_stack_workspace_bytes(M_13B, HIDDEN_13B, FFN_13B), dtype=torch.uint8, device=dev)
        ho = torch.empty_like(xm)
        ms_blk, ms_blk_min = med_min(lambda: fq.fq_stack_forward(one, bv, xm, out=ho, workspace=ws13))
        dec = fq.Stack(copies)
        bv_dec = np.tile(bv, DECODE_LAYERS)
        x1 = torch.empty((1, HIDDEN_13B), dtype=torch.float16, device=dev).normal_()
        o1 = torch.empty_like(x1)
        ws1 = torch.empty(fq.fq_stack_workspace_bytes(1, HIDDEN_13B, FFN_13B), dtype=torch.uint8, device=dev)
        ms_d, ms_d_min = med_min(lambda: fq.fq_stack_forward(dec, bv_dec, x1, out=o1, workspace=ws1))
        gbps = DECODE_LAYERS * bytes13 / ms_d / 1e6
        return {"workload": "llama2-13b-block: bits %s (60/30/10 %% of 2/3/4), random packed bytes" % "/".join(map(str, bv)),
                "gemm_m4096": {"tflops_kernels": round(flops13 / total / 1e9, 1),
                               "frac_mfma_peak": round(flops13 / total / 1e9 / PEAK_MFMA_F16_TFLOPS, 4),
                               "ms_block_forward": round(ms_blk, 4), "ms_block_forward_min": round(ms_blk_min, 4),
                               "tflops_block_forward": round(flops13 / ms_blk / 1e9, 1), "kernels": per_kernel},
                "gemv_m1": {"layers": DECODE_LAYERS, "MB_streamed": round(DECODE_LAYERS * bytes13 / 1e6, 1),
                            "ms_stack_decode": round(ms_d, 4), "ms_stack_decode_min": round(ms_d_min, 4),
                            "GBps_stack_decode": round(gbps, 1), "frac_hbm_peak": round(gbps / PEAK_HBM_GBPS, 4)}}

    def leg_mixed_matrix():
        """Widths mixed within one matrix: a 4096 x 4096 matrix stored as three runs of output rows (60 % at
        2 bits, 30 % at 3, 10 % at 4: 2.5 bits on average), decode (M=1, rotating over cold copies) and M=2048."""
        runs = [(2432, 2), (1232, 3), (432, 4)]
        one_bytes = sum(fq.fq_packed_bytes(N, HIDDEN, bb) + 4 * fq.fq_meta_count(N, HIDDEN) for N, bb in runs)
        copies = -(-ROTATE_BYTES // one_bytes)
        mats = [[random_matrix(N, HIDDEN, bb) for N, bb in runs] for _ in range(copies)]
        x1 = torch.empty((1, HIDDEN), dtype=torch.float16, device=dev).normal_()
        o1 = torch.empty((1, HIDDEN), dtype=torch.float16, device=dev)

        def rot():
            for segs in mats:
                fq.fq_qlinear_mixed(x1, segs, out=o1)

        rot()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            rot()
        us, us_min = med_min(graph.replay, per=copies)
        xm = torch.empty((M_FWD, HIDDEN), dtype=torch.float16, device=dev).normal_()
        om = torch.empty((M_FWD, HIDDEN), dtype=torch.float16, device=dev)
        ms, ms_min = med_min(lambda: fq.fq_qlinear_mixed(xm, mats[0], out=om))
        return {"N": HIDDEN, "K": HIDDEN, "runs": [{"rows": N, "bits": bb} for N, bb in runs],
                "mean_bits": round(sum(N * bb for N, bb in runs) / HIDDEN, 2), "copies": copies,
                "gemv_us": round(us * 1e3, 2), "gemv_us_min": round(us_min * 1e3, 2),
                "gemv_GBps": round(one_bytes / us / 1e6, 1), "gemm_ms": round(ms, 4), "gemm_ms_min": round(ms_min, 4),
                "gemm_tflops": round(2.0 * M_FWD * HIDDEN * HIDDEN / ms / 1e9, 1)}

    def leg_stream_read():
        """The practical ceiling of the decode leg: the library's read-only kernel over a buffer as large as the
        packed bytes one decode pass streams (cold: two such buffers alternate)."""
        n = int(gemv_bytes) // 16 * 16
        bufs = [torch.empty(n, dtype=torch.uint8, device=dev).random_(0, 255) for _ in range(2)]
        sink = torch.empty(fq.STREAM_READ_WORDS, dtype=torch.int32, device=dev)
        turn = [0]

        def read():
            fq.fq_stream_read(bufs[turn[0] & 1], sink)
            turn[0] += 1

        ms, ms_min = med_min(read)
        return {"MB": round(n / 1e6, 1), "us": round(ms * 1e3, 2), "us_min": round(ms_min * 1e3, 2),
                "GBps": round(n / ms / 1e6, 1), "frac_hbm_peak": round(n / ms / 1e6 / PEAK_HBM_GBPS, 4)}

    def leg_hbm_reference():
        """What plain device copies reach on this machine, as context for the HBM-bound figures: bytes read plus bytes
        written per second, for a small and a large buffer."""
        out = []
        for mb in (48, 1024):
            src = torch.empty(mb << 20, dtype=torch.uint8, device=dev).random_(0, 255)
            dst = torch.empty_like(src)
            ms = timed(lambda: dst.copy_(src), reps)
            out.append({"MB": mb, "us": round(ms * 1e3, 2), "GBps_read_plus_write": round(2.0 * (mb << 20) / ms / 1e6, 1)})
            del src, dst
        return out

    def leg_by_width():
        """Every distinct matrix shape of the block at every stored width (random packed bytes, constant scales
        and zeros): the dequant-GEMM at M=2048 and the decode kernel at M=1 (graph replay over 8 copies)."""
        table = []
        for (N, K) in ((4096, 4096), (11008, 4096), (4096, 11008)):
            xm = torch.empty((M_FWD, K), dtype=torch.float16, device=dev).normal_()
            x1 = torch.empty((1, K), dtype=torch.float16, device=dev).normal_()
            om = torch.empty((M_FWD, N), dtype=torch.float16, device=dev)
            o1 = torch.empty((1, N), dtype=torch.float16, device=dev)
            for bb in (2, 3, 4, 8):
                nb, nm = fq.fq_packed_bytes(N, K, bb), fq.fq_meta_count(N, K)
                cps = [fq.PackedMatrix(torch.randint(0, 255, (nb,), dtype=torch.uint8, device=dev),
                                       torch.full((nm,), 0.01, dtype=torch.float16, device=dev),
                                       torch.full((nm,), float((1 << bb) // 2), dtype=torch.float16, device=dev), N, K, bb)
                       for _ in range(DECODE_LAYERS)]
                ms_g = timed(lambda: fq.fq_qlinear(xm, cps[0], out=om), reps)

                def rot1():
                    for w in cps:
                        fq.fq_qlinear(x1, w, out=o1)

                rot1()
                torch.cuda.synchronize()
                g1 = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g1):
                    rot1()
                ms_v = timed(g1.replay, reps) / DECODE_LAYERS
                nbytes = cps[0].nbytes + 2 * K + 2 * N
                table.append({"N": N, "K": K, "bits": bb, "gemm_ms": round(ms_g, 4),
                              "gemm_tflops": round(2.0 * M_FWD * N * K / ms_g / 1e9, 1), "gemv_us": round(ms_v * 1e3, 2),
                              "gemv_GBps": round(nbytes / ms_v / 1e6, 1)})
                del cps, g1
        return table

    def leg_same_process():
        """The seven matrices of the block at M=2048 three ways in one process, repetitions interleaved (GPUs of
        the same model differ by several per cent among themselves, so only such figures compare): the 128-row tile kernels, the
        256-row tile kernel, and the vendor's dense fp16 GEMM (torch.matmul on the dequantized matrix: the same
        product with no unpacking)."""
        reps_ab = 30
        t128 = t256 = tvend = 0.0
        for j, (N, K) in enumerate(shapes):
            w = block[j][int(bitvec[j])]
            xin = mm if K == FFN else u
            o1 = torch.empty((M_FWD, N), dtype=torch.float16, device=dev)
            o2 = torch.empty_like(o1)
            wt = fq.fq_dequant(w, fp16=True).t()
            fns = [lambda: fq.fq_qlinear(xin, w, out=o1, tile_rows=128), lambda: fq.fq_qlinear(xin, w, out=o1, tile_rows=256),
                   lambda: torch.matmul(xin, wt, out=o2)]
            for f in fns:
                f()
            torch.cuda.synchronize()
            ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps_ab)]
                  for _ in fns]
            for r in range(reps_ab):
                for i, f in enumerate(fns):
                    ev[i][r][0].record()
                    f()
                    ev[i][r][1].record()
            torch.cuda.synchronize()
            m = [float(np.median([a.elapsed_time(b) for a, b in e])) for e in ev]
            t128, t256, tvend = t128 + m[0], t256 + m[1], tvend + m[2]
            del wt
        return {"tflops_128_row_tiles": round(gemm_flops / t128 / 1e9, 1), "tflops_256_row_tiles": round(gemm_flops / t256 / 1e9, 1),
                "tflops_vendor_dense_fp16": round(gemm_flops / tvend / 1e9, 1), "repetitions": reps_ab,
                "note": "seven launches each, medians of interleaved repetitions; every third launch is the other kind, so each runs a little slower than alone"}

    same_process = optional(leg_same_process)
    block_13b = optional(leg_13b)
    mixed_matrix = optional(leg_mixed_matrix)
    stream_read = optional(leg_stream_read)
    real_blocks = optional(leg_real_blocks)
    by_width = optional(leg_by_width)
    hbm_reference = optional(leg_hbm_reference)
    full_stack = optional(leg_full_stack)
    transition = optional(leg_transition)
    gemv_large = optional(leg_gemv_large)

    traffic = None
    if GEMM_TRAFFIC["kernel_digest"] == kernel_digest() and GEMM_TRAFFIC["fetch_bytes"]:
        traffic = {"fetch_bytes": GEMM_TRAFFIC["fetch_bytes"], "write_bytes": GEMM_TRAFFIC["write_bytes"]}
    # what the seven launches have to move at least: x and y once, packed weights + scales + zeros once
    gemm_alg_bytes = sum(block[j][int(bitvec[j])].nbytes + 2.0 * M_FWD * (N + K) for j, (N, K) in enumerate(shapes))

    result = {
        "metric": "dequant-GEMM TFLOP/s (M=2048) with dequant-GEMV GB/s (M=1) in roofline_gemv, one Llama-2-7B block",
        "value": round(gemm_tflops, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": "llama2-7b-block: 7 linears, bits %s, group 128; value = the seven dequant-GEMM launches at"
                               " M=2048; a step = block forward M=2048 + fp16 head with fused NLL + M=1 decode over %d"
                               " block copies" % ("/".join(map(str, bitvec)), DECODE_LAYERS),
                   "hidden": HIDDEN, "ffn": FFN, "vocab": VOCAB, "seed": SEED},
        "legs": {
            "whole_step": {"tflops": round(step_flops / ms_per_step / 1e9, 2), "ms": round(ms_per_step, 4),
                           "parts": "block forward M=2048 + head with fused NLL + decode M=1 over %d block copies" % DECODE_LAYERS},
            "llama2_13b_block_outside_the_step": block_13b,
            "mixed_widths_within_a_matrix_outside_the_step": mixed_matrix,
            "gemm_m2048": {"tflops_kernels": round(gemm_tflops, 1),
                           "tflops_block_forward": round(gemm_flops / ms_fwd_block / 1e9, 1),
                           "ms_block_forward": round(ms_fwd_block, 4), "frac_mfma_peak": round(gemm_tflops / PEAK_MFMA_F16_TFLOPS, 4)},
            "head_nll_m2048": {"tflops": round(head_flops / ms_head_nll / 1e9, 1), "ms": round(ms_head_nll, 4)},
            "head_alone_outside_the_step": {"tflops": round(head_flops / ms_head / 1e9, 1), "ms": round(ms_head, 4)},
            "nll_alone_outside_the_step": {"GBps": round(nll_bytes / ms_nll / 1e6, 1), "ms": round(ms_nll, 4),
                                           "max_abs_diff_to_fused": float((nll_two - nll).abs().max().item())},
            "logit_l2_outside_the_step": {"GBps": round(2 * nll_bytes / ms_l2 / 1e6, 1), "ms": round(ms_l2, 4),
                                          "frac_hbm_peak": round(2 * nll_bytes / ms_l2 / 1e6 / PEAK_HBM_GBPS, 4)},
            "real_decode_outside_the_step": real_blocks.get("decode", real_blocks),
            "real_prefill_outside_the_step": real_blocks.get("prefill", real_blocks),
            "device_copy_reference_outside_the_step": hbm_reference,
            "every_shape_at_every_width_outside_the_step": by_width,
            "ensemble_sweep_outside_the_step": full_stack,
            "transition_outside_the_step": transition,
            "gemv_large_outside_the_step": gemv_large,
            "tile_heights_and_vendor_dense_same_process_outside_the_step": same_process,
            "gemv_m1": {"GBps_single_launches": round(block_bytes / gemv_ms_total / 1e6, 1),
                        "GBps_stack_decode": round(gemv_bytes / ms_dec / 1e6, 1),
                        "ms_stack_decode": round(ms_dec, 4), "ms_stack_decode_min": round(ms_dec_min, 4),
                        "layers": DECODE_LAYERS, "MB_streamed": round(gemv_bytes / 1e6, 1),
                        "frac_hbm_peak": round(gemv_bytes / ms_dec / 1e6 / PEAK_HBM_GBPS, 4)},
            "stream_read_of_the_decode_footprint": stream_read,
        },
        "kernels": {"gemm": kernels, "gemv": gemv_kernels},
        "roofline": {"bound": "mfma", "achieved": round(gemm_tflops, 1), "peak": PEAK_MFMA_F16_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(gemm_tflops / PEAK_MFMA_F16_TFLOPS, 4), "traffic": traffic,
                     "kernel": "qgemm_tall_kernel (dequant-GEMM, M=2048, the 7 launches of the block, 256-row tiles)",
                     "algorithmic_flops": gemm_flops, "algorithmic_bytes": gemm_alg_bytes},
        "roofline_gemv": {"bound": "hbm", "achieved": round(gemv_bytes / ms_dec / 1e6, 1), "peak": PEAK_HBM_GBPS,
                          "unit": "GB/s", "frac": round(gemv_bytes / ms_dec / 1e6 / PEAK_HBM_GBPS, 4),
                          "frac_of_stream_read": (round(gemv_bytes / ms_dec / 1e6 / stream_read["GBps"], 4)
                                                  if "GBps" in stream_read else None),
                          "kernel": "gemv_stream_kernel (decode, M=1, 4 launches per block, launch gaps included)"},
    }

    # ---------------------------------------------------- CPU oracle baseline
    if not args.no_cpu_baseline:
        try:
            import oracle

            rows = max(1, min(args.cpu_rows, M_FWD))
            t0 = time.perf_counter()
            mats = [oracle.dequant(*host_q[j]) for j in range(7)]
            t = oracle.block_forward(x_fwd_h[:rows], mats)
            lg = oracle.round_f16(oracle.dense_f16(t["x_next"], head_h))
            ref_nll = oracle.token_nll(lg, labels_h[:rows])
            cpu_s = time.perf_counter() - t0
            cpu_flops = rows / M_FWD * (gemm_flops + head_flops)
            result["cpu_baseline"] = {"value": round(cpu_flops / cpu_s / 1e12, 6), "unit": "TFLOP/s",
                                      "cores": oracle.threads(), "kind": "oracle",
                                      "sample": "leg A on %d of %d rows (dequant + block forward + head + NLL), %.1f s"
                                                % (rows, M_FWD, cpu_s)}
            got = nll[:rows].cpu().numpy().astype(np.float64)
            result["parity"] = {"nll_mean_abs_diff_sample": round(float(abs(got.mean() - ref_nll.mean())), 6)}
        except Exception as e:  # noqa: BLE001 - the GPU figures above stand without the CPU leg
            result["cpu_baseline"] = {"error": "%s: %s" % (type(e).__name__, e)}

    print(json.dumps(result))


if __name__ == "__main__":
    main()
