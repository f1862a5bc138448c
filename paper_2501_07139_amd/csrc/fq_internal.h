// Declarations shared by the translation units of libfq (not part of the ABI).
#ifndef FQ_INTERNAL_H
#define FQ_INTERNAL_H

#include <stddef.h>
#include <stdint.h>

#include "fq.h"

int fq_fail(int code, const char *fmt, ...) __attribute__((format(printf, 2, 3)));
int fq_bits_index(int bits);         // 2,3,4,8 -> 0..3, else -1
int fq_rows_per_supertile(int bits); // 32,64,16,16

struct ihipStream_t;
typedef ihipStream_t *fq_stream;

// One packed matrix as the kernels see it.
struct fq_packed_ref {
    const void *packed;
    const void *scales;
    const void *zeros;
    int N, K, bits;
    int ld = 0; // elements between consecutive rows of the output this matrix writes; 0: N (an output of its own)
};

// Launchers.  Arguments are validated by the callers in fq_api.hip; each returns a hipError_t as int.
int fq_launch_dequant(const fq_packed_ref &w, void *out, int out_is_fp16, fq_stream st);
int fq_launch_gemv(const void *x, int M, const fq_packed_ref &w, void *out, fq_stream st);
// Streaming decode kernel: up to three matrices that share their input and K in one launch (M <= 16).
// The input is x = f(a, b, c), fp16 [M,K] each, with the block's row-wise glue folded in:
//   mode 0: a   1: rms(a)   2: rms(a+b+c)   3: aux = a+b, rms(aux)   4: rms(silu(a)*b)   5: aux = rms(a+b), rms(aux)
//   mode 6: silu(a)*b
struct fq_gemv_input {
    const void *a, *b, *c;
    void *aux;
    int mode;
};
// inputs: how many of a, b, c the mode reads (mode 2: three, modes 3 to 6: two, else one)
bool fq_gemv_can_stream(int M, int K, int bits, int inputs);
// Once per device: raises the streaming kernels' LDS limit and learns their residency (idempotent).
int fq_gemv_prepare();
int fq_launch_gemv_multi(const fq_gemv_input &src, int M, const fq_packed_ref *w, void *const *outs, int count,
                         fq_stream st);
// Persistent decode kernel (M = 1): the whole stack in one launch per sixteen blocks.  Buffers are fp16
// vectors in the caller's workspace (q, k, v, o, d, x1 hidden wide; g, p ffn wide) and 4 KiB for the
// barrier counters.  fq_launch_decode_persist returns 0 once queued, -1 when the kernel does not apply (the
// caller queues the per-phase launches instead), else a hipError_t.  Without may_allocate nothing is set up
// on a device that fq_decode_prepare has not seen (the preparation pins a word of host memory).
struct fq_decode_buffers {
    void *q, *k, *v, *o, *g, *p, *d, *x1, *sync;
};
constexpr size_t fq_decode_sync_bytes = 4096;
int fq_decode_prepare();
int fq_launch_decode_persist(const fq_layer *layers, int L, const uint8_t *bitvec, int H, int F, const void *x_in,
                             void *x_out, const fq_decode_buffers &b, bool may_allocate, fq_stream st);
bool fq_decode_async_error();        // a decode kernel has given up at its grid barrier on this device
void fq_decode_clear_async_error();
unsigned long long fq_decode_set_give_up_ticks(unsigned long long ticks); // returns the previous bound
int fq_decode_set_mode(int mode);    // 0: per-phase launches (default), 1: persistent kernel where it applies; returns the previous
unsigned long long fq_decode_launches(); // persistent launches queued by this process so far
int fq_decode_available(int H, int F); // pages per ring if the persistent kernel would run, else 0
void fq_decode_partition_of(unsigned bits4, int ph, int N, int wg, int grid, int *out6);
// M > 16.  tile_rows: 0 lets the library choose between the 128-row and the 256-row tile kernels, 128 or 256 pins one.
int fq_launch_gemm(const void *x, int M, const fq_packed_ref &w, void *out, fq_stream st, int tile_rows = 0);
// Up to three matrices with the same input (same K) in one launch, M > 16.
int fq_launch_gemm_multi(const void *x, int M, const fq_packed_ref *w, void *const *outs, int count, fq_stream st,
                         int tile_rows = 0);
int fq_launch_dense(const void *x, int M, const void *W, int N, int K, void *out, fq_stream st);
// The same product with 256 x 256 tiles, both operands through LDS; pays once its tiles fill the chip.
bool fq_dense_tiled_pays(int M, int N);
int fq_launch_dense_tiled(const void *x, int M, const void *W, int N, int K, void *out, fq_stream st);
// Head GEMM with the token loss in its epilogue; workspace of fq_head_nll_scratch_bytes(M, V) bytes.
size_t fq_head_nll_scratch_bytes(int M, int V);
int fq_launch_head_nll(const void *x, int M, const void *W, int V, int K, const int32_t *labels, float *nll,
                       void *workspace, fq_stream st);
// Attention of one decode step (head dimension 128): rotary embedding of q and k, cache append, softmax over
// the cached positions; caches [heads][Tmax][128].  Workspace of fq_attn_scratch_bytes(Tmax, n_heads) bytes.
size_t fq_attn_scratch_bytes(int Tmax, int n_heads);
int fq_attn_max_positions(); // largest Tmax the merge of the splits handles
int fq_launch_attn_decode(const void *q, const void *k, const void *v, void *k_cache, void *v_cache, int pos,
                          int Tmax, int n_heads, const float *rope, void *out, void *workspace, fq_stream st);
// Causal attention over positions 0..T-1 of one sequence: rotates q and k, fills the caches, writes out
// [T,H].  Workspace of fq_attn_prefill_scratch_bytes(T, n_heads) bytes.
size_t fq_attn_prefill_scratch_bytes(int T, int n_heads);
int fq_launch_attn_prefill(const void *q, const void *k, const void *v, int T, void *k_cache, void *v_cache,
                           int Tmax, int n_heads, const float *rope, void *out, void *workspace, fq_stream st);
int fq_launch_glue(int op, const void *a, const void *b, const void *c, int M, int H, void *out, fq_stream st);
// Two steps in one pass: op 6: aux = a + b, out = rms(aux); op 7: aux = rms(a + b), out = rms(aux).
int fq_launch_glue2(int op, const void *a, const void *b, int M, int H, void *aux, void *out, fq_stream st);
int fq_launch_nll(const void *logits, const int32_t *labels, int M, int V, float *nll, fq_stream st);
int fq_launch_logit_l2(const void *a, const void *b, int M, int V, float *dist, fq_stream st);
// Plain read of a buffer; one word per workgroup lands in sink[blocks].
int fq_launch_stream_read(const void *src, size_t bytes, uint32_t *sink, int blocks, fq_stream st);

#endif
