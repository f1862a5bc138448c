/*
 * libfq -- mixed-bit weight-only quantized linear layers and token NLL for
 * AMD MI355X (gfx950).
 *
 * The method served here is FlexQuant's hybrid model (arXiv 2501.07139): every
 * module takes its weights from one of several stored quantized models, so the
 * bit-width is a per-matrix choice made by a configuration vector (Section
 * "EQM Generation Philosophy"); arithmetic is FP16 whatever the weight
 * bit-width (Section "Large Language Model Quantization"); a candidate is
 * scored by perplexity over calibration token sequences (Algorithm 1,
 * calibrationEval) and served one token at a time (Section "Introduction").
 *
 * Conventions
 *   - Every function returns FQ_OK (0) or a negative FQ_ERR_* code, never
 *     throws and never allocates device memory.  fq_last_error() gives a
 *     thread-local message for the last failure on the calling thread.
 *   - "host" pointers are ordinary memory; "device" pointers are HIP device
 *     memory of the current device, 16-byte aligned, owned by the caller and
 *     only accessed by stream-ordered work queued by the call.
 *   - `stream` is a hipStream_t passed as void*; NULL means the default
 *     stream.  Device functions only enqueue work; they do not synchronise.
 *     The first device call on a device also prepares the library's kernels
 *     there (see fq_init): call fq_init() before capturing calls into a graph.
 *   - bits is one of 2, 3, 4, 8; group must be 128; K must be a multiple of
 *     128.  fp16 values cross the boundary as IEEE binary16 bit patterns.
 *
 * Packed weight format (device and host, little-endian)
 *   Rows are padded to Np = 64*ceil(N/64); pad rows hold code 0, scale 0.
 *   A supertile covers R rows by one group of 128 k, R = 32/64/16/16 for
 *   bits = 2/3/4/8, and takes R*16*bits bytes (1, 3, 1, 2 planes of 1024
 *   bytes).  Supertile (n/R, k/128) starts at byte
 *   ((n/R)*(K/128) + k/128) * R*16*bits.  Inside it, lane l = 16*c + r owns
 *   the dwords D[j] at byte (j/4)*1024 + 16*l + 4*(j%4): one 128-bit load per
 *   lane per plane, 1024 contiguous bytes per wavefront.
 *   With n % R = 16*u + r and k % 128 = 32*s + 8*c + e (t = 8*s + e), the
 *   weight's chunk is C[i] = D[bits*u + i], i < bits, and its code sits at
 *     bits 4:  C[s],         bit offset 16*(e%2) + 4*(e/2)
 *     bits 8:  C[2*s + e/4], bit offset 16*(e%2) + 8*((e%4)/2)
 *     bits 2:  C[s/2],       bit offset 16*(e%2) + 2*(4*(s%2) + e/2)
 *     bits 3:  t < 30: C[t/10], bit offset 16*(t%2) + 3*((t%10)/2);
 *              t = 30: code bit i is bit 15 of C[i]; t = 31: bit 31 of C[i].
 *   (r, c, s, e) are the row, lane slice, k-step and element of a 16x16x32
 *   matrix-core operand, so a lane's chunk unpacks straight into operands.
 *   Scales and zeros are fp16 arrays of Np*(K/128) entries in tile order:
 *   entry (n, g) is element (n/16)*(K/128)*16 + g*16 + n%16.
 *   The reconstruction is  w = scale * (code - zero): zeros are in code units.
 */
#ifndef FQ_H
#define FQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FQ_OK 0
#define FQ_ERR_NULL (-1)      /* a required pointer is NULL */
#define FQ_ERR_SHAPE (-2)     /* a size is non-positive or K is not a multiple of 128 */
#define FQ_ERR_BITS (-3)      /* bits not in {2,3,4,8} */
#define FQ_ERR_GROUP (-4)     /* group != 128 */
#define FQ_ERR_ALIGN (-5)     /* a device pointer is not 16-byte aligned */
#define FQ_ERR_WORKSPACE (-6) /* workspace too small */
#define FQ_ERR_HIP (-7)       /* a HIP call or kernel launch failed */

/* Message for the last error returned on this thread ("" if none).  Host. */
const char *fq_last_error(void);

/* Library version string.  Host. */
const char *fq_version(void);

/*
 * Prepare the library on the current device: raise the LDS limit of the decode
 * kernels and learn how many of their workgroups the device keeps resident.
 * Idempotent and thread-safe; once per device.  Every device function does this
 * by itself on its first call on a device, which is not something a stream
 * capture may contain: a caller that captures graphs calls fq_init() first,
 * with the device current.  FQ_ERR_HIP if the runtime refuses.
 */
int fq_init(void);

/* ------------------------------------------------------------------ host --- */

/*
 * Group-wise round-to-nearest asymmetric min-max quantization (the quantizer is
 * delegated by the paper, Section "Large Language Model Quantization"; this is
 * the plain one).  Per row and group of 128 consecutive k, in fp32:
 *   lo = min(0, min w), hi = max(0, max w);
 *   hi == lo: scale 1, zero 0, codes 0; otherwise
 *   scale = fp16((hi - lo) / (2^bits - 1)), raised to the smallest normal fp16
 *   if zero or subnormal; zero = clamp(rne(-lo / scale), 0, 2^bits - 1);
 *   code = clamp(rne(w / scale) + zero, 0, 2^bits - 1); rne = half-to-even.
 * W fp32 [N,K] row-major (host, read).  codes u8 [N,K], scales and zeros fp16
 * [N, K/128] row-major (host, written).  Multi-threaded over rows.
 */
int fq_quantize_rtn(const float *W, int N, int K, int bits, int group,
                    uint8_t *codes, uint16_t *scales, uint16_t *zeros);

/*
 * Bytes of the packed buffer for an [N,K] matrix: 64*ceil(N/64) * K * bits / 8,
 * i.e. exactly `bits` bits per weight (the footprint a module of QM(bits) adds to
 * a hybrid model, Section "EQM Generation Philosophy").  0 on bad arguments.
 */
size_t fq_packed_bytes(int N, int K, int bits);

/* Entries of each tiled scale/zero array: 64*ceil(N/64) * K/128.  0 on bad arguments. */
size_t fq_meta_count(int N, int K, int group);

/*
 * Pack codes and lay scales/zeros out in the device format described above: one
 * stored form per matrix and bit-width, the "parameters of QM(n)" a hybrid model
 * draws from (Section "EQM Generation Philosophy").
 * codes u8 [N,K] (values < 2^bits, else FQ_ERR_BITS), scales/zeros fp16
 * [N,K/128] row-major: host, read.  packed_out (fq_packed_bytes bytes),
 * scales_out and zeros_out (fq_meta_count entries each): host, written, pad
 * included.  The caller copies the three outputs to the device unchanged.
 */
int fq_pack_groups(const uint8_t *codes, const uint16_t *scales, const uint16_t *zeros,
                   int N, int K, int bits, int group,
                   void *packed_out, uint16_t *scales_out, uint16_t *zeros_out);

/* ---------------------------------------------------------------- device --- */

/*
 * The n-bit layer as the numerical approximation of its FP16 counterpart that
 * Section "FlexQuant Framework" reasons about, written out: dequantize a packed
 * matrix to a dense row-major [N,K] array: fp32
 * (out_is_fp16 == 0): float(scale) * (float(code) - float(zero)), each step
 * rounded to fp32; or fp16: that value rounded once.  For parity checks.
 * packed, scales, zeros: device, read.  out: device, written.
 */
int fq_dequant(const void *packed, const void *scales, const void *zeros,
               int N, int K, int bits, int group, void *out, int out_is_fp16, void *stream);

/*
 * The quantized linear layer of a hybrid model:
 *   out[m,n] = sum_k x[m,k] * scale[n,k/128] * (code[n,k] - zero[n,k/128]),
 * fp16 inputs, fp32 accumulation, fp16 output (one rounding).  x fp16 [M,K]
 * row-major and the packed triple: device, read.  out fp16 [M,N] row-major:
 * device, written.  M <= 16 runs the bandwidth-bound streaming kernel (decode),
 * larger M the matrix-core tile kernel (calibration forward).  Any M >= 1,
 * N >= 1.  Scales and zeros may be any finite fp16 (e.g. zero/2^d after
 * truncating d code bits, Section "Elastic Serving").  For M > 16 the
 * activations (M*K*2 bytes) and the packed weights must each stay below
 * 4 GiB, else FQ_ERR_SHAPE.  Two tile kernels exist for M > 16: 128 activation
 * rows per workgroup, and 256 rows per workgroup of eight wavefronts with the
 * k-steps of every group split over two wavefront sets (each unpacked weight
 * feeds twice as many matrix instructions); the library takes the 256-row tiles
 * once M > 128 and there is a tile for every compute unit, except from 4096 rows
 * on for 2- and 4-bit matrices wide enough for 128 x 256 tiles (as measured on
 * MI355X).
 * fq_qlinear_tile is the same call with the choice
 * made by the caller: tile_rows = 128 or 256 pins a kernel (any M > 16; for tests
 * and tuning; ignored for M <= 16), 0 leaves it to the library; anything else is
 * FQ_ERR_SHAPE.
 */
int fq_qlinear(const void *x, int M, const void *packed, const void *scales, const void *zeros,
               int N, int K, int bits, int group, void *out, void *stream);
int fq_qlinear_tile(const void *x, int M, const void *packed, const void *scales, const void *zeros,
                    int N, int K, int bits, int group, void *out, int tile_rows, void *stream);

/*
 * Mixed precision WITHIN a matrix (Section "Large Language Model Quantization":
 * the quantizers the paper builds on assign different bit-widths not only across
 * modules but within individual modules).  Here a matrix [N,K] is stored as up to
 * FQ_MAX_SEGMENTS runs of consecutive output rows, each run a packed triple of
 * its own bit-width over the same K, and
 *   out[m, n0_i + n] = fq_qlinear(x, segment i)[m, n],  n0_i = N_0 + ... + N_(i-1),
 * the same arithmetic as fq_qlinear per run; out fp16 [M, sum of N_i] row-major.
 * Runs that share a launch (three at a time) are dealt to the chip together, like
 * q/k/v in the stack forward.  Any M >= 1; every N_i >= 1 (no alignment needed:
 * each run is padded on its own); segments: host array, device pointers inside.
 * (The cited quantizers vary the width along the input dimension; this format
 * keeps a row's groups at one width, so the variation is along the output rows.)
 */
#define FQ_MAX_SEGMENTS 8
typedef struct {
    const void *packed, *scales, *zeros; /* device: the packed triple of this run of rows */
    int N;                               /* rows (output features) of the run */
    int bits;                            /* 2, 3, 4 or 8 */
} fq_segment;
int fq_qlinear_mixed(const void *x, int M, const fq_segment *segments, int count, int K, int group, void *out,
                     void *stream);

/* One matrix in all stored bit-widths; index 0..3 = bits 2, 3, 4, 8.  Unused widths may be NULL. */
typedef struct {
    const void *packed[4];
    const void *scales[4];
    const void *zeros[4];
    int N, K;
} fq_matrix;

/* The seven linears of a decoder block: q, k, v, o, gate, up, down. */
typedef struct {
    fq_matrix m[7];
} fq_layer;

/* Workspace bytes fq_stack_forward needs for M rows of a (hidden, ffn) stack. */
size_t fq_stack_workspace_bytes(int M, int hidden, int ffn);

/*
 * Forward M rows through L blocks whose matrix j of block l uses the packing
 * of bit-width bitvec[7*l + j] -- the configuration vector of a hybrid model
 * (Section "EQM Generation Philosophy").  Synthetic block, every named tensor
 * fp16, rms(t) = t / sqrt(mean(t^2) + 1e-5) per row:
 *   u = rms(x); q,k,v = Lq(u), Lk(u), Lv(u); a = rms(q+k+v); o = Lo(a);
 *   x1 = x + o; u2 = rms(x1); g,p = Lgate(u2), Lup(u2); m = rms(silu(g)*p);
 *   d = Ldown(m); x_next = rms(x1 + d).
 * layers: host array of L entries holding device pointers (read during the
 * call only).  bitvec: host, 7*L entries.  x_in fp16 [M,hidden]: device, read.
 * x_out fp16 [M,hidden]: device, written (may equal x_in).  workspace: device.
 * A NULL packing for a selected bit-width fails with FQ_ERR_NULL before any
 * launch.
 */
int fq_stack_forward(const fq_layer *layers, int L, const uint8_t *bitvec,
                     const void *x_in, int M, void *x_out,
                     void *workspace, size_t workspace_bytes, void *stream);

/*
 * fq_stack_forward for callers that cannot allocate or hold a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * computation and the same kernels, for M <= 16 rows and hidden, ffn <= 16384, with
 * the activations between the launches kept in a 6.5 MiB array that is part of the
 * library's device code (every GPU the library runs on holds it until the process
 * ends).  The call allocates nothing, on the device or through any library; larger
 * M or wider blocks are refused with FQ_ERR_SHAPE.  Every call on a GPU uses that
 * GPU's one array: calls that overlap in time on the same GPU (two streams, two
 * threads) race and must be serialised by the caller; nothing in the array has to
 * survive from one call to the next.  Call fq_init() first if the call is to be
 * captured.
 */
int fq_stack_forward_noalloc(const fq_layer *layers, int L, const uint8_t *bitvec,
                             const void *x_in, int M, void *x_out, void *stream);

/*
 * Decode path and its error reporting.  With M == 1 the stack forwards above can run
 * the whole stack in one persistent launch per sixteen blocks (hidden <= 8192, ffn
 * <= 16384): one workgroup per compute unit, all resident together, streaming the
 * packed weights through LDS rings that keep loading across the block's four
 * dependent phases, and meeting at a grid-wide barrier after each phase.
 *   fq_set_decode_mode(1) selects that kernel for M == 1 where it applies; mode 0,
 *     the default, runs the per-phase launches that also serve 2 <= M <= 16 (four
 *     launches per block).  The previous mode is returned.  Process-wide.  As
 *     measured on MI355X the per-phase launches are the faster of the two.
 * Every wait of the persistent kernel's barrier is bounded by a timer; a workgroup
 * that waits longer gives up, the launch still ends, its results are invalid, and
 * from then on fq_stack_forward and fq_stack_forward_noalloc return FQ_ERR_HIP (the
 * library does not synchronise, so the failure surfaces at the next call, as
 * fq_async_error() does at any time) until fq_clear_async_error() is called.
 *   fq_decode_give_up_ticks(t) sets the bound in ticks of the 100 MHz timer
 *     (default 2 s) and returns the previous one; 0 makes every wait give up at
 *     once, which is how the tests exercise the failure path.
 * The no-alloc variant runs the persistent kernel only after fq_init() on that
 * device (the preparation pins one word of host memory for the error report).
 */
int fq_set_decode_mode(int mode);
/* Non-zero (the depth of a wavefront's LDS ring in KiB) if, on the current device and after fq_init(), the
 * persistent kernel can serve M == 1 forwards through blocks of this size when mode 1 selects it; else 0. */
int fq_decode_persistent(int hidden, int ffn);
/* Launches of the persistent kernel this process has queued so far (tests use it to see which path ran). */
unsigned long long fq_decode_persistent_launches(void);
unsigned long long fq_decode_give_up_ticks(unsigned long long ticks);
/*
 * How the persistent kernel deals a phase's work to its workgroups (host; for tests
 * and tools).  Phase 0..3 = q/k/v, o, gate/up, down of a block whose seven matrices
 * have the bit-widths bits7 (host, 7 entries); N = rows of the phase's matrices.  A
 * work unit is a supertile row (32/64/16/16 weight rows at 2/3/4/8 bits); every
 * matrix of the phase is cut into `grid` contiguous runs of nearly equal length,
 * the odd matrices dealt in reverse workgroup order.  units_out (host, 6 ints)
 * receives [first, end) of workgroup wg's units in each of the phase's (up to
 * three) matrices; unused pairs are 0, 0.
 */
int fq_decode_partition(const uint8_t *bits7, int phase, int N, int wg, int grid, int *units_out);
int fq_async_error(void);
void fq_clear_async_error(void);

/* Single glue steps of the block above, exposed for layer-by-layer parity checks.
 * All tensors fp16 [M,H] row-major on the device; b and c may be NULL where unused.
 *   op 0: out = rms(a)              op 1: out = rms(a + b + c)
 *   op 2: out = a + b               op 3: out = rms(silu(a) * b)
 *   op 4: out = rms(a + b)          op 5: out = silu(a) * b (no norm: real decoder blocks)
 */
int fq_glue(int op, const void *a, const void *b, const void *c, int M, int H, void *out, void *stream);

/*
 * Unquantized fp16 linear: out[m,n] = sum_k x[m,k] W[n,k], fp32 accumulation,
 * fp16 output.  It is the vocabulary head whose logits calibrationEval
 * (Algorithm 1) turns into a perplexity and the sensitivity analysis (Section
 * "Efficient Design Space Navigation") compares; the head is not quantized.
 * x [M,K], W [N,K], out [M,N] row-major, device.  K must be a multiple of 128;
 * x and W must each stay below 4 GiB (FQ_ERR_SHAPE otherwise).  Two kernels serve
 * it: 128-row tiles, and 256-row tiles with both operands in LDS once those fill
 * the chip.  fq_dense_f16_tile is the same call with the choice made by the
 * caller: tile_rows = 128 or 256 pins a kernel (any size; for tests and tuning),
 * 0 leaves it to the library; anything else is FQ_ERR_SHAPE.
 */
int fq_dense_f16(const void *x, int M, const void *W, int N, int K, void *out, void *stream);
int fq_dense_f16_tile(const void *x, int M, const void *W, int N, int K, void *out, int tile_rows, void *stream);

/*
 * Fused log-softmax cross-entropy per token (the quantity whose mean,
 * exponentiated, is the perplexity calibrationEval returns in Algorithm 1):
 *   nll[m] = log(sum_v exp(l[m,v] - max_v l[m,v])) + max_v l[m,v] - l[m,label[m]].
 * logits fp16 [M,V] row-major, labels int32 [M]: device, read.  nll fp32 [M]:
 * device, written.  A label outside [0,V) marks an ignored position (nll 0).
 * One pass over the logits.
 */
int fq_token_nll(const void *logits, const int32_t *labels, int M, int V, float *nll_out, void *stream);

/*
 * The two steps above in one: token losses of the head's logits without storing
 * the logits (calibrationEval of Algorithm 1 needs only the losses),
 *   nll[m] = fq_token_nll(round_fp16(fq_dense_f16(x, W)), labels)[m],
 * the logits rounded to fp16 exactly as fq_dense_f16 would store them.  Every
 * workgroup of the GEMM reduces its tile of logits to one (maximum, sum of
 * exponentials) pair per row and 64 columns; a second kernel merges the pairs.
 * x fp16 [M,K], W fp16 [V,K], labels int32 [M]: device, read.  nll fp32 [M]:
 * device, written.  workspace: device scratch of at least
 * fq_head_nll_workspace_bytes(M, V) bytes, 16-byte aligned, owned by the caller,
 * contents undefined afterwards (FQ_ERR_WORKSPACE if NULL or too small).
 * K a multiple of 128; x and W below 4 GiB each (FQ_ERR_SHAPE).  Always runs the
 * 256-row tiles: meant for M * V large enough to fill the chip.
 */
size_t fq_head_nll_workspace_bytes(int M, int V);
int fq_head_nll(const void *x, int M, const void *W, int V, int K, const int32_t *labels, float *nll_out,
                void *workspace, size_t workspace_bytes, void *stream);

/*
 * Row-wise Euclidean distance between two sets of logits (Section "Efficient
 * Design Space Navigation": the sensitivity value of a module is the Euclidean distance between
 * the logits of the hybrid model with that module lowered and those of
 * QM(n_up)):  dist[m] = sqrt(sum_v (a[m,v] - b[m,v])^2), differences, squares
 * and the sum in fp32.  a, b fp16 [M,V] row-major: device, read, 16-byte
 * aligned.  dist fp32 [M]: device, written.  The distance over a batch of rows
 * is sqrt(sum_m dist[m]^2).  One pass over both arrays.
 */
int fq_logit_l2(const void *a, const void *b, int M, int V, float *dist_out, void *stream);

/*
 * Measurement aid, not a step of the method: reads `bytes` of device memory once
 * (128-bit loads, nothing else) and leaves FQ_STREAM_READ_WORDS checksum words in
 * sink.  Timing it gives the rate a pure read reaches on the device, the
 * practical ceiling for the decode path, which streams every packed weight once
 * per token (Section "Introduction").  src: device, 16-byte aligned, bytes a
 * positive multiple of 16.  sink: device, FQ_STREAM_READ_WORDS uint32, written.
 */
#define FQ_STREAM_READ_WORDS 2048
int fq_stream_read(const void *src, size_t bytes, uint32_t *sink, void *stream);

/*
 * Real decoder blocks around the quantized linears, one decode step (the hosted
 * models of Section "Experiment" are Llama decoders; Section "Introduction":
 * served one token at a time).  Per block, for the token at position pos:
 *   u = rms(x); q,k,v = L(u); q' = rope(q,pos), k' = rope(k,pos);
 *   K[pos] = k', V[pos] = v; a = softmax_t(q'.K[t]/sqrt(128)).V[t], t <= pos, per head;
 *   o = Lo(a); x1 = x + o; u2 = rms(x1); g,p = Lgate(u2),Lup(u2);
 *   d = Ldown(silu(g)*p); x_next = x1 + d.
 * rms(t) = t/sqrt(mean(t^2)+1e-5) without gain (a model's norm gains are folded
 * into the following linears before quantization); rope rotates the adjacent
 * pair (2i, 2i+1) of every head by the angle whose (cos, sin) the table gives;
 * heads are 128 wide, as many key/value heads as query heads; every named tensor
 * is stored as fp16.
 *
 * fq_attn_decode: the attention step alone.  q, k, v fp16 [H] (H = 128 n_heads),
 * device, read.  k_cache, v_cache fp16 [n_heads][Tmax][128] (head-major: a
 * head's positions are contiguous), device: positions < pos read, position pos
 * written.  rope fp32 [Tmax][64][2] = (cos, sin) of pos * theta_i, device, read.
 * out fp16 [H], device, written.  workspace: device scratch of at least
 * fq_attn_workspace_bytes(Tmax, n_heads) bytes, 16-byte aligned, owned by the
 * caller.  FQ_ERR_SHAPE unless 0 <= pos < Tmax <= 131072.
 *
 * fq_decode_step: L blocks.  layers/bitvec as in fq_stack_forward.  x_in, x_out
 * fp16 [hidden], device.  k_cache, v_cache fp16 [L][n_heads][Tmax][128], device,
 * layer l at offset l*Tmax*hidden.  workspace of fq_decode_workspace_bytes(hidden, ffn,
 * Tmax) bytes, 16-byte aligned.  Six launches per block (q/k/v, attention and
 * its merge when pos >= 128, o, gate/up, down), all on `stream`; positions must
 * be fed in order 0, 1, 2, ... for the cache to be complete.
 *
 * fq_attn_prefill / fq_prefill_forward: the same blocks over a whole sequence, rows
 * 0..T-1 of x at positions 0..T-1 (causal attention; Algorithm 1's calibrationEval on
 * real blocks, and the way to fill the caches before decoding).  q, k, v, out and
 * x_in, x_out are fp16 [T,H] row-major; the caches as above, positions 0..T-1
 * written; workspace of fq_attn_prefill_workspace_bytes(T, n_heads) respectively
 * fq_prefill_workspace_bytes(T, hidden, ffn) bytes.  FQ_ERR_SHAPE unless
 * 0 < T <= Tmax <= 131072.
 */
/*
 * fq_rope_table: the (cos, sin) table the calls below take, for positions
 * 0..Tmax-1: out[t][i] = (cos, sin)(t * base^(-2i/head_dim)), i < head_dim/2,
 * evaluated in fp64 and rounded once to fp32.  out: host, Tmax*head_dim floats,
 * written; the caller copies it to the device.  FQ_ERR_SHAPE unless Tmax > 0,
 * head_dim even and positive, base > 0.
 */
int fq_rope_table(int Tmax, int head_dim, double base, float *out);
size_t fq_attn_workspace_bytes(int Tmax, int n_heads);
size_t fq_decode_workspace_bytes(int hidden, int ffn, int Tmax);
int fq_attn_decode(const void *q, const void *k, const void *v, void *k_cache, void *v_cache, int pos, int Tmax,
                   int n_heads, const float *rope, void *out, void *workspace, size_t workspace_bytes, void *stream);
int fq_decode_step(const fq_layer *layers, int L, const uint8_t *bitvec, const void *x_in, void *x_out,
                   void *k_cache, void *v_cache, int pos, int Tmax, const float *rope, void *workspace,
                   size_t workspace_bytes, void *stream);
size_t fq_attn_prefill_workspace_bytes(int T, int n_heads);
size_t fq_prefill_workspace_bytes(int T, int hidden, int ffn);
int fq_attn_prefill(const void *q, const void *k, const void *v, int T, void *k_cache, void *v_cache, int Tmax,
                    int n_heads, const float *rope, void *out, void *workspace, size_t workspace_bytes, void *stream);
int fq_prefill_forward(const fq_layer *layers, int L, const uint8_t *bitvec, const void *x_in, int T, void *x_out,
                       void *k_cache, void *v_cache, int Tmax, const float *rope, void *workspace,
                       size_t workspace_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* FQ_H */
