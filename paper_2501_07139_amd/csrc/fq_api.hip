// C-ABI entry points of the device half: argument checks, dispatch, and the
// block/stack driver that applies a hybrid model's configuration vector
// (FlexQuant, arXiv 2501.07139, Section "EQM Generation Philosophy": each
// module takes its parameters from one stored quantized model).
#include "fq.h"
#include "fq_internal.h"

#include <hip/hip_runtime.h>

#include <mutex>

// Scratch of the entry point that must not allocate (fq_stack_forward_noalloc): the activations of a decode
// stack forward for up to 16 rows of up to 16384 elements.  Every device the library runs on holds its own
// copy of this array until the process ends.  In host code the array's name is only a handle: the device
// address comes from hipGetSymbolAddress (static_scratch below) and is what kernels and copies are given.
constexpr int kNoallocMaxM = 16, kNoallocMaxDim = 16384;
constexpr size_t kNoallocScratchBytes = (size_t)13 * kNoallocMaxM * kNoallocMaxDim * 2 + fq_decode_sync_bytes;
static __device__ __align__(256) unsigned char scratch[kNoallocScratchBytes];

namespace {

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_hip(int e, const char *what)
{
    if (e == 0)
        return FQ_OK;
    return fq_fail(FQ_ERR_HIP, "%s: %s", what, hipGetErrorString((hipError_t)e));
}

int check_matrix(const char *fn, const void *packed, const void *scales, const void *zeros, int N, int K,
                 int bits, int group)
{
    if (!packed || !scales || !zeros)
        return fq_fail(FQ_ERR_NULL, "%s: NULL weight pointer", fn);
    if (fq_bits_index(bits) < 0)
        return fq_fail(FQ_ERR_BITS, "%s: bits=%d not in {2,3,4,8}", fn, bits);
    if (group != 128)
        return fq_fail(FQ_ERR_GROUP, "%s: group=%d, only 128 is supported", fn, group);
    if (N <= 0 || K <= 0 || K % 128 != 0)
        return fq_fail(FQ_ERR_SHAPE, "%s: N=%d K=%d (K must be a positive multiple of 128)", fn, N, K);
    if (!aligned16(packed) || !aligned16(scales) || !aligned16(zeros))
        return fq_fail(FQ_ERR_ALIGN, "%s: weight pointers must be 16-byte aligned", fn);
    return FQ_OK;
}

// The M > 16 kernels address each array through 32-bit byte offsets.
bool below_4gib(size_t a, size_t b, size_t elem_bytes) { return a * b * elem_bytes < ((size_t)1 << 32); }

int qlinear_checked(const void *x, int M, const fq_packed_ref &w, void *out, fq_stream st, int tile_rows = 0)
{
    if (M > 16 && (!below_4gib(M, w.K, 2) || !below_4gib(((size_t)w.N + 63) / 64 * 8, w.K, w.bits)))
        return fq_fail(FQ_ERR_SHAPE, "fq_qlinear: M=%d N=%d K=%d: activations and packed weights must each stay "
                       "below 4 GiB", M, w.N, w.K);
    int e = (M <= 16) ? fq_launch_gemv(x, M, w, out, st) : fq_launch_gemm(x, M, w, out, st, tile_rows);
    return check_hip(e, "fq_qlinear launch");
}

// M > 16: the linears that share an input (q/k/v, gate/up) in one launch.
int qlinear_multi_checked(const void *x, int M, const fq_packed_ref *w, void *const *outs, int count, fq_stream st)
{
    for (int i = 0; i < count; ++i)
        if (!below_4gib(M, w[i].K, 2) || !below_4gib(((size_t)w[i].N + 63) / 64 * 8, w[i].K, w[i].bits))
            return fq_fail(FQ_ERR_SHAPE, "fq_stack_forward: M=%d N=%d K=%d: activations and packed weights must each "
                           "stay below 4 GiB", M, w[i].N, w[i].K);
    return check_hip(fq_launch_gemm_multi(x, M, w, outs, count, st), "fq_stack_forward linears");
}

constexpr int kMaxGlueH = 16384;

size_t align_up(size_t v) { return (v + 255) & ~(size_t)255; }

// Device address of `scratch` on the current device, looked up once per device with that device current.
int static_scratch(void **out)
{
    static void *ptr[16] = {};
    static std::mutex guard;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess)
        return (int)e;
    if (dev < 0 || dev >= 16)
        return (int)hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(guard);
    if (!ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess)
            return (int)e;
        if (!p)
            return (int)hipErrorInvalidSymbol;
        ptr[dev] = p;
    }
    *out = ptr[dev];
    return 0;
}

} // namespace

extern "C" int fq_dequant(const void *packed, const void *scales, const void *zeros, int N, int K, int bits,
                          int group, void *out, int out_is_fp16, void *stream)
{
    if (int rc = check_matrix("fq_dequant", packed, scales, zeros, N, K, bits, group))
        return rc;
    if (!out)
        return fq_fail(FQ_ERR_NULL, "fq_dequant: NULL output");
    fq_packed_ref w{packed, scales, zeros, N, K, bits};
    return check_hip(fq_launch_dequant(w, out, out_is_fp16, static_cast<fq_stream>(stream)), "fq_dequant launch");
}

extern "C" int fq_qlinear(const void *x, int M, const void *packed, const void *scales, const void *zeros,
                          int N, int K, int bits, int group, void *out, void *stream)
{
    return fq_qlinear_tile(x, M, packed, scales, zeros, N, K, bits, group, out, 0, stream);
}

extern "C" int fq_qlinear_tile(const void *x, int M, const void *packed, const void *scales, const void *zeros,
                               int N, int K, int bits, int group, void *out, int tile_rows, void *stream)
{
    if (tile_rows != 0 && tile_rows != 128 && tile_rows != 256)
        return fq_fail(FQ_ERR_SHAPE, "fq_qlinear_tile: tile_rows=%d (0, 128 or 256)", tile_rows);
    if (int rc = check_matrix("fq_qlinear", packed, scales, zeros, N, K, bits, group))
        return rc;
    if (!x || !out)
        return fq_fail(FQ_ERR_NULL, "fq_qlinear: NULL activation or output pointer");
    if (M <= 0)
        return fq_fail(FQ_ERR_SHAPE, "fq_qlinear: M=%d", M);
    if (!aligned16(x) || !aligned16(out))
        return fq_fail(FQ_ERR_ALIGN, "fq_qlinear: x and out must be 16-byte aligned");
    fq_packed_ref w{packed, scales, zeros, N, K, bits};
    return qlinear_checked(x, M, w, out, static_cast<fq_stream>(stream), tile_rows);
}

extern "C" int fq_qlinear_mixed(const void *x, int M, const fq_segment *segments, int count, int K, int group,
                                void *out, void *stream)
{
    if (!segments || !x || !out)
        return fq_fail(FQ_ERR_NULL, "fq_qlinear_mixed: NULL argument");
    if (count < 1 || count > FQ_MAX_SEGMENTS)
        return fq_fail(FQ_ERR_SHAPE, "fq_qlinear_mixed: %d segments (1..%d)", count, FQ_MAX_SEGMENTS);
    if (M <= 0)
        return fq_fail(FQ_ERR_SHAPE, "fq_qlinear_mixed: M=%d", M);
    if (!aligned16(x) || !aligned16(out))
        return fq_fail(FQ_ERR_ALIGN, "fq_qlinear_mixed: x and out must be 16-byte aligned");
    long total = 0;
    for (int i = 0; i < count; ++i) {
        const fq_segment &sg = segments[i];
        if (int rc = check_matrix("fq_qlinear_mixed", sg.packed, sg.scales, sg.zeros, sg.N, K, sg.bits, group))
            return rc;
        if (M > 16 && (!below_4gib(M, K, 2) || !below_4gib(((size_t)sg.N + 63) / 64 * 8, K, sg.bits)))
            return fq_fail(FQ_ERR_SHAPE, "fq_qlinear_mixed: M=%d N=%d K=%d: activations and packed weights must each "
                           "stay below 4 GiB", M, sg.N, K);
        total += sg.N;
    }
    if (total > (1L << 30))
        return fq_fail(FQ_ERR_SHAPE, "fq_qlinear_mixed: %ld output columns", total);
    fq_stream st = static_cast<fq_stream>(stream);
    fq_packed_ref w[FQ_MAX_SEGMENTS];
    void *outs[FQ_MAX_SEGMENTS];
    bool stream_all = M <= 16;
    long col = 0;
    for (int i = 0; i < count; ++i) {
        w[i] = fq_packed_ref{segments[i].packed, segments[i].scales, segments[i].zeros, segments[i].N, K,
                             segments[i].bits, (int)total};
        outs[i] = static_cast<_Float16 *>(out) + col; // row 0 of the segment's column range; rows are `total` apart
        col += segments[i].N;
        stream_all = stream_all && fq_gemv_can_stream(M, K, segments[i].bits, 1);
    }
    // up to three segments share a launch (they share x): the same multi-matrix launches q/k/v and gate/up use
    for (int i = 0; i < count; i += 3) {
        const int n = count - i < 3 ? count - i : 3;
        int e = 0;
        if (M > 16)
            e = fq_launch_gemm_multi(x, M, &w[i], &outs[i], n, st);
        else if (stream_all)
            e = fq_launch_gemv_multi(fq_gemv_input{x, nullptr, nullptr, nullptr, 0}, M, &w[i], &outs[i], n, st);
        else
            for (int j = i; j < i + n && e == 0; ++j)
                e = fq_launch_gemv(x, M, w[j], outs[j], st);
        if (int rc = check_hip(e, "fq_qlinear_mixed launch"))
            return rc;
    }
    return FQ_OK;
}

extern "C" int fq_init(void)
{
    if (int rc = check_hip(fq_gemv_prepare(), "fq_init"))
        return rc;
    if (int rc = check_hip(fq_decode_prepare(), "fq_init: decode kernel"))
        return rc;
    void *p = nullptr;
    return check_hip(static_scratch(&p), "fq_init: static scratch");
}

extern "C" int fq_dense_f16(const void *x, int M, const void *W, int N, int K, void *out, void *stream)
{
    return fq_dense_f16_tile(x, M, W, N, K, out, 0, stream);
}

extern "C" int fq_dense_f16_tile(const void *x, int M, const void *W, int N, int K, void *out, int tile_rows,
                                 void *stream)
{
    if (!x || !W || !out)
        return fq_fail(FQ_ERR_NULL, "fq_dense_f16: NULL argument");
    if (M <= 0 || N <= 0 || K <= 0 || K % 128 != 0)
        return fq_fail(FQ_ERR_SHAPE, "fq_dense_f16: M=%d N=%d K=%d (K must be a positive multiple of 128)", M, N, K);
    if (!aligned16(x) || !aligned16(W) || !aligned16(out))
        return fq_fail(FQ_ERR_ALIGN, "fq_dense_f16: pointers must be 16-byte aligned");
    if (!below_4gib(M, K, 2) || !below_4gib(N, K, 2))
        return fq_fail(FQ_ERR_SHAPE, "fq_dense_f16: M=%d N=%d K=%d: x and W must each stay below 4 GiB", M, N, K);
    if (tile_rows != 0 && tile_rows != 128 && tile_rows != 256)
        return fq_fail(FQ_ERR_SHAPE, "fq_dense_f16_tile: tile_rows=%d not in {0, 128, 256}", tile_rows);
    const bool tiled = tile_rows ? tile_rows == 256 : fq_dense_tiled_pays(M, N);
    if (tiled)
        return check_hip(fq_launch_dense_tiled(x, M, W, N, K, out, static_cast<fq_stream>(stream)),
                         "fq_dense_f16 launch");
    return check_hip(fq_launch_dense(x, M, W, N, K, out, static_cast<fq_stream>(stream)), "fq_dense_f16 launch");
}

extern "C" int fq_glue(int op, const void *a, const void *b, const void *c, int M, int H, void *out, void *stream)
{
    if (op < 0 || op > 5)
        return fq_fail(FQ_ERR_SHAPE, "fq_glue: op=%d not in 0..5", op);
    if (!a || !out || (op != 0 && !b) || (op == 1 && !c))
        return fq_fail(FQ_ERR_NULL, "fq_glue: NULL argument for op %d", op);
    if (M <= 0 || H <= 0 || H % 8 != 0 || H > kMaxGlueH)
        return fq_fail(FQ_ERR_SHAPE, "fq_glue: M=%d H=%d (H must be a multiple of 8, at most %d)", M, H, kMaxGlueH);
    if (!aligned16(a) || !aligned16(out) || (b && !aligned16(b)) || (c && !aligned16(c)))
        return fq_fail(FQ_ERR_ALIGN, "fq_glue: pointers must be 16-byte aligned");
    return check_hip(fq_launch_glue(op, a, b, c, M, H, out, static_cast<fq_stream>(stream)), "fq_glue launch");
}

extern "C" int fq_token_nll(const void *logits, const int32_t *labels, int M, int V, float *nll_out, void *stream)
{
    if (!logits || !labels || !nll_out)
        return fq_fail(FQ_ERR_NULL, "fq_token_nll: NULL argument");
    if (M <= 0 || V <= 0)
        return fq_fail(FQ_ERR_SHAPE, "fq_token_nll: M=%d V=%d", M, V);
    if (!aligned16(logits))
        return fq_fail(FQ_ERR_ALIGN, "fq_token_nll: logits must be 16-byte aligned");
    return check_hip(fq_launch_nll(logits, labels, M, V, nll_out, static_cast<fq_stream>(stream)), "fq_token_nll launch");
}

extern "C" size_t fq_head_nll_workspace_bytes(int M, int V)
{
    if (M <= 0 || V <= 0)
        return 0;
    return (fq_head_nll_scratch_bytes(M, V) + 15) / 16 * 16;
}

extern "C" int fq_head_nll(const void *x, int M, const void *W, int V, int K, const int32_t *labels, float *nll_out,
                           void *workspace, size_t workspace_bytes, void *stream)
{
    if (!x || !W || !labels || !nll_out)
        return fq_fail(FQ_ERR_NULL, "fq_head_nll: NULL argument");
    if (M <= 0 || V <= 0 || K <= 0 || K % 128 != 0)
        return fq_fail(FQ_ERR_SHAPE, "fq_head_nll: M=%d V=%d K=%d (K must be a positive multiple of 128)", M, V, K);
    if (!below_4gib(M, K, 2) || !below_4gib(V, K, 2))
        return fq_fail(FQ_ERR_SHAPE, "fq_head_nll: M=%d V=%d K=%d: x and W must each stay below 4 GiB", M, V, K);
    if (!workspace || workspace_bytes < fq_head_nll_workspace_bytes(M, V))
        return fq_fail(FQ_ERR_WORKSPACE, "fq_head_nll: workspace of %zu bytes, need %zu", workspace ? workspace_bytes : 0,
                       fq_head_nll_workspace_bytes(M, V));
    if (!aligned16(x) || !aligned16(W) || !aligned16(workspace))
        return fq_fail(FQ_ERR_ALIGN, "fq_head_nll: x, W and workspace must be 16-byte aligned");
    return check_hip(fq_launch_head_nll(x, M, W, V, K, labels, nll_out, workspace, static_cast<fq_stream>(stream)),
                     "fq_head_nll launch");
}

extern "C" int fq_logit_l2(const void *a, const void *b, int M, int V, float *dist_out, void *stream)
{
    if (!a || !b || !dist_out)
        return fq_fail(FQ_ERR_NULL, "fq_logit_l2: NULL argument");
    if (M <= 0 || V <= 0)
        return fq_fail(FQ_ERR_SHAPE, "fq_logit_l2: M=%d V=%d", M, V);
    if (!aligned16(a) || !aligned16(b))
        return fq_fail(FQ_ERR_ALIGN, "fq_logit_l2: a and b must be 16-byte aligned");
    return check_hip(fq_launch_logit_l2(a, b, M, V, dist_out, static_cast<fq_stream>(stream)), "fq_logit_l2 launch");
}

extern "C" int fq_stream_read(const void *src, size_t bytes, uint32_t *sink, void *stream)
{
    if (!src || !sink)
        return fq_fail(FQ_ERR_NULL, "fq_stream_read: NULL argument");
    if (bytes == 0 || bytes % 16 != 0)
        return fq_fail(FQ_ERR_SHAPE, "fq_stream_read: %zu bytes (a positive multiple of 16)", bytes);
    if (!aligned16(src))
        return fq_fail(FQ_ERR_ALIGN, "fq_stream_read: src must be 16-byte aligned");
    return check_hip(fq_launch_stream_read(src, bytes, sink, FQ_STREAM_READ_WORDS, static_cast<fq_stream>(stream)),
                     "fq_stream_read launch");
}

// Shapes of the block's seven matrices and the selected packing of each, checked before anything is launched.
static int validate_layers(const char *fn, const fq_layer *layers, int L, const uint8_t *bitvec, int *H_out, int *F_out)
{
    const int H = layers[0].m[0].K, F = layers[0].m[4].N;
    if (H <= 0 || F <= 0 || H % 128 != 0 || F % 128 != 0 || H > kMaxGlueH || F > kMaxGlueH)
        return fq_fail(FQ_ERR_SHAPE, "%s: hidden=%d ffn=%d must be multiples of 128, at most %d", fn, H, F, kMaxGlueH);
    for (int l = 0; l < L; ++l)
        for (int j = 0; j < 7; ++j) {
            const fq_matrix &mx = layers[l].m[j];
            const int wantN = (j == 4 || j == 5) ? F : H, wantK = (j == 6) ? F : H;
            if (mx.N != wantN || mx.K != wantK)
                return fq_fail(FQ_ERR_SHAPE, "%s: layer %d matrix %d is %dx%d, expected %dx%d", fn, l, j, mx.N, mx.K,
                               wantN, wantK);
            const int bi = fq_bits_index(bitvec[7 * l + j]);
            if (bi < 0)
                return fq_fail(FQ_ERR_BITS, "%s: bitvec[%d]=%d not in {2,3,4,8}", fn, 7 * l + j, (int)bitvec[7 * l + j]);
            if (!mx.packed[bi] || !mx.scales[bi] || !mx.zeros[bi])
                return fq_fail(FQ_ERR_NULL, "%s: layer %d matrix %d has no %d-bit packing", fn, l, j,
                               (int)bitvec[7 * l + j]);
            if (!aligned16(mx.packed[bi]) || !aligned16(mx.scales[bi]) || !aligned16(mx.zeros[bi]))
                return fq_fail(FQ_ERR_ALIGN, "%s: layer %d matrix %d is not 16-byte aligned", fn, l, j);
        }
    *H_out = H;
    *F_out = F;
    return FQ_OK;
}

// Workspace: u, q, k, v, a, o, x1, u2, d, xcur (hidden wide), g, p, m (ffn wide), then the counters of the
// persistent decode kernel's grid barrier.
extern "C" size_t fq_stack_workspace_bytes(int M, int hidden, int ffn)
{
    if (M <= 0 || hidden <= 0 || ffn <= 0)
        return 0;
    const size_t h = align_up((size_t)M * hidden * 2), f = align_up((size_t)M * ffn * 2);
    return 10 * h + 3 * f + fq_decode_sync_bytes;
}

static const char kGaveUp[] = "an earlier decode kernel gave up waiting at its grid barrier (its results are invalid); "
                              "fq_clear_async_error() re-arms the library";

extern "C" int fq_set_decode_mode(int mode) { return fq_decode_set_mode(mode); }
extern "C" unsigned long long fq_decode_give_up_ticks(unsigned long long ticks) { return fq_decode_set_give_up_ticks(ticks); }
extern "C" int fq_decode_persistent(int hidden, int ffn) { return fq_decode_available(hidden, ffn); }
extern "C" unsigned long long fq_decode_persistent_launches(void) { return fq_decode_launches(); }
extern "C" int fq_async_error(void) { return fq_decode_async_error() ? FQ_ERR_HIP : FQ_OK; }
extern "C" void fq_clear_async_error(void) { fq_decode_clear_async_error(); }

extern "C" int fq_decode_partition(const uint8_t *bits7, int phase, int N, int wg, int grid, int *units_out)
{
    if (!bits7 || !units_out)
        return fq_fail(FQ_ERR_NULL, "fq_decode_partition: NULL argument");
    if (phase < 0 || phase > 3 || N <= 0 || grid <= 0 || wg < 0 || wg >= grid)
        return fq_fail(FQ_ERR_SHAPE, "fq_decode_partition: phase=%d N=%d wg=%d grid=%d", phase, N, wg, grid);
    unsigned bits4 = 0;
    for (int j = 0; j < 7; ++j) {
        if (fq_bits_index(bits7[j]) < 0)
            return fq_fail(FQ_ERR_BITS, "fq_decode_partition: bits=%d not in {2,3,4,8}", (int)bits7[j]);
        bits4 |= (unsigned)bits7[j] << (4 * j);
    }
    fq_decode_partition_of(bits4, phase, N, wg, grid, units_out);
    return FQ_OK;
}

static int stack_forward_checked(const fq_layer *layers, int L, const uint8_t *bitvec, const void *x_in, int M,
                                 void *x_out, void *workspace, int H, int F, bool may_allocate, fq_stream st);

extern "C" int fq_stack_forward(const fq_layer *layers, int L, const uint8_t *bitvec, const void *x_in, int M,
                                void *x_out, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!layers || !bitvec || !x_in || !x_out || !workspace)
        return fq_fail(FQ_ERR_NULL, "fq_stack_forward: NULL argument");
    if (L <= 0 || M <= 0)
        return fq_fail(FQ_ERR_SHAPE, "fq_stack_forward: L=%d M=%d", L, M);
    int H = 0, F = 0;
    if (int rc = validate_layers("fq_stack_forward", layers, L, bitvec, &H, &F))
        return rc;
    if (workspace_bytes < fq_stack_workspace_bytes(M, H, F))
        return fq_fail(FQ_ERR_WORKSPACE, "fq_stack_forward: workspace of %zu bytes, need %zu", workspace_bytes,
                       fq_stack_workspace_bytes(M, H, F));
    if (!aligned16(x_in) || !aligned16(x_out) || !aligned16(workspace))
        return fq_fail(FQ_ERR_ALIGN, "fq_stack_forward: x_in, x_out and workspace must be 16-byte aligned");
    if (fq_decode_async_error())
        return fq_fail(FQ_ERR_HIP, "fq_stack_forward: %s", kGaveUp);
    return stack_forward_checked(layers, L, bitvec, x_in, M, x_out, workspace, H, F, true, static_cast<fq_stream>(stream));
}

extern "C" int fq_stack_forward_noalloc(const fq_layer *layers, int L, const uint8_t *bitvec, const void *x_in, int M,
                                        void *x_out, void *stream)
{
    if (!layers || !bitvec || !x_in || !x_out)
        return fq_fail(FQ_ERR_NULL, "fq_stack_forward_noalloc: NULL argument");
    if (L <= 0 || M <= 0)
        return fq_fail(FQ_ERR_SHAPE, "fq_stack_forward_noalloc: L=%d M=%d", L, M);
    if (M > kNoallocMaxM)
        return fq_fail(FQ_ERR_SHAPE, "fq_stack_forward_noalloc: M=%d exceeds the %d rows the library's own scratch "
                       "holds; use fq_stack_forward with a workspace", M, kNoallocMaxM);
    int H = 0, F = 0;
    if (int rc = validate_layers("fq_stack_forward_noalloc", layers, L, bitvec, &H, &F))
        return rc;
    if (H > kNoallocMaxDim || F > kNoallocMaxDim || fq_stack_workspace_bytes(M, H, F) > kNoallocScratchBytes)
        return fq_fail(FQ_ERR_SHAPE, "fq_stack_forward_noalloc: hidden=%d ffn=%d exceed the %d elements per row the "
                       "library's own scratch holds; use fq_stack_forward with a workspace", H, F, kNoallocMaxDim);
    if (!aligned16(x_in) || !aligned16(x_out))
        return fq_fail(FQ_ERR_ALIGN, "fq_stack_forward_noalloc: x_in and x_out must be 16-byte aligned");
    void *ws = nullptr;
    if (int rc = check_hip(static_scratch(&ws), "fq_stack_forward_noalloc: static scratch"))
        return rc;
    if (fq_decode_async_error())
        return fq_fail(FQ_ERR_HIP, "fq_stack_forward_noalloc: %s", kGaveUp);
    return stack_forward_checked(layers, L, bitvec, x_in, M, x_out, ws, H, F, false, static_cast<fq_stream>(stream));
}

// The launches of a stack forward; every argument has been validated and the workspace holds
// fq_stack_workspace_bytes(M, H, F) bytes.
static int stack_forward_checked(const fq_layer *layers, int L, const uint8_t *bitvec, const void *x_in, int M,
                                 void *x_out, void *workspace, int H, int F, bool may_allocate, fq_stream st)
{
    fq_packed_ref sel[7];
    const size_t hb = align_up((size_t)M * H * 2), fb = align_up((size_t)M * F * 2);
    char *ws = static_cast<char *>(workspace);
    void *u = ws, *q = ws + hb, *k = ws + 2 * hb, *v = ws + 3 * hb, *a = ws + 4 * hb, *o = ws + 5 * hb,
         *x1 = ws + 6 * hb, *u2 = ws + 7 * hb, *d = ws + 8 * hb, *xc = ws + 9 * hb;
    void *g = ws + 10 * hb, *p = ws + 10 * hb + fb, *mm = ws + 10 * hb + 2 * fb;

    // One token: the whole stack in one persistent launch where that kernel applies.
    if (M == 1) {
        const fq_decode_buffers bufs = {q, k, v, o, g, p, d, x1, ws + 10 * hb + 3 * fb};
        const int e = fq_launch_decode_persist(layers, L, bitvec, H, F, x_in, x_out, bufs, may_allocate, st);
        if (e == 0)
            return FQ_OK;
        if (e > 0)
            return check_hip(e, "decode (persistent kernel)");
    }

    // Decode (M <= 16): four launches per block.  q/k/v and gate/up share a launch each, and every
    // row-wise step is folded into the input staging of the linear that consumes it.
    bool decode = M <= 16;
    for (int l = 0; l < L && decode; ++l)
        for (int j = 0; j < 7; ++j)
            decode = decode && fq_gemv_can_stream(M, layers[l].m[j].K, bitvec[7 * l + j], j == 3 ? 3 : 2);

    const void *xcur = x_in;
    for (int l = 0; l < L; ++l) {
        for (int j = 0; j < 7; ++j) {
            const fq_matrix &mx = layers[l].m[j];
            const int bits = bitvec[7 * l + j], bi = fq_bits_index(bits);
            sel[j] = fq_packed_ref{mx.packed[bi], mx.scales[bi], mx.zeros[bi], mx.N, mx.K, bits};
        }
        void *xnext = (l == L - 1) ? x_out : xc;
        void *const qkv[3] = {q, k, v};
        void *const gp[2] = {g, p};
        int rc;
#define FQ_STEP(call) \
    do { \
        if ((rc = (call)) != FQ_OK) \
            return rc; \
    } while (0)
        if (decode) {
            // the previous block's x_next = rms(x1 + d) is produced (into xc) by this block's first launch
            const fq_gemv_input in_qkv = (l == 0) ? fq_gemv_input{x_in, nullptr, nullptr, nullptr, 1}
                                                  : fq_gemv_input{x1, d, nullptr, xc, 5};
            if (l > 0)
                xcur = xc;
            FQ_STEP(check_hip(fq_launch_gemv_multi(in_qkv, M, &sel[0], qkv, 3, st), "decode q/k/v"));
            FQ_STEP(check_hip(fq_launch_gemv_multi(fq_gemv_input{q, k, v, nullptr, 2}, M, &sel[3], &o, 1, st),
                              "decode o"));
            FQ_STEP(check_hip(fq_launch_gemv_multi(fq_gemv_input{xcur, o, nullptr, x1, 3}, M, &sel[4], gp, 2, st),
                              "decode gate/up"));
            FQ_STEP(check_hip(fq_launch_gemv_multi(fq_gemv_input{g, p, nullptr, nullptr, 4}, M, &sel[6], &d, 1, st),
                              "decode down"));
            if (l == L - 1)
                FQ_STEP(check_hip(fq_launch_glue(4, x1, d, nullptr, M, H, x_out, st), "glue rms(add)"));
            continue;
        }
        // M > 16: the row-wise steps are kernels of their own, two of them per pass where one feeds the other
        // (the residual sum with the norm that reads it; a block's output with the next block's first norm)
        if (l == 0) {
            FQ_STEP(check_hip(fq_launch_glue(0, xcur, nullptr, nullptr, M, H, u, st), "glue rms"));
        }
        FQ_STEP(qlinear_multi_checked(u, M, &sel[0], qkv, 3, st));
        FQ_STEP(check_hip(fq_launch_glue(1, q, k, v, M, H, a, st), "glue rms(q+k+v)"));
        FQ_STEP(qlinear_checked(a, M, sel[3], o, st));
        FQ_STEP(check_hip(fq_launch_glue2(6, xcur, o, M, H, x1, u2, st), "glue add, rms"));
        FQ_STEP(qlinear_multi_checked(u2, M, &sel[4], gp, 2, st));
        FQ_STEP(check_hip(fq_launch_glue(3, g, p, nullptr, M, F, mm, st), "glue rms(silu*mul)"));
        FQ_STEP(qlinear_checked(mm, M, sel[6], d, st));
        if (l == L - 1) {
            FQ_STEP(check_hip(fq_launch_glue(4, x1, d, nullptr, M, H, xnext, st), "glue rms(add)"));
        } else {
            FQ_STEP(check_hip(fq_launch_glue2(7, x1, d, M, H, xnext, u, st), "glue rms(add), rms"));
        }
#undef FQ_STEP
        xcur = xnext;
    }
    return FQ_OK;
}

// Workspace: q, k, v, a, o, x1, d, x (hidden wide), g, p (ffn wide), then the attention's split results.
extern "C" size_t fq_decode_workspace_bytes(int hidden, int ffn, int Tmax)
{
    if (hidden <= 0 || ffn <= 0 || Tmax <= 0 || hidden % 128 != 0)
        return 0;
    return 8 * align_up((size_t)hidden * 2) + 2 * align_up((size_t)ffn * 2) + align_up(fq_attn_scratch_bytes(Tmax, hidden / 128));
}

extern "C" size_t fq_attn_workspace_bytes(int Tmax, int n_heads)
{
    if (Tmax <= 0 || n_heads <= 0)
        return 0;
    return align_up(fq_attn_scratch_bytes(Tmax, n_heads));
}

extern "C" int fq_attn_decode(const void *q, const void *k, const void *v, void *k_cache, void *v_cache, int pos,
                              int Tmax, int n_heads, const float *rope, void *out, void *workspace,
                              size_t workspace_bytes, void *stream)
{
    if (!q || !k || !v || !k_cache || !v_cache || !rope || !out || !workspace)
        return fq_fail(FQ_ERR_NULL, "fq_attn_decode: NULL argument");
    if (n_heads <= 0 || Tmax <= 0 || Tmax > fq_attn_max_positions() || pos < 0 || pos >= Tmax)
        return fq_fail(FQ_ERR_SHAPE, "fq_attn_decode: n_heads=%d Tmax=%d pos=%d (need 0 <= pos < Tmax <= %d)", n_heads, Tmax,
                       pos, fq_attn_max_positions());
    if (workspace_bytes < fq_attn_scratch_bytes(Tmax, n_heads))
        return fq_fail(FQ_ERR_WORKSPACE, "fq_attn_decode: workspace of %zu bytes, need %zu", workspace_bytes,
                       fq_attn_scratch_bytes(Tmax, n_heads));
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(k_cache) || !aligned16(v_cache) ||
        !aligned16(rope) || !aligned16(out) || !aligned16(workspace))
        return fq_fail(FQ_ERR_ALIGN, "fq_attn_decode: pointers must be 16-byte aligned");
    return check_hip(fq_launch_attn_decode(q, k, v, k_cache, v_cache, pos, Tmax, n_heads, rope, out, workspace,
                                           static_cast<fq_stream>(stream)), "fq_attn_decode launch");
}

extern "C" int fq_decode_step(const fq_layer *layers, int L, const uint8_t *bitvec, const void *x_in, void *x_out,
                              void *k_cache, void *v_cache, int pos, int Tmax, const float *rope, void *workspace,
                              size_t workspace_bytes, void *stream)
{
    if (!layers || !bitvec || !x_in || !x_out || !k_cache || !v_cache || !rope || !workspace)
        return fq_fail(FQ_ERR_NULL, "fq_decode_step: NULL argument");
    if (L <= 0 || Tmax <= 0 || Tmax > fq_attn_max_positions() || pos < 0 || pos >= Tmax)
        return fq_fail(FQ_ERR_SHAPE, "fq_decode_step: L=%d Tmax=%d pos=%d (need 0 <= pos < Tmax <= %d)", L, Tmax, pos,
                       fq_attn_max_positions());
    int H = 0, F = 0;
    if (int rc = validate_layers("fq_decode_step", layers, L, bitvec, &H, &F))
        return rc;
    for (int l = 0; l < L; ++l)
        for (int j = 0; j < 7; ++j)
            if (!fq_gemv_can_stream(1, layers[l].m[j].K, bitvec[7 * l + j], 2))
                return fq_fail(FQ_ERR_SHAPE, "fq_decode_step: rows of %d elements do not fit the decode kernel",
                               layers[l].m[j].K);
    if (workspace_bytes < fq_decode_workspace_bytes(H, F, Tmax))
        return fq_fail(FQ_ERR_WORKSPACE, "fq_decode_step: workspace of %zu bytes, need %zu", workspace_bytes,
                       fq_decode_workspace_bytes(H, F, Tmax));
    if (!aligned16(x_in) || !aligned16(x_out) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(rope) ||
        !aligned16(workspace))
        return fq_fail(FQ_ERR_ALIGN, "fq_decode_step: pointers must be 16-byte aligned");

    fq_stream st = static_cast<fq_stream>(stream);
    const int n_heads = H / 128;
    const size_t hb = align_up((size_t)H * 2), fb = align_up((size_t)F * 2), layer_cache = (size_t)Tmax * H * 2;
    char *ws = static_cast<char *>(workspace);
    void *q = ws, *k = ws + hb, *v = ws + 2 * hb, *a = ws + 3 * hb, *o = ws + 4 * hb, *x1 = ws + 5 * hb,
         *d = ws + 6 * hb, *xc = ws + 7 * hb, *g = ws + 8 * hb, *p = ws + 8 * hb + fb, *attn = ws + 8 * hb + 2 * fb;
    fq_packed_ref sel[7];
    const void *xres = x_in;
    for (int l = 0; l < L; ++l) {
        for (int j = 0; j < 7; ++j) {
            const fq_matrix &mx = layers[l].m[j];
            const int bits = bitvec[7 * l + j], bi = fq_bits_index(bits);
            sel[j] = fq_packed_ref{mx.packed[bi], mx.scales[bi], mx.zeros[bi], mx.N, mx.K, bits};
        }
        void *const qkv[3] = {q, k, v};
        void *const gp[2] = {g, p};
        int rc;
#define FQ_STEP(call) \
    do { \
        if ((rc = (call)) != FQ_OK) \
            return rc; \
    } while (0)
        // the previous block's output x1 + d is formed (into xc) by this block's first launch
        const fq_gemv_input in_qkv = (l == 0) ? fq_gemv_input{x_in, nullptr, nullptr, nullptr, 1}
                                              : fq_gemv_input{x1, d, nullptr, xc, 3};
        if (l > 0)
            xres = xc;
        FQ_STEP(check_hip(fq_launch_gemv_multi(in_qkv, 1, &sel[0], qkv, 3, st), "decode q/k/v"));
        FQ_STEP(check_hip(fq_launch_attn_decode(q, k, v, static_cast<char *>(k_cache) + l * layer_cache,
                                                static_cast<char *>(v_cache) + l * layer_cache, pos, Tmax, n_heads, rope, a,
                                                attn, st), "decode attention"));
        FQ_STEP(check_hip(fq_launch_gemv_multi(fq_gemv_input{a, nullptr, nullptr, nullptr, 0}, 1, &sel[3], &o, 1, st),
                          "decode o"));
        FQ_STEP(check_hip(fq_launch_gemv_multi(fq_gemv_input{xres, o, nullptr, x1, 3}, 1, &sel[4], gp, 2, st),
                          "decode gate/up"));
        FQ_STEP(check_hip(fq_launch_gemv_multi(fq_gemv_input{g, p, nullptr, nullptr, 6}, 1, &sel[6], &d, 1, st),
                          "decode down"));
#undef FQ_STEP
    }
    return check_hip(fq_launch_glue(2, x1, d, nullptr, 1, H, x_out, st), "glue add");
}

extern "C" size_t fq_attn_prefill_workspace_bytes(int T, int n_heads)
{
    if (T <= 0 || n_heads <= 0)
        return 0;
    return align_up(fq_attn_prefill_scratch_bytes(T, n_heads));
}

extern "C" int fq_attn_prefill(const void *q, const void *k, const void *v, int T, void *k_cache, void *v_cache,
                               int Tmax, int n_heads, const float *rope, void *out, void *workspace,
                               size_t workspace_bytes, void *stream)
{
    if (!q || !k || !v || !k_cache || !v_cache || !rope || !out || !workspace)
        return fq_fail(FQ_ERR_NULL, "fq_attn_prefill: NULL argument");
    if (n_heads <= 0 || T <= 0 || T > Tmax || Tmax > fq_attn_max_positions() || !below_4gib(T, (size_t)n_heads * 128, 2))
        return fq_fail(FQ_ERR_SHAPE, "fq_attn_prefill: n_heads=%d T=%d Tmax=%d (need 0 < T <= Tmax <= %d)", n_heads, T, Tmax,
                       fq_attn_max_positions());
    if (workspace_bytes < fq_attn_prefill_workspace_bytes(T, n_heads))
        return fq_fail(FQ_ERR_WORKSPACE, "fq_attn_prefill: workspace of %zu bytes, need %zu", workspace_bytes,
                       fq_attn_prefill_workspace_bytes(T, n_heads));
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(k_cache) || !aligned16(v_cache) ||
        !aligned16(rope) || !aligned16(out) || !aligned16(workspace))
        return fq_fail(FQ_ERR_ALIGN, "fq_attn_prefill: pointers must be 16-byte aligned");
    return check_hip(fq_launch_attn_prefill(q, k, v, T, k_cache, v_cache, Tmax, n_heads, rope, out, workspace,
                                            static_cast<fq_stream>(stream)), "fq_attn_prefill launch");
}

// Workspace: u, q, k, v, a, o, x1, d, x (hidden wide), g, p, m (ffn wide), then the attention's scratch.
extern "C" size_t fq_prefill_workspace_bytes(int T, int hidden, int ffn)
{
    if (T <= 0 || hidden <= 0 || ffn <= 0 || hidden % 128 != 0)
        return 0;
    return 9 * align_up((size_t)T * hidden * 2) + 3 * align_up((size_t)T * ffn * 2) +
           align_up(fq_attn_prefill_scratch_bytes(T, hidden / 128));
}

extern "C" int fq_prefill_forward(const fq_layer *layers, int L, const uint8_t *bitvec, const void *x_in, int T,
                                  void *x_out, void *k_cache, void *v_cache, int Tmax, const float *rope,
                                  void *workspace, size_t workspace_bytes, void *stream)
{
    if (!layers || !bitvec || !x_in || !x_out || !k_cache || !v_cache || !rope || !workspace)
        return fq_fail(FQ_ERR_NULL, "fq_prefill_forward: NULL argument");
    if (L <= 0 || T <= 0 || T > Tmax || Tmax > fq_attn_max_positions())
        return fq_fail(FQ_ERR_SHAPE, "fq_prefill_forward: L=%d T=%d Tmax=%d (need 0 < T <= Tmax <= %d)", L, T, Tmax,
                       fq_attn_max_positions());
    int H = 0, F = 0;
    if (int rc = validate_layers("fq_prefill_forward", layers, L, bitvec, &H, &F))
        return rc;
    if (workspace_bytes < fq_prefill_workspace_bytes(T, H, F))
        return fq_fail(FQ_ERR_WORKSPACE, "fq_prefill_forward: workspace of %zu bytes, need %zu", workspace_bytes,
                       fq_prefill_workspace_bytes(T, H, F));
    if (!aligned16(x_in) || !aligned16(x_out) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(rope) ||
        !aligned16(workspace))
        return fq_fail(FQ_ERR_ALIGN, "fq_prefill_forward: pointers must be 16-byte aligned");

    fq_stream st = static_cast<fq_stream>(stream);
    const int n_heads = H / 128, M = T;
    const size_t hb = align_up((size_t)T * H * 2), fb = align_up((size_t)T * F * 2), layer_cache = (size_t)Tmax * H * 2;
    char *ws = static_cast<char *>(workspace);
    void *u = ws, *q = ws + hb, *k = ws + 2 * hb, *v = ws + 3 * hb, *a = ws + 4 * hb, *o = ws + 5 * hb,
         *x1 = ws + 6 * hb, *d = ws + 7 * hb, *xc = ws + 8 * hb;
    void *g = ws + 9 * hb, *p = ws + 9 * hb + fb, *mm = ws + 9 * hb + 2 * fb, *attn = ws + 9 * hb + 3 * fb;
    fq_packed_ref sel[7];
    const void *xcur = x_in;
    for (int l = 0; l < L; ++l) {
        for (int j = 0; j < 7; ++j) {
            const fq_matrix &mx = layers[l].m[j];
            const int bits = bitvec[7 * l + j], bi = fq_bits_index(bits);
            sel[j] = fq_packed_ref{mx.packed[bi], mx.scales[bi], mx.zeros[bi], mx.N, mx.K, bits};
        }
        void *xnext = (l == L - 1) ? x_out : xc;
        void *const qkv[3] = {q, k, v};
        void *const gp[2] = {g, p};
        int rc;
#define FQ_STEP(call) \
    do { \
        if ((rc = (call)) != FQ_OK) \
            return rc; \
    } while (0)
        FQ_STEP(check_hip(fq_launch_glue(0, xcur, nullptr, nullptr, M, H, u, st), "glue rms"));
        if (M > 16) {
            FQ_STEP(qlinear_multi_checked(u, M, &sel[0], qkv, 3, st));
        } else {
            for (int j = 0; j < 3; ++j)
                FQ_STEP(qlinear_checked(u, M, sel[j], qkv[j], st));
        }
        FQ_STEP(check_hip(fq_launch_attn_prefill(q, k, v, T, static_cast<char *>(k_cache) + l * layer_cache,
                                                 static_cast<char *>(v_cache) + l * layer_cache, Tmax, n_heads, rope, a,
                                                 attn, st), "prefill attention"));
        FQ_STEP(qlinear_checked(a, M, sel[3], o, st));
        FQ_STEP(check_hip(fq_launch_glue2(6, xcur, o, M, H, x1, u, st), "glue add, rms"));
        if (M > 16) {
            FQ_STEP(qlinear_multi_checked(u, M, &sel[4], gp, 2, st));
        } else {
            for (int j = 0; j < 2; ++j)
                FQ_STEP(qlinear_checked(u, M, sel[4 + j], gp[j], st));
        }
        FQ_STEP(check_hip(fq_launch_glue(5, g, p, nullptr, M, F, mm, st), "glue silu*mul"));
        FQ_STEP(qlinear_checked(mm, M, sel[6], d, st));
        FQ_STEP(check_hip(fq_launch_glue(2, x1, d, nullptr, M, H, xnext, st), "glue add"));
#undef FQ_STEP
        xcur = xnext;
    }
    return FQ_OK;
}
