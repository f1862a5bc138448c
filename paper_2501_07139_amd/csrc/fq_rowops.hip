// Row-wise kernels: the glue between the linears of the synthetic block, the
// dense dump of a packed matrix, and the fused log-softmax cross-entropy that
// turns head logits into the per-token loss behind the perplexity score
// (FlexQuant, arXiv 2501.07139, Algorithm 1, calibrationEval).  All are
// bandwidth-bound: one pass over their inputs with 128-bit loads.
#include "fq_device.h"
#include "fq_internal.h"
#include "fq_lse.h"

namespace {

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1)
        v += __shfl_xor(v, o, 64);
    return v;
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1)
        v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// ------------------------------------------------------------------ glue
// One workgroup of 256 threads per row; the row lives in registers between the
// sum-of-squares pass and the scaling pass (H <= 256*8*MAXC halves).
constexpr int GLUE_MAXC = 8;

template <int OP>
__global__ __launch_bounds__(256) void glue_kernel(const _Float16 *__restrict__ a, const _Float16 *__restrict__ b,
                                                   const _Float16 *__restrict__ c, int H,
                                                   _Float16 *__restrict__ out)
{
    const size_t row = (size_t)blockIdx.x * H;
    const int chunks = H >> 3;
    float t[GLUE_MAXC][8];
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < GLUE_MAXC; ++i) {
        const int ch = threadIdx.x + 256 * i;
        if (ch < chunks) {
            const h8 va = *reinterpret_cast<const h8 *>(a + row + ch * 8);
            h8 vb = va, vc = va;
            if constexpr (OP != 0)
                vb = *reinterpret_cast<const h8 *>(b + row + ch * 8);
            if constexpr (OP == 1)
                vc = *reinterpret_cast<const h8 *>(c + row + ch * 8);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float v;
                if constexpr (OP == 0)
                    v = (float)va[e];
                else if constexpr (OP == 1)
                    v = (float)va[e] + (float)vb[e] + (float)vc[e];
                else if constexpr (OP == 2 || OP == 4)
                    v = (float)va[e] + (float)vb[e];
                else {
                    const float g = (float)va[e];
                    v = g / (1.0f + __expf(-g)) * (float)vb[e];
                }
                t[i][e] = v;
                ss += v * v;
            }
        }
    }
    float inv = 1.0f;
    if constexpr (OP != 2 && OP != 5) { // 2 and 5 have no norm
        __shared__ float part[4];
        ss = wave_sum(ss);
        if ((threadIdx.x & 63) == 0)
            part[threadIdx.x >> 6] = ss;
        __syncthreads();
        ss = part[0] + part[1] + part[2] + part[3];
        inv = 1.0f / sqrtf(ss / (float)H + 1e-5f);
    }
#pragma unroll
    for (int i = 0; i < GLUE_MAXC; ++i) {
        const int ch = threadIdx.x + 256 * i;
        if (ch < chunks) {
            h8 o;
#pragma unroll
            for (int e = 0; e < 8; ++e)
                o[e] = (_Float16)(t[i][e] * inv);
            *reinterpret_cast<h8 *>(out + row + ch * 8) = o;
        }
    }
}

// Two consecutive row-wise steps of the block in one pass (M > 16), each rounded to fp16 where the separate
// kernels would store it, so the values are those of the two calls:
//   OP 6: aux = a + b,       out = rms(aux)     the residual after the output projection and the FFN's input
//   OP 7: aux = rms(a + b),  out = rms(aux)     a block's output and the next block's first normalisation
template <int OP>
__global__ __launch_bounds__(256) void glue2_kernel(const _Float16 *__restrict__ a, const _Float16 *__restrict__ b, int H,
                                                    _Float16 *__restrict__ aux, _Float16 *__restrict__ out)
{
    const size_t row = (size_t)blockIdx.x * H;
    const int chunks = H >> 3;
    __shared__ float part[2][4];
    auto row_sum = [&](float ss, int which) {
        ss = wave_sum(ss);
        if ((threadIdx.x & 63) == 0)
            part[which][threadIdx.x >> 6] = ss;
        __syncthreads();
        return part[which][0] + part[which][1] + part[which][2] + part[which][3];
    };
    float t[GLUE_MAXC][8];
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < GLUE_MAXC; ++i) {
        const int ch = threadIdx.x + 256 * i;
        if (ch < chunks) {
            const h8 va = *reinterpret_cast<const h8 *>(a + row + ch * 8), vb = *reinterpret_cast<const h8 *>(b + row + ch * 8);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float v = (float)va[e] + (float)vb[e];
                if constexpr (OP == 6)
                    v = (float)(_Float16)v; // the stored sum is what the norm reads
                t[i][e] = v;
                ss += v * v;
            }
        }
    }
    if constexpr (OP == 7) { // first norm; its rounded result is the second one's input
        const float inv = 1.0f / sqrtf(row_sum(ss, 0) / (float)H + 1e-5f);
        ss = 0.f;
#pragma unroll
        for (int i = 0; i < GLUE_MAXC; ++i)
            if (threadIdx.x + 256 * i < chunks) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float v = (float)(_Float16)(t[i][e] * inv);
                    t[i][e] = v;
                    ss += v * v;
                }
            }
    }
    const float inv = 1.0f / sqrtf(row_sum(ss, 1) / (float)H + 1e-5f);
#pragma unroll
    for (int i = 0; i < GLUE_MAXC; ++i) {
        const int ch = threadIdx.x + 256 * i;
        if (ch < chunks) {
            h8 x, o;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                x[e] = (_Float16)t[i][e]; // exact: already an fp16 value
                o[e] = (_Float16)(t[i][e] * inv);
            }
            *reinterpret_cast<h8 *>(aux + row + ch * 8) = x;
            *reinterpret_cast<h8 *>(out + row + ch * 8) = o;
        }
    }
}

// ------------------------------------------------------------------- NLL
// One workgroup per token row; each thread keeps a running (max, sum of
// exp(l - max)) over its 16-byte chunks, then the pairs are merged across the
// wavefront and the workgroup.  The label's logit is read directly.
__global__ __launch_bounds__(256) void nll_kernel(const _Float16 *__restrict__ logits,
                                                  const int32_t *__restrict__ labels, int V,
                                                  float *__restrict__ nll)
{
    const int row = blockIdx.x;
    const int label = labels[row];
    if (label < 0 || label >= V) { // uniform across the workgroup
        if (threadIdx.x == 0)
            nll[row] = 0.f;
        return;
    }
    const _Float16 *l = logits + (size_t)row * V;
    float mx = -INFINITY, se = 0.f;
    // rows start 16-byte aligned only if V % 8 == 0; otherwise take the scalar route
    if ((V & 7) == 0) {
        const int chunks = V >> 3;
        for (int ch = threadIdx.x; ch < chunks; ch += 256) {
            const h8 v = *reinterpret_cast<const h8 *>(l + ch * 8);
            float cm = (float)v[0];
#pragma unroll
            for (int e = 1; e < 8; ++e)
                cm = fmaxf(cm, (float)v[e]);
            float cs = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e)
                cs += __expf((float)v[e] - cm);
            lse_merge(mx, se, cm, cs);
        }
    } else {
        for (int i = threadIdx.x; i < V; i += 256)
            lse_merge(mx, se, (float)l[i], 1.0f);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float m2 = __shfl_xor(mx, o, 64), s2 = __shfl_xor(se, o, 64);
        lse_merge(mx, se, m2, s2);
    }
    __shared__ float pm[4], ps[4];
    if ((threadIdx.x & 63) == 0) {
        pm[threadIdx.x >> 6] = mx;
        ps[threadIdx.x >> 6] = se;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        float m = pm[0], s = ps[0];
        for (int w = 1; w < 4; ++w)
            lse_merge(m, s, pm[w], ps[w]);
        nll[row] = logf(s) + (m - (float)l[label]); // difference first: exact for fp16 inputs
    }
}

// --------------------------------------------------------------- dequant
// Dense dump of a packed matrix, one thread per (sixteen-row block, group, lane)
// chunk: reads the format literally (integer field extraction), then
// float(scale) * (float(code) - float(zero)) with both steps rounded to fp32.
template <int BITS>
__global__ __launch_bounds__(64) void dequant_kernel(const uint32_t *__restrict__ packed,
                                                     const _Float16 *__restrict__ scales,
                                                     const _Float16 *__restrict__ zeros, int N, int K,
                                                     void *__restrict__ out, int out_is_fp16)
{
    constexpr int SUB = Fmt<BITS>::SUB;
    const int G = K >> 7;
    const int g = blockIdx.x, rb16 = blockIdx.y, lane = threadIdx.x;
    const int r = lane & 15, c = lane >> 4;
    const int n = rb16 * 16 + r;
    const uint32_t *tile = packed + ((size_t)(rb16 / SUB) * G + g) * tile_dwords<BITS>();
    uint32_t C[BITS];
    load_chunk<BITS>(tile, rb16 % SUB, lane, C);
    const size_t meta = ((size_t)rb16 * G + g) * 16 + r;
    const float z = (float)zeros[meta], sc = (float)scales[meta];
    if (n >= N)
        return;
#pragma unroll
    for (int t = 0; t < 32; ++t) {
        const int s = t >> 3, e = t & 7;
        const int k = g * 128 + 32 * s + 8 * c + e;
        const float d = __fsub_rn((float)code_at<BITS>(C, t), z);
        const float w = __fmul_rn(sc, d);
        if (out_is_fp16)
            static_cast<_Float16 *>(out)[(size_t)n * K + k] = (_Float16)w;
        else
            static_cast<float *>(out)[(size_t)n * K + k] = w;
    }
}

} // namespace

int fq_launch_glue(int op, const void *a, const void *b, const void *c, int M, int H, void *out, fq_stream st)
{
    dim3 grid(M), block(256);
    const _Float16 *pa = static_cast<const _Float16 *>(a), *pb = static_cast<const _Float16 *>(b),
                   *pc = static_cast<const _Float16 *>(c);
    _Float16 *po = static_cast<_Float16 *>(out);
    switch (op) {
    case 0: hipLaunchKernelGGL(glue_kernel<0>, grid, block, 0, st, pa, pb, pc, H, po); break;
    case 1: hipLaunchKernelGGL(glue_kernel<1>, grid, block, 0, st, pa, pb, pc, H, po); break;
    case 2: hipLaunchKernelGGL(glue_kernel<2>, grid, block, 0, st, pa, pb, pc, H, po); break;
    case 3: hipLaunchKernelGGL(glue_kernel<3>, grid, block, 0, st, pa, pb, pc, H, po); break;
    case 4: hipLaunchKernelGGL(glue_kernel<4>, grid, block, 0, st, pa, pb, pc, H, po); break;
    default: hipLaunchKernelGGL(glue_kernel<5>, grid, block, 0, st, pa, pb, pc, H, po); break;
    }
    return (int)hipGetLastError();
}

int fq_launch_glue2(int op, const void *a, const void *b, int M, int H, void *aux, void *out, fq_stream st)
{
    dim3 grid(M), block(256);
    const _Float16 *pa = static_cast<const _Float16 *>(a), *pb = static_cast<const _Float16 *>(b);
    if (op == 6)
        hipLaunchKernelGGL(glue2_kernel<6>, grid, block, 0, st, pa, pb, H, static_cast<_Float16 *>(aux), static_cast<_Float16 *>(out));
    else
        hipLaunchKernelGGL(glue2_kernel<7>, grid, block, 0, st, pa, pb, H, static_cast<_Float16 *>(aux), static_cast<_Float16 *>(out));
    return (int)hipGetLastError();
}

// Row-wise Euclidean distance between two logit arrays (sensitivity analysis of the search, Section
// "Efficient Design Space Navigation").  One workgroup per row, one pass over both rows with 128-bit loads; differences and
// squares in fp32, four partial sums per thread, then a fixed-order reduction.
__global__ __launch_bounds__(256) void logit_l2_kernel(const _Float16 *__restrict__ a, const _Float16 *__restrict__ b,
                                                       int V, float *__restrict__ dist)
{
    const int row = blockIdx.x;
    const _Float16 *ra = a + (size_t)row * V, *rb = b + (size_t)row * V;
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    // rows start 16-byte aligned only if V % 8 == 0; otherwise take the scalar route
    if ((V & 7) == 0) {
        const int chunks = V >> 3;
        for (int ch = threadIdx.x; ch < chunks; ch += 256) {
            const h8 va = *reinterpret_cast<const h8 *>(ra + ch * 8), vb = *reinterpret_cast<const h8 *>(rb + ch * 8);
            float d[8];
#pragma unroll
            for (int e = 0; e < 8; ++e)
                d[e] = (float)va[e] - (float)vb[e];
            s0 = fmaf(d[0], d[0], s0); s1 = fmaf(d[1], d[1], s1); s2 = fmaf(d[2], d[2], s2); s3 = fmaf(d[3], d[3], s3);
            s0 = fmaf(d[4], d[4], s0); s1 = fmaf(d[5], d[5], s1); s2 = fmaf(d[6], d[6], s2); s3 = fmaf(d[7], d[7], s3);
        }
    } else {
        for (int i = threadIdx.x; i < V; i += 256) {
            const float d = (float)ra[i] - (float)rb[i];
            s0 = fmaf(d, d, s0);
        }
    }
    float ss = (s0 + s1) + (s2 + s3);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1)
        ss += __shfl_xor(ss, o, 64);
    __shared__ float part[4];
    if ((threadIdx.x & 63) == 0)
        part[threadIdx.x >> 6] = ss;
    __syncthreads();
    if (threadIdx.x == 0)
        dist[row] = sqrtf((part[0] + part[1]) + (part[2] + part[3]));
}

int fq_launch_logit_l2(const void *a, const void *b, int M, int V, float *dist, fq_stream st)
{
    hipLaunchKernelGGL(logit_l2_kernel, dim3(M), dim3(256), 0, st, static_cast<const _Float16 *>(a),
                       static_cast<const _Float16 *>(b), V, dist);
    return (int)hipGetLastError();
}

int fq_launch_nll(const void *logits, const int32_t *labels, int M, int V, float *nll, fq_stream st)
{
    hipLaunchKernelGGL(nll_kernel, dim3(M), dim3(256), 0, st, static_cast<const _Float16 *>(logits), labels, V, nll);
    return (int)hipGetLastError();
}

int fq_launch_dequant(const fq_packed_ref &w, void *out, int out_is_fp16, fq_stream st)
{
    const int Np16 = (w.N + 63) / 64 * 4;
    dim3 grid(w.K >> 7, Np16), block(64);
    const uint32_t *p = static_cast<const uint32_t *>(w.packed);
    const _Float16 *s = static_cast<const _Float16 *>(w.scales), *z = static_cast<const _Float16 *>(w.zeros);
    switch (w.bits) {
    case 2: hipLaunchKernelGGL(dequant_kernel<2>, grid, block, 0, st, p, s, z, w.N, w.K, out, out_is_fp16); break;
    case 3: hipLaunchKernelGGL(dequant_kernel<3>, grid, block, 0, st, p, s, z, w.N, w.K, out, out_is_fp16); break;
    case 4: hipLaunchKernelGGL(dequant_kernel<4>, grid, block, 0, st, p, s, z, w.N, w.K, out, out_is_fp16); break;
    default: hipLaunchKernelGGL(dequant_kernel<8>, grid, block, 0, st, p, s, z, w.N, w.K, out, out_is_fp16); break;
    }
    return (int)hipGetLastError();
}

// ------------------------------------------------------------ streaming read
// Reads `bytes` once with 128-bit loads, eight independent loads per lane and round, and keeps one word
// per workgroup: what a kernel that does nothing but read reaches on this device, the practical ceiling
// beside which the decode path's bytes per second are reported (Section "Introduction": single-batch
// decoding streams every weight once per token and is bound by that).
namespace {
__global__ __launch_bounds__(256) void stream_read_kernel(const u4v *__restrict__ src, size_t n16, uint32_t *sink)
{
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    u4v acc = {0u, 0u, 0u, 0u};
    for (; i + 7 * stride < n16; i += 8 * stride) {
        u4v v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k)
            v[k] = __builtin_nontemporal_load(src + i + k * stride);
#pragma unroll
        for (int k = 0; k < 8; ++k)
            acc ^= v[k];
    }
    for (; i < n16; i += stride)
        acc ^= __builtin_nontemporal_load(src + i);
    uint32_t w = acc.x ^ acc.y ^ acc.z ^ acc.w;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1)
        w ^= __shfl_xor(w, o, 64);
    __shared__ uint32_t part[4];
    if ((threadIdx.x & 63) == 0)
        part[threadIdx.x >> 6] = w;
    __syncthreads();
    if (threadIdx.x == 0)
        sink[blockIdx.x] = part[0] ^ part[1] ^ part[2] ^ part[3];
}
} // namespace

int fq_launch_stream_read(const void *src, size_t bytes, uint32_t *sink, int blocks, fq_stream st)
{
    hipLaunchKernelGGL(stream_read_kernel, dim3(blocks), dim3(256), 0, st, static_cast<const u4v *>(src), bytes / 16, sink);
    return (int)hipGetLastError();
}

