// Attention of one decode step over a key/value cache, for real decoder blocks around the quantized
// linears (FlexQuant, arXiv 2501.07139, Section "Experiment": the hosted models are Llama decoders; the
// serving loop of the Introduction runs them one token at a time).
//
// Per head (d = 128): q' = rope(q, pos), k' = rope(k, pos) (RoFormer rotary embedding, adjacent pairs, angles
// from a caller-supplied cos/sin table), cache K[pos] = k', V[pos] = v, and
//   a = softmax_t(q' . K[t] / sqrt(d)) . V[t]   over t <= pos.
// The work is a read of the cache: 2 * (pos+1) * H fp16 values.  The cache is head-major,
// [head][position][128], so that a head's positions are contiguous (256 bytes each) and a workgroup streams
// two 32 KiB runs.  Grid = heads x splits of 128 positions; a workgroup of 256 threads handles 16 positions per step (16 lanes x 8 dims each cover a head's 128 dims with
// 16-byte loads) and issues all its key and value loads before it touches them.  Scores, softmax and the
// weighted sum are fp32; the new token's row is taken from registers by the workgroup that owns the last
// split, which also writes it to the cache (at its end), so no workgroup uses what another writes.  With more than one
// split every workgroup leaves (max, sum, unnormalised output) and a second small kernel merges them.
#include "fq_device.h"
#include "fq_internal.h"

namespace {

constexpr int AD = 128;       // head dimension
constexpr int ACH = 128;      // positions per split
constexpr int ASTEPS = ACH / 16;

struct AttnArgs {
    const _Float16 *q, *k, *v; // [H]
    _Float16 *kc, *vc;         // [heads][Tmax][128]
    const float *rope;         // [Tmax][64][2]
    _Float16 *out;             // [H]
    float *part;               // [heads][splits][2 + 128]
    int pos, Tmax, splits;
};

// rotate the four adjacent pairs a lane holds; cs = (cos, sin) of its four angles; result rounded to fp16
__device__ __forceinline__ h8 rope8(h8 x, const float (&cs)[8])
{
    h8 r;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float a = (float)x[2 * i], b = (float)x[2 * i + 1], c = cs[2 * i], s = cs[2 * i + 1];
        r[2 * i] = (_Float16)(a * c - b * s);
        r[2 * i + 1] = (_Float16)(a * s + b * c);
    }
    return r;
}

__device__ __forceinline__ float sum16(float v) // over the 16 lanes that share a position
{
#pragma unroll
    for (int o = 1; o < 16; o <<= 1)
        v += __shfl_xor(v, o, 64);
    return v;
}

__global__ __launch_bounds__(256) void attn_decode_kernel(AttnArgs p)
{
    __shared__ float red[4][AD];
    __shared__ float wmax[4], wsum[4];

    const int head = blockIdx.x, split = blockIdx.y;
    const int tid = threadIdx.x, r = tid & 15, slot = tid >> 4, wave = tid >> 6;
    const size_t col = (size_t)head * AD + 8 * r;                 // in q, k, v, out
    const size_t base = (size_t)head * p.Tmax * AD + 8 * r;       // in the caches: + position * 128
    const int t0 = split * ACH;
    const bool owns_new = split == p.splits - 1; // the split that contains pos

    // Loads in the order they are needed, none behind a branch: the token's q, k, v and the table row first,
    // then all of the split's cache rows; the rotation then waits for the first five only.  Positions past pos
    // and pos itself re-read row t0 (t0 <= pos, in bounds; the values are not used).
    const h8 q_in = *reinterpret_cast<const h8 *>(p.q + col);
    const h8 k_in = *reinterpret_cast<const h8 *>(p.k + col);
    const h8 vnew = *reinterpret_cast<const h8 *>(p.v + col);
    const f4 cs_lo = *reinterpret_cast<const f4 *>(p.rope + (size_t)p.pos * AD + 8 * r);
    const f4 cs_hi = *reinterpret_cast<const f4 *>(p.rope + (size_t)p.pos * AD + 8 * r + 4);
    h8 kk[ASTEPS], vv[ASTEPS];
#pragma unroll
    for (int i = 0; i < ASTEPS; ++i) {
        const int t = t0 + 16 * i + slot;
        const int tr = t < p.pos ? t : t0;
        kk[i] = *reinterpret_cast<const h8 *>(p.kc + base + (size_t)tr * AD);
        vv[i] = *reinterpret_cast<const h8 *>(p.vc + base + (size_t)tr * AD);
    }
    const float cs[8] = {cs_lo[0], cs_lo[1], cs_lo[2], cs_lo[3], cs_hi[0], cs_hi[1], cs_hi[2], cs_hi[3]};
    const h8 qr = rope8(q_in, cs), knew = rope8(k_in, cs);

    float s[ASTEPS], mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < ASTEPS; ++i) {
        const int t = t0 + 16 * i + slot;
        const h8 kr = (t == p.pos) ? knew : kk[i];
        float dot = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e)
            dot = fmaf((float)qr[e], (float)kr[e], dot);
        dot = sum16(dot) * 0.08838834764831845f; // 1 / sqrt(128)
        s[i] = t <= p.pos ? dot : -INFINITY;
        mx = fmaxf(mx, s[i]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    if ((tid & 63) == 0)
        wmax[wave] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3])); // finite: position t0 <= pos is in this split

    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}, l = 0.f;
#pragma unroll
    for (int i = 0; i < ASTEPS; ++i) {
        const int t = t0 + 16 * i + slot;
        const float w = __expf(s[i] - mx); // exp(-inf) = 0 for the positions past pos
        const h8 vr = (t == p.pos) ? vnew : (t < p.pos ? vv[i] : h8{}); // unused rows may hold anything: 0 * NaN
        l += w;
#pragma unroll
        for (int e = 0; e < 8; ++e)
            acc[e] = fmaf(w, (float)vr[e], acc[e]);
    }
    // over the four position slots of a wavefront, then over the wavefronts
#pragma unroll
    for (int o = 16; o <= 32; o <<= 1) {
        l += __shfl_xor(l, o, 64);
#pragma unroll
        for (int e = 0; e < 8; ++e)
            acc[e] += __shfl_xor(acc[e], o, 64);
    }
    if ((tid & 63) < 16) {
#pragma unroll
        for (int e = 0; e < 8; ++e)
            red[wave][8 * r + e] = acc[e];
        if (r == 0)
            wsum[wave] = l;
    }
    __syncthreads();
    // The new row goes to the cache last: every load of this workgroup has been consumed by now, and no other
    // workgroup reads position pos.
    if (owns_new && slot == (p.pos - t0) % 16) { // one 16-lane group stores the head's row
        *reinterpret_cast<h8 *>(p.kc + base + (size_t)p.pos * AD) = knew;
        *reinterpret_cast<h8 *>(p.vc + base + (size_t)p.pos * AD) = vnew;
    }
    if (tid < AD) {
        const float a = (red[0][tid] + red[1][tid]) + (red[2][tid] + red[3][tid]);
        const float lsum = (wsum[0] + wsum[1]) + (wsum[2] + wsum[3]);
        if (p.splits == 1) {
            p.out[(size_t)head * AD + tid] = (_Float16)(a / lsum);
        } else {
            float *dst = p.part + ((size_t)head * p.splits + split) * (2 + AD);
            if (tid == 0) {
                dst[0] = mx;
                dst[1] = lsum;
            }
            dst[2 + tid] = a;
        }
    }
}

constexpr int AMAXSPLITS = 1024; // splits the merge kernel keeps weights for: contexts up to 131072 positions

// One workgroup of 128 threads per head: merge the splits' (max, sum, output) triples.  Threads first work
// split-parallel (maxima, weights exp(max_s - max), total sum), then dimension-parallel over the outputs with
// the weights in LDS, eight independent loads in flight per thread.
__global__ __launch_bounds__(AD) void attn_merge_kernel(AttnArgs p)
{
    __shared__ float w[AMAXSPLITS];
    __shared__ float red[2];
    const int head = blockIdx.x, tid = threadIdx.x, n = p.splits;
    const float *src = p.part + (size_t)head * n * (2 + AD);
    float mx = -INFINITY;
    for (int sp = tid; sp < n; sp += AD)
        mx = fmaxf(mx, src[(size_t)sp * (2 + AD)]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1)
        mx = fmaxf(mx, __shfl_xor(mx, o, 64));
    if ((tid & 63) == 0)
        red[tid >> 6] = mx;
    __syncthreads();
    mx = fmaxf(red[0], red[1]);
    __syncthreads();
    float l = 0.f;
    for (int sp = tid; sp < n; sp += AD) {
        const float ws = __expf(src[(size_t)sp * (2 + AD)] - mx);
        w[sp] = ws;
        l = fmaf(ws, src[(size_t)sp * (2 + AD) + 1], l);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1)
        l += __shfl_xor(l, o, 64);
    if ((tid & 63) == 0)
        red[tid >> 6] = l;
    __syncthreads();
    l = red[0] + red[1];
    float a = 0.f;
#pragma unroll 8
    for (int sp = 0; sp < n; ++sp)
        a = fmaf(w[sp], src[(size_t)sp * (2 + AD) + 2 + tid], a);
    p.out[(size_t)head * AD + tid] = (_Float16)(a / l);
}

} // namespace

int fq_attn_splits(int positions) { return (positions + ACH - 1) / ACH; }

int fq_attn_max_positions() { return AMAXSPLITS * ACH; }

size_t fq_attn_scratch_bytes(int Tmax, int n_heads) { return (size_t)n_heads * fq_attn_splits(Tmax) * (2 + AD) * sizeof(float); }

// Shapes are validated by the caller: head dimension 128, 0 <= pos < Tmax, workspace of
// fq_attn_scratch_bytes(Tmax, n_heads) bytes.
int fq_launch_attn_decode(const void *q, const void *k, const void *v, void *k_cache, void *v_cache, int pos,
                          int Tmax, int n_heads, const float *rope, void *out, void *workspace, fq_stream st)
{
    AttnArgs a;
    a.q = static_cast<const _Float16 *>(q);
    a.k = static_cast<const _Float16 *>(k);
    a.v = static_cast<const _Float16 *>(v);
    a.kc = static_cast<_Float16 *>(k_cache);
    a.vc = static_cast<_Float16 *>(v_cache);
    a.rope = rope;
    a.out = static_cast<_Float16 *>(out);
    a.part = static_cast<float *>(workspace);
    a.pos = pos;
    a.Tmax = Tmax;
    a.splits = fq_attn_splits(pos + 1);
    hipLaunchKernelGGL(attn_decode_kernel, dim3(n_heads, a.splits), dim3(256), 0, st, a);
    int rc = (int)hipGetLastError();
    if (rc != 0 || a.splits == 1)
        return rc;
    hipLaunchKernelGGL(attn_merge_kernel, dim3(n_heads), dim3(AD), 0, st, a);
    return (int)hipGetLastError();
}
