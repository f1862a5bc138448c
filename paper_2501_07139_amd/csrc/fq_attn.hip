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

// ------------------------------------------------------------------ prefill
// Causal attention over a whole sequence (positions 0..T-1 of one sequence), for running real decoder blocks
// over calibration sequences (Algorithm 1, calibrationEval) and for filling the cache before decoding.
//
// attn_prep_kernel, per (64 positions, head): rotates q (to a scratch array, row-major like q) and k (into
// the head-major key cache), copies v into the value cache and also writes it transposed, [head][128][Tp],
// through an LDS tile, so that the second product below finds the positions of one dimension contiguous.
//
// attn_prefill_kernel, per (64 query rows, head), 4 wavefronts x 16 query rows, over the key/value tiles of
// 64 positions up to the diagonal, both copied straight into double-buffered LDS tiles:
//   S^T = K . Q'^T     16x16x32 MFMA, A = key rows from LDS, B = the wavefront's query rows (registers)
//   a lane then holds scores of ONE query row (column l%16): running max and sum need only in-lane work and
//   two cross-lane steps; P = exp(S - max) rounded to fp16 is, as it stands in the lane, the B operand of
//   O^T = V^T . P^T    A = rows of the transposed values from LDS (the k index runs over the positions in
//   the order the score blocks left them: 4g..4g+3 of one block, then of the next),
// with the accumulators rescaled per lane when the maximum moves.  Heavy query tiles are launched first.
namespace {

constexpr int PT = 64; // positions per tile, queries and keys alike

struct PrefillArgs {
    const _Float16 *q, *k, *v; // [T][H]
    _Float16 *qr;              // [T][H] rotated queries
    _Float16 *kc, *vc;         // [heads][Tmax][128]
    _Float16 *vt;              // [heads][128][Tp]
    const float *rope;         // [Tmax][64][2]
    _Float16 *out;             // [T][H]
    int T, Tp, Tmax, H;
};

__global__ __launch_bounds__(256) void attn_prep_kernel(PrefillArgs p)
{
    __shared__ _Float16 vs[PT][AD + 2]; // +2 halves: the column reads below spread over the banks
    const int t0 = blockIdx.x * PT, head = blockIdx.y, tid = threadIdx.x;
    for (int c = tid; c < PT * 16; c += 256) {
        const int row = c >> 4, r = c & 15, t = t0 + row;
        h8 vv = {};
        if (t < p.T) {
            const size_t src = (size_t)t * p.H + (size_t)head * AD + 8 * r;
            const f4 lo = *reinterpret_cast<const f4 *>(p.rope + (size_t)t * AD + 8 * r);
            const f4 hi = *reinterpret_cast<const f4 *>(p.rope + (size_t)t * AD + 8 * r + 4);
            const float cs[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            *reinterpret_cast<h8 *>(p.qr + src) = rope8(*reinterpret_cast<const h8 *>(p.q + src), cs);
            const size_t dst = ((size_t)head * p.Tmax + t) * AD + 8 * r;
            *reinterpret_cast<h8 *>(p.kc + dst) = rope8(*reinterpret_cast<const h8 *>(p.k + src), cs);
            vv = *reinterpret_cast<const h8 *>(p.v + src);
            *reinterpret_cast<h8 *>(p.vc + dst) = vv;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e)
            vs[row][8 * r + e] = vv[e]; // zeros past T: they meet zero weights, and 0 * 0 stays 0
    }
    __syncthreads();
    for (int c = tid; c < AD * (PT / 8); c += 256) {
        const int d = c >> 3, j = c & 7;
        h8 o;
#pragma unroll
        for (int e = 0; e < 8; ++e)
            o[e] = vs[8 * j + e][d];
        *reinterpret_cast<h8 *>(p.vt + ((size_t)head * AD + d) * p.Tp + t0 + 8 * j) = o;
    }
}

__global__ __launch_bounds__(256, 2) void attn_prefill_kernel(PrefillArgs p)
{
    __shared__ h8 Ks[2][PT * 16];  // chunk ch of key row r at r*16 + (ch ^ (r & 15))
    __shared__ h8 Vs[2][AD * 8];   // 16-byte slot sl of dimension row d at d*8 + (sl ^ ((d >> 1) & 7))

    const int qt = (int)gridDim.x - 1 - (int)blockIdx.x, head = blockIdx.y; // long rows of tiles first
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 15, g = lane >> 4;
    const int q0 = qt * PT + 16 * wave;

    // the wavefront's query rows as B operands of the four k-steps over the head dimension
    h8 qb[4];
    {
        const size_t row = (size_t)min(q0 + col, p.T - 1) * p.H + (size_t)head * AD + 8 * g;
#pragma unroll
        for (int s = 0; s < 4; ++s)
            qb[s] = *reinterpret_cast<const h8 *>(p.qr + row + 32 * s);
    }

    const fq_rsrc kr = make_rsrc(p.kc + (size_t)head * p.Tmax * AD, (uint32_t)p.Tmax * AD * 2u);
    const fq_rsrc vr = make_rsrc(p.vt + (size_t)head * AD * p.Tp, (uint32_t)AD * (uint32_t)p.Tp * 2u);
    // copies: the i-th of a wavefront fills the 64 slots from 64*(wave + 4i) of a tile
    uint32_t koff[4], voff[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int krow = 4 * (wave + 4 * i) + (lane >> 4), kch = (lane & 15) ^ (krow & 15);
        koff[i] = ((uint32_t)krow * AD + (uint32_t)kch * 8u) * 2u; // + tile * 64 rows, clamped below
        const int vrow = 8 * (wave + 4 * i) + (lane >> 3), vsl = (lane & 7) ^ ((vrow >> 1) & 7);
        voff[i] = ((uint32_t)vrow * (uint32_t)p.Tp + (uint32_t)vsl * 8u) * 2u;
    }
    auto copy_tiles = [&](int buffer, int jt) {
        // key rows past the last position re-read the last one: their scores are masked
        const int last = p.T - 1 - jt * PT;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int krow = 4 * (wave + 4 * i) + (lane >> 4);
            const uint32_t off = krow <= last ? koff[i] : koff[i] - (uint32_t)(krow - last) * (AD * 2u);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(kr, &Ks[buffer][64 * (wave + 4 * i)], 16, off,
                                                     (uint32_t)jt * (PT * AD * 2u), 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(vr, &Vs[buffer][64 * (wave + 4 * i)], 16, voff[i],
                                                     (uint32_t)jt * (PT * 2u), 0, 0);
    };

    f4 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
        acc[i] = f4{0.f, 0.f, 0.f, 0.f};
    float mx = -INFINITY, l = 0.f;

    copy_tiles(0, 0);
    __builtin_amdgcn_s_waitcnt(FQ_WAIT_VMCNT0);
    __syncthreads();

    for (int jt = 0; jt <= qt; ++jt) {
        const int cur = jt & 1;
        if (jt < qt)
            copy_tiles(cur ^ 1, jt + 1);

        // scores of 64 positions against the wavefront's 16 query rows, transposed
        f4 st[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            st[b] = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const int row = 16 * b + col, ch = 4 * s + g;
                st[b] = mfma16x16x32(Ks[cur][row * 16 + (ch ^ (row & 15))], qb[s], st[b]);
            }
        }
        // lane: query row q0 + col, positions jt*64 + 16b + 4g + v
        float tmax = -INFINITY;
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int kv = jt * PT + 16 * b + 4 * g + v;
                const float sc = st[b][v] * 0.08838834764831845f; // 1 / sqrt(128)
                st[b][v] = kv <= q0 + col ? sc : -INFINITY;      // causal mask (also hides positions past T)
                tmax = fmaxf(tmax, st[b][v]);
            }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
        const float mnew = fmaxf(mx, tmax); // finite from the first tile on: position 0 is visible to every row
        const float alpha = __expf(mx - mnew);
        mx = mnew;
        h8 pb[2];
        float psum = 0.f;
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float e = __expf(st[b][v] - mnew);
                psum += e;
                pb[b >> 1][4 * (b & 1) + v] = (_Float16)e;
            }
        l = l * alpha + psum;
#pragma unroll
        for (int i = 0; i < 8; ++i)
            acc[i] *= alpha;
        // O^T += V^T . P^T; k-slot e of k-step ks is position 32ks + 4g + e (e < 4) or 32ks + 16 + 4g + e - 4
#pragma unroll
        for (int db = 0; db < 8; ++db) {
            const int d = 16 * db + col, sw = (d >> 1) & 7;
            const uint2 *rowp = reinterpret_cast<const uint2 *>(&Vs[cur][d * 8]);
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                const int s0 = 4 * ks + (g >> 1), s1 = s0 + 2;
                const uint2 lo = rowp[2 * (s0 ^ sw) + (g & 1)], hi = rowp[2 * (s1 ^ sw) + (g & 1)];
                const u4v both = {lo.x, lo.y, hi.x, hi.y};
                acc[db] = mfma16x16x32(__builtin_bit_cast(h8, both), pb[ks], acc[db]);
            }
        }
        __builtin_amdgcn_s_waitcnt(FQ_WAIT_VMCNT0);
        __syncthreads();
    }

    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    const int q = q0 + col;
    if (q < p.T) {
        const float inv = 1.0f / l;
#pragma unroll
        for (int db = 0; db < 8; ++db) {
            const h4 o = {(_Float16)(acc[db][0] * inv), (_Float16)(acc[db][1] * inv), (_Float16)(acc[db][2] * inv),
                          (_Float16)(acc[db][3] * inv)};
            *reinterpret_cast<h4 *>(p.out + (size_t)q * p.H + (size_t)head * AD + 16 * db + 4 * g) = o;
        }
    }
}

} // namespace

static int prefill_tp(int T) { return (T + PT - 1) / PT * PT; }

size_t fq_attn_prefill_scratch_bytes(int T, int n_heads)
{
    return (size_t)T * n_heads * AD * 2 + (size_t)n_heads * AD * prefill_tp(T) * 2;
}

// Shapes validated by the caller: 0 < T <= Tmax, head dimension 128, 16-byte aligned pointers, the byte
// sizes of one head's cache and of one head's transposed values below 4 GiB.
int fq_launch_attn_prefill(const void *q, const void *k, const void *v, int T, void *k_cache, void *v_cache,
                           int Tmax, int n_heads, const float *rope, void *out, void *workspace, fq_stream st)
{
    PrefillArgs a;
    a.q = static_cast<const _Float16 *>(q);
    a.k = static_cast<const _Float16 *>(k);
    a.v = static_cast<const _Float16 *>(v);
    a.qr = static_cast<_Float16 *>(workspace);
    a.vt = a.qr + (size_t)T * n_heads * AD;
    a.kc = static_cast<_Float16 *>(k_cache);
    a.vc = static_cast<_Float16 *>(v_cache);
    a.rope = rope;
    a.out = static_cast<_Float16 *>(out);
    a.T = T;
    a.Tp = prefill_tp(T);
    a.Tmax = Tmax;
    a.H = n_heads * AD;
    const int tiles = a.Tp / PT;
    hipLaunchKernelGGL(attn_prep_kernel, dim3(tiles, n_heads), dim3(256), 0, st, a);
    int rc = (int)hipGetLastError();
    if (rc != 0)
        return rc;
    hipLaunchKernelGGL(attn_prefill_kernel, dim3(tiles, n_heads), dim3(256), 0, st, a);
    return (int)hipGetLastError();
}
