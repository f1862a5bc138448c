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

#include <type_traits>

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
// attn_prefill_kernel, per (128 query rows, head), 4 wavefronts x 2 blocks of 16 query rows, over the
// key/value tiles of 64 positions up to the diagonal, in double-buffered LDS tiles:
//   S^T = K . Q'^T     16x16x32 MFMA, A = key rows from LDS, B = the wavefront's query rows (registers)
//   a lane then holds scores of ONE query row (column l%16): running max and sum need only in-lane work and
//   two cross-lane steps; P = exp(S - max) rounded to fp16 is, as it stands in the lane, the B operand of
//   O^T = V^T . P^T    A = rows of the transposed values from LDS (the key rows are dealt to the score
//   blocks in such an order that a lane's eight weights of a k-step belong to eight contiguous positions),
// with the accumulators rescaled per lane when the maximum moves.  Long and short query tiles are paired
// on a CU through the order of the grid.
namespace {

constexpr int PT = 64; // positions per tile, queries and keys alike

struct PrefillArgs {
    const _Float16 *q, *k, *v; // [T][H]
    _Float16 *qr;              // [T][H] rotated queries
    _Float16 *kc, *vc;         // [heads][Tmax][128]
    _Float16 *vt;              // [heads][128][Tp]
    const float *rope;         // [Tmax][64][2]
    _Float16 *out;             // [T][H]
    int T, Tp, Tmax, H, NQ, heads;
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

constexpr int QB = 2;            // blocks of 16 query rows per wavefront
constexpr int QT = 4 * 16 * QB;  // query rows per workgroup

// row of the key tile that feeds row r of score block b: chosen so that the eight positions a lane ends up
// holding for one k-step of the second product, (4g..4g+3 of blocks 2ks and 2ks+1), are the contiguous
// positions 32ks + 8g .. + 7, i.e. one 16-byte slot of a transposed value row
__device__ __forceinline__ int key_row(int b, int r) { return 32 * (b >> 1) + 8 * (r >> 2) + 4 * (b & 1) + (r & 3); }
// position of 16-byte chunk ch in key row `row`: the sixteen rows a block's operand read touches differ in
// bits 0-1 and 3-4 of the row number
__device__ __forceinline__ int key_slot(int row, int ch) { return row * 16 + (ch ^ ((row & 3) | ((row >> 1) & 12))); }

__global__ __launch_bounds__(256, 2) void attn_prefill_kernel(PrefillArgs p)
{
    // Key tiles [64 positions][16 chunks] (see key_slot); value tiles: 16-byte slot sl (eight positions) of
    // dimension row d at d*8 + (sl ^ ((d >> 1) & 7)).  Two of each, as separate arrays named statically in
    // a loop unrolled by two: the compiler then knows that the key tile being read is not the one the
    // copies in flight write, and does not wait for those copies before the first read.  It keeps track of
    // only a few such copies, so the value tiles take the other road: global memory to registers at the
    // top of a step, registers to LDS at its end.
    __shared__ h8 Ks0[PT * 16], Ks1[PT * 16];
    __shared__ h8 Vs0[AD * 8], Vs1[AD * 8];

    // Jobs (query tile, head) sorted by length, longest first, are dealt so that the first half of the grid
    // takes them from the long end and the second half from the short end: the workgroups b and b + half,
    // which share a CU when the grid is two workgroups per CU, then have about the same total length.
    const int jobs = (int)gridDim.x, half = (jobs + 1) >> 1, bidx = (int)blockIdx.x;
    const int job = bidx < half ? bidx : jobs - 1 - (bidx - half);
    const int qt = p.NQ - 1 - job / p.heads, head = job % p.heads;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 15, g = lane >> 4;
    const int q0 = qt * QT + 16 * QB * wave; // first query row of this wavefront
    const int last_tile = min((qt * QT + QT - 1) / PT, p.Tp / PT - 1);

    // the wavefront's query rows as B operands of the four k-steps over the head dimension
    h8 qb[QB][4];
#pragma unroll
    for (int qi = 0; qi < QB; ++qi) {
        const size_t row = (size_t)min(q0 + 16 * qi + col, p.T - 1) * p.H + (size_t)head * AD + 8 * g;
#pragma unroll
        for (int s = 0; s < 4; ++s)
            qb[qi][s] = *reinterpret_cast<const h8 *>(p.qr + row + 32 * s);
    }

    const fq_rsrc kr = make_rsrc(p.kc + (size_t)head * p.Tmax * AD, (uint32_t)p.Tmax * AD * 2u);
    const fq_rsrc vr = make_rsrc(p.vt + (size_t)head * AD * p.Tp, (uint32_t)AD * (uint32_t)p.Tp * 2u);
    // copies: the i-th of a wavefront fills the 64 slots from 64*(wave + 4i) of a tile
    uint32_t koff[4], voff[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int krow = 4 * (wave + 4 * i) + (lane >> 4);
        const int kch = (lane & 15) ^ ((krow & 3) | ((krow >> 1) & 12));
        koff[i] = ((uint32_t)krow * AD + (uint32_t)kch * 8u) * 2u;
        const int vrow = 8 * (wave + 4 * i) + (lane >> 3), vsl = (lane & 7) ^ ((vrow >> 1) & 7);
        voff[i] = ((uint32_t)vrow * (uint32_t)p.Tp + (uint32_t)vsl * 8u) * 2u;
    }
    h8 vreg[4];
    auto load_tiles = [&](h8 *Kdst, int jt) {
        if (jt * PT + PT <= p.T) { // uniform: only the sequence's last tile can reach past its end
#pragma unroll
            for (int i = 0; i < 4; ++i)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(kr, &Kdst[64 * (wave + 4 * i)], 16, koff[i],
                                                         (uint32_t)jt * (PT * AD * 2u), 0, 0);
        } else { // key rows past the last position re-read the last one: their scores are masked
            const int last = p.T - 1 - jt * PT;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int krow = 4 * (wave + 4 * i) + (lane >> 4);
                const uint32_t off = krow <= last ? koff[i] : koff[i] - (uint32_t)(krow - last) * (AD * 2u);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(kr, &Kdst[64 * (wave + 4 * i)], 16, off,
                                                         (uint32_t)jt * (PT * AD * 2u), 0, 0);
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
            vreg[i] = __builtin_bit_cast(h8, buf_load_b128(vr, voff[i], (uint32_t)jt * (PT * 2u)));
    };
    auto store_values = [&](h8 *Vdst) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            Vdst[64 * (wave + 4 * i) + lane] = vreg[i];
    };

    f4 acc[QB][8];
    float mx[QB], l[QB];
#pragma unroll
    for (int qi = 0; qi < QB; ++qi) {
        mx[qi] = -INFINITY;
        l[qi] = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i)
            acc[qi][i] = f4{0.f, 0.f, 0.f, 0.f};
    }

    load_tiles(Ks0, 0);
    store_values(Vs0);
    __builtin_amdgcn_s_waitcnt(FQ_WAIT_VMCNT0);
    __syncthreads();

    auto tile_step = [&](int jt, auto parity) {
        constexpr int PAR = decltype(parity)::value;
        h8 *const Kcur = PAR ? Ks1 : Ks0, *const Vcur = PAR ? Vs1 : Vs0;
        if (jt < last_tile)
            load_tiles(PAR ? Ks0 : Ks1, jt + 1);

        // a wavefront whose every query row lies before the tile has nothing to add (uniform per wavefront)
        if (jt * PT <= q0 + 16 * QB - 1) {
            // scores of 64 positions against the wavefront's query rows, transposed: S^T = K . Q'^T
            f4 st[QB][4];
#pragma unroll
            for (int b = 0; b < 4; ++b) {
#pragma unroll
                for (int qi = 0; qi < QB; ++qi)
                    st[qi][b] = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const h8 ka = Kcur[key_slot(key_row(b, col), 4 * s + g)];
#pragma unroll
                    for (int qi = 0; qi < QB; ++qi)
                        st[qi][b] = mfma16x16x32(ka, qb[qi][s], st[qi][b]);
                }
            }
            // lane: query row q0 + 16qi + col; st[qi][b][v] belongs to position jt*64 + key_row(b, 4g + v).
            // Scores are kept in units of log2(e) / sqrt(128), so that the exponentials are bare exp2; only
            // tiles that reach the diagonal need the mask (it also hides the positions past T).
            constexpr float kScale = 0.08838834764831845f * 1.4426950408889634f;
            const bool diagonal = jt * PT + PT - 1 > q0; // uniform per wavefront
            h8 pb[QB][2];
#pragma unroll
            for (int qi = 0; qi < QB; ++qi) {
                float tmax = -INFINITY;
                if (diagonal) {
#pragma unroll
                    for (int b = 0; b < 4; ++b)
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            const int kv = jt * PT + key_row(b, 4 * g + v);
                            st[qi][b][v] = kv <= q0 + 16 * qi + col ? st[qi][b][v] * kScale : -INFINITY;
                            tmax = fmaxf(tmax, st[qi][b][v]);
                        }
                } else {
#pragma unroll
                    for (int b = 0; b < 4; ++b)
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            st[qi][b][v] *= kScale;
                            tmax = fmaxf(tmax, st[qi][b][v]);
                        }
                }
                tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
                tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
                // the maximum so far; a row the tile does not reach at all keeps its old one (and gets zeros)
                const float mnew = fmaxf(mx[qi], tmax);
                const float mref = mnew == -INFINITY ? 0.f : mnew;
                float psum = 0.f;
#pragma unroll
                for (int b = 0; b < 4; ++b)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const float e = __builtin_amdgcn_exp2f(st[qi][b][v] - mref);
                        psum += e;
                        pb[qi][b >> 1][4 * (b & 1) + v] = (_Float16)e;
                    }
                if (__builtin_amdgcn_ballot_w64(mnew != mx[qi]) != 0) { // some row's maximum moved: rescale
                    const float alpha = __builtin_amdgcn_exp2f(mx[qi] - mref); // exp2(-inf) = 0 at the start
                    mx[qi] = mnew;
                    l[qi] *= alpha;
#pragma unroll
                    for (int i = 0; i < 8; ++i)
                        acc[qi][i] *= alpha;
                }
                l[qi] += psum;
            }
            // O^T += V^T . P^T; k-slot e of k-step ks is position 32ks + 8g + e: one slot of a value row
#pragma unroll
            for (int db = 0; db < 8; ++db) {
                const int d = 16 * db + col, sw = (d >> 1) & 7;
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) {
                    const h8 va = Vcur[d * 8 + ((4 * ks + g) ^ sw)];
#pragma unroll
                    for (int qi = 0; qi < QB; ++qi)
                        acc[qi][db] = mfma16x16x32(va, pb[qi][ks], acc[qi][db]);
                }
            }
        }
        if (jt < last_tile)
            store_values(PAR ? Vs0 : Vs1); // last read in the previous step, before its barrier
        __builtin_amdgcn_s_waitcnt(FQ_WAIT_VMCNT0);
        __syncthreads();
    };
    int jt = 0;
    for (; jt + 1 <= last_tile; jt += 2) {
        tile_step(jt, std::integral_constant<int, 0>{});
        tile_step(jt + 1, std::integral_constant<int, 1>{});
    }
    if (jt <= last_tile)
        tile_step(jt, std::integral_constant<int, 0>{});

#pragma unroll
    for (int qi = 0; qi < QB; ++qi) {
        float lsum = l[qi];
        lsum += __shfl_xor(lsum, 16, 64);
        lsum += __shfl_xor(lsum, 32, 64);
        const int q = q0 + 16 * qi + col;
        if (q < p.T) {
            const float inv = 1.0f / lsum;
#pragma unroll
            for (int db = 0; db < 8; ++db) {
                const h4 o = {(_Float16)(acc[qi][db][0] * inv), (_Float16)(acc[qi][db][1] * inv),
                              (_Float16)(acc[qi][db][2] * inv), (_Float16)(acc[qi][db][3] * inv)};
                *reinterpret_cast<h4 *>(p.out + (size_t)q * p.H + (size_t)head * AD + 16 * db + 4 * g) = o;
            }
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
    hipLaunchKernelGGL(attn_prep_kernel, dim3(a.Tp / PT, n_heads), dim3(256), 0, st, a);
    int rc = (int)hipGetLastError();
    if (rc != 0)
        return rc;
    a.NQ = (T + QT - 1) / QT;
    a.heads = n_heads;
    hipLaunchKernelGGL(attn_prefill_kernel, dim3(a.NQ * n_heads), dim3(256), 0, st, a);
    return (int)hipGetLastError();
}
