// Decode path: dequant-GEMV for 1 <= M <= 16 rows of activations.
//
// The served hybrid model generates one token at a time on a memory-constrained
// device (FlexQuant, arXiv 2501.07139, Section "Introduction"), so these kernels
// are bound by streaming the packed weights once.  The columns of a 16x16x32
// MFMA hold the M activation rows, its rows sixteen weight rows; a lane's packed
// chunk is already the A operand of four consecutive k-steps.
//
// Streaming kernel (used whenever the activations fit in LDS, i.e. for decode):
//  - Persistent workgroups, as many as fit on the chip, each walking supertile rows of the
//    matrix (or of up to three matrices that share the same input, so that q/k/v or
//    gate/up go out in one launch).  The eight wavefronts of a workgroup interleave
//    over the groups of a supertile row and every wavefront keeps DEPTH groups of
//    packed planes in flight (128-bit loads, 1 KiB contiguous per wavefront), also
//    across supertile rows, so the HBM stream never drains between rows.
//  - The unpack is only the field extraction: a pair of codes becomes two fp16
//    numbers 1024 + code*2^p by one and-or and goes to the matrix core as is.  The
//    activations are staged in LDS already divided by 2^p (exact: a power of two),
//    so the MFMA result is  sum_k x_k code_k + 1024 * sum_k x'_k.  The second term
//    does not depend on the weight row: it is computed once per group while
//    staging, together with sum_k x_k, and the group's contribution is
//        scale * (P - 1024*sum x' - zero * sum x)
//    in fp32: per weight there is neither a subtract nor a multiply, and any fp16
//    zero (integer or not) is handled the same.
//  - Bit-width dispatch happens once per workgroup; each bit-width has its own
//    fully specialised body.
//  - Wavefronts reduce through LDS in a fixed order: results are deterministic.
//
// Generic kernel: same arithmetic as the GEMM (exact code - zero in fp16), x read
// from global memory; used when M*K is too large for LDS.
#include "fq_device.h"
#include "fq_internal.h"

namespace {

// ------------------------------------------------------------------ generic
template <int BITS, int NWAVES>
__global__ __launch_bounds__(64 * NWAVES) void gemv_generic_kernel(const _Float16 *__restrict__ x, int M,
                                                                   const uint32_t *__restrict__ packed,
                                                                   const _Float16 *__restrict__ scales,
                                                                   const _Float16 *__restrict__ zeros, int N, int K,
                                                                   _Float16 *__restrict__ out)
{
    constexpr int SUB = Fmt<BITS>::SUB;
    constexpr int TILE = tile_dwords<BITS>();
    const int G = K >> 7;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int rb = blockIdx.x; // supertile row
    const int m = lane & 15;   // activation row this lane feeds / receives
    const int c = lane >> 4;   // k slice
    const uint32_t *tiles = packed + (size_t)rb * G * TILE;

    f4 acc[SUB];
#pragma unroll
    for (int u = 0; u < SUB; ++u)
        acc[u] = f4{0.f, 0.f, 0.f, 0.f};

    for (int g = wave; g < G; g += NWAVES) {
        const uint32_t *tile = tiles + (size_t)g * TILE;
        h8 xf[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            if (m < M)
                xf[s] = *reinterpret_cast<const h8 *>(x + (size_t)m * K + g * 128 + 32 * s + 8 * c);
            else
                xf[s] = h8{0, 0, 0, 0, 0, 0, 0, 0};
        }
#pragma unroll
        for (int u = 0; u < SUB; ++u) {
            uint32_t C[BITS];
            load_chunk<BITS>(tile, u, lane, C);
            const size_t meta = ((size_t)(rb * SUB + u) * G + g) * 16;
            const _Float16 z = zeros[meta + (lane & 15)];
            const h4 sc = *reinterpret_cast<const h4 *>(scales + meta + 4 * c);
            h2 q[16];
            unpack_codes<BITS>(C, q);
            const h2 z2 = {z, z};
#pragma unroll
            for (int i = 0; i < 16; ++i)
                q[i] = q[i] - z2;
            f4 p = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < 4; ++s)
                p = mfma16x16x32(make_h8(q[4 * s], q[4 * s + 1], q[4 * s + 2], q[4 * s + 3]), xf[s], p);
#pragma unroll
            for (int v = 0; v < 4; ++v)
                acc[u][v] += (float)sc[v] * p[v];
        }
    }

    __shared__ float red[NWAVES][SUB * 4][64];
#pragma unroll
    for (int u = 0; u < SUB; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v)
            red[wave][u * 4 + v][lane] = acc[u][v];
    __syncthreads();
    if (wave == 0 && m < M) {
#pragma unroll
        for (int u = 0; u < SUB; ++u) {
            const int n0 = rb * Fmt<BITS>::ROWS + 16 * u + 4 * c;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                float sum = 0.f;
#pragma unroll
                for (int w = 0; w < NWAVES; ++w)
                    sum += red[w][u * 4 + v][lane];
                if (n0 + v < N)
                    out[(size_t)m * N + n0 + v] = (_Float16)sum;
            }
        }
    }
}

template <int BITS>
int launch_generic(const void *x, int M, const fq_packed_ref &w, void *out, fq_stream st)
{
    constexpr int NWAVES = 4;
    const int Np = (w.N + 63) / 64 * 64;
    dim3 grid(Np / Fmt<BITS>::ROWS), block(64 * NWAVES);
    hipLaunchKernelGGL((gemv_generic_kernel<BITS, NWAVES>), grid, block, 0, st, static_cast<const _Float16 *>(x), M,
                       static_cast<const uint32_t *>(w.packed), static_cast<const _Float16 *>(w.scales),
                       static_cast<const _Float16 *>(w.zeros), w.N, w.K, static_cast<_Float16 *>(out));
    return (int)hipGetLastError();
}

// ---------------------------------------------------------------- streaming
constexpr int GNW = 8; // wavefronts per workgroup

// Groups in flight per wavefront.  HBM throughput here follows the bytes in flight (about 3 us of loaded
// latency): 16 wavefronts per CU times 4-6 KiB each.
template <int BITS>
struct GemvDepth { static constexpr int D = (BITS == 3) ? 2 : (BITS == 8 ? 3 : 4); };

struct GemvJob {
    const uint32_t *packed;
    const _Float16 *scales, *zeros;
    _Float16 *out;
    int N, bits;
    int blk0, nblk; // the workgroups [blk0, blk0 + nblk) of the launch serve this matrix
};

struct GemvJobs {
    GemvJob j[3];
    int count;
};

// Where the linear's input x comes from.  The row-wise steps between the linears of the block are
// folded into the staging of x (rms(t) = t / sqrt(mean(t^2) + 1e-5), results rounded to fp16 where
// the block stores an fp16 tensor):
//   0: x = a                      1: x = rms(a)                 2: x = rms(a + b + c)
//   3: aux = a + b, x = rms(aux)  4: x = rms(silu(a) * b)       5: aux = rms(a + b), x = rms(aux)
// aux (fp16 [M,K]) is written by workgroup 0 only.
struct GemvInput {
    const _Float16 *a, *b, *c;
    _Float16 *aux;
    int mode;
};


// Sum over the workgroup, the same value in every thread (two barriers).
__device__ __forceinline__ float gemv_block_sum(float v, float *part)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1)
        v += __shfl_xor(v, o, 64);
    __syncthreads();
    if ((threadIdx.x & 63) == 0)
        part[threadIdx.x >> 6] = v;
    __syncthreads();
    float sum = 0.f;
#pragma unroll
    for (int w = 0; w < GNW; ++w)
        sum += part[w];
    return sum;
}

template <int BITS>
struct GemvSlot {
    u4v plane[Fmt<BITS>::PLANES];
    h4 scale[Fmt<BITS>::SUB], zero[Fmt<BITS>::SUB];
};

// 2^-pair_shift for element e of k-step s: the factor applied to x while staging.
template <int BITS>
__device__ __forceinline__ float stage_factor(int s, int e)
{
    if constexpr (BITS == 8) {
        return 1.0f;
    } else if constexpr (BITS == 4) {
        return ((e >> 1) & 1) ? 0.0625f : 1.0f;
    } else if constexpr (BITS == 2) {
        constexpr float f[8] = {1.0f, 0.25f, 0.0625f, 0.015625f, 0.00390625f, 1.0f, 0.25f, 0.0625f};
        return f[4 * (s & 1) + (e >> 1)];
    } else {
        constexpr float f[16] = {1.0f, 0.125f, 0.015625f, 1.0f, 0.125f, 1.0f, 0.125f, 0.015625f,
                                 1.0f, 0.125f, 1.0f, 0.125f, 0.015625f, 1.0f, 0.125f, 1.0f};
        return f[4 * s + (e >> 1)];
    }
}

// Position in the stream of (supertile row, group) items of one wavefront.
struct GemvCursor {
    int j, t; // j-th supertile row of this workgroup, t-th group of this wavefront in it
};

template <int BITS>
__device__ __forceinline__ void gemv_body(const GemvJob &job, int bj, const GemvInput &in, int M, int K,
                                          unsigned char *smem, float *part)
{
    constexpr int SUB = Fmt<BITS>::SUB, ROWS = Fmt<BITS>::ROWS, D = GemvDepth<BITS>::D, TILE = tile_dwords<BITS>();
    const int G = K >> 7;
    h8 *xl = reinterpret_cast<h8 *>(smem);                             // [K/8][M] staged activations
    float *xsum = reinterpret_cast<float *>(smem + (size_t)M * K * 2); // [G][M] sum of x over the group
    float *csum = xsum + (size_t)G * M;                                // [G][M] 1024 * sum of staged x
    float *red = csum + (size_t)G * M;                                 // [2][GNW][SUB*4][64]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6); // scalar: keeps tile addressing in SGPRs
    const int m = lane & 15, c = lane >> 4;
    const int NRB = ((job.N + 63) / 64 * 64) / ROWS;
    const int T = (G + GNW - 1) / GNW;                                 // groups per wavefront and supertile row
    const int J = bj < NRB ? (NRB - bj + job.nblk - 1) / job.nblk : 0; // supertile rows of this workgroup
    const int I = J * T;

    if (J == 0)
        return; // uniform: nothing to do for this workgroup

    // Loads are unconditional (indices clamped into the matrix) so that the number of loads in flight is
    // known at compile time and a wavefront only ever waits for the oldest slot of its ring.
    GemvSlot<BITS> ring[D];
    GemvCursor pre = {0, 0};
    auto issue = [&](GemvSlot<BITS> &sl) {
        const int g = min(wave + GNW * pre.t, G - 1);
        const int rb = bj + min(pre.j, J - 1) * job.nblk;
        const uint32_t *tile = job.packed + ((size_t)rb * G + g) * TILE;
#pragma unroll
        for (int p = 0; p < Fmt<BITS>::PLANES; ++p)
            sl.plane[p] = *reinterpret_cast<const u4v *>(tile + p * 256 + lane * 4);
#pragma unroll
        for (int u = 0; u < SUB; ++u) {
            const size_t meta = ((size_t)(rb * SUB + u) * G + g) * 16 + 4 * c;
            sl.scale[u] = *reinterpret_cast<const h4 *>(job.scales + meta);
            sl.zero[u] = *reinterpret_cast<const h4 *>(job.zeros + meta);
        }
        if (++pre.t == T) {
            pre.t = 0;
            ++pre.j;
        }
    };
    // weights first: they do not depend on the staging below
#pragma unroll
    for (int d = 0; d < D; ++d)
        issue(ring[d]);

    // stage x, one activation row at a time: the input transform of the block (see GemvInput) runs here,
    // in every workgroup alike, so that the row-wise glue between two linears costs no launch of its own.
    // The inputs are re-read (from L2) in each pass instead of being held in registers.
    // Chunk kc of row mm (8 halves at k = 8*kc) goes to xl[kc*M + mm], divided by 2^p.
    const int chunks = K >> 3;
    for (int mm = 0; mm < M; ++mm) {
        const size_t row = (size_t)mm * K;
        auto base = [&](int kc, float (&v)[8]) {
            const h8 va = *reinterpret_cast<const h8 *>(in.a + row + kc * 8);
            h8 vb = va, vc = va;
            if (in.mode >= 2)
                vb = *reinterpret_cast<const h8 *>(in.b + row + kc * 8);
            if (in.mode == 2)
                vc = *reinterpret_cast<const h8 *>(in.c + row + kc * 8);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float t = (float)va[e];
                if (in.mode == 2)
                    t = t + (float)vb[e] + (float)vc[e];
                else if (in.mode == 3)
                    t = (float)(_Float16)(t + (float)vb[e]); // the sum is a stored fp16 tensor
                else if (in.mode == 4)
                    t = t / (1.0f + __expf(-t)) * (float)vb[e];
                else if (in.mode == 5)
                    t = t + (float)vb[e];
                v[e] = t;
            }
        };
        float inv1 = 1.0f, inv2 = 1.0f;
        if (in.mode != 0) {
            float ss = 0.f;
            for (int kc = tid; kc < chunks; kc += 64 * GNW) {
                float v[8];
                base(kc, v);
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    ss += v[e] * v[e];
            }
            inv1 = 1.0f / sqrtf(gemv_block_sum(ss, part) / (float)K + 1e-5f);
            if (in.mode == 5) { // rms twice: the first result is the stored fp16 block output
                ss = 0.f;
                for (int kc = tid; kc < chunks; kc += 64 * GNW) {
                    float v[8];
                    base(kc, v);
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float y = (float)(_Float16)(v[e] * inv1);
                        ss += y * y;
                    }
                }
                inv2 = 1.0f / sqrtf(gemv_block_sum(ss, part) / (float)K + 1e-5f);
            }
        }
        for (int kc = tid; kc < chunks; kc += 64 * GNW) { // all 16 lanes of a group take the same trips
            float v[8];
            base(kc, v);
            if (in.mode == 5) {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    v[e] = (float)(_Float16)(v[e] * inv1);
            }
            if ((in.mode == 3 || in.mode == 5) && blockIdx.x == 0) {
                h8 o;
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    o[e] = (_Float16)v[e]; // exact: already fp16 values
                *reinterpret_cast<h8 *>(in.aux + row + kc * 8) = o;
            }
            const float inv = in.mode == 5 ? inv2 : inv1;
            const int s = (kc >> 2) & 3;
            h8 w;
            float sx = 0.f, sc = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float xe = in.mode == 0 ? v[e] : (float)(_Float16)(v[e] * inv);
                w[e] = (_Float16)(xe * stage_factor<BITS>(s, e));
                sx += xe;
                sc += (float)w[e];
            }
            xl[(size_t)kc * M + mm] = w;
#pragma unroll
            for (int o = 8; o > 0; o >>= 1) {
                sx += __shfl_xor(sx, o, 64);
                sc += __shfl_xor(sc, o, 64);
            }
            if ((kc & 15) == 0) {
                xsum[(kc >> 4) * M + mm] = sx;
                csum[(kc >> 4) * M + mm] = 1024.0f * sc;
            }
        }
    }
    __syncthreads();

    f4 acc[SUB];
#pragma unroll
    for (int u = 0; u < SUB; ++u)
        acc[u] = f4{0.f, 0.f, 0.f, 0.f};

    const bool live = m < M;
    const int mc = min(m, M - 1), xlane = c * M + mc;
    GemvCursor cur = {0, 0};
    for (int i0 = 0; i0 < I; i0 += D) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const int g = wave + GNW * cur.t;
            const bool valid = (i0 + d < I) && (g < G); // past the end the slot holds a clamped reload: skipped
            if (valid) {
                // lanes of the unused MFMA columns (m >= M) repeat column M-1; their results are never stored
                const h8 *xg_ptr = xl + (size_t)g * 16 * M + xlane;
                h8 bx[4];
#pragma unroll
                for (int s = 0; s < 4; ++s)
                    bx[s] = xg_ptr[s * 4 * M];
                const float xg = xsum[g * M + mc], ncg = -csum[g * M + mc];
                uint32_t dw[4 * Fmt<BITS>::PLANES];
#pragma unroll
                for (int p = 0; p < Fmt<BITS>::PLANES; ++p) {
                    dw[4 * p + 0] = ring[d].plane[p].x; dw[4 * p + 1] = ring[d].plane[p].y;
                    dw[4 * p + 2] = ring[d].plane[p].z; dw[4 * p + 3] = ring[d].plane[p].w;
                }
#pragma unroll
                for (int u = 0; u < SUB; ++u) {
                    uint32_t C[BITS], h[16];
#pragma unroll
                    for (int i = 0; i < BITS; ++i)
                        C[i] = dw[BITS * u + i];
                    extract_biased<BITS>(C, h);
                    f4 p = {ncg, ncg, ncg, ncg}; // the bias term leaves with the accumulator's start value
#pragma unroll
                    for (int s = 0; s < 4; ++s)
                        p = mfma16x16x32(make_h8_bits(h[4 * s], h[4 * s + 1], h[4 * s + 2], h[4 * s + 3]), bx[s], p);
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const float t = fmaf(-(float)ring[d].zero[u][v], xg, p[v]);
                        acc[u][v] = fmaf((float)ring[d].scale[u][v], t, acc[u][v]);
                    }
                }
            }
            issue(ring[d]); // the item D places ahead reuses this slot
            if (i0 + d < I && ++cur.t == T) {
                // end of a supertile row: fixed-order reduction over the wavefronts, double-buffered
                float *rbuf = red + (size_t)(cur.j & 1) * GNW * SUB * 4 * 64;
#pragma unroll
                for (int u = 0; u < SUB; ++u)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        rbuf[(wave * SUB * 4 + u * 4 + v) * 64 + lane] = acc[u][v];
                        acc[u][v] = 0.f;
                    }
                __syncthreads();
                const int rb = bj + cur.j * job.nblk;
                if (live) {
                    for (int e = wave; e < SUB * 4; e += GNW) {
                        float sum = 0.f;
#pragma unroll
                        for (int w = 0; w < GNW; ++w)
                            sum += rbuf[(w * SUB * 4 + e) * 64 + lane];
                        const int n = rb * ROWS + 16 * (e >> 2) + 4 * c + (e & 3);
                        if (n < job.N)
                            job.out[(size_t)m * job.N + n] = (_Float16)sum;
                    }
                }
                cur.t = 0;
                ++cur.j;
            }
        }
    }
}

__global__ __launch_bounds__(64 * GNW, 2) void gemv_stream_kernel(GemvInput in, int M, int K, GemvJobs jobs)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    __shared__ float part[GNW];
    int ji = 0;
#pragma unroll
    for (int i = 1; i < 3; ++i)
        if (i < jobs.count && (int)blockIdx.x >= jobs.j[i].blk0)
            ji = i;
    const GemvJob &job = jobs.j[ji];
    const int bj = blockIdx.x - job.blk0;
    switch (job.bits) { // uniform across the workgroup
    case 2: gemv_body<2>(job, bj, in, M, K, smem, part); break;
    case 3: gemv_body<3>(job, bj, in, M, K, smem, part); break;
    case 4: gemv_body<4>(job, bj, in, M, K, smem, part); break;
    default: gemv_body<8>(job, bj, in, M, K, smem, part); break;
    }
}

constexpr size_t GEMV_MAX_LDS = 152 * 1024;

size_t gemv_stream_lds(int M, int K, int bits)
{
    const int sub = bits == 3 ? 4 : (bits == 2 ? 2 : 1);
    return (size_t)M * K * 2 + 2 * (size_t)(K >> 7) * M * 4 + 2 * (size_t)GNW * sub * 4 * 64 * 4;
}

int rows_per_supertile(int bits) { return bits == 2 ? 32 : (bits == 3 ? 64 : 16); }

// Resident workgroups of the streaming kernel on the device.
int gemv_resident_blocks(size_t lds, int *out)
{
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, n = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess)
            return (int)e;
        e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess)
            return (int)e;
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(gemv_stream_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)GEMV_MAX_LDS);
        if (e != hipSuccess)
            return (int)e;
        cus = n;
    }
    // the answer depends only on the LDS request: remember the last few
    static size_t seen_lds[8];
    static int seen_blocks[8], seen = 0;
    for (int i = 0; i < seen; ++i)
        if (seen_lds[i] == lds) {
            *out = seen_blocks[i];
            return 0;
        }
    int per_cu = 0;
    hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, gemv_stream_kernel, 64 * GNW, lds);
    if (e != hipSuccess)
        return (int)e;
    *out = cus * (per_cu > 0 ? per_cu : 1);
    if (seen < 8) {
        seen_lds[seen] = lds;
        seen_blocks[seen++] = *out;
    }
    return 0;
}

} // namespace

bool fq_gemv_can_stream(int M, int K, int bits)
{
    return gemv_stream_lds(M, K, bits) <= GEMV_MAX_LDS;
}

// Up to three matrices that share the input (same K): one launch.
int fq_launch_gemv_multi(const fq_gemv_input &src, int M, const fq_packed_ref *w, void *const *outs, int count,
                         fq_stream st)
{
    GemvJobs jobs;
    jobs.count = count;
    size_t lds = 0;
    double bytes[3], total = 0;
    int nrb[3], sum_nrb = 0;
    for (int i = 0; i < count; ++i) {
        const size_t need = gemv_stream_lds(M, w[i].K, w[i].bits);
        lds = lds > need ? lds : need;
        nrb[i] = ((w[i].N + 63) / 64 * 64) / rows_per_supertile(w[i].bits);
        sum_nrb += nrb[i];
        bytes[i] = (double)w[i].N * w[i].K * w[i].bits;
        total += bytes[i];
    }
    int resident = 0;
    if (int e = gemv_resident_blocks(lds, &resident))
        return e;
    int grid = sum_nrb < resident ? sum_nrb : resident;
    if (grid < count)
        grid = count;
    // share the workgroups among the matrices in proportion to their packed bytes
    int left = grid, blk0 = 0;
    for (int i = 0; i < count; ++i) {
        int nb = (i == count - 1) ? left : (int)(grid * bytes[i] / total + 0.5);
        const int reserve = count - 1 - i; // one workgroup at least for every later matrix
        if (nb > left - reserve)
            nb = left - reserve;
        if (nb > nrb[i])
            nb = nrb[i];
        if (nb < 1)
            nb = 1;
        jobs.j[i] = GemvJob{static_cast<const uint32_t *>(w[i].packed), static_cast<const _Float16 *>(w[i].scales),
                            static_cast<const _Float16 *>(w[i].zeros), static_cast<_Float16 *>(outs[i]), w[i].N,
                            w[i].bits, blk0, nb};
        blk0 += nb;
        left -= nb;
    }
    for (int i = count; i < 3; ++i)
        jobs.j[i] = GemvJob{nullptr, nullptr, nullptr, nullptr, 0, 0, blk0, 0};
    const GemvInput in = {static_cast<const _Float16 *>(src.a), static_cast<const _Float16 *>(src.b),
                          static_cast<const _Float16 *>(src.c), static_cast<_Float16 *>(src.aux), src.mode};
    hipLaunchKernelGGL(gemv_stream_kernel, dim3(blk0), dim3(64 * GNW), lds, st, in, M, w[0].K, jobs);
    return (int)hipGetLastError();
}

int fq_launch_gemv(const void *x, int M, const fq_packed_ref &w, void *out, fq_stream st)
{
    if (fq_gemv_can_stream(M, w.K, w.bits)) {
        const fq_gemv_input src = {x, nullptr, nullptr, nullptr, 0};
        return fq_launch_gemv_multi(src, M, &w, &out, 1, st);
    }
    switch (w.bits) {
    case 2: return launch_generic<2>(x, M, w, out, st);
    case 3: return launch_generic<3>(x, M, w, out, st);
    case 4: return launch_generic<4>(x, M, w, out, st);
    default: return launch_generic<8>(x, M, w, out, st);
    }
}
