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
//    activations are staged in LDS as x'_k = x_k * 2^(E - p): E is chosen per group
//    of 128 so that the group's largest |x| lands in [2^14, 2^15), which keeps every
//    value within 2^-20 of that maximum a normal fp16 number whatever the scale of
//    the activations (without it, dividing small activations by 2^p would push them
//    into the subnormal range and lose bits).  The MFMA result is
//        P = 2^E * sum_k x_k code_k + 1024 * sum_k x'_k.
//    The second term does not depend on the weight row: it is computed once per
//    group while staging, together with sum_k x_k, and the group's contribution is
//        scale * (2^-E * (P - 1024*sum x') - zero * sum x)
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
#include "fq_stage.h"

#include <mutex>

namespace {

// ------------------------------------------------------------------ generic
template <int BITS, int NWAVES>
__global__ __launch_bounds__(64 * NWAVES) void gemv_generic_kernel(const _Float16 *__restrict__ x, int M,
                                                                   const uint32_t *__restrict__ packed,
                                                                   const _Float16 *__restrict__ scales,
                                                                   const _Float16 *__restrict__ zeros, int N, int K,
                                                                   _Float16 *__restrict__ out, int ld)
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
                    out[(size_t)m * ld + n0 + v] = (_Float16)sum;
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
                       static_cast<const _Float16 *>(w.zeros), w.N, w.K, static_cast<_Float16 *>(out), w.ld ? w.ld : w.N);
    return (int)hipGetLastError();
}

// ---------------------------------------------------------------- streaming
#ifndef FQ_GNW
#define FQ_GNW 8
#endif
constexpr int GNW = FQ_GNW; // wavefronts per workgroup

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
    int split;      // 2- and 3-bit only: work units are the 16-row sub-blocks of a supertile row, not whole rows
    int ld;         // elements between consecutive rows of out (N, or more when out is a column range of a wider array)
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
//   6: x = silu(a) * b (no norm: the MLP of a real decoder block)
// aux (fp16 [M,K]) is written by workgroup 0 only.
struct GemvInput {
    const _Float16 *a, *b, *c;
    _Float16 *aux;
    int mode;
};


// Sum over the workgroup, the same value in every thread.  part holds two sets of per-wavefront
// partials used in turn (which = 0, 1, 0, ...), so one barrier per sum is enough: a wavefront can only
// be two sums ahead of another after passing the barrier of the sum in between.
__device__ __forceinline__ float gemv_block_sum(float v, float *part, int which)
{
    v = row16_sum(v);
    v += __shfl_xor(v, 16, 64);
    v += __shfl_xor(v, 32, 64);
    if ((threadIdx.x & 63) == 0)
        part[which * GNW + (threadIdx.x >> 6)] = v;
    lds_barrier();
    float sum = 0.f;
#pragma unroll
    for (int w = 0; w < GNW; ++w)
        sum += part[which * GNW + w];
    return sum;
}

// One (work unit, group) item in flight: the packed dwords a lane owns and the scales and zeros.  A unit
// is S sub-blocks of 16 weight rows: a whole supertile row (whole planes, 128-bit loads), or a single
// sub-block of a 2- or 3-bit supertile row (just its BITS dwords).
// Scales and zeros: the item needs 2S values per weight row (value 2u the scale, 2u+1 the zero of sub-block
// u), and every lane of a row's column (lane % 16) would load the same ones.  Instead the four 16-lane
// groups of the wavefront load four different values with ONE instruction (lane group c of load q fetches
// value 4q + c for row lane % 16), and the lanes that need a value take it from its group with a cross-lane
// read when the item runs: a quarter of the vector-memory instructions, which is what this kernel is short of
// (measured: without any scale or zero loads a 7B-shaped decode block takes 36.0 us instead of 41.4).
template <int BITS, int S>
struct GemvSlot {
    static constexpr bool WHOLE = S == Fmt<BITS>::SUB;
    static constexpr int NMETA = (2 * S + 3) / 4;
    u4v plane[WHOLE ? Fmt<BITS>::PLANES : 1];
    uint32_t w[WHOLE ? 1 : BITS];
    uint32_t meta[NMETA]; // fp16 bits: in lane group c of meta[q], value 4q + c of weight row lane % 16
};

// Position in the stream of (work unit, group) items of one wavefront.
struct GemvCursor {
    int ub, t; // work unit, t-th group of this wavefront in it
};

// MV: activation rows a lane finishes per sub-block (1 when M == 1, else 4).
// S: sub-blocks per work unit (all of a supertile row's, or 1).  With F = SUB/S units per supertile row,
// unit ub is part (ub/8) % F of supertile row (ub / (8F)) * 8 + ub % 8: the F workgroups that share a
// supertile row (and read the same cache lines) are 8 apart, i.e. on the same XCD and L2.
template <int BITS, int MODE, int MV, int S>
__device__ __forceinline__ void gemv_body(const GemvJob job, int bj, const GemvInput in, int M, int K,
                                          unsigned char *smem, float *part)
{
    constexpr int SUB = Fmt<BITS>::SUB, ROWS = Fmt<BITS>::ROWS, D = GemvDepth<BITS>::D, TILE = tile_dwords<BITS>();
    constexpr int NIN = GemvInputs<MODE>::N, STEP = 64 * GNW;
    constexpr int F = SUB / S;
    constexpr bool WHOLE = F == 1;
    constexpr int NMETA = GemvSlot<BITS, S>::NMETA;
    const int G = K >> 7;
    const int T = (G + GNW - 1) / GNW; // groups per wavefront and supertile row
    const int GP = T * GNW;            // groups rounded up to whole turns of the wavefronts: the rest is zero
    h8 *xl = reinterpret_cast<h8 *>(smem);                                   // [GP*16][M] staged activations
    float *xsum = reinterpret_cast<float *>(smem + (size_t)GP * 16 * M * 16); // [GP][16] sum of x over the group
    float *csum = xsum + (size_t)GP * 16;                                    // [GP][16] 2^-E * 1024 * sum of staged x
    float *esc = csum + (size_t)GP * 16;                                     // [GP][16] 2^-E of the group
    float *red = esc + (size_t)GP * 16;                                      // [2][GNW][S*MV][64]
    h8 *raw = reinterpret_cast<h8 *>(red); // [NIN][trips][STEP] raw input row; free again before the first reduction

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6); // scalar: keeps tile addressing in SGPRs
    const int NRB = ((job.N + 63) / 64 * 64) / ROWS;
    const int NU = WHOLE ? NRB : (NRB + 7) / 8 * 8 * F; // work units (with F > 1 some may lie past the matrix)
    const int nblk = job.nblk;
    const uint32_t *const packed = job.packed;
    const _Float16 *const scales = job.scales, *const zeros = job.zeros;

    if (bj >= NU) {
        __builtin_amdgcn_s_waitcnt(FQ_WAIT_VMCNT0); // the kernel's copies into this workgroup's LDS land before it ends
        return;                                     // uniform: nothing to do for this workgroup
    }
    auto unit_row = [&](int ub) { return WHOLE ? ub : (ub / (8 * F)) * 8 + (ub & 7); };
    auto unit_part = [&](int ub) { return WHOLE ? 0 : (ub >> 3) & (F - 1); };

    // ---- the input row is on its way already: the kernel issued its copies from global memory straight into
    // `raw` (no registers) before it looked at its job; the staging below waits for these copies only, not
    // for the weights issued behind them.
    const int chunks = K >> 3, trips = (chunks + STEP - 1) / STEP;
    const _Float16 *const src[3] = {in.a, in.b, in.c};
    // The copies land before any weight load is issued.  Measured against the other order (weights issued behind
    // the copies and left in flight by a counted wait): the same or slightly faster, and nothing here depends
    // on how many loads the compiler places where.
    __builtin_amdgcn_s_waitcnt(FQ_WAIT_VMCNT0);
    lds_barrier();

    // ---- weights: unconditional loads (indices clamped into the matrix) so that a wavefront only
    // ever waits for the oldest slot of its ring.
    // Addresses: a per-unit base, recomputed when the stream moves to the next unit, plus a 32-bit
    // offset for the group, plus the lane's own offset.  Units past the end read supertile row 0.
    const uint32_t plane_off = (uint32_t)lane * 4u;
    const size_t row_tiles = (size_t)G * TILE;
    const uint32_t *tile_row;
    const uint16_t *meta_lane[NMETA]; // this lane's scale or zero (see GemvSlot) of group 0 of the unit
    int pre_part;
    auto set_unit = [&](int ub) {
        const int r = unit_row(ub), rb = (ub < NU && r < NRB) ? r : 0;
        pre_part = unit_part(ub);
        tile_row = packed + (size_t)rb * row_tiles;
        const size_t meta = (size_t)(rb * SUB + pre_part * S) * G * 16;
#pragma unroll
        for (int q = 0; q < NMETA; ++q) {
            const int vi = 4 * q + (lane >> 4), u = min(vi >> 1, S - 1); // values past 2S repeat the last sub-block's
            meta_lane[q] = reinterpret_cast<const uint16_t *>((vi & 1) ? zeros : scales) + meta + (size_t)u * G * 16 + (lane & 15);
        }
    };
    GemvSlot<BITS, S> ring[D];
    GemvCursor pre = {bj, 0};
    set_unit(bj);
    auto issue = [&](GemvSlot<BITS, S> &sl) {
        const uint32_t g = (uint32_t)min(wave + GNW * pre.t, G - 1);
        const uint32_t *tile = tile_row + g * (uint32_t)TILE;
        if constexpr (WHOLE) {
#pragma unroll
            for (int p = 0; p < Fmt<BITS>::PLANES; ++p)
                sl.plane[p] = *reinterpret_cast<const u4v *>(tile + p * 256 + plane_off);
        } else if constexpr (BITS == 2) {
            const u2v v = *reinterpret_cast<const u2v *>(tile + plane_off + 2 * pre_part);
            sl.w[0] = v.x;
            sl.w[1] = v.y;
        } else {
#pragma unroll
            for (int i = 0; i < BITS; ++i) {
                const int j = BITS * pre_part + i; // dword j of the lane: plane j / 4, component j % 4
                sl.w[i] = tile[(j >> 2) * 256 + plane_off + (j & 3)];
            }
        }
#pragma unroll
        for (int q = 0; q < NMETA; ++q)
            sl.meta[q] = meta_lane[q][g * 16u];
        if (++pre.t == T) {
            pre.t = 0;
            pre.ub += nblk;
            set_unit(pre.ub);
        }
    };
#pragma unroll
    for (int d = 0; d < D; ++d) {
        issue(ring[d]);
        __builtin_amdgcn_sched_barrier(0); // slot by slot, the order in which the loop below waits for them
    }

    // ---- stage x, one activation row at a time: the input transform of the block (see GemvInput) runs
    // here, in every workgroup alike, so that the row-wise glue between two linears costs no launch of
    // its own.  Chunk kc of row mm (8 halves at k = 8*kc) goes to xl[kc*M + mm], divided by 2^p.
    // MODE 4 (the expensive transform) is evaluated once: the first pass over the row leaves the eight
    // fp32 products in the two 16-byte slots of its inputs, which only this thread touches.
    using Chunk = GemvChunk<MODE>;
    auto fetch = [&](int t, Chunk &v, bool first) { // this thread's chunk of trip t, combined
        h8 r[NIN];
#pragma unroll
        for (int i = 0; i < NIN; ++i)
            r[i] = raw[(i * trips + t) * STEP + tid];
        if constexpr (MODE == 4) {
            if (first) {
                gemv_combine<MODE>(r, v);
                if (t > 0) { // trip 0 stays in registers
                    raw[t * STEP + tid] = __builtin_bit_cast(h8, f4{v.f[0], v.f[1], v.f[2], v.f[3]});
                    raw[(trips + t) * STEP + tid] = __builtin_bit_cast(h8, f4{v.f[4], v.f[5], v.f[6], v.f[7]});
                }
            } else {
                const f4 lo = __builtin_bit_cast(f4, r[0]), hi = __builtin_bit_cast(f4, r[1]);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    v.f[e] = lo[e];
                    v.f[4 + e] = hi[e];
                }
            }
        } else {
            gemv_combine<MODE>(r, v);
        }
    };
    // The chunk of trip 0 stays in registers between the passes over the row (it is the whole row up
    // to K = 4096); later trips are fetched from LDS again.
    int sums = 0; // block sums taken so far: selects the partials' buffer
    auto stage_row = [&](int mm) {
        Chunk v0;
        const bool has0 = tid < chunks;
        if (has0)
            fetch(0, v0, true);
        float inv1 = 1.0f, inv2 = 1.0f;
        if constexpr (MODE != 0 && MODE != 6) {
            // sum of squares of the row; second: of the fp16 result of the first rms
            auto squares = [&](bool second) {
                float ss = 0.f;
                auto add = [&](const Chunk &v) {
                    if constexpr (Chunk::HALF) {
                        ss = gemv_sumsq(v.h, ss);
                    } else if (second) {
                        ss = gemv_sumsq(gemv_scaled(v.f, inv1), ss);
                    } else {
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            ss = fmaf(v.f[e], v.f[e], ss);
                    }
                };
                if (has0)
                    add(v0);
                for (int t = 1; t < trips; ++t)
                    if (tid + STEP * t < chunks) {
                        Chunk v;
                        fetch(t, v, !second);
                        add(v);
                    }
                return ss;
            };
            inv1 = 1.0f / sqrtf(gemv_block_sum(squares(false), part, sums++ & 1) / (float)K + 1e-5f);
            if constexpr (MODE == 5) // rms twice: the first result is the stored fp16 block output
                inv2 = 1.0f / sqrtf(gemv_block_sum(squares(true), part, sums++ & 1) / (float)K + 1e-5f);
        }
        // writes one chunk of x to LDS, and the group sums (the 16 lanes that share a group are all here:
        // chunks is a multiple of 16)
        auto put = [&](int kc, const Chunk &v) {
            h8 xe; // the linear's input, fp16
            if constexpr (MODE == 0) {
                xe = v.h;
            } else if constexpr (MODE == 5) {
                const h8 y = gemv_scaled(v.f, inv1); // the stored block output
                if (blockIdx.x == 0)
                    *reinterpret_cast<h8 *>(in.aux + (size_t)mm * K + (size_t)kc * 8) = y;
                xe = gemv_scaled(y, inv2);
            } else if constexpr (Chunk::HALF) {
                if constexpr (MODE == 3) {
                    if (blockIdx.x == 0)
                        *reinterpret_cast<h8 *>(in.aux + (size_t)mm * K + (size_t)kc * 8) = v.h;
                }
                xe = gemv_scaled(v.h, inv1);
            } else {
                xe = gemv_scaled(v.f, inv1);
            }
            // the group's exponent: its largest |x| (exponent field ex, taken as 1 for zero and subnormal
            // maxima) is brought to 2^14: E = 29 - ex in [-1, 28]
            const int ex = min(max((int)(group_max_bits(xe) >> 10), 1), 30), E = 29 - ex;
            const h8 w = stage_scaled<BITS>(xe, (kc >> 2) & 3, E);
            xl[(size_t)kc * M + mm] = w;
            const float sx = row16_sum(gemv_sum(xe)), sc = row16_sum(gemv_sum(w));
            if ((kc & 15) == 0) {
                const float einv = __builtin_bit_cast(float, (uint32_t)(127 - E) << 23); // 2^-E
                xsum[(kc >> 4) * 16 + mm] = sx;
                csum[(kc >> 4) * 16 + mm] = einv * (1024.0f * sc); // exact scaling
                esc[(kc >> 4) * 16 + mm] = einv;
            }
        };
        if (has0)
            put(tid, v0);
        for (int t = 1; t < trips; ++t)
            if (tid + STEP * t < chunks) {
                Chunk v;
                fetch(t, v, false);
                put(tid + STEP * t, v);
            }
    };
    // Zero what no row writes: the groups past K (items on them then add nothing) and the sums of the
    // activation rows past M.
    for (int i = chunks * M + tid; i < GP * 16 * M; i += STEP)
        xl[i] = h8{0, 0, 0, 0, 0, 0, 0, 0};
    for (int i = tid; i < GP * 16; i += STEP)
        if ((i & 15) >= M || (i >> 4) >= G) {
            xsum[i] = 0.f;
            csum[i] = 0.f;
            esc[i] = 0.f;
        }
    stage_row(0);
    for (int mm = 1; mm < M; ++mm) {
        lds_barrier(); // every thread is done with the previous row
        for (int t = 0; t < trips; ++t) { // through registers: behind the weights whichever way
            const size_t off = (size_t)mm * K + (size_t)min(tid + STEP * t, chunks - 1) * 8;
#pragma unroll
            for (int i = 0; i < NIN; ++i)
                raw[(i * trips + t) * STEP + tid] = *reinterpret_cast<const h8 *>(src[i] + off);
        }
        lds_barrier();
        stage_row(mm);
    }
    lds_barrier(); // x is staged; the raw row (which shares LDS with the reduction buffers) is dead

    float acc[S][MV];
#pragma unroll
    for (int u = 0; u < S; ++u)
#pragma unroll
        for (int v = 0; v < MV; ++v)
            acc[u][v] = 0.f;

    // The activations are the A operand (rows = activation rows m), the packed weights the B operand
    // (columns = weight rows n): lane l receives D[m = 4*(l/16) + v][n = l%16], so one scale and one zero
    // per lane and sub-block finish its results, and with M == 1 only v = 0 is needed at all.
    // (the lane's coordinates are taken afresh here: carried across the staging they cost registers there)
    int lane2 = threadIdx.x & 63;
    asm volatile("" : "+v"(lane2));
    const int m = lane2 & 15, c = lane2 >> 4;
    const int mc = min(m, M - 1), xlane = c * M + mc; // lanes of unused A rows (m >= M) repeat row M-1
    int meta_from[4]; // byte index (lane * 4) of the lane of group k that holds this lane's weight row
#pragma unroll
    for (int k = 0; k < 4; ++k)
        meta_from[k] = (16 * k + (lane & 15)) * 4;
    GemvCursor cur = {bj, 0};
    int parity = 0;
    while (cur.ub < NU) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            // No branch around the item: past the end of a row the slot holds a clamped reload and the
            // item runs on it against the zeroed groups of x; past the last row its results are dropped.
            // With a branch, the compiler could not tell how many loads are in flight and waited for all.
            const int g = wave + GNW * cur.t;
            {
                const h8 *xg_ptr = xl + (size_t)g * 16 * M + xlane;
                h8 ax[4];
#pragma unroll
                for (int s = 0; s < 4; ++s)
                    ax[s] = xg_ptr[s * 4 * M];
                float xg[MV], cg[MV], eg[MV];
                if constexpr (MV == 4) {
                    const f4 a4 = *reinterpret_cast<const f4 *>(xsum + g * 16 + 4 * c);
                    const f4 c4 = *reinterpret_cast<const f4 *>(csum + g * 16 + 4 * c);
                    const f4 e4 = *reinterpret_cast<const f4 *>(esc + g * 16 + 4 * c);
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        xg[v] = a4[v];
                        cg[v] = c4[v];
                        eg[v] = e4[v];
                    }
                } else {
                    xg[0] = xsum[g * 16];
                    cg[0] = csum[g * 16];
                    eg[0] = esc[g * 16];
                }
#pragma unroll
                for (int u = 0; u < S; ++u) {
                    uint32_t C[BITS], h[16];
                    if constexpr (WHOLE) {
#pragma unroll
                        for (int i = 0; i < BITS; ++i) {
                            const int j = BITS * u + i;
                            const u4v pl = ring[d].plane[j >> 2];
                            C[i] = (j & 3) == 0 ? pl.x : ((j & 3) == 1 ? pl.y : ((j & 3) == 2 ? pl.z : pl.w));
                        }
                    } else {
#pragma unroll
                        for (int i = 0; i < BITS; ++i)
                            C[i] = ring[d].w[i];
                    }
                    extract_biased<BITS>(C, h);
                    f4 p = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int s = 0; s < 4; ++s)
                        p = mfma16x16x32(ax[s], make_h8_bits(h[4 * s], h[4 * s + 1], h[4 * s + 2], h[4 * s + 3]), p);
                    // p = 2^E sum x code + 1024 sum x': back to the scale of x (exact), take the bias and
                    // zero * sum x away, then scale
                    // value 2u (scale) and 2u+1 (zero) of this lane's weight row, from the lane group that loaded it;
                    // with one activation row only lanes 0..15 count, and they hold value 0 themselves
                    const uint32_t sraw = (MV == 1 && u == 0)
                                              ? ring[d].meta[0]
                                              : (uint32_t)__builtin_amdgcn_ds_bpermute(meta_from[(2 * u) & 3], (int)ring[d].meta[(2 * u) >> 2]);
                    const uint32_t zraw = (uint32_t)__builtin_amdgcn_ds_bpermute(meta_from[(2 * u + 1) & 3], (int)ring[d].meta[(2 * u + 1) >> 2]);
                    const float zf = (float)__builtin_bit_cast(_Float16, (uint16_t)zraw);
                    const float sf = (float)__builtin_bit_cast(_Float16, (uint16_t)sraw);
#pragma unroll
                    for (int v = 0; v < MV; ++v)
                        acc[u][v] = fmaf(sf, fmaf(eg[v], p[v], -fmaf(zf, xg[v], cg[v])), acc[u][v]);
                }
            }
            issue(ring[d]); // the item D places ahead reuses this slot
            if (cur.ub < NU && ++cur.t == T) {
                // end of a unit: fixed-order reduction over the wavefronts, double-buffered
                float *rbuf = red + (size_t)parity * GNW * S * MV * 64;
#pragma unroll
                for (int u = 0; u < S; ++u)
#pragma unroll
                    for (int v = 0; v < MV; ++v) {
                        rbuf[(wave * S * MV + u * MV + v) * 64 + lane] = acc[u][v];
                        acc[u][v] = 0.f;
                    }
                lds_barrier();
                const int n0 = unit_row(cur.ub) * ROWS + 16 * S * unit_part(cur.ub) + (lane & 15);
                for (int e = wave; e < S * MV; e += GNW) {
                    const int mrow = 4 * c + (e % MV), n = n0 + 16 * (e / MV);
                    if (mrow < M && n < job.N) { // units past the matrix have n >= N
                        float sum = 0.f;
#pragma unroll
                        for (int w = 0; w < GNW; ++w)
                            sum += rbuf[(w * S * MV + e) * 64 + lane];
                        job.out[(size_t)mrow * job.ld + n] = (_Float16)sum;
                    }
                }
                cur.t = 0;
                cur.ub += nblk;
                parity ^= 1;
            }
        }
    }
}

// Four wavefronts per SIMD, i.e. two workgroups per CU.  The inputs, M and K come first and as plain pointers
// and integers: the build asks the compiler to have these ten dwords preloaded into scalar registers at wavefront
// start, so the copies of the input row go out without waiting for a load of the kernel arguments.
template <int MODE, int MV>
__global__ __launch_bounds__(64 * GNW, 4) void gemv_stream_kernel(const _Float16 *in_a, const _Float16 *in_b, const _Float16 *in_c,
                                                                  _Float16 *in_aux, int M, int K, GemvJobs jobs)
{
    const GemvInput in = {in_a, in_b, in_c, in_aux, MODE};
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    __shared__ float part[2 * GNW];
    // The input row first, before anything about the job is known (which matrix, which width: three dependent
    // rounds of kernel-argument loads): row 0 of every input of the mode, copied from global memory straight into
    // LDS.  The i-th copy of a wavefront fills 64 consecutive 16-byte slots, lane by lane; chunk indices past the
    // end of the row are clamped (their slots are never read).  The destination is the region the bodies call
    // `raw` (behind the staged activations and the three group arrays), the same for every width.
    {
        constexpr int NIN = GemvInputs<MODE>::N, STEP = 64 * GNW;
        const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
        const int GP = (((K >> 7) + GNW - 1) / GNW) * GNW;
        h8 *raw = reinterpret_cast<h8 *>(smem + (size_t)GP * 16 * M * 16 + 3 * (size_t)GP * 16 * 4);
        const int chunks = K >> 3, trips = (chunks + STEP - 1) / STEP;
        const _Float16 *const src[3] = {in.a, in.b, in.c};
        for (int t = 0; t < trips; ++t) {
            const size_t off = (size_t)min(tid + STEP * t, chunks - 1) * 8;
#pragma unroll
            for (int i = 0; i < NIN; ++i)
                __builtin_amdgcn_global_load_lds(src[i] + off, &raw[(i * trips + t) * STEP + 64 * wave], 16, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0); // nothing of the job selection moves ahead of the copies
    }
    // the job of this workgroup, selected by value so that its fields stay in scalar registers
    GemvJob job = jobs.j[0];
    if (jobs.count > 1 && (int)blockIdx.x >= jobs.j[1].blk0)
        job = jobs.j[1];
    if (jobs.count > 2 && (int)blockIdx.x >= jobs.j[2].blk0)
        job = jobs.j[2];
    const int bj = blockIdx.x - job.blk0;
    switch (job.bits) { // uniform across the workgroup
    case 2:
        if (job.split)
            gemv_body<2, MODE, MV, 1>(job, bj, in, M, K, smem, part);
        else
            gemv_body<2, MODE, MV, 2>(job, bj, in, M, K, smem, part);
        break;
    case 3:
        if (job.split)
            gemv_body<3, MODE, MV, 1>(job, bj, in, M, K, smem, part);
        else
            gemv_body<3, MODE, MV, 4>(job, bj, in, M, K, smem, part);
        break;
    case 4: gemv_body<4, MODE, MV, 1>(job, bj, in, M, K, smem, part); break;
    default: gemv_body<8, MODE, MV, 1>(job, bj, in, M, K, smem, part); break;
    }
}

typedef void (*GemvKernel)(const _Float16 *, const _Float16 *, const _Float16 *, _Float16 *, int, int, GemvJobs);

// One kernel per input mode, for a single activation row and for up to sixteen.
GemvKernel gemv_kernel_for(int mode, int M, int *slot)
{
    static const GemvKernel table[7][2] = {
        {gemv_stream_kernel<0, 1>, gemv_stream_kernel<0, 4>}, {gemv_stream_kernel<1, 1>, gemv_stream_kernel<1, 4>},
        {gemv_stream_kernel<2, 1>, gemv_stream_kernel<2, 4>}, {gemv_stream_kernel<3, 1>, gemv_stream_kernel<3, 4>},
        {gemv_stream_kernel<4, 1>, gemv_stream_kernel<4, 4>}, {gemv_stream_kernel<5, 1>, gemv_stream_kernel<5, 4>},
        {gemv_stream_kernel<6, 1>, gemv_stream_kernel<6, 4>},
    };
    const int wide = M == 1 ? 0 : 1;
    *slot = 2 * mode + wide;
    return table[mode][wide];
}

constexpr size_t GEMV_MAX_LDS = 152 * 1024;

// Dynamic LDS of a streaming launch: staged x, the group sums and exponents (groups rounded up to whole turns of
// the wavefronts), and one region shared by the raw input row (inputs of the mode, whole trips of 512
// chunks) and the reduction buffers.
size_t gemv_stream_lds(int M, int K, int bits, int inputs)
{
    const int sub = bits == 3 ? 4 : (bits == 2 ? 2 : 1), mv = M == 1 ? 1 : 4;
    const size_t gp = (size_t)(((K >> 7) + GNW - 1) / GNW) * GNW;
    const size_t red = 2 * (size_t)GNW * sub * mv * 64 * 4;
    const size_t raw = (size_t)inputs * (((K >> 3) + 64 * GNW - 1) / (64 * GNW)) * (64 * GNW) * 16;
    return gp * 16 * M * 16 + 3 * gp * 16 * 4 + (red > raw ? red : raw);
}

int rows_per_supertile(int bits) { return bits == 2 ? 32 : (bits == 3 ? 64 : 16); }

// What a launch needs to know about the device, learnt once per device by fq_gemv_prepare (fq_init, or the
// first launch on that device): the CU count, and for each of the 14 kernel variants the largest dynamic-LDS
// request that still leaves p workgroups resident per CU.  Nothing on the launch path then sets attributes
// or queries the runtime, so launches can be captured into a graph.
constexpr int GEMV_VARIANTS = 14, GEMV_MAX_PER_CU = 4;
struct GemvDevice {
    bool ready = false;
    int cus = 0;
    size_t max_lds[GEMV_VARIANTS][GEMV_MAX_PER_CU + 1] = {}; // [slot][p]: largest request with >= p resident
};
GemvDevice g_gemv_dev[16];
std::mutex g_gemv_guard;

int gemv_prepare_locked(GemvDevice &d, int dev)
{
    int n = 0;
    hipError_t e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess)
        return (int)e;
    for (int mode = 0; mode < 7; ++mode)
        for (int wide = 0; wide < 2; ++wide) {
            int slot = 0;
            const GemvKernel kernel = gemv_kernel_for(mode, wide ? 16 : 1, &slot);
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)GEMV_MAX_LDS);
            if (e != hipSuccess)
                return (int)e;
            for (int p = 1; p <= GEMV_MAX_PER_CU; ++p) {
                // occupancy falls as the request grows: bisect for the last request (in KiB) with >= p resident
                int lo = -1, hi = (int)(GEMV_MAX_LDS >> 10) + 1;
                while (hi - lo > 1) {
                    const int mid = (lo + hi) / 2;
                    int per_cu = 0;
                    e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, 64 * GNW, (size_t)mid << 10);
                    if (e != hipSuccess)
                        return (int)e;
                    if (per_cu >= p)
                        lo = mid;
                    else
                        hi = mid;
                }
                d.max_lds[slot][p] = lo < 0 ? 0 : (size_t)lo << 10;
            }
        }
    d.cus = n;
    d.ready = true;
    return 0;
}

// Resident workgroups of variant `slot` on the current device for a request of dynamic LDS.
int gemv_resident_blocks(int slot, size_t lds, int *out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess)
        return (int)e;
    if (dev < 0 || dev >= 16)
        return (int)hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_gemv_guard);
    GemvDevice &d = g_gemv_dev[dev];
    if (!d.ready)
        if (int rc = gemv_prepare_locked(d, dev))
            return rc;
    int per_cu = 1;
    for (int p = 2; p <= GEMV_MAX_PER_CU; ++p)
        if (lds <= d.max_lds[slot][p])
            per_cu = p;
    *out = d.cus * per_cu;
    return 0;
}

} // namespace

int fq_gemv_prepare()
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess)
        return (int)e;
    if (dev < 0 || dev >= 16)
        return (int)hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_gemv_guard);
    return g_gemv_dev[dev].ready ? 0 : gemv_prepare_locked(g_gemv_dev[dev], dev);
}

bool fq_gemv_can_stream(int M, int K, int bits, int inputs)
{
    return gemv_stream_lds(M, K, bits, inputs) <= GEMV_MAX_LDS;
}

// Up to three matrices that share the input (same K): one launch.
int fq_launch_gemv_multi(const fq_gemv_input &src, int M, const fq_packed_ref *w, void *const *outs, int count,
                         fq_stream st)
{
    if (src.mode < 0 || src.mode > 6)
        return (int)hipErrorInvalidValue;
    const int inputs = src.mode == 2 ? 3 : (src.mode >= 3 ? 2 : 1);
    GemvJobs jobs;
    jobs.count = count;
    size_t lds = 0;
    int nrb[3];
    for (int i = 0; i < count; ++i) {
        const size_t need = gemv_stream_lds(M, w[i].K, w[i].bits, inputs);
        lds = lds > need ? lds : need;
        nrb[i] = ((w[i].N + 63) / 64 * 64) / rows_per_supertile(w[i].bits);
    }
    int slot = 0, resident = 0;
    const GemvKernel kernel = gemv_kernel_for(src.mode, M, &slot);
    if (int e = gemv_resident_blocks(slot, lds, &resident))
        return e;
    // Work units.  Whole supertile rows as a rule; but when even the 16-row sub-blocks of the 2- and 3-bit
    // matrices (2 or 4 per supertile row) are no more than the resident workgroups, those matrices are
    // handed out by sub-block, one per workgroup: 4096 x 4096 at 2 bits has only 128 supertile rows, at
    // 3 bits 64, and half or more of the chip would idle.  (With more sub-blocks than workgroups the split
    // loses: a sub-block item carries the fixed cost of a whole one.)  The workgroups that share a
    // supertile row are 8 apart in the grid, i.e. run on one XCD, whose L2 fetches their common lines
    // once; the job's share of the grid is a multiple of 8 * parts.
    int split_units = 0;
    for (int i = 0; i < count; ++i) {
        const int f = w[i].bits == 2 ? 2 : (w[i].bits == 3 ? 4 : 1);
        split_units += f > 1 ? (nrb[i] + 7) / 8 * 8 * f : nrb[i];
    }
    const bool underfull = split_units <= resident;
    int parts[3], units[3], gran[3], nbs[3], order[3];
    double unit_cost[3];
    // cost of a whole supertile row relative to a 4-bit one (2-bit rows are bound by the unpack, not by
    // their bytes, so cost grows more slowly than bytes)
    static const double row_cost[9] = {0, 0, 1.25, 2.5, 1.0, 0, 0, 0, 1.55};
    int used = 0;
    for (int i = 0; i < count; ++i) {
        const int f = w[i].bits == 2 ? 2 : (w[i].bits == 3 ? 4 : 1);
        parts[i] = (underfull && f > 1) ? f : 1;
        units[i] = parts[i] > 1 ? (nrb[i] + 7) / 8 * 8 * parts[i] : nrb[i];
        gran[i] = parts[i] > 1 ? 8 * parts[i] : 1;
        unit_cost[i] = row_cost[w[i].bits] / parts[i];
        nbs[i] = gran[i];
        used += gran[i];
    }
    // Hand the remaining workgroups, a granule at a time, to the matrix that would finish last.
    for (;;) {
        int worst = -1;
        double worst_t = -1.0;
        for (int i = 0; i < count; ++i) {
            if (nbs[i] >= units[i] || used + gran[i] > resident)
                continue;
            const double t = (double)((units[i] + nbs[i] - 1) / nbs[i]) * unit_cost[i];
            if (t > worst_t) {
                worst_t = t;
                worst = i;
            }
        }
        if (worst < 0)
            break;
        nbs[worst] += gran[worst];
        used += gran[worst];
    }
    // split jobs first: their first workgroup must sit at a multiple of 8
    int n_order = 0;
    for (int pass = 0; pass < 2; ++pass)
        for (int i = 0; i < count; ++i)
            if ((parts[i] > 1) == (pass == 0))
                order[n_order++] = i;
    int blk0 = 0;
    for (int k = 0; k < count; ++k) {
        const int i = order[k];
        jobs.j[k] = GemvJob{static_cast<const uint32_t *>(w[i].packed), static_cast<const _Float16 *>(w[i].scales),
                            static_cast<const _Float16 *>(w[i].zeros), static_cast<_Float16 *>(outs[i]), w[i].N,
                            w[i].bits, blk0, nbs[i], parts[i] > 1 ? 1 : 0, w[i].ld ? w[i].ld : w[i].N};
        blk0 += nbs[i];
    }
    for (int i = count; i < 3; ++i)
        jobs.j[i] = GemvJob{nullptr, nullptr, nullptr, nullptr, 0, 0, blk0, 0, 0, 0};
    const GemvInput in = {static_cast<const _Float16 *>(src.a), static_cast<const _Float16 *>(src.b),
                          static_cast<const _Float16 *>(src.c), static_cast<_Float16 *>(src.aux), src.mode};
    hipLaunchKernelGGL(kernel, dim3(blk0), dim3(64 * GNW), lds, st, in.a, in.b, in.c, in.aux, M, w[0].K, jobs);
    return (int)hipGetLastError();
}

int fq_launch_gemv(const void *x, int M, const fq_packed_ref &w, void *out, fq_stream st)
{
    if (fq_gemv_can_stream(M, w.K, w.bits, 1)) {
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
