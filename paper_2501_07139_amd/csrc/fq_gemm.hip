// Calibration-forward path: dequant-GEMM for M > 16 rows of activations, and the
// unquantized fp16 head GEMM.
//
// Scoring one candidate hybrid model means a full forward of the calibration
// sequences (FlexQuant, arXiv 2501.07139, Algorithm 1, calibrationEval), which is
// a dense contraction, so it runs on the matrix cores: 16x16x32 fp16 MFMA with
// fp32 accumulation.
//
// Quantized kernel.  Workgroup tile: BM=128 activation rows x BN=128 weight rows,
// one group of 128 k per iteration, 256 threads = 4 wavefronts side by side along
// N (each 128 x 32), two workgroups resident per CU.  The packed format stores a lane's 32 weights of a group as
// the A operands of four consecutive MFMA k-steps, so every wavefront loads its
// own packed chunks straight from global memory into registers (1 KiB contiguous
// per load), dequantizes them there and feeds the matrix core: weights never
// touch LDS and are unpacked once per workgroup.  Activations are shared by the
// four wavefronts through a double-buffered LDS tile, row-major with 16-byte
// chunks XOR-swizzled by row so that the coalesced copy and the operand reads are
// both free of bank conflicts; the copy goes from global memory straight into LDS.  Loads for group g+1 are issued
// before the MFMAs of group g; one barrier per iteration.
//
// The linears of a block that share their input (q/k/v, gate/up) go out as one launch whose workgroups
// each look up their matrix: a matrix whose tiles do not fill the workgroup slots a whole number of times
// shares its last round with the next one.
//
// The unquantized head runs the same kernel: its fp16 weights are read from the row-major matrix
// directly into the operand registers (sixteen rows by 64 contiguous bytes per load).
#include "fq_device.h"
#include "fq_internal.h"

#include <type_traits>
#include <utility>

namespace {

// ------------------------------------------------------------ quantized GEMM
constexpr int QBM = 128, QMB = QBM / 16; // per wave: QNB weight blocks (template) x QMB activation blocks

constexpr int DENSE = 16; // BITS value of the unquantized fp16 weight path (the vocabulary head)

template <int BITS>
struct WChunk {
    uint32_t c[BITS];
    uint32_t scale, zero; // fp16 bits in the low half, as loaded: nothing touches them before their use
};

// fp16 weights: a lane's operands of the four k-steps, read straight from the row-major matrix
template <>
struct WChunk<DENSE> {
    h8 f[4];
};

// Descriptors of the kernel's arrays (see make_rsrc).
struct GemmBuffers {
    fq_rsrc x, packed, scales, zeros;
};

template <int BITS>
__device__ __forceinline__ void load_wchunk(WChunk<BITS> &w, const GemmBuffers &buf, int rb16, int Np16, int G, int K,
                                            int g, int lane)
{
    if constexpr (BITS == DENSE) {
        // packed is the fp16 matrix [N,K]; Np16 carries N here.  Rows past the end re-read the last row.
        const int row = min(rb16 * 16 + (lane & 15), Np16 - 1);
        const uint32_t lo = ((uint32_t)row * (uint32_t)K + 8u * (uint32_t)(lane >> 4)) * 2u;
#pragma unroll
        for (int s = 0; s < 4; ++s)
            w.f[s] = __builtin_bit_cast(h8, buf_load_b128(buf.packed, lo + 64u * s, (uint32_t)g * 256u));
    } else {
        constexpr int SUB = Fmt<BITS>::SUB;
        // blocks past the end of the matrix re-read the last block: their results are never stored, and
        // loads without a branch keep the count of loads in flight known to the compiler
        const int rb = min(rb16, Np16 - 1);
        const uint32_t tile_off = (uint32_t)((rb / SUB) * G + g) * (uint32_t)(tile_dwords<BITS>() * 4);
        buf_load_chunk<BITS>(buf.packed, tile_off, rb % SUB, lane, w.c);
        const uint32_t meta_off = (uint32_t)(rb * G + g) * 32u, lo = (uint32_t)(lane & 15) * 2u;
        w.scale = buf_load_u16(buf.scales, lo, meta_off);
        w.zero = buf_load_u16(buf.zeros, lo, meta_off);
    }
}

// One output tile of one matrix.  Xs: the workgroup's two activation tiles in LDS, [2][QBM * 16], chunk ch of
// row r at r*16 + (ch ^ (r & 15)).  `tile` numbers the matrix's tiles in bands of four activation row-tiles
// (row-tile fastest): tiles with consecutive numbers share weight tiles and a few activation row-tiles.
template <int BITS, int QNB>
__device__ __forceinline__ void qgemm_tile(h8 (*Xs)[QBM * 16], const _Float16 *__restrict__ x, int M,
                                           const uint32_t *__restrict__ packed, const _Float16 *__restrict__ scales,
                                           const _Float16 *__restrict__ zeros, int N, int K,
                                           _Float16 *__restrict__ out, int ld, int tile)
{
    constexpr int QBN = 64 * QNB;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int NT = (N + QBN - 1) / QBN, MT = (M + QBM - 1) / QBM;
    const int band = tile / (4 * NT), rest = tile - band * 4 * NT, height = min(4, MT - 4 * band);
    const int m0 = (4 * band + rest % height) * QBM, n0 = (rest / height) * QBN;
    const int G = K >> 7;
    const int Np16 = BITS == DENSE ? N : ((N + 63) / 64 * 64) >> 4; // sixteen-row blocks present (dense: rows)
    const int rb0 = (n0 >> 4) + wave * QNB; // first sixteen-row weight block of this wave

    // activation copy, global memory straight into LDS (no register hop): the i-th load of a wavefront
    // fills the 64 consecutive 16-byte slots from 64*wave + 256*i, lane by lane; slot (row, pos) holds
    // chunk pos ^ (row & 15) of its row, so each lane fetches that chunk.  Rows past M re-read row M-1.
    // Source addresses are the group's byte offset in a row (uniform) plus a 32-bit lane offset.
    const int xrow = 4 * wave + (lane >> 4), xch = (lane & 15) ^ (xrow & 15);
    uint32_t xoff[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
        xoff[i] = ((uint32_t)min(m0 + xrow + 16 * i, M - 1) * (uint32_t)K + (uint32_t)xch * 8u) * 2u;
    GemmBuffers buf;
    buf.x = make_rsrc(x, (uint32_t)M * (uint32_t)K * 2u);
    if constexpr (BITS == DENSE) {
        buf.packed = make_rsrc(packed, (uint32_t)N * (uint32_t)K * 2u);
        buf.scales = buf.zeros = buf.packed; // unused
    } else {
        const uint32_t Np = (uint32_t)(N + 63) / 64u * 64u;
        buf.packed = make_rsrc(packed, Np / 8u * (uint32_t)K * (uint32_t)BITS);
        buf.scales = make_rsrc(scales, Np * (uint32_t)G * 2u);
        buf.zeros = make_rsrc(zeros, Np * (uint32_t)G * 2u);
    }

    f4 acc[QNB][QMB];
#pragma unroll
    for (int i = 0; i < QNB; ++i)
#pragma unroll
        for (int j = 0; j < QMB; ++j)
            acc[i][j] = f4{0.f, 0.f, 0.f, 0.f};

    WChunk<BITS> wc[QNB];
#pragma unroll
    for (int i = 0; i < 8; ++i)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(buf.x, &Xs[0][64 * wave + 256 * i], 16, xoff[i], 0, 0, 0);
#pragma unroll
    for (int i = 0; i < QNB; ++i)
        load_wchunk<BITS>(wc[i], buf, rb0 + i, Np16, G, K, 0, lane);
    __builtin_amdgcn_s_waitcnt(FQ_WAIT_VMCNT0); // the copies into LDS have landed ...
    __syncthreads();                            // ... in every wavefront

    // Integer zeros (what the quantizer produces) let bias and zero leave a pair in one addition: look
    // at the zeros of this workgroup's weight rows once and take the matching copy of the main loop.
    bool intz = true;
    if constexpr (BITS != DENSE && QNB != 4) {
        const uint32_t first = (uint32_t)(n0 >> 4) * (uint32_t)G * 16u, count = (QBN / 16) * (uint32_t)G * 16u;
        int frac = 0;
        for (uint32_t i = (uint32_t)tid * 8u; i < count; i += 256u * 8u) { // past the array: zeros
            const h8 z = __builtin_bit_cast(h8, buf_load_b128(buf.zeros, (first + i) * 2u, 0));
#pragma unroll
            for (int e = 0; e < 8; ++e)
                frac |= z[e] != __builtin_truncf16(z[e]);
        }
        intz = !__syncthreads_or(frac);
    }

    auto main_loop = [&](auto intz_tag) {
    constexpr bool INTZ = decltype(intz_tag)::value;
    for (int g = 0; g < G; ++g) {
        const int cur = g & 1;
        // dequantize this group's weights into operands: (code - zero) * scale
        h8 a[QNB][4];
#pragma unroll
        for (int i = 0; i < QNB; ++i) {
            if constexpr (BITS == DENSE) {
#pragma unroll
                for (int s = 0; s < 4; ++s)
                    a[i][s] = wc[i].f[s];
            } else {
                h2 q[16];
                unpack_dequant<BITS, INTZ>(wc[i].c, as_h2(wc[i].zero * 0x10001u), as_h2(wc[i].scale * 0x10001u), q);
#pragma unroll
                for (int s = 0; s < 4; ++s)
                    a[i][s] = make_h8(q[4 * s], q[4 * s + 1], q[4 * s + 2], q[4 * s + 3]);
            }
        }
        // prefetch the next group
        const bool more = g + 1 < G;
        if (more) {
#pragma unroll
            for (int i = 0; i < 8; ++i)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(buf.x, &Xs[cur ^ 1][64 * wave + 256 * i], 16, xoff[i],
                                                         (uint32_t)(g + 1) * 256u, 0, 0);
#pragma unroll
            for (int i = 0; i < QNB; ++i)
                load_wchunk<BITS>(wc[i], buf, rb0 + i, Np16, G, K, g + 1, lane);
        }
        // contraction
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            h8 b[QMB];
#pragma unroll
            for (int j = 0; j < QMB; ++j) {
                const int row = j * 16 + (lane & 15), ch = 4 * s + (lane >> 4);
                b[j] = Xs[cur][row * 16 + (ch ^ (row & 15))];
            }
#pragma unroll
            for (int i = 0; i < QNB; ++i)
#pragma unroll
                for (int j = 0; j < QMB; ++j)
                    acc[i][j] = mfma16x16x32(a[i][s], b[j], acc[i][j]);
        }
        __builtin_amdgcn_s_waitcnt(FQ_WAIT_VMCNT0);
        __syncthreads();
    }
    };
    // Narrow quantized tiles: the same loop, software-pipelined inside the wavefront.  Matrix and vector
    // instructions leave through one issue port, so a wavefront that unpacks first and multiplies afterwards
    // leaves the matrix pipe idle while it unpacks, whatever the other resident wavefront does; here the
    // operands of group g+1 are unpacked between the MFMAs of group g (each MFMA occupies the pipe for four
    // issue slots and needs one).  Two chunk buffers and two operand buffers; the loads of group g+2 go out at
    // the top of iteration g, so everything the end-of-iteration wait covers was issued an iteration ago.
    auto pipelined_loop = [&](auto intz_tag) {
        constexpr bool INTZ = decltype(intz_tag)::value;
        if constexpr (BITS != DENSE) {
            WChunk<BITS> wd[QNB];
            h8 a0[QNB][4], a1[QNB][4];
            auto unpack_all = [&](WChunk<BITS> (&w)[QNB], h8 (&a)[QNB][4]) {
#pragma unroll
                for (int i = 0; i < QNB; ++i) {
                    h2 q[16];
                    unpack_dequant<BITS, INTZ>(w[i].c, as_h2(w[i].zero * 0x10001u), as_h2(w[i].scale * 0x10001u), q);
#pragma unroll
                    for (int s = 0; s < 4; ++s)
                        a[i][s] = make_h8(q[4 * s], q[4 * s + 1], q[4 * s + 2], q[4 * s + 3]);
                }
            };
            auto load_all = [&](WChunk<BITS> (&w)[QNB], int g) {
#pragma unroll
                for (int i = 0; i < QNB; ++i)
                    load_wchunk<BITS>(w[i], buf, rb0 + i, Np16, G, K, min(g, G - 1), lane);
            };
            auto body = [&](int g, h8 (&ac)[QNB][4], h8 (&an)[QNB][4], WChunk<BITS> (&wn)[QNB], WChunk<BITS> (&wl)[QNB]) {
                const int cur = g & 1;
                // past the last group both prefetches repeat it (nobody reads them): no branch in the iteration
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(buf.x, &Xs[cur ^ 1][64 * wave + 256 * i], 16, xoff[i],
                                                             (uint32_t)min(g + 1, G - 1) * 256u, 0, 0);
                load_all(wl, g + 2);
                unpack_all(wn, an); // ahead of the MFMAs in program order: the scheduler fills their shadows with it
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    h8 b[QMB];
#pragma unroll
                    for (int j = 0; j < QMB; ++j) {
                        const int row = j * 16 + (lane & 15), ch = 4 * s + (lane >> 4);
                        b[j] = Xs[cur][row * 16 + (ch ^ (row & 15))];
                    }
#pragma unroll
                    for (int i = 0; i < QNB; ++i)
#pragma unroll
                        for (int j = 0; j < QMB; ++j)
                            acc[i][j] = mfma16x16x32(ac[i][s], b[j], acc[i][j]);
                }
                __builtin_amdgcn_s_waitcnt(FQ_WAIT_VMCNT0);
                __syncthreads();
                __builtin_amdgcn_sched_barrier(0); // nothing moves from one iteration into the other
            };
            unpack_all(wc, a0);
            load_all(wc, 1);
            int g = 0;
            for (; g + 1 < G; g += 2) {
                body(g, a0, a1, wc, wd);
                body(g + 1, a1, a0, wd, wc);
            }
            if (g < G)
                body(g, a0, a1, wc, wd);
        }
    };
    if constexpr (QNB == 4 || BITS == DENSE)
        main_loop(std::false_type{}); // the wide tile has no registers to spare for a second copy of the loop
    else if (intz)
        pipelined_loop(std::true_type{});
    else
        pipelined_loop(std::false_type{});

    // store: lane holds m = lane%16 and n = 4*(lane/16) + v of each 16x16 block; four values at once where
    // every row of the output (a column range of a wider array when ld > N) starts 8-byte aligned
    const bool vec_ok = (ld & 3) == 0 && (reinterpret_cast<uintptr_t>(out) & 7) == 0;
#pragma unroll
    for (int j = 0; j < QMB; ++j) {
        const int m = m0 + j * 16 + (lane & 15);
        if (m >= M)
            continue;
#pragma unroll
        for (int i = 0; i < QNB; ++i) {
            const int n = (rb0 + i) * 16 + 4 * (lane >> 4);
            _Float16 *o = out + (size_t)m * ld + n;
            if (n + 3 < N && vec_ok) {
                h4 v = {(_Float16)acc[i][j][0], (_Float16)acc[i][j][1], (_Float16)acc[i][j][2], (_Float16)acc[i][j][3]};
                *reinterpret_cast<h4 *>(o) = v;
            } else {
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (n + v < N)
                        o[v] = (_Float16)acc[i][j][v];
            }
        }
    }
}

// Workgroups are dealt to the eight XCDs round-robin and each XCD has its own L2: XCD x takes the x-th
// contiguous run of `total` tiles.  Returns -1 for the workgroups past the end (uniform over a workgroup).
__device__ __forceinline__ int xcd_tile(int total)
{
    const int per_xcd = (total + 7) >> 3;
    const int tile = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    return tile < total ? tile : -1;
}

// Two workgroups per CU (two wavefronts per SIMD): a single wavefront cannot keep the matrix pipe
// busy, and two independent workgroups overlap one's unpack/copy phase with the other's MFMAs.
template <int BITS, int QNB>
__global__ __launch_bounds__(256, 2) void qgemm_kernel(const _Float16 *__restrict__ x, int M,
                                                       const uint32_t *__restrict__ packed,
                                                       const _Float16 *__restrict__ scales,
                                                       const _Float16 *__restrict__ zeros, int N, int K,
                                                       _Float16 *__restrict__ out)
{
    __shared__ h8 Xs[2][QBM * 16];
    constexpr int QBN = 64 * QNB;
    const int tile = xcd_tile(((N + QBN - 1) / QBN) * ((M + QBM - 1) / QBM));
    if (tile < 0)
        return; // before any barrier
    qgemm_tile<BITS, QNB>(Xs, x, M, packed, scales, zeros, N, K, out, N, tile);
}

// Up to three matrices with the same input in one launch (q/k/v, gate/up): their tiles form one list, so
// a matrix whose tiles do not fill the chip's workgroup slots a whole number of times shares its last
// round with the next matrix.  Each workgroup looks up its matrix and runs the tile code of that matrix's
// bit-width and tile width.
struct GemmJob {
    const uint32_t *packed;
    const _Float16 *scales, *zeros;
    _Float16 *out;
    int N, bits, qnb, tile0; // tile0: index of the matrix's first tile in the launch's list
    int ld;                  // elements between consecutive rows of out
};
struct GemmJobs {
    GemmJob j[3];
    int count, total;
};

__global__ __launch_bounds__(256, 2) void qgemm_multi_kernel(const _Float16 *__restrict__ x, int M, int K, GemmJobs jobs)
{
    __shared__ h8 Xs[2][QBM * 16];
    int tile = xcd_tile(jobs.total);
    if (tile < 0)
        return;
    int ji = 0;
    if (jobs.count > 1 && tile >= jobs.j[1].tile0)
        ji = 1;
    if (jobs.count > 2 && tile >= jobs.j[2].tile0)
        ji = 2;
    const GemmJob job = ji == 0 ? jobs.j[0] : (ji == 1 ? jobs.j[1] : jobs.j[2]); // selected by value
    tile -= job.tile0;
    switch (job.bits * 8 + job.qnb) {
    case 2 * 8 + 4: qgemm_tile<2, 4>(Xs, x, M, job.packed, job.scales, job.zeros, job.N, K, job.out, job.ld, tile); break;
    case 4 * 8 + 4: qgemm_tile<4, 4>(Xs, x, M, job.packed, job.scales, job.zeros, job.N, K, job.out, job.ld, tile); break;
    case 2 * 8 + 2: qgemm_tile<2, 2>(Xs, x, M, job.packed, job.scales, job.zeros, job.N, K, job.out, job.ld, tile); break;
    case 3 * 8 + 2: qgemm_tile<3, 2>(Xs, x, M, job.packed, job.scales, job.zeros, job.N, K, job.out, job.ld, tile); break;
    case 4 * 8 + 2: qgemm_tile<4, 2>(Xs, x, M, job.packed, job.scales, job.zeros, job.N, K, job.out, job.ld, tile); break;
    default: qgemm_tile<8, 2>(Xs, x, M, job.packed, job.scales, job.zeros, job.N, K, job.out, job.ld, tile); break;
    }
}

// ------------------------------------------------------------ tall tiles
// 256 activation rows x 128 weight rows per workgroup of eight wavefronts, one workgroup per CU, for products
// with many rows.  In the 128-row kernels every unpacked weight operand feeds 8 MFMAs and the unpacking is the
// largest share of what a wavefront issues beside its MFMAs; here a wavefront owns 256 x 32 outputs (128
// accumulator registers), so an operand feeds 16.  A 4096-column product at 2048 rows has only 256 such tiles,
// one per CU, so the second wavefront of every SIMD comes from splitting K inside the workgroup: wavefront
// (kh, nq) multiplies k-steps 2*kh and 2*kh+1 of every group with the weight rows 32*nq..+31, loads only that
// half of a chunk and unpacks only its eight pairs; the two partial sums meet in LDS at the end, in fp32.
// The loop is the narrow tiles' software pipeline (loads two groups ahead, operands of the next group
// unpacked ahead of this group's MFMAs in program order, one barrier per group).
//
// The two activation buffers are two LDS arrays on purpose.  A kernel with more than one LDS object has its LDS
// accesses tagged with alias scopes, and the compiler then waits for every direct-to-LDS load in flight before
// a read that may touch the same object: with both buffers in one array the reads of one buffer wait for the
// copies into the other right after they were issued, and the copy's whole latency (0.6 us per group here)
// lands on the wavefront.  With separate arrays, selected at compile time, the copies stay in flight until the
// wait at the end of the iteration.  As measured on MI355X (2048 rows, 4096 x 4096 and 4096 x 11008, same
// harness): 6-13 % faster than the 128-row kernels at every bit-width.
constexpr int TBM = 256, TBN = 128, TMB = TBM / 16, TNB = 2;

// biased pair P of a chunk (elements 2v, 2v+1 of k-step P/4, v = P%4) and the class of its bit position;
// the same fields and constants as unpack_dequant, one pair at a time
template <int BITS, int P>
struct PairAt {
    static constexpr int T = BITS == 2 ? (P & 7) : BITS == 3 ? (P % 5) : BITS == 4 ? (P & 3) : (P & 1);
    static constexpr int WRAP = BITS == 2 ? 5 : BITS == 3 ? 3 : BITS == 4 ? 2 : 1; // fields per half before the shifted copy
    static constexpr int DW = BITS == 2 ? (P >> 3) : BITS == 3 ? (P / 5) : BITS == 4 ? (P >> 2) : (P >> 1);
    static constexpr int SHIFT = T >= WRAP ? (BITS == 2 ? 10 : BITS == 3 ? 9 : 8) : 0;
    static constexpr int CLS = BITS == 8 ? 0 : (T >= WRAP ? T - WRAP : T);
    static constexpr uint32_t MASK = BITS == 8 ? 0x00ff00ffu : (((1u << BITS) - 1u) * 0x10001u) << (BITS * CLS);
};

template <int BITS>
struct UnpackConsts {
    static constexpr int NS = UnpackPlan<BITS>::NSHIFT;
    uint32_t E[NS]; // exponent of 2^(10-p) per class, in vector registers
    h2 mb[NS];      // -2^(10-p)
    __device__ __forceinline__ void init()
    {
        if constexpr (BITS == 8) {
            E[0] = exp_for_shift<0>(); mb[0] = minus_bias<0>();
        } else if constexpr (BITS == 4) {
            E[0] = exp_for_shift<0>(); E[1] = exp_for_shift<4>();
            mb[0] = minus_bias<0>(); mb[1] = minus_bias<4>();
        } else if constexpr (BITS == 3) {
            E[0] = exp_for_shift<0>(); E[1] = exp_for_shift<3>(); E[2] = exp_for_shift<6>();
            mb[0] = minus_bias<0>(); mb[1] = minus_bias<3>(); mb[2] = minus_bias<6>();
        } else {
            E[0] = exp_for_shift<0>(); E[1] = exp_for_shift<2>(); E[2] = exp_for_shift<4>(); E[3] = exp_for_shift<6>();
            E[4] = exp_for_shift<8>();
            mb[0] = minus_bias<0>(); mb[1] = minus_bias<2>(); mb[2] = minus_bias<4>(); mb[3] = minus_bias<6>();
            mb[4] = minus_bias<8>();
        }
    }
};

template <int BITS, int P>
__device__ __forceinline__ uint32_t biased_pair(const uint32_t (&C)[BITS], const UnpackConsts<BITS> &uc)
{
    if constexpr (BITS == 3 && P == 15) { // the two weights whose bits sit on top of the three dwords
        uint32_t sp = ((C[0] >> 15) & 0x00010001u) | uc.E[0];
        sp |= (C[1] >> 14) & 0x00020002u;
        sp |= (C[2] >> 13) & 0x00040004u;
        return sp;
    } else {
        using A = PairAt<BITS, P>;
        return ((C[A::DW] >> A::SHIFT) & A::MASK) | uc.E[A::CLS];
    }
}

template <int BITS, int P>
constexpr int pair_class() { return (BITS == 3 && P == 15) ? 0 : PairAt<BITS, P>::CLS; }

template <int... I, class F>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>), in order
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(static_cast<F &&>(f), std::make_integer_sequence<int, N>{});
}

// The dwords of a chunk that hold k-steps 2*KH and 2*KH+1 (3 bits: all three, the last pair's bits sit on
// top of every dword), with the row's scale and zero; the other entries of w.c stay unset and unread.
template <int BITS, int KH>
__device__ __forceinline__ void load_whalf(WChunk<BITS> &w, const GemmBuffers &buf, int rb16, int Np16, int G, int g,
                                           int lane)
{
    constexpr int SUB = Fmt<BITS>::SUB;
    const int rb = min(rb16, Np16 - 1); // blocks past the end re-read the last block (see load_wchunk)
    const uint32_t tile_off = (uint32_t)((rb / SUB) * G + g) * (uint32_t)(tile_dwords<BITS>() * 4);
    const int u = rb % SUB;
    const uint32_t lo = (uint32_t)lane * 16u;
    if constexpr (BITS == 2) {
        w.c[KH] = buf_load_b32(buf.packed, lo + 8u * (uint32_t)u + 4u * KH, tile_off);
    } else if constexpr (BITS == 4) {
        const u2v v = buf_load_b64(buf.packed, lo + 8u * KH, tile_off);
        w.c[2 * KH] = v.x; w.c[2 * KH + 1] = v.y;
    } else if constexpr (BITS == 8) {
        const u4v v = buf_load_b128(buf.packed, lo + 1024u * KH, tile_off);
        w.c[4 * KH] = v.x; w.c[4 * KH + 1] = v.y; w.c[4 * KH + 2] = v.z; w.c[4 * KH + 3] = v.w;
    } else {
        buf_load_chunk<BITS>(buf.packed, tile_off, u, lane, w.c);
    }
    const uint32_t meta_off = (uint32_t)(rb * G + g) * 32u, mlo = (uint32_t)(lane & 15) * 2u;
    w.scale = buf_load_u16(buf.scales, mlo, meta_off);
    w.zero = buf_load_u16(buf.zeros, mlo, meta_off);
}

// Operands of k-steps 2*KH and 2*KH+1 of a chunk: (code - zero) * scale per weight in packed fp16, the
// arithmetic of unpack_dequant pair by pair (integer zeros: bias and zero leave in one exact addition).
template <int BITS, bool INTZ, int KH>
__device__ __forceinline__ void unpack_khalf(const WChunk<BITS> &w, const UnpackConsts<BITS> &uc, h8 (&a)[2])
{
    const h2 zero2 = as_h2(w.zero * 0x10001u), scale2 = as_h2(w.scale * 0x10001u);
    static_for<2>([&](auto s_tag) {
        constexpr int s = decltype(s_tag)::value;
        h2 q[4];
        static_for<4>([&](auto v_tag) {
            constexpr int v = decltype(v_tag)::value, P = 4 * (2 * KH + s) + v, CLS = pair_class<BITS, P>();
            const h2 b = as_h2(biased_pair<BITS, P>(w.c, uc));
            if constexpr (INTZ)
                q[v] = (b + (uc.mb[CLS] - zero2)) * scale2;
            else
                q[v] = ((b + uc.mb[CLS]) - zero2) * scale2;
        });
        a[s] = make_h8(q[0], q[1], q[2], q[3]);
    });
}

// One 256 x 128 output tile.  Xs0, Xs1: the two activation tiles (256 rows x 128 k each, laid out like the
// narrow tiles'); after the loop the same memory carries the second K half's partial sums to the first.
template <int BITS>
__device__ __forceinline__ void qgemm_tall_tile(h8 *Xs0, h8 *Xs1, const _Float16 *__restrict__ x, int M,
                                                const uint32_t *__restrict__ packed,
                                                const _Float16 *__restrict__ scales,
                                                const _Float16 *__restrict__ zeros, int N, int K,
                                                _Float16 *__restrict__ out, int ld, int tile)
{
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kh = wave >> 2, nq = wave & 3; // half of every group's k-steps, quarter of the tile's weight rows
    // tiles are numbered in bands of two activation row-tiles (row-tile fastest): the 32 tiles an XCD holds at a
    // time share 512 activation rows (4 MiB at k = 4096, the size of its L2) and 16 weight tiles
    const int NT = (N + TBN - 1) / TBN, MT = (M + TBM - 1) / TBM;
    const int band = tile / (2 * NT), rest = tile - band * 2 * NT, height = min(2, MT - 2 * band);
    const int m0 = (2 * band + rest % height) * TBM, n0 = (rest / height) * TBN;
    const int G = K >> 7;
    const int Np16 = ((N + 63) / 64 * 64) >> 4;
    const int rb0 = (n0 >> 4) + nq * TNB;

    GemmBuffers buf;
    buf.x = make_rsrc(x, (uint32_t)M * (uint32_t)K * 2u);
    const uint32_t Np = (uint32_t)(N + 63) / 64u * 64u;
    buf.packed = make_rsrc(packed, Np / 8u * (uint32_t)K * (uint32_t)BITS);
    buf.scales = make_rsrc(scales, Np * (uint32_t)G * 2u);
    buf.zeros = make_rsrc(zeros, Np * (uint32_t)G * 2u);

    // Activation copies, global memory straight into LDS: copy i of a wavefront fills the 64 slots from
    // 64*wave + 512*i, i.e. rows 4*wave + 32*i + lane/16; slot (row, pos) holds chunk pos ^ (row & 15).  The
    // row is part of the lane offset, which the descriptor's range check covers (the scalar offset, which
    // carries the group's bytes within the row, is not checked): rows past M read as zero and are never stored.
    const int xrow = 4 * wave + (lane >> 4), xch = (lane & 15) ^ (xrow & 15);
    const uint32_t xoff0 = ((uint32_t)(m0 + xrow) * (uint32_t)K + (uint32_t)xch * 8u) * 2u;
    const uint32_t xstep = 64u * (uint32_t)K; // 32 rows

    f4 acc[TNB][TMB];
#pragma unroll
    for (int i = 0; i < TNB; ++i)
#pragma unroll
        for (int j = 0; j < TMB; ++j)
            acc[i][j] = f4{0.f, 0.f, 0.f, 0.f};

#pragma unroll
    for (int i = 0; i < 8; ++i)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(buf.x, &Xs0[64 * wave + 512 * i], 16, xoff0 + xstep * i, 0, 0, 0);

    // integer zeros: one addition takes bias and zero away (see qgemm_tile)
    bool intz;
    {
        const uint32_t first = (uint32_t)(n0 >> 4) * (uint32_t)G * 16u, count = (TBN / 16) * (uint32_t)G * 16u;
        int frac = 0;
        for (uint32_t i = (uint32_t)tid * 8u; i < count; i += 512u * 8u) { // past the array: zeros
            const h8 z = __builtin_bit_cast(h8, buf_load_b128(buf.zeros, (first + i) * 2u, 0));
#pragma unroll
            for (int e = 0; e < 8; ++e)
                frac |= z[e] != __builtin_truncf16(z[e]);
        }
        __builtin_amdgcn_s_waitcnt(FQ_WAIT_VMCNT0); // the first activation tile has landed ...
        intz = !__syncthreads_or(frac);             // ... in every wavefront
    }

    UnpackConsts<BITS> uc;
    uc.init();
    const int brow = lane & 15;

    auto main_loop = [&](auto intz_tag, auto kh_tag) {
        constexpr bool INTZ = decltype(intz_tag)::value;
        constexpr int KH = decltype(kh_tag)::value;
        WChunk<BITS> wc[TNB], wd[TNB];
        h8 a0[TNB][2], a1[TNB][2];
        auto unpack_all = [&](WChunk<BITS> (&w)[TNB], h8 (&a)[TNB][2]) {
#pragma unroll
            for (int i = 0; i < TNB; ++i)
                unpack_khalf<BITS, INTZ, KH>(w[i], uc, a[i]);
        };
        auto load_all = [&](WChunk<BITS> (&w)[TNB], int g) {
#pragma unroll
            for (int i = 0; i < TNB; ++i)
                load_whalf<BITS, KH>(w[i], buf, rb0 + i, Np16, G, min(g, G - 1), lane);
        };
        // Xc: this group's activations, Xn: the buffer the next group's are copied into.  Past the last group
        // both prefetches repeat it (nobody reads them): no branch in the iteration.
        auto body = [&](h8 *Xc, h8 *Xn, int g, h8 (&ac)[TNB][2], h8 (&an)[TNB][2], WChunk<BITS> (&wn)[TNB],
                        WChunk<BITS> (&wl)[TNB]) {
#pragma unroll
            for (int i = 0; i < 8; ++i)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(buf.x, &Xn[64 * wave + 512 * i], 16, xoff0 + xstep * i,
                                                         (uint32_t)min(g + 1, G - 1) * 256u, 0, 0);
            __builtin_amdgcn_sched_barrier(0); // the copies go out first: they have the whole iteration to land
            load_all(wl, g + 2);
            unpack_all(wn, an); // ahead of the MFMAs in program order: the scheduler fills their shadows with it
            constexpr int JB = BITS == 3 ? 4 : 8; // operand reads per batch (3 bits: the fewest registers to spare)
#pragma unroll
            for (int s = 0; s < 2; ++s) {
#pragma unroll
                for (int jh = 0; jh < TMB; jh += JB) {
                    h8 b[JB];
#pragma unroll
                    for (int j = 0; j < JB; ++j) {
                        const int ch = 4 * (2 * KH + s) + (lane >> 4);
                        b[j] = Xc[((jh + j) * 16 + brow) * 16 + (ch ^ brow)];
                    }
#pragma unroll
                    for (int i = 0; i < TNB; ++i)
#pragma unroll
                        for (int j = 0; j < JB; ++j)
                            acc[i][jh + j] = mfma16x16x32(ac[i][s], b[j], acc[i][jh + j]);
                }
            }
            __builtin_amdgcn_s_waitcnt(FQ_WAIT_VMCNT0); // this wavefront's copies into Xn have landed ...
            __syncthreads();                            // ... and everybody's; Xc is free
            __builtin_amdgcn_sched_barrier(0);          // nothing moves from one iteration into the other
        };
        load_all(wc, 0);
        unpack_all(wc, a0);
        load_all(wc, 1);
        int g = 0;
        for (; g + 1 < G; g += 2) {
            body(Xs0, Xs1, g, a0, a1, wc, wd);
            body(Xs1, Xs0, g + 1, a1, a0, wd, wc);
        }
        if (g < G)
            body(Xs0, Xs1, g, a0, a1, wc, wd);
    };
    if (kh == 0) {
        if (intz)
            main_loop(std::true_type{}, std::integral_constant<int, 0>{});
        else
            main_loop(std::false_type{}, std::integral_constant<int, 0>{});
    } else {
        if (intz)
            main_loop(std::true_type{}, std::integral_constant<int, 1>{});
        else
            main_loop(std::false_type{}, std::integral_constant<int, 1>{});
    }

    // The second K half hands its sums over (every iteration ended with a wait for all loads and a barrier, so
    // both arrays are free): block (i, j) of column quarter nq at float4 (nq*16 + j)*64 + lane of array i.
    f4 *red0 = reinterpret_cast<f4 *>(Xs0), *red1 = reinterpret_cast<f4 *>(Xs1);
    if (kh == 1) {
#pragma unroll
        for (int j = 0; j < TMB; ++j) {
            red0[((nq * 16 + j) << 6) + lane] = acc[0][j];
            red1[((nq * 16 + j) << 6) + lane] = acc[1][j];
        }
    }
    __syncthreads();
    if (kh == 1)
        return;
    // store: lane holds m = lane%16 and n = 4*(lane/16) + v of each 16x16 block (see qgemm_tile)
    const bool vec_ok = (ld & 3) == 0 && (reinterpret_cast<uintptr_t>(out) & 7) == 0;
#pragma unroll
    for (int j = 0; j < TMB; ++j) {
        const int m = m0 + j * 16 + (lane & 15);
#pragma unroll
        for (int i = 0; i < TNB; ++i) {
            const f4 r = acc[i][j] + (i ? red1 : red0)[((nq * 16 + j) << 6) + lane];
            const int n = (rb0 + i) * 16 + 4 * (lane >> 4);
            if (m >= M)
                continue;
            _Float16 *o = out + (size_t)m * ld + n;
            if (n + 3 < N && vec_ok) {
                h4 v = {(_Float16)r[0], (_Float16)r[1], (_Float16)r[2], (_Float16)r[3]};
                *reinterpret_cast<h4 *>(o) = v;
            } else {
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (n + v < N)
                        o[v] = (_Float16)r[v];
            }
        }
    }
}

struct TallJob {
    const uint32_t *packed;
    const _Float16 *scales, *zeros;
    _Float16 *out;
    int N, bits, tile0, ld;
};
struct TallJobs {
    TallJob j[3];
    int count, total;
};

// Eight wavefronts of 256 registers each: one workgroup per CU, two wavefronts per SIMD.
__global__ __launch_bounds__(512, 1) void qgemm_tall_kernel(const _Float16 *__restrict__ x, int M, int K, TallJobs jobs)
{
    __shared__ h8 Xs0[TBM * 16];
    __shared__ h8 Xs1[TBM * 16];
    int tile = xcd_tile(jobs.total);
    if (tile < 0)
        return;
    int ji = 0;
    if (jobs.count > 1 && tile >= jobs.j[1].tile0)
        ji = 1;
    if (jobs.count > 2 && tile >= jobs.j[2].tile0)
        ji = 2;
    const TallJob job = ji == 0 ? jobs.j[0] : (ji == 1 ? jobs.j[1] : jobs.j[2]);
    tile -= job.tile0;
    switch (job.bits) {
    case 2: qgemm_tall_tile<2>(Xs0, Xs1, x, M, job.packed, job.scales, job.zeros, job.N, K, job.out, job.ld, tile); break;
    case 3: qgemm_tall_tile<3>(Xs0, Xs1, x, M, job.packed, job.scales, job.zeros, job.N, K, job.out, job.ld, tile); break;
    case 4: qgemm_tall_tile<4>(Xs0, Xs1, x, M, job.packed, job.scales, job.zeros, job.N, K, job.out, job.ld, tile); break;
    default: qgemm_tall_tile<8>(Xs0, Xs1, x, M, job.packed, job.scales, job.zeros, job.N, K, job.out, job.ld, tile); break;
    }
}

// Weight-tile width.  Wide tiles (each wavefront 128 x 64) halve the LDS reads and activation copies per
// MFMA but need at least two workgroups per CU to keep both wavefront slots of every SIMD filled.
int wide_tiles_pay(int M, int N)
{
    const long tiles = (long)((N + 255) / 256) * ((M + QBM - 1) / QBM);
    return tiles >= 2 * 256;
}

int tall_tiles(int M, int N) { return ((N + TBN - 1) / TBN) * ((M + TBM - 1) / TBM); }

// Tile height for a launch of `count` matrices.  A tall tile occupies a whole CU, so tall tiles pay once there is
// one for every CU and the rows fill more than half of a tile: as measured, 3-14 % faster than the 128-row tiles
// at 2048 rows at every bit-width.  From 4096 rows on, the 128 x 256 tiles of 2- and 4-bit matrices run several
// full rounds and are level or 2-6 % ahead, so launches made of such matrices only stay with them.
int choose_tile_rows(int M, const fq_packed_ref *w, int count)
{
    long tall = 0;
    bool all_wide = M >= 4096;
    for (int i = 0; i < count; ++i) {
        tall += tall_tiles(M, w[i].N);
        all_wide = all_wide && (w[i].bits == 2 || w[i].bits == 4) && wide_tiles_pay(M, w[i].N);
    }
    return (M > 128 && tall >= 256 && !all_wide) ? 256 : 128;
}

template <int BITS, int QNB>
int launch_tile(const void *x, int M, const void *packed, const void *scales, const void *zeros, int N, int K,
                void *out, fq_stream st)
{
    constexpr int QBN = 64 * QNB;
    const int total = ((N + QBN - 1) / QBN) * ((M + QBM - 1) / QBM);
    dim3 grid(8 * ((total + 7) / 8)), block(256);
    hipLaunchKernelGGL((qgemm_kernel<BITS, QNB>), grid, block, 0, st, static_cast<const _Float16 *>(x), M,
                       static_cast<const uint32_t *>(packed), static_cast<const _Float16 *>(scales),
                       static_cast<const _Float16 *>(zeros), N, K, static_cast<_Float16 *>(out));
    return (int)hipGetLastError();
}

template <int BITS>
int launch_q(const void *x, int M, const fq_packed_ref &w, void *out, fq_stream st)
{
    // 3- and 8-bit operands do not fit the register budget of a wide tile
    if ((BITS == 2 || BITS == 4) && wide_tiles_pay(M, w.N))
        return launch_tile<(BITS == 2 || BITS == 4) ? BITS : 4, 4>(x, M, w.packed, w.scales, w.zeros, w.N, w.K, out, st);
    return launch_tile<BITS, 2>(x, M, w.packed, w.scales, w.zeros, w.N, w.K, out, st);
}

} // namespace

// The kernels address x, the packed weights and the scales/zeros through 32-bit byte offsets.
static bool fits_32bit(size_t a, size_t b, size_t elem_bytes) { return a * b * elem_bytes < ((size_t)1 << 32); }

static int launch_tall(const void *x, int M, const fq_packed_ref *w, void *const *outs, int count, fq_stream st)
{
    TallJobs jobs;
    jobs.count = count;
    int total = 0;
    for (int i = 0; i < count; ++i) {
        jobs.j[i] = TallJob{static_cast<const uint32_t *>(w[i].packed), static_cast<const _Float16 *>(w[i].scales),
                            static_cast<const _Float16 *>(w[i].zeros), static_cast<_Float16 *>(outs[i]), w[i].N,
                            w[i].bits, total, w[i].ld ? w[i].ld : w[i].N};
        total += tall_tiles(M, w[i].N);
    }
    jobs.total = total;
    hipLaunchKernelGGL(qgemm_tall_kernel, dim3(8 * ((total + 7) / 8)), dim3(512), 0, st,
                       static_cast<const _Float16 *>(x), M, w[0].K, jobs);
    return (int)hipGetLastError();
}

int fq_launch_gemm(const void *x, int M, const fq_packed_ref &w, void *out, fq_stream st, int tile_rows)
{
    const size_t Np = ((size_t)w.N + 63) / 64 * 64;
    if (!fits_32bit(M, w.K, 2) || Np / 8 * w.K * w.bits >= ((size_t)1 << 32))
        return (int)hipErrorInvalidValue;
    if (tile_rows == 0)
        tile_rows = choose_tile_rows(M, &w, 1);
    if (tile_rows == 256)
        return launch_tall(x, M, &w, &out, 1, st);
    if (w.ld && w.ld != w.N) // a column range of a wider output: the multi-matrix kernel carries the row pitch
        return fq_launch_gemm_multi(x, M, &w, &out, 1, st, 128);
    switch (w.bits) {
    case 2: return launch_q<2>(x, M, w, out, st);
    case 3: return launch_q<3>(x, M, w, out, st);
    case 4: return launch_q<4>(x, M, w, out, st);
    default: return launch_q<8>(x, M, w, out, st);
    }
}

// Matrices that share x (same K): one launch.  Shapes are validated by the caller like fq_launch_gemm's.
int fq_launch_gemm_multi(const void *x, int M, const fq_packed_ref *w, void *const *outs, int count, fq_stream st,
                         int tile_rows)
{
    if (count < 1 || count > 3)
        return (int)hipErrorInvalidValue;
    for (int i = 0; i < count; ++i) {
        const size_t Np = ((size_t)w[i].N + 63) / 64 * 64;
        if (w[i].K != w[0].K || !fits_32bit(M, w[i].K, 2) || Np / 8 * w[i].K * w[i].bits >= ((size_t)1 << 32))
            return (int)hipErrorInvalidValue;
    }
    if (tile_rows == 0)
        tile_rows = choose_tile_rows(M, w, count);
    if (tile_rows == 256)
        return launch_tall(x, M, w, outs, count, st);
    GemmJobs jobs;
    jobs.count = count;
    int total = 0;
    for (int i = 0; i < count; ++i) {
        const int qnb = ((w[i].bits == 2 || w[i].bits == 4) && wide_tiles_pay(M, w[i].N)) ? 4 : 2;
        jobs.j[i] = GemmJob{static_cast<const uint32_t *>(w[i].packed), static_cast<const _Float16 *>(w[i].scales),
                            static_cast<const _Float16 *>(w[i].zeros), static_cast<_Float16 *>(outs[i]), w[i].N,
                            w[i].bits, qnb, total, w[i].ld ? w[i].ld : w[i].N};
        total += ((w[i].N + 64 * qnb - 1) / (64 * qnb)) * ((M + QBM - 1) / QBM);
    }
    jobs.total = total;
    hipLaunchKernelGGL(qgemm_multi_kernel, dim3(8 * ((total + 7) / 8)), dim3(256), 0, st,
                       static_cast<const _Float16 *>(x), M, w[0].K, jobs);
    return (int)hipGetLastError();
}

int fq_launch_dense(const void *x, int M, const void *W, int N, int K, void *out, fq_stream st)
{
    if (!fits_32bit(M, K, 2) || !fits_32bit(N, K, 2))
        return (int)hipErrorInvalidValue;
    return launch_tile<DENSE, 2>(x, M, W, nullptr, nullptr, N, K, out, st);
}
