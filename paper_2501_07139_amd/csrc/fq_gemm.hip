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
// 256 activation rows x 128 weight rows per workgroup, for products with many rows.  What bounds the
// 128-row kernels is not the matrix pipe alone: every wavefront re-reads the whole activation tile from LDS
// (one 1 KiB operand read per two MFMAs with 32-column wavefront tiles) and unpacks every weight for only 8
// MFMAs, and LDS reads, vector instructions and MFMAs each fill more than half of their own capacity.  Here a wavefront
// owns 256 x 64 outputs: one operand read per four MFMAs, one unpacked weight operand per sixteen, and the
// 256 accumulator registers that takes leave one wavefront per SIMD, whose own instruction stream overlaps
// loads, unpacking and MFMAs (the operands of the next half group are unpacked between the MFMAs of this one).
// A 4096-column product at 2048 rows has only 128 tiles of 256 x 256, so the four wavefronts of a workgroup
// are two column halves times two halves of K: each K half streams its own activation tiles (64 k per step,
// double buffered, 128 KiB in all) and the two partial sums meet in LDS at the end, in fp32.
// As measured on MI355X (2048 x 4096 x 4096, 2 bits) this kernel takes 77-80 us against 66-67 us for the
// 128-row kernel: with one wavefront per SIMD nothing covers the wait for the next step's activation copies
// (without them 54 us), and LDS has no room for a third buffer.  It is therefore never the library's own
// choice and runs only when a caller asks for 256-row tiles.
constexpr int TBM = 256, TBN = 128, TMB = TBM / 16, TNB = 4;
constexpr int TSLOTS = TBM * 8; // 16-byte slots of one activation tile: 256 rows x 64 k

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

// (code - zero) * scale for pair P of a chunk, as the two fp16 numbers of one operand register, one
// instruction per stage so that the caller can place the stages of two pairs alternately (a packed fp16
// instruction that reads the previous one's result costs a wait state).  The arithmetic is unpack_dequant's:
// stage 0 biased field, then + (bias - zero), * scale with integer zeros (bias + zero is exact, an integer
// below 2048), else + bias, - zero, * scale.  `live` false (a step past the end of this wavefront's share of
// K) gives zeros.  The per-chunk terms are written out at every call; calls on the same chunk share them.
template <int BITS, bool INTZ, int P, int STAGE>
__device__ __forceinline__ uint32_t unpack_stage(uint32_t t, const WChunk<BITS> &w, bool live, const UnpackConsts<BITS> &uc)
{
    constexpr int CLS = pair_class<BITS, P>();
    if constexpr (STAGE == 0) {
        return biased_pair<BITS, P>(w.c, uc);
    } else {
        const h2 zero2 = as_h2(w.zero * 0x10001u), scale2 = as_h2((live ? w.scale : 0u) * 0x10001u);
        if constexpr (INTZ)
            return as_u32(STAGE == 1 ? as_h2(t) + (uc.mb[CLS] - zero2) : as_h2(t) * scale2);
        else
            return as_u32(STAGE == 1 ? as_h2(t) + uc.mb[CLS] : STAGE == 2 ? as_h2(t) - zero2 : as_h2(t) * scale2);
    }
}
template <bool INTZ>
constexpr int unpack_stages() { return INTZ ? 3 : 4; }

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

// c += a . b with the accumulator held in place in an accumulator register.  Written as an instruction
// because the compiler, left to allocate 256 accumulator registers itself, moves them between register
// files around every MFMA.  The compiler does not know what this instruction is, so no result of it may be
// read by anything but another mfma_acc on the same accumulator before settle_mfma().
__device__ __forceinline__ void mfma_acc(f4 &c, h8 a, h8 b)
{
    asm("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
}
// the wait states between the last MFMA and the first other read of its result (at most 18 for this shape)
__device__ __forceinline__ void settle_mfma() { asm volatile("s_nop 15\n\ts_nop 15" ::: "memory"); }

__device__ __forceinline__ int tall_slot(int row, int ch) { return row * 8 + (ch ^ ((row >> 1) & 7)); }

// One 256 x 128 output tile.  Xs: [K half][buffer][TSLOTS]; after the loop the same memory carries the
// second K half's partial sums to the first.
template <int BITS>
__device__ __forceinline__ void qgemm_tall_tile(h8 (*Xs)[2][TSLOTS], const _Float16 *__restrict__ x, int M,
                                                const uint32_t *__restrict__ packed,
                                                const _Float16 *__restrict__ scales,
                                                const _Float16 *__restrict__ zeros, int N, int K,
                                                _Float16 *__restrict__ out, int tile)
{
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kh = wave >> 1, nw = wave & 1; // half of K, half of the tile's weight rows
    const int NT = (N + TBN - 1) / TBN, MT = (M + TBM - 1) / TBM;
    const int band = tile / (4 * NT), rest = tile - band * 4 * NT, height = min(4, MT - 4 * band);
    const int m0 = (4 * band + rest % height) * TBM, n0 = (rest / height) * TBN;
    const int G = K >> 7, Gh = (G + 1) >> 1;
    const int g0 = kh * Gh, gcount = min(G - g0, Gh); // this half's groups; the other half runs as many steps
    const int Np16 = ((N + 63) / 64 * 64) >> 4;
    const int rb0 = (n0 >> 4) + nw * TNB;

    GemmBuffers buf;
    buf.x = make_rsrc(x, (uint32_t)M * (uint32_t)K * 2u);
    const uint32_t Np = (uint32_t)(N + 63) / 64u * 64u;
    buf.packed = make_rsrc(packed, Np / 8u * (uint32_t)K * (uint32_t)BITS);
    buf.scales = make_rsrc(scales, Np * (uint32_t)G * 2u);
    buf.zeros = make_rsrc(zeros, Np * (uint32_t)G * 2u);

    // Activation copies: a K half's tile (256 rows x 64 k) is filled by its two wavefronts, 16 copies of 1 KiB
    // each; copy i of a wavefront fills the slots of rows 128*nw + 8*i + lane/8, position lane%8, which holds
    // chunk position ^ (row/2)%8.  Rows past M re-read row M-1.
    uint32_t xoff[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int row = 128 * nw + 8 * i + (lane >> 3), ch = (lane & 7) ^ ((row >> 1) & 7);
        xoff[i] = ((uint32_t)min(m0 + row, M - 1) * (uint32_t)K + (uint32_t)ch * 8u) * 2u;
    }
    auto copy_x = [&](int buffer, int step) { // step of this half: group g0 + step/2, k-steps 2*(step%2)..+1
        const uint32_t koff = (uint32_t)min(g0 + (step >> 1), G - 1) * 256u + (uint32_t)(step & 1) * 128u;
#pragma unroll
        for (int i = 0; i < 16; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(buf.x, &Xs[kh][buffer][(128 * nw + 8 * i) * 8], 16, xoff[i], koff, 0, 0);
    };

    f4 acc[TNB][TMB];
#pragma unroll
    for (int i = 0; i < TNB; ++i)
#pragma unroll
        for (int j = 0; j < TMB; ++j)
            acc[i][j] = f4{0.f, 0.f, 0.f, 0.f};

    WChunk<BITS> wcur[TNB], wnext[TNB];
    auto load_group = [&](WChunk<BITS> (&w)[TNB], int gl) {
#pragma unroll
        for (int i = 0; i < TNB; ++i)
            load_wchunk<BITS>(w[i], buf, rb0 + i, Np16, G, K, min(g0 + gl, G - 1), lane);
    };
    copy_x(0, 0);
    load_group(wcur, 0);
    __builtin_amdgcn_s_waitcnt(FQ_WAIT_VMCNT0);
    __syncthreads();

    // integer zeros: one addition takes bias and zero away (see qgemm_tile)
    bool intz;
    {
        const uint32_t first = (uint32_t)(n0 >> 4) * (uint32_t)G * 16u, count = (TBN / 16) * (uint32_t)G * 16u;
        int frac = 0;
        for (uint32_t i = (uint32_t)tid * 8u; i < count; i += 256u * 8u) {
            const h8 z = __builtin_bit_cast(h8, buf_load_b128(buf.zeros, (first + i) * 2u, 0));
#pragma unroll
            for (int e = 0; e < 8; ++e)
                frac |= z[e] != __builtin_truncf16(z[e]);
        }
        intz = !__syncthreads_or(frac);
    }

    UnpackConsts<BITS> uc;
    uc.init();
    const int brow = lane & 15, bsw = (brow >> 1) & 7;
    const int bslot0 = brow * 8 + ((lane >> 4) ^ bsw), bslot1 = brow * 8 + ((4 + (lane >> 4)) ^ bsw);

    // A step (64 k) is eight sections of 16 MFMAs: section sec multiplies k-step sec/4 of the step with the four
    // activation row blocks 4*(sec%4)..+3.  The wavefront is alone on its SIMD, so its own instruction order is
    // the overlap: every MFMA is preceded by a few instructions of other work that issue while the previous
    // MFMA occupies the pipe (four issue slots each), and nothing moves between these slots.  Per section: the
    // four operand reads of the next section (two sets of registers), one operand register of the next step
    // unpacked per four MFMAs; the copies of the next step's activations go out over the first two sections
    // and the next group's weight loads in the third, so that they have most of a step to land; the barrier
    // sits ahead of the last section's MFMAs, which cover the first reads of the next step.
    auto main_loop = [&](auto intz_tag) {
        constexpr bool INTZ = decltype(intz_tag)::value;
        u4v ap[TNB][2], aq[TNB][2]; // operands as four registers of one pair each
        h8 b[2][4];
        auto read_b = [&](h8 &dst, int buffer, int sec, int jj) {
            dst = Xs[kh][buffer][((sec >> 2) ? bslot1 : bslot0) + ((sec & 3) * 4 + jj) * 128];
        };
        auto step = [&](int buffer, int next_step, u4v (&ac)[TNB][2], auto other_work) {
            const uint32_t koff = (uint32_t)min(g0 + (next_step >> 1), G - 1) * 256u + (uint32_t)(next_step & 1) * 128u;
            static_for<8>([&](auto sec_tag) {
                constexpr int sec = decltype(sec_tag)::value;
                if constexpr (sec == 7) {
                    __builtin_amdgcn_s_waitcnt(0x0070); // vmcnt(0), lgkmcnt(0): copies, weights, operand reads
                    __syncthreads();                    // the other buffer is complete, this one is free
                    __builtin_amdgcn_sched_barrier(0);
                }
                static_for<16>([&](auto m_tag) {
                    constexpr int m = decltype(m_tag)::value, jj = m >> 2, i = m & 3;
                    if constexpr (m < 4) {
                        if constexpr (sec < 7)
                            read_b(b[(sec + 1) & 1][m], buffer, sec + 1, m);
                        else
                            read_b(b[0][m], buffer ^ 1, 0, m);
                    }
                    if constexpr (sec < 2 && (m & 1) == 0) { // copy 8*sec + m/2 of the next step's activations
                        constexpr int c = 8 * sec + m / 2;
                        __builtin_amdgcn_raw_ptr_buffer_load_lds(buf.x, &Xs[kh][buffer ^ 1][(128 * nw + 8 * c) * 8], 16,
                                                                 xoff[c], koff, 0, 0);
                    }
                    other_work(sec_tag, m_tag);
                    mfma_acc(acc[i][(sec & 3) * 4 + jj], __builtin_bit_cast(h8, ac[i][sec >> 2]), b[sec & 1][jj]);
                    __builtin_amdgcn_sched_barrier(0);
                });
            });
        };
        // the next step's operand of this section (chunk sec/2, k-step KS0 + sec%2): pairs 0,1 in slots 4.., pairs
        // 2,3 in slots 8.., one stage of both pairs per slot
        uint32_t st[2];
        auto unpack_slot = [&](auto ks_tag, auto m_tag, const WChunk<BITS> &w, bool live, u4v &dst) {
            constexpr int KS = decltype(ks_tag)::value, m = decltype(m_tag)::value, NST = unpack_stages<INTZ>();
            constexpr int duo = (m >> 2) - 1, stage = m & 3;
            if constexpr ((duo == 0 || duo == 1) && stage < NST) {
                constexpr int P = 4 * KS + 2 * duo;
                st[0] = unpack_stage<BITS, INTZ, P, stage>(st[0], w, live, uc);
                st[1] = unpack_stage<BITS, INTZ, P + 1, stage>(st[1], w, live, uc);
                if constexpr (stage == NST - 1) {
                    dst[2 * duo] = st[0];
                    dst[2 * duo + 1] = st[1];
                }
            }
        };
        static_for<TNB>([&](auto i_tag) {
            constexpr int i = decltype(i_tag)::value;
            static_for<2>([&](auto ks_tag) {
                static_for<8>([&](auto m8_tag) {
                    unpack_slot(ks_tag, std::integral_constant<int, 4 + decltype(m8_tag)::value>{}, wcur[i], gcount > 0,
                                ap[i][decltype(ks_tag)::value]);
                });
            });
        });
#pragma unroll
        for (int jj = 0; jj < 4; ++jj)
            read_b(b[0][jj], 0, 0, jj);
        for (int gl = 0; gl < Gh; ++gl) {
            // first half of the group; meanwhile k-steps 2 and 3 of this group's chunks become operands, and
            // the next group's chunks are requested
            step(0, 2 * gl + 1, ap, [&](auto sec_tag, auto m_tag) {
                constexpr int sec = decltype(sec_tag)::value, m = decltype(m_tag)::value;
                if constexpr (sec == 2 && (m & 3) == 0)
                    load_wchunk<BITS>(wnext[m >> 2], buf, rb0 + (m >> 2), Np16, G, K, min(g0 + gl + 1, G - 1), lane);
                unpack_slot(std::integral_constant<int, 2 + (sec & 1)>{}, m_tag, wcur[sec >> 1], gl < gcount,
                            aq[sec >> 1][sec & 1]);
            });
            // second half; k-steps 0 and 1 of the next group's chunks become operands
            step(1, 2 * gl + 2, aq, [&](auto sec_tag, auto m_tag) {
                constexpr int sec = decltype(sec_tag)::value;
                unpack_slot(std::integral_constant<int, (sec & 1)>{}, m_tag, wnext[sec >> 1], gl + 1 < gcount,
                            ap[sec >> 1][sec & 1]);
            });
#pragma unroll
            for (int i = 0; i < TNB; ++i)
                wcur[i] = wnext[i];
        }
    };
    if (intz)
        main_loop(std::true_type{});
    else
        main_loop(std::false_type{});

    settle_mfma();
    // the second K half hands its sums over: block (i, j) of column half nw at float4 ((nw*64 + i*16 + j)*64 + lane)
    f4 *red = reinterpret_cast<f4 *>(&Xs[0][0][0]);
    if (kh == 1) {
#pragma unroll
        for (int i = 0; i < TNB; ++i)
#pragma unroll
            for (int j = 0; j < TMB; ++j)
                red[((nw * 64 + i * 16 + j) << 6) + lane] = acc[i][j];
    }
    __syncthreads();
    if (kh == 1)
        return;
    // store: lane holds m = lane%16 and n = 4*(lane/16) + v of each 16x16 block
#pragma unroll
    for (int j = 0; j < TMB; ++j) {
        const int m = m0 + j * 16 + (lane & 15);
#pragma unroll
        for (int i = 0; i < TNB; ++i) {
            const f4 r = acc[i][j] + red[((nw * 64 + i * 16 + j) << 6) + lane];
            const int n = (rb0 + i) * 16 + 4 * (lane >> 4);
            if (m >= M)
                continue;
            _Float16 *o = out + (size_t)m * N + n;
            if (n + 3 < N && (N & 3) == 0) {
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
    int N, bits, tile0;
};
struct TallJobs {
    TallJob j[3];
    int count, total;
};

// One wavefront per SIMD: the whole register file (256 vector + 256 accumulator registers) belongs to it.
__global__ __launch_bounds__(256, 1) void qgemm_tall_kernel(const _Float16 *__restrict__ x, int M, int K, TallJobs jobs)
{
    __shared__ h8 Xs[2][2][TSLOTS];
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
    case 2: qgemm_tall_tile<2>(Xs, x, M, job.packed, job.scales, job.zeros, job.N, K, job.out, tile); break;
    case 3: qgemm_tall_tile<3>(Xs, x, M, job.packed, job.scales, job.zeros, job.N, K, job.out, tile); break;
    case 4: qgemm_tall_tile<4>(Xs, x, M, job.packed, job.scales, job.zeros, job.N, K, job.out, tile); break;
    default: qgemm_tall_tile<8>(Xs, x, M, job.packed, job.scales, job.zeros, job.N, K, job.out, tile); break;
    }
}

// Weight-tile width.  Wide tiles (each wavefront 128 x 64) halve the LDS reads and activation copies per
// MFMA but need at least two workgroups per CU to keep both wavefront slots of every SIMD filled.
int wide_tiles_pay(int M, int N)
{
    const long tiles = (long)((N + 255) / 256) * ((M + QBM - 1) / QBM);
    return tiles >= 2 * 256;
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
    for (int i = 0; i < count; ++i)
        if (w[i].ld && w[i].ld != w[i].N)
            return (int)hipErrorInvalidValue; // this kernel writes outputs of their own only
    TallJobs jobs;
    jobs.count = count;
    int total = 0;
    for (int i = 0; i < count; ++i) {
        jobs.j[i] = TallJob{static_cast<const uint32_t *>(w[i].packed), static_cast<const _Float16 *>(w[i].scales),
                            static_cast<const _Float16 *>(w[i].zeros), static_cast<_Float16 *>(outs[i]), w[i].N,
                            w[i].bits, total};
        total += ((w[i].N + TBN - 1) / TBN) * ((M + TBM - 1) / TBM);
    }
    jobs.total = total;
    hipLaunchKernelGGL(qgemm_tall_kernel, dim3(8 * ((total + 7) / 8)), dim3(256), 0, st,
                       static_cast<const _Float16 *>(x), M, w[0].K, jobs);
    return (int)hipGetLastError();
}

int fq_launch_gemm(const void *x, int M, const fq_packed_ref &w, void *out, fq_stream st, int tile_rows)
{
    const size_t Np = ((size_t)w.N + 63) / 64 * 64;
    if (!fits_32bit(M, w.K, 2) || Np / 8 * w.K * w.bits >= ((size_t)1 << 32))
        return (int)hipErrorInvalidValue;
    if (tile_rows == 256) // never the library's own choice: as measured the 128-row kernels are faster
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
