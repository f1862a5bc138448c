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
                                           _Float16 *__restrict__ out, int tile)
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
    if constexpr (QNB == 4)
        main_loop(std::false_type{}); // the wide tile has no registers to spare for a second copy of the loop
    else if (intz)
        main_loop(std::true_type{});
    else
        main_loop(std::false_type{});

    // store: lane holds m = lane%16 and n = 4*(lane/16) + v of each 16x16 block
#pragma unroll
    for (int j = 0; j < QMB; ++j) {
        const int m = m0 + j * 16 + (lane & 15);
        if (m >= M)
            continue;
#pragma unroll
        for (int i = 0; i < QNB; ++i) {
            const int n = (rb0 + i) * 16 + 4 * (lane >> 4);
            _Float16 *o = out + (size_t)m * N + n;
            if (n + 3 < N && (N & 3) == 0) {
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
    qgemm_tile<BITS, QNB>(Xs, x, M, packed, scales, zeros, N, K, out, tile);
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
    case 2 * 8 + 4: qgemm_tile<2, 4>(Xs, x, M, job.packed, job.scales, job.zeros, job.N, K, job.out, tile); break;
    case 4 * 8 + 4: qgemm_tile<4, 4>(Xs, x, M, job.packed, job.scales, job.zeros, job.N, K, job.out, tile); break;
    case 2 * 8 + 2: qgemm_tile<2, 2>(Xs, x, M, job.packed, job.scales, job.zeros, job.N, K, job.out, tile); break;
    case 3 * 8 + 2: qgemm_tile<3, 2>(Xs, x, M, job.packed, job.scales, job.zeros, job.N, K, job.out, tile); break;
    case 4 * 8 + 2: qgemm_tile<4, 2>(Xs, x, M, job.packed, job.scales, job.zeros, job.N, K, job.out, tile); break;
    default: qgemm_tile<8, 2>(Xs, x, M, job.packed, job.scales, job.zeros, job.N, K, job.out, tile); break;
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

int fq_launch_gemm(const void *x, int M, const fq_packed_ref &w, void *out, fq_stream st)
{
    const size_t Np = ((size_t)w.N + 63) / 64 * 64;
    if (!fits_32bit(M, w.K, 2) || Np / 8 * w.K * w.bits >= ((size_t)1 << 32))
        return (int)hipErrorInvalidValue;
    switch (w.bits) {
    case 2: return launch_q<2>(x, M, w, out, st);
    case 3: return launch_q<3>(x, M, w, out, st);
    case 4: return launch_q<4>(x, M, w, out, st);
    default: return launch_q<8>(x, M, w, out, st);
    }
}

// Matrices that share x (same K): one launch.  Shapes are validated by the caller like fq_launch_gemm's.
int fq_launch_gemm_multi(const void *x, int M, const fq_packed_ref *w, void *const *outs, int count, fq_stream st)
{
    if (count < 1 || count > 3)
        return (int)hipErrorInvalidValue;
    GemmJobs jobs;
    jobs.count = count;
    int total = 0;
    for (int i = 0; i < count; ++i) {
        const size_t Np = ((size_t)w[i].N + 63) / 64 * 64;
        if (w[i].K != w[0].K || !fits_32bit(M, w[i].K, 2) || Np / 8 * w[i].K * w[i].bits >= ((size_t)1 << 32))
            return (int)hipErrorInvalidValue;
        const int qnb = ((w[i].bits == 2 || w[i].bits == 4) && wide_tiles_pay(M, w[i].N)) ? 4 : 2;
        jobs.j[i] = GemmJob{static_cast<const uint32_t *>(w[i].packed), static_cast<const _Float16 *>(w[i].scales),
                            static_cast<const _Float16 *>(w[i].zeros), static_cast<_Float16 *>(outs[i]), w[i].N,
                            w[i].bits, qnb, total};
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
