// Calibration-forward path: dequant-GEMM for M > 16 rows of activations, and the
// unquantized fp16 head GEMM.
//
// Scoring one candidate hybrid model means a full forward of the calibration
// sequences (FlexQuant, arXiv 2501.07139, Algorithm 1, calibrationEval), which is
// a dense contraction: packed weights are unpacked and dequantized once per
// workgroup tile into fp16 operand fragments in LDS and consumed by 16x16x32
// MFMA with fp32 accumulation.
//
// Tile: BM activation rows x BN weight rows x one group of 128 k per step,
// 256 threads = 2x2 wavefronts.  The weight fragments sit in LDS in operand
// order (every read and write is a contiguous 1 KiB per wavefront); the
// activation tile is row-major with its 16-byte chunks XOR-swizzled by row so
// that both the coalesced global->LDS copy and the operand reads are free of
// bank conflicts.
#include "fq_device.h"
#include "fq_internal.h"

namespace {

constexpr int DENSE = 16; // BITS value selecting the fp16 weight path

template <int BITS, int BM, int BN>
__global__ __launch_bounds__(256) void gemm_kernel(const _Float16 *__restrict__ x, int M,
                                                   const uint32_t *__restrict__ packed,
                                                   const _Float16 *__restrict__ scales,
                                                   const _Float16 *__restrict__ zeros,
                                                   int N, int K, _Float16 *__restrict__ out)
{
    constexpr int WM = BM / 2, WN = BN / 2; // per-wave tile
    constexpr int MB = WM / 16, NB = WN / 16;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    h8 *Xs = reinterpret_cast<h8 *>(smem);                // [BM][16 chunks], chunk ch of row r at r*16 + (ch ^ (r & 15))
    h8 *Ws = reinterpret_cast<h8 *>(smem + BM * 256);     // packed: [BN/16][4 k-steps][64 lanes]; dense: like Xs

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int G = K >> 7;
    const int Np16 = ((N + 63) / 64 * 64) >> 4; // sixteen-row blocks that exist in the packed buffer

    f4 acc[NB][MB];
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
        for (int j = 0; j < MB; ++j)
            acc[i][j] = f4{0.f, 0.f, 0.f, 0.f};

    for (int g = 0; g < G; ++g) {
        // ---- activations: BM rows x 16 chunks of 8 halves
#pragma unroll
        for (int i = 0; i < BM * 16 / 256; ++i) {
            const int idx = tid + 256 * i;
            const int row = idx >> 4, ch = idx & 15;
            const int mrow = min(m0 + row, M - 1);
            Xs[row * 16 + (ch ^ (row & 15))] =
                *reinterpret_cast<const h8 *>(x + (size_t)mrow * K + g * 128 + ch * 8);
        }
        // ---- weights
        if constexpr (BITS == DENSE) {
            const _Float16 *Wd = reinterpret_cast<const _Float16 *>(packed);
#pragma unroll
            for (int i = 0; i < BN * 16 / 256; ++i) {
                const int idx = tid + 256 * i;
                const int row = idx >> 4, ch = idx & 15;
                const int nrow = min(n0 + row, N - 1);
                Ws[row * 16 + (ch ^ (row & 15))] =
                    *reinterpret_cast<const h8 *>(Wd + (size_t)nrow * K + g * 128 + ch * 8);
            }
        } else {
            constexpr int SUB = Fmt<BITS>::SUB;
            constexpr int TILE = tile_dwords<BITS>();
#pragma unroll
            for (int i = 0; i < BN / 64; ++i) {
                const int blk = wave + 4 * i;        // sixteen-row block inside the tile
                const int rb16 = (n0 >> 4) + blk;    // ... and in the matrix
                h8 *dst = Ws + (blk * 4) * 64 + lane;
                if (rb16 < Np16) {
                    const int sr = rb16 / SUB, u = rb16 % SUB;
                    const uint32_t *tile = packed + ((size_t)sr * G + g) * TILE;
                    uint32_t C[BITS];
                    load_chunk<BITS>(tile, u, lane, C);
                    const size_t meta = ((size_t)rb16 * G + g) * 16 + (lane & 15);
                    const _Float16 z = zeros[meta], sc = scales[meta];
                    h2 q[16];
                    unpack_codes<BITS>(C, q);
                    const h2 z2 = {z, z}, s2 = {sc, sc};
#pragma unroll
                    for (int p = 0; p < 16; ++p)
                        q[p] = (q[p] - z2) * s2;
#pragma unroll
                    for (int s = 0; s < 4; ++s)
                        dst[s * 64] = make_h8(q[4 * s], q[4 * s + 1], q[4 * s + 2], q[4 * s + 3]);
                } else {
#pragma unroll
                    for (int s = 0; s < 4; ++s)
                        dst[s * 64] = h8{0, 0, 0, 0, 0, 0, 0, 0};
                }
            }
        }
        __syncthreads();
        // ---- contraction over the four k-steps of the group
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            h8 a[NB], b[MB];
#pragma unroll
            for (int i = 0; i < NB; ++i) {
                if constexpr (BITS == DENSE) {
                    const int row = wn * WN + i * 16 + (lane & 15), ch = 4 * s + (lane >> 4);
                    a[i] = Ws[row * 16 + (ch ^ (row & 15))];
                } else {
                    a[i] = Ws[((wn * NB + i) * 4 + s) * 64 + lane];
                }
            }
#pragma unroll
            for (int j = 0; j < MB; ++j) {
                const int row = wm * WM + j * 16 + (lane & 15), ch = 4 * s + (lane >> 4);
                b[j] = Xs[row * 16 + (ch ^ (row & 15))];
            }
#pragma unroll
            for (int i = 0; i < NB; ++i)
#pragma unroll
                for (int j = 0; j < MB; ++j)
                    acc[i][j] = mfma16x16x32(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }

    // ---- store: lane holds m = lane%16, n = 4*(lane/16) + v of each 16x16 block
#pragma unroll
    for (int j = 0; j < MB; ++j) {
        const int m = m0 + wm * WM + j * 16 + (lane & 15);
        if (m >= M)
            continue;
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int n = n0 + wn * WN + i * 16 + 4 * (lane >> 4);
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

template <int BITS, int BM, int BN>
int launch(const void *x, int M, const void *packed, const void *scales, const void *zeros, int N, int K,
           void *out, fq_stream st)
{
    constexpr size_t lds = (size_t)(BM + BN) * 256;
    auto kern = gemm_kernel<BITS, BM, BN>;
    static bool configured = false;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess)
            return (int)e;
        configured = true;
    }
    dim3 grid((N + BN - 1) / BN, (M + BM - 1) / BM), block(256);
    hipLaunchKernelGGL(kern, grid, block, lds, st, static_cast<const _Float16 *>(x), M,
                       static_cast<const uint32_t *>(packed), static_cast<const _Float16 *>(scales),
                       static_cast<const _Float16 *>(zeros), N, K, static_cast<_Float16 *>(out));
    return (int)hipGetLastError();
}

} // namespace

int fq_launch_gemm(const void *x, int M, const fq_packed_ref &w, void *out, fq_stream st)
{
    constexpr int BM = 256, BN = 128;
    switch (w.bits) {
    case 2: return launch<2, BM, BN>(x, M, w.packed, w.scales, w.zeros, w.N, w.K, out, st);
    case 3: return launch<3, BM, BN>(x, M, w.packed, w.scales, w.zeros, w.N, w.K, out, st);
    case 4: return launch<4, BM, BN>(x, M, w.packed, w.scales, w.zeros, w.N, w.K, out, st);
    default: return launch<8, BM, BN>(x, M, w.packed, w.scales, w.zeros, w.N, w.K, out, st);
    }
}

int fq_launch_dense(const void *x, int M, const void *W, int N, int K, void *out, fq_stream st)
{
    return launch<DENSE, 256, 128>(x, M, W, nullptr, nullptr, N, K, out, st);
}
