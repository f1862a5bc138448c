// Unquantized fp16 GEMM for many rows: out[M,N] = x[M,K] . W[N,K]^T, the vocabulary head of the
// calibration forward (FlexQuant, arXiv 2501.07139, Algorithm 1, calibrationEval: the logits whose
// token losses give a candidate's perplexity).
//
// Neither operand needs unpacking, so both go through LDS and every workgroup owns a large output tile:
// 256 activation rows x 256 weight rows, 64 k per iteration, 512 threads = 8 wavefronts in a 2 (rows) x
// 4 (weights) grid, each 128 x 64 = 8 x 4 blocks of 16x16x32 fp16 MFMA with fp32 accumulators.  Per 32
// MFMAs a wavefront reads 12 operands from LDS, and a CU fetches 64 KiB per 8.4 MFLOP.  Both tiles are
// copied from global memory straight into a double-buffered LDS tile (128 KiB, one workgroup per CU),
// row-major with the eight 16-byte chunks of a row XOR-swizzled by (row / 2) % 8: the copy writes whole
// rows and the operand reads of sixteen rows by one chunk touch every bank once.  The copy of iteration
// kt+1 is issued before the MFMAs of iteration kt; one barrier per iteration.
//
// Fused loss (the same calibrationEval, logits never stored): instead of writing its 128 x 64 logits a
// wavefront rounds them to fp16, as the stored logits would be, and reduces every row to the pair
// (maximum, sum of exp(logit - maximum)) over its 64 columns; a second small kernel merges a row's pairs
// over the vocabulary and subtracts the label's logit, which the one lane that holds it has set aside.
#include "fq_device.h"
#include "fq_internal.h"
#include "fq_lse.h"

namespace {

constexpr int DT = 256;        // tile rows of either operand
constexpr int DK = 64;         // k per iteration: 8 chunks of 16 bytes per row
constexpr int DSLOTS = DT * 8; // 16-byte slots of one operand tile

__device__ __forceinline__ int dense_slot(int row, int ch) { return row * 8 + (ch ^ ((row >> 1) & 7)); }

// What the fused-loss variant writes instead of logits.
struct LossParts {
    const int32_t *labels; // [M]
    float2 *pairs;         // [M][ceil(N / 64)]: (maximum, sum of exp(logit - maximum)) of 64 columns
    float *label_logit;    // [M]: the label's logit, written only where the label is in range
};

template <bool FUSED>
__global__ __launch_bounds__(512, 2) void dense_kernel(const _Float16 *__restrict__ x, int M,
                                                       const _Float16 *__restrict__ W, int N, int K,
                                                       _Float16 *__restrict__ out, LossParts loss)
{
    __shared__ h8 tiles[2][2][DSLOTS]; // [buffer][0: activations, 1: weights]

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 1, wn = wave >> 1;
    // Workgroups go to the eight XCDs round-robin, each with its own L2: XCD x takes the x-th contiguous
    // run of tiles, ordered in bands of four activation row-tiles (row-tile fastest).
    const int NT = (N + DT - 1) / DT, MT = (M + DT - 1) / DT, total = NT * MT;
    const int per_xcd = (total + 7) >> 3;
    const int tile = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (tile >= total)
        return; // uniform over the workgroup, before any barrier
    const int band = tile / (4 * NT), rest = tile - band * 4 * NT, height = min(4, MT - 4 * band);
    const int m0 = (4 * band + rest % height) * DT, n0 = (rest / height) * DT;
    const int KT = K / DK;

    // The i-th copy of a wavefront fills the 64 slots from 64*wave + 512*i of a tile, lane by lane: rows
    // 8*wave + 64*i + lane/8, position lane%8, which holds chunk position ^ (row/2)%8 (the same for every
    // i).  Rows past the end of an operand re-read its last row; their products are never stored.
    const int crow = 8 * wave + (lane >> 3), cch = (lane & 7) ^ ((crow >> 1) & 7);
    uint32_t xoff[4], woff[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        xoff[i] = ((uint32_t)min(m0 + crow + 64 * i, M - 1) * (uint32_t)K + (uint32_t)cch * 8u) * 2u;
        woff[i] = ((uint32_t)min(n0 + crow + 64 * i, N - 1) * (uint32_t)K + (uint32_t)cch * 8u) * 2u;
    }
    const fq_rsrc xr = make_rsrc(x, (uint32_t)M * (uint32_t)K * 2u);
    const fq_rsrc wr = make_rsrc(W, (uint32_t)N * (uint32_t)K * 2u);

    auto copy_tiles = [&](int buffer, int kt) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(xr, &tiles[buffer][0][64 * wave + 512 * i], 16, xoff[i],
                                                     (uint32_t)kt * (DK * 2u), 0, 0);
#pragma unroll
        for (int i = 0; i < 4; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(wr, &tiles[buffer][1][64 * wave + 512 * i], 16, woff[i],
                                                     (uint32_t)kt * (DK * 2u), 0, 0);
    };

    f4 acc[4][8];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j)
            acc[i][j] = f4{0.f, 0.f, 0.f, 0.f};

    copy_tiles(0, 0);
    __builtin_amdgcn_s_waitcnt(FQ_WAIT_VMCNT0);
    __syncthreads();

    for (int kt = 0; kt < KT; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < KT)
            copy_tiles(cur ^ 1, kt + 1);
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int ch = 4 * s + (lane >> 4);
            h8 a[4], b[8];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                a[i] = tiles[cur][1][dense_slot(64 * wn + 16 * i + (lane & 15), ch)];
#pragma unroll
            for (int j = 0; j < 8; ++j)
                b[j] = tiles[cur][0][dense_slot(128 * wm + 16 * j + (lane & 15), ch)];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    acc[i][j] = mfma16x16x32(a[i], b[j], acc[i][j]);
        }
        __builtin_amdgcn_s_waitcnt(FQ_WAIT_VMCNT0); // this wavefront's copies have landed ...
        __syncthreads();                            // ... and everyone's, and all reads of `cur` are done
    }

    // lane holds m = lane%16 and n = 4*(lane/16) + v of each 16x16 block
    if constexpr (FUSED) {
        const int nw = n0 + 64 * wn, NC = (N + 63) >> 6;
        if (nw >= N)
            return; // no column of this wavefront exists (after the last barrier)
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int m = m0 + 128 * wm + 16 * j + (lane & 15);
            const int label = m < M ? loss.labels[m] : -1;
            float l[16], mx = -INFINITY;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int n = nw + 16 * i + 4 * (lane >> 4) + v;
                    const float logit = (float)(_Float16)acc[i][j][v]; // what the stored fp16 logit would hold
                    l[4 * i + v] = n < N ? logit : -INFINITY;
                    mx = fmaxf(mx, l[4 * i + v]);
                    if (n == label)
                        loss.label_logit[m] = logit;
                }
            float se = 0.f;
            if (mx != -INFINITY) {
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    se += __expf(l[e] - mx);
            }
#pragma unroll
            for (int o = 16; o <= 32; o <<= 1) { // the four lanes that share a row
                const float m2 = __shfl_xor(mx, o, 64), s2 = __shfl_xor(se, o, 64);
                lse_merge(mx, se, m2, s2);
            }
            if (lane < 16 && m < M)
                loss.pairs[(size_t)m * NC + (nw >> 6)] = make_float2(mx, se);
        }
        return;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int m = m0 + 128 * wm + 16 * j + (lane & 15);
        if (m >= M)
            continue;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int n = n0 + 64 * wn + 16 * i + 4 * (lane >> 4);
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

// One wavefront per row: merge the row's pairs, then nll = log(sum of exp) - label's logit; a label outside
// [0, V) gives 0, as in the unfused loss.
__global__ __launch_bounds__(64) void loss_finish_kernel(LossParts loss, int V, float *__restrict__ nll)
{
    const int row = blockIdx.x, lane = threadIdx.x, NC = (V + 63) >> 6;
    const int label = loss.labels[row];
    if (label < 0 || label >= V) { // uniform across the wavefront
        if (lane == 0)
            nll[row] = 0.f;
        return;
    }
    float mx = -INFINITY, se = 0.f;
    for (int c = lane; c < NC; c += 64) {
        const float2 p = loss.pairs[(size_t)row * NC + c];
        lse_merge(mx, se, p.x, p.y);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float m2 = __shfl_xor(mx, o, 64), s2 = __shfl_xor(se, o, 64);
        lse_merge(mx, se, m2, s2);
    }
    if (lane == 0)
        nll[row] = logf(se) + (mx - loss.label_logit[row]); // difference first: exact for fp16 inputs
}

} // namespace

// Large tiles pay from about half a tile per CU on (measured: 128 tiles of 2048 x 4096 already run 12 % faster
// than 512 tiles of 128 rows); below that the smaller tiles spread the work over more CUs.
bool fq_dense_tiled_pays(int M, int N) { return (long)((M + DT - 1) / DT) * ((N + DT - 1) / DT) >= 128; }

// x and W are addressed through 32-bit byte offsets (checked by the caller); K is a multiple of 128.
int fq_launch_dense_tiled(const void *x, int M, const void *W, int N, int K, void *out, fq_stream st)
{
    const int total = ((N + DT - 1) / DT) * ((M + DT - 1) / DT);
    dim3 grid(8 * ((total + 7) / 8)), block(512);
    hipLaunchKernelGGL(dense_kernel<false>, grid, block, 0, st, static_cast<const _Float16 *>(x), M,
                       static_cast<const _Float16 *>(W), N, K, static_cast<_Float16 *>(out), LossParts{});
    return (int)hipGetLastError();
}

size_t fq_head_nll_scratch_bytes(int M, int V)
{
    const size_t pairs = (size_t)M * ((V + 63) / 64) * sizeof(float2);
    return pairs + (size_t)M * sizeof(float);
}

// workspace: fq_head_nll_scratch_bytes(M, V) bytes, 8-byte aligned.
int fq_launch_head_nll(const void *x, int M, const void *W, int V, int K, const int32_t *labels, float *nll,
                       void *workspace, fq_stream st)
{
    LossParts loss;
    loss.labels = labels;
    loss.pairs = static_cast<float2 *>(workspace);
    loss.label_logit = reinterpret_cast<float *>(loss.pairs + (size_t)M * ((V + 63) / 64));
    const int total = ((V + DT - 1) / DT) * ((M + DT - 1) / DT);
    dim3 grid(8 * ((total + 7) / 8)), block(512);
    hipLaunchKernelGGL(dense_kernel<true>, grid, block, 0, st, static_cast<const _Float16 *>(x), M,
                       static_cast<const _Float16 *>(W), V, K, static_cast<_Float16 *>(nullptr), loss);
    int rc = (int)hipGetLastError();
    if (rc != 0)
        return rc;
    hipLaunchKernelGGL(loss_finish_kernel, dim3(M), dim3(64), 0, st, loss, V, nll);
    return (int)hipGetLastError();
}
