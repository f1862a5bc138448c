// Decode path: dequant-GEMV for 1 <= M <= 16 rows of activations.
//
// The served hybrid model generates one token at a time on a memory-constrained
// device (FlexQuant, arXiv 2501.07139, Section "Introduction"), so this kernel
// is bound by streaming the packed weights once.  Each wavefront owns a
// supertile row (16/32/64 weight rows) and walks the groups of 128 k: one
// 128-bit load per lane per plane (1 KiB contiguous per wavefront), unpack in
// registers straight into matrix-core operands, 16x16x32 MFMA against the x
// fragment (columns = the M activation rows), then one fp32 multiply-add per
// group applies the scale.  Waves of a workgroup split the groups and reduce
// through LDS in a fixed order, so results are deterministic.
#include "fq_device.h"
#include "fq_internal.h"

namespace {

template <int BITS, int NWAVES>
__global__ __launch_bounds__(64 * NWAVES) void gemv_kernel(const _Float16 *__restrict__ x, int M,
                                                           const uint32_t *__restrict__ packed,
                                                           const _Float16 *__restrict__ scales,
                                                           const _Float16 *__restrict__ zeros,
                                                           int N, int K, _Float16 *__restrict__ out)
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

    // fixed-order reduction over the waves of the workgroup
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
int launch(const void *x, int M, const fq_packed_ref &w, void *out, fq_stream st)
{
    constexpr int NWAVES = 4;
    const int Np = (w.N + 63) / 64 * 64;
    dim3 grid(Np / Fmt<BITS>::ROWS), block(64 * NWAVES);
    hipLaunchKernelGGL((gemv_kernel<BITS, NWAVES>), grid, block, 0, st,
                       static_cast<const _Float16 *>(x), M, static_cast<const uint32_t *>(w.packed),
                       static_cast<const _Float16 *>(w.scales), static_cast<const _Float16 *>(w.zeros),
                       w.N, w.K, static_cast<_Float16 *>(out));
    return (int)hipGetLastError();
}

} // namespace

int fq_launch_gemv(const void *x, int M, const fq_packed_ref &w, void *out, fq_stream st)
{
    switch (w.bits) {
    case 2: return launch<2>(x, M, w, out, st);
    case 3: return launch<3>(x, M, w, out, st);
    case 4: return launch<4>(x, M, w, out, st);
    default: return launch<8>(x, M, w, out, st);
    }
}
