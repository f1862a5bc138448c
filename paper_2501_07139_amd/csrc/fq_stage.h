// Staging helpers shared by the decode kernels: the row-wise transforms between the linears of a block
// (folded into the staging of a linear's input), the per-group exponent and bit-field scaling of the staged
// activations, lane-group reductions, and the LDS-only workgroup barrier.
#ifndef FQ_STAGE_H
#define FQ_STAGE_H

#include "fq_device.h"

namespace {

// Workgroup barrier that orders LDS accesses only: waits for this wavefront's LDS operations, then for
// the other wavefronts.  __syncthreads() also fences, and in a kernel that copies into LDS through the
// vector-memory path the compiler makes that fence wait for every vector load in flight: here that
// would be the weights.  The memory clobber keeps the compiler from moving accesses across it.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Sum over each aligned run of 16 lanes, in all of its lanes: four adds whose second operand comes
// through the lane-permute path of the ALU (swap within pairs, swap pairs within quads, rotate the row
// by 4 and by 8).
__device__ __forceinline__ float row16_sum(float v)
{
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x124, 0xF, 0xF, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x128, 0xF, 0xF, true));
    return v;
}

// pair_shift for element e of k-step s: staged x carries the factor 2^-shift against its group's scale.
template <int BITS>
__host__ __device__ constexpr int stage_shift(int s, int e)
{
    return pair_shift<BITS>(4 * s + (e >> 1));
}

// Inputs the transform of each mode reads.
template <int MODE>
struct GemvInputs { static constexpr int N = MODE == 2 ? 3 : (MODE >= 3 ? 2 : 1); };

// One chunk (8 consecutive k) of the block's tensor that feeds the last rms.  Where that tensor is an
// fp16 one (modes 0, 1 and 3: a stored activation, or the stored sum of two) it stays in packed fp16: the
// packed add rounds a + b once, like the fp32 add followed by a conversion, since the fp32 sum of two
// fp16 numbers is exact or already beyond fp16's precision.  Otherwise it is held in fp32.
template <int MODE>
struct GemvChunk {
    static constexpr bool HALF = MODE == 0 || MODE == 1 || MODE == 3;
    h8 h;       // HALF
    float f[8]; // !HALF
};

template <int MODE>
__device__ __forceinline__ void gemv_combine(const h8 (&r)[GemvInputs<MODE>::N], GemvChunk<MODE> &v)
{
    if constexpr (MODE == 0 || MODE == 1) {
        v.h = r[0];
    } else if constexpr (MODE == 3) {
        v.h = r[0] + r[1];
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float t = (float)r[0][e];
            if constexpr (MODE == 2)
                t = t + (float)r[1][e] + (float)r[2][e];
            else if constexpr (MODE == 4 || MODE == 6)
                t = t * __builtin_amdgcn_rcpf(1.0f + __expf(-t)) * (float)r[1][e]; // reciprocal good to 1 ulp
            else
                t = t + (float)r[1][e];
            v.f[e] = t;
        }
    }
}

// sum of the squares / of the elements of a packed chunk, accumulated in fp32 (two products per instruction)
__device__ __forceinline__ float gemv_sumsq(h8 v, float acc)
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const h2 p = {v[2 * i], v[2 * i + 1]};
        acc = __builtin_amdgcn_fdot2(p, p, acc, false);
    }
    return acc;
}

__device__ __forceinline__ float gemv_sum(h8 v)
{
    const h2 one = {(_Float16)1.0f, (_Float16)1.0f};
    float acc = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const h2 p = {v[2 * i], v[2 * i + 1]};
        acc = __builtin_amdgcn_fdot2(p, one, acc, false);
    }
    return acc;
}

// v * scale in fp32, rounded to fp16
__device__ __forceinline__ h8 gemv_scaled(const float (&v)[8], float scale)
{
    h8 r;
#pragma unroll
    for (int e = 0; e < 8; ++e)
        r[e] = (_Float16)(v[e] * scale);
    return r;
}

__device__ __forceinline__ h8 gemv_scaled(h8 v, float scale)
{
    h8 r;
#pragma unroll
    for (int e = 0; e < 8; ++e)
        r[e] = (_Float16)((float)v[e] * scale);
    return r;
}

// The shifts of the four pairs of k-step s, four bits each (pair v = e/2 in bits 4v..4v+3).
template <int BITS>
__host__ __device__ constexpr uint32_t stage_shift_row(int s)
{
    return (uint32_t)stage_shift<BITS>(s, 0) | ((uint32_t)stage_shift<BITS>(s, 2) << 4) |
           ((uint32_t)stage_shift<BITS>(s, 4) << 8) | ((uint32_t)stage_shift<BITS>(s, 6) << 12);
}

// x * 2^(E - pair_shift) for the eight elements of a chunk of k-step s: exact while the result is a normal
// fp16 number, rounded to nearest below that.  s differs from lane to lane, so the row of shifts is
// selected, not branched on.
template <int BITS>
__device__ __forceinline__ h8 stage_scaled(h8 x, int s, int E)
{
    constexpr uint32_t r0 = stage_shift_row<BITS>(0), r1 = stage_shift_row<BITS>(1), r2 = stage_shift_row<BITS>(2),
                       r3 = stage_shift_row<BITS>(3);
    const uint32_t row = s == 0 ? r0 : (s == 1 ? r1 : (s == 2 ? r2 : r3));
    h8 w;
#pragma unroll
    for (int e = 0; e < 8; ++e)
        w[e] = __builtin_ldexpf16(x[e], E - (int)((row >> (4 * (e >> 1))) & 15u));
    return w;
}

// Largest |x| of a chunk as an fp16 bit pattern (positive fp16 numbers order like their bits), then over
// each aligned run of 16 lanes (the 128 values of a group), in all of its lanes.
__device__ __forceinline__ uint32_t group_max_bits(h8 x)
{
    const u4v v = __builtin_bit_cast(u4v, x) & 0x7fff7fffu;
    uint32_t m = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t d = i == 0 ? v.x : (i == 1 ? v.y : (i == 2 ? v.z : v.w));
        m = max(m, max(d & 0xffffu, d >> 16));
    }
    m = max(m, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)m, 0xB1, 0xF, 0xF, true));
    m = max(m, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)m, 0x4E, 0xF, 0xF, true));
    m = max(m, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)m, 0x124, 0xF, 0xF, true));
    m = max(m, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)m, 0x128, 0xF, 0xF, true));
    return m;
}

// s_waitcnt immediate: vector-memory loads in flight <= n (n < 64), the other counters left alone
constexpr int gemv_wait_vmcnt(int n) { return 0x0f70 | (n & 15) | ((n >> 4) << 14); }

} // namespace

#endif
