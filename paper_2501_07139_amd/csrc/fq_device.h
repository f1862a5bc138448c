// Device-side helpers: vector types, the packed-format constants and the
// per-bit-width unpack routines.  One specialisation per bit-width; nothing here
// branches on the bit-width at run time.
#ifndef FQ_DEVICE_H
#define FQ_DEVICE_H

#include <hip/hip_runtime.h>
#include <stdint.h>

typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u2v __attribute__((ext_vector_type(2)));
typedef uint32_t u4v __attribute__((ext_vector_type(4)));

// s_waitcnt immediate that waits for all vector-memory loads only (vmcnt = 0, expcnt and lgkmcnt left at their maxima)
#define FQ_WAIT_VMCNT0 0x0f70

__device__ __forceinline__ h2 as_h2(uint32_t u) { return __builtin_bit_cast(h2, u); }
__device__ __forceinline__ uint32_t as_u32(h2 h) { return __builtin_bit_cast(uint32_t, h); }

// Packed-format constants.  A supertile is ROWS rows by 128 k and holds
// ROWS/16 sixteen-row sub-blocks; each lane owns BITS dwords per sub-block.
template <int BITS>
struct Fmt;
template <>
struct Fmt<2> { static constexpr int ROWS = 32, SUB = 2, PLANES = 1; };
template <>
struct Fmt<3> { static constexpr int ROWS = 64, SUB = 4, PLANES = 3; };
template <>
struct Fmt<4> { static constexpr int ROWS = 16, SUB = 1, PLANES = 1; };
template <>
struct Fmt<8> { static constexpr int ROWS = 16, SUB = 1, PLANES = 2; };

template <int BITS>
__host__ __device__ constexpr int tile_dwords() { return Fmt<BITS>::ROWS * 4 * BITS; }

// Dword j of lane `lane` inside a supertile (dword offset from the supertile base).
__device__ __forceinline__ int lane_dword(int j, int lane) { return (j >> 2) * 256 + lane * 4 + (j & 3); }

// Load the BITS dwords of sub-block `u` owned by `lane`.  Adjacent dwords merge
// into 64/96/128-bit loads where the format makes them contiguous.
template <int BITS>
__device__ __forceinline__ void load_chunk(const uint32_t *tile, int u, int lane, uint32_t (&C)[BITS])
{
    if constexpr (BITS == 4) {
        u4v v = *reinterpret_cast<const u4v *>(tile + lane * 4);
        C[0] = v.x; C[1] = v.y; C[2] = v.z; C[3] = v.w;
    } else if constexpr (BITS == 8) {
        u4v a = *reinterpret_cast<const u4v *>(tile + lane * 4);
        u4v b = *reinterpret_cast<const u4v *>(tile + 256 + lane * 4);
        C[0] = a.x; C[1] = a.y; C[2] = a.z; C[3] = a.w;
        C[4] = b.x; C[5] = b.y; C[6] = b.z; C[7] = b.w;
    } else if constexpr (BITS == 2) {
        u2v v = *reinterpret_cast<const u2v *>(tile + lane * 4 + 2 * u);
        C[0] = v.x; C[1] = v.y;
    } else {
#pragma unroll
        for (int i = 0; i < 3; ++i)
            C[i] = tile[lane_dword(3 * u + i, lane)];
    }
}

// ---------------------------------------------------------------------------
// Buffer addressing: a 128-bit descriptor (base, size in bytes) in scalar registers, a scalar byte
// offset and a 32-bit per-lane byte offset.  A load then costs no vector address arithmetic, and lanes
// past the size read zero.  Every array addressed this way is smaller than 4 GiB (the callers check).
// ---------------------------------------------------------------------------
typedef __amdgpu_buffer_rsrc_t fq_rsrc;

__device__ __forceinline__ fq_rsrc make_rsrc(const void *base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, bytes, 0x00020000);
}

__device__ __forceinline__ u4v buf_load_b128(fq_rsrc r, uint32_t lane_off, uint32_t uniform_off)
{
    return __builtin_bit_cast(u4v, __builtin_amdgcn_raw_buffer_load_b128(r, lane_off, uniform_off, 0));
}

__device__ __forceinline__ u2v buf_load_b64(fq_rsrc r, uint32_t lane_off, uint32_t uniform_off)
{
    return __builtin_bit_cast(u2v, __builtin_amdgcn_raw_buffer_load_b64(r, lane_off, uniform_off, 0));
}

__device__ __forceinline__ uint32_t buf_load_b32(fq_rsrc r, uint32_t lane_off, uint32_t uniform_off)
{
    return __builtin_amdgcn_raw_buffer_load_b32(r, lane_off, uniform_off, 0);
}

// 16 bits, zero-extended
__device__ __forceinline__ uint32_t buf_load_u16(fq_rsrc r, uint32_t lane_off, uint32_t uniform_off)
{
    return __builtin_amdgcn_raw_buffer_load_b16(r, lane_off, uniform_off, 0);
}

// The BITS dwords of sub-block `u` owned by `lane`, from the supertile at byte offset tile_off.
template <int BITS>
__device__ __forceinline__ void buf_load_chunk(fq_rsrc packed, uint32_t tile_off, int u, int lane, uint32_t (&C)[BITS])
{
    const uint32_t lo = (uint32_t)lane * 16u;
    if constexpr (BITS == 4) {
        const u4v v = buf_load_b128(packed, lo, tile_off);
        C[0] = v.x; C[1] = v.y; C[2] = v.z; C[3] = v.w;
    } else if constexpr (BITS == 8) {
        const u4v a = buf_load_b128(packed, lo, tile_off);
        const u4v b = buf_load_b128(packed, lo + 1024u, tile_off);
        C[0] = a.x; C[1] = a.y; C[2] = a.z; C[3] = a.w;
        C[4] = b.x; C[5] = b.y; C[6] = b.z; C[7] = b.w;
    } else if constexpr (BITS == 2) {
        const u2v v = buf_load_b64(packed, lo + 8u * (uint32_t)u, tile_off);
        C[0] = v.x; C[1] = v.y;
    } else {
#pragma unroll
        for (int i = 0; i < 3; ++i)
            C[i] = buf_load_b32(packed, 4u * (uint32_t)lane_dword(3 * u + i, lane), tile_off);
    }
}

// Plain integer code of element t = 8*s + e of a chunk: the format read literally.
template <int BITS>
__device__ __forceinline__ uint32_t code_at(const uint32_t (&C)[BITS], int t)
{
    const int s = t >> 3, e = t & 7;
    const int half = 16 * (e & 1);
    if constexpr (BITS == 4) {
        return (C[s] >> (half + 4 * (e >> 1))) & 0xfu;
    } else if constexpr (BITS == 8) {
        return (C[2 * s + (e >> 2)] >> (half + 8 * ((e & 3) >> 1))) & 0xffu;
    } else if constexpr (BITS == 2) {
        return (C[s >> 1] >> (half + 2 * (4 * (s & 1) + (e >> 1)))) & 0x3u;
    } else {
        if (t < 30)
            return (C[t / 10] >> (half + 3 * ((t % 10) >> 1))) & 0x7u;
        const int b = (t == 30) ? 15 : 31;
        return ((C[0] >> b) & 1u) | (((C[1] >> b) & 1u) << 1) | (((C[2] >> b) & 1u) << 2);
    }
}

// ---------------------------------------------------------------------------
// Fast unpack.  A code field that sits inside the low 10 bits of a 16-bit half
// becomes an fp16 number by OR-ing in the exponent of 1024: the half then reads
// 1024 + code * 2^p, p the field's bit position.  One fused multiply-add by
// (2^-p, -1024 * 2^-p) turns a pair of them into the exact codes.  Fields are
// laid out so that the two weights of a pair share p and sit 16 bits apart.
// q[4*s + v] holds elements e = 2v (low half) and 2v+1 (high half) of k-step s.
// ---------------------------------------------------------------------------
#define FQ_EXP1024 0x64006400u

// The exponent pattern held in a vector register: the three-operand and-or instruction takes no
// literal and only one scalar operand, so with the mask in a scalar register and the exponent in a
// vector register (w & mask) | exp is a single instruction.
__device__ __forceinline__ uint32_t exp1024_reg()
{
    uint32_t e = FQ_EXP1024;
    asm volatile("" : "+v"(e));
    return e;
}

template <int P>
__device__ __forceinline__ h2 debias(uint32_t biased)
{
    constexpr float mul = 1.0f / (float)(1 << P);
    const h2 m = {(_Float16)mul, (_Float16)mul};
    const h2 a = {(_Float16)(-1024.0f * mul), (_Float16)(-1024.0f * mul)};
    return __builtin_elementwise_fma(as_h2(biased), m, a);
}

template <int BITS>
__device__ __forceinline__ void unpack_codes(const uint32_t (&C)[BITS], h2 (&q)[16])
{
    const uint32_t EXP = exp1024_reg();
    if constexpr (BITS == 4) {
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const uint32_t w = C[s], t = w >> 8;
            q[4 * s + 0] = debias<0>((w & 0x000f000fu) | EXP);
            q[4 * s + 1] = debias<4>((w & 0x00f000f0u) | EXP);
            q[4 * s + 2] = debias<0>((t & 0x000f000fu) | EXP);
            q[4 * s + 3] = debias<4>((t & 0x00f000f0u) | EXP);
        }
    } else if constexpr (BITS == 2) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const uint32_t w = C[j], t = w >> 10;
            q[8 * j + 0] = debias<0>((w & 0x00030003u) | EXP);
            q[8 * j + 1] = debias<2>((w & 0x000c000cu) | EXP);
            q[8 * j + 2] = debias<4>((w & 0x00300030u) | EXP);
            q[8 * j + 3] = debias<6>((w & 0x00c000c0u) | EXP);
            q[8 * j + 4] = debias<8>((w & 0x03000300u) | EXP);
            q[8 * j + 5] = debias<0>((t & 0x00030003u) | EXP);
            q[8 * j + 6] = debias<2>((t & 0x000c000cu) | EXP);
            q[8 * j + 7] = debias<4>((t & 0x00300030u) | EXP);
        }
    } else if constexpr (BITS == 8) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t w = C[j];
            // bytes 0 and 2 form one pair, bytes 1 and 3 the next
            q[2 * j + 0] = debias<0>((w & 0x00ff00ffu) | EXP);
            q[2 * j + 1] = debias<0>(((w >> 8) & 0x00ff00ffu) | EXP);
        }
    } else {
#pragma unroll
        for (int d = 0; d < 3; ++d) {
            const uint32_t w = C[d], t = w >> 9;
            q[5 * d + 0] = debias<0>((w & 0x00070007u) | EXP);
            q[5 * d + 1] = debias<3>((w & 0x00380038u) | EXP);
            q[5 * d + 2] = debias<6>((w & 0x01c001c0u) | EXP);
            q[5 * d + 3] = debias<0>((t & 0x00070007u) | EXP);
            q[5 * d + 4] = debias<3>((t & 0x00380038u) | EXP);
        }
        uint32_t sp = ((C[0] >> 15) & 0x00010001u) | EXP;
        sp |= (C[1] >> 14) & 0x00020002u;
        sp |= (C[2] >> 13) & 0x00040004u;
        q[15] = debias<0>(sp);
    }
}

// ---------------------------------------------------------------------------
// Unpack for the matrix-core GEMM: (code - zero) * scale per weight, in packed fp16.
// A code field at bit p of a half's mantissa, OR-ed with the exponent of 2^(10-p), reads 2^(10-p) + code:
// the code itself, not code * 2^p.  Taking the bias away is then an exact addition, and when the zero is
// an integer (what the quantizer produces) bias and zero leave together in one addition:
//     q = (biased + (-(2^(10-p)) - zero)) * scale          3 operations per pair with the and-or
// The sum is exact because bias + zero is an integer below 2048.  With fractional zeros (zeros rescaled
// after truncating code bits) the two additions are taken separately.
// ---------------------------------------------------------------------------
template <int P>
__device__ __forceinline__ uint32_t exp_for_shift()
{
    uint32_t e = (uint32_t)((25 - P) << 10) * 0x10001u; // exponent field of 2^(10-P), both halves
    asm volatile("" : "+v"(e));                          // vector register: see exp1024_reg()
    return e;
}

template <int P>
__device__ __forceinline__ h2 minus_bias()
{
    constexpr float b = -(float)(1 << (10 - P));
    return h2{(_Float16)b, (_Float16)b};
}

// pairs of one k-step: which shift each uses (index into the per-shift constants) and how to extract it
template <int BITS>
struct UnpackPlan;
template <>
struct UnpackPlan<4> { static constexpr int NSHIFT = 2; };
template <>
struct UnpackPlan<2> { static constexpr int NSHIFT = 5; };
template <>
struct UnpackPlan<3> { static constexpr int NSHIFT = 3; };
template <>
struct UnpackPlan<8> { static constexpr int NSHIFT = 1; };

// INTZ: the caller has made sure that the zero is an integer.
template <int BITS, bool INTZ>
__device__ __forceinline__ void unpack_dequant(const uint32_t (&C)[BITS], h2 zero2, h2 scale2, h2 (&q)[16])
{
    constexpr int NS = UnpackPlan<BITS>::NSHIFT;
    uint32_t b[16]; // biased pairs
    int sh[16];     // index of the shift of each pair (compile-time after unrolling)
    h2 mb[NS];      // -2^(10-p) per shift
    if constexpr (BITS == 4) {
        const uint32_t E0 = exp_for_shift<0>(), E4 = exp_for_shift<4>();
        mb[0] = minus_bias<0>(); mb[1] = minus_bias<4>();
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const uint32_t w = C[s], t = w >> 8;
            b[4 * s + 0] = (w & 0x000f000fu) | E0; sh[4 * s + 0] = 0;
            b[4 * s + 1] = (w & 0x00f000f0u) | E4; sh[4 * s + 1] = 1;
            b[4 * s + 2] = (t & 0x000f000fu) | E0; sh[4 * s + 2] = 0;
            b[4 * s + 3] = (t & 0x00f000f0u) | E4; sh[4 * s + 3] = 1;
        }
    } else if constexpr (BITS == 2) {
        const uint32_t E0 = exp_for_shift<0>(), E2 = exp_for_shift<2>(), E4 = exp_for_shift<4>(),
                       E6 = exp_for_shift<6>(), E8 = exp_for_shift<8>();
        mb[0] = minus_bias<0>(); mb[1] = minus_bias<2>(); mb[2] = minus_bias<4>(); mb[3] = minus_bias<6>();
        mb[4] = minus_bias<8>();
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const uint32_t w = C[j], t = w >> 10;
            b[8 * j + 0] = (w & 0x00030003u) | E0; sh[8 * j + 0] = 0;
            b[8 * j + 1] = (w & 0x000c000cu) | E2; sh[8 * j + 1] = 1;
            b[8 * j + 2] = (w & 0x00300030u) | E4; sh[8 * j + 2] = 2;
            b[8 * j + 3] = (w & 0x00c000c0u) | E6; sh[8 * j + 3] = 3;
            b[8 * j + 4] = (w & 0x03000300u) | E8; sh[8 * j + 4] = 4;
            b[8 * j + 5] = (t & 0x00030003u) | E0; sh[8 * j + 5] = 0;
            b[8 * j + 6] = (t & 0x000c000cu) | E2; sh[8 * j + 6] = 1;
            b[8 * j + 7] = (t & 0x00300030u) | E4; sh[8 * j + 7] = 2;
        }
    } else if constexpr (BITS == 8) {
        const uint32_t E0 = exp_for_shift<0>();
        mb[0] = minus_bias<0>();
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t w = C[j];
            b[2 * j + 0] = (w & 0x00ff00ffu) | E0; sh[2 * j + 0] = 0;
            b[2 * j + 1] = ((w >> 8) & 0x00ff00ffu) | E0; sh[2 * j + 1] = 0;
        }
    } else {
        const uint32_t E0 = exp_for_shift<0>(), E3 = exp_for_shift<3>(), E6 = exp_for_shift<6>();
        mb[0] = minus_bias<0>(); mb[1] = minus_bias<3>(); mb[2] = minus_bias<6>();
#pragma unroll
        for (int d = 0; d < 3; ++d) {
            const uint32_t w = C[d], t = w >> 9;
            b[5 * d + 0] = (w & 0x00070007u) | E0; sh[5 * d + 0] = 0;
            b[5 * d + 1] = (w & 0x00380038u) | E3; sh[5 * d + 1] = 1;
            b[5 * d + 2] = (w & 0x01c001c0u) | E6; sh[5 * d + 2] = 2;
            b[5 * d + 3] = (t & 0x00070007u) | E0; sh[5 * d + 3] = 0;
            b[5 * d + 4] = (t & 0x00380038u) | E3; sh[5 * d + 4] = 1;
        }
        uint32_t sp = ((C[0] >> 15) & 0x00010001u) | E0;
        sp |= (C[1] >> 14) & 0x00020002u;
        sp |= (C[2] >> 13) & 0x00040004u;
        b[15] = sp; sh[15] = 0;
    }
    if constexpr (INTZ) {
        h2 mbz[NS];
#pragma unroll
        for (int i = 0; i < NS; ++i)
            mbz[i] = mb[i] - zero2; // exact: an integer below 2048
#pragma unroll
        for (int p = 0; p < 16; ++p)
            q[p] = (as_h2(b[p]) + mbz[sh[p]]) * scale2;
    } else {
#pragma unroll
        for (int p = 0; p < 16; ++p)
            q[p] = ((as_h2(b[p]) + mb[sh[p]]) - zero2) * scale2;
    }
}

// Biased pairs without the fix-up: h[4*s + v] reads, as two fp16 numbers,
// 1024 + code * 2^pair_shift(4*s + v) for elements 2v and 2v+1 of k-step s.  The
// streaming kernel feeds these to the matrix core as they are and removes the
// bias once per group instead of once per weight.
template <int BITS>
__host__ __device__ constexpr int pair_shift(int p)
{
    if (BITS == 4)
        return (p & 1) ? 4 : 0;
    if (BITS == 2) {
        constexpr int sh[8] = {0, 2, 4, 6, 8, 0, 2, 4};
        return sh[p & 7];
    }
    if (BITS == 3) {
        constexpr int sh[5] = {0, 3, 6, 0, 3};
        return p == 15 ? 0 : sh[p % 5];
    }
    return 0;
}

template <int BITS>
__device__ __forceinline__ void extract_biased(const uint32_t (&C)[BITS], uint32_t (&h)[16])
{
    const uint32_t EXP = exp1024_reg();
    if constexpr (BITS == 4) {
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const uint32_t w = C[s], t = w >> 8;
            h[4 * s + 0] = (w & 0x000f000fu) | EXP;
            h[4 * s + 1] = (w & 0x00f000f0u) | EXP;
            h[4 * s + 2] = (t & 0x000f000fu) | EXP;
            h[4 * s + 3] = (t & 0x00f000f0u) | EXP;
        }
    } else if constexpr (BITS == 2) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const uint32_t w = C[j], t = w >> 10;
            h[8 * j + 0] = (w & 0x00030003u) | EXP;
            h[8 * j + 1] = (w & 0x000c000cu) | EXP;
            h[8 * j + 2] = (w & 0x00300030u) | EXP;
            h[8 * j + 3] = (w & 0x00c000c0u) | EXP;
            h[8 * j + 4] = (w & 0x03000300u) | EXP;
            h[8 * j + 5] = (t & 0x00030003u) | EXP;
            h[8 * j + 6] = (t & 0x000c000cu) | EXP;
            h[8 * j + 7] = (t & 0x00300030u) | EXP;
        }
    } else if constexpr (BITS == 8) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t w = C[j];
            h[2 * j + 0] = (w & 0x00ff00ffu) | EXP;
            h[2 * j + 1] = ((w >> 8) & 0x00ff00ffu) | EXP;
        }
    } else {
#pragma unroll
        for (int d = 0; d < 3; ++d) {
            const uint32_t w = C[d], t = w >> 9;
            h[5 * d + 0] = (w & 0x00070007u) | EXP;
            h[5 * d + 1] = (w & 0x00380038u) | EXP;
            h[5 * d + 2] = (w & 0x01c001c0u) | EXP;
            h[5 * d + 3] = (t & 0x00070007u) | EXP;
            h[5 * d + 4] = (t & 0x00380038u) | EXP;
        }
        uint32_t sp = ((C[0] >> 15) & 0x00010001u) | EXP;
        sp |= (C[1] >> 14) & 0x00020002u;
        sp |= (C[2] >> 13) & 0x00040004u;
        h[15] = sp;
    }
}

// Operand for k-step s of a 16x16x32 matrix-core instruction from four pairs.
__device__ __forceinline__ h8 make_h8(h2 a, h2 b, h2 c, h2 d)
{
    h8 r;
    r[0] = a[0]; r[1] = a[1]; r[2] = b[0]; r[3] = b[1];
    r[4] = c[0]; r[5] = c[1]; r[6] = d[0]; r[7] = d[1];
    return r;
}

__device__ __forceinline__ h8 make_h8_bits(uint32_t a, uint32_t b, uint32_t c, uint32_t d)
{
    const u4v v = {a, b, c, d};
    return __builtin_bit_cast(h8, v);
}

__device__ __forceinline__ f4 mfma16x16x32(h8 a, h8 b, f4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}

#endif
