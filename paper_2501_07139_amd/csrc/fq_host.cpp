// Host half of libfq: error reporting, RTN quantizer, packer.
//
// The hybrid model of FlexQuant (arXiv 2501.07139, Section "EQM Generation
// Philosophy") draws each matrix from one of several stored quantized models;
// these routines produce those stored forms from fp32 weights.  They are one-off
// preparation, not part of the timed path.
#include "fq.h"
#include "fq_internal.h"

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <thread>
#include <vector>

namespace {
thread_local char g_err[256] = "";
}

int fq_fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

extern "C" const char *fq_last_error(void) { return g_err; }
extern "C" const char *fq_version(void) { return "libfq 0.1 (gfx950)"; }

int fq_bits_index(int bits)
{
    switch (bits) {
    case 2: return 0;
    case 3: return 1;
    case 4: return 2;
    case 8: return 3;
    }
    return -1;
}

int fq_rows_per_supertile(int bits)
{
    static const int R[4] = {32, 64, 16, 16};
    int i = fq_bits_index(bits);
    return i < 0 ? 0 : R[i];
}

namespace {

inline float half_bits_to_float(uint16_t h)
{
    _Float16 v;
    std::memcpy(&v, &h, 2);
    return (float)v;
}

inline uint16_t float_to_half_bits(float f)
{
    _Float16 v = (_Float16)f; // round-to-nearest-even
    uint16_t h;
    std::memcpy(&h, &v, 2);
    return h;
}

template <class F>
void parallel_rows(int count, F &&body)
{
    unsigned hw = std::thread::hardware_concurrency();
    int nt = (int)std::min<unsigned>(hw ? hw : 1u, 16u);
    nt = std::max(1, std::min(nt, count));
    if (nt == 1) {
        body(0, count);
        return;
    }
    std::vector<std::thread> pool;
    int per = (count + nt - 1) / nt;
    for (int t = 0; t < nt; ++t) {
        int lo = t * per, hi = std::min(count, lo + per);
        if (lo >= hi)
            break;
        pool.emplace_back([=, &body] { body(lo, hi); });
    }
    for (auto &th : pool)
        th.join();
}

} // namespace

extern "C" int fq_quantize_rtn(const float *W, int N, int K, int bits, int group,
                               uint8_t *codes, uint16_t *scales, uint16_t *zeros)
{
    if (!W || !codes || !scales || !zeros)
        return fq_fail(FQ_ERR_NULL, "fq_quantize_rtn: NULL argument");
    if (fq_bits_index(bits) < 0)
        return fq_fail(FQ_ERR_BITS, "fq_quantize_rtn: bits=%d not in {2,3,4,8}", bits);
    if (group != 128)
        return fq_fail(FQ_ERR_GROUP, "fq_quantize_rtn: group=%d, only 128 is supported", group);
    if (N <= 0 || K <= 0 || K % 128 != 0)
        return fq_fail(FQ_ERR_SHAPE, "fq_quantize_rtn: N=%d K=%d (K must be a positive multiple of 128)", N, K);
    const int G = K / 128;
    const float qmax = (float)((1 << bits) - 1);
    parallel_rows(N, [&](int n0, int n1) {
        for (int n = n0; n < n1; ++n) {
            for (int g = 0; g < G; ++g) {
                const float *w = W + (size_t)n * K + (size_t)g * 128;
                uint8_t *q = codes + (size_t)n * K + (size_t)g * 128;
                float mn = 0.0f, mx = 0.0f;
                for (int i = 0; i < 128; ++i) {
                    mn = std::min(mn, w[i]);
                    mx = std::max(mx, w[i]);
                }
                size_t mi = (size_t)n * G + g;
                if (mx == mn) {
                    scales[mi] = 0x3c00; // 1.0
                    zeros[mi] = 0;
                    std::memset(q, 0, 128);
                    continue;
                }
                uint16_t sh = float_to_half_bits((mx - mn) / qmax);
                if ((sh & 0x7c00) == 0)
                    sh = 0x0400; // below the normal range: use 2^-14
                const float s = half_bits_to_float(sh);
                float zr = std::nearbyintf((0.0f - mn) / s); // 0 - 0 is +0: the stored zero is never -0
                zr = std::min(std::max(zr, 0.0f), qmax);
                for (int i = 0; i < 128; ++i) {
                    // stays in floating point until it is inside [0, qmax]: the sum of two integers is exact
                    // wherever it can land in that range, and no out-of-range value is converted
                    const float c = std::nearbyintf(w[i] / s) + zr;
                    q[i] = (uint8_t)std::min(std::max(c, 0.0f), qmax);
                }
                scales[mi] = sh;
                zeros[mi] = float_to_half_bits(zr);
            }
        }
    });
    return FQ_OK;
}

extern "C" size_t fq_packed_bytes(int N, int K, int bits)
{
    if (N <= 0 || K <= 0 || K % 128 != 0 || fq_bits_index(bits) < 0)
        return 0;
    size_t Np = ((size_t)N + 63) / 64 * 64;
    return Np * (size_t)K * (size_t)bits / 8;
}

extern "C" size_t fq_meta_count(int N, int K, int group)
{
    if (N <= 0 || K <= 0 || group != 128 || K % 128 != 0)
        return 0;
    size_t Np = ((size_t)N + 63) / 64 * 64;
    return Np * (size_t)(K / 128);
}

namespace {

// Where code (rho = row in supertile, kap = k in group) lives: dword index inside
// the supertile and the bit offset of each of its `bits` bits.
struct Slot {
    int word[3];
    int shift[3];
    int pieces; // 1: contiguous field; 3: one bit in each of three dwords
};

inline int lane_word(int bits, int u, int i, int lane)
{
    int j = bits * u + i;
    return (j >> 2) * 256 + lane * 4 + (j & 3);
}

inline Slot locate(int bits, int rho, int kap)
{
    const int u = rho >> 4, r = rho & 15;
    const int s = kap >> 5, c = (kap >> 3) & 3, e = kap & 7;
    const int lane = 16 * c + r;
    const int half = 16 * (e & 1);
    Slot sl;
    sl.pieces = 1;
    switch (bits) {
    case 4:
        sl.word[0] = lane_word(4, u, s, lane);
        sl.shift[0] = half + 4 * (e >> 1);
        break;
    case 8:
        sl.word[0] = lane_word(8, u, 2 * s + (e >> 2), lane);
        sl.shift[0] = half + 8 * ((e & 3) >> 1);
        break;
    case 2:
        sl.word[0] = lane_word(2, u, s >> 1, lane);
        sl.shift[0] = half + 2 * (4 * (s & 1) + (e >> 1));
        break;
    default: { // 3
        const int t = 8 * s + e;
        if (t < 30) {
            sl.word[0] = lane_word(3, u, t / 10, lane);
            sl.shift[0] = half + 3 * ((t % 10) >> 1);
        } else {
            sl.pieces = 3;
            for (int i = 0; i < 3; ++i) {
                sl.word[i] = lane_word(3, u, i, lane);
                sl.shift[i] = (t == 30) ? 15 : 31;
            }
        }
    }
    }
    return sl;
}

} // namespace

extern "C" int fq_pack_groups(const uint8_t *codes, const uint16_t *scales, const uint16_t *zeros,
                              int N, int K, int bits, int group,
                              void *packed_out, uint16_t *scales_out, uint16_t *zeros_out)
{
    if (!codes || !scales || !zeros || !packed_out || !scales_out || !zeros_out)
        return fq_fail(FQ_ERR_NULL, "fq_pack_groups: NULL argument");
    if (fq_bits_index(bits) < 0)
        return fq_fail(FQ_ERR_BITS, "fq_pack_groups: bits=%d not in {2,3,4,8}", bits);
    if (group != 128)
        return fq_fail(FQ_ERR_GROUP, "fq_pack_groups: group=%d, only 128 is supported", group);
    if (N <= 0 || K <= 0 || K % 128 != 0)
        return fq_fail(FQ_ERR_SHAPE, "fq_pack_groups: N=%d K=%d (K must be a positive multiple of 128)", N, K);
    const int G = K / 128;
    const int R = fq_rows_per_supertile(bits);
    const int Np = (N + 63) / 64 * 64;
    const size_t tile_words = (size_t)R * 4 * bits;
    uint32_t *out = static_cast<uint32_t *>(packed_out);
    std::memset(out, 0, fq_packed_bytes(N, K, bits));
    const unsigned limit = 1u << bits;
    std::atomic<int> bad{0};
    parallel_rows(Np / R, [&](int b0, int b1) {
        for (int rb = b0; rb < b1; ++rb) {
            for (int rho = 0; rho < R; ++rho) {
                const int n = rb * R + rho;
                if (n >= N)
                    break;
                const uint8_t *row = codes + (size_t)n * K;
                for (int k = 0; k < K; ++k) {
                    const unsigned q = row[k];
                    if (q >= limit) {
                        bad = 1;
                        continue;
                    }
                    uint32_t *tile = out + ((size_t)rb * G + (k >> 7)) * tile_words;
                    const Slot sl = locate(bits, rho, k & 127);
                    if (sl.pieces == 1) {
                        tile[sl.word[0]] |= q << sl.shift[0];
                    } else {
                        for (int i = 0; i < 3; ++i)
                            tile[sl.word[i]] |= ((q >> i) & 1u) << sl.shift[i];
                    }
                }
            }
        }
    });
    if (bad)
        return fq_fail(FQ_ERR_BITS, "fq_pack_groups: a code does not fit in %d bits", bits);
    for (int n = 0; n < Np; ++n)
        for (int g = 0; g < G; ++g) {
            size_t dst = ((size_t)(n >> 4) * G + g) * 16 + (n & 15);
            scales_out[dst] = n < N ? scales[(size_t)n * G + g] : 0;
            zeros_out[dst] = n < N ? zeros[(size_t)n * G + g] : 0;
        }
    return FQ_OK;
}

// Rotary-embedding table of the real decoder blocks: angles pos * base^(-2i/head_dim) in fp64, their cosine
// and sine rounded once to fp32.
extern "C" int fq_rope_table(int Tmax, int head_dim, double base, float *out)
{
    if (!out)
        return fq_fail(FQ_ERR_NULL, "fq_rope_table: NULL output");
    if (Tmax <= 0 || head_dim <= 0 || head_dim % 2 != 0 || !(base > 0.0))
        return fq_fail(FQ_ERR_SHAPE, "fq_rope_table: Tmax=%d head_dim=%d base=%g", Tmax, head_dim, base);
    const int half = head_dim / 2;
    parallel_rows(Tmax, [&](int lo, int hi) {
        for (int t = lo; t < hi; ++t)
            for (int i = 0; i < half; ++i) {
                const double ang = (double)t * std::pow(base, -2.0 * (double)i / (double)head_dim);
                out[((size_t)t * half + i) * 2 + 0] = (float)std::cos(ang);
                out[((size_t)t * half + i) * 2 + 1] = (float)std::sin(ang);
            }
    });
    return FQ_OK;
}
