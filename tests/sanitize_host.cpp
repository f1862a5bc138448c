// Host-only driver for AddressSanitizer / UndefinedBehaviorSanitizer: every buffer is a heap block of exactly
// the documented size, so an access one byte off either end of an input or an output of the library's host
// functions (quantizer, packer, size queries, rotary table) or of the oracle's C functions is reported.
// Built and run by tests/test_sanitizers.py with g++ -fsanitize=address,undefined; no GPU code is involved.
// It also cross-checks the two sides where that is free: library quantizer == oracle quantizer, and the
// oracle's unpack of the library's packing returns the codes.
#include "fq.h"

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

extern "C" {
uint16_t ora_f2h(float v);
int ora_quantize_rtn(const float *W, int N, int K, int bits, int group, uint8_t *codes, uint16_t *scales, uint16_t *zeros);
size_t ora_packed_bytes(int N, int K, int bits);
int ora_unpack(const uint8_t *packed, int N, int K, int bits, uint8_t *codes);
int ora_untile_meta(const uint16_t *tiled, int N, int G, uint16_t *rowmajor);
int ora_dequant(const uint8_t *codes, const uint16_t *scales, const uint16_t *zeros, int N, int K, int group, float *W32);
int ora_truncate(const uint8_t *codes, const uint16_t *scales, const uint16_t *zeros, int N, int K, int group, int d,
                 int midpoint, uint8_t *codes_out, uint16_t *scales_out, uint16_t *zeros_out);
int ora_qlinear(const uint16_t *X, int M, const float *W32, int N, int K, double *Y);
int ora_dense_f16(const uint16_t *X, int M, const uint16_t *W, int N, int K, double *Y);
void ora_round_f16(const double *in, size_t count, uint16_t *out);
void ora_rms_rows(const double *t, int M, int H, double eps, uint16_t *out);
void ora_silu_mul(const uint16_t *g, const uint16_t *p, size_t count, double *out);
int ora_token_nll(const uint16_t *logits, const int32_t *labels, int M, int V, double *nll);
int ora_logit_l2(const uint16_t *a, const uint16_t *b, int M, int V, double *dist);
}

// exact-size heap block (std::vector may over-allocate; malloc'd blocks have red zones right at the end)
template <class T>
struct Block {
    T *p;
    size_t n;
    explicit Block(size_t count) : p(static_cast<T *>(std::malloc(count ? count * sizeof(T) : 1))), n(count) {}
    ~Block() { std::free(p); }
    Block(const Block &) = delete;
    Block &operator=(const Block &) = delete;
    T &operator[](size_t i) { return p[i]; }
};

static uint32_t g_state = 12345u;
static float rnd() // uniform in [-1, 1)
{
    g_state = g_state * 1664525u + 1013904223u;
    return (float)(int32_t)g_state / 2147483648.0f;
}

#define CHECK(cond)                                                                      \
    do {                                                                                 \
        if (!(cond)) {                                                                   \
            std::fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
            return 1;                                                                    \
        }                                                                                \
    } while (0)

static int one_matrix(int N, int K, int bits)
{
    const int G = K / 128;
    Block<float> W((size_t)N * K);
    for (size_t i = 0; i < W.n; ++i)
        W[i] = 0.02f * rnd() * ((i % 977 == 0) ? 40.0f : 1.0f); // a few outliers
    for (int k = 0; k < 128 && N > 1; ++k)                      // one constant group: the hi == lo branch
        W[(size_t)K + k] = 0.0f;
    Block<uint8_t> codes(W.n), codes_o(W.n);
    Block<uint16_t> s((size_t)N * G), z((size_t)N * G), so((size_t)N * G), zo((size_t)N * G);
    CHECK(fq_quantize_rtn(W.p, N, K, bits, 128, codes.p, s.p, z.p) == FQ_OK);
    CHECK(ora_quantize_rtn(W.p, N, K, bits, 128, codes_o.p, so.p, zo.p) == 0);
    CHECK(std::memcmp(codes.p, codes_o.p, W.n) == 0);
    CHECK(std::memcmp(s.p, so.p, s.n * 2) == 0 && std::memcmp(z.p, zo.p, z.n * 2) == 0);

    const size_t pb = fq_packed_bytes(N, K, bits), mc = fq_meta_count(N, K, 128);
    CHECK(pb == ora_packed_bytes(N, K, bits) && pb > 0 && mc >= (size_t)N * G);
    Block<uint8_t> packed(pb);
    Block<uint16_t> st(mc), zt(mc);
    CHECK(fq_pack_groups(codes.p, s.p, z.p, N, K, bits, 128, packed.p, st.p, zt.p) == FQ_OK);
    Block<uint8_t> back(W.n);
    CHECK(ora_unpack(packed.p, N, K, bits, back.p) == 0);
    CHECK(std::memcmp(back.p, codes.p, W.n) == 0);
    Block<uint16_t> s_rm((size_t)N * G);
    CHECK(ora_untile_meta(st.p, N, G, s_rm.p) == 0);
    CHECK(std::memcmp(s_rm.p, s.p, s.n * 2) == 0);

    Block<float> W32(W.n);
    CHECK(ora_dequant(codes.p, s.p, z.p, N, K, 128, W32.p) == 0);
    if (bits > 2) {
        Block<uint8_t> ct(W.n);
        Block<uint16_t> s2(s.n), z2(z.n);
        CHECK(ora_truncate(codes.p, s.p, z.p, N, K, 128, bits - 2, 1, ct.p, s2.p, z2.p) == 0);
    }
    const int M = 3;
    Block<uint16_t> X((size_t)M * K);
    for (size_t i = 0; i < X.n; ++i)
        X[i] = ora_f2h(rnd());
    Block<double> Y((size_t)M * N);
    CHECK(ora_qlinear(X.p, M, W32.p, N, K, Y.p) == 0);
    Block<uint16_t> Yh(Y.n);
    ora_round_f16(Y.p, Y.n, Yh.p);
    // the rounded outputs as a second fp16 matrix [M, N] against itself: the dense product and the row ops
    Block<double> D((size_t)M * M);
    CHECK(ora_dense_f16(Yh.p, M, Yh.p, M, N, D.p) == 0);
    Block<uint16_t> R(Y.n);
    ora_rms_rows(Y.p, M, N, 1e-5, R.p);
    Block<double> SM(Y.n);
    ora_silu_mul(Yh.p, R.p, Y.n, SM.p);
    Block<int32_t> labels(M);
    labels[0] = 0, labels[1] = N - 1, labels[2] = -1;
    Block<double> nll(M), dist(M);
    CHECK(ora_token_nll(Yh.p, labels.p, M, N, nll.p) == 0);
    CHECK(nll.p[2] == 0.0 && std::isfinite(nll.p[0]) && std::isfinite(nll.p[1]));
    CHECK(ora_logit_l2(Yh.p, R.p, M, N, dist.p) == 0);
    return 0;
}

int main()
{
    const int shapes[][2] = {{1, 128}, {70, 256}, {200, 384}, {64, 1280}, {129, 128}};
    const int widths[] = {2, 3, 4, 8};
    for (auto &sh : shapes)
        for (int bits : widths)
            if (one_matrix(sh[0], sh[1], bits)) {
                std::fprintf(stderr, "failed at N=%d K=%d bits=%d: %s\n", sh[0], sh[1], bits, fq_last_error());
                return 1;
            }
    // argument checking returns errors, touches nothing
    uint8_t dummy[16];
    uint16_t d16[8];
    float w[128] = {0};
    if (fq_quantize_rtn(w, 1, 128, 5, 128, dummy, d16, d16) != FQ_ERR_BITS || fq_quantize_rtn(w, 1, 100, 4, 128, dummy, d16, d16) != FQ_ERR_SHAPE ||
        fq_quantize_rtn(nullptr, 1, 128, 4, 128, dummy, d16, d16) != FQ_ERR_NULL || fq_packed_bytes(1, 100, 4) != 0)
        return 2;
    // rotary table: [Tmax][head_dim] floats (cos then sin halves), exactly that many
    const int T = 37, HD = 128;
    Block<float> rope((size_t)T * HD);
    if (fq_rope_table(T, HD, 10000.0, rope.p) != FQ_OK || rope.p[0] != 1.0f)
        return 3;
    std::puts("sanitize_host: ok");
    return 0;
}
