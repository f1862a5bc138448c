/*
 * CPU oracle for the mixed-bit weight-only quantized linear layer and the
 * token-level loss that scores a hybrid (mixed bit-width) model.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is deliberately slow and plain: one loop
 * nest per definition, fp64 accumulation, no blocking, no vector tricks.  It
 * shares no code, header, table or constant with the GPU library; only tests,
 * the smoke check and the benchmark's CPU-baseline leg may call it.
 *
 * What the paper fixes (FlexQuant, arXiv 2501.07139):
 *   - every module of a hybrid model takes its parameters from one of the
 *     stored quantized models, i.e. has its own bit-width
 *     (Section "EQM Generation Philosophy");
 *   - the arithmetic is done in a standard format (FP16) whatever the weight
 *     bit-width, and an n-bit layer approximates its FP16 counterpart
 *     (Section "Large Language Model Quantization", Section "FlexQuant Framework");
 *   - lower precisions can be obtained from a higher one by truncating code
 *     bits (Section "Elastic Serving");
 *   - a candidate is scored by its perplexity on calibration token sequences
 *     (Section "Efficient Design Space Navigation", Algorithm 1, calibrationEval).
 * The paper delegates the quantizer itself; the reading used here is group-wise
 * round-to-nearest asymmetric min-max quantization with fp16 scale and zero,
 * groups of 128 along the input dimension.
 *
 * Functions whose result has no pin other than agreement with the GPU path:
 *   ora_rms_rows / ora_silu_mul (glue of the synthetic stack) -- their closed
 *   forms are pinned, the stack dataflow that strings them together is a
 *   reading of "activations carried layer to layer" and is parity-unpinned
 *   by the paper.
 *
 * Build: gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC fq_oracle.c -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ fp16 */

/* IEEE binary16 -> double, exact. */
double ora_h2d(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int ex = (h >> 10) & 0x1f;
    int man = h & 0x3ff;
    double v;
    if (ex == 0)
        v = ldexp((double)man, -24); /* subnormal or zero */
    else if (ex == 31)
        v = man ? NAN : INFINITY;
    else
        v = ldexp(1.0 + (double)man / 1024.0, ex - 15);
    return sign ? -v : v;
}

float ora_h2f(uint16_t h) { return (float)ora_h2d(h); /* exact: 11 bits fit in 24 */ }

/* double -> IEEE binary16, one rounding, round-half-to-even. */
uint16_t ora_d2h(double v)
{
    uint16_t sign = signbit(v) ? 0x8000u : 0u;
    double a = fabs(v);
    if (isnan(v))
        return 0x7e00u;
    if (a >= 65520.0) /* halfway between 65504 and 2^16 rounds to infinity */
        return sign | 0x7c00u;
    if (a == 0.0)
        return sign;
    int ex;
    (void)frexp(a, &ex); /* a = m * 2^ex, m in [0.5,1)  ->  floor(log2 a) = ex-1 */
    int e = ex - 1;
    if (e < -14)
        e = -14; /* subnormal range shares the quantum of the lowest binade */
    double quantum = ldexp(1.0, e - 10);
    double n = nearbyint(a / quantum); /* power-of-two scaling is exact; RNE */
    double r = n * quantum;            /* value of the result, exactly a half */
    if (r == 0.0)
        return sign;
    if (r < ldexp(1.0, -14))
        return sign | (uint16_t)(r / ldexp(1.0, -24));
    (void)frexp(r, &ex);
    e = ex - 1;
    double frac = r / ldexp(1.0, e) - 1.0; /* in [0,1) */
    return sign | (uint16_t)((e + 15) << 10) | (uint16_t)(frac * 1024.0);
}

uint16_t ora_f2h(float v) { return ora_d2h((double)v); }

/* ------------------------------------------------------------- quantize */

/*
 * Group-wise RTN asymmetric min-max quantization of W[N,K] (fp32, row-major).
 * Per (row, group of `group` consecutive k):
 *   lo = min(0, min w), hi = max(0, max w)                      (fp32)
 *   hi == lo:  s = 1, z = 0, all codes 0
 *   else       s = fp16(  (hi - lo) / maxq  ), raised to the smallest normal
 *              fp16 if it is zero or subnormal;  sf = float(s)
 *              z = clamp(rne(-lo / sf), 0, maxq)                (an integer, stored as fp16)
 *              q = clamp(rne(w / sf) + z, 0, maxq)
 * with maxq = 2^bits - 1 and rne = round-half-to-even.  Reconstruction is
 * w^ = s * (q - z): the zero is in code units.  codes[N,K] u8, scales/zeros
 * [N, K/group] fp16 bit patterns, all row-major.
 */
int ora_quantize_rtn(const float *W, int N, int K, int bits, int group,
                     uint8_t *codes, uint16_t *scales, uint16_t *zeros)
{
    if (!W || !codes || !scales || !zeros)
        return -1;
    if (bits < 1 || bits > 8 || group <= 0 || K % group != 0)
        return -2;
    int G = K / group;
    int maxq = (1 << bits) - 1;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int g = 0; g < G; ++g) {
            const float *w = W + (size_t)n * K + (size_t)g * group;
            uint8_t *q = codes + (size_t)n * K + (size_t)g * group;
            float lo = 0.0f, hi = 0.0f;
            for (int i = 0; i < group; ++i) {
                if (w[i] < lo) lo = w[i];
                if (w[i] > hi) hi = w[i];
            }
            if (hi == lo) {
                scales[(size_t)n * G + g] = ora_f2h(1.0f);
                zeros[(size_t)n * G + g] = 0;
                memset(q, 0, (size_t)group);
                continue;
            }
            float s32 = (hi - lo) / (float)maxq;
            uint16_t sh = ora_f2h(s32);
            if ((sh & 0x7c00u) == 0)
                sh = 0x0400u; /* smallest normal fp16, 2^-14 */
            float sf = ora_h2f(sh);
            float zf = nearbyintf(-lo / sf);
            int z = zf < 0.0f ? 0 : (zf > (float)maxq ? maxq : (int)zf);
            for (int i = 0; i < group; ++i) {
                float r = nearbyintf(w[i] / sf);
                /* r is an integer-valued float; clamp before converting */
                if (r < -1.0e6f) r = -1.0e6f;
                if (r > 1.0e6f) r = 1.0e6f;
                int c = (int)r + z;
                q[i] = (uint8_t)(c < 0 ? 0 : (c > maxq ? maxq : c));
            }
            scales[(size_t)n * G + g] = sh;
            zeros[(size_t)n * G + g] = ora_f2h((float)z);
        }
    }
    return 0;
}

/* ---------------------------------------------------------------- unpack */

/*
 * The packed device format, read back from its written description.
 *
 * Rows are padded to Np = 64*ceil(N/64).  A supertile covers R rows by one
 * group of 128 k, R = 32/64/16/16 for bits 2/3/4/8, and takes R*16*bits bytes
 * (a whole number of 1024-byte planes).  Supertile (n/R, k/128) starts at byte
 * ((n/R)*(K/128) + k/128) * R*16*bits.  Inside it, "lane" l = 16*c + r owns
 * dwords D[j]; D[j] is the little-endian u32 at byte (j/4)*1024 + 16*l + 4*(j%4).
 * With  n % R = 16*u + r  and  k % 128 = 32*s + 8*c + e  (t = 8*s + e), the
 * chunk of the weight is C[i] = D[bits*u + i], i < bits, and the code sits at
 *   bits 4:  C[s],          bit offset 16*(e%2) + 4*(e/2)
 *   bits 8:  C[2*s + e/4],  bit offset 16*(e%2) + 8*((e%4)/2)
 *   bits 2:  C[s/2],        bit offset 16*(e%2) + 2*(4*(s%2) + e/2)
 *   bits 3:  t < 30: C[t/10], bit offset 16*(t%2) + 3*((t%10)/2);
 *            t = 30: code bit i is bit 15 of C[i];  t = 31: bit 31 of C[i].
 */
static uint32_t rd32(const uint8_t *p)
{
    return (uint32_t)p[0] | ((uint32_t)p[1] << 8) | ((uint32_t)p[2] << 16) | ((uint32_t)p[3] << 24);
}

static int rows_per_supertile(int bits)
{
    switch (bits) {
    case 2: return 32;
    case 3: return 64;
    case 4: return 16;
    case 8: return 16;
    }
    return 0;
}

size_t ora_packed_bytes(int N, int K, int bits)
{
    size_t Np = ((size_t)N + 63) / 64 * 64;
    return Np * (size_t)K * (size_t)bits / 8;
}

int ora_unpack(const uint8_t *packed, int N, int K, int bits, uint8_t *codes)
{
    int R = rows_per_supertile(bits);
    if (!packed || !codes)
        return -1;
    if (R == 0 || K % 128 != 0)
        return -2;
    int G = K / 128;
    size_t tile_bytes = (size_t)R * 16 * bits;
    for (int n = 0; n < N; ++n) {
        for (int k = 0; k < K; ++k) {
            int rho = n % R, u = rho / 16, r = rho % 16;
            int kap = k % 128, s = kap / 32, c = (kap % 32) / 8, e = kap % 8;
            int t = 8 * s + e;
            int l = 16 * c + r;
            const uint8_t *tile = packed + ((size_t)(n / R) * G + (size_t)(k / 128)) * tile_bytes;
            uint32_t C[8];
            for (int i = 0; i < bits; ++i) {
                int j = bits * u + i;
                C[i] = rd32(tile + (size_t)(j / 4) * 1024 + 16 * (size_t)l + 4 * (size_t)(j % 4));
            }
            uint32_t q = 0;
            if (bits == 4) {
                q = (C[s] >> (16 * (e % 2) + 4 * (e / 2))) & 0xf;
            } else if (bits == 8) {
                q = (C[2 * s + e / 4] >> (16 * (e % 2) + 8 * ((e % 4) / 2))) & 0xff;
            } else if (bits == 2) {
                q = (C[s / 2] >> (16 * (e % 2) + 2 * (4 * (s % 2) + e / 2))) & 0x3;
            } else { /* 3 */
                if (t < 30) {
                    q = (C[t / 10] >> (16 * (t % 2) + 3 * ((t % 10) / 2))) & 0x7;
                } else {
                    int bitpos = (t == 30) ? 15 : 31;
                    for (int i = 0; i < 3; ++i)
                        q |= ((C[i] >> bitpos) & 1u) << i;
                }
            }
            codes[(size_t)n * K + k] = (uint8_t)q;
        }
    }
    return 0;
}

/*
 * Scales and zeros travel to the device in tile order: entry (n, g) is element
 * (n/16)*G*16 + g*16 + n%16 of an array of Np*G fp16 values.  This puts them
 * back in row-major [N, G].
 */
int ora_untile_meta(const uint16_t *tiled, int N, int G, uint16_t *rowmajor)
{
    if (!tiled || !rowmajor)
        return -1;
    for (int n = 0; n < N; ++n)
        for (int g = 0; g < G; ++g)
            rowmajor[(size_t)n * G + g] = tiled[((size_t)(n / 16) * G + g) * 16 + n % 16];
    return 0;
}

/* ------------------------------------------------------------ dequantize */

/*
 * W32[n,k] = float(s) * (float(q) - float(z)), each operation rounded to fp32.
 * For integer zeros (what RTN produces) and for z/2^d (what truncation
 * produces) both steps are exact.
 */
int ora_dequant(const uint8_t *codes, const uint16_t *scales, const uint16_t *zeros,
                int N, int K, int group, float *W32)
{
    if (!codes || !scales || !zeros || !W32)
        return -1;
    if (group <= 0 || K % group != 0)
        return -2;
    int G = K / group;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k) {
            size_t m = (size_t)n * G + k / group;
            volatile float d = (float)codes[(size_t)n * K + k] - ora_h2f(zeros[m]);
            W32[(size_t)n * K + k] = ora_h2f(scales[m]) * d;
        }
    return 0;
}

/*
 * Nesting by truncation (Section "Elastic Serving": a lower precision is the
 * higher one with code bits dropped).  Drop d low bits of every code:
 *   q' = q >> d,  s' = s * 2^d,  z' = z / 2^d        (lower-edge reconstruction)
 * so that  s' * (q' - z') == s * ((q & ~(2^d - 1)) - z)  exactly.  With
 * midpoint != 0 the reconstruction point moves to the middle of the dropped
 * range: z' = (z - 2^(d-1)) / 2^d.
 */
int ora_truncate(const uint8_t *codes, const uint16_t *scales, const uint16_t *zeros,
                 int N, int K, int group, int d, int midpoint,
                 uint8_t *codes_out, uint16_t *scales_out, uint16_t *zeros_out)
{
    if (!codes || !scales || !zeros || !codes_out || !scales_out || !zeros_out)
        return -1;
    if (d < 0 || d > 7 || group <= 0 || K % group != 0)
        return -2;
    int G = K / group;
    for (size_t i = 0; i < (size_t)N * K; ++i)
        codes_out[i] = (uint8_t)(codes[i] >> d);
    for (size_t i = 0; i < (size_t)N * G; ++i) {
        double s = ora_h2d(scales[i]), z = ora_h2d(zeros[i]);
        double half = (midpoint && d > 0) ? ldexp(1.0, d - 1) : 0.0;
        scales_out[i] = ora_d2h(ldexp(s, d));
        zeros_out[i] = ora_d2h(ldexp(z - half, -d));
    }
    return 0;
}

/* --------------------------------------------------------------- qlinear */

/*
 * Y[m,n] = sum_{k ascending} double(X[m,k]) * double(W32[n,k]); X fp16 [M,K],
 * W32 fp32 [N,K], Y fp64 [M,N].  This is the quantized linear layer: the
 * weights are the dequantized ones, the contraction is the plain definition.
 */
int ora_qlinear(const uint16_t *X, int M, const float *W32, int N, int K, double *Y)
{
    if (!X || !W32 || !Y)
        return -1;
#pragma omp parallel for schedule(static) collapse(2)
    for (int m = 0; m < M; ++m)
        for (int n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int k = 0; k < K; ++k)
                acc += ora_h2d(X[(size_t)m * K + k]) * (double)W32[(size_t)n * K + k];
            Y[(size_t)m * N + n] = acc;
        }
    return 0;
}

/* The unquantized head: same contraction with fp16 weights W[N,K]. */
int ora_dense_f16(const uint16_t *X, int M, const uint16_t *W, int N, int K, double *Y)
{
    if (!X || !W || !Y)
        return -1;
#pragma omp parallel for schedule(static) collapse(2)
    for (int m = 0; m < M; ++m)
        for (int n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int k = 0; k < K; ++k)
                acc += ora_h2d(X[(size_t)m * K + k]) * ora_h2d(W[(size_t)n * K + k]);
            Y[(size_t)m * N + n] = acc;
        }
    return 0;
}

/* Round an fp64 array to fp16 bit patterns (one rounding each). */
void ora_round_f16(const double *in, size_t count, uint16_t *out)
{
    for (size_t i = 0; i < count; ++i)
        out[i] = ora_d2h(in[i]);
}

/* ------------------------------------------------------------------ glue */

/* out[m,:] = fp16( t[m,:] / sqrt(mean(t[m,:]^2) + eps) ), t in fp64. */
void ora_rms_rows(const double *t, int M, int H, double eps, uint16_t *out)
{
    for (int m = 0; m < M; ++m) {
        double ss = 0.0;
        for (int i = 0; i < H; ++i)
            ss += t[(size_t)m * H + i] * t[(size_t)m * H + i];
        double inv = 1.0 / sqrt(ss / (double)H + eps);
        for (int i = 0; i < H; ++i)
            out[(size_t)m * H + i] = ora_d2h(t[(size_t)m * H + i] * inv);
    }
}

/* out = silu(g) * p elementwise in fp64, g and p fp16: silu(g) = g / (1 + exp(-g)). */
void ora_silu_mul(const uint16_t *g, const uint16_t *p, size_t count, double *out)
{
    for (size_t i = 0; i < count; ++i) {
        double gv = ora_h2d(g[i]);
        out[i] = gv / (1.0 + exp(-gv)) * ora_h2d(p[i]);
    }
}

/* ------------------------------------------------------------------- NLL */

/*
 * Token negative log-likelihood from fp16 logits [M,V]:
 *   nll[m] = log(sum_v exp(l[m,v] - max_v l[m,v])) + max_v l[m,v] - l[m,label[m]]
 * A negative label marks an ignored position (nll 0).  Perplexity of a
 * sequence is exp(mean nll) (calibrationEval in Algorithm 1 returns it).
 */
int ora_token_nll(const uint16_t *logits, const int32_t *labels, int M, int V, double *nll)
{
    if (!logits || !labels || !nll)
        return -1;
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m) {
        const uint16_t *row = logits + (size_t)m * V;
        if (labels[m] < 0 || labels[m] >= V) {
            nll[m] = 0.0;
            continue;
        }
        double mx = -INFINITY;
        for (int v = 0; v < V; ++v) {
            double x = ora_h2d(row[v]);
            if (x > mx) mx = x;
        }
        double se = 0.0;
        for (int v = 0; v < V; ++v)
            se += exp(ora_h2d(row[v]) - mx);
        nll[m] = log(se) + mx - ora_h2d(row[labels[m]]);
    }
    return 0;
}

/*
 * Euclidean distance between two sets of fp16 logits, row by row (Section
 * "Efficient Design Space Navigation": the sensitivity value of a module is the Euclidean distance
 * between the logits of the hybrid model and those of QM(n_up)):
 *   dist[m] = sqrt(sum_v (a[m,v] - b[m,v])^2)
 * The distance over a whole batch of rows is sqrt(sum_m dist[m]^2).
 */
int ora_logit_l2(const uint16_t *a, const uint16_t *b, int M, int V, double *dist)
{
    if (!a || !b || !dist)
        return -1;
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m) {
        const uint16_t *ra = a + (size_t)m * V, *rb = b + (size_t)m * V;
        double ss = 0.0;
        for (int v = 0; v < V; ++v) {
            const double d = ora_h2d(ra[v]) - ora_h2d(rb[v]);
            ss += d * d;
        }
        dist[m] = sqrt(ss);
    }
    return 0;
}

