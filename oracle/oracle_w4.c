/*
 * CPU oracle for the W4A16 weight-only-quantised GEMM  Y = X * dequant(Wq).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, scalar, obviously-correct definition the GPU
 * library is compared against.  It shares no code, header, table or constant with the HIP path and
 * must never be linked into or called from the product library.
 *
 * What is defined here and where the definition comes from:
 *   - orc_quantise:   group-wise asymmetric int4 quantiser of the workload recipe
 *                     (s = (max-min)/15 as fp16, z = round(-min/s) in [0,15],
 *                      q = clamp(round(w/s)+z, 0, 15); rounding is round-half-to-even).
 *   - orc_pack_canonical / orc_unpack_canonical:
 *                     "eight INT4 values per 32-bit word" (paper Sec. 3.2, challenge M2): the interchange
 *                     layout handed to the library, u32 [K][N/8], nibble t of word (k,j) = q[k][8j+t].
 *   - orc_pack_n8i / orc_unpack_n8i, orc_pack_k8 / orc_unpack_k8:
 *                     the two other word orders in which 4-bit checkpoints of the families the paper names
 *                     (Sec. 4.1: one pack routine serves several weight formats) keep the same integers:
 *                     N-major words whose nibbles walk the eight columns in the order 0,2,4,6,1,3,5,7, and
 *                     K-major words u32 [K/8][N] holding eight consecutive rows of one column.
 *   - orc_quantise_bits, orc_pack_canonical8 / orc_unpack_canonical8, orc_unpack_packed8:
 *                     the same pipeline for 8-bit weights (paper Sec. 4.1/Sec. 3.3 present packing and the fused
 *                     GEMM as independent of the weight width): codes 0..255, four per 32-bit word.
 *   - orc_fp8e4m3_decode_table, orc_quantise_fp8, orc_dequant_fp8, orc_gemm_fp8:
 *                     FP8 (E4M3) weight codes through the same GEMM (the paper's evaluation includes an FP8 model,
 *                     Sec. 5.3): W^[k][n] = fp8(q[k][n]) * s[k/g][n], no zero-point; the format is the published
 *                     OCP 8-bit floating point E4M3 (finite-only: bias 7, no infinities, S.1111.111 = NaN).
 *   - orc_dequant_gidx, orc_gemm_gidx:
 *                     the same GEMM when the K-group of a row is given by an index array instead of k / g
 *                     (checkpoints quantised in activation order): W^[k][n] = (q[k][n] - z[gidx[k]][n]) * s[gidx[k]][n].
 *   - orc_unpack_packed:
 *                     inverse index map of the library's MFMA-fragment-ordered buffer (the gfx950 analogue
 *                     of the packed fragment store of paper Sec. 4.1 steps (iii)-(iv)); written from the
 *                     layout specification only.
 *   - orc_dequant:    W^[k][n] = (q - z) * s, paper Sec. 3.1 step (iii), evaluated exactly in fp64.
 *   - orc_gemm*:      paper Sec. 3.1 step (iv): a standard matrix multiply of the fp16 activations with the
 *                     dequantised weights; here accumulated in fp64 with k ascending and rounded once to fp16.
 *
 * Parity status: every function here is pinned by tests that do not call it to produce their expected
 * values (exhaustive fp16 tables against numpy.float16, hand-worked quantiser groups, closed-form pack
 * words, brute-force loops, numpy matmul).  Nothing is "parity unpinned".
 *
 * The host compiler has no _Float16, so fp16 <-> fp64 conversion is written out below.
 * OpenMP pragmas only parallelise independent outputs; they never change any sum order.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_API __attribute__((visibility("default")))

/* ---------------------------------------------------------------- fp16 <-> fp64 (IEEE 754 binary16) */

ORC_API double orc_fp16_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1F;
    int frac = h & 0x3FF;
    double v;
    if (expo == 0) {
        v = ldexp((double)frac, -24);              /* zero and subnormals: frac * 2^-24 */
    } else if (expo == 31) {
        v = frac ? NAN : INFINITY;
    } else {
        v = ldexp((double)(1024 + frac), expo - 25); /* (1 + frac/1024) * 2^(expo-15) */
    }
    return sign ? -v : v;
}

/* round-to-nearest, ties-to-even, directly from fp64 (no intermediate fp32: no double rounding) */
ORC_API uint16_t orc_double_to_fp16(double x)
{
    uint16_t sign = signbit(x) ? 0x8000u : 0u;
    if (isnan(x)) return (uint16_t)(sign | 0x7E00u);
    double a = fabs(x);
    if (isinf(a)) return (uint16_t)(sign | 0x7C00u);
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e);                /* a = f * 2^e with f in [0.5,1)  ->  floor(log2 a) = e-1 */
    int p = e - 1;
    if (p < -14) {
        /* subnormal range: spacing 2^-24 */
        double r = nearbyint(ldexp(a, 24));        /* exact scaling, then RNE (default rounding mode) */
        return (uint16_t)(sign | (uint16_t)r);     /* r == 1024 lands on the smallest normal by carry */
    }
    /* normal range: spacing 2^(p-10); r in [1024, 2048] */
    double r = nearbyint(ldexp(a, 10 - p));
    uint32_t bits = ((uint32_t)(p + 15) << 10) + ((uint32_t)r - 1024u); /* r == 2048 carries into the exponent */
    if (bits >= 0x7C00u) bits = 0x7C00u;           /* overflow -> infinity */
    return (uint16_t)(sign | bits);
}

/* ---------------------------------------------------------------- quantiser (workload recipe) */

static float clampf(float v, float lo, float hi) { return v < lo ? lo : (v > hi ? hi : v); }

/*
 * W fp32 [K][N] row-major; group g along K.  Outputs: q u8 [K][N] (values 0..15),
 * s fp16 bits [K/g][N], z fp16 bits [K/g][N] (the integer zero-point stored as fp16).
 * s is rounded to fp16 first; z and q are computed in fp32 with that rounded s.
 * A group whose fp16 scale would be zero (constant group, or range below fp16 resolution) gets s = 1.
 */
ORC_API int orc_quantise_bits(const float* W, int K, int N, int g, int bits, uint8_t* q, uint16_t* s, uint16_t* z)
{
    if (!W || !q || !s || !z || K <= 0 || N <= 0 || g <= 0 || K % g || (bits != 4 && bits != 8)) return -1;
    const float qmax = (float)((1 << bits) - 1);           /* 15 or 255 */
    int G = K / g;
    for (int gi = 0; gi < G; ++gi) {
        for (int n = 0; n < N; ++n) {
            float mn = W[(size_t)(gi * g) * N + n], mx = mn;
            for (int k = gi * g; k < gi * g + g; ++k) {
                float w = W[(size_t)k * N + n];
                if (w < mn) mn = w;
                if (w > mx) mx = w;
            }
            float s32 = (mx - mn) / qmax;
            uint16_t sh = orc_double_to_fp16((double)s32);
            float sf = (float)orc_fp16_to_double(sh);
            if (!(sf > 0.0f) || isinf(sf)) { sf = 1.0f; sh = 0x3C00u; }
            float zf = clampf(rintf(-mn / sf), 0.0f, qmax);
            s[(size_t)gi * N + n] = sh;
            z[(size_t)gi * N + n] = orc_double_to_fp16((double)zf);
            for (int k = gi * g; k < gi * g + g; ++k) {
                float w = W[(size_t)k * N + n];
                float qf = clampf(rintf(w / sf) + zf, 0.0f, qmax);
                q[(size_t)k * N + n] = (uint8_t)qf;
            }
        }
    }
    return 0;
}

/* the 4-bit recipe of the benchmark configurations */
ORC_API int orc_quantise(const float* W, int K, int N, int g, uint8_t* q, uint16_t* s, uint16_t* z)
{
    return orc_quantise_bits(W, K, N, g, 4, q, s, z);
}

/* ---------------------------------------------------------------- canonical interchange layout */

/* q u8 [K][N] -> u32 [K][N/8]; nibble t (bits 4t..4t+3) of word (k,j) is q[k][8j+t] */
ORC_API int orc_pack_canonical(const uint8_t* q, int K, int N, uint32_t* out)
{
    if (!q || !out || K <= 0 || N <= 0 || N % 8) return -1;
    for (int k = 0; k < K; ++k)
        for (int j = 0; j < N / 8; ++j) {
            uint32_t w = 0;
            for (int t = 0; t < 8; ++t) w |= (uint32_t)(q[(size_t)k * N + 8 * j + t] & 0xF) << (4 * t);
            out[(size_t)k * (N / 8) + j] = w;
        }
    return 0;
}

ORC_API int orc_unpack_canonical(const uint32_t* in, int K, int N, uint8_t* q)
{
    if (!q || !in || K <= 0 || N <= 0 || N % 8) return -1;
    for (int k = 0; k < K; ++k)
        for (int n = 0; n < N; ++n)
            q[(size_t)k * N + n] = (uint8_t)((in[(size_t)k * (N / 8) + n / 8] >> (4 * (n % 8))) & 0xF);
    return 0;
}

/* 8-bit codes: q u8 [K][N] -> u32 [K][N/4]; byte t (bits 8t..8t+7) of word (k,j) is q[k][4j+t] */
ORC_API int orc_pack_canonical8(const uint8_t* q, int K, int N, uint32_t* out)
{
    if (!q || !out || K <= 0 || N <= 0 || N % 4) return -1;
    for (int k = 0; k < K; ++k)
        for (int j = 0; j < N / 4; ++j) {
            uint32_t w = 0;
            for (int t = 0; t < 4; ++t) w |= (uint32_t)q[(size_t)k * N + 4 * j + t] << (8 * t);
            out[(size_t)k * (N / 4) + j] = w;
        }
    return 0;
}

ORC_API int orc_unpack_canonical8(const uint32_t* in, int K, int N, uint8_t* q)
{
    if (!q || !in || K <= 0 || N <= 0 || N % 4) return -1;
    for (int k = 0; k < K; ++k)
        for (int n = 0; n < N; ++n)
            q[(size_t)k * N + n] = (uint8_t)((in[(size_t)k * (N / 4) + n / 4] >> (8 * (n % 4))) & 0xFF);
    return 0;
}

/* N-major, interleaved nibbles: u32 [K][N/8]; nibble p of word (k,j) is q[k][8j + ord(p)] with
 * ord = 0,2,4,6,1,3,5,7 (even columns fill the low half of the word, odd columns the high half) */
static const int orc_n8i_order[8] = {0, 2, 4, 6, 1, 3, 5, 7};

ORC_API int orc_pack_n8i(const uint8_t* q, int K, int N, uint32_t* out)
{
    if (!q || !out || K <= 0 || N <= 0 || N % 8) return -1;
    for (int k = 0; k < K; ++k)
        for (int j = 0; j < N / 8; ++j) {
            uint32_t w = 0;
            for (int p = 0; p < 8; ++p)
                w |= (uint32_t)(q[(size_t)k * N + 8 * j + orc_n8i_order[p]] & 0xF) << (4 * p);
            out[(size_t)k * (N / 8) + j] = w;
        }
    return 0;
}

ORC_API int orc_unpack_n8i(const uint32_t* in, int K, int N, uint8_t* q)
{
    if (!q || !in || K <= 0 || N <= 0 || N % 8) return -1;
    for (int k = 0; k < K; ++k)
        for (int j = 0; j < N / 8; ++j)
            for (int p = 0; p < 8; ++p)
                q[(size_t)k * N + 8 * j + orc_n8i_order[p]] =
                    (uint8_t)((in[(size_t)k * (N / 8) + j] >> (4 * p)) & 0xF);
    return 0;
}

/* K-major: u32 [K/8][N]; nibble t of word (i,n) is q[8i+t][n] */
ORC_API int orc_pack_k8(const uint8_t* q, int K, int N, uint32_t* out)
{
    if (!q || !out || K <= 0 || N <= 0 || K % 8) return -1;
    for (int i = 0; i < K / 8; ++i)
        for (int n = 0; n < N; ++n) {
            uint32_t w = 0;
            for (int t = 0; t < 8; ++t) w |= (uint32_t)(q[(size_t)(8 * i + t) * N + n] & 0xF) << (4 * t);
            out[(size_t)i * N + n] = w;
        }
    return 0;
}

ORC_API int orc_unpack_k8(const uint32_t* in, int K, int N, uint8_t* q)
{
    if (!q || !in || K <= 0 || N <= 0 || K % 8) return -1;
    for (int k = 0; k < K; ++k)
        for (int n = 0; n < N; ++n)
            q[(size_t)k * N + n] = (uint8_t)((in[(size_t)(k / 8) * N + n] >> (4 * (k % 8))) & 0xF);
    return 0;
}

/* ---------------------------------------------------------------- the library's packed layout, inverted
 *
 * Weight buffer (u32 words).  The matrix is cut into units of 16 columns x 128 rows; unit (nt, ku) covers
 * columns 16*nt .. 16*nt+15 and rows 128*ku .. 128*ku+127 and occupies the 256 consecutive words starting at
 * word ((nt * (K/128)) + ku) * 256.  Inside a unit, word index = 4*lane + t with lane = 16*h + c
 * (c = 0..15, h = 0..3) and t = 0..3.  That word holds, for column n = 16*nt + c, the eight rows
 * k = 128*ku + 32*t + 8*h + e (e = 0..7); weight e sits in nibble p(e) = 4*(e & 1) + (e >> 1),
 * i.e. bits [4p, 4p+3].
 *
 * Scale/zero buffer (u32 words): word ((nt * (K/g)) + G) * 16 + c holds, for column 16*nt + c and K-group G,
 * the fp16 scale bits in its low half and the fp16 zero-point bits in its high half.
 */
ORC_API int orc_unpack_packed(const uint32_t* wbuf, const uint32_t* szbuf, int K, int N, int g,
                              uint8_t* q, uint16_t* s, uint16_t* z)
{
    if (!wbuf || !szbuf || !q || !s || !z) return -1;
    if (K <= 0 || N <= 0 || g <= 0 || K % 128 || N % 16 || K % g) return -1;
    int KU = K / 128, G = K / g;
    for (int k = 0; k < K; ++k) {
        for (int n = 0; n < N; ++n) {
            int nt = n / 16, c = n % 16;
            int ku = k / 128, kk = k % 128;
            int t = kk / 32, h = (kk % 32) / 8, e = kk % 8;
            int lane = 16 * h + c;
            int p = 4 * (e & 1) + (e >> 1);
            uint32_t w = wbuf[((size_t)nt * KU + ku) * 256 + 4 * lane + t];
            q[(size_t)k * N + n] = (uint8_t)((w >> (4 * p)) & 0xF);
        }
    }
    for (int gi = 0; gi < G; ++gi)
        for (int n = 0; n < N; ++n) {
            uint32_t w = szbuf[((size_t)(n / 16) * G + gi) * 16 + (n % 16)];
            s[(size_t)gi * N + n] = (uint16_t)(w & 0xFFFFu);
            z[(size_t)gi * N + n] = (uint16_t)(w >> 16);
        }
    return 0;
}

/*
 * 8-bit weights.  Units of 16 columns x 64 rows (again 256 words = 1 KiB); unit (nt, ks) covers columns
 * 16*nt .. 16*nt+15 and rows 64*ks .. 64*ks+63 and starts at word ((nt * (K/64)) + ks) * 256.  Word index =
 * 4*lane + 2*tt + hf with lane = 16*h + c (c = 0..15, h = 0..3), tt = 0..1, hf = 0..1; it holds, for column
 * 16*nt + c, rows 64*ks + 32*tt + 8*h + 4*hf + b (b = 0..3), code b in byte b (bits [8b, 8b+7]).
 * The scale/zero buffer is that of the 4-bit layout.
 */
ORC_API int orc_unpack_packed8(const uint32_t* wbuf, const uint32_t* szbuf, int K, int N, int g,
                               uint8_t* q, uint16_t* s, uint16_t* z)
{
    if (!wbuf || !szbuf || !q || !s || !z) return -1;
    if (K <= 0 || N <= 0 || g <= 0 || K % 128 || N % 16 || K % g) return -1;
    int KS = K / 64, G = K / g;
    for (int k = 0; k < K; ++k) {
        for (int n = 0; n < N; ++n) {
            int nt = n / 16, c = n % 16;
            int ks = k / 64, kk = k % 64;
            int tt = kk / 32, h = (kk % 32) / 8, hf = (kk % 8) / 4, b = kk % 4;
            int lane = 16 * h + c;
            uint32_t w = wbuf[((size_t)nt * KS + ks) * 256 + 4 * lane + 2 * tt + hf];
            q[(size_t)k * N + n] = (uint8_t)((w >> (8 * b)) & 0xFF);
        }
    }
    for (int gi = 0; gi < G; ++gi)
        for (int n = 0; n < N; ++n) {
            uint32_t w = szbuf[((size_t)(n / 16) * G + gi) * 16 + (n % 16)];
            s[(size_t)gi * N + n] = (uint16_t)(w & 0xFFFFu);
            z[(size_t)gi * N + n] = (uint16_t)(w >> 16);
        }
    return 0;
}

/* ---------------------------------------------------------------- dequantise and multiply */

/* rows carry their group index explicitly: gidx[k] in [0, G) */
ORC_API int orc_dequant_gidx(const uint8_t* q, const uint16_t* s, const uint16_t* z, const int32_t* gidx, int K, int N,
                             int G, double* What)
{
    if (!q || !s || !z || !gidx || !What || K <= 0 || N <= 0 || G <= 0) return -1;
    for (int k = 0; k < K; ++k) {
        if (gidx[k] < 0 || gidx[k] >= G) return -2;
        for (int n = 0; n < N; ++n) {
            size_t gi = (size_t)gidx[k] * N + n;
            What[(size_t)k * N + n] = ((double)q[(size_t)k * N + n] - orc_fp16_to_double(z[gi])) * orc_fp16_to_double(s[gi]);
        }
    }
    return 0;
}

ORC_API int orc_gemm_gidx(const uint16_t* X, int M, const uint8_t* q, const uint16_t* s, const uint16_t* z,
                          const int32_t* gidx, int K, int N, int G, uint16_t* Y)
{
    if (!X || !q || !s || !z || !gidx || !Y || M < 0 || K <= 0 || N <= 0 || G <= 0) return -1;
    for (int k = 0; k < K; ++k)
        if (gidx[k] < 0 || gidx[k] >= G) return -2;
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
    for (int n = 0; n < N; ++n)
        for (int m = 0; m < M; ++m) {
            double acc = 0.0;
            for (int k = 0; k < K; ++k) {
                size_t gi = (size_t)gidx[k] * N + n;
                double w = ((double)q[(size_t)k * N + n] - orc_fp16_to_double(z[gi])) * orc_fp16_to_double(s[gi]);
                acc += orc_fp16_to_double(X[(size_t)m * K + k]) * w;
            }
            Y[(size_t)m * N + n] = orc_double_to_fp16(acc);
        }
    return 0;
}

/* OCP FP8 E4M3, finite-only: sign(1) exponent(4, bias 7) mantissa(3); exponent 0 is subnormal (m/8 * 2^-6);
 * exponent 15 is an ordinary binade except mantissa 7, which is NaN.  Largest finite value 1.75 * 2^8 = 448. */
static double fp8e4m3_to_double(uint8_t c)
{
    int sign = c >> 7, e = (c >> 3) & 0xF, m = c & 7;
    double v;
    if (e == 15 && m == 7) return NAN;
    if (e == 0) v = ldexp((double)m / 8.0, -6);
    else v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return sign ? -v : v;
}

ORC_API void orc_fp8e4m3_decode_table(double* out256)
{
    for (int c = 0; c < 256; ++c) out256[c] = fp8e4m3_to_double((uint8_t)c);
}

/* nearest finite code to v (|v| <= 448 after clamping); ties go to the code with an even mantissa bit.
 * Brute force over the 127 non-negative finite codes: slow and obviously right. */
static uint8_t fp8e4m3_from_float(float v)
{
    double a = fabs((double)v);
    if (a > 448.0) a = 448.0;
    int best = 0;
    double bestd = a;                                   /* distance to code 0 */
    for (int c = 1; c < 127; ++c) {
        double d = fabs(fp8e4m3_to_double((uint8_t)c) - a);
        if (d < bestd || (d == bestd && (c & 1) == 0)) { best = c; bestd = d; }
    }
    return (uint8_t)(best | ((v < 0.0f || (v == 0.0f && signbit(v))) ? 0x80 : 0));
}

/* recipe: per column and K-group s = fp16(max|w| / 448) (1 if that is 0 or not finite), q = fp8(w / s), fp32 arithmetic */
ORC_API int orc_quantise_fp8(const float* W, int K, int N, int g, uint8_t* q, uint16_t* s)
{
    if (!W || !q || !s || K <= 0 || N <= 0 || g <= 0 || K % g) return -1;
    for (int gi = 0; gi < K / g; ++gi)
        for (int n = 0; n < N; ++n) {
            float amax = 0.0f;
            for (int k = gi * g; k < gi * g + g; ++k) {
                float a = fabsf(W[(size_t)k * N + n]);
                if (a > amax) amax = a;
            }
            uint16_t sh = orc_double_to_fp16((double)(amax / 448.0f));
            float sf = (float)orc_fp16_to_double(sh);
            if (!(sf > 0.0f) || isinf(sf)) { sf = 1.0f; sh = 0x3C00u; }
            s[(size_t)gi * N + n] = sh;
            for (int k = gi * g; k < gi * g + g; ++k)
                q[(size_t)k * N + n] = fp8e4m3_from_float(W[(size_t)k * N + n] / sf);
        }
    return 0;
}

ORC_API int orc_dequant_fp8(const uint8_t* q, const uint16_t* s, int K, int N, int g, double* What)
{
    if (!q || !s || !What || K <= 0 || N <= 0 || g <= 0 || K % g) return -1;
    for (int k = 0; k < K; ++k)
        for (int n = 0; n < N; ++n)
            What[(size_t)k * N + n] = fp8e4m3_to_double(q[(size_t)k * N + n]) * orc_fp16_to_double(s[(size_t)(k / g) * N + n]);
    return 0;
}

/* Y[m][n] = fp16( sum_k X[m][k] * fp8(q[k][n]) * s[k/g][n] ), k ascending in fp64, one rounding */
ORC_API int orc_gemm_fp8(const uint16_t* X, int M, const uint8_t* q, const uint16_t* s, int K, int N, int g,
                         uint16_t* Y, double* Yd)
{
    if (!X || !q || !s || !Y || M < 0 || K <= 0 || N <= 0 || g <= 0 || K % g) return -1;
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
    for (int n = 0; n < N; ++n)
        for (int m = 0; m < M; ++m) {
            double acc = 0.0;
            for (int k = 0; k < K; ++k)
                acc += orc_fp16_to_double(X[(size_t)m * K + k]) *
                       (fp8e4m3_to_double(q[(size_t)k * N + n]) * orc_fp16_to_double(s[(size_t)(k / g) * N + n]));
            if (Yd) Yd[(size_t)m * N + n] = acc;
            Y[(size_t)m * N + n] = orc_double_to_fp16(acc);
        }
    return 0;
}


/* What[k][n] = (q - z) * s in fp64 (exact: an integer of at most 9 bits times an 11-bit significand) */
ORC_API int orc_dequant(const uint8_t* q, const uint16_t* s, const uint16_t* z, int K, int N, int g, double* What)
{
    if (!q || !s || !z || !What || K <= 0 || N <= 0 || g <= 0 || K % g) return -1;
    for (int k = 0; k < K; ++k)
        for (int n = 0; n < N; ++n) {
            size_t gi = (size_t)(k / g) * N + n;
            What[(size_t)k * N + n] = ((double)q[(size_t)k * N + n] - orc_fp16_to_double(z[gi])) * orc_fp16_to_double(s[gi]);
        }
    return 0;
}

/* one output element: sum over k ascending in fp64, one rounding to fp16 */
static uint16_t gemm_element(const uint16_t* X, const uint8_t* q, const uint16_t* s, const uint16_t* z,
                             int K, int N, int g, int m, int n, double* yd_out)
{
    double acc = 0.0;
    for (int k = 0; k < K; ++k) {
        size_t gi = (size_t)(k / g) * N + n;
        double w = ((double)q[(size_t)k * N + n] - orc_fp16_to_double(z[gi])) * orc_fp16_to_double(s[gi]);
        acc += orc_fp16_to_double(X[(size_t)m * K + k]) * w;
    }
    if (yd_out) *yd_out = acc;
    return orc_double_to_fp16(acc);
}

/*
 * Y[m][n] = fp16( sum_k X[m][k] * What[k][n] ), all M x N outputs.
 * Loop order m, k, n with an fp64 row of N running sums: every output still adds its K terms in ascending k,
 * so the result is identical to the element-by-element triple loop (orc_gemm_sampled); rows are independent
 * and are what OpenMP distributes (column blocks when M is small).
 * Yd (optional, may be NULL) receives the unrounded fp64 sums.
 */
ORC_API int orc_gemm(const uint16_t* X, int M, const uint8_t* q, const uint16_t* s, const uint16_t* z,
                     int K, int N, int g, uint16_t* Y, double* Yd)
{
    if (!X || !q || !s || !z || !Y || M < 0 || K <= 0 || N <= 0 || g <= 0 || K % g) return -1;
    if (M == 0) return 0;
    const int NB = 256;                              /* column block handed to one thread */
    int nblocks = (N + NB - 1) / NB;
    long total = (long)M * nblocks;
#pragma omp parallel
    {
        double* acc = (double*)malloc(sizeof(double) * NB);
        double* sc = (double*)malloc(sizeof(double) * NB);
        double* zp = (double*)malloc(sizeof(double) * NB);
#pragma omp for schedule(dynamic, 1)
        for (long task = 0; task < total; ++task) {
            int m = (int)(task / nblocks);
            int n0 = (int)(task % nblocks) * NB;
            int nb = N - n0 < NB ? N - n0 : NB;
            for (int j = 0; j < nb; ++j) acc[j] = 0.0;
            for (int k = 0; k < K; ++k) {
                if (k % g == 0) {
                    size_t gi = (size_t)(k / g) * N + n0;
                    for (int j = 0; j < nb; ++j) {
                        sc[j] = orc_fp16_to_double(s[gi + j]);
                        zp[j] = orc_fp16_to_double(z[gi + j]);
                    }
                }
                double x = orc_fp16_to_double(X[(size_t)m * K + k]);
                const uint8_t* qr = q + (size_t)k * N + n0;
                for (int j = 0; j < nb; ++j) acc[j] += x * (((double)qr[j] - zp[j]) * sc[j]);
            }
            for (int j = 0; j < nb; ++j) {
                Y[(size_t)m * N + n0 + j] = orc_double_to_fp16(acc[j]);
                if (Yd) Yd[(size_t)m * N + n0 + j] = acc[j];
            }
        }
        free(acc); free(sc); free(zp);
    }
    return 0;
}

/* the plain triple loop on a list of (m, n) pairs: used to check sampled outputs of shapes too large to do whole */
ORC_API int orc_gemm_sampled(const uint16_t* X, int M, const uint8_t* q, const uint16_t* s, const uint16_t* z,
                             int K, int N, int g, const int32_t* ms, const int32_t* ns, long count,
                             uint16_t* Y, double* Yd)
{
    if (!X || !q || !s || !z || !Y || !ms || !ns || count < 0 || K <= 0 || N <= 0 || g <= 0 || K % g) return -1;
    for (long i = 0; i < count; ++i)
        if (ms[i] < 0 || ms[i] >= M || ns[i] < 0 || ns[i] >= N) return -2;
#pragma omp parallel for schedule(static)
    for (long i = 0; i < count; ++i) {
        double yd;
        Y[i] = gemm_element(X, q, s, z, K, N, g, ms[i], ns[i], &yd);
        if (Yd) Yd[i] = yd;
    }
    return 0;
}

ORC_API int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
