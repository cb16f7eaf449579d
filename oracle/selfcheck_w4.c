/*
 * Self-check driver for the scalar C oracle (oracle_w4.c), meant to be built with the address and undefined-behaviour
 * sanitizers and run on the CPU:
 *
 *     gcc -std=c11 -O1 -g -fopenmp -fsanitize=address,undefined -fno-sanitize-recover=all \
 *         oracle/selfcheck_w4.c oracle/oracle_w4.c -lm -o selfcheck && ./selfcheck
 *
 * TEST INFRASTRUCTURE ONLY, like the oracle itself.  It calls every exported function on small ragged shapes with heap
 * buffers of exactly the documented sizes, so that an index that runs past a buffer, a shift that overflows or a
 * misaligned access stops the run, and checks the identities that need no second implementation (round trips, the
 * blocked matmul against the element-by-element one, a group index that restates the plain grouping, argument errors).
 * Exit status 0 = every check passed.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

double orc_fp16_to_double(uint16_t h);
uint16_t orc_double_to_fp16(double x);
int orc_quantise_bits(const float* W, int K, int N, int g, int bits, uint8_t* q, uint16_t* s, uint16_t* z);
int orc_quantise(const float* W, int K, int N, int g, uint8_t* q, uint16_t* s, uint16_t* z);
int orc_pack_canonical(const uint8_t* q, int K, int N, uint32_t* out);
int orc_unpack_canonical(const uint32_t* in, int K, int N, uint8_t* q);
int orc_pack_canonical8(const uint8_t* q, int K, int N, uint32_t* out);
int orc_unpack_canonical8(const uint32_t* in, int K, int N, uint8_t* q);
int orc_pack_n8i(const uint8_t* q, int K, int N, uint32_t* out);
int orc_unpack_n8i(const uint32_t* in, int K, int N, uint8_t* q);
int orc_pack_k8(const uint8_t* q, int K, int N, uint32_t* out);
int orc_unpack_k8(const uint32_t* in, int K, int N, uint8_t* q);
int orc_unpack_packed(const uint32_t* wbuf, const uint32_t* szbuf, int K, int N, int g, uint8_t* q, uint16_t* s, uint16_t* z);
int orc_unpack_packed8(const uint32_t* wbuf, const uint32_t* szbuf, int K, int N, int g, uint8_t* q, uint16_t* s, uint16_t* z);
int orc_dequant_gidx(const uint8_t* q, const uint16_t* s, const uint16_t* z, const int32_t* gidx, int K, int N, int G, double* What);
int orc_gemm_gidx(const uint16_t* X, int M, const uint8_t* q, const uint16_t* s, const uint16_t* z, const int32_t* gidx, int K,
                  int N, int G, uint16_t* Y);
void orc_fp8e4m3_decode_table(double* out256);
int orc_quantise_fp8(const float* W, int K, int N, int g, uint8_t* q, uint16_t* s);
int orc_dequant_fp8(const uint8_t* q, const uint16_t* s, int K, int N, int g, double* What);
int orc_gemm_fp8(const uint16_t* X, int M, const uint8_t* q, const uint16_t* s, int K, int N, int g, uint16_t* Y, double* Yd);
int orc_dequant(const uint8_t* q, const uint16_t* s, const uint16_t* z, int K, int N, int g, double* What);
int orc_gemm(const uint16_t* X, int M, const uint8_t* q, const uint16_t* s, const uint16_t* z, int K, int N, int g, uint16_t* Y,
             double* Yd);
int orc_gemm_sampled(const uint16_t* X, int M, const uint8_t* q, const uint16_t* s, const uint16_t* z, int K, int N, int g,
                     const int32_t* ms, const int32_t* ns, long count, uint16_t* Y, double* Yd);
int orc_num_threads(void);

static int failures = 0;
#define CHECK(cond)                                                              \
    do {                                                                         \
        if (!(cond)) {                                                           \
            fprintf(stderr, "selfcheck: line %d: %s\n", __LINE__, #cond);        \
            ++failures;                                                          \
        }                                                                        \
    } while (0)

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(void)                      /* splitmix64, upper half */
{
    uint64_t z = (rng_state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return (uint32_t)((z ^ (z >> 31)) >> 32);
}
static float rnd_unit(void) { return (float)(rnd() >> 8) / 16777216.0f - 0.5f; }
static void* xmalloc(size_t n)
{
    void* p = malloc(n ? n : 1);
    if (!p) { fprintf(stderr, "selfcheck: out of memory\n"); exit(2); }
    return p;
}

static void check_fp16(void)
{
    for (uint32_t h = 0; h < 65536; ++h) {
        int is_nan = ((h >> 10) & 0x1F) == 0x1F && (h & 0x3FF);
        double v = orc_fp16_to_double((uint16_t)h);
        if (is_nan) { CHECK(isnan(v)); continue; }
        CHECK(orc_double_to_fp16(v) == (uint16_t)h);
    }
    CHECK(orc_double_to_fp16(1.0) == 0x3C00 && orc_double_to_fp16(-2.0) == 0xC000);
    CHECK(orc_double_to_fp16(65520.0) == 0x7C00);          /* rounds up to infinity */
    CHECK(orc_double_to_fp16(1.0 + 1.0 / 2048.0) == 0x3C00); /* tie to even */
    CHECK(orc_double_to_fp16(1.0 + 3.0 / 2048.0) == 0x3C02);
    CHECK(orc_double_to_fp16(1e-30) == 0 && orc_double_to_fp16(-1e-30) == 0x8000);
}

static void check_shape(int M, int K, int N, int g, int bits)
{
    const int G = K / g;
    float* W = xmalloc(sizeof(float) * K * N);
    for (long i = 0; i < (long)K * N; ++i) W[i] = 0.04f * rnd_unit();
    uint8_t* q = xmalloc((size_t)K * N);
    uint8_t* q2 = xmalloc((size_t)K * N);
    uint16_t* s = xmalloc(sizeof(uint16_t) * G * N);
    uint16_t* z = xmalloc(sizeof(uint16_t) * G * N);
    CHECK(orc_quantise_bits(W, K, N, g, bits, q, s, z) == 0);
    const int qmax = (1 << bits) - 1;
    for (long i = 0; i < (long)K * N; ++i) CHECK(q[i] <= qmax);
    for (long i = 0; i < (long)G * N; ++i) {
        double zz = orc_fp16_to_double(z[i]);
        CHECK(zz >= 0 && zz <= qmax && zz == floor(zz) && orc_fp16_to_double(s[i]) > 0);
    }
    if (bits == 4) {
        uint32_t* w = xmalloc(sizeof(uint32_t) * K * N / 8);
        CHECK(orc_pack_canonical(q, K, N, w) == 0 && orc_unpack_canonical(w, K, N, q2) == 0 && !memcmp(q, q2, (size_t)K * N));
        CHECK(orc_pack_n8i(q, K, N, w) == 0 && orc_unpack_n8i(w, K, N, q2) == 0 && !memcmp(q, q2, (size_t)K * N));
        CHECK(orc_pack_k8(q, K, N, w) == 0 && orc_unpack_k8(w, K, N, q2) == 0 && !memcmp(q, q2, (size_t)K * N));
        free(w);
    } else {
        uint32_t* w = xmalloc(sizeof(uint32_t) * K * N / 4);
        CHECK(orc_pack_canonical8(q, K, N, w) == 0 && orc_unpack_canonical8(w, K, N, q2) == 0 && !memcmp(q, q2, (size_t)K * N));
        free(w);
    }
    /* the packed-layout inverse on buffers of exactly the packed size (any word pattern is a valid buffer) */
    if (K % 128 == 0 && N % 16 == 0) {
        size_t wwords = (size_t)K * N * bits / 32, szwords = (size_t)G * N;
        uint32_t* wb = xmalloc(sizeof(uint32_t) * wwords);
        uint32_t* sb = xmalloc(sizeof(uint32_t) * szwords);
        for (size_t i = 0; i < wwords; ++i) wb[i] = rnd();
        for (size_t i = 0; i < szwords; ++i) sb[i] = rnd();
        uint16_t* s2 = xmalloc(sizeof(uint16_t) * G * N);
        uint16_t* z2 = xmalloc(sizeof(uint16_t) * G * N);
        int rc = bits == 4 ? orc_unpack_packed(wb, sb, K, N, g, q2, s2, z2) : orc_unpack_packed8(wb, sb, K, N, g, q2, s2, z2);
        CHECK(rc == 0);
        long hist = 0;
        for (long i = 0; i < (long)K * N; ++i) { CHECK(q2[i] <= qmax); hist += q2[i]; }
        CHECK(hist > 0);
        free(wb); free(sb); free(s2); free(z2);
    }
    /* matmul: the column-blocked routine against the element-by-element one, bit for bit, plus the group-index form */
    uint16_t* X = xmalloc(sizeof(uint16_t) * (M ? M : 1) * K);
    for (long i = 0; i < (long)M * K; ++i) X[i] = orc_double_to_fp16(2.0 * rnd_unit());
    uint16_t* Y = xmalloc(sizeof(uint16_t) * (M ? M : 1) * N);
    double* Yd = xmalloc(sizeof(double) * (M ? M : 1) * N);
    CHECK(orc_gemm(X, M, q, s, z, K, N, g, Y, Yd) == 0);
    if (M > 0) {
        long cnt = (long)M * N;
        int32_t* ms = xmalloc(sizeof(int32_t) * cnt);
        int32_t* ns = xmalloc(sizeof(int32_t) * cnt);
        for (long i = 0; i < cnt; ++i) { ms[i] = (int32_t)(i / N); ns[i] = (int32_t)(i % N); }
        uint16_t* Ys = xmalloc(sizeof(uint16_t) * cnt);
        double* Ysd = xmalloc(sizeof(double) * cnt);
        CHECK(orc_gemm_sampled(X, M, q, s, z, K, N, g, ms, ns, cnt, Ys, Ysd) == 0);
        CHECK(!memcmp(Y, Ys, sizeof(uint16_t) * cnt));
        for (long i = 0; i < cnt; ++i) CHECK(Yd[i] == Ysd[i]);
        ms[0] = M;                                          /* an index past the end is an error, not a read */
        CHECK(orc_gemm_sampled(X, M, q, s, z, K, N, g, ms, ns, cnt, Ys, NULL) == -2);
        int32_t* gidx = xmalloc(sizeof(int32_t) * K);
        for (int k = 0; k < K; ++k) gidx[k] = k / g;
        CHECK(orc_gemm_gidx(X, M, q, s, z, gidx, K, N, G, Ys) == 0);
        CHECK(!memcmp(Y, Ys, sizeof(uint16_t) * cnt));
        double* Wh = xmalloc(sizeof(double) * K * N);
        double* Wg = xmalloc(sizeof(double) * K * N);
        CHECK(orc_dequant(q, s, z, K, N, g, Wh) == 0 && orc_dequant_gidx(q, s, z, gidx, K, N, G, Wg) == 0);
        CHECK(!memcmp(Wh, Wg, sizeof(double) * K * N));
        for (int n = 0; n < N; ++n)                         /* closed form on the first row */
            CHECK(Wh[n] == ((double)q[n] - orc_fp16_to_double(z[n])) * orc_fp16_to_double(s[n]));
        free(ms); free(ns); free(Ys); free(Ysd); free(gidx); free(Wh); free(Wg);
    }
    if (bits == 8) {                                        /* the FP8 routes share the 8-bit buffers */
        uint16_t* s8 = xmalloc(sizeof(uint16_t) * G * N);
        CHECK(orc_quantise_fp8(W, K, N, g, q2, s8) == 0);
        double* Wh = xmalloc(sizeof(double) * K * N);
        CHECK(orc_dequant_fp8(q2, s8, K, N, g, Wh) == 0);
        for (long i = 0; i < (long)K * N; ++i) CHECK(isfinite(Wh[i]) && fabs(Wh[i] - W[i]) <= 0.07 * fabs(W[i]) + 1e-4);
        CHECK(orc_gemm_fp8(X, M, q2, s8, K, N, g, Y, Yd) == 0);
        free(s8); free(Wh);
    }
    free(W); free(q); free(q2); free(s); free(z); free(X); free(Y); free(Yd);
}

int main(void)
{
    check_fp16();
    double table[256];
    orc_fp8e4m3_decode_table(table);
    CHECK(table[0] == 0.0 && table[0x38] == 1.0 && table[0x7E] == 448.0 && isnan(table[0x7F]) && table[0xB8] == -1.0);
    CHECK(table[0x01] == ldexp(1.0, -9));
    static const int shapes[][5] = {                        /* M, K, N, group, bits */
        {1, 128, 16, 128, 4}, {3, 384, 80, 64, 4}, {0, 128, 16, 32, 4}, {17, 256, 272, 32, 4}, {5, 96, 24, 32, 4},
        {2, 128, 16, 128, 8}, {9, 384, 48, 64, 8}, {4, 64, 20, 32, 8}, {33, 640, 528, 128, 4},
    };
    for (unsigned i = 0; i < sizeof(shapes) / sizeof(shapes[0]); ++i)
        check_shape(shapes[i][0], shapes[i][1], shapes[i][2], shapes[i][3], shapes[i][4]);
    /* argument errors come back as codes */
    uint8_t b8[8] = {0};
    uint16_t b16[8] = {0};
    uint32_t b32[8] = {0};
    float f[8] = {0};
    double d[8] = {0};
    CHECK(orc_quantise(NULL, 128, 16, 128, b8, b16, b16) == -1 && orc_quantise(f, 100, 16, 128, b8, b16, b16) == -1);
    CHECK(orc_quantise_bits(f, 128, 16, 128, 5, b8, b16, b16) == -1);
    CHECK(orc_pack_canonical(b8, 1, 12, b32) == -1 && orc_pack_k8(b8, 12, 8, b32) == -1 && orc_pack_canonical8(b8, 1, 6, b32) == -1);
    CHECK(orc_gemm(b16, 1, b8, b16, b16, 100, 16, 128, b16, d) == -1 && orc_gemm(NULL, 1, b8, b16, b16, 128, 16, 128, b16, d) == -1);
    CHECK(orc_dequant(b8, b16, b16, 128, 16, 0, d) == -1 && orc_gemm_fp8(b16, 1, b8, b16, 100, 16, 128, b16, d) == -1);
    CHECK(orc_unpack_packed(NULL, b32, 128, 16, 128, b8, b16, b16) == -1);
    CHECK(orc_num_threads() >= 1);
    if (failures) {
        fprintf(stderr, "selfcheck: %d check(s) failed\n", failures);
        return 1;
    }
    printf("selfcheck: all checks passed\n");
    return 0;
}
