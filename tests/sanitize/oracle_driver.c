/* Host sanitizer run of the CPU oracle: every exported function on exactly sized heap buffers, so that
 * AddressSanitizer sees any access one element out of bounds and UBSan any overflow, shift or
 * misaligned access.  Built and run by tests/test_host_sanitizers.py; checks a few invariants
 * on the way so that the calls cannot be optimised into nothing. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_num_threads(void);
int oracle_hadamard(int g, const int8_t *h4, int8_t *H);
int oracle_rotate(const uint16_t *x, int64_t rows, int64_t K, int g, const int8_t *H, double *out);
int oracle_quantize(const double *v, int64_t rows, int64_t K, int qmax, float *scale, int8_t *codes);
int oracle_pack4(const int8_t *codes, int64_t rows, int64_t K, uint8_t *packed);
int oracle_unpack4(const uint8_t *packed, int64_t rows, int64_t K, int8_t *codes);
int oracle_int_gemm(const int8_t *qx, const int8_t *qw, int64_t M, int64_t N, int64_t K, int32_t *acc);
uint16_t oracle_double_to_bf16(double v);
int oracle_dequant(const int32_t *acc, const float *sx, const float *sw, const uint16_t *bias, int64_t M, int64_t N,
                   uint16_t *y);
int oracle_rotquant(const uint16_t *x, int64_t rows, int64_t K, int g, int qmax, int8_t *codes, float *scale);
int oracle_convlinear(const uint16_t *x, const uint16_t *w, const uint16_t *bias, int64_t M, int64_t N, int64_t K,
                      int g, int qmax, uint16_t *y);

#define CHECK(cond)                                                                  \
    do {                                                                             \
        if (!(cond)) {                                                               \
            fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
            exit(1);                                                                 \
        }                                                                            \
    } while (0)

static uint32_t rng_state = 12345u;
static double unit_random(void)   /* xorshift, uniform in (-1, 1) */
{
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 17;
    rng_state ^= rng_state << 5;
    return (double)(int32_t)rng_state / 2147483648.0;
}

static void fill_bf16(uint16_t *p, int64_t n, double amp)
{
    for (int64_t i = 0; i < n; ++i) p[i] = oracle_double_to_bf16(unit_random() * amp);
}

int main(void)
{
    static const int groups[] = {4, 16, 64, 256, 1024};
    CHECK(oracle_num_threads() >= 1);
    for (int gi = 0; gi < 5; ++gi) {
        const int g = groups[gi];
        int8_t *H = malloc((size_t)g * g);
        CHECK(oracle_hadamard(g, NULL, H) == 0);
        int64_t rowsum = 0;
        for (int j = 0; j < g; ++j) rowsum += H[j];
        CHECK(rowsum * rowsum == g);                       /* regular: every row sums to sqrt(g) */

        const int64_t M = 5, N = 7, K = 2 * (int64_t)g < 32 ? 32 : 2 * (int64_t)g;
        uint16_t *x = malloc(sizeof(uint16_t) * M * K), *w = malloc(sizeof(uint16_t) * N * K);
        uint16_t *bias = malloc(sizeof(uint16_t) * N), *y = malloc(sizeof(uint16_t) * M * N);
        fill_bf16(x, M * K, 3.0);
        fill_bf16(w, N * K, 0.05);
        fill_bf16(bias, N, 0.1);
        memset(x + 2 * K, 0, sizeof(uint16_t) * K);        /* an all-zero row: scale 1, codes 0 */

        double *rot = malloc(sizeof(double) * M * K);
        CHECK(oracle_rotate(x, M, K, g, H, rot) == 0);
        int8_t *qx = malloc(M * K), *qw = malloc(N * K), *q2 = malloc(M * K);
        float *sx = malloc(sizeof(float) * M), *sw = malloc(sizeof(float) * N), *s2 = malloc(sizeof(float) * M);
        for (int qmax = 7; qmax <= 127; qmax += 120) {
            CHECK(oracle_quantize(rot, M, K, qmax, sx, qx) == 0);
            CHECK(oracle_rotquant(x, M, K, g, qmax, q2, s2) == 0);
            CHECK(memcmp(qx, q2, M * K) == 0 && memcmp(sx, s2, sizeof(float) * M) == 0);
            CHECK(sx[2] == 1.0f);
            for (int64_t i = 0; i < M * K; ++i) CHECK(qx[i] >= -qmax && qx[i] <= qmax);
            CHECK(oracle_rotquant(w, N, K, g, qmax, qw, sw) == 0);
            int32_t *acc = malloc(sizeof(int32_t) * M * N);
            CHECK(oracle_int_gemm(qx, qw, M, N, K, acc) == 0);
            CHECK(oracle_dequant(acc, sx, sw, bias, M, N, y) == 0);
            uint16_t *y2 = malloc(sizeof(uint16_t) * M * N);
            CHECK(oracle_convlinear(x, w, bias, M, N, K, g, qmax, y2) == 0);
            CHECK(memcmp(y, y2, sizeof(uint16_t) * M * N) == 0);
            CHECK(oracle_dequant(acc, sx, sw, NULL, M, N, y2) == 0);
            free(y2);
            free(acc);
        }
        CHECK(oracle_rotquant(x, M, K, g, 7, qx, sx) == 0);
        uint8_t *packed = malloc(M * K / 2);
        CHECK(oracle_pack4(qx, M, K, packed) == 0);
        CHECK(oracle_unpack4(packed, M, K, q2) == 0);
        CHECK(memcmp(qx, q2, M * K) == 0);
        /* argument errors must be reported, not executed */
        CHECK(oracle_rotate(x, M, K + 1, g, H, rot) != 0);
        CHECK(oracle_hadamard(g + 1, NULL, H) != 0);
        free(packed); free(qx); free(qw); free(q2); free(sx); free(sw); free(s2); free(rot);
        free(x); free(w); free(bias); free(y); free(H);
    }
    /* the accumulator bound: K = 65536 products of +-49, and of +-127^2 */
    {
        const int64_t K = 65536;
        int8_t *a = malloc(K), *b = malloc(K);
        int32_t acc;
        memset(a, 7, K); memset(b, -7, K);
        CHECK(oracle_int_gemm(a, b, 1, 1, K, &acc) == 0 && acc == -49 * 65536);
        memset(a, 127, K); memset(b, 127, K);
        CHECK(oracle_int_gemm(a, b, 1, 1, K, &acc) == 0 && acc == 127 * 127 * 65536);
        free(a); free(b);
    }
    /* bf16 rounding of special values */
    CHECK(oracle_double_to_bf16(0.0) == 0 && oracle_double_to_bf16(1.0) == 0x3F80 && oracle_double_to_bf16(-2.0) == 0xC000);
    CHECK(oracle_double_to_bf16(1e300) == 0x7F80 && oracle_double_to_bf16(-1e300) == 0xFF80);
    CHECK(oracle_double_to_bf16(1e-60) == 0);
    puts("oracle under sanitizers: ok");
    return 0;
}
