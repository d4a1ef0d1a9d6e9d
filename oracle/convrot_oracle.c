/*
 * CPU oracle for the ConvLinear4bit forward path (ConvRot, arXiv 2512.03673).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, double-precision
 * statement of what the path computes.  It shares no code, header, table or
 * helper with the HIP library and is only ever called from tests, from the
 * smoke check and from the benchmark's "cpu_baseline" leg.  Nothing here is
 * blocked, fused or reordered: every step is the definition written out as
 * loops so it can be checked against the paper by eye.
 *
 * Steps (paper notation: N_0 = group size g, X in R^{MxK}, W in R^{NxK}):
 *   H_g      : Thm 3.3 / Eq. 9  - Kronecker powers of the printed order-4
 *              regular Hadamard matrix.
 *   rotate   : Sec. 4.2, Eq. 11-13 - every length-g block of every row is
 *              right-multiplied by H_g / sqrt(g)  (Def. of the normalised
 *              Hadamard matrix, Sec. 3.2).
 *   quantize : Eq. 1, Sec. 5.2 "per-token / per-channel 4-bit" - one scale
 *              per row, q = round(x / s).
 *   int gemm : Sec. 4.3 - acc[m,n] = sum_k qx[m,k] qw[n,k].
 *   dequant  : Sec. 4.3 / supplement Sec. B - Y = acc * s_x[m] * s_w[n], bf16.
 *
 * Readings taken where the paper is silent (also listed in the design notes):
 *   - symmetric signed codes in [-7, 7], s = absmax / 7, s = 1 for a zero row;
 *   - round = round-half-to-even;
 *   - the scale is stored as fp32; the division uses that fp32 value;
 *   - no rounding of the rotated tensor before quantisation;
 *   - K must be a multiple of g (no ragged last block);
 *   - packed layout: byte j of a row = code 2j in bits 0-3, code 2j+1 in bits
 *     4-7, 4-bit two's complement.
 *
 * Parity pins: every function below is pinned by tests/test_oracle_*.py against
 * closed forms, the printed matrix, numpy brute force and invariants.  The one
 * thing the paper gives no number for is the quantised output on random data:
 * "parity unpinned" applies to those absolute values only (they are pinned by
 * the definition plus the special cases, not by a printed example).
 *
 * OpenMP is used over independent rows only.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_ERR_ARG (-1)
#define ORACLE_ERR_OVERFLOW (-2)

/* Eq. 9: the order-4 regular Hadamard matrix as printed (-1 on the anti-diagonal). */
static const int8_t H4_PRINTED[16] = {
     1,  1,  1, -1,
     1,  1, -1,  1,
     1, -1,  1,  1,
    -1,  1,  1,  1,
};

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static int is_power_of_four(int g)
{
    if (g < 1) return 0;
    while (g > 1) {
        if (g % 4) return 0;
        g /= 4;
    }
    return 1;
}

/*
 * Thm 3.3: H_1 = [1], H_{4n} = H_n (x) H_4, i.e. (A (x) B)[i*4+p][j*4+q] = A[i][j] * B[p][q].
 * h4 == NULL selects the printed matrix; a caller may pass another order-4 base
 * (used by a test that compares the J-2I base with the printed one).
 * H is g*g, row-major.
 */
int oracle_hadamard(int g, const int8_t *h4, int8_t *H)
{
    if (!is_power_of_four(g) || !H) return ORACLE_ERR_ARG;
    if (!h4) h4 = H4_PRINTED;
    int8_t *prev = (int8_t *)malloc((size_t)g * g);
    if (!prev) return ORACLE_ERR_ARG;
    int n = 1;
    prev[0] = 1;
    while (n < g) {
        int n4 = n * 4;
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j)
                for (int p = 0; p < 4; ++p)
                    for (int q = 0; q < 4; ++q)
                        H[(size_t)(i * 4 + p) * n4 + (j * 4 + q)] =
                            (int8_t)(prev[(size_t)i * n + j] * h4[p * 4 + q]);
        memcpy(prev, H, (size_t)n4 * n4);
        n = n4;
    }
    if (g == 1) H[0] = 1;
    free(prev);
    return ORACLE_OK;
}

static double bf16_to_double(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/*
 * Sec. 4.2, Eq. 11-13: out[r, b*g + j] = (sum_i x[r, b*g + i] * H[i][j]) / sqrt(g).
 * x: bf16 bits [rows, K]; H: g*g (+-1); out: double [rows, K].
 */
int oracle_rotate(const uint16_t *x, int64_t rows, int64_t K, int g, const int8_t *H, double *out)
{
    if (!x || !H || !out || rows < 0 || K <= 0 || g <= 0 || K % g) return ORACLE_ERR_ARG;
    const double inv_sqrt_g = 1.0 / sqrt((double)g);
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const uint16_t *xr = x + r * K;
        double *orow = out + r * K;
        for (int64_t b = 0; b < K / g; ++b) {
            for (int j = 0; j < g; ++j) {
                double s = 0.0;
                for (int i = 0; i < g; ++i)
                    s += bf16_to_double(xr[b * g + i]) * (double)H[(size_t)i * g + j];
                orow[b * g + j] = s * inv_sqrt_g;
            }
        }
    }
    return ORACLE_OK;
}

/*
 * Eq. 1 with per-row scale (Sec. 5.2: per-token for X, per-output-channel for W).
 *   a = max_j |v[r,j]|, s = a / qmax (fp32), s = 1 if a == 0,
 *   q = clamp(rne(v / s), -qmax, qmax).
 * qmax = 7 for 4-bit.  codes: int8 [rows, K]; scale: float [rows].
 */
int oracle_quantize(const double *v, int64_t rows, int64_t K, int qmax, float *scale, int8_t *codes)
{
    if (!v || !scale || !codes || rows < 0 || K <= 0 || qmax < 1 || qmax > 127) return ORACLE_ERR_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const double *vr = v + r * K;
        double a = 0.0;
        for (int64_t j = 0; j < K; ++j) {
            double t = fabs(vr[j]);
            if (t > a) a = t;
        }
        float s = (a == 0.0) ? 1.0f : (float)(a / (double)qmax);
        scale[r] = s;
        for (int64_t j = 0; j < K; ++j) {
            double q = nearbyint(vr[j] / (double)s); /* default rounding mode: half to even */
            if (q > (double)qmax) q = (double)qmax;
            if (q < -(double)qmax) q = -(double)qmax;
            codes[r * K + j] = (int8_t)q;
        }
    }
    return ORACLE_OK;
}

/* Canonical packed layout: byte j = (code[2j] & 0xF) | ((code[2j+1] & 0xF) << 4). */
int oracle_pack4(const int8_t *codes, int64_t rows, int64_t K, uint8_t *packed)
{
    if (!codes || !packed || rows < 0 || K <= 0 || (K & 1)) return ORACLE_ERR_ARG;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t j = 0; j < K / 2; ++j) {
            uint8_t lo = (uint8_t)codes[r * K + 2 * j] & 0xF;
            uint8_t hi = (uint8_t)codes[r * K + 2 * j + 1] & 0xF;
            packed[r * (K / 2) + j] = (uint8_t)(lo | (hi << 4));
        }
    return ORACLE_OK;
}

int oracle_unpack4(const uint8_t *packed, int64_t rows, int64_t K, int8_t *codes)
{
    if (!codes || !packed || rows < 0 || K <= 0 || (K & 1)) return ORACLE_ERR_ARG;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t j = 0; j < K / 2; ++j) {
            uint8_t b = packed[r * (K / 2) + j];
            int lo = b & 0xF, hi = b >> 4;
            codes[r * K + 2 * j] = (int8_t)(lo >= 8 ? lo - 16 : lo);
            codes[r * K + 2 * j + 1] = (int8_t)(hi >= 8 ? hi - 16 : hi);
        }
    return ORACLE_OK;
}

/*
 * Sec. 4.3: acc[m,n] = sum_k qx[m,k] * qw[n,k]   (X W^T on the integer codes).
 * Accumulated in int64 and checked to fit int32.
 */
int oracle_int_gemm(const int8_t *qx, const int8_t *qw, int64_t M, int64_t N, int64_t K, int32_t *acc)
{
    if (!qx || !qw || !acc || M < 0 || N < 0 || K <= 0) return ORACLE_ERR_ARG;
    int overflow = 0;
#pragma omp parallel for schedule(static) reduction(| : overflow)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            int64_t s = 0;
            for (int64_t k = 0; k < K; ++k)
                s += (int64_t)qx[m * K + k] * (int64_t)qw[n * K + k];
            if (s > INT32_MAX || s < INT32_MIN) overflow = 1;
            acc[m * N + n] = (int32_t)s;
        }
    }
    return overflow ? ORACLE_ERR_OVERFLOW : ORACLE_OK;
}

/* Round a double to the nearest bfloat16 (8 significant bits), ties to even; returns bf16 bits. */
static uint16_t double_to_bf16_rne(double v)
{
    if (isnan(v)) return 0x7FC0;
    uint16_t sign = signbit(v) ? 0x8000 : 0;
    double a = fabs(v);
    if (a == 0.0) return sign;
    if (isinf(a)) return (uint16_t)(sign | 0x7F80);
    int e;
    (void)frexp(a, &e);           /* a = f * 2^e, f in [0.5, 1)  => a in [2^(e-1), 2^e) */
    int ex = e - 1;               /* floor(log2(a)) */
    if (ex < -126) ex = -126;     /* subnormal range keeps the quantum of the smallest normal */
    double quantum = ldexp(1.0, ex - 7);
    double r = nearbyint(a / quantum) * quantum;   /* both operations exact in double */
    if (r >= ldexp(1.0, 128)) return (uint16_t)(sign | 0x7F80);
    float f = (float)r;           /* exact: r has at most 8 significant bits */
    uint32_t u;
    memcpy(&u, &f, 4);
    return (uint16_t)(sign | (u >> 16));
}

uint16_t oracle_double_to_bf16(double v) { return double_to_bf16_rne(v); }

/*
 * Sec. 4.3 / supplement Sec. B: Y[m,n] = bf16( acc[m,n] * s_x[m] * s_w[n] + b[n] ), all in double, one
 * rounding.  The bias b (bf16 [N], may be NULL = none) is not in the paper's Eq. 10; the linear layers
 * the paper replaces carry one, and it is taken as added to the dequantised product before the
 * single rounding to the output type.
 */
int oracle_dequant(const int32_t *acc, const float *sx, const float *sw, const uint16_t *bias, int64_t M, int64_t N,
                   uint16_t *y)
{
    if (!acc || !sx || !sw || !y || M < 0 || N < 0) return ORACLE_ERR_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            double v = (double)acc[m * N + n] * (double)sx[m] * (double)sw[n];
            if (bias) v += bf16_to_double(bias[n]);
            y[m * N + n] = double_to_bf16_rne(v);
        }
    return ORACLE_OK;
}

/*
 * One operand through rotation + quantisation: bf16 rows -> codes + scales.
 * Serves X (rows = tokens) and W (rows = output channels) alike (Eq. 12-13).
 */
int oracle_rotquant(const uint16_t *x, int64_t rows, int64_t K, int g, int qmax, int8_t *codes, float *scale)
{
    if (!x || !codes || !scale || rows < 0 || K <= 0) return ORACLE_ERR_ARG;
    if (!is_power_of_four(g) || K % g) return ORACLE_ERR_ARG;
    int8_t *H = (int8_t *)malloc((size_t)g * g);
    double *rot = (double *)malloc(sizeof(double) * (size_t)(rows > 0 ? rows : 1) * (size_t)K);
    int rc = ORACLE_ERR_ARG;
    if (H && rot) {
        rc = oracle_hadamard(g, NULL, H);
        if (rc == ORACLE_OK) rc = oracle_rotate(x, rows, K, g, H, rot);
        if (rc == ORACLE_OK) rc = oracle_quantize(rot, rows, K, qmax, scale, codes);
    }
    free(H);
    free(rot);
    return rc;
}

/*
 * The whole ConvLinear forward (Sec. 4.3) on bf16 X[M,K] and bf16 W[N,K]: rotate + quantise both,
 * integer GEMM, dequantise (+ optional bias) to bf16 Y[M,N].  qmax = 7 is ConvLinear4bit (W4A4);
 * qmax = 127 is the W8A8 variant of the same layer (Sec. 5, Tables 5-2 and 5-4), read as the same
 * symmetric quantiser with s = absmax / 127.
 */
int oracle_convlinear(const uint16_t *x, const uint16_t *w, const uint16_t *bias, int64_t M, int64_t N, int64_t K,
                      int g, int qmax, uint16_t *y)
{
    if (!x || !w || !y || M < 0 || N < 0 || K <= 0) return ORACLE_ERR_ARG;
    size_t m1 = (size_t)(M > 0 ? M : 1), n1 = (size_t)(N > 0 ? N : 1);
    int8_t *qx = (int8_t *)malloc(m1 * (size_t)K), *qw = (int8_t *)malloc(n1 * (size_t)K);
    float *sx = (float *)malloc(sizeof(float) * m1), *sw = (float *)malloc(sizeof(float) * n1);
    int32_t *acc = (int32_t *)malloc(sizeof(int32_t) * m1 * n1);
    int rc = ORACLE_ERR_ARG;
    if (qx && qw && sx && sw && acc) {
        rc = oracle_rotquant(x, M, K, g, qmax, qx, sx);
        if (rc == ORACLE_OK) rc = oracle_rotquant(w, N, K, g, qmax, qw, sw);
        if (rc == ORACLE_OK) rc = oracle_int_gemm(qx, qw, M, N, K, acc);
        if (rc == ORACLE_OK) rc = oracle_dequant(acc, sx, sw, bias, M, N, y);
    }
    free(qx); free(qw); free(sx); free(sw); free(acc);
    return rc;
}
