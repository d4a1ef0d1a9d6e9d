// Kernel A of libconvrot: group-wise regular-Hadamard rotation + per-row absmax + 4-bit
// quantisation + nibble packing, one pass over the bf16 input (ConvRot paper Sec. 4.2 Eq. 11-13,
// Eq. 1, Sec. 5.2).  Serves activations (rows = tokens) and weights (rows = output channels).
//
// Work split.  A "unit" is 16 consecutive elements of a row (32 B of bf16 in, 8 B of codes out)
// and belongs to one lane.  A row is spread over T = 64*Wv lanes (Wv wavefronts); lane t of the
// row owns units t, t+T, t+2T, ... (U of them), so one wavefront load instruction covers a
// contiguous 2 KB span of the row.  The whole row stays in registers between the absmax
// reduction and the rounding, so X is read from HBM exactly once.
//
// Rotation.  H_g = H_4 (x) ... (x) H_4 (Thm 3.3) is separable: one radix-4 step per base-4 digit
// of the in-group index.  With the printed H_4 (all ones, -1 on the anti-diagonal) a step is
//     y_j = (x_0 + x_1 + x_2 + x_3) - 2 x_{3-j}.
// Digits 0 and 1 live inside a lane's 16 elements, so the index flip 3-j is register renaming.
// Digits 2, 3 (g = 64, 256) run across lanes with DPP adds and digit 4 (g = 1024) with
// wavefront shuffles; there the step is taken as y_j = s - 2 x_j (the matrix J - 2I, which is
// the printed matrix with its columns reversed) and the flip is applied once, for free, to the
// lane's output address.  The 1/sqrt(g) = 2^-k normalisation is folded into the scale.
//
// Quantiser.  a = 2^-k max|z| (exact), s = a / 7 (IEEE division), r = 2^-k / s (IEEE division),
// q = rne(z * r) taken by one fused multiply-add against 1.5 * 2^23, whose low mantissa bits are
// then the two's-complement code.  |z r| <= 7 (1 + 2^-22), so no clamp is needed.  Rows whose
// scale is a short dyadic number divide exactly instead (see the comment at the code).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "convrot_internal.h"

namespace convrot {

namespace {

constexpr int kUnit = 16;  // elements per unit

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

template <int CTRL>
__device__ __forceinline__ float dpp_f32(float x)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, false));
}

// s - 2 x with s the sum over the four lanes that differ in one base-4 digit of the lane id.
template <int CTRL_A, int CTRL_B>
__device__ __forceinline__ float radix4_lanes_dpp(float x)
{
    float t = x + dpp_f32<CTRL_A>(x);
    float s = t + dpp_f32<CTRL_B>(t);
    return fmaf(-2.0f, x, s);
}

__device__ __forceinline__ float radix4_lanes_shfl(float x, int m1, int m2)
{
    float t = x + __shfl_xor(x, m1, 64);
    float s = t + __shfl_xor(t, m2, 64);
    return fmaf(-2.0f, x, s);
}

// Printed H_4 on four registers: y_j = s - 2 x_{3-j}.
__device__ __forceinline__ void radix4_regs(float &a, float &b, float &c, float &d)
{
    float s = (a + b) + (c + d);
    float na = fmaf(-2.0f, d, s);
    float nb = fmaf(-2.0f, c, s);
    float nc = fmaf(-2.0f, b, s);
    float nd = fmaf(-2.0f, a, s);
    a = na; b = nb; c = nc; d = nd;
}

template <int G>
__device__ __forceinline__ void rotate_unit(float (&v)[kUnit])
{
#pragma unroll
    for (int q = 0; q < 4; ++q) radix4_regs(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
    if constexpr (G >= 16) {
#pragma unroll
        for (int e = 0; e < 4; ++e) radix4_regs(v[e], v[e + 4], v[e + 8], v[e + 12]);
    }
    if constexpr (G >= 64) {  // lanes l ^ 1, l ^ 2: quad_perm [1,0,3,2] then [2,3,0,1]
#pragma unroll
        for (int e = 0; e < kUnit; ++e) v[e] = radix4_lanes_dpp<0xB1, 0x4E>(v[e]);
    }
    if constexpr (G >= 256) {  // lanes l ^ 8, l ^ 4 inside a row of 16: row_ror:8 then row_ror:4
#pragma unroll
        for (int e = 0; e < kUnit; ++e) v[e] = radix4_lanes_dpp<0x128, 0x124>(v[e]);
    }
    if constexpr (G >= 1024) {
#pragma unroll
        for (int e = 0; e < kUnit; ++e) v[e] = radix4_lanes_shfl(v[e], 16, 32);
    }
}

template <int G>
constexpr int lane_flip_mask() { return G >= 1024 ? 63 : (G >= 256 ? 15 : (G >= 64 ? 3 : 0)); }

template <int G>
constexpr float group_norm() { return G == 4 ? 0.5f : G == 16 ? 0.25f : G == 64 ? 0.125f : G == 256 ? 0.0625f : 0.03125f; }

}  // namespace

// grid.x = ceil(rows / rows_per_block); block = rows_per_block * T threads, T = 64 * waves_per_row.
template <int G, int U, int BLOCK>
__global__ __launch_bounds__(BLOCK) void rotquant_kernel(const uint16_t *__restrict__ X, int64_t rows, int K,
                                                         int T, uint8_t *__restrict__ Xq,
                                                         float *__restrict__ scale)
{
    __shared__ float s_part[BLOCK / 64];

    const int tid = threadIdx.x;
    const int rib = tid / T;               // row inside the block
    const int t = tid - rib * T;           // lane index inside the row
    const int rows_per_block = BLOCK / T;
    const int64_t row = (int64_t)blockIdx.x * rows_per_block + rib;
    const bool row_ok = row < rows;
    const int units = K / kUnit;

    float v[U][kUnit];
    float amax = 0.0f;

#pragma unroll
    for (int i = 0; i < U; ++i) {
        const int unit = i * T + t;
        u32x4 lo = {0, 0, 0, 0}, hi = {0, 0, 0, 0};
        if (row_ok && unit < units) {
            const u32x4 *p = reinterpret_cast<const u32x4 *>(X + row * (int64_t)K + (int64_t)unit * kUnit);
            lo = __builtin_nontemporal_load(p);
            hi = __builtin_nontemporal_load(p + 1);
        }
        const uint32_t w[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            v[i][2 * j] = __uint_as_float(w[j] << 16);
            v[i][2 * j + 1] = __uint_as_float(w[j] & 0xFFFF0000u);
        }
        rotate_unit<G>(v[i]);
#pragma unroll
        for (int e = 0; e < kUnit; ++e) amax = fmaxf(amax, fabsf(v[i][e]));
    }

    // row absmax: wavefront butterfly, then across the row's wavefronts through LDS
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) amax = fmaxf(amax, __shfl_xor(amax, m, 64));
    if (T > 64) {
        if ((tid & 63) == 0) s_part[tid >> 6] = amax;
        __syncthreads();
        const int w0 = (rib * T) >> 6;
        const int wv = T >> 6;
        float a = s_part[w0];
        for (int w = 1; w < wv; ++w) a = fmaxf(a, s_part[w0 + w]);
        amax = a;
    }

    const float norm = group_norm<G>();
    const float a = amax * norm;                       // exact: power-of-two scaling
    const float s = (a == 0.0f) ? 1.0f : a / 7.0f;     // IEEE division
    const float r = norm / s;                          // IEEE division
    if (row_ok && t == 0) scale[row] = s;

    // Codes.  Fast rows: one fma against 1.5 * 2^23 (ulp 1) rounds z * r to an integer, ties to even,
    // and leaves the two's-complement code in the low mantissa bits.  r carries a relative error of
    // 2^-24, which only matters when z / s is a half-integer to within ~1e-6.  On bf16-grid inputs
    // that happens in bulk in exactly one situation: the row's absmax is a short multiple of 7, so
    // that s itself is a short dyadic number and z = (n + 1/2) s is hit exactly.  Such rows (s has
    // >= 8 trailing zero mantissa bits) take the correctly rounded division instead, which returns
    // n + 1/2 exactly and lets the rounding see the tie.
    constexpr float kMagic = 12582912.0f;
    const bool short_scale = (__float_as_uint(s) & 0xFFu) == 0u;   // uniform over the row
    const float su = s / norm;                                      // scale in un-normalised units (exact)
    const int tf = t ^ lane_flip_mask<G>();
#pragma unroll
    for (int i = 0; i < U; ++i) {
        uint32_t d0 = 0, d1 = 0;
        if (short_scale) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                d0 |= ((uint32_t)(int)rintf(v[i][e] / su) & 0xFu) << (4 * e);
                d1 |= ((uint32_t)(int)rintf(v[i][e + 8] / su) & 0xFu) << (4 * e);
            }
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                d0 |= (__float_as_uint(fmaf(v[i][e], r, kMagic)) & 0xFu) << (4 * e);
                d1 |= (__float_as_uint(fmaf(v[i][e + 8], r, kMagic)) & 0xFu) << (4 * e);
            }
        }
        const int unit = i * T + tf;
        if (row_ok && unit < units) {
            u32x2 *o = reinterpret_cast<u32x2 *>(Xq + row * (int64_t)(K / 2) + (int64_t)unit * (kUnit / 2));
            __builtin_nontemporal_store(u32x2{d0, d1}, o);
        }
    }
}

namespace {

template <int G, int U>
hipError_t launch_gu(const void *X, int64_t rows, int K, int waves_per_row, void *Xq, float *scale,
                     hipStream_t stream)
{
    const int T = 64 * waves_per_row;
    if (T <= 256) {
        const int rpb = 256 / T;
        const unsigned grid = (unsigned)((rows + rpb - 1) / rpb);
        hipLaunchKernelGGL((rotquant_kernel<G, U, 256>), dim3(grid), dim3(256), 0, stream,
                           (const uint16_t *)X, rows, K, T, (uint8_t *)Xq, scale);
    } else if (T <= 512) {
        hipLaunchKernelGGL((rotquant_kernel<G, U, 512>), dim3((unsigned)rows), dim3(512), 0, stream,
                           (const uint16_t *)X, rows, K, 512, (uint8_t *)Xq, scale);
    } else {
        hipLaunchKernelGGL((rotquant_kernel<G, U, 1024>), dim3((unsigned)rows), dim3(1024), 0, stream,
                           (const uint16_t *)X, rows, K, 1024, (uint8_t *)Xq, scale);
    }
    return hipGetLastError();
}

template <int G>
hipError_t launch_g(const void *X, int64_t rows, int K, void *Xq, float *scale, hipStream_t stream)
{
    // Pick the wavefronts per row (1, 2, 4, 8 or 16) so that every lane holds at most 4 units,
    // preferring 3-4 units per lane (enough bytes in flight per wavefront, registers under 128).
    const int chunks = (K / kUnit + 63) / 64;  // 1024-element spans per row
    int wv = 1;
    while (wv < 16 && (chunks + wv - 1) / wv > 4) wv *= 2;
    const int u = (chunks + wv - 1) / wv;
    switch (u) {
        case 1: return launch_gu<G, 1>(X, rows, K, wv, Xq, scale, stream);
        case 2: return launch_gu<G, 2>(X, rows, K, wv, Xq, scale, stream);
        case 3: return launch_gu<G, 3>(X, rows, K, wv, Xq, scale, stream);
        default: return launch_gu<G, 4>(X, rows, K, wv, Xq, scale, stream);
    }
}

}  // namespace

hipError_t launch_rotquant(const void *X, int64_t rows, int64_t K, int group, void *Xq, float *scale,
                           hipStream_t stream)
{
    if (rows == 0) return hipSuccess;
    switch (group) {
        case 4: return launch_g<4>(X, rows, (int)K, Xq, scale, stream);
        case 16: return launch_g<16>(X, rows, (int)K, Xq, scale, stream);
        case 64: return launch_g<64>(X, rows, (int)K, Xq, scale, stream);
        case 256: return launch_g<256>(X, rows, (int)K, Xq, scale, stream);
        case 1024: return launch_g<1024>(X, rows, (int)K, Xq, scale, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace convrot
