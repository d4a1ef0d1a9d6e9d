// Kernel B of libconvrot: W4A4 GEMM on packed 4-bit codes with the dequantisation fused
// (ConvRot paper Sec. 4.3: 4-bit matrix multiplication, then dequantisation).
//
//   acc[m,n] = sum_k q_x[m,k] q_w[n,k]        int32, exact
//   Y[m,n]   = bf16( float(acc) * s_x[m] * s_w[n] )
//
// gfx950 has no 4-bit integer MFMA, so the codes are widened on chip to int8 and fed to
// v_mfma_i32_32x32x32_i8.  Widening keeps each nibble in the top half of its byte:
//     hi = p & 0xF0F0F0F0            (codes 1,3,5,7 of a dword, each as 16*code)
//     lo = (p << 4) & 0xF0F0F0F0     (codes 0,2,4,6, each as 16*code)
// which needs no sign extension.  Both operands are widened the same way, so byte i of one
// always meets byte i of the other (a dot product does not care in which order k is visited)
// and every product is 256 * q_x * q_w.  The accumulator is therefore exactly 256 * acc
// (|256 acc| <= 256 * 49 * K < 2^31 for K <= 65536) and the factor 2^-8 is folded, exactly,
// into the epilogue.
//
// The MFMA's row operand is the W tile and its column operand the X tile, so that a lane ends up
// with four consecutive n for one m and the bf16 output is written in 8-byte pieces.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "convrot_internal.h"

namespace convrot {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kStageBytes = 64;   // packed bytes of K per row per LDS stage (128 codes)
constexpr int kLdsStride = 80;    // row pitch in LDS: 64 + 16 bytes of padding (bank spread for b128 reads)
constexpr int kNumXcd = 8;

__device__ __forceinline__ uint32_t nib_lo(uint32_t p) { return (p << 4) & 0xF0F0F0F0u; }
__device__ __forceinline__ uint32_t nib_hi(uint32_t p) { return p & 0xF0F0F0F0u; }

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Tile order: blocks are dealt round-robin to the 8 XCDs by the hardware, each XCD has its own
// L2.  Give every XCD one contiguous range of logical tile ids, and walk that range in bands of
// `GM` tile rows so that tiles that run together share X and W panels.
__device__ __forceinline__ bool tile_of_block(int bid, int tiles_m, int tiles_n, int &tm, int &tn)
{
    const int ntiles = tiles_m * tiles_n;
    const int per_xcd = (ntiles + kNumXcd - 1) / kNumXcd;
    const int id = (bid % kNumXcd) * per_xcd + bid / kNumXcd;
    if (id >= ntiles) return false;
    constexpr int GM = 6;
    const int band = id / (GM * tiles_n);
    const int first_m = band * GM;
    const int rows_in_band = min(GM, tiles_m - first_m);
    const int local = id - band * GM * tiles_n;
    tm = first_m + local % rows_in_band;
    tn = local / rows_in_band;
    return true;
}

}  // namespace

template <int BM, int BN, int WGM, int WGN, bool RAW>
__global__ __launch_bounds__(WGM *WGN * 64) void gemm_w4a4_kernel(
    const uint8_t *__restrict__ Xq, const float *__restrict__ x_scale, const uint8_t *__restrict__ Wq,
    const float *__restrict__ w_scale, int M, int N, int K, uint16_t *__restrict__ Y,
    int32_t *__restrict__ acc_out, int tiles_m, int tiles_n)
{
    constexpr int NT = WGM * WGN * 64;
    constexpr int WTM = BM / WGM, WTN = BN / WGN;  // wavefront tile
    constexpr int FM = WTM / 32, FN = WTN / 32;    // 32x32 MFMA tiles per wavefront
    constexpr int XP = BM * 4 / NT, WP = BN * 4 / NT;  // 16-byte pieces per thread per stage
    static_assert(BM * 4 % NT == 0 && BN * 4 % NT == 0, "tile/threads mismatch");

    constexpr int kBufBytes = (BM + BN) * kLdsStride;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds_raw[];
    uint8_t(*lds)[kBufBytes] = reinterpret_cast<uint8_t(*)[kBufBytes]>(lds_raw);

    int tm, tn;
    if (!tile_of_block(blockIdx.x, tiles_m, tiles_n, tm, tn)) return;
    const int m0 = tm * BM, n0 = tn * BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave % WGM) * WTM, wn0 = (wave / WGM) * WTN;
    const int Kb = K >> 1;  // packed bytes per row
    const int KT = (Kb + kStageBytes - 1) / kStageBytes;  // the last stage may be partial: zero-filled

    // global -> register staging addresses (rows past the edge re-read the last valid row)
    const uint8_t *xg[XP];
    const uint8_t *wg[WP];
    int xl[XP], wl[WP];
#pragma unroll
    for (int i = 0; i < XP; ++i) {
        const int p = tid + NT * i, r = p >> 2, c = p & 3;
        xg[i] = Xq + (int64_t)min(m0 + r, M - 1) * Kb + c * 16;
        xl[i] = r * kLdsStride + c * 16;
    }
#pragma unroll
    for (int i = 0; i < WP; ++i) {
        const int p = tid + NT * i, r = p >> 2, c = p & 3;
        wg[i] = Wq + (int64_t)min(n0 + r, N - 1) * Kb + c * 16;
        wl[i] = (BM + r) * kLdsStride + c * 16;
    }

    uint4 xr[XP], wr[WP];
    const int piece_col = (tid & 3) * 16;  // NT is a multiple of 4: every piece of a thread has the same column
    auto load_stage = [&](int kt) {
        const int koff = kt * kStageBytes;
        const bool in_row = koff + piece_col < Kb;  // zero codes past the end of K add nothing
#pragma unroll
        for (int i = 0; i < XP; ++i)
            xr[i] = in_row ? *reinterpret_cast<const uint4 *>(xg[i] + koff) : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < WP; ++i)
            wr[i] = in_row ? *reinterpret_cast<const uint4 *>(wg[i] + koff) : make_uint4(0, 0, 0, 0);
    };
    auto store_stage = [&](int buf) {
#pragma unroll
        for (int i = 0; i < XP; ++i) *reinterpret_cast<uint4 *>(&lds[buf][xl[i]]) = xr[i];
#pragma unroll
        for (int i = 0; i < WP; ++i) *reinterpret_cast<uint4 *>(&lds[buf][wl[i]]) = wr[i];
    };

    v16i acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    const int frag_row = lane & 31;
    const int frag_kb = (lane >> 5) * 16;

    load_stage(0);
    store_stage(0);
    __syncthreads();

    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < KT) load_stage(kt + 1);

#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            v4i xop[FM][2], wop[FN][2];
#pragma unroll
            for (int i = 0; i < FM; ++i) {
                const uint4 p = *reinterpret_cast<const uint4 *>(
                    &lds[buf][(wm0 + i * 32 + frag_row) * kLdsStride + ks * 32 + frag_kb]);
                xop[i][0] = v4i{(int)nib_lo(p.x), (int)nib_hi(p.x), (int)nib_lo(p.y), (int)nib_hi(p.y)};
                xop[i][1] = v4i{(int)nib_lo(p.z), (int)nib_hi(p.z), (int)nib_lo(p.w), (int)nib_hi(p.w)};
            }
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                const uint4 p = *reinterpret_cast<const uint4 *>(
                    &lds[buf][(BM + wn0 + j * 32 + frag_row) * kLdsStride + ks * 32 + frag_kb]);
                wop[j][0] = v4i{(int)nib_lo(p.x), (int)nib_hi(p.x), (int)nib_lo(p.y), (int)nib_hi(p.y)};
                wop[j][1] = v4i{(int)nib_lo(p.z), (int)nib_hi(p.z), (int)nib_lo(p.w), (int)nib_hi(p.w)};
            }
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int i = 0; i < FM; ++i)
#pragma unroll
                    for (int j = 0; j < FN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wop[j][h], xop[i][h], acc[i][j], 0, 0, 0);
        }

        if (kt + 1 < KT) store_stage(buf ^ 1);
        __syncthreads();
    }

    // Epilogue.  Lane l, register r of a 32x32 tile: m = l % 32, n = 8 (r/4) + 4 (l/32) + r % 4.
    const bool vec_ok = RAW ? ((N & 3) == 0) : ((N & 3) == 0);
#pragma unroll
    for (int i = 0; i < FM; ++i) {
        const int m = m0 + wm0 + i * 32 + (lane & 31);
        if (m >= M) continue;
        float sxm = 0.0f;
        if constexpr (!RAW) sxm = x_scale[m] * 0.00390625f;  // 2^-8 undoes the 16*16 of the widening
#pragma unroll
        for (int j = 0; j < FN; ++j) {
#pragma unroll
            for (int rb = 0; rb < 4; ++rb) {
                const int n = n0 + wn0 + j * 32 + rb * 8 + (lane >> 5) * 4;
                if (n >= N) continue;
                if constexpr (RAW) {
                    int32_t o[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = acc[i][j][rb * 4 + e] >> 8;
                    int32_t *dst = acc_out + (int64_t)m * N + n;
                    if (vec_ok) {
                        *reinterpret_cast<int4 *>(dst) = make_int4(o[0], o[1], o[2], o[3]);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (n + e < N) dst[e] = o[e];
                    }
                } else {
                    uint16_t o[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float swn = (n + e < N) ? w_scale[n + e] : 0.0f;
                        o[e] = f32_to_bf16_rne(((float)acc[i][j][rb * 4 + e] * sxm) * swn);
                    }
                    uint16_t *dst = Y + (int64_t)m * N + n;
                    if (vec_ok) {
                        *reinterpret_cast<uint2 *>(dst) =
                            make_uint2((uint32_t)o[0] | ((uint32_t)o[1] << 16), (uint32_t)o[2] | ((uint32_t)o[3] << 16));
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (n + e < N) dst[e] = o[e];
                    }
                }
            }
        }
    }
}

namespace {

template <int BM, int BN, int WGM, int WGN>
hipError_t launch_tile(const void *Xq, const float *x_scale, const void *Wq, const float *w_scale, int M, int N,
                       int K, void *Y, int32_t *acc, hipStream_t stream)
{
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const int ntiles = tiles_m * tiles_n;
    const int grid = ((ntiles + kNumXcd - 1) / kNumXcd) * kNumXcd;
    const dim3 block(WGM * WGN * 64);
    constexpr int lds_bytes = 2 * (BM + BN) * kLdsStride;
    static bool attr_done = false;  // raising the dynamic-LDS limit is idempotent; a race only repeats it
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_w4a4_kernel<BM, BN, WGM, WGN, true>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_w4a4_kernel<BM, BN, WGM, WGN, false>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    if (acc) {
        hipLaunchKernelGGL((gemm_w4a4_kernel<BM, BN, WGM, WGN, true>), dim3(grid), block, lds_bytes, stream,
                           (const uint8_t *)Xq, x_scale, (const uint8_t *)Wq, w_scale, M, N, K, (uint16_t *)nullptr,
                           acc, tiles_m, tiles_n);
    } else {
        hipLaunchKernelGGL((gemm_w4a4_kernel<BM, BN, WGM, WGN, false>), dim3(grid), block, lds_bytes, stream,
                           (const uint8_t *)Xq, x_scale, (const uint8_t *)Wq, w_scale, M, N, K, (uint16_t *)Y,
                           (int32_t *)nullptr, tiles_m, tiles_n);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_w4a4(const void *Xq, const float *x_scale, const void *Wq, const float *w_scale,
                            int64_t M, int64_t N, int64_t K, void *Y_bf16, int32_t *acc_i32,
                            hipStream_t stream)
{
    if (M == 0 || N == 0) return hipSuccess;
    return launch_tile<256, 256, 2, 2>(Xq, x_scale, Wq, w_scale, (int)M, (int)N, (int)K, Y_bf16, acc_i32, stream);
}

}  // namespace convrot
