// W8A8 variant of kernel B of libconvrot (the paper's W8A8 rows, Sec. 5, Tables 5-2 and 5-4): the same
// layer with 8-bit codes on both operands,
//
//   acc[m,n] = sum_k q_x[m,k] q_w[n,k]        int8 codes in [-127, 127], int32 accumulate, exact
//   Y[m,n]   = bf16( float(acc) * s_x[m] * s_w[n] + bias[n] )
//
// Same shape as the 4-bit kernel in gemm_w4a4.hip (2 x 2 wavefronts per block, two blocks per compute
// unit, LDS-direct loads into a swizzled ring, one memory instruction per MFMA slot, X fragment
// stationary, scales and bias parked in LDS, LDS-transposed bf16 epilogue), with a ring of 3 stages of
// 64 codes of K: a 16-byte fragment read from LDS is an operand of v_mfma_i32_32x32x32_i8 as it stands.
// Two block tiles of 384 rows per stage are compiled, 192 x 192 (3 x 3 accumulator tiles per wavefront)
// and 256 x 128 (4 x 2): the square one moves fewer operand bytes per product, the other one has 11 %
// less work per block, which wins when the grid is a round or two of the chip; the launcher picks by
// the block count of the busiest compute unit.  A stage is 64 bytes = 64 codes of K per
// row, i.e. two MFMAs per accumulator tile; the panel layout of the operands (panel_layout.h) pads the
// last stage with zero codes.  |acc| <= 127^2 K < 2^31 for K <= 65536.
#include "gemm_common.h"

#include "convrot_internal.h"
#include "panel_layout.h"

namespace convrot {

using gemm::kNumXcd;
using gemm::kRowBytes;
using gemm::kSubSteps;
using gemm::lds_dma16;
using gemm::pack_bf16x2;
using gemm::swz;
using gemm::tile_of_block;
using gemm::v16i;
using gemm::v4i;
using gemm::wait_vmcnt;

namespace {

constexpr int kThreads = 256;                 // 4 wavefronts, 2 x 2
constexpr int kTileRows = 384;                // X rows + W rows of a block tile
constexpr int kStages = 3;
constexpr int kStageBytes = kTileRows * kRowBytes;        // 24 KB
constexpr int kRingBytes = kStages * kStageBytes;         // 72 KB
constexpr int kChunks = kStageBytes / 1024 / 4;           // 1 KB LDS-direct loads per wavefront per stage: 6

// Derived constants of a block tile TM x TN (TM + TN = 384, multiples of 64).
template <int TM_, int TN_>
struct Tile {
    static constexpr int TM = TM_, TN = TN_;
    static constexpr int WM = TM / 2, WN = TN / 2;            // wavefront tile
    static constexpr int XF = WM / 32, WF = WN / 32;          // fragments (32 rows x one K32 step) per wavefront
    static constexpr int NF = XF + WF;
    static constexpr int kMfmas = XF * WF;                    // per K32 step
    static constexpr int kXChunks = TM * kRowBytes / 1024 / 4;   // the first of a wavefront's chunks fetch X rows
    static constexpr int kEpiPitch = WN * 2 + 16;             // bf16 row of the wavefront tile + pad
    static constexpr int kLdsTotal = kRingBytes + (TM + 2 * TN) * 4;   // + the tile's dequantisation scales and bias
    static constexpr int kBandRows = TM == TN ? 8 : 6;        // tile rows per band of the tile order
    static_assert(TM + TN == kTileRows && TM % 64 == 0 && TN % 64 == 0, "tile shape");
    static_assert(kXChunks * 4 * 16 == TM, "X rows must fill whole chunks of all four wavefronts");
    static_assert(4 * 32 * kEpiPitch <= kRingBytes, "epilogue staging must fit the ring");
    static_assert(2 * kLdsTotal <= 160 * 1024, "two blocks per compute unit");
    static_assert(NF == 6 && kMfmas >= 8 && kMfmas <= 9, "slot plan of a step");
};
static_assert(kChunks * 4 * 1024 == kStageBytes && kChunks == 6 && kSubSteps == 2, "slot plan of a step");

}  // namespace

template <bool RAW, class T>
__global__ __launch_bounds__(kThreads, 2) void gemm_w8a8_kernel(
    const uint8_t *__restrict__ Xq, const float *__restrict__ x_scale, const uint8_t *__restrict__ Wq,
    const float *__restrict__ w_scale, const uint16_t *__restrict__ bias, int M, int N, int K,
    uint16_t *__restrict__ Y,
    int32_t *__restrict__ acc_out, int tiles_m, int tiles_n)
{
    // Statically sized: above 64 KB a dynamic allocation would need a per-device function attribute set
    // from the host before the first launch, i.e. hidden library state; a static one needs nothing.
    __shared__ __attribute__((aligned(1024))) uint8_t lds[T::kLdsTotal];
    constexpr int TM = T::TM, TN = T::TN, WM = T::WM, WN = T::WN, XF = T::XF, WF = T::WF, NF = T::NF;
    constexpr int kMfmas = T::kMfmas, kXChunks = T::kXChunks, kEpiPitch = T::kEpiPitch, kBandRows = T::kBandRows;

    int tm, tn;
    if (!tile_of_block<kBandRows>(blockIdx.x, tiles_m, tiles_n, tm, tn)) return;
    const int m0 = tm * TM, n0 = tn * TN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave & 1) * WM, wn0 = (wave >> 1) * WN;
    const int KT = (int)panel::k_panels(K);   // stages = K-panels per row; the last one is zero-padded

    // ---- dequantisation scales of the tile's rows and columns: thread t fetches x_scale[m0 + t] and
    // w_scale[n0 + t] now, so that the latency hides under the main loop, and parks them in LDS (past
    // the ring) once the loop is over.
    float my_sx = 0.0f, my_sw = 0.0f, my_b = 0.0f;
    if constexpr (!RAW) {
        if (tid < TM && m0 + tid < M) my_sx = x_scale[m0 + tid];
        if (tid < TN && n0 + tid < N) {
            my_sw = w_scale[n0 + tid];
            if (bias) my_b = gemm::bf16_to_f32(bias[n0 + tid]);
        }
    }

    // ---- global -> LDS (direct): wavefront w fills chunks w, w+4, ... of every stage; chunk c holds
    // tile rows 16c .. 16c+15 (rows 0..TM-1 are X, the rest W), which is one 1 KB panel of the operand
    // (panel_layout.h), K-panels of the same rows 1 KB apart; lane l fills slot l & 3 of row l >> 2.
    const uint8_t *xtile = Xq + (int64_t)(m0 / panel::kRows) * KT * panel::kBytes;
    const uint8_t *wtile = Wq + (int64_t)(n0 / panel::kRows) * KT * panel::kBytes;
    uint32_t goff[kChunks];   // byte offset of this lane's piece inside the operand's tile rows, stage 0
#pragma unroll
    for (int i = 0; i < kChunks; ++i) {
        const int row_t = 16 * (wave + 4 * i) + lane / 4;
        const int piece = (lane % 4) ^ swz(row_t);
        const int r = i < kXChunks ? min(row_t, M - 1 - m0) : min(row_t - TM, N - 1 - n0);   // edge rows re-read the last valid row
        goff[i] = (uint32_t)(r / panel::kRows) * (uint32_t)KT * panel::kBytes + (r % panel::kRows) * kRowBytes + piece * 16;
    }
    // LDS-direct loads are issued from inline assembly so that the compiler does not serialise every
    // later LDS read behind them; completion is tracked by hand with vmcnt.
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)lds;
    const uint32_t wave_lds = lds_base + __builtin_amdgcn_readfirstlane(wave) * 1024;
    // chunk i of this wavefront's share of stage kt; chunk wave + 4 i sits 4096 i further on
    auto load_chunk = [&](int kt, int i) {
        const uint32_t sl = wave_lds + ((unsigned)kt % kStages) * kStageBytes;
        lds_dma16((i < kXChunks ? xtile : wtile) + (uint32_t)kt * panel::kBytes, goff[i], sl + i * 4096);
    };

    // ---- LDS -> registers: fragment of 32 rows x 32 packed codes per lane-half
    const int frow = lane & 31;
    const int fswz = swz(frow);                              // tile rows differ from frow by multiples of 32
    int foff[kSubSteps];                                     // per K64 step: byte offset inside a 32-row slab
#pragma unroll
    for (int ks = 0; ks < kSubSteps; ++ks) foff[ks] = frow * kRowBytes + (((2 * ks + (lane >> 5)) ^ fswz) << 4);
    const int xslab = wm0 * kRowBytes;
    const int wslab = (TM + wn0) * kRowBytes;

    // fragment f of step ks (32 codes of K) of stage kt: 0..XF-1 X rows 32 f .., then W rows 32 (f - XF) ..
    v4i cur[NF], nxt[NF];
    auto read_frag = [&](v4i (&dst)[NF], int kt, int ks, auto F) {
        constexpr int f = decltype(F)::value;
        const uint8_t *sbase = lds + ((unsigned)kt % kStages) * kStageBytes + foff[ks];
        if constexpr (f < XF) dst[f] = *reinterpret_cast<const v4i *>(sbase + xslab + f * 32 * kRowBytes);
        else dst[f] = *reinterpret_cast<const v4i *>(sbase + wslab + (f - XF) * 32 * kRowBytes);
    };

    v16i acc[XF][WF];
#pragma unroll
    for (int i = 0; i < XF; ++i)
#pragma unroll
        for (int j = 0; j < WF; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    // One step = XF * WF MFMAs (one per accumulator tile) on the fragments in `cur`, slot by slot, in issue
    // order (scheduling barriers pin it): slot m runs MFMA (i = m / WF, j = m % WF), the X fragment
    // staying for WF MFMAs in a row; m < 6 fetches
    // fragment m of the next step (stage nkt, step nks) into `nxt`; with REFILL slots 2..7 also issue
    // the LDS-direct loads of stage rkt.  With SYNC the step opens with the wait for stage nkt (with a
    // ring of three only that stage is in flight) and the block barrier.
    auto step = [&](auto SYNC, auto REFILL, int nkt, int nks, int rkt) {
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (decltype(SYNC)::value) {
            wait_vmcnt<0>();
            __syncthreads();
            __builtin_amdgcn_sched_barrier(0);
        }
        auto slot = [&](auto MI) {
            constexpr int m = decltype(MI)::value, i = m / WF, j = m % WF;
            if constexpr (m < kMfmas) {
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(cur[XF + j], cur[i], acc[i][j], 0, 0, 0);
                if constexpr (m < NF) read_frag(nxt, nkt, nks, std::integral_constant<int, m>{});
                if constexpr (decltype(REFILL)::value && m >= 2 && m - 2 < kChunks) load_chunk(rkt, m - 2);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        slot(std::integral_constant<int, 0>{}); slot(std::integral_constant<int, 1>{});
        slot(std::integral_constant<int, 2>{}); slot(std::integral_constant<int, 3>{});
        slot(std::integral_constant<int, 4>{}); slot(std::integral_constant<int, 5>{});
        slot(std::integral_constant<int, 6>{}); slot(std::integral_constant<int, 7>{});
        slot(std::integral_constant<int, 8>{});
#pragma unroll
        for (int f = 0; f < NF; ++f) cur[f] = nxt[f];   // a renaming
    };

    // ---- pipeline: stages 0 and 1 in flight; when stage 0 has landed its first fragments are fetched.
    // The block meets once per stage, at the start of the stage's second step: stage kt+1 must have
    // landed by then (its first fragments are fetched during that step), and the buffer stage kt-1
    // vacated is refilled with stage kt+2.  The last two stages refill nothing (what they fetch past
    // the last stage is a ring buffer whose contents are unused).
#pragma unroll
    for (int i = 0; i < kChunks; ++i) load_chunk(0, i);
    if (KT > 1) {
#pragma unroll
        for (int i = 0; i < kChunks; ++i) load_chunk(1, i);
        wait_vmcnt<kChunks>();
    } else {
        wait_vmcnt<0>();
    }
    __syncthreads();
#define CONVROT_F(f) read_frag(cur, 0, 0, std::integral_constant<int, f>{});
    CONVROT_F(0) CONVROT_F(1) CONVROT_F(2) CONVROT_F(3) CONVROT_F(4) CONVROT_F(5)
#undef CONVROT_F

    int kt = 0;
    for (; kt < KT - 2; ++kt) {
        step(std::false_type{}, std::false_type{}, kt, 1, 0);
        step(std::true_type{}, std::true_type{}, kt + 1, 0, kt + 2);
    }
    for (; kt < KT; ++kt) {
        step(std::false_type{}, std::false_type{}, kt, 1, 0);
        step(std::true_type{}, std::false_type{}, kt + 1, 0, 0);
    }

    // ---- epilogue.  Lane l, register r of a 32x32 accumulator tile: m = l % 32, n = 8 (r/4) + 4 (l/32) + r % 4.
    if constexpr (RAW) {
        const bool vec_ok = (N & 3) == 0;
#pragma unroll
        for (int i = 0; i < XF; ++i) {
            const int m = m0 + wm0 + i * 32 + (lane & 31);
            if (m >= M) continue;
#pragma unroll
            for (int j = 0; j < WF; ++j) {
#pragma unroll
                for (int rb = 0; rb < 4; ++rb) {
                    const int n = n0 + wn0 + j * 32 + rb * 8 + (lane >> 5) * 4;
                    if (n >= N) continue;
                    int32_t o[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = acc[i][j][rb * 4 + e];
                    int32_t *dst = acc_out + (int64_t)m * N + n;
                    if (vec_ok) {
                        *reinterpret_cast<int4 *>(dst) = make_int4(o[0], o[1], o[2], o[3]);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (n + e < N) dst[e] = o[e];
                    }
                }
            }
        }
    } else {
        float *sx_lds = reinterpret_cast<float *>(lds + kRingBytes), *sw_lds = sx_lds + TM;
        if (tid < TM) sx_lds[tid] = my_sx;
        if (tid < TN) {
            sw_lds[tid] = my_sw;
            sw_lds[TN + tid] = my_b;
        }
        __syncthreads();     // every wavefront has finished reading the ring; the scales are visible
        // `interior`: the tile lies wholly inside Y and rows of Y are 16-byte multiples, so the stores need
        // no bounds checks (uniform over the block).
        const bool interior = m0 + TM <= M && n0 + TN <= N && (N & 7) == 0;
        float sxm[XF];
#pragma unroll
        for (int i = 0; i < XF; ++i) sxm[i] = sx_lds[wm0 + i * 32 + (lane & 31)];
        uint8_t *stage = lds + wave * (32 * kEpiPitch);          // this wavefront's 32 x WN bf16 staging tile
        // read-back: the 32 rows of WN bf16 are 32 * WN / 8 pieces of 16 bytes, dealt to the 64 lanes in order
        // (piece p = 64 pass + lane: row p / (WN / 8), columns 8 (p % (WN / 8)) ...), so every pass has all
        // lanes at work and stores whole rows of the wavefront tile back to back
        constexpr int kRowPieces = WN / 8, kRbPasses = 32 * kRowPieces / 64;
        static_assert(kRbPasses * 64 == 32 * kRowPieces, "read-back passes");
        const int rb_row0 = lane / kRowPieces, rb_piece0 = lane % kRowPieces;   // pass 0; 64 more pieces per pass
        // the column scales of the lane's accumulator registers, fetched once for all XF row blocks
        float4 swv[WF][4];
#pragma unroll
        for (int j = 0; j < WF; ++j)
#pragma unroll
            for (int rb = 0; rb < 4; ++rb)
                swv[j][rb] = *reinterpret_cast<const float4 *>(sw_lds + wn0 + j * 32 + rb * 8 + (lane >> 5) * 4);
        auto body = [&](auto INTERIOR, auto BIAS) {
#pragma unroll
            for (int i = 0; i < XF; ++i) {
                const int mrow = m0 + wm0 + i * 32;
#pragma unroll
                for (int j = 0; j < WF; ++j)
#pragma unroll
                    for (int rb = 0; rb < 4; ++rb) {
                        const int col = j * 32 + rb * 8 + (lane >> 5) * 4;
                        const float4 sw = swv[j][rb];
                        float y[4] = {((float)acc[i][j][rb * 4 + 0] * sxm[i]) * sw.x, ((float)acc[i][j][rb * 4 + 1] * sxm[i]) * sw.y,
                                      ((float)acc[i][j][rb * 4 + 2] * sxm[i]) * sw.z, ((float)acc[i][j][rb * 4 + 3] * sxm[i]) * sw.w};
                        if constexpr (decltype(BIAS)::value) {
                            const float4 b = *reinterpret_cast<const float4 *>(sw_lds + TN + wn0 + col);
                            y[0] += b.x; y[1] += b.y; y[2] += b.z; y[3] += b.w;
                        }
                        *reinterpret_cast<uint2 *>(stage + (lane & 31) * kEpiPitch + col * 2) =
                            make_uint2(pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3]));
                    }
                // the same wavefront reads back row-contiguous
#pragma unroll
                for (int it = 0; it < kRbPasses; ++it) {
                    int piece = rb_piece0 + (it * 64) % kRowPieces, r = rb_row0 + (it * 64) / kRowPieces;
                    if ((it * 64) % kRowPieces != 0 && piece >= kRowPieces) { piece -= kRowPieces; ++r; }
                    const uint4 v = *reinterpret_cast<const uint4 *>(stage + r * kEpiPitch + piece * 16);
                    const int mo = mrow + r, ncol = n0 + wn0 + piece * 8;
                    uint16_t *dst = Y + (int64_t)mo * N + ncol;
                    if constexpr (decltype(INTERIOR)::value) {
                        *reinterpret_cast<uint4 *>(dst) = v;
                    } else {
                        if (mo >= M || ncol >= N) continue;
                        if ((N & 7) == 0) {
                            *reinterpret_cast<uint4 *>(dst) = v;
                        } else {
                            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                            for (int e = 0; e < 8; ++e)
                                if (ncol + e < N) dst[e] = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
                        }
                    }
                }
            }
        };
        if (bias) {
            if (interior) body(std::true_type{}, std::true_type{});
            else body(std::false_type{}, std::true_type{});
        } else {
            if (interior) body(std::true_type{}, std::false_type{});
            else body(std::false_type{}, std::false_type{});
        }
    }
}

namespace {

template <bool RAW, class T>
hipError_t launch_tile(const void *Xq, const float *x_scale, const void *Wq, const float *w_scale, const void *bias,
                       int M, int N, int K, void *Y, int32_t *acc, hipStream_t stream)
{
    const int tiles_m = (M + T::TM - 1) / T::TM, tiles_n = (N + T::TN - 1) / T::TN;
    if ((int64_t)tiles_m * tiles_n > (1 << 30)) return hipErrorInvalidValue;   // the kernel counts tiles in 32 bits
    const int ntiles = tiles_m * tiles_n;
    const int grid = ((ntiles + kNumXcd - 1) / kNumXcd) * kNumXcd;
    hipLaunchKernelGGL((gemm_w8a8_kernel<RAW, T>), dim3(grid), dim3(kThreads), 0, stream, (const uint8_t *)Xq,
                       x_scale, (const uint8_t *)Wq, w_scale, (const uint16_t *)bias, M, N, K, (uint16_t *)Y, acc, tiles_m,
                       tiles_n);
    return hipGetLastError();
}

template <bool RAW>
hipError_t launch_one(const void *Xq, const float *x_scale, const void *Wq, const float *w_scale, const void *bias,
                      int M, int N, int K, void *Y, int32_t *acc, hipStream_t stream)
{
    using Square = Tile<192, 192>;
    using Tall = Tile<256, 128>;
    if (gemm_tile_rows(M, N) == Square::TM)
        return launch_tile<RAW, Square>(Xq, x_scale, Wq, w_scale, bias, M, N, K, Y, acc, stream);
    return launch_tile<RAW, Tall>(Xq, x_scale, Wq, w_scale, bias, M, N, K, Y, acc, stream);
}

}  // namespace

hipError_t launch_gemm_w8a8(const void *Xq, const float *x_scale, const void *Wq, const float *w_scale,
                            const void *bias_bf16, int64_t M, int64_t N, int64_t K, void *Y_bf16,
                            int32_t *acc_i32, hipStream_t stream)
{
    if (M == 0 || N == 0) return hipSuccess;
    if (acc_i32)
        return launch_one<true>(Xq, x_scale, Wq, w_scale, nullptr, (int)M, (int)N, (int)K, nullptr, acc_i32, stream);
    return launch_one<false>(Xq, x_scale, Wq, w_scale, bias_bf16, (int)M, (int)N, (int)K, Y_bf16, nullptr, stream);
}

}  // namespace convrot
