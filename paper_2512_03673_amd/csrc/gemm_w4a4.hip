// Kernel B of libconvrot: W4A4 GEMM on 4-bit codes with the dequantisation fused
// (ConvRot paper Sec. 4.3: 4-bit matrix multiplication, then dequantisation).
//
//   acc[m,n] = sum_k q_x[m,k] q_w[n,k]        exact
//   Y[m,n]   = bf16( float(acc) * s_x[m] * s_w[n] + bias[n] )
//
// gfx950 has no 4-bit integer MFMA, but every code in [-7, 7] is an FP6 (E2M3) number, and
// v_mfma_f32_32x32x64_f8f6f4 on FP6 operands runs at twice the rate of the int8 MFMA.  Products of two
// codes (|.| <= 49) and all their partial sums (|.| <= 49 K < 2^22 for K <= 65536) are integers that
// fp32 holds exactly, so the fp32 accumulators carry the exact integer result whatever the order of
// the additions.  The codes arrive from the rotate+quantise kernel already as FP6 (e2m3_layout.h), six
// bits each, in the register image the MFMA wants: nothing is unpacked or widened here.  (On this
// chip the int8 path is held back by power, not by issue: the same int8 kernel ran 98 us on all-zero
// codes and 113-135 us on real ones, and a register-only loop sustains 2.7 POP/s of int8 MFMA against
// 6.6 POP/s of FP6 MFMA on workload-like data.)
//
// Data movement.  A block of 4 wavefronts (2 x 2) owns an output tile of 384 operand rows per K step,
// in one of two shapes.  192 x 192 (96 x 96 per wavefront: 3 x 3 accumulator tiles, 144 registers per
// lane, nine MFMAs on six fragments per K64 step) moves the fewest operand bytes per product; FLUX's
// layer widths and token counts are multiples of 192, and the headline shape is exactly three rounds of
// 512 such tiles.  256 x 128 (128 x 64 per wavefront: 4 x 2 accumulator tiles, eight MFMAs on six
// fragments) has 11 % less work per block, which wins when the grid is no more than a round or two of
// the chip; the launcher picks by the block count of the busiest compute unit (gemm_tile_rows).
// Either needs 74 KB of LDS, so that two blocks share a compute unit: while one runs
// its prologue or epilogue, or waits at a barrier, the other keeps the MFMA pipe busy.  The operands
// sit in HBM as 3 KB blocks of 32 rows x 128 codes (an A plane of 32 x 64 bytes and a B plane of
// 32 x 32 bytes, both XOR-swizzled for the fragment reads); a K128 stage of the tile is 12 such blocks
// = 36 global_load_lds_dwordx4 of one contiguous kilobyte each, nine per wavefront, straight copies
// into a ring of two stage buffers.  A fragment (32 rows x 64 codes, 24 bytes per lane) is one
// ds_read_b128 from the A plane and one ds_read_b64 from the B plane and is an MFMA operand as read.
//
// The MFMA's row operand is the W tile and its column operand the X tile, so that a lane ends up
// with four consecutive n for one m; the epilogue scales, rounds to bf16, transposes through LDS
// and writes 16 bytes per lane, whole contiguous rows of the wavefront's tile (192 or 128 bytes).
#include "gemm_common.h"

#include "convrot_internal.h"
#include "e2m3_layout.h"

namespace convrot {

using gemm::kNumXcd;
using gemm::lds_dma16;
using gemm::pack_bf16x2;
using gemm::tile_of_block;
using gemm::v4i;
using gemm::wait_vmcnt;
using gemm::wait_vmcnt_lgkm0;

namespace {

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;                 // 4 wavefronts, 2 x 2
constexpr int kTileRows = 384;                // X rows + W rows of a block tile
constexpr int kTileBlocks = kTileRows / e2m3::kRows;             // 32-row blocks of a stage: those of X, then those of W
constexpr int kAPlane = kTileRows * e2m3::kARowBytes;            // LDS stage: A parts, tile row r at r * 64 ... 24 KB
constexpr int kBPlane = kTileRows * e2m3::kBRowBytes;            // ... then B parts, tile row r at r * 32: 12 KB
constexpr int kStageBytes = kAPlane + kBPlane;                   // 36 KB
constexpr int kStages = 2;
constexpr int kRingBytes = kStages * kStageBytes;                // 72 KB
constexpr int kLoads = kStageBytes / 1024 / 4;                   // 1 KB LDS-direct loads per wavefront per stage: 9
static_assert(kLoads * 4 * 1024 == kStageBytes && kTileBlocks * 3 == kLoads * 4, "stage must split into 1 KB loads over 4 wavefronts");

// Derived constants of a block tile TM x TN (TM + TN = 384, multiples of 64).
template <int TM_, int TN_>
struct Tile {
    static constexpr int TM = TM_, TN = TN_;
    static constexpr int WM = TM / 2, WN = TN / 2;            // wavefront tile
    static constexpr int XF = WM / 32, WF = WN / 32;          // fragments (32 rows x one K64 step) per wavefront
    static constexpr int NF = XF + WF;
    static constexpr int kMfmas = XF * WF;                    // per K64 step
    static constexpr int kEpiPitch = WN * 2 + 16;             // bf16 row of the wavefront tile + pad
    static constexpr int kLdsTotal = kRingBytes + (TM + 2 * TN) * 4;   // + the tile's dequantisation scales and bias
    static constexpr int kBandRows = TM == TN ? 8 : 6;        // tile rows per band of the XCD-aware tile order
    static_assert(TM + TN == kTileRows && TM % 64 == 0 && TN % 64 == 0, "tile shape");
    static_assert(4 * 32 * kEpiPitch <= kRingBytes, "epilogue staging must fit the ring");
    static_assert(2 * kLdsTotal <= 160 * 1024, "two blocks per compute unit");
    static_assert(NF == 6 && kLoads == 9 && kMfmas >= 8 && kMfmas <= 9, "slot plan of a K64 step");
};

}  // namespace

template <bool RAW, class T>
__global__ __launch_bounds__(kThreads, 2) void gemm_w4a4_kernel(
    const uint8_t *__restrict__ Xq, const float *__restrict__ x_scale, const uint8_t *__restrict__ Wq,
    const float *__restrict__ w_scale, const uint16_t *__restrict__ bias, int M, int N, int K,
    uint16_t *__restrict__ Y,
    int32_t *__restrict__ acc_out, int tiles_m, int tiles_n)
{
    // Statically sized: above 64 KB a dynamic allocation would need a per-device function attribute set
    // from the host before the first launch, i.e. hidden library state; a static one needs nothing.
    __shared__ __attribute__((aligned(1024))) uint8_t lds[T::kLdsTotal];
    constexpr int TM = T::TM, TN = T::TN, WM = T::WM, WN = T::WN, XF = T::XF, WF = T::WF, NF = T::NF;
    constexpr int kMfmas = T::kMfmas, kEpiPitch = T::kEpiPitch, kBandRows = T::kBandRows;

    int tm, tn;
    if (!tile_of_block<kBandRows>(blockIdx.x, tiles_m, tiles_n, tm, tn)) return;
    const int m0 = tm * TM, n0 = tn * TN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave & 1) * WM, wn0 = (wave >> 1) * WN;
    const int KS = (int)e2m3::stages(K);   // K128 stages per row; the last one is zero-padded

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

    // ---- global -> LDS (direct).  Load j of a stage (0..35) copies kilobyte j % 3 of the 3 KB block of
    // 32-row group j / 3 of the tile (the first TM / 32 groups are X rows, the rest W rows): kilobytes 0, 1 are the A plane
    // (rows 0-15, 16-31), kilobyte 2 the B plane.  Wavefront w issues loads w, w + 4, ...; a group past
    // the operand's last one (edge tiles) re-reads the last one, whose results are never stored.
    const int x_groups = (M + e2m3::kRows - 1) / e2m3::kRows, w_groups = (N + e2m3::kRows - 1) / e2m3::kRows;
    const uint8_t *src[kLoads];   // stage 0 source of each of this wavefront's loads (wavefront-uniform)
    uint32_t dst[kLoads];         // its place in a stage buffer
#pragma unroll
    for (int i = 0; i < kLoads; ++i) {
        const int j = __builtin_amdgcn_readfirstlane(wave) + 4 * i, grp = j / 3, part = j % 3;
        const bool is_x = grp < TM / e2m3::kRows;
        const int g = is_x ? min(m0 / e2m3::kRows + grp, x_groups - 1) : min(n0 / e2m3::kRows + grp - TM / e2m3::kRows, w_groups - 1);
        src[i] = (is_x ? Xq : Wq) + (int64_t)g * KS * e2m3::kBlockBytes + part * 1024;
        dst[i] = part < 2 ? grp * e2m3::kAPlaneBytes + part * 1024 : kAPlane + grp * e2m3::kBPlaneBytes;
    }
    // LDS-direct loads are issued from inline assembly so that the compiler does not serialise every
    // later LDS read behind them; completion is tracked by hand with vmcnt.
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)lds;
    const uint32_t lane16 = lane * 16;
    auto load_stage_part = [&](int s, auto IC) {   // load i of this wavefront's share of stage s
        constexpr int i = decltype(IC)::value;
        lds_dma16(src[i], lane16 + (uint32_t)s * e2m3::kBlockBytes, lds_base + ((unsigned)s % kStages) * kStageBytes + dst[i]);
    };

    // ---- LDS -> registers: a fragment is 32 rows x one K64 step; lane l holds chunk 2 ks + l / 32 of row l % 32
    const int frow = lane & 31;
    int offa[2], offb[2];     // per K64 step: byte offsets of the lane's A part and B part inside a 32-row group
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
        const int c = 2 * ks + (lane >> 5);
        offa[ks] = frow * e2m3::kARowBytes + ((c ^ e2m3::swz_a(frow)) << 4);
        offb[ks] = kAPlane + frow * e2m3::kBRowBytes + ((c ^ e2m3::swz_b(frow)) << 3);
    }
    const int xrow0 = wm0, wrow0 = TM + wn0;   // first tile row of the wavefront's X and W fragments

    v8i op[2][NF];   // [K64 step parity][fragment]: 0..XF-1 X rows 32 f .., then W rows 32 (f - XF) ..; 6 dwords used
    auto read_frag = [&](int s, auto KSI, auto F) {
        constexpr int ks = decltype(KSI)::value, f = decltype(F)::value;
        const uint8_t *sbase = lds + ((unsigned)s % kStages) * kStageBytes;
        const int row0 = f < XF ? xrow0 + f * 32 : wrow0 + (f - XF) * 32;
        const v4i a = *reinterpret_cast<const v4i *>(sbase + offa[ks] + row0 * e2m3::kARowBytes);
        const v2i b = *reinterpret_cast<const v2i *>(sbase + offb[ks] + row0 * e2m3::kBRowBytes);
        v8i o = __builtin_shufflevector(a, a, 0, 1, 2, 3, -1, -1, -1, -1);
        o[4] = b.x;
        o[5] = b.y;
        op[ks][f] = o;
    };

    v16f acc[XF][WF];
#pragma unroll
    for (int i = 0; i < XF; ++i)
#pragma unroll
        for (int j = 0; j < WF; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // One K64 step, slot by slot, in issue order (scheduling barriers pin it): a wavefront issues in
    // order, so every memory instruction gets an MFMA slot of its own instead of queueing up in a burst.
    //   slot m: MFMA (i = m / WF, j = m % WF: the X fragment stays for WF MFMAs, measured 1 % faster than the W
    //   fragment staying) on the fragments of step KSI;  m < 6: fetch fragment m of the next step (stage ns,
    //   the other K64 parity);  REFILL: LDS-direct load m of stage rs (with eight slots the last takes two)
    auto slot = [&](auto MI, auto KSI, auto REFILL, int ns, int rs) {
        constexpr int m = decltype(MI)::value, ks = decltype(KSI)::value, i = m / WF, j = m % WF;
        if constexpr (m < kMfmas) {
            acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(op[ks][XF + j], op[ks][i], acc[i][j], 2, 2, 0, 0, 0, 0);
            if constexpr (decltype(REFILL)::value) {
                load_stage_part(rs, std::integral_constant<int, m>{});
                if constexpr (m == kMfmas - 1 && kMfmas < kLoads) load_stage_part(rs, std::integral_constant<int, kLoads - 1>{});
            }
            if constexpr (m < NF) read_frag(ns, std::integral_constant<int, 1 - ks>{}, std::integral_constant<int, m>{});
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    auto step = [&](auto KSI, auto REFILL, int ns, int rs) {
        __builtin_amdgcn_sched_barrier(0);
#define CONVROT_SLOT(m) slot(std::integral_constant<int, m>{}, KSI, REFILL, ns, rs);
        CONVROT_SLOT(0) CONVROT_SLOT(1) CONVROT_SLOT(2) CONVROT_SLOT(3) CONVROT_SLOT(4) CONVROT_SLOT(5) CONVROT_SLOT(6) CONVROT_SLOT(7)
        CONVROT_SLOT(8)
#undef CONVROT_SLOT
    };
    // The block meets once per stage, between its two K64 steps: every wavefront has then read all of
    // stage s into registers (its own LDS reads have returned), so the buffer can take stage s + 2, and
    // its share of stage s + 1 has landed, which the barrier extends to everybody's share.
    auto meet = [&]() {
        __builtin_amdgcn_sched_barrier(0);
        wait_vmcnt_lgkm0<0>();
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
    };

    // ---- pipeline: stages 0 and 1 in flight; when stage 0 has landed its first fragments are fetched.
    using K0 = std::integral_constant<int, 0>;
    using K1 = std::integral_constant<int, 1>;
#define CONVROT_ALL_LOADS(s) \
    load_stage_part(s, std::integral_constant<int, 0>{}); load_stage_part(s, std::integral_constant<int, 1>{}); \
    load_stage_part(s, std::integral_constant<int, 2>{}); load_stage_part(s, std::integral_constant<int, 3>{}); \
    load_stage_part(s, std::integral_constant<int, 4>{}); load_stage_part(s, std::integral_constant<int, 5>{}); \
    load_stage_part(s, std::integral_constant<int, 6>{}); load_stage_part(s, std::integral_constant<int, 7>{}); \
    load_stage_part(s, std::integral_constant<int, 8>{});
    CONVROT_ALL_LOADS(0)
    if (KS > 1) {
        CONVROT_ALL_LOADS(1)
        wait_vmcnt<kLoads>();
    } else {
        wait_vmcnt<0>();
    }
#undef CONVROT_ALL_LOADS
    __syncthreads();
#define CONVROT_F(f) read_frag(0, K0{}, std::integral_constant<int, f>{});
    CONVROT_F(0) CONVROT_F(1) CONVROT_F(2) CONVROT_F(3) CONVROT_F(4) CONVROT_F(5)
#undef CONVROT_F

    int s = 0;
    for (; s < KS - 2; ++s) {
        step(K0{}, std::false_type{}, s, 0);          // first K64 step of stage s; fetches the fragments of the second
        meet();
        step(K1{}, std::true_type{}, s + 1, s + 2);   // second step; fetches the first fragments of stage s + 1; refill
    }
    for (; s < KS; ++s) {   // the last two stages refill nothing (what the very last step fetches is unused)
        step(K0{}, std::false_type{}, s, 0);
        meet();
        step(K1{}, std::false_type{}, s + 1, 0);
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
                    for (int e = 0; e < 4; ++e) o[e] = (int32_t)acc[i][j][rb * 4 + e];   // exact: an integer below 2^24
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
                        float y[4] = {(acc[i][j][rb * 4 + 0] * sxm[i]) * sw.x, (acc[i][j][rb * 4 + 1] * sxm[i]) * sw.y,
                                      (acc[i][j][rb * 4 + 2] * sxm[i]) * sw.z, (acc[i][j][rb * 4 + 3] * sxm[i]) * sw.w};
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
    hipLaunchKernelGGL((gemm_w4a4_kernel<RAW, T>), dim3(grid), dim3(kThreads), 0, stream, (const uint8_t *)Xq,
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

hipError_t launch_gemm_w4a4(const void *Xq, const float *x_scale, const void *Wq, const float *w_scale,
                            const void *bias_bf16, int64_t M, int64_t N, int64_t K, void *Y_bf16,
                            int32_t *acc_i32, hipStream_t stream)
{
    if (M == 0 || N == 0) return hipSuccess;
    if (acc_i32)
        return launch_one<true>(Xq, x_scale, Wq, w_scale, nullptr, (int)M, (int)N, (int)K, nullptr, acc_i32, stream);
    return launch_one<false>(Xq, x_scale, Wq, w_scale, bias_bf16, (int)M, (int)N, (int)K, Y_bf16, nullptr, stream);
}

}  // namespace convrot
