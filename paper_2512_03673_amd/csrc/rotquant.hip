// Kernel A of libconvrot: group-wise regular-Hadamard rotation + per-row absmax + 4-bit
// quantisation + packing of the codes, one pass over the bf16 input (ConvRot paper Sec. 4.2 Eq. 11-13,
// Eq. 1, Sec. 5.2).  Serves activations (rows = tokens) and weights (rows = output channels).
//
// Work split.  A "unit" is 16 consecutive elements of a row (32 B of bf16 in, 12 B of codes out)
// and belongs to one lane.  A row is spread over T = 64*Wv lanes (Wv wavefronts); lane t of the
// row owns units t, t+T, t+2T, ... (U of them), so the two load instructions of a wavefront for one
// such set of units cover a contiguous 2 KB span of the row.  The whole row stays in registers between the absmax
// reduction and the rounding, so X is read from HBM exactly once.
//
// Rotation.  H_g = H_4 (x) ... (x) H_4 (Thm 3.3) is separable: one radix-4 step per base-4 digit
// of the in-group index.  With the printed H_4 (all ones, -1 on the anti-diagonal) a step is
//     y_j = (x_0 + x_1 + x_2 + x_3) - 2 x_{3-j}.
// Digits 0 and 1 live inside a lane's 16 elements: a 16 x 16 matrix of +-1 (H_4 (x) H_4) applied to
// every unit, which is what the otherwise idle matrix pipe does for 64 units at a time, the bf16 -> fp32
// widening and the hand-over of each unit to its lane included (rotation_operand below): the vector ALU,
// which bounds this kernel on small inputs, sees none of it.
// Digits 2, 3 (g = 64, 256) run across lanes with DPP adds and digit 4 (g = 1024) with
// wavefront shuffles; there the step is taken as y_j = s - 2 x_j (the matrix J - 2I, which is
// the printed matrix with its columns reversed) and the flip is applied once, for free, to the
// lane's output address.  The 1/sqrt(g) = 2^-k normalisation is folded into the scale.
//
// Quantiser.  a = 2^-k max|z| (exact), s = a / 7 (IEEE division), r = 2^-k / s (IEEE division),
// q = rne(z / (2^k s)) decided exactly from two bracketing multiply-adds, with an exact-residual
// fallback for the few wavefronts that hold a (near-)tie (see the comment at the code).
// |z| / (2^k s) <= 7 (1 + 2^-22), so no clamp is needed.
//
// Output.  The codes leave in the layouts the GEMMs load from (e2m3_layout.h for 4-bit codes,
// panel_layout.h for 8-bit ones).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "convrot_internal.h"
#include "e2m3_layout.h"
#include "panel_layout.h"

namespace convrot {

namespace {

constexpr int kUnit = 16;  // elements per unit

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int v6u __attribute__((ext_vector_type(6)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

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

// The digits that live across lanes (in-group index digits 2 and up), on a unit whose digits 0 and 1 are done.
template <int G>
__device__ __forceinline__ void rotate_lanes(float (&v)[kUnit])
{
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

// The digits inside a unit on the matrix pipe.  v_mfma_f32_32x32x16_bf16 computes D = A B with B a 16 x 32
// matrix of bf16 whose column n is spread over lanes n (rows 0-7) and n + 32 (rows 8-15), eight consecutive
// rows = 16 contiguous bytes each, and leaves column n of D in lanes n (rows 8 b + r) and n + 32 (rows
// 8 b + 4 + r), register 4 b + r.  With the 32 units of lanes 0-31 as the columns of B and the 16 rows of
// R = H_4 (x) H_4 (I_4 (x) H_4 for g = 4; both symmetric) put at the rows 8 b + r of A, zeros elsewhere, lane n
// receives its whole rotated unit in element order, as fp32; a second MFMA with the rows of R at 8 b + 4 + r and
// the units of lanes 32-63 as B accumulates the other half of the wavefront on top.  Products with +-1 are
// exact and the sums are taken in fp32, as the register butterflies take them; the bf16 -> fp32 widening
// comes with it.  The price is that a lane fetches halves of two other lanes' units instead of its own.
// Returns this lane's eight entries of A for the MFMA that serves lanes 32 * half ... 32 * half + 31.
template <int G>
__device__ __forceinline__ v8bf rotation_operand(int lane, int half)
{
    const int i = lane & 31, kb = lane >> 5;
    const int o = 4 * (i >> 3) + (i & 3);             // element of the unit that accumulator row i holds
    const bool mine = ((i >> 2) & 1) == half;
    union { v8bf v; uint16_t u[8]; } a;
#pragma unroll
    for (int x = 0; x < 8; ++x) {
        const int k = 8 * kb + x;
        const bool neg = ((o & 3) + (k & 3) == 3) != (G >= 16 && (o >> 2) + (k >> 2) == 3);
        const bool zero = !mine || (G < 16 && (o >> 2) != (k >> 2));
        a.u[x] = zero ? (uint16_t)0 : (neg ? (uint16_t)0xBF80 : (uint16_t)0x3F80);    // bf16 0, -1, +1
    }
    return a.v;
}

// Digits 0 and 1 of 64 units, one per lane: b0 / b1 = bytes 16 (lane / 32) ... + 15 of the units owned by lanes
// lane % 32 and lane % 32 + 32; v = this lane's unit.
__device__ __forceinline__ void rotate_units_mfma(const v8bf &rot0, const v8bf &rot1, const u32x4 &b0, const u32x4 &b1,
                                                  float (&v)[kUnit])
{
    v16f d = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
    d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rot0, __builtin_bit_cast(v8bf, b0), d, 0, 0, 0);
    d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rot1, __builtin_bit_cast(v8bf, b1), d, 0, 0, 0);
#pragma unroll
    for (int e = 0; e < kUnit; ++e) v[e] = d[e];
}

template <int G>
constexpr int lane_flip_mask() { return G >= 1024 ? 63 : (G >= 256 ? 15 : (G >= 64 ? 3 : 0)); }

template <int G>
constexpr float group_norm() { return G == 4 ? 0.5f : G == 16 ? 0.25f : G == 64 ? 0.125f : G == 256 ? 0.0625f : 0.03125f; }

}  // namespace

// T = lanes per row.  Two ways of laying rows over wavefronts:
//   RPW = 1  a wavefront holds 64 lanes of one row (T = 64 * waves per row, BLOCK / T rows per block): any K, any g
//   RPW = 4  a wavefront holds 16 lanes of each of 4 consecutive rows (T = BLOCK / 4, 4 rows per block): g <= 256
//            (the cross-lane digits stay inside 16 lanes), used for K <= 4096.  The four rows' pieces of an output block
//            are adjacent in memory, so a store instruction touches 256- and 128-byte runs instead of 64- and
//            32-byte ones: as few cache lines per instruction as a row-major stream would.
// grid.x = 8 * ceil(rows / (8 * group rows)) * group rows / rows per block (see the row mapping below).
// BITS = 4: codes in [-7, 7], stored as FP6 E2M3 (e2m3_layout.h); BITS = 8 (the W8A8 variant of the layer): one
// int8 per code, [-127, 127] (panel_layout.h).
// (At least two wavefronts per SIMD, i.e. at most 256 registers per lane: then the compiler keeps the MFMA results in
// ordinary registers instead of copying them out of the accumulation registers, one move per element.)
template <int G, int U, int BLOCK, int BITS, int RPW>
__global__ __launch_bounds__(BLOCK, BLOCK <= 256 ? 2 : 1) void rotquant_kernel(const uint16_t *__restrict__ X, int64_t rows, int K,
                                                         int T, uint8_t *__restrict__ Xq,
                                                         float *__restrict__ scale)
{
    static_assert(RPW == 1 || (RPW == 4 && G <= 256), "four rows per wavefront need the rotation inside 16 lanes");
    __shared__ float s_part[BLOCK / 64 * RPW];

    const int tid = threadIdx.x;
    const int rib = RPW == 1 ? tid / T : (tid & 63) >> 4;                        // row inside the block
    const int t = RPW == 1 ? tid - rib * T : (tid >> 6) * 16 + (tid & 15);       // lane index inside the row
    const int rows_per_block = RPW == 1 ? BLOCK / T : RPW;
    // Blocks are dealt round-robin to the 8 XCDs, each with an L2 of its own.  The 16 rows of an output
    // panel go to consecutive blocks of one XCD, so that the 64-byte row pieces of a panel meet in one
    // L2 and leave it as whole lines.
    constexpr int kGroupRows = BITS == 4 ? e2m3::kRows : panel::kRows;   // rows that share an output block
    const int bpp = kGroupRows / rows_per_block;              // thread blocks per group of rows
    const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3;
    const int64_t row = ((int64_t)(idx / bpp) * 8 + xcd) * kGroupRows + (idx % bpp) * rows_per_block + rib;
    const bool row_ok = row < rows;
    const int units = K / kUnit;

    // All loads are issued up front and unconditionally: a unit (or row) that does not exist is replaced
    // by the last unit of the last row, and its owner is masked out of the absmax and the stores.
    // K % g == 0 makes a rotation group all-valid or all-invalid, so such lanes never feed valid ones.
    // The units are fetched as operands of the rotation MFMAs (rotation_operand): for h = 0, 1 this lane
    // loads bytes 16 kb ... 16 kb + 15 (kb = lane / 32) of the units owned by lane (lane % 32) + 32 h.
    const int lane = tid & 63;
    const uint16_t *src[2];
    int t_src[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int otid = (tid & ~63) | (lane & 31) | (h << 5);                     // the owner
        const int orib = RPW == 1 ? rib : (otid & 63) >> 4;                        // (a wavefront lies inside one row if RPW == 1)
        t_src[h] = RPW == 1 ? otid - rib * T : (otid >> 6) * 16 + (otid & 15);
        const int64_t orow = row - rib + orib;
        src[h] = X + (orow < rows ? orow : rows - 1) * (int64_t)K + 8 * (lane >> 5);
    }
    u32x4 raw[U][2];
#pragma unroll
    for (int i = 0; i < U; ++i) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int unit = min(i * T + t_src[h], units - 1);
            raw[i][h] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src[h] + (int64_t)unit * kUnit));
        }
    }
    const v8bf rot0 = rotation_operand<G>(lane, 0), rot1 = rotation_operand<G>(lane, 1);

    float v[U][kUnit];
    float amax = 0.0f;
#pragma unroll
    for (int i = 0; i < U; ++i) {
        rotate_units_mfma(rot0, rot1, raw[i][0], raw[i][1], v[i]);
        rotate_lanes<G>(v[i]);
        float m = 0.0f;
#pragma unroll
        for (int e = 0; e < kUnit; ++e) m = fmaxf(m, fabsf(v[i][e]));
        amax = (row_ok && i * T + t < units) ? fmaxf(amax, m) : amax;
    }

    // row absmax: butterfly over the row's lanes of this wavefront, then across the row's wavefronts through LDS
    if constexpr (RPW == 1) {
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
    } else {
#pragma unroll
        for (int m = 8; m >= 1; m >>= 1) amax = fmaxf(amax, __shfl_xor(amax, m, 64));
        if ((tid & 15) == 0) s_part[(tid >> 6) * RPW + rib] = amax;
        __syncthreads();
        float a = s_part[rib];
#pragma unroll
        for (int w = 1; w < BLOCK / 64; ++w) a = fmaxf(a, s_part[w * RPW + rib]);
        amax = a;
    }

    const float norm = group_norm<G>();
    const float a = amax * norm;                       // exact: power-of-two scaling
    constexpr float kQmax = BITS == 4 ? 7.0f : 127.0f;
    const float s = (a == 0.0f) ? 1.0f : a / kQmax;    // IEEE division
    const float r = norm / s;                          // IEEE division
    if (row_ok && t == 0) scale[row] = s;

    // Codes.  q = rne(z / su) with su = s / norm, decided exactly although the lane only multiplies.
    // r approximates 1 / su to 2^-24, so z / su lies strictly between z * r_lo and z * r_hi
    // (r_lo, r_hi = r (1 -+ 2^-21)); rounding to an integer is monotonic, hence when both products
    // round to the same integer so does the exact quotient.  One fused multiply-add against
    // 1.5 * 2^23 (+ an offset) rounds a product to nearest, ties to even, and leaves the integer in
    // the low mantissa bits.  A wavefront in which any pair disagrees (a few in a thousand on random
    // data; every exact tie, which bf16-grid inputs do produce when the scale is a short dyadic
    // number) redoes its codes through the exact residual e = z - q su (one rounding of a quantity
    // that is representable whenever q is the nearest or a neighbouring integer), which decides the
    // rounding, ties to even, without a division.
    const float su = s / norm;                                      // scale in un-normalised units (exact)
    const float r_lo = r * (1.0f - 0x1p-21f), r_hi = r * (1.0f + 0x1p-21f);
    const float half_su = 0.5f * su;
    const int tf = t ^ lane_flip_mask<G>();
    auto exact_code = [&](float z) {   // rne(z / su) as a float, from the exact residual
        float q = rintf(z * r);
        const float res = fmaf(-q, su, z);
        const bool odd = ((int)q & 1) != 0;
        const bool up = res > half_su || (res == half_su && odd);
        const bool dn = res < -half_su || (res == -half_su && odd);
        return q + ((up ? 1.0f : 0.0f) - (dn ? 1.0f : 0.0f));
    };

    if constexpr (BITS == 4) {
        // 4-bit codes leave as FP6 (E2M3) numbers, the operand format of the GEMM's MFMA: every integer in
        // [-7, 7] is one.  v_cvt_scalef32_2xpk16_fp6_f32 packs 2 x 16 floats into 6 dwords, interleaving
        // its two sources (a0 b0 a1 b1 ...): fed (unit[0..7], next unit[0..7]) and (unit[8..15], next
        // unit[8..15]) it returns this unit's 16 codes in dwords 0-2 and the next unit's in dwords 3-5.
        // The order of the codes inside a unit does not matter to the GEMM as long as it is the same for
        // activations and weights, which it is.
        constexpr float kMagic = 12582912.0f;                       // 1.5 * 2^23
        const int padded_units = (units + e2m3::kUnitsPerStage - 1) / e2m3::kUnitsPerStage * e2m3::kUnitsPerStage;
        const int64_t stages = padded_units / e2m3::kUnitsPerStage;
        uint8_t *const row_block = Xq + (row / e2m3::kRows) * stages * e2m3::kBlockBytes;
        const int r32 = (int)(row % e2m3::kRows);
        auto store_unit = [&](int i, uint32_t w0, uint32_t w1, uint32_t w2) {
            // A 24-byte chunk (the 32 codes one MFMA lane consumes) is an even unit followed by the odd
            // unit next to it, which the neighbouring lane holds: its first 16 bytes go to the A plane of the
            // block, the other 8 to the B plane (e2m3_layout.h).  The even lane fetches the odd lane's first dword.
            const uint32_t nb0 = __builtin_amdgcn_update_dpp(0u, w0, 0xB1, 0xF, 0xF, false);   // quad_perm [1,0,3,2]
            const int unit = i * T + tf;
            if (!(row_ok && unit < padded_units)) return;
            uint32_t nb = nb0;
            if (unit >= units) w0 = w1 = w2 = nb = 0;               // K padding: zero codes (units come in pairs: K % 32 == 0)
            uint8_t *blk = row_block + (int64_t)(unit / e2m3::kUnitsPerStage) * e2m3::kBlockBytes;
            const int c = (unit % e2m3::kUnitsPerStage) >> 1;       // chunk of the K128 stage
            if ((unit & 1) == 0) {
                *reinterpret_cast<u32x4 *>(blk + e2m3::a_offset(r32, c)) = u32x4{w0, w1, w2, nb};
            } else {
                *reinterpret_cast<u32x2 *>(blk + e2m3::b_offset(r32, c)) = u32x2{w1, w2};
            }
        };
#pragma unroll
        for (int i = 0; i < U; i += 2) {
            const bool pair = i + 1 < U;
            const int i1 = pair ? i + 1 : i;
            // the two brackets agree on every code exactly when the sum of |difference of their bit patterns|
            // is zero (the patterns share their upper halves, so the 16-bit SAD sees the whole difference)
            uint32_t disagree = 0;
            v16f qa, qb;    // conversion sources; the halves of a missing second unit stay unset (their output is not used)
#pragma unroll
            for (int e = 0; e < kUnit; ++e) {
                const float lo0 = fmaf(v[i][e], r_lo, kMagic), hi0 = fmaf(v[i][e], r_hi, kMagic);
                disagree = __builtin_amdgcn_sad_u16(__float_as_uint(lo0), __float_as_uint(hi0), disagree);
                if (e < 8) qa[e] = lo0 - kMagic;
                else qb[e - 8] = lo0 - kMagic;
                if (pair) {
                    const float lo1 = fmaf(v[i1][e], r_lo, kMagic), hi1 = fmaf(v[i1][e], r_hi, kMagic);
                    disagree = __builtin_amdgcn_sad_u16(__float_as_uint(lo1), __float_as_uint(hi1), disagree);
                    if (e < 8) qa[8 + e] = lo1 - kMagic;
                    else qb[e] = lo1 - kMagic;
                }
            }
            if (__builtin_amdgcn_ballot_w64(disagree != 0) != 0) {   // wavefront-uniform, rare
#pragma unroll
                for (int e = 0; e < kUnit; ++e) {
                    const float q0 = exact_code(v[i][e]);
                    if (e < 8) qa[e] = q0;
                    else qb[e - 8] = q0;
                    if (pair) {
                        const float q1 = exact_code(v[i1][e]);
                        if (e < 8) qa[8 + e] = q1;
                        else qb[e] = q1;
                    }
                }
            }
            const v6u packed = __builtin_amdgcn_cvt_scalef32_2xpk16_fp6_f32(qa, qb, 1.0f);
            store_unit(i, packed[0], packed[1], packed[2]);
            if (pair) store_unit(i + 1, packed[3], packed[4], packed[5]);
        }
    } else {
        // 8-bit codes: q + 128 in the low byte of the rounded sum, four codes per dword by a Horner sum over
        // the raw float bits, sum_e (C + u_e) 2^(8 e) mod 2^32 with C the magic's bits (the same sum over the
        // other bracket: digits differ by at most one, so the two sums are equal exactly when every pair of
        // codes is).
        constexpr uint32_t kOff = 128u;                            // offset that keeps every digit positive
        constexpr int kPerDword = 4;
        constexpr int kDwords = kUnit / kPerDword;                 // output dwords per unit
        constexpr float kMagic = 12582912.0f + (float)kOff;
        constexpr uint32_t kC = 0x4B400000u;                       // bits of 1.5 * 2^23
        constexpr uint32_t kFlip = 0x80808080u;                    // offset-binary digits -> two's complement
        constexpr uint32_t kBias = kC + (kC << 8);                 // sum_e C 2^(8 e) mod 2^32: only the first terms survive
#pragma unroll
        for (int i = 0; i < U; ++i) {
            uint32_t disagree = 0;
            uint32_t code[kDwords];
#pragma unroll
            for (int w = 0; w < kDwords; ++w) {
                uint32_t acc = 0, acc_hi = 0;
#pragma unroll
                for (int e = kPerDword - 1; e >= 0; --e) {
                    const float z = v[i][kPerDword * w + e];
                    acc = (acc << 8) + __float_as_uint(fmaf(z, r_lo, kMagic));
                    acc_hi = (acc_hi << 8) + __float_as_uint(fmaf(z, r_hi, kMagic));
                }
                disagree |= acc ^ acc_hi;
                code[w] = (acc - kBias) ^ kFlip;
            }
            if (__builtin_amdgcn_ballot_w64(disagree != 0) != 0) {   // wavefront-uniform, rare
#pragma unroll
                for (int w = 0; w < kDwords; ++w) {
                    uint32_t d = 0;
#pragma unroll
                    for (int e = 0; e < kPerDword; ++e)
                        d |= ((uint32_t)(int)exact_code(v[i][kPerDword * w + e]) & 0xFFu) << (8 * e);
                    code[w] = d;
                }
            }
            // Panel layout: 1 KB panels of 16 rows x 64 bytes, a unit is 16 bytes of its row; units past the
            // row's end inside its last K-panel are stored as zero codes.
            const int unit = i * T + tf;
            constexpr int kUnitsPerPanelRow = panel::kRowBytes / kUnit;
            const int padded_units = (units + kUnitsPerPanelRow - 1) / kUnitsPerPanelRow * kUnitsPerPanelRow;
            if (row_ok && unit < padded_units) {
                if (unit >= units) {
#pragma unroll
                    for (int w = 0; w < kDwords; ++w) code[w] = 0;
                }
                uint8_t *o = Xq + ((row >> 4) * (int64_t)(padded_units / kUnitsPerPanelRow) + unit / kUnitsPerPanelRow) * panel::kBytes +
                             (int)(row & 15) * panel::kRowBytes + (unit % kUnitsPerPanelRow) * kUnit;
                // plain (cacheable) stores: the pieces of a line are merged in L2
                *reinterpret_cast<u32x4 *>(o) = u32x4{code[0], code[1], code[2], code[3]};
            }
        }
    }
}

namespace {

// Sylvester (Walsh) Hadamard matrix of order G on a unit: radix-2 butterflies (a, b) -> (a + b, a - b),
// in-group index bits 0-3 inside the lane's 16 elements, the higher ones across lanes.
template <int G>
__device__ __forceinline__ void sylvester_unit(float (&v)[kUnit], int lane)
{
    constexpr int kBitsInUnit = G >= 16 ? 4 : 2;
#pragma unroll
    for (int b = 0; b < kBitsInUnit; ++b)
#pragma unroll
        for (int e = 0; e < kUnit; ++e)
            if (!(e & (1 << b))) {
                const float lo = v[e], hi = v[e | (1 << b)];
                v[e] = lo + hi;
                v[e | (1 << b)] = lo - hi;
            }
    constexpr int kLaneBits = G == 64 ? 2 : G == 256 ? 4 : G == 1024 ? 6 : 0;
#pragma unroll
    for (int b = 0; b < kLaneBits; ++b) {
        const bool upper = (lane >> b) & 1;
#pragma unroll
        for (int e = 0; e < kUnit; ++e) {
            const float other = __shfl_xor(v[e], 1 << b, 64);
            v[e] = upper ? other - v[e] : v[e] + other;
        }
    }
}

}  // namespace

// Diagnostic (the paper's outlier-amplitude metric max |X H|, Sec. 4.2 and Table 5-1): per-row maximum of
// the rotated activations for KIND 0 = no rotation, 1 = the layer's regular Hadamard rotation, 2 = the
// Sylvester Hadamard matrix of the same order.  One wavefront per row, 1024 elements per pass.
template <int G, int KIND>
__global__ __launch_bounds__(256, 2) void rotated_absmax_kernel(const uint16_t *__restrict__ X, int64_t rows, int K,
                                                             float *__restrict__ out)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;                     // wavefront-uniform
    const int units = K / kUnit;
    const uint16_t *xrow = X + row * (int64_t)K;
    float amax = 0.0f;
    v8bf rot0, rot1;
    if constexpr (KIND == 1) { rot0 = rotation_operand<G>(lane, 0); rot1 = rotation_operand<G>(lane, 1); }
    for (int base = 0; base < units; base += 64) {
        const int unit = base + lane;
        const bool ok = unit < units;            // K % g == 0: a rotation group is all-valid or all-invalid
        float v[kUnit];
        if constexpr (KIND == 1) {
            // the layer's rotation, with the arithmetic of the rotate+quantise kernel (bit-identical maxima)
            const int u0 = min(base + (lane & 31), units - 1), u1 = min(base + (lane & 31) + 32, units - 1);
            const uint16_t *half = xrow + 8 * (lane >> 5);
            const u32x4 b0 = *reinterpret_cast<const u32x4 *>(half + (int64_t)u0 * kUnit);
            const u32x4 b1 = *reinterpret_cast<const u32x4 *>(half + (int64_t)u1 * kUnit);
            rotate_units_mfma(rot0, rot1, b0, b1, v);
            rotate_lanes<G>(v);
        } else {
            const u32x4 *p = reinterpret_cast<const u32x4 *>(xrow + (int64_t)(ok ? unit : units - 1) * kUnit);
            const u32x4 lo = p[0], hi = p[1];
            const uint32_t w[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                v[2 * j] = __uint_as_float(w[j] << 16);
                v[2 * j + 1] = __uint_as_float(w[j] & 0xFFFF0000u);
            }
        }
        if constexpr (KIND == 2) sylvester_unit<G>(v, lane);
        float m = 0.0f;
#pragma unroll
        for (int e = 0; e < kUnit; ++e) m = fmaxf(m, fabsf(v[e]));
        amax = ok ? fmaxf(amax, m) : amax;
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) amax = fmaxf(amax, __shfl_xor(amax, m, 64));
    if (lane == 0) out[row] = KIND == 0 ? amax : amax * group_norm<G>();
}

namespace {

template <int G, int U, int BITS>
hipError_t launch_gu(const void *X, int64_t rows, int K, int waves_per_row, void *Xq, float *scale,
                     hipStream_t stream)
{
    const int T = 64 * waves_per_row;
    // grid: 8 XCDs x whole row groups per XCD x blocks per group (see the row mapping in the kernel)
    constexpr int kGroupRows = BITS == 4 ? e2m3::kRows : panel::kRows;
    auto grid_for = [&](int rpb) { return (unsigned)(((rows + 8 * kGroupRows - 1) / (8 * kGroupRows)) * 8 * (kGroupRows / rpb)); };
    if (T <= 256) {
        const int rpb = 256 / T;
        hipLaunchKernelGGL((rotquant_kernel<G, U, 256, BITS, 1>), dim3(grid_for(rpb)), dim3(256), 0, stream,
                           (const uint16_t *)X, rows, K, T, (uint8_t *)Xq, scale);
    } else if (T <= 512) {
        hipLaunchKernelGGL((rotquant_kernel<G, U, 512, BITS, 1>), dim3(grid_for(1)), dim3(512), 0, stream,
                           (const uint16_t *)X, rows, K, 512, (uint8_t *)Xq, scale);
    } else {
        hipLaunchKernelGGL((rotquant_kernel<G, U, 1024, BITS, 1>), dim3(grid_for(1)), dim3(1024), 0, stream,
                           (const uint16_t *)X, rows, K, 1024, (uint8_t *)Xq, scale);
    }
    return hipGetLastError();
}

// four rows per wavefront: 4 wavefronts of 16 lanes per row (blocks of 256 threads; with larger blocks, i.e.
// longer rows, the mapping loses more to the block-wide barrier than the stores gain: measured)
template <int G, int U, int BITS>
hipError_t launch_gu4(const void *X, int64_t rows, int K, void *Xq, float *scale, hipStream_t stream)
{
    constexpr int kGroupRows = BITS == 4 ? e2m3::kRows : panel::kRows;
    const unsigned grid = (unsigned)(((rows + 8 * kGroupRows - 1) / (8 * kGroupRows)) * 8 * (kGroupRows / 4));
    hipLaunchKernelGGL((rotquant_kernel<G, U, 256, BITS, 4>), dim3(grid), dim3(256), 0, stream, (const uint16_t *)X, rows, K,
                       64, (uint8_t *)Xq, scale);
    return hipGetLastError();
}

template <int G, int BITS>
hipError_t launch_g(const void *X, int64_t rows, int K, void *Xq, float *scale, hipStream_t stream)
{
    if constexpr (G <= 256) {
        // four rows per wavefront whenever 4 wavefronts x 16 lanes x 4 units hold a row (K <= 4096)
        const int spans = (K / kUnit + 15) / 16;   // 256-element spans per row
        if (spans <= 16) {
            switch ((spans + 3) / 4) {
                case 1: return launch_gu4<G, 1, BITS>(X, rows, K, Xq, scale, stream);
                case 2: return launch_gu4<G, 2, BITS>(X, rows, K, Xq, scale, stream);
                case 3: return launch_gu4<G, 3, BITS>(X, rows, K, Xq, scale, stream);
                default: return launch_gu4<G, 4, BITS>(X, rows, K, Xq, scale, stream);
            }
        }
    }
    // Pick the wavefronts per row (1, 2, 4, 8 or 16) so that every lane holds at most 4 units,
    // preferring 3-4 units per lane (enough bytes in flight per wavefront, registers under 128).
    const int chunks = (K / kUnit + 63) / 64;  // 1024-element spans per row
    int wv = 1;
    while (wv < 16 && (chunks + wv - 1) / wv > 4) wv *= 2;
    const int u = (chunks + wv - 1) / wv;
    switch (u) {
        case 1: return launch_gu<G, 1, BITS>(X, rows, K, wv, Xq, scale, stream);
        case 2: return launch_gu<G, 2, BITS>(X, rows, K, wv, Xq, scale, stream);
        case 3: return launch_gu<G, 3, BITS>(X, rows, K, wv, Xq, scale, stream);
        default: return launch_gu<G, 4, BITS>(X, rows, K, wv, Xq, scale, stream);
    }
}

template <int BITS>
hipError_t launch_bits(const void *X, int64_t rows, int64_t K, int group, void *Xq, float *scale, hipStream_t stream)
{
    switch (group) {
        case 4: return launch_g<4, BITS>(X, rows, (int)K, Xq, scale, stream);
        case 16: return launch_g<16, BITS>(X, rows, (int)K, Xq, scale, stream);
        case 64: return launch_g<64, BITS>(X, rows, (int)K, Xq, scale, stream);
        case 256: return launch_g<256, BITS>(X, rows, (int)K, Xq, scale, stream);
        case 1024: return launch_g<1024, BITS>(X, rows, (int)K, Xq, scale, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

hipError_t launch_rotquant(const void *X, int64_t rows, int64_t K, int group, int bits, void *Xq, float *scale,
                           hipStream_t stream)
{
    if (rows == 0) return hipSuccess;
    if (bits == 4) return launch_bits<4>(X, rows, K, group, Xq, scale, stream);
    if (bits == 8) return launch_bits<8>(X, rows, K, group, Xq, scale, stream);
    return hipErrorInvalidValue;
}

namespace {

template <int G>
hipError_t launch_absmax_g(const void *X, int64_t rows, int K, int kind, float *out, hipStream_t stream)
{
    const dim3 grid((unsigned)((rows + 3) / 4)), block(256);
    const uint16_t *x = (const uint16_t *)X;
    if (kind == 0) hipLaunchKernelGGL((rotated_absmax_kernel<G, 0>), grid, block, 0, stream, x, rows, K, out);
    else if (kind == 1) hipLaunchKernelGGL((rotated_absmax_kernel<G, 1>), grid, block, 0, stream, x, rows, K, out);
    else hipLaunchKernelGGL((rotated_absmax_kernel<G, 2>), grid, block, 0, stream, x, rows, K, out);
    return hipGetLastError();
}

}  // namespace

// ---- code matrix -> plain int8 codes (gate / debug export)
__global__ __launch_bounds__(256) void unpack_codes_kernel(const uint8_t *__restrict__ Xq, int64_t rows, int K,
                                                           int8_t *__restrict__ codes)
{
    // one thread per unit of 16 codes: its 12 bytes are the first or the last 12 of a 24-byte chunk
    const int units = K / kUnit;
    const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (id >= rows * units) return;
    const int64_t row = id / units;
    const int unit = (int)(id - row * units);
    const uint8_t *blk = Xq + ((row / e2m3::kRows) * e2m3::stages(K) + unit / e2m3::kUnitsPerStage) * e2m3::kBlockBytes;
    const int r = (int)(row % e2m3::kRows), c = (unit % e2m3::kUnitsPerStage) >> 1;
    const uint32_t *pa = reinterpret_cast<const uint32_t *>(blk + e2m3::a_offset(r, c));
    const uint32_t *pb = reinterpret_cast<const uint32_t *>(blk + e2m3::b_offset(r, c));
    uint32_t w[3];
    if ((unit & 1) == 0) { w[0] = pa[0]; w[1] = pa[1]; w[2] = pa[2]; }
    else { w[0] = pa[3]; w[1] = pb[0]; w[2] = pb[1]; }
    int8_t out[kUnit];
#pragma unroll
    for (int e = 0; e < kUnit; ++e) {
        const int bit = 6 * (2 * (e % 8) + e / 8);
        uint32_t f = w[bit / 32] >> (bit % 32);
        if (bit % 32 > 26) f |= w[bit / 32 + 1] << (32 - bit % 32);
        const int ex = (f >> 3) & 3, mant = f & 7;
        const int mag = ex == 0 ? 0 : ((8 | mant) << ex) >> 4;   // E2M3, bias 1: (1 + mant / 8) * 2^(ex - 1)
        out[e] = (int8_t)((f & 32) ? -mag : mag);
    }
    int4 *dst = reinterpret_cast<int4 *>(codes + row * (int64_t)K + (int64_t)unit * kUnit);
    *dst = *reinterpret_cast<const int4 *>(out);
}

hipError_t launch_unpack_codes(const void *Xq, int64_t rows, int64_t K, int8_t *codes, hipStream_t stream)
{
    if (rows == 0) return hipSuccess;
    const int64_t n = rows * (K / kUnit);
    hipLaunchKernelGGL(unpack_codes_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, (const uint8_t *)Xq, rows,
                       (int)K, codes);
    return hipGetLastError();
}

hipError_t launch_rotated_absmax(const void *X, int64_t rows, int64_t K, int group, int kind, float *out,
                                 hipStream_t stream)
{
    if (rows == 0) return hipSuccess;
    if (kind < 0 || kind > 2) return hipErrorInvalidValue;
    switch (group) {
        case 4: return launch_absmax_g<4>(X, rows, (int)K, kind, out, stream);
        case 16: return launch_absmax_g<16>(X, rows, (int)K, kind, out, stream);
        case 64: return launch_absmax_g<64>(X, rows, (int)K, kind, out, stream);
        case 256: return launch_absmax_g<256>(X, rows, (int)K, kind, out, stream);
        case 1024: return launch_absmax_g<1024>(X, rows, (int)K, kind, out, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace convrot
