// Internal launch interface between the C ABI (convrot_api.hip) and the kernels.
// Shapes are validated by the caller; these only pick a configuration and launch.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace convrot {

// Block tile of both GEMM kernels for an [M, N] output: X rows per tile, 192 (with 192 W rows) or 256
// (with 128).  Blocks are dealt to the 256 compute units as slots free up, so a launch lasts about as
// long as the busiest unit's share, ceil(tiles / 256) blocks of TM x TN products each; the square tile
// moves fewer operand bytes per product and takes the ties.
inline int gemm_tile_rows(int64_t M, int64_t N)
{
    auto work = [&](int64_t tm, int64_t tn) {
        const int64_t tiles = ((M + tm - 1) / tm) * ((N + tn - 1) / tn);
        return ((tiles + 255) / 256) * tm * tn;
    };
    return work(192, 192) <= work(256, 128) ? 192 : 256;
}

// Rotate + quantise + pack `rows` rows of K bf16 values (group in {4,16,64,256,1024}; bits 4: FP6 E2M3
// codes in the layout of e2m3_layout.h, bits 8: one int8 per code in the layout of panel_layout.h).
hipError_t launch_rotquant(const void *X, int64_t rows, int64_t K, int group, int bits, void *Xq, float *scale,
                           hipStream_t stream);

// 4-bit code matrix (FP6 layout) -> int8 codes [rows, K], row-major.
hipError_t launch_unpack_codes(const void *Xq, int64_t rows, int64_t K, int8_t *codes, hipStream_t stream);

// Per-row max |R(X)| for kind 0 = no rotation, 1 = the regular Hadamard rotation, 2 = Sylvester (diagnostic).
hipError_t launch_rotated_absmax(const void *X, int64_t rows, int64_t K, int group, int kind, float *out,
                                 hipStream_t stream);

// W4A4 GEMM on 4-bit code matrices (e2m3_layout.h).  Exactly one of Y_bf16 / acc_i32 is non-null:
//   Y_bf16 : dequantised bf16 output (needs x_scale, w_scale; bias_bf16 [N] or null)
//   acc_i32: raw int32 accumulators
hipError_t launch_gemm_w4a4(const void *Xq, const float *x_scale, const void *Wq, const float *w_scale,
                            const void *bias_bf16, int64_t M, int64_t N, int64_t K, void *Y_bf16,
                            int32_t *acc_i32, hipStream_t stream);

// W8A8 GEMM on int8 codes in the panel layout; same contract as launch_gemm_w4a4.
hipError_t launch_gemm_w8a8(const void *Xq, const float *x_scale, const void *Wq, const float *w_scale,
                            const void *bias_bf16, int64_t M, int64_t N, int64_t K, void *Y_bf16,
                            int32_t *acc_i32, hipStream_t stream);

}  // namespace convrot
