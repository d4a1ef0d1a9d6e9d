// HBM layout of the 4-bit code matrices (activations and weights): FP6 E2M3 codes in 3 KB blocks.
//
// A 4-bit code q in [-7, 7] is stored as the FP6 (E2M3: 1 sign, 2 exponent, 3 mantissa bits, bias 1) number
// q, the operand format of v_mfma_f32_32x32x64_f8f6f4: six bits per code, 0.75 byte.  Products of two
// codes and their sums up to K = 65536 are integers below 2^24, so the MFMA's fp32 accumulation is exact.
//
//   unit   16 consecutive codes of a row = 96 bits = 3 dwords, in the order the pack instruction
//          v_cvt_scalef32_2xpk16_fp6_f32 leaves them: code e of the unit at bit 6 (2 (e % 8) + e / 8)
//   chunk  two consecutive units (even, odd) = 32 codes = 24 bytes: what one lane feeds one MFMA.
//          Its first 16 bytes are the chunk's "A part", the last 8 its "B part".
//   stage  4 chunks = 128 codes of a row: one K128 stage of the GEMM (two MFMAs per accumulator tile)
//   block  32 rows x one stage = 3 KB, stored as
//            A plane  32 rows x 64 bytes: the A part of chunk c of row r at  r * 64 + ((c ^ swz_a(r)) * 16)
//            B plane  32 rows x 32 bytes: the B part at               2048 + r * 32 + ((c ^ swz_b(r)) * 8)
//          The XOR swizzles are the ones under which the GEMM's fragment reads from LDS (32 rows, one chunk;
//          ds_read_b128 on the A plane, ds_read_b64 on the B plane) touch every bank once; they are baked into
//          the HBM layout so that the GEMM's LDS-direct loads are straight copies of whole kilobytes.
//   matrix blocks of the same 32 rows adjacent, K-stage minor:  block (R, S) at (R * stages + S) * 3072.
//
// The last stage of a row is padded with zero codes; rows past `rows` in the last block are never read
// or written.
#pragma once
#include <stdint.h>

#include <hip/hip_runtime.h>

namespace convrot {
namespace e2m3 {

constexpr int kRows = 32;             // rows per block
constexpr int kStageCodes = 128;      // codes of a row per block
constexpr int kUnitsPerStage = 8;     // units of 16 codes
constexpr int kARowBytes = 64, kBRowBytes = 32;
constexpr int kAPlaneBytes = kRows * kARowBytes;   // 2 KB
constexpr int kBPlaneBytes = kRows * kBRowBytes;   // 1 KB
constexpr int kBlockBytes = kAPlaneBytes + kBPlaneBytes;

__host__ __device__ inline int swz_a(int r) { return ((r >> 1) ^ (r >> 3)) & 3; }
__host__ __device__ inline int swz_b(int r) { return (r >> 3) & 3; }

// byte offsets inside a block of the two parts of chunk c (0..3) of row r (0..31)
__host__ __device__ inline int a_offset(int r, int c) { return r * kARowBytes + ((c ^ swz_a(r)) << 4); }
__host__ __device__ inline int b_offset(int r, int c) { return kAPlaneBytes + r * kBRowBytes + ((c ^ swz_b(r)) << 3); }

__host__ __device__ inline int64_t stages(int64_t K) { return (K + kStageCodes - 1) / kStageCodes; }

// bytes of the whole matrix, padding included
__host__ __device__ inline int64_t matrix_bytes(int64_t rows, int64_t K)
{
    return ((rows + kRows - 1) / kRows) * stages(K) * kBlockBytes;
}

}  // namespace e2m3
}  // namespace convrot
