// Panel layout of the code matrices (activations and weights, 4-bit packed or 8-bit) in HBM.
//
// A code matrix is a matrix of bytes: `rows` rows of `row_bytes` bytes (K / 2 for 4-bit codes, two per
// byte; K for 8-bit codes).  It is stored as 1 KB panels of 16 rows x 64 bytes, K-panels of the same 16
// rows adjacent:
//
//   byte b of row r  ->  ((r / 16) * kp + b / 64) * 1024 + (r % 16) * 64 + b % 64,   kp = ceil(row_bytes / 64)
//
// so that one K-stage of 16 tile rows - what one LDS-direct load instruction of the GEMM moves - is one
// contiguous, 1 KB-aligned kilobyte instead of sixteen 64-byte pieces a row pitch apart (the vector
// memory path moves the former at more than twice the rate of the latter).  Bytes of the last K-panel
// past row_bytes hold zero codes (they enter the GEMM and add nothing); rows past `rows` in the last
// row panel are never read and never written.
#pragma once
#include <stdint.h>

#include <hip/hip_runtime.h>

namespace convrot {
namespace panel {

constexpr int kRows = 16;        // rows per panel
constexpr int kRowBytes = 64;    // bytes of one row inside a panel
constexpr int kBytes = kRows * kRowBytes;

// K-panels per row
__host__ __device__ inline int64_t k_panels(int64_t row_bytes) { return (row_bytes + kRowBytes - 1) / kRowBytes; }

// bytes of the whole matrix, row padding included
__host__ __device__ inline int64_t matrix_bytes(int64_t rows, int64_t row_bytes)
{
    return ((rows + kRows - 1) / kRows) * k_panels(row_bytes) * kBytes;
}

// byte offset of (row, byte), kp = k_panels(row_bytes)
__host__ __device__ inline int64_t offset(int64_t row, int64_t byte, int64_t kp)
{
    return ((row / kRows) * kp + byte / kRowBytes) * kBytes + (row % kRows) * kRowBytes + byte % kRowBytes;
}

}  // namespace panel
}  // namespace convrot
