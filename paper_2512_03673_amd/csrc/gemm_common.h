// Shared pieces of the GEMM kernels of libconvrot, 4-bit and 8-bit (LDS swizzle, LDS-direct loads,
// tile order).  See gemm_w4a4.hip for the description of the method.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace convrot {
namespace gemm {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v2f __attribute__((ext_vector_type(2)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));

constexpr int kRowBytes = 64;                 // bytes of K per row per stage: 128 4-bit codes or 64 8-bit codes
constexpr int kSubSteps = kRowBytes / 32;     // MFMA K-steps of 32 bytes per row (one ds_read_b128 per fragment) per stage
constexpr int kNumXcd = 8;

// Which of the four 16-byte slots of its LDS row a piece lands in: slot = piece ^ swz(row).
// For any 8 consecutive rows the (row & 1, slot) pairs are distinct (32 banks), and for any 16
// consecutive rows the (row & 3, slot) pairs are distinct (64 banks).
__device__ __forceinline__ int swz(int row) { return ((row >> 1) ^ (row >> 3)) & 3; }

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    // gfx9 encoding: vmcnt = {imm[15:14], imm[3:0]}, expcnt = imm[6:4], lgkmcnt = imm[11:8]
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0xF << 8));
}

// The same, and every LDS (and scalar memory) operation of the wavefront returned as well.
template <int N>
__device__ __forceinline__ void wait_vmcnt_lgkm0()
{
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0x0 << 8));
}

// global_load_lds_dwordx4: lane l copies 16 bytes from its global address to LDS address M0 + 16 l.
// M0 is written here and not named as a clobber.  This relies on a property of the AMDGPU backend, not on a
// documented contract: M0 is a reserved register that the register allocator never assigns a value to; every
// instruction the backend itself emits that reads M0 (LDS-direct loads from the builtin, s_movrel, GWS, s_sendmsg)
// is preceded by its own write in the same block.  Naming a reserved register in a clobber list is rejected with
// a warning ("may not be preserved ... may lead to undefined behaviour") and changes nothing in the generated code,
// so it would only look like a guarantee.  None of the instructions above occurs in the GEMM kernels besides this
// one (the build prints the hipcc version it ran with, and the bit-exact GEMM tests are the check that a new
// toolchain still behaves so: a stale M0 sends a kilobyte of operands to the wrong place in the ring).
__device__ __forceinline__ void lds_dma16(const uint8_t *base, uint32_t lane_off, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(lane_off), "s"(base), "s"(lds_addr) : "memory");
}
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b)
{
    v2bf r = __builtin_convertvector((v2f){a, b}, v2bf);   // v_cvt_pk_bf16_f32: round to nearest even
    return *reinterpret_cast<uint32_t *>(&r);
}

// Tile order: blocks are dealt round-robin to the 8 XCDs by the hardware, each XCD has its own
// L2.  Give every XCD one contiguous range of logical tile ids, and walk that range in bands of
// `GM` tile rows (a template parameter: 6 suits 256 x 128 tiles, 8 square ones) so that tiles that run together share X and W panels.  `bid` may run past the
// grid (a persistent block asks for bid + gridDim.x, ...): false when XCD bid % 8 has no such tile.
template <int GM = 6>
__device__ __forceinline__ bool tile_of_block(int bid, int tiles_m, int tiles_n, int &tm, int &tn)
{
    const int ntiles = tiles_m * tiles_n;
    const int per_xcd = (ntiles + kNumXcd - 1) / kNumXcd;
    if (bid / kNumXcd >= per_xcd) return false;
    const int id = (bid % kNumXcd) * per_xcd + bid / kNumXcd;
    if (id >= ntiles) return false;
    const int band = id / (GM * tiles_n);
    const int first_m = band * GM;
    const int rows_in_band = min(GM, tiles_m - first_m);
    const int local = id - band * GM * tiles_n;
    tm = first_m + local % rows_in_band;
    tn = local / rows_in_band;
    return true;
}

}  // namespace gemm

}  // namespace convrot
