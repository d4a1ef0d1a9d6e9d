// Host sanitizer run of the C ABI's host side: every entry point with arguments that validation must reject
// (or that are no-ops) before anything touches a device, the size queries over a sweep of shapes, and the
// status strings.  Built with -fsanitize=address,undefined on the host pass and run by
// tests/test_host_sanitizers.py; needs no GPU.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "convrot.h"

#define CHECK(cond)                                                                       \
    do {                                                                                  \
        if (!(cond)) {                                                                    \
            std::fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
            std::exit(1);                                                                 \
        }                                                                                 \
    } while (0)

int main()
{
    void *A = reinterpret_cast<void *>(0x10000);          // aligned, never dereferenced on the host
    void *A2 = reinterpret_cast<void *>(0x10002);
    float *F = reinterpret_cast<float *>(0x20000);
    CHECK(convrot_version() == CONVROT_VERSION);
    for (int s = -8; s <= 1; ++s) CHECK(std::strlen(convrot_status_string(s)) > 0);

    // size queries: monotone, padded to whole blocks, zero on bad input, no overflow at the largest shapes
    size_t prev = 0;
    for (int64_t rows = 0; rows <= 130; ++rows) {
        const size_t b = convrot_packed_bytes(rows, 96);
        CHECK(b >= prev && b % 3072 == 0 && b == (size_t)((rows + 31) / 32) * 3072);
        prev = b;
    }
    for (int64_t K = 32; K <= CONVROT_MAX_K; K += 32) {
        CHECK(convrot_packed_bytes(33, K) == 2 * (size_t)((K + 127) / 128) * 3072);
        CHECK(convrot_packed_bytes8(33, K) == 3 * (size_t)((K + 63) / 64) * 1024);
        CHECK(convrot_workspace_bytes(33, K) == convrot_packed_bytes(33, K) + 256);
        CHECK(convrot_workspace_bytes8(33, K) == convrot_packed_bytes8(33, K) + 256);
    }
    CHECK(convrot_packed_bytes(INT32_MAX, CONVROT_MAX_K) == (size_t)(((int64_t)INT32_MAX + 31) / 32) * 512 * 3072);
    CHECK(convrot_packed_bytes(-1, 32) == 0 && convrot_packed_bytes(4, 0) == 0 && convrot_packed_bytes(4, 33) == 0);
    CHECK(convrot_packed_bytes8(-1, 32) == 0 && convrot_workspace_bytes(-1, 32) == 0 && convrot_workspace_bytes8(4, -2) == 0);
    CHECK(convrot_gemm_tile_rows(4608, 12288) == 192 && convrot_gemm_tile_rows(300, 520) == 256);
    CHECK(convrot_gemm_tile_rows(INT32_MAX, INT32_MAX) > 0 && convrot_gemm_tile_rows(-1, 4) == 0);

    // every launching entry point: null, shape, group, alignment, workspace, and the empty no-ops
    static const int bad_groups[] = {0, 1, 2, 8, 32, 128, 512, 2048, -16};
    for (int g : bad_groups) {
        CHECK(convrot_rotquant_act(A, 4, 1024, g, A, F, nullptr) == CONVROT_ERR_GROUP);
        CHECK(convrot_prepare_weight8(A, 4, 1024, g, A, F, nullptr) == CONVROT_ERR_GROUP);
        CHECK(convlinear4bit_forward(A, A, F, nullptr, 4, 4, 1024, g, A, A, 1 << 20, nullptr) == CONVROT_ERR_GROUP);
        CHECK(convlinear4bit_forward_noalloc(A, A, F, nullptr, 4, 4, 1024, g, A, nullptr) == CONVROT_ERR_GROUP);
        CHECK(convrot_rotated_absmax(A, 4, 1024, g, 1, F, nullptr) == CONVROT_ERR_GROUP);
    }
    static const int64_t bad_k[] = {0, -32, 16, 48, 1000, CONVROT_MAX_K + 32, INT64_MAX};
    for (int64_t K : bad_k) {
        CHECK(convrot_rotquant_act(A, 4, K, 16, A, F, nullptr) == CONVROT_ERR_SHAPE);
        CHECK(convrot_rotquant_act8(A, 4, K, 16, A, F, nullptr) == CONVROT_ERR_SHAPE);
        CHECK(convrot_w4a4_gemm_dequant(A, F, A, F, nullptr, 4, 4, K, A, nullptr) == CONVROT_ERR_SHAPE);
        CHECK(convrot_w8a8_gemm_dequant(A, F, A, F, nullptr, 4, 4, K, A, nullptr) == CONVROT_ERR_SHAPE);
        CHECK(convrot_w4a4_gemm_i32(A, A, 4, 4, K, (int32_t *)A, nullptr) == CONVROT_ERR_SHAPE);
        CHECK(convrot_w8a8_gemm_i32(A, A, 4, 4, K, (int32_t *)A, nullptr) == CONVROT_ERR_SHAPE);
        CHECK(convrot_unpack_codes(A, 4, K, (int8_t *)A, nullptr) == CONVROT_ERR_SHAPE);
        CHECK(convlinear8bit_forward(A, A, F, nullptr, 4, 4, K, 16, A, A, 1 << 20, nullptr) == CONVROT_ERR_SHAPE);
        CHECK(convlinear4bit_forward_noalloc(A, A, F, nullptr, 4, 4, K, 16, A, nullptr) == CONVROT_ERR_SHAPE);
    }
    CHECK(convrot_rotquant_act(A, -1, 1024, 16, A, F, nullptr) == CONVROT_ERR_SHAPE);
    CHECK(convrot_rotquant_act(A, (int64_t)INT32_MAX + 1, 1024, 16, A, F, nullptr) == CONVROT_ERR_SHAPE);
    CHECK(convrot_rotquant_act(A, 4, 96, 64, A, F, nullptr) == CONVROT_ERR_SHAPE);
    CHECK(convrot_w4a4_gemm_dequant(A, F, A, F, nullptr, -4, 4, 1024, A, nullptr) == CONVROT_ERR_SHAPE);
    CHECK(convrot_w4a4_gemm_dequant(nullptr, F, A, F, nullptr, 4, 4, 1024, A, nullptr) == CONVROT_ERR_NULL);
    CHECK(convrot_w4a4_gemm_dequant(A, nullptr, A, F, nullptr, 4, 4, 1024, A, nullptr) == CONVROT_ERR_NULL);
    CHECK(convrot_w4a4_gemm_dequant(A, F, A, nullptr, nullptr, 4, 4, 1024, A, nullptr) == CONVROT_ERR_NULL);
    CHECK(convrot_w4a4_gemm_dequant(A, F, A, F, nullptr, 4, 4, 1024, nullptr, nullptr) == CONVROT_ERR_NULL);
    CHECK(convrot_w4a4_gemm_dequant(A2, F, A, F, nullptr, 4, 4, 1024, A, nullptr) == CONVROT_ERR_ALIGN);
    CHECK(convrot_w4a4_gemm_dequant(A, F, A, F, (char *)A + 1, 4, 4, 1024, A, nullptr) == CONVROT_ERR_ALIGN);
    CHECK(convrot_w4a4_gemm_dequant(A, (float *)A2, A, F, nullptr, 4, 4, 1024, A, nullptr) == CONVROT_ERR_ALIGN);
    CHECK(convrot_rotquant_act(nullptr, 4, 1024, 16, A, F, nullptr) == CONVROT_ERR_NULL);
    CHECK(convrot_rotquant_act(A2, 4, 1024, 16, A, F, nullptr) == CONVROT_ERR_ALIGN);
    CHECK(convrot_rotquant_act(A, 4, 1024, 16, (char *)A + 128, F, nullptr) == CONVROT_ERR_ALIGN);
    CHECK(convlinear4bit_forward(A, A, F, nullptr, 4, 4, 1024, 16, A, nullptr, 1 << 20, nullptr) == CONVROT_ERR_NULL);
    CHECK(convlinear4bit_forward(A, A, F, nullptr, 4, 4, 1024, 16, A, (char *)A + 16, 1 << 20, nullptr) == CONVROT_ERR_ALIGN);
    CHECK(convlinear4bit_forward(A, A, F, nullptr, 4, 4, 1024, 16, A, A, convrot_workspace_bytes(4, 1024) - 1, nullptr) == CONVROT_ERR_WORKSPACE);
    CHECK(convlinear8bit_forward(A, A, F, nullptr, 4, 4, 1024, 16, A, A, convrot_workspace_bytes8(4, 1024) - 1, nullptr) == CONVROT_ERR_WORKSPACE);
    CHECK(convlinear4bit_forward_noalloc(A, A, F, nullptr, 16896, 4, 12288, 16, A, nullptr) == CONVROT_ERR_WORKSPACE);
    CHECK(convlinear4bit_forward_noalloc(nullptr, A, F, nullptr, 4, 4, 1024, 16, A, nullptr) == CONVROT_ERR_NULL);
    CHECK(convrot_rotated_absmax(A, 4, 1024, 16, 3, F, nullptr) == CONVROT_ERR_GROUP);
    CHECK(convrot_unpack_codes(A, 4, 1024, (int8_t *)A + 8, nullptr) == CONVROT_ERR_ALIGN);
    // empty problems: valid, nothing launched, null matrices accepted
    CHECK(convrot_rotquant_act(nullptr, 0, 1024, 16, nullptr, nullptr, nullptr) == CONVROT_OK);
    CHECK(convrot_prepare_weight(nullptr, 0, 1024, 16, nullptr, nullptr, nullptr) == CONVROT_OK);
    CHECK(convrot_w4a4_gemm_dequant(nullptr, nullptr, A, F, nullptr, 0, 4, 1024, nullptr, nullptr) == CONVROT_OK);
    CHECK(convrot_w8a8_gemm_dequant(A, F, nullptr, nullptr, nullptr, 4, 0, 1024, nullptr, nullptr) == CONVROT_OK);
    CHECK(convrot_w4a4_gemm_i32(nullptr, A, 0, 4, 1024, nullptr, nullptr) == CONVROT_OK);
    CHECK(convrot_unpack_codes(nullptr, 0, 1024, nullptr, nullptr) == CONVROT_OK);
    CHECK(convrot_rotated_absmax(nullptr, 0, 1024, 16, 2, nullptr, nullptr) == CONVROT_OK);
    CHECK(convlinear4bit_forward_noalloc(nullptr, A, F, nullptr, 0, 4, 1024, 16, nullptr, nullptr) == CONVROT_OK);
    std::puts("C ABI host side under sanitizers: ok");
    return 0;
}
