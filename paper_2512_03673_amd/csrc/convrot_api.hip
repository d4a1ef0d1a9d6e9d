// C ABI of libconvrot (see include/convrot.h): argument validation on the host, then launches.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <mutex>

#include "convrot.h"
#include "convrot_internal.h"
#include "e2m3_layout.h"
#include "panel_layout.h"

namespace {

inline bool aligned(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

int check_group(int g) { return (g == 4 || g == 16 || g == 64 || g == 256 || g == 1024) ? CONVROT_OK : CONVROT_ERR_GROUP; }

int check_k(int64_t K) { return (K > 0 && K <= CONVROT_MAX_K && K % 32 == 0) ? CONVROT_OK : CONVROT_ERR_SHAPE; }

// A matrix with zero rows may come with a null pointer (an empty allocation has no address).
inline bool missing(const void *p, int64_t rows) { return rows > 0 && !p; }

int check_rotquant(const void *in, int64_t rows, int64_t K, int group, const void *out, const float *scale)
{
    if (int rc = check_group(group)) return rc;
    if (rows < 0 || rows > INT32_MAX) return CONVROT_ERR_SHAPE;
    if (int rc = check_k(K)) return rc;
    if (K % group != 0) return CONVROT_ERR_SHAPE;
    if (missing(in, rows) || missing(out, rows) || missing(scale, rows)) return CONVROT_ERR_NULL;
    if (!aligned(in, 16) || !aligned(out, 256) || !aligned(scale, 4)) return CONVROT_ERR_ALIGN;
    return CONVROT_OK;
}

int check_gemm(const void *Xq, const void *Wq, int64_t M, int64_t N, int64_t K, const void *out, uintptr_t out_align)
{
    if (M < 0 || N < 0 || M > INT32_MAX || N > INT32_MAX) return CONVROT_ERR_SHAPE;
    if (int rc = check_k(K)) return rc;
    if (missing(Xq, M) || missing(Wq, N) || missing(out, M * N)) return CONVROT_ERR_NULL;
    if (!aligned(Xq, 256) || !aligned(Wq, 256) || !aligned(out, out_align)) return CONVROT_ERR_ALIGN;
    return CONVROT_OK;
}

inline int from_hip(hipError_t e) { return e == hipSuccess ? CONVROT_OK : CONVROT_ERR_HIP; }

// ---- the static workspace of convlinear4bit_forward_noalloc.  Every device the library's code is loaded
// on holds its own copy of this array at its own address, until the process ends.  In host code the
// name `scratch` is only a handle for hipGetSymbolAddress: the device address it yields (per device)
// is what kernels get.
static __device__ __align__(256) uint8_t scratch[CONVROT_NOALLOC_WORKSPACE_BYTES];

constexpr int kMaxDevices = 64;
std::atomic<uint8_t *> g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_mutex;

// Device address of `scratch` on the calling thread's current device (resolved once per device).
int scratch_of_current_device(uint8_t **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return CONVROT_ERR_HIP;
    uint8_t *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        p = g_scratch_ptr[dev].load(std::memory_order_relaxed);
        if (!p) {
            void *q = nullptr;
            if (hipGetSymbolAddress(&q, HIP_SYMBOL(scratch)) != hipSuccess || !q) return CONVROT_ERR_HIP;
            p = static_cast<uint8_t *>(q);
            g_scratch_ptr[dev].store(p, std::memory_order_release);
        }
    }
    *out = p;
    return CONVROT_OK;
}

// Argument checks shared by the fused forward calls (everything but the workspace).
int check_forward(const void *X_bf16, const void *Wq, const float *w_scale, const void *bias_bf16, int64_t M, int64_t N,
                  int64_t K, int group, const void *Y_bf16)
{
    if (int rc = check_group(group)) return rc;
    if (M < 0 || N < 0 || M > INT32_MAX || N > INT32_MAX) return CONVROT_ERR_SHAPE;
    if (int rc = check_k(K)) return rc;
    if (K % group != 0) return CONVROT_ERR_SHAPE;
    if (missing(X_bf16, M) || missing(Wq, N) || missing(w_scale, N) || missing(Y_bf16, M * N)) return CONVROT_ERR_NULL;
    if (!aligned(X_bf16, 16) || !aligned(Wq, 256) || !aligned(Y_bf16, 16) || !aligned(w_scale, 4) || !aligned(bias_bf16, 2))
        return CONVROT_ERR_ALIGN;
    return CONVROT_OK;
}

}  // namespace

extern "C" {

const char *convrot_status_string(int status)
{
    switch (status) {
        case CONVROT_OK: return "ok";
        case CONVROT_ERR_NULL: return "null pointer";
        case CONVROT_ERR_SHAPE: return "bad shape (need M,N >= 0, 0 < K <= 65536, K % 32 == 0, K % group == 0)";
        case CONVROT_ERR_GROUP: return "bad group size (need 4, 16, 64, 256 or 1024)";
        case CONVROT_ERR_ALIGN: return "misaligned pointer";
        case CONVROT_ERR_WORKSPACE: return "workspace too small";
        case CONVROT_ERR_HIP: return "HIP launch failed";
        default: return "unknown status";
    }
}

int convrot_version(void) { return CONVROT_VERSION; }

#define CONVROT_STR2(x) #x
#define CONVROT_STR(x) CONVROT_STR2(x)
const char *convrot_build_info(void)
{
    return "clang " __clang_version__ ", HIP " CONVROT_STR(HIP_VERSION_MAJOR) "." CONVROT_STR(HIP_VERSION_MINOR) "." CONVROT_STR(HIP_VERSION_PATCH);
}

int convrot_init(void)
{
    uint8_t *p = nullptr;
    return scratch_of_current_device(&p);
}

int convrot_gemm_tile_rows(int64_t M, int64_t N)
{
    if (M < 0 || N < 0) return 0;
    return convrot::gemm_tile_rows(M, N);
}

size_t convrot_packed_bytes(int64_t rows, int64_t K)
{
    if (rows < 0 || K <= 0 || (K & 1)) return 0;
    return (size_t)convrot::e2m3::matrix_bytes(rows, K);
}

size_t convrot_packed_bytes8(int64_t rows, int64_t K)
{
    if (rows < 0 || K <= 0) return 0;
    return (size_t)convrot::panel::matrix_bytes(rows, K);
}

size_t convrot_workspace_bytes(int64_t M, int64_t K)
{
    if (M < 0 || K <= 0 || (K & 1)) return 0;
    return convrot_packed_bytes(M, K) + round_up((size_t)M * sizeof(float), 256);
}

int convrot_prepare_weight(const void *W_bf16, int64_t N, int64_t K, int group, void *Wq, float *w_scale,
                           void *stream)
{
    if (int rc = check_rotquant(W_bf16, N, K, group, Wq, w_scale)) return rc;
    return from_hip(convrot::launch_rotquant(W_bf16, N, K, group, 4, Wq, w_scale, (hipStream_t)stream));
}

int convrot_rotquant_act(const void *X_bf16, int64_t M, int64_t K, int group, void *Xq, float *x_scale,
                         void *stream)
{
    if (int rc = check_rotquant(X_bf16, M, K, group, Xq, x_scale)) return rc;
    return from_hip(convrot::launch_rotquant(X_bf16, M, K, group, 4, Xq, x_scale, (hipStream_t)stream));
}

int convrot_w4a4_gemm_dequant(const void *Xq, const float *x_scale, const void *Wq, const float *w_scale,
                              const void *bias_bf16, int64_t M, int64_t N, int64_t K, void *Y_bf16, void *stream)
{
    if (int rc = check_gemm(Xq, Wq, M, N, K, Y_bf16, 16)) return rc;
    if (missing(x_scale, M) || missing(w_scale, N)) return CONVROT_ERR_NULL;
    if (!aligned(x_scale, 4) || !aligned(w_scale, 4) || !aligned(bias_bf16, 2)) return CONVROT_ERR_ALIGN;
    return from_hip(convrot::launch_gemm_w4a4(Xq, x_scale, Wq, w_scale, bias_bf16, M, N, K, Y_bf16, nullptr,
                                              (hipStream_t)stream));
}

int convrot_w4a4_gemm_i32(const void *Xq, const void *Wq, int64_t M, int64_t N, int64_t K, int32_t *acc,
                          void *stream)
{
    if (int rc = check_gemm(Xq, Wq, M, N, K, acc, 16)) return rc;
    return from_hip(convrot::launch_gemm_w4a4(Xq, nullptr, Wq, nullptr, nullptr, M, N, K, nullptr, acc, (hipStream_t)stream));
}

int convrot_unpack_codes(const void *Xq, int64_t rows, int64_t K, int8_t *codes, void *stream)
{
    if (rows < 0 || rows > INT32_MAX) return CONVROT_ERR_SHAPE;
    if (int rc = check_k(K)) return rc;
    if (missing(Xq, rows) || missing(codes, rows)) return CONVROT_ERR_NULL;
    if (!aligned(Xq, 256) || !aligned(codes, 16)) return CONVROT_ERR_ALIGN;
    return from_hip(convrot::launch_unpack_codes(Xq, rows, K, codes, (hipStream_t)stream));
}

int convlinear4bit_forward(const void *X_bf16, const void *Wq, const float *w_scale, const void *bias_bf16,
                           int64_t M, int64_t N, int64_t K, int group, void *Y_bf16, void *workspace,
                           size_t workspace_bytes, void *stream)
{
    if (int rc = check_forward(X_bf16, Wq, w_scale, bias_bf16, M, N, K, group, Y_bf16)) return rc;
    if (missing(workspace, M)) return CONVROT_ERR_NULL;
    if (!aligned(workspace, 256)) return CONVROT_ERR_ALIGN;
    if (workspace_bytes < convrot_workspace_bytes(M, K)) return CONVROT_ERR_WORKSPACE;

    uint8_t *xq = static_cast<uint8_t *>(workspace);
    float *xs = reinterpret_cast<float *>(xq + convrot_packed_bytes(M, K));
    hipStream_t s = (hipStream_t)stream;
    if (hipError_t e = convrot::launch_rotquant(X_bf16, M, K, group, 4, xq, xs, s); e != hipSuccess) return CONVROT_ERR_HIP;
    return from_hip(convrot::launch_gemm_w4a4(xq, xs, Wq, w_scale, bias_bf16, M, N, K, Y_bf16, nullptr, s));
}

int convlinear4bit_forward_noalloc(const void *X_bf16, const void *Wq, const float *w_scale, const void *bias_bf16,
                                   int64_t M, int64_t N, int64_t K, int group, void *Y_bf16, void *stream)
{
    if (int rc = check_forward(X_bf16, Wq, w_scale, bias_bf16, M, N, K, group, Y_bf16)) return rc;
    if (convrot_workspace_bytes(M, K) > CONVROT_NOALLOC_WORKSPACE_BYTES) return CONVROT_ERR_WORKSPACE;
    if (M == 0 || N == 0) return CONVROT_OK;
    uint8_t *xq = nullptr;
    if (int rc = scratch_of_current_device(&xq)) return rc;
    // Nothing in the array has to start at zero: the rotate+quantise kernel writes every byte of the rows below M
    // (K padding included) and all M scales before the GEMM reads them; what an earlier call left in the rows
    // past M of the last 32-row block only ever meets accumulators that are not stored.
    float *xs = reinterpret_cast<float *>(xq + convrot_packed_bytes(M, K));
    hipStream_t s = (hipStream_t)stream;
    if (hipError_t e = convrot::launch_rotquant(X_bf16, M, K, group, 4, xq, xs, s); e != hipSuccess) return CONVROT_ERR_HIP;
    return from_hip(convrot::launch_gemm_w4a4(xq, xs, Wq, w_scale, bias_bf16, M, N, K, Y_bf16, nullptr, s));
}

int convrot_rotated_absmax(const void *X_bf16, int64_t M, int64_t K, int group, int kind, float *row_absmax,
                           void *stream)
{
    if (int rc = check_group(group)) return rc;
    if (kind < 0 || kind > 2) return CONVROT_ERR_GROUP;
    if (M < 0 || M > INT32_MAX) return CONVROT_ERR_SHAPE;
    if (int rc = check_k(K)) return rc;
    if (K % group != 0) return CONVROT_ERR_SHAPE;
    if (missing(X_bf16, M) || missing(row_absmax, M)) return CONVROT_ERR_NULL;
    if (!aligned(X_bf16, 16) || !aligned(row_absmax, 4)) return CONVROT_ERR_ALIGN;
    return from_hip(convrot::launch_rotated_absmax(X_bf16, M, K, group, kind, row_absmax, (hipStream_t)stream));
}

// ---- W8A8 variant

size_t convrot_workspace_bytes8(int64_t M, int64_t K)
{
    if (M < 0 || K <= 0) return 0;
    return convrot_packed_bytes8(M, K) + round_up((size_t)M * sizeof(float), 256);
}

int convrot_prepare_weight8(const void *W_bf16, int64_t N, int64_t K, int group, void *Wq, float *w_scale,
                            void *stream)
{
    if (int rc = check_rotquant(W_bf16, N, K, group, Wq, w_scale)) return rc;
    return from_hip(convrot::launch_rotquant(W_bf16, N, K, group, 8, Wq, w_scale, (hipStream_t)stream));
}

int convrot_rotquant_act8(const void *X_bf16, int64_t M, int64_t K, int group, void *Xq, float *x_scale,
                          void *stream)
{
    if (int rc = check_rotquant(X_bf16, M, K, group, Xq, x_scale)) return rc;
    return from_hip(convrot::launch_rotquant(X_bf16, M, K, group, 8, Xq, x_scale, (hipStream_t)stream));
}

int convrot_w8a8_gemm_dequant(const void *Xq, const float *x_scale, const void *Wq, const float *w_scale,
                              const void *bias_bf16, int64_t M, int64_t N, int64_t K, void *Y_bf16, void *stream)
{
    if (int rc = check_gemm(Xq, Wq, M, N, K, Y_bf16, 16)) return rc;
    if (missing(x_scale, M) || missing(w_scale, N)) return CONVROT_ERR_NULL;
    if (!aligned(x_scale, 4) || !aligned(w_scale, 4) || !aligned(bias_bf16, 2)) return CONVROT_ERR_ALIGN;
    return from_hip(convrot::launch_gemm_w8a8(Xq, x_scale, Wq, w_scale, bias_bf16, M, N, K, Y_bf16, nullptr,
                                              (hipStream_t)stream));
}

int convrot_w8a8_gemm_i32(const void *Xq, const void *Wq, int64_t M, int64_t N, int64_t K, int32_t *acc,
                          void *stream)
{
    if (int rc = check_gemm(Xq, Wq, M, N, K, acc, 16)) return rc;
    return from_hip(convrot::launch_gemm_w8a8(Xq, nullptr, Wq, nullptr, nullptr, M, N, K, nullptr, acc,
                                              (hipStream_t)stream));
}

int convlinear8bit_forward(const void *X_bf16, const void *Wq, const float *w_scale, const void *bias_bf16,
                           int64_t M, int64_t N, int64_t K, int group, void *Y_bf16, void *workspace,
                           size_t workspace_bytes, void *stream)
{
    if (int rc = check_forward(X_bf16, Wq, w_scale, bias_bf16, M, N, K, group, Y_bf16)) return rc;
    if (missing(workspace, M)) return CONVROT_ERR_NULL;
    if (!aligned(workspace, 256)) return CONVROT_ERR_ALIGN;
    if (workspace_bytes < convrot_workspace_bytes8(M, K)) return CONVROT_ERR_WORKSPACE;

    uint8_t *xq = static_cast<uint8_t *>(workspace);
    float *xs = reinterpret_cast<float *>(xq + convrot_packed_bytes8(M, K));
    hipStream_t s = (hipStream_t)stream;
    if (hipError_t e = convrot::launch_rotquant(X_bf16, M, K, group, 8, xq, xs, s); e != hipSuccess) return CONVROT_ERR_HIP;
    return from_hip(convrot::launch_gemm_w8a8(xq, xs, Wq, w_scale, bias_bf16, M, N, K, Y_bf16, nullptr, s));
}

}  // extern "C"
