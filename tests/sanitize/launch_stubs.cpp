// Stand-ins for the kernel launchers, so that the host side of the C ABI (argument validation, size
// queries, the per-device workspace bookkeeping) can be built with host sanitizers and run without a GPU.
// The driver only makes calls that validation rejects or that are no-ops; a launcher being reached with work
// to do is a failure of that validation, so these abort.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <cstdio>
#include <cstdlib>

#include "convrot_internal.h"

namespace convrot {

static hipError_t reached(const char *what, int64_t rows)
{
    if (rows == 0) return hipSuccess;
    std::fprintf(stderr, "launcher %s reached with %lld rows\n", what, (long long)rows);
    std::abort();
}

hipError_t launch_rotquant(const void *, int64_t rows, int64_t, int, int, void *, float *, hipStream_t) { return reached("rotquant", rows); }
hipError_t launch_unpack_codes(const void *, int64_t rows, int64_t, int8_t *, hipStream_t) { return reached("unpack_codes", rows); }
hipError_t launch_rotated_absmax(const void *, int64_t rows, int64_t, int, int, float *, hipStream_t) { return reached("rotated_absmax", rows); }
hipError_t launch_gemm_w4a4(const void *, const float *, const void *, const float *, const void *, int64_t M, int64_t N, int64_t,
                            void *, int32_t *, hipStream_t) { return reached("gemm_w4a4", M * N); }
hipError_t launch_gemm_w8a8(const void *, const float *, const void *, const float *, const void *, int64_t M, int64_t N, int64_t,
                            void *, int32_t *, hipStream_t) { return reached("gemm_w8a8", M * N); }

}  // namespace convrot
