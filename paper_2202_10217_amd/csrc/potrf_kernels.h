// potrf_kernels.h -- launch interface of the diagonal-tile Cholesky kernel.
#pragma once
#include <hip/hip_runtime_api.h>
#include <stdint.h>

namespace tbs {

// Factors the nb x nb (nb <= 64) diagonal tile at A in place (lower triangle; Algorithm 2 on one
// tile) and writes the inverse of the factor, a 64 x 64 row-major lower triangular matrix (identity
// beyond nb), to Linv.  A pivot that is not > 0 stores index0 + (its 0-based index) + 1 into *info
// if *info is still 0, and leaves the rest of the tile unfactored.  All pointers: device.
hipError_t launch_potrf_tile(bool f32, int nb, void* A, int64_t lda, void* Linv, int32_t* info,
                             int32_t index0, hipStream_t stream);

// dst[0..n) = value, as a kernel (safe to record into a HIP graph, unlike a memset node).
hipError_t launch_fill_i32(int32_t* dst, int32_t value, int n, hipStream_t stream);

}  // namespace tbs
