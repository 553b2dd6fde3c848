// potrf_kernels.h -- launch interface of the diagonal-tile Cholesky kernel.
#pragma once
#include <hip/hip_runtime_api.h>
#include <stdint.h>

namespace tbs {

// Factors the nb x nb (nb <= 64) diagonal tile at A in place (lower triangle; Algorithm 2 on one
// tile).  A pivot that is not > 0 stores index0 + (its 0-based index) + 1 into *info if *info is
// still 0; the columns from that one on are then unspecified.  All pointers: device.
hipError_t launch_potrf_tile(bool f32, int nb, void* A, int64_t lda, int32_t* info, int32_t index0,
                             hipStream_t stream);

// The same for a diagonal block of n <= 128 columns, in one workgroup (factor the first tile, solve and
// update the second, factor it).  Returns hipErrorInvalidValue for n > 128.  `done` (optional): an event
// that happens when the block is factored.
hipError_t launch_potrf_block(bool f32, int n, void* A, int64_t lda, int32_t* info, int32_t index0,
                              hipStream_t stream, hipEvent_t done = nullptr);

// X (m x nb, nb <= 64) <- X * L^{-T} by forward substitution, L the lower triangular nb x nb tile at
// `L` (leading dimension ldl); X in place.  The column-scaling and update steps of Algorithm 2 for
// the rows below a diagonal tile.
hipError_t launch_trsm_tile(bool f32, int64_t m, int nb, const void* L, int64_t ldl, void* X, int64_t ldx,
                            hipStream_t stream);

// The same for a lower triangular block L of n <= 512 columns (n x n, leading dimension ldl): one launch,
// every workgroup takes 32 rows of X through all tile columns.  Returns hipErrorInvalidValue for n > 512.
hipError_t launch_trsm_panel(bool f32, int64_t m, int n, const void* L, int64_t ldl, void* X, int64_t ldx,
                             hipStream_t stream);

// dst[0..n) = value, as a kernel (safe to record into a HIP graph, unlike a memset node).
hipError_t launch_fill_i32(int32_t* dst, int32_t value, int n, hipStream_t stream);

}  // namespace tbs
