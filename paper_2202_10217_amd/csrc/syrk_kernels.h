// syrk_kernels.h -- launch interface of the Triangle Block SYRK kernels (device code in the .hip).
#pragma once
#include <hip/hip_runtime_api.h>
#include <stdint.h>

#include "tbs_plan.h"

namespace tbs {

// C[lower] <- beta*C + alpha*A*A^T for the blocks of `plan`.  All pointers are device pointers; sizes
// have been validated by the caller.  max_workgroups > 0 bounds the launch: a plan with more blocks
// runs as that many persistent workgroups taking blocks in list order (normally the number of
// compute units; fewer leaves units free for kernels of other streams); <= 0: one workgroup per block.
// A plan with sliced blocks needs `workspace`: device memory of syrk_workspace_bytes(), aligned to the
// element size, contents arbitrary; it is only written and read by this launch.
hipError_t launch_syrk(bool f32, const Plan& plan, int64_t N, int64_t M, double alpha, const void* A,
                       int64_t lda, double beta, void* C, int64_t ldc, int max_workgroups, void* workspace,
                       hipStream_t stream);
size_t syrk_workspace_bytes(bool f32, const Plan& plan);

// C (m x n) <- beta*C + alpha * R (m x K) * Q (n x K)^T, all row-major device matrices that do not
// overlap.  `units`: compute units the launch can expect to have (sets the block shape).
hipError_t launch_gemm_nt(bool f32, int64_t m, int64_t n, int64_t K, double alpha, const void* R,
                          int64_t ldr, const void* Q, int64_t ldq, double beta, void* C, int64_t ldc,
                          int units, hipStream_t stream);

}  // namespace tbs
