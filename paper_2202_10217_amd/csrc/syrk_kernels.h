// syrk_kernels.h -- launch interface of the Triangle Block SYRK kernels (device code in the .hip).
#pragma once
#include <hip/hip_runtime_api.h>
#include <stdint.h>

#include "tbs_plan.h"

namespace tbs {

constexpr int kSliceCounters = 512;      // cut blocks per plan (one device counter each)
constexpr int kLaunchCounters = 16;      // of a persistent launch: next block, workgroups done, one per die

// The device counters one launch may use: the kLaunchCounters of the persistent form, the counters of
// the cut blocks, and the event that completes with the launch.  Empty (all null): none could be given.
struct CounterLease {
    unsigned int* ctr = nullptr;
    unsigned int* slice_ctr = nullptr;
    hipEvent_t done = nullptr;
};

// Counters for the next launch on `stream` on the current device.  Launches on one stream share a
// set (they run one after the other); another stream gets a set of its own, or one whose last launch
// has finished; if every set belongs to a launch that may still be running, *out stays empty and the
// caller must launch the form that needs none (max_workgroups <= 0 and a plan without cut blocks).
// Calls no allocation routine except for one event per set, created when the set is first handed out.
hipError_t acquire_counters(hipStream_t stream, CounterLease* out);

// The library's own scratch memory for callers that cannot allocate: a file-scope array in device
// memory, kStaticCounterBytes for the counters of one launch followed by kStaticWorkspaceBytes for the
// parts of cut blocks.  *ptr receives its device address on the current device (looked up once per
// device).  Every call on a device shares the one array.
constexpr size_t kStaticCounterBytes = 4096;
constexpr size_t kStaticWorkspaceBytes = (size_t)128 << 20;
hipError_t static_scratch(unsigned char** ptr);

// An operand matrix as the kernels address it: element (row, k) of its panels is p[row * rs + k * ks]
// (device pointer).  A row-major N x M matrix with the contraction along its rows: rs = leading
// dimension, ks = 1.  The Gram form A^T A of a row-major matrix (panel row = column of A, contraction
// down its rows): rs = 1, ks = leading dimension.
struct OperandDesc {
    const void* p;
    int64_t rs, ks;
};

// C[lower] <- beta*C + alpha*A*A^T for the blocks of `plan`; C is N x N, the contraction has length M.
// All pointers are device pointers; sizes have been validated by the caller.  max_workgroups > 0
// bounds the launch: a plan with more blocks
// runs as that many persistent workgroups taking blocks in list order (normally the number of
// compute units; fewer leaves units free for kernels of other streams); <= 0: one workgroup per block.
// The persistent form and plans with cut blocks need a lease from acquire_counters (same stream).
// A plan with sliced blocks needs `workspace`: device memory of syrk_workspace_bytes(), aligned to the
// element size, contents arbitrary; it is only written and read by this launch.
hipError_t launch_syrk(bool f32, const Plan& plan, int64_t N, int64_t M, double alpha, const OperandDesc& a,
                       double beta, void* C, int64_t ldc, int max_workgroups, void* workspace,
                       const CounterLease& lease, hipStream_t stream);

// C[lower] <- beta*C + alpha*(A*B^T + B*A^T): every block runs over the contraction dimension twice,
// (A rows, B columns) then (B rows, A columns), into the same accumulators.  The plan must consist of
// rectangular blocks (no triangle blocks, no cut blocks); hipErrorInvalidValue otherwise.
hipError_t launch_syr2k(bool f32, const Plan& plan, int64_t N, int64_t M, double alpha, const OperandDesc& a,
                        const OperandDesc& b, double beta, void* C, int64_t ldc, int max_workgroups,
                        const CounterLease& lease, hipStream_t stream);
size_t syrk_workspace_bytes(bool f32, const Plan& plan);

// C (m x n) <- beta*C + alpha * R (m x K) * Q (n x K)^T, all row-major device matrices that do not
// overlap.  `units`: compute units the launch can expect to have (sets the block shape).
hipError_t launch_gemm_nt(bool f32, int64_t m, int64_t n, int64_t K, double alpha, const void* R,
                          int64_t ldr, const void* Q, int64_t ldq, double beta, void* C, int64_t ldc,
                          int units, hipStream_t stream);

}  // namespace tbs
