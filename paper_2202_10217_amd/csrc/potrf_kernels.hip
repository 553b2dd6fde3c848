// potrf_kernels.hip -- Cholesky of one diagonal tile, the sequential core of Large Block Cholesky
// (the paper's Algorithm 5 calls a one-tile Cholesky for A[I0, I0]; at the bottom of the
// recursion that is Algorithm 2 on a tile held in LDS).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "potrf_kernels.h"

namespace tbs {

constexpr int kPT = 64;          // tile side
constexpr int kPLd = kPT + 1;    // padded LDS row

template <typename T>
__global__ __launch_bounds__(256) void potrf_tile_kernel(int nb, T* __restrict__ A, int64_t lda,
                                                         T* __restrict__ Linv, int32_t* info, int32_t index0)
{
    __shared__ T S[kPT * kPLd];      // working copy, trailing part updated in place
    __shared__ T L[kPT * kPLd];      // finished factor
    __shared__ T X[kPT * kPLd];      // inverse of the factor
    __shared__ int s_fail;
    const int tid = threadIdx.x;
    if (tid == 0) s_fail = -1;
    for (int e = tid; e < kPT * kPT; e += 256) {
        const int i = e / kPT, j = e - i * kPT;
        T v = (i == j) ? T(1) : T(0);                      // identity padding beyond nb
        if (i < nb && j <= i) v = A[(int64_t)i * lda + j];
        S[i * kPLd + j] = v;
        L[i * kPLd + j] = (i == j) ? T(1) : T(0);
    }
    __syncthreads();
    // right-looking elimination in the order of Algorithm 2: pivot, scale column k, rank-1 update of
    // the trailing matrix with the scaled column (the same operations on the same values as the plain
    // loops, so integer-valued factors come out exactly).
    const int ti = tid >> 2, tj0 = tid & 3;
    for (int k = 0; k < nb; ++k) {
        const T p = S[k * kPLd + k];
        if (!(p > T(0))) {
            if (tid == 0) s_fail = k;
            break;                                          // p is the same for every thread
        }
        const T d = sqrt(p);
        if (tid >= k && tid < nb) L[tid * kPLd + k] = (tid == k) ? d : S[tid * kPLd + k] / d;
        __syncthreads();
        if (ti > k && ti < nb) {
            const T lik = L[ti * kPLd + k];
            for (int j = k + 1 + tj0; j <= ti; j += 4) S[ti * kPLd + j] -= lik * L[j * kPLd + k];
        }
        __syncthreads();
    }
    __syncthreads();
    const int fail = s_fail;
    if (fail >= 0) {
        if (tid == 0 && *info == 0) *info = index0 + fail + 1;
    }
    // write back the columns that were finished (all of them when nothing failed)
    const int ncol = (fail >= 0) ? fail : nb;
    for (int e = tid; e < kPT * kPT; e += 256) {
        const int i = e / kPT, j = e - i * kPT;
        if (i < nb && j <= i && j < ncol) A[(int64_t)i * lda + j] = L[i * kPLd + j];
    }
    // inverse of L by forward substitution, one column per thread: L x = e_j
    if (tid < kPT) {
        const int j = tid;
        for (int i = 0; i < kPT; ++i) {
            T s = (i == j) ? T(1) : T(0);
            for (int m = j; m < i; ++m) s -= L[i * kPLd + m] * X[m * kPLd + j];
            X[i * kPLd + j] = (i < j) ? T(0) : s / L[i * kPLd + i];
        }
    }
    __syncthreads();
    for (int e = tid; e < kPT * kPT; e += 256) {
        const int i = e / kPT, j = e - i * kPT;
        Linv[i * kPT + j] = X[i * kPLd + j];
    }
}

__global__ void fill_i32_kernel(int32_t* dst, int32_t value, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = value;
}

hipError_t launch_fill_i32(int32_t* dst, int32_t value, int n, hipStream_t stream)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(fill_i32_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, dst, value, n);
    return hipGetLastError();
}

hipError_t launch_potrf_tile(bool f32, int nb, void* A, int64_t lda, void* Linv, int32_t* info,
                             int32_t index0, hipStream_t stream)
{
    if (nb <= 0) return hipSuccess;
    if (f32)
        hipLaunchKernelGGL(potrf_tile_kernel<float>, dim3(1), dim3(256), 0, stream, nb, (float*)A, lda,
                           (float*)Linv, info, index0);
    else
        hipLaunchKernelGGL(potrf_tile_kernel<double>, dim3(1), dim3(256), 0, stream, nb, (double*)A, lda,
                           (double*)Linv, info, index0);
    return hipGetLastError();
}

}  // namespace tbs
