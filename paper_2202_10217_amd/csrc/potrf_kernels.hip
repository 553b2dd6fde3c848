// potrf_kernels.hip -- Cholesky of one diagonal tile, the sequential core of Large Block Cholesky
// (the paper's Algorithm 5 calls a one-tile Cholesky for A[I0, I0]; at the bottom of the
// recursion that is Algorithm 2 on a tile held in LDS).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "potrf_kernels.h"

namespace tbs {

constexpr int kPT = 64;          // tile side
constexpr int kPLd = kPT + 1;    // padded LDS row

// Thread (i, q) = (tid / 4, tid % 4) keeps the elements j = 4 m + q, m = 0..15, of row i of the
// working matrix S and of the inverse X in registers for the whole factorisation.  A step needs two
// things from other threads, both broadcast through LDS: the scaled column k of L (stored so that
// the 16 values a thread needs are contiguous) and row k of X.  The elimination loop is unrolled
// completely, so every register index is a constant and a step only touches the columns that still
// change (j > k of S, j <= k of X).
//
// The operations on S are those of Algorithm 2 in its order (pivot, scale column k by division,
// rank-1 update with the scaled column), so integer-valued factors come out exactly.  The inverse is
// built in the same sweep: L X = I solved by eliminating column k of L from the rows below row k.
// One elimination step; K is a compile-time constant so that every register index is static.
template <typename T, int K>
__device__ __forceinline__ void tile_step(T (&s)[16], T (&x)[16], T* colL, T* rowX, T* pivot, int& fail,
                                          int i, int q, int perm_i)
{
    constexpr int km = K >> 2, kq = K & 3;
    T p = *pivot;
    if (!(p > T(0))) {                                      // uniform: every thread reads the same p
        if (fail < 0) fail = K;
        p = T(1);                                           // keep going on finite numbers; the output
    }                                                       // from column `fail` on is unspecified
    const T d = sqrt(p);
    if (q == kq) {                                          // owners of column K
        const T a = s[km];
        const T l = (i > K) ? a / d : d;
        if (i >= K) s[km] = l;
        colL[perm_i] = (i > K) ? l : T(0);
    }
    if (i == K) {                                           // owners of row K of X
        const T r = T(1) / d;
#pragma unroll
        for (int m = 0; m < 16; ++m) {
            if (m <= km) x[m] *= r;
            rowX[q * 16 + m] = x[m];
        }
    }
    __syncthreads();
    if ((i | 15) > K) {                                     // wavefronts whose 16 rows are all <= K idle
        const T lik = colL[perm_i];
#pragma unroll
        for (int m = 0; m < 16; ++m) {
            if (m >= km) s[m] -= lik * colL[q * 16 + m];    // columns j > K (entries for j <= K are 0)
            if (m <= km) x[m] -= lik * rowX[q * 16 + m];    // columns j <= K
        }
    }
    if (K + 1 < kPT && i == K + 1 && q == ((K + 1) & 3)) *pivot = s[((K + 1) >> 2) & 15];
    __syncthreads();
}

template <typename T, int K>
struct TileSteps {
    static __device__ __forceinline__ void run(int nb, T (&s)[16], T (&x)[16], T* colL, T* rowX, T* pivot,
                                               int& fail, int i, int q, int perm_i)
    {
        if constexpr (K < kPT) {
            if (K < nb) {                                   // uniform
                tile_step<T, K>(s, x, colL, rowX, pivot, fail, i, q, perm_i);
                TileSteps<T, K + 1>::run(nb, s, x, colL, rowX, pivot, fail, i, q, perm_i);
            }
        }
    }
};

// Thread (i, q) = (tid / 4, tid % 4) keeps the elements j = 4 m + q, m = 0..15, of row i of the
// working matrix S and of the inverse X in registers for the whole factorisation.  A step needs two
// things from other threads, both broadcast through LDS: the scaled column k of L (stored so that
// the 16 values a thread needs are contiguous) and row k of X.  The elimination loop is unrolled
// completely (template recursion), so every register index is a constant and a step only touches
// the columns that still change (j > k of S, j <= k of X).
//
// The operations on S are those of Algorithm 2 in its order (pivot, scale column k by division,
// rank-1 update with the scaled column), so integer-valued factors come out exactly.  The inverse is
// built in the same sweep: L X = I solved by eliminating column k of L from the rows below row k.
template <typename T>
__global__ __launch_bounds__(256) void potrf_tile_kernel(int nb, T* __restrict__ A, int64_t lda,
                                                         T* __restrict__ Linv, int32_t* info, int32_t index0)
{
    __shared__ T colL[kPT];          // scaled column k, entry of row j at [(j % 4) * 16 + j / 4]; 0 for j <= k
    __shared__ T rowX[kPT];          // row k of X, same permutation; 0 for j > k
    __shared__ T pivot;              // S[k][k] entering step k
    const int tid = threadIdx.x;
    const int i = tid >> 2, q = tid & 3;
    const int perm_i = (i & 3) * 16 + (i >> 2);
    T s[16], x[16];
#pragma unroll
    for (int m = 0; m < 16; ++m) {
        const int j = 4 * m + q;
        T v = (i == j) ? T(1) : T(0);                      // identity padding beyond nb
        if (i < nb && j <= i) v = A[(int64_t)i * lda + j];
        s[m] = v;
        x[m] = (i == j) ? T(1) : T(0);
    }
    if (tid == 0) pivot = s[0];
    int fail = -1;
    __syncthreads();
    TileSteps<T, 0>::run(nb, s, x, colL, rowX, &pivot, fail, i, q, perm_i);
    if (fail >= 0 && tid == 0 && *info == 0) *info = index0 + fail + 1;
    // write back the columns that were finished (all of them when nothing failed); the inverse is
    // meaningful only then
    const int ncol = (fail >= 0) ? fail : nb;
#pragma unroll
    for (int m = 0; m < 16; ++m) {
        const int j = 4 * m + q;
        if (i < nb && j <= i && j < ncol) A[(int64_t)i * lda + j] = s[m];
        Linv[i * kPT + j] = (j <= i) ? x[m] : T(0);
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
