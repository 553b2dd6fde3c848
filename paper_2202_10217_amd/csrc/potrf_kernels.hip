// potrf_kernels.hip -- Cholesky of one diagonal tile, the sequential core of Large Block Cholesky
// (the paper's Algorithm 5 calls a one-tile Cholesky for A[I0, I0]; at the bottom of the
// recursion that is Algorithm 2 on a tile held in LDS).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "potrf_kernels.h"

namespace tbs {

constexpr int kPT = 64;          // tile side
constexpr int kPLd = kPT + 1;    // padded LDS row

// One elimination step; K is a compile-time constant so that every register index is static.
template <typename T, int K>
__device__ __forceinline__ void tile_step(T (&s)[16], T* colL, T* pivot, int& fail, int i, int q, int perm_i)
{
    constexpr int km = K >> 2, kq = K & 3;
    T p = *pivot;
    if (!(p > T(0))) {                                      // uniform: every thread reads the same p
        if (fail < 0) fail = K;
        p = T(1);                                           // keep going on finite numbers; the output
    }                                                       // from column `fail` on is unspecified
    // d = sqrt(p) and r = 1/d once per step; column entries are a/d computed as a*r followed by one
    // residual correction (q + r*(a - q*d)), which returns the correctly rounded quotient whenever it
    // is representable exactly -- in particular integer factors stay exact -- without a division
    // sequence on the critical path of every step.
    const T d = sqrt(p);
    const T r = T(1) / d;
    if (q == kq) {                                          // owners of column K
        const T a = s[km];
        const T q0 = a * r;
        const T l = (i > K) ? fma(fma(-q0, d, a), r, q0) : d;
        if (i >= K) s[km] = l;
        colL[perm_i] = (i > K) ? l : T(0);
    }
    __syncthreads();
    if ((i | 15) > K) {                                     // wavefronts whose 16 rows are all <= K idle
        const T lik = colL[perm_i];
#pragma unroll
        for (int m = 0; m < 16; ++m)
            if (m >= km) s[m] -= lik * colL[q * 16 + m];    // columns j > K (entries for j <= K are 0)
    }
    if (K + 1 < kPT && i == K + 1 && q == ((K + 1) & 3)) *pivot = s[((K + 1) >> 2) & 15];
    __syncthreads();
}

template <typename T, int K>
struct TileSteps {
    static __device__ __forceinline__ void run(int nb, T (&s)[16], T* colL, T* pivot, int& fail, int i, int q,
                                               int perm_i)
    {
        if constexpr (K < kPT) {
            if (K < nb) {                                   // uniform
                tile_step<T, K>(s, colL, pivot, fail, i, q, perm_i);
                TileSteps<T, K + 1>::run(nb, s, colL, pivot, fail, i, q, perm_i);
            }
        }
    }
};

// Thread (i, q) = (tid / 4, tid % 4) keeps the elements j = 4 m + q, m = 0..15, of row i of the
// working matrix in registers for the whole factorisation.  A step needs one thing from other
// threads, broadcast through LDS: the scaled column k of L (stored so that the 16 values a thread
// needs are contiguous).  The elimination loop is unrolled completely (template recursion), so every
// register index is a constant and a step only touches the columns that still change (j > k).
//
// The operations are those of Algorithm 2 in its order (pivot, scale column k, rank-1 update with the
// scaled column), so integer-valued factors come out exactly.
template <typename T>
__global__ __launch_bounds__(256) void potrf_tile_kernel(int nb, T* __restrict__ A, int64_t lda, int32_t* info,
                                                         int32_t index0)
{
    __shared__ T colL[kPT];          // scaled column k, entry of row j at [(j % 4) * 16 + j / 4]; 0 for j <= k
    __shared__ T pivot;              // S[k][k] entering step k
    const int tid = threadIdx.x;
    const int i = tid >> 2, q = tid & 3;
    const int perm_i = (i & 3) * 16 + (i >> 2);
    T s[16];
#pragma unroll
    for (int m = 0; m < 16; ++m) {
        const int j = 4 * m + q;
        const int ic = min(i, nb - 1), jc = min(j, ic);    // unconditional loads on clamped addresses
        const T a = A[(int64_t)ic * lda + jc];
        s[m] = (i < nb && j <= i) ? a : ((i == j) ? T(1) : T(0));   // identity padding beyond nb
    }
    if (tid == 0) pivot = s[0];
    int fail = -1;
    __syncthreads();
    TileSteps<T, 0>::run(nb, s, colL, &pivot, fail, i, q, perm_i);
    if (fail >= 0 && tid == 0 && *info == 0) *info = index0 + fail + 1;
    // write back the columns that were finished (all of them when nothing failed)
    const int ncol = (fail >= 0) ? fail : nb;
#pragma unroll
    for (int m = 0; m < 16; ++m) {
        const int j = 4 * m + q;
        if (i < nb && j <= i && j < ncol) A[(int64_t)i * lda + j] = s[m];
    }
}

// ---- triangular solve with one diagonal tile ---------------------------------------------------
// X (m x nb, nb <= 64) <- X * L^{-T}, L the nb x nb lower triangular factor of a diagonal tile:
// the "scale column k, update the columns right of it" part of Algorithm 2 for the rows below the
// tile, so the same operations in the same order as the plain loops (forward substitution along
// each row of X; no inverse of L is formed).
//
// A workgroup takes 64 rows.  Four neighbouring lanes share one row: lane q of the quad keeps the
// column pairs {8 g + 2 q, 8 g + 2 q + 1}, g = 0..7, in registers, so a quad reads and writes 64
// contiguous bytes of its row per access.  In step J the lane that owns column J forms
// x_J = b_J / L_JJ and hands it to its quad with one DPP move per 32-bit half; every lane then
// updates its columns right of J with column J of L, which sits in LDS permuted so that the 16
// entries a lane needs are contiguous (entries on and above the diagonal are stored as zeros, so no
// lane needs a mask).
constexpr int kLqLd = kPT + 2;       // padded LDS row: keeps 16-byte alignment, spreads banks

__device__ __forceinline__ int lq_perm(int k) { return ((k >> 1) & 3) * 16 + (k >> 3) * 2 + (k & 1); }

template <int SRC>
__device__ __forceinline__ float quad_bcast(float v)
{
    constexpr int ctrl = SRC * 0x55;                        // quad_perm: [SRC, SRC, SRC, SRC]
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), ctrl, 0xF, 0xF, false));
}
template <int SRC>
__device__ __forceinline__ double quad_bcast(double v)
{
    constexpr int ctrl = SRC * 0x55;
    const long long bits = __double_as_longlong(v);
    const int lo = __builtin_amdgcn_update_dpp(0, (int)(bits & 0xffffffffll), ctrl, 0xF, 0xF, false);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(bits >> 32), ctrl, 0xF, 0xF, false);
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}

// Step J for the R rows a lane holds.  `cur` are the lane's 16 entries of column J of L and
// (d, r) = (L_JJ, 1 / L_JJ), all read from LDS during step J - 1; the step starts by issuing the
// reads for step J + 1, so that LDS latency never sits on the chain x_J -> b_{J+1} -> x_{J+1}.
template <typename T, int R, int J>
struct TrsmSteps {
    static __device__ __forceinline__ void run(T (&b)[R][16], const T (&cur)[16], T d, T r, const T* Lq,
                                               const T* dg, const T* rdg, int q)
    {
        if constexpr (J < kPT) {
            constexpr int gJ = J >> 3, qJ = (J >> 1) & 3, eJ = J & 1;
            constexpr int Jn = (J + 1 < kPT) ? J + 1 : J;
            T nxt[16];
            const T* col = Lq + Jn * kLqLd + q * 16;
#pragma unroll
            for (int c = 2 * (Jn >> 3); c < 16; ++c) nxt[c] = col[c];
            const T dn = dg[Jn], rn = rdg[Jn];
#pragma unroll
            for (int t = 0; t < R; ++t) {
                // x_J = b_J / L_JJ as b_J * (1 / L_JJ) plus one residual correction (exact whenever
                // the quotient is representable); computed by every lane on its own register, the
                // owner's result is the one the quad keeps
                const T bj = b[t][2 * gJ + eJ];
                const T q0 = bj * r;
                const T xj = quad_bcast<qJ>(fma(fma(-q0, d, bj), r, q0));
                if (q == qJ) b[t][2 * gJ + eJ] = xj;
#pragma unroll
                for (int c = 2 * gJ; c < 16; ++c) b[t][c] -= xj * cur[c];
            }
            TrsmSteps<T, R, J + 1>::run(b, nxt, dn, rn, Lq, dg, rdg, q);
        }
    }
};

template <typename T, int R>
__global__ __launch_bounds__(256) void trsm_tile_kernel(int m, int nb, const T* __restrict__ L, int64_t ldl,
                                                        T* X, int64_t ldx)
{
    __shared__ __attribute__((aligned(16))) T Lq[kPT * kLqLd];   // Lq[J][lq_perm(k)] = L[k][J] for k > J, else 0
    __shared__ T dg[kPT], rdg[kPT];                               // L_JJ and 1 / L_JJ (1 beyond nb)
    const int tid = threadIdx.x;
    const int i = tid >> 2, q = tid & 3;
    T b[R][16];
    bool live[R];
    T* xr[R];
    // every load below is unconditional on a clamped (always valid) address and the value is
    // selected afterwards, so that all of a thread's loads are in flight together
    {
        T lv[16];
#pragma unroll
        for (int it = 0; it < 16; ++it) {
            const int k = it * 4 + (tid >> 6), j = tid & 63;      // element L[k][j]; a wavefront reads one row
            const int kc = min(k, nb - 1), jc = min(j, kc);
            lv[it] = L[(int64_t)kc * ldl + jc];
        }
        const int dc = min(tid & 63, nb - 1);
        const T dv = L[(int64_t)dc * ldl + dc];
        T b0[R][16];
#pragma unroll
        for (int t = 0; t < R; ++t) {
            const int64_t row = ((int64_t)blockIdx.x * R + t) * kPT + i;
            live[t] = row < m;
            xr[t] = X + (live[t] ? row : (int64_t)m - 1) * ldx;
#pragma unroll
            for (int c = 0; c < 16; ++c) b0[t][c] = xr[t][min(8 * (c >> 1) + 2 * q + (c & 1), nb - 1)];
        }
#pragma unroll
        for (int it = 0; it < 16; ++it) {
            const int k = it * 4 + (tid >> 6), j = tid & 63;
            Lq[j * kLqLd + lq_perm(k)] = (k < nb && j < k) ? lv[it] : T(0);
        }
        if (tid < kPT) {
            const T d = (tid < nb) ? dv : T(1);
            dg[tid] = d;
            rdg[tid] = T(1) / d;
        }
#pragma unroll
        for (int t = 0; t < R; ++t)
#pragma unroll
            for (int c = 0; c < 16; ++c)
                b[t][c] = (live[t] && 8 * (c >> 1) + 2 * q + (c & 1) < nb) ? b0[t][c] : T(0);
    }
    __syncthreads();
    T cur[16];
#pragma unroll
    for (int c = 0; c < 16; ++c) cur[c] = Lq[q * 16 + c];
    TrsmSteps<T, R, 0>::run(b, cur, dg[0], rdg[0], Lq, dg, rdg, q);
#pragma unroll
    for (int t = 0; t < R; ++t)
#pragma unroll
        for (int c = 0; c < 16; ++c) {
            const int col = 8 * (c >> 1) + 2 * q + (c & 1);
            if (live[t] && col < nb) xr[t][col] = b[t][c];
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

hipError_t launch_potrf_tile(bool f32, int nb, void* A, int64_t lda, int32_t* info, int32_t index0,
                             hipStream_t stream)
{
    if (nb <= 0) return hipSuccess;
    if (f32)
        hipLaunchKernelGGL(potrf_tile_kernel<float>, dim3(1), dim3(256), 0, stream, nb, (float*)A, lda, info,
                           index0);
    else
        hipLaunchKernelGGL(potrf_tile_kernel<double>, dim3(1), dim3(256), 0, stream, nb, (double*)A, lda, info,
                           index0);
    return hipGetLastError();
}

template <typename T>
static void launch_trsm_typed(int64_t m, int nb, const void* L, int64_t ldl, void* X, int64_t ldx,
                              hipStream_t stream)
{
    if (m <= kPT) {
        hipLaunchKernelGGL((trsm_tile_kernel<T, 1>), dim3(1), dim3(256), 0, stream, (int)m, nb, (const T*)L, ldl,
                           (T*)X, ldx);
    } else {
        const unsigned grid = (unsigned)((m + 2 * kPT - 1) / (2 * kPT));
        hipLaunchKernelGGL((trsm_tile_kernel<T, 2>), dim3(grid), dim3(256), 0, stream, (int)m, nb, (const T*)L,
                           ldl, (T*)X, ldx);
    }
}

hipError_t launch_trsm_tile(bool f32, int64_t m, int nb, const void* L, int64_t ldl, void* X, int64_t ldx,
                            hipStream_t stream)
{
    if (m <= 0 || nb <= 0) return hipSuccess;
    if (f32)
        launch_trsm_typed<float>(m, nb, L, ldl, X, ldx, stream);
    else
        launch_trsm_typed<double>(m, nb, L, ldl, X, ldx, stream);
    return hipGetLastError();
}

}  // namespace tbs
