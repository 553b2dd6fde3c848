// potrf_kernels.hip -- Cholesky of one diagonal tile, the sequential core of Large Block Cholesky
// (the paper's Algorithm 5 calls a one-tile Cholesky for A[I0, I0]; at the bottom of the
// recursion that is Algorithm 2 on a tile held in LDS).
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "potrf_kernels.h"

namespace tbs {

constexpr int kPT = 64;          // tile side
constexpr int kPLd = kPT + 1;    // padded LDS row

typedef double f64x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Per-type pieces: the 16x16x4 MFMA (lane l supplies A[l%16][l/16] and B[l/16][l%16]; row_of gives the
// row of result register g), the hardware reciprocal square root, and a read of one lane's value.
template <typename T> struct TileOps;
template <> struct TileOps<double> {
    typedef f64x4 acc_t;
    static __device__ __forceinline__ acc_t mma(double a, double b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int row_of(int g, int lane) { return 4 * g + (lane >> 4); }
    static __device__ __forceinline__ double rsq(double p) { return __builtin_amdgcn_rsq(p); }
    static __device__ __forceinline__ double readlane(double v, int lane)
    {
        const int lo = __builtin_amdgcn_readlane(__double2loint(v), lane);
        const int hi = __builtin_amdgcn_readlane(__double2hiint(v), lane);
        return __hiloint2double(hi, lo);
    }
};
template <> struct TileOps<float> {
    typedef f32x4 acc_t;
    static __device__ __forceinline__ acc_t mma(float a, float b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int row_of(int g, int lane) { return 4 * (lane >> 4) + g; }
    static __device__ __forceinline__ float rsq(float p) { return __builtin_amdgcn_rsqf(p); }
    static __device__ __forceinline__ float readlane(float v, int lane)
    {
        return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
    }
};

// d = sqrt(p) and r ~ 1 / d for a pivot p > 0 (p is the same in every lane), without a branch.  The
// hardware estimate of p^{-1/2} is refined by one coupled Newton step for (sqrt p, 1 / (2 sqrt p)) and
// two residual steps on the root: d is the correctly rounded root whenever the root is representable
// (so integer factors stay exact); r is good to a few ulps, which is all the corrected quotient in
// PanelSteps needs.  Eight dependent operations instead of the several dozen of a library sqrt
// followed by a division -- this sequence sits on the critical path of every column.  No rescaling is
// done: for pivots below 2^-767 the residual p - d*d is no longer exact and d may be off by an ulp.
template <typename T>
__device__ __forceinline__ void sqrt_and_reciprocal(T p, T& d, T& r)
{
    const T y = TileOps<T>::rsq(p);
    T g = p * y, h = T(0.5) * y;
    const T e = fma(-h, g, T(0.5));
    g = fma(g, e, g);
    h = fma(h, e, h);
    g = fma(fma(-g, g, p), h, g);
    d = fma(fma(-g, g, p), h, g);
    r = h + h;
}

// Columns 16 kb .. 16 kb + 15 of the tile for all rows from 16 kb down, by one wavefront: lane l holds
// the 16 entries of row 16 kb + l in registers.  Step K is Algorithm 2's iteration for that column:
// the pivot comes from lane K, every lane scales its entry of column K and updates its entries right
// of it with the scaled entries of the rows K + 1 .. 15 (read from their lanes), so rows of the
// diagonal block and rows below it run the same instructions and nothing goes through LDS.  The
// sixteen steps are one straight line of code (a failed pivot is replaced by 1 with selects), so that
// the updates of one step can fill the stalls of the next step's square root.
template <typename T, int K>
struct PanelSteps {
    static __device__ __forceinline__ void run(T (&s)[16], int lane, int col0, int& fail)
    {
        if constexpr (K < 16) {
            T p = TileOps<T>::readlane(s[K], K);
            const bool bad = !(p > T(0));
            fail = (bad && fail < 0) ? col0 + K : fail;
            p = bad ? T(1) : p;                             // keep going on finite numbers; the output
            T d, r;                                         // from column `fail` on is unspecified
            sqrt_and_reciprocal(p, d, r);
            // a / d as a * r plus one residual correction: exact whenever the quotient is representable
            const T a = s[K];
            const T q0 = a * r;
            const T l = (lane == K) ? d : fma(fma(-q0, d, a), r, q0);
            s[K] = l;
#pragma unroll
            for (int j = K + 1; j < 16; ++j) s[j] -= l * TileOps<T>::readlane(l, j);
            PanelSteps<T, K + 1>::run(s, lane, col0, fail);
        }
    }
};

// Cholesky of one nb x nb tile (nb <= 64), one workgroup.  The tile sits in LDS (identity beyond nb).
// For each block of 16 columns: wavefront 0 factors the block column (PanelSteps); then the four
// wavefronts subtract its outer product from the 16 x 16 blocks to the right of it with MFMAs.
// Within a block column the operations are those of Algorithm 2 in its order; across block columns
// the 16 products of an update are summed by the MFMA before they are subtracted, which changes
// rounding only (integer-valued factors still come out exactly).
// The factorisation proper, on a tile that sits in LDS (rows of kPLd elements, identity beyond nb);
// all 256 threads call it; `fail` (meaningful in wavefront 0) receives the first failed column.
template <typename T>
__device__ __forceinline__ void factor_tile_in_lds(T* S, int nb, int& fail, int lane, int w)
{
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) {
        if (16 * kb < nb) {                                 // uniform
            if (w == 0) {
                const int row = min(16 * kb + lane, kPT - 1);
                const bool live = 16 * kb + lane < kPT;
                T s[16];
#pragma unroll
                for (int c = 0; c < 16; ++c) s[c] = S[row * kPLd + 16 * kb + c];
                PanelSteps<T, 0>::run(s, lane, 16 * kb, fail);
                if (live) {
#pragma unroll
                    for (int c = 0; c < 16; ++c) S[row * kPLd + 16 * kb + c] = s[c];
                }
            }
            __syncthreads();
            if (kb < 3) {
                int idx = 0;
#pragma unroll
                for (int I = kb + 1; I < 4; ++I)
#pragma unroll
                    for (int J = kb + 1; J <= I; ++J) {
                        if ((idx++ & 3) == w) {             // uniform per wavefront
                            typename TileOps<T>::acc_t acc;
                            T* c = S + (16 * I) * kPLd + 16 * J + (lane & 15);
#pragma unroll
                            for (int g = 0; g < 4; ++g) acc[g] = c[TileOps<T>::row_of(g, lane) * kPLd];
                            const T* ra = S + (16 * I + (lane & 15)) * kPLd + 16 * kb + (lane >> 4);
                            const T* rb = S + (16 * J + (lane & 15)) * kPLd + 16 * kb + (lane >> 4);
#pragma unroll
                            for (int k4 = 0; k4 < 4; ++k4) acc = TileOps<T>::mma(ra[4 * k4], -rb[4 * k4], acc);
#pragma unroll
                            for (int g = 0; g < 4; ++g) c[TileOps<T>::row_of(g, lane) * kPLd] = acc[g];
                        }
                    }
                __syncthreads();
            }
        }
    }
}

// Lower triangle of the nb x nb tile at A into LDS (identity beyond nb, zeros above the diagonal):
// unconditional loads on clamped addresses, all in flight together; one row per wavefront and turn.
template <typename T>
__device__ __forceinline__ void load_lower_tile(T* S, const T* A, int64_t lda, int nb, int lane, int w)
{
    T v[16];
#pragma unroll
    for (int it = 0; it < 16; ++it) {
        const int i = it * 4 + w, j = lane;
        const int ic = min(i, nb - 1), jc = min(j, ic);
        v[it] = A[(int64_t)ic * lda + jc];
    }
#pragma unroll
    for (int it = 0; it < 16; ++it) {
        const int i = it * 4 + w, j = lane;
        S[i * kPLd + j] = (i < nb && j <= i) ? v[it] : ((i == j) ? T(1) : T(0));
    }
}

template <typename T>
__global__ __launch_bounds__(256) void potrf_tile_kernel(int nb, T* __restrict__ A, int64_t lda, int32_t* info,
                                                         int32_t index0)
{
    __shared__ T S[kPT * kPLd];
    __shared__ int fail_sh;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    load_lower_tile(S, A, lda, nb, lane, w);
    if (tid == 0) fail_sh = -1;
    __syncthreads();
    int fail = -1;
    factor_tile_in_lds(S, nb, fail, lane, w);
    if (tid == 0 && fail >= 0) {
        fail_sh = fail;
        if (*info == 0) *info = index0 + fail + 1;
    }
    __syncthreads();
    // write back the columns that were finished (all of them when nothing failed)
    const int failed = fail_sh;
    const int ncol = (failed >= 0) ? failed : nb;
#pragma unroll
    for (int it = 0; it < 16; ++it) {
        const int i = it * 4 + w, j = lane;
        if (i < nb && j <= i && j < ncol) A[(int64_t)i * lda + j] = S[i * kPLd + j];
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

// ---- triangular solve with a lower triangular block of up to 512 columns -------------------------
// X (m x n) <- X * L^{-T}, L the n x n lower triangular factor (n <= 512), in one launch: the rows of
// X do not depend on each other, so a workgroup takes 32 of them through all tile columns by itself
// (no ordering between workgroups, no intermediate kernel).  For tile column jt:
//   the 32 x 64 tile X_jt is loaded into MFMA accumulators and the products X_kt * L[jt][kt]^T of the
//   tile columns kt < jt already solved (kept in LDS; L comes straight from global memory in operand
//   layout, it is shared by every workgroup and stays in L2) are subtracted;
//   the result goes through LDS to the four-lanes-per-row layout of TrsmSteps, is solved against the
//   diagonal tile L[jt][jt] by forward substitution, and is written to global memory and, as the
//   operand of the later tile columns, back to LDS.
// The operations on an element are those of Algorithm 2 for the rows below a diagonal block, except
// that the products of 64 columns are summed by the MFMA before they are subtracted.
constexpr int kPR = 32;                                    // rows of X per workgroup
constexpr int kMaxPanelTiles = 8;                          // n <= 512
constexpr int kXsLd = kPT * (kMaxPanelTiles - 1) + 2;      // LDS row of solved tiles (padded)

template <typename T>
__global__ __launch_bounds__(256) void trsm_panel_kernel(int m, int n, const T* __restrict__ L, int64_t ldl,
                                                         T* X, int64_t ldx)
{
    __shared__ __attribute__((aligned(16))) T Xs[kPR * kXsLd];   // solved tiles 0 .. nt-2; also the staging tile
    __shared__ __attribute__((aligned(16))) T Lq[kPT * kLqLd];   // diagonal tile, as in trsm_tile_kernel
    __shared__ T dg[kPT], rdg[kPT];
    typedef typename TileOps<T>::acc_t acc_t;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int64_t row0 = (int64_t)blockIdx.x * kPR;
    const int nt = (n + kPT - 1) / kPT;
    // this lane's elements of a tile of X in accumulator layout (wavefront w owns columns 16 w ..
    // 16 w + 15 of a tile, both groups of 16 rows); requested one tile column ahead, before anything
    // else of the iteration, so that the loads have the whole iteration to arrive
    auto load_x = [&](int jt, T (&x)[2][4]) {
        const int col = jt * kPT + 16 * w + (lane & 15);
#pragma unroll
        for (int rg = 0; rg < 2; ++rg)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int64_t row = row0 + 16 * rg + TileOps<T>::row_of(g, lane);
                const T v = X[min(row, (int64_t)m - 1) * ldx + min(col, n - 1)];
                x[rg][g] = (row < m && col < n) ? v : T(0);
            }
    };
    T xin[2][4], xnext[2][4];
    load_x(0, xin);
    for (int jt = 0; jt < nt; ++jt) {
        const int c0 = jt * kPT;
        const int nbw = min(kPT, n - c0);
        // requests to global memory, in the order in which their data is needed (they complete in
        // order): the first operand values of L, the diagonal tile L[jt][jt] (written to LDS after the
        // products), the next tile of X
        const int col = c0 + 16 * w + (lane & 15);
        const T* lp = L + (int64_t)min(col, n - 1) * ldl + (lane >> 4);   // row `col` of L, this lane's k offset
        const bool lrow_ok = col < n;
        T bcur[16], bnxt[16];
#pragma unroll
        for (int s4 = 0; s4 < 16; ++s4) bcur[s4] = lp[(jt > 0) ? 4 * s4 : 0];
        T lv[16];
#pragma unroll
        for (int it = 0; it < 16; ++it) {
            const int k = it * 4 + w, j = lane;
            const int kc = min(k, nbw - 1), jc = min(j, kc);
            lv[it] = L[(int64_t)(c0 + kc) * ldl + c0 + jc];
        }
        const int dc = min(lane, nbw - 1);
        const T dv = L[(int64_t)(c0 + dc) * ldl + c0 + dc];
        load_x(min(jt + 1, nt - 1), xnext);
        acc_t acc[2];
#pragma unroll
        for (int rg = 0; rg < 2; ++rg)
#pragma unroll
            for (int g = 0; g < 4; ++g) acc[rg][g] = xin[rg][g];
        const T* xa = Xs + (lane & 15) * kXsLd + (lane >> 4);
        // per tile column kt: the operand values of L for kt + 1 are requested from global memory and
        // all operand values of X for kt are read from LDS before the 32 MFMAs of kt are issued
        for (int kt = 0; kt < jt; ++kt) {
            T a0[16], a1[16];
#pragma unroll
            for (int s4 = 0; s4 < 16; ++s4) {
                a0[s4] = xa[kt * kPT + 4 * s4];
                a1[s4] = xa[16 * kXsLd + kt * kPT + 4 * s4];
            }
            const int ktn = (kt + 1 < jt) ? kt + 1 : kt;    // last round: a harmless repeat
#pragma unroll
            for (int s4 = 0; s4 < 16; ++s4) bnxt[s4] = lp[ktn * kPT + 4 * s4];
            T bneg[16];
#pragma unroll
            for (int s4 = 0; s4 < 16; ++s4) bneg[s4] = lrow_ok ? -bcur[s4] : T(0);
            __builtin_amdgcn_sched_barrier(0);              // nothing of the next round moves up into
#pragma unroll                                              // the MFMAs: it would wait for the loads
            for (int s4 = 0; s4 < 16; ++s4) {
                acc[0] = TileOps<T>::mma(a0[s4], bneg[s4], acc[0]);
                acc[1] = TileOps<T>::mma(a1[s4], bneg[s4], acc[1]);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int s4 = 0; s4 < 16; ++s4) bcur[s4] = bnxt[s4];
        }
#pragma unroll
        for (int rg = 0; rg < 2; ++rg)
#pragma unroll
            for (int g = 0; g < 4; ++g) xin[rg][g] = xnext[rg][g];
        // staging tile: the place of X_jt among the solved tiles; the last tile column is no operand
        // of anything, it borrows place 0 once every wavefront is done with the solved tiles
        const int place = (jt < nt - 1) ? jt : 0;
        if (jt == nt - 1 && nt > 1) __syncthreads();
#pragma unroll
        for (int rg = 0; rg < 2; ++rg)
#pragma unroll
            for (int g = 0; g < 4; ++g)
                Xs[(16 * rg + TileOps<T>::row_of(g, lane)) * kXsLd + place * kPT + 16 * w + (lane & 15)] = acc[rg][g];
#pragma unroll
        for (int it = 0; it < 16; ++it) {
            const int k = it * 4 + w, j = lane;
            Lq[j * kLqLd + lq_perm(k)] = (k < nbw && j < k) ? lv[it] : T(0);
        }
        if (tid < kPT) {
            const T d = (tid < nbw) ? dv : T(1);
            dg[tid] = d;
            rdg[tid] = T(1) / d;
        }
        __syncthreads();
        if (tid < 4 * kPR) {                                // two wavefronts: four lanes per row
            const int i = tid >> 2, q = tid & 3;
            T* br = Xs + i * kXsLd + place * kPT;
            T b[1][16], cur[16];
#pragma unroll
            for (int c = 0; c < 16; ++c) {
                b[0][c] = br[8 * (c >> 1) + 2 * q + (c & 1)];
                cur[c] = Lq[q * 16 + c];
            }
            TrsmSteps<T, 1, 0>::run(b, cur, dg[0], rdg[0], Lq, dg, rdg, q);
            const int64_t row = row0 + i;
#pragma unroll
            for (int c = 0; c < 16; ++c) {
                const int cc = 8 * (c >> 1) + 2 * q + (c & 1);
                br[cc] = b[0][c];
                if (row < m && c0 + cc < n) X[row * ldx + c0 + cc] = b[0][c];
            }
        }
        __syncthreads();
    }
}

// ---- Cholesky of a diagonal block of up to 128 columns in one workgroup ---------------------------
// Algorithm 5 on two tiles without leaving the compute unit: factor A11 (64 x 64), solve
// A21 <- A21 L11^{-T}, update A22 <- A22 - A21 A21^T, factor A22 (n - 64 columns).  The three pieces are
// the code of potrf_tile_kernel, trsm_tile_kernel and an MFMA product on tiles held in LDS; as four
// launches they cost three kernel boundaries on the chain of every pair of tile columns.
template <typename T>
__global__ __launch_bounds__(256) void potrf_block_kernel(int n, T* __restrict__ A, int64_t lda, int32_t* info,
                                                          int32_t index0)
{
    __shared__ T S11[kPT * kPLd], S21[kPT * kPLd], S22[kPT * kPLd];
    __shared__ __attribute__((aligned(16))) T Lq[kPT * kLqLd];
    __shared__ T dg[kPT], rdg[kPT];
    __shared__ int fail_sh;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int n2 = n - kPT;                                 // 1 .. 64
    load_lower_tile(S11, A, lda, kPT, lane, w);
    load_lower_tile(S22, A + (int64_t)kPT * lda + kPT, lda, n2, lane, w);
    {
        T v[16];
#pragma unroll
        for (int it = 0; it < 16; ++it) {
            const int i = it * 4 + w, j = lane;
            v[it] = A[(int64_t)(kPT + min(i, n2 - 1)) * lda + j];
        }
#pragma unroll
        for (int it = 0; it < 16; ++it) {
            const int i = it * 4 + w, j = lane;
            S21[i * kPLd + j] = (i < n2) ? v[it] : T(0);
        }
    }
    if (tid == 0) fail_sh = -1;
    __syncthreads();
    int fail1 = -1, fail2 = -1;
    factor_tile_in_lds(S11, kPT, fail1, lane, w);
    // L11 in the layout of the substitution (see trsm_tile_kernel)
#pragma unroll
    for (int it = 0; it < 16; ++it) {
        const int k = it * 4 + w, j = lane;
        Lq[j * kLqLd + lq_perm(k)] = (j < k) ? S11[k * kPLd + j] : T(0);
    }
    if (tid < kPT) {
        const T d = S11[tid * kPLd + tid];
        dg[tid] = d;
        rdg[tid] = T(1) / d;
    }
    __syncthreads();
    {
        const int i = tid >> 2, q = tid & 3;                // four lanes per row of A21
        T* br = S21 + i * kPLd;
        T b[1][16], cur[16];
#pragma unroll
        for (int c = 0; c < 16; ++c) {
            b[0][c] = br[8 * (c >> 1) + 2 * q + (c & 1)];
            cur[c] = Lq[q * 16 + c];
        }
        TrsmSteps<T, 1, 0>::run(b, cur, dg[0], rdg[0], Lq, dg, rdg, q);
#pragma unroll
        for (int c = 0; c < 16; ++c) br[8 * (c >> 1) + 2 * q + (c & 1)] = b[0][c];
    }
    __syncthreads();
    {
        int idx = 0;
#pragma unroll
        for (int I = 0; I < 4; ++I)
#pragma unroll
            for (int J = 0; J <= I; ++J) {
                if ((idx++ & 3) == w) {                     // uniform per wavefront
                    typename TileOps<T>::acc_t acc;
                    T* c = S22 + (16 * I) * kPLd + 16 * J + (lane & 15);
#pragma unroll
                    for (int g = 0; g < 4; ++g) acc[g] = c[TileOps<T>::row_of(g, lane) * kPLd];
                    const T* ra = S21 + (16 * I + (lane & 15)) * kPLd + (lane >> 4);
                    const T* rb = S21 + (16 * J + (lane & 15)) * kPLd + (lane >> 4);
#pragma unroll
                    for (int k4 = 0; k4 < 16; ++k4) acc = TileOps<T>::mma(ra[4 * k4], -rb[4 * k4], acc);
#pragma unroll
                    for (int g = 0; g < 4; ++g) c[TileOps<T>::row_of(g, lane) * kPLd] = acc[g];
                }
            }
    }
    __syncthreads();
    factor_tile_in_lds(S22, n2, fail2, lane, w);
    if (tid == 0) {
        const int f = (fail1 >= 0) ? fail1 : ((fail2 >= 0) ? kPT + fail2 : -1);
        fail_sh = f;
        if (f >= 0 && *info == 0) *info = index0 + f + 1;
    }
    __syncthreads();
    // write back the columns that were finished (all of them when nothing failed)
    const int failed = fail_sh;
    const int ncol = (failed >= 0) ? failed : n;
#pragma unroll
    for (int it = 0; it < 16; ++it) {
        const int i = it * 4 + w, j = lane;
        if (j <= i && j < ncol) A[(int64_t)i * lda + j] = S11[i * kPLd + j];
        if (i < n2 && j < ncol) A[(int64_t)(kPT + i) * lda + j] = S21[i * kPLd + j];
        if (i < n2 && j <= i && kPT + j < ncol) A[(int64_t)(kPT + i) * lda + kPT + j] = S22[i * kPLd + j];
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

hipError_t launch_potrf_block(bool f32, int n, void* A, int64_t lda, int32_t* info, int32_t index0,
                              hipStream_t stream, hipEvent_t done)
{
    if (n > 2 * kPT) return hipErrorInvalidValue;
    if (n <= kPT) {
        const hipError_t e = launch_potrf_tile(f32, n, A, lda, info, index0, stream);
        if (e != hipSuccess || !done) return e;
        return hipEventRecord(done, stream);
    }
    // `done`: the kernel's own completion is the event (no separate packet in the queue between this
    // kernel and the next one of the stream)
    if (f32)
        hipExtLaunchKernelGGL(potrf_block_kernel<float>, dim3(1), dim3(256), 0, stream, nullptr, done, 0, n,
                              (float*)A, lda, info, index0);
    else
        hipExtLaunchKernelGGL(potrf_block_kernel<double>, dim3(1), dim3(256), 0, stream, nullptr, done, 0, n,
                              (double*)A, lda, info, index0);
    return hipGetLastError();
}

hipError_t launch_trsm_panel(bool f32, int64_t m, int n, const void* L, int64_t ldl, void* X, int64_t ldx,
                             hipStream_t stream)
{
    if (m <= 0 || n <= 0) return hipSuccess;
    if (n > kPT * kMaxPanelTiles) return hipErrorInvalidValue;
    const unsigned grid = (unsigned)((m + kPR - 1) / kPR);
    if (f32)
        hipLaunchKernelGGL(trsm_panel_kernel<float>, dim3(grid), dim3(256), 0, stream, (int)m, n, (const float*)L,
                           ldl, (float*)X, ldx);
    else
        hipLaunchKernelGGL(trsm_panel_kernel<double>, dim3(grid), dim3(256), 0, stream, (int)m, n,
                           (const double*)L, ldl, (double*)X, ldx);
    return hipGetLastError();
}

}  // namespace tbs
