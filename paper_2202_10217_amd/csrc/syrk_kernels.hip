// syrk_kernels.hip -- Triangle Block SYRK for gfx950 (MI355X), fp64 and fp32.
//
// One workgroup (4 wavefronts, one per SIMD of a compute unit) executes one block of the plan:
//   * a triangle block TB(R), |R| = k = 4 tile rows: the k(k-1)/2 = 6 tiles C[r_u, r_v], u > v,
//     stay in registers (the paper's fast memory, Section 5.1.4: S = b^2 k(k-1)/2) while the k
//     row panels A[r_u, :] stream through LDS in chunks of KC columns (Algorithm 4's loop over
//     the columns of A, KC columns per step).  Every staged panel is used as left operand
//     (rows of the tile) and as right operand (columns of the tile): the symmetric reuse that
//     Section 5.1 is about;
//   * a rectangular block of at most 2 x 3 tiles (Algorithm 4's square-block part: the last l
//     tile rows and the recursion base), 5 panels for 6 tiles;
//   * a diagonal tile: one panel, only the 10 of 16 sub-tiles on or below the diagonal.
// Within a tile, wavefront w owns the 16-column strip w: 4 MFMA sub-tiles of 16 x 16 per tile.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tbs_plan.h"
#include "syrk_kernels.h"

namespace tbs {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef double f64x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;

// ---- per-type constants and the MFMA instruction --------------------------------------------
template <typename T> struct Cfg;

template <> struct Cfg<double> {
    typedef f64x4 acc_t;
    static constexpr int KC = 16;            // columns of A per staged chunk (128 B per row)
    static constexpr int LDK = KC + 2;       // padded LDS row length, keeps 16 B alignment
    static constexpr int VEC = 2;            // elements per 16 B
    // D = A(16x4) * B(4x16) + C.  Lane l supplies A[l%16][l/16] and B[l/16][l%16]; register g of
    // the result holds D[4*g + l/16][l%16].
    static __device__ __forceinline__ acc_t mfma(double a, double b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int row_of(int g, int lane) { return 4 * g + (lane >> 4); }
};

template <> struct Cfg<float> {
    typedef f32x4 acc_t;
    static constexpr int KC = 32;
    static constexpr int LDK = KC + 4;
    static constexpr int VEC = 4;
    // Same operand layout; register g of the result holds D[4*(l/16) + g][l%16].
    static __device__ __forceinline__ acc_t mfma(float a, float b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int row_of(int g, int lane) { return 4 * (lane >> 4) + g; }
};

constexpr int kLdsBytes = 2 * kMaxPanels * kTile * Cfg<double>::LDK * 8;
static_assert(kLdsBytes == 2 * kMaxPanels * kTile * Cfg<float>::LDK * 4, "one LDS size for both types");

// ---- block shapes ----------------------------------------------------------------------------
// A shape names which LDS panels feed the row side (all four 16-row groups of a panel) and the
// column side (the wavefront's 16-row group) of each accumulator slot.
struct TriShape {                         // panels 0..3 = R in zone order
    static constexpr int NP = 4, NA = 3, NB = 3, NSLOT = 6;
    static constexpr int a_panel(int i) { return i + 1; }
    static constexpr int b_panel(int j) { return j; }
    static constexpr bool col_side(int) { return false; }   // SYRK only: one matrix
    static constexpr bool active(int i, int j) { return j <= i; }
    static constexpr int slot(int i, int j) { return i * (i + 1) / 2 + j; }
};
struct RectShape {                        // panels 0..2 = column side, 3..4 = row side
    static constexpr int NP = 5, NA = 2, NB = 3, NSLOT = 6;
    static constexpr int a_panel(int i) { return 3 + i; }
    static constexpr int b_panel(int j) { return j; }
    static constexpr bool col_side(int p) { return p < 3; }
    static constexpr bool active(int, int) { return true; }
    static constexpr int slot(int i, int j) { return i * 3 + j; }
};

// ---- operands of one launch --------------------------------------------------------------------
// C[rows, cols] <- beta*C + alpha * R[rows, :] * Q[cols, :]^T.  SYRK has R == Q == A and updates
// only tiles strictly below the diagonal; the general product (used by the Cholesky driver for its
// triangular solves) has two different matrices and updates every tile.
template <typename T>
struct Mats {
    const T* R;  int64_t ldr;  int nr;      // row-side matrix, nr rows
    const T* Q;  int64_t ldq;  int nq;      // column-side matrix, nq rows
    T* C;        int64_t ldc;
    int M;                                  // contraction length
    T alpha, beta;
    bool lower;                             // true: SYRK (tile (r,q) only if q < r)
};

// ---- global -> register -> LDS staging of one chunk --------------------------------------------
template <typename T, int NP>
struct Stager {
    static constexpr int KC = Cfg<T>::KC, LDK = Cfg<T>::LDK, VEC = Cfg<T>::VEC;
    u32x4 reg[2 * NP];

    // prow[p]: tile row of panel p (-1: absent) in matrix base[p] with nrows[p] rows.
    __device__ __forceinline__ void load(const T* const (&base)[NP], const int64_t (&ld)[NP],
                                         const int (&nrows)[NP], const int (&prow)[NP], int M, int k0,
                                         bool fast, int tid)
    {
        const int v = tid & 7, r = tid >> 3;
#pragma unroll
        for (int p = 0; p < NP; ++p) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                u32x4 val = {0u, 0u, 0u, 0u};
                const int grow = prow[p] * kTile + h * 32 + r;
                if (prow[p] >= 0 && grow < nrows[p]) {
                    const T* src = base[p] + (int64_t)grow * ld[p] + k0 + v * VEC;
                    if (fast) {
                        val = *reinterpret_cast<const u32x4*>(src);
                    } else {
                        union { u32x4 q; T e[VEC]; } tmp;
                        tmp.q = val;
#pragma unroll
                        for (int e = 0; e < VEC; ++e)
                            if (k0 + v * VEC + e < M) tmp.e[e] = src[e];
                        val = tmp.q;
                    }
                }
                reg[p * 2 + h] = val;
            }
        }
    }

    __device__ __forceinline__ void store(T* __restrict__ buf, int tid) const
    {
        const int v = tid & 7, r = tid >> 3;
#pragma unroll
        for (int p = 0; p < NP; ++p)
#pragma unroll
            for (int h = 0; h < 2; ++h)
                *reinterpret_cast<u32x4*>(&buf[(p * kTile + h * 32 + r) * LDK + v * VEC]) = reg[p * 2 + h];
    }
};

template <typename T>
__device__ __forceinline__ bool vec_ok(const T* p, int64_t ld)
{
    return ((reinterpret_cast<uintptr_t>(p) & 15) == 0) && ((ld * sizeof(T)) % 16 == 0);
}

// ---- one chunk of MFMA work for a triangle or rectangular block --------------------------------
template <typename T, class Shape>
__device__ __forceinline__ void compute_chunk(const T* __restrict__ buf,
                                              typename Cfg<T>::acc_t (&acc)[Shape::NSLOT][4],
                                              uint32_t pmask, int w, int lane)
{
    constexpr int KC = Cfg<T>::KC, LDK = Cfg<T>::LDK;
    const int r16 = lane & 15, g = lane >> 4;
#pragma unroll
    for (int ks = 0; ks < KC / 4; ++ks) {
        T a[Shape::NA][4], b[Shape::NB];
#pragma unroll
        for (int i = 0; i < Shape::NA; ++i)
#pragma unroll
            for (int rb = 0; rb < 4; ++rb)
                a[i][rb] = buf[(Shape::a_panel(i) * kTile + rb * 16 + r16) * LDK + ks * 4 + g];
#pragma unroll
        for (int j = 0; j < Shape::NB; ++j)
            b[j] = buf[(Shape::b_panel(j) * kTile + w * 16 + r16) * LDK + ks * 4 + g];
#pragma unroll
        for (int i = 0; i < Shape::NA; ++i)
#pragma unroll
            for (int j = 0; j < Shape::NB; ++j)
                if (Shape::active(i, j)) {
                    const int s = Shape::slot(i, j);
                    if (pmask & (1u << s)) {
#pragma unroll
                        for (int rb = 0; rb < 4; ++rb)
                            acc[s][rb] = Cfg<T>::mfma(a[i][rb], b[j], acc[s][rb]);
                    }
                }
    }
}

// C tile element update: C <- beta*C + alpha*acc (beta == 0: C is not read)
template <typename T>
__device__ __forceinline__ void store_subtile(const Mats<T>& m, int row0, int col,
                                              const typename Cfg<T>::acc_t& acc, int lane, bool lower_only)
{
    T old[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const int row = row0 + Cfg<T>::row_of(g, lane);
        const bool ok = row < m.nr && col < m.nq && (!lower_only || col <= row);
        old[g] = (ok && m.beta != T(0)) ? m.C[(int64_t)row * m.ldc + col] : T(0);
    }
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const int row = row0 + Cfg<T>::row_of(g, lane);
        const bool ok = row < m.nr && col < m.nq && (!lower_only || col <= row);
        if (ok) {
            const T v = m.alpha * acc[g];
            m.C[(int64_t)row * m.ldc + col] = (m.beta != T(0)) ? m.beta * old[g] + v : v;
        }
    }
}

template <typename T, class Shape>
__device__ __forceinline__ void run_block(const Item& it, const Mats<T>& m, T* lds)
{
    constexpr int KC = Cfg<T>::KC, LDK = Cfg<T>::LDK, NP = Shape::NP;
    constexpr int kBufElems = kMaxPanels * kTile * LDK;
    typedef typename Cfg<T>::acc_t acc_t;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);

    // tile rows of the LDS panels, of the row side and of the column side of every slot
    int prow[NP], arow[Shape::NA], brow[Shape::NB], nrows[NP];
    const T* base[NP];
    int64_t ld[NP];
    uint32_t pmask = 0;
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        prow[p] = it.rows[p];                               // -1: panel absent
        const bool col_side = Shape::col_side(p);
        base[p] = col_side ? m.Q : m.R;
        ld[p] = col_side ? m.ldq : m.ldr;
        nrows[p] = col_side ? m.nq : m.nr;
    }
#pragma unroll
    for (int i = 0; i < Shape::NA; ++i) arow[i] = prow[Shape::a_panel(i)];
#pragma unroll
    for (int j = 0; j < Shape::NB; ++j) brow[j] = prow[Shape::b_panel(j)];
#pragma unroll
    for (int i = 0; i < Shape::NA; ++i)
#pragma unroll
        for (int j = 0; j < Shape::NB; ++j)
            if (Shape::active(i, j) && arow[i] >= 0 && brow[j] >= 0 && (!m.lower || brow[j] < arow[i]))
                pmask |= 1u << Shape::slot(i, j);

    acc_t acc[Shape::NSLOT][4];
#pragma unroll
    for (int s = 0; s < Shape::NSLOT; ++s)
#pragma unroll
        for (int rb = 0; rb < 4; ++rb) acc[s][rb] = acc_t{0, 0, 0, 0};

    const bool aligned = vec_ok(m.R, m.ldr) && vec_ok(m.Q, m.ldq);
    const int M = m.M;
    const int nchunks = (M + KC - 1) / KC;
    Stager<T, NP> st;
    if (nchunks > 0) {
        st.load(base, ld, nrows, prow, M, 0, aligned && KC <= M, tid);
        st.store(lds, tid);
    }
    __syncthreads();
    for (int ch = 0; ch < nchunks; ++ch) {
        const bool more = ch + 1 < nchunks;
        if (more) {
            const int k0 = (ch + 1) * KC;
            st.load(base, ld, nrows, prow, M, k0, aligned && k0 + KC <= M, tid);
        }
        compute_chunk<T, Shape>(lds + (ch & 1) * kBufElems, acc, pmask, w, lane);
        if (more) st.store(lds + ((ch + 1) & 1) * kBufElems, tid);
        __syncthreads();
    }

    const int col16 = w * 16 + (lane & 15);
#pragma unroll
    for (int i = 0; i < Shape::NA; ++i)
#pragma unroll
        for (int j = 0; j < Shape::NB; ++j)
            if (Shape::active(i, j)) {
                const int s = Shape::slot(i, j);
                if (pmask & (1u << s)) {
#pragma unroll
                    for (int rb = 0; rb < 4; ++rb)
                        store_subtile<T>(m, arow[i] * kTile + rb * 16, brow[j] * kTile + col16, acc[s][rb],
                                         lane, false);
                }
            }
}

// ---- diagonal tile: 10 sub-tiles on or below the diagonal, at most 3 per wavefront -------------
template <typename T>
__device__ __forceinline__ void run_diag(const Item& it, const Mats<T>& m, T* lds)
{
    constexpr int KC = Cfg<T>::KC, LDK = Cfg<T>::LDK;
    constexpr int kBufElems = kMaxPanels * kTile * LDK;
    typedef typename Cfg<T>::acc_t acc_t;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    // (row group, column group) of the wavefront's sub-tiles:
    //   w0: (0,0) (1,0) (2,0)   w1: (1,1) (2,1) (3,1)   w2: (2,2) (3,2) (3,0)   w3: (3,3)
    // (the two unused slots of wavefront 3 repeat (3,3) so that every LDS address stays valid)
    const int nsub = (w == 3) ? 1 : 3;
    int srow[3], scol[3];
    srow[0] = w;
    scol[0] = w;
    srow[1] = (w >= 2) ? 3 : w + 1;
    scol[1] = w;
    srow[2] = (w >= 1) ? 3 : 2;
    scol[2] = (w == 2) ? 0 : w;

    acc_t acc[3];
#pragma unroll
    for (int s = 0; s < 3; ++s) acc[s] = acc_t{0, 0, 0, 0};

    const int prow[1] = {it.rows[0]};
    const T* const base[1] = {m.R};
    const int64_t ld[1] = {m.ldr};
    const int nrows[1] = {m.nr};
    const bool aligned = vec_ok(m.R, m.ldr);
    const int M = m.M;
    const int nchunks = (M + KC - 1) / KC;
    Stager<T, 1> st;
    if (nchunks > 0) {
        st.load(base, ld, nrows, prow, M, 0, aligned && KC <= M, tid);
        st.store(lds, tid);
    }
    __syncthreads();
    const int r16 = lane & 15, g = lane >> 4;
    for (int ch = 0; ch < nchunks; ++ch) {
        const bool more = ch + 1 < nchunks;
        if (more) {
            const int k0 = (ch + 1) * KC;
            st.load(base, ld, nrows, prow, M, k0, aligned && k0 + KC <= M, tid);
        }
        const T* buf = lds + (ch & 1) * kBufElems;
#pragma unroll
        for (int ks = 0; ks < KC / 4; ++ks) {
            T a[3], b[3];
#pragma unroll
            for (int s = 0; s < 3; ++s) {
                a[s] = buf[(srow[s] * 16 + r16) * LDK + ks * 4 + g];
                b[s] = buf[(scol[s] * 16 + r16) * LDK + ks * 4 + g];
            }
#pragma unroll
            for (int s = 0; s < 3; ++s)
                if (s < nsub) acc[s] = Cfg<T>::mfma(a[s], b[s], acc[s]);
        }
        if (more) st.store(lds + ((ch + 1) & 1) * kBufElems, tid);
        __syncthreads();
    }
    const int t0 = it.rows[0] * kTile;
#pragma unroll
    for (int s = 0; s < 3; ++s)
        if (s < nsub)
            store_subtile<T>(m, t0 + srow[s] * 16, t0 + scol[s] * 16 + r16, acc[s], lane, true);
}

// ---- the kernels: workgroup index -> block -> code path ---------------------------------------
template <typename T>
__global__ __launch_bounds__(kThreads) void tbs_syrk_kernel(Plan plan, int N, int M, T alpha,
                                                            const T* __restrict__ A, int64_t lda,
                                                            T beta, T* __restrict__ C, int64_t ldc)
{
    __shared__ __attribute__((aligned(16))) unsigned char smem[kLdsBytes];
    T* lds = reinterpret_cast<T*>(smem);
    Item it;
    tbs_decode(plan, (int32_t)blockIdx.x, it);
    const Mats<T> m = {A, lda, N, A, lda, N, C, ldc, M, alpha, beta, true};
    if (it.kind == kTri) {
        run_block<T, TriShape>(it, m, lds);
    } else if (it.kind == kRect) {
        run_block<T, RectShape>(it, m, lds);
    } else if (it.kind == kDiag) {
        run_diag<T>(it, m, lds);
    }
}

// C (m x n) <- beta*C + alpha * R (m x K) * Q (n x K)^T, rectangular blocks of 2 x 3 tiles.
template <typename T>
__global__ __launch_bounds__(kThreads) void gemm_nt_kernel(int m_rows, int n_cols, int K, T alpha,
                                                           const T* R, int64_t ldr, const T* Q,
                                                           int64_t ldq, T beta, T* C, int64_t ldc, int nJ)
{
    __shared__ __attribute__((aligned(16))) unsigned char smem[kLdsBytes];
    T* lds = reinterpret_cast<T*>(smem);
    const int I = blockIdx.x / nJ, J = blockIdx.x - I * nJ;
    const int Tm = (m_rows + kTile - 1) / kTile, Tn = (n_cols + kTile - 1) / kTile;
    Item it;
    it.kind = kRect;
    it.nrow = 0;
    it.ncol = 0;
#pragma unroll
    for (int q = 0; q < kRectCols; ++q) {
        const int t = J * kRectCols + q;
        it.rows[q] = (t < Tn) ? t : -1;
    }
#pragma unroll
    for (int r = 0; r < kRectRows; ++r) {
        const int t = I * kRectRows + r;
        it.rows[kRectCols + r] = (t < Tm) ? t : -1;
    }
    const Mats<T> m = {R, ldr, m_rows, Q, ldq, n_cols, C, ldc, K, alpha, beta, false};
    run_block<T, RectShape>(it, m, lds);
}

template <typename T>
static hipError_t launch_syrk_t(const Plan& plan, int64_t N, int64_t M, double alpha, const void* A,
                                int64_t lda, double beta, void* C, int64_t ldc, hipStream_t stream)
{
    if (plan.n_items <= 0) return hipSuccess;
    hipLaunchKernelGGL(tbs_syrk_kernel<T>, dim3((unsigned)plan.n_items), dim3(kThreads), 0, stream, plan,
                       (int)N, (int)M, (T)alpha, (const T*)A, lda, (T)beta, (T*)C, ldc);
    return hipGetLastError();
}

hipError_t launch_syrk(bool f32, const Plan& plan, int64_t N, int64_t M, double alpha, const void* A,
                       int64_t lda, double beta, void* C, int64_t ldc, hipStream_t stream)
{
    return f32 ? launch_syrk_t<float>(plan, N, M, alpha, A, lda, beta, C, ldc, stream)
               : launch_syrk_t<double>(plan, N, M, alpha, A, lda, beta, C, ldc, stream);
}

template <typename T>
static hipError_t launch_gemm_t(int64_t m, int64_t n, int64_t K, double alpha, const void* R, int64_t ldr,
                                const void* Q, int64_t ldq, double beta, void* C, int64_t ldc,
                                hipStream_t stream)
{
    if (m <= 0 || n <= 0) return hipSuccess;
    const int Tm = (int)((m + kTile - 1) / kTile), Tn = (int)((n + kTile - 1) / kTile);
    const int nI = (Tm + kRectRows - 1) / kRectRows, nJ = (Tn + kRectCols - 1) / kRectCols;
    hipLaunchKernelGGL(gemm_nt_kernel<T>, dim3((unsigned)(nI * nJ)), dim3(kThreads), 0, stream, (int)m,
                       (int)n, (int)K, (T)alpha, (const T*)R, ldr, (const T*)Q, ldq, (T)beta, (T*)C, ldc, nJ);
    return hipGetLastError();
}

hipError_t launch_gemm_nt(bool f32, int64_t m, int64_t n, int64_t K, double alpha, const void* R,
                          int64_t ldr, const void* Q, int64_t ldq, double beta, void* C, int64_t ldc,
                          hipStream_t stream)
{
    return f32 ? launch_gemm_t<float>(m, n, K, alpha, R, ldr, Q, ldq, beta, C, ldc, stream)
               : launch_gemm_t<double>(m, n, K, alpha, R, ldr, Q, ldq, beta, C, ldc, stream);
}

}  // namespace tbs
