// syrk_kernels.hip -- Triangle Block SYRK for gfx950 (MI355X), fp64 and fp32.
//
// One workgroup (4 wavefronts, one per SIMD of a compute unit) executes one block of the plan:
//   * a triangle block TB(R), |R| = k = 4 tile rows: the k(k-1)/2 = 6 tiles C[r_u, r_v], u > v,
//     stay in registers (the paper's fast memory, Section 5.1.4: S = b^2 k(k-1)/2) while the k
//     row panels A[r_u, :] stream through LDS in chunks of KC columns (Algorithm 4's loop over
//     the columns of A, KC columns per step).  Every staged panel is used as left operand
//     (rows of the tile) and as right operand (columns of the tile): the symmetric reuse that
//     Section 5.1 is about;
//   * an augmented triangle block: the same plus two tiles of the diagonal zones, each between a row of
//     the block and one further row (8 tiles, all 256 accumulator registers of a lane in fp64, 6 panels);
//   * a rectangular block of at most 2 x 3 tiles (Algorithm 4's square-block part: the last l
//     tile rows and the recursion base), 5 panels for 6 tiles;
//   * a diagonal tile: one panel, only the 10 of 16 sub-tiles on or below the diagonal.
// Within a tile, wavefront w owns the 16-column strip w: 4 MFMA sub-tiles of 16 x 16 per tile.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <cstdlib>
#include <stdint.h>

#include <atomic>
#include <mutex>

#include "counter_slots.h"
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

// LDS: the assembly loops use a ring of chunk buffers (144 KB of the 160 KB a compute unit has); the
// checked C++ loop uses two padded buffers at the start of the same allocation.
constexpr int kLdsBytes = 144 * 1024;
static_assert(2 * kMaxPanels * kTile * Cfg<double>::LDK * 8 <= kLdsBytes, "checked path fits");
static_assert(2 * kMaxPanels * kTile * Cfg<float>::LDK * 4 <= kLdsBytes, "checked path fits");

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
    static constexpr bool may_be_diagonal(int) { return false; }     // (its tile rows are pairwise different)
};
struct RectShape {                        // panels 0..2 = column side, 3..4 = row side
    static constexpr int NP = 5, NA = 2, NB = 3, NSLOT = 6;
    static constexpr int a_panel(int i) { return 3 + i; }
    static constexpr int b_panel(int j) { return j; }
    static constexpr bool col_side(int p) { return p < 3; }
    static constexpr bool active(int, int) { return true; }
    static constexpr int slot(int i, int j) { return i * 3 + j; }
    static constexpr bool may_be_diagonal(int) { return true; }
};

struct AugShape {                         // panels 0..3 = R in zone order, 4 and 5 = the further rows
    static constexpr int NP = 6, NA = 5, NB = 5, NSLOT = 12;
    static constexpr int a_panel(int i) { return i + 1; }
    static constexpr int b_panel(int j) { return j < 4 ? j : 5; }
    static constexpr bool col_side(int) { return false; }
    // slots 0..5: the triangle block; 6, 7: panel 4 x panel 0 / 1; 8..11: panel 5 x panel 2, panel 2 x
    // panel 5, panel 5 x panel 3, panel 3 x panel 5 (a block has one slot of 6..7 and one of 8..11)
    static constexpr int slot(int i, int j)
    {
        if (i < 3 && j < 3 && j <= i) return i * (i + 1) / 2 + j;
        if (i == 3 && j < 2) return 6 + j;
        if (i == 4 && j == 2) return 8;
        if (i == 1 && j == 4) return 9;
        if (i == 4 && j == 3) return 10;
        if (i == 2 && j == 4) return 11;
        return -1;
    }
    static constexpr bool active(int i, int j) { return slot(i, j) >= 0; }
    static constexpr bool may_be_diagonal(int s) { return s == 6 || s == 7 || s == 8; }
};

// which slots / row-side panels / column-side panels / LDS panels a set of slots needs
template <class Shape> constexpr bool slot_on(uint32_t slots, int i, int j)
{
    return Shape::active(i, j) && ((slots >> (Shape::slot(i, j) & 31)) & 1u);
}
template <class Shape> constexpr bool a_used(uint32_t slots, int i)
{
    bool u = false;
    for (int j = 0; j < Shape::NB; ++j) u = u || slot_on<Shape>(slots, i, j);
    return u;
}
template <class Shape> constexpr bool b_used(uint32_t slots, int j)
{
    bool u = false;
    for (int i = 0; i < Shape::NA; ++i) u = u || slot_on<Shape>(slots, i, j);
    return u;
}
template <class Shape> constexpr uint32_t panels_of(uint32_t slots)
{
    uint32_t pm = 0;
    for (int i = 0; i < Shape::NA; ++i)
        if (a_used<Shape>(slots, i)) pm |= 1u << Shape::a_panel(i);
    for (int j = 0; j < Shape::NB; ++j)
        if (b_used<Shape>(slots, j)) pm |= 1u << Shape::b_panel(j);
    return pm;
}

// ---- operands of one launch --------------------------------------------------------------------
// One operand matrix: element (row, k) of its panels is p[row * rs + k * ks].  Row panels (SYRK, SYR2K,
// the products of the Cholesky driver; the matrix is stored row-major with the contraction index along
// a row): rs = leading dimension, ks = 1.  Column panels (the Gram form A^T A: a "row" of the operand
// is a column of the stored matrix): rs = 1, ks = leading dimension.
template <typename T>
struct Side {
    const T* p;
    int64_t rs, ks;
};

// C[rows, cols] <- beta*C + alpha * sum over the passes of R_pass[rows, :] * Q_pass[cols, :]^T.  SYRK
// has one pass with R == Q == A and updates only tiles strictly below the diagonal (and the lower
// part of diagonal tiles); the general product (used by the Cholesky driver for its triangular solves)
// has two different matrices and updates every tile; SYR2K has two passes, (A, B) and (B, A).
template <typename T, int NPASS_ = 1>
struct Mats {
    static constexpr int NPASS = NPASS_;
    Side<T> R[NPASS_];  int nr;             // row-side operand of every pass, nr panel rows
    Side<T> Q[NPASS_];  int nq;             // column-side operand, nq panel rows
    T* C;        int64_t ldc;
    int M;                                  // contraction length
    T alpha, beta;
    bool lower;                             // true: SYRK (tile (r,q) only if q < r)
};

// ---- global -> register -> LDS staging of one chunk --------------------------------------------
template <typename T>
__device__ __forceinline__ bool vec_ok(const T* p, int64_t ld)
{
    return ((reinterpret_cast<uintptr_t>(p) & 15) == 0) && ((ld * sizeof(T)) % 16 == 0);
}

// Thread t moves, for every panel, two 16-byte pieces: rows t/8 and t/8 + 32, columns
// [ (t%8)*VEC, +VEC ) of the chunk: 8 threads cover the 128 contiguous bytes of one row.
// PANELS (compile time) selects the panels that are staged at all.
template <typename T, int NP, uint32_t PANELS>
struct Stager {
    static constexpr int KC = Cfg<T>::KC, LDK = Cfg<T>::LDK, VEC = Cfg<T>::VEC;
    u32x4 reg[2 * NP];
    const T* base[NP];                     // matrix of each panel (wavefront-uniform)
    int64_t rs[NP], ks[NP];                // its strides between panel rows / along the contraction
    int64_t off[NP];                       // element offset of the thread's first piece in chunk 0
    uint32_t valid;                        // bit 2p+h: piece h of panel p exists (inside the matrix)

    static constexpr bool on(int p) { return (PANELS >> p) & 1u; }

    // prow[p]: tile row of panel p (-1: absent) in matrix base_[p] with nrows[p] rows.
    __device__ __forceinline__ void init(const T* const (&base_)[NP], const int64_t (&rs_)[NP],
                                         const int64_t (&ks_)[NP], const int (&nrows)[NP],
                                         const int (&prow)[NP], int tid)
    {
        const int v = tid & 7, r = tid >> 3;
        valid = 0;
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            if (!on(p)) continue;
            base[p] = base_[p];
            rs[p] = rs_[p];
            ks[p] = ks_[p];
            const int grow = prow[p] * kTile + r;
            off[p] = (int64_t)grow * rs_[p] + (int64_t)(v * VEC) * ks_[p];
            if (prow[p] >= 0 && grow < nrows[p]) valid |= 1u << (2 * p);
            if (prow[p] >= 0 && grow + 32 < nrows[p]) valid |= 2u << (2 * p);
        }
    }

    // General case.  whole: the chunk lies inside [0, M), the contraction index runs along memory
    // and 16-byte loads are legal; otherwise elements are fetched one by one and those beyond M read
    // as zero.  Missing rows read as zero.
    __device__ __forceinline__ void load_checked(int M, int k0, bool whole, int tid)
    {
        const int v = tid & 7;
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            if (!on(p)) continue;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                union { u32x4 q4; T e[VEC]; } tmp;
                tmp.q4 = u32x4{0u, 0u, 0u, 0u};
                if ((valid >> (2 * p + h)) & 1u) {
                    const T* src = base[p] + off[p] + (int64_t)h * 32 * rs[p] + (int64_t)k0 * ks[p];
                    if (whole) {
                        tmp.q4 = *reinterpret_cast<const u32x4*>(src);
                    } else {
#pragma unroll
                        for (int e = 0; e < VEC; ++e)
                            if (k0 + v * VEC + e < M) tmp.e[e] = src[(int64_t)e * ks[p]];
                    }
                }
                reg[p * 2 + h] = tmp.q4;
            }
        }
    }

    __device__ __forceinline__ void store(T* __restrict__ buf, int tid) const
    {
        const int v = tid & 7, r = tid >> 3;
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            if (!on(p)) continue;
#pragma unroll
            for (int h = 0; h < 2; ++h)
                *reinterpret_cast<u32x4*>(&buf[(p * kTile + h * 32 + r) * LDK + v * VEC]) = reg[p * 2 + h];
        }
    }
};

// ---- MFMA operands of one k-step (4 columns of the chunk) ---------------------------------------
// Row side: the four 16-row groups of each row-side panel.  Column side: the wavefront's group of
// each column-side panel.  Lane l holds element [row l%16][column l/16] of its 16 x 4 piece, which
// is the layout of both MFMA inputs, so a panel that is row side of one tile and column side of
// another is read with the same addressing.  SLOTS (compile time) selects what is read at all.
template <typename T, class Shape, uint32_t SLOTS>
struct Operands {
    T a[Shape::NA][4];
    T b[Shape::NB];
    __device__ __forceinline__ void load(const T* __restrict__ buf, int ks, int w, int lane)
    {
        constexpr int LDK = Cfg<T>::LDK;
        const T* base = buf + (lane & 15) * LDK + (lane >> 4) + ks * 4;
#pragma unroll
        for (int i = 0; i < Shape::NA; ++i) {
            if (!a_used<Shape>(SLOTS, i)) continue;
#pragma unroll
            for (int rb = 0; rb < 4; ++rb) a[i][rb] = base[(Shape::a_panel(i) * kTile + rb * 16) * LDK];
        }
#pragma unroll
        for (int j = 0; j < Shape::NB; ++j) {
            if (!b_used<Shape>(SLOTS, j)) continue;
            b[j] = base[(Shape::b_panel(j) * kTile + w * 16) * LDK];
        }
    }
};

// MFMAs of one k-step for the slots of SLOTS that the run-time mask has.
template <typename T, class Shape, uint32_t SLOTS>
__device__ __forceinline__ void mfma_step(const Operands<T, Shape, SLOTS>& op,
                                          typename Cfg<T>::acc_t (&acc)[Shape::NSLOT][4], uint32_t pmask)
{
#pragma unroll
    for (int i = 0; i < Shape::NA; ++i)
#pragma unroll
        for (int j = 0; j < Shape::NB; ++j)
            if (slot_on<Shape>(SLOTS, i, j)) {
                const int s = Shape::slot(i, j);
                if (pmask & (1u << s)) {
#pragma unroll
                    for (int rb = 0; rb < 4; ++rb)
                        acc[s][rb] = Cfg<T>::mfma(op.a[i][rb], op.b[j], acc[s][rb]);
                }
            }
}


// A value that is the same in every lane, moved to a scalar register (the assembly loops take their
// pointers and counts as scalar operands; the compiler cannot always see that a value is uniform).
__device__ __forceinline__ uint32_t to_scalar(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }
template <typename P>
__device__ __forceinline__ const P* to_scalar(const P* p)
{
    const uint64_t u = (uint64_t)(uintptr_t)p;
    const uint32_t lo = to_scalar((uint32_t)u), hi = to_scalar((uint32_t)(u >> 32));
    return (const P*)(uintptr_t)(((uint64_t)hi << 32) | lo);
}

// ---- the main loop in assembly (generated) -----------------------------------------------------
struct AsmLoopArgs {
    uint32_t ada[8];        // LDS byte address of the lane's row-side operand piece for k-step j
    uint32_t adb[8];        // same for the column side (includes the wavefront's 16-row group)
    const void* gP[6];      // first element of each panel the block uses (tile row, first column), in panel order
    uint32_t nch;           // chunks, >= 1
    uint32_t step;          // bytes per chunk along a row
    uint32_t m0base;        // LDS byte address of the wavefront's 1 KB slice in panel 0, half 0, buffer 0
};
#include "syrk_asm_loops.inc"

// The 16 elements of C that one lane holds of a 64 x 16 tile strip (4 row groups x 4 registers).
template <typename T>
struct TileStrip {
    T v[4][4];
    // CHECK: rows / columns beyond the matrix are skipped (ragged last tile)
    // diag: the strip belongs to a diagonal tile; elements above the diagonal are not touched
    template <bool CHECK, class MatsT>
    __device__ __forceinline__ void load(const MatsT& m, int row0, int col, int lane, bool diag)
    {
#pragma unroll
        for (int rb = 0; rb < 4; ++rb)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int row = row0 + rb * 16 + Cfg<T>::row_of(g, lane);
                const bool ok = (!CHECK || (row < m.nr && col < m.nq)) && (!diag || col <= row);
                v[rb][g] = ok ? m.C[(int64_t)row * m.ldc + col] : T(0);
            }
    }
};

// Writes C <- beta*old + alpha*acc for one tile strip (beta == 0: old is not used).
template <typename T, bool CHECK, class MatsT>
__device__ __forceinline__ void store_strip(const MatsT& m, int row0, int col, int lane,
                                            const typename Cfg<T>::acc_t (&acc)[4], const TileStrip<T>& old,
                                            bool diag)
{
#pragma unroll
    for (int rb = 0; rb < 4; ++rb)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int row = row0 + rb * 16 + Cfg<T>::row_of(g, lane);
            if ((!CHECK || (row < m.nr && col < m.nq)) && (!diag || col <= row)) {
                const T v = m.alpha * acc[rb][g];
                m.C[(int64_t)row * m.ldc + col] = (m.beta != T(0)) ? m.beta * old.v[rb][g] + v : v;
            }
        }
}

// The same for whole tiles on the fast path: the lane's 16 elements lie at byte offsets from the first
// element of the wavefront's strip that are the same for every tile (64 rows of C span less than 4 GiB:
// checked by the caller).  MAY_DIAG (a constant once the caller's loops are unrolled): the tile may be a diagonal tile (`diag`, run time), of
// which only the elements on or below the diagonal are read and written.  Nothing here branches around
// a load: the compiler waits for every outstanding memory operation, stores included, wherever a loaded
// value is used behind a branch, which made the sixteen stores of such a strip wait for each other.  A
// lane's element above the diagonal is replaced by the diagonal element of its column for the load (a
// valid address; the value is not used); only the stores are predicated.
template <typename T>
struct StripOffsets {
    uint32_t off[4][4];
    uint32_t on_diagonal;               // the element (c, c) of the lane's column c
    uint32_t on_or_below;               // bit 4 rb + g: the element is on or below the diagonal of a diagonal tile
    __device__ __forceinline__ void init(int64_t ldc, int lane, int w)
    {
        on_or_below = 0;
        const int c = w * 16 + (lane & 15);
        on_diagonal = (uint32_t)(((int64_t)c * ldc + (lane & 15)) * (int64_t)sizeof(T));
#pragma unroll
        for (int rb = 0; rb < 4; ++rb)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int row = rb * 16 + Cfg<T>::row_of(g, lane);
                off[rb][g] = (uint32_t)(((int64_t)row * ldc + (lane & 15)) * (int64_t)sizeof(T));
                if (c <= row) on_or_below |= 1u << (4 * rb + g);
            }
    }
};

template <typename T>
__device__ __forceinline__ void load_strip_fast(TileStrip<T>& old, const T* strip, const StripOffsets<T>& so,
                                                const bool MAY_DIAG, bool diag)
{
    const char* base = reinterpret_cast<const char*>(strip);
#pragma unroll
    for (int rb = 0; rb < 4; ++rb)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            uint32_t o = so.off[rb][g];
            if (MAY_DIAG) o = (!diag || ((so.on_or_below >> (4 * rb + g)) & 1u)) ? o : so.on_diagonal;
            old.v[rb][g] = *reinterpret_cast<const T*>(base + o);
        }
}

template <typename T>
__device__ __forceinline__ void store_strip_fast(T* strip, const StripOffsets<T>& so, T alpha, T beta,
                                                 const typename Cfg<T>::acc_t (&acc)[4], const TileStrip<T>& old,
                                                 const bool MAY_DIAG, bool diag)
{
    char* base = reinterpret_cast<char*>(strip);
#pragma unroll
    for (int rb = 0; rb < 4; ++rb)
#pragma unroll
        for (int g = 0; g < 4; ++g)
            if (!MAY_DIAG || !diag || ((so.on_or_below >> (4 * rb + g)) & 1u)) {
                const T v = alpha * acc[rb][g];
                *reinterpret_cast<T*>(base + so.off[rb][g]) = (beta != T(0)) ? beta * old.v[rb][g] + v : v;
            }
}

// ---- blocks cut along the contraction dimension -------------------------------------------------
// A sliced block is computed by `slices` workgroups, each over its share of the columns of A.  Every
// one writes its accumulators to its own place in the workspace (in register order: coalesced, no
// layout change; device-scope stores, see part_store), then adds one to the block's counter; the workgroup that finds the counter at
// slices - 1 is the last: it reads all parts back, adds them in the order of the slices (so the
// result does not depend on who finished when), and runs the ordinary epilogue on the sum.  No
// workgroup ever waits for another.  part == nullptr: an ordinary, whole block.
// Device-scope accesses to the parts of cut blocks.  The dies of the chip have an L2 each, which are not
// coherent with one another for ordinary loads and stores; a `__threadfence()` makes a workgroup's stores
// visible to the others by writing back every dirty line of its die's L2 and invalidating that L2
// (`buffer_wbl2 sc1` + `buffer_inv sc1`): tens of microseconds per fence next to running blocks whose
// panels the invalidation throws out.  Relaxed atomic stores and loads at device scope instead go through
// to the memory side line by line and need no fence: a part is complete at device scope when its stores have
// been acknowledged (`s_waitcnt vmcnt(0)`), and the counter, a device-scope atomic as well, is bumped after
// that; whoever reads the parts does so after its own bump has returned the full count.
__device__ __forceinline__ void part_store(double* p, double v)
{
    __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), (unsigned long long)__double_as_longlong(v),
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void part_store(float* p, float v)
{
    __hip_atomic_store(reinterpret_cast<unsigned int*>(p), __float_as_uint(v), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ double part_load(const double* p)
{
    return __longlong_as_double((long long)__hip_atomic_load(reinterpret_cast<const unsigned long long*>(p),
                                                             __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}
__device__ __forceinline__ float part_load(const float* p)
{
    return __uint_as_float(__hip_atomic_load(reinterpret_cast<const unsigned int*>(p), __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_AGENT));
}

template <typename T>
struct SliceCtx {
    T* part = nullptr;              // this block's stretch of the workspace: [slices][NSLOT][16][256]
    unsigned int* ctr = nullptr;    // parts finished so far (zero before and after the launch)
    int* flag = nullptr;            // one int of LDS
    int slices = 1, slice = 0;
};

// One block from start to end.  LDS holds two chunks; registers hold the operands of two k-steps
// and one chunk in flight from global memory.  Per chunk: the operands of k-step s+1 are read from
// LDS before the MFMAs of k-step s are issued; before the last k-step the next chunk is written to
// the other LDS buffer, the workgroup synchronises, the first operands of the next chunk are read
// and the chunk after that is requested from global memory, all hidden behind the last k-step's
// MFMAs.
//   FAST: the slots SLOTS are exactly the block's and M >= KC (`ragged`: a
//   panel has fewer than 64 rows inside the matrix; the loop then reads its last row in place of the
//   missing ones and the epilogue checks rows and columns).  The chunk loop over the whole chunks then has no
//   test and no branch, so the accumulators stay in their registers across it; columns beyond the
//   last whole chunk go through the checked loop afterwards.
//   !FAST: anything else (ragged edges, odd leading dimensions, unusual slot sets); same schedule
//   with every access checked.
template <typename T, class Shape, uint32_t SLOTS, bool FAST, bool CAN_SLICE, class MatsT>
__device__ __forceinline__ void block_body(const MatsT& m, const int (&prow)[Shape::NP], uint32_t pmask,
                                           uint32_t dmask, T* lds, const SliceCtx<T>& sc, bool ragged)
{
    constexpr int NP = Shape::NP;
    constexpr int KC = Cfg<T>::KC, KS = KC / 4, LDK = Cfg<T>::LDK;
    constexpr int kBufElems = kMaxPanels * kTile * LDK;
    constexpr uint32_t PANELS = panels_of<Shape>(SLOTS);
    static_assert(KS % 2 == 0, "operand double buffering assumes an even number of k-steps");
    typedef typename Cfg<T>::acc_t acc_t;
    typedef Operands<T, Shape, SLOTS> Ops;
    // (the thread's index passes through an empty assembly statement: what is derived from it -- LDS and
    // global offsets, a dozen or two registers -- is then computed inside each instance of this function,
    // not once for all of them at the top of the kernel, where it would occupy registers across every
    // assembly loop, the largest of which leaves the compiler 136 of them)
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);

    int nrows[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) nrows[p] = Shape::col_side(p) ? m.nq : m.nr;

    acc_t acc[Shape::NSLOT][4];
    {
        // (a zero the compiler cannot see through: otherwise it keeps a vector of zeros in registers for
        // the whole kernel, across every assembly loop)
        T zero = T(0);
        asm volatile("" : "+v"(zero));
#pragma unroll
        for (int s = 0; s < Shape::NSLOT; ++s)
#pragma unroll
            for (int rb = 0; rb < 4; ++rb) acc[s][rb] = acc_t{zero, zero, zero, zero};
    }

    const int M = m.M;
    // one pass over the contraction dimension per operand pair; the accumulators carry over (the
    // operands of a pass are chosen by
    // comparison, not by indexing, so that the kernel's arguments stay in registers)
#pragma unroll
    for (int pass = 0; pass < MatsT::NPASS; ++pass) {
    const Side<T> side_r = (MatsT::NPASS > 1 && pass > 0) ? m.R[MatsT::NPASS - 1] : m.R[0];
    const Side<T> side_q = (MatsT::NPASS > 1 && pass > 0) ? m.Q[MatsT::NPASS - 1] : m.Q[0];
    const T* base[NP];
    int64_t rs[NP], ks[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const Side<T>& sd = Shape::col_side(p) ? side_q : side_r;
        base[p] = sd.p;
        rs[p] = sd.rs;
        ks[p] = sd.ks;
    }
    if (MatsT::NPASS > 1 && pass > 0) __syncthreads();      // every wavefront has left the previous pass's LDS
    if constexpr (FAST) {
        // Addresses for the assembly loop (layout and schedule: gen_asm_loops.py).  In LDS a chunk
        // buffer holds the used panels back to back, 64 rows of 128 bytes each, the 16-byte pieces of
        // row r permuted by XOR with r mod 8.  Global addresses are a 64-bit pointer per panel plus a
        // 32-bit offset per lane; the caller has checked that 64 rows of either matrix span less than 4 GiB.
        constexpr int ES = (int)sizeof(T);
        typedef __attribute__((address_space(3))) unsigned char lds_byte;
        const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_byte*)lds;
        // Column panels (the contraction index runs across memory rows; all operands of a launch are of
        // one kind): a 16-byte piece then holds VEC consecutive panel rows at one k.  The 2 KB of a
        // 16-row group hold its pieces in the order (k, group of VEC rows), so that a wavefront's operand
        // read (16 rows x 4 k) covers 4 x 128 (64) contiguous bytes and a load instruction deposits, for 8
        // (16) values of k, the 128 (64) contiguous bytes of 16 rows: no bank conflicts, no permutation.
        const bool colp = ks[Shape::b_panel(0)] != 1;
        constexpr int VEC = Cfg<T>::VEC;
        AsmLoopArgs g;
        {
            const uint32_t r16 = lane & 15, gq = lane >> 4, x = r16 & 7;
#pragma unroll
            for (int j = 0; j < KS; ++j) {
                uint32_t a;
                if (colp)          // element k = 4 j + gq of row r16: byte (k * 16 + r16) * ES of the group
                    a = ((uint32_t)(4 * j + gq) * 16 + r16) * ES;
                else if (ES == 8)  // element k = 4 ks + gq: piece (2 ks + gq/2) ^ x, half gq & 1
                    a = r16 * 128 + ((((gq >> 1) ^ (x & 1)) | (((uint32_t)j ^ (x >> 1)) << 1)) << 4) + (gq & 1) * 8;
                else               // element k = 4 ks + gq: piece ks ^ x, word gq
                    a = r16 * 128 + (((uint32_t)j ^ x) << 4) + gq * 4;
                g.ada[j] = lds0 + a;
                g.adb[j] = lds0 + a + (uint32_t)w * 2048;
            }
        }
        g.nch = (uint32_t)(M / KC);                         // whole chunks; the rest follows below
        g.step = to_scalar((uint32_t)(KC * ES * ks[Shape::b_panel(0)]));   // (all operands of a launch advance alike)
        g.m0base = lds0 + (uint32_t)w * 1024;
        uint32_t go[2 * NP];
        int q = 0, np_used = 0;
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            if (!((PANELS >> p) & 1u)) continue;
            g.gP[np_used++] = to_scalar(base[p] + (int64_t)prow[p] * kTile * rs[p]);
            const int rows_in = min(kTile, nrows[p] - prow[p] * kTile);
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                if (colp) {
                    // LDS position (16-byte units) h * 256 + w * 64 + lane of the panel's chunk: 16-row
                    // group 2 h + w / 2, piece (w % 2) * 64 + lane inside it = (k, group of VEC rows).
                    // A panel that reaches beyond the matrix has a multiple of VEC rows inside (checked
                    // by the caller); the last whole group of rows stands in for the missing ones.
                    const int piece = (w & 1) * 64 + lane, per_k = 16 / VEC;
                    const int k = piece / per_k;
                    const int row = min((2 * h + (w >> 1)) * 16 + (piece % per_k) * VEC, rows_in - VEC);
                    go[q++] = (uint32_t)(((int64_t)k * ks[p] + row) * ES);
                } else {
                    // this lane's piece of the wavefront's 8 rows: row 8w + lane/8 of the half-panel,
                    // global piece (lane%8) ^ (lane/8) so that it lands at LDS position lane%8; the offset
                    // is relative to the panel's first row (64 rows of a matrix stay below 4 GiB: checked
                    // by the caller)
                    // (a panel that reaches beyond the matrix: its last row stands in for the missing ones;
                    // what is computed from them belongs to rows or columns of C that are never stored)
                    const int64_t row = min(h * 32 + w * 8 + (lane >> 3), rows_in - 1);
                    go[q++] = (uint32_t)(row * rs[p] * ES + (((lane & 7) ^ (lane >> 3)) << 4));
                }
            }
        }
        AsmLoop<T, Shape, SLOTS>::run(acc, g, go);
    }
    // The checked loop over the columns [k_begin, M) (everything, or what the assembly loop left over):
    // two padded LDS buffers, chunks staged through registers, every access checked.
    auto checked_columns = [&](int k_begin) {
        const int nch = (M - k_begin + KC - 1) / KC;
        if (nch <= 0) return;
        Stager<T, NP, PANELS> st;
        st.init(base, rs, ks, nrows, prow, tid);
        const bool aligned = side_r.ks == 1 && side_q.ks == 1 && vec_ok(side_r.p, side_r.rs) &&
                             vec_ok(side_q.p, side_q.rs);
        st.load_checked(M, k_begin, aligned && k_begin + KC <= M, tid);
        st.store(lds, tid);
        __syncthreads();
        if (nch > 1) st.load_checked(M, k_begin + KC, aligned && k_begin + 2 * KC <= M, tid);
        Ops op[2];
        op[0].load(lds, 0, w, lane);
        for (int ch = 0; ch < nch; ++ch) {
            T* cur = lds + (ch & 1) * kBufElems;
            T* nxt = lds + ((ch + 1) & 1) * kBufElems;
            const bool more = ch + 1 < nch;
#pragma unroll
            for (int ks = 0; ks < KS - 1; ++ks) {
                op[(ks + 1) & 1].load(cur, ks + 1, w, lane);
                mfma_step<T, Shape, SLOTS>(op[ks & 1], acc, pmask);
            }
            if (more) st.store(nxt, tid);
            __syncthreads();
            if (more) {
                op[0].load(nxt, 0, w, lane);
                if (ch + 2 < nch) {
                    const int k0 = k_begin + (ch + 2) * KC;
                    st.load_checked(M, k0, aligned && k0 + KC <= M, tid);
                }
            }
            mfma_step<T, Shape, SLOTS>(op[(KS - 1) & 1], acc, pmask);
        }
    };
    if constexpr (FAST) {
        // the columns beyond the last whole chunk (M is no multiple of KC)
        if (M % KC != 0) {
            __syncthreads();                                // the ring is free: every wavefront has left the loop
            checked_columns(M - M % KC);
        }
    } else {
        checked_columns(0);
    }
    }   // passes

    if (CAN_SLICE && sc.part != nullptr) {                  // uniform
        constexpr int NS = Shape::NSLOT;
#pragma unroll
        for (int s = 0; s < NS; ++s)
            if (FAST ? ((SLOTS >> s) & 1u) != 0 : ((pmask >> s) & 1u) != 0) {
                T* dst = sc.part + ((size_t)(sc.slice * NS + s) * 16) * kThreads + tid;
#pragma unroll
                for (int rb = 0; rb < 4; ++rb)
#pragma unroll
                    for (int g = 0; g < 4; ++g) part_store(&dst[(rb * 4 + g) * kThreads], acc[s][rb][g]);
            }
        __builtin_amdgcn_s_waitcnt(0x0F70);                 // vmcnt(0): this thread's share of the part is out ...
        __syncthreads();                                    // ... and everybody's ...
        if (tid == 0)                                       // ... before the count
            *sc.flag = (__hip_atomic_fetch_add(sc.ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) ==
                        (unsigned)(sc.slices - 1)) ? 1 : 0;
        __syncthreads();
        if (*sc.flag == 0) return;                          // not the last part of this block
        T zero = T(0);
        asm volatile("" : "+v"(zero));                      // (as above: no vector of zeros kept for the whole kernel)
#pragma unroll
        for (int s = 0; s < NS; ++s)
            if (FAST ? ((SLOTS >> s) & 1u) != 0 : ((pmask >> s) & 1u) != 0) {
#pragma unroll
                for (int rb = 0; rb < 4; ++rb)
#pragma unroll
                    for (int g = 0; g < 4; ++g) acc[s][rb][g] = zero;
                // two parts are requested together (32 loads in flight per lane), then added in order
                for (int sl0 = 0; sl0 < sc.slices; sl0 += 2) {
                    T v[2][16];
#pragma unroll
                    for (int d = 0; d < 2; ++d) {
                        const int sl = min(sl0 + d, sc.slices - 1);
                        const T* src = sc.part + ((size_t)(sl * NS + s) * 16) * kThreads + tid;
#pragma unroll
                        for (int e = 0; e < 16; ++e) v[d][e] = part_load(&src[e * kThreads]);
                    }
#pragma unroll
                    for (int d = 0; d < 2; ++d)
                        if (sl0 + d < sc.slices) {          // uniform
#pragma unroll
                            for (int rb = 0; rb < 4; ++rb)
#pragma unroll
                                for (int g = 0; g < 4; ++g) acc[s][rb][g] += v[d][rb * 4 + g];
                        }
                }
            }
        if (tid == 0)                                       // for the next launch that uses this counter
            __hip_atomic_store(sc.ctr, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }

    // Epilogue.
    const int col16 = w * 16 + (lane & 15);
    bool any_may_be_diagonal = false;
#pragma unroll
    for (int sl = 0; sl < Shape::NSLOT; ++sl)
        if (((SLOTS >> sl) & 1u) && Shape::may_be_diagonal(sl)) any_may_be_diagonal = true;
    // (eight tiles in fp64 take every accumulator register, the compiler has no room to spare there: only
    // the second form below, which needs fewer address registers)
    constexpr bool kNoSpareRegisters = sizeof(T) == 8 && __builtin_popcount(SLOTS) > 6;
    if (FAST && !ragged && !kNoSpareRegisters && (!any_may_be_diagonal || dmask == 0)) {
        // no diagonal tile in the block: the old values of three tiles are requested at once (the operand
        // registers of the loop are free now), then their strips are computed and stored
        const bool rd = m.beta != T(0);
#pragma unroll
        for (int s0 = 0; s0 < Shape::NSLOT; s0 += 3) {      // three tiles' old values in flight at a time
            TileStrip<T> old[3];
#pragma unroll
            for (int i = 0; i < Shape::NA; ++i)
#pragma unroll
                for (int j = 0; j < Shape::NB; ++j) {
                    const int sl = Shape::slot(i, j);
                    if (slot_on<Shape>(SLOTS, i, j) && sl >= s0 && sl < s0 + 3 && rd)
                        old[sl - s0].template load<false>(m, prow[Shape::a_panel(i)] * kTile,
                                                          prow[Shape::b_panel(j)] * kTile + col16, lane, false);
                }
#pragma unroll
            for (int i = 0; i < Shape::NA; ++i)
#pragma unroll
                for (int j = 0; j < Shape::NB; ++j) {
                    const int sl = Shape::slot(i, j);
                    if (slot_on<Shape>(SLOTS, i, j) && sl >= s0 && sl < s0 + 3)
                        store_strip<T, false>(m, prow[Shape::a_panel(i)] * kTile,
                                              prow[Shape::b_panel(j)] * kTile + col16, lane, acc[sl], old[sl - s0],
                                              false);
                }
        }
    } else if (FAST && !ragged && (int64_t)kTile * m.ldc * (int64_t)sizeof(T) < ((int64_t)1 << 32)) {
        // blocks with diagonal tiles (rectangles of triangular regions, some augmented triangle blocks)
        // the old values of EG tiles are requested at once (the operand registers of the loop are free
        // now), then their strips are computed and stored.  Tiles are taken in the order of their slots;
        // EG is what fits the registers: all tiles in fp32 (at most 128 registers of values), up to four
        // in fp64, plus the 16 offsets.
        const bool rd = m.beta != T(0);
        constexpr int NT = __builtin_popcount(SLOTS);
        constexpr int EG = (sizeof(T) == 4 || NT <= 4) ? NT : (NT + 1) / 2;
        StripOffsets<T> so;
        so.init(m.ldc, lane, w);
#pragma unroll
        for (int t0 = 0; t0 < NT; t0 += EG) {
            TileStrip<T> old[EG];
#pragma unroll
            for (int i = 0; i < Shape::NA; ++i)
#pragma unroll
                for (int j = 0; j < Shape::NB; ++j)
                    if (slot_on<Shape>(SLOTS, i, j)) {
                        const int sl = Shape::slot(i, j);
                        const int d = __builtin_popcount(SLOTS & ((1u << sl) - 1u));    // place among the block's tiles
                        if (d >= t0 && d < t0 + EG && rd)
                            load_strip_fast(old[d - t0],
                                            m.C + (int64_t)prow[Shape::a_panel(i)] * kTile * m.ldc +
                                                prow[Shape::b_panel(j)] * kTile + w * 16,
                                            so, Shape::may_be_diagonal(sl), ((dmask >> sl) & 1u) != 0);
                    }
            // every old value has arrived before the first (predicated) store: s_waitcnt vmcnt(0), told to
            // the compiler so that it places no waits of its own between the stores
            // (only where a tile of the group may be diagonal: otherwise the compiler's own waits let the
            // first tile's arithmetic and stores start while the later tiles' values are still arriving)
            bool any_diag = false;
#pragma unroll
            for (int sl = 0; sl < Shape::NSLOT; ++sl) {
                const int d = __builtin_popcount(SLOTS & ((1u << sl) - 1u));
                if (((SLOTS >> sl) & 1u) && d >= t0 && d < t0 + EG && Shape::may_be_diagonal(sl)) any_diag = true;
            }
            if (rd && any_diag) __builtin_amdgcn_s_waitcnt(0x0F70);
#pragma unroll
            for (int i = 0; i < Shape::NA; ++i)
#pragma unroll
                for (int j = 0; j < Shape::NB; ++j)
                    if (slot_on<Shape>(SLOTS, i, j)) {
                        const int sl = Shape::slot(i, j);
                        const int d = __builtin_popcount(SLOTS & ((1u << sl) - 1u));
                        if (d >= t0 && d < t0 + EG)
                            store_strip_fast(m.C + (int64_t)prow[Shape::a_panel(i)] * kTile * m.ldc +
                                                 prow[Shape::b_panel(j)] * kTile + w * 16,
                                             so, m.alpha, m.beta, acc[sl], old[d - t0], Shape::may_be_diagonal(sl),
                                             ((dmask >> sl) & 1u) != 0);
                    }
        }
    } else {
#pragma unroll
        for (int i = 0; i < Shape::NA; ++i)
#pragma unroll
            for (int j = 0; j < Shape::NB; ++j)
                if (slot_on<Shape>(SLOTS, i, j)) {
                    const int s = Shape::slot(i, j);
                    if (pmask & (1u << s)) {
                        const int row0 = prow[Shape::a_panel(i)] * kTile;
                        const int col = prow[Shape::b_panel(j)] * kTile + col16;
                        TileStrip<T> old;
                        const bool diag = ((dmask >> s) & 1u) != 0;
                        if (m.beta != T(0)) old.template load<true>(m, row0, col, lane, diag);
                        store_strip<T, true>(m, row0, col, lane, acc[s], old, diag);
                    }
                }
    }
}

// The slot sets that have a branch-free instance: a triangle block on 4, 3 or 2 tile rows; a
// rectangle of r x c tiles, r <= 2, c <= 3; a two-row rectangle that straddles the diagonal (its
// first row without its last tile, without its last two tiles of three or two, or empty).
template <class Shape> struct FastSets;
template <> struct FastSets<TriShape> {
    static constexpr int N = 3;
    static constexpr uint32_t set(int n) { return n == 0 ? 0x3Fu : n == 1 ? 0x07u : 0x01u; }
};
template <> struct FastSets<RectShape> {
    static constexpr int N = 9;
    static constexpr uint32_t set(int n)
    {
        return n == 0 ? 0x3Fu : n == 1 ? 0x1Bu : n == 2 ? 0x09u : n == 3 ? 0x07u : n == 4 ? 0x03u : n == 5 ? 0x01u
             : n == 6 ? 0x3Bu : n == 7 ? 0x19u : 0x08u;
    }
};

template <> struct FastSets<AugShape> {
    static constexpr int N = 8;
    static constexpr uint32_t set(int n) { return 0x3Fu | (1u << (6 + (n >> 2))) | (1u << (8 + (n & 3))); }
};

template <typename T, class Shape, int IDX, bool CAN_SLICE, class MatsT>
__device__ __forceinline__ bool try_fast(const MatsT& m, const int (&prow)[Shape::NP], uint32_t pmask,
                                         uint32_t dmask, T* lds, const SliceCtx<T>& sc)
{
    if constexpr (IDX < FastSets<Shape>::N) {
        constexpr uint32_t SLOTS = FastSets<Shape>::set(IDX);
        if (pmask == SLOTS) {
            constexpr uint32_t PANELS = panels_of<Shape>(SLOTS);
            bool whole = true;
#pragma unroll
            for (int p = 0; p < Shape::NP; ++p)
                if ((PANELS >> p) & 1u) {
                    const int nrows = Shape::col_side(p) ? m.nq : m.nr;
                    whole = whole && (prow[p] + 1) * kTile <= nrows;
                }
            // a panel that reaches beyond the matrix (ragged last tile row) keeps the fast loop; the
            // epilogue then checks every row and column
            block_body<T, Shape, SLOTS, true, CAN_SLICE>(m, prow, pmask, dmask, lds, sc, !whole);
            return true;
        }
        return try_fast<T, Shape, IDX + 1, CAN_SLICE>(m, prow, pmask, dmask, lds, sc);
    } else {
        return false;
    }
}

// Whether the operands of a launch suit the assembly loops.
template <typename T, class MatsT>
__device__ __forceinline__ bool fast_path_ok(const MatsT& m)
{
    constexpr int KC = Cfg<T>::KC;
    // the assembly loop addresses a panel's 64 rows with 32-bit byte offsets from the panel's start
    const int64_t lim = (int64_t)1 << 32;
    // (rows need no alignment beyond that of an element: the loads into LDS take 16 bytes from any
    // element-aligned address, at full speed)
    // (column panels: the KC memory rows of a chunk instead, and whole 16-byte pieces inside the matrix)
    bool fast_ok = m.M >= KC;
#pragma unroll
    for (int pass = 0; pass < MatsT::NPASS; ++pass) {
        const Side<T>&r = m.R[pass], &q = m.Q[pass];
        const bool colp = r.ks != 1;
        fast_ok = fast_ok && (q.ks != 1) == colp;
        fast_ok = fast_ok && (colp ? KC * r.ks + kTile : kTile * r.rs) * (int64_t)sizeof(T) < lim &&
                  (colp ? KC * q.ks + kTile : kTile * q.rs) * (int64_t)sizeof(T) < lim;
        if (colp) fast_ok = fast_ok && r.rs == 1 && q.rs == 1 && m.nr % Cfg<T>::VEC == 0 && m.nq % Cfg<T>::VEC == 0;
    }
    return fast_ok;
}

// with_diag: tiles (r, r) belong to the block (their part on and below the diagonal)
template <typename T, class Shape, bool CAN_SLICE = true, class MatsT>
__device__ __forceinline__ void run_block(const Item& it, const MatsT& m, T* lds, const SliceCtx<T>& sc,
                                          bool with_diag = false)
{
    constexpr int NP = Shape::NP;
    int prow[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) prow[p] = it.rows[p];      // -1: panel absent
    uint32_t pmask = 0, dmask = 0;
#pragma unroll
    for (int i = 0; i < Shape::NA; ++i)
#pragma unroll
        for (int j = 0; j < Shape::NB; ++j) {
            const int ar = prow[Shape::a_panel(i)], br = prow[Shape::b_panel(j)];
            if (Shape::active(i, j) && ar >= 0 && br >= 0) {
                if (!m.lower || br < ar) pmask |= 1u << Shape::slot(i, j);
                if (m.lower && with_diag && br == ar) {
                    pmask |= 1u << Shape::slot(i, j);
                    dmask |= 1u << Shape::slot(i, j);
                }
            }
        }
    if (fast_path_ok<T>(m) && try_fast<T, Shape, 0, CAN_SLICE>(m, prow, pmask, dmask, lds, sc)) return;
    block_body<T, Shape, (1u << Shape::NSLOT) - 1, false, CAN_SLICE>(m, prow, pmask, dmask, lds, sc, true);
}

// An augmented triangle block.  There is no general path for eight tiles: plans with such blocks are
// used only where fast_path_ok holds (the host checks the same conditions before it chooses the plan).
template <typename T, class MatsT>
__device__ __forceinline__ void run_aug_block(const Item& it, const MatsT& m, T* lds)
{
    int prow[AugShape::NP];
#pragma unroll
    for (int p = 0; p < AugShape::NP; ++p) prow[p] = it.rows[p];
    const uint32_t pmask = 0x3Fu | (1u << it.aug1) | (1u << it.aug2);
    uint32_t dmask = 0;
    if (it.rows[4] == ((it.aug1 == 6) ? it.rows[0] : it.rows[1])) dmask |= 1u << it.aug1;
    if (it.aug2 == 8 && it.rows[5] == it.rows[2]) dmask |= 1u << 8;
    try_fast<T, AugShape, 0, false>(m, prow, pmask, dmask, lds, SliceCtx<T>{});
}

// ---- the kernels: workgroup -> block(s) -> code path ------------------------------------------
// Where the sliced blocks of a launch keep their parts and counters.
template <typename T>
struct SliceSpace {
    T* ws = nullptr;                // workspace: n_ws_blocks stretches of ws_slices * 6 * 16 * 256 elements
    unsigned int* ctr = nullptr;    // one counter per sliced block
    int* flag = nullptr;            // one int of LDS
};

// What a kernel's plans contain besides rectangular blocks: nothing (SYR2K), triangle blocks (Algorithm 4),
// or augmented triangle blocks.
constexpr int kBlocksRect = 0, kBlocksTri = 1, kBlocksAug = 2;

template <typename T, int KINDS, class MatsT>
__device__ __forceinline__ void run_item(const Plan& plan, int32_t id, const MatsT& m0, T* lds,
                                         const SliceSpace<T>& sp)
{
    Item it;
    tbs_decode(plan, id, it);
    MatsT m = m0;
    SliceCtx<T> sc;
    if (it.slices > 1 && it.kind != kEmpty) {
        // part `slice` of the columns of A, in whole chunks (the last part takes the ragged end)
        constexpr int KC = Cfg<T>::KC;
        const int64_t nch = (m0.M + KC - 1) / KC;
        const int64_t k0 = nch * it.slice / it.slices * KC;
        const int64_t k1 = (it.slice + 1 == it.slices) ? (int64_t)m0.M : nch * (it.slice + 1) / it.slices * KC;
#pragma unroll
        for (int pass = 0; pass < MatsT::NPASS; ++pass) {
            m.R[pass].p = m0.R[pass].p + k0 * m0.R[pass].ks;
            m.Q[pass].p = m0.Q[pass].p + k0 * m0.Q[pass].ks;
        }
        m.M = (int)(k1 > k0 ? k1 - k0 : 0);
        sc.part = sp.ws + (size_t)it.ws_block * ((size_t)plan.ws_slices * 6 * 16 * kThreads);
        sc.ctr = sp.ctr + it.ws_block;
        sc.flag = sp.flag;
        sc.slices = it.slices;
        sc.slice = it.slice;
    }
    // (one call site per shape: each is a copy of that shape's code)
    Item x = it;
    if (x.kind == kDiag) {                                  // a 1 x 1 rectangle on the diagonal
        x.rows[kRectCols] = x.rows[0];
        x.kind = kRectDiag;
    }
    if (x.kind == kTri) {
        if constexpr (KINDS == kBlocksTri) run_block<T, TriShape>(x, m, lds, sc);
    } else if (x.kind == kAug) {
        // (the host hands out augmented plans only for operands that suit the assembly loops)
        if constexpr (KINDS == kBlocksAug) run_aug_block<T>(x, m, lds);
    } else if (x.kind == kRect || x.kind == kRectDiag) {
        run_block<T, RectShape>(x, m, lds, sc, x.kind == kRectDiag);
    }
}

// The SYRK kernel.  NPASS: 1 for SYRK and the Gram form, 2 for SYR2K.  KINDS: which blocks besides
// rectangles its plans have (see kBlocksRect ..): there is one kernel per kind, because the code of all
// block shapes in one kernel leaves the compiler too few registers outside the assembly loops.
//
// ctr == nullptr: one workgroup per block of the plan (used when the plan has no more blocks than the
// launch may have workgroups): workgroup b runs item b.
//
// Persistent form (ctr != nullptr): a fixed number of workgroups (at most one per compute unit; fewer
// when the caller wants to keep units free for kernels of another stream) take blocks from the list in
// order through a counter in device memory, which is what the hardware dispatcher does with one
// workgroup per block, minus the cost of starting a workgroup for every block.  ctr[0] = next block,
// ctr[1] = workgroups that have finished; the last one to finish sets the counters back to zero for the
// next launch that uses the same set.
//
// The Triangle Block Scheme one level up (Section 5.1 with the L2 of a die as fast memory): the first
// plan.team_items items are groups of 32 triangle blocks on 28 tile rows (tbs_plan.h).  The workgroups
// of a die (they share its L2) take the blocks of one group together: die d owns the groups d, d + 8,
// ... and hands them out through its own counter ctr[kTeamCtr + d]; a workgroup whose die has none left
// helps the other dies in turn, so every block is taken exactly once whatever the placement of the
// workgroups, and then all continue with the rest of the list through ctr[0].  Blocks of equal length
// started together stay together, so a group's 28 panels are fetched into the L2 once for 32 blocks.
//
// (All three ways of choosing the next block feed one loop with one call of run_item: the block code is
// large, and every further call site would be another copy of it to compile.)
constexpr int kTeams = 8;                  // accelerator dies, each with its own L2
constexpr int kTeamCtr = 4;                // ctr[kTeamCtr + d]: blocks handed out of die d's groups
static_assert(kTeamCtr + kTeams <= kLaunchCounters, "the counters of a launch fit their set");

__device__ __forceinline__ int die_of_this_workgroup()
{
    uint32_t id;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID, 0, 4)" : "=s"(id));
    return (int)(id % kTeams);
}

template <typename T, int NPASS, int KINDS>
__global__ __launch_bounds__(kThreads) void tbs_syrk_kernel(Plan plan, Mats<T, NPASS> m, unsigned int* ctr, T* ws,
                                                            unsigned int* slice_ctr)
{
    __shared__ __attribute__((aligned(16))) unsigned char smem[kLdsBytes];
    __shared__ int32_t s_item;
    __shared__ int s_flag;
    const SliceSpace<T> sp = {ws, slice_ctr, &s_flag};
    const bool persistent = ctr != nullptr;
    const int32_t n_groups = persistent ? plan.team_items / kGroupItems : 0;
    const int home = die_of_this_workgroup();
    bool groups_left = n_groups > 0, first = true;
    for (;;) {
        int32_t id = -1;
        if (!persistent) {
            if (first) id = (int32_t)blockIdx.x;
            first = false;
        } else {
            __syncthreads();                    // the previous block's LDS reads and s_item are done with
            if (threadIdx.x == 0) {
                int32_t got = -1;
                if (groups_left) {
                    // the home die's next block; when it has none left, the next block of the first die
                    // (in turn) whose counter, read first, says that it has (the atomic's result decides)
                    unsigned int seen[kTeams];
#pragma unroll
                    for (int t = 0; t < kTeams; ++t) seen[t] = 0u;
                    for (int turn = 0; turn < kTeams && got < 0; ++turn) {
                        const int t = (home + turn) % kTeams;
                        const int32_t mine = ((n_groups - t + kTeams - 1) / kTeams) * kGroupItems;   // die t's blocks
                        if (turn == 1) {
#pragma unroll
                            for (int u = 0; u < kTeams; ++u)
                                seen[u] = __hip_atomic_load(&ctr[kTeamCtr + u], __ATOMIC_RELAXED,
                                                            __HIP_MEMORY_SCOPE_AGENT);
                        }
                        if (mine <= 0 || (int32_t)seen[t] >= mine) continue;
                        const int32_t n = (int32_t)atomicAdd(&ctr[kTeamCtr + t], 1u);
                        if (n < mine) got = ((n / kGroupItems) * kTeams + t) * kGroupItems + n % kGroupItems;
                    }
                }
                if (got < 0) {                  // the groups are done (or there are none): the list
                    const int32_t n = plan.team_items + (int32_t)atomicAdd(&ctr[0], 1u);
                    got = n < plan.n_items ? n : -1;
                    if (groups_left) got |= (int32_t)0x40000000;        // tells the others: no groups left
                }
                s_item = got;
            }
            __syncthreads();
            id = __builtin_amdgcn_readfirstlane(s_item);
            if (id >= 0 && (id & 0x40000000)) {
                groups_left = false;
                id &= 0x3FFFFFFF;
            } else if (id < 0) {
                groups_left = false;
            }
        }
        if (id < 0) break;
        run_item<T, KINDS>(plan, id, m, reinterpret_cast<T*>(smem), sp);
    }
    if (persistent && threadIdx.x == 0) {
        // (no fence: the counters are only ever touched by device-scope atomics; this one follows the
        // return of the workgroup's last fetch from the list, and the reset follows the return of this one)
        if (atomicAdd(&ctr[1], 1u) == gridDim.x - 1) {  // every workgroup has left its loop
#pragma unroll
            for (int c = 0; c < kLaunchCounters; ++c)
                __hip_atomic_store(&ctr[c], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// C (m x n) <- beta*C + alpha * R (m x K) * Q (n x K)^T, rectangular blocks of mr x nc tiles
// (mr <= 2, nc <= 3), one workgroup per block.
template <typename T>
__global__ __launch_bounds__(kThreads) void gemm_nt_kernel(int m_rows, int n_cols, int K, T alpha,
                                                           const T* R, int64_t ldr, const T* Q,
                                                           int64_t ldq, T beta, T* C, int64_t ldc, int nJ,
                                                           int mr, int nc)
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
        const int t = J * nc + q;
        it.rows[q] = (q < nc && t < Tn) ? t : -1;
    }
#pragma unroll
    for (int r = 0; r < kRectRows; ++r) {
        const int t = I * mr + r;
        it.rows[kRectCols + r] = (r < mr && t < Tm) ? t : -1;
    }
    const Mats<T> m = {{{R, ldr, 1}}, m_rows, {{Q, ldq, 1}}, n_cols, C, ldc, K, alpha, beta, false};
    run_block<T, RectShape, false>(it, m, lds, SliceCtx<T>{});
}

// `lease`: the counters of this launch (see acquire_counters); needed by the persistent form and by
// plans with cut blocks.  Its event, if any, is attached to the kernel: it completes with the launch.
// NPASS = 1: C <- beta C + alpha A A^T (b unused); NPASS = 2: C <- beta C + alpha (A B^T + B A^T), plan
// of rectangles only.
template <typename T, int NPASS, int KINDS>
hipError_t launch_syrk_t(const Plan& plan, int64_t N, int64_t M, double alpha, const OperandDesc& a,
                         const OperandDesc& b, double beta, void* C, int64_t ldc, int max_workgroups, void* ws,
                         const CounterLease& lease, hipStream_t stream)
{
    if (plan.n_items <= 0) return hipSuccess;
    if (plan.n_ws_blocks > kSliceCounters || (plan.n_ws_blocks > 0 && ws == nullptr)) return hipErrorInvalidValue;
    const bool persistent = max_workgroups > 0 && plan.n_items > max_workgroups;
    if ((persistent && lease.ctr == nullptr) || (plan.n_ws_blocks > 0 && lease.slice_ctr == nullptr))
        return hipErrorInvalidValue;
    Mats<T, NPASS> m;
    const Side<T> sa = {(const T*)a.p, a.rs, a.ks}, sb = {(const T*)b.p, b.rs, b.ks};
    m.R[0] = sa;
    m.Q[0] = NPASS == 1 ? sa : sb;
    if constexpr (NPASS == 2) {
        m.R[1] = sb;
        m.Q[1] = sa;
    }
    m.nr = m.nq = (int)N;
    m.C = (T*)C;
    m.ldc = ldc;
    m.M = (int)M;
    m.alpha = (T)alpha;
    m.beta = (T)beta;
    m.lower = true;
    // (one kernel for both forms: without counters, workgroup b runs item b)
    hipExtLaunchKernelGGL((tbs_syrk_kernel<T, NPASS, KINDS>), dim3((unsigned)(persistent ? max_workgroups : plan.n_items)),
                          dim3(kThreads), 0, stream, nullptr, lease.done, 0, plan, m,
                          persistent ? lease.ctr : (unsigned int*)nullptr, (T*)ws, lease.slice_ctr);
    return hipGetLastError();
}

// The block shape is the one with the shortest estimated time on `units` compute units: rounds of
// blocks, each costing its tiles (K columns at one unit's share of the MFMA peak) plus the fixed
// cost of a block.  A product with few blocks per unit is cut finer so that the last round is full.
template <typename T>
hipError_t launch_gemm_t(int64_t m, int64_t n, int64_t K, double alpha, const void* R, int64_t ldr,
                                const void* Q, int64_t ldq, double beta, void* C, int64_t ldc, int units,
                                hipStream_t stream)
{
    if (m <= 0 || n <= 0) return hipSuccess;
    const int Tm = (int)((m + kTile - 1) / kTile), Tn = (int)((n + kTile - 1) / kTile);
    const double tile_us = (double)K * (sizeof(T) == 4 ? 0.01334 : 0.02668), fixed_us = 15.0;
    const int shapes[5][2] = {{2, 3}, {2, 2}, {1, 3}, {1, 2}, {1, 1}};
    int mr = 2, nc = 3;
    double best = 0.0;
    if (units < 1) units = 1;
    for (const auto& sh : shapes) {
        const int64_t blocks = (int64_t)((Tm + sh[0] - 1) / sh[0]) * ((Tn + sh[1] - 1) / sh[1]);
        const int64_t rounds = (blocks + units - 1) / units;
        const double t = (double)rounds * (sh[0] * sh[1] * tile_us + fixed_us);
        if (best == 0.0 || t < best * 0.97) {               // prefer the larger block on near ties
            best = t;
            mr = sh[0];
            nc = sh[1];
        }
    }
    const int nI = (Tm + mr - 1) / mr, nJ = (Tn + nc - 1) / nc;
    hipLaunchKernelGGL(gemm_nt_kernel<T>, dim3((unsigned)(nI * nJ)), dim3(kThreads), 0, stream, (int)m,
                       (int)n, (int)K, (T)alpha, (const T*)R, ldr, (const T*)Q, ldq, (T)beta, (T*)C, ldc, nJ, mr,
                       nc);
    return hipGetLastError();
}

// ---- translation units ---------------------------------------------------------------------------
// The file is compiled several times in parallel (each kernel template with its many instances takes
// minutes): -DTBS_UNIT_SYRK, -DTBS_UNIT_SYRK_AUG, -DTBS_UNIT_SYR2K or -DTBS_UNIT_GEMM with -DTBS_UNIT_TYPE=double|float instantiates one
// launcher (and the kernels it launches), -DTBS_UNIT_DISPATCH defines the entry points that choose
// between them; without any of these macros one translation unit holds everything.
#define TBS_LAUNCH_SYRK_ARGS \
    const Plan&, int64_t, int64_t, double, const OperandDesc&, const OperandDesc&, double, void*, int64_t, int, \
        void*, const CounterLease&, hipStream_t
#define TBS_LAUNCH_GEMM_ARGS \
    int64_t, int64_t, int64_t, double, const void*, int64_t, const void*, int64_t, double, void*, int64_t, int, \
        hipStream_t
#if defined(TBS_UNIT_SYRK)
template hipError_t launch_syrk_t<TBS_UNIT_TYPE, 1, kBlocksTri>(TBS_LAUNCH_SYRK_ARGS);
#elif defined(TBS_UNIT_SYRK_AUG)
template hipError_t launch_syrk_t<TBS_UNIT_TYPE, 1, kBlocksAug>(TBS_LAUNCH_SYRK_ARGS);
#elif defined(TBS_UNIT_SYR2K)
template hipError_t launch_syrk_t<TBS_UNIT_TYPE, 2, kBlocksRect>(TBS_LAUNCH_SYRK_ARGS);
#elif defined(TBS_UNIT_GEMM)
template hipError_t launch_gemm_t<TBS_UNIT_TYPE>(TBS_LAUNCH_GEMM_ARGS);
#else
#if defined(TBS_UNIT_DISPATCH)
extern template hipError_t launch_syrk_t<double, 1, kBlocksTri>(TBS_LAUNCH_SYRK_ARGS);
extern template hipError_t launch_syrk_t<float, 1, kBlocksTri>(TBS_LAUNCH_SYRK_ARGS);
extern template hipError_t launch_syrk_t<double, 1, kBlocksAug>(TBS_LAUNCH_SYRK_ARGS);
extern template hipError_t launch_syrk_t<float, 1, kBlocksAug>(TBS_LAUNCH_SYRK_ARGS);
extern template hipError_t launch_syrk_t<double, 2, kBlocksRect>(TBS_LAUNCH_SYRK_ARGS);
extern template hipError_t launch_syrk_t<float, 2, kBlocksRect>(TBS_LAUNCH_SYRK_ARGS);
extern template hipError_t launch_gemm_t<double>(TBS_LAUNCH_GEMM_ARGS);
extern template hipError_t launch_gemm_t<float>(TBS_LAUNCH_GEMM_ARGS);
#endif
// ---- counters in device memory --------------------------------------------------------------------
// One set per slot: ctr[kLaunchCounters] of the persistent form (next block, workgroups done, next
// block of each die's groups) and one counter per cut block (parts finished).  All zero at load time; every launch leaves its set zero again (the last
// workgroup of a persistent launch resets the pair, the workgroup that sums a block resets its
// counter).  Which launch may use which slot is decided by SlotTable (counter_slots.h); the event of a
// slot completes with the last launch that used it.
static __device__ unsigned int g_syrk_counters[kCounterSlots][kLaunchCounters];
static __device__ unsigned int g_slice_counters[kCounterSlots][kSliceCounters];

namespace {
struct DeviceCounters {
    unsigned int* pairs = nullptr;      // device address of g_syrk_counters on this device
    unsigned int* slices = nullptr;     // ... of g_slice_counters
    hipEvent_t done[kCounterSlots] = {};
    SlotTable table;
};
constexpr int kMaxDevices = 64;
std::mutex g_counters_mu;
DeviceCounters g_counters[kMaxDevices];
}  // namespace

hipError_t acquire_counters(hipStream_t stream, CounterLease* out)
{
    *out = CounterLease{};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_counters_mu);
    DeviceCounters& dc = g_counters[dev];
    if (!dc.pairs) {                                        // once per device, with that device current
        void* ptr = nullptr;
        void* sptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_syrk_counters));
        if (e != hipSuccess) return e;
        e = hipGetSymbolAddress(&sptr, HIP_SYMBOL(g_slice_counters));
        if (e != hipSuccess) return e;
        dc.slices = static_cast<unsigned int*>(sptr);
        dc.pairs = static_cast<unsigned int*>(ptr);
    }
    SlotOwner who;
    who.stream = stream;
    if (stream == hipStreamPerThread) {                     // one handle, a different stream in every thread
        static thread_local char tag;
        who.thread = (uint64_t)reinterpret_cast<uintptr_t>(&tag);
    }
    const int s = dc.table.acquire(who, [&](int slot) {
        return dc.done[slot] == nullptr || hipEventQuery(dc.done[slot]) == hipSuccess;
    });
    if (s < 0) return hipSuccess;                           // none free: out stays empty
    if (!dc.done[s]) {
        e = hipEventCreateWithFlags(&dc.done[s], hipEventDisableTiming);
        if (e != hipSuccess) return e;
    }
    out->ctr = dc.pairs + (size_t)kLaunchCounters * s;
    out->slice_ctr = dc.slices + (size_t)kSliceCounters * s;
    out->done = dc.done[s];
    return hipSuccess;
}

// ---- scratch memory of the entry point that allocates nothing ---------------------------------------
// Held by every device the library runs on until the process ends.  In host code the name below is
// only a handle for hipGetSymbolAddress; kernels receive the looked-up address as an argument.
static_assert(kStaticCounterBytes >= (kLaunchCounters + kSliceCounters) * sizeof(unsigned int), "counters fit");
static __device__ __align__(256) unsigned char scratch[kStaticCounterBytes + kStaticWorkspaceBytes];

hipError_t static_scratch(unsigned char** out)
{
    static std::mutex mu;
    static unsigned char* per_device[kMaxDevices] = {};
    *out = nullptr;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!per_device[dev]) {                                 // each device has its own copy at its own address
        unsigned char* ptr = nullptr;
        e = hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        per_device[dev] = ptr;
    }
    *out = per_device[dev];
    return hipSuccess;
}

hipError_t launch_syrk(bool f32, const Plan& plan, int64_t N, int64_t M, double alpha, const OperandDesc& a,
                       double beta, void* C, int64_t ldc, int max_workgroups, void* workspace,
                       const CounterLease& lease, hipStream_t stream)
{
    bool aug = false;
    for (int32_t sg = 0; sg < plan.nseg; ++sg) aug = aug || (plan.seg[sg].kind == kSegTri && plan.seg[sg].aug);
    for (int32_t sg = 0; sg < plan.nseg && aug; ++sg)       // (such plans have no other triangle blocks)
        if ((plan.seg[sg].kind == kSegTri && !plan.seg[sg].aug) || plan.seg[sg].kind == kSegTriBase)
            return hipErrorInvalidValue;
    if (aug)
        return f32 ? launch_syrk_t<float, 1, kBlocksAug>(plan, N, M, alpha, a, a, beta, C, ldc, max_workgroups,
                                                         workspace, lease, stream)
                   : launch_syrk_t<double, 1, kBlocksAug>(plan, N, M, alpha, a, a, beta, C, ldc, max_workgroups,
                                                          workspace, lease, stream);
    return f32 ? launch_syrk_t<float, 1, kBlocksTri>(plan, N, M, alpha, a, a, beta, C, ldc, max_workgroups, workspace,
                                                     lease, stream)
               : launch_syrk_t<double, 1, kBlocksTri>(plan, N, M, alpha, a, a, beta, C, ldc, max_workgroups, workspace,
                                                      lease, stream);
}

hipError_t launch_syr2k(bool f32, const Plan& plan, int64_t N, int64_t M, double alpha, const OperandDesc& a,
                        const OperandDesc& b, double beta, void* C, int64_t ldc, int max_workgroups,
                        const CounterLease& lease, hipStream_t stream)
{
    if (plan.n_ws_blocks > 0) return hipErrorInvalidValue;
    for (int32_t sg = 0; sg < plan.nseg; ++sg)
        if (plan.seg[sg].kind == kSegTri || plan.seg[sg].kind == kSegTriBase) return hipErrorInvalidValue;
    return f32 ? launch_syrk_t<float, 2, kBlocksRect>(plan, N, M, alpha, a, b, beta, C, ldc, max_workgroups, nullptr,
                                                      lease, stream)
               : launch_syrk_t<double, 2, kBlocksRect>(plan, N, M, alpha, a, b, beta, C, ldc, max_workgroups, nullptr,
                                                       lease, stream);
}

size_t syrk_workspace_bytes(bool f32, const Plan& plan)
{
    return (size_t)plan.n_ws_blocks * (size_t)plan.ws_slices * 6 * 16 * kThreads * (f32 ? 4 : 8);
}

hipError_t launch_gemm_nt(bool f32, int64_t m, int64_t n, int64_t K, double alpha, const void* R,
                          int64_t ldr, const void* Q, int64_t ldq, double beta, void* C, int64_t ldc,
                          int units, hipStream_t stream)
{
    return f32 ? launch_gemm_t<float>(m, n, K, alpha, R, ldr, Q, ldq, beta, C, ldc, units, stream)
               : launch_gemm_t<double>(m, n, K, alpha, R, ldr, Q, ldq, beta, C, ldc, units, stream);
}

#endif

}  // namespace tbs
