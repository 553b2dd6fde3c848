/*
 * tbs_syrk.h -- C ABI of the Triangle Block SYRK / Large Block Cholesky library for MI355X.
 *
 * The operations are the two kernels of the paper "I/O-Optimal Algorithms for Symmetric Linear
 * Algebra Kernels" (Section 3, Algorithms 1 and 2), scheduled as its Section 5 prescribes:
 *   - tbs_syrk_lower       the symmetric rank-k update under the tiled Triangle Block Scheme
 *                          (Section 5.1, Algorithm 4, tiled form of Section 5.1.4);
 *   - tbs_syrk_lower_square the same update with square blocks only (the OOC_SYRK scheme the
 *                          paper compares with, Sections 5 and 5.1.3): the baseline;
 *   - tbs_potrf_lower      Large Block Cholesky (Section 5.2, Algorithm 5): panel factorisation,
 *                          triangular solve, Triangle Block trailing update.
 *
 * Conventions common to every call
 *   - All matrices are row-major with a leading dimension counted in elements; pointers need the
 *     alignment of an element, leading dimensions need none.
 *   - Matrix pointers are DEVICE pointers; the caller owns them (and the stream) before, during
 *     and after the call.  The library allocates and frees no device memory.
 *   - Only entries on or below the diagonal (column <= row) of a symmetric / triangular matrix
 *     are read or written; everything above the diagonal is left bit-for-bit untouched.
 *   - Calls are asynchronous on `hip_stream` (a hipStream_t passed as void*, NULL = the default
 *     stream) unless stated otherwise.
 *   - Arguments are validated on the host before anything is launched.  Errors are return codes;
 *     nothing is thrown or aborted.  On an error nothing has been launched.
 *   - Functions whose names end in _query, _workspace, _enumerate or _string touch no GPU.
 */
#ifndef TBS_SYRK_H
#define TBS_SYRK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { TBS_F64 = 0, TBS_F32 = 1 } tbs_dtype;

typedef enum {
    TBS_OK = 0,
    TBS_EINVAL = 1,      /* bad size, leading dimension, dtype or NULL pointer                  */
    TBS_EWORKSPACE = 2,  /* workspace smaller than the _workspace call asks for                 */
    TBS_ENOTSPD = 3,     /* potrf met a pivot that is not > 0 (see info_host)                    */
    TBS_EHIP = 4         /* a HIP runtime call failed (launch error, no device)                  */
} tbs_status;

/* Plain-text name of a status code; never NULL. */
const char* tbs_status_string(tbs_status s);

/* ------------------------------------------------------------------------------------------------
 * SYRK, lower triangle (Algorithm 1 with scaling factors):
 *     C[i][j] <- beta * C[i][j] + alpha * sum_{k<M} A[i][k] * A[j][k]      for 0 <= j <= i < N.
 * The paper's update is alpha = beta = 1; the trailing update of Algorithm 5 is alpha = -1.
 * beta == 0 means C is write-only (old contents, NaN included, are not read).
 *   A   device, N x M, lda >= max(M,1), never written
 *   C   device, N x N, ldc >= max(N,1)
 *   N, M >= 0; N == 0 is a no-op; M == 0 scales the lower triangle by beta.
 *   workspace / workspace_bytes: optional device scratch (contents arbitrary, aligned to the
 *   element size; owned by the caller, used only until the call's work on the stream has finished;
 *   calls that may run at the same time need different workspaces).  tbs_syrk_lower_workspace()
 *   reports what the library can use: 0 for most sizes.  For problems with few tiles per compute
 *   unit it is the room for blocks that are computed in parts along the contraction dimension (the
 *   parts are summed in a fixed order, results are reproducible).  With workspace == NULL the call
 *   uses its plan without such blocks (same results up to the order of the floating-point sums,
 *   lower throughput); a workspace that is not NULL must hold the reported number of bytes, else
 *   TBS_EWORKSPACE is returned and nothing is launched.  tbs_syrk_lower_square ignores it.
 *   The persistent form of the kernel and the blocks computed in parts count through small arrays
 *   of device memory inside the library (file scope, no allocation).  A set of counters serves the
 *   launches of one stream; if every set is held by launches of other streams that have not
 *   finished (more than 64 streams busy at once), the call runs one workgroup per block without
 *   blocks computed in parts instead: slower, same contract.
 * The schedule (Section 5.1.4): C is cut into b x b tiles (b = 64); the tile rows are grouped
 * into triangle blocks R^{i,j} = { u*c + f^{i,j}(u) } of k tile rows (an indexing family in the
 * sense of Section 5.1.1: the cyclic one of Section 5.1.2, or its XOR analogue for c = 2^m); one
 * workgroup holds the k(k-1)/2 tiles of TB(R) in registers, streams the k row panels of A through
 * LDS once and uses every staged panel as left and as right operand.  Diagonal zones recurse, the
 * last l tile rows and the recursion base use rectangular blocks, which carry the diagonal tiles
 * of their region (nothing above the diagonal is read or written).
 * ---------------------------------------------------------------------------------------------- */
tbs_status tbs_syrk_lower_workspace(tbs_dtype dtype, int64_t N, int64_t M, size_t* bytes);

tbs_status tbs_syrk_lower(tbs_dtype dtype, int64_t N, int64_t M, double alpha,
                          const void* A, int64_t lda, double beta, void* C, int64_t ldc,
                          void* workspace, size_t workspace_bytes, void* hip_stream);

/* Same contract and arguments; every block is a rectangle of tiles (no triangle blocks). */
tbs_status tbs_syrk_lower_square(tbs_dtype dtype, int64_t N, int64_t M, double alpha,
                                 const void* A, int64_t lda, double beta, void* C, int64_t ldc,
                                 void* workspace, size_t workspace_bytes, void* hip_stream);

/* ------------------------------------------------------------------------------------------------
 * Two more kernels that use an input twice (the extension the paper's conclusion points to), built
 * from the same blocks and main loops.
 *
 * SYR2K, lower triangle:
 *     C[i][j] <- beta * C[i][j] + alpha * sum_{k<M} (A[i][k] * B[j][k] + B[i][k] * A[j][k]),  j <= i.
 *   A, B  device, N x M, lda, ldb >= max(M,1), never written; C device, N x N, ldc >= max(N,1).
 *   Schedule: rectangular blocks of up to 2 x 3 tiles (the square-block scheme of Section 5); a
 *   block streams (rows of A, rows of B) and then (rows of B, rows of A) into one set of
 *   accumulators and touches its part of C once.  A triangle block would need the panels of both
 *   matrices for all of its k tile rows at once, twice what a compute unit's LDS and registers
 *   hold beside k(k-1)/2 tiles, so the triangle-block schedule is not used here.
 *
 * Gram matrix, lower triangle (SYRK of the transpose, A stored as it is):
 *     C[i][j] <- beta * C[i][j] + alpha * sum_{k<N} A[k][i] * A[k][j],  0 <= j <= i < M.
 *   A  device, N x M row-major, lda >= max(M,1), never written; C device, M x M, ldc >= max(M,1).
 *   Schedule: the Triangle Block Scheme of tbs_syrk_lower on the M/b column panels of A (a panel's
 *   "row" is a column of A; a staged chunk is 16 or 32 memory rows of 64 columns); workspace as for
 *   tbs_syrk_lower, sized by tbs_gram_lower_workspace().  When M is no multiple of 2 (fp64) or 4
 *   (fp32) every block takes the slower, fully checked loop.
 * Both: N, M >= 0; an empty contraction scales the lower triangle by beta; beta == 0 means C is
 * write-only; nothing above the diagonal is read or written; asynchronous on hip_stream.
 * ---------------------------------------------------------------------------------------------- */
tbs_status tbs_syr2k_lower(tbs_dtype dtype, int64_t N, int64_t M, double alpha,
                           const void* A, int64_t lda, const void* B, int64_t ldb,
                           double beta, void* C, int64_t ldc, void* hip_stream);

tbs_status tbs_gram_lower_workspace(tbs_dtype dtype, int64_t N, int64_t M, size_t* bytes);

tbs_status tbs_gram_lower(tbs_dtype dtype, int64_t N, int64_t M, double alpha,
                          const void* A, int64_t lda, double beta, void* C, int64_t ldc,
                          void* workspace, size_t workspace_bytes, void* hip_stream);

/* ------------------------------------------------------------------------------------------------
 * tbs_syrk_lower for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same operation and arguments as tbs_syrk_lower called
 * with the workspace that tbs_syrk_lower_workspace() asks for, and the same plan and results bit for bit
 * wherever that plan has no eight-tile blocks (TBS_SYRK_AUGMENT=0 in the environment makes that so at
 * every size; this entry point never uses them, the results then agree within rounding), but
 * the scratch memory (the parts of blocks computed in parts, and the counters of the launch) is an
 * array at file scope in the library's device code: TBS_NOALLOC_SCRATCH_BYTES of device memory that
 * every GPU the library runs on holds from the moment the library is loaded until the process ends.
 * The call allocates and frees nothing on the device, creates no stream or event, and clears the
 * counters it needs with a small kernel on `hip_stream` (not with a memset).
 *   Limit: a plan that needs more than TBS_NOALLOC_WORKSPACE_BYTES for its parts (what
 *   tbs_syrk_lower_workspace() reports: 0 for most sizes, up to 128 MiB for some small N with a long
 *   contraction; more only for plans pinned through TBS_PLAN_TUNING) is rejected with
 *   TBS_EWORKSPACE before anything is launched: use tbs_syrk_lower with a workspace of the
 *   caller's for those.
 *   All calls on one GPU share the one array, which keeps the last call's contents: calls that may
 *   run at the same time on one GPU (different streams, no ordering between them) race and give
 *   wrong results; calls ordered by a stream or by events are fine.
 * ---------------------------------------------------------------------------------------------- */
#define TBS_NOALLOC_WORKSPACE_BYTES ((size_t)128 << 20)
#define TBS_NOALLOC_SCRATCH_BYTES (TBS_NOALLOC_WORKSPACE_BYTES + 4096)

tbs_status tbs_syrk_lower_noalloc(tbs_dtype dtype, int64_t N, int64_t M, double alpha,
                                  const void* A, int64_t lda, double beta, void* C, int64_t ldc,
                                  void* hip_stream);

/* ------------------------------------------------------------------------------------------------
 * The plan the library uses for a given size, for tests and benchmarks (host only).
 * Element counts follow the paper's accounting (Sections 5.1.3, 5.1.4): A elements loaded by
 * every block (k*b*M per triangle block), C elements loaded once.
 * ---------------------------------------------------------------------------------------------- */
typedef struct {
    int32_t k;                 /* side of a triangle block, in tile rows                         */
    int32_t b;                 /* tile side, in elements                                         */
    int32_t c;                 /* top-level modulus of the indexing family (0: no triangle blocks) */
    int32_t l;                 /* top-level leftover tile rows, T - k*c                          */
    int32_t levels;            /* recursion levels that use triangle blocks                      */
    int32_t tile_rows;         /* T = ceil(N / b)                                                */
    int32_t family;            /* top level: 0 = the cyclic family of Section 5.1.2; m > 0 = c is 2^m  */
                               /* and f(0)=j, f(1)=i, f(2)=i^j, f(3)=i^(x j mod x^m+x+1)            */
    int32_t max_slices;        /* blocks are cut along the contraction dimension into at most this many parts */
    int64_t n_items;           /* workgroups launched                                            */
    int64_t n_tri_blocks;      /* triangle blocks, all levels (six tiles, or eight: see _enumerate) */
    int64_t n_rect_blocks;     /* rectangular blocks (leftover rows, recursion base)             */
    int64_t n_diag_tiles;      /* diagonal tiles                                                 */
    int64_t S_C_elems;         /* C elements resident per block: b^2 k(k-1)/2, 8 b^2 for eight-tile blocks */
    int64_t S_res_elems;       /* S_C plus the LDS staging buffers of A                          */
    double  A_elems;           /* A elements this plan loads (all blocks, all levels)            */
    double  A_elems_top;       /* of which top-level triangle blocks: Q1 = c^2 k b M             */
    double  C_elems;           /* N(N+1)/2                                                       */
    double  tbs_bound_elems;   /* N^2 M / (sqrt(2) sqrt(S_C))  (corollary of Section 4.1)        */
    double  tiled_lead_elems;  /* N^2 M / ((k-1) b)            (Section 5.1.4)                   */
    double  square_elems;      /* N^2 M / sqrt(S_C)            (square blocks of equal area)     */
    int64_t n_sliced_blocks;   /* blocks computed in parts (0: none, no workspace needed)        */
    int64_t workspace_bytes;   /* what tbs_syrk_lower_workspace reports for this plan            */
} tbs_plan_info;

/* square = 0: the plan of tbs_syrk_lower when it is given its workspace; 1: the plan of
 * tbs_syrk_lower_square; 2: the plan of tbs_syrk_lower without a workspace. */
tbs_status tbs_syrk_lower_query(tbs_dtype dtype, int64_t N, int64_t M, int32_t square,
                                tbs_plan_info* out);

/* Expands the plan into its work list, with the very index arithmetic the kernels use.
 * Item t occupies items[t*13 .. t*13+12] (TBS_ENUMERATE_COLUMNS values):  [0] kind (0 triangle block,
 * 1 rectangle, 2 diagonal tile, 3 empty, 4 rectangle with diagonal tiles, 5 augmented triangle block:
 * see below), [1] number of row-side tile rows, [2] number of
 * column-side tile rows, [3..7] tile-row ids, -1 = unused (triangle block: the members of R in zone
 * order in [3..6]; rectangle: column side in [3..5], row side in [6..7]; diagonal tile: [3]).  A
 * rectangle updates the tiles (r, q) of its row x column product with q < r only; kind 4 also
 * updates the tiles with q = r (the part on and below the diagonal).  The plan depends on N and, for
 * small N, on M (which sets how finely the tail of the list is cut so that all compute units finish
 * together).  [8], [9]: the item is part [8] of the [9] parts its block is cut into along the
 * contraction dimension (0 of 1: a whole block); the parts of a block are consecutive items.
 * Kind 5: the triangle block on the four tile rows [3..6] plus two tiles of the diagonal zones, each
 * between one of those rows and one further row of the same zone ([7] for the first, [10] for the
 * second; -1 for other kinds): [11] = 6: tile ([7], [3]), 7: tile ([7], [4]); [12] = 8: tile ([10], [5]),
 * 9: tile ([5], [10]), 10: tile ([10], [6]), 11: tile ([6], [10]) (row, column); where the two rows of a
 * tile are equal it is a diagonal tile, updated on and below the diagonal.
 * `square` as for the query.  `capacity` counts items; *n_items receives the number the plan has
 * (call with items == NULL to size the buffer).  HOST pointers. */
#define TBS_ENUMERATE_COLUMNS 13
tbs_status tbs_syrk_lower_enumerate(tbs_dtype dtype, int64_t N, int64_t M, int32_t square,
                                    int32_t* items, int64_t capacity, int64_t* n_items);

/* ------------------------------------------------------------------------------------------------
 * Cholesky, lower triangle, in place (Algorithm 2; schedule: Algorithm 5, Large Block Cholesky):
 * the lower triangle of the symmetric positive definite matrix A (device, N x N, lda >=
 * max(N,1)) is replaced by L with L * L^T = A.
 *   workspace: device scratch of at least tbs_potrf_lower_workspace() bytes.
 *   info_host: HOST pointer or NULL.  If not NULL the call synchronises the stream before it
 *   returns and stores 0, or the 1-based index of the first pivot that is not > 0 (the return
 *   value is then TBS_ENOTSPD and the contents of A are unspecified).  With NULL the call is
 *   asynchronous and a failed pivot goes unreported.
 *   Large matrices are factored with look-ahead on two more streams that the library creates per
 *   device on first use (default priority) and keeps; their work is ordered before and after the
 *   caller's stream by events, so the caller sees an ordinary stream-ordered call.  Calls from
 *   several host threads on one device are enqueued one after the other.
 *   Inside a panel the block columns are processed right-looking (Algorithm 5 again, with a smaller
 *   block); the environment variable TBS_POTRF_PANEL=left, read at every call, selects the
 *   left-looking order (a block column first receives all updates of the panel's earlier block
 *   columns, then is factored and solved: every entry of the panel is written once, as Section 5.2.2
 *   accounts the panel steps).  Same results up to the order of the floating-point sums.
 * ---------------------------------------------------------------------------------------------- */
tbs_status tbs_potrf_lower_workspace(tbs_dtype dtype, int64_t N, size_t* bytes);

tbs_status tbs_potrf_lower(tbs_dtype dtype, int64_t N, void* A, int64_t lda,
                           void* workspace, size_t workspace_bytes,
                           int32_t* info_host, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* TBS_SYRK_H */
