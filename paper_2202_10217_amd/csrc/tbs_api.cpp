// tbs_api.cpp -- the C ABI declared in include/tbs_syrk.h: argument checks, plan cache, launches,
// and the Large Block Cholesky driver (Algorithm 5 of the paper) built from the kernels.
#include "tbs_syrk.h"

#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <map>
#include <mutex>
#include <string>
#include <tuple>
#include <utility>

#include "potrf_kernels.h"
#include "syrk_kernels.h"
#include "tbs_planner.h"

namespace {

using tbs::kK;
using tbs::kTile;

constexpr int64_t kMaxN = (int64_t)kTile << 15;       // descriptor limit: 2^15 tile rows
constexpr int64_t kMaxM = (int64_t)1 << 30;

bool dtype_ok(tbs_dtype d) { return d == TBS_F64 || d == TBS_F32; }
size_t elem_size(tbs_dtype d) { return d == TBS_F32 ? 4 : 8; }

int32_t compute_units()
{
    static int32_t ncu = [] {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            n = 256;                                   // no device (host-only use): MI355X's count
        return (int32_t)n;
    }();
    return ncu;
}

// The environment variables that change what the planner builds (all optional, for measurements).
// They are read at every call and are part of the cache key, so a plan built under one setting is
// never handed out under another.
constexpr bool kAugmentByDefault = true;

struct PlanEnv {
    std::string costs, family, slices, tuning, groups, augment;
    static PlanEnv read()
    {
        auto get = [](const char* name) {
            const char* v = std::getenv(name);
            return std::string(v ? v : "");
        };
        return PlanEnv{get("TBS_PLAN_COSTS"), get("TBS_PLAN_FAMILY"), get("TBS_SYRK_SLICES"), get("TBS_PLAN_TUNING"),
                       get("TBS_SYRK_DIE_GROUPS"), get("TBS_SYRK_AUGMENT")};
    }
};

// A plan depends on the number of tile rows and, for small matrices, on how long a tile takes
// compared with the fixed cost of a block (prologue, epilogue, dispatch: about 20 us against
// M * 2 * 64 * 64 flops at one compute unit's share of the MFMA peak), which decides how finely the
// tail of the work list is cut.  M enters through its power-of-two bucket.  Built once, kept.
// allow_aug = false: no augmented blocks (they have no general path: the caller passes false for operands
// that do not suit the assembly loops, see operands_suit_fast_path).
const tbs::Plan* cached_plan(int32_t T, bool square, tbs_dtype dtype, int64_t M, bool sliced, bool allow_aug = true)
{
    static std::mutex mu;
    static std::map<std::tuple<int32_t, bool, int32_t, int32_t, bool, bool, std::string, std::string, std::string,
                               std::string, std::string, std::string>,
                    tbs::Plan>
        cache;
    int32_t bucket = 0;
    while (bucket < 30 && ((int64_t)3 << bucket) / 2 <= M) ++bucket;     // M ~ 2^bucket
    const PlanEnv env = PlanEnv::read();
    std::lock_guard<std::mutex> lock(mu);
    auto key = std::make_tuple(T, square, (int32_t)dtype, bucket, sliced, allow_aug, env.costs, env.family, env.slices,
                               square ? std::string() : env.tuning, env.groups, env.augment);
    auto it = cache.find(key);
    if (it == cache.end()) {
        const double tile_us = (double)((int64_t)1 << bucket) * (dtype == TBS_F32 ? 0.01334 : 0.02668);
        // fixed costs: a block (prologue, epilogue, taking it from the list), a part of a cut block, and
        // per part of the block again for summing them (TBS_PLAN_COSTS="block_us,part_us,per_part_us"
        // overrides them)
        double block_us = 20.0, slice_us = 0.03 * tile_us, per_part_us = 0.0;
        if (!env.costs.empty()) {
            double b = 0.0, sl = 0.0, pp = 0.0;
            if (std::sscanf(env.costs.c_str(), "%lf,%lf,%lf", &b, &sl, &pp) >= 2 && b >= 0.0 && sl >= 0.0 && pp >= 0.0) {
                block_us = b;
                slice_us = sl;
                per_part_us = pp;
            }
        }
        const double overhead_tiles = block_us / tile_us;
        tbs::Plan p;
        // TBS_PLAN_FAMILY=cyclic: the paper's cyclic family only (no power-of-two moduli)
        const bool xor_family = !(!env.family.empty() && env.family[0] == 'c');
        // Top-level triangle blocks in groups of 32 that one die takes together (they share 28 panels in
        // its L2): less than half the bytes come in from the fabric, and the workgroups of a die run in
        // step, epilogues included.  It pays when A is too large for the last-level cache, so that the
        // fetches would go to HBM (N = 32768, M = 8192 fp32: 136 -> 62 GB fetched, 3 % faster); with a
        // smaller A they are served by that cache anyway and the synchronised epilogues cost 1-2 %.
        // TBS_SYRK_DIE_GROUPS=1 / 0 forces the groups on / off.
        const double a_bytes = (double)T * kTile * (double)((int64_t)1 << bucket) * (dtype == TBS_F32 ? 4.0 : 8.0);
        bool die_groups = a_bytes > 192.0 * 1048576.0;
        if (!env.groups.empty()) die_groups = env.groups[0] != '0';
        // Top-level triangle blocks that take two tiles of the diagonal zones with them (eight tiles per
        // block instead of six: the fixed cost of a block is spread over a third more work, and the zones
        // need no blocks of their own).  TBS_SYRK_AUGMENT=1 / 0 lets the planner consider them or not.
        // By default in fp64, and there only where a compute unit gets at most two top-level blocks (the
        // planner's rule): measured +0.5 to +4.9 % for N = 4096 .. 5632, M = 1024 .. 16384; in fp32 the larger
        // epilogue eats the gain (-1.4 to +5.5 %, most sizes slightly negative).
        bool augment = kAugmentByDefault && dtype == TBS_F64;
        if (!env.augment.empty()) augment = env.augment[0] != '0';
        // (the smallest M of the bucket must give the assembly loops a whole chunk)
        if (!allow_aug || ((int64_t)3 << bucket) / 4 < (dtype == TBS_F32 ? 32 : 16)) augment = false;
        // blocks may be cut along the contraction dimension while a part keeps at least 8 chunks of
        // the smallest M of the bucket; TBS_SYRK_SLICES=0 turns that off, "levels,rows,...,tri,rect,
        // tail_blocks,tail" in TBS_PLAN_TUNING pins it
        const int64_t kc = dtype == TBS_F32 ? 32 : 16;
        const int64_t m_low = ((int64_t)3 << bucket) / 4;
        int32_t max_slices = (int32_t)std::min<int64_t>(tbs::kMaxSlices, m_low / (8 * kc));
        if (!sliced || square || (!env.slices.empty() && env.slices[0] == '0')) max_slices = 1;
        // TBS_PLAN_TUNING="levels,rows,cols,base,zone_rows,zone_cols[,tri,rect,tail_blocks,tail[,augment]]" pins
        // the tuning the planner would otherwise choose (every tuning covers each tile exactly once)
        const char* pin = (square || env.tuning.empty()) ? nullptr : env.tuning.c_str();
        int lv = 0, mr = 0, nc = 0, base = 0, mrd = 0, ncd = 0, st = 1, sr = 1, tb = 0, ts = 1, ag = 0;
        if (pin && std::sscanf(pin, "%d,%d,%d,%d,%d,%d,%d,%d,%d,%d,%d", &lv, &mr, &nc, &base, &mrd, &ncd, &st, &sr, &tb,
                               &ts, &ag) >= 4 &&
            lv >= 0 && lv <= tbs::kMaxLevels && mr >= 1 && mr <= tbs::kRectRows && nc >= 1 && nc <= tbs::kRectCols) {
            tbs::PlanTuning tune{lv, mr, nc, base != 0, mrd, ncd};
            tune.xor_family = xor_family;
            tune.die_groups = die_groups;
            tune.augment = ag != 0 && allow_aug;
            if (!tbs::build_plan(T, tune, &p)) return nullptr;
            if (max_slices > 1 && (st > 1 || sr > 1 || (tb > 0 && ts > 1))) {
                tbs::Plan q;
                if (tbs::apply_slicing(p, tbs::Slicing{st, sr, tb, ts}, &q)) p = q;
            }
        } else if (!tbs::choose_plan(T, square, compute_units(), overhead_tiles, &p, xor_family, max_slices,
                                     slice_us / tile_us, per_part_us / tile_us, die_groups, augment)) {
            return nullptr;
        }
        it = cache.emplace(key, p).first;
    }
    return &it->second;
}

tbs_status check_syrk(tbs_dtype dtype, int64_t N, int64_t M, const void* A, int64_t lda, const void* C,
                      int64_t ldc)
{
    if (!dtype_ok(dtype)) return TBS_EINVAL;
    if (N < 0 || M < 0 || N > kMaxN || M > kMaxM) return TBS_EINVAL;
    if (lda < (M > 1 ? M : 1) || ldc < (N > 1 ? N : 1)) return TBS_EINVAL;
    if (N > 0 && M > 0 && A == nullptr) return TBS_EINVAL;
    if (N > 0 && C == nullptr) return TBS_EINVAL;
    return TBS_OK;
}

// Workgroups of a persistent launch that leaves `reserve_units` compute units free (0: launches are
// not persistent, TBS_SYRK_PERSISTENT=0).
int persistent_workgroups(int reserve_units)
{
    static const bool persistent = [] {
        const char* v = std::getenv("TBS_SYRK_PERSISTENT");
        return !(v && v[0] == '0');
    }();
    // TBS_SYRK_RESERVE=n keeps n compute units out of every persistent launch (for measurements)
    static const int env_reserve = [] {
        const char* v = std::getenv("TBS_SYRK_RESERVE");
        const long n = v ? std::atol(v) : 0;
        return (n > 0 && n < 4096) ? (int)n : 0;
    }();
    return persistent ? std::max(1, compute_units() - std::max(reserve_units, env_reserve)) : 0;
}

// The conditions under which the kernels take the assembly loops (fast_path_ok in syrk_kernels.hip), on
// the host: at least one whole chunk of columns; 64 panel rows (row panels) or one chunk of memory rows
// (column panels) within 4 GiB; column panels: whole 16-byte pieces inside the matrix.
bool operands_suit_fast_path(tbs_dtype dtype, int64_t n_rows, int64_t M, int64_t row_stride, int64_t k_stride)
{
    const int64_t es = dtype == TBS_F32 ? 4 : 8, kc = dtype == TBS_F32 ? 32 : 16, vec = 16 / es;
    const int64_t lim = (int64_t)1 << 32;
    if (M < kc) return false;
    if (k_stride == 1) return kTile * row_stride * es < lim;
    return row_stride == 1 && (kc * k_stride + kTile) * es < lim && n_rows % vec == 0;
}

// The plan a call uses: the one with cut blocks if the caller gave a workspace (which must then hold
// its parts), else the one without.
tbs_status plan_for_call(int32_t T, bool square, tbs_dtype dtype, int64_t M, const void* workspace,
                         size_t workspace_bytes, const tbs::Plan** out, bool allow_aug)
{
    const size_t es = dtype == TBS_F32 ? 4 : 8;
    *out = nullptr;
    if (workspace == nullptr || square) {
        *out = cached_plan(T, square, dtype, M, false, allow_aug);
        return *out ? TBS_OK : TBS_EINVAL;
    }
    const tbs::Plan* sliced = cached_plan(T, square, dtype, M, true, allow_aug);
    if (!sliced) return TBS_EINVAL;
    if (sliced->n_ws_blocks > 0) {
        if (workspace_bytes < tbs::syrk_workspace_bytes(dtype == TBS_F32, *sliced)) return TBS_EWORKSPACE;
        if ((reinterpret_cast<uintptr_t>(workspace) % es) != 0) return TBS_EINVAL;
    }
    *out = sliced;
    return TBS_OK;
}

tbs_status syrk_impl(bool square, tbs_dtype dtype, int64_t N, int64_t M, double alpha, const void* A,
                     int64_t lda, double beta, void* C, int64_t ldc, hipStream_t stream, int reserve_units = 0,
                     void* workspace = nullptr, size_t workspace_bytes = 0)
{
    if (N == 0) return TBS_OK;
    const int32_t T = (int32_t)((N + kTile - 1) / kTile);
    const tbs::Plan* plan = nullptr;
    const bool aug_ok = operands_suit_fast_path(dtype, N, M, lda, 1);
    const tbs_status ps = plan_for_call(T, square, dtype, M, workspace, workspace_bytes, &plan, aug_ok);
    if (ps != TBS_OK) return ps;
    int wgs = persistent_workgroups(reserve_units);
    tbs::CounterLease lease;
    if ((wgs > 0 && plan->n_items > wgs) || plan->n_ws_blocks > 0) {
        if (tbs::acquire_counters(stream, &lease) != hipSuccess) return TBS_EHIP;
        if (!lease.ctr) {
            // every set of counters belongs to a launch on another stream that may still be running:
            // the form that needs none (one workgroup per block, no cut blocks)
            plan = cached_plan(T, square, dtype, M, false, aug_ok);
            if (!plan) return TBS_EINVAL;
            wgs = 0;
        }
    }
    const hipError_t e = tbs::launch_syrk(dtype == TBS_F32, *plan, N, M, alpha, tbs::OperandDesc{A, lda, 1}, beta, C,
                                          ldc, wgs, workspace, lease, stream);
    return e == hipSuccess ? TBS_OK : TBS_EHIP;
}

// ---- Large Block Cholesky ------------------------------------------------------------------------
constexpr size_t kInfoBytes = 256;                     // the workspace holds the info word only

// Two more streams and a few events per device for the look-ahead of Large Block Cholesky (created on
// first use, default priority, kept until the process ends).
constexpr int kSolvePieces = 8;
struct LookAhead {
    hipStream_t panel = nullptr, solve = nullptr;
    hipEvent_t column_ready = nullptr, panel_done = nullptr, rest_done = nullptr;
    hipEvent_t block_done[kSolvePieces] = {};
    bool ok = false;
    std::mutex enqueue;     // held while a call records into the stream and the events: calls from
};                          // several host threads then simply follow each other on the panel stream

LookAhead* look_ahead_for_device()
{
    static std::mutex mu;
    static std::map<int, LookAhead> per_device;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return nullptr;
    std::lock_guard<std::mutex> lock(mu);
    LookAhead& la = per_device[dev];
    if (!la.ok) {
        if (hipStreamCreateWithFlags(&la.panel, hipStreamNonBlocking) != hipSuccess) return nullptr;
        if (hipStreamCreateWithFlags(&la.solve, hipStreamNonBlocking) != hipSuccess) return nullptr;
        for (auto& e : la.block_done)
            if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) return nullptr;
        if (hipEventCreateWithFlags(&la.column_ready, hipEventDisableTiming) != hipSuccess) return nullptr;
        if (hipEventCreateWithFlags(&la.panel_done, hipEventDisableTiming) != hipSuccess) return nullptr;
        if (hipEventCreateWithFlags(&la.rest_done, hipEventDisableTiming) != hipSuccess) return nullptr;
        la.ok = true;
    }
    return &la;
}

struct Lbc {
    tbs_dtype dtype;
    size_t es;
    char* A;
    int64_t lda;
    int32_t* info;
    hipStream_t stream;  // the caller's stream
    int64_t big_block;   // panel width at the top level
    int reserve_units;   // compute units the trailing update leaves to the panel stream
    // A block of up to 512 columns and at most this many rows is solved by one launch (32 rows per
    // workgroup, no kernel boundaries between its tile columns: the short chain that the last panels
    // need); a taller one by the recursion below, whose products run as full-size blocks and make
    // better use of the few compute units the panel stream has next to a long trailing update.
    int64_t fused_trsm_rows = 6144;
    int64_t wide_rows = 8192;   // trailing matrices at least this tall get double-width panels
    // Inside a panel: right-looking (a block column is factored and solved, then the rest of the panel is
    // updated with it: Algorithm 5 again) or left-looking (a block column first receives the updates of
    // all earlier block columns of the panel in one product, then is factored and solved: every entry of
    // the panel is written once, the rule by which Section 5.2.2 accounts the panel steps).  Same
    // operations on the same values either way; TBS_POTRF_PANEL=left selects the second.
    bool left_panel = false;
    bool piecewise_solve = true;   // solve of the rows below block by block on a third stream
    int64_t piecewise_width = 1024; // ... for panels up to this width (at most kSolvePieces diagonal blocks)
    hipError_t err = hipSuccess;

    char* at(int64_t i, int64_t j) const { return A + ((size_t)i * (size_t)lda + (size_t)j) * es; }
    void note(hipError_t e) { if (err == hipSuccess && e != hipSuccess) err = e; }
    void note(tbs_status st) { if (st != TBS_OK) note(hipErrorUnknown); }

    int64_t block_for(int64_t n) const
    {
        if (n >= 4 * big_block) return big_block;
        if (n > 1024) return 256;
        return 128;                                                     // two tiles are one kernel
    }

    // X = A[row0 : row0+m, col0 : col0+nb]  <-  X * L^{-T},  L = A[col0 : col0+nb, col0 : col0+nb]
    // (the solve of Algorithm 5, "TRSM"): a block of up to 64 columns is solved by forward substitution
    // against its diagonal tile, one of up to 512 columns and not too many rows by the kernel that
    // takes 32 rows through all tile columns; other blocks are split in two with a product in between.
    void trsm(int64_t row0, int64_t m, int64_t col0, int64_t nb, hipStream_t st)
    {
        if (m <= 0 || nb <= 0) return;
        const bool f32 = dtype == TBS_F32;
        if (nb <= kTile) {
            note(tbs::launch_trsm_tile(f32, m, (int)nb, at(col0, col0), lda, at(row0, col0), lda, st));
            return;
        }
        if (nb <= 512 && m <= fused_trsm_rows) {
            note(tbs::launch_trsm_panel(f32, m, (int)nb, at(col0, col0), lda, at(row0, col0), lda, st));
            return;
        }
        const int64_t nb1 = ((nb / kTile + 1) / 2) * kTile;
        trsm(row0, m, col0, nb1, st);
        note(tbs::launch_gemm_nt(f32, m, nb - nb1, nb1, -1.0, at(row0, col0), lda, at(col0 + nb1, col0), lda,
                                 1.0, at(row0, col0 + nb1), lda, compute_units(), st));
        trsm(row0, m, col0 + nb1, nb - nb1, st);
    }

    // Algorithm 5 on A[off : off+n, off : off+n], everything on one stream; the one-tile Cholesky of
    // the panel is the same routine with a smaller block (the recursive variant the paper mentions in
    // Section 5.2.1).
    void potrf(int64_t off, int64_t n, hipStream_t st)
    {
        if (n <= 0) return;
        if (n <= 2 * kTile) {                                           // one or two tiles: one workgroup
            note(tbs::launch_potrf_block(dtype == TBS_F32, (int)n, at(off, off), lda, info, (int32_t)off, st));
            return;
        }
        const int64_t B = block_for(n);
        for (int64_t p0 = 0; p0 < n; p0 += B) {
            const int64_t nb = (B < n - p0) ? B : n - p0;
            const int64_t rest = n - p0 - nb, row0 = off + p0 + nb;
            if (left_panel && p0 > 0) update_block_column(off, p0, nb, rest, st);
            potrf(off + p0, nb, st);                                    // A[I0,I0] <- CHOL
            if (rest <= 0) continue;
            trsm(row0, rest, off + p0, nb, st);                         // A[I1,I0] <- TRSM
            if (!left_panel)
                note(syrk_impl(false, dtype, rest, nb, -1.0, at(row0, off + p0), lda, 1.0, at(row0, row0), lda,
                               st));                                    // A[I1,I1] <- TBS
        }
    }

    // Left-looking step inside the panel that starts at `off`: block column [p0, p0 + nb) of the panel
    // (its diagonal block and the `rest` panel rows below it) minus the products with the p0 columns
    // left of it.
    void update_block_column(int64_t off, int64_t p0, int64_t nb, int64_t rest, hipStream_t st)
    {
        note(syrk_impl(false, dtype, nb, p0, -1.0, at(off + p0, off), lda, 1.0, at(off + p0, off + p0), lda, st));
        if (rest > 0)
            note(tbs::launch_gemm_nt(dtype == TBS_F32, rest, nb, p0, -1.0, at(off + p0 + nb, off), lda,
                                     at(off + p0, off), lda, 1.0, at(off + p0 + nb, off + p0), lda, compute_units(),
                                     st));
    }

    // The panel A[off : off+n, off : off+n] factored on the panel stream as in potrf(), and, one
    // diagonal block behind it on the solve stream, the rows below the panel solved block column by
    // block column (right-looking: the product with the block columns already solved, then the
    // substitution against the diagonal block just factored).  When the panel's last diagonal block
    // is done only one block column of the solve is left, instead of the whole solve.  The rows below
    // must be up to date when `rows_ready` has happened.
    void potrf_and_solve_below(int64_t off, int64_t n, int64_t below, LookAhead* la, hipEvent_t rows_ready,
                               hipStream_t solve)
    {
        const bool f32 = dtype == TBS_F32;
        const int64_t B = block_for(n), row0 = off + n;
        note(hipStreamWaitEvent(solve, rows_ready, 0));
        int piece = 0;
        for (int64_t p0 = 0; p0 < n; p0 += B, ++piece) {
            const int64_t nb = (B < n - p0) ? B : n - p0;
            const bool last = p0 + nb >= n;
            // the last block column of the solve stays on the panel stream (it is what the next step
            // waits for, and a hand-over between streams costs about 12 us)
            hipStream_t st = solve;
            if (left_panel && p0 > 0) update_block_column(off, p0, nb, n - p0 - nb, la->panel);
            if (!last) {
                if (nb <= 2 * kTile) {                                  // the kernel's completion is the event
                    note(tbs::launch_potrf_block(f32, (int)nb, at(off + p0, off + p0), lda, info,
                                                 (int32_t)(off + p0), la->panel, la->block_done[piece]));
                } else {
                    potrf(off + p0, nb, la->panel);
                    note(hipEventRecord(la->block_done[piece], la->panel));
                }
                note(hipStreamWaitEvent(solve, la->block_done[piece], 0));
            } else {
                potrf(off + p0, nb, la->panel);
                note(hipEventRecord(la->block_done[piece], solve));
                note(hipStreamWaitEvent(la->panel, la->block_done[piece], 0));
                st = la->panel;
            }
            if (p0 > 0)
                note(tbs::launch_gemm_nt(f32, below, nb, p0, -1.0, at(row0, off), lda, at(off + p0, off), lda, 1.0,
                                         at(row0, off + p0), lda, compute_units(), st));
            trsm(row0, below, off + p0, nb, st);
            const int64_t rest = n - p0 - nb, r1 = off + p0 + nb;
            if (rest <= 0) continue;
            trsm(r1, rest, off + p0, nb, la->panel);
            if (!left_panel)
                note(syrk_impl(false, dtype, rest, nb, -1.0, at(r1, off + p0), lda, 1.0, at(r1, r1), lda, la->panel));
        }
    }

    // Algorithm 5 at the top level with look-ahead.  The trailing update of panel p is split in three:
    // the diagonal block of the next panel (SYRK), the rows below it (a product), the rest.  The next
    // panel's factorisation (a long chain of small kernels) runs on the panel stream: the diagonal
    // block is updated there and factored while the caller's stream computes the product and then the
    // rest of the update (which leaves a few compute units free); the solve of the rows below follows
    // the factorisation block by block on the solve stream (potrf_and_solve_below), or as a whole on the
    // panel stream.  The streams touch disjoint parts of A: diagonal block / rows below it / columns
    // right of the next panel; all read the columns of panel p.
    void potrf_top(int64_t N)
    {
        const int64_t B = block_for(N);
        LookAhead* la = (N > 2 * B) ? look_ahead_for_device() : nullptr;
        if (!la) {
            potrf(0, N, stream);
            return;
        }
        std::lock_guard<std::mutex> lock(la->enqueue);
        const bool f32 = dtype == TBS_F32;
        // panels are twice as wide while the trailing matrix is tall: its update then runs on longer
        // blocks (less of their time is prologue and epilogue), and the wider panel still finishes in
        // the shadow of that update
        auto width_for = [&](int64_t rest) { return (rest >= wide_rows) ? 2 * B : B; };
        int64_t nb = width_for(N);                                      // width of panel p
        if (piecewise_solve && nb <= piecewise_width && (nb + block_for(nb) - 1) / block_for(nb) <= kSolvePieces) {
            // the first panel: factorisation and, block by block behind it, the solve of all other rows
            note(hipEventRecord(la->column_ready, stream));             // the caller's earlier work
            note(hipStreamWaitEvent(la->panel, la->column_ready, 0));
            potrf_and_solve_below(0, nb, N - nb, la, la->column_ready, la->solve);
            note(hipEventRecord(la->panel_done, la->panel));
            note(hipStreamWaitEvent(stream, la->panel_done, 0));
        } else {
            potrf(0, nb, stream);
            trsm(nb, N - nb, 0, nb, stream);
        }
        note(hipEventRecord(la->rest_done, stream));
        for (int64_t c0 = 0; c0 + nb < N;) {                            // c0: first column of panel p
            const int64_t r0 = c0 + nb, rest = N - r0;                  // trailing matrix starts at r0
            const int64_t wn = width_for(rest);
            const int64_t nbn = (wn < rest) ? wn : rest;                // width of panel p + 1
            const int64_t below = rest - nbn;
            // panel stream: the diagonal block of panel p + 1 is brought up to date (it was last written
            // by the previous trailing update) and factored
            note(hipStreamWaitEvent(la->panel, la->rest_done, 0));
            note(syrk_impl(false, dtype, nbn, nb, -1.0, at(r0, c0), lda, 1.0, at(r0, r0), lda, la->panel));
            // the solve of the rows below follows the panel block by block on a third stream (for the
            // last panels the chain of small kernels paces the factorisation; for the first ones the
            // solve gets an earlier start on the few units it has)
            const bool piecewise = piecewise_solve && below > 0 && nbn <= piecewise_width &&
                                   (nbn + block_for(nbn) - 1) / block_for(nbn) <= kSolvePieces;
            // (Order of the calls: streams may share a hardware queue, in which packets keep the order
            // of the calls; the panel's launches come first because they pace the last panels.)
            if (!piecewise) potrf(r0, nbn, la->panel);
            // caller's stream, meanwhile: the rows below that block, then the rest of the update
            if (below > 0)
                note(tbs::launch_gemm_nt(f32, below, nbn, nb, -1.0, at(r0 + nbn, c0), lda, at(r0, c0), lda, 1.0,
                                         at(r0 + nbn, r0), lda, compute_units(), stream));
            note(hipEventRecord(la->column_ready, stream));
            if (piecewise) potrf_and_solve_below(r0, nbn, below, la, la->column_ready, la->solve);
            if (below > 0)
                note(syrk_impl(false, dtype, below, nb, -1.0, at(r0 + nbn, c0), lda, 1.0, at(r0 + nbn, r0 + nbn),
                               lda, stream, reserve_units));
            note(hipEventRecord(la->rest_done, stream));
            if (!piecewise) {
                // panel stream: the solve of the rows below needs them up to date
                note(hipStreamWaitEvent(la->panel, la->column_ready, 0));
                if (below > 0) trsm(r0 + nbn, below, r0, nbn, la->panel);
            }
            note(hipEventRecord(la->panel_done, la->panel));
            note(hipStreamWaitEvent(stream, la->panel_done, 0));
            c0 = r0;
            nb = nbn;
        }
    }
};

// Compute units the trailing update leaves to the panel stream.  The workgroup dispatcher hands the
// workgroups of a kernel round robin to the 32 shader engines (8 dies x 4) and waits when the engine
// whose turn it is has no unit with enough LDS free, so a second kernel only gets going next to a
// persistent one if every engine keeps a unit free: the reserve is a multiple of 32.  (Measured: next
// to 224 resident workgroups a 36-workgroup kernel runs at once; next to 232 it waits for them to end.)
int default_reserve_units()
{
    const char* e = std::getenv("TBS_POTRF_RESERVE");
    if (e) {
        const long v = std::atol(e);
        if (v >= 0 && v <= 128) return (int)v;
    }
    return 32;
}

int64_t default_big_block()
{
    const char* e = std::getenv("TBS_POTRF_BLOCK");
    if (e) {
        const long v = std::atol(e);
        if (v >= kTile && v <= 4096 && v % kTile == 0) return v;
    }
    return 512;
}

}  // namespace

extern "C" {

const char* tbs_status_string(tbs_status s)
{
    switch (s) {
        case TBS_OK: return "ok";
        case TBS_EINVAL: return "invalid argument";
        case TBS_EWORKSPACE: return "workspace too small";
        case TBS_ENOTSPD: return "matrix is not positive definite";
        case TBS_EHIP: return "HIP runtime error";
    }
    return "unknown status";
}

tbs_status tbs_syrk_lower_workspace(tbs_dtype dtype, int64_t N, int64_t M, size_t* bytes)
{
    if (!dtype_ok(dtype) || N < 0 || M < 0 || N > kMaxN || M > kMaxM || !bytes) return TBS_EINVAL;
    *bytes = 0;
    if (N == 0) return TBS_OK;
    const int32_t T = (int32_t)((N + kTile - 1) / kTile);
    // (operands that do not suit the assembly loops get the plan without augmented blocks, which may cut
    // other blocks: the figure covers both)
    const tbs::Plan* plan = cached_plan(T, false, dtype, M, true);
    const tbs::Plan* plain = cached_plan(T, false, dtype, M, true, false);
    if (!plan || !plain) return TBS_EINVAL;
    *bytes = std::max(tbs::syrk_workspace_bytes(dtype == TBS_F32, *plan),
                      tbs::syrk_workspace_bytes(dtype == TBS_F32, *plain));
    return TBS_OK;
}

tbs_status tbs_syrk_lower(tbs_dtype dtype, int64_t N, int64_t M, double alpha, const void* A, int64_t lda,
                          double beta, void* C, int64_t ldc, void* workspace, size_t workspace_bytes,
                          void* hip_stream)
{
    const tbs_status st = check_syrk(dtype, N, M, A, lda, C, ldc);
    if (st != TBS_OK) return st;
    return syrk_impl(false, dtype, N, M, alpha, A, lda, beta, C, ldc, (hipStream_t)hip_stream, 0, workspace,
                     workspace_bytes);
}

tbs_status tbs_syrk_lower_noalloc(tbs_dtype dtype, int64_t N, int64_t M, double alpha, const void* A, int64_t lda,
                                  double beta, void* C, int64_t ldc, void* hip_stream)
{
    const tbs_status st = check_syrk(dtype, N, M, A, lda, C, ldc);
    if (st != TBS_OK) return st;
    if (N == 0) return TBS_OK;
    const int32_t T = (int32_t)((N + kTile - 1) / kTile);
    // (the plan without eight-tile blocks: their fp64 kernel spills a few registers to memory that the
    // runtime provides per queue when such a kernel is first launched, which this entry point must not cause)
    const tbs::Plan* plan = cached_plan(T, false, dtype, M, true, false);
    if (!plan) return TBS_EINVAL;
    if (tbs::syrk_workspace_bytes(dtype == TBS_F32, *plan) > tbs::kStaticWorkspaceBytes) return TBS_EWORKSPACE;
    unsigned char* base = nullptr;
    if (tbs::static_scratch(&base) != hipSuccess) return TBS_EHIP;
    hipStream_t stream = (hipStream_t)hip_stream;
    // the counters start at zero whatever an earlier call (finished, or given up half-way) left there:
    // cleared by a kernel on the caller's stream (no memset node: the call may be recorded into a graph)
    tbs::CounterLease lease;
    lease.ctr = reinterpret_cast<unsigned int*>(base);
    lease.slice_ctr = lease.ctr + tbs::kLaunchCounters;
    if (tbs::launch_fill_i32(reinterpret_cast<int32_t*>(base), 0, tbs::kLaunchCounters + tbs::kSliceCounters, stream) !=
        hipSuccess)
        return TBS_EHIP;
    const hipError_t e = tbs::launch_syrk(dtype == TBS_F32, *plan, N, M, alpha, tbs::OperandDesc{A, lda, 1}, beta, C,
                                          ldc, persistent_workgroups(0), base + tbs::kStaticCounterBytes, lease,
                                          stream);
    return e == hipSuccess ? TBS_OK : TBS_EHIP;
}

tbs_status tbs_syr2k_lower(tbs_dtype dtype, int64_t N, int64_t M, double alpha, const void* A, int64_t lda,
                           const void* B, int64_t ldb, double beta, void* C, int64_t ldc, void* hip_stream)
{
    const tbs_status st = check_syrk(dtype, N, M, A, lda, C, ldc);
    if (st != TBS_OK) return st;
    if (ldb < (M > 1 ? M : 1) || (N > 0 && M > 0 && B == nullptr)) return TBS_EINVAL;
    if (N == 0) return TBS_OK;
    const int32_t T = (int32_t)((N + kTile - 1) / kTile);
    hipStream_t stream = (hipStream_t)hip_stream;
    const tbs::Plan* plan = cached_plan(T, true, dtype, M, false);      // rectangular blocks only
    if (!plan) return TBS_EINVAL;
    int wgs = persistent_workgroups(0);
    tbs::CounterLease lease;
    if (wgs > 0 && plan->n_items > wgs) {
        if (tbs::acquire_counters(stream, &lease) != hipSuccess) return TBS_EHIP;
        if (!lease.ctr) wgs = 0;                            // no counters free: one workgroup per block
    }
    const hipError_t e = tbs::launch_syr2k(dtype == TBS_F32, *plan, N, M, alpha, tbs::OperandDesc{A, lda, 1},
                                           tbs::OperandDesc{B, ldb, 1}, beta, C, ldc, wgs, lease, stream);
    return e == hipSuccess ? TBS_OK : TBS_EHIP;
}

// The Gram form: the order of C is the number of columns of A, the contraction runs down its rows.
static tbs_status check_gram(tbs_dtype dtype, int64_t N, int64_t M, const void* A, int64_t lda, const void* C,
                             int64_t ldc)
{
    if (!dtype_ok(dtype)) return TBS_EINVAL;
    if (N < 0 || M < 0 || M > kMaxN || N > kMaxM) return TBS_EINVAL;
    if (lda < (M > 1 ? M : 1) || ldc < (M > 1 ? M : 1)) return TBS_EINVAL;
    if (N > 0 && M > 0 && A == nullptr) return TBS_EINVAL;
    if (M > 0 && C == nullptr) return TBS_EINVAL;
    return TBS_OK;
}

tbs_status tbs_gram_lower_workspace(tbs_dtype dtype, int64_t N, int64_t M, size_t* bytes)
{
    return tbs_syrk_lower_workspace(dtype, M, N, bytes);    // the plan of a SYRK of order M, contraction N
}

tbs_status tbs_gram_lower(tbs_dtype dtype, int64_t N, int64_t M, double alpha, const void* A, int64_t lda,
                          double beta, void* C, int64_t ldc, void* workspace, size_t workspace_bytes,
                          void* hip_stream)
{
    const tbs_status st = check_gram(dtype, N, M, A, lda, C, ldc);
    if (st != TBS_OK) return st;
    if (M == 0) return TBS_OK;
    const int32_t T = (int32_t)((M + kTile - 1) / kTile);
    hipStream_t stream = (hipStream_t)hip_stream;
    const tbs::Plan* plan = nullptr;
    const bool aug_ok = operands_suit_fast_path(dtype, M, N, 1, lda);
    const tbs_status ps = plan_for_call(T, false, dtype, N, workspace, workspace_bytes, &plan, aug_ok);
    if (ps != TBS_OK) return ps;
    int wgs = persistent_workgroups(0);
    tbs::CounterLease lease;
    if ((wgs > 0 && plan->n_items > wgs) || plan->n_ws_blocks > 0) {
        if (tbs::acquire_counters(stream, &lease) != hipSuccess) return TBS_EHIP;
        if (!lease.ctr) {
            plan = cached_plan(T, false, dtype, N, false, aug_ok);
            if (!plan) return TBS_EINVAL;
            wgs = 0;
        }
    }
    // panel row i of the operand is column i of A: rows one element apart, the contraction one
    // leading dimension apart
    const hipError_t e = tbs::launch_syrk(dtype == TBS_F32, *plan, M, N, alpha, tbs::OperandDesc{A, 1, lda}, beta, C,
                                          ldc, wgs, workspace, lease, stream);
    return e == hipSuccess ? TBS_OK : TBS_EHIP;
}

tbs_status tbs_syrk_lower_square(tbs_dtype dtype, int64_t N, int64_t M, double alpha, const void* A,
                                 int64_t lda, double beta, void* C, int64_t ldc, void* workspace,
                                 size_t workspace_bytes, void* hip_stream)
{
    (void)workspace;
    (void)workspace_bytes;
    const tbs_status st = check_syrk(dtype, N, M, A, lda, C, ldc);
    if (st != TBS_OK) return st;
    return syrk_impl(true, dtype, N, M, alpha, A, lda, beta, C, ldc, (hipStream_t)hip_stream);
}

tbs_status tbs_syrk_lower_query(tbs_dtype dtype, int64_t N, int64_t M, int32_t square, tbs_plan_info* out)
{
    if (!dtype_ok(dtype) || N < 0 || M < 0 || N > kMaxN || M > kMaxM || !out) return TBS_EINVAL;
    const int32_t T = (int32_t)((N + kTile - 1) / kTile);
    const tbs::Plan* plan = cached_plan(T, square == 1, dtype, M, square == 0);
    if (!plan) return TBS_EINVAL;
    tbs::PlanStats st;
    tbs::plan_stats(*plan, N, M, &st);
    tbs_plan_info r{};
    r.k = kK;
    r.b = kTile;
    r.levels = st.levels;
    r.c = st.levels > 0 ? plan->c[0] : 0;
    r.l = st.levels > 0 ? T - kK * plan->c[0] : T;
    r.family = st.levels > 0 ? plan->fam[0] : 0;
    r.max_slices = plan->n_ws_blocks > 0 ? plan->ws_slices : 1;
    r.n_sliced_blocks = plan->n_ws_blocks;
    r.workspace_bytes = (int64_t)tbs::syrk_workspace_bytes(dtype == TBS_F32, *plan);
    r.tile_rows = T;
    r.n_items = plan->n_items;
    r.n_tri_blocks = st.n_tri;
    r.n_rect_blocks = st.n_rect;
    r.n_diag_tiles = st.n_diag;
    // (a plan with eight-tile blocks keeps eight tiles of C per block and stages six panels: the bound it is
    // held against is the one for that larger fast memory)
    bool eight = false;
    for (int32_t sg = 0; sg < plan->nseg; ++sg) eight = eight || (plan->seg[sg].kind == tbs::kSegTri && plan->seg[sg].aug);
    r.S_C_elems = (int64_t)kTile * kTile * (eight ? 8 : kK * (kK - 1) / 2);
    const int64_t kc = dtype == TBS_F32 ? 32 : 16;      // staged columns per chunk, two buffers
    r.S_res_elems = r.S_C_elems + 2 * (int64_t)(eight ? kK + 2 : kK) * kTile * kc;
    r.A_elems = st.A_elems;
    r.A_elems_top = st.A_elems_top;
    r.C_elems = st.C_elems;
    const double n2m = (double)N * (double)N * (double)M;
    r.tbs_bound_elems = n2m / (std::sqrt(2.0) * std::sqrt((double)r.S_C_elems));
    r.tiled_lead_elems = n2m / ((kK - 1.0) * kTile);
    r.square_elems = n2m / std::sqrt((double)r.S_C_elems);
    *out = r;
    return TBS_OK;
}

tbs_status tbs_syrk_lower_enumerate(tbs_dtype dtype, int64_t N, int64_t M, int32_t square, int32_t* items,
                                    int64_t capacity, int64_t* n_items)
{
    if (!dtype_ok(dtype) || N < 0 || N > kMaxN || M < 0 || M > kMaxM || !n_items) return TBS_EINVAL;
    const int32_t T = (int32_t)((N + kTile - 1) / kTile);
    const tbs::Plan* plan = cached_plan(T, square == 1, dtype, M, square == 0);
    if (!plan) return TBS_EINVAL;
    *n_items = plan->n_items;
    if (!items) return TBS_OK;
    if (capacity < plan->n_items) return TBS_EWORKSPACE;
    for (int32_t t = 0; t < plan->n_items; ++t) {
        tbs::Item it;
        tbs::tbs_decode(*plan, t, it);
        int32_t* o = items + (int64_t)t * TBS_ENUMERATE_COLUMNS;
        o[0] = it.kind;
        o[1] = it.nrow;
        o[2] = it.ncol;
        for (int s = 0; s < 5; ++s) o[3 + s] = it.rows[s];
        o[8] = it.slice;
        o[9] = it.slices;
        o[10] = it.rows[5];
        o[11] = it.aug1;
        o[12] = it.aug2;
    }
    return TBS_OK;
}

tbs_status tbs_potrf_lower_workspace(tbs_dtype dtype, int64_t N, size_t* bytes)
{
    if (!dtype_ok(dtype) || N < 0 || N > kMaxN || !bytes) return TBS_EINVAL;
    *bytes = kInfoBytes;
    return TBS_OK;
}

tbs_status tbs_potrf_lower(tbs_dtype dtype, int64_t N, void* A, int64_t lda, void* workspace,
                           size_t workspace_bytes, int32_t* info_host, void* hip_stream)
{
    size_t need = 0;
    if (tbs_potrf_lower_workspace(dtype, N, &need) != TBS_OK) return TBS_EINVAL;
    if (lda < (N > 1 ? N : 1)) return TBS_EINVAL;
    if (N > 0 && A == nullptr) return TBS_EINVAL;
    if (N == 0) {
        if (info_host) *info_host = 0;
        return TBS_OK;
    }
    if (workspace == nullptr || workspace_bytes < need) return TBS_EWORKSPACE;
    if ((reinterpret_cast<uintptr_t>(workspace) & 15) != 0) return TBS_EINVAL;

    Lbc ctx;
    ctx.dtype = dtype;
    ctx.es = elem_size(dtype);
    ctx.A = static_cast<char*>(A);
    ctx.lda = lda;
    ctx.info = static_cast<int32_t*>(workspace);
    ctx.stream = (hipStream_t)hip_stream;
    ctx.big_block = default_big_block();
    ctx.reserve_units = default_reserve_units();
    if (const char* e = std::getenv("TBS_POTRF_WIDE_ROWS")) {
        const long v = std::atol(e);
        if (v > 0) ctx.wide_rows = v;
    }
    if (const char* e = std::getenv("TBS_POTRF_PIECEWISE")) {
        ctx.piecewise_solve = e[0] != '0';
        const long v = std::atol(e);
        if (v >= 64) ctx.piecewise_width = v;
    }
    if (const char* e = std::getenv("TBS_POTRF_PANEL")) ctx.left_panel = e[0] == 'l';
    if (const char* e = std::getenv("TBS_POTRF_FUSED_ROWS")) {
        const long v = std::atol(e);
        if (v >= 0) ctx.fused_trsm_rows = v;
    }
    ctx.note(tbs::launch_fill_i32(ctx.info, 0, 1, ctx.stream));
    ctx.potrf_top(N);
    if (ctx.err != hipSuccess) return TBS_EHIP;
    if (info_host) {
        int32_t info = 0;
        if (hipMemcpyAsync(&info, ctx.info, sizeof(info), hipMemcpyDeviceToHost, ctx.stream) != hipSuccess)
            return TBS_EHIP;
        if (hipStreamSynchronize(ctx.stream) != hipSuccess) return TBS_EHIP;
        *info_host = info;
        if (info != 0) return TBS_ENOTSPD;
    }
    return TBS_OK;
}

}  // extern "C"
