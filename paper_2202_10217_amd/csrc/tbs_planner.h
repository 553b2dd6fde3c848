// tbs_planner.h -- host-side construction of Triangle Block Scheme plans (integer work only).
#pragma once
#include "tbs_plan.h"

namespace tbs {

// Largest c <= upper coprime with every integer of [2, k-2] (hypothesis of the validity lemma of
// Section 5.1.2 for the cyclic family); 0 when upper <= 0.
int32_t choose_c(int32_t upper, int32_t k);

// How a plan covers what the top-level triangle blocks leave: how many recursion levels use
// triangle blocks, the shape of the rectangular blocks, whether a base zone of at most k tile rows
// is one triangle block.
struct PlanTuning {
    int32_t tri_levels;      // levels that use triangle blocks (0: none, i.e. rectangles only)
    int32_t mr, nc;          // rectangular block: mr x nc tiles, mr <= kRectRows, nc <= kRectCols
    bool tri_base;           // base zones of <= k tile rows become one triangle block
    int32_t mr_deep = 0, nc_deep = 0;   // shape of the rectangles of triangular regions (0: as mr, nc);
                                        // one tile row high whenever they carry the diagonal tiles
    bool xor_family = true;  // levels may use c = 2^m with the XOR family where that covers more rows
    bool die_groups = true;  // top-level blocks of the XOR family in groups of 32 that share tile rows
    bool augment = false;    // top-level blocks take two tiles of the diagonal zones each (no recursion then)
};

// How the blocks of a plan are cut along the contraction dimension (1 = not at all): all triangle
// blocks, all rectangular blocks, and the last `tail_blocks` blocks of the list (the ones that decide
// when the last compute unit finishes) more finely.
struct Slicing {
    int32_t tri = 1, rect = 1, tail_blocks = 0, tail = 1;
};
constexpr int32_t kMaxSliceBlocks = 512;   // sliced blocks per plan (each has a counter and workspace)
constexpr int32_t kMaxSlices = 32;

// Sets plan->team_items: the leading whole groups of segment 0 if that segment is grouped and not cut.
void set_team_items(Plan* plan);

// Rewrites the segments of an unsliced plan for the given slicing; false if it does not fit the
// descriptor (too many segments or sliced blocks).
bool apply_slicing(const Plan& base, const Slicing& sl, Plan* out);

// Plan for a matrix of T tile rows with the given tuning.  Returns false when T is out of range for
// the descriptor.
bool build_plan(int32_t T, const PlanTuning& tune, Plan* out);

// The plan the library uses.  square = true: rectangular blocks only (the baseline): 2 x 3 tiles, smaller
// ones for small matrices by the rule below.
// Otherwise the schedule of Algorithm 4; for small matrices, where a compute unit receives only a
// few blocks, the candidates differ in how finely the diagonal zones and the last tile rows are cut,
// and the one with the shortest simulated makespan on `ncu` compute units is taken (blocks are
// dispatched in list order to the first free unit; a block costs its tiles plus `overhead_tiles`).
// max_slices > 1 lets the choice cut blocks along the contraction dimension (at most that finely);
// a part of a block cut into S parts costs `slice_overhead_tiles + S * slice_per_part_tiles` on top
// (storing the part; the last part to finish sums all of them).
bool choose_plan(int32_t T, bool square, int32_t ncu, double overhead_tiles, Plan* out, bool xor_family = true,
                 int32_t max_slices = 1, double slice_overhead_tiles = 0.03, double slice_per_part_tiles = 0.0,
                 bool die_groups = true, bool augment = false);

// Makespan, in tile units, of dispatching the plan's blocks in order onto ncu units.
double simulate_makespan(const Plan& p, int32_t ncu, double overhead_tiles, double slice_overhead_tiles = 0.03,
                         double slice_per_part_tiles = 0.0);

struct PlanStats {
    int32_t levels;
    int64_t n_tri, n_rect, n_diag, n_empty;
    double A_elems, A_elems_top, C_elems;
};

// Walks the work list (tbs_decode on every item) and counts blocks and the A / C elements the
// schedule loads for an N x M problem, with the accounting of Sections 5.1.3 and 5.1.4.
void plan_stats(const Plan& p, int64_t N, int64_t M, PlanStats* st);

}  // namespace tbs
