// tbs_planner.h -- host-side construction of Triangle Block Scheme plans (integer work only).
#pragma once
#include "tbs_plan.h"

namespace tbs {

// Largest c <= upper coprime with every integer of [2, k-2] (hypothesis of the validity lemma of
// Section 5.1.2 for the cyclic family); 0 when upper <= 0.
int32_t choose_c(int32_t upper, int32_t k);

// Plan for a matrix of T tile rows.  square = true: rectangular blocks only (the baseline).
// Returns false when T is out of range for the descriptor.
bool build_plan(int32_t T, bool square, Plan* out);

struct PlanStats {
    int32_t levels;
    int64_t n_tri, n_rect, n_diag, n_empty;
    double A_elems, A_elems_top, C_elems;
};

// Walks the work list (tbs_decode on every item) and counts blocks and the A / C elements the
// schedule loads for an N x M problem, with the accounting of Sections 5.1.3 and 5.1.4.
void plan_stats(const Plan& p, int64_t N, int64_t M, PlanStats* st);

}  // namespace tbs
