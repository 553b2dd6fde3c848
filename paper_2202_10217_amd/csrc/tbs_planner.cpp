// tbs_planner.cpp -- builds the work-list descriptor of the tiled Triangle Block Scheme
// (Algorithm 4 with the changes of Section 5.1.4), flattening its recursion level by level.
#include "tbs_planner.h"

#include <algorithm>
#include <functional>
#include <numeric>
#include <queue>
#include <vector>

namespace tbs {

int32_t choose_c(int32_t upper, int32_t k)
{
    for (int32_t c = upper; c > 0; --c) {
        bool ok = true;
        for (int32_t d = 2; d <= k - 2 && ok; ++d) ok = std::gcd(c, d) == 1;
        if (ok) return c;
    }
    return 0;
}

namespace {

Seg rect_seg(int32_t level, int64_t nz, int32_t r0, int32_t r1, int32_t c0, int32_t c1, int32_t mr,
             int32_t nc, bool diag = false)
{
    Seg s{};
    s.kind = kSegRect;
    s.diag = diag ? 1 : 0;
    s.level = level;
    s.r0 = r0; s.r1 = r1; s.c0 = c0; s.c1 = c1;
    s.mr = mr; s.nc = nc;
    s.nI = (r1 - r0 + s.mr - 1) / s.mr;
    s.nJ = (c1 - c0 + s.nc - 1) / s.nc;
    s.count = (int32_t)(nz * s.nI * s.nJ);
    return s;
}

}  // namespace

bool build_plan(int32_t T, const PlanTuning& tune, Plan* out)
{
    if (T < 0 || T > (1 << 15)) return false;
    if (tune.mr < 1 || tune.mr > kRectRows || tune.nc < 1 || tune.nc > kRectCols) return false;
    if (tune.mr_deep < 0 || tune.mr_deep > kRectRows || tune.nc_deep < 0 || tune.nc_deep > kRectCols) return false;
    Plan p{};
    p.k = kK;
    p.T = T;
    std::vector<Seg> tri, rect, base;
    const int32_t k = p.k;
    // rectangles that cover a triangular region take its diagonal tiles along, unless base zones are
    // triangle blocks (which cannot): then every diagonal tile is an item of its own
    if (tune.augment && tune.tri_base) return false;        // (augmented blocks take diagonal tiles themselves)
    const bool with_diag = !tune.tri_base;
    {
        int32_t level = 0, Tl = T;
        int64_t nz = 1;
        for (;;) {
            const int32_t mr = tune.mr, nc = tune.nc;       // rectangles left of a zone
            // rectangles of a triangular region: their own shape if one is given (a block that
            // straddles the diagonal keeps the tiles on and below it)
            const bool own = tune.mr_deep > 0 && tune.nc_deep > 0;
            const int32_t mrt = own ? tune.mr_deep : tune.mr;
            const int32_t nct = own ? tune.nc_deep : tune.nc;
            int32_t c = choose_c(Tl / k, k), fam = 0;
            if (tune.xor_family && Tl / k >= 4) {
                int32_t m = 0;
                while ((2 << m) <= Tl / k) ++m;             // 2^m = largest power of two <= Tl / k
                if ((1 << m) > c) {
                    c = 1 << m;
                    fam = m;
                }
            }
            const bool room = level < kMaxLevels - 1 && level < tune.tri_levels &&
                              (int)(tri.size() + rect.size()) + 3 < kMaxSegs - 2;
            if (c < k - 1 || !room) {                       // base zones (c too small)
                if (Tl >= (with_diag ? 1 : 2)) {
                    if (Tl <= k && tune.tri_base) {
                        Seg s{};
                        s.kind = kSegTriBase;
                        s.level = level;
                        s.r1 = Tl;
                        s.count = (int32_t)nz;
                        base.push_back(s);
                    } else {
                        rect.push_back(rect_seg(level, nz, 0, Tl, 0, with_diag ? Tl : Tl - 1, mrt, nct, with_diag));
                    }
                }
                break;
            }
            p.c[level] = c;
            p.fam[level] = fam;
            Seg s{};
            s.kind = kSegTri;
            s.level = level;
            s.count = (int32_t)(nz * c * c);
            s.group = (tune.die_groups && level == 0 && fam >= 3) ? 1 : 0;
            s.aug = (tune.augment && level == 0) ? 1 : 0;
            tri.push_back(s);
            const int32_t done = k * c, l = Tl - done;
            if (l > 0) {                                    // the last l tile rows
                rect.push_back(rect_seg(level, nz, done, Tl, 0, done, mr, nc));
                if (l >= (with_diag ? 1 : 2))
                    rect.push_back(rect_seg(level, nz, done, Tl, done, with_diag ? Tl : Tl - 1, mrt, nct, with_diag));
            }
            if (s.aug) {
                // the blocks have taken every tile of the zones except the diagonal tiles of zones 1 and 3
                for (int32_t z = 1; z < k; z += 2) {
                    Seg d{};
                    d.kind = kSegDiagRun;
                    d.r0 = z * c;
                    d.r1 = (z + 1) * c;
                    d.count = c;
                    rect.push_back(d);
                }
                break;
            }
            nz *= k;
            Tl = c;
            ++level;
        }
    }
    // longest blocks first: triangle blocks by level, rectangles, base triangles, diagonal tiles
    // (a base triangle of k rows is as long as a family block: it goes before the rectangles then)
    int32_t n = 0, first = 0;
    auto push = [&](Seg s) {
        if (s.count <= 0) return;
        s.slices = 1;
        s.t0 = 0;
        s.ws0 = 0;
        s.first = first;
        first += s.count;
        p.seg[n++] = s;
    };
    std::vector<Seg> all(tri);
    all.insert(all.end(), rect.begin(), rect.end());
    all.insert(all.end(), base.begin(), base.end());
    auto tiles_of = [&](const Seg& s) {
        if (s.kind == kSegTri) return k * (k - 1) / 2 + (s.aug ? 2 : 0);
        if (s.kind == kSegDiagRun) return 1;
        if (s.kind == kSegTriBase) return s.r1 * (s.r1 - 1) / 2;
        return s.mr * s.nc;
    };
    std::stable_sort(all.begin(), all.end(),
                     [&](const Seg& a, const Seg& b) { return tiles_of(a) > tiles_of(b); });
    for (const Seg& s : all) push(s);
    if (T > 0 && !with_diag) {
        Seg d{};
        d.kind = kSegDiag;
        d.count = T;
        push(d);
    }
    p.nseg = n;
    p.n_items = first;
    p.n_ws_blocks = 0;
    p.ws_slices = 1;
    set_team_items(&p);
    *out = p;
    return true;
}

void set_team_items(Plan* plan)
{
    plan->team_items = 0;
    if (plan->nseg < 1) return;
    const Seg& s = plan->seg[0];
    if (s.kind == kSegTri && s.group && s.level == 0 && s.first == 0 && s.t0 == 0 && s.slices <= 1)
        plan->team_items = s.count / kGroupItems * kGroupItems;
}

bool apply_slicing(const Plan& base, const Slicing& sl, Plan* out)
{
    Plan p = base;
    std::vector<Seg> segs;
    for (int32_t i = 0; i < base.nseg; ++i) {
        Seg s = base.seg[i];                                // unsliced: count = blocks, t0 = 0
        s.slices = (s.kind == kSegTri || s.kind == kSegTriBase) ? sl.tri : sl.rect;
        if (s.kind == kSegTri && s.aug && s.slices > 1) return false;   // (augmented blocks are never cut)
        segs.push_back(s);
    }
    if (sl.tail_blocks > 0 && sl.tail > 1 && !segs.empty()) {   // the end of the list, cut more finely
        int32_t want = sl.tail_blocks;
        std::vector<Seg> tail;
        while (want > 0 && !segs.empty()) {
            Seg& last = segs.back();
            if (last.kind == kSegTri && last.aug) return false;
            const int32_t take = std::min(want, last.count);
            Seg cut = last;
            cut.t0 = last.t0 + last.count - take;
            cut.count = take;
            cut.slices = std::max(sl.tail, last.slices);
            tail.insert(tail.begin(), cut);
            last.count -= take;
            want -= take;
            if (last.count == 0) segs.pop_back();
        }
        segs.insert(segs.end(), tail.begin(), tail.end());
    }
    if ((int32_t)segs.size() > kMaxSegs) return false;
    int32_t first = 0, ws = 0, smax = 1;
    p.nseg = 0;
    for (Seg s : segs) {
        if (s.slices < 1) s.slices = 1;
        if (s.slices > kMaxSlices) return false;
        s.first = first;
        s.ws0 = 0;
        if (s.slices > 1) {
            s.ws0 = ws;
            ws += s.count;
            smax = std::max(smax, s.slices);
        }
        s.count *= s.slices;                                // items
        first += s.count;
        p.seg[p.nseg++] = s;
    }
    if (ws > kMaxSliceBlocks) return false;
    p.n_items = first;
    p.n_ws_blocks = ws;
    p.ws_slices = smax;
    set_team_items(&p);
    *out = p;
    return true;
}

double simulate_makespan(const Plan& p, int32_t ncu, double overhead_tiles, double slice_overhead_tiles,
                         double slice_per_part_tiles)
{
    std::priority_queue<double, std::vector<double>, std::greater<double>> free_at;
    for (int32_t u = 0; u < ncu; ++u) free_at.push(0.0);
    double end = 0.0;
    for (int32_t t = 0; t < p.n_items; ++t) {
        Item it;
        tbs_decode(p, t, it);
        double tiles = 0.0;
        if (it.kind == kTri) {
            tiles = 0.5 * it.nrow * (it.nrow - 1);
        } else if (it.kind == kAug) {
            // (writing eight tiles back takes longer than six: most of a block's fixed cost is its epilogue)
            tiles = 8.0 + 0.6 * overhead_tiles;
        } else if (it.kind == kRect || it.kind == kRectDiag) {
            for (int r = 0; r < kRectRows; ++r)
                for (int q = 0; q < kRectCols; ++q)
                    if (it.rows[kRectCols + r] >= 0 && it.rows[q] >= 0 &&
                        (it.rows[q] < it.rows[kRectCols + r] ||
                         (it.kind == kRectDiag && it.rows[q] == it.rows[kRectCols + r])))
                        tiles += 1.0;
        } else if (it.kind == kDiag) {
            tiles = 1.0;                                    // computed as a whole tile
        } else {
            continue;                                       // empty block: exits at once
        }
        // a part also stores its accumulators, and the last one to finish sums all parts: that cost
        // grows with their number and is what the block's completion waits for
        if (it.slices > 1) tiles = tiles / it.slices + slice_overhead_tiles + slice_per_part_tiles * it.slices;
        const double start = free_at.top();
        free_at.pop();
        const double stop = start + tiles + overhead_tiles;
        free_at.push(stop);
        end = std::max(end, stop);
    }
    return end;
}

bool choose_plan(int32_t T, bool square, int32_t ncu, double overhead_tiles, Plan* out, bool xor_family,
                 int32_t max_slices, double slice_overhead_tiles, double slice_per_part_tiles, bool die_groups,
                 bool augment)
{
    if (square) {
        // rectangles only; for small matrices the block shape with the shortest simulated makespan
        // (the same rule as below, so that the baseline is not handicapped by coarse blocks)
        if (!build_plan(T, PlanTuning{0, kRectRows, kRectCols, false}, out)) return false;
        if (0.5 * (double)T * (double)T / (double)std::max(ncu, 1) > 200.0 || T < 2) return true;
        double best_sq = simulate_makespan(*out, ncu, overhead_tiles, slice_overhead_tiles, slice_per_part_tiles);
        const int32_t sq_shapes[4][2] = {{2, 2}, {1, 3}, {1, 2}, {1, 1}};
        for (const auto& sh : sq_shapes) {
            Plan cand;
            if (!build_plan(T, PlanTuning{0, sh[0], sh[1], false}, &cand)) continue;
            const double span = simulate_makespan(cand, ncu, overhead_tiles, slice_overhead_tiles, slice_per_part_tiles);
            if (span < best_sq * 0.98) {
                best_sq = span;
                *out = cand;
            }
        }
        return true;
    }
    PlanTuning coarse{kMaxLevels, kRectRows, kRectCols, true};
    coarse.xor_family = xor_family;
    coarse.die_groups = die_groups;
    if (!build_plan(T, coarse, out)) return false;
    // with many blocks per compute unit the granularity of the tail does not matter
    const double per_unit = 0.5 * (double)T * (double)T / (double)std::max(ncu, 1);
    if (per_unit > 200.0 || T < 2) return true;
    double best = simulate_makespan(*out, ncu, overhead_tiles, slice_overhead_tiles, slice_per_part_tiles);
    // cutting blocks along the contraction dimension costs a workspace and an extra pass over the
    // parts: only for problems with few tiles per compute unit, and only for a clear gain
    const bool slicing = max_slices > 1 && per_unit <= 40.0;
    double best_sliced = best;
    Plan sliced = *out;
    bool have_sliced = false;
    auto try_slicings = [&](const Plan& base) {
        // all blocks of a kind cut alike (tri, rect), or only the end of the list cut (that many items,
        // that finely): the end decides when the last unit finishes
        const int32_t whole[3] = {1, 2, 4};
        const int32_t tail_items[9] = {16, 24, 32, 36, 40, 48, 64, 96, 128};
        const int32_t tail_parts[6] = {3, 4, 5, 6, 8, 16};
        auto consider = [&](const Slicing& sl) {
            Plan q;
            if (!apply_slicing(base, sl, &q)) return;
            // at most 128 MB of workspace (6 tiles of doubles per part)
            if ((int64_t)q.n_ws_blocks * q.ws_slices * 6 * kTile * kTile * 8 > ((int64_t)128 << 20)) return;
            const double span = simulate_makespan(q, ncu, overhead_tiles, slice_overhead_tiles, slice_per_part_tiles);
            if (span < best_sliced * 0.995) {
                best_sliced = span;
                sliced = q;
                have_sliced = true;
            }
        };
        for (int32_t st : whole)
            for (int32_t sr : whole) {
                if (st > max_slices || sr > max_slices) continue;
                if (st > 1 || sr > 1) consider(Slicing{st, sr, 0, 1});
                for (int32_t tp : {4, 8, 16})
                    if (tp <= max_slices && tp > std::max(st, sr)) consider(Slicing{st, sr, 64, tp});
            }
        for (int32_t ti : tail_items)
            for (int32_t tp : tail_parts)
                if (tp <= max_slices) consider(Slicing{1, 1, ti, tp});
    };
    if (slicing) try_slicings(*out);
    const int32_t shapes[5][2] = {{2, 3}, {2, 2}, {1, 3}, {1, 2}, {1, 1}};
    for (int32_t levels = kMaxLevels; levels >= 0; levels = (levels == kMaxLevels) ? 2 : levels - 1) {
        for (const auto& sh : shapes) {
            for (int32_t mrt = kRectRows; mrt >= 1; --mrt)      // triangular regions: mrt x nct blocks
                for (int32_t nct = kRectCols; nct >= 1; --nct) {
                    PlanTuning tune{levels, sh[0], sh[1], false, mrt, nct};
                    tune.xor_family = xor_family;
                    tune.die_groups = die_groups;
                    Plan cand;
                    if (!build_plan(T, tune, &cand)) continue;
                    const double span = simulate_makespan(cand, ncu, overhead_tiles, slice_overhead_tiles, slice_per_part_tiles);
                    if (span < best * 0.98) {               // prefer the coarser plan on near ties
                        best = span;
                        *out = cand;
                    }
                    if (slicing && sh[0] == 1 && mrt == 1) try_slicings(cand);
                    if (augment && levels == kMaxLevels) {   // the same with augmented top-level blocks
                        tune.augment = true;
                        if (!build_plan(T, tune, &cand) || cand.nseg < 1 || !cand.seg[0].aug) continue;
                        // (measured: with more than two rounds of top-level blocks the finer plain plans do
                        // as well or better; the larger blocks pay where they save a short extra round)
                        if ((int64_t)cand.c[0] * cand.c[0] > 2 * (int64_t)ncu) continue;
                        const double aspan = simulate_makespan(cand, ncu, overhead_tiles, slice_overhead_tiles, slice_per_part_tiles);
                        if (aspan < best * 0.97) {
                            best = aspan;
                            *out = cand;
                        }
                        if (slicing && mrt == 1) try_slicings(cand);
                    }
                }
        }
    }
    if (have_sliced && best_sliced < best * 0.97) *out = sliced;
    return true;
}

void plan_stats(const Plan& p, int64_t N, int64_t M, PlanStats* st)
{
    PlanStats r{};
    for (int32_t s = 0; s < p.nseg; ++s)
        if (p.seg[s].kind == kSegTri) r.levels = std::max(r.levels, p.seg[s].level + 1);
    auto panel_rows = [&](int32_t t) -> double {
        const int64_t lo = (int64_t)t * kTile;
        return (double)std::max<int64_t>(0, std::min<int64_t>(kTile, N - lo));
    };
    for (int32_t s = 0; s < p.nseg; ++s) {
        const Seg& sg = p.seg[s];
        for (int32_t t = 0; t < sg.count; ++t) {
            Item it;
            tbs_decode(p, sg.first + t, it);
            const bool head = it.slice == 0;                // blocks are counted once, at their first part
            double a = 0;
            if (it.kind == kTri) {
                if (head) ++r.n_tri;
                for (int32_t u = 0; u < it.nrow; ++u) a += panel_rows(it.rows[u]);
            } else if (it.kind == kAug) {
                ++r.n_tri;
                for (int32_t u = 0; u < kMaxPanels; ++u) a += panel_rows(it.rows[u]);   // (a diagonal tile's panel twice)
                if (it.rows[4] == it.rows[0]) ++r.n_diag;
                if (it.rows[5] == it.rows[2]) ++r.n_diag;
            } else if (it.kind == kRect || it.kind == kRectDiag) {
                if (head) ++r.n_rect;
                for (int32_t u = 0; u < kMaxPanels; ++u)
                    if (it.rows[u] >= 0) a += panel_rows(it.rows[u]);
                if (it.kind == kRectDiag && head)
                    for (int32_t q = 0; q < kRectCols; ++q)
                        for (int32_t rr = 0; rr < kRectRows; ++rr)
                            if (it.rows[q] >= 0 && it.rows[q] == it.rows[kRectCols + rr]) ++r.n_diag;
            } else if (it.kind == kDiag) {
                if (head) ++r.n_diag;
                a += panel_rows(it.rows[0]);
            } else {
                ++r.n_empty;
            }
            a /= (double)it.slices;                         // a part loads its share of the columns
            r.A_elems += a * (double)M;
            if (sg.kind == kSegTri && sg.level == 0) r.A_elems_top += a * (double)M;
        }
    }
    r.C_elems = 0.5 * (double)N * (double)(N + 1);
    *st = r;
}

}  // namespace tbs
