// tbs_plan.h -- the Triangle Block Scheme work list as a compact descriptor plus index arithmetic.
//
// The partition of C follows Algorithm 4 / Section 5.1.4 of the paper, on b x b tiles:
//   level 0 is the whole matrix (T tile rows); a level with T_L tile rows per zone picks
//   c_L = largest integer <= T_L / k coprime with every integer of [2, k-2] (Section 5.1.2);
//   if c_L >= k-1 its c_L^2 triangle blocks R^{i,j} = { u c_L + f^{i,j}(u) : u < k }, with the
//   cyclic family f(0) = j, f(u) = (i + j (u-1)) mod c_L, cover the k(k-1)/2 square zones
//   (where a power of two 2^m <= T_L / k exceeds that c_L, the level uses c_L = 2^m with the family
//   f(0) = j, f(1) = i, f(2) = i XOR j, f(3) = i XOR (x j mod x^m + x + 1), which is valid by the same
//   definition (Section 5.1.1) and leaves fewer tile rows over),
//   the l_L = T_L - k c_L last tile rows are covered by rectangular blocks, and each of the k
//   diagonal zones (c_L tile rows) becomes a zone of level L+1;  if c_L < k-1 the zone is a base
//   zone: one triangle block on its consecutive rows when it has at most k of them, rectangular
//   blocks otherwise.  Diagonal tiles: the rectangular blocks that cover a triangular region (a base
//   zone, the triangle of the last l_L tile rows) take the diagonal tiles of that region with them
//   (item kind kRectDiag); a plan whose base zones are triangle blocks lists all diagonal tiles
//   separately instead (kDiag).
//
// Augmented plans (a choice of this library, not of the paper: a compute unit has accumulators for eight
// tiles, a triangle block on k = 4 tile rows has six): the top-level triangle blocks each take two tiles
// of the diagonal zones with them, a tile between one of the block's rows and one further row of the
// same zone.  The c^2 blocks absorb every off-diagonal tile of the k zones (2 c^2 - 2 c of them) and the
// diagonal tiles of zones 0 and 2, so there is no recursion: what is left are the diagonal tiles of
// zones 1 and 3 and the last l tile rows.  Which tile goes to which block, for block (i, j):
//   zones 0 and 1 (f(0) = j, f(1) = i):  i > j: tile (i, j) of zone 0;  j > i: tile (j, i) of zone 1;
//     i = j: the diagonal tile (j, j) of zone 0.  Every off-diagonal tile of the two zones exactly once.
//   zones 2 and 3:  j = 0: the diagonal tile of zone 2 on the block's row.  Otherwise a tile {f, f + j}
//     (cyclic family: + modulo c, zone 2 for j < c / 2, zone 3 for j > c / 2, c is odd) or {f, f XOR j}
//     (XOR family: zone 2 if i has the highest bit of j, else zone 3), f the block's row in that zone:
//     for a fixed j the blocks that use a zone give pairwise different pairs whose difference is j,
//     and every pair of rows of a zone has exactly one j (cyclic: one of +-j) that leads to it.
//
// The descriptor is small enough to be a kernel argument; every workgroup turns its index into
// its block with tbs_decode().  The host uses the same function to expand, count and check plans,
// so what is tested on the CPU is what the kernels execute.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define TBS_HD __host__ __device__ inline
#else
#define TBS_HD inline
#endif

namespace tbs {

constexpr int kTile = 64;        // b: tile side in elements
constexpr int kK = 4;            // k: tile rows per triangle block
constexpr int kMaxLevels = 10;
constexpr int kMaxSegs = 28;
constexpr int kRectRows = 2;     // rectangular block: at most 2 x 3 tiles
constexpr int kRectCols = 3;
constexpr int kMaxPanels = 6;    // panels of A a block can stage (k + 2, or kRectRows + kRectCols)
constexpr int kGroupItems = 32;  // blocks of a group that the workgroups of one die take together

// kRect: tiles (r, q) of the block's rows x columns with q < r.  kRectDiag: q <= r, where of a tile
// (r, r) only the part on and below the diagonal belongs to the block.
// kAug: a triangle block on rows[0..3] plus the tiles named by aug1 and aug2 (see Item).
enum ItemKind : int32_t { kTri = 0, kRect = 1, kDiag = 2, kEmpty = 3, kRectDiag = 4, kAug = 5 };

enum SegKind : int32_t {
    kSegTri = 0,       // c^2 triangle blocks in each zone of a level
    kSegTriBase = 1,   // one triangle block on the consecutive rows of each base zone
    kSegRect = 2,      // grid of rectangular blocks inside each zone of a level
    kSegDiag = 3,      // all diagonal tiles (only in plans whose rectangles do not carry them)
    kSegDiagRun = 4    // the diagonal tiles of the tile rows [r0, r1) (augmented plans)
};

struct Seg {
    int32_t kind;
    int32_t first;     // index of the first item of the segment
    int32_t count;     // number of items
    int32_t level;     // zones of this level are addressed (k^level of them)
    int32_t r0, r1;    // kSegRect: tile rows [r0, r1) relative to the zone; kSegTriBase: r1 = zone size
    int32_t c0, c1;    // kSegRect: tile columns [c0, c1) relative to the zone
    int32_t nI, nJ;    // kSegRect: blocks per zone along rows / columns
    int32_t mr, nc;    // kSegRect: block shape in tiles
    int32_t diag;      // kSegRect: 1 = the columns reach the diagonal and tiles (r, r) belong to the blocks
    // Slicing along the contraction dimension: every block of the segment is `slices` consecutive
    // items, item s of a block takes the s-th part of the columns of A; the parts are summed in order
    // by the last one to finish (see the kernels).  `t0`: the segment covers the blocks t0, t0 + 1, ...
    // of the enumeration described above (a list of blocks may be cut into two segments that are
    // sliced differently).  `ws0`: number of this segment's first block among all sliced blocks.
    int32_t slices, t0, ws0;
    // kSegTri, level 0, XOR family with c >= 8: the c^2 blocks are enumerated in groups of 32,
    // (i / 8, j / 4) outermost and (i % 8, j % 4) inside a group.  The blocks of a group lie on 28 tile
    // rows instead of 128 (j: 4 values; i, i XOR j and i XOR x j: 8 values each, because the low three
    // bits form a subspace that contains {0, 1, x, x + 1} and x times it): a group is a triangle block
    // one level up in the sense of Section 5.1, for a fast memory shared by 32 compute units.
    int32_t group;
    // kSegTri, level 0: every block takes two tiles of the diagonal zones with it (item kind kAug)
    int32_t aug;
};

struct Plan {
    int32_t k;
    int32_t T;                  // tile rows of the whole matrix
    int32_t nseg;
    int32_t n_items;
    int32_t c[kMaxLevels];      // modulus of each level that has triangle blocks
    int32_t fam[kMaxLevels];    // 0: cyclic family; m > 0: the XOR family with c = 2^m
    int32_t team_items;         // the first team_items items (a multiple of 32, whole groups of segment 0)
                                // are handed out group by group to the workgroups of one die (0: none)
    int32_t n_ws_blocks;        // sliced blocks (each owns a stretch of the workspace)
    int32_t ws_slices;          // largest `slices` of any segment (the workspace stride per block)
    Seg seg[kMaxSegs];
};

struct Item {
    int32_t kind;
    int32_t nrow;               // triangle block: members of R; rectangle: row-side tile rows
    int32_t ncol;               // rectangle: column-side tile rows; otherwise 0
    // tile rows, -1 = unused.  Triangle block: R in zone order in slots 0..k-1.  Rectangle: column
    // side in slots 0..2, row side in slots 3..4.  Diagonal tile: slot 0.
    // Augmented triangle block: slots 4 and 5 are the further rows of its two extra tiles.
    int32_t rows[kMaxPanels];
    // kAug: which tiles the extra panels form.  aug1 = 6: (rows[4], rows[0]), 7: (rows[4], rows[1]);
    // aug2 = 8: (rows[5], rows[2]), 9: (rows[2], rows[5]), 10: (rows[5], rows[3]), 11: (rows[3], rows[5])
    // (row, column of the tile; equal rows: the diagonal tile, of which the lower part belongs to the block).
    int32_t aug1, aug2;
    int32_t slice, slices;      // this item is part `slice` of `slices` of its block (0 of 1: the whole block)
    int32_t ws_block;           // sliced blocks: which stretch of the workspace
};

// first tile row of zone z of a level: the zone is reached by choosing digit d_m at level m
TBS_HD int32_t zone_base(const Plan& p, int32_t level, int32_t z)
{
    int32_t base = 0;
    for (int32_t m = level - 1; m >= 0; --m) {
        base += (z % kK) * p.c[m];
        z /= kK;
    }
    return base;
}

TBS_HD void tbs_decode(const Plan& p, int32_t id, Item& it)
{
    it.kind = kEmpty;
    it.nrow = 0;
    it.ncol = 0;
    it.slice = 0;
    it.slices = 1;
    it.ws_block = -1;
    it.aug1 = it.aug2 = 0;
    for (int s = 0; s < kMaxPanels; ++s) it.rows[s] = -1;
    int32_t si = 0;
    while (si + 1 < p.nseg && id >= p.seg[si + 1].first) ++si;
    const Seg& sg = p.seg[si];
    const int32_t item = id - sg.first;
    if (item < 0 || item >= sg.count) return;
    const int32_t S = sg.slices > 1 ? sg.slices : 1;
    const int32_t blk = item / S;
    it.slice = item - blk * S;
    it.slices = S;
    if (S > 1) it.ws_block = sg.ws0 + blk;
    const int32_t t = sg.t0 + blk;
    if (sg.kind == kSegTri) {
        const int32_t c = p.c[sg.level];
        const int32_t z = t / (c * c);
        const int32_t ij = t - z * c * c;
        int32_t i = ij / c, j = ij - i * c;
        if (sg.group) {                             // groups of 32 blocks that share tile rows
            const int32_t g = ij >> 5, q = ij & 31, per_row = c >> 2;
            const int32_t gi = g / per_row, gj = g - gi * per_row;
            i = gi * 8 + (q >> 2);
            j = gj * 4 + (q & 3);
        }
        const int32_t base = zone_base(p, sg.level, z);
        it.kind = kTri;
        it.nrow = kK;
        it.rows[0] = base + j;
        const int32_t m = p.fam[sg.level];
        if (m == 0) {
            int32_t f = i;                          // f(1) = i, f(u+1) = f(u) + j mod c
            for (int32_t u = 1; u < kK; ++u) {
                it.rows[u] = base + u * c + f;
                f += j;
                if (f >= c) f -= c;
            }
        } else {                                    // f(u) = i XOR (j * a_u), a = 0, 1, x
            static_assert(kK == 4, "the XOR family is written out for k = 4");
            const int32_t xj = ((j << 1) ^ ((j >> (m - 1)) ? 3 : 0)) & (c - 1);
            it.rows[1] = base + c + i;
            it.rows[2] = base + 2 * c + (i ^ j);
            it.rows[3] = base + 3 * c + (i ^ xj);
        }
        if (sg.aug) {
            it.kind = kAug;
            if (i >= j) {                           // i = j: the diagonal tile of zone 0 (rows[4] = rows[0])
                it.rows[4] = base + i;
                it.aug1 = 6;
            } else {
                it.rows[4] = base + c + j;
                it.aug1 = 7;
            }
            int32_t zone = 2;                       // j = 0: the diagonal tile of zone 2 (rows[5] = rows[2])
            if (j != 0) {
                if (m == 0) {
                    zone = (2 * j < c) ? 2 : 3;
                } else {
                    int32_t hb = 0;
                    while ((j >> (hb + 1)) != 0) ++hb;
                    zone = ((i >> hb) & 1) ? 2 : 3;
                }
            }
            const int32_t f = ((zone == 2) ? it.rows[2] : it.rows[3]) - base - zone * c;   // (no indexing by a variable)
            int32_t other = f;
            if (j != 0) {
                if (m == 0) {
                    other = f + j;
                    if (other >= c) other -= c;
                } else {
                    other = f ^ j;
                }
            }
            it.rows[5] = base + zone * c + other;
            it.aug2 = (zone == 2) ? (other >= f ? 8 : 9) : (other > f ? 10 : 11);
        }
    } else if (sg.kind == kSegTriBase) {
        const int32_t base = zone_base(p, sg.level, t);
        it.kind = kTri;
        it.nrow = sg.r1;
        for (int32_t u = 0; u < kK; ++u)
            if (u < sg.r1) it.rows[u] = base + u;
    } else if (sg.kind == kSegRect) {
        const int32_t per_zone = sg.nI * sg.nJ;
        const int32_t z = t / per_zone;
        const int32_t rem = t - z * per_zone;
        const int32_t I = rem / sg.nJ, J = rem - I * sg.nJ;
        const int32_t base = zone_base(p, sg.level, z);
        const int32_t ra = sg.r0 + I * sg.mr;
        const int32_t rb = (ra + sg.mr < sg.r1) ? ra + sg.mr : sg.r1;
        const int32_t ca = sg.c0 + J * sg.nc;
        const int32_t cb = (ca + sg.nc < sg.c1) ? ca + sg.nc : sg.c1;
        if (ca > rb - 1 - (sg.diag ? 0 : 1)) return;   // no tile on the wanted side of the diagonal: empty
        it.kind = sg.diag ? kRectDiag : kRect;
        it.ncol = cb - ca;
        it.nrow = rb - ra;
        for (int32_t q = 0; q < kRectCols; ++q)
            if (q < it.ncol) it.rows[q] = base + ca + q;
        for (int32_t r = 0; r < kRectRows; ++r)
            if (r < it.nrow) it.rows[kRectCols + r] = base + ra + r;
    } else if (sg.kind == kSegDiagRun) {
        it.kind = kDiag;
        it.nrow = 1;
        it.rows[0] = sg.r0 + t;
    } else {
        it.kind = kDiag;
        it.nrow = 1;
        it.rows[0] = t;
    }
}

}  // namespace tbs
