// Host-side launch planning of the leaf-kernel library: which tiles a product runs on, how a
// grid is cut into launches, how MTTKRP and the streaming kernels split their index ranges, and
// how large the workspaces are.  Plain C++ with no HIP in it: the library includes it, and so
// does a host-only test program that is built with the address and undefined-behaviour
// sanitizers and fuzzes the extents.  Every plan is a function of the extents only, never of
// the device, so summation orders and results are reproducible across devices.
#pragma once
#include <stdint.h>

#include <limits>

#include "tile_map.hpp"

namespace distal {

constexpr int kInnerprodMaxBlocks = 2048;   // partial sums the inner product's workspace holds
// Workgroups of a streaming launch that gives each a contiguous range: one per compute unit of
// the part (256), which is what HBM serves fastest; a constant, so results do not depend on the device.
constexpr int kStreamBlocks = 256;
constexpr int64_t kComputeUnits = 256;

inline bool mul_ok(int64_t a, int64_t b, int64_t *out) { return !__builtin_mul_overflow(a, b, out); }

// ---- streaming kernels: contiguous index ranges per workgroup ---------------------------------
// n items over at most max_blocks workgroups of at least min_per items each: workgroup b owns
// [b * per, min((b + 1) * per, n)), per a multiple of `granule`; no range is empty.
struct RangeSplit { int64_t per, blocks; };

inline RangeSplit split_ranges(int64_t n, int64_t max_blocks, int64_t min_per, int64_t granule) {
    if (n <= 0) return RangeSplit{granule, 0};
    int64_t blocks = (n - 1) / min_per + 1;
    if (blocks > max_blocks) blocks = max_blocks;
    int64_t per = (n - 1) / blocks + 1;
    per = ((per - 1) / granule + 1) * granule;
    return RangeSplit{per, (n - 1) / per + 1};
}

// ---- matrix products: tile choice and the cut into two launches ------------------------------
struct TilePick { int id, bm, bn, bk; double cost; };

// (How many wavefronts share a tile follows from the tile and the size of the grid, see
// launch_by_id; the figures below are measured with that rule in place.)
// A tile shape the straight-line kernels exist for, with its measured efficiency (fraction of
// the MFMA peak of the dtype) on grids that give every compute unit exactly J tiles, for
// J = 1, 2, 3, 4, 8 and 16 or more (aligned products, K = 2048; 4096 for the deep binary64 tile).
// Few tiles per compute unit mean few wavefronts per SIMD and less overlap of one tile's
// prologue and epilogue with another's k-loop, and how much that costs differs by tile: a
// 256 x 256 binary32 tile brings its own four wavefronts per SIMD and loses 1 %, a 64 x 64 one
// alone on a compute unit runs at 60 % of its large-grid speed.
struct TileCandidate { int id; bool eligible; int bm, bn, bk; double eff[6]; };

constexpr int kMaxTileCandidates = 12;

// efficiencies of a narrow tile from one large-grid figure (what a rank-sized product of the
// tensor-times-matrix shapes reaches with it): the small-grid entries follow the 128 x 128
// tile's curve
inline void narrow_eff(TileCandidate &c, double large) {
    const double shape[6] = {0.82, 0.92, 0.96, 0.98, 0.99, 1.0};
    for (int i = 0; i < 6; ++i) c.eff[i] = large * shape[i];
}

inline int tile_candidates(bool f64, bool ta, int64_t M, int64_t N, int64_t K, TileCandidate (&c)[kMaxTileCandidates],
                           bool acc = false) {
    // tiles with a 32-wide (or, in binary32, 64-wide) short side only for an output that is that
    // narrow (rank-sized N, or M under TA)
    const bool n32 = N <= 32, n64 = N <= 64, m32 = M <= 32, m64 = M <= 64;
    (void)ta;
    if (!f64) {
        // added onto an old C the largest tile pays from deeper products on: its one workgroup per
        // compute unit has nothing to overlap the read-modify-write of its 256 KiB of C with
        // (8192 x 8192 x 1024 under accumulate: 82.8 % of peak, 256 x 128 tiles 85.7 %)
        // (the two largest tiles measure within half a point of each other on large grids, 95.1 and
        // 95.0 % at 8192^3: they carry the same last entry, and the larger one, listed first, wins the tie)
        c[0] = {1, K >= (acc ? 4096 : 1024), 256, 256, ta ? 16 : 32, {0.927, 0.931, 0.933, 0.934, 0.940, 0.945}};
        c[1] = {2, K >= (acc ? 512 : 256), 256, 128, 16, {0.882, 0.923, 0.932, 0.938, 0.943, 0.945}};
        // a product of at most 256 terms added onto an old C is bound by the traffic of C: tiles with
        // 128 columns and 64 rows (512-byte runs of C, four workgroups per compute unit) then measure
        // 4..5 points ahead of 128 x 128 and of 128 x 64
        const bool thin_acc = acc && K <= 256;
        c[2] = {3, !thin_acc, 128, 128, 16, {0.843, 0.906, 0.919, 0.927, 0.939, 0.950}};
        c[3] = {4, K < 256, 64, 64, 16, {0.628, 0.759, 0.806, 0.829, 0.835, 0.852}};
        c[4] = {9, !thin_acc && K >= 32, 128, 64, 32, {0.754, 0.849, 0.864, 0.888, 0.889, 0.911}};
        c[5] = {10, K >= 32, 64, 128, 32, {0.732, 0.842, 0.881, 0.877, 0.888, 0.911}};
        // (128 x 128, 128 x 64, 64 x 128 and the 32-deep 64 x 64 run on the 16 x 16 x 4 instruction, eight
        // wavefronts each; see launch_by_id)
        // 64 x 64 with 32-deep slabs: half the barriers per term; pays from K = 256 on (binary32 only:
        // the same in binary64 measured 3..9 % slower)
        c[6] = {11, K >= 256, 64, 64, 32, {0.699, 0.808, 0.844, 0.841, 0.854, 0.867}};
        c[7] = {5, n64, 256, 64, 16, {}};
        c[8] = {6, n32 && K >= 32, 128, 32, 32, {}};
        c[9] = {7, m64, 64, 256, 16, {}};
        c[10] = {8, m32 && K >= 32, 32, 256, 32, {}};
        narrow_eff(c[7], 0.891); narrow_eff(c[8], 0.575); narrow_eff(c[9], 0.883); narrow_eff(c[10], 0.585);
        // 128 x 256: two workgroups per compute unit like 256 x 128, with 1 KiB rows of the right operand
        // and of C; 0.5 to 1.7 points ahead of it at every depth from 128 to 8192 (8192^3: 96.3 against 95.8),
        // level with 128 x 128 on large grids and ahead of it at two tiles per compute unit (4096^3)
        c[11] = {12, K >= (acc ? 512 : 128), 128, 256, 16, {0.905, 0.933, 0.937, 0.945, 0.946, 0.948}};
        return 12;
    }
    c[0] = {2, K >= 2048, 256, 128, 16, {0.877, 0.938, 0.938, 0.938, 0.939, 0.940}};
    // a step of at most 128 terms added onto an old C is bound by C's traffic: 64 x 128 tiles measure
    // 65.2 % of peak at 8192 x 8192 x 128 against 62.4 on 128 x 128
    const bool thin_acc64 = acc && K <= 128;
    c[1] = {3, !thin_acc64, 128, 128, 16, {0.901, 0.935, 0.937, 0.941, 0.949, 0.954}};
    c[2] = {4, true, 64, 64, 16, {0.796, 0.854, 0.889, 0.883, 0.917, 0.909}};
    c[3] = {5, true, 128, 64, 16, {0.818, 0.898, 0.905, 0.911, 0.919, 0.930}};
    c[4] = {7, true, 64, 128, 16, {0.841, 0.902, 0.908, 0.925, 0.941, 0.939}};
    c[5] = {6, n32, 128, 32, 16, {}};
    c[6] = {8, m32, 32, 256, 16, {}};
    narrow_eff(c[5], 0.633); narrow_eff(c[6], 0.560);
    return 7;
}

// Estimated time of a grid, in units of tile area: the most loaded compute unit works
// J = ceil(tiles / 256) tiles at the efficiency measured for J tiles per compute unit
// (interpolated between the measured J; padding counts through the tile count).
inline double rounds_cost(int64_t tiles, const TileCandidate &c) {
    const int64_t J = (tiles + kComputeUnits - 1) / kComputeUnits;
    double e;
    if (J <= 4) e = c.eff[J < 1 ? 0 : J - 1];
    else if (J < 8) e = c.eff[3] + (c.eff[4] - c.eff[3]) * (double)(J - 4) / 4.0;
    else if (J < 16) e = c.eff[4] + (c.eff[5] - c.eff[4]) * (double)(J - 8) / 8.0;
    else e = c.eff[5];
    return (double)J * (double)(c.bm * c.bn) / e;
}

// The tile with the least estimated time for a product run as one launch.
inline TilePick pick_tile(bool f64, bool ta, int64_t M, int64_t N, int64_t K, int64_t batch, bool acc = false) {
    TileCandidate cand[kMaxTileCandidates];
    const int n = tile_candidates(f64, ta, M, N, K, cand, acc);
    TilePick pick{4, 64, 64, 16, 1e300};
    for (int i = 0; i < n; ++i) {
        if (!cand[i].eligible) continue;
        const int64_t tm = (M + cand[i].bm - 1) / cand[i].bm, tn = (N + cand[i].bn - 1) / cand[i].bn;
        const double c = rounds_cost(tm * tn * batch, cand[i]);
        if (c < pick.cost) pick = TilePick{cand[i].id, cand[i].bm, cand[i].bn, cand[i].bk, c};   // earlier candidates win ties
    }
    return pick;
}

// A product as at most two launches: the leading rows (or columns) of the output - a whole
// number of tile rows (columns) whose tiles fill whole rounds of the compute units - with
// `main`, and what remains, if anything, with the tile that suits it alone; so the part of a
// grid that would be a thin last round of large tiles runs as a round of small ones.
// split = 0: one launch; 1: rows [0, cut) and [cut, M); 2: columns [0, cut) and [cut, N).
struct ProductPlan { TilePick main; int split; int64_t cut; TilePick rest; };

inline ProductPlan plan_product(bool f64, bool ta, int64_t M, int64_t N, int64_t K, int64_t batch, bool acc = false) {
    ProductPlan plan{pick_tile(f64, ta, M, N, K, batch, acc), 0, 0, TilePick{0, 0, 0, 0, 0.0}};
    // a second launch costs about 3 us of an otherwise busy part: in units of tile area
    const double launch_cost = 3e-6 * (f64 ? 78.6e12 : 157.3e12) / (double)kComputeUnits / (2.0 * (double)K);
    TileCandidate cand[kMaxTileCandidates];
    const int n = tile_candidates(f64, ta, M, N, K, cand, acc);
    double best = plan.main.cost;
    for (int i = 0; i < n; ++i) {
        if (!cand[i].eligible) continue;
        const TileCandidate &c = cand[i];
        const int64_t tm = (M + c.bm - 1) / c.bm, tn = (N + c.bn - 1) / c.bn;
        const int64_t whole = tm * tn * batch / kComputeUnits * kComputeUnits;     // tiles inside whole rounds
        for (int split = 1; split <= 2; ++split) {
            const int64_t per_line = (split == 1 ? tn : tm) * batch;               // tiles per row (column) of tiles
            const int64_t lines = whole / per_line, cut = lines * (split == 1 ? c.bm : c.bn);
            if (lines < 1 || cut >= (split == 1 ? M : N)) continue;
            const TilePick rest = split == 1 ? pick_tile(f64, ta, M - cut, N, K, batch, acc)
                                             : pick_tile(f64, ta, M, N - cut, K, batch, acc);
            const double total = rounds_cost(lines * per_line, c) + rest.cost + launch_cost;
            if (total < 0.985 * best) {                                             // worth a second launch
                best = total / 0.985;
                plan = ProductPlan{TilePick{c.id, c.bm, c.bn, c.bk, total}, split, cut, rest};
            }
        }
    }
    return plan;
}

// Rows of the right operand that do not end on a 16-byte piece (N not a multiple of 16 / element
// size).  The straight-line kernels can take such rows as they are - the last piece is fetched one
// vector before the end of the row and shifted in registers, about 3 % on the whole launch, and
// N counts with its padding to whole tiles - or the trailing N mod vector columns are peeled off
// to a streaming kernel that reads the left operand once more (about 4.5 TB/s) while the rest
// runs on a whole number of pieces.  Returns the number of columns to peel: the cheaper of the two
// by the estimates of plan_product (a narrow output, where the second pass over the left operand
// doubles the time, stays whole; a wide one, where that pass is a percent, is peeled); all N columns
// when N is narrower than one piece.  A function of the extents only.
inline int64_t peeled_columns(bool f64, bool ta, int64_t M, int64_t N, int64_t K, int64_t batch, bool acc = false) {
    const int64_t vec = f64 ? 2 : 4;
    if (N % vec == 0) return 0;
    if (N < vec) return N;
    const double per_cu = (f64 ? 78.6e12 : 157.3e12) / (double)kComputeUnits, esz = f64 ? 8.0 : 4.0;
    const double whole = 1.03 * plan_product(f64, ta, M, N, K, batch, acc).main.cost;
    // the second pass in units of tile area, as the costs of plan_product are: seconds x rate / (2 K)
    const double pass = ((double)M * (double)K * (double)batch * esz / 4.5e12 + 3e-6) * per_cu / (2.0 * (double)K);
    const double peeled = plan_product(f64, ta, M, N - N % vec, K, batch, acc).main.cost + pass;
    return peeled < whole ? N % vec : 0;
}

// A product with a small output and a long contracted index gives fewer tiles than the part has
// compute units, however the tiles are chosen.  With scratch memory from the caller such a product
// is cut along k into `parts` products of `kchunk` terms each (the last one shorter), run as one
// batch into `parts` M x N slabs of the scratch, which a second kernel adds up in the order of k.
// The number of parts is the one with the least estimated time among a fixed list: the batch on
// the tile the table picks for it, plus the second kernel's traffic over the slabs at 5 TB/s, plus
// 3 us per launch; the product is cut only where that beats the single launch by a tenth.
// parts == 1: not cut (also whenever at least half the compute units have a tile already, or
// the parts would be shallower than 1024 terms).  kchunk is a multiple of 32, so every part keeps
// the alignment of the whole.  A function of the extents only.
struct SplitKPlan { int64_t parts, kchunk; };

inline SplitKPlan plan_split_k(bool f64, int64_t M, int64_t N, int64_t K) {
    SplitKPlan best{1, K};
    if (M <= 0 || N <= 0 || K < 2048) return best;
    const TilePick whole = pick_tile(f64, false, M, N, K, 1);
    int64_t tiles, outs;
    if (!mul_ok((M + whole.bm - 1) / whole.bm, (N + whole.bn - 1) / whole.bn, &tiles) || tiles > kComputeUnits / 2) return best;
    if (!mul_ok(M, N, &outs) || outs > ((int64_t)1 << 40)) return best;
    const double per_cu = (f64 ? 78.6e12 : 157.3e12) / (double)kComputeUnits, esz = f64 ? 8.0 : 4.0;
    auto seconds = [&](double cost, int64_t depth) { return cost * 2.0 * (double)depth / per_cu; };
    double best_time = seconds(whole.cost, K) * 0.9;
    const int options[] = {2, 3, 4, 6, 8, 12, 16, 24, 32, 48, 64};
    for (int want : options) {
        if (want > K / 1024) break;
        const int64_t kchunk = ((K + want - 1) / want + 31) / 32 * 32;
        const int64_t parts = (K + kchunk - 1) / kchunk;
        if (parts < 2) continue;
        const TilePick t = pick_tile(f64, false, M, N, kchunk, parts);
        const double time = seconds(t.cost, kchunk) + (double)(parts + 1) * (double)outs * esz / 5e12 + 2 * 3e-6;
        if (time < best_time) { best_time = time; best = SplitKPlan{parts, kchunk}; }
    }
    return best;
}

// Whether unsigned 32-bit byte offsets from a tile's first element reach every 16-byte piece of
// one slab of it: the straight-line contraction kernels address a slab that way (the slab's base
// is a 64-bit scalar).  The farthest piece starts at (rows of the slab - 1) x leading dimension +
// row length - one vector; the bound leaves the whole last row below 2^32 - 64.  Operands whose
// rows lie farther apart run the pointer-addressed kernel.
inline bool slab_offsets_fit(int64_t esz, bool ta, int bm, int bn, int bk, int64_t lda, int64_t ldb) {
    const int64_t limit = ((int64_t)1 << 32) - 64;
    const int64_t a_rows = ta ? bk : bm, a_len = ta ? bm : bk;
    int64_t a, b;
    if (lda < 0 || ldb < 0) return false;
    if (!mul_ok(a_rows - 1, lda, &a) || !mul_ok(bk - 1, ldb, &b)) return false;
    if (a > limit || b > limit) return false;                    // before the next products can overflow
    return (a + a_len) * esz < limit && (b + bn) * esz < limit;
}

// ---- TTM over the last mode with a rank-sized factor -------------------------------------------
// Slices of the factor per wavefront (1, 2, 3 or 4) for the kernel that keeps the whole factor in the
// registers of a workgroup's eight wavefronts, or 0 where the tiled contraction runs instead:
// at most 32 columns, rows of the tensor that are whole 16-byte pieces and at most 8 x 4 slices
// of 256 bytes long, at least seven eighths of the wavefronts' slices in use, and enough blocks
// of 32 rows to give every compute unit eight.  Three and four slices per wavefront only for
// exactly 24 or 32 slices: the forms for a short last slice spill there and are not built.  (Rows
// beyond a whole number of blocks of 32 are no obstacle: with whole slices the last R mod 32 rows
// run as a small tiled product of their own.)
// A function of the extents only.
inline int ttm_slices_per_wave(bool f64, int64_t R, int64_t K, int64_t L) {
    const int64_t vec = f64 ? 2 : 4, sl = f64 ? 32 : 64;
    if (L < 1 || L > 32 || K < 1 || K % vec != 0 || R < (int64_t)32 * kComputeUnits * 8) return 0;
    const int64_t nslices = (K + sl - 1) / sl;
    const int ns = nslices <= 8 ? 1 : nslices <= 16 ? 2 : nslices <= 24 ? 3 : nslices <= 32 ? 4 : 0;
    if (ns == 0 || nslices * 8 < (int64_t)8 * ns * 7) return 0;
    if (ns >= 3 && K != 8 * ns * sl) return 0;                    // the ragged forms of three and four slices spill
    return ns;
}

// ---- MTTKRP: ranges of the walked index and partial rows --------------------------------------
constexpr int64_t kModeTargetBlocks = 768;

struct MttkrpModePlan {
    int64_t tasks;          // workgroups per range of the walked index
    int64_t isplit, nsplit; // walked indices per range; ranges (none empty)
    int64_t nparts;         // partial rows per output row
    int64_t partial_elems;  // workspace elements (0 when nparts == 1)
    int64_t nslices, spw, kgroups, rblocks /* blocks of 32 output rows */, rgroups, jgroups, kblocks, tiles_n;
    bool ok;
};

inline MttkrpModePlan mttkrp_mode_plan(int dt, int mode, int64_t I, int64_t J, int64_t K, int64_t L) {
    MttkrpModePlan p{};
    const int64_t esz = dt == 1 /* binary64 */ ? 8 : 4;
    // a wavefront takes two column tiles of 32 once the rank exceeds 32
    p.tiles_n = L > 32 ? (L + 63) / 64 : (L + 31) / 32;
    int64_t out_rows, per_split;
    if (mode != 2) {                       // kept index r = i (mode 0) or j (mode 1), the other one is walked
        const int64_t sl = 256 / esz;
        out_rows = mode == 0 ? I : J;
        p.nslices = (K + sl - 1) / sl;
        // four k-slices per workgroup, one per wavefront; a short K gives a workgroup fewer slices
        // and its other wavefronts further blocks of output rows instead
        p.spw = p.nslices >= 3 ? 4 : p.nslices;
        p.kgroups = (p.nslices + p.spw - 1) / p.spw;
        p.rblocks = (out_rows + 31) / 32;
        p.rgroups = (p.rblocks + 4 / p.spw - 1) / (4 / p.spw);
        p.ok = mul_ok(p.kgroups * p.tiles_n, p.rgroups, &p.tasks);
        per_split = p.nslices;
    } else {
        const int64_t kw = 512 / esz;
        p.kblocks = (K + kw - 1) / kw;
        p.jgroups = (J + 63) / 64;
        p.ok = mul_ok(p.kblocks * p.tiles_n, p.jgroups, &p.tasks);
        per_split = p.jgroups;
        out_rows = K;
    }
    if (!p.ok || p.tasks < 1) { p.ok = false; return p; }
    const int64_t walked = mode == 0 ? J : I;                 // the index each workgroup walks a range of
    int64_t want = (kModeTargetBlocks + p.tasks - 1) / p.tasks;
    if (want > walked) want = walked;
    if (want < 1) want = 1;
    p.isplit = (walked + want - 1) / want;
    p.nsplit = (walked + p.isplit - 1) / p.isplit;
    int64_t rows;
    p.ok = mul_ok(p.nsplit, per_split, &p.nparts) && mul_ok(out_rows, p.nparts, &rows) &&
           mul_ok(rows, L, &p.partial_elems) && p.partial_elems <= INT64_MAX / 16 &&
           p.nparts <= std::numeric_limits<int>::max();
    int64_t nblocks;
    p.ok = p.ok && mul_ok(p.tasks, p.nsplit, &nblocks) && nblocks <= std::numeric_limits<int>::max();
    if (p.nparts <= 1) p.partial_elems = 0;
    return p;
}

}  // namespace distal
