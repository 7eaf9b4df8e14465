// Host-only check of the library's launch planning (csrc/host_plan.hpp, csrc/tile_map.hpp),
// built by tests/test_host_sanitizers.py with g++ -fsanitize=address,undefined and run without
// a GPU.  Extents are fuzzed, including ones close to the limits the entry points accept; every
// failed property prints a line and the program exits non-zero.
#include <cinttypes>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../paper_2203_08069_amd/csrc/host_plan.hpp"

using namespace distal;

static int failures = 0;
#define CHECK(cond, ...) do { if (!(cond)) { if (++failures <= 20) { printf("FAIL %s:%d %s | ", __FILE__, __LINE__, #cond); printf(__VA_ARGS__); printf("\n"); } } } while (0)

static uint64_t rng_state = 0x243F6A8885A308D3ull;
static uint64_t rnd() {                       // xorshift64*
    rng_state ^= rng_state >> 12; rng_state ^= rng_state << 25; rng_state ^= rng_state >> 27;
    return rng_state * 0x2545F4914F6CDD1Dull;
}
// an extent in [1, hi], log-uniform so that small and huge values both occur
static int64_t extent(int64_t hi) {
    int bits = 1; while (bits < 62 && ((int64_t)1 << bits) <= hi) ++bits;
    const int b = 1 + (int)(rnd() % bits);
    int64_t v = (int64_t)(rnd() & (((uint64_t)1 << b) - 1)) + 1;
    return v > hi ? hi : v;
}

template <int G>
static void check_tile_map(int tiles_m, int tiles_n) {
    const int n = tiles_m * tiles_n;
    std::vector<unsigned char> seen((size_t)n, 0);
    for (int b = 0; b < n; ++b) {
        int tm = -1, tn = -1;
        tile_of_block<G>(b, n, tiles_m, tiles_n, tm, tn);
        CHECK(tm >= 0 && tm < tiles_m && tn >= 0 && tn < tiles_n, "G=%d grid %dx%d block %d -> (%d,%d)", G, tiles_m, tiles_n, b, tm, tn);
        if (tm < 0 || tm >= tiles_m || tn < 0 || tn >= tiles_n) return;
        CHECK(!seen[(size_t)tm * tiles_n + tn], "G=%d grid %dx%d tile (%d,%d) twice", G, tiles_m, tiles_n, tm, tn);
        seen[(size_t)tm * tiles_n + tn] = 1;
    }
}

static bool known_tile(bool f64, bool ta, int64_t M, int64_t N, int64_t K, const TilePick &t) {
    TileCandidate c[kMaxTileCandidates];
    const int n = tile_candidates(f64, ta, M, N, K, c);
    for (int i = 0; i < n; ++i)
        if (c[i].eligible && c[i].id == t.id) return c[i].bm == t.bm && c[i].bn == t.bn && c[i].bk == t.bk;
    return false;
}

static void check_product(bool f64, bool ta, int64_t M, int64_t N, int64_t K, int64_t batch) {
    const ProductPlan p = plan_product(f64, ta, M, N, K, batch);
    CHECK(known_tile(f64, ta, M, N, K, p.main), "main tile of %" PRId64 "x%" PRId64 "x%" PRId64, M, N, K);
    CHECK(p.main.cost > 0 && p.main.cost < 1e300, "cost");
    CHECK(p.split >= 0 && p.split <= 2, "split %d", p.split);
    if (p.split == 0) return;
    const int64_t ext = p.split == 1 ? M : N, unit = p.split == 1 ? p.main.bm : p.main.bn;
    CHECK(p.cut > 0 && p.cut < ext && p.cut % unit == 0 && p.cut % 32 == 0, "cut %" PRId64 " of %" PRId64, p.cut, ext);
    // the first launch is whole rounds of the compute units
    const int64_t lines = p.cut / unit, per_line = (p.split == 1 ? (N + p.main.bn - 1) / p.main.bn : (M + p.main.bm - 1) / p.main.bm) * batch;
    CHECK(lines * per_line <= ((M + p.main.bm - 1) / p.main.bm) * ((N + p.main.bn - 1) / p.main.bn) * batch, "first launch larger than the grid");
    const int64_t rm = p.split == 1 ? M - p.cut : M, rn = p.split == 2 ? N - p.cut : N;
    CHECK(known_tile(f64, ta, rm, rn, K, p.rest), "rest tile of %" PRId64 "x%" PRId64, rm, rn);
}

static void check_mttkrp(int dt, int mode, int64_t I, int64_t J, int64_t K, int64_t L) {
    const MttkrpModePlan p = mttkrp_mode_plan(dt, mode, I, J, K, L);
    if (!p.ok) return;
    const int64_t walked = mode == 0 ? J : I, out_rows = mode == 0 ? I : (mode == 1 ? J : K);
    CHECK(p.isplit >= 1 && p.nsplit >= 1, "split");
    // the ranges [s*isplit, min((s+1)*isplit, walked)) tile the walked index, none empty
    CHECK((p.nsplit - 1) * p.isplit < walked && walked <= p.nsplit * p.isplit, "ranges %" PRId64 " x %" PRId64 " over %" PRId64, p.nsplit, p.isplit, walked);
    CHECK(p.tasks >= 1 && p.tasks * p.nsplit <= std::numeric_limits<int>::max(), "grid");
    const int64_t per_split = mode == 2 ? p.jgroups : p.nslices;
    CHECK(p.nparts == p.nsplit * per_split, "nparts");
    // the last partial row a workgroup can write: row (out_rows-1) * nparts + (nparts-1), L values
    if (p.nparts > 1) {
        const int64_t last = ((out_rows - 1) * p.nparts + (p.nparts - 1)) * L + (L - 1);
        CHECK(last < p.partial_elems, "partial index %" PRId64 " >= %" PRId64, last, p.partial_elems);
        CHECK(p.partial_elems <= INT64_MAX / 16, "workspace bytes overflow");
    } else {
        CHECK(p.partial_elems == 0, "no workspace for one partial row");
    }
    if (mode != 2) {
        const int64_t sl = dt == 1 ? 32 : 64;
        CHECK(p.nslices * sl >= K && (p.nslices - 1) * sl < K, "k-slices");
        CHECK(p.spw == 1 || p.spw == 2 || p.spw == 4, "spw");
        CHECK(p.kgroups * p.spw >= p.nslices, "k-groups");
        CHECK(p.rblocks * 32 >= out_rows && (p.rblocks - 1) * 32 < out_rows, "row blocks");
        CHECK(p.rgroups * (4 / p.spw) >= p.rblocks, "row groups");
        CHECK(p.tasks == p.kgroups * p.tiles_n * p.rgroups, "tasks");
    } else {
        const int64_t kw = dt == 1 ? 64 : 128;
        CHECK(p.kblocks * kw >= K && (p.kblocks - 1) * kw < K, "k-blocks");
        CHECK(p.jgroups * 64 >= J && (p.jgroups - 1) * 64 < J, "j-groups");
        CHECK(p.tasks == p.kblocks * p.tiles_n * p.jgroups, "tasks");
    }
    CHECK(p.tiles_n * (L > 32 ? 64 : 32) >= L, "column tiles");
}

static void check_ranges(int64_t n, int64_t max_blocks, int64_t min_per, int64_t granule) {
    const RangeSplit r = split_ranges(n, max_blocks, min_per, granule);
    CHECK(r.blocks >= 1 && r.blocks <= max_blocks, "blocks %" PRId64, r.blocks);
    CHECK(r.per >= 1 && r.per % granule == 0, "per %" PRId64, r.per);
    CHECK((r.blocks - 1) * r.per < n && n - (r.blocks - 1) * r.per <= r.per, "ranges %" PRId64 " x %" PRId64 " over %" PRId64, r.blocks, r.per, n);
}

int main() {
    // the block-id -> tile map is a bijection on every grid
    for (int tm = 1; tm <= 40; ++tm)
        for (int tn = 1; tn <= 40; ++tn) { check_tile_map<4>(tm, tn); check_tile_map<8>(tm, tn); }
    for (int it = 0; it < 60; ++it) {
        const int tm = (int)extent(3000), tn = (int)extent(700);
        check_tile_map<4>(tm, tn); check_tile_map<8>(tm, tn);
    }
    check_tile_map<8>(1, 1 << 21); check_tile_map<4>(1 << 21, 1); check_tile_map<8>(32768, 64);

    // products: whatever passes the entry point's own limits (at most 2^31-1 tiles of 128 x 128,
    // at most 2^60 outputs over the batch)
    for (int it = 0; it < 200000; ++it) {
        const bool f64 = rnd() & 1, ta = rnd() & 2;
        int64_t M = extent((int64_t)1 << 40), N = extent((int64_t)1 << 40);
        const int64_t K = extent((int64_t)1 << 40);
        int64_t batch = (rnd() & 3) ? 1 : extent(65535 * 4);
        int64_t tiles, outs;
        if (!mul_ok((M + 127) / 128, (N + 127) / 128, &tiles) || tiles > std::numeric_limits<int>::max()) { N = 1 + N % 4096; M = 1 + M % ((int64_t)1 << 30); }
        if (!mul_ok(M, N, &outs) || outs > ((int64_t)1 << 60) / batch) batch = 1;
        check_product(f64, ta, M, N, K, batch);
    }
    const int64_t shapes[][3] = {{8192, 8192, 8192}, {8200, 8192, 8192}, {8192, 8200, 8192}, {3000, 3000, 3000}, {1 << 20, 256, 1024},
                                 {1 << 20, 32, 1024}, {32, 1 << 20, 1024}, {1, 1, 16}, {INT32_MAX, 128, 16}, {128, (int64_t)INT32_MAX * 128, 16}};
    for (auto &s : shapes)
        for (int f = 0; f < 4; ++f) check_product(f & 1, f & 2, s[0], s[1], s[2], 1);

    // 32-bit slab offsets: whenever the predicate accepts leading dimensions, the farthest byte a
    // lane of the straight-line kernel can touch (computed in 128 bits) lies below 2^32; and it
    // does accept every operand whose tile spans less than 2 GiB
    for (int it = 0; it < 400000; ++it) {
        const int64_t esz = (rnd() & 1) ? 8 : 4;
        const bool ta = rnd() & 1;
        const int bms[] = {32, 64, 128, 256}, bks[] = {16, 32};
        const int bm = bms[rnd() % 4], bn = bms[rnd() % 4], bk = bks[rnd() % 2];
        const int64_t lda = (rnd() % 8 == 0) ? (int64_t)(rnd() >> 1) : extent((int64_t)1 << 36);
        const int64_t ldb = (rnd() % 8 == 0) ? (int64_t)(rnd() >> 1) : extent((int64_t)1 << 36);
        const bool fit = slab_offsets_fit(esz, ta, bm, bn, bk, lda, ldb);
        const unsigned __int128 a_end = ((unsigned __int128)((ta ? bk : bm) - 1) * (unsigned __int128)lda + (ta ? bm : bk)) * esz;
        const unsigned __int128 b_end = ((unsigned __int128)(bk - 1) * (unsigned __int128)ldb + bn) * esz;
        const unsigned __int128 top = (unsigned __int128)1 << 32;
        if (fit) CHECK(a_end < top && b_end < top, "offsets past 2^32 accepted: lda %" PRId64 " ldb %" PRId64, lda, ldb);
        if (a_end < top / 2 && b_end < top / 2) CHECK(fit, "small operand rejected: lda %" PRId64 " ldb %" PRId64, lda, ldb);
    }
    CHECK(slab_offsets_fit(4, false, 256, 128, 16, 4198400, 128), "rows 4.28e9 bytes apart fit");
    CHECK(!slab_offsets_fit(4, false, 256, 128, 16, 8396800, 128), "rows 8.5e9 bytes apart do not");
    CHECK(!slab_offsets_fit(8, true, 128, 128, 16, INT64_MAX, 128), "overflowing product");

    // cuts along k: the parts cover K exactly once, only the last may be shorter, every part keeps
    // 32-element alignment and at least 1024 terms, and there are at most 64 of them
    for (int it = 0; it < 300000; ++it) {
        const bool f64 = rnd() & 1;
        const int64_t M = extent((int64_t)1 << 24), N = extent((int64_t)1 << 24), K = extent((int64_t)1 << 40);
        const SplitKPlan p = plan_split_k(f64, M, N, K);
        CHECK(p.parts >= 1 && p.parts <= 64, "parts %" PRId64, p.parts);
        if (p.parts == 1) { CHECK(p.kchunk == K, "uncut product with a chunk"); continue; }
        CHECK(p.kchunk % 32 == 0 && p.kchunk >= 1024, "chunk %" PRId64, p.kchunk);
        CHECK((p.parts - 1) * p.kchunk < K && K <= p.parts * p.kchunk, "parts %" PRId64 " x %" PRId64 " against K %" PRId64, p.parts, p.kchunk, K);
        CHECK(((M + 63) / 64) * ((N + 63) / 64) >= 1 && K >= 2048, "cut of a shallow product");
    }
    CHECK(plan_split_k(true, 512, 512, 8192).parts == 8 && plan_split_k(true, 512, 512, 8192).kchunk == 1024, "512 x 512 x 8192");
    CHECK(plan_split_k(true, 1024, 1024, 8192).parts == 1, "a tile per compute unit is not cut");

    // trailing columns peeled off a product: none, the N mod vector, or all of a product narrower than a piece
    for (int it = 0; it < 300000; ++it) {
        const bool f64 = rnd() & 1, ta = rnd() & 1, acc = rnd() & 1;
        const int64_t vec = f64 ? 2 : 4;
        const int64_t M = extent((int64_t)1 << 24), N = extent((int64_t)1 << 24), K = extent((int64_t)1 << 30);
        const int64_t batch = 1 + (int64_t)(rnd() % 4) * (int64_t)(rnd() % 300);
        const int64_t c = peeled_columns(f64, ta, M, N, K, batch, acc);
        if (N % vec == 0) CHECK(c == 0, "whole pieces peeled: %" PRId64, c);
        else if (N < vec) CHECK(c == N, "narrower than a piece: %" PRId64 " of %" PRId64, c, N);
        else CHECK(c == 0 || c == N % vec, "peeled %" PRId64 " of N %" PRId64, c, N);
        CHECK(N - c == 0 || N - c >= vec, "what remains is narrower than a piece");
    }

    // where the last-mode TTM keeps its factor in registers: the slices fit the wavefronts and mostly fill them
    for (int it = 0; it < 300000; ++it) {
        const bool f64 = rnd() & 1;
        const int64_t vec = f64 ? 2 : 4, sl = f64 ? 32 : 64;
        const int64_t R = extent((int64_t)1 << 40), K = (rnd() & 3) ? extent(4096) : extent((int64_t)1 << 40), L = extent(40);
        const int ns = ttm_slices_per_wave(f64, R, K, L);
        CHECK(ns >= 0 && ns <= 4, "slices per wavefront %d", ns);
        if (ns == 0) continue;
        const int64_t nslices = (K + sl - 1) / sl;
        CHECK(L >= 1 && L <= 32 && K % vec == 0 && R >= 65536, "extents %" PRId64 " %" PRId64 " %" PRId64, R, K, L);
        CHECK(nslices <= 8 * ns && nslices * 8 >= 56 * ns, "%" PRId64 " slices on %d per wavefront", nslices, ns);
        CHECK(ns < 3 || K == 8 * ns * sl, "a short last slice with %d slices per wavefront", ns);
    }

    // MTTKRP plans: extents whose product stays below 2^60, as the entry point demands
    for (int it = 0; it < 300000; ++it) {
        const int dt = (int)(rnd() & 1), mode = (int)(rnd() % 3);
        int64_t I = extent((int64_t)1 << 40), J = extent((int64_t)1 << 40), K = extent((int64_t)1 << 40);
        const int64_t L = extent(4096);
        int64_t ij, ijk;
        while (!mul_ok(I, J, &ij) || !mul_ok(ij, K, &ijk) || ijk > ((int64_t)1 << 60)) { I = (I + 1) / 2; J = (J + 1) / 2; K = (K + 1) / 2; }
        check_mttkrp(dt, mode, I, J, K, L);
    }
    for (int mode = 0; mode < 3; ++mode)
        for (int dt = 0; dt < 2; ++dt) {
            check_mttkrp(dt, mode, 1024, 1024, 1024, 32);
            check_mttkrp(dt, mode, 1, 1, 1, 1);
            check_mttkrp(dt, mode, (int64_t)1 << 40, 1, 1 << 10, 33);
            check_mttkrp(dt, mode, 3, (int64_t)1 << 40, 5, 64);
            check_mttkrp(dt, mode, 7, 9, (int64_t)1 << 50, 4096);
        }

    // contiguous ranges of the streaming kernels
    for (int it = 0; it < 300000; ++it) {
        const int64_t n = extent(INT64_MAX / 8);
        const int kind = (int)(rnd() % 3);
        if (kind == 0) check_ranges(n, kStreamBlocks, 1, 4 * (1 << (rnd() % 3)));     // TTV rows
        else if (kind == 1) check_ranges(n, kStreamBlocks, 256, 256);                 // inner product, 16-byte pieces
        else check_ranges(n, kInnerprodMaxBlocks, 1024, 256);                         // inner product, elements
    }
    check_ranges(INT64_MAX / 8, kStreamBlocks, 1, 16);
    check_ranges(1, kStreamBlocks, 256, 256);
    CHECK(split_ranges(0, 256, 1, 4).blocks == 0, "empty");

    printf(failures ? "host_plan_check: %d failure(s)\n" : "host_plan_check: ok\n", failures);
    return failures ? 1 : 0;
}
