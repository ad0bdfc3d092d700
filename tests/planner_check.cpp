// Host check of the work maps in paper_2603_28845_amd/csrc/planner.hpp: for every supported width the launches'
// workgroup -> (tile, piece) maps are enumerated exactly as the launchers and kernels use them, and every tile
// (every piece of a split tile) must be owned exactly once, inside the matrix, with token ranges that tile the
// token axis.  Prints "ok <number of checks>" on success, the first failure otherwise.  Plain C++, no GPU.
#include <cstdio>
#include <cstdlib>
#include <set>
#include <utility>
#include <vector>
#include "../paper_2603_28845_amd/csrc/planner.hpp"

using namespace onecomp::plan;

static long n_checks = 0;
#define REQUIRE(cond, ...)                                   \
    do {                                                     \
        ++n_checks;                                          \
        if (!(cond)) {                                       \
            std::printf("FAILED %s: ", #cond);               \
            std::printf(__VA_ARGS__);                        \
            std::printf("\n");                               \
            std::exit(1);                                    \
        }                                                    \
    } while (0)

// the launcher's grid for the register-staged and fp32 kernels: chunk * 8 workgroups, v = (b % 8) * chunk + b / 8
static void check_simple_upper(int d_in, int ts) {
    const int n_t = int(cdiv(d_in, ts)), n_tiles = n_upper_tiles(n_t), chunk = int(cdiv(n_tiles, 8));
    std::set<std::pair<int, int>> seen;
    for (int b = 0; b < chunk * 8; ++b) {
        const int v = (b & 7) * chunk + (b >> 3);
        if (v >= n_tiles) continue;
        int ti, tk;
        tile_from_rank(v, n_t, ti, tk);
        REQUIRE(0 <= ti && ti <= tk && tk < n_t, "d_in %d ts %d rank %d -> (%d, %d)", d_in, ts, v, ti, tk);
        REQUIRE(seen.insert({ti, tk}).second, "d_in %d ts %d tile (%d, %d) owned twice", d_in, ts, ti, tk);
    }
    REQUIRE(int(seen.size()) == n_tiles, "d_in %d ts %d: %zu of %d tiles owned", d_in, ts, seen.size(), n_tiles);
}

// trailing update of the blocked Cholesky: the lower tiles of a matrix of n_t tile rows through the banded order with
// bands of SYRK_BAND, (tn, tm) = tile_from_rank_band(v), rank 0 = tile (0, 0), grid rounded up to a multiple of 8
static void check_syrk_lower(int n_t) {
    const int n_tiles = n_upper_tiles(n_t), chunk = int(cdiv(n_tiles, 8));
    std::set<std::pair<int, int>> seen;
    for (int b = 0; b < chunk * 8; ++b) {
        const int v = (b & 7) * chunk + (b >> 3);
        if (v >= n_tiles) continue;
        int tn, tm;
        tile_from_rank_band<SYRK_BAND>(v, n_t, tn, tm);
        REQUIRE(0 <= tn && tn <= tm && tm < n_t, "syrk n_t %d rank %d -> (%d, %d)", n_t, v, tm, tn);
        REQUIRE(b != 0 || (tm == 0 && tn == 0), "syrk n_t %d: workgroup 0 owns (%d, %d), not the diagonal tile", n_t, tm, tn);
        REQUIRE(seen.insert({tm, tn}).second, "syrk n_t %d tile (%d, %d) owned twice", n_t, tm, tn);
    }
    REQUIRE(int(seen.size()) == n_tiles, "syrk n_t %d: %zu of %d tiles owned", n_t, seen.size(), n_tiles);
}

// ring kernel, symmetric: 256 x 256 tiles with the split plan, 128 x 256 tiles, or 384 x 256 tiles with the
// workspace-only split plan
enum Shape { BIG, MID, WIDE };
static void tile_of(Shape shape, int v, int n_rt, int n_ct, int& ti, int& tk) {
    if (shape == BIG) tile_from_rank(v, n_ct, ti, tk);
    else if (shape == MID) tile128_from_rank(v, n_rt, n_ct, ti, tk);
    else tile_wide_from_rank(v, n_rt, n_ct, ti, tk);
}
// the ranks of a shape's tile map are a bijection onto the tiles that reach the diagonal or lie above it
static void check_tile_set(int d_in, Shape shape) {
    const int tm = shape == BIG ? 256 : shape == MID ? 128 : 384;
    const int n_rt = int(cdiv(d_in, tm)), n_ct = int(cdiv(d_in, 256));
    const int n_tiles = shape == BIG ? n_upper_tiles(n_ct) : shape == MID ? n_tiles128(n_rt, n_ct) : n_tiles_wide(n_rt, n_ct);
    std::set<std::pair<int, int>> seen;
    for (int v = 0; v < n_tiles; ++v) {
        int ti, tk;
        tile_of(shape, v, n_rt, n_ct, ti, tk);
        REQUIRE(seen.insert({ti, tk}).second, "d_in %d tile (%d, %d) has two ranks", d_in, ti, tk);
    }
    // ... and the tile set is everything that reaches the diagonal or lies above it
    int needed = 0;
    for (int i = 0; i < n_rt; ++i)
        for (int k = 0; k < n_ct; ++k)
            if (int64_t(k + 1) * 256 > int64_t(i) * tm) {
                ++needed;
                REQUIRE(seen.count({i, k}) == 1, "d_in %d tile (%d, %d) has no rank", d_in, i, k);
            }
    REQUIRE(needed == n_tiles, "d_in %d: %d tiles needed, %d ranked", d_in, needed, n_tiles);
}

static void check_ring(int d_in, int64_t n_tokens, int n_cus, int64_t ws_slots, Shape shape) {
    const bool big = shape == BIG;
    const int tm = shape == BIG ? 256 : shape == MID ? 128 : 384;
    const int n_rt = int(cdiv(d_in, tm)), n_ct = int(cdiv(d_in, 256));
    const int n_tiles = shape == BIG ? n_upper_tiles(n_ct) : shape == MID ? n_tiles128(n_rt, n_ct) : n_tiles_wide(n_rt, n_ct);
    SplitPlan sp;
    if (big) sp = plan_split(n_tiles, n_ct, d_in, n_tokens, n_cus, ws_slots);
    if (shape == WIDE) {
        sp = plan_split(n_tiles, n_ct, d_in, n_tokens, n_cus, ws_slots, false);
        REQUIRE(sp.n_split == 0 || sp.use_ws, "d_in %d: a 384-row tile split without the workspace", d_in);
    }
    REQUIRE(sp.n_split >= 0 && sp.n_split <= n_tiles && sp.split0 >= 0 && sp.split0 + sp.n_split <= n_tiles,
            "d_in %d plan split0 %d n_split %d of %d", d_in, sp.split0, sp.n_split, n_tiles);
    REQUIRE(sp.n_piece >= 1 && sp.n_piece <= 16, "d_in %d n_piece %d", d_in, sp.n_piece);
    if (sp.use_ws) REQUIRE(int64_t(sp.n_split) * sp.n_piece <= ws_slots, "d_in %d plan exceeds the workspace", d_in);
    if (sp.n_split > 0 && !sp.use_ws) {
        // two halves, the second parked in the mirror position: tiles strictly above the diagonal, inside the matrix,
        // and rank split0 + m must be tile (m % 4, 4 + m / 4) (what the merge kernel assumes)
        REQUIRE(sp.n_piece == 2, "d_in %d mirror plan with %d pieces", d_in, sp.n_piece);
        for (int m = 0; m < sp.n_split; ++m) {
            int ti, tk;
            tile_from_rank(sp.split0 + m, n_ct, ti, tk);
            REQUIRE(ti == m % GRAM_BAND && tk == GRAM_BAND + m / GRAM_BAND, "d_in %d mirror tile %d -> (%d, %d)", d_in, m, ti, tk);
            REQUIRE(tk > ti && (tk + 1) * 256 <= d_in && (ti + 1) * 256 <= d_in, "d_in %d mirror tile (%d, %d) not interior", d_in, ti, tk);
        }
    }
    const int chunk = int(cdiv(n_tiles - sp.n_split, 8));
    const int total = ring_total_blocks(chunk, sp.n_split, sp.n_piece);
    std::vector<int> whole(n_tiles, 0);
    std::vector<std::vector<int>> pieces(n_tiles);
    for (int bid = 0; bid < total; ++bid) {
        RingWork w;
        if (!ring_work(bid, chunk, n_tiles, sp.split0, sp.n_split, w)) continue;
        REQUIRE(w.v >= 0 && w.v < n_tiles, "d_in %d block %d -> rank %d of %d", d_in, bid, w.v, n_tiles);
        int ti, tk;
        tile_of(shape, w.v, n_rt, n_ct, ti, tk);
        REQUIRE(ti >= 0 && ti < n_rt && tk >= 0 && tk < n_ct, "d_in %d rank %d -> (%d, %d)", d_in, w.v, ti, tk);
        // the tile reaches the diagonal or lies above it: its last column is not left of its first row
        REQUIRE(int64_t(tk + 1) * 256 > int64_t(ti) * tm, "d_in %d rank %d below the diagonal", d_in, w.v);
        if (w.piece < 0) {
            REQUIRE(w.v < sp.split0 || w.v >= sp.split0 + sp.n_split, "d_in %d split tile %d taken whole", d_in, w.v);
            ++whole[w.v];
        } else {
            REQUIRE(w.v >= sp.split0 && w.v < sp.split0 + sp.n_split && w.m_split == w.v - sp.split0,
                    "d_in %d piece of a tile outside the split range", d_in);
            REQUIRE(w.piece < sp.n_piece, "d_in %d piece %d of %d", d_in, w.piece, sp.n_piece);
            pieces[w.v].push_back(w.piece);
        }
    }
    for (int v = 0; v < n_tiles; ++v) {
        const bool split = v >= sp.split0 && v < sp.split0 + sp.n_split;
        REQUIRE(whole[v] == (split ? 0 : 1), "d_in %d tile %d owned %d times", d_in, v, whole[v]);
        if (split) {
            std::set<int> s(pieces[v].begin(), pieces[v].end());
            REQUIRE(int(pieces[v].size()) == sp.n_piece && int(s.size()) == sp.n_piece,
                    "d_in %d tile %d has %zu pieces of %d", d_in, v, pieces[v].size(), sp.n_piece);
        }
    }
    // token ranges of the pieces: whole steps of 16, in bounds, tiling the token axis
    if (sp.n_split > 0) {
        int64_t next = 0;
        for (int p = 0; p < sp.n_piece; ++p) {
            int64_t t0, cnt;
            piece_tokens(n_tokens, sp.n_piece, p, 16, t0, cnt);
            REQUIRE(t0 % 16 == 0 && t0 == next, "d_in %d piece %d starts at %lld, expected %lld", d_in, p, (long long)t0, (long long)next);
            if (cnt > 0) { REQUIRE(t0 + cnt <= n_tokens, "d_in %d piece %d runs past the tokens", d_in, p); next = t0 + cnt; }
            else next = t0 + ((n_tokens + 15) / 16 + sp.n_piece - 1) / sp.n_piece * 16;
            if (p + 1 < sp.n_piece && cnt > 0 && t0 + cnt < n_tokens) REQUIRE(cnt % 16 == 0, "d_in %d inner piece of %lld tokens", d_in, (long long)cnt);
        }
        int64_t covered = 0;
        for (int p = 0; p < sp.n_piece; ++p) {
            int64_t t0, cnt;
            piece_tokens(n_tokens, sp.n_piece, p, 16, t0, cnt);
            if (cnt > 0) covered += cnt;
        }
        REQUIRE(covered == n_tokens, "d_in %d pieces cover %lld of %lld tokens", d_in, (long long)covered, (long long)n_tokens);
    }
}

static void check_cross(int d_in, Shape shape) {
    const int n_rt = int(cdiv(d_in, shape == BIG ? 256 : shape == MID ? 128 : 384)), n_ct = int(cdiv(d_in, 256));
    const int n_tiles = n_rt * n_ct, chunk = int(cdiv(n_tiles, 8));
    std::set<std::pair<int, int>> seen;
    for (int bid = 0; bid < ring_total_blocks(chunk, 0, 1); ++bid) {
        RingWork w;
        if (!ring_work(bid, chunk, n_tiles, 0, 0, w)) continue;
        int ti, tk;
        cross_tile_from_rank(w.v, n_rt, n_ct, ti, tk);
        REQUIRE(ti >= 0 && ti < n_rt && tk >= 0 && tk < n_ct, "cross d_in %d rank %d -> (%d, %d)", d_in, w.v, ti, tk);
        REQUIRE(seen.insert({ti, tk}).second, "cross d_in %d tile (%d, %d) owned twice", d_in, ti, tk);
    }
    REQUIRE(int(seen.size()) == n_tiles, "cross d_in %d: %zu of %d tiles", d_in, seen.size(), n_tiles);
}

static void check_trailing(int d_out, int n_cols) {
    const int n_mt = int(cdiv(d_out, 128)), n_nt = int(cdiv(n_cols, 256));
    const int chunk = int(cdiv(int64_t(n_mt) * n_nt, 8));
    std::set<std::pair<int, int>> seen;
    for (int bid = 0; bid < chunk * 8; ++bid) {
        int mt, nt;
        if (!trail_tile(bid, chunk, n_mt, n_nt, mt, nt)) continue;
        REQUIRE(mt >= 0 && mt < n_mt && nt >= 0 && nt < n_nt, "trailing %d x %d block %d -> (%d, %d)", d_out, n_cols, bid, mt, nt);
        REQUIRE(seen.insert({mt, nt}).second, "trailing %d x %d tile (%d, %d) owned twice", d_out, n_cols, mt, nt);
    }
    REQUIRE(int(seen.size()) == n_mt * n_nt, "trailing %d x %d: %zu of %d tiles", d_out, n_cols, seen.size(), n_mt * n_nt);
}

int main() {
    const int n_cus = 256;
#ifdef PLANNER_CHECK_THIN
    const int step = 16 * 37;   // a thinned set of widths for the sanitizer build
#else
    const int step = 16;
#endif
    for (int n_t = 1; n_t <= 512; ++n_t) check_syrk_lower(n_t);   // every trailing matrix up to d_in 65536
    for (int d_in = 16; d_in <= 32768; d_in += step) {
        if (d_in <= 4096 || d_in % 256 == 0) {            // every width up to 4096, then every multiple of 256 (set-based checks)
            check_simple_upper(d_in, 128);
        }
        if (d_in >= 1024) {
            // token counts around the thresholds of the plan, with and without a workspace, small and large
            const int64_t toks[] = {1, 17, 1000, 1024, 4095, 4096, 9001, 17001, 32768, 65535, 131072, 262144};
            const int64_t slots[] = {0, 3, 64, 1000, int64_t(1) << 40};
            const bool dense = d_in % 1024 == 0 || d_in <= 4096;
            for (int64_t t : toks)
                for (int64_t s : slots) {
                    if (!dense && !(t == 262144 || t == 9001)) continue;
                    check_ring(d_in, t, n_cus, s, BIG);
                    // slots of the 384 x 256 shape are 1.5 times as large: the same workspace holds two thirds as many
                    check_ring(d_in, t, n_cus, s / 3 * 2, WIDE);
                }
            check_ring(d_in, 262144, n_cus, 0, MID);
            for (Shape sh : {BIG, MID, WIDE}) check_tile_set(d_in, sh);
            if (d_in % 256 == 0 || d_in <= 4096) { check_cross(d_in, BIG); check_cross(d_in, MID); check_cross(d_in, WIDE); }
        }
    }
    for (int d_out : {1, 7, 64, 128, 129, 1000, 4096, 8192, 14336, 28672})
        for (int cols = 8; cols <= 28672; cols = cols < 2048 ? cols + 8 : cols + 512) check_trailing(d_out, cols);
    // super-block widths: a wide group is a run of whole super-blocks, each a run of whole 128-column blocks
    for (int G = 16; G <= 32768; G += 16) {
        for (int64_t d_in : {int64_t(G), int64_t(2) * G, int64_t(3) * G}) {
            if (d_in % 128 != 0 || d_in > 65535) continue;
            if (G > 128 && G % 128 != 0) continue;
            if (G < 128 && 128 % G != 0) continue;
            const int w = sweep_superblock_width(G, d_in);
            REQUIRE(w % 128 == 0 && w >= 128 && w <= 512, "G %d d_in %lld width %d", G, (long long)d_in, w);
            if (G > 128 && G != d_in) REQUIRE(G % w == 0, "G %d d_in %lld width %d does not divide the group", G, (long long)d_in, w);
        }
    }
    std::printf("ok %ld\n", n_checks);
    return 0;
}
