// Work maps of the launches: which tile (and which piece of the token axis) a workgroup owns, how a Gram call is cut
// into pieces, how wide the sweep's super-blocks are.  Plain integer logic shared by the kernels (device) and the
// launchers (host); it compiles as ordinary C++ too, so that a host program can enumerate the maps and check that
// every tile is owned exactly once (tests/planner_check.cpp).  No arithmetic of the method lives here.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define ONECOMP_HD __host__ __device__ inline
#else
#define ONECOMP_HD inline
#endif

namespace onecomp {
namespace plan {

ONECOMP_HD int imin(int a, int b) { return a < b ? a : b; }
ONECOMP_HD int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

// ---- symmetric Gram, square tiles: rank v in the banded order -> (ti, tk), ti <= tk < n_t.  Bands of GRAM_BAND tile
// rows; inside a band first the triangle on the diagonal (column by column), then the rectangle right of it column
// by column, rows fastest.
constexpr int GRAM_BAND = 4;
template <int BAND>
ONECOMP_HD void tile_from_rank_band(int v, int n_t, int& ti, int& tk) {
    int a = 0;
    while (true) {
        int rows = imin(BAND, n_t - a * BAND);
        int cols = n_t - a * BAND;
        int cnt = rows * cols - rows * (rows - 1) / 2;
        if (v < cnt) {
            int tri = rows * (rows + 1) / 2;
            if (v < tri) {
                int c = 0;
                while ((c + 1) * (c + 2) / 2 <= v) ++c;
                tk = a * BAND + c;
                ti = a * BAND + (v - c * (c + 1) / 2);
            } else {
                int w = v - tri;
                tk = a * BAND + rows + w / rows;
                ti = a * BAND + w % rows;
            }
            return;
        }
        v -= cnt;
        ++a;
    }
}
ONECOMP_HD void tile_from_rank(int v, int n_t, int& ti, int& tk) { tile_from_rank_band<GRAM_BAND>(v, n_t, ti, tk); }
// ---- factor: the lower tiles of a trailing update go through the same banded order with bands of SYRK_BAND tile
// columns ((tn, tm) = tile_from_rank_band<SYRK_BAND>): two workgroups per CU, 64 tiles of an XCD in flight, an 8 x 8
// patch of them shares 16 operand panels.
constexpr int SYRK_BAND = 8;
ONECOMP_HD int n_upper_tiles(int n_t) { return n_t * (n_t + 1) / 2; }

// ---- symmetric Gram, 128 x 256 tiles: tile (i, k) = rows [128 i, +128) x columns [256 k, +256) is computed when it
// reaches above the diagonal (k >= i / 2).  Bands of GRAM_RBAND tile rows, inside a band column by column, rows fastest.
constexpr int GRAM_RBAND = 8;
ONECOMP_HD void tile128_from_rank(int v, int n_rt, int n_ct, int& ti, int& tk) {
    for (int a = 0;; ++a) {
        const int r0 = a * GRAM_RBAND, rows = imin(GRAM_RBAND, n_rt - r0);
        for (int k = r0 / 2; k < n_ct; ++k) {
            const int valid = imin(rows, 2 * k + 2 - r0);   // rows r0 .. r0+valid-1 satisfy i / 2 <= k
            if (v < valid) { ti = r0 + v; tk = k; return; }
            v -= valid;
        }
    }
}
ONECOMP_HD int n_tiles128(int n_rt, int n_ct) {
    int n = 0;
    for (int i = 0; i < n_rt; ++i) n += n_ct - i / 2;
    return n;
}

// ---- symmetric Gram, 384 x 256 tiles: tile (i, k) = rows [384 i, +384) x columns [256 k, +256) is computed when it
// reaches above the diagonal (256 (k + 1) > 384 i, i.e. k >= floor(3 i / 2)).  Bands of GRAM_BAND tile rows, inside a
// band column by column, rows fastest.
ONECOMP_HD void tile_wide_from_rank(int v, int n_rt, int n_ct, int& ti, int& tk) {
    for (int a = 0;; ++a) {
        const int r0 = a * GRAM_BAND, rows = imin(GRAM_BAND, n_rt - r0);
        for (int k = 3 * r0 / 2; k < n_ct; ++k) {
            const int valid = imin(rows, (2 * k + 1) / 3 - r0 + 1);   // rows r0 .. r0+valid-1 satisfy 3 i / 2 <= k
            if (v < valid) { ti = r0 + v; tk = k; return; }
            v -= valid;
        }
    }
}
ONECOMP_HD int n_tiles_wide(int n_rt, int n_ct) {
    int n = 0;
    for (int i = 0; i < n_rt; ++i) n += n_ct - 3 * i / 2;
    return n;
}

// ---- cross-Gram (every tile): bands of GRAM_BAND tile rows, column by column inside a band
ONECOMP_HD void cross_tile_from_rank(int v, int n_rt, int n_ct, int& ti, int& tk) {
    const int band = imin(v / (GRAM_BAND * n_ct), (n_rt - 1) / GRAM_BAND);
    const int w = v - band * GRAM_BAND * n_ct, rows = imin(GRAM_BAND, n_rt - band * GRAM_BAND);
    tk = w / rows;
    ti = band * GRAM_BAND + w % rows;
}

// ---- ring kernel: workgroup `bid` of the whole schedule -> tile rank and piece.
// Workgroups 0 .. 8 chunk - 1 take whole tiles: the ranks outside [split0, split0 + n_split), `chunk` of them per
// XCD (hardware deals consecutive workgroups round-robin to the 8 XCDs, so workgroup b takes position
// (b % 8) * chunk + b / 8: each XCD owns a contiguous run of the order).  The workgroups after them take the n_split
// tiles of that range in n_piece pieces of the token axis each; on an XCD the pieces run tile after tile for one
// range of tokens, then for the next.  Returns false for a workgroup with nothing to do.
struct RingWork {
    int v;         // tile rank in the order of the tile map
    int piece;     // -1: the whole token axis; else the piece number
    int m_split;   // index of the tile among the split ones
};
ONECOMP_HD bool ring_work(int bid, int chunk, int n_tiles, int split0, int n_split, RingWork& w) {
    w.piece = -1;
    w.m_split = 0;
    if (bid < 8 * chunk) {
        w.v = (bid & 7) * chunk + (bid >> 3);
        if (w.v >= n_tiles - n_split) return false;
        if (w.v >= split0) w.v += n_split;
        return true;
    }
    const int b = bid - 8 * chunk, per_xcd = (n_split + 7) >> 3, j = b >> 3;
    w.m_split = (b & 7) * per_xcd + j % per_xcd;
    if (w.m_split >= n_split) return false;
    w.v = split0 + w.m_split;
    w.piece = j / per_xcd;
    return true;
}
// total workgroups of the schedule
ONECOMP_HD int ring_total_blocks(int chunk, int n_split, int n_piece) { return chunk * 8 + 8 * n_piece * int(cdiv(n_split, 8)); }
// tokens [t_begin, t_begin + count) of a piece: whole steps of kt tokens; count <= 0: nothing left for this piece
ONECOMP_HD void piece_tokens(int64_t n_tokens, int n_piece, int piece, int kt, int64_t& t_begin, int64_t& count) {
    const int64_t n_st_all = (n_tokens + kt - 1) / kt;
    const int64_t t_piece = (n_st_all + n_piece - 1) / n_piece * kt;
    t_begin = piece * t_piece;
    count = n_tokens - t_begin < t_piece ? n_tokens - t_begin : t_piece;
}

// ---- which 256 x 256 tiles of the symmetric Gram are computed in pieces of the token axis, and the estimated
// duration of the launch in units of one whole tile on one CU.
// Without a workspace only two pieces per tile are possible (the second partial sum is parked in the tile's mirror
// position), for tiles strictly above the diagonal and inside the matrix: the short last round is taken from the
// rectangular part of the first band.  With a workspace any tile can be cut into 2 .. 16 pieces: either the tiles
// left over after whole rounds, or all of them when there are fewer than two rounds.  A piece costs its share of
// the tile plus about half a percent of a tile for filling the pipeline and storing the partial sum, and it must
// keep at least 2048 tokens.
// ws_slots: how many 256 x 256 partial sums the workspace holds (0: none).
struct SplitPlan {
    int split0 = 0, n_split = 0, n_piece = 1;
    bool use_ws = false;
    double rounds = 0.0;
};
// mirror_ok: the tiles are 256 x 256, so the workspace-free form exists (other tile shapes split only with a workspace,
// whose slots are then partial sums of that shape).
inline SplitPlan plan_split(int64_t n_tiles, int64_t n_ct, int64_t d_in, int64_t n_tokens, int n_cus, int64_t ws_slots,
                            bool mirror_ok = true) {
    SplitPlan best;
    best.rounds = double(cdiv(n_tiles, n_cus));
    const int64_t r = n_tiles % n_cus;
    if (mirror_ok && r > 0 && r <= n_cus / 2 && n_tokens >= 1024 && n_ct >= GRAM_BAND + cdiv(r, GRAM_BAND) &&
        (GRAM_BAND + cdiv(r, GRAM_BAND)) * 256 <= d_in) {
        best.split0 = GRAM_BAND * (GRAM_BAND + 1) / 2;
        best.n_split = int(r);
        best.n_piece = 2;
        best.rounds = double(n_tiles / n_cus) + 0.5 * 1.06;
    }
    const int max_pc = mirror_ok ? 16 : 8;   // the larger slots of the other shapes: fewer of them
    for (int pc = 2; pc <= max_pc; ++pc) {
        if (n_tokens / pc < 2048) break;
        const double piece_cost = 1.0 / pc + 0.005;
        if (r > 0 && n_tiles > n_cus && r * pc <= ws_slots) {   // the leftover tiles, from the end of the rank order
            const double rounds = double(n_tiles / n_cus) + double(cdiv(r * pc, n_cus)) * piece_cost;
            if (rounds < best.rounds) best = SplitPlan{int(n_tiles - r), int(r), pc, true, rounds};
        }
        if (n_tiles < 2 * n_cus && n_tiles * pc <= ws_slots) {   // every tile
            const double rounds = double(cdiv(n_tiles * pc, n_cus)) * piece_cost;
            if (rounds < best.rounds) best = SplitPlan{0, int(n_tiles), pc, true, rounds};
        }
    }
    return best;
}

// ---- sweep: far-update tiles.  Workgroup bid -> tile (mt, nt) of n_mt x n_nt; each XCD (bid % 8) owns a contiguous
// run of `chunk` positions, m fastest inside bands of TRAIL_BAND row tiles.  Returns false for an idle workgroup.
constexpr int TRAIL_BAND = 8;
ONECOMP_HD bool trail_tile(int bid, int chunk, int n_mt, int n_nt, int& mt, int& nt) {
    const int v = (bid & 7) * chunk + (bid >> 3);
    if (v >= n_mt * n_nt) return false;
    const int band = imin(v / (TRAIL_BAND * n_nt), (n_mt - 1) / TRAIL_BAND);
    const int rem = v - band * TRAIL_BAND * n_nt;
    const int mb = imin(TRAIL_BAND, n_mt - TRAIL_BAND * band);
    mt = band * TRAIL_BAND + rem % mb;
    nt = rem / mb;
    return true;
}

// ---- sweep: width of a super-block.  512 columns; for groups wider than a 128-column block that are not the whole
// row, the largest of 512 / 384 / 256 / 128 that divides the group, so that a group is a run of whole super-blocks.
inline int sweep_superblock_width(int group_size, int64_t d_in) {
    if (group_size > 128 && group_size != d_in)
        for (int c = 512; c >= 128; c -= 128)
            if (group_size % c == 0) return c;
    return 512;
}

}  // namespace plan
}  // namespace onecomp
