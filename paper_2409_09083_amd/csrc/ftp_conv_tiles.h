// Tile geometry of the matrix-core convolution kernel (ftp_mfma_conv.hip), shared by the kernel, its launcher and the
// host check of tests/host_checks (plain integer arithmetic, no device types): how a stack's rectangle is cut into the
// tiles of one workgroup each, which patch of the input a tile stages in LDS, and the choice of the tile shape.
#pragma once
#include <cstddef>
#include "ftp_plan.h"

namespace ftp {

FTP_HD constexpr bool conv_dl_quads(size_t elem, bool pool_in, bool up_in) { return elem == 4 && !pool_in && !up_in; }
// 16-bit maps on the bfloat matrix-core path (stride-1 1x1 / 3x3), patch not gathered through pool winners: the patch may
// stay packed in LDS, two bytes a position, loaded 8 positions (16 bytes) a lane
FTP_HD constexpr bool conv_dl_packable(size_t elem, int K, int stride, bool pool_in) { return elem == 2 && K <= 3 && stride == 1 && !pool_in; }
// (a multiple of 256; quads pad every patch row to a multiple of 4 positions, which costs the narrow rectangles of deep
// layers up to a fifth more positions: their 128-pixel tiles get the room of the 256-pixel ones)
// (packed bfloats: twice the positions in the same bytes, in blocks of 512)
FTP_HD constexpr int conv_dl_max_positions(int K, int BN, bool strided_fwd, bool quad, bool packed = false)          // patch positions in LDS
{
    return packed ? (K == 3 && BN == 256 ? 1024 : 512)
                  : strided_fwd ? 768 : K >= 5 ? (BN == 256 ? 768 : 512) : K == 1 ? 256 : (BN == 256 || quad ? 512 : 256);
}


// Geometry of one tile.  A rectangle is cut into column blocks of TC columns and runs of whole rows (c0 = 0), or, where
// the launch says so (a rectangle of one column block whose rows fill a tile badly), into runs of `cap` consecutive pixels
// of its row-major pixel list, counted through the batch: a tile then starts at column c0 of flattened row R0 and need not
// end at a row end, so every tile but a stack's last is full.  The patch covers the rows R0 .. R0+nrows-1 in full.
struct TileGeom {
    int rw, rh;            // the stack's rectangle
    int TC, ox0;           // column block
    int R0, nrows;         // flattened rows
    int c0, npx;           // first pixel's column in row R0; pixels (pool windows) of the tile
    int n_a, y_a;          // first image and its first row
    int PW;                // patch row length
    int first_cnt, per_cnt;// patch rows of the first image / of every further image
    int npos;              // patch positions
    bool empty;
};

// Q: positions of a patch row a lane loads at once (0: one; 4: fp32 quads; 8: packed bfloats, whose rows start up to one
// position early, on the dword grid of the map): patch rows are padded to whole units.
FTP_HD inline TileGeom conv_tile_geom(int tiles_x, int TC, int cap, int flat, int batch, int x0, int x1, int y0, int y1, int bx, int S, int P, int Q)
{
    TileGeom g;
    g.rw = x1 - x0 + 1; g.rh = y1 - y0 + 1;
    const int tx = bx % tiles_x, tb = bx / tiles_x;
    g.TC = tiles_x == 1 ? g.rw : TC;
    g.ox0 = x0 + tx * g.TC;
    const int rtot = batch * g.rh;
    if (flat) {
        const int p0 = tb * cap, total = rtot * g.rw;
        g.empty = p0 >= total;
        g.R0 = p0 / g.rw; g.c0 = p0 - g.R0 * g.rw;
        g.npx = total - p0 < cap ? total - p0 : cap;
        g.nrows = (g.c0 + g.npx + g.rw - 1) / g.rw;
    } else {
        int trf = cap / g.TC; if (trf < 1) trf = 1;
        g.R0 = tb * trf; g.c0 = 0;
        g.empty = g.ox0 > x1 || g.R0 >= rtot;
        g.nrows = rtot - g.R0 < trf ? rtot - g.R0 : trf;
        g.npx = g.nrows * g.TC;
    }
    g.n_a = g.R0 / g.rh; g.y_a = g.R0 - g.n_a * g.rh;
    const int n_l = (g.R0 + g.nrows - 1) / g.rh;
    g.PW = g.TC * S + 2 * P;
    if (Q == 4) g.PW = (g.PW + 3) & ~3;
    if (Q == 8) g.PW = (g.PW + 1 + 7) & ~7;
    const int first_rows = g.rh - g.y_a < g.nrows ? g.rh - g.y_a : g.nrows;
    g.first_cnt = S * first_rows + 2 * P;
    g.per_cnt = S * g.rh + 2 * P;
    g.npos = (S * g.nrows + 2 * P * (n_l - g.n_a + 1)) * g.PW;
    return g;
}

// Pixel (or pool window) wq of a tile -> image, row (relative to the rectangle), column, and its patch row.
struct TilePix { int n, y, xl, prow; bool valid; };
FTP_HD inline TilePix conv_tile_pix(const TileGeom& g, int wq, int x1, int S, int P)
{
    TilePix t;
    const int lin = g.c0 + wq;
    const int fr = lin / g.TC;
    t.xl = lin - fr * g.TC;
    const int R = g.R0 + fr;
    t.n = R / g.rh;
    t.y = R - t.n * g.rh;
    t.prow = S * fr + 2 * P * (t.n - g.n_a);
    t.valid = wq < g.npx && fr < g.nrows && g.ox0 + t.xl <= x1;
    return t;
}

struct TileChoice { int TC, tiles_x, tiles_r, cap, cs, max_img, flat; };

// Tile capacity (pixels or pool windows), column blocking and the worst-case patch size over all stacks.
// npl: positions of a patch row the kernel loads per lane (0, 4 or 8): rows are padded as tile_geom pads them.
// gather: every further patch position is expensive (the patch is collected element by element - through pool winners,
// between inserted zeros - or the kernel is bound by the latency of its patch loads).
inline TileChoice choose_tile(const int* rws, const int* rhs, int N, int M, int batch, int cap0, int S, int P, int max_pos, int npl, bool gather)
{
    int mw = 0;
    for (int t = 0; t < M; ++t) mw = mw > rws[t] ? mw : rws[t];
    const int max_tc = 64 / S;                         // widest column block of a tile
    // One way of cutting: `tx` column blocks and runs of whole rows, or (flat) runs of pixels.  The tile capacity is cut
    // down until the largest patch fits LDS; `tiles` = workgroups of one channel block, each of which costs the same
    // matrix-core work however many of its slots are filled.
    auto eval = [&](int tx, bool flat, double* tiles_out) -> TileChoice {
        TileChoice c;
        c.tiles_x = tx; c.flat = flat ? 1 : 0;
        c.TC = (mw + tx - 1) / tx;
        c.cap = cap0;
        for (;;) {
            c.tiles_r = 1; c.cs = 1; c.max_img = 1;
            bool fits = true;
            double tiles_all = 0;
            for (int i = 0; i < N; ++i)
                for (int j = 0; j < M; ++j) {
                    const int rw = rws[j], rh = rhs[i];
                    const int rtot = batch * rh;
                    const int tc = tx == 1 ? rw : c.TC;
                    int tiles, rows;                       // tiles of this stack (per column block); most rows one of them touches
                    if (flat) {
                        tiles = (int)(((long long)rtot * rw + c.cap - 1) / c.cap);
                        rows = (c.cap + 2 * tc - 2) / tc;          // a run of cap pixels that starts at the last column of a row
                    } else {
                        int trf = c.cap / tc; if (trf < 1) trf = 1;
                        tiles = (rtot + trf - 1) / trf;
                        rows = trf;
                    }
                    if (rows > rtot) rows = rtot;
                    if (tiles > c.tiles_r) c.tiles_r = tiles;
                    tiles_all += (double)tiles * ((rw + tc - 1) / tc);
                    int nimg = (rows + rh - 2) / rh + 1; if (nimg > batch) nimg = batch;
                    if (nimg > c.max_img) c.max_img = nimg;
                    const int pw = npl == 8 ? (tc * S + 2 * P + 1 + 7) & ~7 : npl == 4 ? (tc * S + 2 * P + 3) & ~3 : tc * S + 2 * P;
                    const int npos = (S * rows + 2 * P * nimg) * pw;
                    if (npos > c.cs) c.cs = npos;
                    if (npos > max_pos && rows > 1) fits = false;
                }
            *tiles_out = tiles_all;
            if (fits || c.cap <= 8) break;
            c.cap -= c.cap / 8;
        }
        return c;
    };
    // Whole rows of the fewest column blocks are the reference.  Narrower blocks can fill the slots of a tile better (rows
    // of 25 pool windows put 50 into 64 slots, blocks of 9 + 9 + 7 put 63 + 63 + 49 into 192): up to three more blocks are
    // tried and taken if they save more than 9 % of the tiles (a block more costs a filter halo more; config 4, delta through
    // the first pool: rows of 54 pixels fill 216 of 256 slots, blocks of 18 fill 252, 2.39 -> 2.16 ms).  A rectangle of one
    // column block can be cut into runs of pixels, which leaves no slot empty but makes a tile touch one or two rows more (a
    // larger patch): taken if it saves tiles at all, but not where patch positions are expensive (config 4, delta pass
    // through the first pool: 16 % fewer tiles, a third more patch positions, 13 % slower).
    const int base = (mw + max_tc - 1) / max_tc;
    int tx_rows = base;
    {
        // (slots of the uncut capacity: what the split is judged by)
        auto slots_for = [&](int tx) -> double {
            const int TCt = (mw + tx - 1) / tx;
            double slots = 0;
            for (int i = 0; i < N; ++i)
                for (int j = 0; j < M; ++j) {
                    const int rw = rws[j], rh = rhs[i];
                    const int tc = tx == 1 ? rw : TCt;
                    int trf = cap0 / tc; if (trf < 1) trf = 1;
                    slots += (double)(((long long)batch * rh + trf - 1) / trf) * ((rw + tc - 1) / tc);
                }
            return slots;
        };
        double best_slots = slots_for(base);
        for (int tx = base + 1; tx <= base + 3 && (mw + tx - 1) / tx >= 4; ++tx) {
            const double sl = slots_for(tx);
            if (sl < 0.91 * best_slots) { best_slots = sl; tx_rows = tx; }
        }
    }
    double best_tiles = 0;
    TileChoice best = eval(tx_rows, false, &best_tiles);
    if (base == 1 && !gather) {
        double t = 0;
        const TileChoice c = eval(1, true, &t);
        if (t < 0.99 * best_tiles) { best = c; best_tiles = t; }
    }
    return best;
}

// Tiles one stack's rectangle is cut into (what tile_geom() enumerates).
inline long long tile_slots(const TileChoice& tc, int rw, int rh, int batch)
{
    const long long rtot = (long long)batch * rh;
    if (tc.flat) return (rtot * rw + tc.cap - 1) / tc.cap;
    const int tcw = tc.tiles_x == 1 ? rw : tc.TC;
    int trf = tc.cap / tcw; if (trf < 1) trf = 1;
    return ((rtot + trf - 1) / trf) * ((rw + tcw - 1) / tcw);
}

}  // namespace ftp
