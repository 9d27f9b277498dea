// Exhaustive host check of the tile geometry of the matrix-core convolution kernel: for every rectangle size, batch,
// tile capacity and patch limit in the ranges below, the tile shape the launcher chooses must make every tile the kernel
// enumerates fit - the patch inside the LDS area the kernel is compiled with, the pixels inside the tile capacity, the
// images inside the bound the 32-bit offset check uses - and the tiles of a stack must cover each of its pixels exactly
// once, every pixel's patch (filter halo included) lying inside the tile's patch.  An overflow here would be an
// out-of-bounds LDS write on the GPU.  Built and run by tests/test_chunks_host.py with the host compiler.
#include <cstdio>
#include <vector>
#include "ftp_conv_tiles.h"

using namespace ftp;

static long g_checked = 0;

static bool check_one(const int* rws, const int* rhs, int N, int M, int batch, int cap0, int S, int P, int max_pos, int npl, bool gather)
{
    const TileChoice tc = choose_tile(rws, rhs, N, M, batch, cap0, S, P, max_pos, npl, gather);
    if (tc.cs > max_pos) return true;                      // the launcher declines this shape (the caller takes another kernel)
    if (tc.cap < 1 || tc.cap > cap0 || tc.tiles_x < 1) { std::printf("bad choice cap %d tiles_x %d\n", tc.cap, tc.tiles_x); return false; }
    const int Q = npl;
    for (int i = 0; i < N; ++i)
        for (int j = 0; j < M; ++j) {
            const int rw = rws[j], rh = rhs[i];
            const int x0 = 5, y0 = 3, x1 = x0 + rw - 1, y1 = y0 + rh - 1;
            std::vector<int> hits((size_t)batch * rh * rw, 0);
            const int ntiles = tc.tiles_x * tc.tiles_r;
            long long nonempty = 0;
            for (int bx = 0; bx < ntiles; ++bx) {
                const TileGeom g = conv_tile_geom(tc.tiles_x, tc.TC, tc.cap, tc.flat, batch, x0, x1, y0, y1, bx, S, P, Q);
                if (g.empty) continue;
                ++nonempty;
                ++g_checked;
                const int n_l = (g.R0 + g.nrows - 1) / g.rh;
                bool ok = g.npos <= tc.cs && g.npos <= max_pos && g.npx >= 1 && g.npx <= tc.cap && n_l - g.n_a + 1 <= tc.max_img && n_l < batch;
                ok = ok && g.PW >= g.TC * S + 2 * P + (Q == 8 ? 1 : 0) && (Q == 0 || g.PW % Q == 0);
                if (!ok) {
                    std::printf("tile does not fit: rw %d rh %d batch %d cap0 %d S %d P %d max_pos %d npl %d: cap %d tiles_x %d flat %d bx %d npos %d cs %d npx %d images %d max_img %d\n",
                                rw, rh, batch, cap0, S, P, max_pos, npl, tc.cap, tc.tiles_x, tc.flat, bx, g.npos, tc.cs, g.npx, n_l - g.n_a + 1, tc.max_img);
                    return false;
                }
                for (int wq = 0; wq < cap0; ++wq) {
                    const TilePix t = conv_tile_pix(g, wq, x1, S, P);
                    if (!t.valid) continue;
                    if (t.n < 0 || t.n >= batch || t.y < 0 || t.y >= rh || g.ox0 + t.xl < x0 || g.ox0 + t.xl > x1) { std::printf("pixel outside the rectangle\n"); return false; }
                    ++hits[((size_t)t.n * rh + t.y) * rw + (g.ox0 + t.xl - x0)];
                    // the last patch position the pixel (window) reads: S + 2P - 1 rows and columns beyond its first (+1 for the early start of packed rows)
                    const int last = (t.prow + S - 1 + 2 * P) * g.PW + t.xl * S + (S - 1) + 2 * P + (Q == 8 ? 1 : 0);
                    if (last >= g.npos) { std::printf("patch position %d beyond the patch (%d): rw %d rh %d batch %d cap %d flat %d S %d P %d\n", last, g.npos, rw, rh, batch, tc.cap, tc.flat, S, P); return false; }
                }
            }
            for (size_t k = 0; k < hits.size(); ++k)
                if (hits[k] != 1) { std::printf("pixel %zu covered %d times: rw %d rh %d batch %d cap0 %d S %d P %d npl %d flat %d tiles_x %d\n", k, hits[k], rw, rh, batch, cap0, S, P, npl, tc.flat, tc.tiles_x); return false; }
            if (nonempty != tile_slots(tc, rw, rh, batch)) { std::printf("tile count %lld != %lld\n", nonempty, tile_slots(tc, rw, rh, batch)); return false; }
        }
    return true;
}

int main()
{
    // (K, pixels per tile, pooled / strided forward, loading mode) as the kernel is instantiated
    struct Mode { int K, BN, S, npl; bool strided; };
    const Mode modes[] = {
        {3, 256, 1, 4, false}, {3, 128, 1, 4, false}, {3, 256, 1, 0, false}, {3, 128, 1, 0, false},     // fp32 3x3: quads / element-wise (gathered patches)
        {3, 256, 2, 4, false}, {3, 128, 2, 4, false},                                                   // ... with the fused pool (tiles of windows)
        {1, 256, 1, 4, false}, {1, 128, 1, 4, false}, {1, 256, 1, 0, false},
        {5, 256, 1, 4, false}, {7, 128, 1, 4, false},
        {3, 128, 2, 4, true},                                                                           // strided forward
        {3, 128, 1, 8, false}, {3, 256, 1, 8, false}, {3, 128, 2, 8, false}, {1, 256, 1, 8, false},     // packed bfloats
    };
    for (const Mode& m : modes) {
        const int P = m.K / 2;
        const int max_pos = conv_dl_max_positions(m.K, m.BN, m.strided, m.npl == 4, m.npl == 8);
        const int cap0 = (m.S == 2 && !m.strided) ? m.BN / 4 : m.BN;
        for (int rw = 1; rw <= 70; rw += (rw < 34 ? 1 : 3))
            for (int rh = 1; rh <= 40; rh += (rh < 12 ? 1 : 5))
                for (int batch = 1; batch <= 7; batch += 3)
                    for (int gather = 0; gather <= 1; ++gather) {
                        // a grid of 2 x 2 stacks with slightly different rectangles, as clamped halos make them
                        const int rws[2] = {rw, rw > 2 ? rw - 2 : rw}, rhs[2] = {rh, rh > 1 ? rh - 1 : rh};
                        if (!check_one(rws, rhs, 2, 2, batch, cap0, m.S, P, max_pos, m.npl, gather != 0)) return 1;
                    }
    }
    std::printf("ok %ld tiles\n", g_checked);
    return 0;
}
