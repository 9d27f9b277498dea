// Exhaustive host check of the chunk geometry the matrix-core filter-gradient kernels stage into LDS: every chunk
// must fit the pixel and patch-position limits the kernels size their LDS for (an overflow would be an
// out-of-bounds LDS write on the GPU).  Built and run by tests/test_chunks_host.py with the host compiler.
#include <cstdio>
#include "ftp_plan.h"

int main()
{
    long checked = 0;
    for (int S = 1; S <= 2; ++S)
    for (int P = 0; P <= (S == 2 ? 1 : 3); ++P) {
        const int XPOS = ftp::wgrad_xpos(P, S);
        if (XPOS % 64 != 0 || XPOS > 384) { std::printf("patch size %d\n", XPOS); return 1; }      // whole load passes, at most 6
        for (int rw = 1; rw <= 160; ++rw)
            for (int rh = 1; rh <= 160; rh += (rh < 40 ? 1 : 7))
                for (int batch = 1; batch <= 9; batch += 2) {
                    const ftp::WgradChunks c = ftp::wgrad_chunks(rw, rh, batch, P, S);
                    ++checked;
                    bool ok = c.TC >= 1 && c.TCp >= c.TC && (c.TCp & 1) == 0 && c.PW == S * c.TCp + 2 * P && c.TR >= 1 && c.TI >= 1 &&
                              c.col_blocks * c.TC >= rw && c.row_blocks * c.TR >= rh && c.img_blocks * c.TI >= batch &&
                              c.total == c.img_blocks * c.row_blocks * c.col_blocks;
                    ok = ok && c.TI * c.TR * c.TCp <= 64;                              // pixels of dZ
                    ok = ok && c.TI * (S * c.TR + 2 * P) * c.PW <= XPOS;               // patch positions of X
                    if (c.TI > 1) ok = ok && c.TR == rh && c.col_blocks == 1;          // several images only for whole rectangles
                    if (!ok) {
                        std::printf("wgrad_chunks(rw=%d, rh=%d, batch=%d, P=%d, S=%d): TC=%d TCp=%d PW=%d TR=%d TI=%d blocks %d x %d x %d\n",
                                    rw, rh, batch, P, S, c.TC, c.TCp, c.PW, c.TR, c.TI, c.img_blocks, c.row_blocks, c.col_blocks);
                        return 1;
                    }
                }
    }
    // bfloat 3x3 kernel: 16 groups of 8 patch positions to a chunk; the patch (rows + 2 halo rows per image, PWp = 8 G
    // elements each) fits the LDS row of a channel; one lane loads one 16-byte unit, one lane clears one patch row
    for (int waves_ci = 1; waves_ci <= 2; ++waves_ci) {
        const int pe = ftp::w16_patch_elems(waves_ci);
        if (ftp::w16_row_bytes(waves_ci) % 32 != 16 || pe * 2 > ftp::w16_row_bytes(waves_ci)) { std::printf("row bytes\n"); return 1; }
        for (int xs = 0; xs <= 1; ++xs)
            for (int rw = 1; rw <= 200; ++rw)
                for (int rh = 1; rh <= 160; rh += (rh < 40 ? 1 : 7))
                    for (int batch = 1; batch <= 9; batch += 2) {
                        const ftp::Wgrad16Chunks c = ftp::wgrad16_chunks(rw, rh, batch, pe, xs);
                        ++checked;
                        const int rows = c.TI > 1 ? c.TI * (rh + 2) : c.RB + 2;
                        bool ok = c.TC >= 1 && c.TC <= 64 && c.G >= 1 && c.PWp == 8 * c.G && c.PWp >= c.TC + 2 + xs && c.RB >= 1 && c.TI >= 1 &&
                                  c.col_blocks * c.TC >= rw && c.row_blocks * c.RB >= rh && c.img_blocks * c.TI >= batch &&
                                  c.total == c.img_blocks * c.row_blocks * c.col_blocks;
                        ok = ok && (c.col_blocks == 1 || c.TC % 8 == 0);                   // column blocks start at even columns
                        ok = ok && (c.TI > 1 ? c.TI * rh : c.RB) * c.G <= ftp::kW16Groups;  // groups of a chunk
                        ok = ok && rows * c.PWp <= pe && rows * c.G <= 64 && rows <= 64;    // patch elements, units, rows
                        if (c.TI > 1) ok = ok && c.RB == rh && c.col_blocks == 1 && c.TI <= batch;
                        if (!ok) {
                            std::printf("wgrad16_chunks(rw=%d, rh=%d, batch=%d, pe=%d, xs=%d): TC=%d G=%d PWp=%d RB=%d TI=%d\n", rw, rh, batch, pe, xs, c.TC, c.G, c.PWp, c.RB, c.TI);
                            return 1;
                        }
                    }
    }
    // thin-layer kernel: a chunk holds at most PK pixels (rows padded to even), whole pool windows behind a pool
    for (int pooled = 0; pooled <= 1; ++pooled)
        for (int rw = 1; rw <= 320; ++rw) {
            if (pooled && (rw & 1)) continue;
            const int wpad = (rw + 1) & ~1;
            const int PK = ftp::thin_wgrad_pk(wpad, pooled != 0);
            for (int rh = pooled ? 2 : 1; rh <= 120; rh += pooled ? 2 : 1)
                for (int batch = 1; batch <= 9; batch += 4) {
                    const ftp::ThinChunks c = ftp::thin_wgrad_chunks(rw, rh, batch, PK, pooled != 0);
                    ++checked;
                    bool ok = c.TCp == wpad && c.TR >= 1 && c.TI >= 1 && c.TI * c.TR * c.TCp <= PK &&
                              c.row_blocks * c.TR >= rh && c.img_blocks * c.TI >= batch && c.total == c.img_blocks * c.row_blocks;
                    if (pooled) ok = ok && (c.TR & 1) == 0;
                    if (!ok) {
                        std::printf("thin_wgrad_chunks(rw=%d, rh=%d, batch=%d, PK=%d, pooled=%d): TCp=%d TR=%d TI=%d\n", rw, rh, batch, PK, pooled, c.TCp, c.TR, c.TI);
                        return 1;
                    }
                }
        }
    // streamed form of the thin-layer kernel: two stages of (dZ rows of 32 channels, patch) in LDS; every stack's chunk
    // fits the stage the launch is sized for, the load instructions stay inside their rows, the last operand read
    // inside the patch
    for (int pooled = 0; pooled <= 1; ++pooled)
        for (int K = 1; K <= 7; K += 2)
            for (int S = 1; S <= 2; ++S) {
                if (pooled && (S != 1 || K > 3)) continue;
                const int P = K / 2;
                for (int cin = 1; cin <= 4; ++cin)
                    for (int rw0 = pooled ? 2 : 1; rw0 <= 620; rw0 += pooled ? 2 : 3)
                        for (int d = 0; d <= 4; d += 2)
                            for (int rh0 = pooled ? 2 : 1; rh0 <= 80; rh0 += pooled ? 6 : 7)
                                for (int batch = 1; batch <= 9; batch += 4) {
                                    const int rws[2] = {rw0, rw0 + d}, rhs[2] = {rh0, rh0 + d};
                                    const ftp::ThinStream g = ftp::thin_stream_geom(rws, rhs, 2, 2, batch, cin, K, S, pooled != 0);
                                    ++checked;
                                    if (!g.fits) continue;
                                    bool ok = g.zs % 64 == 2 && g.lds <= 64 * 1024 && 2 * (size_t)g.stage_words * 4 <= g.lds && g.wgs_per_cu >= 1;
                                    for (int i = 0; i < 2 && ok; ++i)
                                        for (int j = 0; j < 2 && ok; ++j) {
                                            const ftp::ThinStreamChunks c = ftp::thin_stream_chunks(rws[j], rhs[i], batch, pooled != 0, g.cb_max);
                                            const int nzp = pooled ? c.TI * (c.TR >> 1) * (c.TC >> 1) : c.TI * c.TR * c.TC;
                                            const int passes = (nzp + 63) / 64;
                                            const int PW = S * c.TC + 2 * P, PH = S * c.TR + 2 * P, XCS = c.TI * PH * PW;
                                            const int zwords = 32 * g.zs * (pooled ? 2 : 1);
                                            ok = ok && c.TC >= 2 && (c.TC & 1) == 0 && c.TC <= g.cb_max && c.col_blocks * c.TC >= rws[j] && (c.col_blocks - 1) * c.TC < rws[j];
                                            ok = ok && c.TR >= 1 && c.row_blocks * c.TR >= rhs[i] && c.TI >= 1 && c.img_blocks * c.TI >= batch;
                                            ok = ok && c.total == c.img_blocks * c.row_blocks * c.col_blocks && c.total <= g.max_chunks && c.TI <= g.max_ti;
                                            ok = ok && (c.TI == 1 || (c.TR == rhs[i] && c.col_blocks == 1));
                                            ok = ok && (!pooled || (c.TR & 1) == 0);
                                            ok = ok && passes <= ftp::kThinZPass(pooled != 0) && 64 * passes <= g.zs - 2;
                                            ok = ok && zwords + cin * XCS <= g.stage_words;
                                            // last B operand: lane (last channel, last tap, second pixel of the pair), last row, last pair
                                            const int last = (cin - 1) * XCS + (K - 1) * PW + (K - 1) + S + ((c.TI - 1) * PH + S * (c.TR - 1)) * PW + S * (c.TC - 2);
                                            ok = ok && last < cin * XCS;
                                        }
                                    if (!ok) {
                                        std::printf("thin_stream_geom(rw=%d+%d, rh=%d+%d, batch=%d, cin=%d, K=%d, S=%d, pooled=%d): block=%d zs=%d stage=%d lds=%zu\n",
                                                    rw0, d, rh0, d, batch, cin, K, S, pooled, g.cb_max, g.zs, g.stage_words, g.lds);
                                        return 1;
                                    }
                                }
            }
    // parity-class delta kernel: the blocks of 32 cells cover every pixel of the rectangle exactly once (pixel = cell +
    // class), a block's patch fits its LDS stride, the last operand read lies inside the patch
    for (int nc = 8; nc <= 32; nc *= 2)
        for (int K = 1; K <= 3; K += 2)
            for (int x0 = 0; x0 <= 3; ++x0)
                for (int w = 1; w <= 70; w += (w < 12 ? 1 : 7))
                    for (int y0 = 0; y0 <= 3; ++y0)
                        for (int h = 1; h <= 23; h += (h < 8 ? 1 : 5)) {
                            const int x1 = x0 + w - 1, y1 = y0 + h - 1, batch = 3, NR = 32 / nc, P = K / 2;
                            const ftp::S2Blocks b = ftp::s2_blocks(x0, x1, y0, y1, batch, nc);
                            ++checked;
                            long long covered = 0;
                            bool ok = (NR + P) * (nc + P) <= ftp::kS2XCS;
                            for (int q = 0; q < b.total && ok; ++q) {
                                const int img = q / (b.gr * b.gc), rem = q - img * (b.gr * b.gc), rg = rem / b.gc;
                                const int J0 = (y0 >> 1) + NR * rg, I0 = (x0 >> 1) + nc * (rem - rg * b.gc);
                                ok = ok && img < batch;
                                for (int l = 0; l < 32; ++l) {
                                    const int cr = l / nc, cc = l - cr * nc;
                                    // last operand read of the lane: second channel of a pair, neighbour (P, P)
                                    ok = ok && (cr + P) * (nc + P) + cc + P < (NR + P) * (nc + P);
                                    for (int c = 0; c < 4; ++c) {
                                        const int y = 2 * (J0 + cr) + (c >> 1), x = 2 * (I0 + cc) + (c & 1);
                                        if (y >= y0 && y <= y1 && x >= x0 && x <= x1) ++covered;
                                    }
                                }
                            }
                            ok = ok && covered == (long long)batch * w * h;
                            if (!ok) { std::printf("s2_blocks(x0=%d, w=%d, y0=%d, h=%d, NC=%d, K=%d): gc=%d gr=%d total=%d covered=%lld\n", x0, w, y0, h, nc, K, b.gc, b.gr, b.total, covered); return 1; }
                        }
    std::printf("ok %ld\n", checked);
    return 0;
}
