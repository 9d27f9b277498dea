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
    std::printf("ok %ld\n", checked);
    return 0;
}
