// Exhaustive host check of the chunk geometry the matrix-core filter-gradient kernels stage into LDS: every chunk
// must fit the pixel and patch-position limits the kernels size their LDS for (an overflow would be an
// out-of-bounds LDS write on the GPU).  Built and run by tests/test_chunks_host.py with the host compiler.
#include <cstdio>
#include "ftp_plan.h"

int main()
{
    long checked = 0;
    for (int P = 0; P <= 3; ++P) {
        const int XPOS = ftp::wgrad_xpos(P);
        for (int rw = 1; rw <= 160; ++rw)
            for (int rh = 1; rh <= 160; rh += (rh < 40 ? 1 : 7))
                for (int batch = 1; batch <= 9; batch += 2) {
                    const ftp::WgradChunks c = ftp::wgrad_chunks(rw, rh, batch, P);
                    ++checked;
                    bool ok = c.TC >= 1 && c.TCp >= c.TC && (c.TCp & 1) == 0 && c.PW == c.TCp + 2 * P && c.TR >= 1 && c.TI >= 1 &&
                              c.col_blocks * c.TC >= rw && c.row_blocks * c.TR >= rh && c.img_blocks * c.TI >= batch &&
                              c.total == c.img_blocks * c.row_blocks * c.col_blocks;
                    ok = ok && c.TI * c.TR * c.TCp <= 64;                              // pixels of dZ
                    ok = ok && c.TI * (c.TR + 2 * P) * c.PW <= XPOS;                   // patch positions of X
                    if (c.TI > 1) ok = ok && c.TR == rh && c.col_blocks == 1;          // several images only for whole rectangles
                    if (!ok) {
                        std::printf("wgrad_chunks(rw=%d, rh=%d, batch=%d, P=%d): TC=%d TCp=%d PW=%d TR=%d TI=%d blocks %d x %d x %d\n",
                                    rw, rh, batch, P, c.TC, c.TCp, c.PW, c.TR, c.TI, c.img_blocks, c.row_blocks, c.col_blocks);
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
