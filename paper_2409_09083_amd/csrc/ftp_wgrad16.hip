// Per-stack filter gradient of 3x3 stride-1 convolutions over 16-bit (bfloat) maps on the matrix cores of gfx950
// (Sec. 4.1: the filter gradient of a tile is the correlation of its input map with the delta map of its output, summed
// over the batch and over the pixels the tile owns):
//   dW[co][ci][ky][kx] = sum over images and owned output pixels (y, c) of dZ[co][y][c] * X[ci][y + ky - 1][c + kx - 1]
// is a GEMM with M = co, N = ci and the pixels as reduction dimension, one accumulator tile per tap.
//
// v_mfma_f32_32x32x16_bf16 takes, per lane, 8 consecutive reduction elements of one row of A and one column of B
// (A[m = lane%32][k = 8*(lane/32) + j], B[k = 8*(lane/32) + j][n = lane%32], j < 8).  The maps are pixel-contiguous
// per channel in HBM, so 8 consecutive reduction elements are 16 contiguous bytes if the reduction index is the
// position e in a row of the input patch:
//   dW[..][ky][kx] = sum over rows y and patch positions e of dZrow[y][e - kx] * Xpatch[y + ky][e]
// where Xpatch row positions count from the patch's first element and dZrow is the row of deltas moved to where its
// first pixel reads tap kx = 0, zero outside the owned pixels.  So:
//   X   stays packed (two bfloats to a dword) and channel-major in LDS, as in HBM, and goes HBM -> LDS with
//       buffer_load_dwordx4 ... lds, 16 bytes per lane, no registers in between.  The patch starts on the dword grid of
//       the map (one element before column x0 - 1 where that is odd).  Units outside the map come from out-of-range
//       offsets, which read as zero; elements a unit brings along beyond the needed columns are cleared afterwards by
//       the wavefront that loaded it.  One aligned 16-byte LDS read serves the three taps of a filter row.
//   dZ  goes through registers (it needs per-pixel treatment: the ends of a row, and behind a pool the routing of each
//       pooled delta to its window's winner) and is written to LDS as [group of 8 positions][co][16 bytes]; the tap
//       kx = 1, 2 operands are that group shifted by one and two elements, cut from it and the last dword of the group
//       before it in the row (kept in a small table of its own, so that every LDS read is free of bank conflicts).
// Two patch buffers alternate, so the loads of chunk i+1 are in flight while the matrix cores work on chunk i.
#include "ftp_device.h"
#include "ftp_launch.h"

namespace ftp {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

struct Wgrad16Args {
    View in, din, mask;
    RectTab own;                                    // owned rectangle at the convolution output (before the pool)
    float* partial;                                 // [stacks][n_params]
    float* scratch;                                 // [stacks][splits][Cout*Cin*9] when splits > 1
    long long n_params, w_off;
    int Cin, Cout, Hc, Wc;                          // map extent at the convolution (stride 1: input = output)
    int splits, M, batch;
    int gx, stacks;                                 // blocks per (stack, share); stacks (the grid is 1-D, see xcd_order)
};

#define FTP_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
constexpr unsigned kOob16 = 0x80000000u;            // beyond the records of every buffer resource below: reads as zero
constexpr unsigned kRecords16 = 0x7FFFFFFFu;


__device__ __forceinline__ uint32_t alignhalf(uint32_t hi, uint32_t lo) { return __builtin_amdgcn_alignbit(hi, lo, 16); }

// HALF: 0 = deltas at the resolution of the owned rectangle; 1 = a 2x2 pool follows the convolution: the deltas sit
// at pooled resolution and a pixel receives its window's delta only if it is the window's winner.
template <int WAVES_CI, int HALF>
__global__ void __launch_bounds__(256, 2)
k_wgrad_mfma16(Wgrad16Args a)
{
    constexpr int WAVES_CO = 2, WAVES_K = 4 / (WAVES_CO * WAVES_CI);
    constexpr int BCO = 32 * WAVES_CO, BCI = 32 * WAVES_CI;
    constexpr int NG = kW16Groups;
    constexpr int XSB = w16_row_bytes(WAVES_CI);
    constexpr int XBUF = BCI * XSB;
    constexpr int ZBYTES = NG * BCO * 16, PBYTES = NG * BCO * 4;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds16[];
    unsigned char* const Xl0 = lds16;
    unsigned char* const Xl1 = lds16 + XBUF;
    unsigned char* const Zl = lds16 + 2 * XBUF;           // [group][co (rotated by the group index)][8 bfloats]
    uint32_t* const Zp = (uint32_t*)(Zl + ZBYTES);        // [group][co]: last dword of the group before it in the row (or 0)
    int* const gtab = (int*)(Zl + ZBYTES + PBYTES);       // [group] -> byte offset of its 8 positions in a patch row (ky = 0)

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_co = wave % WAVES_CO, wave_ci = (wave / WAVES_CO) % WAVES_CI, wave_k = wave / (WAVES_CO * WAVES_CI);
    const int hi = lane >> 5, l32 = lane & 31;
    // (block, share, stack), block fastest, in XCD order: the blocks of one stack and share read the same maps
    int vgroup, bx;
    if (!xcd_order(a.splits * a.stacks, a.gx, vgroup, bx)) return;
    const int split = vgroup % a.splits;
    const int stack = vgroup / a.splits, ti = stack / a.M, tj = stack % a.M;
    const int x0 = a.own.x0[tj], x1 = a.own.x1[tj], y0 = a.own.y0[ti], y1 = a.own.y1[ti];
    const int rw = x1 - x0 + 1, rh = y1 - y0 + 1;
    const int tiles_ci = (a.Cin + BCI - 1) / BCI;
    const int co0 = (bx / tiles_ci) * BCO, ci0 = (bx % tiles_ci) * BCI;

    // what the per-chunk code needs of the argument block, once
    const int Hc = a.Hc, Wc = a.Wc, Cin = a.Cin, Cout = a.Cout, batch = a.batch;
    const int in_x0 = a.in.x0[tj], in_y0 = a.in.y0[ti], in_pitch = a.in.pitch, in_cs = (int)a.in.cs, in_ns = (int)a.in.ns;
    const int d_x0 = a.din.x0[tj], d_y0 = a.din.y0[ti], d_pitch = a.din.pitch, d_cs = (int)a.din.cs, d_ns = (int)a.din.ns;
    const int m_x0 = a.mask.x0[tj], m_y0 = a.mask.y0[ti], m_pitch = a.mask.pitch, m_cs = (int)a.mask.cs, m_ns = (int)a.mask.ns;
    // Parity of the patch's first column (x0 - 1) in the input view: the patch starts one element earlier where it is
    // odd (strides of the view are even, column blocks a multiple of 8 wide: the same for every row, channel and chunk
    // of the stack).  Patch position e is map column xb - 1 - xs + e; pixel c of a row reads positions c + xs + kx.
    // Group gi holds the deltas of pixels 8 gi - xs .. 8 gi - xs + 7 (the pixels whose tap kx = 0 sits at positions
    // 8 gi .. 8 gi + 7), zero where there is no such pixel.
    const int xs = (x0 - 1 - in_x0) & 1;
    const Wgrad16Chunks wc = wgrad16_chunks(rw, rh, batch, w16_patch_elems(WAVES_CI), xs);
    const int G = wc.G, PWp = wc.PWp;
    const int id0 = (int)((long long)split * wc.total / a.splits), id1 = (int)((long long)(split + 1) * wc.total / a.splits);

    // LDS starts as zeros (everything a multiply reads is written first, except patch rows beyond a short chunk's)
    for (int i = tid; i < (2 * XBUF + ZBYTES + PBYTES + NG * 4) / 4; i += 256) ((uint32_t*)lds16)[i] = 0u;

    v16f acc[9];
#pragma unroll
    for (int t = 0; t < 9; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[t][i] = 0.0f;

    // Chunks: (image block, row block, column block), column block fastest.  Either a chunk is RB rows of one image
    // (TI == 1), or TI whole images of rh rows: in both cases a patch position or a group index splits into (image, row,
    // column part) the same way in every chunk of the stack, so each lane does that once.
    struct Chunk { int n0, ni, yb, nr, xb, nc; };
    const int RB = wc.RB, TI = wc.TI, TC = wc.TC, row_blocks = wc.row_blocks, col_blocks = wc.col_blocks;
    auto chunk_of = [&](int ib, int rb, int cb) {
        Chunk c;
        c.n0 = ib * TI; c.ni = (batch - c.n0) < TI ? (batch - c.n0) : TI;
        c.yb = y0 + rb * RB; c.nr = (y1 - c.yb + 1) < RB ? (y1 - c.yb + 1) : RB;
        c.xb = x0 + cb * TC; c.nc = (x1 - c.xb + 1) < TC ? (x1 - c.xb + 1) : TC;
        return c;
    };
    const int prh_full = (TI > 1 ? rh : RB) + 2;                   // patch rows per image (TI > 1: always whole images)
    // lane -> 16-byte unit of the patch: (image, row of its patch, unit of the row; G units to a row); a chunk with fewer
    // rows (TI == 1: one image) has the same split, only fewer positions
    const int x_pr = lane / G, x_u = lane - x_pr * G;
    const int x_il = TI > 1 ? x_pr / prh_full : 0, x_lr = TI > 1 ? x_pr - x_il * prh_full : x_pr;
    // thread -> group of the chunk: (row of the chunk, group of the row); row -> (image, row of the image)
    const int zg = tid & 15, zco = tid >> 4;
    const int z_fr = zg / G, z_gi = zg - z_fr * G;
    const int z_il = TI > 1 ? z_fr / rh : 0, z_r = TI > 1 ? z_fr - z_il * rh : z_fr;

    // ---- X: HBM -> LDS ------------------------------------------------------------------------------------------
    // One lane moves 16 bytes (8 elements, a "unit"; the memory pipeline handles four lanes a clock whatever their width,
    // so dword loads would take four times as many instructions).  A unit is loaded if its row lies in the map and it
    // overlaps the needed columns [xb - 1, xb + nc] cut to the map.  Its address is a multiple of 4 bytes, possibly
    // 4 bytes before the view (the buffer resource starts 4 bytes early).
    const bf16_t* const xstack = (const bf16_t*)a.in.p + (long long)stack * a.in.ss - 2;
    auto issue_x = [&](unsigned char* Xb, const Chunk& c) {
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)(xstack + (long long)c.n0 * in_ns), (short)0, (int)kRecords16, 0x00020000);
        const int pu = c.ni * (c.nr + 2) * G;                      // units of the patch: at most 64
        const int na = c.xb - 1 > 0 ? c.xb - 1 : 0, nb = c.xb + c.nc < Wc ? c.xb + c.nc : Wc - 1;
        if (lane < pu) {                                            // (lanes beyond the patch must not write into the next channel's row)
            const int y = c.yb - 1 + x_lr, mx = c.xb - 1 - xs + 8 * x_u;
            unsigned vo = kOob16;
            if (y >= 0 && y < Hc && mx + 7 >= na && mx <= nb)
                vo = 4u + 2u * (unsigned)(x_il * in_ns + (y - in_y0) * in_pitch + (mx - in_x0));
#pragma unroll
            for (int k = 0; k < BCI / 4; ++k) {
                const int ci = wave + 4 * k;
                const unsigned v = ci0 + ci < Cin ? vo : kOob16;
                const unsigned so = 2u * (unsigned)((ci0 + ci) * in_cs);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, FTP_LDS_PTR(Xb + ci * XSB), 16, v, so, 0, 0);
            }
        }
    };
    // The first and the last loaded unit of a row bring elements outside the needed columns along: zero padding beyond
    // the map's first / last column (read by real pixels), or columns that only meet zero deltas (other stacks' data,
    // another buffer, or memory nobody wrote: it has to be finite at least).  The wavefront that loaded a channel clears
    // them once its loads have landed: lane = patch row, a few zero stores per channel.
    auto fixup_x = [&](unsigned char* Xb, const Chunk& c) {
        const int na = c.xb - 1 > 0 ? c.xb - 1 : 0, nb = c.xb + c.nc < Wc ? c.xb + c.nc : Wc - 1;
        const int e_first = na - (c.xb - 1) + xs, e_last = nb - (c.xb - 1) + xs;      // first / last needed position (e_first <= 2)
        int z = e_last + 1;
        const int zend = (e_last | 7) + 1;                         // positions [e_last + 1, zend) of the last unit are cleared
        const bool w16 = (z & 1) != 0; z += z & 1;
        const bool w32 = (z & 2) && z < zend; const int z32 = z; z += w32 ? 2 : 0;
        const bool w64 = (z & 4) && z < zend; const int z64 = z;
        if (lane < c.ni * (c.nr + 2)) {
            unsigned char* row = Xb + wave * XSB + lane * PWp * 2;
            if (e_first == 1) {
#pragma unroll
                for (int k = 0; k < BCI / 4; ++k) *(uint16_t*)(row + 4 * k * XSB) = (uint16_t)0;
            }
            if (e_first == 2) {
#pragma unroll
                for (int k = 0; k < BCI / 4; ++k) *(uint32_t*)(row + 4 * k * XSB) = 0u;
            }
            if (w16) {
#pragma unroll
                for (int k = 0; k < BCI / 4; ++k) *(uint16_t*)(row + 4 * k * XSB + 2 * (e_last + 1)) = (uint16_t)0;
            }
            if (w32) {
#pragma unroll
                for (int k = 0; k < BCI / 4; ++k) *(uint32_t*)(row + 4 * k * XSB + 2 * z32) = 0u;
            }
            if (w64) {
#pragma unroll
                for (int k = 0; k < BCI / 4; ++k) *(uint2*)(row + 4 * k * XSB + 2 * z64) = make_uint2(0u, 0u);
            }
        }
    };

    // ---- dZ: HBM -> registers -> LDS ----------------------------------------------------------------------------
    // thread -> group g = tid % 16 of the chunk and output channels tid / 16 + 16 * it.  A group's 8 pixels are 16
    // contiguous bytes in HBM that start on a 2-byte boundary: 4 dwords from the even element at or before them, and a
    // fifth when the start is odd.  Behind a pool: the 5 pooled deltas (3 dwords) and 5 code bytes (2 dwords) of the
    // windows the group touches.  Pixels outside the row are masked; the loads may start 4 bytes before a map and run a
    // few bytes past it (the workspace has margins for that): the buffer resources start 4 bytes early.
    uint32_t zr[4][5];
    int zlo = 0, zhi = 0, zsh = 0, zwant = 0, zgoff = 0, zbo0 = 0;
    bool zfrom_next = false;
    const bf16_t* const zstack = (const bf16_t*)a.din.p + (long long)stack * a.din.ss - 2;
    const uint8_t* const mstack = (const uint8_t*)a.mask.p + (long long)stack * a.mask.ss - 4;
    auto load_z = [&](const Chunk& c) {
        const int ngroups = c.ni * c.nr * G;
        const int gi = z_gi, il = z_il, r = z_r;
        const int cs0 = 8 * gi - xs;                               // first pixel of the group, relative to the row
        int lo = cs0 < 0 ? -cs0 : 0, hi_ = c.nc - cs0; hi_ = hi_ > 8 ? 8 : hi_;
        const bool inrow = zg < ngroups, exists = inrow && hi_ > lo;
        zlo = exists ? lo : 0; zhi = exists ? hi_ : 0;
        zgoff = inrow ? 2 * ((il * (c.nr + 2) + r) * PWp + 8 * gi) : 0;
        const __amdgpu_buffer_rsrc_t zrsrc = __builtin_amdgcn_make_buffer_rsrc((void*)(zstack + (long long)c.n0 * d_ns), (short)0, (int)kRecords16, 0x00020000);
        typedef uint32_t v4u __attribute__((ext_vector_type(4)));
        typedef uint32_t v3u __attribute__((ext_vector_type(3)));
        typedef uint32_t v2u __attribute__((ext_vector_type(2)));
        if (HALF == 0) {
            const int eo = il * d_ns + (c.yb + r - d_y0) * d_pitch + (c.xb + cs0 - d_x0);       // (-1 at the very first pixel of a view)
            const int odd = eo & 1;
            zsh = odd * 16;
            // the fifth dword is the first dword of the next group of the row, which the next lane loads (same channel);
            // only where the row's pixels end with this group it takes a load of its own
            const bool fifth = odd && zhi == 8;
            zfrom_next = fifth && c.nc - cs0 > 8;
            const bool extra = fifth && !zfrom_next;
            const bool any_extra = __builtin_amdgcn_ballot_w64(extra) != 0ull;
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                const int gco = co0 + zco + 16 * it;
                const bool ok = exists && gco < Cout;
                const unsigned base = 4u + 2u * (unsigned)((eo & ~1) + gco * d_cs);
                const v4u q = __builtin_amdgcn_raw_buffer_load_b128(zrsrc, ok ? base : kOob16, 0, 0);
                zr[it][0] = q[0]; zr[it][1] = q[1]; zr[it][2] = q[2]; zr[it][3] = q[3];
                zr[it][4] = 0u;
                if (any_extra) zr[it][4] = __builtin_amdgcn_raw_buffer_load_b32(zrsrc, ok && extra ? base + 16u : kOob16, 0, 0);
            }
        } else {
            const __amdgpu_buffer_rsrc_t mrsrc = __builtin_amdgcn_make_buffer_rsrc((void*)(mstack + (long long)c.n0 * m_ns), (short)0, (int)kRecords16, 0x00020000);
            // first window the group touches (the rectangle starts at an even column: windows are whole inside it)
            const int py = (c.yb + r) >> 1, pw = (c.xb >> 1) + 4 * gi - xs;
            zwant = 2 * ((c.yb + r) & 1);
            const int eo = il * d_ns + (py - d_y0) * d_pitch + (pw - d_x0);
            zsh = (eo & 1) * 16;
            zbo0 = il * m_ns + (py - m_y0) * m_pitch + (pw - m_x0);
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                const int gco = co0 + zco + 16 * it;
                const bool ok = exists && gco < Cout;
                const unsigned base = 4u + 2u * (unsigned)((eo & ~1) + gco * d_cs);
                const v3u q = __builtin_amdgcn_raw_buffer_load_b96(zrsrc, ok ? base : kOob16, 0, 0);
                zr[it][0] = q[0]; zr[it][1] = q[1]; zr[it][2] = q[2];
                const int bo = zbo0 + gco * m_cs;
                const v2u k2 = __builtin_amdgcn_raw_buffer_load_b64(mrsrc, ok ? 4u + (unsigned)(bo & ~3) : kOob16, 0, 0);
                zr[it][3] = k2[0]; zr[it][4] = k2[1];
            }
        }
    };
    // which elements of output dword i (elements 2i, 2i+1) lie in [lo, hi)
    auto keep = [](int lo, int hi_, int i) -> uint32_t {
        return ((2 * i >= lo && 2 * i < hi_) ? 0x0000FFFFu : 0u) | ((2 * i + 1 >= lo && 2 * i + 1 < hi_) ? 0xFFFF0000u : 0u);
    };
    auto store_z = [&]() {
        if (tid < NG) gtab[zg] = zgoff;
        const uint32_t k0 = keep(zlo, zhi, 0), k1 = keep(zlo, zhi, 1), k2 = keep(zlo, zhi, 2), k3 = keep(zlo, zhi, 3);
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int co = zco + 16 * it;
            uint32_t o[4];
            if (HALF == 0) {
                const uint32_t nxt = (uint32_t)__shfl_down((int)zr[it][0], 1, 16);      // first dword of the next lane's group
                const uint32_t q4 = zfrom_next ? nxt : zr[it][4];
#pragma unroll
                for (int i = 0; i < 4; ++i) o[i] = __builtin_amdgcn_alignbit(i < 3 ? zr[it][i + 1] : q4, zr[it][i], (uint32_t)zsh);
            } else {
                // 5 pooled deltas and their winner codes; element j of the group is pixel 8 gi - xs + j: window
                // ((j - xs) >> 1) + xs of the 5, left or right pixel by the parity of j + xs
                const uint32_t d01 = __builtin_amdgcn_alignbit(zr[it][1], zr[it][0], (uint32_t)zsh);
                const uint32_t d23 = __builtin_amdgcn_alignbit(zr[it][2], zr[it][1], (uint32_t)zsh);
                const uint32_t d4 = zr[it][2] >> zsh;
                const int bo = zbo0 + (co0 + co) * m_cs;
                const unsigned long long kk = (((unsigned long long)zr[it][4] << 32) | zr[it][3]) >> (8 * (bo & 3));
                uint32_t dv[5], wn[5];
                dv[0] = d01 & 0xFFFFu; dv[1] = d01 >> 16; dv[2] = d23 & 0xFFFFu; dv[3] = d23 >> 16; dv[4] = d4 & 0xFFFFu;
#pragma unroll
                for (int w = 0; w < 5; ++w) wn[w] = (uint32_t)(kk >> (8 * w + 1)) & 3u;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    uint32_t v = 0;
                    if (xs == 0) {
                        // elements 2i, 2i+1 are the left and right pixel of window i
                        if (wn[i] == (uint32_t)zwant) v = dv[i];
                        if (wn[i] == (uint32_t)zwant + 1u) v = dv[i] << 16;
                    } else {
                        // element 2i is the right pixel of window i, element 2i+1 the left pixel of window i+1
                        if (wn[i] == (uint32_t)zwant + 1u) v = dv[i];
                        if (wn[i + 1] == (uint32_t)zwant) v |= dv[i + 1] << 16;
                    }
                    o[i] = v;
                }
            }
            o[0] &= k0; o[1] &= k1; o[2] &= k2; o[3] &= k3;
            *(uint4*)(Zl + (zg * BCO + ((co + zg) & (BCO - 1))) * 16) = make_uint4(o[0], o[1], o[2], o[3]);
            // the next group of the row finds this group's last dword in the table; the first group of a row finds zero
            if (z_gi + 1 < G && zg + 1 < NG) Zp[(zg + 1) * BCO + co] = o[3];
            if (z_gi == 0) Zp[zg * BCO + co] = 0u;
        }
    };

    // ---- multiply ---------------------------------------------------------------------------------------------
    // A step multiplies two groups (lanes 0-31 one, lanes 32-63 the next).  Per group: the deltas at the group's 8
    // positions for tap kx = 0 (a0), and the same row of deltas one and two elements earlier for kx = 1, 2 (a1, a2), against
    // the three patch rows ky = 0, 1, 2 at those positions.  The operands of the next filter row are read from LDS
    // before the matrix-core instructions of the current one are issued.
    const int co_l = wave_co * 32 + l32, ci_l = wave_ci * 32 + l32;
    constexpr int NSTEP = NG / 2 / WAVES_K;              // steps of one wavefront per chunk, at most
    auto multiply = [&](const unsigned char* Xb, int ngroups) {
        const int nsteps = (ngroups + 1) >> 1;
        if (wave_k >= nsteps) return;
        const unsigned char* xrow = Xb + ci_l * XSB;
        auto read_row = [&](int goff, int ky) { return *(const uint4*)(xrow + goff + ky * PWp * 2); };
        auto read_a = [&](int i) {
            const int g = 2 * (wave_k + WAVES_K * i) + hi;
            return *(const uint4*)(Zl + (g * BCO + ((co_l + g) & (BCO - 1))) * 16);
        };
        auto read_p = [&](int i) { return Zp[(2 * (wave_k + WAVES_K * i) + hi) * BCO + co_l]; };
        int gcur = gtab[2 * wave_k + hi];
        uint4 a_cur = read_a(0);
        uint32_t p_cur = read_p(0);
        uint4 r_cur = read_row(gcur, 0);
        for (int s = wave_k, i = 0; s < nsteps; s += WAVES_K, ++i) {
            // (the step after the last one reads a group slot that exists in LDS, and is not used)
            const int inext = i + 1 < NSTEP ? i + 1 : i;
            const int gnext = gtab[2 * (wave_k + WAVES_K * inext) + hi];
            const uint4 a1 = make_uint4(alignhalf(a_cur.x, p_cur), alignhalf(a_cur.y, a_cur.x), alignhalf(a_cur.z, a_cur.y), alignhalf(a_cur.w, a_cur.z));
            const uint4 a2 = make_uint4(p_cur, a_cur.x, a_cur.y, a_cur.z);
            const v8bf A0 = __builtin_bit_cast(v8bf, a_cur), A1 = __builtin_bit_cast(v8bf, a1), A2 = __builtin_bit_cast(v8bf, a2);
            uint4 a_next = a_cur;
            uint32_t p_next = p_cur;
#pragma unroll
            for (int ky = 0; ky < 3; ++ky) {
                uint4 r_next;
                if (ky < 2) r_next = read_row(gcur, ky + 1);
                else { r_next = read_row(gnext, 0); a_next = read_a(inext); p_next = read_p(inext); }
                __builtin_amdgcn_sched_barrier(0);     // keep these reads ahead of the matrix-core instructions below
                const v8bf B = __builtin_bit_cast(v8bf, r_cur);
                acc[3 * ky + 0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A0, B, acc[3 * ky + 0], 0, 0, 0);
                acc[3 * ky + 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A1, B, acc[3 * ky + 1], 0, 0, 0);
                acc[3 * ky + 2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A2, B, acc[3 * ky + 2], 0, 0, 0);
                r_cur = r_next;
            }
            a_cur = a_next; p_cur = p_next;
            gcur = gnext;
        }
    };

    __syncthreads();                                    // the cleared LDS is visible
    if (id0 < id1) {
        const int per_img = row_blocks * col_blocks;
        int ib = id0 / per_img, rb = (id0 - ib * per_img) / col_blocks, cb = id0 - ib * per_img - rb * col_blocks;
        Chunk cur = chunk_of(ib, rb, cb);
        issue_x(Xl0, cur);
        load_z(cur);
        int buf = 0;
        for (int id = id0;; ++id) {
            unsigned char* Xb = buf ? Xl1 : Xl0;
            __builtin_amdgcn_s_waitcnt(0x0F70);        // vmcnt(0): this wavefront's patch loads and delta registers have landed
            fixup_x(Xb, cur);
            store_z();
            __syncthreads();                            // chunk `id` is complete in LDS
            const bool more = id + 1 < id1;
            Chunk nxt = cur;
            if (more) {
                if (++cb == col_blocks) { cb = 0; if (++rb == row_blocks) { rb = 0; ++ib; } }
                nxt = chunk_of(ib, rb, cb);
                issue_x(buf ? Xl0 : Xl1, nxt);
                load_z(nxt);
            }
            multiply(Xb, cur.ni * cur.nr * G);
            if (!more) break;
            __syncthreads();                            // everybody is done with the deltas and the table of chunk `id`
            cur = nxt; buf ^= 1;
        }
    }

    // ---- combine the pixel-split wavefronts (fixed order), then store -----------------------------------------
    if (WAVES_K > 1) {
        __syncthreads();
        float* red = (float*)lds16;                     // [WAVES_CO*WAVES_CI][16][64]
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            if (wave_k == 1) {
#pragma unroll
                for (int i = 0; i < 16; ++i) red[((wave % (WAVES_CO * WAVES_CI)) * 16 + i) * 64 + lane] = acc[t][i];
            }
            __syncthreads();
            if (wave_k == 0) {
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[t][i] += red[((wave % (WAVES_CO * WAVES_CI)) * 16 + i) * 64 + lane];
            }
            __syncthreads();
        }
    }
    if (wave_k == 0) {
        const long long layer_params = (long long)a.Cout * a.Cin * 9;
        float* dst = a.splits > 1 ? a.scratch + ((long long)stack * a.splits + split) * layer_params
                                  : a.partial + (long long)stack * a.n_params + a.w_off;
        const int ci = ci0 + ci_l;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int co = co0 + wave_co * 32 + 8 * (i >> 2) + 4 * hi + (i & 3);
            if (co < a.Cout && ci < a.Cin) {
#pragma unroll
                for (int t = 0; t < 9; ++t) dst[((long long)co * a.Cin + ci) * 9 + t] = acc[t][i];
            }
        }
    }
}


namespace {

bool even_view(const View& v)
{
    return ((uintptr_t)v.p & 3) == 0 && !(v.pitch & 1) && !(v.cs & 1) && !(v.ns & 1) && !(v.ss & 1);
}

}  // namespace

// 16-bit maps, 3x3, stride 1, no bias, with or without the fused pool; every row of the input view on a 4-byte
// boundary (pairs of pixels travel as dwords), offsets inside one stack within 31 bits.
bool wgrad16_eligible(const ConvArgs& c)
{
    if (!c.bf16 || c.K != 3 || c.S != 1 || c.has_bias || c.Cout < 32 || c.Cin < 16) return false;
    if (c.pooled && ((c.Hc | c.Wc) & 1)) return false;
    if (!even_view(c.in) || ((uintptr_t)c.din.p & 3) || ((uintptr_t)c.mask.p & 3)) return false;
    const double img = (double)kW16Groups;              // a chunk spans at most this many images
    if (2.0 * (img * (double)c.in.ns + (double)c.Cin * (double)c.in.cs) >= 2.0e9) return false;
    if (2.0 * (img * (double)c.din.ns + (double)c.Cout * (double)c.din.cs) >= 2.0e9) return false;
    if (c.pooled && img * (double)c.mask.ns + (double)c.Cout * (double)c.mask.cs >= 2.0e9) return false;
    return true;
}

// c.rect = owned rectangle at the convolution output (before the pool); scratch holds the shares.
void wgrad16(const ConvArgs& c, float* scratch, hipStream_t s)
{
    Wgrad16Args a;
    a.in = c.in; a.din = c.din; a.mask = c.mask; a.own = c.rect;
    a.partial = c.partial; a.scratch = scratch; a.n_params = c.n_params; a.w_off = c.w_off;
    a.Cin = c.Cin; a.Cout = c.Cout; a.Hc = c.Hi; a.Wc = c.Wi; a.M = c.M; a.batch = c.batch;
    a.splits = c.wgrad_shares16;
    const int waves_ci = w16_waves_ci(c.Cin);
    const int BCI = 32 * waves_ci;
    const size_t lds = (size_t)2 * BCI * w16_row_bytes(waves_ci) + (size_t)kW16Groups * 64 * 20 + (size_t)kW16Groups * 4;
    const int tiles = ((c.Cout + 63) / 64) * ((c.Cin + BCI - 1) / BCI);
    a.gx = tiles; a.stacks = c.N * c.M;
    dim3 grid(xcd_grid(a.splits * a.stacks, a.gx)), block(256);
#define FTP_W16(WCI, HF) do { \
        static thread_local bool granted = false; \
        if (!granted) { (void)hipFuncSetAttribute((const void*)k_wgrad_mfma16<WCI, HF>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); granted = true; } \
        g_kernel_label = "k_wgrad_mfma16<" #WCI ", " #HF ">"; \
        hipLaunchKernelGGL((k_wgrad_mfma16<WCI, HF>), grid, block, lds, s, a); } while (0)
    if (waves_ci == 2) { if (c.pooled) FTP_W16(2, 1); else FTP_W16(2, 0); }
    else               { if (c.pooled) FTP_W16(1, 1); else FTP_W16(1, 0); }
#undef FTP_W16
}

}  // namespace ftp
