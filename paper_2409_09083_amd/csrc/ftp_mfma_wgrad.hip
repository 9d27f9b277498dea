// fp32 matrix-core (MFMA) per-stack filter gradient for gfx950.
//   dW[co][ci][tap] = sum over the batch and the stack's owned output pixels q of dZ[co][q] * X[ci][q + tap - P]
// is a GEMM with M = co, N = ci and the pixels as reduction dimension, one accumulator tile per tap.
// A workgroup (4 wavefronts) owns a 32*WAVES_CO x 32*WAVES_CI block of (co, ci) for one stack and one
// share of the batch.  Per step it stages TI images x TR rows of the owned rectangle in LDS, pixel-major
// (channel contiguous) so that v_mfma_f32_32x32x2_f32 finds A[m = co][k = pixel] and B[k = pixel][n = ci]
// at consecutive addresses: dZ as [pixel][co], X as [(row, column) incl. filter halo][ci].
// Rows are padded to an even number of pixels (dZ = 0 there) because one MFMA consumes two pixels.
// HALF: 0 = the deltas sit at the resolution of the owned rectangle; 1 = a pool follows the convolution: the
// rectangle is at the convolution output, the deltas at pooled resolution, and a pixel receives its window's delta
// only if it is the window's winner; 2 = stride-2 convolution: the rectangle is the stack's owned part of the
// *input* map and pixel (y, x) carries delta (y/2, x/2) if both are even, else zero (the filter gradient of a strided
// convolution is the stride-1 one of the deltas with zeros in between; three quarters of the products are zero; no
// longer launched); 3 = stride-2 convolution run over the stack's owned *output* pixels: pixel (y, x) reads the
// patch of the input map at (2y + ky, 2x + kx), no zeros are multiplied, the patch of a chunk is four times as large
// (fp32 arithmetic for both storage types: 16-bit maps arrive one element per dword and are widened at the read).
// fp32 maps: the patch of X does not pass through registers.  It goes HBM -> LDS with buffer_load_dword ... lds, one
// element per lane, channel-major ([ci][patch position], odd channel stride), positions outside the map from
// out-of-range offsets (= 0); the deltas still go through registers (masking, pool routing), loaded during the
// previous chunk's multiply.
// 16-bit (bfloat) maps multiply with v_mfma_f32_32x32x8_bf16_1k: 8 pixels per instruction (lanes 0-31 the first 4,
// lanes 32-63 the next 4), counted through the chunk's pixel list; a small table in LDS gives each pixel's patch
// position.  The staged values are widened bfloats, so taking their upper halves back is exact.
// TROWS: filter rows per workgroup (5x5: 2, 7x7: 1, else all): one accumulator tile per tap has to fit the registers,
// so larger filters are split over blockIdx.x, each part staging the same chunks.
#include "ftp_device.h"
#include "ftp_launch.h"
#include <type_traits>

namespace ftp {

typedef float v16f __attribute__((ext_vector_type(16)));

// LDS positions of one staged chunk: pixels of dZ, patch positions of X (a multiple of 64).
constexpr int kWgradZPos = 64;                         // the limits wgrad_chunks() cuts to: this and wgrad_xpos(P)

template <typename T, int K, int WAVES_CO, int WAVES_CI, int HALF, int TROWS>
__global__ void __launch_bounds__(256, 2)
k_wgrad_mfma(MfmaWgradArgs a)
{
    constexpr bool POOL = HALF == 1;
    constexpr bool BF = sizeof(T) == 2 && HALF != 3;   // 16-bit maps on the bfloat matrix cores, staged through registers
    constexpr bool DL = !BF;                           // fp32 arithmetic: the patch is loaded straight into LDS (16-bit maps: the
                                                       // output-pixel form of stride 2 only, an element a dword, widened at the read)
    constexpr unsigned ES = sizeof(T);
    constexpr int S = HALF == 3 ? 2 : 1;               // patch positions per chunk pixel and dimension
    constexpr bool HALF_RES = HALF == 1 || HALF == 2;  // the deltas sit at half the resolution of the rectangle
    constexpr int WAVES_K = 4 / (WAVES_CO * WAVES_CI);
    constexpr int KK = K * K, P = K / 2, NTAP = TROWS * K;
    constexpr int BCO = 32 * WAVES_CO, BCI = 32 * WAVES_CI;
    constexpr int ZP = BCO + 1, XP = BCI + 1;          // odd strides: conflict-free transposing writes
    constexpr int NZ = BCO / 4, NX = BCI / 4;          // channels each wavefront stages
    constexpr int ZPOS = kWgradZPos, XPOS = wgrad_xpos(P, S), XPASS = XPOS / 64;
    constexpr int XS = XPOS + 1;                       // DL: dwords between the patch rows of two channels

    extern __shared__ float lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // uniform: keeps the loop control scalar
    const int wave_co = wave % WAVES_CO, wave_ci = (wave / WAVES_CO) % WAVES_CI, wave_k = wave / (WAVES_CO * WAVES_CI);
    const int hi = lane >> 5, l32 = lane & 31;
    // (block, share, stack), block fastest, in XCD order: the blocks of one stack and share read the same maps
    int vgroup, bx;
    if (!xcd_order(a.splits * a.stacks, a.gx, vgroup, bx)) return;
    const int split = vgroup % a.splits;
    const int stack = vgroup / a.splits, ti = stack / a.M, tj = stack % a.M;
    const int x0 = a.own.x0[tj], x1 = a.own.x1[tj], y0 = a.own.y0[ti], y1 = a.own.y1[ti];
    const int rw = x1 - x0 + 1, rh = y1 - y0 + 1;
    const int tiles_ci = (a.Cin + BCI - 1) / BCI, tiles = tiles_ci * ((a.Cout + BCO - 1) / BCO);
    const int tile = TROWS == K ? bx : bx % tiles;
    const int trow0 = TROWS == K ? 0 : (bx / tiles) * TROWS;       // first filter row of this workgroup
    const int co0 = (tile / tiles_ci) * BCO, ci0 = (tile % tiles_ci) * BCI;

    // Chunk geometry of this stack: TI images x TR rows x TC columns of the owned rectangle, at most ZPOS
    // pixels (rows padded to an even length TCp) and at most XPOS patch positions.  The stack's chunk list
    // (image block, row block, column block) is cut into a.splits contiguous shares.
    const WgradChunks wc = wgrad_chunks(rw, rh, a.batch, P, S);
    const int col_blocks = wc.col_blocks, TC = wc.TC, TCp = wc.TCp, PW = wc.PW, TR = wc.TR, row_blocks = wc.row_blocks, TI = wc.TI;
    const int id0 = (int)((long long)split * wc.total / a.splits), id1 = (int)((long long)(split + 1) * wc.total / a.splits);
    float* Zl = lds;                                   // [pixel][ZP]
    float* Xl = lds + ZPOS * ZP;                       // [patch position][XP]; DL: [ci][XS]
    int* posl = (int*)(Xl + XPOS * XP);                // bfloat path: [pixel] -> XP * patch position of its tap (0, 0)

    v16f acc[NTAP];
#pragma unroll
    for (int t = 0; t < NTAP; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[t][i] = 0.0f;

    const int co_l = wave_co * 32 + l32, ci_l = wave_ci * 32 + l32;

    struct Chunk { int n0, yb, xb, ni, nr, nc; };
    auto chunk_at = [&](int ib, int rb, int cb) {
        Chunk c;
        c.n0 = ib * TI; c.ni = (a.batch - c.n0) < TI ? (a.batch - c.n0) : TI;
        c.yb = y0 + rb * TR; c.nr = (y1 - c.yb + 1) < TR ? (y1 - c.yb + 1) : TR;
        c.xb = x0 + cb * TC; c.nc = (x1 - c.xb + 1) < TC ? (x1 - c.xb + 1) : TC;
        return c;
    };

    // Registers that carry one chunk from HBM to LDS.  Lane -> position (pixel of dZ, patch position of X,
    // both row-major over the chunk), wavefront -> every fourth channel; all loads are independent, so they are in flight
    // together.  16-bit maps: the loads are unconditional (clamped addresses) and what must be zero is zeroed at the LDS
    // write; fp32 maps: a lane that has nothing to stage loads from beyond the buffer's records (= 0).  zinfo: bit 0 position exists, bit 1 padding column, bits 2-3 the pixel's place in its pool
    // window.  xinfo: per pass bit 0 position exists, bit 1 inside the map.
    // zinfo bit 4: the position lies in the pixel list rounded up to a multiple of 8 (bfloat path; zero if it does not
    // exist); zpos: XP * patch position of the pixel.
    uint32_t zm[NZ]; float zg[NZ]; float xg[DL ? 1 : XPASS][DL ? 1 : NX];
    int zinfo = 0, xinfo = 0, zpos = 0;

    // fp32 path: which (image, row, column) of a chunk a lane stages never changes from chunk to chunk - chunks of
    // several images hold whole rectangles, all others one image - so the divisions are done once, here.  (While the
    // other workgroup's wavefront keeps this SIMD's matrix cores busy, every vector-ALU instruction of the staging code
    // waits for a gap between its instructions: the per-chunk part is kept to a few of them.)
    int z_il = 0, z_r = 0, z_c = 0;
    int x_il[DL ? XPASS : 1], x_r[DL ? XPASS : 1], x_c[DL ? XPASS : 1];
    if constexpr (DL) {
        const int zrow = lane / TCp;
        z_c = lane - zrow * TCp;
        if (TI > 1) { z_il = zrow / rh; z_r = zrow - z_il * rh; } else { z_r = zrow; }
        const int nph_all = S * rh + 2 * P;
#pragma unroll
        for (int pass = 0; pass < XPASS; ++pass) {
            const int pp = lane + 64 * pass;
            const int prow = pp / PW;
            x_c[pass] = pp - prow * PW;
            if (TI > 1) { x_il[pass] = prow / nph_all; x_r[pass] = prow - x_il[pass] * nph_all; } else { x_il[pass] = 0; x_r[pass] = prow; }
        }
    }
    // whole blocks of channels (every layer of the paper's networks): no per-channel range checks in the staging code
    const bool co_full = co0 + BCO <= a.Cout, ci_full = ci0 + BCI <= a.Cin;

    // fp32: buffer loads - one 32-bit offset per lane, the channel as a scalar offset; a lane without a pixel (beyond
    // the chunk, padding column) loads from beyond the buffer's records and receives the zero it has to stage
    auto load_dl = [&](const Chunk& c, auto full) {
        if constexpr (DL) {
            const bool ok = z_il < c.ni && z_r < c.nr && z_c < c.nc;
            const int qy = c.yb + z_r, qx = c.xb + z_c;
            const int sy = HALF_RES ? (qy >> 1) : qy, sx = HALF_RES ? (qx >> 1) : qx;
            zinfo = (((qy & 1) << 1) | (qx & 1)) << 2;
            const T* gbase = (const T*)a.din.p + (long long)stack * a.din.ss + (long long)c.n0 * a.din.ns;
            const __amdgpu_buffer_rsrc_t grsrc = __builtin_amdgcn_make_buffer_rsrc((void*)gbase, (short)0, 0x7FFFFFFF, 0x00020000);
            const unsigned gvo = ok ? ES * (unsigned)(z_il * (int)a.din.ns + (sy - a.din.y0[ti]) * a.din.pitch + (sx - a.din.x0[tj])) : 0x80000000u;
            const uint8_t* mbase = (const uint8_t*)a.mask.p + (long long)stack * a.mask.ss + (long long)c.n0 * a.mask.ns;
            const __amdgpu_buffer_rsrc_t mrsrc = __builtin_amdgcn_make_buffer_rsrc((void*)mbase, (short)0, 0x7FFFFFFF, 0x00020000);
            const unsigned mvo = (POOL && ok) ? (unsigned)(z_il * (int)a.mask.ns + (sy - a.mask.y0[ti]) * a.mask.pitch + (sx - a.mask.x0[tj])) : 0x80000000u;
#pragma unroll
            for (int k = 0; k < NZ; ++k) {
                const int ch = wave + 4 * k;
                unsigned gv = gvo, mv = mvo;
                if constexpr (!decltype(full)::value)
                    if (co0 + ch >= a.Cout) { gv = 0x80000000u; mv = 0x80000000u; }
                zm[k] = POOL ? (uint32_t)__builtin_amdgcn_raw_buffer_load_b8(mrsrc, mv, (unsigned)((co0 + ch) * (int)a.mask.cs), 0) : 0u;      // only the pool winner is needed
                if constexpr (sizeof(T) == 4) zg[k] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(grsrc, gv, 4u * (unsigned)((co0 + ch) * (int)a.din.cs), 0));
                else                          zg[k] = __uint_as_float((uint32_t)__builtin_amdgcn_raw_buffer_load_b16(grsrc, gv, 2u * (unsigned)((co0 + ch) * (int)a.din.cs), 0) << 16);
            }
        }
    };
    auto load = [&](const Chunk& c) {
        if constexpr (DL) {
            if (co_full) load_dl(c, std::true_type{}); else load_dl(c, std::false_type{});
        } else {
            const int npos = c.ni * c.nr * TCp;
            const bool ok = lane < npos;
            const int p = ok ? lane : 0;
            const int row = p / TCp, zc = p - row * TCp;
            const int il = row / c.nr, r = row - il * c.nr;
            const int qy = c.yb + r, qx = c.xb + (zc < c.nc ? zc : c.nc - 1);
            const int sy = HALF_RES ? (qy >> 1) : qy, sx = HALF_RES ? (qx >> 1) : qx;
            zinfo = (ok ? 1 : 0) | (zc >= c.nc ? 2 : 0) | ((((qy & 1) << 1) | (qx & 1)) << 2) | (lane < ((npos + 7) & ~7) ? 16 : 0);
            zpos = ok ? ((il * (c.nr + 2 * P) + r) * PW + zc) * XP : 0;
            {
                const uint8_t* mp = at<uint8_t>(a.mask, stack, ti, tj, c.n0 + il, 0, sy, sx);
                const T* gp = at<T>(a.din, stack, ti, tj, c.n0 + il, 0, sy, sx);
#pragma unroll
                for (int k = 0; k < NZ; ++k) {
                    const int ch = wave + 4 * k;
                    const int co = co0 + ch < a.Cout ? co0 + ch : a.Cout - 1;
                    zm[k] = POOL ? (uint32_t)mp[(long long)co * a.mask.cs] : 0u;      // only the pool winner is needed
                    zg[k] = ld(gp + (long long)co * a.din.cs);
                }
            }
        }
        if constexpr (!DL) {
            const int nph = c.nr + 2 * P;
            const int npos = c.ni * nph * PW;
            xinfo = 0;
#pragma unroll
            for (int pass = 0; pass < XPASS; ++pass) {
                if (pass * 64 < npos) {
                    const int pp = lane + 64 * pass;
                    const bool ok = pp < npos;
                    const int p = ok ? pp : 0;
                    const int prow = p / PW, xc = p - prow * PW;
                    const int il = prow / nph, r = prow - il * nph;
                    const int gy = c.yb - P + r, gx = c.xb - P + xc;
                    const bool inside = xc < c.nc + 2 * P && gy >= 0 && gy < a.Hc && gx >= 0 && gx < a.Wc;
                    xinfo |= ((ok ? 1 : 0) | (inside ? 2 : 0)) << (2 * pass);
                    const T* xp = at<T>(a.in, stack, ti, tj, c.n0 + il, 0, inside ? gy : y0, inside ? gx : x0);
#pragma unroll
                    for (int k = 0; k < NX; ++k) {
                        const int ch = wave + 4 * k;
                        const int ci = ci0 + ch < a.Cin ? ci0 + ch : a.Cin - 1;
                        xg[pass][k] = ld(xp + (long long)ci * a.in.cs);
                    }
                }
            }
        }
    };

    auto store = [&]() {
        if constexpr (DL) {
            // (lanes without a pixel received zeros; those beyond the chunk write them where nothing is read)
            float* zdst = Zl + lane * ZP;
            const uint32_t code = (uint32_t)(zinfo >> 2) & 3u;
#pragma unroll
            for (int k = 0; k < NZ; ++k) {
                float v = zg[k];                                       // the delta maps hold dLoss/dZ
                if (POOL && ((zm[k] >> 1) & 3u) != code) v = 0.0f;
                zdst[wave + 4 * k] = v;
            }
            return;
        }
        if (!DL) __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): every load of the chunk has landed
        if (zinfo & (BF ? 16 : 1)) {
            float* zdst = Zl + lane * ZP;
            const int code = (zinfo >> 2) & 3;
#pragma unroll
            for (int k = 0; k < NZ; ++k) {
                const int ch = wave + 4 * k;
                float v = zg[k];                                       // the delta maps hold dLoss/dZ
                if (POOL && ((zm[k] >> 1) & 3) != (uint32_t)code) v = 0.0f;
                if (HALF == 2 && code != 0) v = 0.0f;
                if ((zinfo & 2) || !(zinfo & 1) || co0 + ch >= a.Cout) v = 0.0f;
                zdst[ch] = v;
            }
            if (BF && wave == 0) posl[lane] = zpos;
        }
        if constexpr (!DL)
#pragma unroll
        for (int pass = 0; pass < XPASS; ++pass) {
            const int f = xinfo >> (2 * pass);
            if (f & 1) {
                float* xdst = Xl + (lane + 64 * pass) * XP;
#pragma unroll
                for (int k = 0; k < NX; ++k) {
                    const int ch = wave + 4 * k;
                    xdst[ch] = ((f & 2) && ci0 + ch < a.Cin) ? xg[pass][k] : 0.0f;
                }
            }
        }
    };

    // DL: one chunk's patch, HBM -> LDS.  Lane -> patch position (64 to an instruction), wavefront -> every fourth
    // channel.  Returns the number of load instructions this wavefront issued.
    auto issue_x_dl = [&](const Chunk& c, auto full) -> int {
        int issued = 0;
        if constexpr (DL) {
            const int nph = S * c.nr + 2 * P, npos = c.ni * nph * PW, ncn = S * c.nc + 2 * P;
            const T* base = (const T*)a.in.p + (long long)stack * a.in.ss + (long long)c.n0 * a.in.ns;
            const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)base, (short)0, 0x7FFFFFFF, 0x00020000);
            const int gy0 = S * c.yb - P, gx0 = S * c.xb - P;
#pragma unroll
            for (int pass = 0; pass < XPASS; ++pass) {
                if (pass * 64 < npos) {
                    const int gy = gy0 + x_r[pass], gx = gx0 + x_c[pass];
                    const bool inside = x_il[pass] < c.ni && x_r[pass] < nph && x_c[pass] < ncn && (unsigned)gy < (unsigned)a.Hc && (unsigned)gx < (unsigned)a.Wc;
                    const unsigned vo = inside ? ES * (unsigned)(x_il[pass] * (int)a.in.ns + (gy - a.in.y0[ti]) * a.in.pitch + (gx - a.in.x0[tj])) : 0x80000000u;
#pragma unroll
                    for (int k = 0; k < NX; ++k) {
                        const int ch = wave + 4 * k;
                        unsigned v = vo;
                        if constexpr (!decltype(full)::value)
                            if (ci0 + ch >= a.Cin) v = 0x80000000u;
                        const unsigned so = ES * (unsigned)((ci0 + ch) * (int)a.in.cs);
                        if constexpr (sizeof(T) == 4) __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (__attribute__((address_space(3))) void*)(Xl + ch * XS + pass * 64), 4, v, so, 0, 0);
                        else                          __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (__attribute__((address_space(3))) void*)(Xl + ch * XS + pass * 64), 2, v, so, 0, 0);
                    }
                    issued += NX;
                }
            }
        }
        return issued;
    };
    auto issue_x = [&](const Chunk& c) -> int {
        if constexpr (DL) return ci_full ? issue_x_dl(c, std::true_type{}) : issue_x_dl(c, std::false_type{});
        return 0;
    };
    // waits until at most `n` of this wavefront's loads are outstanding (loads return in order)
    auto wait_vm = [&](int n) {
        switch (n) {
            case 0: __builtin_amdgcn_s_waitcnt(0x0F70); break;
            case 8: __builtin_amdgcn_s_waitcnt(0x0F78); break;
            case 16: __builtin_amdgcn_s_waitcnt(0x4F70); break;
            case 24: __builtin_amdgcn_s_waitcnt(0x4F78); break;
            case 32: __builtin_amdgcn_s_waitcnt(0x8F70); break;
            case 40: __builtin_amdgcn_s_waitcnt(0x8F78); break;
            case 48: __builtin_amdgcn_s_waitcnt(0xCF70); break;
            default: __builtin_amdgcn_s_waitcnt(0x0F70); break;
        }
    };

    auto multiply = [&](const Chunk& c) {
        if constexpr (BF) {
            typedef short v4s __attribute__((ext_vector_type(4)));
            const int nblk = (c.ni * c.nr * TCp + 7) >> 3;
            // wavefronts that share a (co, ci) tile take alternate blocks of 8 pixels
            for (int b = wave_k; b < nblk; b += WAVES_K) {
                const int4 po = *(const int4*)(posl + 8 * b + 4 * hi);
                const float* zp = Zl + (8 * b + 4 * hi) * ZP + co_l;
                const uint32_t z0 = __float_as_uint(zp[0]), z1 = __float_as_uint(zp[ZP]), z2 = __float_as_uint(zp[2 * ZP]), z3 = __float_as_uint(zp[3 * ZP]);
                // upper halves of two dwords -> one dword of two bfloats
                const uint2 av = make_uint2(__builtin_amdgcn_perm(z1, z0, 0x07060302u), __builtin_amdgcn_perm(z3, z2, 0x07060302u));
                const float* xb = Xl + ci_l;
#pragma unroll
                for (int t = 0; t < NTAP; ++t) {
                    if (TROWS != K && trow0 + t / K >= K) break;
                    const int off = ((trow0 + t / K) * PW + (t % K)) * XP;
                    const uint32_t x0 = __float_as_uint(xb[po.x + off]), x1 = __float_as_uint(xb[po.y + off]);
                    const uint32_t x2 = __float_as_uint(xb[po.z + off]), x3 = __float_as_uint(xb[po.w + off]);
                    const uint2 bv = make_uint2(__builtin_amdgcn_perm(x1, x0, 0x07060302u), __builtin_amdgcn_perm(x3, x2, 0x07060302u));
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(__builtin_bit_cast(v4s, av), __builtin_bit_cast(v4s, bv), acc[t], 0, 0, 0);
                }
            }
            return;
        }
        const int nrows = c.ni * c.nr, nph = S * c.nr + 2 * P, ncp = (c.nc + 1) & ~1;
        for (int rr = 0; rr < nrows; ++rr) {
            const int il = rr / c.nr, r = rr - il * c.nr;
            const float* zrow = Zl + (rr * TCp + hi) * ZP + co_l;
            const float* xrow = DL ? Xl + ci_l * XS + (il * nph + S * r) * PW + S * hi : Xl + ((il * nph + r) * PW + hi) * XP + ci_l;
            // wavefronts that share a (co, ci) tile take alternate pixel pairs of every row
            for (int xp = 2 * wave_k; xp < ncp; xp += 2 * WAVES_K) {
                const float av = zrow[xp * ZP];
#pragma unroll
                for (int t = 0; t < NTAP; ++t) {
                    if (TROWS != K && trow0 + t / K >= K) break;           // (the last part of a split filter may be short)
                    float bv = xrow[((trow0 + t / K) * PW + S * xp + (t % K)) * (DL ? 1 : XP)];
                    if constexpr (DL && sizeof(T) == 2) bv = __uint_as_float(__float_as_uint(bv) << 16);      // (a 16-bit element in the lower half of its dword)
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[t], 0, 0, 0);
                }
            }
        }
    };

    // The next chunk travels from HBM into registers while the matrix cores work on the current one.
    if (id0 < id1) {
        int id = id0;
        int ib = id / (row_blocks * col_blocks), rem = id - ib * (row_blocks * col_blocks);
        int rb = rem / col_blocks, cb = rem - rb * col_blocks;
        Chunk cur = chunk_at(ib, rb, cb);
        load(cur);
        for (;;) {
            __syncthreads();                            // the previous chunk has been consumed
            if constexpr (DL) {
                // the patch loads start first; the deltas (loaded during the previous multiply) are stored while they fly
                const int nx = issue_x(cur);
                wait_vm(nx);
                store();
                __builtin_amdgcn_s_waitcnt(0x0F70);    // vmcnt(0): this wavefront's part of the patch has landed
            } else {
                store();
            }
            __syncthreads();
            if (++cb == col_blocks) { cb = 0; if (++rb == row_blocks) { rb = 0; ++ib; } }
            const bool more = ++id < id1;
            Chunk nxt = cur;
            if (more) { nxt = chunk_at(ib, rb, cb); load(nxt); }
            multiply(cur);
            if (!more) break;
            cur = nxt;
        }
    }

    // ---- combine the pixel-split wavefronts (fixed order), then store -----------------------------------------
    if (WAVES_K > 1) {
        __syncthreads();
        float* red = lds;                               // [WAVES_CO*WAVES_CI][16][64]
#pragma unroll
        for (int t = 0; t < NTAP; ++t)
#pragma unroll
            for (int k = 1; k < WAVES_K; ++k) {            // in wavefront order
                if (wave_k == k) {
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
        const long long layer_params = (long long)a.Cout * a.Cin * KK;
        float* dst = a.splits > 1 ? a.scratch + ((long long)stack * a.splits + split) * layer_params
                                  : a.partial + (long long)stack * a.n_params + a.w_off;
        const int ci = ci0 + ci_l;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int co = co0 + wave_co * 32 + 8 * (i >> 2) + 4 * hi + (i & 3);
            if (co < a.Cout && ci < a.Cin) {
#pragma unroll
                for (int t = 0; t < NTAP; ++t)
                    if (TROWS == K || trow0 + t / K < K) dst[((long long)co * a.Cin + ci) * KK + trow0 * K + t] = acc[t][i];
            }
        }
    }
}

// Sum of the batch shares of one layer's partial gradient, in share order.  V = 4: four consecutive parameters per thread,
// the shares' 16-byte loads four at a time in flight (layers whose parameter count is a multiple of 4); V = 1 otherwise.
template <int V>
__global__ void __launch_bounds__(256)
k_wgrad_splitk_reduce(const float* __restrict__ scratch, float* __restrict__ partial, long long layer_params, long long n_params,
                      long long w_off, int splits)
{
    const long long i = ((long long)blockIdx.x * blockDim.x + threadIdx.x) * V;
    const int stack = blockIdx.y;
    if (i >= layer_params) return;
    const float* src = scratch + (long long)stack * splits * layer_params + i;
    float* dst = partial + (long long)stack * n_params + w_off + i;
    if constexpr (V == 4) {
        auto ld4 = [&](int sh) { return *(const float4*)(src + (long long)sh * layer_params); };
        auto add = [](float4& v, const float4& b) { v.x += b.x; v.y += b.y; v.z += b.z; v.w += b.w; };
        float4 v = ld4(0);
        int sh = 1;
        for (; sh + 3 < splits; sh += 4) {
            const float4 b0 = ld4(sh), b1 = ld4(sh + 1), b2 = ld4(sh + 2), b3 = ld4(sh + 3);
            add(v, b0); add(v, b1); add(v, b2); add(v, b3);
        }
        for (; sh < splits; ++sh) add(v, ld4(sh));
        dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;     // (the layer's place in the parameter vector need not be 16-byte aligned)
    } else {
        float v = src[0];
        for (int sh = 1; sh < splits; ++sh) v += src[(long long)sh * layer_params];
        dst[0] = v;
    }
}

// Geometry: stride 1 with K = 1, 3 (with or without the fused pool), K = 5, 7 without; stride 2 with K = 1, 3.
bool mfma_wgrad_eligible(const ConvArgs& c)
{
    if (c.pooled && (c.S != 1 || c.K > 3)) return false;
    if (c.S == 2 && c.K > 3) return false;
    // (the fp32 patch loads address one stack's images with 32-bit byte offsets; a chunk spans at most 64 images)
    const bool direct = !c.bf16 || c.S == 2;           // (the patch goes straight into LDS)
    if (direct && 4.0 * (64.0 * (double)c.in.ns + (double)c.Cin * (double)c.in.cs) >= 2.0e9) return false;
    if (direct && 4.0 * (64.0 * (double)c.din.ns + (double)c.Cout * (double)c.din.cs) >= 2.0e9) return false;
    if (!c.bf16 && c.pooled && 64.0 * (double)c.mask.ns + (double)c.Cout * (double)c.mask.cs >= 2.0e9) return false;
    return !c.has_bias && c.Cout >= 32 && c.Cin >= 16;
}

// c.rect = owned rectangle at the convolution output (before the pool), c.own = owned rectangle at the convolution
// input (used for strided convolutions); scratch holds the batch shares.
void mfma_wgrad(const ConvArgs& c, float* scratch, hipStream_t s)
{
    MfmaWgradArgs a;
    // (stride 2: the gradient runs over the owned output pixels, pixel (y, x) reading the patch at (2y + ky, 2x + kx))
    const int half = c.pooled ? 1 : c.S == 2 ? 3 : 0;
    a.in = c.in; a.din = c.din; a.mask = c.mask; a.own = c.rect;
    a.partial = c.partial; a.scratch = scratch; a.n_params = c.n_params; a.w_off = c.w_off;
    a.Cin = c.Cin; a.Cout = c.Cout; a.Hc = c.Hi; a.Wc = c.Wi; a.slope = c.slope; a.M = c.M; a.batch = c.batch;
    a.splits = c.wgrad_shares;
    a.PK = kWgradZPos;
    // (64 input channels per workgroup where the patch of a 5x5 / 7x7 filter would not leave LDS for two workgroups)
    // (... or of the fourfold patch of the output-pixel form of stride 2)
    const int waves_ci = (c.Cin >= 64 && c.K <= 3 && half != 3) ? 2 : 1;
    // (32 output channels per workgroup for the 3x3 layers that have no more: all four wavefronts then split the pixels)
    const int waves_co = (c.Cout <= 32 && c.K == 3 && waves_ci == 1) ? 1 : 2;
    const int BCO = 32 * waves_co, BCI = 32 * waves_ci;
    // (+ the bfloat path's table of patch positions)
    // (the fp32 patch layout is [ci][positions + 1], the bfloat one [position][ci + 1] + the table of patch positions)
    const size_t lds = (c.bf16 && half != 3) ? ((size_t)kWgradZPos * (BCO + 1) + (size_t)wgrad_xpos(c.K / 2) * (BCI + 1) + kWgradZPos) * sizeof(float)
                              : ((size_t)kWgradZPos * (BCO + 1) + (size_t)BCI * (wgrad_xpos(c.K / 2, half == 3 ? 2 : 1) + 1)) * sizeof(float);
    const int tiles = ((c.Cout + BCO - 1) / BCO) * ((c.Cin + BCI - 1) / BCI);
    const int parts = c.K == 5 ? 3 : c.K == 7 ? 7 : 1;                 // filter rows 2 + 2 + 1, or one at a time
    a.gx = tiles * parts; a.stacks = c.N * c.M;
    dim3 grid(xcd_grid(a.splits * a.stacks, a.gx)), block(256);
    // more than 64 KB of dynamic LDS has to be granted per kernel, once
#define FTP_WG1(TT, TN, KK, WCO, WCI, HF, TR) do { \
        static thread_local bool granted = false; \
        if (!granted) { (void)hipFuncSetAttribute((const void*)k_wgrad_mfma<TT, KK, WCO, WCI, HF, TR>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); granted = true; } \
        g_kernel_label = "k_wgrad_mfma<" TN ", " #KK ", " #WCO ", " #WCI ", " #HF ", " #TR ">"; \
        hipLaunchKernelGGL((k_wgrad_mfma<TT, KK, WCO, WCI, HF, TR>), grid, block, lds, s, a); } while (0)
#define FTP_WG(KK, WCO, WCI, HF, TR) do { if (c.bf16) FTP_WG1(bf16_t, "unsigned short", KK, WCO, WCI, HF, TR); else FTP_WG1(float, "float", KK, WCO, WCI, HF, TR); } while (0)
    if (c.K == 7) FTP_WG(7, 2, 1, 0, 1);
    else if (c.K == 5) FTP_WG(5, 2, 1, 0, 2);
    else if (c.K == 3) {
        if (half == 3)          { if (waves_co == 1) FTP_WG(3, 1, 1, 3, 3); else FTP_WG(3, 2, 1, 3, 3); }
        else if (waves_co == 1) { if (half == 1) FTP_WG(3, 1, 1, 1, 3); else FTP_WG(3, 1, 1, 0, 3); }
        else if (waves_ci == 2) { if (half == 1) FTP_WG(3, 2, 2, 1, 3); else FTP_WG(3, 2, 2, 0, 3); }
        else                    { if (half == 1) FTP_WG(3, 2, 1, 1, 3); else FTP_WG(3, 2, 1, 0, 3); }
    } else {
        if (half == 3)     FTP_WG(1, 2, 1, 3, 1);
        else if (waves_ci == 2) { if (half == 1) FTP_WG(1, 2, 2, 1, 1); else FTP_WG(1, 2, 2, 0, 1); }
        else               { if (half == 1) FTP_WG(1, 2, 1, 1, 1); else FTP_WG(1, 2, 1, 0, 1); }
    }
#undef FTP_WG
#undef FTP_WG1
}

// Sums the `shares` partial results one of the filter-gradient kernels left in the scratch area into the layer's place
// in the per-stack gradient vectors, in share order.
void wgrad_share_sum(const ConvArgs& c, const float* scratch, int shares, hipStream_t s)
{
    const long long lp = (long long)c.Cout * c.Cin * c.K * c.K;
    g_kernel_label = "k_wgrad_splitk_reduce";
    // (the share scratch is 256-byte aligned, so with a parameter count that is a multiple of 4 every share's slice is too)
    if (lp % 4 == 0 && ((uintptr_t)scratch & 15) == 0) {
        dim3 g2((unsigned)((lp / 4 + 255) / 256), c.N * c.M);
        hipLaunchKernelGGL(k_wgrad_splitk_reduce<4>, g2, dim3(256), 0, s, scratch, c.partial, lp, c.n_params, c.w_off, shares);
    } else {
        dim3 g2((unsigned)((lp + 255) / 256), c.N * c.M);
        hipLaunchKernelGGL(k_wgrad_splitk_reduce<1>, g2, dim3(256), 0, s, scratch, c.partial, lp, c.n_params, c.w_off, shares);
    }
}

}  // namespace ftp
