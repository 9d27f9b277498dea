// Per-stack filter gradient of 3x3 stride-1 convolutions over 16-bit (bfloat) maps on the matrix cores of gfx950
// (Sec. 4.1: the filter gradient of a tile is the correlation of its input map with the delta map of its output, summed
// over the batch and over the pixels the tile owns):
//   dW[co][ci][tap] = sum over images and owned output pixels q of dZ[co][q] * X[ci][q + tap - 1]
// is a GEMM with M = co, N = ci and the pixels as reduction dimension, one accumulator tile per tap.
//
// v_mfma_f32_32x32x16_bf16 takes, per lane, 8 consecutive reduction elements of one row of A and one column of B
// (A[m = lane%32][k = 8*(lane/32) + j], B[k = 8*(lane/32) + j][n = lane%32], j < 8).  With the pixels as reduction
// dimension and maps stored pixel-contiguous per channel, those 8 elements are 8 consecutive pixels of one row of the
// owned rectangle: 16 contiguous bytes of dZ, and for tap (ky, kx) 16 bytes of X that start kx elements further.
// So the maps stay packed (two bfloats to a dword) and channel-major in LDS, as they are in HBM:
//   X   HBM -> LDS with buffer_load ... lds, one dword (two neighbouring pixels) per lane, no registers in between;
//       dwords outside the map (zero padding) come from out-of-range offsets, which read as zero; where the map ends in
//       the middle of a dword the loading wavefront clears that one element afterwards.  The three taps of a filter
//       row are cut out of 6 loaded dwords, the odd ones with v_alignbit.
//   dZ  through registers (it needs per-pixel treatment: the rectangle's ragged end, and behind a pool the routing of
//       each pooled delta to its window's winner), written to LDS as [group of 8 pixels][co][16 bytes].
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
    constexpr int ZBYTES = NG * BCO * 16;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds16[];
    unsigned char* const Xl0 = lds16;
    unsigned char* const Xl1 = lds16 + XBUF;
    unsigned char* const Zl = lds16 + 2 * XBUF;           // [group][co (rotated by the group index)][8 bfloats]
    int* const gtab = (int*)(Zl + ZBYTES);                // [group] -> byte offset of its pixels' tap (0, 0) in a patch row (even floor)

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_co = wave % WAVES_CO, wave_ci = (wave / WAVES_CO) % WAVES_CI, wave_k = wave / (WAVES_CO * WAVES_CI);
    const int hi = lane >> 5, l32 = lane & 31;
    const int stack = blockIdx.z, ti = stack / a.M, tj = stack % a.M;
    const int x0 = a.own.x0[tj], x1 = a.own.x1[tj], y0 = a.own.y0[ti], y1 = a.own.y1[ti];
    const int rw = x1 - x0 + 1, rh = y1 - y0 + 1;
    const int tiles_ci = (a.Cin + BCI - 1) / BCI;
    const int co0 = (blockIdx.x / tiles_ci) * BCO, ci0 = (blockIdx.x % tiles_ci) * BCI;
    const int split = blockIdx.y;

    const Wgrad16Chunks wc = wgrad16_chunks(rw, rh, a.batch, w16_patch_elems(WAVES_CI));
    const int G = wc.G, PWp = wc.PWp, HW = wc.PWp >> 1;
    const int id0 = (int)((long long)split * wc.total / a.splits), id1 = (int)((long long)(split + 1) * wc.total / a.splits);

    // LDS starts as zeros: patch elements no load ever writes are multiplied with zero deltas only, and must be finite
    for (int i = tid; i < (2 * XBUF + ZBYTES + NG * 4) / 4; i += 256) ((uint32_t*)lds16)[i] = 0u;

    v16f acc[9];
#pragma unroll
    for (int t = 0; t < 9; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[t][i] = 0.0f;

    struct Chunk { int n0, ni, yb, nr, xb, nc; };
    auto chunk_at = [&](int id) {
        const int per_img = wc.row_blocks * wc.col_blocks;
        const int ib = id / per_img, rem = id - ib * per_img;
        const int rb = rem / wc.col_blocks, cb = rem - rb * wc.col_blocks;
        Chunk c;
        c.n0 = ib * wc.TI; c.ni = (a.batch - c.n0) < wc.TI ? (a.batch - c.n0) : wc.TI;
        c.yb = y0 + rb * wc.RB; c.nr = (y1 - c.yb + 1) < wc.RB ? (y1 - c.yb + 1) : wc.RB;
        c.xb = x0 + cb * wc.TC; c.nc = (x1 - c.xb + 1) < wc.TC ? (x1 - c.xb + 1) : wc.TC;
        return c;
    };
    // parity of the patch's first column in the input view: the even element of every loaded dword is the element
    // just before it when the start is odd (strides of the view are even, so this holds for every row and channel)
    auto patch_shift = [&](const Chunk& c) { return (c.xb - 1 - a.in.x0[tj]) & 1; };

    // ---- X: HBM -> LDS ------------------------------------------------------------------------------------------
    const bf16_t* const xstack = (const bf16_t*)a.in.p + (long long)stack * a.in.ss;
    auto issue_x = [&](unsigned char* Xb, const Chunk& c) {
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)(xstack + (long long)c.n0 * a.in.ns), (short)0, (int)kRecords16, 0x00020000);
        const int xs = patch_shift(c);
        const int prh = c.nr + 2, pdw = c.ni * prh * HW;
        const int na = c.xb - 1 > 0 ? c.xb - 1 : 0, nb = c.xb + c.nc < a.Wc ? c.xb + c.nc : a.Wc - 1;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (j * 64 < pdw) {
                const int p = j * 64 + lane;
                if (p < pdw) {                      // (lanes beyond the patch must not write into the next channel's row)
                    const int pr = p / HW, d = p - pr * HW;
                    const int il = pr / prh, lr = pr - il * prh;
                    const int y = c.yb - 1 + lr, mx = c.xb - 1 - xs + 2 * d;
                    unsigned vo = kOob16;
                    if (y >= 0 && y < a.Hc && mx + 1 >= na && mx <= nb)
                        vo = 2u * (unsigned)(il * (int)a.in.ns + (y - a.in.y0[ti]) * a.in.pitch + (mx - a.in.x0[tj]));
#pragma unroll
                    for (int k = 0; k < BCI / 4; ++k) {
                        const int ci = wave + 4 * k;
                        const unsigned v = ci0 + ci < a.Cin ? vo : kOob16;
                        const unsigned so = 2u * (unsigned)((ci0 + ci) * (int)a.in.cs);
                        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, FTP_LDS_PTR(Xb + ci * XSB + j * 256), 4, v, so, 0, 0);
                    }
                }
            }
        }
    };
    // Where the needed columns end on the even element of a dword, the odd element came along: it is the zero padding
    // beyond the map's last column, or lies beyond everything a valid pixel reads.  The wavefront that loaded a channel
    // clears it (after its loads have landed).
    auto fixup_x = [&](unsigned char* Xb, const Chunk& c) {
        const int xs = patch_shift(c);
        const int nb = c.xb + c.nc < a.Wc ? c.xb + c.nc : a.Wc - 1;
        const int eb = nb - (c.xb - 1) + xs;                       // patch element of the last needed column
        if (eb & 1) return;
        const int prows = c.ni * (c.nr + 2), items = (BCI / 4) * prows;
        for (int it = lane; it < items; it += 64) {
            const int k = it / prows, pr = it - k * prows;
            *(uint16_t*)(Xb + (wave + 4 * k) * XSB + (pr * PWp + eb + 1) * 2) = (uint16_t)0;
        }
    };

    // ---- dZ: HBM -> registers -> LDS ----------------------------------------------------------------------------
    // thread -> group g = tid % 16 of the chunk and output channels tid / 16 + 16 * it
    const int zg = tid & 15, zco = tid >> 4;
    uint32_t zr[4][5];
    int zvalid = 0, zsh = 0, zwant = 0, zgoff = 0;
    const bf16_t* const zstack = (const bf16_t*)a.din.p + (long long)stack * a.din.ss;
    const uint8_t* const mstack = (const uint8_t*)a.mask.p + (long long)stack * a.mask.ss;
    auto load_z = [&](const Chunk& c) {
        const int ngroups = c.ni * c.nr * G;
        const int fr = zg / G, gi = zg - fr * G;
        const int il = fr / c.nr, r = fr - il * c.nr;
        const int c0 = 8 * gi;
        int valid = c.nc - c0; valid = valid > 8 ? 8 : valid;
        const bool exists = zg < ngroups && valid > 0;
        zvalid = exists ? valid : 0;
        zgoff = exists ? 2 * ((il * (c.nr + 2) + r) * PWp + c0) : 0;
        const __amdgpu_buffer_rsrc_t zrsrc = __builtin_amdgcn_make_buffer_rsrc((void*)(zstack + (long long)c.n0 * a.din.ns), (short)0, (int)kRecords16, 0x00020000);
        if (HALF == 0) {
            const int eo = il * (int)a.din.ns + (c.yb + r - a.din.y0[ti]) * a.din.pitch + (c.xb + c0 - a.din.x0[tj]);
            const int odd = eo & 1, nd = (odd + zvalid + 1) >> 1;
            zsh = odd * 16;
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                const int gco = co0 + zco + 16 * it;
                const bool ok = exists && gco < a.Cout;
                const unsigned base = 2u * (unsigned)((eo & ~1) + gco * (int)a.din.cs);
#pragma unroll
                for (int i = 0; i < 5; ++i) {
                    const int ii = i < nd ? i : nd - 1;
                    zr[it][i] = __builtin_amdgcn_raw_buffer_load_b32(zrsrc, ok ? base + 4u * (unsigned)ii : kOob16, 0, 0);
                }
            }
        } else {
            const __amdgpu_buffer_rsrc_t mrsrc = __builtin_amdgcn_make_buffer_rsrc((void*)(mstack + (long long)c.n0 * a.mask.ns), (short)0, (int)kRecords16, 0x00020000);
            const int py = (c.yb + r) >> 1, pc = (c.xb + c0) >> 1, nwin = (zvalid + 1) >> 1;
            zwant = 2 * ((c.yb + r) & 1);
            const int eo = il * (int)a.din.ns + (py - a.din.y0[ti]) * a.din.pitch + (pc - a.din.x0[tj]);
            const int odd = eo & 1, nd = (odd + nwin + 1) >> 1;
            zsh = odd * 16;
            const int bo0 = il * (int)a.mask.ns + (py - a.mask.y0[ti]) * a.mask.pitch + (pc - a.mask.x0[tj]);
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                const int gco = co0 + zco + 16 * it;
                const bool ok = exists && gco < a.Cout;
                const unsigned base = 2u * (unsigned)((eo & ~1) + gco * (int)a.din.cs);
#pragma unroll
                for (int i = 0; i < 3; ++i) {
                    const int ii = i < nd ? i : nd - 1;
                    zr[it][i] = __builtin_amdgcn_raw_buffer_load_b32(zrsrc, ok ? base + 4u * (unsigned)ii : kOob16, 0, 0);
                }
                const int bo = bo0 + gco * (int)a.mask.cs;
                const int ncd = ((bo & 3) + nwin + 3) >> 2;
                zr[it][3] = __builtin_amdgcn_raw_buffer_load_b32(mrsrc, ok ? (unsigned)(bo & ~3) : kOob16, 0, 0);
                zr[it][4] = __builtin_amdgcn_raw_buffer_load_b32(mrsrc, ok ? (unsigned)(bo & ~3) + (ncd > 1 ? 4u : 0u) : kOob16, 0, 0);
            }
        }
    };
    // element mask of output dword i of a group with `n` valid pixels
    auto keep = [](int n, int i) -> uint32_t { return n >= 2 * i + 2 ? 0xFFFFFFFFu : n == 2 * i + 1 ? 0x0000FFFFu : 0u; };
    auto store_z = [&](const Chunk& c) {
        if (tid < NG) gtab[zg] = zgoff;
        int bo0 = 0;
        if (HALF == 1) {
            const int fr = zg / G, gi = zg - fr * G;
            const int il = fr / c.nr, r = fr - il * c.nr;
            const int py = (c.yb + r) >> 1, pc = (c.xb + 8 * gi) >> 1;
            bo0 = il * (int)a.mask.ns + (py - a.mask.y0[ti]) * a.mask.pitch + (pc - a.mask.x0[tj]);
        }
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int co = zco + 16 * it;
            uint32_t o[4];
            if (HALF == 0) {
#pragma unroll
                for (int i = 0; i < 4; ++i) o[i] = __builtin_amdgcn_alignbit(zr[it][i + 1], zr[it][i], (uint32_t)zsh) & keep(zvalid, i);
            } else {
                // 4 pooled deltas and their 4 winner codes; window j feeds pixels 2j and 2j+1 of this row
                const uint32_t d01 = __builtin_amdgcn_alignbit(zr[it][1], zr[it][0], (uint32_t)zsh);
                const uint32_t d23 = __builtin_amdgcn_alignbit(zr[it][2], zr[it][1], (uint32_t)zsh);
                const int bo = bo0 + (co0 + co) * (int)a.mask.cs;
                const uint32_t cw = __builtin_amdgcn_alignbyte(zr[it][4], zr[it][3], (uint32_t)(bo & 3));
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t dj = ((j & 2) ? d23 : d01) >> ((j & 1) * 16) & 0xFFFFu;
                    const uint32_t win = (cw >> (8 * j + 1)) & 3u;
                    uint32_t v = 0;
                    if (win == (uint32_t)zwant) v = dj;
                    if (win == (uint32_t)zwant + 1u) v = dj << 16;
                    o[j] = v & keep(zvalid, j);
                }
            }
            *(uint4*)(Zl + (zg * BCO + ((co + zg) & (BCO - 1))) * 16) = make_uint4(o[0], o[1], o[2], o[3]);
        }
    };

    // ---- multiply ---------------------------------------------------------------------------------------------
    const int co_l = wave_co * 32 + l32, ci_l = wave_ci * 32 + l32;
    auto multiply = [&](const unsigned char* Xb, const Chunk& c) {
        const int nsteps = (c.ni * c.nr * G + 1) >> 1;
        const int xs = patch_shift(c);
        const unsigned char* xrow = Xb + ci_l * XSB;
        for (int s = wave_k; s < nsteps; s += WAVES_K) {
            const int g = 2 * s + hi;
            const int goff = gtab[g];
            const uint4 av = *(const uint4*)(Zl + (g * BCO + ((co_l + g) & (BCO - 1))) * 16);
            const v8bf A = __builtin_bit_cast(v8bf, av);
#pragma unroll
            for (int ky = 0; ky < 3; ++ky) {
                const unsigned char* rp = xrow + goff + ky * PWp * 2;
                const uint4 d = *(const uint4*)rp;
                const uint2 e = *(const uint2*)(rp + 16);
                uint4 t0, t1, t2;
                if (xs == 0) {
                    t0 = d;
                    t1 = make_uint4(alignhalf(d.y, d.x), alignhalf(d.z, d.y), alignhalf(d.w, d.z), alignhalf(e.x, d.w));
                    t2 = make_uint4(d.y, d.z, d.w, e.x);
                } else {
                    t0 = make_uint4(alignhalf(d.y, d.x), alignhalf(d.z, d.y), alignhalf(d.w, d.z), alignhalf(e.x, d.w));
                    t1 = make_uint4(d.y, d.z, d.w, e.x);
                    t2 = make_uint4(alignhalf(d.z, d.y), alignhalf(d.w, d.z), alignhalf(e.x, d.w), alignhalf(e.y, e.x));
                }
                acc[3 * ky + 0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, __builtin_bit_cast(v8bf, t0), acc[3 * ky + 0], 0, 0, 0);
                acc[3 * ky + 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, __builtin_bit_cast(v8bf, t1), acc[3 * ky + 1], 0, 0, 0);
                acc[3 * ky + 2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, __builtin_bit_cast(v8bf, t2), acc[3 * ky + 2], 0, 0, 0);
            }
        }
    };

    __syncthreads();                                    // the cleared LDS is visible
    if (id0 < id1) {
        Chunk cur = chunk_at(id0);
        issue_x(Xl0, cur);
        load_z(cur);
        int buf = 0;
        for (int id = id0;; ++id) {
            unsigned char* Xb = buf ? Xl1 : Xl0;
            __builtin_amdgcn_s_waitcnt(0x0F70);        // vmcnt(0): this wavefront's patch loads and delta registers have landed
            fixup_x(Xb, cur);
            store_z(cur);
            __syncthreads();                            // chunk `id` is complete in LDS
            const bool more = id + 1 < id1;
            Chunk nxt = cur;
            if (more) { nxt = chunk_at(id + 1); issue_x(buf ? Xl0 : Xl1, nxt); load_z(nxt); }
            multiply(Xb, cur);
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

// Sum of the shares of one layer's partial gradient, in share order.
__global__ void __launch_bounds__(256)
k_wgrad_mfma16_share_sum(const float* __restrict__ scratch, float* __restrict__ partial, long long layer_params, long long n_params,
                    long long w_off, int splits)
{
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const int stack = blockIdx.y;
    if (i >= layer_params) return;
    const float* src = scratch + (long long)stack * splits * layer_params + i;
    float v = src[0];
    for (int s = 1; s < splits; ++s) v += src[(long long)s * layer_params];
    partial[(long long)stack * n_params + w_off + i] = v;
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
    const size_t lds = (size_t)2 * BCI * w16_row_bytes(waves_ci) + (size_t)kW16Groups * 64 * 16 + (size_t)kW16Groups * 4;
    const int tiles = ((c.Cout + 63) / 64) * ((c.Cin + BCI - 1) / BCI);
    dim3 grid(tiles, a.splits, c.N * c.M), block(256);
#define FTP_W16(WCI, HF) do { \
        static bool granted = false; \
        if (!granted) { (void)hipFuncSetAttribute((const void*)k_wgrad_mfma16<WCI, HF>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); granted = true; } \
        g_kernel_label = "k_wgrad_mfma16<" #WCI ", " #HF ">"; \
        hipLaunchKernelGGL((k_wgrad_mfma16<WCI, HF>), grid, block, lds, s, a); } while (0)
    if (waves_ci == 2) { if (c.pooled) FTP_W16(2, 1); else FTP_W16(2, 0); }
    else               { if (c.pooled) FTP_W16(1, 1); else FTP_W16(1, 0); }
#undef FTP_W16
    if (a.splits > 1) {
        const long long lp = (long long)c.Cout * c.Cin * 9;
        dim3 g2((unsigned)((lp + 255) / 256), c.N * c.M);
        hipLaunchKernelGGL(k_wgrad_mfma16_share_sum, g2, dim3(256), 0, s, scratch, c.partial, lp, c.n_params, c.w_off, a.splits);
    }
}

}  // namespace ftp
