// Kernels for the thin first layer (a handful of input channels, e.g. the 3-channel image), gfx950.
// The layer is far from a dense contraction in its input-channel dimension, so
//  * the delta towards the image (3 output channels) is a coalesced, LDS-tiled direct convolution:
//    the dZ patch of 16 channels is staged once and every thread produces all input channels of a pixel;
//  * the filter gradient puts (input channel, tap) - 27 columns - on the N side of one 32x32 MFMA tile
//    and reduces over pixels, so the matrix cores are used without padding the 3 channels to 32.
#include "ftp_device.h"
#include "ftp_launch.h"
#include <algorithm>

namespace ftp {

typedef float v16f __attribute__((ext_vector_type(16)));

__device__ __forceinline__ bool in_rect_thin(const RectTab& r, int ti, int tj, int y, int x)
{
    return y >= r.y0[ti] && y <= r.y1[ti] && x >= r.x0[tj] && x <= r.x1[tj];
}

// dZ of one element from the delta and the owner's decision code (see ftp_direct.hip: delta_z).
// ---- forward of a K = 3 convolution with at most 4 input channels (+ leaky ReLU, + fused 2x2 pool) ---------------
// Workgroup = ntx x nty threads on one (stack, image); a thread produces one pool window (2 x 2 convolution outputs)
// or, without a pool, two neighbouring pixels, for every output channel in turn.  The input patch of the tile
// (all input channels, filter halo, zero outside the map) and the filter with its bias sit in LDS; a thread keeps
// its own 4 x 4 (or 3 x 4) patch per input channel in registers and reads the 9 * CI weights of an output channel
// as broadcast vectors.  A thread sees all channels of its pixel, so it writes the sign words itself.
constexpr int kThinFwdPatch = 1280, kThinFwdCout = 64;     // floats of one channel's patch; channels whose weights fit LDS

template <typename T, bool POOL, int CI>
__global__ void __launch_bounds__(256)
k_conv_fwd_thin(View in, View out, View mask, View osign, RectTab rt, RectTab own, const T* __restrict__ w,
                const T* __restrict__ bias, int Cin, int Cout, int Hc, int Wc, float slope, int M, int batch,
                int ntx, int nty, int tiles_x)
{
    constexpr int PH = POOL ? 4 : 3, PWD = 4, WR = 9 * CI;         // register patch rows / columns, weights per channel
    constexpr int SY = POOL ? 2 : 1, SX = 2;                        // convolution pixels per thread
    __shared__ __attribute__((aligned(16))) float xp[CI * kThinFwdPatch];
    __shared__ __attribute__((aligned(16))) float wl[kThinFwdCout * (WR + 1)];
    const int tid = threadIdx.x;
    const int stack = blockIdx.z / batch, n = blockIdx.z % batch;
    const int ti = stack / M, tj = stack % M;
    // the rectangle is in output coordinates (pooled if POOL); tiles of ntx x nty threads
    const int bx = blockIdx.x % tiles_x, by = blockIdx.x / tiles_x;
    const int OX = POOL ? 1 : 2;                                    // output pixels per thread along x
    const int ox0 = rt.x0[tj] + bx * ntx * OX, oy0 = rt.y0[ti] + by * nty;
    if (ox0 > rt.x1[tj] || oy0 > rt.y1[ti]) return;
    // convolution-resolution origin of the patch and its extent
    const int cx0 = ox0 * (POOL ? 2 : 1) - 1, cy0 = oy0 * SY - 1;
    const int PW = SX * ntx + 2, PHT = SY * nty + 2, PP = (PW + 1) & ~1;
    for (int i = tid; i < CI * PHT * PW; i += 256) {
        const int ci = i / (PHT * PW), rem = i - ci * (PHT * PW), r = rem / PW, q = rem - r * PW;
        const int y = cy0 + r, x = cx0 + q;
        // positions only pixels beyond the rectangle would read may lie outside the input view
        const int ylim = (rt.y1[ti] + 1) * SY, xlim = (rt.x1[tj] + 1) * (POOL ? 2 : 1);
        const bool okp = ci < Cin && y >= 0 && y < Hc && x >= 0 && x < Wc && y <= ylim && x <= xlim;
        xp[ci * kThinFwdPatch + r * PP + q] = okp ? ld(at<T>(in, stack, ti, tj, n, ci, y, x)) : 0.0f;
    }
    for (int i = tid; i < Cout * (WR + 1); i += 256) {
        const int co = i / (WR + 1), r = i - co * (WR + 1);
        float v = 0.0f;
        if (r < WR) { const int ci = r / 9, t = r - ci * 9; if (ci < Cin) v = ld(w + ((size_t)co * Cin + ci) * 9 + t); }
        else if (bias) v = ld(bias + co);
        wl[i] = v;
    }
    __syncthreads();
    const int tx = tid % ntx, ty = tid / ntx;
    if (ty >= nty) return;
    const int oy = oy0 + ty, ox = ox0 + tx * OX;
    float p[CI][PH][PWD];
#pragma unroll
    for (int ci = 0; ci < CI; ++ci)
#pragma unroll
        for (int r = 0; r < PH; ++r) {
            const float* row = xp + ci * kThinFwdPatch + (SY * ty + r) * PP + SX * tx;
            const float2 a = *(const float2*)row, b = *(const float2*)(row + 2);
            p[ci][r][0] = a.x; p[ci][r][1] = a.y; p[ci][r][2] = b.x; p[ci][r][3] = b.y;
        }
    const bool v0 = oy <= rt.y1[ti] && ox <= rt.x1[tj];
    const bool v1 = !POOL && oy <= rt.y1[ti] && ox + 1 <= rt.x1[tj];
    const bool o0 = v0 && in_rect_thin(own, ti, tj, oy, ox), o1 = v1 && in_rect_thin(own, ti, tj, oy, ox + 1);
    uint32_t s0 = 0, s1 = 0;
    for (int co = 0; co < Cout; ++co) {
        const float* wc = wl + co * (WR + 1);
        float acc[SY][SX];
#pragma unroll
        for (int a = 0; a < SY; ++a)
#pragma unroll
            for (int b = 0; b < SX; ++b) acc[a][b] = 0.0f;
#pragma unroll
        for (int ci = 0; ci < CI; ++ci)
#pragma unroll
            for (int ky = 0; ky < 3; ++ky)
#pragma unroll
                for (int kx = 0; kx < 3; ++kx) {
                    const float wv = wc[ci * 9 + ky * 3 + kx];
#pragma unroll
                    for (int a = 0; a < SY; ++a)
#pragma unroll
                        for (int b = 0; b < SX; ++b) acc[a][b] = fmaf(wv, p[ci][a + ky][b + kx], acc[a][b]);
                }
        const float bv = wc[WR];
        if (POOL) {
            // candidates are compared as the map would hold them; the first maximum in window order wins
            float best = stored(leaky(acc[0][0] + bv, slope), (const T*)nullptr);
            int bi = 0;
            const float c1 = stored(leaky(acc[0][1] + bv, slope), (const T*)nullptr);
            const float c2 = stored(leaky(acc[SY - 1][0] + bv, slope), (const T*)nullptr);
            const float c3 = stored(leaky(acc[SY - 1][1] + bv, slope), (const T*)nullptr);
            if (c1 > best) { best = c1; bi = 1; }
            if (c2 > best) { best = c2; bi = 2; }
            if (c3 > best) { best = c3; bi = 3; }
            if (v0) {
                st(at<T>(out, stack, ti, tj, n, co, oy, ox), best);
                if (o0) *at<uint8_t>(mask, stack, ti, tj, n, co, oy, ox) = (uint8_t)((bi << 1) | (best > 0.0f ? 1 : 0));
            }
            s0 |= (best > 0.0f ? 1u : 0u) << (co & 31);
        } else {
            const float a0 = stored(leaky(acc[0][0] + bv, slope), (const T*)nullptr);
            const float a1 = stored(leaky(acc[0][1] + bv, slope), (const T*)nullptr);
            if (v0) st(at<T>(out, stack, ti, tj, n, co, oy, ox), a0);
            if (v1) st(at<T>(out, stack, ti, tj, n, co, oy, ox + 1), a1);
            s0 |= (a0 > 0.0f ? 1u : 0u) << (co & 31);
            s1 |= (a1 > 0.0f ? 1u : 0u) << (co & 31);
        }
        if ((co & 31) == 31 || co == Cout - 1) {
            if (o0) *at<uint32_t>(osign, stack, ti, tj, n, co >> 5, oy, ox) = s0;
            if (o1) *at<uint32_t>(osign, stack, ti, tj, n, co >> 5, oy, ox + 1) = s1;
            s0 = s1 = 0;
        }
    }
}

bool thin_conv_fwd_eligible(const ConvArgs& a) { return a.K == 3 && a.Cin <= 4 && a.Cout <= kThinFwdCout; }

void thin_conv_fwd(const ConvArgs& a, hipStream_t s)
{
    int mw = 0, mh = 0;
    for (int t = 0; t < a.M; ++t) mw = mw > a.rect.x1[t] - a.rect.x0[t] + 1 ? mw : a.rect.x1[t] - a.rect.x0[t] + 1;
    for (int t = 0; t < a.N; ++t) mh = mh > a.rect.y1[t] - a.rect.y0[t] + 1 ? mh : a.rect.y1[t] - a.rect.y0[t] + 1;
    const int OX = a.pooled ? 1 : 2, SY = a.pooled ? 2 : 1;
    // threads along x cover the widest rectangle without a ragged last tile; at most 32 of them
    const int need_x = (mw + OX - 1) / OX;
    int tiles_x = (need_x + 31) / 32;
    const int ntx = (need_x + tiles_x - 1) / tiles_x;
    tiles_x = (need_x + ntx - 1) / ntx;
    int nty_max = 256 / ntx; if (nty_max > 32) nty_max = 32;
    const int tiles_y = (mh + nty_max - 1) / nty_max;
    const int nty = (mh + tiles_y - 1) / tiles_y;
    const int PP = (2 * ntx + 2 + 1) & ~1;
    if ((SY * nty + 2) * PP > kThinFwdPatch) { direct_conv_fwd(a, s); return; }
    dim3 grid(tiles_x * tiles_y, 1, a.N * a.M * a.batch), block(256);
    g_kernel_label = "k_conv_fwd_thin";
#define FTP_TF(T, PL, CI) hipLaunchKernelGGL((k_conv_fwd_thin<T, PL, CI>), grid, block, 0, s, a.in, a.out, a.mask, a.osign, a.rect, a.own, (const T*)a.w, (const T*)a.bias, a.Cin, a.Cout, a.Hc, a.Wc, a.slope, a.M, a.batch, ntx, nty, tiles_x)
#define FTP_TFC(T, PL) do { if (a.Cin <= 3) FTP_TF(T, PL, 3); else FTP_TF(T, PL, 4); } while (0)
    if (a.bf16) { if (a.pooled) FTP_TFC(bf16_t, true); else FTP_TFC(bf16_t, false); }
    else        { if (a.pooled) FTP_TFC(float, true); else FTP_TFC(float, false); }
#undef FTP_TFC
#undef FTP_TF
}

// ---- forward of the other thin first layers: 5x5 / 7x7 filters, stride 2 (no fused pool) ------------------------------
// Workgroup = 16 x 16 output pixels of one (stack, image), one pixel per thread.  The input patch of the tile (all
// input channels, zero outside the map) is staged in LDS once; a thread copies its own K x K x CI patch into registers
// and then walks the output channels, 16 at a time: their filters (+ bias) are staged in LDS as rows of whole float4s
// and read as broadcast vectors, K * K * CI multiply-adds per channel.  A thread sees all channels of its pixel, so
// it writes the sign words itself.
constexpr int kThinGenTile = 16, kThinGenCoc = 16;

template <typename T, int K, int S, int CI>
__global__ void __launch_bounds__(256)
k_conv_fwd_thin_gen(View in, View out, View osign, RectTab rt, RectTab own, const T* __restrict__ w,
                    const T* __restrict__ bias, int Cin, int Cout, int Hi, int Wi, float slope, int M, int batch, int tiles_x)
{
    constexpr int P = K / 2, KK = K * K, TS = kThinGenTile, COC = kThinGenCoc;
    constexpr int PD = S * (TS - 1) + K, PP = PD | 1;               // patch extent, odd pitch
    constexpr int WR = CI * KK, WRP = (WR + 1 + 3) & ~3;            // weights of a channel (+ bias), padded to float4s
    __shared__ __attribute__((aligned(16))) float xp[CI * PD * PP];
    __shared__ __attribute__((aligned(16))) float wl[COC * WRP];
    const int tid = threadIdx.x;
    const int stack = blockIdx.z / batch, n = blockIdx.z % batch;
    const int ti = stack / M, tj = stack % M;
    const int bx = blockIdx.x % tiles_x, by = blockIdx.x / tiles_x;
    const int ox0 = rt.x0[tj] + bx * TS, oy0 = rt.y0[ti] + by * TS;
    if (ox0 > rt.x1[tj] || oy0 > rt.y1[ti]) return;
    const int ix0 = S * ox0 - P, iy0 = S * oy0 - P;
    // positions only pixels beyond the rectangle would read may lie outside the input view
    const int ylim = S * rt.y1[ti] + P, xlim = S * rt.x1[tj] + P;
    for (int i = tid; i < CI * PD * PD; i += 256) {
        const int ci = i / (PD * PD), rem = i - ci * (PD * PD), r = rem / PD, q = rem - r * PD;
        const int y = iy0 + r, x = ix0 + q;
        const bool okp = ci < Cin && y >= 0 && y < Hi && x >= 0 && x < Wi && y <= ylim && x <= xlim;
        xp[(ci * PD + r) * PP + q] = okp ? ld(at<T>(in, stack, ti, tj, n, ci, y, x)) : 0.0f;
    }
    __syncthreads();
    const int tx = tid % TS, ty = tid / TS;
    const int oy = oy0 + ty, ox = ox0 + tx;
    float p[WR];
#pragma unroll
    for (int ci = 0; ci < CI; ++ci)
#pragma unroll
        for (int ky = 0; ky < K; ++ky)
#pragma unroll
            for (int kx = 0; kx < K; ++kx) p[ci * KK + ky * K + kx] = xp[(ci * PD + S * ty + ky) * PP + S * tx + kx];
    const bool v0 = oy <= rt.y1[ti] && ox <= rt.x1[tj];
    const bool o0 = v0 && in_rect_thin(own, ti, tj, oy, ox);
    uint32_t s0 = 0;
    for (int c0 = 0; c0 < Cout; c0 += COC) {
        __syncthreads();                               // the previous block's filters have been consumed
        for (int i = tid; i < COC * WRP; i += 256) {
            const int c = i / WRP, r = i - c * WRP;
            float v = 0.0f;
            if (c0 + c < Cout) {
                if (r < WR) { const int ci = r / KK, t = r - ci * KK; if (ci < Cin) v = ld(w + ((size_t)(c0 + c) * Cin + ci) * KK + t); }
                else if (r == WR && bias) v = ld(bias + c0 + c);
            }
            wl[i] = v;
        }
        __syncthreads();
        for (int c = 0; c < COC; ++c) {
            const int co = c0 + c;
            if (co >= Cout) break;
            const float4* w4 = (const float4*)(wl + c * WRP);
            float acc = 0.0f;
#pragma unroll
            for (int q = 0; q < WRP / 4; ++q) {
                const float4 wv = w4[q];
                if (4 * q + 0 < WR) acc = fmaf(wv.x, p[4 * q + 0 < WR ? 4 * q + 0 : 0], acc);
                if (4 * q + 1 < WR) acc = fmaf(wv.y, p[4 * q + 1 < WR ? 4 * q + 1 : 0], acc);
                if (4 * q + 2 < WR) acc = fmaf(wv.z, p[4 * q + 2 < WR ? 4 * q + 2 : 0], acc);
                if (4 * q + 3 < WR) acc = fmaf(wv.w, p[4 * q + 3 < WR ? 4 * q + 3 : 0], acc);
            }
            const float bv = wl[c * WRP + WR];
            const float a0 = stored(leaky(acc + bv, slope), (const T*)nullptr);
            if (v0) st(at<T>(out, stack, ti, tj, n, co, oy, ox), a0);
            s0 |= (a0 > 0.0f ? 1u : 0u) << (co & 31);
            if ((co & 31) == 31 || co == Cout - 1) {
                if (o0) *at<uint32_t>(osign, stack, ti, tj, n, co >> 5, oy, ox) = s0;
                s0 = 0;
            }
        }
    }
}

bool thin_conv_fwd_gen_eligible(const ConvArgs& a)
{
    return a.Cin <= 4 && !a.pooled && (a.K == 5 || a.K == 7 || (a.S == 2 && (a.K == 1 || a.K == 3))) && (a.S == 1 || a.S == 2);
}

void thin_conv_fwd_gen(const ConvArgs& a, hipStream_t s)
{
    int mw = 0, mh = 0;
    for (int t = 0; t < a.M; ++t) mw = std::max(mw, a.rect.x1[t] - a.rect.x0[t] + 1);
    for (int t = 0; t < a.N; ++t) mh = std::max(mh, a.rect.y1[t] - a.rect.y0[t] + 1);
    const int tiles_x = (mw + kThinGenTile - 1) / kThinGenTile, tiles_y = (mh + kThinGenTile - 1) / kThinGenTile;
    dim3 grid(tiles_x * tiles_y, 1, a.N * a.M * a.batch), block(256);
    g_kernel_label = "k_conv_fwd_thin_gen";
#define FTP_TG(T, KK, SS, CI) hipLaunchKernelGGL((k_conv_fwd_thin_gen<T, KK, SS, CI>), grid, block, 0, s, a.in, a.out, a.osign, a.rect, a.own, (const T*)a.w, (const T*)a.bias, a.Cin, a.Cout, a.Hi, a.Wi, a.slope, a.M, a.batch, tiles_x)
#define FTP_TGC(T, KK, SS) do { if (a.Cin <= 3) FTP_TG(T, KK, SS, 3); else FTP_TG(T, KK, SS, 4); } while (0)
#define FTP_TGK(T) do { \
        if (a.K == 7)      { if (a.S == 2) FTP_TGC(T, 7, 2); else FTP_TGC(T, 7, 1); } \
        else if (a.K == 5) { if (a.S == 2) FTP_TGC(T, 5, 2); else FTP_TGC(T, 5, 1); } \
        else if (a.K == 3) FTP_TGC(T, 3, 2); \
        else               FTP_TGC(T, 1, 2); } while (0)
    if (a.bf16) FTP_TGK(bf16_t); else FTP_TGK(float);
#undef FTP_TGK
#undef FTP_TGC
#undef FTP_TG
}

// ---- delta at the input of a convolution with at most CIT input channels ------------------------------------
// Workgroup = 64 x 4 pixels of one (stack, image): wide tiles keep the reads of the (pooled) delta rows long.
// LDS = dZ patch of COC channels with the filter halo.
template <typename T, int K, bool POOL, int CIT>
__global__ void __launch_bounds__(256)
k_conv_bwd_data_thin(View din, View mask, View dout, View isign, int scale_out, float in_slope, RectTab rt,
                     const T* __restrict__ w, int Cin, int Cout, int Hc, int Wc, int M, int batch, int tiles_x)
{
    constexpr int P = K / 2, TSX = 64, TSY = 4, PSX = TSX + 2 * P, PSY = TSY + 2 * P, PP = PSX + 1, COC = 16;
    __shared__ float dz[COC][PSY][PP];
    const int stack = blockIdx.z / batch, n = blockIdx.z % batch;
    const int ti = stack / M, tj = stack % M;
    const int bx = blockIdx.x % tiles_x, by = blockIdx.x / tiles_x;
    const int ox0 = rt.x0[tj] + bx * TSX, oy0 = rt.y0[ti] + by * TSY;
    if (ox0 > rt.x1[tj] || oy0 > rt.y1[ti]) return;
    const int tx = threadIdx.x % TSX, ty = threadIdx.x / TSX;
    const int ix = ox0 + tx, iy = oy0 + ty;
    float acc[CIT];
#pragma unroll
    for (int j = 0; j < CIT; ++j) acc[j] = 0.0f;
    for (int c0 = 0; c0 < Cout; c0 += COC) {
        __syncthreads();
        // every thread owns fixed patch positions and walks the channels, 4 loads in flight at a time
        for (int sp = threadIdx.x; sp < PSY * PSX; sp += 256) {
            const int r = sp / PSX, q = sp - r * PSX;
            const int qy = oy0 - P + r, qx = ox0 - P + q;
            // dZ positions that only out-of-rectangle pixels of the tile would read may lie outside the delta view
            const bool ok = qy >= 0 && qy < Hc && qx >= 0 && qx < Wc && qy <= rt.y1[ti] + P && qx <= rt.x1[tj] + P;
            const int cy = ok ? qy : rt.y0[ti], cx = ok ? qx : rt.x0[tj];
            const int sy = POOL ? (cy >> 1) : cy, sx = POOL ? (cx >> 1) : cx;
            const int code = ((cy & 1) << 1) | (cx & 1);
            const uint8_t* mp = at<uint8_t>(mask, stack, ti, tj, n, 0, sy, sx);
            const T* gp = at<T>(din, stack, ti, tj, n, 0, sy, sx);
#pragma unroll
            for (int cb = 0; cb < COC; cb += 4) {
                uint8_t m[4]; float g[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int co = c0 + cb + k < Cout ? c0 + cb + k : Cout - 1;
                    m[k] = POOL ? mp[(long long)co * mask.cs] : (uint8_t)0;      // only the pool winner is needed
                    g[k] = ld(gp + (long long)co * din.cs);
                }
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    float v = g[k];                                          // the delta maps hold dLoss/dZ
                    if (POOL && ((m[k] >> 1) & 3) != code) v = 0.0f;
                    if (!ok || c0 + cb + k >= Cout) v = 0.0f;
                    dz[cb + k][r][q] = v;
                }
            }
        }
        __syncthreads();
#pragma unroll 4
        for (int c = 0; c < COC; ++c) {
            const int co = c0 + c;
            if (co >= Cout) break;
#pragma unroll
            for (int ky = 0; ky < K; ++ky)
#pragma unroll
                for (int kx = 0; kx < K; ++kx) {
                    const float d = dz[c][ty + 2 * P - ky][tx + 2 * P - kx];
#pragma unroll
                    for (int j = 0; j < CIT; ++j)
                        if (j < Cin) acc[j] = fmaf(ld(w + (((size_t)co * Cin + j) * K + ky) * K + kx), d, acc[j]);
                }
        }
    }
    if (ix <= rt.x1[tj] && iy <= rt.y1[ti]) {
#pragma unroll
        for (int j = 0; j < CIT; ++j)
            if (j < Cin) {
                float v = acc[j];
                if (scale_out) v = scaled_delta<T>(v, sign_bit(isign, stack, ti, tj, n, j, iy, ix), in_slope);
                st(at<T>(dout, stack, ti, tj, n, j, iy, ix), v);
            }
    }
}

// ---- the same for K = 3, register-tiled: every thread produces 4 neighbouring pixels of all CI input channels ----
// Workgroup = TW x TH pixels of one (stack, image), TW = 4 * ntx <= 64, TH = nty <= 64, ntx * nty <= 256, chosen
// on the host from the largest rectangle so that its tiles leave no ragged last column.  Per 4 output channels the
// routed dZ patch (tile + filter halo) is staged in LDS - behind a pool one (delta, winner) pair per window
// serves its 4 pixels - next to the filter slice [co][ci][tap].  A thread reads 3 x 6 patch values and 9 * CI
// weights per output channel for 36 * CI multiply-adds.  Four channels per stage (22 KB of LDS) and at most 80 registers:
// six workgroups share a CU and cover each other's staging (8 channels, three workgroups: config 4 1.16 instead of 0.90 ms).
constexpr int kThin4Coc = 4, kThin4Patch = 1344;     // channels per stage, floats of one channel's patch

template <typename T, bool POOL, int CI>
__global__ void __launch_bounds__(256, 6)              // (six wavefronts a SIMD: the kernel waits for LDS and memory, not for registers)
k_conv_bwd_data_thin4(View din, View mask, View dout, View isign, int scale_out, float in_slope, RectTab rt,
                      const T* __restrict__ w, int Cin, int Cout, int Hc, int Wc, int M, int batch,
                      int ntx, int nty, int tiles_x, int tiles, int images)
{
    constexpr int COC = kThin4Coc, CH = kThin4Patch, WR = (9 * CI + 3) & ~3;        // (filter rows on 16-byte boundaries: read four weights at a time)
    __shared__ __attribute__((aligned(16))) float dz[COC * CH];
    __shared__ __attribute__((aligned(16))) float wl[COC * WR];
    const int tid = threadIdx.x;
    // 1-D grid in XCD order: the tiles of one (stack, image), whose patches overlap, run on one XCD and share its L2
    int image, tile;
    if (!xcd_order(images, tiles, image, tile)) return;
    const int stack = image / batch, n = image % batch;
    const int ti = stack / M, tj = stack % M;
    const int TW = 4 * ntx, TH = nty, PP = (TW + 2 + 3) & ~3;
    const int bx = tile % tiles_x, by = tile / tiles_x;
    const int ox0 = rt.x0[tj] + bx * TW, oy0 = rt.y0[ti] + by * TH;
    if (ox0 > rt.x1[tj] || oy0 > rt.y1[ti]) return;
    const int tx = tid % ntx, ty = tid / ntx;
    const bool worker = ty < nty;
    const int px0 = ox0 - 1, py0 = oy0 - 1;            // map coordinates of the patch origin
    float acc[CI][4];
#pragma unroll
    for (int j = 0; j < CI; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) acc[j][q] = 0.0f;

    for (int c0 = 0; c0 < Cout; c0 += COC) {
        __syncthreads();
        for (int i = tid; i < COC * WR; i += 256) {
            const int c = i / WR, r = i - c * WR, ci = r / 9, t = r - ci * 9;
            wl[i] = (c0 + c < Cout && ci < Cin) ? ld(w + ((size_t)(c0 + c) * Cin + ci) * 9 + t) : 0.0f;
        }
        if (POOL) {
            // windows that overlap the patch; one that no pixel of the rectangle reads may lie outside the delta view
            const int wy0 = py0 >> 1, wx0 = px0 >> 1;
            const int nwy = ((oy0 + TH) >> 1) - wy0 + 1, nwx = ((ox0 + TW) >> 1) - wx0 + 1;
            for (int idx = tid; idx < nwy * nwx; idx += 256) {
                const int wyi = idx / nwx, wy = wy0 + wyi, wx = wx0 + (idx - wyi * nwx);
                const bool need = wy >= 0 && 2 * wy < Hc && wx >= 0 && 2 * wx < Wc &&
                                  2 * wy + 1 >= rt.y0[ti] - 1 && 2 * wy <= rt.y1[ti] + 1 &&
                                  2 * wx + 1 >= rt.x0[tj] - 1 && 2 * wx <= rt.x1[tj] + 1;
                const int sy = need ? wy : (rt.y0[ti] >> 1), sx = need ? wx : (rt.x0[tj] >> 1);
                const uint8_t* mp = at<uint8_t>(mask, stack, ti, tj, n, 0, sy, sx);
                const T* gp = at<T>(din, stack, ti, tj, n, 0, sy, sx);
                float g[COC]; uint8_t m[COC];
#pragma unroll
                for (int c = 0; c < COC; ++c) {
                    const int co = c0 + c < Cout ? c0 + c : Cout - 1;
                    g[c] = ld(gp + (long long)co * din.cs);
                    m[c] = mp[(long long)co * mask.cs];
                }
                const int r0 = 2 * wy - py0, q0 = 2 * wx - px0;
#pragma unroll
                for (int pos = 0; pos < 4; ++pos) {
                    const int r = r0 + (pos >> 1), q = q0 + (pos & 1);
                    if (r >= 0 && r < TH + 2 && q >= 0 && q < TW + 2) {
#pragma unroll
                        for (int c = 0; c < COC; ++c)
                            dz[c * CH + r * PP + q] = (need && c0 + c < Cout && ((m[c] >> 1) & 3) == pos) ? g[c] : 0.0f;
                    }
                }
            }
        } else {
            for (int idx = tid; idx < (TH + 2) * (TW + 2); idx += 256) {
                const int r = idx / (TW + 2), q = idx - r * (TW + 2);
                const int qy = py0 + r, qx = px0 + q;
                const bool need = qy >= 0 && qy < Hc && qx >= 0 && qx < Wc && qy <= rt.y1[ti] + 1 && qx <= rt.x1[tj] + 1;
                const T* gp = at<T>(din, stack, ti, tj, n, 0, need ? qy : rt.y0[ti], need ? qx : rt.x0[tj]);
                float g[COC];
#pragma unroll
                for (int c = 0; c < COC; ++c) {
                    const int co = c0 + c < Cout ? c0 + c : Cout - 1;
                    g[c] = ld(gp + (long long)co * din.cs);
                }
#pragma unroll
                for (int c = 0; c < COC; ++c) dz[c * CH + r * PP + q] = (need && c0 + c < Cout) ? g[c] : 0.0f;
            }
        }
        __syncthreads();
        if (worker) {
#pragma unroll 2
            for (int c = 0; c < COC; ++c) {
                float d[3][6];
#pragma unroll
                for (int rr = 0; rr < 3; ++rr) {
                    const float* row = dz + c * CH + (ty + rr) * PP + 4 * tx;
                    const float4 a4 = *(const float4*)row;
                    const float2 a2 = *(const float2*)(row + 4);
                    d[rr][0] = a4.x; d[rr][1] = a4.y; d[rr][2] = a4.z; d[rr][3] = a4.w; d[rr][4] = a2.x; d[rr][5] = a2.y;
                }
                const float* wc = wl + c * WR;
#pragma unroll
                for (int j = 0; j < CI; ++j)
#pragma unroll
                    for (int ky = 0; ky < 3; ++ky)
#pragma unroll
                        for (int kx = 0; kx < 3; ++kx) {
                            const float wv = wc[j * 9 + ky * 3 + kx];
                            // dX[y][x] += W[ky][kx] * dZ[y + 1 - ky][x + 1 - kx]; the patch starts at (y0 - 1, x0 - 1)
#pragma unroll
                            for (int q = 0; q < 4; ++q) acc[j][q] = fmaf(wv, d[2 - ky][q + 2 - kx], acc[j][q]);
                        }
            }
        }
    }
    if (!worker) return;
    const int iy = oy0 + ty;
    if (iy > rt.y1[ti]) return;
#pragma unroll
    for (int j = 0; j < CI; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int ix = ox0 + 4 * tx + q;
            if (j < Cin && ix <= rt.x1[tj]) {
                float v = acc[j][q];
                if (scale_out) v = scaled_delta<T>(v, sign_bit(isign, stack, ti, tj, n, j, iy, ix), in_slope);
                st(at<T>(dout, stack, ti, tj, n, j, iy, ix), v);
            }
        }
}

// ---- delta at the input of a stride-2 convolution with at most 4 input channels (the image side of a strided stem) ----
// Input pixel (2j + a, 2i + b) receives W[ky][kx] dZ[qy][qx] from the taps with ky = a + P, kx = b + P (mod 2), at
// qy = j + (a + P - ky) / 2, qx likewise: the four pixels of a cell (j, i) together use every tap exactly once and
// read the deltas of the cells [j + QLO, j + QHI] x [i + QLO, i + QHI] (4 x 4 for a 7x7 filter).
// Workgroup = 16 x 32 cells (32 x 64 pixels) of one (stack, image), two neighbouring cells per thread.  Per 8 output channels the
// delta patch (tile + that halo; zero outside the stack's delta rectangle) and the filter slice [co][tap][ci padded
// to 4] (fp32) are staged in LDS; a thread reads its NQ x NQ deltas and one 16-byte filter vector per tap for
// K * K * CI multiply-adds per output channel.
template <int K> struct StridedTaps {
    static constexpr int P = K / 2;
    static constexpr int QLO = -((K - 1 - P) / 2), QHI = (1 + P) / 2, NQ = QHI - QLO + 1;
};
constexpr int kThinS2PerThread = 2;                   // cells per thread along a row: they share 3 of 4 delta columns and every weight read (1: 2.87 ms on the 7x7 stem, 2: 2.09, 4: 2.27)
constexpr int kThinS2Coc = 8, kThinS2Cells = 16;      // (8 channels a stage, 18 KB of LDS: five workgroups a CU; 16 channels, four workgroups: 3.37 instead of 2.85 ms on the 7x7 stem)

template <typename T, int K, int CI>
__global__ void __launch_bounds__(256, 5)
k_conv_bwd_data_thin_s2(View din, View dout, View isign, int scale_out, float in_slope, RectTab rt, RectTab ext,
                        const T* __restrict__ w, int Cin, int Cout, int M, int batch, int tiles_x)
{
    typedef StridedTaps<K> G;
    constexpr int P = G::P, QLO = G::QLO, NQ = G::NQ, KK = K * K;
    constexpr int COC = kThinS2Coc, TC = kThinS2Cells, NCX = kThinS2PerThread;
    constexpr int TCX = NCX * TC, PDY = TC + NQ - 1, PDX = TCX + NQ - 1, PDP = PDX + 1;     // tile, patch extent, padded pitch
    __shared__ __attribute__((aligned(16))) float dzl[COC * PDY * PDP];
    __shared__ __attribute__((aligned(16))) float wl[COC * KK * 4];
    const int tid = threadIdx.x;
    const int stack = blockIdx.z / batch, n = blockIdx.z % batch;
    const int ti = stack / M, tj = stack % M;
    const int bx = blockIdx.x % tiles_x, by = blockIdx.x / tiles_x;
    const int J0 = (rt.y0[ti] >> 1) + by * TC, I0 = (rt.x0[tj] >> 1) + bx * TCX;     // first cell of the tile
    if (2 * J0 > rt.y1[ti] || 2 * I0 > rt.x1[tj]) return;
    const int cy = tid / TC, cx = NCX * (tid % TC);     // this thread's cells: (cy, cx) .. (cy, cx + NCX - 1)
    float acc[NCX][2][2][CI];
#pragma unroll
    for (int u = 0; u < NCX; ++u)
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int c = 0; c < CI; ++c) acc[u][a][b][c] = 0.0f;

    for (int c0 = 0; c0 < Cout; c0 += COC) {
        __syncthreads();                               // the previous slice has been consumed
        // delta patch: rows QLO .. of the tile's cells, COC channels; lanes run along a patch row
        for (int e = tid; e < COC * PDY * PDX; e += 256) {
            const int c = e / (PDY * PDX), r = e - c * (PDY * PDX);
            const int py = r / PDX, px = r - py * PDX;
            const int qy = J0 + QLO + py, qx = I0 + QLO + px;
            float v = 0.0f;
            if (c0 + c < Cout && qy >= ext.y0[ti] && qy <= ext.y1[ti] && qx >= ext.x0[tj] && qx <= ext.x1[tj])
                v = ld(at<T>(din, stack, ti, tj, n, c0 + c, qy, qx));
            dzl[(c * PDY + py) * PDP + px] = v;
        }
        // filter slice as fp32, [co][tap][ci (4)]
        for (int e = tid; e < COC * KK * 4; e += 256) {
            const int c = e / (KK * 4), r = e - c * (KK * 4);
            const int t = r >> 2, ci = r & 3;
            wl[e] = (c0 + c < Cout && ci < Cin) ? ld(w + ((size_t)(c0 + c) * Cin + ci) * KK + t) : 0.0f;
        }
        __syncthreads();
        for (int c = 0; c < COC; ++c) {
            if (c0 + c >= Cout) break;
            // neighbouring cells share all but one column of their deltas, and every weight
            float dv[NQ][NQ + NCX - 1];
#pragma unroll
            for (int y = 0; y < NQ; ++y)
#pragma unroll
                for (int x = 0; x < NQ + NCX - 1; ++x) dv[y][x] = dzl[(c * PDY + cy + y) * PDP + cx + x];
            const float4* wc = (const float4*)(wl + c * KK * 4);
#pragma unroll
            for (int ky = 0; ky < K; ++ky)
#pragma unroll
                for (int kx = 0; kx < K; ++kx) {
                    const int a = (ky + P) & 1, b = (kx + P) & 1;
                    const int dy = (a + P - ky) / 2 - QLO, dx = (b + P - kx) / 2 - QLO;     // compile-time after unrolling
                    const float4 wv = wc[ky * K + kx];
#pragma unroll
                    for (int u = 0; u < NCX; ++u) {
                        const float d = dv[dy][dx + u];
                        acc[u][a][b][0] = fmaf(wv.x, d, acc[u][a][b][0]);
                        if (CI > 1) acc[u][a][b][1] = fmaf(wv.y, d, acc[u][a][b][1]);
                        if (CI > 2) acc[u][a][b][2] = fmaf(wv.z, d, acc[u][a][b][2]);
                        if (CI > 3) acc[u][a][b][3] = fmaf(wv.w, d, acc[u][a][b][3]);
                    }
                }
        }
    }
#pragma unroll
    for (int u = 0; u < NCX; ++u)
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                const int iy = 2 * (J0 + cy) + a, ix = 2 * (I0 + cx + u) + b;
                if (iy < rt.y0[ti] || iy > rt.y1[ti] || ix < rt.x0[tj] || ix > rt.x1[tj]) continue;
#pragma unroll
                for (int c = 0; c < CI; ++c)
                    if (c < Cin) {
                        float v = acc[u][a][b][c];
                        if (scale_out) v = scaled_delta<T>(v, sign_bit(isign, stack, ti, tj, n, c, iy, ix), in_slope);
                        st(at<T>(dout, stack, ti, tj, n, c, iy, ix), v);
                    }
            }
}

bool thin_bwd_data_strided_eligible(const ConvArgs& a) { return a.S == 2 && a.Cin <= 4 && !a.pooled && a.K >= 3; }

// c.rect = backward rectangle at the input boundary; ext = extent of the delta view per stack.
void thin_conv_bwd_data_strided(const ConvArgs& a, const RectTab& ext, hipStream_t s)
{
    int mw = 0, mh = 0;                                // cells per dimension of the largest rectangle
    for (int t = 0; t < a.M; ++t) mw = std::max(mw, (a.rect.x1[t] >> 1) - (a.rect.x0[t] >> 1) + 1);
    for (int t = 0; t < a.N; ++t) mh = std::max(mh, (a.rect.y1[t] >> 1) - (a.rect.y0[t] >> 1) + 1);
    const int tcx = kThinS2PerThread * kThinS2Cells;
    const int tiles_x = (mw + tcx - 1) / tcx, tiles_y = (mh + kThinS2Cells - 1) / kThinS2Cells;
    dim3 grid(tiles_x * tiles_y, 1, a.N * a.M * a.batch), block(256);
    g_kernel_label = "k_conv_bwd_data_thin_s2";
#define FTP_S2(T, KK, CI) hipLaunchKernelGGL((k_conv_bwd_data_thin_s2<T, KK, CI>), grid, block, 0, s, a.din, a.dout, a.isign, a.scale_out, a.in_slope, a.rect, ext, (const T*)a.w, a.Cin, a.Cout, a.M, a.batch, tiles_x)
#define FTP_S2C(T, KK) do { if (a.Cin <= 3) FTP_S2(T, KK, 3); else FTP_S2(T, KK, 4); } while (0)
#define FTP_S2K(T) do { if (a.K == 7) FTP_S2C(T, 7); else if (a.K == 5) FTP_S2C(T, 5); else FTP_S2C(T, 3); } while (0)
    if (a.bf16) FTP_S2K(bf16_t); else FTP_S2K(float);
#undef FTP_S2K
#undef FTP_S2C
#undef FTP_S2
}

bool thin_bwd_data_eligible(const ConvArgs& a) { return a.Cin <= 4; }

void thin_conv_bwd_data(const ConvArgs& a, hipStream_t s)
{
    int mw = 0, mh = 0;
    for (int t = 0; t < a.M; ++t) mw = mw > a.rect.x1[t] - a.rect.x0[t] + 1 ? mw : a.rect.x1[t] - a.rect.x0[t] + 1;
    for (int t = 0; t < a.N; ++t) mh = mh > a.rect.y1[t] - a.rect.y0[t] + 1 ? mh : a.rect.y1[t] - a.rect.y0[t] + 1;
    if (a.K == 3) {
        // tile = 4*ntx x nty pixels fitted to the largest rectangle
        int tiles_x = (mw + 63) / 64;
        const int ntx = ((mw + tiles_x - 1) / tiles_x + 3) / 4;
        tiles_x = (mw + 4 * ntx - 1) / (4 * ntx);
        int nty_max = 256 / ntx; if (nty_max > 64) nty_max = 64;
        const int tiles_y = (mh + nty_max - 1) / nty_max;
        const int nty = (mh + tiles_y - 1) / tiles_y;
        const int PP = (4 * ntx + 2 + 3) & ~3;
        if ((nty + 2) * PP <= kThin4Patch) {
            const int tiles = tiles_x * tiles_y, images = a.N * a.M * a.batch;
            dim3 grid(xcd_grid(images, tiles)), block(256);
            g_kernel_label = "k_conv_bwd_data_thin4";
#define FTP_T4(T, PL, CI) hipLaunchKernelGGL((k_conv_bwd_data_thin4<T, PL, CI>), grid, block, 0, s, a.din, a.mask, a.dout, a.isign, a.scale_out, a.in_slope, a.rect, (const T*)a.w, a.Cin, a.Cout, a.Hc, a.Wc, a.M, a.batch, ntx, nty, tiles_x, tiles, images)
#define FTP_T4C(T, PL) do { if (a.Cin <= 3) FTP_T4(T, PL, 3); else FTP_T4(T, PL, 4); } while (0)
            if (a.bf16) { if (a.pooled) FTP_T4C(bf16_t, true); else FTP_T4C(bf16_t, false); }
            else        { if (a.pooled) FTP_T4C(float, true); else FTP_T4C(float, false); }
#undef FTP_T4C
#undef FTP_T4
            return;
        }
    }
    const int tiles_x = (mw + 63) / 64, tiles_y = (mh + 3) / 4;
    dim3 grid(tiles_x * tiles_y, 1, a.N * a.M * a.batch), block(256);
    g_kernel_label = "k_conv_bwd_data_thin";
#define FTP_TB(T, KK, PL) hipLaunchKernelGGL((k_conv_bwd_data_thin<T, KK, PL, 4>), grid, block, 0, s, a.din, a.mask, a.dout, a.isign, a.scale_out, a.in_slope, a.rect, (const T*)a.w, a.Cin, a.Cout, a.Hc, a.Wc, a.M, a.batch, tiles_x)
    if (a.bf16) {
        if (a.K == 3) { if (a.pooled) FTP_TB(bf16_t, 3, true); else FTP_TB(bf16_t, 3, false); }
        else          { if (a.pooled) FTP_TB(bf16_t, 1, true); else FTP_TB(bf16_t, 1, false); }
    } else {
        if (a.K == 3) { if (a.pooled) FTP_TB(float, 3, true); else FTP_TB(float, 3, false); }
        else          { if (a.pooled) FTP_TB(float, 1, true); else FTP_TB(float, 1, false); }
    }
#undef FTP_TB
}

// ---- per-stack filter gradient of layers with very few input channels (Cin <= 4) ------------------------------
// D[m = co][n = (ci, tap)] += sum over pixel pairs of dZ[co][pixel] * X[ci][S * pixel + tap - P], NB blocks of 32
// columns n (one for 3x3 filters, five for a 7x7 filter on 3 channels).
// Workgroup = 32 output channels of one stack and one batch share; its 4 wavefronts take alternate pixel
// pairs of each staged block and are summed in wavefront order at the end.
template <typename T, int K, int S, int NB, bool POOL>
__global__ void __launch_bounds__(256)
k_wgrad_mfma_thin(MfmaWgradArgs a)
{
    constexpr int KK = K * K, P = K / 2, ZP = 33;
    extern __shared__ float lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // uniform: row bookkeeping stays scalar
    const int hi = lane >> 5, l32 = lane & 31;
    const int stack = blockIdx.z, ti = stack / a.M, tj = stack % a.M;
    const int x0 = a.own.x0[tj], x1 = a.own.x1[tj], y0 = a.own.y0[ti], y1 = a.own.y1[ti];
    const int rw = x1 - x0 + 1, rh = y1 - y0 + 1;
    const int co0 = blockIdx.x * 32;
    const int split = blockIdx.y;

    const ThinChunks tc = thin_wgrad_chunks(rw, rh, a.batch, a.PK, POOL);
    const int TCp = tc.TCp, TR = tc.TR, TI = tc.TI, row_blocks = tc.row_blocks;
    // this share's part of the stack's chunk list (image block, row block)
    const int id0 = (int)((long long)split * tc.total / a.splits), id1 = (int)((long long)(split + 1) * tc.total / a.splits);
    const int PW = S * TCp + 2 * P, PH = S * TR + 2 * P;
    const int XCS = TI * PH * PW;                      // channel stride of the X patch
    float* Zl = lds;                                   // [TI*TR*TCp][ZP]
    float* Xl = lds + a.PK * ZP;                       // [Cin][TI][PH][PW]

    // B operand of lane n = (ci, tap): fixed offset into the patch
    int lane_off[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int nn = nb * 32 + l32 < a.Cin * KK ? nb * 32 + l32 : 0;
        lane_off[nb] = (nn / KK) * XCS + ((nn % KK) / K) * PW + (nn % KK) % K + S * hi;
    }

    v16f acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[nb][i] = 0.0f;

    // Behind a pool a chunk of up to 256 pixels is at most 64 windows: one (delta, winner) pair per lane and channel.
    // They are loaded one chunk ahead, during the previous chunk's multiply, so that their latency is hidden.
    const bool ahead = POOL && a.PK <= 256;
    uint8_t pm[8]; float pg[8];
    int p_il = 0, p_wr = 0, p_wx = 0;
    bool p_ok = false;
    auto load_ahead = [&](int id) {
        const int ib = id / row_blocks, rb = id - ib * row_blocks;
        const int n0 = ib * TI;
        const int ni = (a.batch - n0) < TI ? (a.batch - n0) : TI;
        const int yb = y0 + rb * TR;
        const int nr = (y1 - yb + 1) < TR ? (y1 - yb + 1) : TR;
        const int wpr = TCp >> 1, wrows = nr >> 1;
        const int nwin = ni * wrows * wpr;
        p_ok = lane < nwin;
        const int wi = p_ok ? lane : 0;
        const int wrow = wi / wpr;
        p_wx = wi - wrow * wpr;
        p_il = wrow / wrows; p_wr = wrow - p_il * wrows;
        const int sy = (yb >> 1) + p_wr, sx = (x0 >> 1) + p_wx;
        const uint8_t* mp = at<uint8_t>(a.mask, stack, ti, tj, n0 + p_il, 0, sy, sx);
        const T* gp = at<T>(a.din, stack, ti, tj, n0 + p_il, 0, sy, sx);
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int co = co0 + wave + 4 * k < a.Cout ? co0 + wave + 4 * k : a.Cout - 1;
            pm[k] = mp[(long long)co * a.mask.cs];
            pg[k] = ld(gp + (long long)co * a.din.cs);
        }
    };
    if (ahead && id0 < id1) load_ahead(id0);

    for (int id = id0; id < id1; ++id) {
        {
            const int ib = id / row_blocks, rb = id - ib * row_blocks;
            const int n0 = ib * TI;
            const int ni = (a.batch - n0) < TI ? (a.batch - n0) : TI;
            const int yb = y0 + rb * TR;
            const int nr = (y1 - yb + 1) < TR ? (y1 - yb + 1) : TR;
            __syncthreads();
            // dZ, pixel-major [pixel][co]: wavefront w takes channels w, w+4, ... (8 of them).  All loads of a pass
            // are unconditional (clamped) and issued together; what must be zero is zeroed at the LDS write.
            if (ahead) {
                if (p_ok) {
#pragma unroll
                    for (int pos = 0; pos < 4; ++pos) {
                        float* zdst = Zl + ((p_il * nr + 2 * p_wr + (pos >> 1)) * TCp + 2 * p_wx + (pos & 1)) * ZP + wave;
#pragma unroll
                        for (int k = 0; k < 8; ++k)
                            zdst[4 * k] = (((pm[k] >> 1) & 3) == pos && co0 + wave + 4 * k < a.Cout) ? pg[k] : 0.0f;
                    }
                }
            } else if (POOL) {
                // behind a pool one (delta, winner) pair per window and channel serves the window's 4 pixels;
                // owned rectangles of a pooled convolution start and end on window borders
                const int wpr = TCp >> 1, wrows = nr >> 1;
                const int nwin = ni * wrows * wpr;
                for (int wb = 0; wb < nwin; wb += 64) {
                    const bool ok = wb + lane < nwin;
                    const int wi = ok ? wb + lane : 0;
                    const int wrow = wi / wpr, wx = wi - wrow * wpr;
                    const int il = wrow / wrows, wr = wrow - il * wrows;
                    const int sy = (yb >> 1) + wr, sx = (x0 >> 1) + wx;
                    const uint8_t* mp = at<uint8_t>(a.mask, stack, ti, tj, n0 + il, 0, sy, sx);
                    const T* gp = at<T>(a.din, stack, ti, tj, n0 + il, 0, sy, sx);
                    uint8_t m[8]; float g[8];
#pragma unroll
                    for (int k = 0; k < 8; ++k) {
                        const int co = co0 + wave + 4 * k < a.Cout ? co0 + wave + 4 * k : a.Cout - 1;
                        m[k] = mp[(long long)co * a.mask.cs];
                        g[k] = ld(gp + (long long)co * a.din.cs);
                    }
                    if (ok) {
#pragma unroll
                        for (int pos = 0; pos < 4; ++pos) {
                            float* zdst = Zl + ((il * nr + 2 * wr + (pos >> 1)) * TCp + 2 * wx + (pos & 1)) * ZP + wave;
#pragma unroll
                            for (int k = 0; k < 8; ++k)
                                zdst[4 * k] = (((m[k] >> 1) & 3) == pos && co0 + wave + 4 * k < a.Cout) ? g[k] : 0.0f;
                        }
                    }
                }
            } else {
                const int npos = ni * nr * TCp;
                for (int pb = 0; pb < npos; pb += 64) {
                    const bool ok = pb + lane < npos;
                    const int pos = ok ? pb + lane : 0;
                    const int row = pos / TCp, col = pos - row * TCp;
                    const int il = row / nr, r = row - il * nr;
                    const T* gp = at<T>(a.din, stack, ti, tj, n0 + il, 0, yb + r, x0 + (col < rw ? col : rw - 1));
                    float g[8];
#pragma unroll
                    for (int k = 0; k < 8; ++k) {
                        const int co = co0 + wave + 4 * k < a.Cout ? co0 + wave + 4 * k : a.Cout - 1;
                        g[k] = ld(gp + (long long)co * a.din.cs);
                    }
                    if (ok) {
#pragma unroll
                        for (int k = 0; k < 8; ++k)
                            Zl[pos * ZP + wave + 4 * k] = (col < rw && co0 + wave + 4 * k < a.Cout) ? g[k] : 0.0f;
                    }
                }
            }
            // X patch in natural order [ci][image][row][column]: a wavefront takes whole rows (the row's place in the
            // patch is wave-uniform, no per-lane division), 4 rows in flight
            {
                const int nph = S * nr + 2 * P;
                const int rows = a.Cin * ni * nph;
                for (int pr0 = 0; pr0 < rows; pr0 += 16)
                for (int cb = 0; cb < PW; cb += 64) {
                    const int col = cb + lane;
                    const int gx = S * x0 - P + col;
                    const bool xin = col < S * rw + 2 * P && gx >= 0 && gx < a.Wc;
                    float v[4]; int dst[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int prow = pr0 + wave + 4 * u;
                        const bool rok = prow < rows;
                        const int pc = rok ? prow : 0;
                        const int ci = pc / (ni * nph), rem = pc - ci * (ni * nph);
                        const int il = rem / nph, r = rem - il * nph;
                        const int gy = S * yb - P + r;
                        const bool inside = xin && gy >= 0 && gy < a.Hc;
                        v[u] = ld(at<T>(a.in, stack, ti, tj, n0 + il, ci, inside ? gy : S * y0, inside ? gx : S * x0));
                        if (!inside) v[u] = 0.0f;
                        dst[u] = (rok && col < PW) ? ci * XCS + (il * PH + r) * PW + col : -1;
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u) if (dst[u] >= 0) Xl[dst[u]] = v[u];
                }
            }
            __syncthreads();
            if (ahead && id + 1 < id1) load_ahead(id + 1);       // in flight during the multiply below
            // the 4 wavefronts take alternate pixel pairs of every row
            const int nrows = ni * nr;
            for (int rr = 0; rr < nrows; ++rr) {
                const int il = rr / nr, r = rr - il * nr;
                const float* zrow = Zl + (rr * TCp + hi) * ZP + l32;
                const float* xrow = Xl + (il * PH + S * r) * PW;
                for (int xp = 2 * wave; xp < TCp; xp += 8) {
                    const float av = zrow[xp * ZP];
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
                        acc[nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, xrow[lane_off[nb] + S * xp], acc[nb], 0, 0, 0);
                }
            }
        }
    }

    // sum the 4 wavefronts in order, then wavefront 0 stores D[co][(ci, tap)]
    float* red = lds;                                  // [3][16][64]
    const long long layer_params = (long long)a.Cout * a.Cin * KK;
    float* dst = a.splits > 1 ? a.scratch + ((long long)stack * a.splits + split) * layer_params
                              : a.partial + (long long)stack * a.n_params + a.w_off;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        __syncthreads();
        if (wave > 0) {
#pragma unroll
            for (int i = 0; i < 16; ++i) red[((wave - 1) * 16 + i) * 64 + lane] = acc[nb][i];
        }
        __syncthreads();
        if (wave == 0) {
            const int n = nb * 32 + l32;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float v = ((acc[nb][i] + red[(0 * 16 + i) * 64 + lane]) + red[(1 * 16 + i) * 64 + lane]) + red[(2 * 16 + i) * 64 + lane];
                const int co = co0 + 8 * (i >> 2) + 4 * hi + (i & 3);
                if (co < a.Cout && n < a.Cin * KK) dst[(long long)co * a.Cin * KK + n] = v;
            }
        }
    }
}

// ---- the same gradient, its chunks streamed into LDS by the load unit ------------------------------------------
// Two stages of LDS: while the matrix cores work on one chunk, the next one travels HBM -> LDS without passing through
// registers (one barrier a chunk).  A stage holds dZ as [32 channels][zs positions] - at the pooled resolution behind a
// pool, followed by the winner codes in the same layout - and the patch [ci][image][row][column] in natural order; 16-bit
// maps occupy one dword a position (the bits in the lower half).  zs = 2 mod 64 keeps the A-operand reads (32 channels
// x 2 neighbouring pixels) on 64 different banks.  A chunk = a column block of the rectangle (at most 128 pixels wide) x
// the rows that 128 pixels (64 pool windows) allow x, for small rectangles, several images (thin_stream_chunks).
// Five wavefronts: the fifth only issues the loads (lane -> position of a row, one instruction per channel / patch row)
// and waits for them, so that the address arithmetic never sits between the matrix instructions of the four that
// multiply; these split the pixel pairs of every row among themselves as in the kernel above.
#define FTP_THIN_LDS(p) ((__attribute__((address_space(3))) void*)(p))
template <typename T, int K, int S, int NB, bool POOL>
__global__ void __launch_bounds__(320)
k_wgrad_thin_dl(MfmaWgradArgs a)
{
    constexpr int KK = K * K, P = K / 2, ES = sizeof(T);
    constexpr int ZPASS = kThinZPass(POOL);
    constexpr unsigned OOB = 0x80000000u;              // beyond the records of the buffer resources below: reads as zero
    extern __shared__ float lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int hi = lane >> 5, l32 = lane & 31;
    const int stack = blockIdx.z, ti = stack / a.M, tj = stack % a.M;
    const int x0 = a.own.x0[tj], x1 = a.own.x1[tj], y0 = a.own.y0[ti], y1 = a.own.y1[ti];
    const int rw = x1 - x0 + 1, rh = y1 - y0 + 1;
    const int co0 = blockIdx.x * 32;
    const int split = blockIdx.y;

    const ThinStreamChunks tc = thin_stream_chunks(rw, rh, a.batch, POOL, a.PK);      // (a.PK: widest column block)
    const int TCp = tc.TC, TR = tc.TR, TI = tc.TI, row_blocks = tc.row_blocks, col_blocks = tc.col_blocks;
    const int id0 = (int)((long long)split * tc.total / a.splits), id1 = (int)((long long)(split + 1) * tc.total / a.splits);
    const int PW = S * TCp + 2 * P, PH = S * TR + 2 * P;
    const int XCS = TI * PH * PW;                      // channel stride of the patch
    const int zs = a.zs;
    const int zwords = 32 * zs * (POOL ? 2 : 1);
    const int wpr = TCp >> 1, wrT = TR >> 1;           // POOL: windows per row, window rows of a full chunk
    const int nzp = POOL ? TI * wrT * wpr : TI * TR * TCp;     // dZ positions of a full chunk

    int lane_off[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int nn = nb * 32 + l32 < a.Cin * KK ? nb * 32 + l32 : 0;
        lane_off[nb] = (nn / KK) * XCS + ((nn % KK) / K) * PW + (nn % KK) % K + S * hi;
    }
    v16f acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[nb][i] = 0.0f;

    // which (image, row, column) of a chunk a lane stages is the same for every chunk (chunks of several images hold
    // whole rectangles): divided once.  z_r: pixel row inside the chunk.
    int z_il[ZPASS], z_r[ZPASS], z_c[ZPASS]; unsigned z_vo[ZPASS], z_mo[ZPASS];
#pragma unroll
    for (int p = 0; p < ZPASS; ++p) {
        const int zi = lane + 64 * p;
        const int row = zi / (POOL ? wpr : TCp), c = zi - row * (POOL ? wpr : TCp);
        const int rows_img = POOL ? wrT : TR;
        const int il = TI > 1 ? row / rows_img : 0;
        const int r = row - il * rows_img;
        z_r[p] = POOL ? 2 * r : r;
        z_c[p] = POOL ? 2 * c : c;                     // pixel column inside the chunk
        const bool ok = zi < nzp;
        z_il[p] = ok ? il : a.batch;                   // (a.batch: never inside a chunk)
        z_vo[p] = ok ? (unsigned)ES * (unsigned)(il * (int)a.din.ns + r * a.din.pitch + c) : 0u;
        z_mo[p] = POOL && ok ? (unsigned)(il * (int)a.mask.ns + r * a.mask.pitch + c) : 0u;
    }

    // chunk list: image block, row block, column block (fastest); walked with counters, divided once
    struct Chunk { int ib, n0, ni, yb, nr, rb, cb, nc; };      // nc: columns of the block that lie in the rectangle
    auto fill = [&](Chunk& c) {
        c.n0 = c.ib * TI; c.ni = (a.batch - c.n0) < TI ? (a.batch - c.n0) : TI;
        c.yb = y0 + c.rb * TR; c.nr = (y1 - c.yb + 1) < TR ? (y1 - c.yb + 1) : TR;
        c.nc = (rw - c.cb * TCp) < TCp ? (rw - c.cb * TCp) : TCp;
    };
    auto chunk_at = [&](int id) {
        Chunk c;
        c.ib = id / (row_blocks * col_blocks);
        const int rem = id - c.ib * (row_blocks * col_blocks);
        c.rb = rem / col_blocks; c.cb = rem - c.rb * col_blocks;
        fill(c);
        return c;
    };
    auto next_chunk = [&](Chunk& c) {
        if (++c.cb == col_blocks) { c.cb = 0; if (++c.rb == row_blocks) { c.rb = 0; ++c.ib; } }
        fill(c);
    };

    // Per load instruction only a scalar offset changes: the channel's (a channel beyond the layer's last loads the last
    // one again - its row of the product is never stored); a chunk's own origin goes into the base address of the
    // buffer resource.
    const int z_cs = (int)a.din.cs, m_cs = POOL ? (int)a.mask.cs : 0, co_last = a.Cout - 1 - co0;
    const T* const zstack = (const T*)a.din.p + (long long)stack * a.din.ss
                            + ((POOL ? (y0 >> 1) : y0) - a.din.y0[ti]) * a.din.pitch + ((POOL ? (x0 >> 1) : x0) - a.din.x0[tj]);
    const uint8_t* const mstack = POOL ? (const uint8_t*)a.mask.p + (long long)stack * a.mask.ss
                                         + ((y0 >> 1) - a.mask.y0[ti]) * a.mask.pitch + ((x0 >> 1) - a.mask.x0[tj]) : nullptr;
    const long long z_ns = a.din.ns, m_ns = a.mask.ns, x_ns = a.in.ns;
    const int z_rowstep = (POOL ? TR >> 1 : TR) * a.din.pitch, m_rowstep = POOL ? (TR >> 1) * a.mask.pitch : 0;
    const int z_colstep = POOL ? TCp >> 1 : TCp;
    // the patch: column offsets of this lane (the same for every chunk), rows relative to the map row S * y0 - P
    const T* const xstack = (const T*)a.in.p + (long long)stack * a.in.ss - (long long)a.in.y0[ti] * a.in.pitch - a.in.x0[tj];
    const int x_pitch = a.in.pitch, x_cs = (int)a.in.cs;
    const int gx00 = S * x0 - P;
    const int Hc = a.Hc, Cin = a.Cin;

    auto issue = [&](const Chunk& c, int rb, float* st) {
        // dZ (and the winner codes): lanes without a pixel receive zeros
        {
            const T* gbase = zstack + c.n0 * z_ns + rb * z_rowstep + c.cb * z_colstep;
            const __amdgpu_buffer_rsrc_t grsrc = __builtin_amdgcn_make_buffer_rsrc((void*)gbase, (short)0, 0x7FFFFFFF, 0x00020000);
            const uint8_t* mbase = POOL ? mstack + c.n0 * m_ns + rb * m_rowstep + c.cb * z_colstep : nullptr;
            const __amdgpu_buffer_rsrc_t mrsrc = __builtin_amdgcn_make_buffer_rsrc((void*)mbase, (short)0, 0x7FFFFFFF, 0x00020000);
#pragma unroll
            for (int p = 0; p < ZPASS; ++p) {
                if (64 * p < nzp) {
                    const bool ok = z_il[p] < c.ni && z_r[p] < c.nr && z_c[p] < c.nc;
                    const unsigned gv = ok ? z_vo[p] : OOB, mv = ok ? z_mo[p] : OOB;
#pragma unroll 8
                    for (int ch = 0; ch < 32; ++ch) {
                        const int co = co0 + (ch < co_last ? ch : co_last);
                        float* zd = st + ch * zs + 64 * p;
                        if constexpr (sizeof(T) == 4) __builtin_amdgcn_raw_ptr_buffer_load_lds(grsrc, FTP_THIN_LDS(zd), 4, gv, (unsigned)ES * (unsigned)(co * z_cs), 0, 0);
                        else                          __builtin_amdgcn_raw_ptr_buffer_load_lds(grsrc, FTP_THIN_LDS(zd), 2, gv, (unsigned)ES * (unsigned)(co * z_cs), 0, 0);
                        if constexpr (POOL)
                            __builtin_amdgcn_raw_ptr_buffer_load_lds(mrsrc, FTP_THIN_LDS(zd + 32 * zs), 1, mv, (unsigned)(co * m_cs), 0, 0);
                    }
                }
            }
        }
        // the patch, 64 columns of a row to an instruction; rows and columns outside the map are filled with zeros
        {
            const int nph = S * c.nr + 2 * P, ncol = S * c.nc + 2 * P;
            const int gy0 = S * c.yb - P, gx0 = gx00 + S * c.cb * TCp;
            const T* base = xstack + c.n0 * x_ns + (long long)gy0 * x_pitch;       // (row gy0 may lie above the map: never read)
            const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)base, (short)0, 0x7FFFFFFF, 0x00020000);
            float* xs = st + zwords;
            for (int cb = 0; cb < PW; cb += 64) {
                const int col = cb + lane, gx = gx0 + col;
                const unsigned vo = (col < ncol && gx >= 0 && gx < a.Wc) ? (unsigned)ES * (unsigned)gx : OOB;
                if (col < PW) {
                    for (int ci = 0; ci < Cin; ++ci)
                        for (int il = 0; il < c.ni; ++il) {
                            int so = ES * (ci * x_cs + il * (int)x_ns);
                            float* xd = xs + ci * XCS + il * PH * PW + cb;
                            for (int r = 0; r < nph; ++r, so += ES * x_pitch, xd += PW) {
                                const bool rok = (unsigned)(gy0 + r) < (unsigned)Hc;   // (uniform)
                                if constexpr (sizeof(T) == 4) __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, FTP_THIN_LDS(xd), 4, rok ? vo : OOB, rok ? (unsigned)so : 0u, 0, 0);
                                else                          __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, FTP_THIN_LDS(xd), 2, rok ? vo : OOB, rok ? (unsigned)so : 0u, 0, 0);
                            }
                        }
                }
            }
        }
    };

    auto widen = [](float v) -> float { return ES == 4 ? v : __uint_as_float(__float_as_uint(v) << 16); };

    // (the LDS reads of the next pixel pair are issued before the matrix instructions of the current one)
    auto multiply = [&](const Chunk& c, const float* st) {
        const float* xs = st + zwords;
        if constexpr (POOL) {
            const int wrows = c.nr >> 1;
            for (int il = 0; il < c.ni; ++il)
                for (int wr = 0; wr < wrows; ++wr) {
                    const float* zrow = st + l32 * zs + (il * wrT + wr) * wpr;
                    const float* xrow = xs + (il * PH + 2 * wr) * PW;
                    // this wavefront's windows wave, wave + 4, ...: two to a turn of the loop, the LDS reads of each issued
                    // before the matrix instructions of the one before
                    const int n = ((c.nc >> 1) - wave + 3) >> 2;
                    if (n <= 0) continue;
                    const float* pz = zrow + wave;
                    const float* px[NB];
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) px[nb] = xrow + lane_off[nb] + 2 * wave;
                    float zA, cA, x0A[NB], x1A[NB], zB, cB, x0B[NB], x1B[NB];
                    auto ldw = [&](int i, float& z, float& cw, float (&x0v)[NB], float (&x1v)[NB]) {
                        z = pz[4 * i]; cw = pz[32 * zs + 4 * i];
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb) { x0v[nb] = px[nb][8 * i]; x1v[nb] = px[nb][PW + 8 * i]; }
                    };
                    auto mm = [&](float z, float cw, const float (&x0v)[NB], const float (&x1v)[NB]) {
                        const float zv = widen(z);
                        const uint32_t cd = (__float_as_uint(cw) >> 1) & 3u;
                        const float a0 = cd == (uint32_t)hi ? zv : 0.0f, a1 = cd == (uint32_t)(2 + hi) ? zv : 0.0f;
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb)
                            acc[nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, widen(x0v[nb]), acc[nb], 0, 0, 0);
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb)
                            acc[nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, widen(x1v[nb]), acc[nb], 0, 0, 0);
                    };
                    ldw(0, zA, cA, x0A, x1A);
                    int i = 0;
                    for (; i + 2 < n; i += 2) {
                        ldw(i + 1, zB, cB, x0B, x1B);
                        __builtin_amdgcn_sched_barrier(0);
                        mm(zA, cA, x0A, x1A);
                        __builtin_amdgcn_sched_barrier(0);
                        ldw(i + 2, zA, cA, x0A, x1A);
                        __builtin_amdgcn_sched_barrier(0);
                        mm(zB, cB, x0B, x1B);
                        __builtin_amdgcn_sched_barrier(0);
                        asm volatile("" : "+v"(zA), "+v"(cA));         // (a value of this turn, not a read of the next)
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb) asm volatile("" : "+v"(x0A[nb]), "+v"(x1A[nb]));
                    }
                    if (i + 1 < n) {
                        ldw(i + 1, zB, cB, x0B, x1B);
                        __builtin_amdgcn_sched_barrier(0);
                        mm(zA, cA, x0A, x1A);
                        mm(zB, cB, x0B, x1B);
                    } else {
                        mm(zA, cA, x0A, x1A);
                    }
                }
        } else {
            for (int il = 0; il < c.ni; ++il)
                for (int r = 0; r < c.nr; ++r) {
                    const float* zrow = st + l32 * zs + (il * TR + r) * TCp + hi;
                    const float* xrow = xs + (il * PH + S * r) * PW;
                    const int ncp = (c.nc + 1) & ~1;
                    if (2 * wave >= ncp) continue;
                    float zc = zrow[2 * wave], xc[NB];
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) xc[nb] = xrow[lane_off[nb] + S * 2 * wave];
                    for (int xp = 2 * wave; xp < ncp; xp += 8) {
                        const int xn = xp + 8 < ncp ? xp + 8 : xp;
                        const float zn = zrow[xn];
                        float xnv[NB];
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb) xnv[nb] = xrow[lane_off[nb] + S * xn];
                        __builtin_amdgcn_sched_barrier(0);
                        const float av = widen(zc);
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb)
                            acc[nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, widen(xc[nb]), acc[nb], 0, 0, 0);
                        __builtin_amdgcn_sched_barrier(0);
                        zc = zn;
                        asm volatile("" : "+v"(zc));
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb) { xc[nb] = xnv[nb]; asm volatile("" : "+v"(xc[nb])); }
                    }
                }
        }
    };

    if (wave == 4) {
        // the loader: chunk id + 1 is on its way while the others multiply chunk id
        Chunk c = chunk_at(id0);
        if (id0 < id1) issue(c, c.rb, lds);
        for (int id = id0; id < id1; ++id) {
            __builtin_amdgcn_s_waitcnt(0x0F70);        // vmcnt(0): chunk id has landed
            __syncthreads();                           // ... and the stage of chunk id - 1 has been consumed
            if (id + 1 < id1) { next_chunk(c); issue(c, c.rb, lds + ((id + 1 - id0) & 1) * a.stage_words); }
        }
    } else {
        Chunk c = chunk_at(id0);
        for (int id = id0; id < id1; ++id) {
            __syncthreads();
            multiply(c, lds + ((id - id0) & 1) * a.stage_words);
            next_chunk(c);
        }
    }

    // sum the 4 wavefronts in order, then wavefront 0 stores D[co][(ci, tap)]
    float* red = lds;                                  // [3][16][64]
    const long long layer_params = (long long)a.Cout * a.Cin * KK;
    float* dst = a.splits > 1 ? a.scratch + ((long long)stack * a.splits + split) * layer_params
                              : a.partial + (long long)stack * a.n_params + a.w_off;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        __syncthreads();
        if (wave > 0 && wave < 4) {
#pragma unroll
            for (int i = 0; i < 16; ++i) red[((wave - 1) * 16 + i) * 64 + lane] = acc[nb][i];
        }
        __syncthreads();
        if (wave == 0) {
            const int n = nb * 32 + l32;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float v = ((acc[nb][i] + red[(0 * 16 + i) * 64 + lane]) + red[(1 * 16 + i) * 64 + lane]) + red[(2 * 16 + i) * 64 + lane];
                const int co = co0 + 8 * (i >> 2) + 4 * hi + (i & 3);
                if (co < a.Cout && n < a.Cin * KK) dst[(long long)co * a.Cin * KK + n] = v;
            }
        }
    }
}
#undef FTP_THIN_LDS

namespace {

struct ThinGeom { int PK; size_t lds; };

ThinGeom thin_geom(const ConvArgs& c)
{
    ThinGeom g;
    const int P = c.K / 2;
    int wmax = 0, max_pos = 1;
    for (int t = 0; t < c.M; ++t) wmax = std::max(wmax, (c.rect.x1[t] - c.rect.x0[t] + 2) & ~1);
    g.PK = thin_wgrad_pk(wmax, c.pooled != 0);
    for (int i = 0; i < c.N; ++i)
        for (int j = 0; j < c.M; ++j) {
            const ThinChunks tc = thin_wgrad_chunks(c.rect.x1[j] - c.rect.x0[j] + 1, c.rect.y1[i] - c.rect.y0[i] + 1, c.batch, g.PK, c.pooled != 0);
            const int pos = tc.TI * (c.S * tc.TR + 2 * P) * (c.S * tc.TCp + 2 * P);
            if (pos > max_pos) max_pos = pos;
        }
    size_t words = (size_t)g.PK * 33 + (size_t)max_pos * c.Cin + 2 * c.S;   // the second pixel of the last pair
    if (words < 3 * 16 * 64) words = 3 * 16 * 64;                         // final sum of the wavefronts
    g.lds = words * sizeof(float);
    return g;
}

}  // namespace

namespace {

ThinStream stream_geom(const ConvArgs& c)
{
    int rws[kTabGrid], rhs[kTabGrid];
    for (int j = 0; j < c.M; ++j) rws[j] = c.rect.x1[j] - c.rect.x0[j] + 1;
    for (int i = 0; i < c.N; ++i) rhs[i] = c.rect.y1[i] - c.rect.y0[i] + 1;
    ThinStream g = thin_stream_geom(rws, rhs, c.N, c.M, c.batch, c.Cin, c.K, c.S, c.pooled != 0);
    // the kernel addresses one chunk's images with 32-bit byte offsets
    const int ti_max = g.max_ti;
    const long long es = c.bf16 ? 2 : 4, lim = 0x7FFFFFFFll;
    if ((ti_max * c.in.ns + (long long)c.Cin * c.in.cs) * es > lim || (ti_max * c.din.ns + (long long)c.Cout * c.din.cs) * es > lim) g.fits = false;
    if (c.pooled && ti_max * c.mask.ns + (long long)c.Cout * c.mask.cs > lim) g.fits = false;
    return g;
}

}  // namespace

// c.rect must hold the owned rectangles.
bool thin_wgrad_eligible(const ConvArgs& c)
{
    if (c.has_bias || !(c.Cin * c.K * c.K <= 32 || (c.Cin <= 4 && c.Cin * c.K * c.K <= 160))) return false;
    if (c.pooled && (c.S != 1 || c.K > 3)) return false;
    if (c.pooled) {
        // owned rectangles of a pooled convolution consist of whole windows; anything else goes to the generic kernel
        for (int t = 0; t < c.M; ++t) if ((c.rect.x0[t] & 1) || !((c.rect.x1[t] - c.rect.x0[t]) & 1)) return false;
        for (int t = 0; t < c.N; ++t) if ((c.rect.y0[t] & 1) || !((c.rect.y1[t] - c.rect.y0[t]) & 1)) return false;
    }
    if (c.Cin <= 4 && stream_geom(c).fits) return true;
    return thin_geom(c).lds <= 64 * 1024;
}

void thin_wgrad(const ConvArgs& c, float* scratch, hipStream_t s)
{
    MfmaWgradArgs a;
    a.in = c.in; a.din = c.din; a.mask = c.mask; a.own = c.rect;
    a.partial = c.partial; a.scratch = scratch; a.n_params = c.n_params; a.w_off = c.w_off;
    a.Cin = c.Cin; a.Cout = c.Cout; a.Hc = c.Hi; a.Wc = c.Wi; a.slope = c.slope; a.M = c.M; a.batch = c.batch;
    a.splits = c.wgrad_shares_thin;
    const int nb = (c.Cin * c.K * c.K + 31) / 32;      // 1 (up to 3x3), 2 or 4 (5x5), 4 to 7 (7x7: 5 for 3 channels)
    dim3 grid((c.Cout + 31) / 32, a.splits, c.N * c.M), block(256);
    const ThinStream ts = c.Cin <= 4 ? stream_geom(c) : ThinStream{0, 0, 0, 1, 1, 1, 0, false};
    const bool stream = ts.fits;
    const ThinGeom g = stream ? ThinGeom{ts.cb_max, ts.lds} : thin_geom(c);
    a.PK = g.PK; a.zs = ts.zs; a.stage_words = ts.stage_words;
    // more than 64 KB of dynamic LDS has to be granted per kernel, once
#define FTP_TW(T, TN, KK, SS, NB, PL) do { \
        if (stream) { \
            static thread_local size_t granted = 64 * 1024; \
            if (g.lds > granted) { (void)hipFuncSetAttribute((const void*)k_wgrad_thin_dl<T, KK, SS, NB, PL>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)g.lds); granted = g.lds; } \
            g_kernel_label = "k_wgrad_thin_dl<" TN ", " #KK ", " #SS ", " #NB ", " #PL ">"; \
            hipLaunchKernelGGL((k_wgrad_thin_dl<T, KK, SS, NB, PL>), grid, dim3(320), g.lds, s, a); \
        } else { \
            g_kernel_label = "k_wgrad_mfma_thin"; \
            hipLaunchKernelGGL((k_wgrad_mfma_thin<T, KK, SS, NB, PL>), grid, block, g.lds, s, a); \
        } } while (0)
#define FTP_TWS(T, TN, KK, NB) do { if (c.S == 2) FTP_TW(T, TN, KK, 2, NB, false); else FTP_TW(T, TN, KK, 1, NB, false); } while (0)
#define FTP_TWK(T, TN) do { \
        if (c.K == 7)      { if (nb <= 4) FTP_TWS(T, TN, 7, 4); else FTP_TWS(T, TN, 7, 5); } \
        else if (c.K == 5) { if (nb <= 2) FTP_TWS(T, TN, 5, 2); else FTP_TWS(T, TN, 5, 4); } \
        else if (c.K == 3) { if (nb <= 1) { if (c.pooled) FTP_TW(T, TN, 3, 1, 1, true); else FTP_TWS(T, TN, 3, 1); } \
                             else         { if (c.pooled) FTP_TW(T, TN, 3, 1, 2, true); else FTP_TWS(T, TN, 3, 2); } } \
        else               { if (c.pooled) FTP_TW(T, TN, 1, 1, 1, true); else FTP_TWS(T, TN, 1, 1); } } while (0)
    if (c.bf16) FTP_TWK(bf16_t, "unsigned short"); else FTP_TWK(float, "float");
#undef FTP_TWK
#undef FTP_TWS
#undef FTP_TW
}

}  // namespace ftp
