// fp32 matrix-core (MFMA) implicit-GEMM convolution for gfx950, used for the forward pass and for the
// delta back-propagation (which is the same convolution with the 180-degree rotated, transposed
// filter applied to dZ).  D[m][pixel] = sum_k Wt[k][m] * patch[k][pixel], k = (tap, channel).
//
// One workgroup (4 wavefronts) produces BM = 32*WAVES_M output channels for a tile of 256 pixels of
// one stack: TI images x TR rows x TC columns of the stack's rectangle (pooled layers: 64 windows of
// 4 pixels).  The input patch (tile + filter halo, zero outside the real map) and the filter slice
// of 8 channels x K*K taps are staged in LDS; v_mfma_f32_32x32x2_f32 reads both from there.
// MFMA lane layout (64 lanes): A[m = lane%32][k = lane/32], B[k = lane/32][n = lane%32],
// D[m = 8*(i/4) + 4*(lane/32) + i%4][n = lane%32] for accumulator register i of 16.
#include "ftp_device.h"
#include "ftp_launch.h"

namespace ftp {

typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kBN = 256;        // pixels per workgroup tile

// Filter relayout: OIHW -> [tap][reduction channel][output channel], so that a stage's slice is a set of
// contiguous rows.  fwd: Wt[t][ci][co] = W[co][ci][t].  bwd: Wt[t][co][ci] = W[co][ci][K*K-1-t] (rotated).
__global__ void __launch_bounds__(256, 2)
k_prep_filter(const float* __restrict__ w, float* __restrict__ wt_fwd, float* __restrict__ wt_bwd, int Cout, int Cin, int KK)
{
    const long long n = (long long)Cout * Cin * KK;
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int t = (int)(i % KK);
    const int ci = (int)((i / KK) % Cin);
    const int co = (int)(i / ((long long)KK * Cin));
    const float v = w[i];
    if (wt_fwd) wt_fwd[((long long)t * Cin + ci) * Cout + co] = v;
    if (wt_bwd) wt_bwd[((long long)(KK - 1 - t) * Cout + co) * Cin + ci] = v;
}

// Reduction channels staged per step: fewer for the 128-channel tile, whose accumulators leave fewer registers
// for the prefetched next stage.
__host__ __device__ constexpr int conv_stage_channels(int K, int BM) { return K == 1 ? (BM == 128 ? 16 : 32) : (BM == 128 ? 4 : 8); }

// Pixel (or pool window) q of a tile -> image, row, column inside the tile.
struct TilePix { int il, yl, xl; };
__device__ __forceinline__ TilePix tile_pix(int wq, int per_img, int TC)
{
    TilePix t;
    t.il = wq / per_img;
    const int rem = wq - t.il * per_img;
    t.yl = rem / TC;
    t.xl = rem - t.yl * TC;
    return t;
}

// WAVES_M x WAVES_N wavefronts; each computes MT x NT tiles of 32 channels x 32 pixels.
template <int K, int WAVES_M, int MT, bool POOL_OUT, bool DELTA_IN, bool POOL_IN>
__global__ void __launch_bounds__(256, 2)
k_conv_mfma(MfmaConvArgs a)
{
    constexpr int kCK = conv_stage_channels(K, 32 * MT * WAVES_M);   // reduction channels per LDS stage
    constexpr int WAVES_N = 4 / WAVES_M;
    constexpr int NT = kBN / 32 / WAVES_N;           // 32-pixel MFMA tiles per wavefront
    constexpr int BM = 32 * MT * WAVES_M;
    constexpr int KK = K * K, P = K / 2;
    constexpr int S = POOL_OUT ? 2 : 1;

    extern __shared__ float lds[];
    float* Wl = lds;                                   // [KK][kCK][BM]
    float* Xl = lds + KK * kCK * BM;                   // [kCK][TI][PH][PW]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_m = wave % WAVES_M, wave_n = wave / WAVES_M;
    const int hi = lane >> 5, l32 = lane & 31;
    const int stack = blockIdx.z, ti = stack / a.M, tj = stack % a.M;
    const int x0 = a.rect.x0[tj], x1 = a.rect.x1[tj], y0 = a.rect.y0[ti], y1 = a.rect.y1[ti];
    const int bx = blockIdx.x;
    const int tx = bx % a.tiles_x, ty = (bx / a.tiles_x) % a.tiles_y, tb = bx / (a.tiles_x * a.tiles_y);
    const int ox0 = x0 + tx * a.TC, oy0 = y0 + ty * a.TR, n0 = tb * a.TI;
    if (ox0 > x1 || oy0 > y1) return;                 // this stack's rectangle is smaller than the largest one
    const int m0 = blockIdx.y * BM;
    const int PW = a.TC * S + 2 * P, PH = a.TR * S + 2 * P;
    const int IS = PH * PW, CS = a.TI * IS;
    const int px0 = ox0 * S - P, py0 = oy0 * S - P;   // patch origin in the coordinates of the convolution input
    const int per_img = a.TR * a.TC;

    // ---- LDS offset of each lane's pixel, per 32-pixel tile ---------------------------------------------
    int baseB[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int q = (wave_n * NT + t) * 32 + l32;
        const TilePix tp = tile_pix(POOL_OUT ? (q >> 2) : q, per_img, a.TC);
        const int pos = POOL_OUT ? (q & 3) : 0;
        const bool v = tp.il < a.TI && n0 + tp.il < a.batch && oy0 + tp.yl <= y1 && ox0 + tp.xl <= x1;
        baseB[t] = (v ? tp.il * IS + (tp.yl * S + (pos >> 1)) * PW + tp.xl * S + (pos & 1) : 0) + hi * CS;
    }
    const int baseA = hi * BM + wave_m * (32 * MT) + l32;

    // ---- per-thread patch positions (fixed over the channel loop): 32-bit offsets from per-workgroup bases ------
    constexpr int MAXPOS = K == 1 ? 1 : 2;
    const int npos = a.TI * IS;
    const View& sv = DELTA_IN ? a.din : a.in;          // source of the patch values
    const float* __restrict__ src = (const float*)sv.p + (long long)stack * sv.ss + (long long)n0 * sv.ns;
    const uint8_t* __restrict__ msk = (const uint8_t*)a.mask.p + (long long)stack * a.mask.ss + (long long)n0 * a.mask.ns;
    int goff[MAXPOS];               // source element offset (channel 0); -1: zero padding / outside the view
    int moff[MAXPOS];               // DELTA_IN: offset in the decision-code map, winner code in the top bits
#pragma unroll
    for (int j = 0; j < MAXPOS; ++j) {
        const int s = tid + j * 256;
        goff[j] = -1; moff[j] = 0;
        if (s < npos) {
            const int il = s / IS, rem = s - il * IS;
            const int r = rem / PW, c = rem - r * PW;
            const int gy = py0 + r, gx = px0 + c;
            if (n0 + il < a.batch && gy >= 0 && gy < a.Hc && gx >= 0 && gx < a.Wc) {
                const int sy = POOL_IN ? (gy >> 1) : gy, sx = POOL_IN ? (gx >> 1) : gx;
                // positions no valid output pixel of this stack reads may lie outside the view
                if (sy >= a.iy0[ti] && sy <= a.iy1[ti] && sx >= a.ix0[tj] && sx <= a.ix1[tj]) {
                    goff[j] = il * (int)sv.ns + (sy - sv.y0[ti]) * sv.pitch + (sx - sv.x0[tj]);
                    if (DELTA_IN) {
                        moff[j] = il * (int)a.mask.ns + (sy - a.mask.y0[ti]) * a.mask.pitch + (sx - a.mask.x0[tj]);
                        if (POOL_IN) moff[j] |= (((gy & 1) << 1) | (gx & 1)) << 29;
                    }
                }
            }
        }
    }

    v16f acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[mt][t][i] = 0.0f;

    const float* __restrict__ wt = a.wt;
    // Software pipeline: the next stage's filter slice and patch are fetched into registers while the matrix
    // cores work on the current stage, and written to LDS between two barriers.
    constexpr int WREG = (KK * kCK * (BM / 4) + 255) / 256;
    float4 wreg[WREG];
    float greg[MAXPOS][kCK];
    uint8_t mreg[MAXPOS][kCK];
    auto prefetch = [&](int c0) {
#pragma unroll
        for (int u = 0; u < WREG; ++u) {
            const int idx = tid + u * 256;
            const int row = idx / (BM / 4), c4 = idx - row * (BM / 4);
            const int tap = row / kCK, cl = row - tap * kCK;
            const int ci = c0 + cl, m = m0 + c4 * 4;
            wreg[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (idx < KK * kCK * (BM / 4) && ci < a.C && m < a.Mtot) wreg[u] = *(const float4*)(wt + ((long long)tap * a.C + ci) * a.Mtot + m);
        }
#pragma unroll
        for (int j = 0; j < MAXPOS; ++j) {
            const int go = goff[j] >= 0 ? goff[j] : 0, mo = moff[j] & 0x1FFFFFFF;
#pragma unroll
            for (int k = 0; k < kCK; ++k) {
                const int ci = c0 + k < a.C ? c0 + k : a.C - 1;
                greg[j][k] = src[go + (long long)ci * sv.cs];
                if (DELTA_IN) mreg[j][k] = msk[mo + (long long)ci * a.mask.cs];
            }
        }
    };
    auto commit = [&](int c0) {
#pragma unroll
        for (int u = 0; u < WREG; ++u) {
            const int idx = tid + u * 256;
            if (idx < KK * kCK * (BM / 4)) *(float4*)(Wl + idx * 4) = wreg[u];
        }
#pragma unroll
        for (int j = 0; j < MAXPOS; ++j) {
            const int s = tid + j * 256;
            if (s < npos) {
                const bool inside = goff[j] >= 0;
                const unsigned code = (unsigned)moff[j] >> 29;
#pragma unroll
                for (int k = 0; k < kCK; ++k) {
                    float v = greg[j][k];
                    if (DELTA_IN) {
                        v = (mreg[j][k] & 1) ? v : a.slope * v;
                        if (POOL_IN && ((mreg[j][k] >> 1) & 3) != code) v = 0.0f;
                    }
                    if (!inside || c0 + k >= a.C) v = 0.0f;
                    Xl[k * CS + s] = v;
                }
            }
        }
    };
    prefetch(0);
    for (int c0 = 0; c0 < a.C; c0 += kCK) {
        __syncthreads();
        commit(c0);
        __syncthreads();
        if (c0 + kCK < a.C) prefetch(c0 + kCK);
#pragma unroll
        for (int tap = 0; tap < KK; ++tap) {
            const int toff = (tap / K) * PW + (tap % K);
#pragma unroll
            for (int i = 0; i < kCK / 2; ++i) {
                float av[MT], bv[NT];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) av[mt] = Wl[(tap * kCK + 2 * i) * BM + baseA + 32 * mt];
#pragma unroll
                for (int t = 0; t < NT; ++t) bv[t] = Xl[baseB[t] + 2 * i * CS + toff];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int t = 0; t < NT; ++t)
                        acc[mt][t] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[mt], bv[t], acc[mt][t], 0, 0, 0);
            }
        }
    }

    // ---- epilogue ------------------------------------------------------------------------------------------
    // A lane holds, per 32x32 tile, 16 channels (8*(i/4) + 4*hi + i%4) of one pixel.
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int q = (wave_n * NT + t) * 32 + l32;
        const TilePix tp = tile_pix(POOL_OUT ? (q >> 2) : q, per_img, a.TC);
        const int pn = n0 + tp.il, py = oy0 + tp.yl, pxx = ox0 + tp.xl;
        bool pvalid = tp.il < a.TI && pn < a.batch && py <= y1 && pxx <= x1;
        if (POOL_OUT) pvalid = pvalid && (lane & 3) == 0;       // the window's first lane stores
        const bool powned = pvalid && !DELTA_IN && py >= a.own.y0[ti] && py <= a.own.y1[ti] && pxx >= a.own.x0[tj] && pxx <= a.own.x1[tj];
        const View& ov = DELTA_IN ? a.dout : a.out;
        float* __restrict__ optr = at<float>(ov, stack, ti, tj, pn, 0, py, pxx);
        uint8_t* __restrict__ mptr = at<uint8_t>(a.mask, stack, ti, tj, pn, 0, py, pxx);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int m = m0 + (wave_m * MT + mt) * 32 + 8 * (i >> 2) + 4 * hi + (i & 3);
                float v = acc[mt][t][i];
                if (DELTA_IN) {
                    if (pvalid && m < a.Mtot) optr[(long long)m * ov.cs] = v;
                } else {
                    const float b = (a.bias && m < a.Mtot) ? a.bias[m] : 0.0f;
                    v = leaky(v + b, a.slope);
                    int bi = 0;
                    if (POOL_OUT) {
                        // the 4 pixels of a window sit in 4 adjacent lanes, in window order; the first lane decides
                        const float o1 = __shfl_xor(v, 1, 64), o2 = __shfl_xor(v, 2, 64), o3 = __shfl_xor(v, 3, 64);
                        if (o1 > v) { v = o1; bi = 1; }
                        if (o2 > v) { v = o2; bi = 2; }
                        if (o3 > v) { v = o3; bi = 3; }
                    }
                    if (pvalid && m < a.Mtot) {
                        optr[(long long)m * ov.cs] = v;
                        if (powned) mptr[(long long)m * a.mask.cs] = (uint8_t)((bi << 1) | (v > 0.0f ? 1 : 0));
                    }
                }
            }
        }
    }
}

// ---- host side ------------------------------------------------------------------------------------------------
namespace {

struct TileChoice { int TI, TR, TC, tiles_x, tiles_y, tiles_i, npos; };

// Largest rectangle of any stack decides the tile shape: whole rectangles of several images when they are
// small, bands of rows otherwise, column blocks only for rectangles wider than a tile.
TileChoice choose_tile(int rw, int rh, int batch, int cap /* pixels (or windows) per tile */, int S, int P)
{
    TileChoice c;
    c.TC = rw <= cap ? rw : cap;
    if (c.TC > 64) c.TC = 64;
    c.tiles_x = (rw + c.TC - 1) / c.TC;
    c.TC = (rw + c.tiles_x - 1) / c.tiles_x;
    int rows = cap / c.TC; if (rows < 1) rows = 1;
    if (rows >= rh) {
        c.TR = rh; c.tiles_y = 1;
        c.TI = cap / (c.TC * c.TR); if (c.TI < 1) c.TI = 1; if (c.TI > batch) c.TI = batch;
    } else {
        c.tiles_y = (rh + rows - 1) / rows;
        c.TR = (rh + c.tiles_y - 1) / c.tiles_y;
        c.TI = 1;
    }
    c.tiles_i = (batch + c.TI - 1) / c.TI;
    c.npos = c.TI * (c.TR * S + 2 * P) * (c.TC * S + 2 * P);
    // the staging registers hold at most 2*256 patch positions per workgroup (256 without a filter halo)
    while (c.npos > (P > 0 ? 512 : 256)) {
        if (c.TI > 1) { --c.TI; c.tiles_i = (batch + c.TI - 1) / c.TI; }
        else { ++c.tiles_y; c.TR = (rh + c.tiles_y - 1) / c.tiles_y; }
        c.npos = c.TI * (c.TR * S + 2 * P) * (c.TC * S + 2 * P);
    }
    return c;
}

template <int K, bool POOL_OUT, bool DELTA_IN, bool POOL_IN>
void launch_m(MfmaConvArgs& a, int stacks, hipStream_t s)
{
    const int KK = K * K;
    // output channels per workgroup: 128 (2x2 wavefronts of 64 x 128 pixels), 64 (1x4 of 64 x 64) or 32 (1x4 of 32 x 64)
    const int BM = a.Mtot >= 128 ? 128 : a.Mtot > 32 ? 64 : 32;
    const int CS = a.TI * (a.TR * (POOL_OUT ? 2 : 1) + 2 * (K / 2)) * (a.TC * (POOL_OUT ? 2 : 1) + 2 * (K / 2));
    const int kCK = conv_stage_channels(K, BM);
    const size_t lds = (size_t)(KK * kCK * BM + kCK * CS) * sizeof(float);
    dim3 grid(a.tiles_x * a.tiles_y * a.tiles_i, (a.Mtot + BM - 1) / BM, stacks), block(256);
    if (BM == 128) hipLaunchKernelGGL((k_conv_mfma<K, 2, 2, POOL_OUT, DELTA_IN, POOL_IN>), grid, block, lds, s, a);
    else if (BM == 64) hipLaunchKernelGGL((k_conv_mfma<K, 1, 2, POOL_OUT, DELTA_IN, POOL_IN>), grid, block, lds, s, a);
    else hipLaunchKernelGGL((k_conv_mfma<K, 1, 1, POOL_OUT, DELTA_IN, POOL_IN>), grid, block, lds, s, a);
}

void rect_max(const RectTab& rt, int N, int M, int& mw, int& mh)
{
    mw = 0; mh = 0;
    for (int t = 0; t < M; ++t) mw = mw > rt.x1[t] - rt.x0[t] + 1 ? mw : rt.x1[t] - rt.x0[t] + 1;
    for (int t = 0; t < N; ++t) mh = mh > rt.y1[t] - rt.y0[t] + 1 ? mh : rt.y1[t] - rt.y0[t] + 1;
}

}  // namespace

bool mfma_conv_eligible(const ConvArgs& a, bool backward)
{
    if (a.bf16) return false;
    const int Mtot = backward ? a.Cin : a.Cout, C = backward ? a.Cout : a.Cin;
    return Mtot >= 16 && Mtot % 4 == 0 && C >= 8;
}

void prep_filter(const float* w, float* wt_fwd, float* wt_bwd, int Cout, int Cin, int K, hipStream_t s)
{
    const long long n = (long long)Cout * Cin * K * K;
    hipLaunchKernelGGL(k_prep_filter, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, w, wt_fwd, wt_bwd, Cout, Cin, K * K);
}

// Forward: a.rect = held rectangle at the unit's output boundary; a.inrect = extent of the input view per stack.
void mfma_conv_fwd(const ConvArgs& c, const RectTab& inrect, const float* wt, hipStream_t s)
{
    MfmaConvArgs a;
    a.in = c.in; a.out = c.out; a.mask = c.mask; a.din = c.din; a.dout = c.dout; a.rect = c.rect; a.own = c.own;
    for (int t = 0; t < kTabGrid; ++t) { a.ix0[t] = inrect.x0[t]; a.ix1[t] = inrect.x1[t]; a.iy0[t] = inrect.y0[t]; a.iy1[t] = inrect.y1[t]; }
    a.wt = wt; a.bias = (const float*)c.bias;
    a.C = c.Cin; a.Mtot = c.Cout; a.Hc = c.Hc; a.Wc = c.Wc; a.slope = c.slope; a.M = c.M; a.batch = c.batch;
    int mw, mh; rect_max(c.rect, c.N, c.M, mw, mh);
    const int S = c.pooled ? 2 : 1, P = c.K / 2;
    const TileChoice tc = choose_tile(mw, mh, c.batch, c.pooled ? kBN / 4 : kBN, S, P);
    a.TI = tc.TI; a.TR = tc.TR; a.TC = tc.TC; a.tiles_x = tc.tiles_x; a.tiles_y = tc.tiles_y; a.tiles_i = tc.tiles_i;
    const int stacks = c.N * c.M;
    if (c.K == 3) { if (c.pooled) launch_m<3, true, false, false>(a, stacks, s); else launch_m<3, false, false, false>(a, stacks, s); }
    else          { if (c.pooled) launch_m<1, true, false, false>(a, stacks, s); else launch_m<1, false, false, false>(a, stacks, s); }
}

// Backward data: a.rect = backward rectangle at the unit's input boundary; inrect = extent of the delta view
// (at the unit's output boundary, pooled coordinates if the unit has a pool).
void mfma_conv_bwd_data(const ConvArgs& c, const RectTab& inrect, const float* wt, hipStream_t s)
{
    MfmaConvArgs a;
    a.in = c.in; a.out = c.out; a.mask = c.mask; a.din = c.din; a.dout = c.dout; a.rect = c.rect; a.own = c.own;
    for (int t = 0; t < kTabGrid; ++t) { a.ix0[t] = inrect.x0[t]; a.ix1[t] = inrect.x1[t]; a.iy0[t] = inrect.y0[t]; a.iy1[t] = inrect.y1[t]; }
    a.wt = wt; a.bias = nullptr;
    a.C = c.Cout; a.Mtot = c.Cin; a.Hc = c.Hc; a.Wc = c.Wc; a.slope = c.slope; a.M = c.M; a.batch = c.batch;
    int mw, mh; rect_max(c.rect, c.N, c.M, mw, mh);
    const TileChoice tc = choose_tile(mw, mh, c.batch, kBN, 1, c.K / 2);
    a.TI = tc.TI; a.TR = tc.TR; a.TC = tc.TC; a.tiles_x = tc.tiles_x; a.tiles_y = tc.tiles_y; a.tiles_i = tc.tiles_i;
    const int stacks = c.N * c.M;
    if (c.K == 3) { if (c.pooled) launch_m<3, false, true, true>(a, stacks, s); else launch_m<3, false, true, false>(a, stacks, s); }
    else          { if (c.pooled) launch_m<1, false, true, true>(a, stacks, s); else launch_m<1, false, true, false>(a, stacks, s); }
}

}  // namespace ftp
