// fp32 matrix-core (MFMA) per-stack filter gradient for gfx950.
//   dW[co][ci][tap] = sum over the batch and the stack's owned output pixels q of dZ[co][q] * X[ci][q + tap - P]
// is a GEMM with M = co, N = ci and the pixels as reduction dimension, one accumulator tile per tap.
// A workgroup (4 wavefronts) owns a 32*WAVES_CO x 32*WAVES_CI block of (co, ci) for one stack and one
// share of the batch.  Per step it stages TI images x TR rows of the owned rectangle in LDS, pixel-major
// (channel contiguous) so that v_mfma_f32_32x32x2_f32 finds A[m = co][k = pixel] and B[k = pixel][n = ci]
// at consecutive addresses: dZ as [pixel][co], X as [(row, column) incl. filter halo][ci].
// Rows are padded to an even number of pixels (dZ = 0 there) because one MFMA consumes two pixels.
#include "ftp_device.h"
#include "ftp_launch.h"

namespace ftp {

typedef float v16f __attribute__((ext_vector_type(16)));

template <typename T, int K, int WAVES_CO, int WAVES_CI, bool POOL>
__global__ void __launch_bounds__(256)
k_wgrad_mfma(MfmaWgradArgs a)
{
    constexpr int WAVES_K = 4 / (WAVES_CO * WAVES_CI);
    constexpr int KK = K * K, P = K / 2;
    constexpr int BCO = 32 * WAVES_CO, BCI = 32 * WAVES_CI;
    constexpr int ZP = BCO + 1, XP = BCI + 1;          // odd strides: conflict-free transposing writes

    extern __shared__ float lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_co = wave % WAVES_CO, wave_ci = (wave / WAVES_CO) % WAVES_CI, wave_k = wave / (WAVES_CO * WAVES_CI);
    const int hi = lane >> 5, l32 = lane & 31;
    const int stack = blockIdx.z, ti = stack / a.M, tj = stack % a.M;
    const int x0 = a.own.x0[tj], x1 = a.own.x1[tj], y0 = a.own.y0[ti], y1 = a.own.y1[ti];
    const int rw = x1 - x0 + 1, rh = y1 - y0 + 1;
    const int tiles_ci = (a.Cin + BCI - 1) / BCI;
    const int co0 = (blockIdx.x / tiles_ci) * BCO, ci0 = (blockIdx.x % tiles_ci) * BCI;
    const int split = blockIdx.y;
    const int nb0 = (int)((long long)split * a.batch / a.splits), nb1 = (int)((long long)(split + 1) * a.batch / a.splits);

    // chunk geometry for this stack: TI images x TR rows x rw columns (rows padded to even)
    const int TCp = (rw + 1) & ~1;
    int TR = a.PK / TCp; if (TR < 1) TR = 1; if (TR > rh) TR = rh;
    int TI = 1;
    if (TR == rh) { TI = a.PK / (TCp * rh); if (TI < 1) TI = 1; }
    const int PW = TCp + 2 * P, PH = TR + 2 * P;      // patch rows as wide as the padded pixel rows
    float* Zl = lds;                                   // [TI*TR*TCp][ZP]
    float* Xl = lds + a.PK * ZP;                       // [TI*PH*PW][XP]
    const int row_blocks = (rh + TR - 1) / TR;

    v16f acc[KK];
#pragma unroll
    for (int t = 0; t < KK; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[t][i] = 0.0f;

    const int co_l = wave_co * 32 + l32, ci_l = wave_ci * 32 + l32;
    // staging: lane -> (row within a pass, column)
    const int zrows = 64 / TCp > 0 ? 64 / TCp : 1, zsub = lane / TCp, zcol = lane - zsub * TCp;
    const int xrows = 64 / PW > 0 ? 64 / PW : 1, xsub = lane / PW, xcol = lane - xsub * PW;

    for (int n0 = nb0; n0 < nb1; n0 += TI) {
        const int ni = (nb1 - n0) < TI ? (nb1 - n0) : TI;
        for (int rb = 0; rb < row_blocks; ++rb) {
            const int yb = y0 + rb * TR;
            const int nr = (y1 - yb + 1) < TR ? (y1 - yb + 1) : TR;
            __syncthreads();
            // ---- stage dZ: [image][row][padded column][co] -------------------------------------------------
            // A wavefront covers `zrows` rows of TCp columns at once (lane -> row, column) and walks its share
            // of the channels 8 at a time, so that 16 independent loads are in flight.
            {
                const int nrows = ni * nr;
                for (int rbase = 0; rbase < nrows; rbase += zrows)
                for (int cofs = 0; cofs < TCp; cofs += 64) {             // rows wider than a wavefront take several passes
                    const int row = rbase + zsub, zc = zcol + cofs;
                    const bool rok = zsub < zrows && row < nrows && zc < TCp;
                    const int rowc = rok ? row : 0;
                    const int il = rowc / nr, r = rowc - il * nr;
                    const int qy = yb + r, qx = x0 + (zc < rw ? zc : rw - 1);
                    const int sy = POOL ? (qy >> 1) : qy, sx = POOL ? (qx >> 1) : qx;
                    const int code = ((qy & 1) << 1) | (qx & 1);
                    const uint8_t* mp = at<uint8_t>(a.mask, stack, ti, tj, n0 + il, 0, sy, sx);
                    const T* gp = at<T>(a.din, stack, ti, tj, n0 + il, 0, sy, sx);
                    float* zdst = Zl + (rowc * TCp + (rok ? zc : 0)) * ZP;
                    // all of this lane's loads are issued before the first use
                    uint8_t m[BCO / 4]; float g[BCO / 4];
#pragma unroll
                    for (int k = 0; k < BCO / 4; ++k) {
                        const int c = wave + 4 * k;
                        const int co = co0 + c < a.Cout ? co0 + c : a.Cout - 1;
                        m[k] = mp[(long long)co * a.mask.cs];
                        g[k] = ld(gp + (long long)co * a.din.cs);
                    }
#pragma unroll
                    for (int k = 0; k < BCO / 4; ++k) {
                        const int c = wave + 4 * k;
                        float v = (m[k] & 1) ? g[k] : a.slope * g[k];
                        if (POOL && ((m[k] >> 1) & 3) != code) v = 0.0f;
                        if (zc >= rw || co0 + c >= a.Cout) v = 0.0f;
                        if (rok) zdst[c] = v;
                    }
                }
            }
            // ---- stage X: [image][patch row][patch column][ci] --------------------------------------------
            {
                const int nph = nr + 2 * P;
                const int nprow = ni * nph;
                for (int rbase = 0; rbase < nprow; rbase += xrows)
                for (int cofs = 0; cofs < PW; cofs += 64) {
                    const int prow = rbase + xsub, xc = xcol + cofs;
                    const bool rok = xsub < xrows && prow < nprow && xc < PW;
                    const int prc = rok ? prow : 0;
                    const int il = prc / nph, r = prc - il * nph;
                    const int gy = yb - P + r, gx = x0 - P + xc;
                    const bool inside = xc < rw + 2 * P && gy >= 0 && gy < a.Hc && gx >= 0 && gx < a.Wc;
                    const T* xp = at<T>(a.in, stack, ti, tj, n0 + il, 0, inside ? gy : y0, inside ? gx : x0);
                    float* xdst = Xl + ((il * PH + r) * PW + (rok ? xc : 0)) * XP;
                    float g[BCI / 4];
#pragma unroll
                    for (int k = 0; k < BCI / 4; ++k) {
                        const int c = wave + 4 * k;
                        const int ci = ci0 + c < a.Cin ? ci0 + c : a.Cin - 1;
                        g[k] = ld(xp + (long long)ci * a.in.cs);
                    }
#pragma unroll
                    for (int k = 0; k < BCI / 4; ++k) {
                        const int c = wave + 4 * k;
                        if (rok) xdst[c] = (inside && ci0 + c < a.Cin) ? g[k] : 0.0f;
                    }
                }
            }
            __syncthreads();
            // ---- multiply ------------------------------------------------------------------------------------
            const int nrows = ni * nr;
            for (int rr = wave_k; rr < nrows; rr += WAVES_K) {
                const int il = rr / nr, r = rr - il * nr;
                const float* zrow = Zl + (rr * TCp + hi) * ZP + co_l;
                const float* xrow = Xl + ((il * PH + r) * PW + hi) * XP + ci_l;
                for (int xp = 0; xp < TCp; xp += 2) {
                    const float av = zrow[xp * ZP];
#pragma unroll
                    for (int t = 0; t < KK; ++t) {
                        const float bv = xrow[((t / K) * PW + xp + (t % K)) * XP];
                        acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[t], 0, 0, 0);
                    }
                }
            }
        }
    }

    // ---- combine the pixel-split wavefronts (fixed order), then store -----------------------------------------
    if (WAVES_K > 1) {
        __syncthreads();
        float* red = lds;                               // [WAVES_CO*WAVES_CI][16][64]
#pragma unroll
        for (int t = 0; t < KK; ++t) {
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
        const long long layer_params = (long long)a.Cout * a.Cin * KK;
        float* dst = a.splits > 1 ? a.scratch + ((long long)stack * a.splits + split) * layer_params
                                  : a.partial + (long long)stack * a.n_params + a.w_off;
        const int ci = ci0 + ci_l;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int co = co0 + wave_co * 32 + 8 * (i >> 2) + 4 * hi + (i & 3);
            if (co < a.Cout && ci < a.Cin) {
#pragma unroll
                for (int t = 0; t < KK; ++t) dst[((long long)co * a.Cin + ci) * KK + t] = acc[t][i];
            }
        }
    }
}

// Sum of the batch shares of one layer's partial gradient, in share order.
__global__ void __launch_bounds__(256)
k_wgrad_splitk_reduce(const float* __restrict__ scratch, float* __restrict__ partial, long long layer_params, long long n_params,
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

struct WgradGeom { int PK; size_t lds; int waves_ci; };

// Pixels staged per step and the LDS the largest stack needs (c.rect = owned rectangles).
WgradGeom wgrad_geom(const ConvArgs& c)
{
    WgradGeom g;
    g.PK = 64;
    const int P = c.K / 2;
    int max_pos = 1;
    for (int t = 0; t < c.M; ++t) { const int w = ((c.rect.x1[t] - c.rect.x0[t] + 2) & ~1); if (w > g.PK) g.PK = w; }   // one full padded row at least
    for (int i = 0; i < c.N; ++i)
        for (int j = 0; j < c.M; ++j) {
            const int rw = c.rect.x1[j] - c.rect.x0[j] + 1, rh = c.rect.y1[i] - c.rect.y0[i] + 1;
            const int TCp = (rw + 1) & ~1;
            int TR = g.PK / TCp; if (TR < 1) TR = 1; if (TR > rh) TR = rh;
            int TI = 1; if (TR == rh) { TI = g.PK / (TCp * rh); if (TI < 1) TI = 1; }
            const int pos = TI * (TR + 2 * P) * (TCp + 2 * P);
            if (pos > max_pos) max_pos = pos;
        }
    g.waves_ci = c.Cin >= 64 ? 2 : 1;
    g.lds = ((size_t)g.PK * (64 + 1) + (size_t)max_pos * (32 * g.waves_ci + 1)) * sizeof(float);
    return g;
}

}  // namespace

// c.rect must hold the owned rectangles.
bool mfma_wgrad_eligible(const ConvArgs& c)
{
    if (c.has_bias || c.Cout < 32 || c.Cin < 16) return false;
    return wgrad_geom(c).lds <= 64 * 1024;
}

int mfma_wgrad_splits(const ConvArgs& c)
{
    return wgrad_batch_shares(c.Cout, c.Cin, c.N * c.M, c.batch);
}

// c.rect = owned rectangle at the convolution output (before the pool); scratch holds the batch shares.
void mfma_wgrad(const ConvArgs& c, float* scratch, hipStream_t s)
{
    MfmaWgradArgs a;
    a.in = c.in; a.din = c.din; a.mask = c.mask; a.own = c.rect;
    a.partial = c.partial; a.scratch = scratch; a.n_params = c.n_params; a.w_off = c.w_off;
    a.Cin = c.Cin; a.Cout = c.Cout; a.Hc = c.Hc; a.Wc = c.Wc; a.slope = c.slope; a.M = c.M; a.batch = c.batch;
    a.splits = mfma_wgrad_splits(c);
    const WgradGeom g = wgrad_geom(c);
    a.PK = g.PK;
    const int waves_ci = g.waves_ci;
    const int BCO = 64, BCI = 32 * waves_ci;
    const size_t lds = g.lds;
    const int tiles = ((c.Cout + BCO - 1) / BCO) * ((c.Cin + BCI - 1) / BCI);
    dim3 grid(tiles, a.splits, c.N * c.M), block(256);
#define FTP_WG(KK, WCI, PL) do { if (c.bf16) { g_kernel_label = "k_wgrad_mfma<unsigned short, " #KK ", 2, " #WCI ", " #PL ">"; hipLaunchKernelGGL((k_wgrad_mfma<bf16_t, KK, 2, WCI, PL>), grid, block, lds, s, a); } else { g_kernel_label = "k_wgrad_mfma<float, " #KK ", 2, " #WCI ", " #PL ">"; hipLaunchKernelGGL((k_wgrad_mfma<float, KK, 2, WCI, PL>), grid, block, lds, s, a); } } while (0)
    if (c.K == 3) {
        if (waves_ci == 2) { if (c.pooled) FTP_WG(3, 2, true); else FTP_WG(3, 2, false); }
        else               { if (c.pooled) FTP_WG(3, 1, true); else FTP_WG(3, 1, false); }
    } else {
        if (waves_ci == 2) { if (c.pooled) FTP_WG(1, 2, true); else FTP_WG(1, 2, false); }
        else               { if (c.pooled) FTP_WG(1, 1, true); else FTP_WG(1, 1, false); }
    }
#undef FTP_WG
    if (a.splits > 1) {
        const long long lp = (long long)c.Cout * c.Cin * c.K * c.K;
        dim3 g2((unsigned)((lp + 255) / 256), c.N * c.M);
        hipLaunchKernelGGL(k_wgrad_splitk_reduce, g2, dim3(256), 0, s, scratch, c.partial, lp, c.n_params, c.w_off, a.splits);
    }
}

}  // namespace ftp
