// Delta back-propagation through a 3x3 (or 1x1) stride-2 convolution on the matrix cores without multiplying zeros, gfx950.
// Eq. (2) with S_l = 2: input pixel (2j + a, 2i + b) receives W[ky][kx]^T dZ[qy][qx] only from the taps with
// ky = a + 1 (mod 2), kx = b + 1 (mod 2), at qy = j + (a + 1 - ky) / 2, qx likewise.  The four pixels of a cell (j, i)
// form four parity classes with 1, 2, 2 and 4 taps: together they use each of the 9 taps once, on the 2 x 2
// neighbourhood dZ[j .. j+1][i .. i+1].  A stack's cells are cut into blocks of 32 (1 x 32, 2 x 16 or 4 x 8, whichever gives
// the fewest blocks; listed over image, row group, column group); a workgroup takes four consecutive blocks and 32 * MT
// input channels; each of its four multiplying wavefronts owns one block (32 cells = the N side of a 32x32x2 MFMA)
// and keeps one accumulator tile per class and channel block, so every MFMA multiplies deltas that exist.
// The reduction runs over the output channels in stages of 8: filter slice [tap][8][channels] and delta patch
// [block][8][(rows + 1) x (columns + 1) positions] travel HBM -> LDS with buffer_load ... lds, issued by a fifth wavefront one stage ahead (two LDS
// stages, one barrier a stage).  Positions outside the map (zero padding) or outside the stack's delta view (never
// needed by a valid pixel) are loaded from beyond the buffer's records and read as zero.
#include "ftp_device.h"
#include "ftp_launch.h"
#include <algorithm>

namespace ftp {

typedef float v16f_s2 __attribute__((ext_vector_type(16)));

struct DeltaS2Args {
    View din, dout, isign;
    RectTab rect;                                   // pixels of the delta each stack has to produce (input side)
    int ix0[kTabGrid], ix1[kTabGrid], iy0[kTabGrid], iy1[kTabGrid];   // extent of the delta view at the output side
    const float* wt;                                // [K * K - 1 - tap][C][Mtot]: the relaid filter of the backward pass
    int C, Mtot;                                    // reduction (output) channels, produced (input) channels
    int Hd, Wd;                                     // extent of the delta map at the output side
    int scale_out; float in_slope;
    int M, batch;
};

constexpr int kS2CK = 8;                            // reduction channels per stage
#define FTP_S2_LDS(p) ((__attribute__((address_space(3))) void*)(p))

template <typename T, int K, int MT, int NC>
__global__ void __launch_bounds__(320)
k_delta_s2_mfma(DeltaS2Args a)
{
    static_assert(K == 1 || K == 3, "1x1 and 3x3 filters");
    constexpr int BM = 32 * MT, ES = sizeof(T), NR = 32 / NC, KK = K * K, P = K / 2;
    constexpr int PW = NC + P, NPOS = (NR + P) * PW, XPASS = (NPOS + 63) / 64;     // (a 1x1 filter reads no neighbour: only the pixels (2j, 2i) receive a delta)
    constexpr int WF = KK * kS2CK * BM;                // dwords of a filter slice
    constexpr int XB = kS2CK * kS2XCS;                 // dwords of one block's patch
    constexpr int STAGE = WF + 4 * XB;
    constexpr unsigned OOB = 0x80000000u;
    static_assert(NPOS <= kS2XCS, "a block's patch fits its channel stride");
    __shared__ __attribute__((aligned(16))) float lds[2 * STAGE];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int hi = lane >> 5, l32 = lane & 31;
    const int stack = blockIdx.z, ti = stack / a.M, tj = stack % a.M;
    const int x0 = a.rect.x0[tj], x1 = a.rect.x1[tj], y0 = a.rect.y0[ti], y1 = a.rect.y1[ti];
    const S2Blocks sb = s2_blocks(x0, x1, y0, y1, a.batch, NC);
    if (4 * (int)blockIdx.x >= sb.total) return;
    const int m0 = blockIdx.y * BM;
    const int nst = (a.C + kS2CK - 1) / kS2CK;
    // block q of the stack -> image and first cell
    auto block_at = [&](int q, int& img, int& J0, int& I0) {
        img = q / (sb.gr * sb.gc);
        const int rem = q - img * (sb.gr * sb.gc), rg = rem / sb.gc;
        J0 = (y0 >> 1) + NR * rg; I0 = (x0 >> 1) + NC * (rem - rg * sb.gc);
    };

    if (wave == 4) {
        // ---- the loader ------------------------------------------------------------------------------------------
        const T* src = (const T*)a.din.p + (long long)stack * a.din.ss;
        const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc((void*)src, (short)0, 0x7FFFFFFF, 0x00020000);
        const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc((void*)a.wt, (short)0, 0x7FFFFFFF, 0x00020000);
        unsigned xvo[4][XPASS];
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const int q = 4 * blockIdx.x + w;
            int img, J0, I0;
            block_at(q < sb.total ? q : 0, img, J0, I0);
#pragma unroll
            for (int u = 0; u < XPASS; ++u) {
                const int p = lane + 64 * u;
                const int prow = p / PW, pcol = p - prow * PW;
                const int qy = J0 + prow, qx = I0 + pcol;
                const bool ok = q < sb.total && p < NPOS && qy >= 0 && qy < a.Hd && qx >= 0 && qx < a.Wd &&
                                qy >= a.iy0[ti] && qy <= a.iy1[ti] && qx >= a.ix0[tj] && qx <= a.ix1[tj];
                xvo[w][u] = ok ? (unsigned)ES * (unsigned)(img * (int)a.din.ns + (qy - a.din.y0[ti]) * a.din.pitch + (qx - a.din.x0[tj])) : OOB;
            }
        }
        constexpr int RPP = 256 / BM, WINSTR = (WF + 255) / 256;     // filter rows per load instruction; instructions per slice
        const int wrow = lane / (BM / 4), wcol = 4 * (lane % (BM / 4));
        auto issue = [&](int sg, float* buf) {
            const int c0 = sg * kS2CK;
#pragma unroll
            for (int idx = 0; idx < WINSTR; ++idx) {
                const int row = idx * RPP + wrow, tap = row / kS2CK, k = row - tap * kS2CK;
                if (row < KK * kS2CK) {                                              // (the last instruction of a slice may be half empty)
                    const bool ok = c0 + k < a.C && m0 + wcol < a.Mtot;
                    const unsigned vo = ok ? 4u * (unsigned)(((KK - 1 - tap) * a.C + c0 + k) * a.Mtot + m0 + wcol) : OOB;
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(wrsrc, FTP_S2_LDS(buf + idx * 256), 16, vo, 0u, 0, 0);
                }
            }
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                float* xs = buf + WF + w * XB;
#pragma unroll
                for (int u = 0; u < XPASS; ++u) {
                    if (lane + 64 * u < NPOS) {
#pragma unroll
                        for (int k = 0; k < kS2CK; ++k) {
                            const bool chok = c0 + k < a.C;                               // (uniform)
                            const unsigned so = (unsigned)ES * (unsigned)((c0 + k) * (int)a.din.cs);
                            if constexpr (sizeof(T) == 4) __builtin_amdgcn_raw_ptr_buffer_load_lds(xrsrc, FTP_S2_LDS(xs + k * kS2XCS + 64 * u), 4, chok ? xvo[w][u] : OOB, chok ? so : 0u, 0, 0);
                            else                          __builtin_amdgcn_raw_ptr_buffer_load_lds(xrsrc, FTP_S2_LDS(xs + k * kS2XCS + 64 * u), 2, chok ? xvo[w][u] : OOB, chok ? so : 0u, 0, 0);
                        }
                    }
                }
            }
        };
        issue(0, lds);
        for (int sg = 0; sg < nst; ++sg) {
            __builtin_amdgcn_s_waitcnt(0x0F70);        // vmcnt(0): stage sg has landed
            __syncthreads();                           // ... and the buffer of stage sg - 1 has been consumed
            if (sg + 1 < nst) issue(sg + 1, lds + ((sg + 1) & 1) * STAGE);
        }
        return;
    }

    // ---- the four multiplying wavefronts, one block of 32 cells each ----------------------------------------------------------
    v16f_s2 acc[4][MT];
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[c][mt][i] = 0.0f;
    const int cr = l32 / NC, cc = l32 - cr * NC;       // this lane's cell inside the block
    const int pb = wave * XB + cr * PW + cc + hi * kS2XCS;
    auto widen = [](float v) -> float { return ES == 4 ? v : __uint_as_float(__float_as_uint(v) << 16); };

    for (int sg = 0; sg < nst; ++sg) {
        __syncthreads();
        const float* Wl = lds + (sg & 1) * STAGE;
        const float* Xl = Wl + WF;
#pragma unroll
        for (int ky = 0; ky < K; ++ky)
#pragma unroll
            for (int kx = 0; kx < K; ++kx) {
                const int pa = (ky + P) & 1, pbx = (kx + P) & 1;                 // parity class of the pixels this tap reaches
                const int dj = (pa + P - ky) / 2, di = (pbx + P - kx) / 2;       // ... and where in the 2 x 2 neighbourhood
                const int cls = 2 * pa + pbx, tap = ky * K + kx;
#pragma unroll
                for (int i = 0; i < kS2CK / 2; ++i) {
                    const float bv = widen(Xl[2 * i * kS2XCS + pb + dj * PW + di]);
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        const float av = Wl[(tap * kS2CK + 2 * i + hi) * BM + 32 * mt + l32];
                        acc[cls][mt] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[cls][mt], 0, 0, 0);
                    }
                }
            }
    }

    // ---- store: accumulator row 8 * (i / 4) + 4 * hi + i % 4 = channel, column l32 = cell ----------------------------------
    // (the 32 channels of a block share one word of the sign map; their addresses differ by multiples of the channel stride)
    const int q = 4 * blockIdx.x + wave;
    if (q >= sb.total) return;
    int n, J0, I0;
    block_at(q, n, J0, I0);
    const int j = J0 + cr, ic = I0 + cc;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const int y = 2 * j + (c >> 1), x = 2 * ic + (c & 1);
        if (y < y0 || y > y1 || x < x0 || x > x1) continue;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int cb = m0 + 32 * mt;
            if (cb >= a.Mtot) continue;
            const uint32_t sw = a.scale_out ? *at<uint32_t>(a.isign, stack, ti, tj, n, cb >> 5, y, x) : 0u;
            T* const p = at<T>(a.dout, stack, ti, tj, n, cb + 4 * hi, y, x);
            const long long cs = a.dout.cs;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int r = 8 * (i >> 2) + (i & 3);
                if (cb + 4 * hi + r < a.Mtot) {
                    float v = acc[c][mt][i];
                    if (a.scale_out) v = scaled_delta<T>(v, (sw >> (4 * hi + r)) & 1u, a.in_slope);
                    st(p + r * cs, v);
                }
            }
        }
    }
}
#undef FTP_S2_LDS

// c.rect = backward rectangle at the input boundary; inrect = extent of the delta view per stack; wt = the backward
// pass's relaid filter.  Returns non-zero where the layer does not fit (the caller then takes the general kernel).
int delta_s2_mfma(const ConvArgs& c, const RectTab& inrect, const float* wt, hipStream_t s)
{
    if ((c.K != 3 && c.K != 1) || c.S != 2 || c.pooled || c.Cin % 4 != 0 || c.Cin < 16) return 1;
    const double es = c.bf16 ? 2.0 : 4.0;
    if (es * ((double)c.Cout * (double)c.din.cs + (double)c.batch * (double)c.din.ns) >= 2.0e9) return 1;   // 32-bit byte offsets inside one stack's maps
    if (4.0 * 9.0 * (double)c.Cout * (double)c.Cin >= 2.0e9) return 1;
    DeltaS2Args a;
    a.din = c.din; a.dout = c.dout; a.isign = c.isign; a.rect = c.rect;
    for (int t = 0; t < kTabGrid; ++t) { a.ix0[t] = inrect.x0[t]; a.ix1[t] = inrect.x1[t]; a.iy0[t] = inrect.y0[t]; a.iy1[t] = inrect.y1[t]; }
    a.wt = wt; a.C = c.Cout; a.Mtot = c.Cin; a.Hd = c.Hc; a.Wd = c.Wc;
    a.scale_out = c.scale_out; a.in_slope = c.in_slope; a.M = c.M; a.batch = c.batch;
    // block shape: the one that cuts the stacks' cell rectangles into the cheapest set of blocks of 32 cells
    int best_nc = 16; long long best_blocks = -1; int max_total = 1;
    for (int nc = 8; nc <= 32; nc *= 2) {
        long long blocks = 0; int mx = 1;
        for (int i = 0; i < c.N; ++i)
            for (int j = 0; j < c.M; ++j) {
                const S2Blocks b = s2_blocks(c.rect.x0[j], c.rect.x1[j], c.rect.y0[i], c.rect.y1[i], c.batch, nc);
                blocks += b.total; mx = std::max(mx, b.total);
            }
        blocks *= 160 + (32 / nc + c.K / 2) * (nc + c.K / 2);      // (a block costs its matrix work plus the loads of its patch: flat blocks have the larger halo)
        if (best_blocks < 0 || blocks < best_blocks) { best_blocks = blocks; best_nc = nc; max_total = mx; }
    }
    // 32 produced channels per workgroup: 64 (two accumulator tiles per class) need 151 registers and leave room for two
    // workgroups a CU instead of four - measured slower (gen_stem: 0.46 / 0.21 ms against 0.44 / 0.14 ms)
    const int mt = 1;
    dim3 grid((max_total + 3) / 4, (c.Cin + 32 * mt - 1) / (32 * mt), c.N * c.M);
    static const char* const labels[2][2][3] = {
        {{"k_delta_s2_mfma<float, 1, 1, 8>", "k_delta_s2_mfma<float, 1, 1, 16>", "k_delta_s2_mfma<float, 1, 1, 32>"},
         {"k_delta_s2_mfma<float, 3, 1, 8>", "k_delta_s2_mfma<float, 3, 1, 16>", "k_delta_s2_mfma<float, 3, 1, 32>"}},
        {{"k_delta_s2_mfma<unsigned short, 1, 1, 8>", "k_delta_s2_mfma<unsigned short, 1, 1, 16>", "k_delta_s2_mfma<unsigned short, 1, 1, 32>"},
         {"k_delta_s2_mfma<unsigned short, 3, 1, 8>", "k_delta_s2_mfma<unsigned short, 3, 1, 16>", "k_delta_s2_mfma<unsigned short, 3, 1, 32>"}}};
    g_kernel_label = labels[c.bf16 ? 1 : 0][c.K == 3 ? 1 : 0][best_nc == 8 ? 0 : best_nc == 16 ? 1 : 2];
#define FTP_S2L(T, MTv, NCv) do { if (c.K == 3) hipLaunchKernelGGL((k_delta_s2_mfma<T, 3, MTv, NCv>), grid, dim3(320), 0, s, a); \
                                   else          hipLaunchKernelGGL((k_delta_s2_mfma<T, 1, MTv, NCv>), grid, dim3(320), 0, s, a); } while (0)
#define FTP_S2N(T, MTv) do { if (best_nc == 8) FTP_S2L(T, MTv, 8); else if (best_nc == 16) FTP_S2L(T, MTv, 16); else FTP_S2L(T, MTv, 32); } while (0)
    if (c.bf16) FTP_S2N(bf16_t, 1); else FTP_S2N(float, 1);
#undef FTP_S2N
#undef FTP_S2L
    return 0;
}

}  // namespace ftp
