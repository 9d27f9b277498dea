// Direct (non-matrix-core) kernels of libftp for gfx950: the general path for every layer geometry
// (K = 1, 3, 5, 7; stride 1 or 2, Eq. (1)/(2) with any K_l, S_l; pools over odd maps), and the path of lone pools.
// One workgroup serves one (stack, image); stacks only read the rectangles the plan entitles them to.
#include "ftp_device.h"
#include "ftp_launch.h"
#include <algorithm>

namespace ftp {

__device__ __forceinline__ float4 operator+(float4 a, float4 b) { return make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w); }

// ---- delta at the convolution output ---------------------------------------------------------------
// The delta maps hold dLoss/dZ (the activation derivative is folded in by whoever writes them).  With a pool
// behind the convolution the delta sits at pooled resolution and reaches only the window's recorded winner
// (Sec. 4.1, back-propagation of the delta); the winner comes from the decision code the owning stack wrote
// in the forward pass.
// (Hp, Wp) = pooled extent: the last row / column of an odd convolution output lies in no window and has delta 0.
template <typename T, bool POOL>
__device__ __forceinline__ float delta_z(const View& din, const View& mask, int stack, int ti, int tj,
                                         int n, int co, int qy, int qx, int Hp, int Wp)
{
    if (!POOL) return ld(at<T>(din, stack, ti, tj, n, co, qy, qx));
    const int sy = qy >> 1, sx = qx >> 1;
    if (sy >= Hp || sx >= Wp) return 0.0f;
    const uint8_t m = *at<uint8_t>(mask, stack, ti, tj, n, co, sy, sx);
    if (((m >> 1) & 3) != (((qy & 1) << 1) | (qx & 1))) return 0.0f;
    return ld(at<T>(din, stack, ti, tj, n, co, sy, sx));
}

__device__ __forceinline__ bool in_rect(const RectTab& r, int ti, int tj, int y, int x)
{
    return y >= r.y0[ti] && y <= r.y1[ti] && x >= r.x0[tj] && x <= r.x1[tj];
}

// ---- forward: convolution + leaky ReLU (+ 2x2 max-pool) ------------------------------------------------
// (Hi, Wi) = extent of the input map; output position o of a stride-S convolution reads inputs o*S - P + k.
template <typename T, int K, int S, bool POOL, int COB>
__global__ void __launch_bounds__(64)
k_conv_fwd_direct(View in, View out, View mask, View osign, RectTab rt, RectTab own, const T* __restrict__ w,
                  const T* __restrict__ bias, int Cin, int Cout, int Hi, int Wi, float slope, int M, int batch)
{
    static_assert(COB == 8, "a workgroup's channels fill one byte of the sign word");
    const int stack = blockIdx.z / batch, n = blockIdx.z % batch;
    const int ti = stack / M, tj = stack % M;
    const int rw = rt.x1[tj] - rt.x0[tj] + 1, rh = rt.y1[ti] - rt.y0[ti] + 1;
    const int pid = blockIdx.x * blockDim.x + threadIdx.x;
    if (pid >= rw * rh) return;
    const int oy = rt.y0[ti] + pid / rw, ox = rt.x0[tj] + pid % rw;
    const int co0 = blockIdx.y * COB;
    constexpr int NP = POOL ? 2 : 1, P = K / 2, R = (NP - 1) * S + K;
    float acc[COB][NP * NP];
#pragma unroll
    for (int j = 0; j < COB; ++j)
#pragma unroll
        for (int d = 0; d < NP * NP; ++d) acc[j][d] = 0.0f;
    const int by = oy * NP * S - P, bx = ox * NP * S - P;
    for (int ci = 0; ci < Cin; ++ci) {
        float patch[R * R];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int c = 0; c < R; ++c) {
                const int y = by + r, x = bx + c;
                patch[r * R + c] = (y >= 0 && y < Hi && x >= 0 && x < Wi) ? ld(at<T>(in, stack, ti, tj, n, ci, y, x)) : 0.0f;
            }
#pragma unroll
        for (int j = 0; j < COB; ++j) {
            const int co = co0 + j;
            if (co >= Cout) break;
            const T* wp = w + ((size_t)co * Cin + ci) * K * K;
#pragma unroll
            for (int ky = 0; ky < K; ++ky)
#pragma unroll
                for (int kx = 0; kx < K; ++kx) {
                    const float wv = ld(wp + ky * K + kx);
#pragma unroll
                    for (int dy = 0; dy < NP; ++dy)
#pragma unroll
                        for (int dx = 0; dx < NP; ++dx)
                            acc[j][dy * NP + dx] = fmaf(wv, patch[(dy * S + ky) * R + dx * S + kx], acc[j][dy * NP + dx]);
                }
        }
    }
    const bool owned = in_rect(own, ti, tj, oy, ox);
    uint32_t signs = 0;
#pragma unroll
    for (int j = 0; j < COB; ++j) {
        const int co = co0 + j;
        if (co >= Cout) break;
        const float b = bias ? ld(bias + co) : 0.0f;
        // the pool compares activations as the map would hold them (rounded to the storage type), so the
        // winner does not depend on whether the pool is evaluated here or as a layer of its own
        float best = stored(leaky(acc[j][0] + b, slope), (const T*)nullptr);
        int bi = 0;
        if (POOL) {
#pragma unroll
            for (int d = 1; d < NP * NP; ++d) {
                const float v = stored(leaky(acc[j][d] + b, slope), (const T*)nullptr);
                if (v > best) { best = v; bi = d; }        // first maximum in window order wins
            }
        }
        st(at<T>(out, stack, ti, tj, n, co, oy, ox), best);
        if (POOL && owned) *at<uint8_t>(mask, stack, ti, tj, n, co, oy, ox) = (uint8_t)((bi << 1) | (best > 0.0f ? 1 : 0));
        signs |= (best > 0.0f ? 1u : 0u) << j;
    }
    // these 8 channels are byte (co0 / 8) % 4 of their sign word
    if (owned) ((uint8_t*)at<uint32_t>(osign, stack, ti, tj, n, co0 >> 5, oy, ox))[(co0 >> 3) & 3] = (uint8_t)signs;
}

// ---- backward: delta at the convolution input -------------------------------------------------------
// (Hc, Wc) = extent of the convolution output; input position i receives W[k] dZ[q] from every (q, k) with
// q*S - P + k == i (for stride 2 only the taps of matching parity contribute).
template <typename T, int K, int S, bool POOL, int CIB>
__global__ void __launch_bounds__(64)
k_conv_bwd_data_direct(View din, View mask, View dout, View isign, int scale_out, float in_slope, RectTab rt,
                       const T* __restrict__ w, int Cin, int Cout, int Hc, int Wc, int M, int batch, int blocks_per_class)
{
    const int stack = blockIdx.z / batch, n = blockIdx.z % batch;
    const int ti = stack / M, tj = stack % M;
    const int rw = rt.x1[tj] - rt.x0[tj] + 1, rh = rt.y1[ti] - rt.y0[ti] + 1;
    int ry, rx, cls = 0;
    if (S == 2) {
        // a workgroup serves one of the four parity classes of the rectangle: its taps, and with them the filter
        // elements it reads, are the same for all its lanes (scalar loads)
        cls = blockIdx.x / blocks_per_class;
        const int idx = (blockIdx.x - cls * blocks_per_class) * blockDim.x + threadIdx.x;
        const int rw2 = (rw + 1) >> 1, rh2 = (rh + 1) >> 1;
        ry = 2 * (idx / rw2) + (cls >> 1); rx = 2 * (idx % rw2) + (cls & 1);
        if (idx >= rw2 * rh2 || ry >= rh || rx >= rw) return;
    } else {
        const int pid = blockIdx.x * blockDim.x + threadIdx.x;
        if (pid >= rw * rh) return;
        ry = pid / rw; rx = pid - ry * rw;
    }
    const int iy = rt.y0[ti] + ry, ix = rt.x0[tj] + rx;
    const int ci0 = blockIdx.y * CIB;
    constexpr int P = K / 2;
    float acc[CIB];
#pragma unroll
    for (int j = 0; j < CIB; ++j) acc[j] = 0.0f;
    // stride 2: only the taps with ky = (iy + P) mod 2, + 2, ... (and likewise kx) meet an output position
    constexpr int NTAP = (K + S - 1) / S;
    const int ky0 = S == 2 ? ((rt.y0[ti] + (cls >> 1) + P) & 1) : 0, kx0 = S == 2 ? ((rt.x0[tj] + (cls & 1) + P) & 1) : 0;
    if constexpr (!POOL) {
        // where each tap's delta sits inside a channel plane of the delta view is the same for every output channel:
        // element offsets once (-1: outside the map), then one load and CIB multiply-adds per (co, tap)
        int off[NTAP * NTAP];
#pragma unroll
        for (int my = 0; my < NTAP; ++my)
#pragma unroll
            for (int mx = 0; mx < NTAP; ++mx) {
                const int ky = ky0 + S * my, kx = kx0 + S * mx;
                const int sy = iy + P - ky, sx = ix + P - kx;
                const int qy = sy / S, qx = sx / S;
                const bool ok = ky < K && kx < K && sy >= 0 && sx >= 0 && qy < Hc && qx < Wc;
                off[my * NTAP + mx] = ok ? (qy - din.y0[ti]) * din.pitch + (qx - din.x0[tj]) : -1;
            }
        const T* dp = at<T>(din, stack, ti, tj, n, 0, din.y0[ti], din.x0[tj]);
        for (int co = 0; co < Cout; ++co, dp += din.cs) {
#pragma unroll
            for (int my = 0; my < NTAP; ++my)
#pragma unroll
                for (int mx = 0; mx < NTAP; ++mx) {
                    const int ky = ky0 + S * my, kx = kx0 + S * mx;
                    if (ky >= K || kx >= K) continue;                   // (the same for every lane of a strided workgroup)
                    const int o = off[my * NTAP + mx];
                    const float dz = o >= 0 ? ld(dp + o) : 0.0f;
#pragma unroll
                    for (int j = 0; j < CIB; ++j) {
                        const int ci = ci0 + j;
                        if (ci < Cin) acc[j] = fmaf(ld(w + (((size_t)co * Cin + ci) * K + ky) * K + kx), dz, acc[j]);
                    }
                }
        }
    } else {
    for (int co = 0; co < Cout; ++co) {
#pragma unroll
        for (int my = 0; my < NTAP; ++my)
#pragma unroll
            for (int mx = 0; mx < NTAP; ++mx) {
                const int ky = ky0 + S * my, kx = kx0 + S * mx;
                if (ky >= K || kx >= K) continue;
                const int sy = iy + P - ky, sx = ix + P - kx;
                if (sy < 0 || sx < 0) continue;
                const int qy = sy / S, qx = sx / S;
                if (qy >= Hc || qx >= Wc) continue;
                const float dz = delta_z<T, POOL>(din, mask, stack, ti, tj, n, co, qy, qx, Hc >> 1, Wc >> 1);
#pragma unroll
                for (int j = 0; j < CIB; ++j) {
                    const int ci = ci0 + j;
                    if (ci < Cin) acc[j] = fmaf(ld(w + (((size_t)co * Cin + ci) * K + ky) * K + kx), dz, acc[j]);
                }
            }
    }
    }
#pragma unroll
    for (int j = 0; j < CIB; ++j)
        if (ci0 + j < Cin) {
            float v = acc[j];
            if (scale_out) v = scaled_delta<T>(v, sign_bit(isign, stack, ti, tj, n, ci0 + j, iy, ix), in_slope);
            st(at<T>(dout, stack, ti, tj, n, ci0 + j, iy, ix), v);
        }
}

// ---- backward: per-stack partial filter gradient -----------------------------------------------------
// One workgroup per (ci, co, stack) sums dZ * X over the batch and the stack's owned output pixels.
// Lanes are combined with wavefront shuffles, waves through LDS in a fixed order: deterministic.
template <typename T, int K, int S, bool POOL>
__global__ void __launch_bounds__(256)
k_wgrad_direct(View xin, View din, View mask, RectTab own, float* __restrict__ partial, long long n_params,
               long long w_off, long long b_off, int has_bias, int Cin, int Cout, int Hi, int Wi, int Hc, int Wc, int M, int batch)
{
    const int ci = blockIdx.x, co = blockIdx.y, stack = blockIdx.z;
    const int ti = stack / M, tj = stack % M;
    const int rw = own.x1[tj] - own.x0[tj] + 1, rh = own.y1[ti] - own.y0[ti] + 1;
    const int px = rw * rh, items = px * batch;
    constexpr int P = K / 2, KK = K * K;
    float acc[KK + 1];
#pragma unroll
    for (int t = 0; t <= KK; ++t) acc[t] = 0.0f;
    for (int it = threadIdx.x; it < items; it += 256) {
        const int n = it / px, r = it - n * px;
        const int qy = own.y0[ti] + r / rw, qx = own.x0[tj] + r % rw;
        const float dz = delta_z<T, POOL>(din, mask, stack, ti, tj, n, co, qy, qx, Hc >> 1, Wc >> 1);
        acc[KK] += dz;
#pragma unroll
        for (int ky = 0; ky < K; ++ky)
#pragma unroll
            for (int kx = 0; kx < K; ++kx) {
                const int y = qy * S - P + ky, x = qx * S - P + kx;
                if (y >= 0 && y < Hi && x >= 0 && x < Wi)
                    acc[ky * K + kx] = fmaf(dz, ld(at<T>(xin, stack, ti, tj, n, ci, y, x)), acc[ky * K + kx]);
            }
    }
    __shared__ float red[4][KK + 1];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int t = 0; t <= KK; ++t) {
        float v = acc[t];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
        if (lane == 0) red[wave][t] = v;
    }
    __syncthreads();
    if (threadIdx.x <= KK) {
        const int t = threadIdx.x;
        const float v = (red[0][t] + red[1][t]) + (red[2][t] + red[3][t]);
        float* base = partial + (long long)stack * n_params;
        if (t < KK) base[w_off + ((long long)co * Cin + ci) * KK + t] = v;
        else if (has_bias && ci == 0) base[b_off + co] = v;
    }
}

// ---- lone 2x2 max-pool ---------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(64)
k_pool_fwd(View in, View out, View mask, RectTab rt, RectTab own, int C, int M, int batch)
{
    const int stack = blockIdx.z / batch, n = blockIdx.z % batch;
    const int ti = stack / M, tj = stack % M;
    const int rw = rt.x1[tj] - rt.x0[tj] + 1, rh = rt.y1[ti] - rt.y0[ti] + 1;
    const int pid = blockIdx.x * blockDim.x + threadIdx.x;
    if (pid >= rw * rh) return;
    const int oy = rt.y0[ti] + pid / rw, ox = rt.x0[tj] + pid % rw;
    const int c = blockIdx.y;
    float best = ld(at<T>(in, stack, ti, tj, n, c, 2 * oy, 2 * ox));
    int bi = 0;
#pragma unroll
    for (int d = 1; d < 4; ++d) {
        const float v = ld(at<T>(in, stack, ti, tj, n, c, 2 * oy + (d >> 1), 2 * ox + (d & 1)));
        if (v > best) { best = v; bi = d; }
    }
    st(at<T>(out, stack, ti, tj, n, c, oy, ox), best);
    if (in_rect(own, ti, tj, oy, ox)) *at<uint8_t>(mask, stack, ti, tj, n, c, oy, ox) = (uint8_t)((bi << 1) | (best > 0.0f ? 1 : 0));
}

// One pool window (2 x 2 input pixels) per thread: the winner code and the pooled delta are loaded once (and
// independently of each other), the four results are written row by row, two pixels at a time where both lie in the
// rectangle and the pair sits on an aligned address.  Windows that only touch the rectangle's border, and the last row
// / column of an odd map (which lies in no window and gets 0), are handled element by element.
template <typename T>
__global__ void __launch_bounds__(256)
k_pool_bwd(View din, View mask, View dout, View isign, int scale_out, float in_slope, RectTab rt, int C, int Ho, int Wo, int M, int batch)
{
    const int stack = blockIdx.z / batch, n = blockIdx.z % batch;
    const int ti = stack / M, tj = stack % M;
    const int x0 = rt.x0[tj], x1 = rt.x1[tj], y0 = rt.y0[ti], y1 = rt.y1[ti];
    const int wx0 = x0 >> 1, wy0 = y0 >> 1, ww = (x1 >> 1) - wx0 + 1, wh = (y1 >> 1) - wy0 + 1;
    const int pid = blockIdx.x * blockDim.x + threadIdx.x;
    if (pid >= ww * wh) return;
    const int wy = wy0 + pid / ww, wx = wx0 + pid % ww;
    const int c = blockIdx.y;
    const bool has = wy < Ho && wx < Wo;
    // the loads are unconditional: a window of the dropped row / column reads the rectangle's first window instead,
    // which (like every window the rectangle touches) lies inside the stack's delta rectangle at the pooled boundary
    const int sy = has ? wy : wy0, sx = has ? wx : wx0;
    const uint8_t code = *at<uint8_t>(mask, stack, ti, tj, n, c, sy, sx);
    const float gd = ld(at<T>(din, stack, ti, tj, n, c, sy, sx));
    const int win = has ? ((code >> 1) & 3) : -1;
#pragma unroll
    for (int dy = 0; dy < 2; ++dy) {
        const int iy = 2 * wy + dy;
        if (iy < y0 || iy > y1) continue;
        float g[2]; bool ok[2];
#pragma unroll
        for (int dx = 0; dx < 2; ++dx) {
            const int ix = 2 * wx + dx;
            ok[dx] = ix >= x0 && ix <= x1;
            g[dx] = win == 2 * dy + dx ? gd : 0.0f;
            if (scale_out && ok[dx]) g[dx] = scaled_delta<T>(g[dx], sign_bit(isign, stack, ti, tj, n, c, iy, ix), in_slope);
        }
        T* p = at<T>(dout, stack, ti, tj, n, c, iy, 2 * wx);
        if (ok[0] && ok[1] && ((uintptr_t)p & (2 * sizeof(T) - 1)) == 0) {
            if constexpr (sizeof(T) == 4) *(float2*)p = make_float2(g[0], g[1]);
            else *(uint32_t*)p = bf16_bits(g[0]) | (bf16_bits(g[1]) << 16);
        } else {
            if (ok[0]) st(p, g[0]);
            if (ok[1]) st(p + 1, g[1]);
        }
    }
}

// ---- sum of the per-stack partial gradients ------------------------------------------------------------
// Balanced pairwise order over the stack index (pairs (2k, 2k+1) at each level, an odd tail is carried
// up), evaluated with a binary-counter stack so that one pass over the partials suffices.
// Balanced pairwise sum of up to 8 items, n of them present: pairs (2k, 2k+1) at each level, an item without a
// partner is carried up unchanged.  All indices are compile-time, so everything stays in registers.
template <typename V>
__device__ __forceinline__ V tree8(const V (&b)[8], int n)
{
    V p[4], q[2];
#pragma unroll
    for (int j = 0; j < 4; ++j) p[j] = 2 * j + 1 < n ? b[2 * j] + b[2 * j + 1] : b[2 * j];
    const int n1 = (n + 1) >> 1;
#pragma unroll
    for (int j = 0; j < 2; ++j) q[j] = 2 * j + 1 < n1 ? p[2 * j] + p[2 * j + 1] : p[2 * j];
    const int n2 = (n1 + 1) >> 1;
    return n2 > 1 ? q[0] + q[1] : q[0];
}

// The balanced pairwise tree over up to 512 stacks, evaluated as nested 8-way trees (the tree over the whole list
// restricted to an aligned group of 8 is the 8-way tree of that group).  The 8 loads of a group are in flight together.
template <typename V>
__device__ __forceinline__ V pairwise_stack_sum(const V* __restrict__ partial, long long stride, int stacks)
{
    V top[8];
    const int n_top = (stacks + 63) >> 6;
    for (int a = 0; a < 8; ++a) {
        if (a >= n_top) break;
        V mid[8];
        const int left_a = stacks - 64 * a, n_mid = left_a >= 64 ? 8 : (left_a + 7) >> 3;
#pragma unroll
        for (int m = 0; m < 8; ++m) {
            if (m < n_mid) {
                V buf[8];
                const int s0 = 64 * a + 8 * m, n = stacks - s0 >= 8 ? 8 : stacks - s0;
#pragma unroll
                for (int u = 0; u < 8; ++u) buf[u] = partial[(long long)(s0 + (u < n ? u : 0)) * stride];
                mid[m] = tree8(buf, n);
            } else {
                mid[m] = mid[0];
            }
        }
        const V v = tree8(mid, n_mid);
#pragma unroll
        for (int t = 0; t < 8; ++t) if (t == a) top[t] = v;
    }
#pragma unroll
    for (int t = 1; t < 8; ++t) if (t >= n_top) top[t] = top[0];
    return tree8(top, n_top);
}

// 4 parameters per thread where the vector is long and aligned enough, one per thread for the rest.
__global__ void __launch_bounds__(256)
k_reduce_wgrad(const float* __restrict__ partial, float* __restrict__ wgrad, long long n_params, int stacks)
{
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long n4 = (n_params % 4 == 0) ? n_params / 4 : 0;        // rows of the partials stay 16-byte aligned
    if (i < n4) {
        ((float4*)wgrad)[i] = pairwise_stack_sum((const float4*)partial + i, n_params / 4, stacks);
    } else {
        const long long p = 4 * n4 + (i - n4);
        if (p < n_params) wgrad[p] = pairwise_stack_sum(partial + p, n_params, stacks);
    }
}

// The same sum fused with the gradient-descent step on one parameter tensor (Sec. 4.1, filter update).
template <typename T>
__global__ void __launch_bounds__(256)
k_sgd_update(const float* __restrict__ partial, long long n_params, int stacks, T* __restrict__ w, long long count, float lr,
             float* __restrict__ wgrad)
{
    const long long p = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= count) return;
    const float g = pairwise_stack_sum(partial + p, n_params, stacks);
    if (wgrad) wgrad[p] = g;
    st(w + p, ld(w + p) - lr * g);
}

// ---- launchers ---------------------------------------------------------------------------------------------
namespace {

inline int rect_max_px(const RectTab& rt, int N, int M)
{
    int mw = 0, mh = 0;
    for (int t = 0; t < M; ++t) mw = mw > rt.x1[t] - rt.x0[t] + 1 ? mw : rt.x1[t] - rt.x0[t] + 1;
    for (int t = 0; t < N; ++t) mh = mh > rt.y1[t] - rt.y0[t] + 1 ? mh : rt.y1[t] - rt.y0[t] + 1;
    return mw * mh;
}

// Picks the instantiation for (K, stride, pooled); the planner admits K in {1, 3, 5, 7} and stride in {1, 2} only,
// and fuses a pool into the convolution in front of it only for stride 1 and K <= 3.
#define FTP_GEOMETRY_S(LAUNCH, KK) \
    do { if (a.pooled) { if constexpr ((KK) <= 3) LAUNCH(KK, 1, true); } \
         else if (a.S == 2) LAUNCH(KK, 2, false); else LAUNCH(KK, 1, false); } while (0)
#define FTP_GEOMETRY(LAUNCH) \
    do { switch (a.K) { case 1: FTP_GEOMETRY_S(LAUNCH, 1); break; case 3: FTP_GEOMETRY_S(LAUNCH, 3); break; \
                        case 5: FTP_GEOMETRY_S(LAUNCH, 5); break; default: FTP_GEOMETRY_S(LAUNCH, 7); break; } } while (0)

template <typename T>
void conv_fwd_t(const ConvArgs& a, hipStream_t s)
{
    constexpr int COB = 8;
    dim3 grid((rect_max_px(a.rect, a.N, a.M) + 63) / 64, (a.Cout + COB - 1) / COB, a.N * a.M * a.batch), block(64);
    const T* w = (const T*)a.w; const T* b = (const T*)a.bias;
#define FTP_FWD(KK, SS, PL) hipLaunchKernelGGL((k_conv_fwd_direct<T, KK, SS, PL, COB>), grid, block, 0, s, a.in, a.out, a.mask, a.osign, a.rect, a.own, w, b, a.Cin, a.Cout, a.Hi, a.Wi, a.slope, a.M, a.batch)
    FTP_GEOMETRY(FTP_FWD);
#undef FTP_FWD
}

template <typename T>
void conv_bwd_data_t(const ConvArgs& a, hipStream_t s)
{
    constexpr int CIB = 8;
    int mw = 0, mh = 0;
    for (int t = 0; t < a.M; ++t) mw = std::max(mw, a.rect.x1[t] - a.rect.x0[t] + 1);
    for (int t = 0; t < a.N; ++t) mh = std::max(mh, a.rect.y1[t] - a.rect.y0[t] + 1);
    const int bpc = (((mw + 1) / 2) * ((mh + 1) / 2) + 63) / 64;                       // stride 2: workgroups per parity class
    dim3 grid(a.S == 2 ? 4 * bpc : (mw * mh + 63) / 64, (a.Cin + CIB - 1) / CIB, a.N * a.M * a.batch), block(64);
    const T* w = (const T*)a.w;
#define FTP_BWD(KK, SS, PL) hipLaunchKernelGGL((k_conv_bwd_data_direct<T, KK, SS, PL, CIB>), grid, block, 0, s, a.din, a.mask, a.dout, a.isign, a.scale_out, a.in_slope, a.rect, w, a.Cin, a.Cout, a.Hc, a.Wc, a.M, a.batch, bpc)
    FTP_GEOMETRY(FTP_BWD);
#undef FTP_BWD
}

template <typename T>
void wgrad_t(const ConvArgs& a, hipStream_t s)
{
    dim3 grid(a.Cin, a.Cout, a.N * a.M), block(256);
#define FTP_WG(KK, SS, PL) hipLaunchKernelGGL((k_wgrad_direct<T, KK, SS, PL>), grid, block, 0, s, a.in, a.din, a.mask, a.rect, a.partial, a.n_params, a.w_off, a.b_off, a.has_bias, a.Cin, a.Cout, a.Hi, a.Wi, a.Hc, a.Wc, a.M, a.batch)
    FTP_GEOMETRY(FTP_WG);
#undef FTP_WG
}

}  // namespace

void direct_conv_fwd(const ConvArgs& a, hipStream_t s) { g_kernel_label = "k_conv_fwd_direct"; if (a.bf16) conv_fwd_t<bf16_t>(a, s); else conv_fwd_t<float>(a, s); }
void direct_conv_bwd_data(const ConvArgs& a, hipStream_t s) { g_kernel_label = "k_conv_bwd_data_direct"; if (a.bf16) conv_bwd_data_t<bf16_t>(a, s); else conv_bwd_data_t<float>(a, s); }
void direct_wgrad(const ConvArgs& a, hipStream_t s) { g_kernel_label = "k_wgrad_direct"; if (a.bf16) wgrad_t<bf16_t>(a, s); else wgrad_t<float>(a, s); }

void pool_fwd(const PoolArgs& a, hipStream_t s)
{
    g_kernel_label = "k_pool_fwd";
    dim3 grid((rect_max_px(a.rect, a.N, a.M) + 63) / 64, a.C, a.N * a.M * a.batch), block(64);
    if (a.bf16) hipLaunchKernelGGL(k_pool_fwd<bf16_t>, grid, block, 0, s, a.in, a.out, a.mask, a.rect, a.own, a.C, a.M, a.batch);
    else        hipLaunchKernelGGL(k_pool_fwd<float>, grid, block, 0, s, a.in, a.out, a.mask, a.rect, a.own, a.C, a.M, a.batch);
}

void pool_bwd(const PoolArgs& a, hipStream_t s)
{
    g_kernel_label = "k_pool_bwd";
    int mw = 0, mh = 0;                                // windows touched by the largest rectangle
    for (int t = 0; t < a.M; ++t) mw = std::max(mw, (a.rect.x1[t] >> 1) - (a.rect.x0[t] >> 1) + 1);
    for (int t = 0; t < a.N; ++t) mh = std::max(mh, (a.rect.y1[t] >> 1) - (a.rect.y0[t] >> 1) + 1);
    const int bs = mw * mh <= 64 ? 64 : mw * mh <= 128 ? 128 : 256;          // small rectangles: no idle wavefronts
    dim3 grid((mw * mh + bs - 1) / bs, a.C, a.N * a.M * a.batch), block(bs);
    if (a.bf16) hipLaunchKernelGGL(k_pool_bwd<bf16_t>, grid, block, 0, s, a.din, a.mask, a.dout, a.isign, a.scale_out, a.in_slope, a.rect, a.C, a.Ho, a.Wo, a.M, a.batch);
    else        hipLaunchKernelGGL(k_pool_bwd<float>, grid, block, 0, s, a.din, a.mask, a.dout, a.isign, a.scale_out, a.in_slope, a.rect, a.C, a.Ho, a.Wo, a.M, a.batch);
}

// 4 consecutive elements of one (image, channel) plane per thread (HW is a multiple of 4: the rows of a plane and of
// the sign words then stay 16-byte aligned), else one element per thread.
template <typename T, int V>
__global__ void __launch_bounds__(256)
k_scale_dy(const T* __restrict__ dy, const uint32_t* __restrict__ sign, T* __restrict__ dst, int C, long long HW, long long total, float slope)
{
    const long long e = ((long long)blockIdx.x * blockDim.x + threadIdx.x) * V;
    if (e >= total) return;
    const long long plane = e / HW, off = e - plane * HW;
    const int c = (int)(plane % C), G = (C + 31) / 32;
    const long long n = plane / C;
    const uint32_t* sg = sign + (n * G + (c >> 5)) * HW + off;
    if (V == 4 && sizeof(T) == 4) {
        const float4 v = *(const float4*)(dy + e);
        const uint4 w = *(const uint4*)sg;
        float4 r;
        r.x = scaled_delta<T>(v.x, (w.x >> (c & 31)) & 1u, slope);
        r.y = scaled_delta<T>(v.y, (w.y >> (c & 31)) & 1u, slope);
        r.z = scaled_delta<T>(v.z, (w.z >> (c & 31)) & 1u, slope);
        r.w = scaled_delta<T>(v.w, (w.w >> (c & 31)) & 1u, slope);
        *(float4*)(dst + e) = r;
    } else {
#pragma unroll
        for (int u = 0; u < V; ++u) st(dst + e + u, scaled_delta<T>(ld(dy + e + u), (sg[u] >> (c & 31)) & 1u, slope));
    }
}

void scale_dy(const void* dy, const uint32_t* sign, void* dst, int batch, int C, long long HW, float slope, int bf16, hipStream_t s)
{
    g_kernel_label = "k_scale_dy";
    const long long total = (long long)batch * C * HW;
    const int V = HW % 4 == 0 ? 4 : 1;
    dim3 grid((unsigned)((total / V + 255) / 256)), block(256);
    if (bf16) {
        if (V == 4) hipLaunchKernelGGL((k_scale_dy<bf16_t, 4>), grid, block, 0, s, (const bf16_t*)dy, sign, (bf16_t*)dst, C, HW, total, slope);
        else        hipLaunchKernelGGL((k_scale_dy<bf16_t, 1>), grid, block, 0, s, (const bf16_t*)dy, sign, (bf16_t*)dst, C, HW, total, slope);
    } else {
        if (V == 4) hipLaunchKernelGGL((k_scale_dy<float, 4>), grid, block, 0, s, (const float*)dy, sign, (float*)dst, C, HW, total, slope);
        else        hipLaunchKernelGGL((k_scale_dy<float, 1>), grid, block, 0, s, (const float*)dy, sign, (float*)dst, C, HW, total, slope);
    }
}

void sgd_update(const float* partial, long long n_params, int stacks, void* w, long long count, float lr, float* wgrad,
                int bf16, hipStream_t s)
{
    g_kernel_label = "k_sgd_update";
    dim3 grid((unsigned)((count + 255) / 256)), block(256);
    if (bf16) hipLaunchKernelGGL(k_sgd_update<bf16_t>, grid, block, 0, s, partial, n_params, stacks, (bf16_t*)w, count, lr, wgrad);
    else      hipLaunchKernelGGL(k_sgd_update<float>, grid, block, 0, s, partial, n_params, stacks, (float*)w, count, lr, wgrad);
}

void reduce_wgrad(const float* partial, float* wgrad, long long n_params, int stacks, hipStream_t s)
{
    g_kernel_label = "k_reduce_wgrad";
    const long long threads = n_params % 4 == 0 ? n_params / 4 : n_params;
    dim3 grid((unsigned)((threads + 255) / 256)), block(256);
    hipLaunchKernelGGL(k_reduce_wgrad, grid, block, 0, s, partial, wgrad, n_params, stacks);
}

}  // namespace ftp
