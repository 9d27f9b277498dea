// fp32 matrix-core (MFMA) implicit-GEMM convolution for gfx950, used for the forward pass and for the
// delta back-propagation (which is the same convolution with the 180-degree rotated, transposed
// filter applied to dZ).  D[m][pixel] = sum_k Wt[k][m] * patch[k][pixel], k = (tap, channel).
//
// One workgroup (4 wavefronts) produces BM = 32/64/128 output channels for a tile of up to 128 or 256 pixels of
// one stack (pooled layers: 32 or 64 windows of 4 pixels).  A tile is a run of consecutive rows of the
// stack's rectangle, counted through the batch (row index R = image * rows + row), times a block of
// columns, so that small rectangles of several images fill one tile and medium ones leave no ragged
// last tile per image.  The input patch (tile rows + filter halo per image, zero outside the real map)
// and the filter slice of a few channels x K*K taps sit in LDS; v_mfma_f32_32x32x2_f32 reads both from there.
// MFMA lane layout (64 lanes): A[m = lane%32][k = lane/32], B[k = lane/32][n = lane%32],
// D[m = 8*(i/4) + 4*(lane/32) + i%4][n = lane%32] for accumulator register i of 16.
// With 16-bit (bfloat) maps and filters the stride-1 1x1 / 3x3 layers multiply with v_mfma_f32_32x32x16_bf16
// instead (A[m][k = 8*(lane/32) + j], B[k = 8*(lane/32) + j][n], j < 8, same D): products of two bfloats are exact in
// fp32 and the sums are accumulated in fp32, so this is the same arithmetic at sixteen times the rate (the older
// 32x32x8 form runs at half of that on this chip).
#include "ftp_device.h"
#include "ftp_launch.h"
#include "ftp_conv_tiles.h"
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>

namespace ftp {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));


// Filter relayout: OIHW -> [tap][reduction channel][output channel], so that a stage's slice is a set of
// contiguous rows.  fwd: Wt[t][ci][co] = W[co][ci][t].  bwd: Wt[t][co][ci] = W[co][ci][K*K-1-t] (rotated).
template <typename T>
__global__ void __launch_bounds__(256)
k_prep_filter(const T* __restrict__ w, float* __restrict__ wt_fwd, float* __restrict__ wt_bwd, int Cout, int Cin, int KK)
{
    const long long n = (long long)Cout * Cin * KK;
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int t = (int)(i % KK);
    const int ci = (int)((i / KK) % Cin);
    const int co = (int)(i / ((long long)KK * Cin));
    const float v = ld(w + i);
    if (wt_fwd) wt_fwd[((long long)t * Cin + ci) * Cout + co] = v;
    if (wt_bwd) wt_bwd[((long long)(KK - 1 - t) * Cout + co) * Cin + ci] = v;
}

// Filter relayout for the bfloat matrix-core path: [tap][group of 8 reduction channels][output channel][8 bfloats],
// taps padded to an even count with zeros (one instruction multiplies 8 channels of two taps, or 16 channels of
// one), reduction channels padded to whole groups with zeros.  fwd: reduction = ci, output = co; bwd: reduction = co,
// output = ci, taps rotated by 180 degrees.
__global__ void __launch_bounds__(256)
k_prep_filter16(const bf16_t* __restrict__ w, bf16_t* __restrict__ wt_fwd, bf16_t* __restrict__ wt_bwd, int Cout, int Cin, int KK, int taps)
{
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const int j = (int)(i & 7);
    if (wt_fwd) {
        const int C8 = (Cin + 7) / 8;
        const long long n = (long long)taps * C8 * Cout;
        if ((i >> 3) < n) {
            const long long e = i >> 3;
            const int co = (int)(e % Cout), q = (int)((e / Cout) % C8), t = (int)(e / ((long long)Cout * C8));
            const int ci = 8 * q + j;
            wt_fwd[i] = (t < KK && ci < Cin) ? w[((long long)co * Cin + ci) * KK + t] : (bf16_t)0;
        }
    }
    if (wt_bwd) {
        const int C8 = (Cout + 7) / 8;
        const long long n = (long long)taps * C8 * Cin;
        if ((i >> 3) < n) {
            const long long e = i >> 3;
            const int ci = (int)(e % Cin), q = (int)((e / Cin) % C8), t = (int)(e / ((long long)Cin * C8));
            const int co = 8 * q + j;
            wt_bwd[i] = (t < KK && co < Cout) ? w[((long long)co * Cin + ci) * KK + (KK - 1 - t)] : (bf16_t)0;
        }
    }
}

// (tile geometry: ftp_conv_tiles.h)
template <int S, int P, int Q>
__device__ __forceinline__ TileGeom tile_geom(const MfmaConvArgs& a, int x0, int x1, int y0, int y1, int bx)
{
    return conv_tile_geom(a.tiles_x, a.TC, a.cap, a.flat, a.batch, x0, x1, y0, y1, bx, S, P, Q);
}
template <int S, int P>
__device__ __forceinline__ TilePix tile_pix(const TileGeom& g, int wq, int x1) { return conv_tile_pix(g, wq, x1, S, P); }

// Epilogue shared by the convolution kernels: bias, leaky ReLU, the fused 2x2 max-pool, the decision codes and
// the stores.  A lane holds, per 32x32 tile, 16 channels (8*(i/4) + 4*hi + i%4) of one pixel.  `bias_lds` is LDS
// no wavefront reads any more once all of them have arrived here (BM floats are used).
// Every map store is a buffer store: the lane's 32-bit byte offset carries the pixel (and the lane half's 4 channels),
// the channel travels as a scalar offset, and a lane that has nothing to store uses an offset beyond the buffer's
// records, which the hardware drops - no address arithmetic in 64 bits, no branch and no scalar reload per element.
__device__ __forceinline__ void store_elem(__amdgpu_buffer_rsrc_t r, unsigned vo, unsigned so, float v, const float*)
{
    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), r, vo, so, 0);
}
__device__ __forceinline__ void store_elem(__amdgpu_buffer_rsrc_t r, unsigned vo, unsigned so, float v, const bf16_t*)
{
    __builtin_amdgcn_raw_buffer_store_b16((uint16_t)bf16_bits(v), r, vo, so, 0);
}

// ... of a value that already is what the map holds (a bfloat widened to fp32: its upper half is stored)
__device__ __forceinline__ void store_rounded(__amdgpu_buffer_rsrc_t r, unsigned vo, unsigned so, float v, const float*)
{
    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), r, vo, so, 0);
}
__device__ __forceinline__ void store_rounded(__amdgpu_buffer_rsrc_t r, unsigned vo, unsigned so, float v, const bf16_t*)
{
    __builtin_amdgcn_raw_buffer_store_b16((uint16_t)(__float_as_uint(v) >> 16), r, vo, so, 0);
}

template <typename T, int K, int S, int WAVES_M, int MT, bool POOL_OUT, bool DELTA_IN, int NT>
__device__ __forceinline__ void conv_epilogue(const MfmaConvArgs& a, const TileGeom& g, v16f (&acc)[MT][NT], float* bias_lds,
                                              int m0, int x0, int x1, int y0, int stack, int ti, int tj)
{
    constexpr int BM = 32 * MT * WAVES_M;
    constexpr int P = K / 2;                           // S: patch positions per tile pixel and dimension (pool or stride)
    constexpr unsigned ES = sizeof(T);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_m = wave % WAVES_M, wave_n = wave / WAVES_M;
    const int hi = lane >> 5, l32 = lane & 31;
    const View& ov = DELTA_IN ? a.dout : a.out;
    // the tile's images start at image n_a of the stack; offsets from there fit 32 bits (checked by the launcher)
    const __amdgpu_buffer_rsrc_t orsrc = __builtin_amdgcn_make_buffer_rsrc((void*)((T*)ov.p + (long long)stack * ov.ss + (long long)g.n_a * ov.ns),
                                                                            (short)0, (int)0x7FFFFFFF, 0x00020000);
    const unsigned ocs = ES * (unsigned)ov.cs;         // bytes between channels
    // The bias goes through LDS: a global load between the stores below would make every store wait for all
    // earlier ones (loads and stores share one counter).
    if (!DELTA_IN) {
        __syncthreads();                               // every wavefront has left the multiply loop
        if (tid < BM) bias_lds[tid] = (a.bias && m0 + tid < a.Mtot) ? ld((const T*)a.bias + m0 + tid) : 0.0f;
        __syncthreads();
    }
    if (DELTA_IN) {
        // Deltas are stored as dLoss/dZ: where the boundary written to carries an activation, its derivative is
        // applied now.  A lane's 16 channels of a 32-channel block share one sign word; all words are loaded
        // before the first store, so that no load has to wait for stores.
        unsigned vo[NT];
        uint32_t sw[NT][MT];
        float in_slope = a.in_slope;
        asm volatile("" : "+v"(in_slope));             // (kept in a register: not re-read from the argument block per element)
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int q = (wave_n * NT + t) * 32 + l32;
            const TilePix tp = tile_pix<S, P>(g, q, x1);
            const int pn = tp.valid ? tp.n : 0, py = tp.valid ? y0 + tp.y : y0, pxx = tp.valid ? g.ox0 + tp.xl : x0;
            vo[t] = tp.valid ? ES * (unsigned)((pn - g.n_a) * (int)ov.ns + (py - ov.y0[ti]) * ov.pitch + (pxx - ov.x0[tj])) + 4u * hi * ocs : 0x80000000u;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const int mb = m0 + (wave_m * MT + mt) * 32;            // first channel of the block
                sw[t][mt] = (a.scale_out && mb < a.Mtot) ? *at<uint32_t>(a.isign, stack, ti, tj, pn, mb >> 5, py, pxx) : 0xFFFFFFFFu;
            }
        }
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const int mb = m0 + (wave_m * MT + mt) * 32;
                const uint32_t w = sw[t][mt] >> (4 * hi);
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    // (the channel count is a multiple of 4: a group of 4 channels exists as a whole or not at all)
                    const unsigned vg = mb + 8 * g4 + 4 * hi < a.Mtot ? vo[t] : 0x80000000u;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int i = 4 * g4 + e;
                        float v = acc[mt][t][i];
                        if (a.scale_out) v = scaled_delta<T>(v, (w >> (8 * g4 + e)) & 1u, in_slope);
                        store_elem(orsrc, vg, (unsigned)(mb + 8 * g4 + e) * ocs, v, (const T*)nullptr);
                    }
                }
            }
        return;
    }
    // While another workgroup's wavefront keeps the matrix cores of this SIMD busy, every vector-ALU instruction issued
    // here waits for a gap between its instructions, so the loop below is written for few of them: the bias is added in a
    // pass of its own that layers without bias skip, the sign bits are collected with constant masks and brought into
    // place once per word, scalar offsets carry the channel.
    float slope = a.slope;
    asm volatile("" : "+v"(slope));
    if (a.bias) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const float4 b4 = *(const float4*)(bias_lds + (wave_m * MT + mt) * 32 + 8 * g4 + 4 * hi);
                const float bb[4] = {b4.x, b4.y, b4.z, b4.w};
#pragma unroll
                for (int t = 0; t < NT; ++t)
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[mt][t][4 * g4 + e] += bb[e];
            }
    }
    const __amdgpu_buffer_rsrc_t mrsrc = __builtin_amdgcn_make_buffer_rsrc(
        POOL_OUT ? (void*)((uint8_t*)a.mask.p + (long long)stack * a.mask.ss + (long long)g.n_a * a.mask.ns) : (void*)ov.p, (short)0, (int)0x7FFFFFFF, 0x00020000);
    const unsigned mcs = (unsigned)a.mask.cs;
    // which of the lane's 4 groups of 4 channels exist, as a mask over its 16 sign bits (before they are shifted by 4 * hi)
    uint32_t gmask[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int mb = m0 + (wave_m * MT + mt) * 32;
        gmask[mt] = 0;
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4)
            if (mb + 8 * g4 + 4 * hi < a.Mtot) gmask[mt] |= 0xFu << (8 * g4);
    }
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int q = (wave_n * NT + t) * 32 + l32;
        const TilePix tp = tile_pix<S, P>(g, POOL_OUT ? (q >> 2) : q, x1);
        const int pn = tp.n, py = y0 + tp.y, pxx = g.ox0 + tp.xl;
        bool pvalid = tp.valid;
        if (POOL_OUT) pvalid = pvalid && (lane & 3) == 0;       // the window's first lane stores
        const bool powned = pvalid && py >= a.own.y0[ti] && py <= a.own.y1[ti] && pxx >= a.own.x0[tj] && pxx <= a.own.x1[tj];
        const unsigned vo = pvalid ? ES * (unsigned)((pn - g.n_a) * (int)ov.ns + (py - ov.y0[ti]) * ov.pitch + (pxx - ov.x0[tj])) + 4u * hi * ocs : 0x80000000u;
        // (code bytes exist only behind a pool, and only for owned pixels)
        const unsigned mvo = (POOL_OUT && powned) ? (unsigned)((pn - g.n_a) * (int)a.mask.ns + (py - a.mask.y0[ti]) * a.mask.pitch + (pxx - a.mask.x0[tj])) + 4u * hi * mcs
                                                  : 0x80000000u;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int mb = m0 + (wave_m * MT + mt) * 32;
            uint32_t signs = 0;                                 // this lane's 16 channels of the block's sign word, bits 8 * g4 + e
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const bool gok = (gmask[mt] >> (8 * g4)) & 1u;
                const unsigned vg = gok ? vo : 0x80000000u, mvg = gok ? mvo : 0x80000000u;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int i = 4 * g4 + e;
                    // compared and recorded as the map will hold it (rounded to the storage type)
                    float v;
                    bool pos;
                    int bi = 0;
                    if constexpr (sizeof(T) == 4 && !POOL_OUT) {
                        // (slopes are >= 0, so the activation is positive exactly where the convolution's result is)
                        const float z = acc[mt][t][i];
                        pos = z > 0.0f;
                        v = pos ? z : slope * z;
                    } else {
                        v = stored(leaky(acc[mt][t][i], slope), (const T*)nullptr);
                        if (POOL_OUT) {
                            // the 4 pixels of a window sit in 4 adjacent lanes, in window order; the first lane decides
                            const float o1 = quad_xor<1>(v), o2 = quad_xor<2>(v), o3 = quad_xor<3>(v);
                            if (o1 > v) { v = o1; bi = 1; }
                            if (o2 > v) { v = o2; bi = 2; }
                            if (o3 > v) { v = o3; bi = 3; }
                        }
                        pos = v > 0.0f;
                    }
                    const unsigned so = (unsigned)(mb + 8 * g4 + e);
                    store_rounded(orsrc, vg, so * ocs, v, (const T*)nullptr);
                    if (POOL_OUT) __builtin_amdgcn_raw_buffer_store_b8((uint8_t)((bi << 1) | (pos ? 1 : 0)), mrsrc, mvg, so * mcs, 0);
                    signs |= (pos ? 1u : 0u) << (8 * g4 + e);
                }
            }
            signs = (pvalid ? signs & gmask[mt] : 0u) << (4 * hi);
            // the other half of the block's channels sits 32 lanes away (same pixel)
            signs |= (uint32_t)__shfl_xor((int)signs, 32, 64);
            if (powned && hi == 0 && mb < a.Mtot)
                *at<uint32_t>(a.osign, stack, ti, tj, pn, mb >> 5, py, pxx) = signs;
        }
    }
}

// ---- the kernel ----------------------------------------------------------------------------------------------
// WAVES_M x WAVES_N wavefronts; each computes MT x NT tiles of 32 channels x 32 pixels.  A stage's patch and
// filter slice travel with buffer_load ... lds: every lane's element lands in LDS at (wave-uniform base +
// 4 * lane), no registers and no LDS-write instructions in between, and offsets beyond the buffer's records read
// as zero, which provides the zero padding.  16-bit (bfloat) elements arrive zero-extended in a dword and are
// shifted into place when the multiply loop reads them.  Two LDS buffers alternate: stage i+1 is in flight while
// the matrix cores work on stage i.
#define FTP_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
// LDS dword as loaded -> value: fp32 as is, a zero-extended bfloat shifted into the high half
__device__ __forceinline__ float widen(float v, const float*) { return v; }
__device__ __forceinline__ float widen(float v, const bf16_t*) { return __uint_as_float(__float_as_uint(v) << 16); }
constexpr unsigned kOobOffset = 0x80000000u;          // beyond the records of every buffer resource below
constexpr unsigned kBufRecords = 0x7FFFFFFFu;
// Reduction channels per stage: the same for every workgroup shape, so that the summation order, and with it every
// bit of the result, does not depend on which shape the launch heuristics pick (they look at the batch size).
// (5x5 and 7x7 filters take 2 channels per stage so that a slice of all taps still fits; a strided forward pass
// reads a patch four times the size of its tile.)
// (the bfloat matrix-core path takes 8 channels of a 3x3 filter per stage: one instruction multiplies 8 of them)
__host__ __device__ constexpr int conv_dl_stage_channels(int K, bool strided_fwd, bool bf_mfma) { return K >= 5 ? 2 : (K == 1 && !strided_fwd) ? 16 : bf_mfma ? 8 : 4; }
// POOL_IN (delta back-propagation through a fused pool): the patch lives at the convolution output, the delta at
// pooled resolution; a patch position receives its window's delta only if it is the window's winner for that
// channel.  The winner codes of the stage after next are loaded into registers one stage ahead, and a lane whose
// position lost simply loads from an out-of-range offset (= 0).
// STRIDE = 2, forward: output pixel (y, x) reads the patch at (2y, 2x), as the first pixel of a pool window does.
// STRIDE = 2, delta back-propagation: the adjoint of a strided convolution is the stride-1 one applied to the
// deltas with zeros inserted between them; a patch position at even coordinates loads delta (y/2, x/2), every
// other one loads from an out-of-range offset (three quarters of the matrix-core work multiply zeros).
// Wavefronts per SIMD the register allocation aims at: two as a rule (the fp32 tiles have 128 accumulator registers; the
// small tiles of the bfloat path then come out at about 160 registers, three wavefronts per SIMD); four for the pooled
// forward kernels of the bfloat path (32 accumulator registers; their epilogue is what needs the registers), which wait for
// loads more than they multiply and are as fast as the number of workgroups a CU holds (LDS holds four): config 5,
// forward of the three pooled layers 0.45 / 0.28 / 0.22 -> 0.44 / 0.26 / 0.21 ms; the same target made the unpooled and the
// delta kernels of the deep layers slower (more workgroups competing for the L2) and is not used there.
__host__ __device__ constexpr int conv_dl_waves(size_t elem, int K, int stride, int MT, int BN, int WAVES_M, bool pool_out)
{
    // (fp32 3x3, 256 pixels, at most 64 accumulator registers: these came out at 131-134 registers, one too many for a
    // fourth workgroup on the CU, which LDS would hold: config 4, forward of the 32 -> 64 layer 2.34 -> 2.22 ms)
    if (elem == 4 && K == 3 && stride == 1 && BN == 256 && MT * (BN / 32 / (4 / WAVES_M)) <= 4) return 4;
    return (elem == 2 && K <= 3 && stride == 1 && pool_out && BN == 128 && MT * (BN / 32 / (4 / WAVES_M)) <= 2) ? 4 : 2;
}

template <typename T, int K, int WAVES_M, int MT, int BN, bool POOL_OUT, bool DELTA_IN, bool POOL_IN, int STRIDE, bool WIDE>
__global__ void __launch_bounds__(256, conv_dl_waves(sizeof(T), K, STRIDE, MT, BN, WAVES_M, POOL_OUT))
k_conv_mfma_dl(MfmaConvArgs a)
{
    // WIDE: the patch travels 16 bytes a lane (fp32: quads of positions; bfloat matrix-core path: packed, 8 positions)
    static_assert(!WIDE || conv_dl_packable(sizeof(T), K, STRIDE, POOL_IN) || conv_dl_quads(sizeof(T), POOL_IN, STRIDE == 2 && DELTA_IN),
                  "wide patch loads: fp32 patches that are not gathered element by element, and the bfloat matrix-core path");
    static_assert(STRIDE == 1 || !(POOL_OUT || POOL_IN), "strided convolutions with a fused pool take the direct kernels");
    constexpr bool STRIDED_FWD = STRIDE == 2 && !DELTA_IN, UP_IN = STRIDE == 2 && DELTA_IN, HALF_IN = POOL_IN || UP_IN;
    constexpr unsigned ES = sizeof(T);                 // bytes per map element
    constexpr int WAVES_N = 4 / WAVES_M;
    constexpr int NT = BN / 32 / WAVES_N;
    constexpr int BM = 32 * MT * WAVES_M;
    constexpr bool BF = sizeof(T) == 2 && K <= 3 && STRIDE == 1;
    constexpr int kCK = conv_dl_stage_channels(K, STRIDED_FWD, BF);
    constexpr int KK = K * K, P = K / 2;
    constexpr int S = (POOL_OUT || STRIDED_FWD) ? 2 : 1;
    constexpr bool XH = WIDE && sizeof(T) == 2;        // the patch stays packed: [channel][position] bfloats
    constexpr bool XQ = WIDE && sizeof(T) == 4;        // fp32 quads
    constexpr int XMAX = conv_dl_max_positions(K, BN, STRIDED_FWD, XQ, XH);
    constexpr int MAXPOS = XMAX / 256;
    // fp32 patches (not those gathered element by element through pool winners or between inserted zeros) travel 16
    // bytes a lane: a quad of consecutive positions of one patch row (rows are padded to whole quads), 64 quads = 256
    // positions to an instruction, NQB such blocks per channel; the wavefronts take (block, channel) pairs in turn.
    // Packed bfloat patches travel the same way, 8 positions (16 bytes) a lane, 512 positions to an instruction; their rows
    // begin on the dword grid of the map (up to one position before the first column the tile needs).
    constexpr bool XW = XQ || XH;                      // wide loads
    constexpr int NPL = XH ? 8 : 4;                    // positions per lane
    constexpr int NQB = XMAX / (64 * NPL), NXI = (NQB * kCK + 3) / 4;
    constexpr bool ONEBLK = 4 % NQB == 0;              // a wavefront always meets the same block
    constexpr int NXB = ONEBLK ? 1 : NXI;
    // bfloat matrix-core path: the filter slice is ROWS rows of [BM][8 bfloats]; a row is (tap, the stage's 8
    // channels) for 3x3 (9 taps + 1 row of zeros) and (channels 8r .. 8r+7) for 1x1; step s multiplies rows 2s, 2s+1
    constexpr int ROWS = K == 3 ? 10 : kCK / 8;
    constexpr int WF = BF ? ROWS * BM * 4 : KK * kCK * BM;   // dwords of one filter slice (fp32: [tap][channel][BM])
    constexpr int WPIECES = WF / 64;                   // 64-dword pieces of the slice, dealt round-robin to the 4 wavefronts
    constexpr int WINSTR = (WPIECES + 3) / 4;
    static_assert(WF % 64 == 0, "the filter slice is loaded in 64-float pieces");
    constexpr int XDW = XH ? kCK * XMAX / 2 : kCK * XMAX;      // dwords of one stage's patch
    __shared__ __attribute__((aligned(16))) float bufA[WF + XDW];
    __shared__ __attribute__((aligned(16))) float bufB[WF + XDW];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_m = wave % WAVES_M, wave_n = wave / WAVES_M;
    const int hi = lane >> 5, l32 = lane & 31;
    // (tile, channel block, stack), tile fastest.  Where the launch says so the workgroups are renumbered in XCD order:
    // the tiles of one stack and channel block then run on one XCD, and as the channel-block count divides 8, an XCD
    // only ever meets one channel block's slice of the filter (with all blocks on every XCD the filters of the
    // 256 -> 512 layers do not stay in a 4 MB L2).
    int vgroup, vtile;
    const int ntiles = a.tiles_x * a.tiles_r;
    if (a.xcd_groups) {
        if (!xcd_order(a.mblocks * a.stacks, ntiles, vgroup, vtile)) return;
    } else {
        vgroup = (int)blockIdx.x / ntiles; vtile = (int)blockIdx.x - vgroup * ntiles;
    }
    const int stack = vgroup / a.mblocks, ti = stack / a.M, tj = stack % a.M;
    const int x0 = a.rect.x0[tj], x1 = a.rect.x1[tj], y0 = a.rect.y0[ti], y1 = a.rect.y1[ti];
    const TileGeom g = tile_geom<S, P, XH ? 8 : XQ ? 4 : 0>(a, x0, x1, y0, y1, vtile);
    if (g.empty) return;
    const int m0 = (vgroup % a.mblocks) * BM;
    const int PW = g.PW, CS = a.cs;                    // CS: whole 64-position blocks cover every patch

    // packed patches: a row starts `sh` (0 or 1) positions before the tile's first patch column, where the map's dword grid falls
    const int sh = XH ? ((g.ox0 * S - P - (DELTA_IN ? a.din : a.in).x0[tj]) & 1) : 0;
    int baseB[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int q = (wave_n * NT + t) * 32 + l32;
        const TilePix tp = tile_pix<S, P>(g, POOL_OUT ? (q >> 2) : q, x1);
        const int pos = POOL_OUT ? (q & 3) : 0;
        baseB[t] = (tp.valid ? (tp.prow + (pos >> 1)) * PW + tp.xl * S + (pos & 1) + sh : 0) + (BF ? 0 : hi * CS);
    }
    const int baseA = (BF ? 0 : hi * BM) + wave_m * (32 * MT) + l32;

    // ---- byte offset of each lane's patch positions from the workgroup's base (channel 0); padding -> out of range
    const int npos = g.npos;
    const View& sv = DELTA_IN ? a.din : a.in;
    const T* src = (const T*)sv.p + (long long)stack * sv.ss + (long long)g.n_a * sv.ns;
    unsigned xoff[XW ? NXB : MAXPOS];
    int moff[MAXPOS];               // POOL_IN: element offset in the code map (channel 0), this position's place in its window in the top bits
    unsigned xfix[NXB];             // wide loads: elements of the lane's unit that lie beside the map (zero padding): cleared once the unit has landed
    const uint8_t* __restrict__ msk = (const uint8_t*)a.mask.p + (long long)stack * a.mask.ss + (long long)g.n_a * a.mask.ns;
    if constexpr (XW) {
        // The buffer starts one unit in front of the images' first element, so that a unit that begins beside the map's
        // left border still has a non-negative offset (the maps lie inside the workspace, which has margins).
        src -= NPL;
#pragma unroll
        for (int ub = 0; ub < NXB; ++ub) {
            const int blk = ONEBLK ? wave % NQB : (wave + 4 * ub) % NQB;
            const int s = NPL * (blk * 64 + lane);
            xoff[ub] = kOobOffset; xfix[ub] = 0;
            if (s < npos) {
                const int pr = s / PW, c = s - pr * PW;
                int k = 0, lr = pr, ybase = g.y_a * S;
                if (pr >= g.first_cnt) {
                    const int t = pr - g.first_cnt;
                    k = 1 + t / g.per_cnt; lr = t - (k - 1) * g.per_cnt; ybase = 0;
                }
                const int gy = y0 * S + ybase + lr - P, gx = g.ox0 * S - P - sh + c;
                // rows no valid output pixel of this stack reads may lie outside the view; columns beside the needed ones
                // just bring along what lies there (never multiplied into a valid pixel)
                if (g.n_a + k < a.batch && gy >= 0 && gy < a.Hc && gy >= a.iy0[ti] && gy <= a.iy1[ti] && gx + NPL - 1 >= 0 && gx < a.Wc) {
                    xoff[ub] = ES * (unsigned)(NPL + k * (int)sv.ns + (gy - sv.y0[ti]) * sv.pitch + (gx - sv.x0[tj]));
#pragma unroll
                    for (int e = 0; e < NPL; ++e)
                        if (gx + e < 0 || gx + e >= a.Wc) xfix[ub] |= 1u << e;
                }
            }
        }
    }
#pragma unroll
    for (int j = 0; j < (XW ? 0 : MAXPOS); ++j) {
        const int s = tid + j * 256;
        xoff[j] = kOobOffset; moff[j] = 0;
        if (s < npos) {
            const int pr = s / PW, c = s - pr * PW;
            int k = 0, lr = pr, ybase = g.y_a * S;
            if (pr >= g.first_cnt) {
                const int t = pr - g.first_cnt;
                k = 1 + t / g.per_cnt; lr = t - (k - 1) * g.per_cnt; ybase = 0;
            }
            const int gy = y0 * S + ybase + lr - P, gx = g.ox0 * S - P + c;
            if (g.n_a + k < a.batch && gy >= 0 && gy < a.Hc && gx >= 0 && gx < a.Wc) {
                const int sy = HALF_IN ? (gy >> 1) : gy, sx = HALF_IN ? (gx >> 1) : gx;
                // positions no valid output pixel of this stack reads may lie outside the view
                if (sy >= a.iy0[ti] && sy <= a.iy1[ti] && sx >= a.ix0[tj] && sx <= a.ix1[tj] && !(UP_IN && ((gy | gx) & 1))) {
                    xoff[j] = ES * (unsigned)(k * (int)sv.ns + (sy - sv.y0[ti]) * sv.pitch + (sx - sv.x0[tj]));
                    if (POOL_IN) moff[j] = (k * (int)a.mask.ns + (sy - a.mask.y0[ti]) * a.mask.pitch + (sx - a.mask.x0[tj]))
                                           | ((((gy & 1) << 1) | (gx & 1)) << 29);
                }
            }
        }
    }
    // winner codes of one stage, per position and channel
    uint8_t codes[MAXPOS][kCK];
    auto load_codes = [&](int c0) {
        if (!POOL_IN) return;
#pragma unroll
        for (int j = 0; j < MAXPOS; ++j)
#pragma unroll
            for (int k = 0; k < kCK; ++k) {
                const int ci = c0 + k < a.C ? c0 + k : a.C - 1;
                codes[j][k] = msk[(moff[j] & 0x1FFFFFFF) + (long long)ci * a.mask.cs];
            }
    };
    // filter: a load instruction covers 64 consecutive floats of the slice; with BM >= 64 that is (part of) one
    // row, with BM = 32 two rows (two consecutive reduction channels)
    // (bfloat path: one 16-byte load per lane = the 8 bfloats of one output channel; 64 channels to an instruction)
    // (fp32 slices whose 1 KB pieces hold rows of one tap only: 16 bytes per lane, lane -> (row of the piece, 4 channels))
    constexpr bool W16 = !BF && kCK % (256 / BM) == 0 && WF % 256 == 0;
    unsigned woff;
    int wrow = 0;
    if constexpr (W16) {
        const int col = 4 * (lane % (BM / 4));
        wrow = lane / (BM / 4);
        woff = m0 + col < a.Mtot ? 4u * (unsigned)(wrow * a.Mtot + col) : kOobOffset;
    } else {
        const int col = BM >= 64 ? (wave % (BM / 64 > 0 ? BM / 64 : 1)) * 64 + lane : (lane & 31);
        woff = m0 + col < a.Mtot ? 4u * (unsigned)((BM >= 64 ? 0 : (lane >> 5) * a.Mtot) + col) : kOobOffset;
    }
    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc((void*)src, (short)0, (int)kBufRecords, 0x00020000);
    const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc((void*)a.wt, (short)0, (int)kBufRecords, 0x00020000);

    v16f acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[mt][t][i] = 0.0f;

    auto issue = [&](float* buf, int c0) {
        float* Wl = buf;
        float* Xl = buf + WF;
        if constexpr (BF) {
            // rows x parts of 64 output channels, dealt round-robin to the 4 wavefronts
            constexpr int PARTS = (BM + 63) / 64, NLOAD = ROWS * PARTS;
            const int C8 = (a.C + 7) >> 3;
#pragma unroll
            for (int u = 0; u < (NLOAD + 3) / 4; ++u) {
                const int idx = wave + 4 * u;
                if (idx < NLOAD) {
                    const int r = idx / PARTS, part = idx - r * PARTS;
                    const int tap = K == 3 ? r : 0, oct = (c0 >> 3) + (K == 3 ? 0 : r);
                    const int col = part * 64 + lane;
                    if (col < BM) {
                        const unsigned so = 16u * (unsigned)((tap * C8 + oct) * a.Mtot + m0);
                        const unsigned vo = (oct < C8 && m0 + col < a.Mtot) ? 16u * (unsigned)col : kOobOffset;
                        __builtin_amdgcn_raw_ptr_buffer_load_lds(wrsrc, FTP_LDS_PTR(Wl + (r * BM + part * 64) * 4), 16, vo, so, 0, 0);
                    }
                }
            }
        }
        if constexpr (W16) {
            // a load instruction covers 256 consecutive floats of the slice: 16 bytes per lane, RPP rows of one tap
            constexpr int RPP = 256 / BM, WP4 = WF / 256;
#pragma unroll
            for (int u = 0; u < (WP4 + 3) / 4; ++u) {
                const int idx = wave + 4 * u;
                if (idx >= WP4) break;
                const int row0 = idx * RPP, tap = row0 / kCK, k0 = row0 - tap * kCK;
                const unsigned so = 4u * (unsigned)((tap * a.C + c0 + k0) * a.Mtot + m0);
                const unsigned vo = c0 + k0 + wrow < a.C ? woff : kOobOffset;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(wrsrc, FTP_LDS_PTR(Wl + idx * 256), 16, vo, so, 0, 0);
            }
        }
#pragma unroll
        for (int u = 0; u < WINSTR; ++u) {
            const int idx = wave + 4 * u;                              // 64-dword piece of the slice
            if (idx >= WPIECES) break;
            if constexpr (BF || W16) continue;
            const int row = BM >= 64 ? idx / (BM / 64 > 0 ? BM / 64 : 1) : 2 * idx;
            const int tap = row / kCK, k = row - tap * kCK;
            const unsigned so = 4u * (unsigned)((tap * a.C + c0 + k) * a.Mtot + m0);
            unsigned vo;
            if (BM >= 64) vo = c0 + k < a.C ? woff : kOobOffset;
            else          vo = c0 + k + (lane >> 5) < a.C ? woff : kOobOffset;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(wrsrc, FTP_LDS_PTR(Wl + idx * 64), 4, vo, so, 0, 0);
        }
        if constexpr (XW) {
#pragma unroll
            for (int u = 0; u < NXI; ++u) {
                const int id = wave + 4 * u;
                const int blk = id % NQB, k = id / NQB;
                if (id < NQB * kCK && blk * (64 * NPL) < npos) {
                    const unsigned vo = c0 + k < a.C ? xoff[ONEBLK ? 0 : u] : kOobOffset;
                    const unsigned so = ES * (unsigned)((c0 + k) * (int)sv.cs);
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(xrsrc, FTP_LDS_PTR((char*)Xl + (int)ES * (k * CS + blk * (64 * NPL))), 16, vo, so, 0, 0);
                }
            }
        }
#pragma unroll
        for (int j = 0; j < (XW ? 0 : MAXPOS); ++j) {
            const int blk = wave + 4 * j;
            if (blk * 64 < npos) {
#pragma unroll
                for (int k = 0; k < kCK; ++k) {
                    unsigned vo = c0 + k < a.C ? xoff[j] : kOobOffset;
                    if (POOL_IN && ((codes[j][k] >> 1) & 3) != ((unsigned)moff[j] >> 29)) vo = kOobOffset;
                    const unsigned so = ES * (unsigned)((c0 + k) * (int)sv.cs);
                    // (the element size has to be a literal)
                    if constexpr (sizeof(T) == 4) __builtin_amdgcn_raw_ptr_buffer_load_lds(xrsrc, FTP_LDS_PTR(Xl + k * CS + blk * 64), 4, vo, so, 0, 0);
                    else                          __builtin_amdgcn_raw_ptr_buffer_load_lds(xrsrc, FTP_LDS_PTR(Xl + k * CS + blk * 64), 2, vo, so, 0, 0);
                }
            }
        }
    };

    // one step = 2 reduction channels of one tap; the operands of step j+1 are read from LDS before the
    // matrix-core instructions of step j are issued
    auto multiply = [&](const float* buf) {
        const float* Wl = buf;
        const float* Xl = buf + WF;
        if constexpr (BF) {
            // one step = rows 2s and 2s+1 of the slice: lanes 0-31 feed row 2s, lanes 32-63 row 2s+1 (8 reduction
            // elements each); the 8 patch values of a lane are zero-extended bfloats and are packed two to a dword
            constexpr int NSTEP16 = ROWS / 2;
            uint4 av[2][MT], bv[2][NT];
            auto load_step = [&](int s2, int b) {
                const int r = 2 * s2 + hi;
                int boff;
                if (K == 3) { const int tap = r < KK ? r : 0; boff = (tap / 3) * PW + (tap - (tap / 3) * 3); }
                else        boff = 8 * r * CS;
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) av[b][mt] = *(const uint4*)(Wl + ((r * BM + baseA + 32 * mt) << 2));
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    uint32_t x[8];
                    if constexpr (XH) {
                        const bf16_t* xp = (const bf16_t*)Xl + baseB[t] + boff;
#pragma unroll
                        for (int k = 0; k < 8; ++k) x[k] = xp[k * CS];
                    } else {
                        const float* xp = Xl + baseB[t] + boff;
#pragma unroll
                        for (int k = 0; k < 8; ++k) x[k] = __float_as_uint(xp[k * CS]);
                    }
                    bv[b][t] = make_uint4(x[0] | (x[1] << 16), x[2] | (x[3] << 16), x[4] | (x[5] << 16), x[6] | (x[7] << 16));
                }
            };
            load_step(0, 0);
#pragma unroll
            for (int j = 0; j < NSTEP16; ++j) {
                if (j + 1 < NSTEP16) load_step(j + 1, (j + 1) & 1);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int t = 0; t < NT; ++t)
                        acc[mt][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, av[j & 1][mt]),
                                                                            __builtin_bit_cast(v8bf, bv[j & 1][t]), acc[mt][t], 0, 0, 0);
            }
            return;
        }
        constexpr int NSTEP = KK * (kCK / 2);
        float av[2][MT], bv[2][NT];
        auto load_step = [&](int j, int b) {
            const int tap = j / (kCK / 2), i = j - tap * (kCK / 2);
            const int toff = (tap / K) * PW + (tap % K);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) av[b][mt] = Wl[(tap * kCK + 2 * i) * BM + baseA + 32 * mt];
#pragma unroll
            for (int t = 0; t < NT; ++t) bv[b][t] = widen(Xl[baseB[t] + 2 * i * CS + toff], (const T*)nullptr);
        };
        load_step(0, 0);
#pragma unroll
        for (int j = 0; j < NSTEP; ++j) {
            if (j + 1 < NSTEP) load_step(j + 1, (j + 1) & 1);
            __builtin_amdgcn_sched_barrier(0);         // keep these reads ahead of the matrix-core instructions below
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    acc[mt][t] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[j & 1][mt], bv[j & 1][t], acc[mt][t], 0, 0, 0);
        }
    };

    // wide loads: once this wavefront's units of a stage have landed, the elements beside the map become the zero padding
    auto fixup = [&](float* buf) {
        if constexpr (XW) {
            T* Xl = (T*)(buf + WF);                    // (elements as the maps hold them)
#pragma unroll
            for (int u = 0; u < NXI; ++u) {
                const int id = wave + 4 * u;
                const int blk = id % NQB, k = id / NQB;
                const unsigned f = xfix[ONEBLK ? 0 : u];
                if (id < NQB * kCK && f) {
                    T* q = Xl + k * CS + blk * (64 * NPL) + NPL * lane;
#pragma unroll
                    for (int e = 0; e < NPL; ++e)
                        if ((f >> e) & 1u) q[e] = (T)0;
                }
            }
        }
    };
    const int nst = (a.C + kCK - 1) / kCK;
    load_codes(0);
    issue(bufA, 0);                                     // (waits for the codes it selects by)
    load_codes(kCK);
    for (int st = 0; st < nst; st += 2) {
        __builtin_amdgcn_s_waitcnt(0x0F70);            // vmcnt(0): this wavefront's share of the stage has landed
        fixup(bufA);
        __syncthreads();                               // ... and everybody's; the other buffer is free again
        if (st + 1 < nst) { issue(bufB, (st + 1) * kCK); load_codes((st + 2) * kCK); }
        multiply(bufA);
        if (st + 1 < nst) {
            __builtin_amdgcn_s_waitcnt(0x0F70);
            fixup(bufB);
            __syncthreads();
            if (st + 2 < nst) { issue(bufA, (st + 2) * kCK); load_codes((st + 3) * kCK); }
            multiply(bufB);
        }
    }
    conv_epilogue<T, K, S, WAVES_M, MT, POOL_OUT, DELTA_IN>(a, g, acc, bufA, m0, x0, x1, y0, stack, ti, tj);
}

// ---- host side ------------------------------------------------------------------------------------------------
namespace {

// Largest byte offset a workgroup forms from its base pointer: the images a tile can span plus all channels.
bool offsets_fit_32bit(const MfmaConvArgs& a, const View& v, int max_img, int K)
{
    const double bytes = 4.0 * ((double)max_img * (double)v.ns + (double)a.C * (double)v.cs);      // (fp32 element size as the bound)
    return bytes < 2.0e9 && 4.0 * K * K * (double)a.C * (double)a.Mtot < 2.0e9;
}

// Workgroup shapes of the direct-load kernel: output channels x pixels, and the workgroups of each that share a CU.
struct DlShape { int BM, BN, per_cu; };

// The largest workgroup whose filter slice (all taps of a stage) still fits LDS next to the patch.
constexpr int conv_dl_max_bm(int K) { return K >= 7 ? 64 : 128; }

template <typename T, int K, bool POOL_OUT, bool DELTA_IN, bool POOL_IN, int STRIDE>
void launch_dl(const MfmaConvArgs& a, DlShape sh, bool wide, dim3 grid, hipStream_t s)
{
    static char label[12][104];                  // (every write of an entry stores the same text: entries depend on the template and the shape only)
    const int v = ((sh.BM == 128 ? 0 : sh.BM == 64 ? 1 : 2) * 2 + (sh.BN == 256 ? 0 : 1)) * 2 + (wide ? 1 : 0);
    std::snprintf(label[v], sizeof(label[v]), "k_conv_mfma_dl<%s, %d, %d, %d, %d, %s, %s, %s, %d, %s>", sizeof(T) == 4 ? "float" : "unsigned short",
                  K, sh.BM == 128 ? 2 : 1, sh.BM == 32 ? 1 : 2, sh.BN, POOL_OUT ? "true" : "false", DELTA_IN ? "true" : "false",
                  POOL_IN ? "true" : "false", STRIDE, wide ? "true" : "false");
    g_kernel_label = label[v];
    constexpr bool STRIDED_FWD = STRIDE == 2 && !DELTA_IN;
    // (which forms exist: the delta maps always lie inside the workspace, so an fp32 delta pass that can load wide always does)
    constexpr bool QUADABLE = conv_dl_quads(sizeof(T), POOL_IN, STRIDE == 2 && DELTA_IN);
    constexpr bool WIDEABLE = QUADABLE || conv_dl_packable(sizeof(T), K, STRIDE, POOL_IN);
    constexpr bool NARROWABLE = !(QUADABLE && DELTA_IN);
#define FTP_DL(WM, MT, BN) do { \
        if (wide) { if constexpr (WIDEABLE) hipLaunchKernelGGL((k_conv_mfma_dl<T, K, WM, MT, BN, POOL_OUT, DELTA_IN, POOL_IN, STRIDE, true>), grid, dim3(256), 0, s, a); } \
        else { if constexpr (NARROWABLE) hipLaunchKernelGGL((k_conv_mfma_dl<T, K, WM, MT, BN, POOL_OUT, DELTA_IN, POOL_IN, STRIDE, false>), grid, dim3(256), 0, s, a); } } while (0)
    if (sh.BN == 256) {
        if constexpr (!STRIDED_FWD) {
            // (the 3x3 bfloat path never takes 128 channels x 256 pixels: its 8-channel stages would not fit 64 KB of LDS)
            if (sh.BM == 128) { if constexpr (conv_dl_max_bm(K) >= 128 && !(sizeof(T) == 2 && K == 3 && STRIDE == 1)) FTP_DL(2, 2, 256); }
            else if (sh.BM == 64) FTP_DL(1, 2, 256); else FTP_DL(1, 1, 256);
        }
    } else {
        if (sh.BM == 128) { if constexpr (conv_dl_max_bm(K) >= 128) FTP_DL(2, 2, 128); }
        else if (sh.BM == 64) FTP_DL(1, 2, 128); else FTP_DL(1, 1, 128);
    }
#undef FTP_DL
}

// Picks the workgroup shape whose launch finishes first.  All workgroups of a launch do the same amount of
// matrix-core work (BM x BN x reduction), `per_cu` of them share one CU's matrix cores, and the last, partly
// filled round of a launch leaves CUs idle: few large workgroups waste most there, many small ones least, while
// larger ones re-read less.  cost = (full rounds + the last round's depth per CU) x work of one workgroup.
template <int K, bool POOL_OUT, bool STRIDED_FWD>
DlShape choose_dl_shape(const MfmaConvArgs& a, const ConvArgs& c, int npl, bool gather, TileChoice* tc_out)
{
    const int S = (POOL_OUT || STRIDED_FWD) ? 2 : 1;
    DlShape best = {0, 0, 0}; double best_cost = 0;
    int rws[kTabGrid], rhs[kTabGrid];                   // widths / heights of the stacks' rectangles per tile column / row
    for (int j = 0; j < c.M; ++j) rws[j] = a.rect.x1[j] - a.rect.x0[j] + 1;
    for (int i = 0; i < c.N; ++i) rhs[i] = a.rect.y1[i] - a.rect.y0[i] + 1;
    // as many output channels per workgroup as the layer has (up to 128): every further channel block re-reads the
    // whole input patch, and with many blocks in flight the filter no longer stays in the L2 cache
    int BM = a.Mtot >= 128 ? 128 : a.Mtot > 32 ? 64 : 32;
    if (BM > conv_dl_max_bm(K)) BM = conv_dl_max_bm(K);
    // The bfloat path finishes a stage's multiply long before the next stage's loads arrive; what hides that is more
    // workgroups per CU, so its 3x3 layers take 64-channel workgroups (half the accumulator registers): config 5
    // forward of the 64 -> 128 layer 0.89 -> 0.41 ms.  (32 channels re-read the patch too often; 1x1 layers lose.)
    if (c.bf16 && K == 3 && !STRIDED_FWD && c.S == 1 && BM > 64) BM = 64;
    // (the cost model below is for kernels bound by the matrix cores; the bfloat 3x3 path is bound by latency and
    // does best with the most workgroups per CU: 64 channels x 128 pixels; config 5: 14.6 -> 14.4 ms per step)
    const bool small_wg = c.bf16 && K == 3 && !STRIDED_FWD && c.S == 1 && BM == 64;
    auto consider = [&](int bm, int BN) -> long long {
        const int max_pos = conv_dl_max_positions(K, BN, STRIDED_FWD, npl == 4, npl == 8);
        const TileChoice tc = choose_tile(rws, rhs, c.N, c.M, c.batch, POOL_OUT ? BN / 4 : BN, S, K / 2, max_pos, npl, gather);
        if (tc.cs > max_pos) return -1;
        // tiles that exist: every stack has its own count, the grid is sized for the largest
        long long wgs = 0;
        for (int i = 0; i < c.N; ++i)
            for (int j = 0; j < c.M; ++j) {
                const int rw = a.rect.x1[j] - a.rect.x0[j] + 1, rh = a.rect.y1[i] - a.rect.y0[i] + 1;
                wgs += tile_slots(tc, rw, rh, c.batch);
            }
        const int mblocks = (a.Mtot + bm - 1) / bm;
        wgs *= mblocks;
        const int per_cu = BN == 256 ? (bm == 32 ? 3 : 2) : (bm == 32 ? 4 : 3);
        const long long slots = 256LL * per_cu;
        const double rounds = (double)(wgs / slots) * per_cu + (double)((wgs % slots + 255) / 256);
        // in units of 1/128 cycle: multiply loop, epilogue (about 25k cycles for 128 x 256), set-up (about 10k cycles)
        const double work = (double)bm * BN * a.C * K * K + 3.2e6 * (bm * BN) / (128.0 * 256.0) + 1.3e6;
        const double cost = rounds * work * (BN == 256 ? 1.0 : 1.03);
        if (best.BM == 0 || cost < best_cost) { best = {bm, BN, per_cu}; best_cost = cost; *tc_out = tc; }
        return wgs;
    };
    long long widest_wgs = 0;
    int bn_first = (STRIDED_FWD || small_wg) ? 128 : 256;
    if (small_wg && POOL_OUT) {
        // ... unless 128-pixel tiles (32 pool windows) fit the rows of the rectangles badly: a row of 19 windows leaves
        // 13 of 32 slots empty, while three such rows fill 57 of 64 (config 5, the 32 -> 64 layer: 0.68 -> 0.58 ms)
        long long units = 0, slots = 0;
        const TileChoice t128 = choose_tile(rws, rhs, c.N, c.M, c.batch, 32, S, K / 2, conv_dl_max_positions(K, 128, STRIDED_FWD, npl == 4, npl == 8), npl, gather);
        for (int i = 0; i < c.N; ++i)
            for (int j = 0; j < c.M; ++j) {
                const int rw = a.rect.x1[j] - a.rect.x0[j] + 1, rh = a.rect.y1[i] - a.rect.y0[i] + 1;
                units += (long long)c.batch * rh * rw;
                slots += tile_slots(t128, rw, rh, c.batch) * t128.cap;
            }
        if (slots > 0 && (double)units < 0.7 * (double)slots) bn_first = 256;
    }
    for (int BN = bn_first; BN >= (bn_first == 256 && small_wg ? 256 : 128); BN /= 2) {
        const long long w = consider(BM, BN);
        if (w > widest_wgs) widest_wgs = w;
    }
    // A launch that does not even fill the CUs once (small batches) is bound by the length of one workgroup's chain
    // of matrix-core instructions: narrower channel blocks shorten it and bring more CUs to work (config 2, batch 1).
    if (widest_wgs > 0 && widest_wgs < 256)
        for (int bm = BM / 2; bm >= 32; bm /= 2)
            for (int BN = STRIDED_FWD ? 128 : 256; BN >= 128; BN /= 2) consider(bm, BN);
    return best;
}

// Returns non-zero if the layer's geometry does not fit the kernel (offsets beyond 32 bits, a row of some stack
// wider than the patch buffer); the caller then uses a direct kernel.
template <typename T, int K, bool POOL_OUT, bool DELTA_IN, bool POOL_IN, int STRIDE>
int launch_t(MfmaConvArgs& a, const ConvArgs& c, hipStream_t s)
{
    constexpr bool STRIDED_FWD = STRIDE == 2 && !DELTA_IN;
    TileChoice td;
    // fp32 patches are loaded 16 bytes a lane, a few bytes beyond the ends of map rows: only inside the workspace (the
    // caller's input, which a wide first layer reads, is loaded element by element)
    constexpr bool quadable = conv_dl_quads(sizeof(T), POOL_IN && DELTA_IN, STRIDE == 2 && DELTA_IN);
    const bool quad = quadable && (DELTA_IN ? c.din_ws : c.in_ws);
    if (quadable && DELTA_IN && !quad) return 1;
    // 16-bit maps on the bfloat matrix-core path: the patch stays packed in LDS and travels 16 bytes a lane where every row
    // of the view starts on a 4-byte boundary (even strides) inside the workspace; otherwise element by element
    bool pack = false;
    if constexpr (conv_dl_packable(sizeof(T), K, STRIDE, POOL_IN && DELTA_IN)) {
        const View& iv = DELTA_IN ? a.din : a.in;
        pack = (DELTA_IN ? c.din_ws : c.in_ws) && ((uintptr_t)iv.p & 3) == 0 && !(iv.pitch & 1) && !(iv.cs & 1) && !(iv.ns & 1) && !(iv.ss & 1);
    }
    const int npl = quad ? 4 : pack ? 8 : 0;
    // (16-bit maps through a fused pool: the kernel waits for its patch more than it multiplies, and runs of pixels, which
    // touch more patch rows, were measured slower: config 5 forward of the pooled layers 0.45 / 0.28 / 0.22 -> 0.50 / 0.33 / 0.24 ms)
    const bool costly_patch = ((POOL_IN || STRIDE == 2) && DELTA_IN) || (sizeof(T) == 2 && POOL_OUT && !DELTA_IN);
    const DlShape sh = choose_dl_shape<K, POOL_OUT, STRIDED_FWD>(a, c, npl, costly_patch, &td);
    if (!sh.BM) return 1;
    // (the kernel keeps code-map offsets in 29 bits)
    if (POOL_IN && DELTA_IN && (double)td.max_img * (double)a.mask.ns >= 5.0e8) return 1;
    if (!offsets_fit_32bit(a, DELTA_IN ? a.din : a.in, td.max_img, K)) return 1;
    // (the epilogue's buffer stores: the images a tile spans plus all output channels, maps and code bytes alike)
    {
        const View& ov = DELTA_IN ? a.dout : a.out;
        if (4.0 * ((double)td.max_img * (double)ov.ns + ((double)a.Mtot + 8.0) * (double)ov.cs) >= 2.0e9) return 1;
        if (POOL_OUT && !DELTA_IN && (double)td.max_img * (double)a.mask.ns + ((double)a.Mtot + 8.0) * (double)a.mask.cs >= 2.0e9) return 1;
    }
    a.TC = td.TC; a.tiles_x = td.tiles_x; a.tiles_r = td.tiles_r; a.cap = td.cap; a.flat = td.flat; a.cs = pack ? (td.cs + 511) & ~511 : quad ? (td.cs + 255) & ~255 : (td.cs + 63) & ~63;
    a.mblocks = (a.Mtot + sh.BM - 1) / sh.BM; a.stacks = c.N * c.M;
    // XCD order pays where several channel blocks compete for the L2 and the groups spread evenly over the 8 XCDs;
    // with one channel block the plain order (neighbouring tiles on different XCDs) balances better
    const int groups = a.mblocks * a.stacks, ntiles = a.tiles_x * a.tiles_r;
    a.xcd_groups = (a.mblocks >= 2 && 8 % a.mblocks == 0 && groups % 8 == 0) ? 1 : 0;
    const unsigned nwg = a.xcd_groups ? xcd_grid(groups, ntiles) : (unsigned)(groups * ntiles);
    launch_dl<T, K, POOL_OUT && !DELTA_IN, DELTA_IN, POOL_IN && DELTA_IN, STRIDE>(a, sh, quad || pack, dim3(nwg), s);
    return 0;
}

template <int K, bool POOL_OUT, bool DELTA_IN, bool POOL_IN, int STRIDE = 1>
int launch_m(MfmaConvArgs& a, const ConvArgs& c, hipStream_t s)
{
    return c.bf16 ? launch_t<bf16_t, K, POOL_OUT, DELTA_IN, POOL_IN, STRIDE>(a, c, s) : launch_t<float, K, POOL_OUT, DELTA_IN, POOL_IN, STRIDE>(a, c, s);
}

void fill_common(MfmaConvArgs& a, const ConvArgs& c, const RectTab& inrect)
{
    a.in = c.in; a.out = c.out; a.mask = c.mask; a.din = c.din; a.dout = c.dout; a.rect = c.rect; a.own = c.own;
    for (int t = 0; t < kTabGrid; ++t) { a.ix0[t] = inrect.x0[t]; a.ix1[t] = inrect.x1[t]; a.iy0[t] = inrect.y0[t]; a.iy1[t] = inrect.y1[t]; }
    a.Hc = c.Hc; a.Wc = c.Wc; a.slope = c.slope; a.M = c.M; a.batch = c.batch;
    a.osign = c.osign; a.isign = c.isign; a.scale_out = c.scale_out; a.in_slope = c.in_slope;
}

}  // namespace

// Geometry: stride 1 with K = 1, 3 (with or without the fused pool over an even map) or K = 5, 7 (no fused pool);
// stride 2 with K = 1, 3 and no fused pool.
bool mfma_conv_eligible(const ConvArgs& a, bool backward)
{
    const int Mtot = backward ? a.Cin : a.Cout, C = backward ? a.Cout : a.Cin;
    if (a.pooled && (a.S != 1 || a.K > 3 || ((a.Hc | a.Wc) & 1))) return false;
    if (a.S == 2 && a.K > 3) return false;
    return Mtot >= 16 && Mtot % 4 == 0 && C >= 8;
}

bool mfma_conv_packs_bf16(const ConvArgs& a) { return a.bf16 && a.K <= 3 && a.S == 1; }

void prep_filter(const void* w, int bf16, int packed16, float* wt_fwd, float* wt_bwd, int Cout, int Cin, int K, hipStream_t s)
{
    if (packed16) {
        // (fits the fp32 areas: at most 10 taps x (C + 7) x M x 2 bytes against K*K x C x M x 4, C >= 8)
        const int taps = K == 3 ? 10 : 1;
        const long long cmax = (long long)taps * (((wt_fwd ? Cin : Cout) + 7) / 8) * (wt_fwd ? Cout : Cin) * 8;
        const long long cboth = (long long)taps * ((std::max(Cin, Cout) + 7) / 8) * std::max(Cin, Cout) * 8;
        const long long n16 = wt_fwd && wt_bwd ? cboth : cmax;
        hipLaunchKernelGGL(k_prep_filter16, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, s, (const bf16_t*)w, (bf16_t*)wt_fwd, (bf16_t*)wt_bwd,
                           Cout, Cin, K * K, taps);
        return;
    }
    const long long n = (long long)Cout * Cin * K * K;
    const dim3 grid((unsigned)((n + 255) / 256)), block(256);
    if (bf16) hipLaunchKernelGGL(k_prep_filter<bf16_t>, grid, block, 0, s, (const bf16_t*)w, wt_fwd, wt_bwd, Cout, Cin, K * K);
    else      hipLaunchKernelGGL(k_prep_filter<float>, grid, block, 0, s, (const float*)w, wt_fwd, wt_bwd, Cout, Cin, K * K);
}

// Forward: c.rect = forward rectangle at the unit's output boundary; inrect = extent of the input view per stack.
// Returns non-zero if the layer's geometry does not fit this kernel (the caller then uses the direct kernel).
int mfma_conv_fwd(const ConvArgs& c, const RectTab& inrect, const float* wt, hipStream_t s)
{
    MfmaConvArgs a;
    fill_common(a, c, inrect);
    a.wt = wt; a.bias = c.bias;
    a.C = c.Cin; a.Mtot = c.Cout;
    a.Hc = c.Hi; a.Wc = c.Wi;                           // the patch is cut from the input map
    if (c.S == 2) return c.K == 3 ? launch_m<3, false, false, false, 2>(a, c, s) : launch_m<1, false, false, false, 2>(a, c, s);
    if (c.K == 7) return launch_m<7, false, false, false>(a, c, s);
    if (c.K == 5) return launch_m<5, false, false, false>(a, c, s);
    if (c.K == 3) return c.pooled ? launch_m<3, true, false, false>(a, c, s) : launch_m<3, false, false, false>(a, c, s);
    return c.pooled ? launch_m<1, true, false, false>(a, c, s) : launch_m<1, false, false, false>(a, c, s);
}

// Backward data: c.rect = backward rectangle at the unit's input boundary; inrect = extent of the delta view
// (at the unit's output boundary, pooled coordinates if the unit has a pool).
int mfma_conv_bwd_data(const ConvArgs& c, const RectTab& inrect, const float* wt, hipStream_t s)
{
    // (stride 2: the kernel that splits the pixels into their four parity classes multiplies no inserted zeros)
    if (c.S == 2 && (c.K == 3 || c.K == 1) && delta_s2_mfma(c, inrect, wt, s) == 0) return 0;
    MfmaConvArgs a;
    fill_common(a, c, inrect);
    a.wt = wt; a.bias = nullptr;
    a.C = c.Cout; a.Mtot = c.Cin;
    // the patch is cut from the deltas as the stride-1 convolution sees them: at the convolution output (stride 1,
    // also through a pool), or with zeros inserted between them (stride 2: twice the extent)
    a.Hc = c.S == 2 ? 2 * c.Hc : c.Hc; a.Wc = c.S == 2 ? 2 * c.Wc : c.Wc;
    if (c.S == 2) return c.K == 3 ? launch_m<3, false, true, false, 2>(a, c, s) : launch_m<1, false, true, false, 2>(a, c, s);
    if (c.K == 7) return launch_m<7, false, true, false>(a, c, s);
    if (c.K == 5) return launch_m<5, false, true, false>(a, c, s);
    if (c.K == 3) return c.pooled ? launch_m<3, false, true, true>(a, c, s) : launch_m<3, false, true, false>(a, c, s);
    return c.pooled ? launch_m<1, false, true, true>(a, c, s) : launch_m<1, false, true, false>(a, c, s);
}

}  // namespace ftp
