// Host-side launch descriptors of libftp's kernels.
#pragma once
#include <hip/hip_runtime.h>
#include "ftp_device.h"
#include "ftp_plan.h"

namespace ftp {

// Name of the main kernel of the most recent launch on this thread (for the timing records).
extern thread_local const char* g_kernel_label;

// One convolution unit (convolution + leaky ReLU, optionally with the 2x2 pool behind it).
// Which fields a pass reads:
//   forward        in (activation at the input), out (activation at the output), mask (decision codes at the
//                  output boundary, written for owned pixels), rect = forward rectangle at the output boundary,
//                  own = owned rectangle there
//   backward data  din (delta at the output boundary), mask (pooled units: winners), dout (delta at the input),
//                  rect = backward rectangle at the input boundary; isign / scale_out / in_slope: see below
//   filter grad    in, din, mask, rect = owned rectangle at the convolution output (before the pool)
// Decision code: bit 0 = activation > 0, bits 1-2 = winner 2*dy+dx of the 2x2 window (pooled units).
// The forward pass also packs bit 0 into the sign map of the output boundary (osign): 32-bit words
// [image][channel / 32][y][x], bit channel % 32.
// Deltas are stored as dLoss/dZ: a delta map already carries the leaky-ReLU derivative of the convolution unit
// that produced its boundary, so readers only route through pool winners.  A pass that writes the delta of its
// input boundary applies that boundary's derivative itself (scale_out: the bit in isign selects 1 or in_slope).
struct ConvArgs {
    View in, out, mask, din, dout;
    View osign, isign;              // sign maps at the output / input boundary
    int scale_out = 0;
    float in_slope = 1.0f;
    RectTab rect, own;
    const void* w = nullptr;        // filter, OIHW
    const void* bias = nullptr;
    float* partial = nullptr;       // [stacks][n_params]
    long long n_params = 0, w_off = 0, b_off = 0;
    int has_bias = 0;
    int K = 3, Cin = 0, Cout = 0;
    int S = 1;                      // stride
    int Hc = 0, Wc = 0;             // map extent at the convolution output (before the pool)
    int Hi = 0, Wi = 0;             // map extent at the convolution input (equal to the output for stride 1)
    int pooled = 0;
    float slope = 0.1f;
    int N = 1, M = 1, batch = 1;
    int bf16 = 0;
    int wgrad_shares = 1, wgrad_shares_thin = 1;   // shares of the matrix-core filter-gradient kernels (from the plan, which sized the scratch)
    int wgrad_shares16 = 1;
    int in_ws = 0, din_ws = 0;      // the activation at the input / the delta at the output lie inside the workspace (which has margins)
};

struct PoolArgs {
    View in, out, mask, din, dout;
    View isign;                     // sign map at the input boundary (backward: see ConvArgs)
    int scale_out = 0;
    float in_slope = 1.0f;
    RectTab rect, own;
    int C = 0, N = 1, M = 1, batch = 1, bf16 = 0;
    int Ho = 0, Wo = 0;             // pooled map extent (floor of half the input extent)
};

// w[i] <- w[i] - lr * sum over stacks of partial[stack][i] (pairwise order of reduce_wgrad), i < count; partial and
// wgrad point at the first parameter of the tensor inside the parameter vector (stride n_params between stacks).
void sgd_update(const float* partial, long long n_params, int stacks, void* w, long long count, float lr, float* wgrad,
                int bf16, hipStream_t s);

// dst = dy * (activation > 0 ? 1 : slope) over a whole map [batch][C][HW]; sign = packed signs of that boundary.
void scale_dy(const void* dy, const uint32_t* sign, void* dst, int batch, int C, long long HW, float slope, int bf16, hipStream_t s);

// Kernel argument block of the matrix-core convolution (forward and delta back-propagation).
struct MfmaConvArgs {
    View in, out, mask, din, dout;
    RectTab rect;                                   // output rectangle each stack computes
    RectTab own;                                    // forward: owned part of it (decision codes are written there)
    int ix0[kTabGrid], ix1[kTabGrid], iy0[kTabGrid], iy1[kTabGrid];   // extent of the input view per tile column / row
    const float* wt;                                // relaid filter [tap][reduction channel][output channel]
    const void* bias;                               // element type of the maps
    int C, Mtot;                                    // reduction channels, output channels
    int Hc, Wc;                                     // map extent at the convolution
    int TC, tiles_x, tiles_r;                       // column block (when tiles_x > 1), column / row-run tile counts
    int mblocks, stacks, xcd_groups;                // output-channel blocks; stacks; 1: workgroups in XCD order (the grid is 1-D, see xcd_order)
    int cap;                                        // pixels (pool windows) per tile
    int flat;                                       // 1: tiles are runs of cap pixels of the rectangle's pixel list, not runs of whole rows
    int cs;                                         // LDS channel stride of the patch = largest patch of any stack
    float slope;
    int M, batch;
    View osign;                                     // forward: sign map of the output boundary
    View isign;                                     // backward: sign map of the boundary the deltas are written to
    int scale_out;                                  // ... whose activation derivative (1 or in_slope) the epilogue applies
    float in_slope;
};

bool mfma_conv_eligible(const ConvArgs& a, bool backward);
// packed16: relay the filter for the bfloat matrix-core path (what mfma_conv_packs_bf16 says for the layer)
bool mfma_conv_packs_bf16(const ConvArgs& a);
void prep_filter(const void* w, int bf16, int packed16, float* wt_fwd, float* wt_bwd, int Cout, int Cin, int K, hipStream_t s);
int mfma_conv_fwd(const ConvArgs& c, const RectTab& inrect, const float* wt, hipStream_t s);       // non-zero: does not fit
int mfma_conv_bwd_data(const ConvArgs& c, const RectTab& inrect, const float* wt, hipStream_t s);
// delta through a 3x3 stride-2 convolution by parity classes (ftp_delta_s2.hip); non-zero: does not fit
int delta_s2_mfma(const ConvArgs& c, const RectTab& inrect, const float* wt, hipStream_t s);

// Kernel argument block of the matrix-core filter gradient.
struct MfmaWgradArgs {
    View in, din, mask;
    RectTab own;                                    // owned rectangle at the convolution output (before the pool)
    float* partial;                                 // [stacks][n_params]
    float* scratch;                                 // [stacks][splits][Cout*Cin*K*K] when splits > 1
    long long n_params, w_off;
    int Cin, Cout, Hc, Wc;
    int splits;                                     // batch shares per stack
    int gx, stacks;                                 // blocks per (stack, share); stacks (the grid is 1-D, see xcd_order)
    int PK;                                         // pixels staged per step
    int zs = 0, stage_words = 0;                    // streamed thin-layer kernel: dwords between the dZ rows of two channels; dwords of a stage
    float slope;
    int M, batch;
};

bool mfma_wgrad_eligible(const ConvArgs& a);
// bfloat 3x3 stride-1 filter gradient with packed staging (ftp_wgrad16.hip)
bool wgrad16_eligible(const ConvArgs& a);
void wgrad16(const ConvArgs& c, float* scratch, hipStream_t s);
void mfma_wgrad(const ConvArgs& c, float* scratch, hipStream_t s);
// The three matrix-core filter-gradient kernels leave `shares` > 1 partial results per stack in the scratch area;
// this sums them into the per-stack gradient vectors (a launch, and a timing record, of its own).
void wgrad_share_sum(const ConvArgs& c, const float* scratch, int shares, hipStream_t s);

bool thin_conv_fwd_eligible(const ConvArgs& a);
void thin_conv_fwd(const ConvArgs& a, hipStream_t s);
// ... with a 5x5 / 7x7 filter or stride 2 (no fused pool)
bool thin_conv_fwd_gen_eligible(const ConvArgs& a);
void thin_conv_fwd_gen(const ConvArgs& a, hipStream_t s);
bool thin_bwd_data_strided_eligible(const ConvArgs& a);
void thin_conv_bwd_data_strided(const ConvArgs& a, const RectTab& ext, hipStream_t s);   // ext: extent of the delta view per stack
bool thin_bwd_data_eligible(const ConvArgs& a);
void thin_conv_bwd_data(const ConvArgs& a, hipStream_t s);
bool thin_wgrad_eligible(const ConvArgs& c);
void thin_wgrad(const ConvArgs& c, float* scratch, hipStream_t s);

void direct_conv_fwd(const ConvArgs& a, hipStream_t s);
void direct_conv_bwd_data(const ConvArgs& a, hipStream_t s);
void direct_wgrad(const ConvArgs& a, hipStream_t s);
void pool_fwd(const PoolArgs& a, hipStream_t s);
void pool_bwd(const PoolArgs& a, hipStream_t s);
void reduce_wgrad(const float* partial, float* wgrad, long long n_params, int stacks, hipStream_t s);

}  // namespace ftp
