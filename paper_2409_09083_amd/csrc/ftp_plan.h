// Internal plan structures of libftp (host side, integers only).
#pragma once
#include <cstdint>
#include <cstddef>
#include <vector>
#include "ftp.h"

struct ftp_plan_s;

namespace ftp {

constexpr int kMaxGrid = 16;   // tiles per dimension

struct Seg { int a, b; };      // inclusive 1-D interval; a rectangle is (x-seg, y-seg)

inline int seg_len(Seg s) { return s.b - s.a + 1; }
inline bool seg_contains(Seg o, Seg i) { return o.a <= i.a && o.b >= i.b; }

// Rectangles are separable: the x interval of tile (ti, tj) depends on tj only, the y interval on ti only.
struct GroupRects {
    int s = 0, e = 0;
    // seg[kind][boundary - s][dim][tile index]; dim 0 = x (columns, M tiles), dim 1 = y (rows, N tiles)
    std::vector<Seg> seg;
    Seg& at(int kind, int l, int dim, int t) { return seg[(((size_t)kind * (e - s + 1) + (l - s)) * 2 + dim) * kMaxGrid + t]; }
    const Seg& at(int kind, int l, int dim, int t) const { return seg[(((size_t)kind * (e - s + 1) + (l - s)) * 2 + dim) * kMaxGrid + t]; }
};

// Where a map (activation, pool winner or delta) of one boundary lives.
enum BufKind : int { BUF_NONE = 0, BUF_X, BUF_Y, BUF_DY, BUF_DX, BUF_WS };

struct BufRef {
    int kind = BUF_NONE;      // user buffer or workspace
    size_t offset = 0;        // byte offset inside the workspace (BUF_WS)
    bool per_stack = false;   // per-stack slots over a held / delta rectangle, else one whole map
    int slot_w = 0, slot_h = 0;   // slot extent (per-stack) or map extent
    int channels = 0;
    int rect_kind = 0;        // rectangle family giving each stack's slot origin (per-stack only)
    size_t bytes = 0;
};

enum UnitKind : int { UNIT_CONV = 0, UNIT_POOL = 1 };

// One kernel-level step: a convolution with its leaky ReLU and, if a pool follows inside the same
// group, that pool evaluated in the epilogue; or a pool on its own.
struct Unit {
    int kind = UNIT_CONV;
    int group = 0;
    int layer = 0;            // primitive layer of the convolution (or of the lone pool)
    bool pooled = false;
    int bi = 0, bo = 0;       // input / output boundary
    BufRef in_act, out_act, out_mask;         // forward (out_mask: decision codes at the output boundary)
    BufRef in_delta, out_delta;               // backward (in_delta lives at bo, out_delta at bi)
    BufRef out_sign, in_sign;                 // packed activation signs at bo (written forward) and at bi (read backward)
    bool scale_out_delta = false;             // the delta written at bi is multiplied by the activation derivative there
    float in_slope = 1.0f;                    // leaky slope of the convolution whose output is boundary bi
    size_t param_offset = 0;                  // first filter element in the parameter vector
    size_t bias_offset = 0;
    size_t wt_fwd_offset = 0, wt_bwd_offset = 0;   // relaid filter copies in the workspace (bytes)
    int wgrad_shares = 1, wgrad_shares_thin = 1;   // shares of the two matrix-core filter-gradient kernels (the scratch is sized for them)
    int wgrad_shares16 = 1;                        // ... and of the bfloat 3x3 kernel
};

struct Plan {
    std::vector<ftp_layer> layers;
    int n_layers = 0, batch = 0, N = 0, M = 0;
    ftp_dtype dtype = FTP_F32;
    size_t esize = 4;
    std::vector<int> C, H, W;                 // per boundary
    std::vector<GroupRects> groups;
    std::vector<int> group_of_layer;
    std::vector<Unit> units;
    std::vector<BufRef> act, mask, delta;     // home of each boundary's activation / decision codes / delta
    std::vector<BufRef> sign;                 // packed activation signs (outputs of convolution units), 32 channels a word
    std::vector<int> home_group;              // group whose rectangles address a per-stack boundary
    // Deltas are kept as dLoss/dZ: where boundary b is the output of a convolution unit (act_slope[b] >= 0), the
    // delta map of b holds dLoss/dY_b times the leaky-ReLU derivative (1 or slope, from the sign map of b);
    // -1 marks boundaries without an activation (the input, outputs of stand-alone pools).
    std::vector<float> act_slope;
    BufRef dy_scaled;                         // whole map at boundary L: the caller's dy times the derivative (if any)
    size_t workspace_bytes = 0, n_params = 0;
    size_t wgrad_scratch_offset = 0;          // batch shares of one layer's partial gradients (bytes)
    size_t split[4] = {0, 0, 0, 0};
    double useful_macs = 0, executed_macs = 0, halo_bytes[2] = {0, 0};
};

#if defined(__HIPCC__)
#define FTP_HD __host__ __device__
#else
#define FTP_HD
#endif

// How the matrix-core filter-gradient kernel cuts one stack's owned rectangle (rw x rh, batch images) into chunks
// of at most 64 pixels (rows padded to an even length) and 192 patch positions: column blocks of TC, row blocks
// of TR, and, where a whole rectangle is smaller than a chunk, TI images at once.  Used by the kernel and by the
// host (share count), so both see the same numbers.
// (Patch positions: a 1x1 filter reads exactly the chunk's 64 pixels; 192 for 3x3 filters, 256 for 5x5 and 7x7.
// The smaller the patch, the more workgroups share a CU's LDS.)
FTP_HD constexpr int wgrad_xpos(int P, int S = 1) { return S == 2 ? (P == 0 ? 256 : 384) : P == 0 ? 64 : P == 1 ? 192 : 256; }
struct WgradChunks { int col_blocks, TC, TCp, PW, TR, row_blocks, TI, img_blocks, total; };
// S = 2: a stride-2 convolution run over its owned *output* pixels (K = 1, 3): pixel (r, c) of a chunk reads the patch
// at (2 r + ky, 2 c + kx), so the patch of a chunk is about four times the chunk.
FTP_HD inline WgradChunks wgrad_chunks(int rw, int rh, int batch, int P, int S = 1)
{
    const int ZPOS = 64, XPOS = wgrad_xpos(P, S);
    int MAXC = ((XPOS / (S + 2 * P) - 2 * P) / S) & ~1;      // widest column block: one row of pixels and its halo rows fit XPOS
    if (MAXC > 64 - 2 * P) MAXC = 64 - 2 * P;
    WgradChunks c;
    c.col_blocks = (rw + MAXC - 1) / MAXC;
    c.TC = (rw + c.col_blocks - 1) / c.col_blocks;
    c.TCp = (c.TC + 1) & ~1; c.PW = S * c.TCp + 2 * P;
    c.TR = ZPOS / c.TCp; if (c.TR > rh) c.TR = rh;
    while (c.TR > 1 && (S * c.TR + 2 * P) * c.PW > XPOS) --c.TR;
    c.row_blocks = (rh + c.TR - 1) / c.TR;
    c.TI = 1;
    if (c.TR == rh && c.col_blocks == 1) {
        c.TI = ZPOS / (c.TCp * rh);
        const int by_patch = XPOS / ((S * rh + 2 * P) * c.PW);
        if (c.TI > by_patch) c.TI = by_patch;
        if (c.TI < 1) c.TI = 1;
    }
    c.img_blocks = (batch + c.TI - 1) / c.TI;
    c.total = c.img_blocks * c.row_blocks * c.col_blocks;
    return c;
}

// Number of shares the matrix-core filter-gradient kernel splits one stack's chunk list into (contiguous ranges,
// summed afterwards in share order).  A workgroup handles one 64 x 64 block of (co, ci) of one stack and one share;
// two workgroups share a CU's matrix cores, so a launch takes ceil(workgroups / 512) rounds of 2 x ceil(chunks /
// shares) chunk times (1x1 filters: four smaller workgroups per CU, bound by staging rather than by the matrix
// cores, hence 1024 slots at the same time per round).  The count that minimises that plus the cost of writing and re-reading the shares is taken.
// chunks = chunk count of the largest stack.
inline int wgrad_shares(int cout, int cin, int k, int stacks, int chunks)
{
    const double blocks = (double)((cout + 63) / 64) * ((cin + 63) / 64) * stacks;
    const double unit_us = 64.0 * k * k * 32.0 / 2400.0 / 0.7;                          // one chunk of one block
    const double share_us = (double)stacks * cout * cin * k * k * 8.0 / 3.0e6;          // one more share: write + read
    const double slots = k == 1 ? 1024.0 : 512.0;                                       // 1x1: four workgroups per CU
    const int smax = chunks < 256 ? chunks : 256;
    int best = 1; double best_t = 0;
    for (int s = 1; s <= smax; ++s) {
        const double rounds = (double)(long long)((blocks * s + slots - 1) / slots);
        const double t = rounds * 2.0 * ((chunks + s - 1) / s) * unit_us + (s > 1 ? s * share_us : 0.0);
        if (s == 1 || t < best_t) { best = s; best_t = t; }
    }
    return best;
}

// Chunks of the bfloat 3x3 filter-gradient kernel (ftp_wgrad16.hip).  The reduction runs over the elements of a patch
// row of the input map, in groups of 8 that start on a 16-byte boundary of the patch; the patch starts `xs` elements
// (0 or 1) before column x0 - 1, where the dword grid of the map falls.  A row of TC pixels reads TC + 2 + xs
// elements: G = ceil((TC + 2 + xs) / 8) groups, PWp = 8 G elements per patch row.  16 groups to a chunk: RB rows of
// one image, or, where a whole rectangle has fewer groups, TI whole images.  The patch of a chunk (rows + 2 halo rows
// per image) has to fit the LDS row of a channel: an odd multiple of 16 bytes (lanes of consecutive channels then read
// 16 bytes each without bank conflicts), twice as long where a workgroup holds 32 input channels only.
constexpr int kW16Groups = 16;
FTP_HD constexpr int w16_row_bytes(int waves_ci) { return waves_ci == 1 ? 944 : 464; }
FTP_HD constexpr int w16_patch_elems(int waves_ci) { return w16_row_bytes(waves_ci) / 2; }
FTP_HD constexpr int w16_waves_ci(int cin) { return cin > 32 ? 2 : 1; }
struct Wgrad16Chunks { int col_blocks, TC, G, PWp, RB, TI, row_blocks, img_blocks, total; };
FTP_HD inline Wgrad16Chunks wgrad16_chunks(int rw, int rh, int batch, int patch_elems, int xs)
{
    Wgrad16Chunks c;
    c.col_blocks = (rw + 63) / 64;
    c.TC = c.col_blocks == 1 ? rw : (((rw + c.col_blocks - 1) / c.col_blocks + 7) & ~7);   // (blocks start at even columns)
    c.col_blocks = (rw + c.TC - 1) / c.TC;
    c.G = (c.TC + 2 + xs + 7) / 8;
    c.PWp = 8 * c.G;
    c.RB = kW16Groups / c.G; if (c.RB > rh) c.RB = rh;
    while (c.RB > 1 && (c.RB + 2) * c.PWp > patch_elems) --c.RB;
    c.TI = 1;
    if (c.RB == rh && c.col_blocks == 1) {
        c.TI = kW16Groups / (c.G * rh);
        const int by_patch = patch_elems / ((rh + 2) * c.PWp);
        if (c.TI > by_patch) c.TI = by_patch;
        if (c.TI > batch) c.TI = batch;
        if (c.TI < 1) c.TI = 1;
    }
    c.row_blocks = (rh + c.RB - 1) / c.RB;
    c.img_blocks = (batch + c.TI - 1) / c.TI;
    c.total = c.img_blocks * c.row_blocks * c.col_blocks;
    return c;
}
// Shares of one stack's chunk list for that kernel: blocks x shares should fill whole rounds of 512 workgroup slots
// (two workgroups per CU) while a share keeps at least a few chunks; one more share costs a write and a read of the
// layer's partial gradients.
inline int wgrad16_shares(int cout, int cin, int stacks, int chunks)
{
    const double blocks = (double)((cout + 63) / 64) * ((cin + 63) / 64) * stacks;
    const double unit_us = 1.6;                                                        // one chunk of one block
    const double share_us = (double)stacks * cout * cin * 9 * 8.0 / 3.0e6;
    const int smax = chunks / 2 < 64 ? (chunks / 2 < 1 ? 1 : chunks / 2) : 64;
    int best = 1; double best_t = 0;
    for (int s = 1; s <= smax; ++s) {
        const double rounds = (double)(long long)((blocks * s + 511.0) / 512.0);
        const double t = rounds * 2.0 * ((chunks + s - 1) / s) * unit_us + (s > 1 ? s * share_us : 0.0);
        if (s == 1 || t < best_t) { best = s; best_t = t; }
    }
    return best;
}

// The kernel for layers with very few input channels stages PK pixels per chunk: TI images x TR rows of the owned
// rectangle (rows padded to even; behind a pool TR is even so that a chunk holds whole windows).
FTP_HD inline int thin_wgrad_pk(int widest_padded_row, bool pooled)
{
    const int need = widest_padded_row * (pooled ? 2 : 1);
    return need > 256 ? need : 256;
}
struct ThinChunks { int TCp, TR, TI, row_blocks, img_blocks, total; };
FTP_HD inline ThinChunks thin_wgrad_chunks(int rw, int rh, int batch, int PK, bool pooled)
{
    ThinChunks c;
    c.TCp = (rw + 1) & ~1;
    c.TR = PK / c.TCp; if (c.TR < 1) c.TR = 1; if (c.TR > rh) c.TR = rh;
    if (pooled && c.TR > 1) c.TR &= ~1;
    c.TI = 1;
    if (c.TR == rh) { c.TI = PK / (c.TCp * rh); if (c.TI < 1) c.TI = 1; }
    c.row_blocks = (rh + c.TR - 1) / c.TR;
    c.img_blocks = (batch + c.TI - 1) / c.TI;
    c.total = c.img_blocks * c.row_blocks;
    return c;
}
// The streamed form of that kernel keeps two chunks in LDS (dZ as [32 channels][zs positions], at the pooled resolution
// behind a pool, where the winner codes follow in the same layout; then the patch), one dword a position.  Its chunks: a
// column block of at most 128 pixels (the rectangle's width in equal, even blocks) x as many rows as 128 pixels - behind a
// pool 64 windows - allow, x several images where one image's rectangle is smaller than that.  cb_max: widest column block
// (128, or 64 / 32 where the patch of wider blocks - large strided filters - would not fit LDS).
FTP_HD constexpr int kThinZPass(bool pooled) { return pooled ? 1 : 2; }      // dZ positions of a chunk, in blocks of 64
struct ThinStreamChunks { int TC, col_blocks, TR, row_blocks, TI, img_blocks, total; };
FTP_HD inline ThinStreamChunks thin_stream_chunks(int rw, int rh, int batch, bool pooled, int cb_max)
{
    ThinStreamChunks c;
    const int rwp = (rw + 1) & ~1;
    c.col_blocks = (rwp + cb_max - 1) / cb_max;
    c.TC = (((rwp + c.col_blocks - 1) / c.col_blocks) + 1) & ~1;
    const int room = pooled ? 256 : 128;               // pixels of a chunk
    c.TR = room / c.TC; if (c.TR < 1) c.TR = 1;
    if (pooled) { c.TR &= ~1; if (c.TR < 2) c.TR = 2; }
    if (c.TR > rh) c.TR = rh;
    c.TI = 1;
    if (c.TR == rh && c.col_blocks == 1) { c.TI = room / (c.TC * rh); if (c.TI < 1) c.TI = 1; }
    c.row_blocks = (rh + c.TR - 1) / c.TR;
    c.img_blocks = (batch + c.TI - 1) / c.TI;
    c.total = c.img_blocks * c.row_blocks * c.col_blocks;
    return c;
}
struct ThinStream { int cb_max, zs, stage_words, wgs_per_cu, max_chunks, max_ti; size_t lds; bool fits; };
inline ThinStream thin_stream_geom(const int* rws, const int* rhs, int N, int M, int batch, int cin, int K, int S, bool pooled)
{
    ThinStream g;
    const int P = K / 2;
    for (g.cb_max = 128; ; g.cb_max /= 2) {
        int nzp = 1, xmax = 1;
        g.max_chunks = 1; g.max_ti = 1;
        for (int i = 0; i < N; ++i)
            for (int j = 0; j < M; ++j) {
                const ThinStreamChunks tc = thin_stream_chunks(rws[j], rhs[i], batch, pooled, g.cb_max);
                const int z = pooled ? tc.TI * (tc.TR >> 1) * (tc.TC >> 1) : tc.TI * tc.TR * tc.TC;
                const int x = cin * tc.TI * (S * tc.TR + 2 * P) * (S * tc.TC + 2 * P);
                if (z > nzp) nzp = z;
                if (x > xmax) xmax = x;
                if (tc.total > g.max_chunks) g.max_chunks = tc.total;
                if (tc.TI > g.max_ti) g.max_ti = tc.TI;
            }
        g.zs = ((nzp + 63) & ~63) + 2;
        g.stage_words = 32 * g.zs * (pooled ? 2 : 1) + xmax + 4;
        size_t words = 2 * (size_t)g.stage_words;
        if (words < 3 * 16 * 64) words = 3 * 16 * 64;                          // final sum of the wavefronts
        g.lds = words * sizeof(float);
        g.fits = nzp <= 64 * kThinZPass(pooled) && g.lds <= 64 * 1024;
        break;                                         // (narrower blocks for patches that do not fit were measured: slower than the
                                                       // register-staged kernel, which takes those layers)
    }
    const int per_cu = (int)((160 * 1024) / g.lds);
    g.wgs_per_cu = per_cu < 1 ? 1 : per_cu > 4 ? 4 : per_cu;
    return g;
}
// Shares of its chunk list: blocks of 32 output channels x stacks x shares should come close to `slots` workgroups, the
// number that runs at a time (1024: four to a CU), without exceeding it - a few workgroups over would start a second
// round as long as the first (36 stacks x 29 shares = 1044 took nearly twice as long as 36 x 28).
inline int wgrad_shares_thin(int cout, int stacks, int chunks, int slots = 1024)
{
    const int blocks = ((cout + 31) / 32) * stacks;
    int shares = slots / blocks;
    if (shares > chunks) shares = chunks;
    if (shares > 256) shares = 256;
    return shares < 1 ? 1 : shares;
}

// The parity-class delta kernel of stride-2 layers (ftp_delta_s2.hip) cuts the cells (2 x 2 input pixels) that cover a
// stack's rectangle into blocks of 32: 32 / NC rows x NC columns, listed over image, row group, column group (fastest).
constexpr int kS2XCS = 67;                          // dwords between two channels of a block's patch (at most 2 x 33 positions)
struct S2Blocks { int gc, gr, total; };
FTP_HD inline S2Blocks s2_blocks(int x0, int x1, int y0, int y1, int batch, int NC)
{
    S2Blocks b;
    const int cw = (x1 >> 1) - (x0 >> 1) + 1, ch = (y1 >> 1) - (y0 >> 1) + 1, NR = 32 / NC;
    b.gc = (cw + NC - 1) / NC; b.gr = (ch + NR - 1) / NR;
    b.total = batch * b.gr * b.gc;
    return b;
}

int build_plan(const ftp_layer* layers, int n_layers, int batch, int in_c, int in_h, int in_w,
               int N, int M, const int32_t* group_ends, int n_groups, ftp_dtype dtype, ftp_plan_s** out);

}  // namespace ftp

// Optional per-kernel timing (benchmarks): HIP events around every launch of the three passes.
// Host objects only; created on first use and owned by the plan.
namespace ftp {
struct Profiler {
    typedef void* event_t;              // hipEvent_t, kept opaque so that this header needs no HIP
    struct Rec { int pass, layer; event_t a, b; const char* kernel; };
    struct Agg { int pass, layer, launches; double ms; const char* kernel; };
    bool on = false;
    std::vector<Rec> pending;
    std::vector<event_t> free_list;
    std::vector<Agg> agg;
    event_t get();
    void recycle();
    ~Profiler();
};
}  // namespace ftp

// Second stream of the backward pass (optional): the filter gradient of a unit runs beside the delta
// back-propagation of the same unit.  Host objects only, created on first use and owned by the plan.
namespace ftp {
struct Overlap {
    bool on = false;
    void* aux = nullptr;                // hipStream_t (default priority)
    std::vector<void*> events;          // hipEvent_t, reused call after call
    ~Overlap();
};
}  // namespace ftp

struct ftp_plan_s {
    ftp::Plan p;
    mutable ftp::Profiler prof;
    mutable ftp::Overlap overlap;
};
