// C ABI of libftp: plan queries and the three device passes (forward, backward, gradient sum).
#include "ftp.h"
#include "ftp_plan.h"
#include "ftp_launch.h"

#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <mutex>

using namespace ftp;

// Workspace of ftp_forward_static.  On the host this name is only a handle for hipGetSymbolAddress: the device
// address, one per GPU, is looked up once per device and kept in g_static_ws.
static __device__ __align__(256) unsigned char scratch[FTP_STATIC_WORKSPACE_BYTES];

namespace {

constexpr int kMaxDevices = 64;
void* g_static_ws[kMaxDevices] = {};
std::mutex g_static_ws_lock;

thread_local int g_last_hip = 0;

struct UserBufs {
    const void* x = nullptr; void* y = nullptr; const void* dy = nullptr; void* dx = nullptr; void* ws = nullptr;
};

View make_view(const Plan& p, const BufRef& b, int group, int boundary, const UserBufs& ub)
{
    View v;
    std::memset(&v, 0, sizeof(v));
    switch (b.kind) {
        case BUF_X: v.p = const_cast<void*>(ub.x); break;
        case BUF_Y: v.p = ub.y; break;
        case BUF_DY: v.p = const_cast<void*>(ub.dy); break;
        case BUF_DX: v.p = ub.dx; break;
        case BUF_WS: v.p = (char*)ub.ws + b.offset; break;
        default: v.p = nullptr; break;
    }
    v.pitch = b.slot_w;
    v.cs = (long long)b.slot_w * b.slot_h;
    v.ns = v.cs * b.channels;
    if (b.per_stack) {
        v.ss = v.ns * p.batch;
        const GroupRects& g = p.groups[group];
        for (int t = 0; t < p.M; ++t) v.x0[t] = g.at(b.rect_kind, boundary, 0, t).a;
        for (int t = 0; t < p.N; ++t) v.y0[t] = g.at(b.rect_kind, boundary, 1, t).a;
    }
    return v;
}

RectTab make_rect(const Plan& p, int group, int kind, int boundary)
{
    RectTab r;
    std::memset(&r, 0, sizeof(r));
    const GroupRects& g = p.groups[group];
    for (int t = 0; t < p.M; ++t) { r.x0[t] = g.at(kind, boundary, 0, t).a; r.x1[t] = g.at(kind, boundary, 0, t).b; }
    for (int t = 0; t < p.N; ++t) { r.y0[t] = g.at(kind, boundary, 1, t).a; r.y1[t] = g.at(kind, boundary, 1, t).b; }
    return r;
}

// Extent of a view per tile column / row: the stack's rectangle for per-stack slots, else the whole map.
RectTab view_extent(const Plan& p, const BufRef& b, int group, int boundary)
{
    if (b.per_stack) return make_rect(p, group, b.rect_kind, boundary);
    RectTab r;
    std::memset(&r, 0, sizeof(r));
    for (int t = 0; t < kTabGrid; ++t) { r.x1[t] = b.slot_w - 1; r.y1[t] = b.slot_h - 1; }
    return r;
}

// FTP_KERNELS=direct keeps every layer on the direct kernels (debugging aid).
bool use_mfma()
{
    static const bool on = [] { const char* e = std::getenv("FTP_KERNELS"); return !(e && std::strcmp(e, "direct") == 0); }();
    return on;
}

// The thin-layer kernels and the matrix-core filter gradient are written for the geometry of the paper's networks:
// stride 1, K <= 3 and, behind the convolution, a pool over an even map (the matrix-core convolution states its own
// limits).  Everything else runs on the general direct kernels.
bool plain_geometry(const ConvArgs& a)
{
    return a.S == 1 && a.K <= 3 && !(a.pooled && ((a.Hc | a.Wc) & 1));
}

ConvArgs conv_args(const Plan& p, const Unit& u, const UserBufs& ub, const void* const* weights, const void* const* biases)
{
    ConvArgs a;
    const ftp_layer& ly = p.layers[u.layer];
    a.in = make_view(p, u.in_act, u.group, u.bi, ub);
    a.out = make_view(p, u.out_act, u.group, u.bo, ub);
    a.mask = make_view(p, u.out_mask, u.group, u.bo, ub);
    a.din = make_view(p, u.in_delta, u.group, u.bo, ub);
    a.dout = make_view(p, u.out_delta, u.group, u.bi, ub);
    a.osign = make_view(p, u.out_sign, u.group, u.bo, ub);
    a.isign = make_view(p, u.in_sign, u.group, u.bi, ub);
    a.scale_out = u.scale_out_delta ? 1 : 0;
    a.in_slope = u.in_slope;
    a.w = weights[u.layer];
    a.bias = (biases && ly.has_bias) ? biases[u.layer] : nullptr;
    a.n_params = (long long)p.n_params; a.w_off = (long long)u.param_offset; a.b_off = (long long)u.bias_offset;
    a.has_bias = ly.has_bias;
    a.K = ly.k; a.Cin = ly.cin; a.Cout = ly.cout;
    a.S = ly.stride;
    a.Hi = p.H[u.layer]; a.Wi = p.W[u.layer];
    a.Hc = p.H[u.layer + 1]; a.Wc = p.W[u.layer + 1];
    a.pooled = u.pooled ? 1 : 0;
    a.slope = ly.leaky_slope;
    a.N = p.N; a.M = p.M; a.batch = p.batch;
    a.bf16 = p.dtype == FTP_BF16;
    a.wgrad_shares = u.wgrad_shares; a.wgrad_shares_thin = u.wgrad_shares_thin; a.wgrad_shares16 = u.wgrad_shares16;
    a.in_ws = u.in_act.kind == BUF_WS ? 1 : 0; a.din_ws = u.in_delta.kind == BUF_WS ? 1 : 0;
    return a;
}

PoolArgs pool_args(const Plan& p, const Unit& u, const UserBufs& ub)
{
    PoolArgs a;
    a.in = make_view(p, u.in_act, u.group, u.bi, ub);
    a.out = make_view(p, u.out_act, u.group, u.bo, ub);
    a.mask = make_view(p, u.out_mask, u.group, u.bo, ub);
    a.din = make_view(p, u.in_delta, u.group, u.bo, ub);
    a.dout = make_view(p, u.out_delta, u.group, u.bi, ub);
    a.isign = make_view(p, u.in_sign, u.group, u.bi, ub);
    a.scale_out = u.scale_out_delta ? 1 : 0;
    a.in_slope = u.in_slope;
    a.C = p.C[u.bi]; a.N = p.N; a.M = p.M; a.batch = p.batch;
    a.bf16 = p.dtype == FTP_BF16;
    a.Ho = p.H[u.bo]; a.Wo = p.W[u.bo];
    return a;
}

template <class Fn>
int timed(const ftp_plan_s* plan, int pass, int layer, hipStream_t s, Fn&& launch);

int check_hip()
{
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) { g_last_hip = (int)e; return FTP_EHIP; }
    return FTP_OK;
}

// Runs one kernel launch; while profiling is on, brackets it with two HIP events on the same stream.
template <class Fn>
int timed(const ftp_plan_s* plan, int pass, int layer, hipStream_t s, Fn&& launch)
{
    Profiler& pr = plan->prof;
    if (!pr.on) { launch(); return check_hip(); }
    hipEvent_t a = (hipEvent_t)pr.get(), b = (hipEvent_t)pr.get();
    if (!a || !b) { g_last_hip = (int)hipGetLastError(); return FTP_EHIP; }
    (void)hipEventRecord(a, s);
    launch();
    (void)hipEventRecord(b, s);
    pr.pending.push_back(Profiler::Rec{pass, layer, a, b, g_kernel_label});
    return check_hip();
}

int check_weights(const Plan& p, const void* const* weights, const void* const* biases)
{
    if (!weights) return FTP_EINVAL;
    for (int l = 0; l < p.n_layers; ++l) {
        if (p.layers[l].kind != FTP_CONV) continue;
        if (!weights[l]) return FTP_EINVAL;
        if (p.layers[l].has_bias && biases && !biases[l]) return FTP_EINVAL;
    }
    return FTP_OK;
}

// FTP_OVERLAP=1: plans start with the two-stream backward pass switched on (see ftp_set_overlap).
bool overlap_default()
{
    const char* e = std::getenv("FTP_OVERLAP");
    return e && std::strcmp(e, "1") == 0;
}

bool any_bias(const Plan& p)
{
    for (const ftp_layer& ly : p.layers) if (ly.kind == FTP_CONV && ly.has_bias) return true;
    return false;
}

}  // namespace

extern "C" {

int ftp_plan(const ftp_layer* layers, int32_t n_layers, int32_t batch, int32_t in_c, int32_t in_h, int32_t in_w,
             int32_t grid_rows, int32_t grid_cols, const int32_t* group_ends, int32_t n_groups,
             ftp_dtype dtype, ftp_plan_t** out_plan)
{
    const int rc = build_plan(layers, n_layers, batch, in_c, in_h, in_w, grid_rows, grid_cols, group_ends, n_groups, dtype, out_plan);
    if (rc == FTP_OK && overlap_default()) (void)ftp_set_overlap(*out_plan, 1);
    return rc;
}

int ftp_set_overlap(ftp_plan_t* plan, int32_t enable)
{
    if (!plan) return FTP_EINVAL;
    Overlap& ov = plan->overlap;
    ov.on = enable != 0;
    if (ov.on && !ov.aux) {
        // The second stream and the events of one backward pass are created here, so that ftp_backward creates no
        // object (it may run under stream capture).  Without a usable device (a host that only plans) this is put
        // off to the first ftp_backward.
        hipStream_t st = nullptr;
        if (hipStreamCreateWithFlags(&st, hipStreamNonBlocking) == hipSuccess) {
            ov.aux = st;
            const size_t want = 3 * plan->p.units.size() + 4;
            while (ov.events.size() < want) {
                hipEvent_t e = nullptr;
                if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) break;
                ov.events.push_back(e);
            }
        }
        (void)hipGetLastError();
    }
    return FTP_OK;
}

void ftp_plan_destroy(ftp_plan_t* plan) { delete plan; }

int ftp_plan_rect(const ftp_plan_t* plan, int32_t group, int32_t boundary, int32_t ti, int32_t tj,
                  ftp_rect_kind kind, int32_t out[4])
{
    if (!plan || !out) return FTP_EINVAL;
    const Plan& p = plan->p;
    if (group < 0 || group >= (int)p.groups.size() || ti < 0 || ti >= p.N || tj < 0 || tj >= p.M) return FTP_EINVAL;
    if ((int)kind < 0 || (int)kind > FTP_RECT_BWD) return FTP_EINVAL;
    const GroupRects& g = p.groups[group];
    if (boundary < g.s || boundary > g.e) return FTP_EINVAL;
    const Seg sx = g.at(kind, boundary, 0, tj), sy = g.at(kind, boundary, 1, ti);
    out[0] = sx.a; out[1] = sy.a; out[2] = sx.b; out[3] = sy.b;
    return FTP_OK;
}

int ftp_plan_map_shape(const ftp_plan_t* plan, int32_t boundary, int32_t out_chw[3])
{
    if (!plan || !out_chw) return FTP_EINVAL;
    const Plan& p = plan->p;
    if (boundary < 0 || boundary > p.n_layers) return FTP_EINVAL;
    out_chw[0] = p.C[boundary]; out_chw[1] = p.H[boundary]; out_chw[2] = p.W[boundary];
    return FTP_OK;
}

int ftp_plan_sizes(const ftp_plan_t* plan, size_t* workspace_bytes, size_t* wgrad_partial_bytes, size_t* n_params,
                   size_t per_stack_split[4])
{
    if (!plan) return FTP_EINVAL;
    const Plan& p = plan->p;
    if (workspace_bytes) *workspace_bytes = p.workspace_bytes;
    if (wgrad_partial_bytes) *wgrad_partial_bytes = (size_t)p.N * p.M * p.n_params * sizeof(float);
    if (n_params) *n_params = p.n_params;
    if (per_stack_split) for (int i = 0; i < 4; ++i) per_stack_split[i] = p.split[i];
    return FTP_OK;
}

int ftp_plan_work(const ftp_plan_t* plan, double* useful_macs, double* executed_macs, double halo_bytes[2])
{
    if (!plan) return FTP_EINVAL;
    const Plan& p = plan->p;
    if (useful_macs) *useful_macs = p.useful_macs;
    if (executed_macs) *executed_macs = p.executed_macs;
    if (halo_bytes) { halo_bytes[0] = p.halo_bytes[0]; halo_bytes[1] = p.halo_bytes[1]; }
    return FTP_OK;
}

int ftp_plan_buffer(const ftp_plan_t* plan, int32_t boundary, ftp_buf_kind which, int64_t out[8])
{
    if (!plan || !out) return FTP_EINVAL;
    const Plan& p = plan->p;
    if (boundary < 0 || boundary > p.n_layers) return FTP_EINVAL;
    const BufRef* b = nullptr;
    switch (which) {
        case FTP_BUF_ACT: b = &p.act[boundary]; break;
        case FTP_BUF_MASK: b = &p.mask[boundary]; break;
        case FTP_BUF_DELTA: b = &p.delta[boundary]; break;
        case FTP_BUF_SIGN: b = &p.sign[boundary]; break;
        default: return FTP_EINVAL;
    }
    out[0] = b->kind; out[1] = (int64_t)b->offset; out[2] = b->per_stack ? 1 : 0;
    out[3] = b->slot_w; out[4] = b->slot_h; out[5] = b->channels; out[6] = b->rect_kind; out[7] = p.home_group[boundary];
    return FTP_OK;
}

int ftp_forward(const ftp_plan_t* plan, const void* x, const void* const* weights, const void* const* biases,
                void* workspace, void* y, void* stream)
{
    if (!plan || !x || !workspace || !y) return FTP_EINVAL;
    const Plan& p = plan->p;
    int rc = check_weights(p, weights, biases);
    if (rc != FTP_OK) return rc;
    if (any_bias(p) && !biases) return FTP_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    UserBufs ub; ub.x = x; ub.y = y; ub.ws = workspace;
    for (const Unit& u : p.units) {
        if (u.kind == UNIT_CONV) {
            ConvArgs a = conv_args(p, u, ub, weights, biases);
            a.rect = make_rect(p, u.group, FTP_RECT_FWD, u.bo);
            a.own = make_rect(p, u.group, FTP_RECT_OWN, u.bo);
            const bool fast = use_mfma() && plain_geometry(a);
            if (use_mfma() && mfma_conv_eligible(a, false)) {
                float* wt = (float*)((char*)workspace + u.wt_fwd_offset);
                const RectTab ext = view_extent(p, u.in_act, u.group, u.bi);
                rc = timed(plan, FTP_PASS_CONV_FWD, u.layer, s, [&] {
                    prep_filter(a.w, a.bf16, mfma_conv_packs_bf16(a), wt, nullptr, a.Cout, a.Cin, a.K, s);
                    if (mfma_conv_fwd(a, ext, wt, s)) direct_conv_fwd(a, s);
                });
            } else if (fast && thin_conv_fwd_eligible(a)) {
                rc = timed(plan, FTP_PASS_CONV_FWD, u.layer, s, [&] { thin_conv_fwd(a, s); });
            } else if (use_mfma() && thin_conv_fwd_gen_eligible(a)) {
                rc = timed(plan, FTP_PASS_CONV_FWD, u.layer, s, [&] { thin_conv_fwd_gen(a, s); });
            } else {
                rc = timed(plan, FTP_PASS_CONV_FWD, u.layer, s, [&] { direct_conv_fwd(a, s); });
            }
        } else {
            PoolArgs a = pool_args(p, u, ub);
            a.rect = make_rect(p, u.group, FTP_RECT_FWD, u.bo);
            a.own = make_rect(p, u.group, FTP_RECT_OWN, u.bo);
            rc = timed(plan, FTP_PASS_POOL_FWD, u.layer, s, [&] { pool_fwd(a, s); });
        }
        if (rc != FTP_OK) return rc;
    }
    return FTP_OK;
}

int ftp_forward_static(const ftp_plan_t* plan, const void* x, const void* const* weights, const void* const* biases,
                       void* y, void* stream)
{
    if (!plan) return FTP_EINVAL;
    if (plan->p.workspace_bytes > (size_t)FTP_STATIC_WORKSPACE_BYTES) return FTP_ETOOLARGE;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) { g_last_hip = (int)hipGetLastError(); return FTP_EHIP; }
    if (dev < 0 || dev >= kMaxDevices) return FTP_EINVAL;
    void* ws = nullptr;
    {
        std::lock_guard<std::mutex> hold(g_static_ws_lock);
        if (!g_static_ws[dev]) {
            void* p = nullptr;
            const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));       // this device's copy of the array
            if (e != hipSuccess || !p) { g_last_hip = (int)e; (void)hipGetLastError(); return FTP_EHIP; }
            g_static_ws[dev] = p;
        }
        ws = g_static_ws[dev];
    }
    return ftp_forward(plan, x, weights, biases, ws, y, stream);
}

int ftp_backward(const ftp_plan_t* plan, const void* dy, const void* x, const void* const* weights,
                 void* workspace, void* dx, float* wgrad_partials, void* stream)
{
    if (!plan || !dy || !x || !workspace || !dx) return FTP_EINVAL;
    const Plan& p = plan->p;
    if (!wgrad_partials && p.n_params > 0) return FTP_EINVAL;       // (a network of pools only has no parameters)
    int rc = check_weights(p, weights, nullptr);
    if (rc != FTP_OK) return rc;
    hipStream_t s = (hipStream_t)stream;
    UserBufs ub; ub.x = x; ub.dy = dy; ub.dx = dx; ub.ws = workspace;
    const int L = p.n_layers;
    if (p.act_slope[L] >= 0.0f) {
        // deltas are kept as dLoss/dZ: fold the last activation's derivative into a copy of dy
        const uint32_t* sg = (const uint32_t*)((const char*)workspace + p.sign[L].offset);
        void* dst = (char*)workspace + p.dy_scaled.offset;
        rc = timed(plan, FTP_PASS_SCALE_DY, p.units.back().layer, s, [&] {
            scale_dy(dy, sg, dst, p.batch, p.C[L], (long long)p.H[L] * p.W[L], p.act_slope[L], p.dtype == FTP_BF16, s);
        });
        if (rc != FTP_OK) return rc;
    }
    // Optional second stream: the filter gradient of unit i (reads the delta at its output boundary, writes the
    // partial gradients) runs beside the delta back-propagation of unit i (reads the same delta, writes the delta at
    // its input boundary).  The next step on `s` overwrites the ping-pong region the gradient is reading, so it waits
    // for it; the next gradient waits for the step that produces its delta.
    Overlap& ov = plan->overlap;
    const bool overlap = ov.on;
    hipStream_t aux = s;
    size_t next_event = 0;
    auto new_event = [&]() -> hipEvent_t {
        if (next_event == ov.events.size()) {
            hipEvent_t e = nullptr;
            if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) return nullptr;
            ov.events.push_back(e);
        }
        return (hipEvent_t)ov.events[next_event++];
    };
    // makes stream `to` wait for everything enqueued on `from` so far
    auto order = [&](hipStream_t from, hipStream_t to) -> int {
        hipEvent_t e = new_event();
        if (!e || hipEventRecord(e, from) != hipSuccess || hipStreamWaitEvent(to, e, 0) != hipSuccess) { g_last_hip = (int)hipGetLastError(); return FTP_EHIP; }
        return FTP_OK;
    };
    if (overlap) {
        if (!ov.aux) {
            hipStream_t st = nullptr;
            if (hipStreamCreateWithFlags(&st, hipStreamNonBlocking) != hipSuccess) { g_last_hip = (int)hipGetLastError(); return FTP_EHIP; }
            ov.aux = st;
        }
        aux = (hipStream_t)ov.aux;
        if ((rc = order(s, aux)) != FTP_OK) return rc;          // the forward pass, dy scaling, earlier calls
    }
    bool gradient_in_flight = false;
    for (int i = (int)p.units.size() - 1; i >= 0; --i) {
        const Unit& u = p.units[i];
        if (u.kind == UNIT_CONV) {
            ConvArgs a = conv_args(p, u, ub, weights, nullptr);
            a.partial = wgrad_partials;
            a.rect = make_rect(p, u.group, FTP_RECT_OWN, u.layer + 1);
            a.own = make_rect(p, u.group, FTP_RECT_OWN, u.layer);
            float* scratch = (float*)((char*)workspace + p.wgrad_scratch_offset);
            const bool fast = use_mfma() && plain_geometry(a);
            // (the previous gradient is still reading the region this unit's delta step will overwrite; gradients
            // are serial among themselves on `aux`, they share the scratch)
            if (overlap && gradient_in_flight && (rc = order(aux, s)) != FTP_OK) return rc;
            int shares = 1;
            if (use_mfma() && thin_wgrad_eligible(a)) {
                shares = a.wgrad_shares_thin;
                rc = timed(plan, FTP_PASS_WGRAD, u.layer, aux, [&] { thin_wgrad(a, scratch, aux); });
            } else if (use_mfma() && plain_geometry(a) && u.in_act.kind == BUF_WS && u.in_delta.kind == BUF_WS && wgrad16_eligible(a)) {
                // (its wide loads round addresses down and may run a few bytes past a map: only inside the workspace, which has margins)
                shares = a.wgrad_shares16;
                rc = timed(plan, FTP_PASS_WGRAD, u.layer, aux, [&] { wgrad16(a, scratch, aux); });
            } else if (use_mfma() && mfma_wgrad_eligible(a)) {
                shares = a.wgrad_shares;
                rc = timed(plan, FTP_PASS_WGRAD, u.layer, aux, [&] { mfma_wgrad(a, scratch, aux); });
            } else {
                rc = timed(plan, FTP_PASS_WGRAD, u.layer, aux, [&] { direct_wgrad(a, aux); });
            }
            if (rc == FTP_OK && shares > 1)
                rc = timed(plan, FTP_PASS_WGRAD_SUM, u.layer, aux, [&] { wgrad_share_sum(a, scratch, shares, aux); });
            if (rc != FTP_OK) return rc;
            gradient_in_flight = overlap;
            a.rect = make_rect(p, u.group, FTP_RECT_BWD, u.bi);
            if (use_mfma() && mfma_conv_eligible(a, true)) {
                float* wt = (float*)((char*)workspace + u.wt_bwd_offset);
                const RectTab ext = view_extent(p, u.in_delta, u.group, u.bo);
                rc = timed(plan, FTP_PASS_CONV_BWD_DATA, u.layer, s, [&] {
                    prep_filter(a.w, a.bf16, mfma_conv_packs_bf16(a), nullptr, wt, a.Cout, a.Cin, a.K, s);
                    if (mfma_conv_bwd_data(a, ext, wt, s)) direct_conv_bwd_data(a, s);
                });
            } else if (use_mfma() && thin_bwd_data_strided_eligible(a)) {
                const RectTab ext = view_extent(p, u.in_delta, u.group, u.bo);
                rc = timed(plan, FTP_PASS_CONV_BWD_DATA, u.layer, s, [&] { thin_conv_bwd_data_strided(a, ext, s); });
            } else if (fast && thin_bwd_data_eligible(a)) {
                rc = timed(plan, FTP_PASS_CONV_BWD_DATA, u.layer, s, [&] { thin_conv_bwd_data(a, s); });
            } else {
                rc = timed(plan, FTP_PASS_CONV_BWD_DATA, u.layer, s, [&] { direct_conv_bwd_data(a, s); });
            }
        } else {
            PoolArgs a = pool_args(p, u, ub);
            a.rect = make_rect(p, u.group, FTP_RECT_BWD, u.bi);
            if (overlap && gradient_in_flight) { if ((rc = order(aux, s)) != FTP_OK) return rc; gradient_in_flight = false; }
            rc = timed(plan, FTP_PASS_POOL_BWD, u.layer, s, [&] { pool_bwd(a, s); });
        }
        if (rc != FTP_OK) return rc;
        if (overlap && i > 0 && (rc = order(s, aux)) != FTP_OK) return rc;      // the next gradient reads the delta just written
    }
    if (overlap && (rc = order(aux, s)) != FTP_OK) return rc;                   // the caller's stream sees every partial gradient
    return FTP_OK;
}

int ftp_reduce_wgrad(const ftp_plan_t* plan, const float* wgrad_partials, float* wgrad, void* stream)
{
    if (!plan) return FTP_EINVAL;
    const Plan& p = plan->p;
    if (p.n_params == 0) return FTP_OK;                               // (a network of pools only: nothing to sum)
    if (!wgrad_partials || !wgrad) return FTP_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    return timed(plan, FTP_PASS_REDUCE, -1, s, [&] { reduce_wgrad(wgrad_partials, wgrad, (long long)p.n_params, p.N * p.M, s); });
}

int ftp_sgd_step(const ftp_plan_t* plan, const float* wgrad_partials, void* const* weights, void* const* biases,
                 float lr, float* wgrad, void* stream)
{
    if (!plan) return FTP_EINVAL;
    const Plan& p = plan->p;
    if (p.n_params == 0) return FTP_OK;                               // (a network of pools only: nothing to update)
    if (!wgrad_partials || !weights) return FTP_EINVAL;
    int rc = check_weights(p, (const void* const*)weights, (const void* const*)biases);
    if (rc != FTP_OK) return rc;
    if (any_bias(p) && !biases) return FTP_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    const int stacks = p.N * p.M, bf16 = p.dtype == FTP_BF16;
    for (const Unit& u : p.units) {
        if (u.kind != UNIT_CONV) continue;
        const ftp_layer& ly = p.layers[u.layer];
        const long long wcount = (long long)ly.cout * ly.cin * ly.k * ly.k;
        rc = timed(plan, FTP_PASS_UPDATE, u.layer, s, [&] {
            sgd_update(wgrad_partials + u.param_offset, (long long)p.n_params, stacks, weights[u.layer], wcount, lr,
                       wgrad ? wgrad + u.param_offset : nullptr, bf16, s);
            if (ly.has_bias)
                sgd_update(wgrad_partials + u.bias_offset, (long long)p.n_params, stacks, biases[u.layer], ly.cout, lr,
                           wgrad ? wgrad + u.bias_offset : nullptr, bf16, s);
        });
        if (rc != FTP_OK) return rc;
    }
    return FTP_OK;
}

int ftp_profile(ftp_plan_t* plan, int32_t enable)
{
    if (!plan) return FTP_EINVAL;
    Profiler& pr = plan->prof;
    if (enable) { pr.recycle(); pr.agg.clear(); }
    pr.on = enable != 0;
    return FTP_OK;
}

int ftp_profile_read(ftp_plan_t* plan, ftp_kernel_time* out, int32_t capacity, int32_t* count)
{
    if (!plan || !count || (capacity > 0 && !out)) return FTP_EINVAL;
    Profiler& pr = plan->prof;
    const Plan& p = plan->p;
    for (const Profiler::Rec& r : pr.pending) {
        if (hipEventSynchronize((hipEvent_t)r.b) != hipSuccess) { g_last_hip = (int)hipGetLastError(); return FTP_EHIP; }
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, (hipEvent_t)r.a, (hipEvent_t)r.b) != hipSuccess) { g_last_hip = (int)hipGetLastError(); return FTP_EHIP; }
        Profiler::Agg* hit = nullptr;
        for (Profiler::Agg& g : pr.agg) if (g.pass == r.pass && g.layer == r.layer) { hit = &g; break; }
        if (!hit) { pr.agg.push_back(Profiler::Agg{r.pass, r.layer, 0, 0.0, r.kernel}); hit = &pr.agg.back(); }
        hit->launches += 1; hit->ms += ms;
    }
    pr.recycle();
    *count = (int32_t)pr.agg.size();
    const double es = (double)p.esize, B = p.batch, stacks = (double)p.N * p.M;
    for (int i = 0; i < (int)pr.agg.size() && i < capacity; ++i) {
        const Profiler::Agg& g = pr.agg[i];
        ftp_kernel_time t;
        t.pass = g.pass; t.layer = g.layer; t.launches = g.launches; t.reserved = 0; t.total_ms = g.ms;
        t.flops_per_launch = 0; t.bytes_per_launch = 0; t.executed_flops_per_launch = 0;
        std::memset(t.kernel, 0, sizeof(t.kernel));
        if (g.kernel) std::strncpy(t.kernel, g.kernel, sizeof(t.kernel) - 1);
        if (g.pass == FTP_PASS_REDUCE) {
            t.bytes_per_launch = (stacks + 1.0) * (double)p.n_params * 4.0;
            t.flops_per_launch = (stacks - 1.0) * (double)p.n_params;
        } else {
            const ftp_layer& ly = p.layers[g.layer];
            const Unit* u = nullptr;
            for (const Unit& q : p.units) if (q.layer == g.layer) { u = &q; break; }
            const double in_el = B * p.C[u->bi] * p.H[u->bi] * p.W[u->bi];
            const double out_el = B * p.C[u->bo] * p.H[u->bo] * p.W[u->bo];
            const double has_arg = (u->pooled || u->kind == UNIT_POOL) ? 1.0 : 0.0;
            if (g.pass == FTP_PASS_UPDATE) {
                const double wel = (double)ly.cout * ly.cin * ly.k * ly.k + (ly.has_bias ? ly.cout : 0);
                t.flops_per_launch = (stacks + 1.0) * wel;
                t.bytes_per_launch = stacks * wel * 4.0 + 2.0 * wel * es;
            } else if (g.pass == FTP_PASS_WGRAD_SUM) {
                const double wel = (double)ly.cout * ly.cin * ly.k * ly.k;
                const double sh = g.kernel == nullptr ? 1.0 : (double)std::max(std::max(u->wgrad_shares, u->wgrad_shares_thin), u->wgrad_shares16);
                t.flops_per_launch = stacks * wel * (sh - 1.0);
                t.bytes_per_launch = stacks * wel * 4.0 * (sh + 1.0);              // (upper bound: the largest share count of the layer)
            } else if (g.pass == FTP_PASS_SCALE_DY) {
                t.flops_per_launch = out_el;
                t.bytes_per_launch = out_el * (2.0 * es + 1.0);
            } else if (u->kind == UNIT_CONV) {
                const double wel = (double)ly.cout * ly.cin * ly.k * ly.k;
                t.flops_per_launch = 2.0 * wel * B * p.H[g.layer + 1] * p.W[g.layer + 1];
                {
                    // rectangles the stacks evaluate: forward F at the convolution output, delta B at its input
                    const GroupRects& gr = p.groups[u->group];
                    const int kind = g.pass == FTP_PASS_CONV_FWD ? FTP_RECT_FWD : g.pass == FTP_PASS_CONV_BWD_DATA ? FTP_RECT_BWD : FTP_RECT_OWN;
                    const int lb = g.pass == FTP_PASS_CONV_BWD_DATA ? g.layer : g.layer + 1;
                    double sx = 0, sy = 0;
                    for (int t2 = 0; t2 < p.M; ++t2) sx += seg_len(gr.at(kind, lb, 0, t2));
                    for (int t2 = 0; t2 < p.N; ++t2) sy += seg_len(gr.at(kind, lb, 1, t2));
                    // (delta pass of a strided convolution: a pixel of the input rectangle meets 1 / S^2 of the taps)
                    const double per_px = g.pass == FTP_PASS_CONV_BWD_DATA ? 1.0 / ((double)ly.stride * ly.stride) : 1.0;
                    t.executed_flops_per_launch = 2.0 * wel * B * sx * sy * per_px;
                }
                if (g.pass == FTP_PASS_CONV_FWD) t.bytes_per_launch = (in_el + out_el + wel) * es + out_el * has_arg;
                else if (g.pass == FTP_PASS_CONV_BWD_DATA) t.bytes_per_launch = (in_el + 2.0 * out_el + wel) * es + out_el * has_arg;
                else t.bytes_per_launch = (in_el + 2.0 * out_el) * es + out_el * has_arg + stacks * wel * 4.0;
            } else {
                t.bytes_per_launch = (in_el + out_el) * es + out_el;
            }
        }
        out[i] = t;
    }
    return FTP_OK;
}

const char* ftp_strerror(int code)
{
    switch (code) {
        case FTP_OK: return "ok";
        case FTP_EINVAL: return "invalid argument";
        case FTP_EUNSUPPORTED: return "unsupported layer (conv needs stride 1 or 2, K in {1,3,5,7}, pad K/2, slope >= 0; pool needs 2x2 stride 2)";
        case FTP_EGRID: return "tile grid does not fit the maps (empty tile, map too small for its pool, or more than 16 tiles per side)";
        case FTP_EGROUPS: return "group ends must be strictly increasing and end at the number of layers";
        case FTP_ENOMEM: return "host allocation failed";
        case FTP_EHIP: return "HIP call failed";
        case FTP_ECHANNELS: return "channel counts of consecutive layers do not match";
        case FTP_ETOOLARGE: return "the plan's workspace exceeds the fixed array of ftp_forward_static (FTP_STATIC_WORKSPACE_BYTES)";
        default: return "unknown error";
    }
}

int ftp_last_hip_error(void) { return g_last_hip; }

}  // extern "C"

namespace ftp {

thread_local const char* g_kernel_label = "";

Profiler::event_t Profiler::get()
{
    if (!free_list.empty()) { event_t e = free_list.back(); free_list.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

void Profiler::recycle()
{
    for (const Rec& r : pending) { free_list.push_back(r.a); free_list.push_back(r.b); }
    pending.clear();
}

Overlap::~Overlap()
{
    for (void* e : events) (void)hipEventDestroy((hipEvent_t)e);
    if (aux) (void)hipStreamDestroy((hipStream_t)aux);
}

Profiler::~Profiler()
{
    recycle();
    for (event_t e : free_list) (void)hipEventDestroy((hipEvent_t)e);
}

}  // namespace ftp
