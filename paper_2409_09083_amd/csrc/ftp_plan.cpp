// Host planner of libftp: map sizes, tile rectangles, kernel-level units and workspace layout.
// Integer arithmetic only; no GPU call.  Rectangle recursions follow Sec. 4.2, Eq. (1a-d), (2a-d).
#include "ftp_plan.h"

#include <algorithm>
#include <cmath>
#include <new>

namespace ftp {

namespace {

inline int floordiv(int a, int b) { int q = a / b; return (a % b != 0 && ((a < 0) != (b < 0))) ? q - 1 : q; }
inline int ceildiv(int a, int b) { return -floordiv(-a, b); }
inline Seg clampseg(Seg s, int len) { return Seg{std::max(s.a, 0), std::min(s.b, len - 1)}; }
inline Seg hull(Seg p, Seg q) { return Seg{std::min(p.a, q.a), std::max(p.b, q.b)}; }
inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// Eq. (1): interval at the input of `ly` that an output interval depends on (Eq. (1c-d) with its (S - 1) term, as
// printed).  A pool has no kernel overlap: its windows are exactly [2a, 2b+1].
inline Seg dep_back(Seg o, const ftp_layer& ly)
{
    if (ly.kind == FTP_CONV) {
        const int S = ly.stride, h = ly.k / 2;
        return Seg{o.a * S - h, o.b * S + h + (S - 1)};
    }
    return Seg{2 * o.a, 2 * o.b + 1};
}

// Eq. (1) without the kernel term: the input pixels the outputs sit on.
inline Seg own_back(Seg o, const ftp_layer& ly)
{
    const int S = ly.stride;
    return Seg{o.a * S, o.b * S + (S - 1)};
}

// A pool on an odd length drops the last position; the tile that reaches the last pooled position keeps it, so
// that the owned intervals still cover the map (it is produced by the layer before; its delta is zero).
inline Seg keep_dropped(Seg back, Seg o, const ftp_layer& ly, int out_len, int in_len)
{
    if (ly.kind == FTP_MAXPOOL && o.b == out_len - 1) back.b = in_len - 1;
    return back;
}

// Eq. (2): delta interval at the output of `ly` that a delta interval at its input depends on.
inline Seg dep_forth(Seg i, const ftp_layer& ly)
{
    if (ly.kind == FTP_CONV) {
        const int S = ly.stride, h = ly.k / 2;
        return Seg{ceildiv(i.a - h, S), floordiv(i.b + h, S)};
    }
    return Seg{floordiv(i.a, 2), floordiv(i.b, 2)};
}

int fill_group(const Plan& p, GroupRects& g)
{
    const int nb = g.e - g.s + 1;
    g.seg.assign((size_t)3 * nb * 2 * kMaxGrid, Seg{0, -1});
    for (int dim = 0; dim < 2; ++dim) {
        const int parts = dim == 0 ? p.M : p.N;
        auto len = [&](int l) { return dim == 0 ? p.W[l] : p.H[l]; };
        for (int t = 0; t < parts; ++t) {
            // owned: equal split of the group's output map, then stride-only projection towards s
            const long L = len(g.e);
            Seg o{(int)((long)t * L / parts), (int)((long)(t + 1) * L / parts) - 1};
            if (o.b < o.a) return FTP_EGRID;
            g.at(FTP_RECT_OWN, g.e, dim, t) = o;
            g.at(FTP_RECT_FWD, g.e, dim, t) = o;
            for (int l = g.e; l > g.s; --l) {
                const ftp_layer& ly = p.layers[l - 1];
                const Seg o1 = g.at(FTP_RECT_OWN, l, dim, t), f1 = g.at(FTP_RECT_FWD, l, dim, t);
                g.at(FTP_RECT_OWN, l - 1, dim, t) = clampseg(keep_dropped(own_back(o1, ly), o1, ly, len(l), len(l - 1)), len(l - 1));
                g.at(FTP_RECT_FWD, l - 1, dim, t) = clampseg(keep_dropped(dep_back(f1, ly), f1, ly, len(l), len(l - 1)), len(l - 1));
            }
            g.at(FTP_RECT_BWD, g.s, dim, t) = g.at(FTP_RECT_OWN, g.s, dim, t);
            for (int l = g.s; l < g.e; ++l)
                g.at(FTP_RECT_BWD, l + 1, dim, t) = clampseg(dep_forth(g.at(FTP_RECT_BWD, l, dim, t), p.layers[l]), len(l + 1));
        }
        // invariants the kernels rely on
        for (int l = g.s; l <= g.e; ++l) {
            int next = 0;
            for (int t = 0; t < parts; ++t) {
                const Seg o = g.at(FTP_RECT_OWN, l, dim, t);
                if (o.a != next || o.b < o.a) return FTP_EGRID;      // disjoint cover, in order
                next = o.b + 1;
                const Seg f = g.at(FTP_RECT_FWD, l, dim, t), b = g.at(FTP_RECT_BWD, l, dim, t);
                if (!seg_contains(f, o) || !seg_contains(b, o)) return FTP_EGRID;
                if (l < g.e) {
                    // forward reads stay inside what the stack holds; the filter-gradient ring too
                    if (!seg_contains(f, clampseg(dep_back(g.at(FTP_RECT_FWD, l + 1, dim, t), p.layers[l]), len(l)))) return FTP_EGRID;
                    if (!seg_contains(f, clampseg(dep_back(g.at(FTP_RECT_OWN, l + 1, dim, t), p.layers[l]), len(l)))) return FTP_EGRID;
                    if (!seg_contains(g.at(FTP_RECT_BWD, l + 1, dim, t), clampseg(dep_forth(b, p.layers[l]), len(l + 1)))) return FTP_EGRID;
                }
            }
            if (next != len(l)) return FTP_EGRID;
        }
    }
    return FTP_OK;
}

int max_len(const GroupRects& g, int kind, int l, int dim, int parts)
{
    int m = 0;
    for (int t = 0; t < parts; ++t) m = std::max(m, seg_len(g.at(kind, l, dim, t)));
    return m;
}

}  // namespace

int build_plan(const ftp_layer* layers, int n_layers, int batch, int in_c, int in_h, int in_w,
               int N, int M, const int32_t* group_ends, int n_groups, ftp_dtype dtype, ftp_plan_s** out)
{
    if (!layers || !group_ends || !out) return FTP_EINVAL;
    *out = nullptr;
    if (n_layers < 1 || batch < 1 || in_c < 1 || in_h < 1 || in_w < 1 || N < 1 || M < 1 || n_groups < 1) return FTP_EINVAL;
    if (dtype != FTP_F32 && dtype != FTP_BF16) return FTP_EINVAL;
    if (N > kMaxGrid || M > kMaxGrid) return FTP_EGRID;
    if ((long)N * M * batch > 65535) return FTP_EUNSUPPORTED;      // one workgroup plane per (stack, image)

    ftp_plan_s* holder = new (std::nothrow) ftp_plan_s();
    if (!holder) return FTP_ENOMEM;
    Plan& p = holder->p;
    auto fail = [&](int code) { delete holder; return code; };

    p.n_layers = n_layers; p.batch = batch; p.N = N; p.M = M; p.dtype = dtype;
    p.esize = dtype == FTP_F32 ? 4 : 2;
    p.layers.assign(layers, layers + n_layers);
    p.C.push_back(in_c); p.H.push_back(in_h); p.W.push_back(in_w);
    for (int l = 0; l < n_layers; ++l) {
        const ftp_layer& ly = p.layers[l];
        const int c = p.C.back(), h = p.H.back(), w = p.W.back();
        if (ly.kind == FTP_CONV) {
            if ((ly.stride != 1 && ly.stride != 2) || (ly.k != 1 && ly.k != 3 && ly.k != 5 && ly.k != 7) || ly.pad != ly.k / 2)
                return fail(FTP_EUNSUPPORTED);
            if (!(ly.leaky_slope >= 0.0f) || !std::isfinite(ly.leaky_slope)) return fail(FTP_EUNSUPPORTED);
            if (ly.cout < 1) return fail(FTP_EINVAL);
            if (ly.cin != c) return fail(FTP_ECHANNELS);
            p.C.push_back(ly.cout);
            p.H.push_back((h + 2 * ly.pad - ly.k) / ly.stride + 1); p.W.push_back((w + 2 * ly.pad - ly.k) / ly.stride + 1);
        } else if (ly.kind == FTP_MAXPOOL) {
            if (ly.k != 2 || ly.stride != 2 || ly.pad != 0) return fail(FTP_EUNSUPPORTED);
            if (ly.cin != c || ly.cout != c) return fail(FTP_ECHANNELS);
            if (h < 2 || w < 2) return fail(FTP_EGRID);
            p.C.push_back(c); p.H.push_back(h / 2); p.W.push_back(w / 2);
        } else {
            return fail(FTP_EUNSUPPORTED);
        }
    }
    {
        int prev = 0;
        for (int g = 0; g < n_groups; ++g) {
            if (group_ends[g] <= prev || group_ends[g] > n_layers) return fail(FTP_EGROUPS);
            prev = group_ends[g];
        }
        if (prev != n_layers) return fail(FTP_EGROUPS);
    }
    p.group_of_layer.assign(n_layers, 0);
    {
        int s = 0;
        for (int g = 0; g < n_groups; ++g) {
            GroupRects gr;
            gr.s = s; gr.e = group_ends[g];
            const int rc = fill_group(p, gr);
            if (rc != FTP_OK) return fail(rc);
            for (int l = s; l < gr.e; ++l) p.group_of_layer[l] = g;
            p.groups.push_back(std::move(gr));
            s = group_ends[g];
        }
    }

    // ---- kernel-level units and buffers -------------------------------------------------------
    const int L = n_layers;
    const size_t stacks = (size_t)N * M;
    std::vector<bool> is_group_edge(L + 1, false);
    is_group_edge[0] = true;
    for (const GroupRects& g : p.groups) is_group_edge[g.e] = true;

    size_t ws = 256;                           // (a margin in front: the 16-bit kernels round addresses down to whole dwords)
    auto alloc = [&](size_t bytes) { const size_t off = ws; ws = align256(ws + bytes); return off; };

    std::vector<BufRef>& act = p.act; std::vector<BufRef>& mask = p.mask; std::vector<BufRef>& delta = p.delta;
    act.assign(L + 1, BufRef()); mask.assign(L + 1, BufRef()); delta.assign(L + 1, BufRef());
    p.sign.assign(L + 1, BufRef());
    p.home_group.assign(L + 1, 0);
    size_t pp_bytes = 0;                       // size of one ping-pong slot set for interior deltas
    for (int g = 0; g < (int)p.groups.size(); ++g) {
        const GroupRects& gr = p.groups[g];
        int l = gr.s, ordinal = 0;
        while (l < gr.e) {
            Unit u;
            u.group = g; u.layer = l; u.bi = l;
            if (p.layers[l].kind == FTP_CONV) {
                u.kind = UNIT_CONV;
                // the pool behind a convolution is evaluated in its epilogue where the fast kernels can do that:
                // stride 1, K <= 3, even map; otherwise it stays a step of its own
                u.pooled = (l + 1 < gr.e) && p.layers[l + 1].kind == FTP_MAXPOOL && p.layers[l].stride == 1 && p.layers[l].k <= 3 &&
                           !((p.H[l + 1] | p.W[l + 1]) & 1);
                u.bo = l + 1 + (u.pooled ? 1 : 0);
            } else {
                u.kind = UNIT_POOL; u.pooled = false; u.bo = l + 1;
            }
            const int b = u.bo;
            // homes of boundary b: activation, decision codes, delta (boundary 0 handled below)
            if (act[b].kind == BUF_NONE) {
                BufRef a, w, d;
                a.channels = w.channels = d.channels = p.C[b];
                const size_t map_elems = (size_t)batch * p.C[b] * p.H[b] * p.W[b];
                // decision codes (pool winner + sign): one byte per element of the whole map, written by the owners;
                // kept only where a pool produced the boundary - elsewhere the packed sign map below says it all
                if (u.pooled || u.kind == UNIT_POOL) {
                    w.kind = BUF_WS; w.slot_w = p.W[b]; w.slot_h = p.H[b]; w.bytes = map_elems; w.offset = alloc(w.bytes);
                }
                if (is_group_edge[b]) {
                    a.slot_w = d.slot_w = p.W[b];
                    a.slot_h = d.slot_h = p.H[b];
                    if (b == L) { a.kind = BUF_Y; d.kind = BUF_DY; }
                    else {
                        a.kind = BUF_WS; a.bytes = map_elems * p.esize; a.offset = alloc(a.bytes);
                        d.kind = BUF_WS; d.bytes = map_elems * p.esize; d.offset = alloc(d.bytes);
                    }
                } else {
                    a.per_stack = d.per_stack = true;
                    a.rect_kind = FTP_RECT_FWD; d.rect_kind = FTP_RECT_BWD;
                    a.slot_w = max_len(gr, FTP_RECT_FWD, b, 0, M);
                    a.slot_h = max_len(gr, FTP_RECT_FWD, b, 1, N);
                    d.slot_w = max_len(gr, FTP_RECT_BWD, b, 0, M);
                    d.slot_h = max_len(gr, FTP_RECT_BWD, b, 1, N);
                    // 16-bit maps: an even row length keeps every row of a slot on a 4-byte boundary (pairs of elements
                    // are loaded as one dword)
                    if (dtype == FTP_BF16) { a.slot_w = (a.slot_w + 1) & ~1; d.slot_w = (d.slot_w + 1) & ~1; }
                    a.kind = BUF_WS; a.bytes = stacks * batch * p.C[b] * a.slot_w * a.slot_h * p.esize; a.offset = alloc(a.bytes);
                    d.kind = BUF_WS; d.bytes = stacks * batch * p.C[b] * d.slot_w * d.slot_h * p.esize;
                    d.offset = (size_t)(ordinal & 1);       // ping-pong index, resolved below
                    pp_bytes = std::max(pp_bytes, d.bytes);
                    ++ordinal;
                }
                act[b] = a; mask[b] = w; delta[b] = d;
                p.home_group[b] = g;
                if (u.kind == UNIT_CONV) {
                    BufRef sg;
                    sg.kind = BUF_WS; sg.channels = (p.C[b] + 31) / 32; sg.slot_w = p.W[b]; sg.slot_h = p.H[b];
                    sg.bytes = (size_t)batch * sg.channels * p.H[b] * p.W[b] * 4; sg.offset = alloc(sg.bytes);
                    p.sign[b] = sg;
                }
            }
            p.units.push_back(u);
            l = u.bo;
        }
    }
    // activation derivative folded into the stored deltas
    p.act_slope.assign(L + 1, -1.0f);
    for (const Unit& u : p.units)
        if (u.kind == UNIT_CONV) p.act_slope[u.bo] = p.layers[u.layer].leaky_slope;
    if (p.act_slope[L] >= 0.0f) {
        // the caller's dy is read-only: its scaled copy lives in the workspace and takes its place as delta of L
        BufRef d = delta[L];
        d.kind = BUF_WS; d.bytes = (size_t)batch * p.C[L] * p.H[L] * p.W[L] * p.esize; d.offset = alloc(d.bytes);
        p.dy_scaled = d;
        delta[L] = d;
    }
    act[0].kind = BUF_X; act[0].channels = p.C[0]; act[0].slot_w = p.W[0]; act[0].slot_h = p.H[0];
    delta[0].kind = BUF_DX; delta[0].channels = p.C[0]; delta[0].slot_w = p.W[0]; delta[0].slot_h = p.H[0];
    const size_t pp0 = alloc(pp_bytes), pp1 = alloc(pp_bytes);
    for (int b = 1; b <= L; ++b)
        if (delta[b].kind == BUF_WS && delta[b].per_stack) delta[b].offset = delta[b].offset ? pp1 : pp0;
    // relaid filters for the matrix-core kernels (fp32, two orders per convolution: forward and rotated)
    for (Unit& u : p.units) {
        if (u.kind != UNIT_CONV) continue;
        const ftp_layer& ly = p.layers[u.layer];
        const size_t bytes = (size_t)ly.cout * ly.cin * ly.k * ly.k * sizeof(float);
        u.wt_fwd_offset = alloc(bytes);
        u.wt_bwd_offset = alloc(bytes);
    }
    {
        size_t scratch = 0;
        for (Unit& u : p.units) {
            if (u.kind != UNIT_CONV) continue;
            const ftp_layer& ly = p.layers[u.layer];
            // chunk count of the largest owned rectangle at the convolution output (a strided convolution's filter
            // gradient runs over the owned input pixels: its deltas are read with zeros in between)
            const GroupRects& gr = p.groups[u.group];
            int chunks = 1;
            const int wb = ly.stride == 2 ? u.layer : u.layer + 1;
            for (int i = 0; i < N; ++i)
                for (int j = 0; j < M; ++j) {
                    const Seg sx = gr.at(FTP_RECT_OWN, wb, 0, j), sy = gr.at(FTP_RECT_OWN, wb, 1, i);
                    chunks = std::max(chunks, wgrad_chunks(sx.b - sx.a + 1, sy.b - sy.a + 1, batch, ly.k / 2).total);
                }
            u.wgrad_shares = wgrad_shares(ly.cout, ly.cin, ly.k, N * M, chunks);
            int wmax = 0, tchunks = 1;
            for (int j = 0; j < M; ++j) { const Seg sx = gr.at(FTP_RECT_OWN, u.layer + 1, 0, j); wmax = std::max(wmax, (sx.b - sx.a + 2) & ~1); }
            const int PK = thin_wgrad_pk(wmax, u.pooled);
            for (int i = 0; i < N; ++i)
                for (int j = 0; j < M; ++j) {
                    const Seg sx = gr.at(FTP_RECT_OWN, u.layer + 1, 0, j), sy = gr.at(FTP_RECT_OWN, u.layer + 1, 1, i);
                    tchunks = std::max(tchunks, thin_wgrad_chunks(sx.b - sx.a + 1, sy.b - sy.a + 1, batch, PK, u.pooled).total);
                }
            u.wgrad_shares_thin = wgrad_shares_thin(ly.cout, N * M, tchunks);
            if (ly.cin * ly.k * ly.k <= 160 && ly.cin <= 4) {
                // (the streamed form of the thin-layer kernel has chunks and an occupancy of its own)
                int rws[kMaxGrid], rhs[kMaxGrid];
                for (int j = 0; j < M; ++j) { const Seg sx = gr.at(FTP_RECT_OWN, u.layer + 1, 0, j); rws[j] = sx.b - sx.a + 1; }
                for (int i = 0; i < N; ++i) { const Seg sy = gr.at(FTP_RECT_OWN, u.layer + 1, 1, i); rhs[i] = sy.b - sy.a + 1; }
                const ThinStream ts = thin_stream_geom(rws, rhs, N, M, batch, ly.cin, ly.k, ly.stride, u.pooled);
                if (ts.fits) u.wgrad_shares_thin = wgrad_shares_thin(ly.cout, N * M, ts.max_chunks, 256 * ts.wgs_per_cu);
            }
            if (dtype == FTP_BF16 && ly.k == 3 && ly.stride == 1) {
                int c16 = 1;
                for (int i = 0; i < N; ++i)
                    for (int j = 0; j < M; ++j) {
                        const Seg sx = gr.at(FTP_RECT_OWN, u.layer + 1, 0, j), sy = gr.at(FTP_RECT_OWN, u.layer + 1, 1, i);
                        c16 = std::max(c16, wgrad16_chunks(sx.b - sx.a + 1, sy.b - sy.a + 1, batch, w16_patch_elems(w16_waves_ci(ly.cin)), 1).total);
                    }
                u.wgrad_shares16 = wgrad16_shares(ly.cout, ly.cin, N * M, c16);
            }
            const int shares = std::max(std::max(u.wgrad_shares, u.wgrad_shares_thin), u.wgrad_shares16);
            if (shares > 1) scratch = std::max(scratch, stacks * shares * (size_t)ly.cout * ly.cin * ly.k * ly.k * sizeof(float));
        }
        p.wgrad_scratch_offset = alloc(scratch);
    }
    // (a margin at the end: wide loads of the 16-bit kernels may run a few bytes past the last map)
    p.workspace_bytes = std::max<size_t>(ws, 256) + 256;

    size_t poff = 0;
    for (Unit& u : p.units) {
        u.in_act = act[u.bi]; u.out_act = act[u.bo]; u.out_mask = mask[u.bo];
        u.in_delta = delta[u.bo]; u.out_delta = delta[u.bi];
        u.out_sign = p.sign[u.bo]; u.in_sign = p.sign[u.bi];
        u.scale_out_delta = p.act_slope[u.bi] >= 0.0f;
        u.in_slope = u.scale_out_delta ? p.act_slope[u.bi] : 1.0f;
    }
    std::vector<size_t> layer_poff(L, 0), layer_boff(L, 0);
    for (int l = 0; l < L; ++l) {
        const ftp_layer& ly = p.layers[l];
        if (ly.kind != FTP_CONV) continue;
        layer_poff[l] = poff; poff += (size_t)ly.cout * ly.cin * ly.k * ly.k;
        layer_boff[l] = poff; if (ly.has_bias) poff += ly.cout;
    }
    p.n_params = poff;
    for (Unit& u : p.units)
        if (u.kind == UNIT_CONV) { u.param_offset = layer_poff[u.layer]; u.bias_offset = layer_boff[u.layer]; }

    // ---- work and memory accounting -------------------------------------------------------------
    auto area_sum = [&](const GroupRects& gr, int kind, int l) {
        double sx = 0, sy = 0;
        for (int t = 0; t < M; ++t) sx += seg_len(gr.at(kind, l, 0, t));
        for (int t = 0; t < N; ++t) sy += seg_len(gr.at(kind, l, 1, t));
        return sx * sy;                           // separable: sum over tiles of w*h
    };
    auto area_max = [&](const GroupRects& gr, int kind, int l) {
        return (double)max_len(gr, kind, l, 0, M) * max_len(gr, kind, l, 1, N);
    };
    double fmap = 0, dmap = 0, other = 0;
    for (const Unit& u : p.units) {
        const GroupRects& gr = p.groups[u.group];
        if (u.kind == UNIT_CONV) {
            const ftp_layer& ly = p.layers[u.layer];
            const double kk = (double)ly.k * ly.k * ly.cin * ly.cout * batch;
            const double full = (double)p.H[u.layer + 1] * p.W[u.layer + 1];
            p.useful_macs += 3.0 * kk * full;
            p.executed_macs += kk * (area_sum(gr, FTP_RECT_FWD, u.layer + 1) + area_sum(gr, FTP_RECT_BWD, u.layer) + full);
        }
        if (u.bi == gr.s) {
            p.halo_bytes[0] += (area_sum(gr, FTP_RECT_FWD, u.bi) - (double)p.H[u.bi] * p.W[u.bi]) * p.C[u.bi] * batch * p.esize;
        }
        if (u.bo == gr.e) {
            const double halo_px = area_sum(gr, FTP_RECT_BWD, u.bo) - (double)p.H[u.bo] * p.W[u.bo];
            p.halo_bytes[1] += halo_px * p.C[u.bo] * batch * (p.esize + 1.0);      // delta + decision code
        } else {
            // interior boundary: only decision codes cross tiles (collected when the backward pass enters the group)
            p.halo_bytes[1] += (area_sum(gr, FTP_RECT_BWD, u.bo) - (double)p.H[u.bo] * p.W[u.bo]) * p.C[u.bo] * batch;
        }
        const int kind_out = u.bo == gr.e ? FTP_RECT_OWN : FTP_RECT_FWD;
        fmap += area_max(gr, kind_out, u.bo) * p.C[u.bo] * batch * p.esize;
        // decisions of the own tile: a winner code byte per element behind a pool, a sign bit per element (32
        // channels to a word) behind a convolution
        other += area_max(gr, FTP_RECT_OWN, u.bo) * batch *
                 ((u.pooled || u.kind == UNIT_POOL ? (double)p.C[u.bo] : 0.0) + (u.kind == UNIT_CONV ? 4.0 * ((p.C[u.bo] + 31) / 32) : 0.0));
        dmap = std::max(dmap, (area_max(gr, FTP_RECT_BWD, u.bo) * p.C[u.bo] + area_max(gr, FTP_RECT_BWD, u.bi) * p.C[u.bi]) * batch * p.esize);
    }
    fmap += area_max(p.groups[0], FTP_RECT_FWD, 0) * p.C[0] * batch * p.esize;
    p.split[0] = (size_t)fmap; p.split[1] = (size_t)dmap;
    p.split[2] = p.n_params * (p.esize + 4);      // own copy of all filters + own partial gradient set
    p.split[3] = (size_t)other;

    *out = holder;
    return FTP_OK;
}

}  // namespace ftp
