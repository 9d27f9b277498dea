"""Helpers of the GPU parity tests: run libftp and the CPU oracle on the same seeded tensors.

Bars (max |a-b| / max |b| per tensor): activations 1e-5 and gradients 1e-4 in fp32, 2e-2 with bf16
storage.  Gradients are compared twice:
  * "given state": the oracle's forward maps are copied into the plan's workspace (oracle -> GPU, never
    the other way), so both sides back-propagate through identical leaky signs and pool winners.  This
    is the strict elementwise check of back-propagation.
  * "chain": ftp_forward followed by ftp_backward.  A rounding difference in a forward value that sits on
    a kink (a pre-activation within rounding of 0, two pool candidates within rounding of each other)
    legitimately flips a decision and changes a few gradient entries by O(1); the chain check is strict
    only where the oracle shows every decision is clear of its kink, else it is held to a norm-wise bound.
"""
import numpy as np

from ftp_synth import configs as C
from ftp_synth.configs import CONV

TOL_ACT_F32 = 1e-5     # activations, fp32
TOL_GRAD_F32 = 1e-4    # dX and dW, fp32
TOL_BF16 = 2e-2        # everything, bf16 storage
# Chain check with flipped decisions (see check_case): relative L2 bounds and the largest share of decisions
# that may flip, each about twice the largest value measured on the MI355X over the whole test suite:
#   fp32  at most 9.9e-7 of the decisions flip, error at most 5.3e-3 (config 4);
#   bf16  at most 2.4e-4 of the decisions flip (config 5: 9567 of 39.9 million), error at most 0.142 in dx, 0.075 in dW.
CHAIN_L2_F32 = 1.1e-2
CHAIN_L2_BF16 = 3e-1
CHAIN_MAX_FLIP_SHARE = {False: 2e-6, True: 5e-4}


def rel_inf(a, b):
    """max |a - b| / max |b| over one tensor (the 'relative' of the parity bars)."""
    d = float(np.max(np.abs(a.astype(np.float64) - b.astype(np.float64))))
    s = float(np.max(np.abs(b)))
    return d / s if s > 0 else d


def rel_l2(a, b):
    d = float(np.linalg.norm((a.astype(np.float64) - b.astype(np.float64)).ravel()))
    s = float(np.linalg.norm(b.astype(np.float64).ravel()))
    return d / s if s > 0 else d


def oracle_run(oracle, cfg, x, ws, bs, dy, want_db=False):
    bf = cfg.dtype == "bf16"
    acts, args = oracle.forward(cfg.layers, x, ws, bs, bf16_store=bf)
    dx, dws, dbs = oracle.backward(cfg.layers, acts, args, ws, dy, bf16_store=bf, want_db=want_db)
    return acts, args, dx, dws, dbs


def pool_gap(a):
    """Top-2 gap of every 2x2 window of a map (n, c, h, w) -> (n, c, floor(h/2), floor(w/2))."""
    n, c, h, w = a.shape
    a = a[:, :, :h // 2 * 2, :w // 2 * 2]            # an odd map's last row / column lies in no window
    win = a.reshape(n, c, h // 2, 2, w // 2, 2).transpose(0, 1, 2, 4, 3, 5).reshape(n, c, h // 2, w // 2, 4)
    srt = np.sort(win, axis=-1)
    return srt[..., 3] - srt[..., 2]


def min_decision_margin(layers, acts):
    """Smallest distance of any forward decision from its kink, relative to the map's max magnitude:
    |Y| for the leaky signs that back-propagation reads (pooled outputs where a pool follows), and the
    top-2 gap of every pool window."""
    m = np.inf
    L = len(layers)
    for l, ly in enumerate(layers):
        out = acts[l + 1]
        scale = float(np.max(np.abs(out))) or 1.0
        if ly.kind == CONV:
            if not (l + 1 < L and layers[l + 1].kind != CONV):
                m = min(m, float(np.min(np.abs(out))) / scale)
        else:
            m = min(m, float(np.min(pool_gap(acts[l]))) / scale)
            if l > 0 and layers[l - 1].kind == CONV:
                m = min(m, float(np.min(np.abs(out))) / scale)
    return m


class _BiasLayer:
    def __init__(self, ly):
        self.kind, self.k, self.stride, self.pad, self.cin, self.cout, self.slope = \
            ly.kind, ly.k, ly.stride, ly.pad, ly.cin, ly.cout, ly.slope
        self.has_bias = 1


def make_session(cfg, batch, has_bias=False):
    from paper_2409_09083_amd.harness import Session
    layers = cfg.layers
    if has_bias:
        layers = [_BiasLayer(ly) if ly.kind == CONV else ly for ly in layers]
    return Session(layers, batch, cfg.in_c, cfg.in_h, cfg.in_w, cfg.grid, cfg.group_ends, cfg.dtype)


def gpu_run(cfg, x, ws, bs, dy, has_bias=False):
    import torch
    s = make_session(cfg, x.shape[0], has_bias)
    s.load(x=x, weights=ws, dy=dy, biases=bs if has_bias else None)
    s.step()
    torch.cuda.synchronize()
    return {"y": s.to_np(s.y), "dx": s.to_np(s.dx), "wgrad": s.to_np(s.wgrad), "partials": s.to_np(s.partials),
            "session": s}


def flat_grad(cfg, dws, dbs=None, has_bias=False):
    parts = []
    for l, ly in enumerate(cfg.layers):
        if ly.kind == CONV:
            parts.append(dws[l].ravel())
            if has_bias:
                parts.append(dbs[l].ravel())
    return np.concatenate(parts)


def param_slices(cfg, has_bias=False):
    """[(layer, start, stop)] of each convolution's filter inside the parameter vector."""
    out, off = [], 0
    for l, ly in enumerate(cfg.layers):
        if ly.kind == CONV:
            n = ly.cout * ly.cin * ly.k * ly.k
            out.append((l, off, off + n))
            off += n + (ly.cout if has_bias else 0)
    return out


def groups_of(cfg):
    out, s = [], 0
    for e in cfg.group_ends:
        out.append((s, e))
        s = e
    return out


def oracle_mask(acts, args, b):
    """Decision code of boundary b as the library defines it: bit 0 = value > 0, bits 1-2 = pool winner."""
    m = (acts[b] > 0).astype(np.uint8)
    if args[b - 1] is not None:
        m |= (args[b - 1].astype(np.uint8) << 1)
    return m


def pack_signs(act):
    """Sign map as the library lays it out: int32 words [image][ceil(C/32)][H][W], bit c % 32 = act[:, c] > 0."""
    n, c, h, w = act.shape
    g = (c + 31) // 32
    words = np.zeros((n, g, h, w), dtype=np.uint32)
    for ch in range(c):
        words[:, ch // 32] |= (act[:, ch] > 0).astype(np.uint32) << np.uint32(ch % 32)
    return words.view(np.int32)


def unpack_signs(words, c):
    w = words.view(np.uint32)
    return np.stack([(w[:, ch // 32] >> np.uint32(ch % 32)) & 1 for ch in range(c)], axis=1).astype(bool)


def check_forward_state(s, cfg, acts, args, tol_a, images=None):
    """Every map the plan keeps equals the oracle's: the assembled owned tiles, and each stack's whole
    forward rectangle (recomputed halo included).  Decision codes may differ from the oracle's only where
    the oracle's own value is within the activation tolerance of the kink (|Y| small, top-2 gap small).
    images: the images of the session's batch that `acts` / `args` hold (default: all of them)."""
    import paper_2409_09083_amd as F
    for b in range(1, len(cfg.layers) + 1):
        got = s.get_boundary(b, images=images)
        scale = float(np.max(np.abs(acts[b])))
        if got is not None:
            e = rel_inf(got, acts[b])
            assert e <= tol_a, ("activation at boundary", b, e)
            for (r, slot) in s.get_slots(b, images=images):
                ref = acts[b][:, :, r[1]:r[3] + 1, r[0]:r[2] + 1]
                assert np.max(np.abs(slot - ref)) <= tol_a * scale, ("held rectangle", b, r)
        gm = s.get_boundary(b, F.FTP_BUF_MASK, images=images)       # behind pools only
        gs = s.get_boundary(b, F.FTP_BUF_SIGN, images=images)       # behind convolutions only
        if gs is not None:
            sg = unpack_signs(gs, acts[b].shape[1])
            bad = sg != (acts[b] > 0)
            if bad.any():
                assert float(np.abs(acts[b][bad]).max()) <= tol_a * scale, ("activation signs", b, int(bad.sum()))
            if gm is not None:
                # bit 0 of the code bytes is the same decision
                assert np.array_equal(sg, (gm & 1).astype(bool)), ("packed signs", b)
        if gm is not None and args[b - 1] is not None:
            bad = ((gm >> 1) & 3) != args[b - 1]
            if bad.any():
                gap = pool_gap(acts[b - 1])
                assert float(gap[bad].max()) <= 2 * tol_a * scale, ("pool winners", b, int(bad.sum()))


def decision_flips(s, cfg, acts, args, images=None):
    """(flipped, total): how many of the decisions the GPU's forward pass recorded (leaky signs, pool winners)
    differ from the oracle's, and how many decisions there are."""
    import paper_2409_09083_amd as F
    flipped = total = 0
    for b in range(1, len(cfg.layers) + 1):
        gs = s.get_boundary(b, F.FTP_BUF_SIGN, images=images)
        if gs is not None:
            flipped += int((unpack_signs(gs, acts[b].shape[1]) != (acts[b] > 0)).sum())
            total += acts[b].size
        gm = s.get_boundary(b, F.FTP_BUF_MASK, images=images)
        if gm is not None and args[b - 1] is not None:
            flipped += int((((gm >> 1) & 3) != args[b - 1]).sum())
            total += args[b - 1].size
    return flipped, total


def decisions_agree(s, cfg, acts, args, images=None):
    """True if every leaky sign and pool winner the GPU's forward pass recorded equals the oracle's."""
    return decision_flips(s, cfg, acts, args, images)[0] == 0


def import_forward_state(s, cfg, acts, args, images=None):
    """oracle -> GPU: the plan's workspace receives the oracle's forward maps and decision codes."""
    import paper_2409_09083_amd as F
    for b in range(1, len(cfg.layers) + 1):
        s.set_boundary(b, acts[b], images=images)
        s.set_boundary(b, oracle_mask(acts, args, b), F.FTP_BUF_MASK, images=images)
        s.set_boundary(b, pack_signs(acts[b]), F.FTP_BUF_SIGN, images=images)


def check_grads(cfg, got_dx, got_wgrad, dx, dws, dbs, has_bias, tol_g, label):
    e = rel_inf(got_dx, dx)
    assert e <= tol_g, (label, "dx", e)
    ref = flat_grad(cfg, dws, dbs, has_bias)
    assert got_wgrad.shape == ref.shape
    for (l, a, b) in param_slices(cfg, has_bias):
        e = rel_inf(got_wgrad[a:b], ref[a:b])
        assert e <= tol_g, (label, "dW", l, e)
        if has_bias:
            eb = rel_inf(got_wgrad[b:b + cfg.layers[l].cout], dbs[l])
            assert eb <= tol_g, (label, "db", l, eb)


def check_case(oracle, cfg, seed=C.rng.MASTER_SEED, has_bias=False, strict_chain=None, partial_check=True):
    import torch
    import paper_2409_09083_amd as F
    x, ws, bs, dy = C.make_tensors(cfg, master_seed=seed)
    bf = cfg.dtype == "bf16"
    if has_bias:
        bs = [None if b is None else C.rng.normal("b/%d" % l, b.shape, 0.2, seed) for l, b in enumerate(bs)]
        if bf:
            bs = [None if b is None else C.rng.to_bf16_rne(b) for b in bs]
    acts, args, dx, dws, dbs = oracle_run(oracle, cfg, x, ws, bs if has_bias else None, dy, want_db=has_bias)
    tol_a, tol_g = (TOL_BF16, TOL_BF16) if bf else (TOL_ACT_F32, TOL_GRAD_F32)
    ref = flat_grad(cfg, dws, dbs, has_bias)

    s = make_session(cfg, x.shape[0], has_bias)
    s.load(x=x, weights=ws, dy=dy, biases=bs if has_bias else None)
    s.forward()
    torch.cuda.synchronize()
    assert rel_inf(s.to_np(s.y), acts[-1]) <= tol_a
    check_forward_state(s, cfg, acts, args, tol_a)

    # chain: back-propagation through the GPU's own forward state
    s.backward()
    s.reduce()
    torch.cuda.synchronize()
    chain_dx, chain_w, chain_p = s.to_np(s.dx), s.to_np(s.wgrad), s.to_np(s.partials)
    flipped, total = decision_flips(s, cfg, acts, args)
    agree = flipped == 0
    if strict_chain is None:
        strict_chain = agree
    if strict_chain:
        # both sides took the same decisions (leaky signs, pool winners): elementwise comparison is well posed
        assert agree
        check_grads(cfg, chain_dx, chain_w, dx, dws, dbs, has_bias, tol_g, "chain")
    else:
        # some decisions sit on their kink and flipped: each flip moves a few gradient entries by O(1), so only a
        # norm-wise bound is meaningful here; the elementwise bars are enforced on the forward state above and on
        # given state below.  The bound is twice the largest error measured on the MI355X for that storage type
        # (the test prints what it measures, with the share of flipped decisions).
        e_dx, e_w = rel_l2(chain_dx, dx), rel_l2(chain_w, ref)
        bound = CHAIN_L2_BF16 if bf else CHAIN_L2_F32
        print("chain %s: %d of %d decisions flipped (%.3g %%), rel L2 error dx %.3g dW %.3g (bound %.3g)"
              % (cfg.name, flipped, total, 100.0 * flipped / max(total, 1), e_dx, e_w, bound))
        assert flipped <= max(4, CHAIN_MAX_FLIP_SHARE[bf] * total), ("flipped decisions", flipped, total)   # (a handful in a small net)
        assert e_dx <= bound, ("chain dx", e_dx)
        assert e_w <= bound, ("chain dW", e_w)
    assert np.allclose(chain_p.astype(np.float64).sum(axis=0), chain_w, rtol=1e-5, atol=1e-6 * np.abs(ref).max())

    # given state: identical decisions on both sides, strict elementwise bars
    import_forward_state(s, cfg, acts, args)
    s.backward()
    s.reduce()
    torch.cuda.synchronize()
    got_dx, got_w, got_p = s.to_np(s.dx), s.to_np(s.wgrad), s.to_np(s.partials)
    check_grads(cfg, got_dx, got_w, dx, dws, dbs, has_bias, tol_g, "given state")
    if partial_check:
        # one stack's partial = the oracle's filter-gradient sum restricted to that stack's owned pixels
        ti, tj = cfg.grid[0] - 1, cfg.grid[1] // 2
        stack = ti * cfg.grid[1] + tj
        groups = groups_of(cfg)
        for (l, a, b) in param_slices(cfg, has_bias):
            g = [k for k, (s0, e0) in enumerate(groups) if s0 <= l < e0][0]
            own = F.ftp_plan_rect(s.plan, g, l + 1, ti, tj, F.FTP_RECT_OWN)
            _, dres, _ = oracle.backward(cfg.layers, acts, args, ws, dy, rect_of_layer=lambda q: own if q == l else None,
                                         bf16_store=bf, want_db=False)
            assert rel_inf(got_p[stack, a:b], dres[l].ravel()) <= tol_g, ("partial", l)
    s.close()
