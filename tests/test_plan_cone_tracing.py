"""The planner's intervals against a derivation that shares nothing with Eq. (1)/(2) as formulas: index sets traced
pixel by pixel.  Rectangles are separable, so every check is done per dimension on sets of integer positions:

  * ownership by labelling: a position of a layer's input belongs to the tile that owns the output position sitting
    on it (convolution: position o sits on inputs o*S .. o*S + S - 1, cut to the map; pool: its window 2o, 2o + 1;
    the row / column a pool drops from an odd map goes with the last window);
  * the forward family by cone tracing: the inputs that a set of outputs reads, position by position
    (o*S - P + k for every tap k inside the map; the two inputs of a pool window);
  * the backward family by adjoint tracing: the outputs whose cone meets a set of inputs.

Against that, through the C ABI (ftp_plan_rect): OWN and BWD are exactly the traced sets' hulls; FWD starts where
the traced set starts and ends exactly S - 1 positions behind its end, cut to the map - the (S - 1) term Eq. (1c-d)
carries as printed (zero for stride 1 and for pools).
"""
import random

import pytest

from ftp_synth import configs as C
from ftp_synth.configs import conv, pool, CONV


@pytest.fixture(scope="module")
def F():
    import paper_2409_09083_amd as F
    return F


def _out_len(n, ly):
    return (n + 2 * ly.pad - ly.k) // ly.stride + 1 if ly.kind == CONV else n // 2


def _reads(o, ly, n_in):
    """Input positions output position o reads (inside the map)."""
    if ly.kind == CONV:
        return [i for i in (o * ly.stride - ly.pad + k for k in range(ly.k)) if 0 <= i < n_in]
    return [2 * o, 2 * o + 1]


def _sits_on(o, ly, n_in, n_out):
    """Input positions that belong with output position o (ownership labelling)."""
    if ly.kind == CONV:
        lo, hi = o * ly.stride, o * ly.stride + ly.stride - 1
    else:
        lo, hi = 2 * o, 2 * o + 1
        if o == n_out - 1:
            hi = n_in - 1                      # the row / column an odd map's pool drops
    return [i for i in range(lo, hi + 1) if i < n_in]


def _check_dim(F, plan, layers, lens, groups, parts, dim):
    for g, (s, e) in enumerate(groups):
        for t in range(parts):
            def rect(kind, l):
                r = F.ftp_plan_rect(plan, g, l, t if dim == 1 else 0, t if dim == 0 else 0, kind)
                return (r[0], r[2]) if dim == 0 else (r[1], r[3])
            n_e = lens[e]
            own = set(range(t * n_e // parts, (t + 1) * n_e // parts))
            assert rect(F.FTP_RECT_OWN, e) == (min(own), max(own))
            assert rect(F.FTP_RECT_FWD, e) == (min(own), max(own))
            fwd_hull = rect(F.FTP_RECT_FWD, e)
            for l in range(e, s, -1):
                ly, n_in, n_out = layers[l - 1], lens[l - 1], lens[l]
                own = {i for o in own for i in _sits_on(o, ly, n_in, n_out)}
                assert rect(F.FTP_RECT_OWN, l - 1) == (min(own), max(own)), ("own", g, t, l - 1, dim)
                assert own == set(range(min(own), max(own) + 1))
                # the forward family is traced from the planner's own interval one layer up: every step is checked
                need = {i for o in range(fwd_hull[0], fwd_hull[1] + 1) for i in _reads(o, ly, n_in)}
                if ly.kind != CONV and fwd_hull[1] == n_out - 1:
                    need |= set(range(2 * n_out, n_in))             # the dropped row stays with the last tile
                extra = ly.stride - 1 if ly.kind == CONV else 0
                got = rect(F.FTP_RECT_FWD, l - 1)
                assert got == (min(need), min(max(need) + extra, n_in - 1)), ("fwd", g, t, l - 1, dim, got, min(need), max(need))
                fwd_hull = got
            bwd_hull = rect(F.FTP_RECT_BWD, s)
            assert bwd_hull == rect(F.FTP_RECT_OWN, s)
            for l in range(s, e):
                ly, n_in, n_out = layers[l], lens[l], lens[l + 1]
                src = set(range(bwd_hull[0], bwd_hull[1] + 1))
                hit = {o for o in range(n_out) if src.intersection(_reads(o, ly, n_in))}
                got = rect(F.FTP_RECT_BWD, l + 1)
                if hit:
                    assert got == (min(hit), max(hit)), ("bwd", g, t, l + 1, dim, got)
                else:
                    # only the row / column dropped by a pool on an odd map reaches no output: nothing to hold
                    assert ly.kind != CONV
                bwd_hull = got


def _check(F, layers, h, w, N, M, ends):
    plan = F.ftp_plan(list(layers), 1, layers[0].cin, h, w, N, M, list(ends))
    try:
        hs, ws = [h], [w]
        for ly in layers:
            hs.append(_out_len(hs[-1], ly)); ws.append(_out_len(ws[-1], ly))
        groups, s = [], 0
        for e in ends:
            groups.append((s, e)); s = e
        _check_dim(F, plan, layers, ws, groups, M, 0)
        _check_dim(F, plan, layers, hs, groups, N, 1)
    finally:
        F.ftp_plan_destroy(plan)


def _all_configs():
    out = [C.tiny(), C.config2(False), C.config2(True), C.config3(), C.config4()]
    out += [C.config5(g) for g in (1, 2, 4, 8, 16)]
    return out


@pytest.mark.parametrize("cfg", _all_configs(), ids=lambda c: c.name)
def test_planner_against_traced_sets_on_configs(F, cfg):
    _check(F, cfg.layers, cfg.in_h, cfg.in_w, cfg.grid[0], cfg.grid[1], cfg.group_ends)


def test_planner_against_traced_sets_general_geometry(F):
    rnd = random.Random(97)
    done = 0
    while done < 120:
        L = rnd.randint(1, 7)
        in_h, in_w = rnd.randint(17, 90), rnd.randint(17, 90)
        layers, c, h, w = [], rnd.randint(1, 3), in_h, in_w
        for _ in range(L):
            if rnd.random() < 0.3 and h >= 4 and w >= 4:
                layers.append(pool(c)); h //= 2; w //= 2
            else:
                co, st = rnd.randint(1, 4), rnd.choice([1, 1, 2])
                layers.append(conv(c, co, rnd.choice([1, 3, 5, 7]), stride=st))
                c, h, w = co, (h - 1) // st + 1, (w - 1) // st + 1
        N, M = rnd.randint(1, 4), rnd.randint(1, 4)
        if h < N or w < M:
            continue
        cuts = sorted(rnd.sample(range(1, L), rnd.randint(0, L - 1))) if L > 1 else []
        try:
            _check(F, layers, in_h, in_w, N, M, tuple(cuts + [L]))
        except F.binding.FtpError as e:
            assert e.code == F.FTP_EGRID
            continue
        done += 1
