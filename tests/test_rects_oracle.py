"""Pins of the integer tile/halo maps (oracle/rects.py): closed forms, invariants, brute-force
dependency tracing and the paper's invariant that fused-tiled evaluation equals the untiled one."""
import numpy as np
import pytest

from ftp_synth import configs as C
from ftp_synth.configs import Layer, conv, pool, CONV, MAXPOOL
from oracle import rects as R


def _all_configs():
    out = [C.tiny(), C.config2(False), C.config2(True), C.config3(), C.config4()]
    out += [C.config5(g) for g in (1, 2, 4, 8, 16)]
    return out


def test_tiny_hand_derived():
    """Two 3x3 stride-1 convolutions on 32x32, 2x2 grid, one group: each convolution adds one halo
    pixel towards the group input (forward) / group output (backward); the map edge clamps."""
    cfg = C.tiny()
    _, plan = R.plan(cfg.layers, 32, 32, 2, 2, cfg.group_ends)
    t = plan[0][(0, 0)]
    assert [t[R.OWN][l] for l in (0, 1, 2)] == [(0, 0, 15, 15)] * 3
    assert [t[R.FWD][l] for l in (0, 1, 2)] == [(0, 0, 17, 17), (0, 0, 16, 16), (0, 0, 15, 15)]
    assert [t[R.BWD][l] for l in (0, 1, 2)] == [(0, 0, 15, 15), (0, 0, 16, 16), (0, 0, 17, 17)]
    t = plan[0][(1, 0)]                          # row 1, column 0
    assert [t[R.FWD][l] for l in (0, 1, 2)] == [(0, 14, 17, 31), (0, 15, 16, 31), (0, 16, 15, 31)]
    assert [t[R.BWD][l] for l in (0, 1, 2)] == [(0, 16, 15, 31), (0, 15, 16, 31), (0, 14, 17, 31)]


@pytest.mark.parametrize("n_conv", [1, 2, 3, 5])
def test_halo_closed_form_stride1(n_conv):
    """n stride-1 3x3 convolutions: F_s = O_e grown by n per side (Eq. 1 with S = 1), then clamped;
    B_e likewise from O_s (Eq. 2)."""
    layers = [conv(4, 4) for _ in range(n_conv)]
    H = W = 60
    _, plan = R.plan(layers, H, W, 3, 3, (n_conv,))
    for (i, j), rk in plan[0].items():
        o = rk[R.OWN][n_conv]
        exp = (max(o[0] - n_conv, 0), max(o[1] - n_conv, 0), min(o[2] + n_conv, W - 1), min(o[3] + n_conv, H - 1))
        assert rk[R.FWD][0] == exp
        assert rk[R.BWD][n_conv] == exp
        for k in range(n_conv + 1):              # mirror symmetry of the two passes
            assert rk[R.BWD][k] == rk[R.FWD][n_conv - k]


def test_pool_doubles_halo():
    """conv3, pool, conv3, pool, conv3 (config 2, fused): halo at the input = 1 + 2*(1 + 2*1) = 7."""
    cfg = C.config2(True)
    _, plan = R.plan(cfg.layers, 416, 416, 3, 3, cfg.group_ends)
    mid = plan[0][(1, 1)]
    assert mid[R.OWN][5] == (34, 34, 68, 68)
    assert mid[R.OWN][0] == (136, 136, 275, 275)
    assert mid[R.FWD][0] == (129, 129, 282, 282)
    # config 5 with one group of 16 layers: 59-pixel halo at the 608x608 input
    c5 = C.config5(16)
    _, plan = R.plan(c5.layers, 608, 608, 8, 8, c5.group_ends)
    rk = plan[0][(4, 4)]
    assert rk[R.OWN][0] == (304, 304, 367, 367)
    assert rk[R.FWD][0] == (304 - 59, 304 - 59, 367 + 59, 367 + 59)


@pytest.mark.parametrize("cfg", _all_configs(), ids=lambda c: c.name)
def test_invariants_on_configs(cfg):
    N, M = cfg.grid
    sizes, plan = R.plan(cfg.layers, cfg.in_h, cfg.in_w, N, M, cfg.group_ends)
    for g, (s, e) in enumerate(R.groups_from_ends(cfg.group_ends)):
        for l in range(s, e + 1):
            h, w = sizes[l]
            cover = np.zeros((h, w), dtype=np.int32)
            for (i, j), rk in plan[g].items():
                o, f, b = rk[R.OWN][l], rk[R.FWD][l], rk[R.BWD][l]
                assert R.area(o) > 0
                cover[o[1]:o[3] + 1, o[0]:o[2] + 1] += 1
                assert R.contains(f, o) and R.contains(b, o)
                if l < e:
                    ly = cfg.layers[l]
                    # Eq. 1 after Eq. 2 covers the rectangle it started from
                    back = R._clamp(R.eq1_back(rk[R.BWD][l + 1], ly), sizes[l])
                    assert R.contains(back, b)
                    if ly.kind == CONV:
                        # the filter-gradient ring around the owned outputs is already in the forward data
                        ring = R._clamp(R.eq1_back(rk[R.OWN][l + 1], ly), sizes[l])
                        assert R.contains(f, ring)
            assert (cover == 1).all()
        # every halo pixel exchanged at a group boundary (F_s forward, B_e backward) belongs to one of
        # the <= 8 adjacent tiles (Sec. 4.2, group-boundary communication)
        for l, kind in ((s, R.FWD), (e, R.BWD)):
            for (i, j), rk in plan[g].items():
                r = rk[kind][l]
                for (i2, j2), rk2 in plan[g].items():
                    o2 = rk2[R.OWN][l]
                    if max(r[0], o2[0]) <= min(r[2], o2[2]) and max(r[1], o2[1]) <= min(r[3], o2[3]):
                        assert abs(i2 - i) <= 1 and abs(j2 - j) <= 1, (g, l, (i, j), (i2, j2))


def test_dependency_tracing_brute_force(oracle):
    """Set one input pixel at a time; with all-positive filters and slope 1 the non-zero outputs are
    exactly the pixels that depend on it.  F_s must be the bounding box of what O_e depends on, B_e the
    bounding box of what O_s influences."""
    layers = [Layer(CONV, 3, 1, 1, 1, 1, 1.0), pool(1), Layer(CONV, 1, 1, 0, 1, 1, 1.0), Layer(CONV, 3, 1, 1, 1, 1, 1.0)]
    H, W = 12, 16
    ws = [None if ly.kind != CONV else np.ones((1, 1, ly.k, ly.k)) for ly in layers]
    sizes, plan = R.plan(layers, H, W, 2, 3, (4,))
    Ho, Wo = sizes[4]
    dep = np.zeros((H, W, Ho, Wo), dtype=bool)
    for y in range(H):
        for x in range(W):
            xin = np.full((1, 1, H, W), 1.0)         # positive background keeps pool winners meaningful
            base, _ = oracle.forward(layers, xin, ws)
            xin[0, 0, y, x] = 50.0
            acts, _ = oracle.forward(layers, xin, ws)
            dep[y, x] = (acts[-1][0, 0] != base[-1][0, 0])
    for (i, j), rk in plan[0].items():
        o_e, o_s = rk[R.OWN][4], rk[R.OWN][0]
        need = dep[:, :, o_e[1]:o_e[3] + 1, o_e[0]:o_e[2] + 1].any(axis=(2, 3))
        ys, xs = np.nonzero(need)
        assert rk[R.FWD][0] == (xs.min(), ys.min(), xs.max(), ys.max())
        infl = dep[o_s[1]:o_s[3] + 1, o_s[0]:o_s[2] + 1].any(axis=(0, 1))
        ys, xs = np.nonzero(infl)
        assert rk[R.BWD][4] == (xs.min(), ys.min(), xs.max(), ys.max())


def test_strided_conv_hand_derived():
    """One 3x3 stride-2 convolution, 16 columns cut in two: Eq. (1a,c) gives [2a - 1, 2b + 2], Eq. (2a,c)
    [ceil((a - 1)/2), floor((b + 1)/2)], both clamped; the owned input columns are [2a, 2b + 1]."""
    layers = [conv(1, 1, 3, stride=2)]
    sizes, plan = R.plan(layers, 16, 16, 1, 2, (1,))
    assert sizes == [(16, 16), (8, 8)]
    t0, t1 = plan[0][(0, 0)], plan[0][(0, 1)]
    assert (t0[R.OWN][1], t1[R.OWN][1]) == ((0, 0, 3, 7), (4, 0, 7, 7))
    assert (t0[R.OWN][0], t1[R.OWN][0]) == ((0, 0, 7, 15), (8, 0, 15, 15))
    assert (t0[R.FWD][0], t1[R.FWD][0]) == ((0, 0, 8, 15), (7, 0, 15, 15))
    assert (t0[R.BWD][1], t1[R.BWD][1]) == ((0, 0, 4, 7), (4, 0, 7, 7))
    # 7x7 stride 2 on an odd map: 15 -> 8 positions; halo 3 + the (S - 1) term
    layers = [conv(1, 1, 7, stride=2)]
    sizes, plan = R.plan(layers, 15, 15, 2, 1, (1,))
    assert sizes[1] == (8, 8)
    t0, t1 = plan[0][(0, 0)], plan[0][(1, 0)]
    assert (t0[R.FWD][0], t1[R.FWD][0]) == ((0, 0, 14, 10), (0, 5, 14, 14))
    assert (t0[R.OWN][0], t1[R.OWN][0]) == ((0, 0, 14, 7), (0, 8, 14, 14))
    assert (t0[R.BWD][1], t1[R.BWD][1]) == ((0, 0, 7, 5), (0, 3, 7, 7))


def test_pool_on_odd_map_last_tile_takes_dropped_row():
    layers = [pool(1)]
    sizes, plan = R.plan(layers, 9, 7, 2, 3, (1,))
    assert sizes[1] == (4, 3)
    assert plan[0][(1, 2)][R.OWN][1] == (2, 2, 2, 3)
    assert plan[0][(1, 2)][R.OWN][0] == (4, 4, 6, 8) == plan[0][(1, 2)][R.FWD][0]
    assert plan[0][(0, 0)][R.OWN][0] == (0, 0, 1, 3)
    assert plan[0][(1, 2)][R.BWD][1] == (2, 2, 2, 3)


def test_strided_dependency_tracing_brute_force(oracle):
    """Strided convolutions and a pool on an odd map, traced pixel by pixel (all-positive filters, slope 1, one
    large input pixel at a time): B_e is exactly the bounding box of what O_s influences (Eq. 2 is the exact cone);
    F_s starts where the bounding box of what O_e depends on starts and exceeds it at the far side by at most the
    (S - 1) terms of Eq. (1c-d) carried down to the group input."""
    layers = [Layer(CONV, 3, 2, 1, 1, 1, 1.0), Layer(CONV, 5, 1, 2, 1, 1, 1.0), pool(1), Layer(CONV, 3, 2, 1, 1, 1, 1.0)]
    H, W = 23, 26
    ws = [None if ly.kind != CONV else np.ones((1, 1, ly.k, ly.k)) for ly in layers]
    sizes, plan = R.plan(layers, H, W, 2, 2, (4,))
    assert sizes == [(23, 26), (12, 13), (12, 13), (6, 6), (3, 3)]
    Ho, Wo = sizes[4]
    dep = np.zeros((H, W, Ho, Wo), dtype=bool)
    base_in = np.full((1, 1, H, W), 1.0)
    base, _ = oracle.forward(layers, base_in, ws)
    for y in range(H):
        for x in range(W):
            xin = base_in.copy()
            xin[0, 0, y, x] = 50.0                   # whatever it reaches becomes the largest value of its pool window
            acts, _ = oracle.forward(layers, xin, ws)
            dep[y, x] = (acts[-1][0, 0] != base[-1][0, 0])
    slack = ((2 - 1) * 2) * 2 + (2 - 1)              # last layer's term, doubled by the pool and by layer 0, plus layer 0's own
    for (i, j), rk in plan[0].items():
        o_e, o_s = rk[R.OWN][4], rk[R.OWN][0]
        need = dep[:, :, o_e[1]:o_e[3] + 1, o_e[0]:o_e[2] + 1].any(axis=(2, 3))
        ys, xs = np.nonzero(need)
        f = rk[R.FWD][0]
        assert (f[0], f[1]) == (xs.min(), ys.min())
        assert 0 <= f[2] - xs.max() <= slack and 0 <= f[3] - ys.max() <= slack
        infl = dep[o_s[1]:o_s[3] + 1, o_s[0]:o_s[2] + 1].any(axis=(0, 1))
        ys, xs = np.nonzero(infl)
        assert rk[R.BWD][4] == (xs.min(), ys.min(), xs.max(), ys.max())


_EMU_NETS = {
    "convs": ([conv(2, 3), conv(3, 4), conv(4, 2)], 13, 11),
    "strided": ([conv(2, 3, 3, stride=2), conv(3, 4, 5), conv(4, 3, 1, stride=2), conv(3, 2, 7, stride=2)], 37, 30),
    "oddpools": ([conv(2, 3, 5), pool(3), conv(3, 4), pool(4), pool(4), conv(4, 2, 3, stride=2)], 31, 27),
    "pools": ([conv(2, 4), pool(4), conv(4, 3), conv(3, 4, 1), pool(4), conv(4, 2)], 24, 20),
    "poolfirst": ([pool(2), conv(2, 3), pool(3), pool(3), conv(3, 2)], 32, 24),
}


@pytest.mark.parametrize("net", sorted(_EMU_NETS))
@pytest.mark.parametrize("grid", [(1, 1), (2, 2), (3, 2)])
@pytest.mark.parametrize("grouping", ["whole", "each", "split"])
def test_fused_tiled_equals_untiled(oracle, net, grid, grouping):
    """Tiles that read only their entitled rectangles reproduce y, dx and dW of the untiled network,
    and each tile's partial filter gradient is the oracle's sum restricted to that tile's pixels."""
    from tests import tiled_emulation as T
    layers, H, W = _EMU_NETS[net]
    L = len(layers)
    ends = {"whole": (L,), "each": tuple(range(1, L + 1)), "split": (L // 2, L)}[grouping]
    rs = np.random.RandomState(23)
    x = rs.standard_normal((2, layers[0].cin, H, W))
    ws = [None if ly.kind != CONV else rs.standard_normal((ly.cout, ly.cin, ly.k, ly.k)) * 0.4 for ly in layers]
    acts, args = oracle.forward(layers, x, ws)
    dy = rs.standard_normal(acts[-1].shape)
    dx, dws, _ = oracle.backward(layers, acts, args, ws, dy, want_db=False)
    y_t, dx_t, partials = T.run(layers, x, ws, dy, grid[0], grid[1], ends)
    assert np.allclose(y_t, acts[-1], rtol=1e-13, atol=1e-13)
    assert np.allclose(dx_t, dx, rtol=1e-12, atol=1e-12)
    sizes, plan = R.plan(layers, H, W, grid[0], grid[1], ends)
    groups = R.groups_from_ends(ends)
    for l, ly in enumerate(layers):
        if ly.kind != CONV:
            continue
        total = sum(p[l] for p in partials)
        assert np.allclose(total, dws[l], rtol=1e-11, atol=1e-12), l
        g = [k for k, (s, e) in enumerate(groups) if s <= l < e][0]
        for t, (i, j) in enumerate([(i, j) for i in range(grid[0]) for j in range(grid[1])]):
            own = plan[g][(i, j)][R.OWN][l + 1]
            _, dres, _ = oracle.backward(layers, acts, args, ws, dy, rect_of_layer=lambda q: own if q == l else None,
                                         want_db=False)
            assert np.allclose(partials[t][l], dres[l], rtol=1e-11, atol=1e-12)
