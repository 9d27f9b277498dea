"""CPU emulation of fused-tile execution built from oracle ops only (test helper).

Every tile of every group evaluates its layers on nothing but (a) the rectangle of the
group-input map it is entitled to read at the group boundary and (b) what it computed
itself; any read outside those rectangles raises.  Reproducing the untiled oracle this way
shows that the integer maps of oracle/rects.py are sufficient (Sec. 4.2: within a group
all intermediate data is computed locally from data collected at the group input).
"""
import numpy as np

from oracle import rects as R
from oracle import reference as O

CONV, MAXPOOL = 0, 1


class Held:
    """A map fragment: data over an inclusive global rectangle of one boundary."""

    def __init__(self, rect, data):
        self.rect, self.data = rect, data
        assert data.shape[2] == rect[3] - rect[1] + 1 and data.shape[3] == rect[2] - rect[0] + 1

    def crop(self, r):
        assert R.contains(self.rect, r), ("read outside held data", self.rect, r)
        x0, y0 = self.rect[0], self.rect[1]
        return np.ascontiguousarray(self.data[:, :, r[1] - y0:r[3] - y0 + 1, r[0] - x0:r[2] - x0 + 1])

    def crop_zero_padded(self, r, hw):
        """Values over r; positions outside the real map are that layer's zero padding."""
        h, w = hw
        inside = (max(r[0], 0), max(r[1], 0), min(r[2], w - 1), min(r[3], h - 1))
        out = np.zeros(self.data.shape[:2] + (r[3] - r[1] + 1, r[2] - r[0] + 1), dtype=self.data.dtype)
        out[:, :, inside[1] - r[1]:inside[3] - r[1] + 1, inside[0] - r[0]:inside[2] - r[0] + 1] = self.crop(inside)
        return out


def full(a):
    return Held((0, 0, a.shape[3] - 1, a.shape[2] - 1), a)


def grow(r, p):
    return (r[0] - p, r[1] - p, r[2] + p, r[3] + p)


def run(layers, x, weights, dy, N, M, group_ends):
    """Fused-tile forward + backward; returns y, dx, per-tile partial dW (list over tiles of list over layers)."""
    L = len(layers)
    sizes, plan = R.plan(layers, x.shape[2], x.shape[3], N, M, group_ends)
    groups = R.groups_from_ends(group_ends)
    chans = [x.shape[1]] + [ly.cout for ly in layers]
    nb = x.shape[0]
    glob = {0: x}
    globarg = {}
    held = [dict() for _ in groups]      # held[g][(i,j)] = {l: Held}, args likewise
    heldarg = [dict() for _ in groups]
    for g, (s, e) in enumerate(groups):
        out = np.full((nb, chans[e]) + sizes[e], np.nan)
        outarg = np.zeros((nb, chans[e]) + sizes[e], dtype=np.uint8)
        for tile, rk in plan[g].items():
            Hd = rk[R.HELD]
            h = {s: Held(Hd[s], full(glob[s]).crop(Hd[s]))}     # group-boundary read: tile + halo
            ha = {}
            for l in range(s, e):
                ly = layers[l]
                if ly.kind == CONV:
                    src = h[l].crop_zero_padded(R.eq1_back(Hd[l + 1], ly), sizes[l])
                    y = O.leaky_fwd(O.conv_fwd(src, weights[l], None, ly.stride, 0), ly.slope)
                else:
                    y, a = O.pool_fwd(h[l].crop(R.eq1_back(Hd[l + 1], ly)))
                    ha[l + 1] = Held(Hd[l + 1], a)
                h[l + 1] = Held(Hd[l + 1], y)
            r = Hd[e]
            assert r == rk[R.OWN][e]
            out[:, :, r[1]:r[3] + 1, r[0]:r[2] + 1] = h[e].data
            if e in ha:
                outarg[:, :, r[1]:r[3] + 1, r[0]:r[2] + 1] = ha[e].data
            held[g][tile], heldarg[g][tile] = h, ha
        assert not np.isnan(out).any()
        glob[e] = out
        globarg[e] = outarg

    tiles = [(i, j) for i in range(N) for j in range(M)]
    partial = {t: [None] * L for t in tiles}
    gdelta = {L: dy}
    for g in range(len(groups) - 1, -1, -1):
        s, e = groups[g]
        out = np.full((nb, chans[s]) + sizes[s], np.nan)
        for tile, rk in plan[g].items():
            B, Ow = rk[R.BWD], rk[R.OWN]
            h, ha = held[g][tile], heldarg[g][tile]
            d = Held(B[e], full(gdelta[e]).crop(B[e]))           # group-boundary read of the delta map
            l = e - 1
            while l >= s:
                ly = layers[l]
                ysrc = full(glob[e]) if l + 1 == e else h[l + 1]
                if ly.kind == MAXPOOL and l > s and layers[l - 1].kind == CONV and l + 1 == e:
                    # pool closing the group behind a convolution: sign and winner come with the
                    # group-boundary maps; leaky is monotone, so the winner's sign is the pooled sign
                    lc = layers[l - 1]
                    pm = O.leaky_bwd(d.data, ysrc.crop(B[l + 1]), lc.slope)
                    dzfull = Held(R.eq1_back(B[l + 1], ly), O.pool_bwd(pm, full(globarg[e]).crop(B[l + 1]),
                                  (2 * pm.shape[2], 2 * pm.shape[3])))
                    dz = Held(B[l], dzfull.crop(B[l]))
                    l -= 1
                    ly = lc
                    d = _conv_backward(ly, l, dz, h, glob, s, sizes, weights, B, Ow, partial[tile], premasked=True)
                elif ly.kind == MAXPOOL:
                    asrc = full(globarg[e]) if l + 1 == e else ha[l + 1]
                    dxf = O.pool_bwd(d.data, asrc.crop(B[l + 1]), (2 * d.data.shape[2], 2 * d.data.shape[3]))
                    d = Held(B[l], Held(R.eq1_back(B[l + 1], ly), dxf).crop(B[l]))
                else:
                    dz = Held(B[l + 1], O.leaky_bwd(d.data, ysrc.crop(B[l + 1]), ly.slope))
                    d = _conv_backward(ly, l, dz, h, glob, s, sizes, weights, B, Ow, partial[tile], premasked=True)
                l -= 1
            r = B[s]
            out[:, :, r[1]:r[3] + 1, r[0]:r[2] + 1] = d.data
        assert not np.isnan(out).any()
        gdelta[s] = out
    return glob[L], gdelta[0], [partial[t] for t in tiles]


def _conv_backward(ly, l, dz, h, glob, s, sizes, weights, B, Ow, partial, premasked):
    """dz: Held over B[l+1] (already multiplied by the activation derivative)."""
    xsrc = h[l]
    own = Ow[l + 1]
    xin = xsrc.crop_zero_padded(grow(own, ly.pad), sizes[l])
    partial[l], _ = O.conv_bwd_weight(xin, dz.crop(own), ly.k, ly.stride, 0, want_db=False)
    wrot = np.ascontiguousarray(weights[l][:, :, ::-1, ::-1].transpose(1, 0, 2, 3))
    dzp = dz.crop_zero_padded(grow(B[l], ly.pad), sizes[l + 1])
    return Held(B[l], O.conv_fwd(dzp, wrot, None, 1, 0))
