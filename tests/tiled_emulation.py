"""CPU emulation of fused-tile execution built from oracle ops only (test helper).

Every tile of every group evaluates its layers on nothing but (a) what it is entitled to collect at a
group boundary: the forward rectangle F_s of the group-input map, the backward rectangle B_e of the
delta map, and the decision codes (activation sign, pool winner) on its backward rectangles, which the
owning tiles publish when the backward pass enters the group; and (b) what it computed itself.  Any
read outside those rectangles raises.  Reproducing the untiled oracle this way shows that the integer
maps of oracle/rects.py are sufficient (Sec. 4.2: within a group all intermediate data is computed
locally from data collected at the group input).
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


    def crop_zero_outside(self, r):
        """Values over r; positions this fragment does not cover are zero (deltas nothing contributes to)."""
        x0, y0, x1, y1 = max(r[0], self.rect[0]), max(r[1], self.rect[1]), min(r[2], self.rect[2]), min(r[3], self.rect[3])
        out = np.zeros(self.data.shape[:2] + (r[3] - r[1] + 1, r[2] - r[0] + 1), dtype=self.data.dtype)
        if x0 <= x1 and y0 <= y1:
            out[:, :, y0 - r[1]:y1 - r[1] + 1, x0 - r[0]:x1 - r[0] + 1] = self.crop((x0, y0, x1, y1))
        return out


def windows(r):
    """Input positions of the 2x2 pool windows r."""
    return (2 * r[0], 2 * r[1], 2 * r[2] + 1, 2 * r[3] + 1)


def taps(r, ly):
    """Input positions the convolution outputs r touch: [S a - P, S b + P] per dimension."""
    S, P = ly.stride, ly.pad
    return (S * r[0] - P, S * r[1] - P, S * r[2] + P, S * r[3] + P)


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
    # decision codes published by the owners: sign[l] = (map at boundary l > 0), win[l] = pool winners of layer l-1
    sign = {l: np.zeros((nb, chans[l]) + sizes[l], dtype=bool) for l in range(1, L + 1)}
    win = {l: np.zeros((nb, chans[l]) + sizes[l], dtype=np.uint8) for l in range(1, L + 1) if layers[l - 1].kind == MAXPOOL}
    held = [dict() for _ in groups]
    for g, (s, e) in enumerate(groups):
        out = np.full((nb, chans[e]) + sizes[e], np.nan)
        for tile, rk in plan[g].items():
            F, Ow = rk[R.FWD], rk[R.OWN]
            h = {s: Held(F[s], full(glob[s]).crop(F[s]))}        # group-boundary read: tile + halo
            for l in range(s, e):
                ly = layers[l]
                if ly.kind == CONV:
                    src = h[l].crop_zero_padded(taps(F[l + 1], ly), sizes[l])
                    y = O.leaky_fwd(O.conv_fwd(src, weights[l], None, ly.stride, 0), ly.slope)
                else:
                    y, a = O.pool_fwd(h[l].crop(windows(F[l + 1])))
                    o = Ow[l + 1]
                    win[l + 1][:, :, o[1]:o[3] + 1, o[0]:o[2] + 1] = Held(F[l + 1], a).crop(o)
                h[l + 1] = Held(F[l + 1], y)
                o = Ow[l + 1]
                sign[l + 1][:, :, o[1]:o[3] + 1, o[0]:o[2] + 1] = h[l + 1].crop(o) > 0
            r = F[e]
            assert r == Ow[e]
            out[:, :, r[1]:r[3] + 1, r[0]:r[2] + 1] = h[e].data
            held[g][tile] = h
        assert not np.isnan(out).any()
        glob[e] = out

    tiles = [(i, j) for i in range(N) for j in range(M)]
    partial = {t: [None] * L for t in tiles}
    gdelta = {L: dy}
    for g in range(len(groups) - 1, -1, -1):
        s, e = groups[g]
        out = np.full((nb, chans[s]) + sizes[s], np.nan)
        for tile, rk in plan[g].items():
            B, Ow = rk[R.BWD], rk[R.OWN]
            h = held[g][tile]
            # collected when the backward pass enters the group: delta on B_e, decision codes on B_l
            d = Held(B[e], full(gdelta[e]).crop(B[e]))
            sg = {l: Held(B[l], full(sign[l]).crop(B[l])) for l in range(s + 1, e + 1)}
            wn = {l: Held(B[l], full(win[l]).crop(B[l])) for l in range(s + 1, e + 1) if l in win}
            for l in range(e - 1, s - 1, -1):
                ly = layers[l]
                if ly.kind == MAXPOOL:
                    dxf = O.pool_bwd(d.data, wn[l + 1].data, (2 * d.data.shape[2], 2 * d.data.shape[3]))
                    d = Held(B[l], Held(windows(B[l + 1]), dxf).crop_zero_outside(B[l]))     # a dropped row / column gets 0
                else:
                    # leaky'(Y) from the sign code: slope where the sign is not positive
                    yy = np.where(sg[l + 1].data, 1.0, -1.0)
                    dz = Held(B[l + 1], O.leaky_bwd(d.data, yy, ly.slope))
                    own = Ow[l + 1]
                    xin = h[l].crop_zero_padded(taps(own, ly), sizes[l])
                    partial[tile][l], _ = O.conv_bwd_weight(xin, dz.crop(own), ly.k, ly.stride, 0, want_db=False)
                    if ly.stride == 1:
                        # correlation with the 180-degree rotated filter (Sec. 4.1)
                        wrot = np.ascontiguousarray(weights[l][:, :, ::-1, ::-1].transpose(1, 0, 2, 3))
                        dzp = dz.crop_zero_padded(grow(B[l], ly.pad), sizes[l + 1])
                        d = Held(B[l], O.conv_fwd(dzp, wrot, None, 1, 0))
                    else:
                        # adjoint of the strided convolution on the positions the held deltas touch
                        reach = taps(B[l + 1], ly)
                        dxf = O.conv_bwd_data(dz.data, weights[l], (reach[3] - reach[1] + 1, reach[2] - reach[0] + 1), ly.stride, 0)
                        d = Held(B[l], Held(reach, dxf).crop_zero_outside(B[l]))
            r = B[s]
            out[:, :, r[1]:r[3] + 1, r[0]:r[2] + 1] = d.data
        assert not np.isnan(out).any()
        gdelta[s] = out
    return glob[L], gdelta[0], [partial[t] for t in tiles]
