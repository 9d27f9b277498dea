"""Integer tile/halo maps of fused tile partitioning, written out from Sec. 4.2.

TEST INFRASTRUCTURE ONLY (second, independent implementation of the maps the
GPU library's planner produces; compared bit-exactly in the tests).

Notation follows the paper: a tile (i, j) of an N x M grid (i = row, j = column)
spans, at the input of layer l ("boundary" l), the inclusive rectangle
(x1, y1)-(x2, y2); layer l has kernel K_l and stride S_l; a group (s, e) starts at
the input of layer s and ends at the input of layer e.

Three families per group, all clamped to the map after every step:
  OWN  O_l : O_e is the equal split of the group's output map (tile index t of n parts
             over a length W owns [floor(t*W/n), floor((t+1)*W/n) - 1]); O_{l-1} is O_l
             scaled by the stride only (no kernel term).  A disjoint cover of every map.
  FWD  F_l : F_e = O_e, then Eq. (1a-d) walked from e down to s: what the forward pass of
             the tile computes and keeps.
  BWD  B_l : B_s = O_s, then Eq. (2a-d) walked from s up to e: where the tile holds deltas.
B_l can stick out of F_l (second half of a group).  The activation signs and pool winners
back-propagation needs there are one small code per element; like the delta halo they are
collected from the owning neighbours at the synchronisation point where the backward pass
enters the group, so nothing is exchanged inside a group.
For a 2x2/2 pool the exact dependence is used in both directions (Eq. (1) and (2) are
stated for convolutions): back a' = 2a, b' = 2b + 1; forth a' = floor(a/2), b' = floor(b/2).
A pool on an odd-sized map drops the last row / column (no padding); so that the owned rectangles
still cover that map, the tile holding the last pooled row / column also takes the dropped one
(OWN and FWD alike: it is produced by the layer before and its delta is zero).
A strided convolution (stride S, kernel K, padding floor(K/2)) maps H to floor((H - 1)/S) + 1
positions; Eq. (1c-d) is used as printed, with its (S - 1) term, and then clamped to the map.
"""

CONV, MAXPOOL = 0, 1
OWN, FWD, BWD = 0, 1, 2


def map_sizes(layers, in_h, in_w):
    """[(H_l, W_l)] for boundaries 0..L."""
    out = [(in_h, in_w)]
    h, w = in_h, in_w
    for ly in layers:
        h = (h + 2 * ly.pad - ly.k) // ly.stride + 1
        w = (w + 2 * ly.pad - ly.k) // ly.stride + 1
        out.append((h, w))
    return out


def _clamp(r, hw):
    h, w = hw
    x1, y1, x2, y2 = r
    return (max(x1, 0), max(y1, 0), min(x2, w - 1), min(y2, h - 1))


def equal_split(length, parts, t):
    return (t * length) // parts, ((t + 1) * length) // parts - 1


def eq1_back(r, ly):
    """Region at the input of layer `ly` needed for region r of its output (Eq. 1a-d)."""
    x1, y1, x2, y2 = r
    if ly.kind == CONV:
        S, h = ly.stride, ly.k // 2
        return (x1 * S - h, y1 * S - h, x2 * S + h + (S - 1), y2 * S + h + (S - 1))
    return (2 * x1, 2 * y1, 2 * x2 + 1, 2 * y2 + 1)


def stride_back(r, ly):
    """Eq. 1 with the kernel term dropped: the input pixels a tile's outputs sit on."""
    x1, y1, x2, y2 = r
    S = ly.stride
    return (x1 * S, y1 * S, x2 * S + (S - 1), y2 * S + (S - 1))


def _ceil_div(a, b):
    return -((-a) // b)


def eq2_forth(r, ly):
    """Delta region at the output of layer `ly` needed for delta region r at its input (Eq. 2a-d)."""
    x1, y1, x2, y2 = r
    if ly.kind == CONV:
        S, h = ly.stride, ly.k // 2
        return (_ceil_div(x1 - h, S), _ceil_div(y1 - h, S), (x2 + h) // S, (y2 + h) // S)
    return (x1 // 2, y1 // 2, x2 // 2, y2 // 2)


def _keep_dropped(back, r, ly, out_hw, in_hw):
    """Pool on an odd map: the rectangle that reaches the last pooled row / column extends to the map's end."""
    if ly.kind != MAXPOOL:
        return back
    x1, y1, x2, y2 = back
    if r[2] == out_hw[1] - 1:
        x2 = in_hw[1] - 1
    if r[3] == out_hw[0] - 1:
        y2 = in_hw[0] - 1
    return (x1, y1, x2, y2)


def group_rects(layers, sizes, s, e, N, M, i, j):
    """{kind: {l: (x1,y1,x2,y2)}} for tile (i,j) of group (s,e), boundaries s..e."""
    He, We = sizes[e]
    ya, yb = equal_split(He, N, i)
    xa, xb = equal_split(We, M, j)
    O = {e: (xa, ya, xb, yb)}
    F = {e: O[e]}
    for l in range(e, s, -1):
        O[l - 1] = _clamp(_keep_dropped(stride_back(O[l], layers[l - 1]), O[l], layers[l - 1], sizes[l], sizes[l - 1]), sizes[l - 1])
        F[l - 1] = _clamp(_keep_dropped(eq1_back(F[l], layers[l - 1]), F[l], layers[l - 1], sizes[l], sizes[l - 1]), sizes[l - 1])
    B = {s: O[s]}
    for l in range(s, e):
        B[l + 1] = _clamp(eq2_forth(B[l], layers[l]), sizes[l + 1])
    return {OWN: O, FWD: F, BWD: B}


def groups_from_ends(group_ends):
    out, s = [], 0
    for e in group_ends:
        out.append((s, e))
        s = e
    return out


def plan(layers, in_h, in_w, N, M, group_ends):
    """rects[g][(i,j)][kind][l]."""
    sizes = map_sizes(layers, in_h, in_w)
    res = []
    for (s, e) in groups_from_ends(group_ends):
        res.append({(i, j): group_rects(layers, sizes, s, e, N, M, i, j)
                    for i in range(N) for j in range(M)})
    return sizes, res


def area(r):
    return max(0, r[2] - r[0] + 1) * max(0, r[3] - r[1] + 1)


def contains(outer, inner):
    return outer[0] <= inner[0] and outer[1] <= inner[1] and outer[2] >= inner[2] and outer[3] >= inner[3]
