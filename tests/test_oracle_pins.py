"""Pins of the CPU oracle against things other than itself: finite differences, adjoint
identities, closed forms, library routines (numpy matmul, scipy correlate, torch CPU autograd)."""
import numpy as np
import pytest

from ftp_synth.configs import Layer, conv, pool, CONV, MAXPOOL


def _rand(rs, shape, dtype=np.float64):
    return rs.standard_normal(shape).astype(dtype)


def _net_small():
    return [conv(3, 4), pool(4), conv(4, 5, 1), conv(5, 2)]


def _weights(rs, layers, dtype=np.float64):
    return [None if ly.kind != CONV else _rand(rs, (ly.cout, ly.cin, ly.k, ly.k), dtype) * 0.5 for ly in layers]


def _loss(oracle, layers, x, ws, bs, g):
    acts, _ = oracle.forward(layers, x, ws, bs)
    return float(np.sum(acts[-1] * g))


def test_finite_differences_fp64(oracle):
    """Central differences of L = <G, f(X, W, b)> reproduce dX, dW and db (fp64 everywhere)."""
    rs = np.random.RandomState(7)
    layers = _net_small()
    x = _rand(rs, (2, 3, 8, 8))
    ws = _weights(rs, layers)
    bs = [None if w is None else _rand(rs, (w.shape[0],)) * 0.1 for w in ws]
    acts, args = oracle.forward(layers, x, ws, bs)
    g = _rand(rs, acts[-1].shape)
    # keep clear of the kinks: every pre-activation and every pool top-2 gap is well away from 0
    for l, ly in enumerate(layers):
        if ly.kind == CONV:
            assert np.abs(acts[l + 1]).min() > 1e-5
    dx, dws, dbs = oracle.backward(layers, acts, args, ws, g)
    eps = 1e-6
    checked = 0
    for (arr, grad) in [(x, dx)] + [(ws[l], dws[l]) for l in range(len(layers)) if ws[l] is not None] \
            + [(bs[l], dbs[l]) for l in range(len(layers)) if bs[l] is not None]:
        flat, gflat = arr.reshape(-1), grad.reshape(-1)
        for idx in rs.choice(flat.size, size=min(25, flat.size), replace=False):
            old = flat[idx]
            flat[idx] = old + eps
            lp = _loss(oracle, layers, x, ws, bs, g)
            flat[idx] = old - eps
            lm = _loss(oracle, layers, x, ws, bs, g)
            flat[idx] = old
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - gflat[idx]) <= 1e-6 * max(1.0, abs(fd)), (idx, fd, gflat[idx])
            checked += 1
    assert checked > 100


def test_adjoint_identities_fp64(oracle):
    """slope = 1, no pool: the layer is linear, so <G, A x> == <A^T G, x> and <dW, W> == <G, Y>."""
    rs = np.random.RandomState(3)
    for k in (1, 3):
        ly = Layer(CONV, k, 1, k // 2, 3, 5, 1.0)
        x = _rand(rs, (2, 3, 7, 9))
        w = _rand(rs, (5, 3, k, k))
        acts, args = oracle.forward([ly], x, [w], None)
        g = _rand(rs, acts[-1].shape)
        dx, dws, _ = oracle.backward([ly], acts, args, [w], g)
        lhs = np.sum(g * acts[-1])
        assert abs(lhs - np.sum(dx * x)) <= 1e-12 * abs(lhs)
        assert abs(lhs - np.sum(dws[0] * w)) <= 1e-12 * abs(lhs)


def test_all_ones_closed_form(oracle):
    """All-ones input and 3x3 filters, pad 1: Z = 9 Cin inside, 6 Cin on edges, 4 Cin in corners."""
    cin = 3
    x = np.ones((1, cin, 6, 7))
    w = np.ones((2, cin, 3, 3))
    z = oracle.conv_fwd(x, w, None, 1, 1)
    exp = np.full((6, 7), 9.0 * cin)
    exp[0, :] = exp[-1, :] = 6.0 * cin
    exp[:, 0] = exp[:, -1] = 6.0 * cin
    exp[0, 0] = exp[0, -1] = exp[-1, 0] = exp[-1, -1] = 4.0 * cin
    for co in range(2):
        assert np.array_equal(z[0, co], exp)


def test_conv1x1_is_matmul(oracle):
    rs = np.random.RandomState(5)
    x = _rand(rs, (2, 6, 5, 4))
    w = _rand(rs, (3, 6, 1, 1))
    z = oracle.conv_fwd(x, w, None, 1, 0)
    W2 = w[:, :, 0, 0]
    ref = np.einsum("oc,nchw->nohw", W2, x)
    assert np.allclose(z, ref, rtol=1e-13, atol=1e-13)
    g = _rand(rs, z.shape)
    dx = oracle.conv_bwd_data(g, w, (5, 4), 1, 0)
    assert np.allclose(dx, np.einsum("oc,nohw->nchw", W2, g), rtol=1e-13, atol=1e-13)
    dw, db = oracle.conv_bwd_weight(x, g, 1, 1, 0)
    assert np.allclose(dw[:, :, 0, 0], np.einsum("nohw,nchw->oc", g, x), rtol=1e-13, atol=1e-13)
    assert np.allclose(db, g.sum(axis=(0, 2, 3)), rtol=1e-13, atol=1e-13)


def test_conv3x3_is_scipy_correlate(oracle):
    from scipy.signal import correlate2d, convolve2d
    rs = np.random.RandomState(11)
    x = _rand(rs, (1, 2, 9, 8))
    w = _rand(rs, (3, 2, 3, 3))
    z = oracle.conv_fwd(x, w, None, 1, 1)
    for co in range(3):
        ref = sum(correlate2d(x[0, ci], w[co, ci], mode="same") for ci in range(2))
        assert np.allclose(z[0, co], ref, rtol=1e-13, atol=1e-13)
    # delta back-propagation is the correlation with the 180-degree rotated filter = a true convolution
    g = _rand(rs, z.shape)
    dx = oracle.conv_bwd_data(g, w, (9, 8), 1, 1)
    for ci in range(2):
        ref = sum(convolve2d(g[0, co], w[co, ci], mode="same") for co in range(3))
        assert np.allclose(dx[0, ci], ref, rtol=1e-13, atol=1e-13)
        ref2 = sum(correlate2d(g[0, co], w[co, ci, ::-1, ::-1], mode="same") for co in range(3))
        assert np.allclose(dx[0, ci], ref2, rtol=1e-13, atol=1e-13)


def test_pool_and_leaky_pointwise(oracle):
    rs = np.random.RandomState(2)
    x = _rand(rs, (2, 3, 6, 8))
    y, arg = oracle.pool_fwd(x)
    ref = x.reshape(2, 3, 3, 2, 4, 2).transpose(0, 1, 2, 4, 3, 5).reshape(2, 3, 3, 4, 4)
    assert np.array_equal(y, ref.max(axis=-1))
    assert np.array_equal(arg, ref.argmax(axis=-1))       # numpy argmax = first maximum
    g = _rand(rs, y.shape)
    dx = oracle.pool_bwd(g, arg, (6, 8))
    win = dx.reshape(2, 3, 3, 2, 4, 2).transpose(0, 1, 2, 4, 3, 5).reshape(2, 3, 3, 4, 4)
    assert np.array_equal((win != 0).sum(axis=-1), np.ones_like(arg))
    assert np.array_equal(win.sum(axis=-1), g)
    # ties: the first maximum in window order wins
    t = np.zeros((1, 1, 2, 2))
    _, a = oracle.pool_fwd(t)
    assert a[0, 0, 0, 0] == 0
    t[0, 0, 0, 1] = t[0, 0, 1, 0] = 1.0
    _, a = oracle.pool_fwd(t)
    assert a[0, 0, 0, 0] == 1
    z = np.array([-2.0, -0.0, 0.0, 3.0])
    yv = oracle.leaky_fwd(z, 0.1)
    assert np.allclose(yv, [-0.2, 0.0, 0.0, 3.0])
    assert np.allclose(oracle.leaky_bwd(np.ones(4), yv, 0.1), [0.1, 0.1, 0.1, 1.0])


def test_against_torch_cpu_autograd(oracle):
    """Library pin: torch's CPU conv2d / leaky_relu / max_pool2d and its autograd, in fp64."""
    torch = pytest.importorskip("torch")
    import torch.nn.functional as F
    rs = np.random.RandomState(13)
    layers = [conv(3, 6), pool(6), conv(6, 8), conv(8, 4, 1), pool(4), conv(4, 5)]
    x = _rand(rs, (2, 3, 16, 12))
    ws = _weights(rs, layers)
    bs = [None if w is None else _rand(rs, (w.shape[0],)) * 0.1 for w in ws]
    acts, args = oracle.forward(layers, x, ws, bs)
    g = _rand(rs, acts[-1].shape)
    dx, dws, dbs, deltas = oracle.backward(layers, acts, args, ws, g, keep_deltas=True)

    tx = torch.tensor(x, requires_grad=True)
    tws = [None if w is None else torch.tensor(w, requires_grad=True) for w in ws]
    tbs = [None if b is None else torch.tensor(b, requires_grad=True) for b in bs]
    t = tx
    tacts = [t]
    for l, ly in enumerate(layers):
        if ly.kind == CONV:
            t = F.leaky_relu(F.conv2d(t, tws[l], tbs[l], stride=1, padding=ly.pad), ly.slope)
        else:
            t = F.max_pool2d(t, 2, 2)
        t.retain_grad()
        tacts.append(t)
    (t * torch.tensor(g)).sum().backward()
    for l in range(len(layers) + 1):
        assert np.allclose(acts[l], tacts[l].detach().numpy(), rtol=1e-12, atol=1e-12), l
    assert np.allclose(dx, tx.grad.numpy(), rtol=1e-11, atol=1e-12)
    for l in range(1, len(layers) + 1):
        assert np.allclose(deltas[l], tacts[l].grad.numpy(), rtol=1e-11, atol=1e-12), l
    for l, ly in enumerate(layers):
        if ly.kind == CONV:
            assert np.allclose(dws[l], tws[l].grad.numpy(), rtol=1e-11, atol=1e-12), l
            assert np.allclose(dbs[l], tbs[l].grad.numpy(), rtol=1e-11, atol=1e-12), l


def test_fp32_mode_rounds_fp64_result_once(oracle):
    """fp32 tensors + fp64 accumulators: each op equals the fp64 op on the same values, rounded once."""
    rs = np.random.RandomState(17)
    x = _rand(rs, (2, 3, 9, 10), np.float32)
    w = (_rand(rs, (4, 3, 3, 3), np.float32) * 0.3).astype(np.float32)
    b = _rand(rs, (4,), np.float32)
    z32 = oracle.conv_fwd(x, w, b, 1, 1)
    z64 = oracle.conv_fwd(x.astype(np.float64), w.astype(np.float64), b.astype(np.float64), 1, 1)
    assert z32.dtype == np.float32 and np.array_equal(z32, z64.astype(np.float32))
    g = _rand(rs, z32.shape, np.float32)
    d32 = oracle.conv_bwd_data(g, w, (9, 10), 1, 1)
    d64 = oracle.conv_bwd_data(g.astype(np.float64), w.astype(np.float64), (9, 10), 1, 1)
    assert np.array_equal(d32, d64.astype(np.float32))
    w32, b32 = oracle.conv_bwd_weight(x, g, 3, 1, 1)
    w64, b64 = oracle.conv_bwd_weight(x.astype(np.float64), g.astype(np.float64), 3, 1, 1)
    assert np.array_equal(w32, w64.astype(np.float32)) and np.array_equal(b32, b64.astype(np.float32))


def test_batch_sum_and_tile_partial_sums(oracle):
    """dW of a batch = sum of per-image dW (one update per batch); the filter-gradient partial sums of
    a disjoint cover of the output pixels add up to the whole gradient (Sec. 4.1)."""
    rs = np.random.RandomState(19)
    x = _rand(rs, (3, 2, 8, 10))
    g = _rand(rs, (3, 4, 8, 10))
    full, fullb = oracle.conv_bwd_weight(x, g, 3, 1, 1)
    per = sum(oracle.conv_bwd_weight(x[n:n + 1].copy(), g[n:n + 1].copy(), 3, 1, 1)[0] for n in range(3))
    assert np.allclose(full, per, rtol=1e-12, atol=1e-12)
    parts, partb = 0.0, 0.0
    for (y0, y1) in ((0, 2), (3, 7)):
        for (x0, x1) in ((0, 3), (4, 4), (5, 9)):
            dw, db = oracle.conv_bwd_weight(x, g, 3, 1, 1, rect=(x0, y0, x1, y1))
            parts, partb = parts + dw, partb + db
    assert np.allclose(full, parts, rtol=1e-12, atol=1e-12)
    assert np.allclose(fullb, partb, rtol=1e-12, atol=1e-12)


def test_bf16_rounding(oracle):
    from ftp_synth import rng
    a = np.array([1.0, 1.00390625, 1.01171875, 3.14159, -2.71828, 1e-30, 65504.0], dtype=np.float32)
    r = oracle.round_bf16(a.copy())
    assert np.array_equal(r, rng.to_bf16_rne(a))
    assert r[1] == 1.0 and r[2] == np.float32(1.015625)     # ties go to the even mantissa


# ---- general geometry: strided convolutions, K = 5 and 7, pools on odd maps (Eq. (1)/(2) are stated for any K_l, S_l) ----

def _net_general():
    return [conv(3, 4, 5, stride=2), pool(4), conv(4, 5, 3, stride=2), conv(5, 3, 7), pool(3), conv(3, 2, 1, stride=2)]


def test_general_geometry_finite_differences_fp64(oracle):
    """Central differences through strided / 5x5 / 7x7 convolutions and pools on odd maps (19 -> 10 -> 5 -> 3 -> 3 -> 1 -> 1)."""
    rs = np.random.RandomState(23)
    layers = _net_general()
    x = _rand(rs, (2, 3, 19, 21))
    ws = _weights(rs, layers)
    bs = [None if w is None else _rand(rs, (w.shape[0],)) * 0.1 for w in ws]
    acts, args = oracle.forward(layers, x, ws, bs)
    assert [a.shape[2:] for a in acts] == [(19, 21), (10, 11), (5, 5), (3, 3), (3, 3), (1, 1), (1, 1)]
    g = _rand(rs, acts[-1].shape)
    for l, ly in enumerate(layers):
        if ly.kind == CONV:
            assert np.abs(acts[l + 1]).min() > 1e-5
    dx, dws, dbs = oracle.backward(layers, acts, args, ws, g)
    eps, checked = 1e-6, 0
    for (arr, grad) in [(x, dx)] + [(ws[l], dws[l]) for l in range(len(layers)) if ws[l] is not None] \
            + [(bs[l], dbs[l]) for l in range(len(layers)) if bs[l] is not None]:
        flat, gflat = arr.reshape(-1), grad.reshape(-1)
        for idx in rs.choice(flat.size, size=min(25, flat.size), replace=False):
            old = flat[idx]
            flat[idx] = old + eps
            lp = _loss(oracle, layers, x, ws, bs, g)
            flat[idx] = old - eps
            lm = _loss(oracle, layers, x, ws, bs, g)
            flat[idx] = old
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - gflat[idx]) <= 1e-6 * max(1.0, abs(fd)), (idx, fd, gflat[idx])
            checked += 1
    assert checked > 100


@pytest.mark.parametrize("k", [1, 3, 5, 7])
@pytest.mark.parametrize("stride", [1, 2])
def test_general_geometry_adjoints_fp64(oracle, k, stride):
    """Linear layer (slope 1): <G, A x> == <A^T G, x> == <dW, W> for every kernel size and stride, odd and even maps."""
    rs = np.random.RandomState(100 + 10 * k + stride)
    for (h, w) in ((8, 11), (9, 6)):
        ly = Layer(CONV, k, stride, k // 2, 2, 3, 1.0)
        x = _rand(rs, (2, 2, h, w))
        wt = _rand(rs, (3, 2, k, k))
        acts, args = oracle.forward([ly], x, [wt], None)
        assert acts[-1].shape[2:] == ((h - 1) // stride + 1, (w - 1) // stride + 1)
        g = _rand(rs, acts[-1].shape)
        dx, dws, _ = oracle.backward([ly], acts, args, [wt], g)
        lhs = np.sum(g * acts[-1])
        assert abs(lhs - np.sum(dx * x)) <= 1e-12 * abs(lhs)
        assert abs(lhs - np.sum(dws[0] * wt)) <= 1e-12 * abs(lhs)


@pytest.mark.parametrize("k", [3, 5, 7])
def test_strided_conv_is_subsampled_scipy_correlate(oracle, k):
    """A stride-2 convolution is the stride-1 'same' correlation kept at every second position."""
    from scipy.signal import correlate2d
    rs = np.random.RandomState(31 + k)
    x = _rand(rs, (1, 2, 11, 8))
    w = _rand(rs, (3, 2, k, k))
    z1 = oracle.conv_fwd(x, w, None, 1, k // 2)
    z2 = oracle.conv_fwd(x, w, None, 2, k // 2)
    for co in range(3):
        ref = sum(correlate2d(x[0, ci], w[co, ci], mode="same") for ci in range(2))
        assert np.allclose(z1[0, co], ref, rtol=1e-13, atol=1e-13)
        assert np.allclose(z2[0, co], ref[::2, ::2], rtol=1e-13, atol=1e-13)
    # the adjoint of subsampling is zero insertion: strided delta back-propagation = stride-1 one of the upsampled delta
    g = _rand(rs, z2.shape)
    up = np.zeros_like(z1)
    up[:, :, ::2, ::2] = g
    assert np.allclose(oracle.conv_bwd_data(g, w, (11, 8), 2, k // 2), oracle.conv_bwd_data(up, w, (11, 8), 1, k // 2),
                       rtol=1e-13, atol=1e-13)
    dw2, db2 = oracle.conv_bwd_weight(x, g, k, 2, k // 2)
    dw1, db1 = oracle.conv_bwd_weight(x, up, k, 1, k // 2)
    assert np.allclose(dw2, dw1, rtol=1e-13, atol=1e-13) and np.allclose(db2, db1, rtol=1e-13, atol=1e-13)


def test_strided_all_ones_closed_form(oracle):
    """All-ones 7x7 input, 5x5 filter of ones, stride 2, pad 2: Z[o] = (rows covered) x (columns covered) x Cin."""
    x = np.ones((1, 2, 7, 7))
    w = np.ones((1, 2, 5, 5))
    z = oracle.conv_fwd(x, w, None, 2, 2)
    cover = np.array([3, 5, 5, 3])                       # taps of [2o-2, 2o+2] that fall inside [0, 6]
    assert np.array_equal(z[0, 0], 2.0 * np.outer(cover, cover))


def test_pool_on_odd_map_drops_last_row_and_column(oracle):
    rs = np.random.RandomState(41)
    x = _rand(rs, (1, 2, 7, 5))
    y, arg = oracle.pool_fwd(x)
    y2, arg2 = oracle.pool_fwd(np.ascontiguousarray(x[:, :, :6, :4]))
    assert y.shape == (1, 2, 3, 2) and np.array_equal(y, y2) and np.array_equal(arg, arg2)
    g = _rand(rs, y.shape)
    dx = oracle.pool_bwd(g, arg, (7, 5))
    assert np.all(dx[:, :, 6, :] == 0) and np.all(dx[:, :, :, 4] == 0)
    assert np.array_equal(dx[:, :, :6, :4], oracle.pool_bwd(g, arg, (6, 4)))


def test_general_geometry_against_torch_cpu_autograd(oracle):
    """Library pin for strides, 5x5 / 7x7 kernels and floor-mode pools on odd maps."""
    torch = pytest.importorskip("torch")
    import torch.nn.functional as F
    rs = np.random.RandomState(43)
    layers = [conv(3, 6, 7, stride=2), pool(6), conv(6, 8, 5), conv(8, 4, 3, stride=2), pool(4), conv(4, 5, 1, stride=2)]
    x = _rand(rs, (2, 3, 37, 30))
    ws = _weights(rs, layers)
    bs = [None if w is None else _rand(rs, (w.shape[0],)) * 0.1 for w in ws]
    acts, args = oracle.forward(layers, x, ws, bs)
    g = _rand(rs, acts[-1].shape)
    dx, dws, dbs, deltas = oracle.backward(layers, acts, args, ws, g, keep_deltas=True)
    tx = torch.tensor(x, requires_grad=True)
    tws = [None if w is None else torch.tensor(w, requires_grad=True) for w in ws]
    tbs = [None if b is None else torch.tensor(b, requires_grad=True) for b in bs]
    t, tacts = tx, [tx]
    for l, ly in enumerate(layers):
        if ly.kind == CONV:
            t = F.leaky_relu(F.conv2d(t, tws[l], tbs[l], stride=ly.stride, padding=ly.pad), ly.slope)
        else:
            t = F.max_pool2d(t, 2, 2)
        t.retain_grad()
        tacts.append(t)
    (t * torch.tensor(g)).sum().backward()
    for l in range(len(layers) + 1):
        assert acts[l].shape == tuple(tacts[l].shape), l
        assert np.allclose(acts[l], tacts[l].detach().numpy(), rtol=1e-12, atol=1e-12), l
    assert np.allclose(dx, tx.grad.numpy(), rtol=1e-11, atol=1e-12)
    for l in range(1, len(layers) + 1):
        assert np.allclose(deltas[l], tacts[l].grad.numpy(), rtol=1e-11, atol=1e-12), l
    for l, ly in enumerate(layers):
        if ly.kind == CONV:
            assert np.allclose(dws[l], tws[l].grad.numpy(), rtol=1e-11, atol=1e-12), l
            assert np.allclose(dbs[l], tbs[l].grad.numpy(), rtol=1e-11, atol=1e-12), l


def test_bf16_storage_branch_layer_by_layer_with_torch(oracle):
    """Pin of the reduced-precision storage branch (bf16_store=True): the network re-derived one layer at a time with
    torch's fp64 conv2d / max_pool2d and its autograd, rounding to bf16 with the input generator's own rounding routine
    exactly where a map is stored: every activation after its leaky ReLU (pools pick among stored values), every
    delta dLoss/dX once it leaves a layer; dZ = dY * leaky' and the filter gradients are not stored as bf16."""
    torch = pytest.importorskip("torch")
    import torch.nn.functional as F
    from ftp_synth import rng

    rs = np.random.RandomState(11)
    layers = [conv(3, 6), pool(6), conv(6, 8), conv(8, 4, 1), pool(4), conv(4, 5)]
    x = rng.to_bf16_rne(rs.uniform(0, 1, (2, 3, 24, 20)).astype(np.float32))
    ws = [None if ly.kind != CONV else
          rng.to_bf16_rne((rs.standard_normal((ly.cout, ly.cin, ly.k, ly.k)) * np.sqrt(2.0 / (ly.cin * ly.k * ly.k))).astype(np.float32))
          for ly in layers]
    acts, args = oracle.forward(layers, x, ws, None, bf16_store=True)
    g = rng.to_bf16_rne(rs.standard_normal(acts[-1].shape).astype(np.float32))
    dx, dws, _ = oracle.backward(layers, acts, args, ws, g, bf16_store=True, want_db=False)
    # every stored map holds bf16 values, and storing in bf16 really changes the result
    for a in acts:
        assert np.array_equal(rng.to_bf16_rne(a), a)
    acts_plain, _ = oracle.forward(layers, x, ws, None, bf16_store=False)
    assert not np.array_equal(acts_plain[-1], acts[-1])

    slope32 = np.float32(0.1)
    # forward
    t_acts, t_arg = [x], [None] * len(layers)
    for l, ly in enumerate(layers):
        a = torch.tensor(t_acts[-1].astype(np.float64))
        if ly.kind == CONV:
            z = F.conv2d(a, torch.tensor(ws[l].astype(np.float64)), None, ly.stride, ly.pad).numpy().astype(np.float32)
            y = np.where(z > 0, z, slope32 * z).astype(np.float32)           # leaky in the storage precision's fp32
            t_acts.append(rng.to_bf16_rne(y))
        else:
            y, ind = F.max_pool2d(a, 2, 2, return_indices=True)
            t_acts.append(y.numpy().astype(np.float32))
            t_arg[l] = ind
    for l in range(len(layers) + 1):
        assert np.array_equal(t_acts[l], acts[l]), ("stored activation", l)
    # backward
    tg = g
    for l in range(len(layers) - 1, -1, -1):
        ly = layers[l]
        if ly.kind == CONV:
            dz = np.where(t_acts[l + 1] > 0, tg, slope32 * tg).astype(np.float32)      # kept in fp32, not stored as bf16
            a = torch.tensor(t_acts[l].astype(np.float64), requires_grad=True)
            w = torch.tensor(ws[l].astype(np.float64), requires_grad=True)
            (F.conv2d(a, w, None, ly.stride, ly.pad) * torch.tensor(dz.astype(np.float64))).sum().backward()
            dw = w.grad.numpy().astype(np.float32)
            scale = np.abs(dw).max()
            assert np.max(np.abs(dw - dws[l])) <= 2e-7 * scale, ("filter gradient", l)       # fp64 sums rounded to fp32 once
            assert not np.array_equal(rng.to_bf16_rne(dws[l]), dws[l])
            tg = rng.to_bf16_rne(a.grad.numpy().astype(np.float32))
        else:
            a = torch.tensor(t_acts[l].astype(np.float64), requires_grad=True)
            (F.max_pool2d(a, 2, 2) * torch.tensor(tg.astype(np.float64))).sum().backward()
            tg = rng.to_bf16_rne(a.grad.numpy().astype(np.float32))
    assert np.array_equal(tg, dx)
    # the same with the rounding of the deltas left out is a different result (the pin sees that rounding)
    dx_plain, _, _ = oracle.backward(layers, acts, args, ws, g, bf16_store=False, want_db=False)
    assert not np.array_equal(dx_plain, dx)
