"""ctypes front end of the CPU oracle plus the layer-by-layer network driver.

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the benchmark's
cpu_baseline leg.  The GPU library never imports or calls this module.

The network is evaluated untiled, one primitive layer at a time, on whole maps:
that is the result the tiled/fused/grouped evaluation has to reproduce exactly
up to rounding order (Sec. 1: no loss of accuracy; Sec. 4.1: partial filter
gradients of the tiles add up to the full gradient).

A layer is any object with attributes kind (0 = convolution with leaky-ReLU,
1 = 2x2/2 max-pool), k, stride, pad, cin, cout, slope.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

CONV, MAXPOOL = 0, 1


def lib():
    global _LIB
    if _LIB is None:
        path = os.path.join(_HERE, "libftp_oracle.so")
        if not os.path.exists(path):
            from . import build as _b
            _b.build()
        _LIB = ctypes.CDLL(path)
        _LIB.oracle_num_threads.restype = ctypes.c_int
    return _LIB


def num_threads():
    return int(lib().oracle_num_threads())


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p) if a is not None else None


def _fn(name, dtype):
    return getattr(lib(), "oracle_%s_%s" % ("f64" if dtype == np.float64 else "f32", name))


def _chk(a, dtype):
    assert a.dtype == dtype and a.flags["C_CONTIGUOUS"], (a.dtype, dtype)
    return a


def conv_fwd(x, w, b, stride, pad):
    dt = x.dtype.type
    n, cin, h, wd = x.shape
    cout, cin2, k, _ = w.shape
    assert cin == cin2
    ho, wo = (h + 2 * pad - k) // stride + 1, (wd + 2 * pad - k) // stride + 1
    z = np.empty((n, cout, ho, wo), dtype=dt)
    _fn("conv_fwd", dt)(_p(_chk(x, dt)), _p(_chk(w, dt)), _p(None if b is None else _chk(b, dt)), _p(z),
                        n, cin, h, wd, cout, k, stride, pad)
    return z


def conv_bwd_data(dz, w, in_hw, stride, pad):
    dt = dz.dtype.type
    n, cout, ho, wo = dz.shape
    cout2, cin, k, _ = w.shape
    h, wd = in_hw
    assert cout == cout2 and ho == (h + 2 * pad - k) // stride + 1 and wo == (wd + 2 * pad - k) // stride + 1
    dx = np.empty((n, cin, h, wd), dtype=dt)
    _fn("conv_bwd_data", dt)(_p(_chk(dz, dt)), _p(_chk(w, dt)), _p(dx), n, cin, h, wd, cout, k, stride, pad)
    return dx


def conv_bwd_weight(x, dz, k, stride, pad, rect=None, want_db=True):
    """rect = inclusive (ox0, oy0, ox1, oy1) of output pixels to sum over; None = whole map."""
    dt = x.dtype.type
    n, cin, h, wd = x.shape
    _, cout, ho, wo = dz.shape
    if rect is None:
        rect = (0, 0, wo - 1, ho - 1)
    ox0, oy0, ox1, oy1 = rect
    assert 0 <= ox0 and ox1 < wo and 0 <= oy0 and oy1 < ho
    dw = np.empty((cout, cin, k, k), dtype=dt)
    db = np.empty((cout,), dtype=dt) if want_db else None
    _fn("conv_bwd_weight", dt)(_p(_chk(x, dt)), _p(_chk(dz, dt)), _p(dw), _p(db),
                               n, cin, h, wd, cout, k, stride, pad, oy0, oy1, ox0, ox1)
    return dw, db


def leaky_fwd(z, slope):
    dt = z.dtype.type
    y = np.empty_like(z)
    _fn("leaky_fwd", dt)(_p(_chk(z, dt)), _p(y), ctypes.c_size_t(z.size), ctypes.c_double(slope))
    return y


def leaky_bwd(g, y, slope):
    dt = g.dtype.type
    dz = np.empty_like(g)
    _fn("leaky_bwd", dt)(_p(_chk(g, dt)), _p(_chk(y, dt)), _p(dz), ctypes.c_size_t(g.size), ctypes.c_double(slope))
    return dz


def pool_fwd(x):
    dt = x.dtype.type
    n, c, h, w = x.shape
    y = np.empty((n, c, h // 2, w // 2), dtype=dt)
    arg = np.empty((n, c, h // 2, w // 2), dtype=np.uint8)
    _fn("pool_fwd", dt)(_p(_chk(x, dt)), _p(y), _p(arg), n * c, h, w)
    return y, arg


def pool_bwd(g, arg, in_hw):
    dt = g.dtype.type
    n, c, ho, wo = g.shape
    h, w = in_hw
    dx = np.empty((n, c, h, w), dtype=dt)
    _fn("pool_bwd", dt)(_p(_chk(g, dt)), _p(_chk(arg, np.uint8)), _p(dx), n * c, h, w)
    return dx


def round_bf16(a):
    """In place: nearest-even rounding of fp32 values to bf16 precision."""
    assert a.dtype == np.float32 and a.flags["C_CONTIGUOUS"]
    lib().oracle_round_bf16(_p(a), ctypes.c_size_t(a.size))
    return a


def forward(layers, x, weights, biases=None, bf16_store=False):
    """Returns (acts, args): acts[l] = map at boundary l (acts[0] = x), args[l] = pool argmax of layer l.

    bf16_store: round every stored activation to bf16 (the reduced-precision storage variant;
    accumulation stays fp64 here).
    """
    acts, args = [np.ascontiguousarray(x)], [None] * len(layers)
    for l, ly in enumerate(layers):
        a = acts[-1]
        if ly.kind == CONV:
            b = None if biases is None else biases[l]
            z = conv_fwd(a, weights[l], b, ly.stride, ly.pad)
            y = leaky_fwd(z, ly.slope)
            if bf16_store:
                round_bf16(y)
        else:
            y, args[l] = pool_fwd(a)
        acts.append(y)
    return acts, args


def backward(layers, acts, args, weights, dy, rect_of_layer=None, bf16_store=False, want_db=True,
             keep_deltas=False):
    """Back-propagation through the list of primitive layers.

    Returns (dx, dws, dbs[, deltas]); dws[l]/dbs[l] are None for pool layers.
    rect_of_layer(l) -> inclusive (ox0, oy0, ox1, oy1) restricts the filter-gradient sum of
    convolution l to those output pixels (one tile's partial sum); the delta chain is unaffected.
    deltas[l] = dLoss/d(map at boundary l).
    """
    L = len(layers)
    g = np.ascontiguousarray(dy)
    dws, dbs = [None] * L, [None] * L
    deltas = [None] * (L + 1)
    deltas[L] = g
    for l in range(L - 1, -1, -1):
        ly = layers[l]
        h, w = acts[l].shape[2], acts[l].shape[3]
        if ly.kind == CONV:
            dz = leaky_bwd(g, acts[l + 1], ly.slope)
            rect = None if rect_of_layer is None else rect_of_layer(l)
            dws[l], dbs[l] = conv_bwd_weight(acts[l], dz, ly.k, ly.stride, ly.pad, rect, want_db)
            g = conv_bwd_data(dz, weights[l], (h, w), ly.stride, ly.pad)
        else:
            g = pool_bwd(g, args[l], (h, w))
        if bf16_store:
            round_bf16(g)
        if keep_deltas:
            deltas[l] = g
    if keep_deltas:
        return g, dws, dbs, deltas
    return g, dws, dbs


def flat_params(layers, dws, dbs=None, has_bias=False):
    """Concatenation over convolution layers in layer order: filters, then (if any) biases."""
    parts = []
    for l, ly in enumerate(layers):
        if ly.kind == CONV:
            parts.append(dws[l].ravel())
            if has_bias:
                parts.append(dbs[l].ravel())
    return np.concatenate(parts)
