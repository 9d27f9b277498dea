"""GPU parity of the whole training cycle (Sec. 4.1: forward, back-propagation, gradient sum, filter update):
ftp_sgd_step against the oracle's gradients, and two cycles in a row against the oracle run with its own
updated filters."""
import numpy as np
import pytest

from ftp_synth import configs as C
from ftp_synth.configs import Config, conv, pool
from tests import parity as P

pytestmark = pytest.mark.gpu

_LAYERS = (conv(3, 8), pool(8), conv(8, 16), conv(16, 8, 1), pool(8), conv(8, 12))


def _cfg(dtype="f32", grouping=(3, 6)):
    return Config("cycle", 2, 3, 48, 40, _LAYERS, (2, 3), grouping, dtype)


def _lr_for(ws, dws):
    """A step that changes the filters by about 5 % of their largest entry."""
    wmax = max(float(np.abs(w).max()) for w in ws if w is not None)
    gmax = max(float(np.abs(g).max()) for g in dws if g is not None)
    return np.float32(0.05 * wmax / gmax)


@pytest.mark.parametrize("has_bias", [False, True])
def test_sgd_step_on_given_state(oracle, has_bias):
    """W <- W - lr * dW with the oracle's decisions imported: (W_old - W_new) / lr equals the oracle's dW, the
    gradient the fused kernel reports equals ftp_reduce_wgrad bit for bit."""
    import torch
    cfg = _cfg()
    x, ws, bs, dy = C.make_tensors(cfg)
    if has_bias:
        bs = [None if b is None else C.rng.normal("b/%d" % l, b.shape, 0.2, C.rng.MASTER_SEED) for l, b in enumerate(bs)]
    acts, args, dx, dws, dbs = P.oracle_run(oracle, cfg, x, ws, bs if has_bias else None, dy, want_db=has_bias)
    lr = _lr_for(ws, dws)
    s = P.make_session(cfg, x.shape[0], has_bias)
    s.load(x=x, weights=ws, dy=dy, biases=bs if has_bias else None)
    s.forward()
    P.import_forward_state(s, cfg, acts, args)
    s.backward()
    s.reduce()
    torch.cuda.synchronize()
    reduced = s.to_np(s.wgrad).copy()
    s.wgrad.zero_()
    s.sgd_step(float(lr))
    torch.cuda.synchronize()
    assert np.array_equal(s.to_np(s.wgrad), reduced)          # same summation order in both kernels
    for l, ly in enumerate(cfg.layers):
        if ws[l] is None:
            continue
        w_new = s.to_np(s.weights[l])
        step = (ws[l].astype(np.float64) - w_new.astype(np.float64)) / float(lr)
        # the subtraction rounds at the magnitude of W: allow that on top of the gradient tolerance
        slack = np.finfo(np.float32).eps * float(np.abs(ws[l]).max()) / float(lr)
        assert np.max(np.abs(step - dws[l])) <= P.TOL_GRAD_F32 * float(np.abs(dws[l]).max()) + 2 * slack, ("dW step", l)
        if has_bias:
            b_new = s.to_np(s.biases[l])
            stepb = (bs[l].astype(np.float64) - b_new.astype(np.float64)) / float(lr)
            slack = np.finfo(np.float32).eps * float(np.abs(bs[l]).max()) / float(lr)
            assert np.max(np.abs(stepb - dbs[l])) <= P.TOL_GRAD_F32 * float(np.abs(dbs[l]).max()) + 2 * slack, ("db step", l)
    s.close()


def test_two_training_cycles(oracle):
    """Two cycles on the same batch with L = <dy, y>: the GPU's second forward pass equals the oracle's forward pass
    with the oracle's own updated filters, and the loss went down by about lr * |dW|^2."""
    import torch
    cfg = _cfg()
    x, ws, bs, dy = C.make_tensors(cfg)
    acts, args, dx, dws, dbs = P.oracle_run(oracle, cfg, x, ws, None, dy)
    lr = np.float32(0.04) * _lr_for(ws, dws)          # small enough for the first-order estimate below
    ws1 = [None if w is None else (w - lr * dws[l].astype(np.float32)).astype(np.float32) for l, w in enumerate(ws)]
    acts1, _ = oracle.forward(cfg.layers, x, ws1, None, bf16_store=False)

    s = P.make_session(cfg, x.shape[0])
    s.load(x=x, weights=ws, dy=dy)
    s.forward()
    torch.cuda.synchronize()
    y0 = s.to_np(s.y)
    agree = P.decisions_agree(s, cfg, acts, args)
    s.backward()
    s.sgd_step(float(lr))
    s.forward()
    torch.cuda.synchronize()
    y1 = s.to_np(s.y)
    loss0, loss1 = float(np.sum(dy.astype(np.float64) * y0)), float(np.sum(dy.astype(np.float64) * y1))
    gnorm2 = sum(float(np.sum(g.astype(np.float64) ** 2)) for g in dws if g is not None)
    assert loss1 < loss0
    assert abs((loss0 - loss1) - float(lr) * gnorm2) <= 0.25 * float(lr) * gnorm2      # first order, small step
    if agree:
        # both sides took the same decisions in the first cycle, so their filters agree to the gradient tolerance
        assert P.rel_inf(y1, acts1[-1]) <= 10 * P.TOL_ACT_F32
    s.close()


def test_sgd_step_bf16(oracle):
    """bf16 storage: the updated filter is the fp32 result rounded to bf16 (nearest even)."""
    import torch
    cfg = _cfg("bf16")
    x, ws, bs, dy = C.make_tensors(cfg)
    s = P.make_session(cfg, x.shape[0])
    s.load(x=x, weights=ws, dy=dy)
    s.step()
    torch.cuda.synchronize()
    g = s.to_np(s.wgrad)
    lr = np.float32(0.05) * np.float32(max(float(np.abs(w).max()) for w in ws if w is not None) / float(np.abs(g).max()))
    s.sgd_step(float(lr))
    torch.cuda.synchronize()
    for (l, a, b) in P.param_slices(cfg):
        want = C.rng.to_bf16_rne((ws[l].ravel() - lr * g[a:b]).astype(np.float32))
        got = s.to_np(s.weights[l]).ravel()
        # a fused multiply-add may round the fp32 intermediate differently: at most one bf16 step apart
        assert np.max(np.abs(got - want)) <= 2.0 ** -7 * float(np.abs(want).max()), l
    s.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_two_stream_backward_is_bit_identical(oracle, dtype):
    """ftp_set_overlap: the filter gradients on a second stream beside the delta back-propagation give the same bits
    (the same kernels in the same order per buffer), call after call, also through several groups and lone pools."""
    import torch
    layers = (conv(3, 16), pool(16), conv(16, 32), conv(32, 32, 1), pool(32), pool(32), conv(32, 48), conv(48, 32, 5), conv(32, 64, 3, stride=2))
    cfg = Config("overlap", 3, 3, 96, 80, layers, (2, 3), (3, 6, 9), dtype)
    x, ws, bs, dy = C.make_tensors(cfg)
    s = P.make_session(cfg, x.shape[0])
    s.load(x=x, weights=ws, dy=dy)
    s.step()
    torch.cuda.synchronize()
    ref = [t.clone() for t in (s.y, s.dx, s.wgrad, s.partials)]
    s.set_overlap(True)
    for _ in range(3):
        for t in (s.dx, s.wgrad, s.partials):
            t.fill_(float("nan"))
        s.step()
        torch.cuda.synchronize()
        for a, b in zip(ref, (s.y, s.dx, s.wgrad, s.partials)):
            assert torch.equal(a, b)
    s.set_overlap(False)
    s.step()
    torch.cuda.synchronize()
    for a, b in zip(ref, (s.y, s.dx, s.wgrad, s.partials)):
        assert torch.equal(a, b)
    s.close()
