"""GPU parity at the full sizes of the five configurations, in the launch configuration bench.py times.

Configurations 1-3 are checked whole against the oracle.  For the 16-layer stacks (configurations 4
and 5) the oracle checks a 2-image batch of the same shape, grid and grouping element by element; the
full batch is then tied to it by properties that hold at any size: sampled images of the full batch
equal the oracle's forward, per-image results do not depend on the batch they sit in, and the filter
gradient is additive over the batch (one update per batch, Sec. 3).
"""
import numpy as np
import pytest

from ftp_synth import configs as C
from tests import parity as P

pytestmark = pytest.mark.gpu


def test_config3_full(oracle):
    P.check_case(oracle, C.config3(), partial_check=False)


def test_config4_shape_two_images(oracle):
    P.check_case(oracle, C.config4().with_(batch=2), partial_check=False)


@pytest.mark.parametrize("g", [1, 4, 16])
def test_config5_shape_two_images(oracle, g):
    P.check_case(oracle, C.config5(g).with_(batch=2), partial_check=False)


def _full_batch_properties(oracle, cfg, sample):
    import torch
    bf = cfg.dtype == "bf16"
    tol_a = P.TOL_BF16 if bf else P.TOL_ACT_F32
    x, ws, bs, dy = C.make_tensors(cfg)
    s = P.make_session(cfg, cfg.batch)
    s.load(x=x, weights=ws, dy=dy)
    s.step()
    torch.cuda.synchronize()
    y_full = s.to_np(s.y[sample])
    dx_full = s.to_np(s.dx[sample])
    w_all = s.to_np(s.wgrad)
    # sampled images against the oracle's forward
    acts, _ = oracle.forward(cfg.layers, np.ascontiguousarray(x[sample]), ws, None, bf16_store=bf)
    assert P.rel_inf(y_full, acts[-1]) <= tol_a
    # additivity over the batch: dW(all) = dW(first half only) + dW(second half only)
    half = cfg.batch // 2
    dy_a = dy.copy(); dy_a[half:] = 0
    dy_b = dy.copy(); dy_b[:half] = 0
    parts = []
    for d in (dy_a, dy_b):
        s.load(dy=d)
        s.backward(); s.reduce()
        torch.cuda.synchronize()
        parts.append(s.to_np(s.wgrad))
    scale = np.abs(w_all).max()
    for (l, a, b) in P.param_slices(cfg):
        sc = np.abs(w_all[a:b]).max()
        assert np.max(np.abs(parts[0][a:b] + parts[1][a:b] - w_all[a:b])) <= (2e-3 if bf else 2e-5) * sc, l
    # only the sampled images carry a loss gradient: equals the 2-image batch of the same images
    dy_s = np.zeros_like(dy); dy_s[sample] = dy[sample]
    s.load(dy=dy_s)
    s.backward(); s.reduce()
    torch.cuda.synchronize()
    w_s = s.to_np(s.wgrad)
    s.close()
    del s
    torch.cuda.empty_cache()
    s2 = P.make_session(cfg, len(sample))
    s2.load(x=np.ascontiguousarray(x[sample]), weights=ws, dy=np.ascontiguousarray(dy[sample]))
    s2.step()
    torch.cuda.synchronize()
    # the same images in a batch of another size: other launch shapes, same summation order
    assert P.rel_inf(s2.to_np(s2.y), y_full) <= 1e-6
    assert P.rel_inf(s2.to_np(s2.dx), dx_full) <= (1e-3 if bf else 1e-5)
    w2 = s2.to_np(s2.wgrad)
    for (l, a, b) in P.param_slices(cfg):
        assert P.rel_inf(w_s[a:b], w2[a:b]) <= (2e-3 if bf else 2e-5), l
    s2.close()


def test_config4_full_batch(oracle):
    _full_batch_properties(oracle, C.config4(), [0, 63])


def test_config5_full_batch(oracle):
    _full_batch_properties(oracle, C.config5(4), [0, 31])
