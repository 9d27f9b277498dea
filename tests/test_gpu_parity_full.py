"""GPU parity at the full sizes of the five configurations, in the launch configuration bench.py times.

Configurations 1-3 are checked whole against the oracle.  The 16-layer stacks (configurations 4 and 5) are
checked twice: a 2-image batch of the same shape, grid and grouping through check_case (every grouping of the
sweep), and the full batch against the oracle run in chunks of 8 images: every kept map and decision of the
forward pass chunk by chunk, then ONE ftp_backward at the full batch whose dx is compared image by image and whose
filter gradient is compared with the fp64 sum of the chunks' oracle gradients (Sec. 4.1: partial sums add up;
Sec. 3: one update per batch).  Further properties that hold at any size tie batch sizes together: per-image
results do not depend on the batch they sit in, and the filter gradient is additive over the batch.
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


@pytest.mark.parametrize("g", [1, 2, 4, 8, 16])
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


def _full_batch_against_oracle(oracle, cfg, chunk=8):
    """The whole batch in the launch configuration bench.py times, against the oracle run chunk by chunk."""
    import torch
    bf = cfg.dtype == "bf16"
    tol_a, tol_g = (P.TOL_BF16, P.TOL_BF16) if bf else (P.TOL_ACT_F32, P.TOL_GRAD_F32)
    x, ws, bs, dy = C.make_tensors(cfg)
    s = P.make_session(cfg, cfg.batch)
    s.load(x=x, weights=ws, dy=dy)
    # chain: back-propagation through the GPU's own forward state
    s.step()
    torch.cuda.synchronize()
    chain_dx, chain_w = s.to_np(s.dx), s.to_np(s.wgrad)
    s.forward()                                   # (the state the checks below read is that of a forward pass)
    torch.cuda.synchronize()
    y = s.to_np(s.y)
    ref_dx = np.empty_like(x)
    ref_w = np.zeros(s.n_params, dtype=np.float64)
    flipped = total = 0
    for c0 in range(0, cfg.batch, chunk):
        idx = list(range(c0, min(cfg.batch, c0 + chunk)))
        acts, args = oracle.forward(cfg.layers, np.ascontiguousarray(x[idx]), ws, None, bf16_store=bf)
        assert P.rel_inf(y[idx], acts[-1]) <= tol_a, ("y", c0)
        P.check_forward_state(s, cfg, acts, args, tol_a, images=idx)
        f, t = P.decision_flips(s, cfg, acts, args, images=idx)
        flipped += f; total += t
        dxc, dws, _ = oracle.backward(cfg.layers, acts, args, ws, np.ascontiguousarray(dy[idx]), bf16_store=bf, want_db=False)
        ref_dx[idx] = dxc
        ref_w += P.flat_grad(cfg, dws).astype(np.float64)
        # oracle -> GPU: from here on this chunk's images carry the oracle's forward state
        P.import_forward_state(s, cfg, acts, args, images=idx)
        del acts, args, dws, dxc
    e_dx, e_w = P.rel_l2(chain_dx, ref_dx), P.rel_l2(chain_w, ref_w)
    print("full batch %s: %d of %d decisions flipped (%.3g %%), chain rel L2 error dx %.3g dW %.3g"
          % (cfg.name, flipped, total, 100.0 * flipped / total, e_dx, e_w))
    if flipped == 0:
        for n in range(cfg.batch):
            assert P.rel_inf(chain_dx[n], ref_dx[n]) <= tol_g, ("chain dx", n)
    else:
        bound = P.CHAIN_L2_BF16 if bf else P.CHAIN_L2_F32
        assert flipped <= max(4, P.CHAIN_MAX_FLIP_SHARE[bf] * total)
        assert e_dx <= bound and e_w <= bound, (e_dx, e_w)
    # given state: one back-propagation of the whole batch through the oracle's decisions, strict bars
    s.backward()
    s.reduce()
    torch.cuda.synchronize()
    got_dx, got_w = s.to_np(s.dx), s.to_np(s.wgrad)
    for n in range(cfg.batch):
        e = P.rel_inf(got_dx[n], ref_dx[n])
        assert e <= tol_g, ("dx of image", n, e)
    for (l, a, b) in P.param_slices(cfg):
        e = P.rel_inf(got_w[a:b], ref_w[a:b])
        assert e <= tol_g, ("dW of layer", l, e)
    s.close()


def test_config4_full_batch_oracle(oracle):
    _full_batch_against_oracle(oracle, C.config4())


def test_config5_full_batch_oracle(oracle):
    _full_batch_against_oracle(oracle, C.config5(4))
