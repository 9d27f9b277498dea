"""ftp_forward_static (the entry point that allocates nothing: its workspace is a fixed array inside the library's
device image) against ftp_forward, through the C ABI: bit-identical outputs on two calls in a row, the second with a
smaller input, and a clear error for plans beyond the array's size."""
import numpy as np
import pytest

from ftp_synth import configs as C
from ftp_synth.configs import Config, conv, pool
from tests import parity as P

pytestmark = pytest.mark.gpu


def _both_ways(cfg):
    import torch
    import paper_2409_09083_amd as F
    x, ws, bs, dy = C.make_tensors(cfg)
    s = P.make_session(cfg, cfg.batch)
    assert s.sizes["workspace_bytes"] <= F.FTP_STATIC_WORKSPACE_BYTES
    s.load(x=x, weights=ws, dy=dy)
    s.forward()
    torch.cuda.synchronize()
    want = s.to_np(s.y)
    s.y.zero_()
    before = torch.cuda.memory_allocated()
    F.ftp_forward_static(s.plan, s.x.data_ptr(), s._wptrs(), s._bptrs(), s.y.data_ptr(), s._stream())
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    got = s.to_np(s.y)
    s.close()
    return want, got


def test_forward_static_matches_forward_twice_and_rejects_large_plans(oracle):
    import paper_2409_09083_amd as F
    big = C.config2(True)                                     # 416 x 416, batch 1: 36.6 MiB of workspace
    want, got = _both_ways(big)
    assert np.array_equal(want, got)
    acts, _ = oracle.forward(big.layers, C.make_tensors(big)[0], C.make_tensors(big)[1])
    assert P.rel_inf(got, acts[-1]) <= P.TOL_ACT_F32
    # a smaller input right after it: the array still holds the previous call's maps
    layers = (conv(3, 8), pool(8), conv(8, 16), conv(16, 8, 1), pool(8), conv(8, 12))
    small = Config("static_small", 2, 3, 48, 40, layers, (3, 2), (3, 6))
    want, got = _both_ways(small)
    assert np.array_equal(want, got)
    # the bfloat path too
    want, got = _both_ways(small.with_(dtype="bf16", grid=(2, 2)))
    assert np.array_equal(want, got)
    # beyond the array: rejected before anything is launched
    c3 = C.config3()
    s = P.make_session(c3, c3.batch)
    assert s.sizes["workspace_bytes"] > F.FTP_STATIC_WORKSPACE_BYTES
    with pytest.raises(F.binding.FtpError) as ei:
        F.ftp_forward_static(s.plan, s.x.data_ptr(), [1] * len(c3.layers), None, s.y.data_ptr(), 0)
    assert ei.value.code == F.FTP_ETOOLARGE and "FTP_STATIC_WORKSPACE_BYTES" in str(ei.value)
    s.close()
