"""GPU parity, small cases: libftp through the C ABI against the CPU oracle, element by element,
on shapes that span several tiles, ragged tails, every grouping and both storage types."""
import numpy as np
import pytest

from ftp_synth import configs as C
from ftp_synth.configs import Config, conv, pool
from tests import parity as P

pytestmark = pytest.mark.gpu


def test_tiny_config(oracle):
    P.check_case(oracle, C.tiny())


_NETS = {
    "convs": ((conv(3, 8), conv(8, 16), conv(16, 8, 1), conv(8, 12)), 40, 36),
    "pools": ((conv(3, 8), pool(8), conv(8, 16), conv(16, 8, 1), pool(8), conv(8, 12)), 48, 40),
    "poolfirst": ((pool(3), conv(3, 6), pool(6), pool(6), conv(6, 10), conv(10, 4, 1)), 64, 48),
    "wide": ((conv(3, 20), pool(20), conv(20, 40), conv(40, 24, 1), conv(24, 33)), 28, 36),
    # 4 input channels, 128-channel workgroups, 1x1 with many reduction channels, tiles wider than one column block
    "deep": ((conv(4, 32), pool(32), conv(32, 128), conv(128, 64, 1), pool(64), conv(64, 160), conv(160, 128)), 144, 136),
}


# general geometry (Eq. (1)/(2) with any K_l, S_l): strides, 5x5 / 7x7 kernels, pools on odd maps, fused and lone
_NETS.update({
    "strided": ((conv(3, 8, 7, stride=2), pool(8), conv(8, 12, 5), conv(12, 16, 3, stride=2), conv(16, 8, 1, stride=2), conv(8, 6)), 75, 62),
    "oddpools": ((conv(3, 8, 5), pool(8), conv(8, 16), pool(16), pool(16), conv(16, 8, 3, stride=2), conv(8, 5, 7)), 61, 51),
    # wide enough for the matrix-core kernels: strided 3x3 / 1x1, 5x5 and 7x7, odd maps
    "stridedmfma": ((conv(8, 32, 3, stride=2), conv(32, 64, 5), conv(64, 32, 7), conv(32, 64, 1, stride=2), conv(64, 48, 3, stride=2), conv(48, 32, 5)), 91, 70),
    # 32 output channels: the filter-gradient kernel's 32-channel workgroups (plain, pooled, strided)
    "cout32": ((conv(3, 16), pool(16), conv(16, 32), pool(32), conv(32, 32), conv(32, 32, 3, stride=2), conv(32, 32)), 88, 72),
    "stridedwide": ((conv(3, 32, 3, stride=2), conv(32, 64, 3, stride=2), pool(64), conv(64, 32, 1), conv(32, 48, 5)), 70, 90),
})


def _mk(net, grid, grouping, dtype="f32", batch=2):
    layers, h, w = _NETS[net]
    L = len(layers)
    ends = {"whole": (L,), "each": tuple(range(1, L + 1)), "split": (L // 2, L)}[grouping]
    return Config("%s_%s" % (net, grouping), batch, layers[0].cin, h, w, layers, grid, ends, dtype)


@pytest.mark.parametrize("net", ["convs", "poolfirst", "pools", "wide"])
@pytest.mark.parametrize("grouping", ["whole", "each", "split"])
@pytest.mark.parametrize("grid", [(1, 1), (3, 2), (2, 4)])
def test_small_nets_f32(oracle, net, grouping, grid):
    P.check_case(oracle, _mk(net, grid, grouping))


@pytest.mark.parametrize("net", ["pools", "wide", "poolfirst"])
@pytest.mark.parametrize("grouping", ["whole", "each"])
def test_small_nets_bf16(oracle, net, grouping):
    P.check_case(oracle, _mk(net, (3, 2), grouping, "bf16"))


@pytest.mark.parametrize("net", ["strided", "oddpools", "stridedwide", "stridedmfma", "cout32"])
@pytest.mark.parametrize("grouping", ["whole", "each", "split"])
@pytest.mark.parametrize("grid", [(1, 1), (2, 3)])
def test_general_geometry_f32(oracle, net, grouping, grid):
    P.check_case(oracle, _mk(net, grid, grouping))


@pytest.mark.parametrize("net", ["strided", "oddpools", "stridedmfma", "cout32"])
def test_general_geometry_bf16_and_bias(oracle, net):
    P.check_case(oracle, _mk(net, (2, 2), "split", "bf16"))
    P.check_case(oracle, _mk(net, (3, 2), "whole"), has_bias=True)


# 16-bit storage, 3x3 filters wide enough for the packed filter-gradient kernel: rectangles wider than one column
# block, odd widths and odd first columns, tiles narrower than one group of 8 pixels, several images per chunk,
# channel counts that are no multiple of the workgroup's block, with and without the fused pool
_NETS.update({
    "w16plain": ((conv(4, 16), conv(16, 48), conv(48, 80), conv(80, 32)), 70, 54),
    "w16pools": ((conv(4, 32), pool(32), conv(32, 64), pool(64), conv(64, 96), conv(96, 40)), 120, 88),
})


@pytest.mark.parametrize("net", ["w16plain", "w16pools"])
@pytest.mark.parametrize("grouping", ["whole", "each"])
@pytest.mark.parametrize("grid", [(1, 1), (3, 5), (7, 4)])
def test_bf16_filter_gradient_shapes(oracle, net, grouping, grid):
    P.check_case(oracle, _mk(net, grid, grouping, "bf16", batch=3))


@pytest.mark.parametrize("grid", [(1, 1), (2, 3)])
@pytest.mark.parametrize("grouping", ["whole", "split"])
def test_deep_net_f32(oracle, grid, grouping):
    P.check_case(oracle, _mk("deep", grid, grouping, batch=3))


def test_deep_net_bf16(oracle):
    P.check_case(oracle, _mk("deep", (2, 2), "split", "bf16", batch=2))


@pytest.mark.parametrize("grid,grouping", [((16, 16), "whole"), ((16, 16), "each"), ((8, 16), "split")])
def test_many_tiny_tiles(oracle, grid, grouping):
    """The largest grid: tiles of 4 x 4 pixels (2 x 2 behind the pool), several images per chunk in the
    filter-gradient kernels, one column of threads in the thin kernels."""
    layers = (conv(3, 16), pool(16), conv(16, 32), conv(32, 16, 1), conv(16, 32))
    L = len(layers)
    ends = {"whole": (L,), "each": tuple(range(1, L + 1)), "split": (L // 2, L)}[grouping]
    P.check_case(oracle, Config("tiny_tiles_%s" % grouping, 3, 3, 64, 64, layers, grid, ends, "f32"), partial_check=False)


@pytest.mark.parametrize("grouping", ["whole", "split"])
def test_bias(oracle, grouping):
    P.check_case(oracle, _mk("pools", (2, 3), grouping), has_bias=True)


def test_batch_one_and_odd_batch(oracle):
    P.check_case(oracle, _mk("pools", (2, 2), "split", batch=1))
    P.check_case(oracle, _mk("convs", (2, 2), "whole", batch=3))


@pytest.mark.parametrize("fused", [False, True])
def test_config2(oracle, fused):
    P.check_case(oracle, C.config2(fused), strict_chain=False)


def test_deterministic_bitwise(oracle):
    """Two runs give bitwise identical y, dx and reduced gradients (no float atomics anywhere)."""
    cfg = _mk("pools", (3, 2), "split")
    x, ws, bs, dy = C.make_tensors(cfg)
    a = P.gpu_run(cfg, x, ws, bs, dy)
    b = P.gpu_run(cfg, x, ws, bs, dy)
    for k in ("y", "dx", "wgrad", "partials"):
        assert np.array_equal(a[k], b[k]), k
    a["session"].close()
    b["session"].close()


@pytest.mark.parametrize("overlap", [False, True])
def test_step_under_graph_capture(oracle, overlap):
    """The three device calls allocate nothing and use no host synchronisation, so a step can be captured in a HIP
    graph: every replay (with eager work and synchronisations in between) reproduces the eager results bit for bit.
    With the two-stream backward pass switched on the second stream joins the capture through its events (the stream
    and the events exist before the capture starts: ftp_set_overlap creates them)."""
    import torch
    cfg = _mk("pools", (3, 2), "split")
    x, ws, bs, dy = C.make_tensors(cfg)
    s = P.make_session(cfg, x.shape[0])
    s.load(x=x, weights=ws, dy=dy)
    s.set_overlap(overlap)
    s.step()
    torch.cuda.synchronize()
    ref = [s.y.clone(), s.dx.clone(), s.wgrad.clone()]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        s.step()                                   # first launches outside the capture (one-time kernel attributes)
        side.synchronize()
        with torch.cuda.graph(g, stream=side):
            s.step()
    torch.cuda.synchronize()
    for _ in range(3):
        for t in (s.y, s.dx, s.wgrad, s.partials):
            t.fill_(float("nan"))                  # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for a, b in zip(ref, (s.y, s.dx, s.wgrad)):
            assert torch.equal(a, b)
    s.close()


def _random_net(seed):
    """A random small network over the whole admitted geometry (K, stride, pools on any map, channel counts on both
    sides of the matrix-core thresholds), a random grid and grouping."""
    import random
    rnd = random.Random(seed)
    while True:
        h, w = rnd.randint(28, 84), rnd.randint(28, 84)
        c = rnd.choice([3, 4, 8, 16, 32])
        layers, ch, hh, ww = [], c, h, w
        for _ in range(rnd.randint(3, 6)):
            if rnd.random() < 0.25 and hh >= 8 and ww >= 8:
                layers.append(pool(ch))
                hh, ww = hh // 2, ww // 2
            else:
                co = rnd.choice([4, 8, 16, 24, 32, 48, 64, 96])
                st = 2 if (rnd.random() < 0.3 and hh >= 12 and ww >= 12) else 1
                layers.append(conv(ch, co, rnd.choice([1, 3, 3, 5, 7]), stride=st))
                ch, hh, ww = co, (hh - 1) // st + 1, (ww - 1) // st + 1
        N, M = rnd.randint(1, 3), rnd.randint(1, 3)
        if hh < 2 * N or ww < 2 * M or all(ly.kind != 0 for ly in layers):
            continue
        L = len(layers)
        cuts = sorted(rnd.sample(range(1, L), rnd.randint(0, min(2, L - 1))))
        dtype = "bf16" if rnd.random() < 0.4 else "f32"
        return Config("random_%d" % seed, rnd.randint(1, 3), c, h, w, tuple(layers), (N, M), tuple(cuts + [L]), dtype)


@pytest.mark.parametrize("seed", list(range(48)))
def test_random_general_networks(oracle, seed):
    P.check_case(oracle, _random_net(seed))


def test_network_without_parameters(oracle):
    """Degenerate case: pools only.  No filter, no gradient vector; y and dx still have to match (winner routing through
    two pools, the second on an odd map)."""
    import torch
    layers = (pool(5), pool(5))
    cfg = Config("pools_only", 2, 5, 42, 30, layers, (2, 2), (1, 2))
    x, ws, bs, dy = C.make_tensors(cfg)
    acts, args = oracle.forward(cfg.layers, x, ws)
    dx, _, _ = oracle.backward(cfg.layers, acts, args, ws, dy, want_db=False)
    s = P.make_session(cfg, x.shape[0])
    assert s.n_params == 0
    s.load(x=x, weights=ws, dy=dy)
    s.step()
    torch.cuda.synchronize()
    assert np.array_equal(s.to_np(s.y), acts[-1])
    assert np.array_equal(s.to_np(s.dx), dx)
    s.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_one_pixel_tiles_and_single_channels(oracle, dtype):
    """Degenerate tilings: every tile owns a single pixel of the group outputs (everything else it touches is halo),
    and layers with a single input or output channel."""
    layers = (conv(1, 8), pool(8), conv(8, 16), conv(16, 1, 1), conv(1, 4, 5))
    P.check_case(oracle, Config("one_pixel_%s" % dtype, 2, 1, 12, 10, layers, (6, 5), (2, 5), dtype), partial_check=False)
    layers = (conv(3, 16), conv(16, 32), conv(32, 16, 3, stride=2))
    P.check_case(oracle, Config("one_pixel_s2_%s" % dtype, 1, 3, 16, 14, layers, (8, 7), (3,), dtype), partial_check=False)


@pytest.mark.parametrize("grid", [(1, 1), (2, 2)])
def test_filters_larger_than_the_map(oracle, grid):
    """7x7 and 5x5 filters on maps of a few pixels: most taps fall into the zero padding, halos cover the whole map."""
    layers = (conv(4, 16, 7), conv(16, 32, 5, stride=2), conv(32, 16, 7), conv(16, 8, 3))
    P.check_case(oracle, Config("tiny_maps", 3, 4, 5, 4, layers, grid, (2, 4)), partial_check=False)
    layers = (conv(16, 32, 5), pool(32), conv(32, 32, 7))
    P.check_case(oracle, Config("tiny_maps_pool", 2, 16, 6, 7, layers, grid, (3,), "bf16"), partial_check=False)


def test_largest_grid_general_geometry(oracle):
    """16 x 16 tiles of 2 x 2 output pixels through a strided layer, a lone pool and a 5x5 layer."""
    layers = (conv(3, 16, 3, stride=2), conv(16, 32), pool(32), conv(32, 16, 5))
    P.check_case(oracle, Config("grid16_general", 2, 3, 128, 128, layers, (16, 16), (2, 4)), partial_check=False)


def _random_wide_net(seed):
    """Like _random_net with wider layers (several channel blocks per kernel), larger grids and optional biases."""
    import random
    rnd = random.Random(1000 + seed)
    while True:
        h, w = rnd.randint(40, 100), rnd.randint(40, 100)
        c = rnd.choice([3, 16, 32, 64])
        layers, ch, hh, ww = [], c, h, w
        for _ in range(rnd.randint(2, 5)):
            if rnd.random() < 0.25 and hh >= 8 and ww >= 8:
                layers.append(pool(ch))
                hh, ww = hh // 2, ww // 2
            else:
                co = rnd.choice([32, 64, 80, 128, 160])
                st = 2 if (rnd.random() < 0.25 and hh >= 16 and ww >= 16) else 1
                layers.append(conv(ch, co, rnd.choice([1, 3, 3, 3, 5]), stride=st))
                ch, hh, ww = co, (hh - 1) // st + 1, (ww - 1) // st + 1
        N, M = rnd.randint(1, 4), rnd.randint(1, 4)
        if hh < 2 * N or ww < 2 * M or all(ly.kind != 0 for ly in layers):
            continue
        L = len(layers)
        cuts = sorted(rnd.sample(range(1, L), rnd.randint(0, min(2, L - 1))))
        dtype = "bf16" if rnd.random() < 0.5 else "f32"
        return Config("random_wide_%d" % seed, rnd.randint(1, 4), c, h, w, tuple(layers), (N, M), tuple(cuts + [L]), dtype), rnd.random() < 0.25


@pytest.mark.parametrize("seed", list(range(24)))
def test_random_wide_networks(oracle, seed):
    cfg, has_bias = _random_wide_net(seed)
    P.check_case(oracle, cfg, has_bias=has_bias, partial_check=False)


_THIN = {
    # rows of 120 pool windows (two blocks of 64 positions per channel), 40 output channels (a partial block of 32)
    "wide_rows": ((conv(2, 40), pool(40), conv(40, 8)), 2, 2, 40, 480, (1, 2), "f32"),
    # rectangles of a few pixels: a chunk holds several images; 5x5 filter on 3 channels (75 columns: three blocks of 32)
    "small_rects_5x5": ((conv(3, 24, 5), conv(24, 8)), 7, 3, 26, 22, (3, 3), "f32"),
    # the same behind a pool, 4 input channels (36 columns), bfloat maps
    "small_rects_pool": ((conv(4, 16), pool(16), conv(16, 8)), 9, 4, 24, 24, (3, 3), "bf16"),
    # strided 7x7 stem on one channel, odd map, 33 output channels
    "stem_7x7": ((conv(1, 33, 7, stride=2), conv(33, 8)), 3, 1, 75, 61, (2, 2), "f32"),
    # three column blocks, the last one of odd width; no pool
    "wide_odd": ((conv(3, 16), conv(16, 8)), 2, 3, 9, 301, (1, 1), "f32"),
    # odd rectangle widths (rows padded to an even length) and a 1x1 filter on 3 channels
    "odd_1x1": ((conv(3, 20, 1), conv(20, 8)), 2, 3, 45, 39, (3, 3), "bf16"),
}


@pytest.mark.parametrize("name", sorted(_THIN))
def test_thin_first_layer_shapes(oracle, name):
    """First layers with 1 to 4 input channels: the kernels written for them (forward, delta, filter gradient streamed
    through LDS) on chunk shapes the networks above do not reach."""
    layers, batch, cin, h, w, grid, dtype = _THIN[name]
    L = len(layers)
    P.check_case(oracle, Config("thin_%s" % name, batch, cin, h, w, layers, grid, (L,), dtype), partial_check=False)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("grid,grouping", [((1, 1), (4,)), ((4, 3), (4,)), ((2, 5), (1, 2, 3, 4))])
def test_strided_delta_parity_classes(oracle, dtype, grid, grouping):
    """3x3 stride-2 layers whose delta pass splits the input pixels into their four parity classes: odd maps (rectangles
    that start at odd pixels), 20 and 48 produced channels (partial blocks of 32), rectangles of a few cells (a workgroup's
    blocks then span several images), both storage types."""
    layers = (conv(16, 20), conv(20, 48, 3, stride=2), conv(48, 40, 3, stride=2), conv(40, 8, 3, stride=2))
    P.check_case(oracle, Config("s2_classes_%s" % dtype, 3, 16, 61, 75, layers, grid, grouping, dtype), partial_check=False)
