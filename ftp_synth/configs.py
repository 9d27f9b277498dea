"""Workload tables: the five synthetic configurations and their tensors.

A network is a list of primitive layers, each either a convolution (with its
leaky-ReLU folded in) or a 2x2/2 max-pool.  Boundaries are numbered 0..L:
boundary l is the input of primitive layer l, boundary L the network output.
A grouping is the list of group end boundaries (strictly increasing, last = L).
Shapes follow the early layers of a detection network (3-channel square
images, 3x3/1x1 convolutions, leaky slope 0.1, 2x2 pools), as in the paper's
experiments on the first 16 layers of its detection CNN (Sec. 5).
"""
from dataclasses import dataclass, field
from typing import List, Tuple
import math

from . import rng

CONV, MAXPOOL = 0, 1


@dataclass(frozen=True)
class Layer:
    kind: int
    k: int
    stride: int
    pad: int
    cin: int
    cout: int
    slope: float = 0.1

    def out_hw(self, h, w):
        return ((h + 2 * self.pad - self.k) // self.stride + 1,
                (w + 2 * self.pad - self.k) // self.stride + 1)


def conv(cin, cout, k=3, slope=0.1, stride=1):
    return Layer(CONV, k, stride, k // 2, cin, cout, slope)


def pool(c):
    return Layer(MAXPOOL, 2, 2, 0, c, c, 1.0)


@dataclass(frozen=True)
class Config:
    name: str
    batch: int
    in_c: int
    in_h: int
    in_w: int
    layers: Tuple[Layer, ...]
    grid: Tuple[int, int]          # (rows N, cols M)
    group_ends: Tuple[int, ...]
    dtype: str = "f32"             # storage type of maps and filters: "f32" | "bf16"

    @property
    def n_layers(self):
        return len(self.layers)

    def boundary_shapes(self):
        """[(C,H,W)] for boundaries 0..L."""
        c, h, w = self.in_c, self.in_h, self.in_w
        out = [(c, h, w)]
        for ly in self.layers:
            h, w = ly.out_hw(h, w)
            c = ly.cout
            out.append((c, h, w))
        return out

    def with_(self, **kw):
        d = dict(name=self.name, batch=self.batch, in_c=self.in_c, in_h=self.in_h, in_w=self.in_w,
                 layers=self.layers, grid=self.grid, group_ends=self.group_ends, dtype=self.dtype)
        d.update(kw)
        return Config(**d)


def uniform_groups(n_layers, g):
    ends = list(range(g, n_layers, g)) + [n_layers]
    return tuple(ends)


def _stack16():
    return (
        conv(3, 32), pool(32),
        conv(32, 64), pool(64),
        conv(64, 128), conv(128, 64, 1), conv(64, 128), pool(128),
        conv(128, 256), conv(256, 128, 1), conv(128, 256), pool(256),
        conv(256, 512), conv(512, 256, 1), conv(256, 512), conv(512, 256, 1),
    )


def tiny():
    return Config("tiny", 1, 3, 32, 32, (conv(3, 8), conv(8, 16)), (2, 2), (2,))


def config2(fused: bool):
    layers = (conv(3, 16), pool(16), conv(16, 32), pool(32), conv(32, 64))
    return Config("cfg2_fused" if fused else "cfg2_perblock", 1, 3, 416, 416, layers, (3, 3),
                  (5,) if fused else (2, 4, 5))


def config3():
    layers = (conv(3, 16), pool(16), conv(16, 32), pool(32), conv(32, 64),
              conv(64, 128), pool(128), conv(128, 64, 1), conv(64, 128), pool(128),
              conv(128, 64, 1), conv(64, 128))
    return Config("cfg3", 8, 3, 608, 608, layers, (4, 4), (7, 12))


def config4():
    return Config("cfg4", 64, 3, 608, 608, _stack16(), (6, 6), (4, 8, 12, 16))


def config5(group_size=4):
    return Config("cfg5_g%d" % group_size, 32, 3, 608, 608, _stack16(), (8, 8),
                  uniform_groups(16, group_size), dtype="bf16")


def general_stem():
    """General-geometry workload (not one of the paper's networks): a 7x7 stride-2 stem on an odd-sized image,
    strided 3x3 convolutions in place of two pools, a 5x5 layer and a pool that meets an odd map (19 -> 9)."""
    layers = (conv(3, 64, 7, stride=2), pool(64), conv(64, 64),
              conv(64, 128, 3, stride=2), conv(128, 64, 1), conv(64, 128, 5),
              pool(128), conv(128, 256, 3, stride=2), pool(256), conv(256, 256))
    return Config("gen_stem", 32, 3, 607, 607, layers, (3, 3), (3, 6, 10))


ALL = {
    "tiny": tiny,
    "cfg2_perblock": lambda: config2(False),
    "cfg2_fused": lambda: config2(True),
    "cfg3": config3,
    "cfg4": config4,
    "cfg5": config5,
    "gen_stem": general_stem,
}


def make_tensors(cfg: Config, master_seed: int = rng.MASTER_SEED, batch=None, images=None):
    """x ~ U[0,1), W_l ~ N(0, 2/(Cin K^2)) (He-normal), zero bias, dy ~ N(0,1).

    `images`: optional list of image indices; image n of the batch is always
    generated from its own stream ("x/n", "dy/n"), so a subset of a batch
    holds exactly the values the full batch holds for those images.
    For bf16 storage the values are rounded to bf16 (nearest even) and still
    returned as fp32 arrays.
    """
    import numpy as np
    shapes = cfg.boundary_shapes()
    if images is None:
        images = list(range(cfg.batch if batch is None else batch))
    c0, h0, w0 = shapes[0]
    cl, hl, wl = shapes[-1]
    x = np.stack([rng.uniform01("x/%d" % n, (c0, h0, w0), master_seed) for n in images])
    dy = np.stack([rng.normal("dy/%d" % n, (cl, hl, wl), 1.0, master_seed) for n in images])
    weights, biases = [], []
    for li, ly in enumerate(cfg.layers):
        if ly.kind == CONV:
            std = math.sqrt(2.0 / (ly.cin * ly.k * ly.k))
            weights.append(rng.normal("W/%d" % li, (ly.cout, ly.cin, ly.k, ly.k), std, master_seed))
            biases.append(np.zeros(ly.cout, dtype=np.float32))
        else:
            weights.append(None)
            biases.append(None)
    if cfg.dtype == "bf16":
        x = rng.to_bf16_rne(x)
        dy = rng.to_bf16_rne(dy)
        weights = [None if w is None else rng.to_bf16_rne(w) for w in weights]
    return x, weights, biases, dy
