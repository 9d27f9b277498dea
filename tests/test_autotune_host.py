"""Host logic of the grouping search: the dynamic programme over measured group costs (no GPU needed)."""
import itertools

import pytest

from paper_2409_09083_amd.autotune import best_partition, boundary_shapes, candidate_profiles
from ftp_synth.configs import Config
from ftp_synth.configs import conv, pool


def _brute(cost, L, max_group):
    best = None
    for k in range(L):
        for cuts in itertools.combinations(range(1, L), k):
            ends = list(cuts) + [L]
            s, tot, ok = 0, 0.0, True
            for e in ends:
                if (s, e) not in cost or e - s > max_group:
                    ok = False
                    break
                tot += cost[(s, e)]
                s = e
            if ok and (best is None or tot < best[1] - 1e-12):
                best = (tuple(ends), tot)
    return best


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_partition_is_optimal(seed):
    import random
    rnd = random.Random(seed)
    L, mg = 7, 4
    cost = {(s, e): rnd.uniform(1.0, 3.0) * (e - s) ** rnd.uniform(0.7, 1.3) for s in range(L) for e in range(s + 1, min(L, s + mg) + 1)}
    del cost[(2, 4)]                      # a group the plan would reject
    ends, tot = best_partition(cost, L, mg)
    want = _brute(cost, L, mg)
    assert abs(tot - want[1]) < 1e-9 and ends[-1] == L
    s = 0
    for e in ends:
        assert (s, e) in cost
        s = e


def test_additive_costs_prefer_the_cheaper_side():
    # superadditive group cost (halo recompute grows with the group) -> singletons; subadditive -> one group
    L = 5
    sup = {(s, e): float((e - s) ** 2) for s in range(L) for e in range(s + 1, L + 1)}
    sub = {(s, e): float((e - s) ** 0.5) for s in range(L) for e in range(s + 1, L + 1)}
    assert best_partition(sup, L, L)[0] == (1, 2, 3, 4, 5)
    assert best_partition(sub, L, L)[0] == (5,)
    with pytest.raises(ValueError):
        best_partition({(0, 1): 1.0}, 2, 2)


def test_boundary_shapes_come_from_the_planner():
    # strides, 5x5 / 7x7 kernels and a pool on an odd map: the shapes are the library's, not a re-derivation
    layers = (conv(3, 8, 7, stride=2), pool(8), conv(8, 16, 1), conv(16, 8, 3, stride=2), pool(8))
    cfg = Config("shapes", 1, 3, 75, 62, layers, (1, 2), (5,))
    assert boundary_shapes(cfg) == [(3, 75, 62), (8, 38, 31), (8, 19, 15), (16, 19, 15), (8, 10, 8), (8, 5, 4)]


def test_candidates_include_every_uniform_profile():
    c = candidate_profiles(6, (2, 6), (3, 6))
    assert c["searched"] == (2, 6) and c["as configured"] == (3, 6)
    assert c["uniform 1"] == (1, 2, 3, 4, 5, 6) and c["uniform 4"] == (4, 6) and c["uniform 6"] == (6,)
