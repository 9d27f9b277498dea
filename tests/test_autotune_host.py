"""Host logic of the grouping search: the dynamic programme over measured group costs (no GPU needed)."""
import itertools

import pytest

from paper_2409_09083_amd.autotune import best_partition, boundary_shapes
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


def test_boundary_shapes():
    layers = (conv(3, 8), pool(8), conv(8, 16, 1))
    assert boundary_shapes(layers, 3, 32, 48) == [(3, 32, 48), (8, 32, 48), (8, 16, 24), (16, 16, 24)]
