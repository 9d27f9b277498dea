"""Grouping-profile search on the GPU (Sec. 4.2: the trade-off between recomputed halo and boundary exchange): the
profile it returns is a valid grouping whose results still match the oracle, and it is the fastest of the profiles
the search itself timed on the whole network, the uniform ones included."""
import pytest

from ftp_synth.configs import Config, conv, pool
from tests import parity as P

pytestmark = pytest.mark.gpu


def test_search_returns_the_fastest_measured_profile_and_parity_holds(oracle):
    from paper_2409_09083_amd import autotune
    layers = (conv(4, 32), pool(32), conv(32, 64), conv(64, 32, 1), pool(32), conv(32, 64), conv(64, 48))
    cfg = Config("autotune_small", 4, 4, 96, 80, layers, (2, 3), (4, 7))
    ends, ms, det = autotune.search(cfg, max_group=4, steps=2)
    L = len(layers)
    assert ends[-1] == L and all(a < b for a, b in zip(ends, ends[1:]))
    timed = {k: v["ms_per_step"] for k, v in det["profiles"].items() if "ms_per_step" in v}
    uniform = {k: v for k, v in timed.items() if k.startswith("uniform")}
    assert uniform and "searched" in timed
    print("autotune: chosen %s %s %.3f ms; predicted %.3f ms; %s" % (det["chosen"], list(ends), ms, det["predicted_ms"],
                                                                       {k: round(v, 3) for k, v in timed.items()}))
    assert ms == min(timed.values())
    assert ms <= 1.02 * min(uniform.values())
    P.check_case(oracle, cfg.with_(group_ends=tuple(ends)))
