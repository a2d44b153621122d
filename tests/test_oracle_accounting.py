"""Pins for the storage arithmetic of Sec. 6.4 against the values the paper prints."""
import os

import numpy as np

from paper_2604_03143_amd import workload as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "capacity_sec6_4.txt")


def _rows():
    out = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                out.append([float(t) for t in line.split()])
    return out


def test_family_cost_matches_printed_values(tdo):
    rows = _rows()
    assert len(rows) == 2
    for n, r, cost, reduction, pct in rows:
        c = tdo.family_cost(int(n), r)
        assert abs(c - cost) < 0.05               # printed to one decimal
        assert abs(n / c - reduction) < 0.1       # "5.6x", "6.7x"
        assert abs(100.0 / r - pct) < 0.5         # "roughly 9%", "about 6%"
    assert tdo.family_cost(1, 11.2) == 1.0
    assert abs(tdo.family_cost(10, 1.0) - 10.0) < 1e-12   # no compression: N full caches


def test_mirror_ratio_closed_forms(tdo):
    g = tdo.geom(8, 128, 16, 1.0e6)
    assert tdo.dense_bytes(g, 5000) == 5000 * 4096
    assert tdo.diff_bytes(g, 19) == 19 * 65536 + 19 * 4 + 12
    assert tdo.diff_bytes(g, 0) == 12
    # synthetic workloads: f = 6 % -> R ~ 16.5 (inside the paper's 11-17x band), 3 % -> ~33, 10 % -> ~10
    for name, lo, hi in (("session", 16.0, 17.0), ("long", 32.5, 34.0), ("llama70b", 9.9, 10.1)):
        spec = wl.CONFIGS[name]
        r = tdo.mirror_ratio(g, spec.span_tokens, spec.perturbed_pages_per_agent)
        assert lo < r < hi, (name, r)
    # ratio * diff == dense
    assert np.isclose(tdo.mirror_ratio(g, 5000, 19) * tdo.diff_bytes(g, 19), tdo.dense_bytes(g, 5000))


def test_config_shapes_match_workload_table():
    """Shapes of the five synthetic rounds (sessions x agents, span, pages, perturbed pages)."""
    exp = {"tiny": (4, 256, 16, 1), "session": (25, 5000, 313, 19), "batched250": (250, 5000, 313, 19),
           "long": (100, 25600, 1600, 48), "llama70b": (64, 12800, 800, 80)}
    for name, (a, s, p, k) in exp.items():
        spec = wl.CONFIGS[name]
        assert (spec.n_agents, spec.span_tokens, spec.span_pages, spec.perturbed_pages_per_agent) == (a, s, p, k)
