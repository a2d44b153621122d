"""The seeded generator: structure invariants (non-overlapping slots, canaries, determinism)."""
import numpy as np

from paper_2604_03143_amd import workload as wl


def test_round_structure_tiny_and_session():
    for name in ("tiny", "session"):
        spec = wl.CONFIGS[name]
        rnd = wl.make_round(spec)
        T = spec.page_tokens
        assert rnd.n_agents == spec.n_agents
        assert np.all(rnd.agent_pos0 >= spec.hist_lo) and np.all(rnd.agent_pos0 <= spec.hist_hi)
        used = []
        for i, bt in enumerate(rnd.block_tables):
            h = int(rnd.agent_pos0[i])
            assert len(bt) == (h + spec.span_tokens - 1) // T + 1
            assert np.all(bt[: h // T] == rnd.dummy_page)
            used.append(bt[h // T:])
        used = np.concatenate(used)
        # the paper's grouping precondition: non-overlapping slot mappings (Sec. 4.2)
        assert len(np.unique(used)) == len(used)
        assert rnd.dummy_page not in used and not np.intersect1d(used, rnd.canary_pages).size
        assert len(used) + len(rnd.canary_pages) + 1 == rnd.pool_pages
        for p in rnd.perturbed:
            assert len(p) == spec.perturbed_pages_per_agent and np.all(np.diff(p) > 0)
    assert not np.all(wl.make_round(wl.CONFIGS["session"]).agent_pos0 % 16 == 0)


def test_generator_is_deterministic():
    a, b = wl.make_round(wl.CONFIGS["tiny"]), wl.make_round(wl.CONFIGS["tiny"])
    assert np.array_equal(a.agent_pos0, b.agent_pos0)
    assert all(np.array_equal(x, y) for x, y in zip(a.block_tables, b.block_tables))
    ka, va = wl.master_host(a, 0)
    kb, vb = wl.master_host(b, 0)
    assert np.array_equal(ka, kb) and np.array_equal(va, vb)
    assert not np.array_equal(ka, wl.master_host(a, 1)[0])


def test_master_values_are_standard_normal():
    rnd = wl.make_round(wl.CONFIGS["tiny"])
    k, v = wl.master_host(rnd, 0)
    for x in (wl.bf16_bits_to_f32(k), wl.bf16_bits_to_f32(v)):
        assert abs(x.mean()) < 0.01 and abs(x.std() - 1.0) < 0.01


def test_perturbation_exceeds_threshold_on_every_perturbed_page():
    spec = wl.CONFIGS["tiny"]
    rnd = wl.make_round(spec)
    k, v = wl.pool_host(rnd, 0)
    k[:] = 0x3F80
    v[:] = 0x3F80
    k0 = k.copy()
    wl.perturb_host(rnd, 0, k, v)
    T = spec.page_tokens
    for i in range(rnd.n_agents):
        for p in range(spec.span_pages):
            rows = rnd.dst_rows(i, np.arange(p * T, (p + 1) * T))
            d = np.abs(wl.bf16_bits_to_f32(k[rows]) - wl.bf16_bits_to_f32(k0[rows])).max()
            assert (d > 10 * spec.eps) == (p in rnd.perturbed[i])
