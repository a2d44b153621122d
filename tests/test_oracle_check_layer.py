"""Pins for the oracle's check-layer functions (Sec. 4.2: batched key-difference pass, important
positions, master = lowest total deviation)."""
import numpy as np
import pytest

from paper_2604_03143_amd import workload as wl
from helpers import OracleRun, small_spec


def test_deviation_is_zero_for_reused_keys_and_exact_for_one_changed_element(tdo):
    rnd = wl.make_round(small_spec(H=2, D=8, T=4, agents=3, blocks=2, block_tokens=9))
    run = OracleRun(tdo, rnd)
    run.rerotate()
    sc = tdo.key_deviation(run.g, run.hr, run.mk, run.pk)
    assert sc.shape == (3 * 18,) and np.all(sc == 0.0)
    # one element of agent 1, token 7 moved from x to x + 0.5 (exactly representable step)
    row = int(rnd.dst_rows(1, np.array([7]))[0])
    x = wl.bf16_bits_to_f32(run.pk[row, 3:4])[0]
    run.pk[row, 3] = 0x3F00 if x == 0 else run.pk[row, 3]
    newv = wl.bf16_bits_to_f32(run.pk[row, 3:4])[0]
    run.pk[row, 3] = wl.f32_to_bf16_bits(np.array([np.float32(4.0)]))[0]
    d = 4.0 - float(x)
    sc = tdo.key_deviation(run.g, run.hr, run.mk, run.pk)
    exp = np.zeros_like(sc)
    exp[18 + 7] = d * d
    assert np.allclose(sc, exp, rtol=1e-12, atol=0)
    # V never matters
    run.pv[:] ^= np.uint16(0x0101)
    assert np.array_equal(tdo.key_deviation(run.g, run.hr, run.mk, run.pk), sc)


def test_deviation_bruteforce_against_numpy(tdo):
    """Separate evaluator: numpy complex rotation in double, rounded to bf16 by the generator's helper."""
    spec = small_spec(H=2, D=8, T=4, agents=2, blocks=2, block_tokens=6, theta=1.0e4)
    rnd = wl.make_round(spec)
    run = OracleRun(tdo, rnd)          # pool = unrelated bits: large deviations everywhere
    sc = tdo.key_deviation(run.g, run.hr, run.mk, run.pk).reshape(2, 12)
    j = np.arange(4)
    for i in range(2):
        w = np.exp(1j * (int(rnd.agent_pos0[i]) * np.power(1.0e4, -2.0 * j / 8)))
        for m in range(12):
            x = wl.bf16_bits_to_f32(run.mk[m]).astype(np.float64).reshape(2, 8)
            z = (x[:, :4] + 1j * x[:, 4:]) * w
            ref_exact = np.concatenate([z.real, z.imag], axis=1).reshape(-1)
            ref = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(ref_exact.astype(np.float32))).astype(np.float64)
            fresh = wl.bf16_bits_to_f32(run.pk[int(rnd.dst_rows(i, np.array([m]))[0])]).astype(np.float64)
            ok = np.isfinite(fresh).all()
            if ok:
                # fp32-math reference may differ from the double one by a bf16 ulp on rare elements
                assert abs(sc[i, m] - np.sum((fresh - ref) ** 2)) <= 0.05 * max(1.0, sc[i, m])


def test_select_matches_stable_argsort(tdo):
    rng = np.random.default_rng(3)
    for S, ratio, ms in ((50, 0.15, 0.0), (64, 1.0, 0.0), (1000, 0.1, 0.5), (7, 0.01, 0.0), (300, 0.3, 10.0)):
        sc = rng.random(S).astype(np.float32)
        sc[rng.integers(0, S, S // 3)] = 0.25          # many ties
        sc[rng.integers(0, S, S // 4)] = 0.0
        got = tdo.select_important(sc, ratio, ms)
        k = int(np.ceil(float(np.float32(ratio)) * S))      # the ratio is an fp32 argument
        cand = np.flatnonzero(sc > ms)
        order = cand[np.argsort(-sc[cand], kind="stable")]     # ties keep ascending index
        exp = np.sort(order[:k])
        assert np.array_equal(got, exp), (S, ratio, ms)
    # a tie across the cut: the lower token numbers win
    assert tdo.select_important(np.full(8, 0.5, np.float32), 0.5, 0.0).tolist() == [0, 1, 2, 3]
    assert tdo.select_important(np.array([1, 2, 1, 2, 1, 2, 1, 2], np.float32), 0.75, 0.0).tolist() == [0, 1, 2, 3, 5, 7]
    # NaN is the most important; nothing qualifies -> empty
    sc = np.array([0.1, np.nan, 0.3, 0.2], np.float32)
    assert tdo.select_important(sc, 0.5, 0.0).tolist() == [1, 2]
    assert tdo.select_important(np.zeros(9, np.float32), 0.5, 0.0).size == 0


def test_master_is_argmin_of_totals(tdo):
    rnd = wl.make_round(small_spec(H=2, D=8, T=4, sessions=3, agents=4, blocks=1, block_tokens=4))
    hr = tdo.HostRound(rnd)
    rng = np.random.default_rng(9)
    for _ in range(5):
        tot = rng.random(12).astype(np.float32)
        exp = [int(np.argmin(tot[4 * s:4 * s + 4])) + 4 * s for s in range(3)]
        assert tdo.choose_master(hr, tot).tolist() == exp
    tot = np.array([3, 1, 1, 2, np.nan, 5, 4, 4, np.nan, np.nan, np.nan, np.nan], np.float32)
    assert tdo.choose_master(hr, tot).tolist() == [1, 6, 8]


def test_perturbed_tokens_are_the_important_ones(tdo):
    """On the synthetic workload the refreshed pages carry all the deviation: with ratio = their share
    and min_score = 0 the important positions are exactly their tokens."""
    spec = wl.CONFIGS["tiny"]
    rnd = wl.make_round(spec)
    run = OracleRun(tdo, rnd)
    run.rerotate(); run.perturb()
    sc = tdo.key_deviation(run.g, run.hr, run.mk, run.pk).reshape(rnd.n_agents, spec.span_tokens)
    T = spec.page_tokens
    for i in range(rnd.n_agents):
        got = tdo.select_important(sc[i].astype(np.float32), 1.0, 0.0)
        exp = np.concatenate([np.arange(p * T, (p + 1) * T) for p in rnd.perturbed[i]])
        assert np.array_equal(got, exp)
