"""Pins of the oracle's attention over a Mirror that is never restored (Sec. 4.4, the diff applied as
attention tiles are loaded): a library routine on the restored cache, a separately written complex-number
evaluator, closed forms, and the log-sum-exp merge identity."""
import numpy as np
import pytest
import torch

from paper_2604_03143_amd import workload as wl
from helpers import OracleRun, small_spec


def _queries(rnd, n_q, Hq, seed=5):
    g = np.random.default_rng([rnd.spec.stream, seed])
    q = g.standard_normal((rnd.n_agents, n_q, Hq, rnd.spec.head_dim)).astype(np.float32)
    return wl.f32_to_bf16_bits(q)


def _mirror(tdo, spec, hist=None, style=0):
    rnd = wl.make_round(spec, hist=hist)
    run = OracleRun(tdo, rnd, style=style)
    run.rerotate(); run.perturb()
    d = run.encode()
    assert d.offset[-1] > 0
    return rnd, run, d


def _sdpa_on_rows(k_rows, v_rows, q_bits, H, scale):
    """torch's scaled_dot_product_attention in double on explicit K/V rows [S][H*D] (double)."""
    S = k_rows.shape[0]
    n_q, Hq, D = q_bits.shape
    G = Hq // H
    k = torch.from_numpy(k_rows.reshape(S, H, D)).permute(1, 0, 2).repeat_interleave(G, dim=0)   # [Hq][S][D]
    v = torch.from_numpy(v_rows.reshape(S, H, D)).permute(1, 0, 2).repeat_interleave(G, dim=0)
    q = torch.from_numpy(wl.bf16_bits_to_f32(q_bits).astype(np.float64)).permute(1, 0, 2)      # [Hq][n_q][D]
    o = torch.nn.functional.scaled_dot_product_attention(q[None], k[None], v[None], scale=scale)[0]
    return o.permute(1, 0, 2).numpy()                                                          # [n_q][Hq][D]


def test_equals_library_attention_on_the_restored_cache_when_nothing_rotates(tdo):
    """Histories of 0 tokens and masters at position 0: the restored cache holds exactly the keys the
    definition uses, so torch's attention on the restored rows must agree to rounding."""
    spec = small_spec(H=2, D=8, T=4, sessions=2, agents=3, blocks=3, block_tokens=7, frac=0.4)
    rnd, run, d = _mirror(tdo, spec, hist=np.zeros(6, np.int64))
    q = _queries(rnd, 2, 4)
    scale = 0.37
    out, lse = tdo.attend_shared(run.g, run.hr, run.mk, run.mv, d, q, 2, 4, scale)
    pk, pv = wl.pool_host(rnd, 0)
    tdo.diff_decode(run.g, run.hr, run.mk, run.mv, pk, pv, d)
    for i in range(rnd.n_agents):
        rows = rnd.dst_rows(i, np.arange(spec.span_tokens))
        ref = _sdpa_on_rows(wl.bf16_bits_to_f32(pk[rows]).astype(np.float64), wl.bf16_bits_to_f32(pv[rows]).astype(np.float64),
                            q[i], spec.num_kv_heads, scale)
        assert np.max(np.abs(out[i] - ref)) < 1e-12


@pytest.mark.parametrize("style", [0, 1])
def test_equals_library_attention_on_the_restored_cache_up_to_the_rounding_of_restored_keys(tdo, style):
    spec = small_spec(H=2, D=16, T=4, sessions=1, agents=4, blocks=4, block_tokens=9, frac=0.3, hist=(3, 900))
    rnd, run, d = _mirror(tdo, spec, style=style)
    q = _queries(rnd, 3, 6)
    scale = 1.0 / np.sqrt(spec.head_dim)
    out, lse = tdo.attend_shared(run.g, run.hr, run.mk, run.mv, d, q, 3, 6, scale)
    pk, pv = wl.pool_host(rnd, 0)
    tdo.diff_decode(run.g, run.hr, run.mk, run.mv, pk, pv, d)
    worst = 0.0
    for i in range(rnd.n_agents):
        rows = rnd.dst_rows(i, np.arange(spec.span_tokens))
        ref = _sdpa_on_rows(wl.bf16_bits_to_f32(pk[rows]).astype(np.float64), wl.bf16_bits_to_f32(pv[rows]).astype(np.float64),
                            q[i], spec.num_kv_heads, scale)
        worst = max(worst, float(np.max(np.abs(out[i] - ref))))
    # restored keys carry one bf16 rounding (2^-9 relative) each; with |q|,|k| ~ 1 the scores move by ~1e-2
    # at most and the normalised outputs by a few 1e-3; a wrong sign, table or head mapping moves them by O(1)
    assert 0.0 < worst < 2e-2


def test_against_a_complex_number_evaluator_including_moved_diff_pages(tdo):
    """Scores and log-sum-exp from a separately written evaluator: keys as complex numbers times
    exp(i * delta * theta^(-2j/D)); listed pages from the payload, moved by their own distance."""
    spec = small_spec(H=2, D=8, T=4, sessions=2, agents=3, blocks=3, block_tokens=7, frac=0.4, theta=1.0e4)
    old, run, d = _mirror(tdo, spec)
    grow = np.array([5, 0, 17, 8, 33, 4], np.int64)
    new = wl.make_round(spec, hist=old.agent_pos0 + grow)
    hr = tdo.HostRound(new, diff_pos0=old.agent_pos0)
    n_q, Hq, D, H, T = 2, 4, spec.head_dim, spec.num_kv_heads, spec.page_tokens
    q = _queries(new, n_q, Hq)
    scale = 0.5
    out, lse = tdo.attend_shared(run.g, hr, run.mk, run.mv, d, q, n_q, Hq, scale)
    inv = np.power(spec.rope_theta, -2.0 * np.arange(D // 2) / D)
    f = lambda bits: wl.bf16_bits_to_f32(bits).astype(np.float64)
    for i in range(new.n_agents):
        s = int(new.agent_session[i])
        S = int(new.span_tokens[s])
        listed = {int(p): int(d.offset[i]) + k for k, p in enumerate(d.idx[int(d.offset[i]):int(d.offset[i + 1])])}
        K = np.zeros((S, H, D)); V = np.zeros((S, H, D))
        for m in range(S):
            if m // T in listed:
                page = d.payload[listed[m // T]].reshape(2, T, H, D)
                k, v, dist = f(page[0, m % T]), f(page[1, m % T]), int(grow[i])
            else:
                row = int(new.master_row0[s]) + m
                k, v = f(run.mk[row]).reshape(H, D), f(run.mv[row]).reshape(H, D)
                dist = int(new.agent_pos0[i]) - int(new.master_pos0[s])
            z = (k[:, : D // 2] + 1j * k[:, D // 2:]) * np.exp(1j * dist * inv)
            K[m] = np.concatenate([z.real, z.imag], axis=-1); V[m] = v
        for qi in range(n_q):
            for hq in range(Hq):
                sc = scale * K[:, hq // (Hq // H), :] @ f(q[i, qi, hq])
                ref_lse = np.log(np.sum(np.exp(sc - sc.max()))) + sc.max()
                p = np.exp(sc - ref_lse)
                assert abs(lse[i, qi, hq] - ref_lse) < 1e-10
                assert np.max(np.abs(out[i, qi, hq] - p @ V[:, hq // (Hq // H), :])) < 1e-10


def test_closed_forms_and_merge_identity(tdo):
    spec = small_spec(H=2, D=8, T=4, sessions=1, agents=3, blocks=3, block_tokens=7, frac=0.4)
    rnd, run, d = _mirror(tdo, spec)
    S, H, D = spec.span_tokens, spec.num_kv_heads, spec.head_dim
    # a zero query weighs every token equally: the output is the mean of the Mirror's V, lse = log S
    q0 = np.zeros((rnd.n_agents, 1, 2, D), np.uint16)
    out, lse = tdo.attend_shared(run.g, run.hr, run.mk, run.mv, d, q0, 1, 2, 1.0)
    pk, pv = wl.pool_host(rnd, 0)
    tdo.diff_decode(run.g, run.hr, run.mk, run.mv, pk, pv, d)
    for i in range(rnd.n_agents):
        v = wl.bf16_bits_to_f32(pv[rnd.dst_rows(i, np.arange(S))]).astype(np.float64).reshape(S, H, D)
        assert np.allclose(out[i, 0], v.mean(axis=0), atol=1e-12) and np.allclose(lse[i], np.log(S), atol=1e-12)
    # the scale multiplies the scores: q at scale 2c equals 2q... at scale c only if doubling q is exact (it is in bf16)
    q = _queries(rnd, 1, 4)
    q2 = wl.f32_to_bf16_bits(2.0 * wl.bf16_bits_to_f32(q))
    a, la = tdo.attend_shared(run.g, run.hr, run.mk, run.mv, d, q, 1, 4, 0.5)
    b, lb = tdo.attend_shared(run.g, run.hr, run.mk, run.mv, d, q2, 1, 4, 0.25)
    assert np.allclose(a, b, atol=1e-13) and np.allclose(la, lb, atol=1e-13)
    # two sessions that split a span: merging their partial results with the log-sum-exp weights gives the whole
    whole = wl.make_round(small_spec(H=2, D=8, T=4, sessions=1, agents=1, blocks=2, block_tokens=8, frac=0.0, stream=7), hist=np.array([6]))
    mk, mv = wl.master_host(whole, 0)
    empty = tdo.Diff(1, 0, 2 * 4 * 16)
    g = tdo.geom_of(whole.spec)
    qq = _queries(whole, 1, 2)
    o_all, l_all = tdo.attend_shared(g, tdo.HostRound(whole), mk, mv, empty, qq, 1, 2, 0.3)
    parts = []
    for lo, hi in ((0, 8), (8, 16)):
        half = wl.make_round(small_spec(H=2, D=8, T=4, sessions=1, agents=1, blocks=1, block_tokens=8, frac=0.0, stream=7), hist=np.array([6 + lo]))
        half.master_pos0 = np.array([lo], np.int64)          # this half of the master sits at positions lo..
        parts.append(tdo.attend_shared(g, tdo.HostRound(half), mk[lo:hi], mv[lo:hi], empty, qq, 1, 2, 0.3))
    (o1, l1), (o2, l2) = parts
    w1, w2 = np.exp(l1 - l_all), np.exp(l2 - l_all)
    assert np.allclose(w1 + w2, 1.0, atol=1e-12)
    assert np.allclose(o_all, w1[..., None] * o1 + w2[..., None] * o2, atol=1e-12)


def test_only_the_owner_of_a_changed_payload_page_sees_it_and_bad_arguments(tdo):
    spec = small_spec(H=2, D=8, T=4, sessions=1, agents=3, blocks=3, block_tokens=7, frac=0.4)
    rnd, run, d = _mirror(tdo, spec)
    q = _queries(rnd, 1, 2)
    a, _ = tdo.attend_shared(run.g, run.hr, run.mk, run.mv, d, q, 1, 2, 0.4)
    slot = int(d.offset[1])                                   # first listed page of agent 1: change its V plane
    page = d.payload[slot].reshape(2, spec.page_tokens, -1)
    page[1] ^= 0x0100
    b, _ = tdo.attend_shared(run.g, run.hr, run.mk, run.mv, d, q, 1, 2, 0.4)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[2], b[2]) and not np.array_equal(a[1], b[1])
    with pytest.raises(ValueError):
        tdo.attend_shared(run.g, run.hr, run.mk, run.mv, d, _queries(rnd, 1, 3), 1, 3, 0.4)   # 3 query heads on 2 KV heads
