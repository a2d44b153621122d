"""Rounds whose sessions differ in span and in agent count (sessions of different sizes batched into one
round): a ragged span, a span shorter than one attention step, an empty span, a session without agents.
Every call of the library against the oracle on such a round: rerotate, encode, decode bit for bit (several
launch shapes), the check layer, and the attention over the mirrors (workspace filled with NaN patterns)."""
import numpy as np
import pytest

import attend_bounds as ab
from paper_2604_03143_amd import workload as wl
from helpers import lists_of

pytestmark = pytest.mark.gpu

SPANS = [1993, 40, 0, 700, 333]
AGENTS = [7, 2, 3, 12, 0]


def ragged_round(T=16, H=8, frac=0.2, spans=SPANS, agents=AGENTS, stream=88):
    spec = wl.RoundSpec("ragged", stream, 2, H, 128, T, 1.0e6, len(spans), max(agents), 5, 70, 3, 900, frac)
    return wl.make_round(spec, spans=spans, agents=agents)


@pytest.mark.parametrize("group,flags", [(0, None), (1, 191 + 512), (3, None), (32, 1023), (2, 63 + 256)])
def test_pipeline_on_ragged_sessions(tdo, group, flags):
    """(flags: the work items handed out statically, from the per-XCD queues whatever the round's size, tapered)"""
    from test_gpu_parity import run_pipeline
    rnd = ragged_round()
    o, od = run_pipeline(tdo, rnd, group=group, flags=flags)
    for i, lst in enumerate(lists_of(od, rnd.n_agents)):
        assert np.array_equal(lst, rnd.perturbed[i]), i


def test_pipeline_on_ragged_sessions_with_32_token_pages_and_own_block_orders(tdo):
    from test_gpu_parity import run_pipeline
    run_pipeline(tdo, ragged_round(T=32, H=2, stream=89))
    # per-agent block orders need spans that are whole blocks: 5 blocks of 70 tokens and 3 of 70
    spec = wl.RoundSpec("ragged_perm", 90, 1, 4, 128, 16, 1.0e6, 2, 6, 5, 70, 3, 900, 0.2)
    rnd = wl.make_round(spec, spans=[350, 350], agents=[6, 2])
    run_pipeline(tdo, wl.permute_blocks(rnd, seed_tag=5))


def test_check_layer_on_ragged_sessions(tdo):
    from test_gpu_check_layer import run_case
    o, gs, gi, gn, gt, gm = run_case(tdo, ragged_round(), 0.15, 0.0, noise_everywhere=0.02)
    assert gm[4] == -1                    # a session without agents has no master
    assert list(gn[9:12]) == [0, 0, 0]    # agents of the empty span have no positions


@pytest.mark.parametrize("n_q,Hq,scale", [(1, 40, None), (3, 16, None), (1, 8, 1.0), (5, 40, None)])
def test_attention_on_ragged_sessions(tdo, n_q, Hq, scale):
    """Chunks past a shorter session's span, row blocks beyond a smaller session's rows, parts of the merge
    that a session never writes: 5 and 40 rows per agent and KV head cover the shared launch and the separate
    kernels; (5, 40) gives the large session 300 rows per KV head (three row blocks), the small one 50."""
    import torch
    from paper_2604_03143_amd import tdk
    import gpu_helpers as gh
    from helpers import OracleRun
    rnd = ragged_round()
    spec = rnd.spec
    o = OracleRun(tdo, rnd)
    o.rerotate(); o.perturb()
    d = o.encode()
    g = np.random.default_rng([spec.stream, n_q, Hq])
    q = wl.f32_to_bf16_bits(g.standard_normal((rnd.n_agents, n_q, Hq, 128)).astype(np.float32))
    scale = 1.0 / np.sqrt(128.0) if scale is None else scale
    want_o, want_l, tol_o, tol_l = ab.expected_and_bounds(tdo, o.g, o.hr, o.mk, o.mv, d, q, n_q, Hq, scale)
    empty = np.array([int(rnd.span_tokens[s]) == 0 for s in rnd.agent_session])
    assert np.all(np.isneginf(want_l[empty])) and np.all(want_o[empty] == 0) and np.all(np.isfinite(want_l[~empty]))
    r = tdk.round_from_workload(rnd)
    try:
        n = int(d.offset[-1])
        mk, mv = gh.up(o.mk), gh.up(o.mv)
        cnt, off = torch.from_numpy(d.count).cuda(), torch.from_numpy(d.offset).cuda()
        idx, pay = torch.from_numpy(d.idx[:max(n, 1)].copy()).cuda(), gh.up(d.payload[:max(n, 1)].copy())
        dd = tdk.diff(cnt, off, idx, pay, n, torch.zeros(1, dtype=torch.int32, device="cuda"))
        nbytes = tdk.tdk_attend_workspace_bytes(r, n_q, Hq)
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        ws.fill_(0xFF)
        out = torch.full((rnd.n_agents, n_q, Hq, 128), float("nan"), dtype=torch.float32, device="cuda")
        lse = torch.full((rnd.n_agents, n_q, Hq), float("nan"), dtype=torch.float32, device="cuda")
        tdk.tdk_attend_shared(r, 0, tdk.layer_io(mk, mv, None, None, 0), dd,
                              tdk.attend_io(gh.up(q), n_q, Hq, scale, out, lse, ws, nbytes))
        torch.cuda.synchronize()
        ab.assert_within(out.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64),
                         want_o, want_l, tol_o, tol_l, what=(n_q, Hq, scale))
    finally:
        r.destroy()
