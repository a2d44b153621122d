"""A seeded sweep of small rounds with independently drawn shapes (sessions, agents per session, block
sizes, histories, page size, KV heads, pair style, launch shape, cache policy, layout): the whole
pipeline against the oracle bit for bit, every stage, plus the attention path by tolerance.  The shapes are fixed by the seed, so every run tests the same 24 rounds."""
import numpy as np
import pytest

from paper_2604_03143_amd import workload as wl
from helpers import OracleRun, lists_of

pytestmark = pytest.mark.gpu


def _draw(case: int):
    g = np.random.default_rng([20260403, 4242, case])
    T = int(g.choice([16, 32]))
    H = int(g.choice([1, 2, 3, 4, 8]))
    sessions = int(g.integers(1, 4))
    agents = int(g.integers(1, 12))
    blocks = int(g.integers(1, 6))
    block_tokens = int(g.integers(T, 90))            # at least a page long: a page meets at most two blocks
    lo = int(g.integers(0, 50))
    hi = lo + int(g.integers(0, 3000))
    frac = float(g.choice([0.0, 0.1, 0.3, 1.0]))
    spec = wl.RoundSpec(f"rnd{case}", 300 + case, 1, H, 128, T, float(g.choice([1.0e4, 5.0e5, 1.0e6])),
                        sessions, agents, blocks, block_tokens, lo, hi, frac)
    return dict(spec=spec, style=int(g.integers(0, 2)), group=int(g.choice([0, 1, 3, 7, 32])),
                flags=int(g.integers(0, 128)) | (128 if case % 2 else 0) | (256 if case % 4 < 2 else 0) | (512 if case % 3 else 1024) | (2048 if case % 5 < 3 else 0), permuted=bool(g.integers(0, 3) == 0), clustered=bool(g.integers(0, 2)))


@pytest.mark.parametrize("case", range(24))
def test_random_round(tdo, case):
    import torch
    from paper_2604_03143_amd import tdk
    import gpu_helpers as gh
    from test_gpu_parity import run_pipeline
    c = _draw(case)
    spec = c["spec"]
    rnd = wl.make_round(spec, clustered=c["clustered"])
    if c["permuted"]:
        rnd = wl.permute_blocks(rnd, seed_tag=case + 1)
    o, od = run_pipeline(tdo, rnd, style=c["style"], group=c["group"], flags=c["flags"])
    for i, lst in enumerate(lists_of(od, rnd.n_agents)):
        assert np.array_equal(lst, rnd.perturbed[i]), (case, i)
    # attention over the same mirrors, never restored
    n_q, Hq = 1 + case % 3, spec.num_kv_heads * (1 + case % 4)
    g = np.random.default_rng([spec.stream, 9])
    q = wl.f32_to_bf16_bits(g.standard_normal((rnd.n_agents, n_q, Hq, 128)).astype(np.float32))
    # every other round with near one-hot weights (scale 1: a dropped or doubled token moves the rows it dominates
    # far above the bounds, which flat weights would hide); per-row bounds as derived in attend_bounds.py
    import attend_bounds as ab
    sharp = case % 2 == 1
    scale = 1.0 if sharp else 1.0 / np.sqrt(128.0)
    want_o, want_l, tol_o, tol_l = ab.expected_and_bounds(tdo, o.g, o.hr, o.mk, o.mv, od, q, n_q, Hq, scale)
    r = tdk.round_from_workload(rnd, style=c["style"])
    try:
        n = int(od.offset[-1])
        mk, mv = gh.up(o.mk), gh.up(o.mv)
        cnt, off = torch.from_numpy(od.count).cuda(), torch.from_numpy(od.offset).cuda()
        idx, pay = torch.from_numpy(od.idx[:max(n, 1)].copy()).cuda(), gh.up(od.payload[:max(n, 1)].copy())
        dd = tdk.diff(cnt, off, idx, pay, n, torch.zeros(1, dtype=torch.int32, device="cuda"))
        nbytes = tdk.tdk_attend_workspace_bytes(r, n_q, Hq)
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        ws.fill_(0xFF)
        out = torch.full((rnd.n_agents, n_q, Hq, 128), float("nan"), dtype=torch.float32, device="cuda")
        lse = torch.full((rnd.n_agents, n_q, Hq), float("nan"), dtype=torch.float32, device="cuda")
        tdk.tdk_attend_shared(r, 0, tdk.layer_io(mk, mv, None, None, 0), dd,
                              tdk.attend_io(gh.up(q), n_q, Hq, scale, out, lse, ws, nbytes))
        torch.cuda.synchronize()
        if rnd.agent_tokens() > 0:
            ab.assert_within(out.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64),
                             want_o, want_l, tol_o, tol_l, what=case)
    finally:
        r.destroy()
