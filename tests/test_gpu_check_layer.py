"""Check-layer pass on the GPU against the oracle.  Scores are fp32 sums on the GPU (order
unspecified) and double sums in the oracle: compared within a tolerance derived from the arithmetic
(1024 fp32 additions of non-negative terms: relative error <= 1024 * 2^-24 ~ 6.1e-5).  The selection
and the master choice are integer work: given the GPU's own fp32 scores / totals they must equal the
oracle's selection bit for bit; against the oracle's own scores they must agree wherever the
decision is not within that tolerance of a tie."""
import numpy as np
import pytest

from paper_2604_03143_amd import workload as wl
from helpers import OracleRun

pytestmark = pytest.mark.gpu
REL = 1024 * 2.0 ** -24 * 2


def run_case(tdo, rnd, ratio, min_score, noise_everywhere=0.0, style=0, fill=None):
    import torch
    from paper_2604_03143_amd import tdk
    import gpu_helpers as gh
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    spec = rnd.spec
    o = OracleRun(tdo, rnd, style=style)
    if fill is None:
        o.rerotate(); o.perturb()
        if noise_everywhere > 0:
            rng = np.random.default_rng(21)
            x = wl.bf16_bits_to_f32(o.pk)
            o.pk[:] = wl.f32_to_bf16_bits(x + rng.standard_normal(x.shape).astype(np.float32) * np.float32(noise_everywhere))
    else:
        fill(o)
    g = gh.GpuRun(rnd, style=style, mk=o.mk, mv=o.mv, pk=o.pk, pv=o.pv)
    A = rnd.n_agents
    spans = [int(rnd.span_tokens[s]) for s in rnd.agent_session]
    n_tok = sum(spans)
    kmax = max([int(np.ceil(float(np.float32(ratio)) * s)) for s in spans] + [1])
    score = torch.full((max(n_tok, 1),), -1.0, dtype=torch.float32, device="cuda")
    imp = torch.full((max(A, 1), kmax), -1, dtype=torch.int32, device="cuda")
    n_imp = torch.full((max(A, 1),), -1, dtype=torch.int32, device="cuda")
    total = torch.full((max(A, 1),), -1.0, dtype=torch.float32, device="cuda")
    master = torch.full((max(rnd.n_sessions, 1),), -7, dtype=torch.int32, device="cuda")
    plan = tdk.reuse_plan(score, imp, kmax, n_imp, total, master)
    try:
        tdk.tdk_check_layer(g.r, 0, g.io, ratio, min_score, plan, g.stream)
        torch.cuda.synchronize()
    finally:
        g.close()
    gs, gi, gn, gt, gm = (score.cpu().numpy()[:n_tok], imp.cpu().numpy(), n_imp.cpu().numpy()[:A],
                          total.cpu().numpy()[:A], master.cpu().numpy()[:rnd.n_sessions])
    os_ = tdo.key_deviation(o.g, o.hr, o.mk, o.pk)
    fin = np.isfinite(os_)
    assert np.array_equal(np.isfinite(gs), fin)
    assert np.all(np.abs(gs[fin] - os_[fin]) <= REL * os_[fin] + 1e-30)
    off = np.concatenate([[0], np.cumsum(spans)])
    for i in range(A):
        mine = gs[off[i]:off[i + 1]]
        # (a) integer work, bit-exact given the same fp32 scores
        exp = tdo.select_important(mine, ratio, min_score)
        assert gn[i] == len(exp)
        assert np.array_equal(gi[i, :gn[i]], exp), f"agent {i}"
        # (b) against the oracle's own double scores: identical unless within tolerance of a tie / of min_score
        theirs = os_[off[i]:off[i + 1]]
        ref = tdo.select_important(theirs.astype(np.float32), ratio, min_score)
        if len(ref) and len(ref) == len(exp) and np.all(np.isfinite(theirs)):
            kth = np.sort(theirs[ref])[0]
            sure_in = np.flatnonzero((theirs > kth * (1 + 4 * REL)) & (theirs > min_score * (1 + 4 * REL)))
            assert np.all(np.isin(sure_in, exp))
            assert np.all(theirs[exp] >= kth * (1 - 4 * REL))
        # totals
        t = float(np.sum(theirs[np.isfinite(theirs)])) if np.all(np.isfinite(theirs)) else float("nan")
        if np.isfinite(t):
            assert abs(gt[i] - t) <= 4 * REL * t + 1e-30
    assert np.array_equal(gm, tdo.choose_master(o.hr, gt))
    return o, gs, gi, gn, gt, gm


def spec_of(**kw):
    d = dict(H=8, T=16, theta=1.0e6, sessions=2, agents=5, blocks=3, block_tokens=70, hist=(0, 300), frac=0.2)
    d.update(kw)
    return wl.RoundSpec("chk", 66, 2, d["H"], 128, d["T"], d["theta"], d["sessions"], d["agents"], d["blocks"],
                        d["block_tokens"], d["hist"][0], d["hist"][1], d["frac"])


def test_refreshed_tokens_are_the_important_positions(tdo):
    rnd = wl.make_round(spec_of())
    o, gs, gi, gn, gt, gm = run_case(tdo, rnd, 1.0, 0.0)
    T = rnd.spec.page_tokens
    S = rnd.spec.span_tokens
    for i in range(rnd.n_agents):
        toks = np.concatenate([np.arange(p * T, min(S, (p + 1) * T)) for p in rnd.perturbed[i]])
        assert np.array_equal(gi[i, :gn[i]], toks)


@pytest.mark.parametrize("ratio,min_score", [(0.15, 0.0), (0.05, 0.0), (0.5, 2.0), (1.0, 1e9)])
def test_noise_on_every_token(tdo, ratio, min_score):
    run_case(tdo, wl.make_round(spec_of()), ratio, min_score, noise_everywhere=0.02)


def test_many_exact_ties_and_zeros(tdo):
    """Only a few distinct score values: the tie-break (lower token first) decides most of the list."""
    def fill(o):
        o.rerotate()
        rows = np.concatenate([o.rnd.dst_rows(i) for i in range(o.rnd.n_agents)])
        pick = rows[::3]
        o.pk[pick, 5] = np.uint16(0x4000)          # the same element set to 2.0 on every third token
    run_case(tdo, wl.make_round(spec_of(frac=0.0)), 0.2, 0.0, fill=fill)


@pytest.mark.parametrize("kw,style", [(dict(H=4), 0), (dict(T=32), 0), (dict(H=8), 1), (dict(hist=(5000, 30000), theta=5.0e5), 0),
                                      (dict(H=1), 0), (dict(H=3, T=32), 1), (dict(H=2, agents=33, sessions=1), 0)])
def test_geometries(tdo, kw, style):
    run_case(tdo, wl.make_round(spec_of(**kw)), 0.15, 0.0, noise_everywhere=0.02, style=style)


def test_nan_scores_and_argument_errors(tdo):
    import torch
    from paper_2604_03143_amd import tdk
    def fill(o):
        o.rerotate()
        o.pk[int(o.rnd.dst_rows(1, np.array([9]))[0]), 100] = 0x7FC0
    o, gs, gi, gn, gt, gm = run_case(tdo, wl.make_round(spec_of(frac=0.0, sessions=1, agents=3)), 0.1, 0.0, fill=fill)
    assert gn.tolist() == [0, 1, 0] and gi[1, 0] == 9
    assert gm.tolist() == [0]          # the NaN total of agent 1 counts as +inf; 0 and 2 tie at 0 -> first
    import gpu_helpers as gh
    rnd = wl.make_round(spec_of(sessions=1, agents=2))
    g = gh.GpuRun(rnd)
    try:
        z = torch.zeros(2048, dtype=torch.float32, device="cuda")
        zi = torch.zeros(2048, dtype=torch.int32, device="cuda")
        for ratio, ms, ks in ((0.0, 0.0, 64), (1.5, 0.0, 64), (0.1, -1.0, 64), (0.1, float("nan"), 64), (0.5, 0.0, 8)):
            with pytest.raises(tdk.TdkError):
                tdk.tdk_check_layer(g.r, 0, g.io, ratio, ms, tdk.reuse_plan(z, zi, ks, zi, z, zi))
    finally:
        g.close()


def test_check_layer_with_permuted_blocks(tdo):
    rnd = wl.permute_blocks(wl.make_round(spec_of(blocks=4, block_tokens=45)))
    run_case(tdo, rnd, 0.15, 0.0, noise_everywhere=0.02)
