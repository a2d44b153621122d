"""Attention over mirrors that are never restored (Sec. 4.4, the diff applied as attention tiles are loaded),
through the C ABI against the oracle.  The GPU path rounds the back-rotated queries and the softmax weights
to bf16 for its two MFMA products and accumulates in fp32, so the comparison is by tolerance: a bound per query
row and output element, derived from that arithmetic in attend_bounds.py (score error from the bf16 queries,
2^-8 for the bf16 weights, both times the row's own sum of weights x |V|; the log-sum-exp within the score
error).  A wrong table sign, head mapping, page mask or plane offset moves the results far outside it."""
import numpy as np
import pytest

import attend_bounds as ab
from paper_2604_03143_amd import workload as wl
from helpers import OracleRun

pytestmark = pytest.mark.gpu


def _case(tdo, spec, n_q, Hq, style=0, grow=None, seed=3, scale=None, perturb=True):
    import torch
    from paper_2604_03143_amd import tdk
    import gpu_helpers as gh
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    old = wl.make_round(spec)
    o = OracleRun(tdo, old, style=style)
    o.rerotate()
    if perturb:
        o.perturb()
    d = o.encode()
    rnd, diff_pos0 = old, None
    if grow is not None:
        rnd = wl.make_round(spec, hist=old.agent_pos0 + np.asarray(grow, np.int64))
        diff_pos0 = old.agent_pos0
    g = np.random.default_rng([spec.stream, seed])
    q = wl.f32_to_bf16_bits(g.standard_normal((rnd.n_agents, n_q, Hq, spec.head_dim)).astype(np.float32))
    scale = 1.0 / np.sqrt(spec.head_dim) if scale is None else scale
    want_o, want_l, tol_o, tol_l = ab.expected_and_bounds(tdo, o.g, tdo.HostRound(rnd, diff_pos0=diff_pos0), o.mk, o.mv, d,
                                                          q, n_q, Hq, scale)

    r = tdk.round_from_workload(rnd, style=style, diff_pos0=diff_pos0)
    try:
        n = int(d.offset[-1])
        mk, mv = gh.up(o.mk), gh.up(o.mv)
        cnt, off = torch.from_numpy(d.count).cuda(), torch.from_numpy(d.offset).cuda()
        idx, pay = torch.from_numpy(d.idx[:max(n, 1)].copy()).cuda(), gh.up(d.payload[:max(n, 1)].copy())
        dd = tdk.diff(cnt, off, idx, pay, n, torch.zeros(1, dtype=torch.int32, device="cuda"))
        io = tdk.layer_io(mk, mv, None, None, 0)
        nbytes = tdk.tdk_attend_workspace_bytes(r, n_q, Hq)
        assert nbytes > 0
        ws = torch.empty(nbytes + 256, dtype=torch.uint8, device="cuda")
        ws.fill_(0xFF)                                   # NaN patterns: stale workspace must not leak into results
        out = torch.full((rnd.n_agents, n_q, Hq, spec.head_dim), float("nan"), dtype=torch.float32, device="cuda")
        lse = torch.full((rnd.n_agents, n_q, Hq), float("nan"), dtype=torch.float32, device="cuda")
        a = tdk.attend_io(gh.up(q), n_q, Hq, scale, out, lse, ws, nbytes)
        tdk.tdk_attend_shared(r, 0, io, dd, a, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        got_o, got_l = out.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64)
    finally:
        r.destroy()
    return ab.assert_within(got_o, got_l, want_o, want_l, tol_o, tol_l, what=(spec.name, n_q, Hq, scale))


def test_one_query_token_per_agent(tdo):
    """Decode step: 1 query token, 40 query heads on 8 KV heads, ragged span, several tiles and chunks."""
    spec = wl.RoundSpec("att", 61, 1, 8, 128, 16, 1.0e6, 2, 5, 4, 73, 5, 3000, 0.2)
    _case(tdo, spec, 1, 40)


@pytest.mark.parametrize("scale", [-0.11, 0.0, 0.25, 1.0])
def test_negative_zero_and_large_scales(tdo, scale):
    """The kernels work with the magnitude of the scale and carry its sign in the query copies; a zero scale
    gives uniform weights (out = mean of V over the span, lse = log S).  At scale 1 the softmax of random data is
    nearly one-hot (scores of +-30): a token that is dropped, counted twice or taken from the wrong source moves
    the rows it dominates by O(|V|), far above the bound, which flat weights would hide."""
    spec = wl.RoundSpec("att6", 66, 1, 2, 128, 16, 1.0e6, 1, 3, 3, 50, 0, 300, 0.3)
    _case(tdo, spec, 2, 6, scale=scale)


def test_sharp_weights_on_several_sessions_and_moved_diffs(tdo):
    """The same near one-hot weights on a round with two sessions, ragged pages, 40 query heads on 8 KV heads and
    mirrors stored when the histories were shorter (payload keys meet turned-back queries)."""
    spec = wl.RoundSpec("att9", 69, 1, 8, 128, 16, 1.0e6, 2, 4, 4, 73, 5, 900, 0.25)
    # With one token carrying nearly all the weight the log-sum-exp takes that token's score error whole (no
    # averaging over tokens), which is what the per-row bound allows for.
    _case(tdo, spec, 1, 40, scale=1.0, grow=[0, 16, 7, 250, 1, 31, 1000, 64])


@pytest.mark.parametrize("n_q,Hq", [(1, 6), (9, 6)])
def test_no_page_listed(tdo, n_q, Hq):
    """Mirrors identical to the rotated master: empty diffs (capacity 0), the listed-pages pass finds nothing and
    the merge takes the master pass's parts alone."""
    spec = wl.RoundSpec("att10", 70, 1, 2, 128, 16, 1.0e6, 2, 3, 5, 60, 0, 90, 0.2)
    _case(tdo, spec, n_q, Hq, perturb=False)


@pytest.mark.parametrize("n_q,Hq", [(1, 6), (9, 6)])
def test_every_page_listed(tdo, n_q, Hq):
    """Every page of every mirror differs from the master: the master pass has nothing left to do (all its
    scores are switched off), the lists are 44 pages long = six pieces of 128 listed tokens, more than the four
    wavefronts launched per list (the pieces are walked in turn); 3 and 27 rows per agent and KV head."""
    spec = wl.RoundSpec("att8", 68, 1, 2, 128, 16, 1.0e6, 1, 3, 7, 100, 0, 90, 1.0)
    _case(tdo, spec, n_q, Hq)


def test_long_span_with_chunks_above_512_tokens(tdo):
    """Four sessions of 10280 tokens on 8 KV heads: on a 256-CU device the planner gives every workgroup of the
    master pass 704 tokens = 44 pages (more than one 64-bit word of a row's page mask)."""
    spec = wl.RoundSpec("att7", 67, 1, 8, 128, 16, 1.0e6, 4, 3, 40, 257, 5, 900, 0.1)
    _case(tdo, spec, 1, 8)


# (the last two: 48 and 40 rows per agent and KV head, past the shared launch: the three kernels one after another,
#  the listed-pages pass walking its pieces once per block of 32 rows)
@pytest.mark.parametrize("H,Hq,T,style,n_q", [(4, 28, 16, 0, 3), (8, 8, 32, 0, 2), (2, 4, 16, 1, 5), (1, 7, 16, 0, 1),
                                               (2, 8, 16, 0, 12), (1, 5, 32, 1, 8)])
def test_head_counts_page_sizes_styles_and_several_query_tokens(tdo, H, Hq, T, style, n_q):
    spec = wl.RoundSpec("att2", 62, 1, H, 128, T, 1.0e6, 1, 4, 3, 50, 0, 500, 0.3)
    _case(tdo, spec, n_q, Hq, style=style)


def test_more_query_rows_than_one_block_and_mirrors_stored_elsewhere(tdo):
    """160 query rows per KV head (two row blocks), and a diff that was stored when the histories were shorter."""
    spec = wl.RoundSpec("att3", 63, 1, 2, 128, 16, 5.0e5, 1, 8, 3, 40, 10, 200, 0.4)
    _case(tdo, spec, 5, 8, grow=[0, 16, 7, 250, 1, 31, 1000, 64])


@pytest.mark.parametrize("T,style,block_tokens,n_q,Hq", [(16, 0, 40, 1, 10), (16, 1, 23, 2, 4), (32, 0, 50, 1, 2), (16, 0, 157, 3, 6)])
def test_agents_with_their_own_block_order(tdo, T, style, block_tokens, n_q, Hq):
    """Every agent orders the shared blocks its own way (Eq. 2): each block has its own offset per agent,
    steps of 64 tokens run over block borders that differ from row to row; two agents keep the identity layout."""
    import torch
    from paper_2604_03143_amd import tdk
    import gpu_helpers as gh
    spec = wl.RoundSpec("att5", 65, 1, 2, 128, T, 1.0e6, 2, 6, 5, block_tokens, 3, 700, 0.25)
    rnd = wl.permute_blocks(wl.make_round(spec), seed_tag=6)
    rnd.segments[1] = np.zeros((0, 3), np.int64)
    rnd.segments[8] = np.zeros((0, 3), np.int64)
    o = OracleRun(tdo, rnd, style=style)
    o.rerotate(); o.perturb()
    d = o.encode()
    g = np.random.default_rng([spec.stream, block_tokens])
    q = wl.f32_to_bf16_bits(g.standard_normal((rnd.n_agents, n_q, Hq, 128)).astype(np.float32))
    scale = 1.0 / np.sqrt(128.0)
    want_o, want_l, tol_o, tol_l = ab.expected_and_bounds(tdo, o.g, o.hr, o.mk, o.mv, d, q, n_q, Hq, scale)
    r = tdk.round_from_workload(rnd, style=style)
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
                         want_o, want_l, tol_o, tol_l, what=(T, style, block_tokens, n_q))
    finally:
        r.destroy()


@pytest.mark.parametrize("T,style,block_tokens,n_q,sharp", [(16, 0, 40, 2, False), (16, 1, 23, 2, False), (32, 0, 50, 2, True),
                                                             (16, 0, 40, 6, False), (16, 0, 40, 2, True), (16, 0, 40, 6, True)])
def test_own_block_order_and_mirrors_stored_under_another_order(tdo, T, style, block_tokens, n_q, sharp):
    """The mirrors were stored in an earlier round, under another block order and shorter histories: every
    block of a listed page meets the queries turned back by its own distance; one agent did not move at all."""
    import torch
    from paper_2604_03143_amd import tdk
    import gpu_helpers as gh
    spec = wl.RoundSpec("att6", 66, 1, 2, 128, T, 1.0e6, 2, 4, 4, block_tokens, 5, 300, 0.3)
    old = wl.permute_blocks(wl.make_round(spec), seed_tag=4)
    old.segments[5] = np.zeros((0, 3), np.int64)
    o = OracleRun(tdo, old, style=style)
    o.rerotate(); o.perturb()
    d = o.encode()
    grow = np.array([0, 16, 7, 250, 1, 31, 1000, 64], np.int64)
    new = wl.permute_blocks(wl.make_round(spec, hist=old.agent_pos0 + grow), seed_tag=9)
    new.segments[5] = np.zeros((0, 3), np.int64)
    new.segments[0] = old.segments[0].copy()
    seg_diff = [sg[:, 1] if len(sg) else np.zeros(0, np.int64) for sg in old.segments]
    Hq = 6                                          # 3 query heads per KV head: 6 or 18 rows per agent and KV head
    scale = 1.0 if sharp else 1.0 / np.sqrt(128.0)  # sharp: near one-hot weights
    g = np.random.default_rng([spec.stream, T, block_tokens])
    q = wl.f32_to_bf16_bits(g.standard_normal((new.n_agents, n_q, Hq, 128)).astype(np.float32))
    hr = tdo.HostRound(new, diff_pos0=old.agent_pos0, segment_diff_pos=seg_diff)
    want_o, want_l, tol_o, tol_l = ab.expected_and_bounds(tdo, o.g, hr, o.mk, o.mv, d, q, n_q, Hq, scale)
    r = tdk.round_from_workload(new, style=style, diff_pos0=old.agent_pos0, segment_diff_pos=seg_diff)
    try:
        n = int(d.offset[-1])
        mk, mv = gh.up(o.mk), gh.up(o.mv)
        cnt, off = torch.from_numpy(d.count).cuda(), torch.from_numpy(d.offset).cuda()
        idx, pay = torch.from_numpy(d.idx[:n].copy()).cuda(), gh.up(d.payload[:n].copy())
        dd = tdk.diff(cnt, off, idx, pay, n, torch.zeros(1, dtype=torch.int32, device="cuda"))
        nbytes = tdk.tdk_attend_workspace_bytes(r, n_q, Hq)
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        ws.fill_(0xFF)
        out = torch.full((new.n_agents, n_q, Hq, 128), float("nan"), dtype=torch.float32, device="cuda")
        lse = torch.full((new.n_agents, n_q, Hq), float("nan"), dtype=torch.float32, device="cuda")
        tdk.tdk_attend_shared(r, 0, tdk.layer_io(mk, mv, None, None, 0), dd,
                              tdk.attend_io(gh.up(q), n_q, Hq, scale, out, lse, ws, nbytes))
        torch.cuda.synchronize()
        ab.assert_within(out.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64),
                         want_o, want_l, tol_o, tol_l, what=(T, style, block_tokens, n_q, sharp))
    finally:
        r.destroy()


def test_argument_errors(tdo):
    import torch
    from paper_2604_03143_amd import tdk
    import gpu_helpers as gh
    spec = wl.RoundSpec("att4", 64, 1, 2, 128, 16, 1.0e6, 1, 2, 2, 20, 0, 50, 0.5)
    rnd = wl.make_round(spec)
    r = tdk.round_from_workload(rnd)
    try:
        assert tdk.tdk_attend_workspace_bytes(r, 1, 3) == 0 and tdk.tdk_attend_workspace_bytes(r, 0, 2) == 0
        nbytes = tdk.tdk_attend_workspace_bytes(r, 1, 2)
        mk, mv = (gh.up(x) for x in wl.master_host(rnd, 0))      # kept alive: layer_io holds raw pointers
        io = tdk.layer_io(mk, mv, None, None, 0)
        d = gh.DevDiff(rnd.n_agents, 4, 2 * 16 * 256)
        d.count.zero_(); d.offset.zero_()
        q = torch.zeros((2, 1, 2, 128), dtype=torch.int16, device="cuda")
        out = torch.zeros((2, 1, 2, 128), dtype=torch.float32, device="cuda")
        lse = torch.zeros((2, 1, 2), dtype=torch.float32, device="cuda")
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        for bad in (tdk.attend_io(q, 1, 2, 1.0, out, lse, ws, nbytes - 1), tdk.attend_io(q, 1, 3, 1.0, out, lse, ws, nbytes),
                    tdk.attend_io(None, 1, 2, 1.0, out, lse, ws, nbytes), tdk.attend_io(q, 1, 2, float("inf"), out, lse, ws, nbytes)):
            with pytest.raises(tdk.TdkError):
                tdk.tdk_attend_shared(r, 0, io, d.c, bad)
        tdk.tdk_attend_shared(r, 0, io, d.c, tdk.attend_io(q, 1, 2, 1.0, out, lse, ws, nbytes))
        torch.cuda.synchronize()
        # zero queries: uniform weights, lse = log S
        assert torch.allclose(lse, torch.full_like(lse, float(np.log(spec.span_tokens))), atol=1e-4)
    finally:
        r.destroy()
