"""Parity at the full sizes of the benchmark configurations, in the launch shape bench.py times (automatic
agent groups, default flags): EVERY agent of the round against the oracle, bit for bit, on layer 0 and on one
seeded layer, for rerotate, encode (count, offset, idx, payload) and decode.  Grouping agents into work items
and batching sessions must change the order of the work, never the result (Sec. 6.6).  The pool is brought to
the host in pieces of at most 25 agents of one session, so that the oracle's copies stay small.  Then the
attention call over the same mirrors: sampled agents against the oracle, by the per-row bound derived in
attend_bounds.py."""
import numpy as np
import pytest

from paper_2604_03143_amd import workload as wl

pytestmark = pytest.mark.gpu

PIECE = 25     # agents per host-side piece


def seeded_layer(spec):
    return int(np.random.default_rng([wl.SEED_BASE, spec.stream, 77]).integers(1, spec.num_layers))


def agent_pieces(rnd):
    """Agents grouped by session, each session cut into pieces of at most PIECE agents."""
    out = []
    for s in range(rnd.n_sessions):
        ids = np.nonzero(rnd.agent_session == s)[0]
        for k in range(0, len(ids), PIECE):
            out.append([int(a) for a in ids[k:k + PIECE]])
    return out


class Piece:
    """The host view of some agents of a round: compact block tables and the pool rows behind them."""

    def __init__(self, tdo, rnd, agents, mk, mv, dev):
        import torch
        T = rnd.spec.page_tokens
        self.agents = agents
        self.sub, page_map = wl.subround(rnd, agents)
        self.rows = (torch.from_numpy(page_map).to(dev)[:, None] * T + torch.arange(T, device=dev)[None, :]).reshape(-1)
        sess = self.sub.extra["sessions"]
        m_rows = np.concatenate([np.arange(rnd.master_row0[s], rnd.master_row0[s + 1]) for s in sess])
        m_rows = torch.from_numpy(m_rows).to(dev)
        self.mk = mk[m_rows].cpu().numpy().view(np.uint16)
        self.mv = mv[m_rows].cpu().numpy().view(np.uint16)
        self.hr = tdo.HostRound(self.sub)
        self.shared = wl.shared_row_mask(self.sub)

    def sample(self, pk, pv):
        return pk[self.rows].cpu().numpy().view(np.uint16), pv[self.rows].cpu().numpy().view(np.uint16)


@pytest.mark.parametrize("which", ["layer0", "seeded"])
@pytest.mark.parametrize("name", ["session", "batched250", "long", "llama70b"])
def test_every_agent_against_the_oracle(tdo, name, which):
    import torch
    from paper_2604_03143_amd import tdk
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    tdk.load()
    spec = wl.CONFIGS[name]
    rnd = wl.make_round(spec)
    layer = 0 if which == "layer0" else seeded_layer(spec)
    dev = torch.device("cuda:0")
    T, RE, A = spec.page_tokens, spec.row_elems, rnd.n_agents
    rows = rnd.pool_pages * T
    mk, mv = wl.master_device(rnd, layer, dev)
    pk = torch.zeros((rows, RE), dtype=torch.int16, device=dev)
    pv = torch.zeros((rows, RE), dtype=torch.int16, device=dev)
    r = tdk.round_from_workload(rnd)
    io = tdk.layer_io(mk, mv, pk, pv, rnd.pool_pages)
    st = torch.cuda.current_stream().cuda_stream
    g = tdo.geom_of(spec)
    pieces = [Piece(tdo, rnd, ag, mk, mv, dev) for ag in agent_pieces(rnd)]
    assert sorted(a for p in pieces for a in p.agents) == list(range(A))

    # --- rerotate: every row of every agent's pages (rows outside the spans stay as they were: zero)
    tdk.tdk_rerotate_round(r, layer, io, st)
    torch.cuda.synchronize()
    for p in pieces:
        gk, gv = p.sample(pk, pv)
        ok = np.zeros_like(gk); ov = np.zeros_like(gv)
        tdo.rerotate_round(g, p.hr, p.mk, p.mv, ok, ov)
        assert np.array_equal(gk, ok) and np.array_equal(gv, ov), ("rerotate", p.agents[0])

    # --- the model refreshes the seeded pages; encode the whole round, decode it into a second, empty pool
    wl.perturb_device(rnd, layer, pk, pv)
    n_pert = sum(len(q) for q in rnd.perturbed)
    cap = n_pert + 7
    pe = 2 * T * RE
    count = torch.zeros(A, dtype=torch.int32, device=dev)
    offset = torch.zeros(A + 1, dtype=torch.int64, device=dev)
    idx = torch.full((cap,), -1, dtype=torch.int32, device=dev)
    payload = torch.zeros((cap, pe), dtype=torch.int16, device=dev)
    ovf = torch.zeros(1, dtype=torch.int32, device=dev)
    d = tdk.diff(count, offset, idx, payload, cap, ovf)
    tdk.tdk_diff_encode(r, layer, io, spec.eps, d, st)
    pk2, pv2 = torch.zeros_like(pk), torch.zeros_like(pv)
    io2 = tdk.layer_io(mk, mv, pk2, pv2, rnd.pool_pages)
    tdk.tdk_diff_decode(r, layer, io2, d, st)
    torch.cuda.synchronize()
    h_off, h_idx, h_cnt = offset.cpu().numpy(), idx.cpu().numpy(), count.cpu().numpy()
    assert int(ovf.item()) == 0 and int(h_off[-1]) == n_pert
    assert np.array_equal(h_off, np.concatenate([[0], np.cumsum(h_cnt)]))
    for i in range(A):                      # ground truth that needs no oracle
        assert np.array_equal(h_idx[h_off[i]:h_off[i + 1]], rnd.perturbed[i])
    assert torch.equal(pk2, pk) and torch.equal(pv2, pv)        # the round trip, whole pool, on the device
    for p in pieces:
        mir_k, mir_v = p.sample(pk, pv)
        od = tdo.diff_encode(g, p.hr, p.mk, p.mv, mir_k, mir_v, spec.eps, len(p.agents) * spec.span_pages)
        assert int(od.overflow[0]) == 0
        lo = int(h_off[p.agents[0]])
        n = int(od.offset[-1])
        # the agents of a piece are consecutive in the round, so are their payload slots
        assert p.agents == list(range(p.agents[0], p.agents[0] + len(p.agents)))
        assert np.array_equal(h_cnt[p.agents[0]:p.agents[0] + len(p.agents)], od.count), ("count", p.agents[0])
        assert np.array_equal(h_off[p.agents[0]:p.agents[0] + len(p.agents) + 1] - lo, od.offset), ("offset", p.agents[0])
        assert np.array_equal(h_idx[lo:lo + n], od.idx[:n]), ("idx", p.agents[0])
        assert np.array_equal(payload[lo:lo + n].cpu().numpy().view(np.uint16), od.payload[:n]), ("payload", p.agents[0])
        dk = np.zeros_like(mir_k); dv = np.zeros_like(mir_v)
        tdo.diff_decode(g, p.hr, p.mk, p.mv, dk, dv, od)
        gk, gv = p.sample(pk2, pv2)
        assert np.array_equal(gk, dk) and np.array_equal(gv, dv), ("decode", p.agents[0])
    r.destroy()


@pytest.mark.parametrize("name", ["batched250", "long", "llama70b"])
def test_attention_over_mirrors_at_full_size(tdo, name):
    """One query token, 5 query heads per KV head (the shape bench.py --mode attend times): sampled agents against
    the oracle, by the per-row bounds of attend_bounds.py, at the usual scale and at scale 1 (near one-hot weights:
    a token dropped, doubled or taken from the wrong source moves the rows it dominates by O(|V|))."""
    import torch
    from paper_2604_03143_amd import tdk
    import attend_bounds as ab
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    tdk.load()
    spec = wl.CONFIGS[name]
    rnd = wl.make_round(spec)
    layer = 3
    dev = torch.device("cuda:0")
    T, RE, A = spec.page_tokens, spec.row_elems, rnd.n_agents
    rows = rnd.pool_pages * T
    mk, mv = wl.master_device(rnd, layer, dev)
    pk = torch.zeros((rows, RE), dtype=torch.int16, device=dev)
    pv = torch.zeros((rows, RE), dtype=torch.int16, device=dev)
    r = tdk.round_from_workload(rnd)
    io = tdk.layer_io(mk, mv, pk, pv, rnd.pool_pages)
    st = torch.cuda.current_stream().cuda_stream
    g = tdo.geom_of(spec)
    pick = sorted(set([0, A - 1] + np.random.default_rng(5).choice(A, size=3, replace=False).tolist()))
    p = Piece(tdo, rnd, pick, mk, mv, dev)
    tdk.tdk_rerotate_round(r, layer, io, st)
    wl.perturb_device(rnd, layer, pk, pv)
    n_pert = sum(len(q) for q in rnd.perturbed)
    cap = n_pert + 7
    count = torch.zeros(A, dtype=torch.int32, device=dev)
    offset = torch.zeros(A + 1, dtype=torch.int64, device=dev)
    idx = torch.full((cap,), -1, dtype=torch.int32, device=dev)
    payload = torch.zeros((cap, 2 * T * RE), dtype=torch.int16, device=dev)
    ovf = torch.zeros(1, dtype=torch.int32, device=dev)
    d = tdk.diff(count, offset, idx, payload, cap, ovf)
    tdk.tdk_diff_encode(r, layer, io, spec.eps, d, st)
    torch.cuda.synchronize()
    mir_k, mir_v = p.sample(pk, pv)
    od = tdo.diff_encode(g, p.hr, p.mk, p.mv, mir_k, mir_v, spec.eps, len(pick) * spec.span_pages)

    n_q, Hq, D = 1, 5 * spec.num_kv_heads, spec.head_dim
    gen = torch.Generator(device=dev); gen.manual_seed(11)
    q = torch.randn((A, n_q, Hq, D), generator=gen, device=dev).to(torch.bfloat16).view(torch.int16)
    out = torch.full((A, n_q, Hq, D), float("nan"), dtype=torch.float32, device=dev)
    lse = torch.full((A, n_q, Hq), float("nan"), dtype=torch.float32, device=dev)
    nbytes = tdk.tdk_attend_workspace_bytes(r, n_q, Hq)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    pick_d = torch.tensor(pick, device=dev)
    hq = q[pick_d].cpu().numpy().view(np.uint16)
    for scale in (1.0 / float(np.sqrt(D)), 1.0):
        out.fill_(float("nan")); lse.fill_(float("nan"))
        tdk.tdk_attend_shared(r, layer, io, d, tdk.attend_io(q, n_q, Hq, scale, out, lse, ws, nbytes), st)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(out).all()) and bool(torch.isfinite(lse).all())
        want_o, want_l, tol_o, tol_l = ab.expected_and_bounds(tdo, g, p.hr, p.mk, p.mv, od, hq, n_q, Hq, scale)
        got_o = out[pick_d].cpu().numpy().astype(np.float64)
        got_l = lse[pick_d].cpu().numpy().astype(np.float64)
        ab.assert_within(got_o, got_l, want_o, want_l, tol_o, tol_l, what=(name, scale))
        if scale < 1.0:
            # the bound has teeth at the usual scale too: an output taken from the neighbouring KV head, or an
            # output of all zeros, lies outside it (planted in the expected value, the kernel is untouched)
            G = Hq // spec.num_kv_heads
            wrong = np.roll(want_o, G, axis=2)
            assert not ab.within(got_o, got_l, wrong, want_l, tol_o, tol_l)
            assert not ab.within(np.zeros_like(got_o), got_l, want_o, want_l, tol_o, tol_l)
    r.destroy()
