"""Parity at the full sizes of the benchmark configurations, one layer, in the launch shape bench.py
times (automatic agent groups, default flags): sampled agents against the oracle bit for bit, and
properties that hold at any size for everything else; then the attention call over the same mirrors, the
sampled agents against the oracle by tolerance."""
import numpy as np
import pytest

from paper_2604_03143_amd import workload as wl

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["batched250", "long", "llama70b"])
def test_full_size_layer(tdo, name):
    import torch
    from paper_2604_03143_amd import tdk
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

    # sampled agents: first, last, and a few seeded ones (different sessions where there are several)
    pick = sorted(set([0, A - 1] + np.random.default_rng(5).choice(A, size=3, replace=False).tolist()))
    sub, page_map = wl.subround(rnd, pick)
    srows = (torch.from_numpy(page_map).to(dev)[:, None] * T + torch.arange(T, device=dev)[None, :]).reshape(-1)
    sess = sub.extra["sessions"]
    m_rows = np.concatenate([np.arange(rnd.master_row0[s], rnd.master_row0[s + 1]) for s in sess])
    m_rows_d = torch.from_numpy(m_rows).to(dev)
    hmk = mk[m_rows_d].cpu().numpy().view(np.uint16)
    hmv = mv[m_rows_d].cpu().numpy().view(np.uint16)
    g = tdo.geom_of(spec)
    hr = tdo.HostRound(sub)
    shared = wl.shared_row_mask(sub)

    def sample():
        torch.cuda.synchronize()
        return pk[srows].cpu().numpy().view(np.uint16), pv[srows].cpu().numpy().view(np.uint16)

    # --- rerotate
    tdk.tdk_rerotate_round(r, layer, io, st)
    gk, gv = sample()
    ok = np.zeros_like(gk); ov = np.zeros_like(gv)
    tdo.rerotate_round(g, hr, hmk, hmv, ok, ov)
    assert np.array_equal(gk, ok) and np.array_equal(gv, ov)
    # V rows are copies of the master everywhere (property, all agents): spot-check a seeded agent in full
    a = int(pick[1])
    s0 = int(rnd.master_row0[rnd.agent_session[a]])
    S = int(rnd.span_tokens[rnd.agent_session[a]])
    dst = torch.from_numpy(rnd.dst_rows(a)).to(dev)
    assert torch.equal(pv[dst], mv[s0:s0 + S])

    # --- the model refreshes the seeded pages; encode
    wl.perturb_device(rnd, layer, pk, pv)
    n_pert = sum(len(p) for p in rnd.perturbed)
    cap = n_pert + 7
    pe = 2 * T * RE
    count = torch.zeros(A, dtype=torch.int32, device=dev)
    offset = torch.zeros(A + 1, dtype=torch.int64, device=dev)
    idx = torch.full((cap,), -1, dtype=torch.int32, device=dev)
    payload = torch.zeros((cap, pe), dtype=torch.int16, device=dev)
    ovf = torch.zeros(1, dtype=torch.int32, device=dev)
    d = tdk.diff(count, offset, idx, payload, cap, ovf)
    tdk.tdk_diff_encode(r, layer, io, spec.eps, d, st)
    torch.cuda.synchronize()
    h_off, h_idx, h_cnt = offset.cpu().numpy(), idx.cpu().numpy(), count.cpu().numpy()
    assert int(ovf.item()) == 0 and int(h_off[-1]) == n_pert
    assert np.array_equal(h_off, np.concatenate([[0], np.cumsum(h_cnt)]))
    for i in range(A):                      # ground truth that needs no oracle
        assert np.array_equal(h_idx[h_off[i]:h_off[i + 1]], rnd.perturbed[i])
    mir_k, mir_v = sample()
    od = tdo.diff_encode(g, hr, hmk, hmv, mir_k, mir_v, spec.eps, len(pick) * spec.span_pages)
    for j, ag in enumerate(pick):
        lo, n = int(h_off[ag]), int(h_cnt[ag])
        assert n == int(od.count[j])
        o0 = int(od.offset[j])
        assert np.array_equal(h_idx[lo:lo + n], od.idx[o0:o0 + n])
        assert np.array_equal(payload[lo:lo + n].cpu().numpy().view(np.uint16), od.payload[o0:o0 + n])

    # --- decode into a second, empty pool: the whole pool must come back (on-device compare)
    pk2, pv2 = torch.zeros_like(pk), torch.zeros_like(pv)
    io2 = tdk.layer_io(mk, mv, pk2, pv2, rnd.pool_pages)
    tdk.tdk_diff_decode(r, layer, io2, d, st)
    torch.cuda.synchronize()
    assert torch.equal(pk2, pk) and torch.equal(pv2, pv)
    dk, dv = ok.copy(), ov.copy()
    tdo.diff_decode(g, hr, hmk, hmv, dk, dv, od)
    assert np.array_equal(pk2[srows].cpu().numpy().view(np.uint16)[shared], dk[shared])
    assert np.array_equal(pv2[srows].cpu().numpy().view(np.uint16)[shared], dv[shared])

    # --- attention over the never-restored mirrors (one query token, 5 query heads per KV head: the shape
    # bench.py --mode attend times), the sampled agents against the oracle by the tolerances of test_gpu_attend.py
    n_q, Hq, D = 1, 5 * spec.num_kv_heads, spec.head_dim
    gen = torch.Generator(device=dev); gen.manual_seed(11)
    q = torch.randn((A, n_q, Hq, D), generator=gen, device=dev).to(torch.bfloat16).view(torch.int16)
    out = torch.full((A, n_q, Hq, D), float("nan"), dtype=torch.float32, device=dev)
    lse = torch.full((A, n_q, Hq), float("nan"), dtype=torch.float32, device=dev)
    nbytes = tdk.tdk_attend_workspace_bytes(r, n_q, Hq)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    pick_d = torch.tensor(pick, device=dev)
    vmax = float(np.max(np.abs(wl.bf16_bits_to_f32(hmv))))
    # the usual scale, then scale 1 (near one-hot weights: any token dropped, doubled or taken from the wrong
    # source moves the rows it dominates far above the bound; bounds as derived in test_gpu_attend.py)
    for scale, lse_tol in ((1.0 / float(np.sqrt(D)), 5e-3), (1.0, 8e-3)):
        k = scale * float(np.sqrt(D))
        out.fill_(float("nan")); lse.fill_(float("nan"))
        tdk.tdk_attend_shared(r, layer, io, d, tdk.attend_io(q, n_q, Hq, scale, out, lse, ws, nbytes), st)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(out).all()) and bool(torch.isfinite(lse).all())
        want_o, want_l = tdo.attend_shared(g, hr, hmk, hmv, od, q[pick_d].cpu().numpy().view(np.uint16), n_q, Hq, scale)
        err_o = float(np.max(np.abs(out[pick_d].cpu().numpy().astype(np.float64) - want_o)))
        err_l = float(np.max(np.abs(lse[pick_d].cpu().numpy().astype(np.float64) - want_l)))
        assert err_o <= k * 1e-2 * max(1.0, vmax) and err_l <= k * lse_tol, (scale, err_o, err_l)
    r.destroy()
