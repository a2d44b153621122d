"""From token ids to attention: prompts with separator tokens are planned on the host (Sec. 4.1), the plan's
segment lists build the round, the collective rerotate places every shared block at each agent's positions
(bit-exact against the oracle), and new queries attend to the shared blocks straight from the master."""
from types import SimpleNamespace

import numpy as np
import pytest

from paper_2604_03143_amd import workload as wl

pytestmark = pytest.mark.gpu
SEP = 151_000


def test_prompts_to_round_to_attention(tdo):
    import torch
    from paper_2604_03143_amd import tdk
    import gpu_helpers as gh
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    g = np.random.default_rng(21)
    T, H, D = 16, 2, 128
    shared = [list(g.integers(0, 150_000, size=n)) for n in (40, 57, 23, 64)]     # the round's shared updates
    prompts = []
    for hist, order in ((37, (0, 1, 2, 3)), (5, (2, 0, 3, 1)), (211, (3, 2, 1, 0)), (90, (1, 3, 0, 2))):
        p = list(g.integers(0, 150_000, size=hist))
        for k in order:
            p += [SEP] + shared[k]
        prompts.append(p + [SEP] + list(g.integers(0, 150_000, size=9)))            # the round's task, private
    spans, session_of, segs = tdk.tdk_prompt_plan(prompts, SEP)
    assert spans == [184] and session_of == [0, 0, 0, 0]
    # paged KV memory: every prompt gets its own pages, scattered
    n_pages = [-(-len(p) // T) for p in prompts]
    perm = g.permutation(sum(n_pages) + 3)
    tables, at = [], 0
    for n in n_pages:
        tables.append(perm[at:at + n].astype(np.int32))
        at += n
    pool_pages = int(perm.max()) + 1
    seg_arr = [np.array(s, np.int64).reshape(-1, 3) for s in segs]
    rnd = SimpleNamespace(span_tokens=np.array(spans, np.int32), master_pos0=np.zeros(1, np.int64),
                          agent_session=np.zeros(4, np.int32), agent_pos0=np.array([s[0][1] for s in segs], np.int64),
                          block_tables=tables, segments=seg_arr, pool_pages=pool_pages)
    geom = tdo.geom(H, D, T, 1.0e6)
    hr = tdo.HostRound(rnd)
    S, re = spans[0], H * D
    mk = wl.f32_to_bf16_bits(g.standard_normal((S, re)).astype(np.float32))
    mv = wl.f32_to_bf16_bits(g.standard_normal((S, re)).astype(np.float32))
    pk = np.full((pool_pages * T, re), 0x7FC1, np.uint16)
    pv = pk.copy()
    opk, opv = pk.copy(), pv.copy()
    tdo.rerotate_round(geom, hr, mk, mv, opk, opv)

    r = tdk.tdk_round_create(tdk.model(1, H, D, T, 1.0e6), spans, [0], [0] * 4, rnd.agent_pos0, tables, None, seg_arr)
    try:
        dmk, dmv, dpk, dpv = gh.up(mk), gh.up(mv), gh.up(pk), gh.up(pv)
        io = tdk.layer_io(dmk, dmv, dpk, dpv, pool_pages)
        tdk.tdk_rerotate_round(r, 0, io)
        torch.cuda.synchronize()
        assert np.array_equal(gh.down16(dpk), opk) and np.array_equal(gh.down16(dpv), opv)
        # every shared token sits where the prompt has it: block k of agent i at the position of its first token
        for i, p in enumerate(prompts):
            for (src, dst, n) in segs[i]:
                rows = tables[i][(dst + np.arange(n)) // T].astype(np.int64) * T + (dst + np.arange(n)) % T
                assert np.array_equal(opv[rows], mv[src:src + n])
        # nothing was refreshed: empty diff; 2 query tokens per agent, 6 query heads
        d = gh.DevDiff(4, 4, 2 * T * re)
        tdk.tdk_diff_encode(r, 0, io, 1e-2, d.c)
        torch.cuda.synchronize()
        assert int(d.offset.cpu()[-1]) == 0
        n_q, Hq, scale = 2, 6, 1.0 / np.sqrt(D)
        q = wl.f32_to_bf16_bits(g.standard_normal((4, n_q, Hq, D)).astype(np.float32))
        od = tdo.Diff(4, 0, 2 * T * re)
        want_o, want_l = tdo.attend_shared(geom, hr, mk, mv, od, q, n_q, Hq, scale)
        nbytes = tdk.tdk_attend_workspace_bytes(r, n_q, Hq)
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        out = torch.zeros((4, n_q, Hq, D), dtype=torch.float32, device="cuda")
        lse = torch.zeros((4, n_q, Hq), dtype=torch.float32, device="cuda")
        tdk.tdk_attend_shared(r, 0, io, d.c, tdk.attend_io(gh.up(q), n_q, Hq, scale, out, lse, ws, nbytes))
        torch.cuda.synchronize()
        assert float(np.max(np.abs(out.cpu().numpy() - want_o))) <= 1e-2 * max(1.0, float(np.abs(wl.bf16_bits_to_f32(mv)).max()))
        assert float(np.max(np.abs(lse.cpu().numpy() - want_l))) <= 5e-3
    finally:
        r.destroy()
