"""Layerwise ping-pong restore (Alg. 1) through the C ABI against the oracle, layer by layer."""
import numpy as np
import pytest

from paper_2604_03143_amd import workload as wl
from helpers import OracleRun

pytestmark = pytest.mark.gpu


def _setup(tdo, layers=5, **kw):
    import torch
    from paper_2604_03143_amd import tdk
    import gpu_helpers as gh
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    spec = wl.RoundSpec("restore", 55, layers, 8, 128, 16, 1.0e6, 2, 4, 3, 70, 5, 300, 0.15)
    rnd = wl.make_round(spec)
    runs, diffs, want = [], [], []
    for layer in range(layers):
        o = OracleRun(tdo, rnd, layer=layer)
        o.rerotate(); o.perturb()
        diffs.append(o.encode())
        want.append((o.pk.copy(), o.pv.copy()))
        runs.append(o)
    return torch, tdk, gh, spec, rnd, runs, diffs, want


def test_pingpong_restore_matches_oracle_per_layer(tdo):
    torch, tdk, gh, spec, rnd, runs, diffs, want = _setup(tdo)
    L = spec.num_layers
    # oracle: Alg. 1 as stated
    opools = [wl.pool_host(rnd, layer) for layer in range(L)]
    tdo.restore_layers(runs[0].g, runs[0].hr, [o.mk for o in runs], [o.mv for o in runs],
                       [p[0] for p in opools], [p[1] for p in opools], diffs)
    # GPU: masters in pinned host memory, diffs and pools on the device
    hk = [torch.from_numpy(o.mk.view(np.int16)).pin_memory() for o in runs]
    hv = [torch.from_numpy(o.mv.view(np.int16)).pin_memory() for o in runs]
    mbytes = hk[0].numel() * 2
    stage = [torch.zeros(mbytes // 2, dtype=torch.int16, device="cuda") for _ in range(4)]
    pp = tdk.pingpong(stage[0], stage[1], stage[2], stage[3], mbytes)
    pools = [(gh.up(wl.pool_host(rnd, layer)[0]), gh.up(wl.pool_host(rnd, layer)[1])) for layer in range(L)]
    ddev = []
    for layer in range(L):
        d = diffs[layer]
        n = int(d.offset[-1])
        t = dict(count=torch.from_numpy(d.count).cuda(), offset=torch.from_numpy(d.offset).cuda(),
                 idx=torch.from_numpy(d.idx[:max(n, 1)].copy()).cuda(),
                 payload=gh.up(d.payload[:max(n, 1)].copy()), ovf=torch.zeros(1, dtype=torch.int32, device="cuda"))
        t["c"] = tdk.diff(t["count"], t["offset"], t["idx"], t["payload"], n, t["ovf"])
        ddev.append(t)
    r = tdk.round_from_workload(rnd)
    ios = [tdk.layer_io(None, None, pools[l][0], pools[l][1], rnd.pool_pages) for l in range(L)]
    comp, copy = torch.cuda.Stream(), torch.cuda.Stream()
    try:
        for rep in range(2):      # the second call reuses the staging buffers right behind the first
            tdk.tdk_restore_layers(r, 0, hk, hv, ios, [t["c"] for t in ddev], pp, comp.cuda_stream, copy.cuda_stream)
        comp.synchronize(); copy.synchronize()
        for l in range(L):
            assert np.array_equal(gh.down16(pools[l][0]), opools[l][0]), f"K layer {l}"
            assert np.array_equal(gh.down16(pools[l][1]), opools[l][1]), f"V layer {l}"
        mask = wl.shared_row_mask(rnd)
        for l in range(L):
            assert np.array_equal(opools[l][0][mask], want[l][0][mask])
        # a sub-range of layers, one stream for both roles
        for l in (1, 2, 3):
            pools[l][0].zero_(); pools[l][1].zero_()
        tdk.tdk_restore_layers(r, 1, hk[1:4], hv[1:4], ios[1:4], [t["c"] for t in ddev[1:4]], pp,
                               comp.cuda_stream, comp.cuda_stream)
        comp.synchronize()
        for l in (1, 2, 3):
            assert np.array_equal(gh.down16(pools[l][0])[mask], want[l][0][mask])
            assert np.array_equal(gh.down16(pools[l][1])[mask], want[l][1][mask])
        # argument errors are caught before anything is enqueued
        small = tdk.pingpong(stage[0], stage[1], stage[2], stage[3], mbytes - 16)
        with pytest.raises(tdk.TdkError):
            tdk.tdk_restore_layers(r, 0, hk, hv, ios, [t["c"] for t in ddev], small, comp.cuda_stream, copy.cuda_stream)
        same = tdk.pingpong(stage[0], stage[0], stage[2], stage[3], mbytes)
        with pytest.raises(tdk.TdkError):
            tdk.tdk_restore_layers(r, 0, hk, hv, ios, [t["c"] for t in ddev], same, comp.cuda_stream, copy.cuda_stream)
        with pytest.raises(tdk.TdkError):
            tdk.tdk_restore_layers(r, 3, hk, hv, ios, [t["c"] for t in ddev], pp, comp.cuda_stream, copy.cuda_stream)
    finally:
        torch.cuda.synchronize()
        r.destroy()


@pytest.mark.parametrize("style,T", [(0, 16), (1, 16), (0, 32)])
def test_restore_at_new_offsets_matches_oracle(tdo, style, T):
    """A mirror stored in one round is restored in the next, where every history has grown: diff pages
    are re-rotated from the position they were encoded at, the rest comes from the master."""
    import torch
    from paper_2604_03143_amd import tdk
    import gpu_helpers as gh
    spec = wl.RoundSpec("next", 56, 1, 8, 128, T, 1.0e6, 2, 4, 3, 70, 5, 300, 0.2)
    old = wl.make_round(spec)
    o = OracleRun(tdo, old, style=style)
    o.rerotate(); o.perturb()
    d = o.encode()
    grow = np.array([0, 16, 7, 250, 1, 31, 1000, 64], np.int64)
    new = wl.make_round(spec, hist=old.agent_pos0 + grow)
    opk, opv = wl.pool_host(new, 0)
    tdo.diff_decode(o.g, tdo.HostRound(new, diff_pos0=old.agent_pos0), o.mk, o.mv, opk, opv, d)
    n = int(d.offset[-1])
    g = gh.GpuRun(new, style=style, mk=o.mk, mv=o.mv)
    g.r.destroy()
    g.r = tdk.round_from_workload(new, style=style, diff_pos0=old.agent_pos0)
    try:
        cnt, off = torch.from_numpy(d.count).cuda(), torch.from_numpy(d.offset).cuda()
        idx, pay = torch.from_numpy(d.idx[:n].copy()).cuda(), gh.up(d.payload[:n].copy())
        dd = tdk.diff(cnt, off, idx, pay, n, torch.zeros(1, dtype=torch.int32, device="cuda"))
        tdk.tdk_diff_decode(g.r, 0, g.io, dd, g.stream)
        gk, gv = g.pool()
        assert np.array_equal(gk, opk) and np.array_equal(gv, opv)
    finally:
        g.close()


@pytest.mark.parametrize("style,T,block_tokens", [(0, 16, 40), (1, 16, 23), (0, 32, 50)])
def test_restore_at_new_offsets_with_reordered_blocks_matches_oracle(tdo, style, T, block_tokens):
    """The next round orders the shared blocks differently as well (Eq. 2): every block of a stored
    page is re-rotated by its own distance, pages hold rows of two blocks, blocks that did not move
    are copied bit for bit; one agent keeps the identity layout in both rounds."""
    import torch
    from paper_2604_03143_amd import tdk
    import gpu_helpers as gh
    spec = wl.RoundSpec("next_perm", 57, 1, 8, 128, T, 1.0e6, 2, 4, 4, block_tokens, 5, 300, 0.3)
    old = wl.permute_blocks(wl.make_round(spec), seed_tag=4)
    old.segments[5] = np.zeros((0, 3), np.int64)
    o = OracleRun(tdo, old, style=style)
    o.rerotate(); o.perturb()
    d = o.encode()
    grow = np.array([0, 16, 7, 250, 1, 31, 1000, 64], np.int64)
    new = wl.permute_blocks(wl.make_round(spec, hist=old.agent_pos0 + grow), seed_tag=9)
    new.segments[5] = np.zeros((0, 3), np.int64)
    new.segments[0] = old.segments[0].copy()              # agent 0: same order, same history: nothing moved
    seg_diff = [sg[:, 1] if len(sg) else np.zeros(0, np.int64) for sg in old.segments]
    opk, opv = wl.pool_host(new, 0)
    tdo.diff_decode(o.g, tdo.HostRound(new, diff_pos0=old.agent_pos0, segment_diff_pos=seg_diff), o.mk, o.mv, opk, opv, d)
    n = int(d.offset[-1])
    g = gh.GpuRun(new, style=style, mk=o.mk, mv=o.mv)
    g.r.destroy()
    g.r = tdk.round_from_workload(new, style=style, diff_pos0=old.agent_pos0, segment_diff_pos=seg_diff)
    try:
        cnt, off = torch.from_numpy(d.count).cuda(), torch.from_numpy(d.offset).cuda()
        idx, pay = torch.from_numpy(d.idx[:n].copy()).cuda(), gh.up(d.payload[:n].copy())
        dd = tdk.diff(cnt, off, idx, pay, n, torch.zeros(1, dtype=torch.int32, device="cuda"))
        tdk.tdk_diff_decode(g.r, 0, g.io, dd, g.stream)
        gk, gv = g.pool()
        assert np.array_equal(gk, opk) and np.array_equal(gv, opv)
    finally:
        g.close()
