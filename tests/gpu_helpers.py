"""GPU-side twin of helpers.OracleRun: the same seeded inputs, pushed through the C-ABI library."""
from __future__ import annotations

import numpy as np
import torch

from paper_2604_03143_amd import tdk, workload as wl


def up(a: np.ndarray) -> torch.Tensor:
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def down16(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint16)


class DevDiff:
    def __init__(self, n_agents: int, capacity: int, page_elems: int, guard_pages: int = 1):
        self.capacity = capacity
        self.count = torch.full((max(n_agents, 1),), -7, dtype=torch.int32, device="cuda")
        self.offset = torch.full((n_agents + 1,), -7, dtype=torch.int64, device="cuda")
        # guard entries after the capacity must never be written
        self.idx = torch.full((capacity + guard_pages,), -1, dtype=torch.int32, device="cuda")
        self.payload = torch.full((capacity + guard_pages, page_elems), 0x5A5A, dtype=torch.int16, device="cuda")
        self.overflow = torch.full((1,), -7, dtype=torch.int32, device="cuda")
        self.c = tdk.diff(self.count, self.offset, self.idx, self.payload, capacity, self.overflow)

    def host(self, n_agents):
        return (self.count.cpu().numpy()[:n_agents], self.offset.cpu().numpy(), self.idx.cpu().numpy(),
                down16(self.payload), int(self.overflow.item()))


class GpuRun:
    def __init__(self, rnd: wl.Round, layer: int = 0, style=tdk.ROPE_HALF, group: int = 0, flags=None,
                 mk=None, mv=None, pk=None, pv=None):
        self.rnd = rnd
        self.layer = layer
        if mk is None:
            mk, mv = wl.master_host(rnd, layer)
        if pk is None:
            pk, pv = wl.pool_host(rnd, layer)
        self.mk, self.mv, self.pk, self.pv = up(mk), up(mv), up(pk), up(pv)
        self.r = tdk.round_from_workload(rnd, style=style)
        if group or flags is not None:
            tdk.tdk_round_tune(self.r, group, tdk.TUNE_DEFAULT if flags is None else flags)
        self.io = tdk.layer_io(self.mk, self.mv, self.pk, self.pv, rnd.pool_pages)
        self.stream = torch.cuda.current_stream().cuda_stream

    def set_pool(self, pk: np.ndarray, pv: np.ndarray):
        self.pk.copy_(up(pk)); self.pv.copy_(up(pv))

    def pool(self):
        torch.cuda.synchronize()
        return down16(self.pk), down16(self.pv)

    def rerotate(self):
        tdk.tdk_rerotate_round(self.r, self.layer, self.io, self.stream)

    def new_diff(self, capacity=None) -> DevDiff:
        sp = self.rnd.spec
        if capacity is None:
            capacity = self.rnd.n_agents * sp.span_pages
        return DevDiff(self.rnd.n_agents, capacity, 2 * sp.page_tokens * sp.row_elems)

    def encode(self, eps=None, capacity=None, d: DevDiff = None) -> DevDiff:
        eps = self.rnd.spec.eps if eps is None else eps
        d = self.new_diff(capacity) if d is None else d
        tdk.tdk_diff_encode(self.r, self.layer, self.io, eps, d.c, self.stream)
        torch.cuda.synchronize()
        return d

    def decode(self, d: DevDiff):
        tdk.tdk_diff_decode(self.r, self.layer, self.io, d.c, self.stream)
        torch.cuda.synchronize()

    def close(self):
        self.r.destroy()


def assert_diff_equal(dev: DevDiff, od, n_agents: int):
    cnt, off, idx, pay, ovf = dev.host(n_agents)
    assert np.array_equal(cnt, od.count), "count"
    assert np.array_equal(off, od.offset), "offset"
    assert ovf == int(od.overflow[0]), "overflow"
    n = min(int(od.offset[-1]), dev.capacity)
    assert np.array_equal(idx[:n], od.idx[:n]), "idx"
    assert np.array_equal(pay[:n], od.payload[:n]), "payload"
    # nothing at or past the listed pages / the capacity was written
    assert np.all(idx[n:] == -1), "idx written past the list"
    assert np.all(pay[n:] == 0x5A5A), "payload written past the list"
