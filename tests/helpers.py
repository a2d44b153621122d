"""Shared test helpers: small rounds and an oracle runner (host only)."""
from __future__ import annotations

import dataclasses

import numpy as np

from paper_2604_03143_amd import workload as wl


def small_spec(name="small", H=2, D=8, T=4, sessions=1, agents=3, blocks=3, block_tokens=7,
               hist=(5, 40), frac=0.2, theta=1.0e4, stream=99, layers=1) -> wl.RoundSpec:
    return wl.RoundSpec(name, stream, layers, H, D, T, theta, sessions, agents, blocks, block_tokens,
                        hist[0], hist[1], frac)


def with_(spec: wl.RoundSpec, **kw) -> wl.RoundSpec:
    return dataclasses.replace(spec, **kw)


class OracleRun:
    """Runs the whole path on the oracle for one layer of a round."""

    def __init__(self, tdo, rnd: wl.Round, layer: int = 0, math=0, style=0):
        self.tdo = tdo
        self.rnd = rnd
        self.g = tdo.geom_of(rnd.spec, math=math, style=style)
        self.hr = tdo.HostRound(rnd)
        self.mk, self.mv = wl.master_host(rnd, layer)
        self.pk, self.pv = wl.pool_host(rnd, layer)
        self.layer = layer

    def rerotate(self):
        self.tdo.rerotate_round(self.g, self.hr, self.mk, self.mv, self.pk, self.pv)

    def perturb(self):
        wl.perturb_host(self.rnd, self.layer, self.pk, self.pv)

    def encode(self, eps=None, capacity=None):
        eps = self.rnd.spec.eps if eps is None else eps
        if capacity is None:
            capacity = self.rnd.n_agents * self.rnd.spec.span_pages
        return self.tdo.diff_encode(self.g, self.hr, self.mk, self.mv, self.pk, self.pv, eps, capacity)

    def decode(self, d, pk=None, pv=None):
        pk = self.pk if pk is None else pk
        pv = self.pv if pv is None else pv
        self.tdo.diff_decode(self.g, self.hr, self.mk, self.mv, pk, pv, d)


def lists_of(d, n_agents):
    return [d.idx[int(d.offset[i]):int(d.offset[i]) + int(d.count[i])].copy() for i in range(n_agents)]
