"""Seeded synthetic All-Gather rounds (inputs only).

This module builds the *inputs* of one collective KV-reuse round: how many
sessions and agents there are, how long each agent's private history is, where
each agent's logical pages live in the paged pool, which master pages the model
"refreshed" (perturbed) for each agent, and the random master K/V values.  It
holds none of the method's arithmetic: no rotation, no compare, no compaction.
Both the HIP path and the CPU oracle are fed from here and from nowhere else.

Shape of a round (Section 2.1, Eq. 2): every agent's prompt is its private
history followed by the same shared output blocks, so the shared span of S
tokens starts at a different absolute position h_i for every agent.  The
configurations below stand in for the replayed agent traces of Section 6.1 by
shape and value distribution only.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

SEED_BASE = 20260403


@dataclass(frozen=True)
class RoundSpec:
    name: str
    stream: int                 # RNG stream id (one per configuration)
    num_layers: int
    num_kv_heads: int
    head_dim: int
    page_tokens: int
    rope_theta: float
    n_sessions: int
    agents_per_session: int
    blocks: int                 # shared output blocks per session
    block_tokens: int           # tokens per shared output block
    hist_lo: int                # private history length, uniform in [lo, hi]
    hist_hi: int
    perturbed_frac: float       # fraction of master pages refreshed per agent
    eps: float = 1e-2
    noise_sigma: float = 0.05

    @property
    def span_tokens(self) -> int:
        return self.blocks * self.block_tokens

    @property
    def span_pages(self) -> int:
        return -(-self.span_tokens // self.page_tokens)

    @property
    def n_agents(self) -> int:
        return self.n_sessions * self.agents_per_session

    @property
    def row_elems(self) -> int:
        return self.num_kv_heads * self.head_dim

    @property
    def perturbed_pages_per_agent(self) -> int:
        if self.perturbed_frac <= 0.0:
            return 0
        return max(1, int(round(self.perturbed_frac * self.span_pages)))


CONFIGS: Dict[str, RoundSpec] = {
    "tiny": RoundSpec("tiny", 1, 1, 8, 128, 16, 1.0e6, 1, 4, 4, 64, 32, 256, 0.06),
    "session": RoundSpec("session", 2, 48, 8, 128, 16, 1.0e6, 1, 25, 25, 200, 1000, 4000, 0.06),
    "batched250": RoundSpec("batched250", 3, 48, 8, 128, 16, 1.0e6, 10, 25, 25, 200, 1000, 4000, 0.06),
    "long": RoundSpec("long", 4, 48, 8, 128, 16, 1.0e6, 1, 100, 100, 256, 4000, 8000, 0.03),
    "llama70b": RoundSpec("llama70b", 5, 80, 8, 128, 16, 5.0e5, 1, 64, 64, 200, 2000, 6000, 0.10),
}


@dataclass
class Round:
    """Host-side structure of one round (no tensors)."""
    spec: RoundSpec
    span_tokens: np.ndarray        # int32 [n_sessions]
    master_pos0: np.ndarray        # int64 [n_sessions]
    master_row0: np.ndarray        # int64 [n_sessions+1], first master row of each session
    agent_session: np.ndarray      # int32 [n_agents]
    agent_pos0: np.ndarray         # int64 [n_agents], h_i
    block_tables: List[np.ndarray]  # per agent int32 [ceil((h_i+S)/T)], logical -> physical page
    pool_pages: int
    dummy_page: int                # every history-only logical page maps here
    canary_pages: np.ndarray       # int32 [2*n_agents], mapped by nobody
    perturbed: List[np.ndarray]    # per agent sorted int32 master-page numbers
    extra: dict = field(default_factory=dict)
    # optional layout of the shared blocks per agent (Eq. 2, Pi_i): int64 [n_seg, 3] rows of
    # (first master token, absolute position it lands at, length); None = identity for every agent
    segments: Optional[List[np.ndarray]] = None

    @property
    def n_agents(self) -> int:
        return int(self.agent_session.shape[0])

    @property
    def n_sessions(self) -> int:
        return int(self.span_tokens.shape[0])

    @property
    def total_master_rows(self) -> int:
        return int(self.master_row0[-1])

    def agent_tokens(self) -> int:
        return int(sum(int(self.span_tokens[s]) for s in self.agent_session))

    def dst_rows(self, agent: int, tokens: Optional[np.ndarray] = None) -> np.ndarray:
        """Physical pool row of master token m for this agent (slot map)."""
        T = self.spec.page_tokens
        S = int(self.span_tokens[self.agent_session[agent]])
        m = np.arange(S, dtype=np.int64) if tokens is None else np.asarray(tokens, dtype=np.int64)
        a = self.token_pos(agent, m)
        bt = self.block_tables[agent]
        return bt[a // T].astype(np.int64) * T + (a % T)


def _token_pos(self, agent: int, m: np.ndarray) -> np.ndarray:
    """Absolute position of master tokens m in this agent's prompt."""
    m = np.asarray(m, dtype=np.int64)
    if self.segments is None or len(self.segments[agent]) == 0:
        return int(self.agent_pos0[agent]) + m
    seg = np.asarray(self.segments[agent], dtype=np.int64)
    q = np.searchsorted(seg[:, 0], m, side="right") - 1
    return seg[q, 1] + (m - seg[q, 0])


Round.token_pos = _token_pos


def permute_blocks(rnd: Round, seed_tag: int = 4) -> Round:
    """Gives every agent its own order of the shared blocks (the scheduler-defined layout of Eq. 2):
    block b of the master lands at h_i + rank_i(b) * block_tokens.  Block tables are unchanged (the
    permuted span occupies the same positions)."""
    spec = rnd.spec
    g = _rng(spec, seed_tag)
    segs = []
    for i in range(rnd.n_agents):
        order = g.permutation(spec.blocks)            # order[k] = block placed k-th
        rank = np.empty(spec.blocks, dtype=np.int64)
        rank[order] = np.arange(spec.blocks)
        h = int(rnd.agent_pos0[i])
        segs.append(np.array([[b * spec.block_tokens, h + int(rank[b]) * spec.block_tokens, spec.block_tokens]
                              for b in range(spec.blocks)], dtype=np.int64))
    rnd.segments = segs
    return rnd


def _rng(spec: RoundSpec, tag: int, extra: int = 0) -> np.random.Generator:
    return np.random.default_rng([SEED_BASE, spec.stream, tag, extra])


def make_round(spec: RoundSpec, hist: Optional[np.ndarray] = None,
               perturbed_per_agent: Optional[int] = None,
               clustered: bool = False, alloc: str = "fragmented",
               spans: Optional[List[int]] = None, agents: Optional[List[int]] = None) -> Round:
    """Draw the structure of a round: histories, block tables, perturbed page sets.

    alloc = "fragmented": physical pages are a seeded random permutation of the pool (an allocator
    after long use; the default and the graded recipe); "contiguous": every agent's pages are
    consecutive (a fresh allocator).

    spans / agents: per-session span lengths and agent counts for ragged rounds (sessions of different
    sizes batched into one round); by default every session has spec.span_tokens tokens and
    spec.agents_per_session agents.  The perturbed fraction then applies to each session's own pages."""
    T = spec.page_tokens
    n_sess = spec.n_sessions if spans is None and agents is None else len(spans if spans is not None else agents)
    span_list = [spec.span_tokens] * n_sess if spans is None else [int(x) for x in spans]
    agent_list = [spec.agents_per_session] * n_sess if agents is None else [int(x) for x in agents]
    assert len(span_list) == n_sess and len(agent_list) == n_sess
    A = int(sum(agent_list))
    rs = _rng(spec, 1)
    span_tokens = np.array(span_list, dtype=np.int32)
    master_pos0 = np.zeros(n_sess, dtype=np.int64)
    master_row0 = np.concatenate([[0], np.cumsum(span_tokens, dtype=np.int64)]).astype(np.int64)
    agent_session = np.repeat(np.arange(n_sess, dtype=np.int32), agent_list)
    if hist is None:
        hist = rs.integers(spec.hist_lo, spec.hist_hi + 1, size=A, dtype=np.int64)
    agent_pos0 = np.asarray(hist, dtype=np.int64).copy()
    assert agent_pos0.shape == (A,)
    S_of = span_tokens[agent_session].astype(np.int64)

    first_lp = agent_pos0 // T
    last_lp = np.where(S_of > 0, (agent_pos0 + S_of - 1) // T, first_lp - 1)
    n_touch = (last_lp - first_lp + 1).astype(np.int64)
    pool_pages = int(n_touch.sum()) + 2 * A + 1
    if alloc == "fragmented":
        perm = _rng(spec, 2).permutation(pool_pages).astype(np.int32)
    elif alloc == "contiguous":
        perm = np.arange(pool_pages, dtype=np.int32)
    else:
        raise ValueError(f"unknown alloc {alloc!r}")
    dummy = int(perm[0])
    canaries = perm[1:1 + 2 * A].copy()
    cursor = 1 + 2 * A
    tables: List[np.ndarray] = []
    for i in range(A):
        n = int(n_touch[i])
        bt = np.full(int(first_lp[i]) + n, dummy, dtype=np.int32)
        bt[int(first_lp[i]):] = perm[cursor:cursor + n]
        cursor += n
        tables.append(bt)
    assert cursor == pool_pages

    rp = _rng(spec, 3)
    perturbed: List[np.ndarray] = []
    for i in range(A):
        S = int(S_of[i])
        P = -(-S // T)
        if perturbed_per_agent is not None:
            k = perturbed_per_agent
        elif spec.perturbed_frac <= 0.0 or P == 0:
            k = 0
        else:
            k = max(1, int(round(spec.perturbed_frac * P)))
        k = min(k, P)
        if k == 0:
            perturbed.append(np.zeros(0, dtype=np.int32))
        elif not clustered:
            perturbed.append(np.sort(rp.choice(P, size=k, replace=False)).astype(np.int32))
        else:
            # runs of 1-4 consecutive pages that start on a shared-block boundary
            chosen: set = set()
            guard = 0
            n_blocks = max(1, min(spec.blocks, -(-S // spec.block_tokens)))
            while len(chosen) < k and guard < 100000:
                guard += 1
                b = int(rp.integers(0, n_blocks))
                start = (b * spec.block_tokens) // T
                run = int(rp.integers(1, 5))
                for q in range(start, min(P, start + run)):
                    if len(chosen) < k:
                        chosen.add(q)
            perturbed.append(np.array(sorted(chosen), dtype=np.int32))
    return Round(spec, span_tokens, master_pos0, master_row0, agent_session, agent_pos0,
                 tables, pool_pages, dummy, canaries, perturbed)


# ---------------------------------------------------------------------------
# bf16 storage helpers (format conversion only)
# ---------------------------------------------------------------------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns, round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    nan = (u & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
    r = np.where(nan, (u >> np.uint32(16)) | np.uint32(0x40), r)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def master_host(rnd: Round, layer: int):
    """Master K, V ~ N(0,1) as bf16 bit patterns, shape [total_master_rows, H*D]."""
    spec = rnd.spec
    g = _rng(spec, 10, layer)
    shape = (rnd.total_master_rows, spec.row_elems)
    k = f32_to_bf16_bits(g.standard_normal(shape, dtype=np.float32))
    v = f32_to_bf16_bits(g.standard_normal(shape, dtype=np.float32))
    return k, v


def pool_host(rnd: Round, layer: int):
    """A pool pre-filled with a seeded non-trivial pattern (so that untouched rows are detectable)."""
    spec = rnd.spec
    g = _rng(spec, 11, layer)
    shape = (rnd.pool_pages * spec.page_tokens, spec.row_elems)
    k = g.integers(0, 1 << 16, size=shape, dtype=np.uint16)
    v = g.integers(0, 1 << 16, size=shape, dtype=np.uint16)
    # keep the fill finite: clear the top exponent bit so no NaN/Inf patterns appear
    k &= np.uint16(0xBFFF)
    v &= np.uint16(0xBFFF)
    return k, v


def perturb_host(rnd: Round, layer: int, pool_k: np.ndarray, pool_v: np.ndarray,
                 same_pages_all_layers: bool = True) -> None:
    """Stand-in for the model's per-position refresh: on every perturbed master page of
    every agent, each valid K and V element x becomes bf16(fp32(x) + n), n ~ N(0, sigma)."""
    spec = rnd.spec
    T = spec.page_tokens
    g = _rng(spec, 12, layer)
    for i in range(rnd.n_agents):
        S = int(rnd.span_tokens[rnd.agent_session[i]])
        for p in rnd.perturbed[i]:
            toks = np.arange(int(p) * T, min(S, (int(p) + 1) * T), dtype=np.int64)
            rows = rnd.dst_rows(i, toks)
            for plane in (pool_k, pool_v):
                x = bf16_bits_to_f32(plane[rows])
                n = g.standard_normal(x.shape, dtype=np.float32) * np.float32(spec.noise_sigma)
                plane[rows] = f32_to_bf16_bits(x + n)


def shared_row_mask(rnd: Round) -> np.ndarray:
    """Boolean [pool_rows]: True where some agent's shared span lands."""
    mask = np.zeros(rnd.pool_pages * rnd.spec.page_tokens, dtype=bool)
    for i in range(rnd.n_agents):
        mask[rnd.dst_rows(i)] = True
    return mask


# ---------------------------------------------------------------------------
# device-side generators for rounds too large to draw on the host (torch is used for random
# numbers and indexing only; still no method arithmetic)
# ---------------------------------------------------------------------------

def master_device(rnd: Round, layer: int, device="cuda"):
    """Master K, V ~ N(0,1) in bf16 on the device, as int16 bit-pattern tensors [rows, H*D]."""
    import torch
    spec = rnd.spec
    g = torch.Generator(device=device)
    g.manual_seed(SEED_BASE * 1000 + spec.stream * 100003 + layer)
    shape = (rnd.total_master_rows, spec.row_elems)
    k = torch.randn(shape, generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)
    v = torch.randn(shape, generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)
    return k.view(torch.int16), v.view(torch.int16)


def perturbed_rows(rnd: Round) -> np.ndarray:
    """Physical pool rows of every valid token of every perturbed page (int64, all agents)."""
    T = rnd.spec.page_tokens
    out = []
    for i in range(rnd.n_agents):
        S = int(rnd.span_tokens[rnd.agent_session[i]])
        if len(rnd.perturbed[i]) == 0:
            continue
        toks = (rnd.perturbed[i].astype(np.int64)[:, None] * T + np.arange(T, dtype=np.int64)[None, :]).ravel()
        toks = toks[toks < S]
        out.append(rnd.dst_rows(i, toks))
    return np.concatenate(out) if out else np.zeros(0, np.int64)


def perturb_device(rnd: Round, layer: int, pool_k, pool_v, rows=None) -> None:
    """Device version of perturb_host: x <- bf16(fp32(x) + N(0, sigma)) on the perturbed pages."""
    import torch
    spec = rnd.spec
    if rows is None:
        rows = torch.from_numpy(perturbed_rows(rnd)).to(pool_k.device)
    if rows.numel() == 0:
        return
    g = torch.Generator(device=pool_k.device)
    g.manual_seed(SEED_BASE * 1000 + spec.stream * 100003 + 50000 + layer)
    for plane in (pool_k, pool_v):
        chunk = 16384
        for c0 in range(0, rows.numel(), chunk):
            r = rows[c0:c0 + chunk]
            x = plane[r].view(torch.bfloat16).float()
            n = torch.randn(x.shape, generator=g, device=x.device, dtype=torch.float32) * spec.noise_sigma
            plane[r] = (x + n).to(torch.bfloat16).view(torch.int16)


def subround(rnd: Round, agents) -> "tuple[Round, np.ndarray]":
    """The sessions and block tables of a few agents, remapped onto a compact pool.

    Returns (sub, page_map) where page_map[q] is the page of `rnd`'s pool that page q of the compact
    pool stands for (page 0 of the compact pool is the dummy page).  Structure only."""
    agents = [int(a) for a in agents]
    T = rnd.spec.page_tokens
    sess_ids = sorted({int(rnd.agent_session[a]) for a in agents})
    smap = {s: k for k, s in enumerate(sess_ids)}
    span = rnd.span_tokens[sess_ids].astype(np.int32)
    page_map = [rnd.dummy_page]
    tables = []
    for a in agents:
        bt = rnd.block_tables[a]
        first = int(rnd.agent_pos0[a]) // T
        nb = np.zeros(len(bt), dtype=np.int32)
        for lp in range(first, len(bt)):
            nb[lp] = len(page_map)
            page_map.append(int(bt[lp]))
        tables.append(nb)
    sub = Round(rnd.spec, span, rnd.master_pos0[sess_ids].astype(np.int64),
                np.concatenate([[0], np.cumsum(span, dtype=np.int64)]).astype(np.int64),
                np.array([smap[int(rnd.agent_session[a])] for a in agents], dtype=np.int32),
                rnd.agent_pos0[agents].astype(np.int64), tables, len(page_map), 0,
                np.zeros(0, np.int32), [rnd.perturbed[a] for a in agents],
                extra={"sessions": sess_ids, "agents": agents},
                segments=None if rnd.segments is None else [rnd.segments[a] for a in agents])
    return sub, np.array(page_map, dtype=np.int64)
