"""Plain reference of the round-aware prompt index (TEST INFRASTRUCTURE ONLY, like the rest of oracle/).

Sec. 4.1 (round-aware prompt interface) and Sec. 5 (segment-based hash table): prompts are split at a
reserved separator token; every block is identified by its content, not by its position, so the same
shared update is recognised in prompts whose private histories differ in length.  Here the content
itself (a tuple of token ids) is the dictionary key: no hashing, nothing to collide.

plan_prompts(prompts, separator) returns
  sessions:  list of dicts {span: tokens of the shared span, blocks: list of content tuples in master order}
  session_of: per prompt the session index, or -1 (no group of at least two prompts shares its blocks:
              the single-request path)
  segments:  per prompt a list of (src_tok, dst_pos, len): master tokens src_tok.. sit at positions dst_pos..
Rules: empty blocks are ignored; a content is shared if it occurs in at least two prompts; prompts are
grouped by the SET of shared contents they hold (at least two prompts per group, groups numbered by their
first prompt); the master lists the shared blocks in the order of the group's first prompt; if a content
occurs twice in one prompt its first occurrence counts.
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple


def split_blocks(tokens: Sequence[int], separator: int) -> List[Tuple[int, Tuple[int, ...]]]:
    """(position of the block's first token, content) for every non-empty run between separators."""
    out, start, cur = [], 0, []
    for pos, t in enumerate(tokens):
        if int(t) == separator:
            if cur:
                out.append((start, tuple(cur)))
            cur, start = [], pos + 1
        else:
            cur.append(int(t))
    if cur:
        out.append((start, tuple(cur)))
    return out


def plan_prompts(prompts: Sequence[Sequence[int]], separator: int):
    blocks = [split_blocks(p, separator) for p in prompts]
    holders: Dict[Tuple[int, ...], set] = {}
    for i, bl in enumerate(blocks):
        for _, content in bl:
            holders.setdefault(content, set()).add(i)
    shared = {c for c, who in holders.items() if len(who) >= 2}
    key_of = [frozenset(c for _, c in bl if c in shared) for bl in blocks]
    members: Dict[frozenset, List[int]] = {}
    for i, k in enumerate(key_of):
        if k:
            members.setdefault(k, []).append(i)
    groups = sorted((m for m in members.values() if len(m) >= 2), key=lambda m: m[0])
    sessions, session_of, segments = [], [-1] * len(prompts), [[] for _ in prompts]
    for s, m in enumerate(groups):
        first = m[0]
        order, seen = [], set()
        for _, c in blocks[first]:
            if c in shared and c not in seen:
                order.append(c)
                seen.add(c)
        src, at = {}, 0
        for c in order:
            src[c] = at
            at += len(c)
        sessions.append(dict(span=at, blocks=order))
        for i in m:
            session_of[i] = s
            placed = {}
            for pos, c in blocks[i]:
                if c in src and c not in placed:
                    placed[c] = pos
            segments[i] = [(src[c], placed[c], len(c)) for c in order]
    return sessions, session_of, segments
