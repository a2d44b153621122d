"""Pins of the prompt-index reference (Sec. 4.1): worked examples written out by hand."""
import numpy as np

from oracle import prompt_index as pi

SEP = 9000


def _prompt(*blocks):
    out = []
    for k, b in enumerate(blocks):
        if k:
            out.append(SEP)
        out.extend(b)
    return out


def test_three_agents_with_histories_of_different_length():
    """The layout of the paper's prompt-interface figure: a private history, then the same shared updates
    and the round task, separators in between."""
    u1, u2, u3, task = [11, 12, 13], [21, 22], [31, 32, 33, 34], [41]
    a = _prompt([1, 2], u1, u2, u3, task)                   # history of 2 tokens
    b = _prompt([5, 6, 7, 8, 9], u1, u2, u3, task)          # history of 5
    c = _prompt([3], u1, u2, u3, task)                      # history of 1
    sessions, session_of, segs = pi.plan_prompts([a, b, c], SEP)
    assert session_of == [0, 0, 0] and len(sessions) == 1
    assert sessions[0]["span"] == 3 + 2 + 4 + 1
    assert sessions[0]["blocks"] == [tuple(u1), tuple(u2), tuple(u3), tuple(task)]
    # prompt a: history 0..1, sep at 2, u1 at 3..5, sep 6, u2 at 7..8, sep 9, u3 at 10..13, sep 14, task at 15
    assert segs[0] == [(0, 3, 3), (3, 7, 2), (5, 10, 4), (9, 15, 1)]
    assert segs[1] == [(0, 6, 3), (3, 10, 2), (5, 13, 4), (9, 18, 1)]
    assert segs[2] == [(0, 2, 3), (3, 6, 2), (5, 9, 4), (9, 14, 1)]


def test_block_order_may_differ_and_private_blocks_are_ignored():
    x, y, z = [1, 1, 1], [2, 2], [3, 3, 3, 3]
    a = _prompt([70], x, y, z)
    b = _prompt([71, 72], z, [99, 98], x, y)                # another order, one private block in between
    sessions, session_of, segs = pi.plan_prompts([a, b], SEP)
    assert session_of == [0, 0] and sessions[0]["span"] == 9
    assert segs[0] == [(0, 2, 3), (3, 6, 2), (5, 9, 4)]
    # b: 71 72 | z at 3..6 | 99 98 at 8..9 | x at 11..13 | y at 15..16 ; master order is a's: x, y, z
    assert segs[1] == [(0, 11, 3), (3, 15, 2), (5, 3, 4)]


def test_groups_singletons_empty_blocks_and_repeats():
    x, y, w = [1, 2, 3], [4, 5], [6]
    p0 = _prompt([50], x, y)
    p1 = _prompt([51], x, y)
    p2 = _prompt([52], w, x)            # shares x with p0/p1 and w with p3, but nobody has its set {x, w}
    p3 = _prompt([53], w)
    p4 = _prompt([54], w)
    p5 = [SEP, SEP] + _prompt([], x, x, y) + [SEP]          # empty blocks and a repeated block
    sessions, session_of, segs = pi.plan_prompts([p0, p1, p2, p3, p4, p5], SEP)
    assert session_of == [0, 0, -1, 1, 1, 0]
    assert [s["span"] for s in sessions] == [5, 1]
    assert segs[2] == [] and segs[3] == [(0, 2, 1)]
    # p5 = SEP SEP SEP x(3..5) SEP x(7..9) SEP y(11..12) SEP: the first x counts
    assert segs[5] == [(0, 3, 3), (3, 11, 2)]
    assert pi.plan_prompts([], SEP) == ([], [], []) and pi.plan_prompts([[SEP]], SEP) == ([], [-1], [[]])


def test_segments_reassemble_the_master_everywhere():
    """Property on seeded random rounds: reading each prompt at the positions its segments name gives the
    master's token sequence, and positions never overlap."""
    g = np.random.default_rng(5)
    for _ in range(20):
        n_blocks = int(g.integers(1, 6))
        shared = [list(g.integers(0, 1000, size=int(g.integers(1, 9)))) for _ in range(n_blocks)]
        prompts = []
        for _ in range(int(g.integers(2, 6))):
            order = g.permutation(n_blocks)
            hist = list(g.integers(1000, 2000, size=int(g.integers(1, 30))))
            prompts.append(_prompt(hist, *[shared[k] for k in order]))
        sessions, session_of, segs = pi.plan_prompts(prompts, SEP)
        assert set(session_of) == {0}
        master = [t for b in sessions[0]["blocks"] for t in b]
        assert sorted(master) == sorted(t for b in shared for t in b)
        for p, sg in zip(prompts, segs):
            got = [p[dst + k] for (_, dst, n) in sg for k in range(n)]
            assert got == master
            pos = [dst + k for (_, dst, n) in sg for k in range(n)]
            assert len(set(pos)) == len(pos)
