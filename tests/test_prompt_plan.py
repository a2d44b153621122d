"""The library's host-side prompt plan (Sec. 4.1, Sec. 5) against the plain reference: same sessions,
same grouping, same segments, on worked examples and on seeded random rounds.  Host code only: runs
without a GPU."""
import numpy as np
import pytest

from oracle import prompt_index as pi
from paper_2604_03143_amd import tdk

SEP = 151_000


def _prompt(*blocks):
    out = []
    for k, b in enumerate(blocks):
        if k:
            out.append(SEP)
        out.extend(int(x) for x in b)
    return out


def _same(prompts):
    sessions, session_of, segs = pi.plan_prompts(prompts, SEP)
    spans, got_of, got_segs = tdk.tdk_prompt_plan(prompts, SEP)
    assert spans == [s["span"] for s in sessions]
    assert got_of == session_of
    assert got_segs == [list(x) for x in segs]
    return sessions, session_of, segs


def test_worked_examples():
    x, y, w = [1, 2, 3], [4, 5], [6]
    _same([_prompt([50], x, y), _prompt([51], x, y), _prompt([52], w, x), _prompt([53], w), _prompt([54], w),
           [SEP, SEP] + _prompt([], x, x, y) + [SEP]])
    _same([])
    _same([[SEP], [], [7, 8, 9]])
    _same([_prompt([1], [2, 3]), _prompt([9, 9], [2, 3])])


def test_seeded_random_rounds_with_reordered_blocks_and_strangers():
    g = np.random.default_rng(11)
    for _ in range(40):
        pools = [[list(g.integers(0, 50, size=int(g.integers(1, 12)))) for _ in range(int(g.integers(1, 7)))]
                 for _ in range(int(g.integers(1, 4)))]                       # several rounds' shared blocks
        prompts = []
        for _ in range(int(g.integers(1, 9))):
            pool = pools[int(g.integers(0, len(pools)))]
            order = g.permutation(len(pool))
            take = order[: int(g.integers(1, len(pool) + 1))] if g.integers(0, 4) == 0 else order
            hist = list(g.integers(100, 200, size=int(g.integers(0, 40))))
            extra = [list(g.integers(300, 400, size=int(g.integers(0, 5))))]
            prompts.append(_prompt(hist, *[pool[k] for k in take], *extra))
        _same(prompts)


def test_the_plan_feeds_round_create_without_a_gpu_error_path():
    """Segments from the plan are accepted by the round planner's host-side validation (a page may meet at
    most two segments, so blocks here are at least a page long)."""
    g = np.random.default_rng(3)
    shared = [list(g.integers(0, 1000, size=n)) for n in (40, 23, 57)]
    prompts = [_prompt(list(g.integers(2000, 3000, size=h)), *[shared[k] for k in order])
               for h, order in ((5, (0, 1, 2)), (31, (2, 0, 1)), (17, (1, 2, 0)))]
    sessions, session_of, segs = _same(prompts)
    assert session_of == [0, 0, 0] and sessions[0]["span"] == 120
    for p, sg in zip(prompts, segs):
        master = [t for b in sessions[0]["blocks"] for t in b]
        assert [p[dst + k] for (_, dst, n) in sg for k in range(n)] == master


def test_bad_arguments():
    with pytest.raises(tdk.TdkError):
        import ctypes as C
        out = C.c_void_p()
        tdk._check(tdk.load().tdk_prompt_plan_create(None, 3, SEP, C.byref(out)), "tdk_prompt_plan_create")
