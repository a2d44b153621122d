"""ctypes loader for the plain-C oracle (libtdo.so).  TEST INFRASTRUCTURE ONLY.

Argument marshalling only; every result is computed by oracle/tdo.c.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libtdo.so")
_SRC = os.path.join(_HERE, "tdo.c")
_HDR = os.path.join(_HERE, "tdo.h")

ROPE_HALF, ROPE_INTERLEAVED = 0, 1
MATH_F32, MATH_F64 = 0, 1


def build(force: bool = False) -> str:
    """Compile oracle/tdo.c with gcc.  No implicit FMA contraction: the fp32 path pins its op order."""
    stale = (not os.path.exists(_SO)) or any(
        os.path.getmtime(p) > os.path.getmtime(_SO) for p in (_SRC, _HDR))
    if force or stale:
        cmd = ["gcc", "-std=c11", "-O2", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True, cwd=_HERE)
    return _SO


class Geom(C.Structure):
    _fields_ = [("num_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("page_tokens", C.c_int32),
                ("rope_style", C.c_int32), ("rope_theta", C.c_double), ("math", C.c_int32)]


class RoundDesc(C.Structure):
    _fields_ = [("n_sessions", C.c_int32), ("span_tokens", C.c_void_p), ("master_pos0", C.c_void_p),
                ("n_agents", C.c_int32), ("agent_session", C.c_void_p), ("agent_pos0", C.c_void_p),
                ("bt_flat", C.c_void_p), ("bt_offset", C.c_void_p), ("agent_diff_pos0", C.c_void_p),
                ("seg_offset", C.c_void_p), ("seg_src", C.c_void_p), ("seg_len", C.c_void_p),
                ("seg_dst", C.c_void_p), ("seg_diff_dst", C.c_void_p)]


_lib: Optional[C.CDLL] = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        # TDO_LIBRARY: another build of the same source (the sanitizer test's instrumented one)
        L = C.CDLL(os.environ.get("TDO_LIBRARY") or build())
        for name in ("tdo_dense_bytes", "tdo_diff_bytes", "tdo_mirror_ratio", "tdo_family_cost"):
            getattr(L, name).restype = C.c_double
        L.tdo_dense_bytes.argtypes = [C.POINTER(Geom), C.c_int64]
        L.tdo_diff_bytes.argtypes = [C.POINTER(Geom), C.c_int64]
        L.tdo_mirror_ratio.argtypes = [C.POINTER(Geom), C.c_int64, C.c_int64]
        L.tdo_family_cost.argtypes = [C.c_int64, C.c_double]
        L.tdo_rope_table_f64.argtypes = [C.c_double, C.c_int32, C.c_int64, C.c_void_p, C.c_void_p]
        L.tdo_rope_table_f32.argtypes = [C.c_double, C.c_int32, C.c_int64, C.c_void_p, C.c_void_p]
        L.tdo_rotate_rows_f32.argtypes = [C.POINTER(Geom), C.c_int64, C.c_int64, C.c_void_p, C.c_void_p]
        L.tdo_rotate_rows_f32_bf16.argtypes = [C.POINTER(Geom), C.c_int64, C.c_int64, C.c_void_p, C.c_void_p]
        L.tdo_rotate_rows_bf16.argtypes = [C.POINTER(Geom), C.c_int64, C.c_int64, C.c_void_p, C.c_void_p]
        L.tdo_rerotate_round.argtypes = [C.POINTER(Geom), C.POINTER(RoundDesc)] + [C.c_void_p] * 4 + [C.c_int64]
        L.tdo_diff_encode.argtypes = ([C.POINTER(Geom), C.POINTER(RoundDesc)] + [C.c_void_p] * 4 +
                                      [C.c_int64, C.c_float] + [C.c_void_p] * 4 + [C.c_int64, C.c_void_p])
        L.tdo_diff_decode.argtypes = ([C.POINTER(Geom), C.POINTER(RoundDesc)] + [C.c_void_p] * 4 +
                                      [C.c_int64] + [C.c_void_p] * 4)
        L.tdo_diff_encode_plane.argtypes = ([C.POINTER(Geom), C.POINTER(RoundDesc)] + [C.c_void_p] * 4 +
                                            [C.c_int64, C.c_float, C.c_int32] + [C.c_void_p] * 4 + [C.c_int64, C.c_void_p])
        L.tdo_diff_decode_plane.argtypes = ([C.POINTER(Geom), C.POINTER(RoundDesc)] + [C.c_void_p] * 4 +
                                            [C.c_int64, C.c_int32] + [C.c_void_p] * 4)
        L.tdo_key_deviation.argtypes = [C.POINTER(Geom), C.POINTER(RoundDesc), C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        L.tdo_select_important.argtypes = [C.c_void_p, C.c_int64, C.c_float, C.c_float, C.c_void_p, C.c_void_p]
        L.tdo_choose_master.argtypes = [C.POINTER(RoundDesc), C.c_void_p, C.c_void_p]
        L.tdo_restore_layers.argtypes = ([C.POINTER(Geom), C.POINTER(RoundDesc), C.c_int32] +
                                         [C.POINTER(C.c_void_p)] * 4 + [C.c_int64] + [C.POINTER(C.c_void_p)] * 4)
        L.tdo_attend_shared.argtypes = ([C.POINTER(Geom), C.POINTER(RoundDesc)] + [C.c_void_p] * 7 +
                                        [C.c_int32, C.c_int32, C.c_double, C.c_void_p, C.c_void_p])
        _lib = L
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data


def _chk(rc: int, what: str) -> None:
    if rc != 0:
        raise ValueError(f"{what} failed with oracle status {rc}")


def geom(H=8, D=128, T=16, theta=1.0e6, style=ROPE_HALF, math=MATH_F32) -> Geom:
    return Geom(H, D, T, style, float(theta), math)


def geom_of(spec, math=MATH_F32, style=ROPE_HALF) -> Geom:
    return geom(spec.num_kv_heads, spec.head_dim, spec.page_tokens, spec.rope_theta, style, math)


class HostRound:
    """Flattened, contiguous host arrays of a workload Round, kept alive for the C calls."""

    def __init__(self, rnd, diff_pos0=None, segment_diff_pos=None):
        self.span_tokens = np.ascontiguousarray(rnd.span_tokens, dtype=np.int32)
        self.master_pos0 = np.ascontiguousarray(rnd.master_pos0, dtype=np.int64)
        self.agent_session = np.ascontiguousarray(rnd.agent_session, dtype=np.int32)
        self.agent_pos0 = np.ascontiguousarray(rnd.agent_pos0, dtype=np.int64)
        lens = np.array([len(b) for b in rnd.block_tables], dtype=np.int64)
        self.bt_offset = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
        self.bt_flat = (np.concatenate(rnd.block_tables).astype(np.int32)
                        if len(rnd.block_tables) else np.zeros(0, np.int32))
        self.desc = RoundDesc(len(self.span_tokens), _p(self.span_tokens), _p(self.master_pos0),
                              len(self.agent_session), _p(self.agent_session), _p(self.agent_pos0),
                              _p(self.bt_flat), _p(self.bt_offset), None, None, None, None, None, None)
        segs = getattr(rnd, "segments", None)
        if segs is not None:
            # per agent an int64 array [n_seg, 3] = (src_tok, dst_pos, len); empty = identity layout
            n = np.array([len(x) for x in segs], dtype=np.int64)
            self.seg_offset = np.concatenate([[0], np.cumsum(n)]).astype(np.int64)
            flat = np.concatenate([np.asarray(x, dtype=np.int64).reshape(-1, 3) for x in segs]) if n.sum() else np.zeros((0, 3), np.int64)
            self.seg_src = np.ascontiguousarray(flat[:, 0], dtype=np.int32)
            self.seg_dst = np.ascontiguousarray(flat[:, 1], dtype=np.int64)
            self.seg_len = np.ascontiguousarray(flat[:, 2], dtype=np.int32)
            self.desc.seg_offset, self.desc.seg_src = _p(self.seg_offset), _p(self.seg_src)
            self.desc.seg_len, self.desc.seg_dst = _p(self.seg_len), _p(self.seg_dst)
        if segment_diff_pos is not None:
            # per agent one position per segment: where the segment sat when the stored diff was encoded
            self.seg_diff_dst = np.ascontiguousarray(
                np.concatenate([np.asarray(x, dtype=np.int64).reshape(-1) for x in segment_diff_pos])
                if len(segment_diff_pos) else np.zeros(0, np.int64), dtype=np.int64)
            assert segs is not None and len(self.seg_diff_dst) == len(self.seg_dst)
            self.desc.seg_diff_dst = _p(self.seg_diff_dst)
        self.diff_pos0 = None
        if diff_pos0 is not None:
            self.diff_pos0 = np.ascontiguousarray(diff_pos0, dtype=np.int64)
            self.desc.agent_diff_pos0 = _p(self.diff_pos0)
        self.pool_pages = int(rnd.pool_pages)


def rope_table(theta: float, head_dim: int, delta: int, f64: bool = False):
    dt = np.float64 if f64 else np.float32
    c = np.zeros(head_dim // 2, dtype=dt)
    s = np.zeros(head_dim // 2, dtype=dt)
    fn = lib().tdo_rope_table_f64 if f64 else lib().tdo_rope_table_f32
    _chk(fn(float(theta), head_dim, int(delta), _p(c), _p(s)), "rope_table")
    return c, s


def rotate_rows_f32(g: Geom, delta: int, x: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    re = g.num_kv_heads * g.head_dim
    assert x.size % re == 0
    y = np.empty_like(x)
    _chk(lib().tdo_rotate_rows_f32(C.byref(g), int(delta), x.size // re, _p(x), _p(y)), "rotate_rows_f32")
    return y


def rotate_rows_f32_bf16(g: Geom, delta: int, x: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    re = g.num_kv_heads * g.head_dim
    assert x.size % re == 0
    y = np.empty(x.shape, dtype=np.uint16)
    _chk(lib().tdo_rotate_rows_f32_bf16(C.byref(g), int(delta), x.size // re, _p(x), _p(y)), "rotate_rows_f32_bf16")
    return y


def rotate_rows_bf16(g: Geom, delta: int, x: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.uint16)
    re = g.num_kv_heads * g.head_dim
    assert x.size % re == 0
    y = np.empty_like(x)
    _chk(lib().tdo_rotate_rows_bf16(C.byref(g), int(delta), x.size // re, _p(x), _p(y)), "rotate_rows_bf16")
    return y


def _u16(a):
    assert a.dtype == np.uint16 and a.flags["C_CONTIGUOUS"]
    return a


def rerotate_round(g: Geom, hr: HostRound, master_k, master_v, pool_k, pool_v) -> None:
    _chk(lib().tdo_rerotate_round(C.byref(g), C.byref(hr.desc), _p(_u16(master_k)), _p(_u16(master_v)),
                                  _p(_u16(pool_k)), _p(_u16(pool_v)), hr.pool_pages), "rerotate_round")


class Diff:
    def __init__(self, n_agents: int, capacity_pages: int, page_elems: int):
        self.count = np.zeros(n_agents, dtype=np.int32)
        self.offset = np.zeros(n_agents + 1, dtype=np.int64)
        self.idx = np.full(max(capacity_pages, 1), -1, dtype=np.int32)
        # non-zero fill: rows the encoder must zero are then visibly its own work
        self.payload = np.full((max(capacity_pages, 1), page_elems), 0xFFFF, dtype=np.uint16)
        self.capacity_pages = int(capacity_pages)
        self.overflow = np.zeros(1, dtype=np.int32)


def diff_encode(g: Geom, hr: HostRound, master_k, master_v, pool_k, pool_v, eps: float,
                capacity_pages: int) -> Diff:
    d = Diff(hr.desc.n_agents, capacity_pages, 2 * g.page_tokens * g.num_kv_heads * g.head_dim)
    _chk(lib().tdo_diff_encode(C.byref(g), C.byref(hr.desc), _p(_u16(master_k)), _p(_u16(master_v)),
                               _p(_u16(pool_k)), _p(_u16(pool_v)), hr.pool_pages, C.c_float(eps),
                               _p(d.count), _p(d.offset), _p(d.idx), _p(d.payload),
                               d.capacity_pages, _p(d.overflow)), "diff_encode")
    return d


def diff_encode_plane(g: Geom, hr: HostRound, master_k, master_v, pool_k, pool_v, eps: float, plane: int,
                      capacity_pages: int) -> Diff:
    d = Diff(hr.desc.n_agents, capacity_pages, g.page_tokens * g.num_kv_heads * g.head_dim)
    _chk(lib().tdo_diff_encode_plane(C.byref(g), C.byref(hr.desc), _p(_u16(master_k)), _p(_u16(master_v)),
                                     _p(_u16(pool_k)), _p(_u16(pool_v)), hr.pool_pages, C.c_float(eps), plane,
                                     _p(d.count), _p(d.offset), _p(d.idx), _p(d.payload),
                                     d.capacity_pages, _p(d.overflow)), "diff_encode_plane")
    return d


def diff_decode_plane(g: Geom, hr: HostRound, master_k, master_v, pool_k, pool_v, plane: int, d: Diff) -> None:
    _chk(lib().tdo_diff_decode_plane(C.byref(g), C.byref(hr.desc), _p(_u16(master_k)), _p(_u16(master_v)),
                                     _p(_u16(pool_k)), _p(_u16(pool_v)), hr.pool_pages, plane,
                                     _p(d.count), _p(d.offset), _p(d.idx), _p(d.payload)), "diff_decode_plane")


def diff_decode(g: Geom, hr: HostRound, master_k, master_v, pool_k, pool_v, d: Diff) -> None:
    _chk(lib().tdo_diff_decode(C.byref(g), C.byref(hr.desc), _p(_u16(master_k)), _p(_u16(master_v)),
                               _p(_u16(pool_k)), _p(_u16(pool_v)), hr.pool_pages,
                               _p(d.count), _p(d.offset), _p(d.idx), _p(d.payload)), "diff_decode")


def key_deviation(g: Geom, hr: HostRound, master_k, pool_k) -> np.ndarray:
    n = int(sum(int(hr.span_tokens[s]) for s in hr.agent_session))
    score = np.zeros(n, dtype=np.float64)
    _chk(lib().tdo_key_deviation(C.byref(g), C.byref(hr.desc), _p(_u16(master_k)), _p(_u16(pool_k)),
                                 hr.pool_pages, _p(score)), "key_deviation")
    return score


def select_important(score: np.ndarray, ratio: float, min_score: float) -> np.ndarray:
    score = np.ascontiguousarray(score, dtype=np.float32)
    out = np.zeros(max(len(score), 1), dtype=np.int32)
    n = np.zeros(1, dtype=np.int32)
    _chk(lib().tdo_select_important(_p(score), len(score), C.c_float(ratio), C.c_float(min_score), _p(out), _p(n)),
         "select_important")
    return out[:int(n[0])].copy()


def choose_master(hr: HostRound, total: np.ndarray) -> np.ndarray:
    total = np.ascontiguousarray(total, dtype=np.float32)
    master = np.zeros(max(hr.desc.n_sessions, 1), dtype=np.int32)
    _chk(lib().tdo_choose_master(C.byref(hr.desc), _p(total), _p(master)), "choose_master")
    return master[:hr.desc.n_sessions].copy()


def restore_layers(g: Geom, hr: HostRound, masters_k, masters_v, pools_k, pools_v, diffs) -> None:
    """Alg. 1 over len(diffs) layers; every argument is a per-layer list."""
    n = len(diffs)

    def arr(xs):
        return (C.c_void_p * max(n, 1))(*[_p(x) for x in xs])

    _chk(lib().tdo_restore_layers(C.byref(g), C.byref(hr.desc), n, arr(masters_k), arr(masters_v),
                                  arr(pools_k), arr(pools_v), hr.pool_pages,
                                  arr([d.count for d in diffs]), arr([d.offset for d in diffs]),
                                  arr([d.idx for d in diffs]), arr([d.payload for d in diffs])), "restore_layers")


def dense_bytes(g: Geom, span_tokens: int) -> float:
    return lib().tdo_dense_bytes(C.byref(g), int(span_tokens))


def diff_bytes(g: Geom, pages: int) -> float:
    return lib().tdo_diff_bytes(C.byref(g), int(pages))


def mirror_ratio(g: Geom, span_tokens: int, pages: int) -> float:
    return lib().tdo_mirror_ratio(C.byref(g), int(span_tokens), int(pages))


def family_cost(n_agents: int, ratio: float) -> float:
    return lib().tdo_family_cost(int(n_agents), float(ratio))


def attend_shared(g: Geom, hr: HostRound, master_k, master_v, d: "Diff", q, n_q: int, n_q_heads: int, scale: float):
    """Attention of q [A][n_q][n_q_heads][D] (bf16 bits) over every Mirror's shared span, from Master + diff.
    Returns (out float64 [A][n_q][n_q_heads][D], lse float64 [A][n_q][n_q_heads])."""
    A = int(hr.desc.n_agents)
    q = np.ascontiguousarray(q, dtype=np.uint16)
    assert q.size == A * n_q * n_q_heads * g.head_dim
    out = np.zeros((A, n_q, n_q_heads, g.head_dim), np.float64)
    lse = np.zeros((A, n_q, n_q_heads), np.float64)
    _chk(lib().tdo_attend_shared(C.byref(g), C.byref(hr.desc), _p(_u16(master_k)), _p(_u16(master_v)),
                                 _p(d.count), _p(d.offset), _p(d.idx), _p(d.payload), _p(q), n_q, n_q_heads,
                                 float(scale), _p(out), _p(lse)), "attend_shared")
    return out, lse


def max_threads() -> int:
    return int(lib().tdo_max_threads())


def set_threads(n: int) -> None:
    """Threads the agent loops use from now on (for timing; results do not depend on it)."""
    lib().tdo_set_threads(int(n))
