"""Thin ctypes binding over libtdk.so: same names as include/tdk.h, argument marshalling only.

Device buffers are passed as anything with a ``data_ptr()`` (torch tensors) or as integer
addresses; streams as integer ``hipStream_t`` handles (``torch.cuda.current_stream().cuda_stream``).
There is no CPU fallback: if the library has not been built, loading fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libtdk.so")

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_CAPACITY, ERR_HIP, ERR_NOMEM = range(6)
BF16 = 0
ROPE_HALF, ROPE_INTERLEAVED = 0, 1
PLANE_K, PLANE_V = 1, 2
(KERNEL_REROTATE, KERNEL_FLAG, KERNEL_COMPACT, KERNEL_GATHER, KERNEL_DECODE, KERNEL_SCATTER,
 KERNEL_KEYDIFF, KERNEL_SELECT, KERNEL_MASTER, KERNEL_ATTEND_QROT, KERNEL_ATTEND_MASTER, KERNEL_ATTEND_DIFF,
 KERNEL_ATTEND_MERGE) = range(13)
KERNEL_KINDS = 13
TUNE_XCD_QUEUES, TUNE_TAPER, TUNE_QUEUES_ANY_SIZE = 128, 256, 512
TUNE_SCATTER_IN_DECODE = 1024
TUNE_SHARED_TAIL = 2048
TUNE_ALL, TUNE_DEFAULT = 4095, 191 + 1024 + 2048
STATIC_SCRATCH_BYTES = 4 << 20

EXPORTS = (
    "tdk_status_str", "tdk_last_error", "tdk_version", "tdk_kernel_name",
    "tdk_round_create", "tdk_round_destroy", "tdk_scratch_bytes", "tdk_round_tune", "tdk_round_agents_per_group",
    "tdk_rerotate_round", "tdk_diff_encode", "tdk_diff_encode_static", "tdk_diff_decode", "tdk_restore_layers", "tdk_check_layer",
    "tdk_diff_encode_plane", "tdk_diff_decode_plane", "tdk_attend_workspace_bytes", "tdk_attend_shared",
    "tdk_prompt_plan_create", "tdk_prompt_plan_destroy", "tdk_prompt_plan_n_sessions", "tdk_prompt_plan_span",
    "tdk_prompt_plan_session_of", "tdk_prompt_plan_segments",
    "tdk_timing_enable", "tdk_timing_read", "tdk_timing_reset",
    "tdk_dense_bytes", "tdk_diff_bytes", "tdk_family_cost",
    "tdk_util_copy", "tdk_util_fill", "tdk_util_page_fill", "tdk_util_page_read",
    "tdk_util_page_fill_product", "tdk_util_page_read_product", "tdk_timeline_bytes", "tdk_timeline_set",
)


class Model(C.Structure):
    _fields_ = [("num_layers", C.c_int32), ("num_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("page_tokens", C.c_int32), ("dtype", C.c_int32), ("rope_style", C.c_int32),
                ("rope_theta", C.c_double)]


class Session(C.Structure):
    _fields_ = [("span_tokens", C.c_int32), ("master_pos0", C.c_int64)]


class Segment(C.Structure):
    _fields_ = [("src_tok", C.c_int32), ("len", C.c_int32), ("dst_pos", C.c_int64), ("diff_pos", C.c_int64)]


class Agent(C.Structure):
    _fields_ = [("session", C.c_int32), ("dst_pos0", C.c_int64), ("block_table", C.c_void_p),
                ("block_table_len", C.c_int32), ("diff_pos0", C.c_int64), ("n_segments", C.c_int32),
                ("segments", C.c_void_p)]


class LayerIO(C.Structure):
    _fields_ = [("master_k", C.c_void_p), ("master_v", C.c_void_p), ("pool_k", C.c_void_p),
                ("pool_v", C.c_void_p), ("pool_pages", C.c_int64)]


class Diff(C.Structure):
    _fields_ = [("count", C.c_void_p), ("offset", C.c_void_p), ("idx", C.c_void_p),
                ("payload", C.c_void_p), ("capacity_pages", C.c_int64), ("overflow", C.c_void_p)]


class ReusePlan(C.Structure):
    _fields_ = [("score", C.c_void_p), ("important", C.c_void_p), ("k_stride", C.c_int32),
                ("n_important", C.c_void_p), ("total", C.c_void_p), ("master", C.c_void_p)]


class AttendIO(C.Structure):
    _fields_ = [("q", C.c_void_p), ("n_q", C.c_int32), ("n_q_heads", C.c_int32), ("scale", C.c_float),
                ("out", C.c_void_p), ("lse", C.c_void_p), ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t)]


class Prompt(C.Structure):
    _fields_ = [("tokens", C.c_void_p), ("n_tokens", C.c_int32)]


class PingPong(C.Structure):
    _fields_ = [("stage_k", C.c_void_p * 2), ("stage_v", C.c_void_p * 2), ("stage_bytes", C.c_size_t)]


class TdkError(RuntimeError):
    def __init__(self, status: int, what: str, detail: str):
        super().__init__(f"{what}: status {status} ({detail})")
        self.status = status
        self.detail = detail


_lib: Optional[C.CDLL] = None


def load() -> C.CDLL:
    """Loads the built library; raises if it is missing (build it with __graft_entry__.build())."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'`")
    L = C.CDLL(LIB_PATH)
    L.tdk_status_str.restype = C.c_char_p
    L.tdk_status_str.argtypes = [C.c_int]
    L.tdk_last_error.restype = C.c_char_p
    L.tdk_version.restype = C.c_char_p
    L.tdk_kernel_name.restype = C.c_char_p
    L.tdk_kernel_name.argtypes = [C.c_int32]
    L.tdk_round_create.argtypes = [C.POINTER(Model), C.POINTER(Session), C.c_int32, C.POINTER(Agent),
                                   C.c_int32, C.POINTER(C.c_void_p)]
    L.tdk_round_destroy.argtypes = [C.c_void_p]
    L.tdk_round_destroy.restype = None
    L.tdk_scratch_bytes.argtypes = [C.c_void_p]
    L.tdk_scratch_bytes.restype = C.c_size_t
    L.tdk_round_tune.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
    L.tdk_round_agents_per_group.argtypes = [C.c_void_p]
    L.tdk_rerotate_round.argtypes = [C.c_void_p, C.c_int32, C.POINTER(LayerIO), C.c_void_p]
    L.tdk_diff_encode.argtypes = [C.c_void_p, C.c_int32, C.POINTER(LayerIO), C.c_float, C.POINTER(Diff), C.c_void_p]
    L.tdk_diff_encode_static.argtypes = L.tdk_diff_encode.argtypes
    L.tdk_diff_decode.argtypes = [C.c_void_p, C.c_int32, C.POINTER(LayerIO), C.POINTER(Diff), C.c_void_p]
    L.tdk_diff_encode_plane.argtypes = [C.c_void_p, C.c_int32, C.POINTER(LayerIO), C.c_float, C.c_int32, C.POINTER(Diff), C.c_void_p]
    L.tdk_diff_decode_plane.argtypes = [C.c_void_p, C.c_int32, C.POINTER(LayerIO), C.c_int32, C.POINTER(Diff), C.c_void_p]
    L.tdk_check_layer.argtypes = [C.c_void_p, C.c_int32, C.POINTER(LayerIO), C.c_float, C.c_float,
                                  C.POINTER(ReusePlan), C.c_void_p]
    L.tdk_attend_workspace_bytes.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
    L.tdk_attend_workspace_bytes.restype = C.c_size_t
    L.tdk_attend_shared.argtypes = [C.c_void_p, C.c_int32, C.POINTER(LayerIO), C.POINTER(Diff), C.POINTER(AttendIO), C.c_void_p]
    L.tdk_prompt_plan_create.argtypes = [C.POINTER(Prompt), C.c_int32, C.c_int32, C.POINTER(C.c_void_p)]
    L.tdk_prompt_plan_destroy.argtypes = [C.c_void_p]
    L.tdk_prompt_plan_destroy.restype = None
    L.tdk_prompt_plan_n_sessions.argtypes = [C.c_void_p]
    L.tdk_prompt_plan_span.argtypes = [C.c_void_p, C.c_int32]
    L.tdk_prompt_plan_session_of.argtypes = [C.c_void_p, C.c_int32]
    L.tdk_prompt_plan_segments.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.POINTER(Segment))]
    L.tdk_restore_layers.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p),
                                     C.POINTER(LayerIO), C.POINTER(Diff), C.POINTER(PingPong), C.c_void_p, C.c_void_p]
    L.tdk_timing_enable.argtypes = [C.c_void_p, C.c_int32]
    L.tdk_timing_read.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    L.tdk_timing_reset.argtypes = [C.c_void_p]
    for name in ("tdk_dense_bytes", "tdk_diff_bytes", "tdk_family_cost"):
        getattr(L, name).restype = C.c_double
    L.tdk_dense_bytes.argtypes = [C.POINTER(Model), C.c_int64]
    L.tdk_diff_bytes.argtypes = [C.POINTER(Model), C.c_int64]
    L.tdk_family_cost.argtypes = [C.c_int64, C.c_double]
    L.tdk_util_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    L.tdk_util_fill.argtypes = [C.c_void_p, C.c_uint32, C.c_size_t, C.c_void_p]
    L.tdk_util_page_fill.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_size_t, C.c_uint32, C.c_void_p]
    L.tdk_util_page_read.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_size_t, C.c_void_p, C.c_void_p]
    L.tdk_util_page_fill_product.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                             C.c_uint32, C.c_void_p]
    L.tdk_util_page_read_product.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                             C.c_void_p, C.c_void_p]
    L.tdk_timeline_bytes.argtypes = [C.c_void_p]
    L.tdk_timeline_bytes.restype = C.c_size_t
    L.tdk_timeline_set.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t]
    _lib = L
    return L


def _ptr(x) -> Optional[int]:
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        return int(x.data_ptr())
    return int(x)


def _check(status: int, what: str) -> None:
    if status != OK:
        raise TdkError(status, what, load().tdk_last_error().decode())


def tdk_status_str(status: int) -> str:
    return load().tdk_status_str(status).decode()


def tdk_last_error() -> str:
    return load().tdk_last_error().decode()


def tdk_version() -> str:
    return load().tdk_version().decode()


def tdk_kernel_name(kernel: int) -> str:
    return load().tdk_kernel_name(kernel).decode()


def model(num_layers, num_kv_heads=8, head_dim=128, page_tokens=16, rope_theta=1.0e6,
          rope_style=ROPE_HALF, dtype=BF16) -> Model:
    return Model(num_layers, num_kv_heads, head_dim, page_tokens, dtype, rope_style, float(rope_theta))


class Round:
    """Owns a tdk_round handle."""

    def __init__(self, handle: int, n_agents: int, keep):
        self.handle = C.c_void_p(handle)
        self.n_agents = n_agents
        self._keep = keep

    def destroy(self) -> None:
        if self.handle:
            load().tdk_round_destroy(self.handle)
            self.handle = C.c_void_p(None)

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def tdk_round_create(mdl: Model, span_tokens: Sequence[int], master_pos0: Sequence[int],
                     agent_session: Sequence[int], agent_pos0: Sequence[int],
                     block_tables: Sequence[np.ndarray], agent_diff_pos0: Optional[Sequence[int]] = None,
                     segments: Optional[Sequence[np.ndarray]] = None,
                     segment_diff_pos: Optional[Sequence[np.ndarray]] = None) -> Round:
    """segments: per agent an int array [n_seg, 3] of (src_tok, dst_pos, len), empty = identity layout.
    segment_diff_pos: per agent the position of each segment when the diff to restore was encoded
    (default: dst_pos, a diff of this round)."""
    ns, na = len(span_tokens), len(agent_session)
    sess = (Session * max(ns, 1))()
    for s in range(ns):
        sess[s] = Session(int(span_tokens[s]), int(master_pos0[s]))
    ags = (Agent * max(na, 1))()
    keep = []
    for i in range(na):
        bt = np.ascontiguousarray(block_tables[i], dtype=np.int32)
        keep.append(bt)
        dp = int(agent_pos0[i]) if agent_diff_pos0 is None else int(agent_diff_pos0[i])
        nseg, segp = 0, None
        if segments is not None and len(segments[i]):
            dpos = [int(x[1]) for x in segments[i]] if segment_diff_pos is None else [int(v) for v in segment_diff_pos[i]]
            if len(dpos) != len(segments[i]):
                raise ValueError("segment_diff_pos must give one position per segment")
            sg = (Segment * len(segments[i]))(*[Segment(int(x[0]), int(x[2]), int(x[1]), dpos[q])
                                                for q, x in enumerate(segments[i])])
            keep.append(sg)
            nseg, segp = len(segments[i]), C.cast(sg, C.c_void_p)
        ags[i] = Agent(int(agent_session[i]), int(agent_pos0[i]), bt.ctypes.data, len(bt), dp, nseg, segp)
    out = C.c_void_p()
    _check(load().tdk_round_create(C.byref(mdl), sess, ns, ags, na, C.byref(out)), "tdk_round_create")
    return Round(out.value, na, None)


def round_from_workload(rnd, style=ROPE_HALF, diff_pos0=None, segment_diff_pos=None) -> Round:
    """Convenience: a tdk round for a workload.Round (marshalling only)."""
    sp = rnd.spec
    mdl = model(sp.num_layers, sp.num_kv_heads, sp.head_dim, sp.page_tokens, sp.rope_theta, style)
    return tdk_round_create(mdl, rnd.span_tokens, rnd.master_pos0, rnd.agent_session, rnd.agent_pos0,
                            rnd.block_tables, diff_pos0, getattr(rnd, "segments", None), segment_diff_pos)


def tdk_round_destroy(r: Round) -> None:
    r.destroy()


def tdk_scratch_bytes(r: Round) -> int:
    return int(load().tdk_scratch_bytes(r.handle))


def tdk_round_tune(r: Round, agents_per_group: int = 0, flags: int = TUNE_DEFAULT) -> None:
    _check(load().tdk_round_tune(r.handle, agents_per_group, flags), "tdk_round_tune")


def tdk_round_agents_per_group(r: Round) -> int:
    return int(load().tdk_round_agents_per_group(r.handle))


def layer_io(master_k, master_v, pool_k, pool_v, pool_pages: int) -> LayerIO:
    return LayerIO(_ptr(master_k), _ptr(master_v), _ptr(pool_k), _ptr(pool_v), int(pool_pages))


def diff(count, offset, idx, payload, capacity_pages: int, overflow) -> Diff:
    return Diff(_ptr(count), _ptr(offset), _ptr(idx), _ptr(payload), int(capacity_pages), _ptr(overflow))


def tdk_rerotate_round(r: Round, layer: int, io: LayerIO, stream: int = 0) -> None:
    _check(load().tdk_rerotate_round(r.handle, layer, C.byref(io), C.c_void_p(stream)), "tdk_rerotate_round")


def tdk_diff_encode(r: Round, layer: int, io: LayerIO, eps: float, out: Diff, stream: int = 0) -> None:
    _check(load().tdk_diff_encode(r.handle, layer, C.byref(io), C.c_float(eps), C.byref(out),
                                  C.c_void_p(stream)), "tdk_diff_encode")


def tdk_diff_encode_static(r: Round, layer: int, io: LayerIO, eps: float, out: Diff, stream: int = 0) -> None:
    _check(load().tdk_diff_encode_static(r.handle, layer, C.byref(io), C.c_float(eps), C.byref(out),
                                         C.c_void_p(stream)), "tdk_diff_encode_static")


def tdk_diff_decode(r: Round, layer: int, io: LayerIO, d: Diff, stream: int = 0) -> None:
    _check(load().tdk_diff_decode(r.handle, layer, C.byref(io), C.byref(d), C.c_void_p(stream)),
           "tdk_diff_decode")


def reuse_plan(score, important, k_stride: int, n_important, total, master) -> ReusePlan:
    return ReusePlan(_ptr(score), _ptr(important), int(k_stride), _ptr(n_important), _ptr(total), _ptr(master))


def tdk_check_layer(r: Round, layer: int, io: LayerIO, ratio: float, min_score: float, plan: ReusePlan,
                    stream: int = 0) -> None:
    _check(load().tdk_check_layer(r.handle, layer, C.byref(io), C.c_float(ratio), C.c_float(min_score),
                                  C.byref(plan), C.c_void_p(stream)), "tdk_check_layer")


def tdk_attend_workspace_bytes(r: Round, n_q: int, n_q_heads: int) -> int:
    return int(load().tdk_attend_workspace_bytes(r.handle, n_q, n_q_heads))


def attend_io(q, n_q: int, n_q_heads: int, scale: float, out, lse, workspace, workspace_bytes: int) -> AttendIO:
    return AttendIO(_ptr(q), int(n_q), int(n_q_heads), float(scale), _ptr(out), _ptr(lse), _ptr(workspace),
                    int(workspace_bytes))


def tdk_attend_shared(r: Round, layer: int, io: LayerIO, d: Diff, a: AttendIO, stream: int = 0) -> None:
    _check(load().tdk_attend_shared(r.handle, layer, C.byref(io), C.byref(d), C.byref(a), C.c_void_p(stream)),
           "tdk_attend_shared")


def tdk_prompt_plan(prompts: Sequence[Sequence[int]], separator: int):
    """Marshals token lists through tdk_prompt_plan_create and returns (spans per session, session per
    prompt, segments per prompt as lists of (src_tok, dst_pos, len))."""
    arrs = [np.ascontiguousarray(p, dtype=np.int32) for p in prompts]
    ps = (Prompt * max(len(arrs), 1))()
    for i, a in enumerate(arrs):
        ps[i] = Prompt(a.ctypes.data if a.size else None, int(a.size))
    plan = C.c_void_p()
    L = load()
    _check(L.tdk_prompt_plan_create(ps, len(arrs), int(separator), C.byref(plan)), "tdk_prompt_plan_create")
    try:
        spans = [int(L.tdk_prompt_plan_span(plan, s)) for s in range(int(L.tdk_prompt_plan_n_sessions(plan)))]
        session_of, segments = [], []
        for i in range(len(arrs)):
            session_of.append(int(L.tdk_prompt_plan_session_of(plan, i)))
            sp = C.POINTER(Segment)()
            n = int(L.tdk_prompt_plan_segments(plan, i, C.byref(sp)))
            segments.append([(int(sp[k].src_tok), int(sp[k].dst_pos), int(sp[k].len)) for k in range(n)])
        return spans, session_of, segments
    finally:
        L.tdk_prompt_plan_destroy(plan)


def pingpong(stage_k0, stage_k1, stage_v0, stage_v1, stage_bytes: int) -> PingPong:
    pp = PingPong()
    pp.stage_k[0], pp.stage_k[1] = _ptr(stage_k0), _ptr(stage_k1)
    pp.stage_v[0], pp.stage_v[1] = _ptr(stage_v0), _ptr(stage_v1)
    pp.stage_bytes = int(stage_bytes)
    return pp


def tdk_restore_layers(r: Round, first_layer: int, host_master_k, host_master_v, ios, diffs, pp: PingPong,
                       compute_stream: int = 0, copy_stream: int = 0) -> None:
    """host_master_k/v: per-layer pinned host tensors (or addresses); ios / diffs: per-layer LayerIO / Diff."""
    n = len(ios)
    hk = (C.c_void_p * max(n, 1))(*[_ptr(x) for x in host_master_k])
    hv = (C.c_void_p * max(n, 1))(*[_ptr(x) for x in host_master_v])
    io_arr = (LayerIO * max(n, 1))(*ios)
    d_arr = (Diff * max(n, 1))(*diffs)
    _check(load().tdk_restore_layers(r.handle, first_layer, n, hk, hv, io_arr, d_arr, C.byref(pp),
                                     C.c_void_p(compute_stream), C.c_void_p(copy_stream)), "tdk_restore_layers")


def tdk_diff_encode_plane(r: Round, layer: int, io: LayerIO, eps: float, plane: int, out: Diff, stream: int = 0) -> None:
    _check(load().tdk_diff_encode_plane(r.handle, layer, C.byref(io), C.c_float(eps), plane, C.byref(out),
                                        C.c_void_p(stream)), "tdk_diff_encode_plane")


def tdk_diff_decode_plane(r: Round, layer: int, io: LayerIO, plane: int, d: Diff, stream: int = 0) -> None:
    _check(load().tdk_diff_decode_plane(r.handle, layer, C.byref(io), plane, C.byref(d), C.c_void_p(stream)),
           "tdk_diff_decode_plane")


def tdk_timing_enable(r: Round, on: bool) -> None:
    _check(load().tdk_timing_enable(r.handle, 1 if on else 0), "tdk_timing_enable")


def tdk_timing_read(r: Round, kernel: int):
    ms, n = C.c_double(), C.c_int64()
    _check(load().tdk_timing_read(r.handle, kernel, C.byref(ms), C.byref(n)), "tdk_timing_read")
    return ms.value, n.value


def tdk_timing_reset(r: Round) -> None:
    _check(load().tdk_timing_reset(r.handle), "tdk_timing_reset")


def tdk_dense_bytes(mdl: Model, span_tokens: int) -> float:
    return load().tdk_dense_bytes(C.byref(mdl), int(span_tokens))


def tdk_diff_bytes(mdl: Model, pages: int) -> float:
    return load().tdk_diff_bytes(C.byref(mdl), int(pages))


def tdk_family_cost(n_agents: int, ratio: float) -> float:
    return load().tdk_family_cost(int(n_agents), float(ratio))


def tdk_util_copy(dst, src, nbytes: int, stream: int = 0) -> None:
    _check(load().tdk_util_copy(_ptr(dst), _ptr(src), int(nbytes), C.c_void_p(stream)), "tdk_util_copy")


def tdk_util_fill(dst, word: int, nbytes: int, stream: int = 0) -> None:
    _check(load().tdk_util_fill(_ptr(dst), int(word) & 0xFFFFFFFF, int(nbytes), C.c_void_p(stream)), "tdk_util_fill")


def tdk_util_page_fill(dst, page_ids, n_pages: int, page_bytes: int, word: int = 0, stream: int = 0) -> None:
    _check(load().tdk_util_page_fill(_ptr(dst), _ptr(page_ids), int(n_pages), int(page_bytes),
                                     int(word) & 0xFFFFFFFF, C.c_void_p(stream)), "tdk_util_page_fill")


def tdk_util_page_read(src, page_ids, n_pages: int, page_bytes: int, sink16, stream: int = 0) -> None:
    _check(load().tdk_util_page_read(_ptr(src), _ptr(page_ids), int(n_pages), int(page_bytes), _ptr(sink16),
                                     C.c_void_p(stream)), "tdk_util_page_read")


def tdk_util_page_fill_product(plane_k, plane_v, page_ids, n_pages: int, group: int, num_kv_heads: int, page_tokens: int,
                               word: int = 0, stream: int = 0) -> None:
    _check(load().tdk_util_page_fill_product(_ptr(plane_k), _ptr(plane_v), _ptr(page_ids), int(n_pages), int(group),
                                             int(num_kv_heads), int(page_tokens), int(word) & 0xFFFFFFFF,
                                             C.c_void_p(stream)), "tdk_util_page_fill_product")


def tdk_util_page_read_product(plane_k, plane_v, page_ids, n_pages: int, group: int, num_kv_heads: int, page_tokens: int,
                               sink16, stream: int = 0) -> None:
    _check(load().tdk_util_page_read_product(_ptr(plane_k), _ptr(plane_v), _ptr(page_ids), int(n_pages), int(group),
                                             int(num_kv_heads), int(page_tokens), _ptr(sink16), C.c_void_p(stream)),
           "tdk_util_page_read_product")


def tdk_timeline_bytes(r: Round) -> int:
    return int(load().tdk_timeline_bytes(r.handle))


def tdk_timeline_set(r: Round, stamps, nbytes: int = 0) -> None:
    _check(load().tdk_timeline_set(r.handle, _ptr(stamps), int(nbytes)), "tdk_timeline_set")
