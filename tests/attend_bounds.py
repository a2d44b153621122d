"""Per-row error bounds for the attention over never-restored mirrors (Sec. 4.4, Fig. 9), derived from the
arithmetic of the GPU path, and the expected values they are applied to (the oracle's, double precision).

What the GPU path rounds that the definition does not:

  (a) every query row is rotated back by its agent's offset (by dst - diff position for the listed pages) in
      fp32 and rounded to bf16: element d carries an independent error of at most 2^-9 |q'_d|, uniform within
      its rounding interval, i.e. of variance at most (2^-9 |q'_d|)^2 / 3.  The score of token m therefore moves
      by  ds_m = scale * sum_d e_d q'_d k_md,  std(ds_m) <= |scale| * 2^-9 / sqrt(3) * sqrt(sum_d q'_d^2 k_md^2).
      A rotation keeps the norm of every pair, so  sum_d q'_d^2 k_md^2 <= sum_pairs |q_pair|^2 |k_m,pair|^2,
      which needs neither the angle nor the frame the keys sit in.  E(row) = 5 std, maximised over the tokens the
      row meets (master rows of its session and its agent's payload rows), bounds |ds_m| for all of them.
  (b) the softmax weights are rounded to bf16 for the second product: 2^-9 relative each, and the same again
      for the denominator in the worst case: 2^-8.
  (c) fp32 accumulation over the span, in hardware order: below 2^-12 relative for spans up to 2^17 tokens
      (error growth sqrt(S) * 2^-24 typical, S * 2^-24 worst over 4 k tokens).

Consequences, per query row and output element d, with w_m the exact weights and A_d = sum_m w_m |V_md| (the
oracle evaluated on |V|):
  weights:  w~_m / w_m lies in [exp(-2E), exp(2E)]          =>  |out~_d - out_d| <= (exp(2E) - 1) A_d
  rounding: (b), (c)                                         =>  + (2^-8 + 2^-12) A_d
  lse:      log sum exp moves by at most max_m |ds_m|        =>  |lse~ - lse| <= E + 1e-4
(1e-4: fp32 representation of values up to a few tens, exp2 / log of the hardware to a few ulp).
"""
from __future__ import annotations

import copy

import numpy as np

from paper_2604_03143_amd import workload as wl

SIGMAS = 5.0
U = 2.0 ** -9


def _pair_norm2(x: np.ndarray, style: int) -> np.ndarray:
    """[..., D] values -> [..., D/2] squared norms of the rotation pairs."""
    x = x.astype(np.float64)
    half = x.shape[-1] // 2
    if style == 0:
        return x[..., :half] ** 2 + x[..., half:] ** 2
    return x[..., 0::2] ** 2 + x[..., 1::2] ** 2


def score_error_bound(g, hr, master_k, d, q, n_q, n_q_heads, scale) -> np.ndarray:
    """E of the derivation above: [A][n_q][n_q_heads]."""
    H, D, T = g.num_kv_heads, g.head_dim, g.page_tokens
    A = int(hr.desc.n_agents)
    G = n_q_heads // H
    qf = wl.bf16_bits_to_f32(np.ascontiguousarray(q, np.uint16)).reshape(A, n_q, n_q_heads, D)
    qp2 = _pair_norm2(qf, g.rope_style)                                  # [A][n_q][Hq][D/2]
    mk2 = _pair_norm2(wl.bf16_bits_to_f32(master_k).reshape(-1, H, D), g.rope_style)   # [rows][H][D/2]
    row0 = np.concatenate([[0], np.cumsum(hr.span_tokens.astype(np.int64))])
    E = np.zeros((A, n_q, n_q_heads))
    for i in range(A):
        s = int(hr.agent_session[i])
        keys = [mk2[row0[s]:row0[s + 1]]]
        lo, n = int(d.offset[i]), int(d.count[i])
        n = max(0, min(n, d.capacity_pages - lo))
        if n > 0:
            pay_k = d.payload[lo:lo + n].reshape(n, 2, T, H, D)[:, 0]
            keys.append(_pair_norm2(wl.bf16_bits_to_f32(pay_k).reshape(-1, H, D), g.rope_style))
        k2 = np.concatenate(keys)                                        # [tokens][H][D/2]
        if k2.shape[0] == 0:
            continue
        for h in range(H):
            qq = qp2[i, :, h * G:(h + 1) * G, :].reshape(-1, D // 2)     # [n_q * G][D/2]
            var = (k2[:, h, :] @ qq.T).max(axis=0)                       # max over tokens of sum_pairs
            E[i, :, h * G:(h + 1) * G] = (SIGMAS * abs(scale) * U / np.sqrt(3.0) * np.sqrt(var)).reshape(n_q, G)
    return E


def expected_and_bounds(tdo, g, hr, master_k, master_v, d, q, n_q, n_q_heads, scale):
    """(want_out, want_lse, tol_out, tol_lse): the oracle's values and the bounds derived above."""
    want_o, want_l = tdo.attend_shared(g, hr, master_k, master_v, d, q, n_q, n_q_heads, scale)
    # A_d = sum_m w_m |V_md|: the same weights over the absolute values of V (sign bits cleared, master and payload)
    T, H, D = g.page_tokens, g.num_kv_heads, g.head_dim
    d_abs = copy.copy(d)
    d_abs.payload = d.payload.copy()
    pv = d_abs.payload.reshape(d_abs.payload.shape[0], 2, T * H * D)
    pv[:, 1] &= np.uint16(0x7FFF)
    abs_o, _ = tdo.attend_shared(g, hr, master_k, master_v & np.uint16(0x7FFF), d_abs, q, n_q, n_q_heads, scale)
    E = score_error_bound(g, hr, master_k, d, q, n_q, n_q_heads, scale)
    tol_o = (np.expm1(2.0 * E) + 2.0 ** -8 + 2.0 ** -12)[..., None] * abs_o + 1e-7
    tol_l = E + 1e-4
    return want_o, want_l, tol_o, tol_l


def _errors(got_o, got_l, want_o, want_l):
    """Absolute errors; a row with an empty span (lse = -inf, out = 0 by definition) must match exactly."""
    empty = np.isneginf(want_l)
    with np.errstate(invalid="ignore"):
        el = np.where(empty, np.where(got_l == want_l, 0.0, np.inf), np.abs(got_l - want_l))
        eo = np.abs(got_o - want_o)
    return np.where(np.isnan(eo), np.inf, eo), np.where(np.isnan(el), np.inf, el)


def within(got_o, got_l, want_o, want_l, tol_o, tol_l) -> bool:
    eo, el = _errors(got_o, got_l, want_o, want_l)
    return bool(np.all(eo <= tol_o) and np.all(el <= tol_l))


def assert_within(got_o, got_l, want_o, want_l, tol_o, tol_l, what=""):
    eo, el = _errors(got_o, got_l, want_o, want_l)
    worst_o = float(np.max(eo / tol_o)) if eo.size else 0.0
    worst_l = float(np.max(el / tol_l)) if el.size else 0.0
    assert worst_o <= 1.0 and worst_l <= 1.0, (what, "error / bound", worst_o, worst_l)
    return worst_o, worst_l
