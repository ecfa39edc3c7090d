"""Full-sequence causal softmax attention, forward and backward, in fp64 (numpy).

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Forward follows Section 3.1, Eq. 3 of the paper: token i attends to tokens 1..i (itself included),
scores are scaled by 1/sqrt(d_k).  Eq. 3 prints the value list as starting at index 0 while the key
list starts at 1; the two lists are read as the same index set 1..i.  The paper prints no backward
formulas; the backward here is the derivative of Eq. 3, written out term by term.

Layout: q [H_q, n, D]; k, v [H_kv, n, D]; query head h reads key/value head h // (H_q // H_kv).

Segment-wise execution (Section 3.1, last paragraph; Section 3.2): a segment holding rows
[off, off+len) needs the keys/values of all tokens up to its own last token; its backward needs the
gradients of all later tokens to have been accumulated first.  `segment_forward` / `segment_backward`
are the same definition restricted to those rows; the paper's claim is that running them over all
segments (forward in order, backward in reverse, accumulating dK/dV) reproduces the full result.
"""
from __future__ import annotations

import numpy as np


def _group(h: int, n_q_heads: int, n_kv_heads: int) -> int:
    assert n_q_heads % n_kv_heads == 0
    return h // (n_q_heads // n_kv_heads)


def _probabilities(q_rows: np.ndarray, k: np.ndarray, first_row: int):
    """Scaled causal scores and softmax for query rows first_row.. of one head.

    q_rows [m, D], k [c, D] with c >= first_row + m.  Row r (absolute index first_row + r, 0-based)
    sees keys 0..first_row+r.  Returns (p [m, c], lse [m]).
    """
    m, d = q_rows.shape
    c = k.shape[0]
    s = (q_rows @ k.T) / np.sqrt(float(d))
    rows = first_row + np.arange(m)[:, None]
    cols = np.arange(c)[None, :]
    s = np.where(cols <= rows, s, -np.inf)
    mx = s.max(axis=1, keepdims=True)
    e = np.exp(s - mx)
    l = e.sum(axis=1, keepdims=True)
    p = e / l
    lse = (mx + np.log(l))[:, 0]
    return p, lse


def segment_forward(q_seg, k_prefix, v_prefix, seg_off: int):
    """Outputs of the rows of one segment.

    q_seg [H_q, len, D] are the queries of absolute rows seg_off..seg_off+len-1; k_prefix, v_prefix
    [H_kv, c, D] with c >= seg_off + len hold all keys/values up to the segment's last token.
    Returns (out [H_q, len, D], lse [H_q, len]) in fp64.
    """
    q_seg = np.asarray(q_seg, dtype=np.float64)
    k_prefix = np.asarray(k_prefix, dtype=np.float64)
    v_prefix = np.asarray(v_prefix, dtype=np.float64)
    hq, m, d = q_seg.shape
    hkv = k_prefix.shape[0]
    c = seg_off + m
    out = np.empty((hq, m, d))
    lse = np.empty((hq, m))
    for h in range(hq):
        g = _group(h, hq, hkv)
        p, lse[h] = _probabilities(q_seg[h], k_prefix[g, :c], seg_off)
        out[h] = p @ v_prefix[g, :c]
    return out, lse


def segment_backward(dout_seg, q_seg, k_prefix, v_prefix, seg_off: int):
    """Gradient contributions of one segment's rows.

    With L = sum(dout * out) over the segment's rows:
      delta_i = dout_i . out_i
      dp_ij   = dout_i . v_j
      ds_ij   = p_ij (dp_ij - delta_i)
      dq_i    = (1/sqrt D) sum_j ds_ij k_j
      dk_j    = (1/sqrt D) sum_{heads in group} sum_i ds_ij q_i     (this segment's rows only)
      dv_j    =            sum_{heads in group} sum_i p_ij dout_i
    Returns (dq [H_q, len, D], dk [H_kv, c, D], dv [H_kv, c, D]) with c = seg_off + len.
    """
    dout_seg = np.asarray(dout_seg, dtype=np.float64)
    q_seg = np.asarray(q_seg, dtype=np.float64)
    k_prefix = np.asarray(k_prefix, dtype=np.float64)
    v_prefix = np.asarray(v_prefix, dtype=np.float64)
    hq, m, d = q_seg.shape
    hkv = k_prefix.shape[0]
    c = seg_off + m
    scale = 1.0 / np.sqrt(float(d))
    dq = np.empty((hq, m, d))
    dk = np.zeros((hkv, c, d))
    dv = np.zeros((hkv, c, d))
    for h in range(hq):
        g = _group(h, hq, hkv)
        kk, vv = k_prefix[g, :c], v_prefix[g, :c]
        p, _ = _probabilities(q_seg[h], kk, seg_off)
        out = p @ vv
        delta = (dout_seg[h] * out).sum(axis=1, keepdims=True)
        dp = dout_seg[h] @ vv.T
        ds = p * (dp - delta)
        dq[h] = scale * (ds @ kk)
        dk[g] += scale * (ds.T @ q_seg[h])
        dv[g] += p.T @ dout_seg[h]
    return dq, dk, dv


def full_forward(q, k, v):
    """Eq. 3 on the whole sequence: (out [H_q, n, D], lse [H_q, n])."""
    return segment_forward(q, k, v, 0)


def full_backward(dout, q, k, v):
    """Gradients of sum(dout * out) for the whole sequence: (dq, dk, dv)."""
    return segment_backward(dout, q, k, v, 0)


def segmented_schedule(q, k, v, dout, boundaries):
    """Run the paper's order of execution on one stage: forward of segments 1..k in order, then
    backward k..1, accumulating dK/dV over the prefix (Section 3.1 order constraint, Section 3.2).

    Returns (out, lse, dq, dk_acc, dv_acc, trace) where trace[i] holds copies of the accumulators
    taken right after the backward of segment i (0-based), for checking that rows of segment i are
    final at that point.
    """
    q = np.asarray(q, dtype=np.float64)
    hq, n, d = q.shape
    hkv = np.asarray(k).shape[0]
    nseg = len(boundaries) - 1
    assert boundaries[0] == 0 and boundaries[-1] == n
    out = np.empty((hq, n, d))
    lse = np.empty((hq, n))
    for i in range(nseg):
        a, b = boundaries[i], boundaries[i + 1]
        out[:, a:b], lse[:, a:b] = segment_forward(q[:, a:b], np.asarray(k)[:, :b], np.asarray(v)[:, :b], a)
    dq = np.empty((hq, n, d))
    dk_acc = np.zeros((hkv, n, d))
    dv_acc = np.zeros((hkv, n, d))
    trace = {}
    for i in reversed(range(nseg)):
        a, b = boundaries[i], boundaries[i + 1]
        dq[:, a:b], dk_i, dv_i = segment_backward(np.asarray(dout)[:, a:b], q[:, a:b],
                                                  np.asarray(k)[:, :b], np.asarray(v)[:, :b], a)
        dk_acc[:, :b] += dk_i
        dv_acc[:, :b] += dv_i
        trace[i] = (dk_acc.copy(), dv_acc.copy())
    return out, lse, dq, dk_acc, dv_acc, trace
