"""CPU oracle of the MoE-layer forward:  y = sum_k g_k(x) * E_k(x).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of what the
HIP library computes; it exists so that tests, the smoke check and the bench's
`cpu_baseline` leg have something independent to compare with and to time.  The
product path never imports it.  It shares no code with the HIP sources.

What is defined here (paper, Section 2.2: an MoE layer is a gating network plus
E expert networks; the gate routes each token to its assigned experts; under
expert parallelism a scatter sends tokens to their experts and a gather collects
and reorders the expert outputs; Section 3.3 / 4.1: the load of expert e is the
number of tokens routed to it):

  gate_scores       logits of the bias-free linear gate (Section 5 and 6.6 give
                    the gate/predictor as a plain d x E linear map), fp64 sums,
                    rounded once to fp32
  topk_select       the k largest fp32 scores per token, ties to the lowest
                    expert index, in descending order
  routing_weights   softmax over all E scores (fp64), read at the selected
                    experts, optionally renormalised to sum to one
  expert_load       W_l = per-expert token counts, and their exclusive prefix sum
  permutation       the stable expert-contiguous order of the T*k assignments
  permute_rows      the single-GPU "scatter"
  expert_ffn        SwiGLU expert  W2 (silu(W1 x) * (W3 x)), fp64, no rounding
  grouped_ffn       the above on every expert's row segment
  combine           the single-GPU "gather": weighted sum in assignment order

All floating point is fp64 except where a value is *defined* as fp32 (the gate
score that decides the integer top-k choice, and the stored routing weights).
Every function is pinned by tests/test_oracle_pins.py against brute force,
closed forms, invariants and library routines; nothing here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np


# ----------------------------------------------------------------------------- storage
def to_f64(a: np.ndarray) -> np.ndarray:
    """Exact widening of a stored tensor (float32, or uint16 bfloat16 bits) to fp64."""
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


# ----------------------------------------------------------------------------- routing
def gate_scores(x, w_gate, gate_bias=None) -> np.ndarray:
    """score[t,e] = fp32( sum_i x[t,i] * w_gate[e,i]  (+ bias[e]) ), sums in fp64."""
    logits = to_f64(x) @ to_f64(w_gate).T
    if gate_bias is not None:
        logits = logits + gate_bias.astype(np.float64)[None, :]
    return logits.astype(np.float32)


def topk_select(score: np.ndarray, k: int) -> np.ndarray:
    """Pick k times the largest remaining fp32 score of each row; equal scores go to
    the lowest expert index.  Returns int32 [T,k] in pick order (descending score)."""
    T, E = score.shape
    assert 1 <= k <= E
    work = score.astype(np.float32).copy()
    idx = np.empty((T, k), dtype=np.int32)
    rows = np.arange(T)
    for j in range(k):
        pick = np.argmax(work, axis=1)          # first occurrence of the maximum
        idx[:, j] = pick
        work[rows, pick] = -np.inf
    return idx


def routing_weights(score: np.ndarray, idx: np.ndarray, renorm: int) -> np.ndarray:
    """w[t,j] = softmax_E(score[t,:])[idx[t,j]], divided by sum_j w[t,j] if renorm."""
    s = score.astype(np.float64)
    s = s - s.max(axis=1, keepdims=True)
    p = np.exp(s)
    p /= p.sum(axis=1, keepdims=True)
    w = np.take_along_axis(p, idx.astype(np.int64), axis=1)
    if renorm:
        w = w / w.sum(axis=1, keepdims=True)
    return w.astype(np.float32)


def route(x, w_gate, k, renorm, gate_bias=None):
    """(topk_idx int32 [T,k], topk_w float32 [T,k], score float32 [T,E])."""
    score = gate_scores(x, w_gate, gate_bias)
    idx = topk_select(score, k)
    return idx, routing_weights(score, idx, renorm), score


# ----------------------------------------------------------------------------- load + dispatch
def expert_load(idx: np.ndarray, E: int):
    """counts[e] = number of (token, slot) assignments routed to expert e;
    offsets = exclusive prefix sum with offsets[E] = T*k."""
    counts = np.zeros(E, dtype=np.int32)
    for e in idx.reshape(-1):
        counts[e] += 1
    offsets = np.zeros(E + 1, dtype=np.int32)
    for e in range(E):
        offsets[e + 1] = offsets[e] + counts[e]
    return counts, offsets


def permutation(idx: np.ndarray, E: int):
    """Stable expert-contiguous order.  Assignments a = t*k + j are visited in
    ascending a; dst_row[a] = offsets[e] + (earlier assignments of the same expert);
    src_assign is the inverse map."""
    _, offsets = expert_load(idx, E)
    flat = idx.reshape(-1)
    fill = offsets[:-1].astype(np.int64).copy()
    dst_row = np.empty(flat.size, dtype=np.int32)
    src_assign = np.empty(flat.size, dtype=np.int32)
    for a, e in enumerate(flat):
        r = fill[e]
        fill[e] += 1
        dst_row[a] = r
        src_assign[r] = a
    return dst_row, src_assign


def permute_rows(x: np.ndarray, dst_row: np.ndarray, k: int) -> np.ndarray:
    """x_perm[dst_row[a]] = x[a // k]  (a copy: storage type is kept)."""
    out = np.empty((dst_row.size, x.shape[1]), dtype=x.dtype)
    for a, r in enumerate(dst_row):
        out[r] = x[a // k]
    return out


# ----------------------------------------------------------------------------- experts
def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def expert_ffn(rows, w1_e, w3_e, w2_e, return_h=False):
    """SwiGLU expert on fp64 rows [m,d]: W2 (silu(W1 x) * (W3 x)).
    w1_e, w3_e are [F,d]; w2_e is [d,F]."""
    r = to_f64(rows)
    g = r @ to_f64(w1_e).T
    u = r @ to_f64(w3_e).T
    h = silu(g) * u
    y = h @ to_f64(w2_e).T
    return (y, h) if return_h else y


def grouped_ffn(x_perm, offsets, w1, w3, w2, return_h=False):
    """Expert e is applied to rows offsets[e] .. offsets[e+1]-1 of x_perm."""
    A = x_perm.shape[0]
    E, F, d = w1.shape
    y = np.zeros((A, d), dtype=np.float64)
    h = np.zeros((A, F), dtype=np.float64) if return_h else None
    for e in range(E):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi == lo:
            continue
        res = expert_ffn(x_perm[lo:hi], w1[e], w3[e], w2[e], return_h=return_h)
        if return_h:
            y[lo:hi], h[lo:hi] = res
        else:
            y[lo:hi] = res
    return (y, h) if return_h else y


def combine(y_perm, dst_row, topk_w) -> np.ndarray:
    """y[t] = sum_{j<k} w[t,j] * y_perm[dst_row[t*k+j]], fp64, j ascending."""
    T, k = topk_w.shape
    yp = to_f64(y_perm)
    w = topk_w.astype(np.float64)
    y = np.zeros((T, yp.shape[1]), dtype=np.float64)
    rows = dst_row.reshape(T, k)
    for j in range(k):
        y += w[:, j:j + 1] * yp[rows[:, j]]
    return y


# ----------------------------------------------------------------------------- whole layer
def moe_layer(x, w_gate, w1, w3, w2, k, renorm, gate_bias=None):
    """All steps in order; returns a dict with every intermediate."""
    E = w_gate.shape[0]
    idx, w, score = route(x, w_gate, k, renorm, gate_bias)
    counts, offsets = expert_load(idx, E)
    dst_row, src_assign = permutation(idx, E)
    x_perm = permute_rows(x, dst_row, k)
    y_perm, h = grouped_ffn(x_perm, offsets, w1, w3, w2, return_h=True)
    y = combine(y_perm, dst_row, w)
    return dict(score=score, topk_idx=idx, topk_w=w, counts=counts, offsets=offsets,
                dst_row=dst_row, src_assign=src_assign, x_perm=x_perm, h=h, y_perm=y_perm, y=y)


def topk_margin(score: np.ndarray, k: int) -> np.ndarray:
    """Per row: (k-th largest score - (k+1)-th largest) / max|score|; inf when k = E.
    Rows with a tiny margin are the ones where a differently ordered fp32 gate sum may
    legitimately pick another expert."""
    T, E = score.shape
    if k >= E:
        return np.full(T, np.inf)
    s = np.sort(score.astype(np.float64), axis=1)[:, ::-1]
    scale = np.maximum(np.abs(score).max(axis=1).astype(np.float64), 1e-30)
    return (s[:, k - 1] - s[:, k]) / scale
