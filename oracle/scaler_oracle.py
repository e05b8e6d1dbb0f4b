"""CPU oracle of the consumers of the expert-load statistic: the coefficient of variation of
the loads, the Expert Scaling heuristic (paper, Algorithm 1 and Section 4.2) and the even
split of an expert's rows over its replicas (Section 3.3, serving step).

TEST INFRASTRUCTURE ONLY.  Slow, plain and independent of the HIP sources: tests and the
smoke check compare the library with it; the product path never imports it.

What is defined here:

  cv                 coefficient of variation of the per-replica loads of a layer.  Section 3.3
                     splits an expert's load W_e evenly over its R_e replicas (per-replica load
                     W_e / R_e); Algorithm 1 removes an expert's replica loads from the multiset
                     W_l and puts the re-split ones back, so CV is taken over that multiset
                     (sum_e R_e values).  Population form: standard deviation / mean with the
                     1/N variance; an all-zero multiset has CV 0.
  expert_scaling     Algorithm 1 in the paper's order: all experts start with one replica and no
                     extra memory allocated; while memory remains and CV exceeds the threshold V,
                     the expert whose replicas carry the largest load gets one more replica, the
                     allocated memory grows by the expert's footprint M_e, and its load is
                     re-split evenly.  Returns the replica counts and the CV after every step.
  replica_segments   the rows [offsets[e], offsets[e+1]) of expert e cut into R_e consecutive
                     pieces whose sizes differ by at most one row (Section 3.3: each expert's
                     load is distributed evenly across its replicas).

Readings of the garbled or silent points (also listed in the design notes):
  * the re-split load of the chosen expert is its ORIGINAL load divided by the new replica
    count (the listing's "w_r <- w_r / R" applied to the already split value would divide
    twice and contradict Section 3.3's W_e / R_e);
  * a replica is added only while it still fits: M_alloc + M_e <= M_cap.  For a cap that is a
    multiple of M_e this is the listing's "M_alloc < M_cap";
  * "largest load" compares per-replica loads exactly (as fractions); equal loads go to the
    lowest expert index; an expert with zero load is never split;
  * the decision CV > V is taken in fp64.

Pinned by tests/test_scaler_pins.py (hand-worked cases, closed forms, invariants, a brute-force
re-derivation on small inputs, planted mistakes); nothing here is "parity unpinned".
"""
from __future__ import annotations

from fractions import Fraction

import numpy as np


def replica_loads(loads, replicas) -> np.ndarray:
    """The multiset W_l as an fp64 array: expert e contributes R_e values W_e / R_e."""
    loads = np.asarray(loads, dtype=np.int64)
    replicas = np.asarray(replicas, dtype=np.int64)
    assert loads.shape == replicas.shape and np.all(replicas >= 1) and np.all(loads >= 0)
    per = loads.astype(np.float64) / replicas.astype(np.float64)
    return np.repeat(per, replicas)


def cv(loads, replicas=None) -> float:
    """Population coefficient of variation of the per-replica loads (0 for all-zero loads)."""
    loads = np.asarray(loads, dtype=np.int64)
    if replicas is None:
        replicas = np.ones_like(loads)
    w = replica_loads(loads, replicas)
    mean = w.mean()
    if mean == 0.0:
        return 0.0
    return float(np.sqrt(np.mean((w - mean) ** 2)) / mean)


def expert_scaling(loads, expert_mem: int, mem_cap: int, cv_threshold: float):
    """Algorithm 1.  loads: int [E] (predicted) token counts of one layer; expert_mem = M_e > 0;
    mem_cap = M_cap >= 0 (memory for ADDITIONAL replicas of this layer); cv_threshold = V.
    Returns (replicas int32 [E], cv_trace list: CV before the first step and after each step)."""
    loads = [int(v) for v in np.asarray(loads).ravel()]
    E = len(loads)
    assert E >= 1 and expert_mem > 0 and mem_cap >= 0 and all(v >= 0 for v in loads)
    replicas = [1] * E
    allocated = 0
    trace = [cv(loads, replicas)]
    while allocated + expert_mem <= mem_cap and trace[-1] > cv_threshold:
        # the straggler: the expert whose replicas carry the largest load
        best = 0
        for e in range(1, E):
            if Fraction(loads[e], replicas[e]) > Fraction(loads[best], replicas[best]):
                best = e
        if loads[best] == 0:
            break
        replicas[best] += 1
        allocated += expert_mem
        trace.append(cv(loads, replicas))
    return np.asarray(replicas, dtype=np.int32), trace


def replica_segments(offsets, replicas):
    """Row ranges of the replicas, expert-major: returns (seg_offsets int32 [S+1], seg_expert
    int32 [S]) with S = sum(replicas).  Replica r of an expert with c rows starting at row o gets
    rows [o + floor(c r / R), o + floor(c (r+1) / R))."""
    offsets = np.asarray(offsets, dtype=np.int64)
    replicas = np.asarray(replicas, dtype=np.int64)
    E = replicas.shape[0]
    assert offsets.shape[0] == E + 1 and np.all(replicas >= 1)
    seg = [int(offsets[0])]
    who = []
    for e in range(E):
        c = int(offsets[e + 1] - offsets[e])
        R = int(replicas[e])
        for r in range(R):
            seg.append(int(offsets[e]) + (c * (r + 1)) // R)
            who.append(e)
    return np.asarray(seg, dtype=np.int32), np.asarray(who, dtype=np.int32)
