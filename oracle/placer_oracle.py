"""CPU oracle of Expert Placement (paper, Algorithm 2 and Section 4.3): which GPU every expert
replica of a layer goes to, given the replica counts of Algorithm 1, the expert loads, the GPUs
and the previous placement.

TEST INFRASTRUCTURE ONLY.  Slow, plain and independent of the HIP sources; the product path
never imports it.

The algorithm, in the paper's order: all per-GPU loads start at zero; replicas are taken from
the most loaded to the least loaded (a replica of expert e carries W_e / R_e, Section 3.3); a
replica that was placed in the previous round and is still alive on a GPU stays there (warm
start); any other replica joins the GPU with the smallest aggregated load so far
(join-the-shortest-queue); the GPU's load grows by the replica's load.

Readings of the garbled or silent points (also in the design notes):
  * a replica is identified across rounds by (expert, replica index): replica r of expert e is
    warm if the previous round had more than r replicas of e and its entry names a GPU
    (an entry of -1 means that replica is no longer alive);
  * "per-GPU capacity constraints" (Section 4.3 text; the listing has none) are replica slots per
    GPU: a GPU without a free slot takes no further replica, warm or not; a replica that finds no
    GPU with a free slot stays unplaced (-1);
  * equal replica loads are taken in ascending (expert, replica) order, equal GPU loads go to the
    lowest GPU index; replicas with zero load are placed like any other;
  * GPU loads are fp64 sums of the fp64 values W_e / R_e in placement order (the comparison that
    picks the shortest queue is made on these sums).

Pinned by tests/test_placer_pins.py; nothing here is "parity unpinned".
"""
from __future__ import annotations

from fractions import Fraction

import numpy as np


def expert_placement(loads, replicas, n_gpus: int, prev_offsets=None, prev_gpu=None, gpu_slots=None):
    """Returns (gpu_of int32 [S], gpu_load float64 [G], gpu_count int32 [G], n_warm int).
    S = sum(replicas); entry s of gpu_of belongs to the s-th replica in expert-major order (the
    order of the replica segments).  prev_offsets [E+1] / prev_gpu [prev_offsets[E]]: GPU of every
    replica of the previous round, expert-major, -1 if not alive; None = no previous round.
    gpu_slots [G]: replicas each GPU can hold; None = unlimited."""
    loads = [int(v) for v in np.asarray(loads).ravel()]
    replicas = [int(v) for v in np.asarray(replicas).ravel()]
    E, G = len(loads), int(n_gpus)
    assert E >= 1 and G >= 1 and len(replicas) == E and all(r >= 1 for r in replicas)
    slots = [1 << 62] * G if gpu_slots is None else [int(v) for v in gpu_slots]
    start = np.concatenate([[0], np.cumsum(replicas)]).astype(np.int64)
    gpu_of = np.full(int(start[-1]), -1, dtype=np.int32)
    gpu_load = [0.0] * G
    gpu_count = [0] * G
    n_warm = 0
    # most loaded first; the replicas of one expert carry the same load and stay together
    order = sorted(range(E), key=lambda e: (-Fraction(max(loads[e], 0), replicas[e]), e))
    for e in order:
        w = float(max(loads[e], 0)) / float(replicas[e])
        for r in range(replicas[e]):
            g = -1
            if prev_offsets is not None and r < int(prev_offsets[e + 1]) - int(prev_offsets[e]):
                pg = int(prev_gpu[int(prev_offsets[e]) + r])
                if 0 <= pg < G and gpu_count[pg] < slots[pg]:
                    g = pg
                    n_warm += 1
            if g < 0:
                for cand in range(G):
                    if gpu_count[cand] < slots[cand] and (g < 0 or gpu_load[cand] < gpu_load[g]):
                        g = cand
            if g >= 0:
                gpu_of[start[e] + r] = g
                gpu_load[g] += w
                gpu_count[g] += 1
    return gpu_of, np.asarray(gpu_load, dtype=np.float64), np.asarray(gpu_count, dtype=np.int32), n_warm
