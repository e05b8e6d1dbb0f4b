"""Expert-parallel latency model on one GPU (paper, Section 4.3: a layer's latency is that of its
most loaded GPU).

The grouped FFN of every simulated GPU ("rank") runs alone, one rank after the other, on the rows
that rank would receive: under the static placement of plain expert parallelism (expert e on GPU
e // (E / G), one replica each), or under the replica counts of Algorithm 1 and the placement of
Algorithm 2 (moe_scale_replicas, moe_replica_segments, moe_place_replicas).  What is reported is
each rank's FFN time, and the maximum over ranks; the all-to-all that would move the rows is not
part of this (one GPU, no collectives).  The rows every rank computes are checked against the
un-sharded call: an output row does not depend on which tile, call or rank computes it.

Index bookkeeping (which rows go to which rank) is done on the host from the small tables the
device calls produce; every FFN row is computed by the library's kernels.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B


def static_shares(offsets: np.ndarray, E: int, G: int):
    """Plain expert parallelism: rank g hosts experts [g*E/G, (g+1)*E/G).  Returns, per rank,
    (hosted expert ids, row index array, local offsets [len(hosted)+1])."""
    if E % G:
        raise ValueError("static placement needs E divisible by the number of GPUs")
    per = E // G
    shares = []
    for g in range(G):
        hosted = np.arange(g * per, (g + 1) * per, dtype=np.int64)
        lo, hi = int(offsets[g * per]), int(offsets[(g + 1) * per])
        rows = np.arange(lo, hi, dtype=np.int64)
        local = (offsets[g * per:(g + 1) * per + 1] - lo).astype(np.int32)
        shares.append((hosted, rows, local))
    return shares


def placed_shares(seg_offsets: np.ndarray, seg_expert: np.ndarray, gpu_of: np.ndarray,
                  n_segments: int, G: int):
    """Shares under a replica placement: segment s (rows [seg_offsets[s], seg_offsets[s+1]) of the
    permuted order, expert seg_expert[s]) goes to rank gpu_of[s].  Replicas of one expert that land
    on the same rank form one local segment, in row order."""
    shares = []
    for g in range(G):
        mine = [s for s in range(n_segments) if int(gpu_of[s]) == g]
        hosted = sorted({int(seg_expert[s]) for s in mine})
        rows, local = [], [0]
        for e in hosted:
            n = 0
            for s in mine:                       # ascending s = ascending rows within an expert
                if int(seg_expert[s]) == e:
                    lo, hi = int(seg_offsets[s]), int(seg_offsets[s + 1])
                    rows.append(np.arange(lo, hi, dtype=np.int64))
                    n += hi - lo
            local.append(local[-1] + n)
        rows = np.concatenate(rows) if rows else np.zeros((0,), np.int64)
        shares.append((np.asarray(hosted, np.int64), rows, np.asarray(local, np.int32)))
    return shares


def check_partition(shares, A: int):
    """Every row of the permuted order belongs to exactly one rank."""
    seen = np.zeros((A,), np.int32)
    for _, rows, local in shares:
        seen[rows] += 1
        if int(local[-1]) != rows.size:
            raise AssertionError("local offsets do not cover the rank's rows")
    if not (seen == 1).all():
        raise AssertionError("the shares are not a partition of the rows")


def run_shares(shares, x_perm, w1, w3, w2, d, F, dtype, iters=10, y_full=None, stream=None):
    """Runs moe_grouped_ffn for every rank's share, alone, and times it.  Returns a list of
    dicts (rows, experts, ms).  If y_full ([A, d], the un-sharded call's output rows) is given,
    asserts that every rank reproduces its rows bit for bit."""
    st = torch.cuda.current_stream() if stream is None else stream
    out = []
    for hosted, rows, local in shares:
        n = int(rows.size)
        if n == 0:
            out.append({"rows": 0, "experts": int(hosted.size), "ms": 0.0})
            continue
        idx = torch.from_numpy(rows).to(x_perm.device)
        x_g = x_perm.index_select(0, idx)
        hosted_t = torch.from_numpy(hosted).to(x_perm.device)
        contiguous = hosted.size > 0 and int(hosted[-1] - hosted[0]) + 1 == hosted.size
        if contiguous:                          # a slice of the weights, no copy
            lo, hi = int(hosted[0]), int(hosted[-1]) + 1
            w1_g, w3_g, w2_g = w1[lo:hi], w3[lo:hi], w2[lo:hi]
        else:                                   # the rank's replicas, as its own memory would hold them
            w1_g, w3_g, w2_g = (w.index_select(0, hosted_t) for w in (w1, w3, w2))
        off_g = torch.from_numpy(local).to(x_perm.device)
        sh = B.make_shape(n, d, int(hosted.size), 1, F, dtype, 1)
        h_g = torch.empty((n, F), dtype=x_perm.dtype, device=x_perm.device)
        y_g = torch.empty((n, d), dtype=x_perm.dtype, device=x_perm.device)

        def call():
            B.moe_grouped_ffn(sh, x_g, off_g, w1_g, w3_g, w2_g, h_g, y_g, st)

        for _ in range(2):
            call()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record(st)
        for _ in range(iters):
            call()
        e1.record(st)
        torch.cuda.synchronize()
        if y_full is not None and not torch.equal(y_g, y_full.index_select(0, idx)):
            raise AssertionError("a rank's rows differ from the un-sharded call's")
        out.append({"rows": n, "experts": int(hosted.size), "ms": e0.elapsed_time(e1) / iters})
        del x_g, h_g, y_g, w1_g, w3_g, w2_g
    return out


def simulate(buf, x, w1, w3, w2, G, cv_threshold=0.2, max_extra=None, iters=10, check=True):
    """buf: a layer.MoeBuffers on which route and moe_count_and_permute (with x_perm) have run.
    Returns the per-rank FFN times under static expert parallelism and under Algorithms 1 + 2."""
    E, d, F, A = buf.E, buf.d, buf.F, buf.T * buf.k
    dtype = buf.shape.dtype
    st = torch.cuda.current_stream()
    y_full = None
    if check:
        B.moe_grouped_ffn(buf.shape, buf.x_perm, buf.offsets, w1, w3, w2, buf.h, buf.y_perm, st)
        torch.cuda.synchronize()
        y_full = buf.y_perm
    offsets = buf.offsets.cpu().numpy()
    static = static_shares(offsets, E, G)
    check_partition(static, A)
    res_static = run_shares(static, buf.x_perm, w1, w3, w2, d, F, dtype, iters, y_full)

    max_extra = E if max_extra is None else int(max_extra)
    max_seg = E + max_extra
    dev = dict(device=buf.x_perm.device)
    replicas = torch.empty((E,), dtype=torch.int32, **dev)
    cv = torch.empty((2,), dtype=torch.float64, **dev)
    seg_offsets = torch.empty((max_seg + 1,), dtype=torch.int32, **dev)
    seg_expert = torch.empty((max_seg,), dtype=torch.int32, **dev)
    n_seg = torch.empty((1,), dtype=torch.int32, **dev)
    gpu_of = torch.full((max_seg,), -1, dtype=torch.int32, **dev)
    gpu_load = torch.empty((G,), dtype=torch.float64, **dev)
    gpu_count = torch.empty((G,), dtype=torch.int32, **dev)
    n_warm = torch.empty((1,), dtype=torch.int32, **dev)
    B.moe_scale_replicas(E, buf.counts, 1, max_extra, cv_threshold, replicas, cv, st)
    B.moe_replica_segments(E, buf.offsets, replicas, max_seg, seg_offsets, seg_expert, n_seg, st)
    B.moe_place_replicas(E, buf.counts, replicas, G, None, None, None, max_seg, gpu_of, gpu_load,
                         gpu_count, n_warm, st)
    torch.cuda.synchronize()
    S = int(n_seg.item())
    placed = placed_shares(seg_offsets.cpu().numpy(), seg_expert.cpu().numpy(),
                           gpu_of.cpu().numpy(), S, G)
    check_partition(placed, A)
    res_placed = run_shares(placed, buf.x_perm, w1, w3, w2, d, F, dtype, iters, y_full)

    def summary(res):
        ms = [r["ms"] for r in res]
        return {"rows_per_rank": [r["rows"] for r in res],
                "experts_per_rank": [r["experts"] for r in res],
                "ffn_ms_per_rank": ms, "max_ms": max(ms), "mean_ms": sum(ms) / len(ms)}

    s_static, s_placed = summary(res_static), summary(res_placed)
    cvs = [float(v) for v in cv.cpu()]
    return {
        "n_gpus": G,
        "static_expert_parallel": s_static,
        "scaled_and_placed": s_placed,
        "replicas_total": int(replicas.sum().item()), "segments": S,
        "cv_of_per_replica_loads": {"before": cvs[0], "after": cvs[1], "threshold": cv_threshold},
        "straggler_ffn_time_ratio": s_placed["max_ms"] / s_static["max_ms"],
        "rows_checked_against_unsharded_call": bool(check),
    }
