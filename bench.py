#!/usr/bin/env python3
"""MoE-layer forward benchmark on one MI355X.

A step is one pass of the whole hot path (moe_route -> moe_count_and_permute ->
moe_grouped_ffn_gather -> moe_combine; with --materialize-x-perm the four-call form
with moe_grouped_ffn on a written x_perm) over one seeded synthetic batch that is
already resident in HBM.  Prints ONE JSON line: whole-layer tokens/s, per-call times, the
roofline of the dominant kernel (the gated up-projection GEMM of the grouped FFN)
and the CPU oracle timed on the host cores on a bounded sample of the same batch.

usage: python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload mixtral]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_MFMA_TFLOPS = 2500.0   # MI355X dense bf16
PEAK_HBM_GBS = 8000.0            # MI355X HBM3E

# HBM-bound calls at a batch where bandwidth, not launch latency, decides: T tokens of the Mixtral
# hidden size and routing fan-out (x is 512 MiB, x_perm and y_perm 1 GiB each, so every call
# streams far more than the 256 MB last-level cache holds; two buffer sets alternate on top)
HBM_BOUND_SHAPE = dict(T=65536, d=4096, E=8, k=2)
HBM_BOUND_ITERS = 200


def algorithmic_work(cfg):
    """Algorithmic bytes / flops of one launch of each call (per-unit figures x units)."""
    T, d, E, k, F, b = cfg.T, cfg.d, cfg.E, cfg.k, cfg.F, cfg.itemsize
    A = T * k
    return {
        "route_bytes": T * d * b + E * d * b + 8 * A,
        "permute_bytes": T * d * b + A * d * b + 4 * A + 8 * A + 8 * E,
        "permute_maps_only_bytes": 4 * A + 8 * A + 8 * E,
        "ffn_up_flops": 4 * d * F * A,        # two d x F products per routed row
        # W1 and W3 of every expert once, the activation rows once, h written once
        "ffn_up_bytes": 2 * E * d * F * b + A * d * b + A * F * b,
        "ffn_down_flops": 2 * d * F * A,
        "combine_bytes": A * d * b + T * d * b + 8 * A,
    }


def cpu_baseline(cfg, L, n_tokens):
    """The oracle, as it stands, on the first n_tokens tokens of the batch (all experts' weights)."""
    from oracle import moe_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    t0 = time.perf_counter()
    orc.moe_layer(L["x"][:n_tokens], L["w_gate"], L["w1"], L["w3"], L["w2"], cfg.k, cfg.renorm,
                  L["gate_bias"])
    dt = time.perf_counter() - t0
    which = "the whole batch" if n_tokens == cfg.T else f"first {n_tokens} of {cfg.T} tokens"
    return {"value": n_tokens / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{which} ({n_tokens} tokens) through the full layer (all {cfg.E} "
                      f"experts' weights, fp64), {dt:.1f} s wall"}


def measured_hbm_traffic(cfg_name, entry_point):
    """HBM bytes of one launch of the dominant call from the rocprofv3 --pmc summary under profiles/
    (FETCH_SIZE and WRITE_SIZE runs of this script, each scaled by what the counter reads for the
    1 GiB calibration copy).  The summary names the workload, the entry point and the SHA-256 of
    csrc/ffn.hip it was taken with; a figure taken with another kernel source, another entry point
    or another workload is not reported (None)."""
    import hashlib
    import re
    path = os.path.join(ROOT, "profiles", f"{cfg_name}_ffn_up_hbm_traffic.md")
    if not os.path.exists(path):
        return None
    fields = dict(re.findall(r"^([a-z_0-9]+):\s*(\S+)\s*$", open(path).read(), flags=re.M))
    src = os.path.join(ROOT, "paper_2603_06350_amd", "csrc", "ffn.hip")
    sha = hashlib.sha256(open(src, "rb").read()).hexdigest()
    if fields.get("ffn_hip_sha256") != sha or fields.get("entry_point") != entry_point or \
            fields.get("workload") != cfg_name:
        return None
    return {"read_bytes": float(fields["hbm_read_bytes"]), "written_bytes": float(fields["hbm_written_bytes"]),
            "source": os.path.relpath(path, ROOT)}


def achievable_peaks():
    """What the box itself sustains on the two rooflines, from the stand-alone micro-benchmarks under
    csrc/microbench, each run in a fresh child process after the timed region: back-to-back
    independent v_mfma_f32_16x16x32_bf16 on random operands held in registers (no memory traffic),
    a read-only stream over 4 GiB of HBM, and the up-projection's operand tiles streamed L2 -> LDS
    with no arithmetic.  Context for the published peaks the roofline fractions are priced against;
    None for a program that is not built."""
    import re
    import subprocess
    mb = os.path.join(ROOT, "paper_2603_06350_amd", "csrc", "microbench")

    def run(name, unit, pick):
        exe = os.path.join(mb, name + ".exe")
        if not os.path.exists(exe):
            return None
        try:
            txt = subprocess.run([exe], capture_output=True, text=True, timeout=120).stdout
        except (OSError, subprocess.TimeoutExpired):
            return None
        vals = [float(m.group(1)) for line in txt.splitlines() if pick in line
                for m in [re.search(r"([0-9.]+) " + unit, line)] if m]
        return max(vals) if vals else None

    mfma = run("mfma_rate", "TFLOP/s", "16x16x32")
    hbm = run("hbm_read_stream", "TB/s", "contiguous")
    l2 = run("l2_to_lds_stream", "TB/s", "buffer_load")
    return {"mfma_bf16_16x16x32_tflops": mfma,
            "mfma_frac_of_published_peak": None if mfma is None else mfma / PEAK_BF16_MFMA_TFLOPS,
            "hbm_read_stream_gbs": None if hbm is None else hbm * 1e3,
            "hbm_frac_of_published_peak": None if hbm is None else hbm * 1e3 / PEAK_HBM_GBS,
            "l2_to_lds_operand_stream_gbs": None if l2 is None else l2 * 1e3,
            "source": "paper_2603_06350_amd/csrc/microbench/{mfma_rate,hbm_read_stream,l2_to_lds_stream}.exe, "
                      "best line of each, child processes after the timed region"}


def vendor_dense_gemm(torch, cfg, x, w1, w2):
    """Context, not part of the path: the vendor library's dense GEMM (torch.matmul, hipBLASLt on
    ROCm) on the dense equivalents of the two projections (all A = T*k rows against one expert's
    [W1;W3] and W2, the same flops as the grouped calls) with operands of the workload's own value
    distributions (the figure depends on them: all-zero operands run about a third faster on this
    chip), and the same contractions on all-zero operands.  After the timed region."""
    A = cfg.T * cfg.k
    rows = x[torch.arange(A, device="cuda") % cfg.T]
    w13 = torch.cat([w1[0], w1[0]], dim=0)            # [2F, d]
    h = torch.randn((A, cfg.F), device="cuda", dtype=torch.float32).mul_(0.5).to(rows.dtype)
    out = {}
    for name, a, b in (("up", rows, w13), ("down", h, w2[0])):
        for kind in ("workload_values", "zeros"):
            aa, bb = (a, b) if kind == "workload_values" else (torch.zeros_like(a), torch.zeros_like(b))
            f = lambda: torch.matmul(aa, bb.t())
            for _ in range(3):
                f()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(10):
                f()
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / 10
            out[f"{name}_{kind}_tflops"] = 2.0 * aa.shape[0] * bb.shape[0] * aa.shape[1] / (ms * 1e-3) / 1e12
    out["shapes"] = f"up [{A} x {cfg.d}] x [{cfg.d} x {2 * cfg.F}], down [{A} x {cfg.F}] x [{cfg.F} x {cfg.d}]"
    return out


def calibration_copy(torch):
    """One plain copy kernel of known size (1 GiB read + 1 GiB written) so that a profiler's HBM
    byte counters can be scaled against a known quantity.  Outside every timed region."""
    calib_src = torch.ones((512 << 20,), dtype=torch.bfloat16, device="cuda")
    calib_dst = torch.empty_like(calib_src)
    torch.mul(calib_src, 1, out=calib_dst)
    torch.cuda.synchronize()


def hbm_bound_calls(torch, si, B, layer, st):
    """moe_route, moe_count_and_permute (with the row copy) and moe_combine at a bandwidth-bound
    batch: average time of HBM_BOUND_ITERS launches each (HIP events on the launch stream), two
    buffer sets alternating, algorithmic bytes / time against the HBM peak."""
    T, d, E, k = (HBM_BOUND_SHAPE[n] for n in "TdEk")
    cfg = si.small_config("hbm_bound", T=T, d=d, E=E, k=k, F=64, dtype=si.BF16, renorm=1, seed=8008)
    L = si.make_layer(cfg, parts=("x", "w_gate"))
    wg = layer.to_device(L["w_gate"])
    sh = B.make_shape(T, d, E, k, 64, B.MOE_BF16, 1)
    A = T * k
    ws_bytes = B.moe_workspace_bytes(sh)
    sets = []
    for _ in range(2):
        kw = dict(device="cuda")
        sets.append(dict(
            x=layer.to_device(L["x"]),
            topk_idx=torch.empty((T, k), dtype=torch.int32, **kw),
            topk_w=torch.empty((T, k), dtype=torch.float32, **kw),
            counts=torch.empty((E,), dtype=torch.int32, **kw),
            offsets=torch.empty((E + 1,), dtype=torch.int32, **kw),
            dst_row=torch.empty((A,), dtype=torch.int32, **kw),
            src_assign=torch.empty((A,), dtype=torch.int32, **kw),
            x_perm=torch.empty((A, d), dtype=torch.bfloat16, **kw),
            y=torch.empty((T, d), dtype=torch.bfloat16, **kw),
            ws=torch.empty((ws_bytes,), dtype=torch.uint8, **kw)))
    del L

    def route(b):
        B.moe_route_ws(sh, b["x"], wg, None, b["topk_idx"], b["topk_w"], None, b["ws"], ws_bytes, st)

    def permute(b):
        B.moe_count_and_permute(sh, b["x"], b["topk_idx"], b["counts"], b["offsets"], b["dst_row"],
                                b["src_assign"], b["x_perm"], b["ws"], ws_bytes, st)

    def combine(b):       # the permuted activations stand in for the expert outputs: same bytes moved
        B.moe_combine(sh, b["x_perm"], b["dst_row"], b["topk_w"], b["y"], st)

    b = 2  # bytes per element
    work = {"route": T * d * b + E * d * b + 8 * A,
            "count_and_permute": T * d * b + A * d * b + 4 * A + 8 * A + 8 * E,
            "combine": A * d * b + T * d * b + 8 * A}
    out = {"shape": f"T={T} d={d} E={E} k={k} bf16", "iterations": HBM_BOUND_ITERS,
           "buffer_sets": len(sets), "hbm_peak_gbs": PEAK_HBM_GBS}
    def plain_copy(b):    # context: what the box gives a copy of x (a PyTorch kernel, not part of the path)
        b["y"].copy_(b["x"])

    work["plain_copy_of_x"] = 2 * T * d * b
    for name, fn in (("route", route), ("count_and_permute", permute), ("combine", combine),
                     ("plain_copy_of_x", plain_copy)):
        for bset in sets:
            fn(bset)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record(st)
        for it in range(HBM_BOUND_ITERS):
            fn(sets[it & 1])
        e1.record(st)
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / HBM_BOUND_ITERS * 1e3
        gbs = work[name] / (us * 1e-6) / 1e9
        out[name] = {"us": us, "algorithmic_bytes": work[name], "gbs": gbs, "frac_of_hbm_peak": gbs / PEAK_HBM_GBS}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="mixtral")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--materialize-x-perm", action="store_true",
                    help="write the permuted activations and run the FFN on them (the four-call form); "
                         "default: the up-projection reads x through the permutation map")
    ap.add_argument("--ep-sim", type=int, default=0, metavar="G",
                    help="also report the expert-parallel latency model for G simulated GPUs: every "
                         "rank's grouped FFN run alone, static placement against Algorithms 1 + 2")
    ap.add_argument("--predictor-accuracy", action="store_true",
                    help="also report how the loads predicted from x match those the same gate gives "
                         "on x + eps * noise (a residual-stream stand-in), for several eps")
    ap.add_argument("--tokens", type=int, default=0, metavar="T",
                    help="run the workload's layer on a batch of T tokens instead of its own size "
                         "(same seeds and shapes otherwise; the JSON line names the batch)")
    ap.add_argument("--ffn-split", action="store_true",
                    help="give the grouped FFN the workspace that lets it cut the tiles of an under-filled "
                         "last round along K (moe_grouped_ffn_ws)")
    ap.add_argument("--no-hbm-bound", action="store_true",
                    help="skip the timings of route / count+permute / combine at the bandwidth-bound batch")
    ap.add_argument("--hbm-bound-only", action="store_true",
                    help="time only route / count+permute / combine at the bandwidth-bound batch and "
                         "print that object (for a profile of those kernels alone)")
    ap.add_argument("--no-achievable-peaks", action="store_true",
                    help="skip the micro-benchmarks that measure what the box sustains on MFMA and HBM, "
                         "and the vendor library's dense GEMM on the same flops")
    ap.add_argument("--no-consumers", action="store_true",
                    help="skip the timings of the load-statistic consumers (scaler, predictor)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py measures one GPU: this build has no sharded path (one process, one "
              "MI355X); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import synth_inputs as si
    from paper_2603_06350_amd import binding as B
    from paper_2603_06350_amd import layer

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    B.load()
    if args.hbm_bound_only:
        calibration_copy(torch)
        print(json.dumps({"hbm_bound_calls": hbm_bound_calls(torch, si, B, layer, torch.cuda.current_stream())}))
        return
    cfg = si.CONFIGS[args.workload]
    if args.tokens > 0 and args.tokens != cfg.T:
        import dataclasses
        cfg = dataclasses.replace(cfg, name=f"{cfg.name}@T={args.tokens}", T=args.tokens)
    L = si.make_layer(cfg)
    x, wg, w1, w3, w2 = (layer.to_device(L[n]) for n in ("x", "w_gate", "w1", "w3", "w2"))
    bias = layer.to_device(L["gate_bias"])
    buf = layer.MoeBuffers(cfg.T, cfg.d, cfg.E, cfg.k, cfg.F, cfg.dtype, cfg.renorm,
                           split_tiles=args.ffn_split)
    st = torch.cuda.current_stream()
    sh = buf.shape

    def ffn_entry(fused):
        return ("moe_grouped_ffn_ws" if args.ffn_split else
                "moe_grouped_ffn_gather" if fused else "moe_grouped_ffn")

    def make_calls(fused, combine_in_ffn=False):
        def call_route():
            B.moe_route_ws(sh, x, wg, bias, buf.topk_idx, buf.topk_w, None, buf.workspace, buf.ws_bytes, st)

        def call_permute():
            B.moe_count_and_permute(sh, x, buf.topk_idx, buf.counts, buf.offsets, buf.dst_row,
                                    buf.src_assign, None if fused else buf.x_perm, buf.workspace,
                                    buf.ws_bytes, st)

        def call_ffn(part=None):
            if combine_in_ffn:
                if part in (None, 2):      # (its two GEMMs cannot be called apart: timed as the down call)
                    B.moe_grouped_ffn_combine_k1(sh, x, buf.src_assign, buf.offsets, w1, w3, w2, buf.topk_w,
                                                 buf.h, buf.y, st)
            elif args.ffn_split:
                B.moe_grouped_ffn_ws(sh, x if fused else buf.x_perm, buf.src_assign if fused else None,
                                     buf.offsets, w1, w3, w2, buf.h, buf.y_perm, 3 if part is None else part,
                                     buf.ffn_ws, buf.ffn_ws_bytes, st)
            elif fused and part is None:
                B.moe_grouped_ffn_gather(sh, x, buf.src_assign, buf.offsets, w1, w3, w2, buf.h, buf.y_perm, st)
            elif fused:
                B.moe_grouped_ffn_gather_part(sh, x, buf.src_assign, buf.offsets, w1, w3, w2, buf.h,
                                              buf.y_perm, part, st)
            elif part is None:
                B.moe_grouped_ffn(sh, buf.x_perm, buf.offsets, w1, w3, w2, buf.h, buf.y_perm, st)
            else:
                B.moe_grouped_ffn_part(sh, buf.x_perm, buf.offsets, w1, w3, w2, buf.h, buf.y_perm, part, st)

        def call_combine():
            if not combine_in_ffn:
                B.moe_combine(sh, buf.y_perm, buf.dst_row, buf.topk_w, buf.y, st)

        return call_route, call_permute, call_ffn, call_combine

    def time_form(fused, warmup, steps, combine_in_ffn=False):
        """ms per step of the whole path (wall clock around `steps` steps), and the average, minimum and
        median duration of every call from HIP events recorded on the launch stream."""
        call_route, call_permute, call_ffn, call_combine = make_calls(fused, combine_in_ffn)
        for _ in range(warmup):
            call_route(), call_permute(), call_ffn(), call_combine()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            call_route(), call_permute(), call_ffn(), call_combine()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        # (torch events record on the current stream, which is the stream every call is given)
        names = ["route", "count_and_permute", "ffn_up", "ffn_down", "combine"]
        fns = [call_route, call_permute, lambda: call_ffn(1), lambda: call_ffn(2), call_combine]
        n_ev = min(steps, 50)
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(len(names) + 1)] for _ in range(n_ev)]
        for it in range(n_ev):
            evs[it][0].record(st)
            for i, fn in enumerate(fns):
                fn()
                evs[it][i + 1].record(st)
        torch.cuda.synchronize()
        samples = {n: sorted(evs[it][i].elapsed_time(evs[it][i + 1]) for it in range(n_ev))
                   for i, n in enumerate(names)}
        return ms, {"avg": {n: sum(v) / len(v) for n, v in samples.items()},
                    "min": {n: v[0] for n, v in samples.items()},
                    "median": {n: v[len(v) // 2] for n, v in samples.items()}}

    fused = not args.materialize_x_perm

    def step():
        for fn in make_calls(fused):
            fn()

    calibration_copy(torch)

    ms_per_step, calls = time_form(fused, args.warmup, args.steps)
    per_call_ms, per_call_ms_min, per_call_ms_median = calls["avg"], calls["min"], calls["median"]
    # the boundary's four calls with a written x_perm (moe_grouped_ffn on it), timed the same way
    four_call = None
    if fused and not args.ffn_split:
        ms4, calls4 = time_form(False, min(args.warmup, 5), args.steps)
        four_call = {"ms_per_step": ms4, "tokens_per_s": cfg.T / (ms4 * 1e-3), "per_call_ms": calls4["avg"],
                     "calls": "moe_route_ws, moe_count_and_permute (maps + x_perm rows), moe_grouped_ffn, "
                              "moe_combine"}
        if cfg.dtype == si.BF16:
            w4 = algorithmic_work(cfg)
            four_call["ffn_pct_of_bf16_mfma_peak"] = 100.0 * (w4["ffn_up_flops"] + w4["ffn_down_flops"]) / (
                (calls4["avg"]["ffn_up"] + calls4["avg"]["ffn_down"]) * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS

    # layers with one expert per token: the combine folded into the down-projection's store
    k1_form = None
    if cfg.k == 1 and cfg.dtype == si.BF16 and not args.ffn_split:
        ms1, calls1 = time_form(True, min(args.warmup, 5), args.steps, combine_in_ffn=True)
        k1_form = {"ms_per_step": ms1, "tokens_per_s": cfg.T / (ms1 * 1e-3),
                   "grouped_ffn_and_combine_ms": calls1["avg"]["ffn_down"],
                   "calls": "moe_route_ws, moe_count_and_permute (maps only), moe_grouped_ffn_combine_k1"}

    # Consumers of the load statistic (not part of the step): Algorithm 1 on the layer's own counts,
    # and a speculative predictor pass (a second gate matrix on the same x) on a side stream.
    consumers = None
    if not args.no_consumers:
        pred = layer.LoadPredictor(cfg.T, cfg.d, cfg.E, cfg.k, cfg.dtype, cfg.renorm,
                                   max_extra_replicas=cfg.E, n_gpus=8)
        w_pred = layer.to_device(si.make_layer(
            si.small_config("predictor_gate", T=cfg.T, d=cfg.d, E=cfg.E, k=cfg.k, F=cfg.F,
                            dtype=cfg.dtype, renorm=cfg.renorm, seed=cfg.seed + 1),
            parts=("w_gate",))["w_gate"])
        rep = torch.empty((cfg.E,), dtype=torch.int32, device="cuda")
        cvs = torch.empty((2,), dtype=torch.float64, device="cuda")
        n_it = 200

        def timed(fn):
            for _ in range(5):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record(st)
            for _ in range(n_it):
                fn()
            e1.record(st)
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / n_it * 1e3

        scale_us = timed(lambda: (
            B.moe_scale_replicas(cfg.E, buf.counts, 1, cfg.E, 0.2, rep, cvs, st),
            B.moe_replica_segments(cfg.E, buf.offsets, rep, pred.max_segments, pred.seg_offsets,
                                   pred.seg_expert, pred.n_segments, st)))
        cv_before, cv_after = (float(v) for v in cvs.cpu())
        extra = int(rep.sum().item()) - cfg.E
        pred_us = timed(lambda: pred.enqueue(x, w_pred, None, 0.2, st))
        side = torch.cuda.Stream()
        fork = torch.cuda.Event()

        def step_with_predictor():
            fork.record(st)
            side.wait_event(fork)
            pred.enqueue(x, w_pred, None, 0.2, side)
            step()
            st.wait_stream(side)

        for _ in range(3):
            step_with_predictor()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(args.steps):
            step_with_predictor()
        torch.cuda.synchronize()
        ms_with = (time.perf_counter() - t1) * 1e3 / args.steps
        consumers = {
            "scale_and_segments_us": scale_us,
            "scaling": {"M_e": 1, "M_cap": cfg.E, "V": 0.2, "cv_before": cv_before,
                        "cv_after": cv_after, "extra_replicas": extra},
            "predictor_pass_us": pred_us,
            "predictor_pass": "moe_route with a second seeded gate matrix + counts + Algorithm 1 + "
                              "replica segments + Algorithm 2 for 8 GPUs, alone on the stream",
            "ms_per_step_with_predictor_on_side_stream": ms_with,
            "added_ms_per_step": ms_with - ms_per_step,
            "paper_prediction_delay_ms": "< 0.2 per layer (Section 6.6, other hardware)",
        }

    work = algorithmic_work(cfg)
    up_s = per_call_ms["ffn_up"] * 1e-3
    achieved = work["ffn_up_flops"] / up_s / 1e12
    tr = measured_hbm_traffic(cfg.name, ffn_entry(fused))
    roofline = {"bound": "mfma",
                "kernel": "the gated up-projection GEMM: part 1 of " + ffn_entry(fused),
                "achieved": achieved, "peak": PEAK_BF16_MFMA_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / PEAK_BF16_MFMA_TFLOPS,
                "traffic": (tr["read_bytes"] + tr["written_bytes"]) if tr else None,
                "traffic_unit": "bytes per launch (HBM read + written); null when profiles/ holds no summary "
                                "taken with this kernel source, entry point and workload",
                "traffic_detail": tr,
                "algorithmic_bytes_per_launch": work["ffn_up_bytes"],
                "flops_per_launch": work["ffn_up_flops"], "avg_launch_ms": per_call_ms["ffn_up"]}
    others = {
        "ffn_down_tflops": work["ffn_down_flops"] / (per_call_ms["ffn_down"] * 1e-3) / 1e12,
        "ffn_total_frac_of_mfma_peak": (work["ffn_up_flops"] + work["ffn_down_flops"]) /
        ((per_call_ms["ffn_up"] + per_call_ms["ffn_down"]) * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS,
        "route_gbs": work["route_bytes"] / (per_call_ms["route"] * 1e-3) / 1e9,
        "count_and_permute_gbs": (work["permute_maps_only_bytes"] if fused else work["permute_bytes"]) /
        (per_call_ms["count_and_permute"] * 1e-3) / 1e9,
        "count_and_permute_form": "maps only: the up-projection reads x through src_assign (latency-bound "
                                  "integer work, no HBM roofline claim)" if fused else "maps + x_perm rows",
        "combine_gbs": work["combine_bytes"] / (per_call_ms["combine"] * 1e-3) / 1e9,
        "hbm_peak_gbs": PEAK_HBM_GBS,
        "note": "every step re-uses the same buffers, but a step streams several GB of weights and "
                "activations between two uses of a buffer, far more than the 256 MB last-level "
                "cache holds, so the HBM-bound calls start cold; event timings include launch gaps",
    }
    out = {
        "metric": "MoE-layer tokens/sec + grouped-FFN % of bf16 MFMA peak (Mixtral shape)"
        if cfg.name == "mixtral" else f"MoE-layer tokens/sec + grouped-FFN % of bf16 MFMA peak ({cfg.name})",
        "value": cfg.T / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == si.BF16 else "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: T={cfg.T} d={cfg.d} E={cfg.E} k={cfg.k} F={cfg.F} "
                               f"renorm={cfg.renorm} seed={cfg.seed}, one MoE-layer forward",
                   "ffn_input": ("x through the permutation map (%s)" % ffn_entry(fused)) if fused
                   else "materialised x_perm (%s)" % ffn_entry(fused),
                   "ffn_split_tiles": bool(args.ffn_split)},
        "ffn_pct_of_bf16_mfma_peak": 100.0 * others["ffn_total_frac_of_mfma_peak"],
        "per_call_ms": per_call_ms, "per_call_ms_min": per_call_ms_min,
        "per_call_ms_median": per_call_ms_median, "roofline": roofline, "other_calls": others,
    }
    if four_call is not None:
        out["four_call_form"] = four_call
        out["four_call_form_ms_per_step"] = four_call["ms_per_step"]
    if k1_form is not None:
        out["combine_in_ffn_form"] = k1_form
    if consumers is not None:
        out["load_consumers"] = consumers
    if not args.no_hbm_bound:
        out["hbm_bound_calls"] = hbm_bound_calls(torch, si, B, layer, st)
    if args.predictor_accuracy:
        import numpy as np
        w_acc = layer.to_device(si.make_layer(
            si.small_config("predictor_gate", T=cfg.T, d=cfg.d, E=cfg.E, k=cfg.k, F=cfg.F,
                            dtype=cfg.dtype, renorm=cfg.renorm, seed=cfg.seed + 1),
            parts=("w_gate",))["w_gate"])
        p_acc = layer.LoadPredictor(cfg.T, cfg.d, cfg.E, cfg.k, cfg.dtype, cfg.renorm, cfg.E)
        rows = []
        for eps in (0.0, 0.1, 0.25, 0.5, 1.0):
            x_later = layer.to_device(si.residual_step(cfg, L["x"], eps))
            cp, ca, same = layer.predicted_vs_actual_loads(p_acc, x, x_later, w_acc, bias, st)
            cp, ca = cp.astype(np.float64), ca.astype(np.float64)
            r = float(np.corrcoef(cp, ca)[0, 1]) if cp.std() > 0 and ca.std() > 0 else 1.0
            rows.append({"eps": eps, "pearson_r_of_counts": r,
                         "mean_abs_count_error_over_mean_count": float(np.abs(cp - ca).mean() / ca.mean()),
                         "max_abs_count_error_over_max_count": float(np.abs(cp - ca).max() / ca.max()),
                         "token_choices_kept": same})
        out["predictor_accuracy"] = {
            "model": "x_later = x + eps * N(0,1) per element (x ~ N(0,1)); the predictor is the later "
                     "layer's gate (a second seeded gate matrix) applied to x, the truth the same gate "
                     "on x_later; the workload's gate bias is applied to both",
            "rows": rows}
    if args.ep_sim > 0:
        # outside the timed region: the permuted rows are materialised once, then every simulated
        # rank's grouped FFN runs alone
        from paper_2603_06350_amd import ep_sim
        B.moe_route_ws(sh, x, wg, bias, buf.topk_idx, buf.topk_w, None, buf.workspace, buf.ws_bytes, st)
        B.moe_count_and_permute(sh, x, buf.topk_idx, buf.counts, buf.offsets, buf.dst_row,
                                buf.src_assign, buf.x_perm, buf.workspace, buf.ws_bytes, st)
        out["ep_simulation"] = ep_sim.simulate(buf, x, w1, w3, w2, args.ep_sim)
    if not args.no_achievable_peaks:
        torch.cuda.synchronize()
        roofline["achievable_peak"] = achievable_peaks()
        if cfg.dtype == si.BF16:
            roofline["vendor_dense_gemm"] = vendor_dense_gemm(torch, cfg, x, w1, w2)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, L, cfg.T)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
