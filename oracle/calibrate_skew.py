"""Find the Zipf bias scale of the skewed-load workload (run once; result is pasted
into synth_inputs.ZIPF_SCALE_SKEW).

TEST INFRASTRUCTURE ONLY: calls the CPU oracle router and the input generator.

The skewed layer adds b_e = s * ln(p_e), p_e ~ rank^-1.2 (expert 0 hottest), to the gate
logits.  An expert can receive at most one of a token's k assignments, so its share
of the T*k assignments is at most 1/k (16.7% at k = 6); the 20% the workload
description asks for is out of reach and the target used is "chosen by 95% of the
tokens", a 15.8% share.  s is bisected on a dyadic grid so it prints exactly.

usage: python -m oracle.calibrate_skew
"""
from dataclasses import replace

import numpy as np

from oracle import moe_oracle as orc
import synth_inputs as si


def hottest_share(cfg):
    L = si.make_layer(cfg, parts=("x", "w_gate"))
    idx, _, _ = orc.route(L["x"], L["w_gate"], cfg.k, cfg.renorm, L["gate_bias"])
    counts, _ = orc.expert_load(idx, cfg.E)
    return counts.max() / float(cfg.A), counts


def main():
    base = si.CONFIGS["skew"]
    target = min(0.20, 0.95 / base.k)
    lo, hi = 0.0, 16.0
    for _ in range(14):
        mid = 0.5 * (lo + hi)
        share, _ = hottest_share(replace(base, zipf_scale=mid))
        if share < target:
            lo = mid
        else:
            hi = mid
    share, counts = hottest_share(replace(base, zipf_scale=hi))
    cv = counts.std() / counts.mean()
    print(f"ZIPF_SCALE_SKEW = {hi!r}")
    print(f"hottest share of T*k = {share:.4f} (target {target:.4f}); CV = {cv:.3f}; "
          f"empty experts = {(counts == 0).sum()}; counts[:8] = {counts[:8].tolist()}; "
          f"min count = {counts.min()}")


if __name__ == "__main__":
    main()
