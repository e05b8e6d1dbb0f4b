"""Writes tests/golden/route_margins.txt: for every named workload, the oracle's
per-expert token counts and the smallest relative top-k margin
(score_(k) - score_(k+1)) / max|score| over all tokens.

Calls only the CPU oracle and the input generator.  The margins justify comparing
the HIP router's indices with the oracle's on every row: a differently ordered
fp32 gate sum moves a score by ~1e-6 relative, so a workload whose smallest margin
is above 1e-4 cannot legitimately flip a choice.  A seed is only accepted if it
gives zero rows below that threshold.

usage: python tests/golden/make_route_margins.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import moe_oracle as orc  # noqa: E402
import synth_inputs as si  # noqa: E402

DELTA = 1e-4


def main():
    lines = ["# name seed min_margin rows_below_1e-4 hottest_share empty_experts counts_crc"]
    for name, cfg in si.CONFIGS.items():
        L = si.make_layer(cfg, parts=("x", "w_gate"))
        idx, _, score = orc.route(L["x"], L["w_gate"], cfg.k, cfg.renorm, L["gate_bias"])
        counts, _ = orc.expert_load(idx, cfg.E)
        m = orc.topk_margin(score, cfg.k)
        crc = int(np.bitwise_xor.reduce((counts.astype(np.int64) * 2654435761) % (1 << 32)))
        lines.append(f"{name} {cfg.seed} {m.min():.6e} {(m < DELTA).sum()} "
                     f"{counts.max() / cfg.A:.4f} {(counts == 0).sum()} {crc}")
        print(lines[-1])
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "route_margins.txt"),
              "w") as f:
        f.write("\n".join(lines) + "\n")


if __name__ == "__main__":
    main()
