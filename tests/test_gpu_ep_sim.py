"""The expert-parallel latency model (paper, Section 4.3): shares of simulated ranks under the
static placement and under Algorithms 1 + 2 partition the rows, and every rank's grouped FFN
reproduces the un-sharded call's rows bit for bit."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import moe_oracle as orc
from oracle import scaler_oracle as sco

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from paper_2603_06350_amd import binding as B  # noqa: E402
from paper_2603_06350_amd import ep_sim, layer  # noqa: E402


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    B.load()


def routed_buffers(cfg):
    L = si.make_layer(cfg)
    x, wg, w1, w3, w2 = (layer.to_device(L[n]) for n in ("x", "w_gate", "w1", "w3", "w2"))
    bias = layer.to_device(L["gate_bias"])
    buf = layer.MoeBuffers(cfg.T, cfg.d, cfg.E, cfg.k, cfg.F, cfg.dtype, cfg.renorm)
    st = torch.cuda.current_stream()
    B.moe_route_ws(buf.shape, x, wg, bias, buf.topk_idx, buf.topk_w, None, buf.workspace, buf.ws_bytes, st)
    B.moe_count_and_permute(buf.shape, x, buf.topk_idx, buf.counts, buf.offsets, buf.dst_row,
                            buf.src_assign, buf.x_perm, buf.workspace, buf.ws_bytes, st)
    torch.cuda.synchronize()
    return L, buf, x, w1, w3, w2


def test_ranks_reproduce_the_unsharded_rows_and_scaling_cuts_the_straggler_share():
    # a Zipf-skewed batch over 16 experts, 4 simulated GPUs
    cfg = si.small_config("ep_sim", T=3000, d=256, E=16, k=2, F=384, zipf_alpha=1.2, zipf_scale=1.0)
    L, buf, x, w1, w3, w2 = routed_buffers(cfg)
    res = ep_sim.simulate(buf, x, w1, w3, w2, 4, cv_threshold=0.2, iters=2, check=True)
    A = cfg.T * cfg.k
    for key in ("static_expert_parallel", "scaled_and_placed"):
        assert sum(res[key]["rows_per_rank"]) == A
    # the replica counts and the placement are the oracle's (Algorithms 1 and 2 on the same counts)
    idx, _, _ = orc.route(L["x"], L["w_gate"], cfg.k, cfg.renorm, gate_bias=L["gate_bias"])
    counts, _ = orc.expert_load(idx, cfg.E)
    assert np.array_equal(counts, buf.counts.cpu().numpy())
    rep, _ = sco.expert_scaling(counts, 1, cfg.E, 0.2)
    assert int(np.sum(rep)) == res["replicas_total"]
    # the most loaded rank holds fewer rows once hot experts are replicated and placed by load
    assert max(res["scaled_and_placed"]["rows_per_rank"]) < max(res["static_expert_parallel"]["rows_per_rank"])
    assert res["cv_of_per_replica_loads"]["after"] <= res["cv_of_per_replica_loads"]["before"]
