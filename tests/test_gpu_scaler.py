"""GPU parity of the load-statistic consumers: moe_scale_replicas (Algorithm 1) and
moe_replica_segments against oracle/scaler_oracle.py, bit-exact on every integer output; the two
CV values within 1e-12 relative (both sides compute them in fp64, in a different summation order).
The decision CV > V is taken in fp64 on both sides; each case first checks, on the oracle's trace,
that no step sits on the knife edge |CV - V| < 1e-9 where the order of an fp64 sum could decide."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import moe_oracle as orc
from oracle import scaler_oracle as sc

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from paper_2603_06350_amd import binding as B  # noqa: E402
from paper_2603_06350_amd import layer  # noqa: E402


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    B.load()


def gpu_scale(loads, mem, cap, V):
    E = len(loads)
    d_loads = torch.tensor(np.asarray(loads, dtype=np.int32), device="cuda")
    rep = torch.full((E,), -7, dtype=torch.int32, device="cuda")
    cvs = torch.full((2,), -1.0, dtype=torch.float64, device="cuda")
    B.moe_scale_replicas(E, d_loads, mem, cap, V, rep, cvs)
    torch.cuda.synchronize()
    return rep.cpu().numpy(), cvs.cpu().numpy()


def off_the_edge(cv, V):
    """A balanced layer has CV exactly 0 on both sides (every deviation is an exact zero)."""
    return abs(cv - V) > 1e-9 or (cv == 0.0 and V == 0.0)


def check_scale(loads, mem, cap, V):
    want, trace = sc.expert_scaling(loads, mem, cap, V)
    assert all(off_the_edge(t, V) for t in trace), "case sits on the CV == V knife edge"
    got, cvs = gpu_scale(loads, mem, cap, V)
    assert np.array_equal(got, want), f"replicas differ: gpu {got} oracle {want}"
    assert cvs[0] == pytest.approx(trace[0], rel=1e-12, abs=1e-15)
    assert cvs[1] == pytest.approx(trace[-1], rel=1e-12, abs=1e-15)
    return got


SCALE_CASES = [
    # E, total, alpha, seed, M_e, M_cap, V
    (8, 8192, 1.2, 1, 1, 16, 0.2),
    (8, 8192, 1.2, 1, 1, 3, 0.2),
    (16, 4096, 2.0, 4, 3, 50, 0.05),
    (64, 49152, 1.2, 2, 1, 64, 0.2),
    (64, 49152, 1.2, 2, 1, 1000, 0.0),        # never balanced: stops at the cap, 1000 steps
    (128, 256, 0.8, 3, 2, 7, 0.0),
    (200, 100000, 1.0, 5, 1, 300, 0.1),
    (256, 1 << 20, 1.5, 6, 1, 2048, 0.02),
    (1, 500, 1.0, 7, 1, 10, 0.0),             # a single expert: CV 0, nothing to do
]


@pytest.mark.parametrize("case", SCALE_CASES, ids=lambda c: "E{}_cap{}_V{}".format(c[0], c[5], c[6]))
def test_scale_replicas_matches_oracle(case):
    E, total, alpha, seed, mem, cap, V = case
    check_scale(si.zipf_loads(E, total, alpha, seed), mem, cap, V)


def test_scale_replicas_degenerate_loads():
    assert check_scale([50] * 8, 1, 100, 0.0).tolist() == [1] * 8          # uniform
    assert check_scale([0] * 8, 1, 100, 0.0).tolist() == [1] * 8           # no tokens
    assert check_scale([1000, 0, 0, 0], 1, 5, 0.0).tolist() == [6, 1, 1, 1]  # one hot expert
    assert check_scale([8, 8, 1], 1, 1, 0.0).tolist() == [2, 1, 1]          # equal stragglers
    assert check_scale([3000, 1000], 1, 10, 0.2).tolist() == [2, 1]         # the hand-worked case
    assert check_scale([3000, 1000], 1, 10, 0.1).tolist() == [3, 1]
    assert check_scale([900, 100, 100, 100], 3, 2, 0.2).tolist() == [1, 1, 1, 1]   # cap below M_e
    assert check_scale([900, 100, 100, 100], 3, 8, 0.2).tolist() == [3, 1, 1, 1]
    big = [2 ** 31 - 1, 2 ** 30, 5, 0]                                      # largest counts
    check_scale(big, 1, 40, 0.0)


def test_scale_replicas_largest_budget():
    """MOE_MAX_EXTRA_REPLICAS steps (V < 0: only the cap stops the loop).  Too many steps for the
    oracle's per-step CV; checked through what is unique about the greedy result: all the budget
    is used, and no replica could move from one expert to another and lower the largest
    per-replica load (W_a / R_a <= W_b / (R_b - 1) for every pair with R_b > 1)."""
    from fractions import Fraction
    loads = si.zipf_loads(16, 1 << 22, 1.1, 8)
    got, _ = gpu_scale(loads, 1, B.MOE_MAX_EXTRA_REPLICAS, -1.0)
    assert int(got.sum()) == 16 + B.MOE_MAX_EXTRA_REPLICAS and got.min() >= 1
    top = max(Fraction(int(w), int(r)) for w, r in zip(loads, got))
    for w, r in zip(loads, got):
        if r > 1:
            assert top <= Fraction(int(w), int(r) - 1)
    # and a prefix of the same run agrees with the oracle step by step
    check_scale(loads, 1, 3000, -1.0)


def test_scale_replicas_on_the_layer_counts():
    """Loads taken from the dispatch of a skewed layer, on the device, without a host round trip."""
    cfg = si.small_config("scaler_skew", T=600, d=256, E=64, k=6, F=128, renorm=0, zipf_alpha=1.2,
                          zipf_scale=0.9, empty_tail=4)
    L = si.make_layer(cfg, parts=("x", "w_gate"))
    idx, _, _ = orc.route(L["x"], L["w_gate"], cfg.k, cfg.renorm, L["gate_bias"])
    counts_ref = np.bincount(idx.ravel(), minlength=cfg.E)
    buf = layer.MoeBuffers(cfg.T, cfg.d, cfg.E, cfg.k, cfg.F, cfg.dtype, cfg.renorm)
    st = torch.cuda.current_stream()
    B.moe_route(buf.shape, layer.to_device(L["x"]), layer.to_device(L["w_gate"]),
                layer.to_device(L["gate_bias"]), buf.topk_idx, buf.topk_w, None, st)
    B.moe_count_and_permute(buf.shape, None, buf.topk_idx, buf.counts, buf.offsets, buf.dst_row,
                            buf.src_assign, None, buf.workspace, buf.ws_bytes, st)
    rep = torch.zeros(cfg.E, dtype=torch.int32, device="cuda")
    cvs = torch.zeros(2, dtype=torch.float64, device="cuda")
    B.moe_scale_replicas(cfg.E, buf.counts, 1, 32, 0.2, rep, cvs, st)
    S_max = cfg.E + 32
    seg = torch.full((S_max + 1,), -1, dtype=torch.int32, device="cuda")
    who = torch.full((S_max,), -1, dtype=torch.int32, device="cuda")
    n = torch.zeros(1, dtype=torch.int32, device="cuda")
    B.moe_replica_segments(cfg.E, buf.offsets, rep, S_max, seg, who, n, st)
    torch.cuda.synchronize()
    assert np.array_equal(buf.counts.cpu().numpy(), counts_ref)
    want, trace = sc.expert_scaling(counts_ref, 1, 32, 0.2)
    assert all(off_the_edge(t, 0.2) for t in trace)
    assert np.array_equal(rep.cpu().numpy(), want)
    assert cvs.cpu().numpy()[0] == pytest.approx(sc.cv(counts_ref), rel=1e-12)
    offsets = np.concatenate([[0], np.cumsum(counts_ref)])
    seg_ref, who_ref = sc.replica_segments(offsets, want)
    S = int(want.sum())
    assert int(n.item()) == S
    assert np.array_equal(seg.cpu().numpy()[:S + 1], seg_ref)
    assert np.array_equal(who.cpu().numpy()[:S], who_ref)


def test_replica_segments_matches_oracle_and_respects_the_bound():
    rng = np.random.default_rng(31)
    for E in (1, 7, 64, 256):
        counts = rng.integers(0, 500, size=E)
        reps = rng.integers(1, 9, size=E).astype(np.int32)
        offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
        seg_ref, who_ref = sc.replica_segments(offsets, reps)
        S = int(reps.sum())
        for max_seg in (S + 5, S, max(S // 2, 0)):
            seg = torch.full((max_seg + 1,), -9, dtype=torch.int32, device="cuda")
            who = torch.full((max(max_seg, 1),), -9, dtype=torch.int32, device="cuda")
            n = torch.zeros(1, dtype=torch.int32, device="cuda")
            B.moe_replica_segments(E, torch.tensor(offsets, device="cuda"),
                                   torch.tensor(reps, device="cuda"), max_seg, seg, who, n)
            torch.cuda.synchronize()
            m = min(S, max_seg)
            assert int(n.item()) == S
            assert np.array_equal(seg.cpu().numpy()[:m + 1], seg_ref[:m + 1])
            assert np.array_equal(who.cpu().numpy()[:m], who_ref[:m])
            assert np.all(seg.cpu().numpy()[m + 1:] == -9)          # nothing past the bound
            assert np.all(who.cpu().numpy()[m:max_seg] == -9)


def test_predictor_on_a_side_stream_next_to_the_layer():
    """Section 4.1 / 5: the gate of a later layer (here: a second seeded gate matrix; fine-tuning is
    out of scope) scores the current layer's input on a side stream while the layer itself runs.
    The predicted counts and the replica plan match the oracle bit-exactly, and the layer's own
    outputs are the same bits with and without the predictor beside it."""
    cfg = si.small_config("pred_layer", T=1400, d=256, E=8, k=2, F=512)
    pred_cfg = si.small_config("pred_gate", T=1400, d=256, E=8, k=2, F=512, seed=cfg.seed + 1)
    L = si.make_layer(cfg)
    w_pred = si.make_layer(pred_cfg, parts=("w_gate",))["w_gate"]
    dev = {n: layer.to_device(L[n]) for n in ("x", "w_gate", "w1", "w3", "w2")}
    d_pred = layer.to_device(w_pred)
    buf = layer.MoeBuffers(cfg.T, cfg.d, cfg.E, cfg.k, cfg.F, cfg.dtype, cfg.renorm)
    buf.forward(dev["x"], dev["w_gate"], dev["w1"], dev["w3"], dev["w2"])
    torch.cuda.synchronize()
    alone = {n: layer.to_host(getattr(buf, n)).copy() for n in ("topk_idx", "counts", "dst_row", "h", "y")}

    pred = layer.LoadPredictor(cfg.T, cfg.d, cfg.E, cfg.k, cfg.dtype, cfg.renorm, max_extra_replicas=8)
    side = torch.cuda.Stream()
    main = torch.cuda.current_stream()
    for n in ("h", "y"):
        getattr(buf, n).zero_()
    ready = torch.cuda.Event()
    ready.record(main)                       # x is resident; the side stream starts from here
    side.wait_event(ready)
    pred.enqueue(dev["x"], d_pred, cv_threshold=0.05, stream=side)
    buf.forward(dev["x"], dev["w_gate"], dev["w1"], dev["w3"], dev["w2"], stream=main)
    main.wait_stream(side)
    torch.cuda.synchronize()
    for n, v in alone.items():
        assert np.array_equal(layer.to_host(getattr(buf, n)), v), f"{n} changed beside the predictor"

    idx_p, _, _ = orc.route(L["x"], w_pred, cfg.k, cfg.renorm, None)
    counts_p = np.bincount(idx_p.ravel(), minlength=cfg.E)
    assert np.array_equal(pred.counts.cpu().numpy(), counts_p)
    want, trace = sc.expert_scaling(counts_p, 1, 8, 0.05)
    assert all(off_the_edge(t, 0.05) for t in trace)
    assert np.array_equal(pred.replicas.cpu().numpy(), want)
    seg_ref, who_ref = sc.replica_segments(np.concatenate([[0], np.cumsum(counts_p)]), want)
    S = int(want.sum())
    assert int(pred.n_segments.item()) == S
    assert np.array_equal(pred.seg_offsets.cpu().numpy()[:S + 1], seg_ref)
    assert np.array_equal(pred.seg_expert.cpu().numpy()[:S], who_ref)
    # the prediction of a gate that differs from the layer's own is a different load vector
    assert not np.array_equal(counts_p, alone["counts"])
