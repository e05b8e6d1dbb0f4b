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


def test_predicted_and_later_loads_on_a_residual_stream_match_the_oracle():
    """Section 4.1: the loads predicted from the current hidden states against the loads the same
    gate produces one layer later (stand-in: x + eps * noise).  Both count vectors and the share of
    token choices that survive are the oracle's on the same input bytes; eps = 0 predicts exactly."""
    cfg = si.small_config("pred_acc", T=900, d=256, E=16, k=2, F=64, zipf_alpha=1.2, zipf_scale=0.5)
    L = si.make_layer(cfg, parts=("x", "w_gate"))
    bias = L["gate_bias"]
    w_pred = si.make_layer(si.small_config("pred_gate", T=cfg.T, d=cfg.d, E=cfg.E, k=cfg.k, F=64,
                                           seed=cfg.seed + 1), parts=("w_gate",))["w_gate"]
    pred = layer.LoadPredictor(cfg.T, cfg.d, cfg.E, cfg.k, cfg.dtype, cfg.renorm, max_extra_replicas=8)
    x_dev, w_dev, b_dev = layer.to_device(L["x"]), layer.to_device(w_pred), layer.to_device(bias)
    for eps in (0.0, 0.5):
        x_later = si.residual_step(cfg, L["x"], eps)
        cp, ca, kept = layer.predicted_vs_actual_loads(pred, x_dev, layer.to_device(x_later), w_dev, b_dev)
        idx_now, _, _ = orc.route(L["x"], w_pred, cfg.k, cfg.renorm, bias)
        idx_later, _, _ = orc.route(x_later, w_pred, cfg.k, cfg.renorm, bias)
        assert np.array_equal(cp, np.bincount(idx_now.ravel(), minlength=cfg.E))
        assert np.array_equal(ca, np.bincount(idx_later.ravel(), minlength=cfg.E))
        kept_ref = np.mean([[idx_now[t, j] in idx_later[t] for j in range(cfg.k)] for t in range(cfg.T)])
        assert abs(kept - kept_ref) < 1e-6
        if eps == 0.0:
            assert np.array_equal(cp, ca) and kept == 1.0
        else:
            assert 0.3 < kept < 1.0 and not np.array_equal(cp, ca)


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


# ----------------------------------------------------------------------------- placement
from oracle import placer_oracle as pl  # noqa: E402


def gpu_place(loads, replicas, G, prev_offsets=None, prev_gpu=None, slots=None, max_segments=None):
    E = len(loads)
    S = int(np.sum(replicas))
    max_segments = S if max_segments is None else max_segments
    i32 = lambda a: None if a is None else torch.tensor(np.asarray(a, dtype=np.int32), device="cuda")
    gpu_of = torch.full((max(max_segments, 1),), -9, dtype=torch.int32, device="cuda")
    load = torch.full((G,), -1.0, dtype=torch.float64, device="cuda")
    count = torch.full((G,), -1, dtype=torch.int32, device="cuda")
    warm = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    d_prev_gpu = i32(prev_gpu)
    if prev_gpu is not None and len(prev_gpu) == 0:        # a zero-size tensor has no address
        d_prev_gpu = torch.zeros(1, dtype=torch.int32, device="cuda")
    prev_replicas = None if prev_offsets is None else np.diff(np.asarray(prev_offsets))
    B.moe_place_replicas(E, i32(loads), i32(replicas), G, i32(prev_replicas), d_prev_gpu, i32(slots),
                         max_segments, gpu_of, load, count, warm)
    torch.cuda.synchronize()
    return gpu_of.cpu().numpy(), load.cpu().numpy(), count.cpu().numpy(), int(warm.item())


def check_place(loads, replicas, G, prev_offsets=None, prev_gpu=None, slots=None):
    want_of, want_load, want_count, want_warm = pl.expert_placement(loads, replicas, G, prev_offsets,
                                                                    prev_gpu, slots)
    got_of, got_load, got_count, got_warm = gpu_place(loads, replicas, G, prev_offsets, prev_gpu, slots)
    assert np.array_equal(got_of[:len(want_of)], want_of)
    assert np.array_equal(got_count, want_count) and got_warm == want_warm
    assert np.array_equal(got_load, want_load)            # the same fp64 sums in the same order
    return got_of


def test_place_replicas_hand_worked():
    assert check_place([6, 4, 2], [2, 1, 1], 2).tolist() == [1, 1, 0, 0]
    assert check_place([6, 4, 2], [2, 1, 1], 2, [0, 1, 2, 3], [-1, 1, -1]).tolist() == [0, 0, 1, 1]
    assert check_place([10, 9], [1, 1], 2, [0, 1, 2], [0, 0]).tolist() == [0, 0]
    assert check_place([6, 4, 2], [2, 1, 1], 2, slots=[1, 3]).tolist() == [1, 1, 0, 1]
    assert check_place([6, 4, 2], [2, 1, 1], 2, slots=[1, 1]).tolist() == [1, -1, 0, -1]
    assert check_place([5, 4], [1, 1], 2, [0, 1, 2], [0, 0], slots=[1, 1]).tolist() == [0, 1]
    check_place([0, 0, 0], [1, 2, 1], 3)                                   # zero loads are placed too
    check_place([7], [5], 1)                                               # one GPU


def test_place_replicas_matches_oracle():
    rng = np.random.default_rng(53)
    for trial in range(40):
        E = int(rng.choice([1, 3, 8, 16, 64, 200, 256]))
        loads = si.zipf_loads(E, int(rng.integers(E, 200000)), float(rng.uniform(0.2, 1.8)), 500 + trial)
        replicas, _ = sc.expert_scaling(loads, 1, int(rng.integers(0, 2 * E + 1)), 0.1)
        G = int(rng.choice([1, 2, 7, 8, 16, 64]))
        kind = trial % 4
        prev_offsets = prev_gpu = slots = None
        if kind in (1, 3):
            prev_r = rng.integers(0, 4, size=E)
            prev_offsets = np.concatenate([[0], np.cumsum(prev_r)])
            prev_gpu = rng.integers(-1, G, size=int(prev_offsets[-1]))
        if kind in (2, 3):
            S = int(replicas.sum())
            slots = rng.integers(0, max(2, 2 * S // G + 2), size=G)
        check_place(loads, replicas, G, prev_offsets, prev_gpu, slots)


def test_place_replicas_respects_the_output_bound():
    loads, replicas = [9, 7, 5, 3], [3, 2, 1, 1]
    want, _, _, _ = pl.expert_placement(loads, replicas, 2)
    got, _, count, _ = gpu_place(loads, replicas, 2, max_segments=4)
    assert np.array_equal(got[:4], want[:4]) and count.sum() == 7          # all placed, four reported


def test_scale_segments_place_chain_on_device():
    """counts -> Algorithm 1 -> segments -> Algorithm 2, one stream, no host round trip; then a second
    round that re-uses the first round's placement as its warm set."""
    E, G = 64, 8
    loads = si.zipf_loads(E, 49152, 1.2, 77)
    d_loads = torch.tensor(loads.astype(np.int32), device="cuda")
    rep = torch.zeros(E, dtype=torch.int32, device="cuda")
    S_max = E + 32
    gpu_of = torch.full((S_max,), -9, dtype=torch.int32, device="cuda")
    load = torch.zeros(G, dtype=torch.float64, device="cuda")
    count = torch.zeros(G, dtype=torch.int32, device="cuda")
    warm = torch.zeros(1, dtype=torch.int32, device="cuda")
    B.moe_scale_replicas(E, d_loads, 1, 32, 0.2, rep, None)
    B.moe_place_replicas(E, d_loads, rep, G, None, None, None, S_max, gpu_of, load, count, warm)
    torch.cuda.synchronize()
    want_rep, _ = sc.expert_scaling(loads, 1, 32, 0.2)
    want_of, want_load, want_count, _ = pl.expert_placement(loads, want_rep, G)
    S = int(want_rep.sum())
    assert np.array_equal(rep.cpu().numpy(), want_rep)
    assert np.array_equal(gpu_of.cpu().numpy()[:S], want_of)
    assert np.array_equal(load.cpu().numpy(), want_load)
    # balanced: no GPU is above the mean by more than the largest replica load
    per = (loads / want_rep).max()
    assert want_load.max() - want_load.mean() <= per
    # second round: a different batch, the previous placement kept alive
    loads2 = si.zipf_loads(E, 49152, 1.2, 78)
    prev_offsets = np.concatenate([[0], np.cumsum(want_rep)]).astype(np.int32)
    want_rep2, _ = sc.expert_scaling(loads2, 1, 32, 0.2)
    want2 = pl.expert_placement(loads2, want_rep2, G, prev_offsets, want_of)
    got2 = gpu_place(loads2, want_rep2, G, prev_offsets, want_of)
    assert np.array_equal(got2[0][:len(want2[0])], want2[0]) and got2[3] == want2[3] and want2[3] > 0


def test_predictor_with_placement_keeps_warm_replicas_over_rounds():
    cfg = si.small_config("pred_place", T=900, d=256, E=16, k=2, F=128, zipf_alpha=1.2, zipf_scale=0.9)
    L = si.make_layer(cfg, parts=("x", "w_gate"))
    x, wg, bias = (layer.to_device(L[n]) for n in ("x", "w_gate", "gate_bias"))
    G = 4
    pred = layer.LoadPredictor(cfg.T, cfg.d, cfg.E, cfg.k, cfg.dtype, cfg.renorm, max_extra_replicas=8,
                               n_gpus=G)
    idx, _, _ = orc.route(L["x"], L["w_gate"], cfg.k, cfg.renorm, L["gate_bias"])
    counts = np.bincount(idx.ravel(), minlength=cfg.E)
    rep, _ = sc.expert_scaling(counts, 1, 8, 0.2)
    first = pl.expert_placement(counts, rep, G)
    pred.enqueue(x, wg, bias, 0.2)
    torch.cuda.synchronize()
    S = int(rep.sum())
    assert np.array_equal(pred.replicas.cpu().numpy(), rep)
    assert np.array_equal(pred.gpu_of[0].cpu().numpy()[:S], first[0]) and int(pred.n_warm.item()) == 0
    # same batch again: every replica is warm and nothing moves
    pred.enqueue(x, wg, bias, 0.2)
    torch.cuda.synchronize()
    second = pl.expert_placement(counts, rep, G, np.concatenate([[0], np.cumsum(rep)]), first[0])
    assert second[3] == S and np.array_equal(second[0], first[0])
    assert np.array_equal(pred.gpu_of[1].cpu().numpy()[:S], second[0]) and int(pred.n_warm.item()) == S
    assert np.array_equal(pred.gpu_load.cpu().numpy(), second[1])
