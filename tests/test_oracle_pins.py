"""Pins for the CPU oracle: each oracle function is checked against something that
is not itself - brute force in scalar Python, closed forms, invariants, special
cases that reduce to a NumPy/SciPy routine - chosen so that a dropped term, a
wrong sign or index, or a transposed operand fails at least one test.  The last
tests plant such mistakes in copies of the oracle and check they are caught.
"""
import math

import numpy as np
import pytest
import scipy.special

from oracle import moe_oracle as orc
import synth_inputs as si


def tiny_layer(**kw):
    cfg = si.small_config(T=kw.pop("T", 13), d=kw.pop("d", 24), E=kw.pop("E", 5),
                          k=kw.pop("k", 2), F=kw.pop("F", 16), **kw)
    return cfg, si.make_layer(cfg)


# ----------------------------------------------------------------------------- formats
def test_bf16_widening_is_exact_and_rne():
    vals = np.array([1.0, -2.5, 3.140625, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1e-20, 65504.0],
                    dtype=np.float32)
    bits = si.f32_to_bf16_bits(vals)
    back = orc.to_f64(bits)
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7: even mantissa wins -> 1.0
    assert back[3] == 1.0
    # 1 + 3*2^-8 is a tie between 1+2^-7 and 1+2^-6: even mantissa -> 1 + 2^-6
    assert back[4] == 1.0 + 2 ** -6
    assert back[0] == 1.0 and back[1] == -2.5 and back[2] == 3.140625
    assert np.all(np.abs(back - vals.astype(np.float64)) <= np.abs(vals) * 2.0 ** -8)
    assert np.array_equal(orc.to_f64(bits), si.bf16_bits_to_f32(bits).astype(np.float64))


# ----------------------------------------------------------------------------- gate
@pytest.mark.parametrize("dtype", [si.F32, si.BF16])
def test_gate_scores_scalar_loop(dtype):
    cfg, L = tiny_layer(dtype=dtype)
    bias = np.linspace(-0.5, 0.5, cfg.E).astype(np.float32)
    got = orc.gate_scores(L["x"], L["w_gate"], bias)
    x = orc.to_f64(L["x"])
    w = orc.to_f64(L["w_gate"])
    for t in range(cfg.T):
        for e in range(cfg.E):
            acc = math.fsum(float(x[t, i]) * float(w[e, i]) for i in range(cfg.d))
            assert got[t, e] == np.float32(acc + float(bias[e]))
    assert got.dtype == np.float32 and got.shape == (cfg.T, cfg.E)


def test_topk_brute_force_with_ties():
    rng = np.random.default_rng(3)
    # few distinct values -> many exact ties
    score = rng.integers(-2, 3, size=(200, 9)).astype(np.float32)
    for k in (1, 2, 4, 9):
        got = orc.topk_select(score, k)
        for t in range(score.shape[0]):
            order = sorted(range(score.shape[1]), key=lambda e: (-float(score[t, e]), e))
            assert got[t].tolist() == order[:k]


def test_topk_engineered_ties_from_the_gate():
    cfg, L = tiny_layer(E=6, k=3)
    wg = L["w_gate"].copy()
    wg[4] = wg[1]                       # experts 1 and 4 always tie
    idx, w, score = orc.route(L["x"], wg, 3, 1)
    assert np.array_equal(score[:, 1], score[:, 4])
    for t in range(cfg.T):
        row = idx[t].tolist()
        if 4 in row:                    # 4 may only appear directly after 1
            assert row.index(1) + 1 == row.index(4)
    # all-zero tokens: every score 0 -> experts 0..k-1, uniform probabilities
    x0 = np.zeros_like(L["x"])
    idx0, w0, _ = orc.route(x0, wg, 3, 0)
    assert np.array_equal(idx0, np.tile(np.arange(3, dtype=np.int32), (cfg.T, 1)))
    assert np.allclose(w0, 1.0 / 6.0, rtol=1e-7)


def test_routing_weights_closed_forms():
    cfg, L = tiny_layer(T=40, E=7, k=3)
    idx, w, score = orc.route(L["x"], L["w_gate"], 3, 1)
    assert np.allclose(w.sum(axis=1), 1.0, atol=1e-6)
    # renormalised top-k of the full softmax == softmax over the k selected scores
    sel = np.take_along_axis(score.astype(np.float64), idx.astype(np.int64), axis=1)
    assert np.allclose(w, scipy.special.softmax(sel, axis=1), rtol=1e-6)
    # without renormalisation: entries of the full softmax
    _, w_raw, _ = orc.route(L["x"], L["w_gate"], 3, 0)
    full = scipy.special.softmax(score.astype(np.float64), axis=1)
    assert np.allclose(w_raw, np.take_along_axis(full, idx.astype(np.int64), axis=1), rtol=1e-6)
    assert np.all(w_raw.sum(axis=1) < 1.0)
    # k = E: all experts, in descending-score order, weights = full softmax (sum 1 either way)
    idx_all, w_all, _ = orc.route(L["x"], L["w_gate"], 7, 0)
    assert np.array_equal(np.sort(idx_all, axis=1), np.tile(np.arange(7), (cfg.T, 1)))
    assert np.allclose(w_all.sum(axis=1), 1.0, atol=1e-6)
    assert np.all(np.diff(w_all, axis=1) <= 0)


def test_gate_bias_shifts_scores_and_steers_choice():
    cfg, L = tiny_layer(E=5, k=2)
    bias = np.zeros(5, np.float32)
    bias[3] = 1e9
    idx, w, _ = orc.route(L["x"], L["w_gate"], 2, 1, bias)
    assert np.all(idx[:, 0] == 3)
    assert np.allclose(w[:, 0], 1.0)


# ----------------------------------------------------------------------------- load + dispatch
def test_expert_load_and_permutation_invariants():
    rng = np.random.default_rng(11)
    T, k, E = 257, 3, 10
    idx = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    idx[idx == 9] = 0                                # force expert 9 empty (may duplicate 0)
    counts, offsets = orc.expert_load(idx, E)
    assert counts.sum() == T * k and offsets[E] == T * k and offsets[0] == 0
    assert np.array_equal(counts, np.bincount(idx.reshape(-1), minlength=E))
    assert np.array_equal(offsets[1:], np.cumsum(counts))
    assert counts[9] == 0
    dst, src = orc.permutation(idx, E)
    A = T * k
    assert np.array_equal(np.sort(dst), np.arange(A))              # bijection
    assert np.array_equal(src[dst], np.arange(A))                  # inverse
    assert np.array_equal(src, np.argsort(idx.reshape(-1), kind="stable"))
    expert_of_row = idx.reshape(-1)[src]
    assert np.all(np.diff(expert_of_row) >= 0)                     # expert-contiguous
    for e in range(E):                                             # ascending inside an expert
        seg = src[offsets[e]:offsets[e + 1]]
        assert np.all(np.diff(seg) > 0)


def test_permute_rows_then_combine_closed_form():
    # skip the experts: y_perm := x_perm  =>  y[t] = (sum_j w[t,j]) * x[t]
    cfg, L = tiny_layer(T=50, E=6, k=3, dtype=si.F32)
    for renorm in (0, 1):
        idx, w, _ = orc.route(L["x"], L["w_gate"], 3, renorm)
        dst, _ = orc.permutation(idx, cfg.E)
        xp = orc.permute_rows(L["x"], dst, 3)
        assert xp.dtype == L["x"].dtype
        for a in range(cfg.A):
            assert np.array_equal(xp[dst[a]], L["x"][a // 3])
        y = orc.combine(xp, dst, w)
        want = w.astype(np.float64).sum(axis=1, keepdims=True) * L["x"].astype(np.float64)
        assert np.allclose(y, want, rtol=1e-12, atol=0)


def test_combine_scalar_loop():
    rng = np.random.default_rng(5)
    T, k, d = 9, 3, 4
    yp = rng.standard_normal((T * k, d))
    dst = rng.permutation(T * k).astype(np.int32)
    w = rng.random((T, k)).astype(np.float32)
    got = orc.combine(yp, dst, w)
    for t in range(T):
        for i in range(d):
            acc = 0.0
            for j in range(k):
                acc += float(w[t, j]) * yp[dst[t * k + j], i]
            assert abs(got[t, i] - acc) <= 1e-14 * max(1.0, abs(acc))


# ----------------------------------------------------------------------------- experts
def test_expert_ffn_scalar_loop():
    rng = np.random.default_rng(9)
    m, d, F = 3, 5, 7
    x = rng.standard_normal((m, d))
    w1, w3 = rng.standard_normal((F, d)), rng.standard_normal((F, d))
    w2 = rng.standard_normal((d, F))
    y, h = orc.expert_ffn(x, w1, w3, w2, return_h=True)
    for r in range(m):
        hh = []
        for f in range(F):
            g = sum(w1[f, i] * x[r, i] for i in range(d))
            u = sum(w3[f, i] * x[r, i] for i in range(d))
            hh.append(g / (1.0 + math.exp(-g)) * u)
            assert abs(h[r, f] - hh[-1]) < 1e-12
        for i in range(d):
            assert abs(y[r, i] - sum(w2[i, f] * hh[f] for f in range(F))) < 1e-12


def identity_expert(d, F, c=1.5):
    """SwiGLU weights with E(x) = x for every x whose feature 0 equals 1:
    W1 rows = c*e0 (gate = silu(c) everywhere), W3 = [I;0], W2 = [I/silu(c), 0]."""
    assert F >= d
    s0 = c / (1.0 + math.exp(-c))
    w1 = np.zeros((F, d)); w1[:, 0] = c
    w3 = np.zeros((F, d)); w3[:d, :d] = np.eye(d)
    w2 = np.zeros((d, F)); w2[:d, :d] = np.eye(d) / s0
    return w1, w3, w2


def test_identity_experts_reproduce_the_input():
    rng = np.random.default_rng(21)
    T, d, E, k, F = 33, 12, 4, 2, 20
    x = rng.standard_normal((T, d)).astype(np.float32)
    x[:, 0] = 1.0
    wg = rng.standard_normal((E, d)).astype(np.float32)
    w1, w3, w2 = (np.stack([m] * E) for m in identity_expert(d, F))
    out = orc.moe_layer(x, wg, w1, w3, w2, k, renorm=1)
    assert np.allclose(out["y"], x.astype(np.float64), rtol=1e-6, atol=1e-6)
    # without renormalisation the layer scales x by the kept probability mass
    out0 = orc.moe_layer(x, wg, w1, w3, w2, k, renorm=0)
    mass = out0["topk_w"].astype(np.float64).sum(axis=1, keepdims=True)
    assert np.allclose(out0["y"], mass * x, rtol=1e-6, atol=1e-6)


def test_linear_expert_closed_form_when_F_less_than_d():
    # constant gate: E(x) = silu(c) * W2 W3 x  -- a plain matrix product
    rng = np.random.default_rng(22)
    m, d, F, c = 6, 16, 8, 0.7
    x = rng.standard_normal((m, d)); x[:, 0] = 1.0
    w1 = np.zeros((F, d)); w1[:, 0] = c
    w3 = rng.standard_normal((F, d)); w2 = rng.standard_normal((d, F))
    s0 = c / (1.0 + math.exp(-c))
    assert np.allclose(orc.expert_ffn(x, w1, w3, w2), s0 * (x @ w3.T @ w2.T), rtol=1e-12)


def test_single_expert_layer_is_a_dense_ffn():
    cfg, L = tiny_layer(T=20, E=1, k=1, dtype=si.F32)
    out = orc.moe_layer(L["x"], L["w_gate"], L["w1"], L["w3"], L["w2"], 1, 1)
    x = L["x"].astype(np.float64)
    g = x @ L["w1"][0].astype(np.float64).T
    u = x @ L["w3"][0].astype(np.float64).T
    want = (g * scipy.special.expit(g) * u) @ L["w2"][0].astype(np.float64).T
    assert np.allclose(out["y"], want, rtol=1e-10, atol=1e-18)
    assert np.allclose(out["topk_w"], 1.0)
    assert out["counts"].tolist() == [20]


def test_dense_special_case_k_equals_E():
    # k = E: y = sum_e softmax_e * E_e(x), computed with no routing or permutation
    cfg, L = tiny_layer(T=17, E=4, k=4, dtype=si.BF16)
    out = orc.moe_layer(L["x"], L["w_gate"], L["w1"], L["w3"], L["w2"], 4, 0)
    x = orc.to_f64(L["x"])
    p = scipy.special.softmax(orc.gate_scores(L["x"], L["w_gate"]).astype(np.float64), axis=1)
    want = np.zeros_like(x)
    for e in range(4):
        g = x @ orc.to_f64(L["w1"][e]).T
        u = x @ orc.to_f64(L["w3"][e]).T
        want += p[:, e:e + 1].astype(np.float32).astype(np.float64) * (
            (g * scipy.special.expit(g) * u) @ orc.to_f64(L["w2"][e]).T)
    assert np.allclose(out["y"], want, rtol=1e-9, atol=1e-12)


def test_whole_layer_brute_force_per_token_on_tiny_config():
    cfg = si.CONFIGS["tiny"]
    L = si.make_layer(cfg)
    out = orc.moe_layer(L["x"], L["w_gate"], L["w1"], L["w3"], L["w2"], cfg.k, cfg.renorm)
    x = L["x"].astype(np.float64)
    wg = L["w_gate"].astype(np.float64)
    for t in range(0, cfg.T, 7):
        logits = np.array([np.float32(math.fsum(x[t] * wg[e])) for e in range(cfg.E)])
        order = sorted(range(cfg.E), key=lambda e: (-float(logits[e]), e))[:cfg.k]
        assert out["topk_idx"][t].tolist() == order
        ex = np.exp(logits.astype(np.float64) - float(logits.max()))
        p = ex / ex.sum()
        w = np.array([p[e] for e in order])
        w = (w / w.sum()).astype(np.float32).astype(np.float64)
        y = np.zeros(cfg.d)
        for j, e in enumerate(order):
            g = L["w1"][e].astype(np.float64) @ x[t]
            u = L["w3"][e].astype(np.float64) @ x[t]
            y += w[j] * (L["w2"][e].astype(np.float64) @ (g / (1 + np.exp(-g)) * u))
        assert np.allclose(out["y"][t], y, rtol=1e-9, atol=1e-20)
    assert out["counts"].sum() == cfg.A


# ----------------------------------------------------------------------------- degenerate cases
def test_degenerate_all_to_one_expert_and_single_token_and_k1():
    cfg, L = tiny_layer(T=19, E=5, k=1, dtype=si.F32)
    bias = np.zeros(5, np.float32); bias[2] = 1e9
    out = orc.moe_layer(L["x"], L["w_gate"], L["w1"], L["w3"], L["w2"], 1, 1, bias)
    assert out["counts"].tolist() == [0, 0, 19, 0, 0]
    assert out["offsets"].tolist() == [0, 0, 0, 19, 19, 19]
    assert np.array_equal(out["dst_row"], np.arange(19))
    want = orc.expert_ffn(L["x"], L["w1"][2], L["w3"][2], L["w2"][2])
    assert np.allclose(out["y"], want, rtol=1e-12)
    one = orc.moe_layer(L["x"][:1], L["w_gate"], L["w1"], L["w3"], L["w2"], 2, 1)
    assert one["y"].shape == (1, cfg.d) and one["counts"].sum() == 2


def test_topk_margin_hand_worked_and_scalar_sort():
    """The margin is pinned by values worked out by hand and by a scalar sort per row: the gap
    between the last chosen and the first rejected score, over the row's largest magnitude."""
    score = np.array([[4.0, -8.0, 1.0, 3.0],      # sorted 4 3 1 -8, scale 8
                      [0.5, 0.5, 0.25, -1.0],     # a tie at the top, scale 1
                      [-2.0, -3.0, -5.0, -4.0],   # all negative: sorted -2 -3 -4 -5, scale 5
                      [0.0, 0.0, 0.0, 0.0]],      # all-zero row: gap 0 (the scale floor avoids 0/0)
                     dtype=np.float32)
    assert orc.topk_margin(score, 1).tolist() == [1 / 8, 0.0, 1 / 5, 0.0]
    assert orc.topk_margin(score, 2).tolist() == [2 / 8, 0.25, 1 / 5, 0.0]
    assert orc.topk_margin(score, 3).tolist() == [9 / 8, 1.25, 1 / 5, 0.0]
    assert np.all(np.isinf(orc.topk_margin(score, 4))) and np.all(orc.topk_margin(score, 4) > 0)
    # scalar sort on random rows with repeated values, every k
    rng = np.random.default_rng(11)
    score = (rng.integers(-6, 7, size=(60, 7)) / 4).astype(np.float32)
    for k in range(1, 7):
        got = orc.topk_margin(score, k)
        for t in range(score.shape[0]):
            desc = sorted((float(v) for v in score[t]), reverse=True)
            scale = max(max(abs(v) for v in desc), 1e-30)
            assert got[t] == (desc[k - 1] - desc[k]) / scale
    # the margin is the gap that separates what topk_select keeps from what it drops
    for k in (1, 3, 6):
        idx = orc.topk_select(score, k)
        for t in range(score.shape[0]):
            kept = score[t, idx[t]].astype(np.float64)
            dropped = np.delete(score[t], idx[t]).astype(np.float64)
            scale = max(np.abs(score[t]).max(), 1e-30)
            assert orc.topk_margin(score, k)[t] == (kept.min() - dropped.max()) / scale

    # planted slips: the gap one position early / late, or a scale taken from the signed maximum
    def slipped(shift, signed_scale=False):
        def f(score, k):
            s = np.sort(score.astype(np.float64), axis=1)[:, ::-1]
            scale = score.max(axis=1) if signed_scale else np.abs(score).max(axis=1)
            return (s[:, k - 1 + shift] - s[:, k + shift]) / np.maximum(scale.astype(np.float64), 1e-30)
        return f
    hand = np.array([[4.0, -8.0, 1.0, 3.0]], dtype=np.float32)
    assert slipped(-1)(hand, 2)[0] != 2 / 8 and slipped(1)(hand, 2)[0] != 2 / 8
    assert slipped(0, True)(hand, 2)[0] != 2 / 8 and slipped(0)(hand, 2)[0] == 2 / 8


def test_named_workloads_match_the_stored_margin_file(repo_root):
    import os
    rows = {}
    with open(os.path.join(repo_root, "tests", "golden", "route_margins.txt")) as f:
        for line in f:
            if not line.startswith("#"):
                p = line.split()
                rows[p[0]] = p
    # the file is regenerated whenever a workload is added: it lists every named one
    assert set(rows) == set(si.CONFIGS)
    for name, p in rows.items():
        assert int(p[1]) == si.CONFIGS[name].seed
    for name in ("tiny", "decode", "mixtral"):
        cfg = si.CONFIGS[name]
        L = si.make_layer(cfg, parts=("x", "w_gate"))
        idx, _, score = orc.route(L["x"], L["w_gate"], cfg.k, cfg.renorm, L["gate_bias"])
        counts, _ = orc.expert_load(idx, cfg.E)
        assert int(rows[name][1]) == cfg.seed
        assert abs(orc.topk_margin(score, cfg.k).min() - float(rows[name][2])) < 1e-9
        assert int(rows[name][5]) == int((counts == 0).sum())
    # the skewed layer: hottest expert near the 95%-of-tokens target (15.8% of T*k),
    # and its empty-tail variant really has four empty experts
    assert abs(float(rows["skew"][4]) - 0.95 / 6) < 2e-3
    assert int(rows["skew_empty"][5]) == 4


def test_paper_shape_facts(repo_root):
    """Byte accounting the paper prints (tests/golden/paper_facts.txt)."""
    import os
    facts = {}
    with open(os.path.join(repo_root, "tests", "golden", "paper_facts.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                key, val = line.split("=", 1)
                facts[key.strip()] = val.split("#")[0].strip()
    cfg = si.CONFIGS["mixtral"]
    expert_bytes = 3 * cfg.d * cfg.F * cfg.itemsize
    assert abs(expert_bytes / 2 ** 30 - float(facts["mixtral_expert_gb"])) < 0.005
    assert (cfg.k, cfg.E) == tuple(int(v) for v in facts["mixtral_active_total"].split("/"))
    # largest gate/predictor = 80 K parameters = a bias-free d x E linear map (5120 x 16)
    assert abs(5120 * 16 - float(facts["largest_gate_params"])) / 81920 < 0.03
    # the other two models of Table 1: widths come from the public model configurations; the
    # experts (three d x F matrices each) must account for most of the printed parameter totals
    for name, layers, total in (("phi", "phi_layers", "phi_params_total_b"),
                                ("llama4", "llama4_layers", "llama4_params_total_b")):
        c = si.CONFIGS[name]
        experts = 3 * c.d * c.F * c.E * int(facts[layers]) / 1e9
        assert 0.85 * float(facts[total]) <= experts <= float(facts[total])
    assert (si.CONFIGS["phi"].k, si.CONFIGS["phi"].E) == tuple(int(v) for v in facts["phi_active_total"].split("/"))
    assert (si.CONFIGS["llama4"].k, si.CONFIGS["llama4"].E) == tuple(
        int(v) for v in facts["llama4_active_total"].split("/"))


# ----------------------------------------------------------------------------- planted mistakes
def _layer_with(monkeypatch, **patches):
    for name, fn in patches.items():
        monkeypatch.setattr(orc, name, fn)


def test_planted_mistakes_are_caught(monkeypatch):
    """Each plausible slip, planted in the oracle, must break a pin above."""
    rng = np.random.default_rng(21)
    T, d, E, k, F = 33, 12, 4, 2, 20
    x = rng.standard_normal((T, d)).astype(np.float32); x[:, 0] = 1.0
    wg = rng.standard_normal((E, d)).astype(np.float32)
    w1, w3, w2 = (np.stack([m] * E) for m in identity_expert(d, F))

    def layer_err():
        out = orc.moe_layer(x, wg, w1, w3, w2, k, renorm=1)
        return np.abs(out["y"] - x).max()

    assert layer_err() < 1e-6
    good_ffn, good_combine, good_silu = orc.expert_ffn, orc.combine, orc.silu

    # (1) W1 and W3 swapped
    monkeypatch.setattr(orc, "expert_ffn",
                        lambda r, a, b, c, return_h=False: good_ffn(r, b, a, c, return_h))
    assert layer_err() > 1e-2
    monkeypatch.setattr(orc, "expert_ffn", good_ffn)
    # (2) sign slip in silu
    monkeypatch.setattr(orc, "silu", lambda z: z / (1.0 + np.exp(z)))
    assert layer_err() > 1e-2
    monkeypatch.setattr(orc, "silu", good_silu)
    # (3) combine forgets the permutation (reads rows in assignment order)
    monkeypatch.setattr(orc, "combine",
                        lambda yp, dst, w: good_combine(yp, np.arange(dst.size, dtype=np.int32), w))
    xr = rng.standard_normal((T, d)).astype(np.float32)
    out = orc.moe_layer(xr, wg, *(rng.standard_normal(s.shape) for s in (w1, w3, w2)), k, 1)
    monkeypatch.setattr(orc, "combine", good_combine)
    ref = good_combine(out["y_perm"], out["dst_row"], out["topk_w"])
    assert np.abs(out["y"] - ref).max() > 1e-3
    # (4) a transposed gate operand cannot even be formed for E != d; with E == d it is caught
    #     by the scalar-loop pin; (5) unstable permutation is caught by the argsort pin:
    idx = np.array([[1, 0], [1, 0], [0, 1]], dtype=np.int32)
    dst, src = orc.permutation(idx, 2)
    assert src.tolist() == [1, 3, 4, 0, 2, 5]
