"""GPU parity at the full sizes of the five named workloads, in the launch configurations
bench.py times (the calls chained on one stream, buffers from MoeBuffers; both the four-call form
with a written x_perm and the default form in which the FFN reads x through the permutation map).

Routing, expert load and the permutation are compared with the full oracle on every
token (the oracle's routing is cheap at any size).  The expert FFN and the combine are
compared on sampled tokens: for every sampled token the oracle computes the k expert
outputs (h row, y_perm row) one by one from the same input bytes and combines them.
On top of the random tokens, rows are chosen by where they sit in their expert's segment, because
that is what decides which tile, which wave and which launch computes them at full size: the
first and the last row of every segment, the two rows either side of every multiple of 16 rows
inside it (every possible tile and sub-tile boundary, whatever the tile height), the whole tail
of the segment past its last multiple of 256 rows (and at least its last 64 rows), and every row
of the smallest non-empty and of the largest expert.  Each of those rows is compared (h and
y_perm) on its own scale.
The decode-shaped layer is small enough for the full oracle.
"""
import numpy as np
import pytest

import synth_inputs as si
from oracle import moe_oracle as orc

torch = pytest.importorskip("torch")
pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]

from paper_2603_06350_amd import binding as B  # noqa: E402
from paper_2603_06350_amd import layer  # noqa: E402


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    B.load()


def run_layer(cfg, L):
    dev = {n: layer.to_device(L[n]) for n in ("x", "w_gate", "w1", "w3", "w2")}
    buf = layer.MoeBuffers(cfg.T, cfg.d, cfg.E, cfg.k, cfg.F, cfg.dtype, cfg.renorm)
    bias = layer.to_device(L["gate_bias"])
    # the four-call form first (it writes x_perm, which check_routing_and_dispatch compares) ...
    buf.forward(dev["x"], dev["w_gate"], dev["w1"], dev["w3"], dev["w2"], gate_bias=bias,
                export_scores=True)
    torch.cuda.synchronize()
    first = {n: getattr(buf, n).clone() for n in ("h", "y_perm", "y")}
    for n in first:
        getattr(buf, n).zero_()
    # ... then the form bench.py times by default: the up-projection reads x through the permutation
    # map.  Its outputs, which the sampled checks below look at, must be the same bits.
    buf.forward(dev["x"], dev["w_gate"], dev["w1"], dev["w3"], dev["w2"], gate_bias=bias,
                export_scores=True, gather_in_ffn=True)
    torch.cuda.synchronize()
    for n, v in first.items():
        assert torch.equal(getattr(buf, n), v), f"{n} differs between the two forms of the FFN call"
    return buf


def check_routing_and_dispatch(cfg, L, buf):
    ridx, rw, rsc = orc.route(L["x"], L["w_gate"], cfg.k, cfg.renorm, L["gate_bias"])
    idx = layer.to_host(buf.topk_idx)
    bad = np.nonzero((idx != ridx).any(axis=1))[0]
    assert bad.size == 0, f"top-k differs on {bad.size} rows, first {bad[:5]}"
    w = layer.to_host(buf.topk_w)
    assert np.all(np.abs(w - rw) <= 1e-5 * np.abs(rw) + 1e-9)
    if cfg.renorm:
        assert np.abs(w.sum(axis=1) - 1.0).max() <= 1e-5
    sc = layer.to_host(buf.scores)
    finite = np.abs(rsc) < 1e8                      # forced-empty experts sit at -1e9
    scale = np.maximum(np.abs(np.where(finite, rsc, 0)).max(axis=1, keepdims=True), 1e-30)
    assert (np.abs(sc - rsc) * finite / scale).max() <= 1e-5
    rc, ro = orc.expert_load(ridx, cfg.E)
    rd, rs = orc.permutation(ridx, cfg.E)
    counts = layer.to_host(buf.counts)
    assert np.array_equal(counts, rc) and counts.sum() == cfg.A
    assert np.array_equal(layer.to_host(buf.offsets), ro)
    assert np.array_equal(layer.to_host(buf.dst_row), rd)
    assert np.array_equal(layer.to_host(buf.src_assign), rs)
    xp = layer.to_host(buf.x_perm)
    x = L["x"]
    assert np.array_equal(xp[rd.reshape(cfg.T, cfg.k)[:, 0]], x)     # slot 0 of every token
    assert np.array_equal(xp[rd], np.repeat(x, cfg.k, axis=0))       # every assignment
    return ridx, rw, ro, rd


def check_sampled_outputs(cfg, L, buf, ridx, rw, rd, n_tokens, seed=0):
    rng = np.random.default_rng(seed)
    toks = np.unique(np.concatenate([[0, cfg.T - 1], rng.integers(0, cfg.T, size=n_tokens)]))
    rows = rd.reshape(cfg.T, cfg.k)[toks]                    # [S,k] rows in expert order
    experts = ridx[toks]
    h_gpu = buf.h[torch.from_numpy(rows.reshape(-1).astype(np.int64)).cuda()]
    yp_gpu = buf.y_perm[torch.from_numpy(rows.reshape(-1).astype(np.int64)).cuda()]
    h_gpu = orc.to_f64(layer.to_host(h_gpu)).reshape(len(toks), cfg.k, cfg.F)
    yp_gpu = orc.to_f64(layer.to_host(yp_gpu)).reshape(len(toks), cfg.k, cfg.d)
    h_ref = np.zeros_like(h_gpu)
    yp_ref = np.zeros_like(yp_gpu)
    for e in np.unique(experts):
        s, j = np.nonzero(experts == e)
        y, h = orc.expert_ffn(L["x"][toks[s]], L["w1"][e], L["w3"][e], L["w2"][e], return_h=True)
        h_ref[s, j], yp_ref[s, j] = h, y
    y_ref = np.einsum("sj,sjd->sd", rw[toks].astype(np.float64), yp_ref)
    y_gpu = orc.to_f64(layer.to_host(buf.y[torch.from_numpy(toks.astype(np.int64)).cuda()]))
    tol = 1e-4 if cfg.dtype == si.F32 else 2e-2
    for name, g, r in (("h", h_gpu, h_ref), ("y_perm", yp_gpu, yp_ref), ("y", y_gpu, y_ref)):
        err = np.abs(g - r).max() / np.abs(r).max()
        assert err <= tol, f"{name}: max rel err {err:.3e}"
    # every sampled row on its own scale, so one bad row cannot hide behind a large one
    row_err = np.abs(y_gpu - y_ref).max(axis=1) / (np.abs(y_ref).max(axis=1) + 1e-30)
    assert row_err.max() <= 4 * tol


def structural_rows(offsets, E):
    """Permuted rows picked by their position in the expert's segment (see the module text)."""
    counts = np.diff(offsets)
    nonempty = np.nonzero(counts > 0)[0]
    whole = {int(nonempty[np.argmin(counts[nonempty])]), int(np.argmax(counts))}
    rows, experts = [], []
    for e in range(E):
        lo, c = int(offsets[e]), int(counts[e])
        if c == 0:
            continue
        if e in whole:
            rel = np.arange(c)
        else:
            b = np.arange(16, c, 16)
            tail = np.arange(min((c // 256) * 256, max(c - 64, 0)), c)
            rel = np.unique(np.concatenate([[0, c - 1], b - 1, b, tail]))
        rows.append(lo + rel)
        experts.append(np.full(rel.size, e))
    return np.concatenate(rows), np.concatenate(experts)


def check_structural_rows(cfg, L, buf, ro, rs):
    rows, experts = structural_rows(ro, cfg.E)
    sel = torch.from_numpy(rows.astype(np.int64)).cuda()
    h_gpu = orc.to_f64(layer.to_host(buf.h[sel]))
    yp_gpu = orc.to_f64(layer.to_host(buf.y_perm[sel]))
    toks = rs[rows] // cfg.k
    tol = 1e-4 if cfg.dtype == si.F32 else 2e-2
    worst = {"h": 0.0, "y_perm": 0.0}
    scale = {"h": 0.0, "y_perm": 0.0}
    for e in np.unique(experts):
        m = experts == e
        y_ref, h_ref = orc.expert_ffn(L["x"][toks[m]], L["w1"][e], L["w3"][e], L["w2"][e], return_h=True)
        for name, g, r in (("h", h_gpu[m], h_ref), ("y_perm", yp_gpu[m], y_ref)):
            row_err = np.abs(g - r).max(axis=1) / (np.abs(r).max(axis=1) + 1e-30)
            bad = np.nonzero(row_err > 4 * tol)[0]
            assert bad.size == 0, (f"{name}: expert {e}, segment row {rows[m][bad[0]] - ro[e]} of "
                                   f"{ro[e + 1] - ro[e]}: rel err {row_err[bad[0]]:.3e} on the row's scale")
            worst[name] = max(worst[name], float(np.abs(g - r).max()))
            scale[name] = max(scale[name], float(np.abs(r).max()))
    for name in worst:
        assert worst[name] <= tol * scale[name], f"{name}: max rel err {worst[name] / scale[name]:.3e}"
    return rows.size


@pytest.mark.parametrize("name,n_tokens", [("mixtral", 40), ("finegrained", 48), ("skew", 48),
                                           ("skew_empty", 24), ("phi", 24), ("llama4", 16)])
def test_full_size_sampled(name, n_tokens):
    cfg = si.CONFIGS[name]
    print(f"workload {name}: generating", flush=True)
    L = si.make_layer(cfg)
    print("running the layer", flush=True)
    buf = run_layer(cfg, L)
    print("checking routing and dispatch", flush=True)
    ridx, rw, ro, rd = check_routing_and_dispatch(cfg, L, buf)
    if name == "skew_empty":
        assert (layer.to_host(buf.counts)[-4:] == 0).all()
    print("checking sampled expert outputs", flush=True)
    check_sampled_outputs(cfg, L, buf, ridx, rw, rd, n_tokens)
    print("checking rows chosen by their place in the expert's segment", flush=True)
    n = check_structural_rows(cfg, L, buf, ro, layer.to_host(buf.src_assign))
    print(f"{n} of {cfg.A} permuted rows compared one by one", flush=True)
    # property that holds at any size: all of y is finite and no row was left unwritten
    y = buf.y.float()
    assert torch.isfinite(y).all() and (y.abs().amax(dim=1) > 0).all()
    if cfg.k == 1:
        # one expert per token: the form with the combine folded into the down-projection's store
        # gives, at full size, the two-call form's y up to one rounding of the storage type
        print("the combine folded into the grouped FFN", flush=True)
        dev = {n: layer.to_device(L[n]) for n in ("x", "w_gate", "w1", "w3", "w2")}
        two_calls = buf.y.float().clone()
        buf.y.zero_()
        buf.forward(dev["x"], dev["w_gate"], dev["w1"], dev["w3"], dev["w2"],
                    gate_bias=layer.to_device(L["gate_bias"]), combine_in_ffn=True)
        torch.cuda.synchronize()
        fused = buf.y.float()
        assert bool((fused - two_calls).abs().le(2.0 ** -7 * two_calls.abs() + 1e-30).all())
        assert (fused.abs().amax(dim=1) > 0).all()


@pytest.mark.parametrize("name", ["tiny", "decode"])
def test_full_size_full_oracle(name):
    cfg = si.CONFIGS[name]
    print(f"workload {name}: generating", flush=True)
    L = si.make_layer(cfg)
    buf = run_layer(cfg, L)
    print("full oracle", flush=True)
    ref = orc.moe_layer(L["x"], L["w_gate"], L["w1"], L["w3"], L["w2"], cfg.k, cfg.renorm,
                        L["gate_bias"])
    for n in ("topk_idx", "counts", "offsets", "dst_row", "src_assign", "x_perm"):
        assert np.array_equal(layer.to_host(getattr(buf, n)), ref[n]), n
    assert np.all(np.abs(layer.to_host(buf.topk_w) - ref["topk_w"]) <= 1e-5 * ref["topk_w"] + 1e-9)
    tol = 1e-4 if cfg.dtype == si.F32 else 2e-2
    for n in ("h", "y_perm", "y"):
        got = orc.to_f64(layer.to_host(getattr(buf, n)))
        err = np.abs(got - ref[n]).max() / np.abs(ref[n]).max()
        assert err <= tol, f"{n}: {err:.3e}"


def test_large_batch_route_permute_combine():
    """The bandwidth-bound batch on which bench.py times moe_route_ws, moe_count_and_permute and
    moe_combine one by one (same shape, seed, entry points and workspace): routing and the
    permutation against the full oracle on every token, the copied rows bit for bit, and the
    combine (with the permuted activations standing in for the expert outputs, as in bench.py) on
    sampled tokens and by what holds for every token."""
    import bench
    T, d, E, k = (bench.HBM_BOUND_SHAPE[n] for n in "TdEk")
    cfg = si.small_config("hbm_bound", T=T, d=d, E=E, k=k, F=64, dtype=si.BF16, renorm=1, seed=8008)
    print("generating", flush=True)
    L = si.make_layer(cfg, parts=("x", "w_gate"))
    st = torch.cuda.current_stream()
    sh = B.make_shape(T, d, E, k, 64, B.MOE_BF16, 1)
    A = T * k
    ws_bytes = B.moe_workspace_bytes(sh)
    kw = dict(device="cuda")
    x, wg = layer.to_device(L["x"]), layer.to_device(L["w_gate"])
    topk_idx = torch.empty((T, k), dtype=torch.int32, **kw)
    topk_w = torch.empty((T, k), dtype=torch.float32, **kw)
    counts = torch.empty((E,), dtype=torch.int32, **kw)
    offsets = torch.empty((E + 1,), dtype=torch.int32, **kw)
    dst_row = torch.empty((A,), dtype=torch.int32, **kw)
    src_assign = torch.empty((A,), dtype=torch.int32, **kw)
    x_perm = torch.zeros((A, d), dtype=torch.bfloat16, **kw)
    y = torch.zeros((T, d), dtype=torch.bfloat16, **kw)
    ws = torch.empty((ws_bytes,), dtype=torch.uint8, **kw)
    print("running the three calls", flush=True)
    B.moe_route_ws(sh, x, wg, None, topk_idx, topk_w, None, ws, ws_bytes, st)
    B.moe_count_and_permute(sh, x, topk_idx, counts, offsets, dst_row, src_assign, x_perm, ws,
                            ws_bytes, st)
    B.moe_combine(sh, x_perm, dst_row, topk_w, y, st)
    torch.cuda.synchronize()
    print("oracle routing", flush=True)
    ridx, rw, _ = orc.route(L["x"], L["w_gate"], k, 1)
    bad = np.nonzero((layer.to_host(topk_idx) != ridx).any(axis=1))[0]
    assert bad.size == 0, f"top-k differs on {bad.size} rows, first {bad[:5]}"
    w = layer.to_host(topk_w)
    assert np.all(np.abs(w - rw) <= 1e-5 * np.abs(rw) + 1e-9)
    print("oracle permutation", flush=True)
    rc, ro = orc.expert_load(ridx, E)
    rd, rs = orc.permutation(ridx, E)
    assert np.array_equal(layer.to_host(counts), rc)
    assert np.array_equal(layer.to_host(offsets), ro)
    assert np.array_equal(layer.to_host(dst_row), rd)
    assert np.array_equal(layer.to_host(src_assign), rs)
    xp = layer.to_host(x_perm)
    assert np.array_equal(xp[rd], np.repeat(L["x"], k, axis=0))
    print("oracle combine on sampled tokens", flush=True)
    rng = np.random.default_rng(3)
    toks = np.unique(np.concatenate([[0, T - 1], rng.integers(0, T, size=512)]))
    rows = rd.reshape(T, k)[toks].reshape(-1)
    y_ref = orc.combine(xp[rows], np.arange(rows.size, dtype=np.int32), rw[toks])
    y_gpu = orc.to_f64(layer.to_host(y[torch.from_numpy(toks.astype(np.int64)).cuda()]))
    # fp32 accumulation of k products, one rounding to bf16 on the store
    assert np.all(np.abs(y_gpu - y_ref) <= 2.0 ** -8 * np.abs(y_ref) + 1e-30)
    # for every token: its k permuted rows are copies of x[t] and its weights sum to one, so
    # y[t] is x[t] up to the rounding of the weights' sum and of the store
    yf, xf = y.float(), x.float()
    assert bool((yf - xf).abs().le(2.0 ** -7 * xf.abs() + 1e-30).all())
