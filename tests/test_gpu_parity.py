"""GPU parity: every C-ABI call against the CPU oracle, element by element, on seeded
inputs.  Each call is first tested alone with oracle-made inputs (so one stage's
parity does not lean on another's), then the four calls are chained.

Bars: indices, counts, offsets and both permutation maps bit-exact; x_perm bit-exact
(a copy); routing weights 1e-5 relative; scores 1e-5 of the row's largest magnitude;
h, y_perm, y within max|gpu - ref| / max|ref| <= 2e-2 (bf16) or 1e-4 (fp32).
"""
import numpy as np
import pytest

import synth_inputs as si
from oracle import moe_oracle as orc

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from paper_2603_06350_amd import binding as B  # noqa: E402
from paper_2603_06350_amd import layer  # noqa: E402


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    B.load()


def tol_of(dtype):
    return 1e-4 if dtype == si.F32 else 2e-2


def rel_err(got, ref):
    ref = np.asarray(ref, dtype=np.float64)
    scale = np.abs(ref).max()
    return float(np.abs(np.asarray(got, dtype=np.float64) - ref).max() / (scale if scale > 0 else 1.0))


def dev(a):
    return layer.to_device(a)


def host(t):
    return layer.to_host(t)


def shape_of(cfg):
    return B.make_shape(cfg.T, cfg.d, cfg.E, cfg.k, cfg.F, cfg.dtype, cfg.renorm)


def tdtype(cfg):
    return torch.float32 if cfg.dtype == si.F32 else torch.bfloat16


# ----------------------------------------------------------------------------- route
def gpu_route(cfg, x, w_gate, bias):
    T, E, k = cfg.T, cfg.E, cfg.k
    idx = torch.full((T, k), -1, dtype=torch.int32, device="cuda")
    w = torch.zeros((T, k), dtype=torch.float32, device="cuda")
    sc = torch.zeros((T, E), dtype=torch.float32, device="cuda")
    B.moe_route(shape_of(cfg), dev(x), dev(w_gate), dev(bias), idx, w, sc)
    torch.cuda.synchronize()
    return host(idx), host(w), host(sc)


def check_route(cfg, x, w_gate, bias):
    idx, w, sc = gpu_route(cfg, x, w_gate, bias)
    ridx, rw, rsc = orc.route(x, w_gate, cfg.k, cfg.renorm, bias)
    row_scale = np.maximum(np.abs(rsc).max(axis=1, keepdims=True), 1e-30)
    assert (np.abs(sc - rsc) / row_scale).max() <= 1e-5
    bad = np.nonzero((idx != ridx).any(axis=1))[0]
    assert bad.size == 0, f"{cfg.name}: top-k differs on rows {bad[:8]} gpu {idx[bad[:3]]} ref {ridx[bad[:3]]}"
    assert np.abs(w - rw).max() <= 1e-5 * max(1e-30, np.abs(rw).max())
    assert np.all(np.abs(w - rw) <= 1e-5 * np.abs(rw) + 1e-9)
    return idx, w


ROUTE_CASES = [
    dict(T=300, d=256, E=8, k=2, renorm=1),
    dict(T=1000, d=512, E=64, k=6, renorm=0),
    dict(T=77, d=1024, E=128, k=8, renorm=1),
    dict(T=130, d=264, E=200, k=5, renorm=1),     # d not a multiple of 32, E > 128
    dict(T=50, d=64, E=16, k=1, renorm=1),        # k = 1 (Llama-4-Scout style)
    dict(T=33, d=128, E=4, k=4, renorm=0),        # k = E
    dict(T=1, d=4096, E=8, k=2, renorm=1),        # one token
    dict(T=40, d=96, E=24, k=3, renorm=1, dtype=si.F32),
]


@pytest.mark.parametrize("case", ROUTE_CASES, ids=lambda c: "T{T}_d{d}_E{E}_k{k}".format(**c))
def test_route_matches_oracle(case):
    cfg = si.small_config(F=64, **case)
    L = si.make_layer(cfg, parts=("x", "w_gate"))
    check_route(cfg, L["x"], L["w_gate"], None)


def test_route_exact_ties_go_to_lowest_index():
    cfg = si.small_config(T=200, d=256, E=16, k=4, F=64)
    L = si.make_layer(cfg, parts=("x", "w_gate"))
    wg = L["w_gate"].copy()
    wg[9] = wg[2]
    wg[13] = wg[2]
    check_route(cfg, L["x"], wg, None)
    idx, w = check_route(cfg, np.zeros_like(L["x"]), wg, None)
    assert np.array_equal(idx, np.tile(np.arange(4, dtype=np.int32), (cfg.T, 1)))


def test_route_with_bias_and_forced_expert():
    cfg = si.small_config(T=150, d=256, E=64, k=6, F=64, renorm=0)
    L = si.make_layer(cfg, parts=("x", "w_gate"))
    bias = np.linspace(-2, 2, 64).astype(np.float32)
    check_route(cfg, L["x"], L["w_gate"], bias)
    bias[5] = 1e9
    bias[60:] = -1e9
    idx, _ = check_route(cfg, L["x"], L["w_gate"], bias)
    assert np.all(idx[:, 0] == 5) and idx.max() < 60


def test_route_near_ties_are_decided_like_the_oracle():
    # experts 1 and 3 share their weights and differ by a 1e-6 bias: their scores are a few
    # fp32 ulps apart, which a differently ordered fp32 sum cannot resolve but the exact pass must
    cfg = si.small_config(T=256, d=512, E=8, k=2, F=64)
    L = si.make_layer(cfg, parts=("x", "w_gate"))
    wg = L["w_gate"].copy()
    wg[3] = wg[1]
    bias = np.zeros(8, dtype=np.float32)
    bias[3] = 1e-6
    _, _, rsc = orc.route(L["x"], wg, 2, 1, bias)
    m = orc.topk_margin(rsc, 2)
    assert ((m < 1e-4) & (m > 0)).sum() > 5     # near-ties (not exact ties) at the k-th place
    check_route(cfg, L["x"], wg, bias)
    bias[3] = -1e-6
    check_route(cfg, L["x"], wg, bias)


def cancelling_tokens(T, d, E, seed):
    """bf16 inputs whose large terms cancel: the first 3/8 of a token are A*u, the next 3/8 are
    -A*u, against gate rows that repeat the same positive vector on both parts, so those products
    add up to exactly zero; the logit is what the last quarter contributes, thousands of times
    smaller than the partial sums on the way.  Experts 2i and 2i+1 differ in one element of the last
    quarter by one bf16 step: their logits are a hair apart, which is larger depends on the token,
    and every token's leading experts are such a pair."""
    rng = np.random.default_rng(seed)
    m = 3 * d // 8
    u = np.abs(rng.standard_normal((T, m), dtype=np.float32)) * 16.0
    sig = rng.standard_normal((T, d - 2 * m), dtype=np.float32) * 0.02
    x = si.f32_to_bf16_bits(np.concatenate([u, -u, sig], axis=1))
    x[:, m:2 * m] = x[:, :m] ^ np.uint16(0x8000)              # exactly the negated bf16 values
    c = np.abs(rng.standard_normal(m, dtype=np.float32)) / 16.0
    g = rng.standard_normal((E, d - 2 * m), dtype=np.float32) / 32.0
    g[1::2] = g[0::2]
    wg = si.f32_to_bf16_bits(np.concatenate([np.tile(c, (E, 1)), np.tile(c, (E, 1)), g], axis=1))
    wg[1::2, 2 * m + 5] += 1                                 # one bf16 step in one element
    return x, wg


@pytest.mark.parametrize("T,d,E,k,ws", [
    (200, 1024, 8, 2, False),      # per-tile kernel
    (2000, 1024, 8, 2, False),     # large-batch kernel, 2 tiles per block
    (3000, 1024, 64, 6, False),    # ... 64 experts
    (100, 1024, 128, 8, True),     # gate product as a kernel of its own, norms through the workspace
    (40, 2048, 256, 8, False),     # per-tile kernel, 256 experts (grouped norm tiles)
])
def test_route_when_large_terms_cancel(T, d, E, k, ws):
    """The fast pass's rounding errors follow the size of the terms it adds, not of their sum: a
    margin taken from the logits would let these tokens through with the wrong order."""
    cfg = si.small_config(T=T, d=d, E=E, k=k, F=64, renorm=1)
    x, wg = cancelling_tokens(T, d, E, seed=77)
    ridx, rw, rsc = orc.route(x, wg, k, 1, None)
    # not vacuous: the gap between experts 0 and 1 is far below what an fp32 sum of these terms
    # can resolve, and both orders occur
    gap = np.abs(rsc[:, 0] - rsc[:, 1])
    xf, wf = si.bf16_bits_to_f32(x), si.bf16_bits_to_f32(wg)
    part = np.abs(np.cumsum(xf[:8].astype(np.float64) * wf[0].astype(np.float64), axis=1)).max(axis=1)
    assert np.all(gap[:8] > 0) and np.all(gap[:8] < part * 2.0 ** -24)
    assert 0.2 < (rsc[:, 0] > rsc[:, 1]).mean() < 0.8
    if ws:
        idx, w, sc = gpu_route_ws(cfg, x, wg, None, True, True)
    else:
        idx, w, sc = gpu_route(cfg, x, wg, None)
    bad = np.nonzero((idx != ridx).any(axis=1))[0]
    assert bad.size == 0, f"top-k differs on rows {bad[:8]} gpu {idx[bad[:3]]} ref {ridx[bad[:3]]}"
    assert np.all(np.abs(w - rw) <= 1e-5 * np.abs(rw) + 1e-9)


# Batches large enough for the large-batch routing kernel (from 96 blocks of 2, 4 or 8 token tiles on;
# gate matrices of at most 128 KB take the fewest tiles per block, larger ones the most that still
# give 256 blocks; 4 or 8 tiles for 65 to 128 experts, 4 for more; k <= 16, whole 64-element stages
# per slice of the hidden dimension).  The hidden size is small so that the oracle stays fast,
# except where only a large gate matrix reaches a form.  T is never a multiple of the block.
BIG_ROUTE_CASES = [
    dict(T=8195, d=256, E=64, k=6, renorm=1),      # 2 tiles per block, 4 slices
    dict(T=8200, d=512, E=40, k=8, renorm=0),      # experts not a multiple of 16
    dict(T=8193, d=256, E=5, k=5, renorm=1),       # k = E
    dict(T=9000, d=768, E=16, k=16, renorm=0),     # the largest k this path takes, k = E
    dict(T=16400, d=256, E=16, k=1, renorm=1),     # 4 tiles per block, 2 slices
    dict(T=16390, d=384, E=33, k=3, renorm=1),
    dict(T=32800, d=128, E=8, k=2, renorm=1),
    dict(T=33000, d=64, E=64, k=15, renorm=0),     # one stage
    dict(T=32800, d=5120, E=16, k=1, renorm=0),    # 160 KB gate matrix: 8 tiles per block, up to 16 experts
    dict(T=16400, d=5120, E=16, k=2, renorm=1),    # ... 4 tiles per block
    dict(T=32800, d=2304, E=32, k=4, renorm=1),    # 8 tiles per block, up to 32 experts
    dict(T=32800, d=1088, E=64, k=6, renorm=0),    # 8 tiles per block, up to 64 experts
    dict(T=16400, d=256, E=128, k=8, renorm=1),    # more than 64 experts: 4 tiles per block only
    dict(T=16390, d=128, E=100, k=6, renorm=0),
    dict(T=16400, d=256, E=65, k=16, renorm=1),
    dict(T=32800, d=128, E=100, k=6, renorm=1),    # 8 tiles per block with more than 64 experts
    dict(T=16400, d=256, E=256, k=8, renorm=1),    # the most experts the library takes
    dict(T=16390, d=128, E=200, k=6, renorm=0),
    dict(T=3100, d=2048, E=64, k=6, renorm=1),     # 256 KB gate matrix: taken from 96 blocks on
    dict(T=6200, d=1024, E=128, k=8, renorm=0),
    dict(T=16400, d=192, E=8, k=2, renorm=1),      # slices would not be whole stages: per-tile kernel
    dict(T=8195, d=256, E=32, k=17, renorm=1),     # k too large for it: per-tile kernel
]


@pytest.mark.parametrize("case", BIG_ROUTE_CASES, ids=lambda c: "T{T}_d{d}_E{E}_k{k}".format(**c))
def test_route_large_batch_matches_oracle(case):
    cfg = si.small_config(F=64, **case)
    L = si.make_layer(cfg, parts=("x", "w_gate"))
    check_route(cfg, L["x"], L["w_gate"], None)
    bias = np.linspace(-1.5, 1.5, cfg.E).astype(np.float32)
    check_route(cfg, L["x"], L["w_gate"], bias)


@pytest.mark.parametrize("T,E", [(8195, 32), (16400, 32), (32800, 32), (16400, 128), (32800, 128),
                                 (16400, 256)])
def test_route_large_batch_ties_and_near_ties(T, E):
    # duplicated gate rows (exact ties), all-zero tokens (every score equal: more candidates than
    # the exact pass lists, so all experts are re-scored), a 1e-6 bias between two equal rows
    # (near-ties that only the exact pass resolves), experts masked by a huge negative bias
    cfg = si.small_config(T=T, d=256, E=E, k=4, F=64)
    L = si.make_layer(cfg, parts=("x", "w_gate"))
    x, wg = L["x"].copy(), L["w_gate"].copy()
    wg[9] = wg[2]
    wg[13] = wg[2]
    wg[30] = wg[17]
    x[::7] = 0
    idx, _ = check_route(cfg, x, wg, None)
    assert np.array_equal(idx[::7], np.tile(np.arange(4, dtype=np.int32), (idx[::7].shape[0], 1)))
    bias = np.zeros(E, dtype=np.float32)
    bias[13] = 1e-6
    bias[30] = -1e-6
    _, _, rsc = orc.route(x, wg, 4, 1, bias)
    m = orc.topk_margin(rsc, 4)
    assert ((m < 1e-4) & (m > 0)).sum() > 5
    check_route(cfg, x, wg, bias)
    bias[20:] = -1e9
    bias[3] = 1e9
    idx, _ = check_route(cfg, x, wg, bias)
    assert np.all(idx[:, 0] == 3) and idx.max() < 20


def test_route_large_batch_without_scores_output():
    cfg = si.small_config(T=8200, d=256, E=64, k=6, F=64)
    L = si.make_layer(cfg, parts=("x", "w_gate"))
    idx = torch.full((cfg.T, cfg.k), -1, dtype=torch.int32, device="cuda")
    w = torch.zeros((cfg.T, cfg.k), dtype=torch.float32, device="cuda")
    B.moe_route(shape_of(cfg), dev(L["x"]), dev(L["w_gate"]), None, idx, w, None)
    torch.cuda.synchronize()
    ridx, rw, _ = orc.route(L["x"], L["w_gate"], cfg.k, cfg.renorm, None)
    assert np.array_equal(host(idx), ridx)
    assert np.all(np.abs(host(w) - rw) <= 1e-5 * np.abs(rw) + 1e-9)


# Small batches with a gate matrix of at least 256 KB: with a workspace (or a score output) the
# gate product runs as a kernel of its own over the whole chip and the selection reads its scores.
SMALL_ROUTE_WS_CASES = [
    dict(T=32, d=4096, E=128, k=8, renorm=1),      # the decode-shaped layer's routing
    dict(T=77, d=1024, E=128, k=8, renorm=0),      # exactly 256 KB
    dict(T=130, d=2056, E=200, k=5, renorm=1),     # ragged hidden size, E > 128, E % 16 != 0
    dict(T=512, d=2048, E=64, k=6, renorm=1),
    dict(T=2048, d=1024, E=128, k=8, renorm=1),    # enough token tiles for 64-expert gate tiles
    dict(T=3000, d=520, E=256, k=8, renorm=0),     # more than 128 experts, ragged hidden size
    dict(T=1, d=4096, E=33, k=33, renorm=1),       # one token, k = E
]


def gpu_route_ws(cfg, x, w_gate, bias, with_ws, with_scores):
    T, E, k = cfg.T, cfg.E, cfg.k
    sh = shape_of(cfg)
    idx = torch.full((T, k), -1, dtype=torch.int32, device="cuda")
    w = torch.zeros((T, k), dtype=torch.float32, device="cuda")
    sc = torch.full((T, E), -3.0, dtype=torch.float32, device="cuda") if with_scores else None
    nb = B.moe_workspace_bytes(sh)
    assert nb >= T * E * 4 or T >= 8192     # room for the scores of every batch that can use them
    ws = torch.full((nb,), 0x5A, dtype=torch.uint8, device="cuda") if with_ws else None
    B.moe_route_ws(sh, dev(x), dev(w_gate), dev(bias), idx, w, sc, ws, nb if with_ws else 0)
    torch.cuda.synchronize()
    return host(idx), host(w), (host(sc) if with_scores else None)


@pytest.mark.parametrize("case", SMALL_ROUTE_WS_CASES, ids=lambda c: "T{T}_d{d}_E{E}_k{k}".format(**c))
def test_route_with_workspace_matches_oracle_and_plain_route(case):
    cfg = si.small_config(F=64, **case)
    L = si.make_layer(cfg, parts=("x", "w_gate"))
    x, wg = L["x"].copy(), L["w_gate"].copy()
    wg[cfg.E - 1] = wg[0]                           # an exact tie between the first and the last expert
    x[cfg.T // 2] = 0                               # and a token whose scores are all equal
    bias = np.linspace(-1.0, 1.0, cfg.E).astype(np.float32)
    for b in (None, bias):
        ridx, rw, rsc = orc.route(x, wg, cfg.k, cfg.renorm, b)
        pidx, pw, psc = gpu_route(cfg, x, wg, b)    # moe_route: one kernel
        assert np.array_equal(pidx, ridx)
        for with_ws, with_scores in ((True, False), (False, True), (True, True)):
            idx, w, sc = gpu_route_ws(cfg, x, wg, b, with_ws, with_scores)
            assert np.array_equal(idx, ridx), (with_ws, with_scores)
            assert np.all(np.abs(w - rw) <= 1e-5 * np.abs(rw) + 1e-9)
            # the two forms take the choice on the same fast scores and re-score near-ties exactly;
            # which tokens count as near-ties may differ in the last bits of the margin, so weights
            # and scores agree to the oracle's tolerance rather than bit for bit
            assert np.all(np.abs(w - pw) <= 1e-5 * np.abs(pw) + 1e-9)
            if with_scores:
                assert np.all(np.abs(sc - psc) <= 1e-5 * np.abs(psc).max(axis=1, keepdims=True))


def test_route_ws_without_usable_workspace_is_plain_route():
    cfg = si.small_config(T=32, d=4096, E=128, k=8, F=64)
    L = si.make_layer(cfg, parts=("x", "w_gate"))
    ridx, rw, _ = orc.route(L["x"], L["w_gate"], cfg.k, cfg.renorm, None)
    idx = torch.full((cfg.T, cfg.k), -1, dtype=torch.int32, device="cuda")
    w = torch.zeros((cfg.T, cfg.k), dtype=torch.float32, device="cuda")
    small = torch.zeros((256,), dtype=torch.uint8, device="cuda")       # too small: ignored
    B.moe_route_ws(shape_of(cfg), dev(L["x"]), dev(L["w_gate"]), None, idx, w, None, small, 256)
    torch.cuda.synchronize()
    assert np.array_equal(host(idx), ridx)
    assert np.all(np.abs(host(w) - rw) <= 1e-5 * np.abs(rw) + 1e-9)


def test_route_ws_with_room_for_the_scores_but_not_the_norms_is_plain_route():
    # the two-kernel form needs T*E scores and T + E norms: a workspace of exactly T*E*4 bytes is
    # not enough for it, and the call must behave like moe_route
    cfg = si.small_config(T=48, d=2048, E=128, k=8, F=64)
    L = si.make_layer(cfg, parts=("x", "w_gate"))
    ridx, rw, _ = orc.route(L["x"], L["w_gate"], cfg.k, cfg.renorm, None)
    idx = torch.full((cfg.T, cfg.k), -1, dtype=torch.int32, device="cuda")
    w = torch.zeros((cfg.T, cfg.k), dtype=torch.float32, device="cuda")
    nb = cfg.T * cfg.E * 4
    ws = torch.full((nb + 256,), 0x5A, dtype=torch.uint8, device="cuda")
    B.moe_route_ws(shape_of(cfg), dev(L["x"]), dev(L["w_gate"]), None, idx, w, None, ws, nb)
    torch.cuda.synchronize()
    assert np.array_equal(host(idx), ridx)
    assert np.all(np.abs(host(w) - rw) <= 1e-5 * np.abs(rw) + 1e-9)
    assert bool((ws[nb:] == 0x5A).all())            # nothing written past the size it was given


# ----------------------------------------------------------------------------- count + permute
def gpu_dispatch(cfg, x, idx):
    T, E, k, d = cfg.T, cfg.E, cfg.k, cfg.d
    sh = shape_of(cfg)
    A = T * k
    counts = torch.full((E,), -7, dtype=torch.int32, device="cuda")
    offsets = torch.full((E + 1,), -7, dtype=torch.int32, device="cuda")
    dst = torch.full((max(A, 1),), -7, dtype=torch.int32, device="cuda")
    src = torch.full((max(A, 1),), -7, dtype=torch.int32, device="cuda")
    xp = torch.zeros((max(A, 1), d), dtype=tdtype(cfg), device="cuda")
    nb = B.moe_workspace_bytes(sh)
    ws = torch.full((nb,), 0x5A, dtype=torch.uint8, device="cuda")   # garbage on entry
    B.moe_count_and_permute(sh, dev(x), dev(idx), counts, offsets, dst, src, xp, ws, nb)
    torch.cuda.synchronize()
    return host(counts), host(offsets), host(dst)[:A], host(src)[:A], host(xp)[:A]


def check_dispatch(cfg, x, idx):
    counts, offsets, dst, src, xp = gpu_dispatch(cfg, x, idx)
    rc, ro = orc.expert_load(idx, cfg.E)
    rd, rs = orc.permutation(idx, cfg.E)
    assert np.array_equal(counts, rc)
    assert np.array_equal(offsets, ro)
    assert np.array_equal(dst, rd)
    assert np.array_equal(src, rs)
    assert np.array_equal(xp, orc.permute_rows(x, rd, cfg.k))
    assert counts.sum() == cfg.T * cfg.k


DISPATCH_CASES = [
    dict(T=300, d=256, E=8, k=2),
    dict(T=1000, d=128, E=64, k=6),       # several blocks of 256 tokens, ragged tail
    dict(T=513, d=64, E=128, k=8),
    dict(T=700, d=72, E=256, k=3),        # 128-thread variant, row not a multiple of 64 B
    dict(T=1, d=4096, E=8, k=2),
    dict(T=40, d=96, E=24, k=3, dtype=si.F32),
    dict(T=128, d=64, E=16, k=2),         # 256 assignments: the largest single-launch dispatch
    dict(T=512, d=64, E=16, k=2),         # 1024 assignments: two launches
    dict(T=86, d=64, E=16, k=3),          # 258: the smallest that takes the general path
    dict(T=32, d=64, E=256, k=8),         # single launch, most experts
]


@pytest.mark.parametrize("case", DISPATCH_CASES, ids=lambda c: "T{T}_d{d}_E{E}_k{k}".format(**c))
def test_count_and_permute_matches_oracle(case):
    cfg = si.small_config(F=64, **case)
    L = si.make_layer(cfg, parts=("x", "w_gate"))
    idx, _, _ = orc.route(L["x"], L["w_gate"], cfg.k, cfg.renorm)
    check_dispatch(cfg, L["x"], idx)


def test_count_and_permute_degenerate_loads():
    cfg = si.small_config(T=600, d=64, E=16, k=2, F=64)
    L = si.make_layer(cfg, parts=("x",))
    idx = np.zeros((cfg.T, 2), dtype=np.int32)
    idx[:, 0], idx[:, 1] = 7, 3                       # two experts take everything, 14 are empty
    check_dispatch(cfg, L["x"], idx)
    rng = np.random.default_rng(0)
    idx = rng.integers(0, 16, size=(cfg.T, 2)).astype(np.int32)   # a token may repeat an expert
    check_dispatch(cfg, L["x"], idx)
    cfg1 = si.small_config(T=600, d=64, E=16, k=1, F=64)
    check_dispatch(cfg1, L["x"], np.full((cfg.T, 1), 15, dtype=np.int32))
    # the same degenerate loads in a batch small enough for the single-launch dispatch
    cfg2 = si.small_config(T=120, d=64, E=16, k=2, F=64)
    L2 = si.make_layer(cfg2, parts=("x",))
    idx = np.zeros((cfg2.T, 2), dtype=np.int32)
    idx[:, 0], idx[:, 1] = 7, 3
    check_dispatch(cfg2, L2["x"], idx)
    idx = np.random.default_rng(1).integers(0, 16, size=(cfg2.T, 2)).astype(np.int32)   # repeats
    check_dispatch(cfg2, L2["x"], idx)


def test_count_and_permute_no_tokens():
    cfg = si.small_config(T=0, d=64, E=8, k=2, F=64)
    sh = shape_of(cfg)
    counts = torch.full((8,), -7, dtype=torch.int32, device="cuda")
    offsets = torch.full((9,), -7, dtype=torch.int32, device="cuda")
    nb = B.moe_workspace_bytes(sh)
    ws = torch.empty((nb,), dtype=torch.uint8, device="cuda")
    B.moe_count_and_permute(sh, None, None, counts, offsets, None, None, None, ws, nb)
    torch.cuda.synchronize()
    assert host(counts).tolist() == [0] * 8 and host(offsets).tolist() == [0] * 9


# ----------------------------------------------------------------------------- grouped FFN
def gpu_ffn(cfg, x_perm, offsets, w1, w3, w2):
    A = cfg.T * cfg.k
    h = torch.zeros((A, cfg.F), dtype=tdtype(cfg), device="cuda")
    yp = torch.zeros((A, cfg.d), dtype=tdtype(cfg), device="cuda")
    args = (dev(x_perm), None, dev(offsets), dev(w1), dev(w3), dev(w2))
    B.moe_grouped_ffn(shape_of(cfg), args[0], *args[2:], h, yp)
    # Inputs this small leave the last (only) round of tiles under-filled, so the call above cuts
    # its tiles along the rows into pieces; with 4 added to `parts` every tile stays whole, which is
    # how the tiles of a full-size batch run.  Both forms are checked: same bits, and the caller
    # compares them with the oracle.
    h_whole, yp_whole = torch.zeros_like(h), torch.zeros_like(yp)
    B.moe_grouped_ffn_ws(shape_of(cfg), *args, h_whole, yp_whole, 3 | 4, None, 0)
    torch.cuda.synchronize()
    assert torch.equal(h, h_whole), "h differs between cut and whole tiles"
    assert torch.equal(yp, yp_whole), "y_perm differs between cut and whole tiles"
    return orc.to_f64(host(h)), orc.to_f64(host(yp))


def check_ffn(cfg, L, idx):
    _, offsets = orc.expert_load(idx, cfg.E)
    dst, _ = orc.permutation(idx, cfg.E)
    x_perm = orc.permute_rows(L["x"], dst, cfg.k)
    ry, rh = orc.grouped_ffn(x_perm, offsets, L["w1"], L["w3"], L["w2"], return_h=True)
    h, yp = gpu_ffn(cfg, x_perm, offsets, L["w1"], L["w3"], L["w2"])
    tol = tol_of(cfg.dtype)
    assert rel_err(h, rh) <= tol, f"h: {rel_err(h, rh):.3e}"
    assert rel_err(yp, ry) <= tol, f"y_perm: {rel_err(yp, ry):.3e}"
    # per-row check too: a wrong row hiding behind a large global scale would show here
    row_scale = np.abs(ry).max(axis=1) + 1e-30
    assert (np.abs(yp - ry).max(axis=1) / row_scale).max() <= 4 * tol
    return x_perm, offsets, dst


FFN_CASES = [
    dict(T=300, d=256, E=8, k=2, F=384),          # MFMA path, 75 rows/expert: 64-row tiles only, ragged
    dict(T=600, d=256, E=8, k=2, F=384),          # 150 rows/expert: partial 256-row tiles + remainders
    dict(T=1500, d=128, E=2, k=1, F=256),         # MFMA path, 256-row tiles (>= 512 rows/expert)
    dict(T=900, d=192, E=3, k=2, F=320),          # 256-row tiles, N tails (320 = 2.5 x 128, 192 < 256)
    dict(T=64, d=512, E=64, k=6, F=128),          # many small / empty experts
    dict(T=100, d=200, E=4, k=2, F=104),          # bf16 generic path (d, F not multiples of 64)
    dict(T=64, d=128, E=8, k=2, F=256, dtype=si.F32, x_std=0.02, w_std=0.02),
    dict(T=45, d=36, E=5, k=2, F=52, dtype=si.F32),
]


def test_grouped_ffn_few_rows_per_expert_with_one_hot_expert():
    # few rows per expert on average (everything runs as 64-row tiles in one launch per GEMM),
    # but one expert holds several tiles' worth of rows and most are empty
    cfg = si.small_config(T=400, d=256, E=64, k=1, F=384)
    L = si.make_layer(cfg)
    rng = np.random.default_rng(5)
    idx = np.where(rng.random((cfg.T, 1)) < 0.8, 5, rng.integers(0, 64, size=(cfg.T, 1))).astype(np.int32)
    counts, _ = orc.expert_load(idx, cfg.E)
    assert counts[5] > 4 * 64 and (counts == 0).sum() > 10
    check_ffn(cfg, L, idx)


@pytest.mark.parametrize("case", FFN_CASES, ids=lambda c: "T{T}_d{d}_E{E}_k{k}_F{F}".format(**c))
def test_grouped_ffn_matches_oracle(case):
    cfg = si.small_config(**case)
    L = si.make_layer(cfg)
    idx, _, _ = orc.route(L["x"], L["w_gate"], cfg.k, cfg.renorm)
    check_ffn(cfg, L, idx)


@pytest.mark.parametrize("d,F", [(64, 704), (128, 640), (192, 576), (256, 512), (320, 448), (384, 384)])
def test_grouped_ffn_every_stage_count_of_the_two_stage_pipeline(d, F):
    # K stages of 64 elements: the up-projection takes d / 64 of them and the down-projection F / 64,
    # so the six cases run the even tiles' two-buffer pipeline over 1 to 11 stages (prologue only,
    # odd and even counts); the experts hold one tile of 256 rows (every wave four sub-tiles), one of
    # 300 rows (19 sub-tiles: waves with five and with four) and two tiles of 224 rows (waves with
    # four and with three sub-tiles)
    cfg = si.small_config(T=1000, d=d, E=3, k=1, F=F)
    L = si.make_layer(cfg)
    idx = np.zeros((cfg.T, 1), dtype=np.int32)
    idx[:256] = 0
    idx[256:256 + 300] = 1
    idx[556:] = 2
    check_ffn(cfg, L, idx)


@pytest.mark.parametrize("rows", [1, 15, 16, 17, 47, 64, 65, 130, 255, 257, 319, 320, 321, 336, 641, 1000])
def test_grouped_ffn_even_tiles_every_wave_share(rows):
    # one hot expert with `rows` rows among experts of 128 rows (so that the mean stays above the
    # even tiles' threshold): its tiles give the waves every count of sub-tiles from 0 to 5, tiles
    # below and at the 320-row limit, and segments that need two or three tiles; both ways of
    # sharing the loads among the waves (the threshold on the mean rows per expert picks one)
    for E, others in ((3, 600), (9, 150)):             # mean rows per expert above / below 384
        cfg = si.small_config(T=rows + (E - 1) * others, d=128, E=E, k=1, F=256, seed=rows + E)
        L = si.make_layer(cfg)
        idx = np.zeros((cfg.T, 1), dtype=np.int32)
        idx[:rows] = 1
        pos = rows
        for e in range(E):
            if e != 1:
                idx[pos:pos + others] = e
                pos += others
        check_ffn(cfg, L, idx)


ROUND_CASES = [
    # (rows per expert, d, F): enough tiles for whole rounds of the chip's 256 compute units plus a
    # last round that is under-filled (its tiles are cut along their rows), just over half full
    # (left whole) or absent; every element of h and y_perm is compared
    ([2048] * 8, 128, 640),                      # up 280 tiles (1 round + 24), down 56 (a fifth of a round)
    ([1500] * 16, 512, 384),                     # up 240 (under a round, whole tiles), down 160
    ([3000, 17, 0, 2500, 64, 700, 1, 4000, 0, 333, 2100, 65, 1290, 1280, 320, 321], 256, 1152),
    ([1024] * 9, 1024, 512),                     # up 144, down 144: just over half a round, not cut
    ([640] * 40, 128, 896),                      # up 560 (2 rounds + 48), down 80
]


@pytest.mark.parametrize("rows,d,F", ROUND_CASES, ids=lambda v: str(v) if isinstance(v, int) else f"E{len(v)}")
def test_grouped_ffn_whole_rounds_and_under_filled_last_rounds(rows, d, F):
    cfg = si.small_config(T=sum(rows), d=d, E=len(rows), k=1, F=F, seed=len(rows) + d + F)
    L = si.make_layer(cfg)
    idx = np.repeat(np.arange(len(rows), dtype=np.int32), rows).reshape(-1, 1)
    check_ffn(cfg, L, idx)


SPLIT_CASES = [
    # (shape, whether some tile must have been split); a GEMM is eligible from K = 6144 on
    (dict(T=600, d=1024, E=2, k=1, F=6144), True),    # even tiles, down-projection cut in 4
    (dict(T=64, d=1024, E=4, k=2, F=6144), True),     # 64-row tiles only (32 rows per expert)
    (dict(T=600, d=6144, E=2, k=1, F=256), True),     # up-projection (gated) cut in 4
    (dict(T=700, d=1024, E=2, k=1, F=6144, seed=11), None),   # 350 rows per expert: two even tiles of 176 rows each
    (dict(T=300, d=1024, E=2, k=1, F=2048), False),   # reductions too short: exactly the plain call
]


@pytest.mark.parametrize("case,expect_split", SPLIT_CASES,
                         ids=lambda c: "T{T}_d{d}_E{E}_k{k}_F{F}".format(**c) if isinstance(c, dict) else "")
@pytest.mark.parametrize("gathered", [False, True])
def test_grouped_ffn_with_split_tiles(case, expect_split, gathered):
    """moe_grouped_ffn_ws: tiles of an under-filled last round are computed in parts along K and
    added up by the launch after the GEMM.  Oracle parity, run-to-run identical bits whatever the
    workspace held before, rows within a bf16 step of the call without a workspace; where the
    case says so, the split did happen (some bits differ) or cannot (identical bits)."""
    cfg = si.small_config(**case)
    L = si.make_layer(cfg)
    idx, _, _ = orc.route(L["x"], L["w_gate"], cfg.k, cfg.renorm)
    _, offsets = orc.expert_load(idx, cfg.E)
    dst, src = orc.permutation(idx, cfg.E)
    x_perm = orc.permute_rows(L["x"], dst, cfg.k)
    ry, rh = orc.grouped_ffn(x_perm, offsets, L["w1"], L["w3"], L["w2"], return_h=True)
    sh = shape_of(cfg)
    A = cfg.T * cfg.k
    nb = B.moe_ffn_workspace_bytes(sh)
    d_x = dev(L["x"]) if gathered else dev(x_perm)
    d_src = dev(src) if gathered else None
    d_off, w1, w3, w2 = dev(offsets), dev(L["w1"]), dev(L["w3"]), dev(L["w2"])
    outs = []
    for fill in (0, 0x7F):                           # 0x7F7F7F7F is a large finite float: stale data would show
        ws = torch.full((nb,), fill, dtype=torch.uint8, device="cuda")
        h = torch.zeros((A, cfg.F), dtype=tdtype(cfg), device="cuda")
        yp = torch.zeros((A, cfg.d), dtype=tdtype(cfg), device="cuda")
        B.moe_grouped_ffn_ws(sh, d_x, d_src, d_off, w1, w3, w2, h, yp, 3, ws, nb)
        torch.cuda.synchronize()
        outs.append((h, yp))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])
    h, yp = outs[0]
    tol = tol_of(cfg.dtype)
    assert rel_err(orc.to_f64(host(h)), rh) <= tol
    assert rel_err(orc.to_f64(host(yp)), ry) <= tol
    # against the call without a workspace: the same rows up to the grouping of the fp32 sum
    h0 = torch.zeros_like(h)
    y0 = torch.zeros_like(yp)
    B.moe_grouped_ffn_ws(sh, d_x, d_src, d_off, w1, w3, w2, h0, y0, 3, None, 0)
    torch.cuda.synchronize()
    assert (h.float() - h0.float()).abs().max().item() <= 2.0 ** -7 * h0.float().abs().max().item()
    assert (yp.float() - y0.float()).abs().max().item() <= 2.0 ** -6 * y0.float().abs().max().item()
    same = torch.equal(h, h0) and torch.equal(yp, y0)
    if expect_split is True:
        assert not same, "no tile was split"
    elif expect_split is False:
        assert same


def test_grouped_ffn_skewed_and_empty_experts():
    cfg = si.small_config(T=700, d=128, E=8, k=2, F=256)
    L = si.make_layer(cfg)
    idx = np.zeros((cfg.T, 2), dtype=np.int32)
    idx[:, 0] = 2                                     # 700 rows: 256-row tiles with a tail
    idx[:, 1] = np.where(np.arange(cfg.T) < 5, 6, 4)  # 5 rows and 695 rows; 5 experts empty
    check_ffn(cfg, L, idx)


def test_identity_experts_reproduce_the_input_on_gpu():
    # closed form: W1 rows = c*e0, W3 = [I;0], W2 = [I/silu(c), 0]  =>  E(x) = x when x[:,0] = 1
    T, d, E, k, F = 200, 128, 4, 2, 192
    cfg = si.small_config(T=T, d=d, E=E, k=k, F=F, dtype=si.F32)
    L = si.make_layer(cfg, parts=("x", "w_gate"))
    x = L["x"].copy()
    x[:, 0] = 1.0
    c = 1.5
    s0 = c / (1.0 + np.exp(-c))
    w1 = np.zeros((E, F, d), np.float32); w1[:, :, 0] = c
    w3 = np.zeros((E, F, d), np.float32); w3[:, :d, :d] = np.eye(d)
    w2 = np.zeros((E, d, F), np.float32); w2[:, :d, :d] = np.eye(d) / s0
    buf = layer.MoeBuffers(T, d, E, k, F, cfg.dtype, 1)
    buf.forward(dev(x), dev(L["w_gate"]), dev(w1), dev(w3), dev(w2))
    torch.cuda.synchronize()
    assert rel_err(host(buf.y), x) <= 1e-5


# ----------------------------------------------------------------------------- combine
@pytest.mark.parametrize("case", [dict(T=300, d=256, E=8, k=2), dict(T=257, d=1032, E=64, k=6),
                                  dict(T=31, d=4096, E=128, k=8),
                                  dict(T=40, d=100, E=6, k=3, dtype=si.F32)],
                         ids=lambda c: "T{T}_d{d}_k{k}".format(**c))
def test_combine_matches_oracle(case):
    cfg = si.small_config(F=64, **case)
    L = si.make_layer(cfg, parts=("x", "w_gate"))
    idx, w, _ = orc.route(L["x"], L["w_gate"], cfg.k, cfg.renorm)
    dst, _ = orc.permutation(idx, cfg.E)
    # any rows will do as "expert outputs": draw them with the generator
    yp = si.make_layer(si.small_config(T=cfg.A, d=cfg.d, E=1, k=1, F=8, dtype=cfg.dtype, seed=99),
                       parts=("x",))["x"]
    y = torch.zeros((cfg.T, cfg.d), dtype=tdtype(cfg), device="cuda")
    B.moe_combine(shape_of(cfg), dev(yp), dev(dst), dev(w), y)
    torch.cuda.synchronize()
    ref = orc.combine(yp, dst, w)
    assert rel_err(orc.to_f64(host(y)), ref) <= (1e-6 if cfg.dtype == si.F32 else 4e-3)


# ----------------------------------------------------------------------------- whole layer
LAYER_CASES = [
    si.CONFIGS["tiny"],
    si.small_config("bf16_small", T=300, d=256, E=8, k=2, F=384),
    si.small_config("bf16_fine", T=500, d=256, E=64, k=6, F=128, renorm=0),
    si.small_config("bf16_big_tiles", T=1400, d=128, E=2, k=2, F=256),
    si.small_config("bf16_decode_like", T=32, d=512, E=128, k=8, F=192),
    si.small_config("bf16_skew", T=600, d=256, E=64, k=6, F=128, renorm=0, zipf_alpha=1.2,
                    zipf_scale=0.9, empty_tail=4),
    si.small_config("bf16_limits", T=100, d=128, E=256, k=64, F=64),       # the largest E and k
    si.small_config("bf16_top1", T=700, d=128, E=16, k=1, F=192),          # one expert per token
    si.small_config("bf16_all_experts", T=150, d=128, E=8, k=8, F=64, renorm=0),   # k = E
    si.small_config("bf16_many_tokens", T=20000, d=64, E=8, k=2, F=64),    # many dispatch blocks
    si.small_config("f32_odd", T=130, d=100, E=12, k=3, F=52, dtype=si.F32),
]


@pytest.mark.parametrize("cfg", LAYER_CASES, ids=lambda c: c.name)
def test_layer_end_to_end(cfg):
    L = si.make_layer(cfg)
    ref = orc.moe_layer(L["x"], L["w_gate"], L["w1"], L["w3"], L["w2"], cfg.k, cfg.renorm,
                        L["gate_bias"])
    buf = layer.MoeBuffers(cfg.T, cfg.d, cfg.E, cfg.k, cfg.F, cfg.dtype, cfg.renorm)
    args = [dev(L[n]) for n in ("x", "w_gate", "w1", "w3", "w2")]
    buf.forward(*args, gate_bias=dev(L["gate_bias"]), export_scores=True)
    torch.cuda.synchronize()
    first = {n: host(getattr(buf, n)).copy() for n in
             ("topk_idx", "topk_w", "counts", "offsets", "dst_row", "src_assign", "x_perm", "h",
              "y_perm", "y")}
    for n in ("topk_idx", "counts", "offsets", "dst_row", "src_assign", "x_perm"):
        assert np.array_equal(first[n], ref[n]), n
    assert np.all(np.abs(first["topk_w"] - ref["topk_w"]) <= 1e-5 * ref["topk_w"] + 1e-9)
    tol = tol_of(cfg.dtype)
    for n in ("h", "y_perm", "y"):
        e = rel_err(orc.to_f64(first[n]), ref[n])
        assert e <= tol, f"{n}: {e:.3e}"
    assert first["counts"].sum() == cfg.A
    # determinism: a second run gives the same bits everywhere
    buf.forward(*args, gate_bias=dev(L["gate_bias"]), export_scores=True)
    torch.cuda.synchronize()
    for n, v in first.items():
        assert np.array_equal(host(getattr(buf, n)), v), f"{n} differs between two runs"


def test_layer_replays_from_a_hip_graph():
    """The four calls captured into one HIP graph replay to the eager bits.  Eager work and
    synchronisations sit between the replays; no call allocates or clears memory."""
    cfg = si.small_config("bf16_graph", T=1400, d=128, E=2, k=2, F=256)
    L = si.make_layer(cfg)
    buf = layer.MoeBuffers(cfg.T, cfg.d, cfg.E, cfg.k, cfg.F, cfg.dtype, cfg.renorm)
    args = [dev(L[n]) for n in ("x", "w_gate", "w1", "w3", "w2")]
    bias = dev(L["gate_bias"])
    names = ("topk_idx", "topk_w", "counts", "offsets", "dst_row", "src_assign", "x_perm", "h",
             "y_perm", "y")
    buf.forward(*args, gate_bias=bias)
    torch.cuda.synchronize()
    eager = {n: host(getattr(buf, n)).copy() for n in names}
    ref = orc.moe_layer(L["x"], L["w_gate"], L["w1"], L["w3"], L["w2"], cfg.k, cfg.renorm,
                        L["gate_bias"])
    assert rel_err(orc.to_f64(eager["y"]), ref["y"]) <= tol_of(cfg.dtype)

    graph = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        buf.forward(*args, gate_bias=bias)          # first use of this stream happens outside the capture
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=s):
        buf.forward(*args, gate_bias=bias)
    torch.cuda.synchronize()
    for rep in range(3):
        for n in names:                             # eager fills between the replays
            getattr(buf, n).zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for n in names:
            assert np.array_equal(host(getattr(buf, n)), eager[n]), f"replay {rep}: {n} differs"


def test_layer_with_split_tiles_replays_from_a_hip_graph():
    """The layer with the split-tile workspace (the down-projection's tiles cut along K, summed by
    the launch after the GEMM) captured into a HIP graph: every replay gives the eager bits, with
    the workspace overwritten between the replays."""
    cfg = si.small_config("bf16_graph_split", T=64, d=256, E=4, k=2, F=6144)
    L = si.make_layer(cfg)
    buf = layer.MoeBuffers(cfg.T, cfg.d, cfg.E, cfg.k, cfg.F, cfg.dtype, cfg.renorm, split_tiles=True)
    plain = layer.MoeBuffers(cfg.T, cfg.d, cfg.E, cfg.k, cfg.F, cfg.dtype, cfg.renorm)
    args = [dev(L[n]) for n in ("x", "w_gate", "w1", "w3", "w2")]
    names = ("topk_idx", "counts", "dst_row", "h", "y_perm", "y")
    buf.forward(*args)
    plain.forward(*args)
    torch.cuda.synchronize()
    eager = {n: host(getattr(buf, n)).copy() for n in names}
    ref = orc.moe_layer(L["x"], L["w_gate"], L["w1"], L["w3"], L["w2"], cfg.k, cfg.renorm, None)
    assert rel_err(orc.to_f64(eager["y"]), ref["y"]) <= tol_of(cfg.dtype)
    assert not np.array_equal(eager["y_perm"], host(plain.y_perm)), "no tile was split"
    graph = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        buf.forward(*args)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=s):
        buf.forward(*args)
    torch.cuda.synchronize()
    for rep in range(3):
        for n in names:
            getattr(buf, n).zero_()
        buf.ffn_ws.fill_(0x7F)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for n in names:
            assert np.array_equal(host(getattr(buf, n)), eager[n]), f"replay {rep}: {n} differs"


@pytest.mark.parametrize("cfg", LAYER_CASES, ids=lambda c: c.name)
def test_ffn_reading_x_through_the_permutation_gives_the_same_bits(cfg):
    """moe_grouped_ffn_gather (no x_perm) against moe_grouped_ffn on the materialised x_perm."""
    L = si.make_layer(cfg)
    buf = layer.MoeBuffers(cfg.T, cfg.d, cfg.E, cfg.k, cfg.F, cfg.dtype, cfg.renorm)
    args = [dev(L[n]) for n in ("x", "w_gate", "w1", "w3", "w2")]
    bias = dev(L["gate_bias"])
    buf.forward(*args, gate_bias=bias)
    torch.cuda.synchronize()
    want = {n: host(getattr(buf, n)).copy() for n in ("src_assign", "h", "y_perm", "y")}
    for n in ("x_perm", "h", "y_perm", "y"):
        getattr(buf, n).zero_()
    buf.forward(*args, gate_bias=bias, gather_in_ffn=True)
    torch.cuda.synchronize()
    for n, v in want.items():
        assert np.array_equal(host(getattr(buf, n)), v), n
    assert not host(buf.x_perm).any()                   # x_perm was not touched
    ref = orc.moe_layer(L["x"], L["w_gate"], L["w1"], L["w3"], L["w2"], cfg.k, cfg.renorm,
                        L["gate_bias"])
    assert rel_err(orc.to_f64(host(buf.y)), ref["y"]) <= tol_of(cfg.dtype)


def test_ffn_gather_rejects_missing_map_and_survives_bad_entries():
    cfg = si.small_config("gather_bad", T=200, d=128, E=4, k=2, F=128)
    L = si.make_layer(cfg)
    buf = layer.MoeBuffers(cfg.T, cfg.d, cfg.E, cfg.k, cfg.F, cfg.dtype, cfg.renorm)
    args = [dev(L[n]) for n in ("x", "w_gate", "w1", "w3", "w2")]
    buf.forward(*args, gather_in_ffn=True)
    with pytest.raises(B.MoeError):
        B.moe_grouped_ffn_gather(buf.shape, args[0], None, buf.offsets, args[2], args[3], args[4],
                                 buf.h, buf.y_perm)
    # entries outside [0, T*k) are clamped to a valid row: values unspecified, no fault
    bad = buf.src_assign.clone()
    bad[::7] = 1 << 30
    bad[3::11] = -5
    B.moe_grouped_ffn_gather(buf.shape, args[0], bad, buf.offsets, args[2], args[3], args[4], buf.h,
                             buf.y_perm)
    torch.cuda.synchronize()
    assert np.isfinite(orc.to_f64(host(buf.y_perm))).all()


def test_two_host_threads_on_two_streams():
    """The header promises that calls from several host threads are independent (the library keeps
    no state of its own).  Two threads, each with its own stream and buffers, run the layer
    repeatedly at the same time; every result equals the one obtained alone."""
    import threading
    cfgs = [si.small_config("thr_a", T=1400, d=128, E=2, k=2, F=256),
            si.small_config("thr_b", T=900, d=256, E=4, k=2, F=128, seed=11)]
    jobs = []
    for cfg in cfgs:
        L = si.make_layer(cfg)
        args = [dev(L[n]) for n in ("x", "w_gate", "w1", "w3", "w2")]
        buf = layer.MoeBuffers(cfg.T, cfg.d, cfg.E, cfg.k, cfg.F, cfg.dtype, cfg.renorm)
        buf.forward(*args)
        torch.cuda.synchronize()
        jobs.append((cfg, args, buf, host(buf.y).copy(), torch.cuda.Stream()))
    errors = []

    def run(job):
        cfg, args, buf, want, stream = job
        try:
            for it in range(20):
                with torch.cuda.stream(stream):
                    buf.y.zero_()
                    buf.forward(*args, stream=stream, gather_in_ffn=bool(it & 1))
                stream.synchronize()
                if not np.array_equal(host(buf.y), want):
                    errors.append(f"{cfg.name}: iteration {it} differs")
                    return
        except Exception as exc:  # noqa: BLE001
            errors.append(f"{cfg.name}: {exc!r}")

    threads = [threading.Thread(target=run, args=(j,)) for j in jobs]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=100)
    assert not any(t.is_alive() for t in threads), "a thread did not finish"
    assert not errors, errors


# ----------------------------------------------------------------------------- k = 1: combine in the FFN
@pytest.mark.parametrize("cfg", [
    si.small_config("k1_even", T=1500, d=256, E=3, k=1, F=384, renorm=0),       # even tiles, several per expert
    si.small_config("k1_ring", T=300, d=128, E=8, k=1, F=256, renorm=0, seed=5),  # ring tiles
    si.small_config("k1_odd", T=200, d=96, E=4, k=1, F=160, renorm=0, seed=6),  # bf16, no MFMA shape
    si.small_config("k1_f32", T=150, d=64, E=4, k=1, F=96, dtype=si.F32, renorm=0, seed=7),
], ids=lambda c: c.name)
def test_ffn_with_the_combine_folded_in_for_one_expert_per_token(cfg):
    """moe_grouped_ffn_combine_k1 against the oracle's layer and against the two-call form (which
    rounds y_perm before the weight is applied: at most one more rounding)."""
    L = si.make_layer(cfg)
    ref = orc.moe_layer(L["x"], L["w_gate"], L["w1"], L["w3"], L["w2"], cfg.k, cfg.renorm, L["gate_bias"])
    args = [dev(L[n]) for n in ("x", "w_gate", "w1", "w3", "w2")]
    buf = layer.MoeBuffers(cfg.T, cfg.d, cfg.E, cfg.k, cfg.F, cfg.dtype, cfg.renorm)
    buf.forward(*args, gather_in_ffn=True)
    torch.cuda.synchronize()
    two_calls = orc.to_f64(host(buf.y))
    h_two = host(buf.h).copy()
    buf.y.zero_()
    buf.y_perm.fill_(7)                              # must stay untouched
    buf.forward(*args, combine_in_ffn=True)
    torch.cuda.synchronize()
    fused = orc.to_f64(host(buf.y))
    assert np.array_equal(host(buf.topk_idx), ref["topk_idx"])
    assert np.array_equal(host(buf.h), h_two)
    assert (orc.to_f64(host(buf.y_perm)) == 7).all()
    tol = tol_of(cfg.dtype)
    assert rel_err(fused, ref["y"]) <= tol
    row_scale = np.abs(ref["y"]).max(axis=1) + 1e-30
    assert (np.abs(fused - ref["y"]).max(axis=1) / row_scale).max() <= 4 * tol
    # one rounding of the storage type apart from the two-call form, element by element
    ulp = 2.0 ** -8 if cfg.dtype == si.BF16 else 2.0 ** -23
    assert np.all(np.abs(fused - two_calls) <= 2 * ulp * np.abs(two_calls) + 1e-30)
    # every row of y was written
    assert (np.abs(fused).max(axis=1) > 0).all()


def test_ffn_combine_k1_rejects_layers_with_more_experts_per_token():
    cfg = si.small_config("k2", T=64, d=64, E=4, k=2, F=64)
    buf = layer.MoeBuffers(cfg.T, cfg.d, cfg.E, cfg.k, cfg.F, cfg.dtype, cfg.renorm)
    z = torch.zeros((cfg.E, cfg.F, cfg.d), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(B.MoeError) as err:
        B.moe_grouped_ffn_combine_k1(buf.shape, buf.y, buf.src_assign, buf.offsets, z, z, z, buf.topk_w,
                                     buf.h, buf.y)
    assert err.value.code == -2
