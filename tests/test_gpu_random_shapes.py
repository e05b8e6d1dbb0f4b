"""GPU parity on seeded random shapes: the whole layer (both forms of the FFN call) and the routing
call alone (all three kernel forms: per-tile, large-batch, small-batch with a workspace) against
the CPU oracle.  The shapes are drawn from a fixed seed, so every run tests the same cases; they
mix sizes that are and are not multiples of the tile sizes, expert counts that are not multiples
of 16, k = 1 and k = E, skewed gates, duplicated gate rows (exact ties) and all-zero tokens.
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


def layer_cases(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        E = int(rng.choice([1, 2, 3, 8, 16, 17, 40, 64, 100, 128, 200, 256]))
        k = int(min(E, rng.choice([1, 2, 3, 6, 8, 16])))
        mf = rng.random() < 0.7                      # d and F multiples of 64: the MFMA path
        d = int(rng.integers(1, 21)) * 64 if mf else int(rng.integers(2, 40)) * 8
        F = int(rng.integers(1, 21)) * 64 if mf else int(rng.integers(2, 40)) * 8
        T = int(rng.choice([1, 5, 31, 64, 200, 257, 700, 1500]))
        dtype = si.BF16 if rng.random() < 0.8 else si.F32
        if dtype == si.F32:
            d, F = max(4, d // 4 * 4), max(4, F // 4 * 4)
        kw = dict(zipf_alpha=1.2, zipf_scale=0.9) if rng.random() < 0.3 else {}
        out.append(si.small_config(f"rl{i}", T=T, d=d, E=E, k=k, F=F, dtype=dtype,
                                   renorm=int(rng.integers(0, 2)), seed=1000 + i, **kw))
    return out


@pytest.mark.parametrize("cfg", layer_cases(14, 11), ids=lambda c: f"T{c.T}_d{c.d}_E{c.E}_k{c.k}_F{c.F}_t{c.dtype}")
def test_random_layer(cfg):
    L = si.make_layer(cfg)
    ref = orc.moe_layer(L["x"], L["w_gate"], L["w1"], L["w3"], L["w2"], cfg.k, cfg.renorm, L["gate_bias"])
    buf = layer.MoeBuffers(cfg.T, cfg.d, cfg.E, cfg.k, cfg.F, cfg.dtype, cfg.renorm)
    args = [layer.to_device(L[n]) for n in ("x", "w_gate", "w1", "w3", "w2")]
    tol = 1e-4 if cfg.dtype == si.F32 else 2e-2
    for fused in (False, True):
        for n in ("h", "y_perm", "y"):
            getattr(buf, n).zero_()
        buf.forward(*args, gate_bias=layer.to_device(L["gate_bias"]), gather_in_ffn=fused)
        torch.cuda.synchronize()
        for n in ("topk_idx", "counts", "offsets", "dst_row", "src_assign"):
            assert np.array_equal(layer.to_host(getattr(buf, n)), ref[n]), (n, fused)
        for n in ("h", "y_perm", "y"):
            got = orc.to_f64(layer.to_host(getattr(buf, n)))
            scale = np.abs(ref[n]).max()
            err = np.abs(got - ref[n]).max() / (scale if scale > 0 else 1.0)
            assert err <= tol, (n, fused, err)
        # the same call with every tile kept whole (inputs this small leave a round of tiles
        # under-filled, whose tiles the call above cuts along their rows): the same bits
        h, yp = torch.zeros_like(buf.h), torch.zeros_like(buf.y_perm)
        B.moe_grouped_ffn_ws(buf.shape, args[0] if fused else buf.x_perm, buf.src_assign if fused else None,
                             buf.offsets, args[2], args[3], args[4], h, yp, 3 | 4, None, 0)
        torch.cuda.synchronize()
        assert torch.equal(h, buf.h) and torch.equal(yp, buf.y_perm), fused


def route_cases(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        E = int(rng.choice([1, 2, 5, 8, 15, 16, 17, 31, 32, 40, 48, 63, 64, 65, 100, 128, 200]))
        k = int(min(E, rng.choice([1, 2, 3, 6, 8, 15, 16, 17])))
        big = rng.random() < 0.5                     # enough tokens for the large-batch kernel
        if big:
            T = int(rng.choice([8193, 9000, 16385, 17000, 32769, 33000]))
            d = int(rng.choice([64, 128, 192, 256, 384, 512]))
        else:
            T = int(rng.choice([1, 5, 31, 33, 128, 129, 257, 512, 700, 3000]))
            d = int(rng.integers(1, 17)) * 256 if rng.random() < 0.7 else int(rng.integers(1, 40)) * 8
        out.append(dict(T=T, d=d, E=E, k=k, renorm=int(rng.integers(0, 2)), seed=5000 + i,
                        mode=int(rng.integers(0, 4))))
    return out


@pytest.mark.parametrize("case", route_cases(28, 12),
                         ids=lambda c: "T{T}_d{d}_E{E}_k{k}_m{mode}".format(**c))
def test_random_route(case):
    mode = case["mode"]      # 0 plain, 1 skewed gate, 2 exact ties and zero tokens, 3 masked experts
    kw = {}
    if mode == 1:
        kw = dict(zipf_alpha=1.2, zipf_scale=0.9)
    if mode == 3 and case["E"] - case["k"] > 0:
        kw = dict(zipf_alpha=1.2, zipf_scale=0.9, empty_tail=min(4, case["E"] - case["k"]))
    cfg = si.small_config("rr", T=case["T"], d=case["d"], E=case["E"], k=case["k"], F=64,
                          dtype=si.BF16, renorm=case["renorm"], seed=case["seed"], **kw)
    L = si.make_layer(cfg, parts=("x", "w_gate"))
    x, wg = L["x"].copy(), L["w_gate"].copy()
    if mode == 2:
        rng = np.random.default_rng(case["seed"])
        for _ in range(max(1, cfg.E // 4)):
            a, b = rng.integers(0, cfg.E, 2)
            wg[a] = wg[b]
        x[rng.integers(0, cfg.T, max(1, cfg.T // 10))] = 0
    ridx, rw, rsc = orc.route(x, wg, cfg.k, cfg.renorm, L["gate_bias"])
    sh = B.make_shape(cfg.T, cfg.d, cfg.E, cfg.k, 64, si.BF16, cfg.renorm)
    xd, wd, bias = layer.to_device(x), layer.to_device(wg), layer.to_device(L["gate_bias"])
    nb = B.moe_workspace_bytes(sh)
    ws = torch.empty((nb,), dtype=torch.uint8, device="cuda")
    for with_scores, with_ws in ((False, False), (True, False), (False, True)):
        idx = torch.full((cfg.T, cfg.k), -7, dtype=torch.int32, device="cuda")
        w = torch.full((cfg.T, cfg.k), -7.0, dtype=torch.float32, device="cuda")
        sc = torch.full((cfg.T, cfg.E), -7.0, dtype=torch.float32, device="cuda") if with_scores else None
        if with_ws:
            B.moe_route_ws(sh, xd, wd, bias, idx, w, sc, ws, nb)
        else:
            B.moe_route(sh, xd, wd, bias, idx, w, sc)
        torch.cuda.synchronize()
        got = layer.to_host(idx)
        assert np.array_equal(got, ridx), np.argwhere(got != ridx)[:5]
        assert np.all(np.abs(layer.to_host(w) - rw) <= 1e-5 * np.abs(rw) + 1e-9)
        if with_scores:
            row_scale = np.maximum(np.abs(rsc).max(axis=1, keepdims=True), 1e-30)
            assert (np.abs(layer.to_host(sc) - rsc) / row_scale).max() <= 1e-5
