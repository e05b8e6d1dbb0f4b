"""CPU-side checks of the boundary: the shared library loads, exports every symbol that
include/moe.h declares, and its host-only logic (argument validation, workspace sizing,
status text) behaves as documented.  No kernel is launched here."""
import ctypes
import os
import re

import pytest

from paper_2603_06350_amd import binding as B


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.lib_path()):
        from paper_2603_06350_amd import build
        build.build()
    return B.load()


def declared_functions(repo_root):
    text = open(os.path.join(repo_root, "include", "moe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib, repo_root):
    names = declared_functions(repo_root)
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_header_has_no_torch_or_cpp_types(repo_root):
    text = open(os.path.join(repo_root, "include", "moe.h")).read()
    assert 'extern "C"' in text
    for banned in ("torch", "at::", "std::", "hipStream_t "):
        assert banned not in re.sub(r"/\*.*?\*/", "", text, flags=re.S)


def test_strerror(lib):
    assert B.strerror(0) == "ok"
    for code in (-1, -2, -3, -4):
        assert B.strerror(code) not in ("ok", "unknown status")
    assert B.strerror(-99) == "unknown status"


def test_shape_validation_happens_before_any_launch(lib):
    ok = B.make_shape(64, 128, 8, 2, 256, B.MOE_BF16, 1)
    assert B.moe_workspace_bytes(ok) >= 8 * 4
    bad = [
        B.make_shape(64, 128, 8, 9, 256, B.MOE_BF16, 1),     # k > E
        B.make_shape(64, 128, 8, 0, 256, B.MOE_BF16, 1),     # k < 1
        B.make_shape(64, 124, 8, 2, 256, B.MOE_BF16, 1),     # d*2 not a multiple of 16
        B.make_shape(64, 128, 8, 2, 250, B.MOE_BF16, 1),     # F*2 not a multiple of 16
        B.make_shape(64, 128, 8, 2, 256, 7, 1),              # dtype
        B.make_shape(64, 128, 8, 2, 256, B.MOE_BF16, 2),     # renorm
        B.make_shape(-1, 128, 8, 2, 256, B.MOE_BF16, 1),     # T < 0
    ]
    for s in bad:
        with pytest.raises(B.MoeError) as ei:
            B.moe_workspace_bytes(s)
        assert ei.value.code == -1
    for s in (B.make_shape(64, 128, 300, 2, 256, B.MOE_BF16, 1),      # E > 256
              B.make_shape(1 << 30, 128, 8, 4, 256, B.MOE_BF16, 1)):  # T*k >= 2^31
        with pytest.raises(B.MoeError) as ei:
            B.moe_workspace_bytes(s)
        assert ei.value.code == -2
    # null pointers are rejected by every call, on the host
    for call in (lambda: B.moe_route(ok, None, None, None, None, None),
                 lambda: B.moe_route_ws(ok, None, None, None, None, None, None, None, 0),
                 lambda: B.moe_count_and_permute(ok, None, None, None, None, None, None, None,
                                                 None, 0),
                 lambda: B.moe_grouped_ffn(ok, None, None, None, None, None, None, None),
                 lambda: B.moe_grouped_ffn_gather(ok, None, None, None, None, None, None, None, None),
                 lambda: B.moe_combine(ok, None, None, None, None)):
        with pytest.raises(B.MoeError) as ei:
            call()
        assert ei.value.code == -1
    # misaligned pointer
    with pytest.raises(B.MoeError):
        B.moe_combine(ok, 0x1008, 0x1000, 0x1000, 0x1000)
    # T = 0 is a no-op for the calls that only touch per-token data
    empty = B.make_shape(0, 128, 8, 2, 256, B.MOE_BF16, 1)
    B.moe_route(empty, None, None, None, None, None)
    B.moe_route_ws(empty, None, None, None, None, None, None, None, 0)
    B.moe_grouped_ffn(empty, None, None, None, None, None, None, None)
    B.moe_combine(empty, None, None, None, None)


def test_workspace_size_grows_with_tokens(lib):
    small = B.moe_workspace_bytes(B.make_shape(16384, 128, 64, 6, 256, B.MOE_BF16, 0))
    large = B.moe_workspace_bytes(B.make_shape(131072, 128, 64, 6, 256, B.MOE_BF16, 0))
    assert large >= 512 * 64 * 4 and small >= 64 * 64 * 4 and large > small
    assert small % 256 == 0 and large % 256 == 0
    # batches of fewer than 8192 tokens: room for T x E fp32 scores and T + E norms between
    # moe_route_ws's two kernels
    decode = B.moe_workspace_bytes(B.make_shape(32, 4096, 128, 8, 1536, B.MOE_BF16, 1))
    assert decode >= (32 * 128 + 32 + 128) * 4
    assert B.moe_workspace_bytes(B.make_shape(8191, 128, 256, 8, 256, B.MOE_BF16, 1)) >= (8191 * 256 + 8191 + 256) * 4


def test_product_package_does_not_import_the_oracle(repo_root):
    pkg = os.path.join(repo_root, "paper_2603_06350_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".h")):
                src = open(os.path.join(dirpath, fn)).read()
                assert "oracle" not in src.replace("no CPU fallback", ""), fn
    for fn in os.listdir(os.path.join(repo_root, "oracle")):
        if fn.endswith(".py"):
            assert "paper_2603_06350_amd" not in open(os.path.join(repo_root, "oracle", fn)).read()


def test_scaler_calls_validate_on_the_host(lib):
    one = 0x1000   # never dereferenced: every case below fails validation first
    cases = [
        (lambda: B.moe_scale_replicas(0, one, 1, 4, 0.2, one), -1),          # E < 1
        (lambda: B.moe_scale_replicas(8, None, 1, 4, 0.2, one), -1),         # no loads
        (lambda: B.moe_scale_replicas(8, one, 1, 4, 0.2, None), -1),         # no output
        (lambda: B.moe_scale_replicas(8, one, 0, 4, 0.2, one), -1),          # M_e < 1
        (lambda: B.moe_scale_replicas(8, one, 1, -1, 0.2, one), -1),         # M_cap < 0
        (lambda: B.moe_scale_replicas(8, one, 1, 4, float("nan"), one), -1),
        (lambda: B.moe_scale_replicas(300, one, 1, 4, 0.2, one), -2),        # E > 256
        (lambda: B.moe_scale_replicas(8, one, 1, B.MOE_MAX_EXTRA_REPLICAS + 1, 0.2, one), -2),
        (lambda: B.moe_replica_segments(0, one, one, 16, one, one, one), -1),
        (lambda: B.moe_replica_segments(8, None, one, 16, one, one, one), -1),
        (lambda: B.moe_replica_segments(8, one, one, -1, one, one, one), -1),
        (lambda: B.moe_replica_segments(8, one, one, 16, one, one, None), -1),
        (lambda: B.moe_replica_segments(300, one, one, 16, one, one, one), -2),
        (lambda: B.moe_place_replicas(0, one, one, 2, None, None, None, 8, one, one, one, one), -1),
        (lambda: B.moe_place_replicas(8, one, one, 0, None, None, None, 8, one, one, one, one), -1),
        (lambda: B.moe_place_replicas(8, None, one, 2, None, None, None, 8, one, one, one, one), -1),
        (lambda: B.moe_place_replicas(8, one, one, 2, one, None, None, 8, one, one, one, one), -1),
        (lambda: B.moe_place_replicas(8, one, one, 2, None, None, None, -1, one, one, one, one), -1),
        (lambda: B.moe_place_replicas(8, one, one, 65, None, None, None, 8, one, one, one, one), -2),
        (lambda: B.moe_place_replicas(300, one, one, 2, None, None, None, 8, one, one, one, one), -2),
    ]
    for call, code in cases:
        with pytest.raises(B.MoeError) as ei:
            call()
        assert ei.value.code == code


def test_grouped_ffn_ws_validates_on_the_host(lib):
    import synth_inputs as si
    sh = B.make_shape(16, 64, 4, 2, 64, si.BF16, 1)
    nb = B.moe_ffn_workspace_bytes(sh)
    assert nb >= 256 * 256 * 4 and nb % (256 * 256 * 4) == 0      # one fp32 tile per compute unit
    one = 0x1000   # never dereferenced: every case below fails validation first
    args = (one, None, one, one, one, one, one, one)
    cases = [
        (lambda: B.moe_grouped_ffn_ws(sh, *args, 0, one, nb), -1),             # parts out of range
        (lambda: B.moe_grouped_ffn_ws(sh, *args, 4, one, nb), -1),             # the whole-tile flag alone
        (lambda: B.moe_grouped_ffn_ws(sh, *args, 8, one, nb), -1),
        (lambda: B.moe_grouped_ffn_ws(sh, *args, 11, one, nb), -1),
        (lambda: B.moe_grouped_ffn_ws(sh, *args, 3, one + 4, nb), -1),         # workspace misaligned
        (lambda: B.moe_grouped_ffn_ws(sh, *args, 3, one, nb - 1), -3),         # workspace too small
        (lambda: B.moe_grouped_ffn_ws(sh, None, None, one, one, one, one, one, one, 3, one, nb), -1),
        (lambda: B.moe_grouped_ffn_ws(sh, one, None, None, one, one, one, one, one, 3, None, 0), -1),
    ]
    for call, code in cases:
        with pytest.raises(B.MoeError) as ei:
            call()
        assert ei.value.code == code
    # no tokens: nothing to do, with or without a workspace
    empty = B.make_shape(0, 64, 4, 2, 64, si.BF16, 1)
    B.moe_grouped_ffn_ws(empty, None, None, None, None, None, None, None, None, 3, None, 0)


def test_expert_parallel_shares_partition_the_rows():
    """Host logic of the expert-parallel latency model (Section 4.3): under the static placement
    and under the oracle's Algorithm 1 + 2 outputs every permuted row belongs to exactly one rank,
    a rank's local offsets cover its rows expert by expert, and replicas of one expert on one rank
    merge in row order."""
    import numpy as np
    import synth_inputs as si
    from oracle import placer_oracle as pl
    from oracle import scaler_oracle as sc
    from paper_2603_06350_amd import ep_sim

    E, G = 16, 4
    counts = si.zipf_loads(E, 5000, 1.2, seed=3).astype(np.int64)
    counts[5] = 0
    offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    A = int(offsets[-1])
    static = ep_sim.static_shares(offsets, E, G)
    ep_sim.check_partition(static, A)
    assert [int(s[1].size) for s in static] == [int(counts[g * 4:(g + 1) * 4].sum()) for g in range(G)]

    replicas, _ = sc.expert_scaling(counts, 1, E, 0.2)
    seg_offsets, seg_expert = sc.replica_segments(offsets, replicas)
    gpu_of = pl.expert_placement(counts, replicas, G)[0]
    S = int(np.sum(replicas))
    placed = ep_sim.placed_shares(seg_offsets, seg_expert, np.asarray(gpu_of), S, G)
    ep_sim.check_partition(placed, A)
    for hosted, rows, local in placed:
        assert np.all(np.diff(hosted) > 0) and local.size == hosted.size + 1
        for i, e in enumerate(hosted):
            mine = rows[local[i]:local[i + 1]]
            assert np.all(np.diff(mine) > 0)                      # row order kept
            assert mine.size == 0 or (mine[0] >= offsets[e] and mine[-1] < offsets[e + 1])
    # the point of scaling + placement: the most loaded rank holds fewer rows
    assert max(r.size for _, r, _ in placed) < max(r.size for _, r, _ in static)
