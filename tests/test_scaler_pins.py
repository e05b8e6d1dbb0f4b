"""Pins of oracle/scaler_oracle.py (CPU only): the CV of the per-replica loads, the paper's
Algorithm 1 (Expert Scaling) and the even split of an expert's rows over its replicas are
checked against hand-worked cases, closed forms, a library routine, invariants, a brute-force
optimum on tiny inputs and an independently written heap formulation; planted mistakes must
break a pin."""
import heapq
import itertools
import math
from fractions import Fraction

import numpy as np
import pytest

import synth_inputs as si
from oracle import scaler_oracle as sc


# ----------------------------------------------------------------------------- CV
def test_cv_closed_forms():
    assert sc.cv([7, 7, 7, 7]) == 0.0
    assert sc.cv([0, 0, 0]) == 0.0
    # two values a, b: mean (a+b)/2, population std |a-b|/2
    for a, b in ((3, 1), (10, 0), (5, 4)):
        assert sc.cv([a, b]) == pytest.approx(abs(a - b) / (a + b), rel=1e-15)
    # one hot expert among E: loads (A, 0, ..., 0) -> CV = sqrt(E - 1)
    for E in (2, 8, 64):
        assert sc.cv([1000] + [0] * (E - 1)) == pytest.approx(math.sqrt(E - 1), rel=1e-14)


def test_cv_is_over_the_replica_multiset():
    # (3w, w) with the first expert split in two: multiset {1.5w, 1.5w, w}; by hand
    # mean = 4w/3, deviations (w/6, w/6, -w/3), variance w^2/18, CV = 3 / (4 sqrt(18)) = 1/(4 sqrt 2)
    for w in (1, 40, 4096):
        assert sc.cv([3 * w, w], [2, 1]) == pytest.approx(1.0 / (4.0 * math.sqrt(2.0)), rel=1e-14)
    # a perfectly split straggler balances the layer
    assert sc.cv([300, 100], [3, 1]) == 0.0
    # identity through the two moments: CV^2 = N * sum(W_e^2 / R_e) / (sum W_e)^2 - 1
    rng = np.random.default_rng(5)
    for _ in range(20):
        E = int(rng.integers(2, 40))
        loads = rng.integers(0, 5000, size=E)
        reps = rng.integers(1, 6, size=E)
        if loads.sum() == 0:
            continue
        s1 = Fraction(int(loads.sum()))
        s2 = sum(Fraction(int(w) ** 2, int(r)) for w, r in zip(loads, reps))
        n = int(reps.sum())
        want = math.sqrt(max(0.0, float(s2 * n / (s1 * s1) - 1)))
        assert sc.cv(loads, reps) == pytest.approx(want, rel=1e-9, abs=1e-12)


def test_cv_matches_library_routine():
    stats = pytest.importorskip("scipy.stats")
    rng = np.random.default_rng(11)
    loads = rng.integers(0, 9000, size=64)
    reps = rng.integers(1, 5, size=64)
    expanded = np.repeat(loads / reps, reps)
    assert sc.cv(loads, reps) == pytest.approx(float(stats.variation(expanded, ddof=0)), rel=1e-12)


# ----------------------------------------------------------------------------- Algorithm 1
def test_scaling_hand_worked():
    w = 1000
    # CV(3w, w) = 0.5.  One split gives {1.5w, 1.5w, w}: CV = 0.1768 <= 0.2 -> stop.
    r, trace = sc.expert_scaling([3 * w, w], expert_mem=1, mem_cap=10, cv_threshold=0.2)
    assert r.tolist() == [2, 1]
    assert trace == pytest.approx([0.5, 1 / (4 * math.sqrt(2))], rel=1e-14)
    # With V = 0.1 the largest per-replica load is still expert 0's (1.5w > w): {w, w, w, w}, CV 0.
    r, trace = sc.expert_scaling([3 * w, w], expert_mem=1, mem_cap=10, cv_threshold=0.1)
    assert r.tolist() == [3, 1]
    assert trace == pytest.approx([0.5, 1 / (4 * math.sqrt(2)), 0.0], abs=1e-15)
    # (5, 4): after one split {2.5, 2.5, 4} the straggler is expert 1, not expert 0 again
    r, _ = sc.expert_scaling([5, 4], expert_mem=1, mem_cap=2, cv_threshold=0.01)
    assert r.tolist() == [2, 2]


def test_scaling_memory_cap_and_threshold_edges():
    loads = [900, 100, 100, 100]
    assert sc.expert_scaling(loads, 3, 0, 0.2)[0].tolist() == [1, 1, 1, 1]      # no memory
    assert sc.expert_scaling(loads, 3, 2, 0.2)[0].tolist() == [1, 1, 1, 1]      # less than one expert
    assert sc.expert_scaling(loads, 3, 3, 0.2)[0].tolist() == [2, 1, 1, 1]      # exactly one
    assert sc.expert_scaling(loads, 3, 8, 0.2)[0].tolist() == [3, 1, 1, 1]      # two fit, 2 units left over
    # uniform loads never scale, whatever the budget; nor do all-zero loads
    assert sc.expert_scaling([50] * 8, 1, 100, 0.0)[0].tolist() == [1] * 8
    assert sc.expert_scaling([0] * 8, 1, 100, 0.0)[0].tolist() == [1] * 8
    # a threshold at or above the initial CV leaves the layer alone (the test is strict: CV > V)
    assert sc.expert_scaling([3, 1], 1, 100, 0.5)[0].tolist() == [1, 1]
    # equal stragglers: the lowest index is split first
    assert sc.expert_scaling([8, 8, 1], 1, 1, 0.0)[0].tolist() == [2, 1, 1]
    # a single hot expert and zero loads elsewhere: replicas go to the hot expert only
    r, _ = sc.expert_scaling([1000, 0, 0, 0], 1, 5, 0.0)
    assert r.tolist() == [6, 1, 1, 1]


def _zipf_loads(E, total, alpha, seed):
    return si.zipf_loads(E, total, alpha, seed)


@pytest.mark.parametrize("E,total,alpha,seed", [(8, 8192, 1.2, 1), (64, 49152, 1.2, 2),
                                                 (128, 256, 0.8, 3), (16, 4096, 2.0, 4)])
def test_scaling_invariants(E, total, alpha, seed):
    loads = _zipf_loads(E, total, alpha, seed)
    for mem, cap, V in ((1, 16, 0.2), (3, 50, 0.05), (1, 1000, 0.2), (2, 7, 0.0)):
        r, trace = sc.expert_scaling(loads, mem, cap, V)
        extra = int(r.sum()) - E
        assert np.all(r >= 1)
        assert extra * mem <= cap                                   # the cap is respected
        assert len(trace) == extra + 1
        # stopped for a reason the algorithm states: balanced, or no room for one more replica
        assert trace[-1] <= V or (extra + 1) * mem > cap
        assert all(t > V for t in trace[:-1])                       # every earlier step was needed
        # heavier experts never end with fewer replicas than lighter ones
        order = np.argsort(-loads, kind="stable")
        for a, b in zip(order[:-1], order[1:]):
            if loads[a] > loads[b]:
                assert r[a] >= r[b]
        # replaying the counts: the largest per-replica load never grows from step to step
        reps = np.ones(E, dtype=np.int64)
        last = max(Fraction(int(w)) for w in loads)
        for _ in range(extra):
            per = [Fraction(int(w), int(q)) for w, q in zip(loads, reps)]
            e = max(range(E), key=lambda i: (per[i], -i))
            reps[e] += 1
            now = max(Fraction(int(w), int(q)) for w, q in zip(loads, reps))
            assert now <= last
            last = now
        assert reps.tolist() == r.tolist()


def test_scaling_greedy_is_the_min_max_optimum_on_tiny_inputs():
    """For a fixed number of extra replicas, splitting the current straggler each time minimises
    the largest per-replica load; brute force over every allocation checks it."""
    rng = np.random.default_rng(3)
    for _ in range(40):
        E = int(rng.integers(2, 5))
        loads = rng.integers(1, 60, size=E)
        n = int(rng.integers(1, 6))
        r, _ = sc.expert_scaling(loads, 1, n, -1.0)                  # V < 0: only the cap stops it
        assert int(r.sum()) - E == n
        got = max(Fraction(int(w), int(q)) for w, q in zip(loads, r))
        best = None
        for alloc in itertools.product(range(n + 1), repeat=E):
            if sum(alloc) != n:
                continue
            m = max(Fraction(int(w), 1 + a) for w, a in zip(loads, alloc))
            best = m if best is None or m < best else best
        assert got == best


def _scaling_with_heap(loads, mem, cap, V):
    """Independent formulation (the paper's text: a max heap of stragglers; CV from the two
    moments S1 = sum W_e, S2 = sum W_e^2 / R_e kept as exact fractions)."""
    E = len(loads)
    reps = [1] * E
    heap = [(-Fraction(int(w)), e) for e, w in enumerate(loads)]
    heapq.heapify(heap)
    s1 = Fraction(int(sum(int(w) for w in loads)))
    s2 = sum(Fraction(int(w) ** 2) for w in loads)
    n = E
    used = 0

    def cv_now():
        if s1 == 0:
            return 0.0
        return math.sqrt(max(0.0, float(s2 * n / (s1 * s1) - 1)))

    while used + mem <= cap and cv_now() > V:
        neg, e = heapq.heappop(heap)
        if neg == 0:
            break
        w = int(loads[e])
        s2 += Fraction(w * w, reps[e] + 1) - Fraction(w * w, reps[e])
        reps[e] += 1
        n += 1
        used += mem
        heapq.heappush(heap, (-Fraction(w, reps[e]), e))
    return reps


def test_scaling_matches_heap_formulation():
    rng = np.random.default_rng(17)
    for trial in range(60):
        E = int(rng.integers(2, 70))
        loads = _zipf_loads(E, int(rng.integers(E, 60000)), float(rng.uniform(0.3, 2.0)), 100 + trial)
        mem = int(rng.integers(1, 4))
        cap = int(rng.integers(0, 200))
        V = float(rng.choice([0.0, 0.05, 0.2, 0.5]))
        r, trace = sc.expert_scaling(loads, mem, cap, V)
        # the comparison is only meaningful away from the knife edge CV == V
        assert all(abs(t - V) > 1e-9 for t in trace)
        assert _scaling_with_heap(loads, mem, cap, V) == r.tolist()


def test_paper_facts_for_the_scaler(repo_root):
    import os
    facts = {}
    with open(os.path.join(repo_root, "tests", "golden", "paper_facts.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                key, val = line.split("=", 1)
                facts[key.strip()] = val.split("#")[0].strip()
    # Section 4.2 quotes CV <= 0.2 as the example threshold and Section 6.4 selects it; every expert
    # starts with a single instance
    assert float(facts["cv_threshold"]) == 0.2
    assert int(facts["initial_replicas"]) == 1
    loads = _zipf_loads(8, 8192, 1.2, 9)
    r, trace = sc.expert_scaling(loads, 1, 64, float(facts["cv_threshold"]))
    assert trace[0] > 0.2 >= trace[-1] and r.min() == int(facts["initial_replicas"])


# ----------------------------------------------------------------------------- replica segments
def test_replica_segments_are_an_even_cover():
    rng = np.random.default_rng(23)
    for _ in range(50):
        E = int(rng.integers(1, 40))
        counts = rng.integers(0, 300, size=E)
        reps = rng.integers(1, 9, size=E)
        offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
        seg, who = sc.replica_segments(offsets, reps)
        assert seg.shape[0] == reps.sum() + 1 and who.shape[0] == reps.sum()
        assert seg[0] == 0 and seg[-1] == counts.sum() and np.all(np.diff(seg) >= 0)
        assert who.tolist() == np.repeat(np.arange(E), reps).tolist()
        pos = 0
        for e in range(E):
            sizes = np.diff(seg[pos:pos + reps[e] + 1])
            assert seg[pos] == offsets[e] and seg[pos + reps[e]] == offsets[e + 1]
            assert sizes.max() - sizes.min() <= 1
            # the same multiset of piece sizes as the library's even split
            want = sorted(len(p) for p in np.array_split(np.arange(counts[e]), reps[e]))
            assert sorted(sizes.tolist()) == want
            pos += reps[e]


# ----------------------------------------------------------------------------- planted mistakes
def test_planted_mistakes_are_caught(monkeypatch):
    def run_pins():
        test_cv_closed_forms()
        test_cv_is_over_the_replica_multiset()
        test_scaling_hand_worked()
        test_scaling_memory_cap_and_threshold_edges()

    run_pins()
    real_cv, real_loads = sc.cv, sc.replica_loads

    # (1) sample standard deviation (1/(N-1)) instead of the population form
    def cv_sample(loads, replicas=None):
        loads = np.asarray(loads, dtype=np.int64)
        replicas = np.ones_like(loads) if replicas is None else replicas
        w = real_loads(loads, replicas)
        return 0.0 if w.mean() == 0 else float(np.std(w, ddof=1) / w.mean())
    monkeypatch.setattr(sc, "cv", cv_sample)
    with pytest.raises(AssertionError):
        run_pins()
    monkeypatch.setattr(sc, "cv", real_cv)

    # (2) CV over the experts' total loads instead of the per-replica multiset
    monkeypatch.setattr(sc, "cv", lambda loads, replicas=None: real_cv(loads))
    with pytest.raises(AssertionError):
        run_pins()
    monkeypatch.setattr(sc, "cv", real_cv)

    # (3) the listing's double division: re-splitting the already split load
    def loads_twice(loads, replicas):
        loads = np.asarray(loads, dtype=np.float64)
        replicas = np.asarray(replicas, dtype=np.int64)
        per = loads.copy()
        for e, r in enumerate(replicas):
            for q in range(2, int(r) + 1):
                per[e] = per[e] / q
        return np.repeat(per, replicas)
    monkeypatch.setattr(sc, "replica_loads", loads_twice)
    with pytest.raises(AssertionError):
        run_pins()
    monkeypatch.setattr(sc, "replica_loads", real_loads)

    # (4) the straggler chosen by total load instead of per-replica load
    real_fraction = sc.Fraction
    monkeypatch.setattr(sc, "Fraction", lambda num, den=1: real_fraction(num, 1))
    with pytest.raises(AssertionError):
        run_pins()
    monkeypatch.setattr(sc, "Fraction", real_fraction)
    run_pins()
