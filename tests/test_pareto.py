"""Pareto front of (makespan, largest peak) and re-capping: oracle pins (CPU) and GPU parity of
fpsched_pareto / fpsched_apply_caps."""
import numpy as np
import pytest

import oracle
import workloads


def evaluated_batch(index=2, n=1500):
    spec = workloads.config(index, n)
    words = workloads.generate(spec, threads=4)
    return spec, words, oracle.evaluate(spec.problem, words, threads=4)


def synthetic_results(n, D, seed, ms_range, pk_range, fail=0.05):
    """Result arrays with chosen value ranges (narrow ranges give many ties), as evaluate writes them."""
    rng = np.random.default_rng(seed)
    ms = rng.integers(ms_range[0], ms_range[1], n).astype(np.int64)
    peak = rng.integers(pk_range[0], pk_range[1], (n, D)).astype(np.int32)
    flags = np.where(rng.random(n) < fail, rng.integers(1, 4, n), 0).astype(np.uint8)
    flags |= np.where((flags == 0) & (rng.random(n) < 0.3), 4, 0).astype(np.uint8)
    bad = (flags & 3) != 0
    ms[bad] = oracle.INT64_MAX
    peak[bad] = -1
    return dict(makespan=ms, idle=np.zeros((n, D), np.int64), peak=peak, flags=flags)


def staircase_front(res):
    """Another route to the same set: sort by (makespan, peak, index) and keep every point whose peak
    is below all peaks seen before it."""
    ok = np.flatnonzero((res["flags"] & 3) == 0)
    ms, pk = res["makespan"][ok], res["peak"][ok].max(1).astype(np.int64)
    order = np.lexsort((ok, pk, ms))
    best = np.iinfo(np.int64).max
    out = []
    for i in order:
        if pk[i] < best:
            best = pk[i]
            out.append((ok[i], ms[i], pk[i]))
    return out


def check_front(res, kmax, idx, ms, pk, cnt):
    expect = staircase_front(res)
    assert cnt == min(kmax, len(expect))
    assert [(int(a), int(b), int(c)) for a, b, c in zip(idx[:cnt], ms[:cnt], pk[:cnt])] == \
        [(int(a), int(b), int(c)) for a, b, c in expect[:cnt]]
    assert np.all(idx[cnt:] == -1) and np.all(ms[cnt:] == oracle.INT64_MAX) and np.all(pk[cnt:] == -1)


def test_hand_worked_front():
    # (makespan, largest peak): c0 (5, 2), c1 (3, 3), c2 (3, 4) dominated by c1, c3 (9, 1), c4 (5, 2) twin of c0,
    # c5 (7, 2) dominated by c0, c6 deadlocked, c7 (2, 9) over the cap but on the front
    r = dict(makespan=np.array([5, 3, 3, 9, 5, 7, oracle.INT64_MAX, 2]),
             peak=np.array([[2, 1], [3, 1], [1, 4], [1, 1], [2, 2], [2, 0], [-1, -1], [9, 1]], dtype=np.int32),
             flags=np.array([0, 0, 0, 0, 0, 0, 1, 4], dtype=np.uint8))
    idx, ms, pk, cnt = oracle.pareto(r, 6)
    assert cnt == 4
    assert list(idx) == [7, 1, 0, 3, -1, -1]
    assert list(ms[:4]) == [2, 3, 5, 9] and list(pk[:4]) == [9, 3, 2, 1]
    # a shorter output keeps the head of the list
    idx, ms, pk, cnt = oracle.pareto(r, 2)
    assert cnt == 2 and list(idx) == [7, 1]


@pytest.mark.parametrize("seed", range(6))
def test_oracle_front_is_the_staircase(seed):
    # narrow ranges: many equal makespans, equal peaks and equal pairs
    res = synthetic_results(700, 3, seed, (10, 40 + 30 * seed), (1, 6 + 5 * seed))
    for kmax in (1, 4, 64):
        check_front(res, kmax, *oracle.pareto(res, kmax))


def test_front_of_evaluated_schedules():
    _, _, res = evaluated_batch(2, 1200)
    idx, ms, pk, cnt = oracle.pareto(res, 256)
    check_front(res, 256, idx, ms, pk, cnt)
    assert cnt >= 1
    # the head of the front is the best makespan over all completed candidates, whatever the cap
    r_idx, r_k1, r_k2, _ = oracle.rank(res, 1, "makespan_peak", include_over_cap=True)
    assert idx[0] == r_idx[0] and ms[0] == r_k1[0] and pk[0] == r_k2[0]
    # its tail is the smallest peak, at that peak's best makespan
    r_idx, r_k1, r_k2, _ = oracle.rank(res, 1, "peak_makespan", include_over_cap=True)
    assert idx[cnt - 1] == r_idx[0] and pk[cnt - 1] == r_k1[0] and ms[cnt - 1] == r_k2[0]
    assert np.all(np.diff(ms[:cnt]) > 0) and np.all(np.diff(pk[:cnt]) < 0)


def test_front_ignores_dominated_additions_and_equal_peaks():
    res = synthetic_results(300, 2, 11, (100, 200), (5, 30), fail=0.1)
    idx, ms, pk, cnt = oracle.pareto(res, 64)
    # appending candidates that are worse in both values changes nothing
    extra = 50
    grown = dict(makespan=np.concatenate([res["makespan"], np.full(extra, 1000)]),
                 peak=np.concatenate([res["peak"], np.full((extra, 2), 99, np.int32)]),
                 flags=np.concatenate([res["flags"], np.zeros(extra, np.uint8)]))
    g = oracle.pareto(grown, 64)
    assert g[3] == cnt and np.array_equal(g[0], idx)
    # with one peak value everywhere the front is the single best (makespan, index)
    flat = dict(res, peak=np.where(res["peak"] >= 0, 7, -1).astype(np.int32))
    f_idx, f_ms, _, f_cnt = oracle.pareto(flat, 8)
    t_idx, t_ms, _ = oracle.topk(flat["makespan"], (flat["flags"] & 3).astype(np.uint8), 1)
    assert f_cnt == 1 and f_idx[0] == t_idx[0] and f_ms[0] == t_ms[0]


def test_front_of_nothing():
    r = dict(makespan=np.array([oracle.INT64_MAX] * 3), peak=np.full((3, 2), -1, np.int32),
             flags=np.array([1, 2, 3], dtype=np.uint8))
    idx, ms, pk, cnt = oracle.pareto(r, 4)
    assert cnt == 0 and np.all(idx == -1)
    r = dict(makespan=np.zeros(0, np.int64), peak=np.zeros((0, 2), np.int32), flags=np.zeros(0, np.uint8))
    assert oracle.pareto(r, 4)[3] == 0


def test_apply_caps_reproduces_the_evaluator_and_moves_with_the_cap():
    spec, words, res = evaluated_batch(2, 800)
    cap = np.asarray(spec.problem.mem_cap, np.int32)
    # the problem's own caps give back the evaluator's flags
    assert np.array_equal(oracle.apply_caps(res, cap), res["flags"])
    # the same schedules evaluated under another cap: the flags are those of a re-capped result
    import copy
    loose = copy.copy(spec.problem)
    loose.mem_cap = [c + 3 for c in spec.problem.mem_cap]
    res2 = oracle.evaluate(loose, words, threads=4)
    assert np.array_equal(res2["peak"], res["peak"])
    assert np.array_equal(oracle.apply_caps(res, cap + 3), res2["flags"])
    # caps per candidate: row c judged by its own row of caps
    n, D = res["peak"].shape
    rng = np.random.default_rng(5)
    caps = rng.integers(0, int(res["peak"].max()) + 2, (n, D)).astype(np.int32)
    fl = oracle.apply_caps(res, caps)
    ok = (res["flags"] & 3) == 0
    over = (res["peak"] > caps).any(1) & ok
    assert np.array_equal((fl & 4) != 0, over)
    assert np.array_equal(fl & 3, res["flags"] & 3)
    # no cap at all
    assert not np.any(oracle.apply_caps(res, np.full(D, 2**31 - 1, np.int32)) & 4)
