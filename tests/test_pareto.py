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


def to_cuda(res):
    import torch
    return {k: torch.from_numpy(np.ascontiguousarray(v)).cuda() for k, v in res.items()}


def gpu_front(h, res_gpu, kmax):
    import torch
    out = h.pareto(res_gpu, kmax)
    torch.cuda.synchronize()
    return (out["idx"].cpu().numpy(), out["makespan"].cpu().numpy(), out["peak"].cpu().numpy(),
            int(out["count"].item()))


@pytest.mark.gpu
@pytest.mark.parametrize("index,n", [(2, 5000), (5, 3000), (1, 200)])
def test_gpu_front_of_evaluated_schedules_matches_the_oracle(index, n):
    import torch

    import paper_2510_05112_amd as fp
    spec, words, ref = evaluated_batch(index, n)
    h = fp.Problem(spec.problem, spec.stride, device=0)
    res = h.evaluate(torch.from_numpy(words.view(np.int16)).cuda())
    for kmax in (1, 7, 1024):
        got = gpu_front(h, res, kmax)
        exp = oracle.pareto(ref, kmax)
        assert got[3] == exp[3], kmax
        for g, e in zip(got[:3], exp[:3]):
            assert np.array_equal(g, e), kmax
    h.close()


@pytest.mark.gpu
def test_gpu_front_with_ties_long_fronts_and_ragged_tiles():
    import paper_2510_05112_amd as fp
    spec = workloads.config(1, 8)
    h = fp.Problem(spec.problem, spec.stride, device=0)
    D = int(spec.problem.n_devices)
    cases = [
        synthetic_results(3000, D, 1, (10, 60), (1, 8)),            # few values, many equal pairs, two tiles
        synthetic_results(2048, D, 2, (0, 10**6), (1, 10**6)),      # exactly one tile, wide values
        synthetic_results(2049, D, 3, (0, 10**12), (1, 2**31 - 1)),  # one candidate in the second tile
        synthetic_results(4500, D, 4, (5, 6), (3, 4)),              # every pair the same: lowest index wins
        synthetic_results(1, D, 5, (5, 6), (3, 4), fail=0.0),
        synthetic_results(700, D, 6, (0, 50), (0, 50), fail=1.0),   # nothing completed
    ]
    # a front longer than kmax and longer than a tile: makespan rises while the peak falls
    n = 5000
    stair = dict(makespan=np.arange(n, dtype=np.int64) * 3, idle=np.zeros((n, D), np.int64),
                 peak=np.repeat((n - np.arange(n, dtype=np.int32))[:, None], D, 1), flags=np.zeros(n, np.uint8))
    # the same staircase in a scrambled order
    perm = np.random.default_rng(9).permutation(n)
    shuffled = {k: v[perm] for k, v in stair.items()}
    for ci, res in enumerate(cases + [stair, shuffled]):
        gres = to_cuda(res)
        for kmax in (1, 5, 1024):
            got = gpu_front(h, gres, kmax)
            check_front(res, kmax, *got)
            if res["makespan"].size <= 3000:
                exp = oracle.pareto(res, kmax)
                assert got[3] == exp[3] and all(np.array_equal(g, e) for g, e in zip(got[:3], exp[:3])), (ci, kmax)
    # the empty batch, and argument errors
    empty = to_cuda({k: v[:0] for k, v in stair.items()})
    got = gpu_front(h, empty, 4)
    assert got[3] == 0 and np.all(got[0] == -1) and np.all(got[2] == -1)
    with pytest.raises(fp.FpschedError):
        h.pareto(empty, 0)
    with pytest.raises(fp.FpschedError):
        h.pareto(empty, 1025)
    h.close()


@pytest.mark.gpu
def test_gpu_apply_caps_matches_the_oracle():
    import torch

    import paper_2510_05112_amd as fp
    spec, words, ref = evaluated_batch(2, 3000)
    h = fp.Problem(spec.problem, spec.stride, device=0)
    res = h.evaluate(torch.from_numpy(words.view(np.int16)).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(res["flags"].cpu().numpy(), ref["flags"])
    n, D = ref["peak"].shape
    cap = np.asarray(spec.problem.mem_cap, np.int32)
    rng = np.random.default_rng(3)
    per_cand = rng.integers(0, int(ref["peak"].max()) + 2, (n, D)).astype(np.int32)
    for caps in (cap - 2, cap + 1, np.zeros(D, np.int32), np.full(D, 2**31 - 1, np.int32), per_cand, cap):
        h.apply_caps(res, torch.from_numpy(caps).cuda())
        torch.cuda.synchronize()
        assert np.array_equal(res["flags"].cpu().numpy(), oracle.apply_caps(ref, caps))
    # top-k under the new cap is the oracle's top-k under that cap
    h.apply_caps(res, torch.from_numpy(cap - 2).cuda())
    top = h.topk(res, 32)
    torch.cuda.synchronize()
    e_idx, e_ms, e_cnt = oracle.topk(ref["makespan"], oracle.apply_caps(ref, cap - 2), 32)
    assert int(top["count"].item()) == e_cnt and np.array_equal(top["idx"].cpu().numpy(), e_idx)
    with pytest.raises(ValueError):
        h.apply_caps(res, torch.zeros(D + 1, dtype=torch.int32, device="cuda"))
    h.close()
