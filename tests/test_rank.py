"""Ranking by two-part keys: oracle pins (CPU) and GPU parity of fpsched_rank."""
import numpy as np
import pytest

import oracle
import workloads

MODES = ["makespan", "makespan_peak", "peak_makespan", "idle"]


def evaluated_batch(index=2, n=1500):
    spec = workloads.config(index, n)
    words = workloads.generate(spec, threads=4)
    return spec, words, oracle.evaluate(spec.problem, words, threads=4)


def numpy_rank(res, k, mode, include_over_cap):
    """The definition, with numpy's lexicographic sort."""
    fl = res["flags"]
    keep = (fl & 3) == 0
    if not include_over_cap:
        keep &= (fl & 4) == 0
    idx = np.flatnonzero(keep)
    ms, pk, idle = res["makespan"][idx], res["peak"][idx].max(1).astype(np.int64), res["idle"][idx].sum(1)
    k1, k2 = {"makespan": (ms, 0 * ms), "makespan_peak": (ms, pk), "peak_makespan": (pk, ms),
              "idle": (idle, 0 * ms)}[mode]
    order = np.lexsort((idx, k2, k1))[:k]
    return idx[order], k1[order], k2[order]


def test_hand_worked_case():
    # four candidates: (makespan, largest peak) = (5, 2), (3, 3) over cap, (3, 2), (9, 1); a fifth deadlocks
    r = dict(makespan=np.array([5, 3, 3, 9, oracle.INT64_MAX]),
             idle=np.array([[1, 1], [2, 0], [0, 1], [4, 4], [-1, -1]]),
             peak=np.array([[2, 1], [3, 1], [1, 2], [1, 1], [-1, -1]], dtype=np.int32),
             flags=np.array([0, 4, 0, 0, 1], dtype=np.uint8))
    assert list(oracle.rank(r, 4, "makespan_peak")[0]) == [2, 0, 3, -1]
    assert list(oracle.rank(r, 4, "makespan_peak", True)[0]) == [2, 1, 0, 3]
    assert list(oracle.rank(r, 4, "peak_makespan", True)[0]) == [3, 2, 0, 1]
    assert list(oracle.rank(r, 4, "idle")[0]) == [2, 0, 3, -1]      # sums of idle 1, 2, 8
    assert oracle.rank(r, 4, "idle")[3] == 3


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("include_over_cap", [False, True])
def test_oracle_rank_is_the_lexicographic_sort(mode, include_over_cap):
    _, _, res = evaluated_batch()
    for k in (1, 17, 300, 1024):
        idx, k1, k2, cnt = oracle.rank(res, k, mode, include_over_cap)
        e_idx, e_k1, e_k2 = numpy_rank(res, k, mode, include_over_cap)
        assert cnt == len(e_idx)
        assert np.array_equal(idx[:cnt], e_idx) and np.array_equal(k1[:cnt], e_k1) and np.array_equal(k2[:cnt], e_k2)
        assert np.all(idx[cnt:] == -1)


def test_makespan_mode_is_topk():
    _, _, res = evaluated_batch()
    idx, ms, cnt = oracle.topk(res["makespan"], res["flags"], 64)
    r_idx, r_k1, _, r_cnt = oracle.rank(res, 64, "makespan")
    assert cnt == r_cnt and np.array_equal(idx, r_idx) and np.array_equal(ms, r_k1)


@pytest.mark.gpu
@pytest.mark.parametrize("index,n", [(2, 5000), (5, 3000), (1, 200)])
def test_gpu_rank_matches_the_oracle(index, n):
    import torch

    import paper_2510_05112_amd as fp
    spec, words, ref = evaluated_batch(index, n)
    h = fp.Problem(spec.problem, spec.stride, device=0)
    res = h.evaluate(torch.from_numpy(words.view(np.int16)).cuda())
    for mode in MODES:
        for include in (False, True):
            for k in (1, 33, 1024):
                out = h.rank(res, k, mode, include)
                torch.cuda.synchronize()
                idx, k1, k2, cnt = oracle.rank(ref, k, mode, include)
                assert int(out["count"].item()) == cnt, (mode, include, k)
                assert np.array_equal(out["idx"].cpu().numpy(), idx), (mode, include, k)
                key = out["key"].cpu().numpy()
                two = mode in ("makespan_peak", "peak_makespan")
                expect = np.where(idx >= 0, (k1 << 32 | k2) if two else k1, oracle.INT64_MAX)
                assert np.array_equal(key, expect), (mode, include, k)
    # an empty batch and argument errors
    empty = {name: t[:0] for name, t in res.items()}
    out = h.rank(empty, 4)
    torch.cuda.synchronize()
    assert int(out["count"].item()) == 0 and np.all(out["idx"].cpu().numpy() == -1)
    with pytest.raises(fp.FpschedError):
        h.rank(res, 0)
    h.close()
