"""GPU parity of fpsched_wslide_evaluate (the sliding pass without its lists) against oracle/fpslideoracle.c."""
import copy

import numpy as np
import pytest
import torch

import oracle
import paper_2510_05112_amd as fp
import workloads
from workloads.problem import B, F, chain_problem, pack_lists

pytestmark = pytest.mark.gpu

NAMES = ("makespan", "idle", "peak", "flags")


def to_gpu(words):
    return torch.from_numpy(np.ascontiguousarray(words).view(np.int16)).cuda()


def run_gpu(h, words):
    out = h.wslide_evaluate(to_gpu(words))
    torch.cuda.synchronize()
    return {k: v.cpu().numpy() for k, v in out.items()}


def assert_same(got, ref, what=""):
    for name in NAMES:
        bad = np.argwhere(got[name] != ref[name])
        assert bad.size == 0, (what, name, bad[:5].tolist(), got[name][tuple(bad[0])], ref[name][tuple(bad[0])])


@pytest.mark.parametrize("links", [False, True])
@pytest.mark.parametrize("index,n", [(2, 3001), (3, 700), (5, 2000), (4, 130)])
def test_matches_the_oracle_on_the_configurations(index, n, links):
    spec = workloads.config(index, n)
    words = workloads.generate(spec, threads=16)
    print(f"cfg{index}: {n} candidates, links={links}", flush=True)
    h = fp.Problem(spec.problem, spec.stride, device=0)
    h.set_link_occupancy(links)
    got = run_gpu(h, words)
    ref = oracle.wslide(spec.problem, words, spec.stride, threads=16, links=links)
    assert_same(got, ref, f"cfg{index}")
    assert ((ref["flags"] & 3) == 0).sum() > n // 2
    # and what the two-pass form reports
    two = h.wslide(to_gpu(words), spec.stride)
    torch.cuda.synchronize()
    for name in NAMES:
        assert np.array_equal(two[name].cpu().numpy(), got[name]), name
    h.close()


def test_lists_without_w_words_and_free_or_huge_items():
    spec = workloads.config(2, 1500)
    prob = spec.problem
    words = workloads.generate(spec, threads=16)
    kinds = words >> 13
    longest = int(((kinds != 0) & (kinds != 3)).sum(2).max())
    stride_in = -(-longest // 8) * 8
    stripped = np.zeros((words.shape[0], words.shape[1], stride_in), np.uint16)
    for c in range(words.shape[0]):
        for d in range(words.shape[1]):
            row = words[c, d]
            keep = row[((row >> 13) != 0) & ((row >> 13) != 3)]
            stripped[c, d, :len(keep)] = keep
    h = fp.Problem(prob, spec.stride, device=0)
    ref = oracle.wslide(prob, words, spec.stride, threads=16)
    assert_same(run_gpu(h, stripped), ref, "stripped")
    assert_same(run_gpu(h, words), ref, "with W words")
    h.close()
    # weight-gradient items that cost nothing, and ones longer than any idle time (every stash grows to all the
    # B items of its device: 64 entries, twice what the kernel's queue holds)
    for w_cost in (0, 5000):
        p2 = copy.deepcopy(prob)
        p2.dur[3] = w_cost
        h = fp.Problem(p2, spec.stride, device=0)
        assert_same(run_gpu(h, words[:600]), oracle.wslide(p2, words[:600], spec.stride, threads=16), f"W cost {w_cost}")
        h.close()


def test_small_cases_and_errors():
    prob = chain_problem(2, 2, v=1, f=2, b=2, w=1, comm=1)
    prob.dur[3] = [1, 3]
    lists = [[(F, 0, 0), (F, 0, 1), (B, 0, 0), (B, 0, 1)], [(F, 0, 0), (B, 0, 0), (F, 0, 1), (B, 0, 1)]]
    deadlock = [[(F, 0, 0), (B, 0, 0), (F, 0, 1), (B, 0, 1)], [(F, 0, 1), (B, 0, 1), (F, 0, 0), (B, 0, 0)]]
    malformed = [[(F, 0, 0), (F, 1, 0)], [(F, 0, 0), (B, 0, 0)]]
    early_end = [[(F, 0, 0)], [(F, 0, 0)]]
    words = np.stack([pack_lists(x, stride=8) for x in (lists, deadlock, malformed, early_end)])
    h = fp.Problem(prob, 8, device=0)
    got = run_gpu(h, words)
    ref = oracle.wslide(prob, words, 8)
    assert_same(got, ref, "small")
    assert list(ref["flags"]) == [0, 1, 3, 2] and ref["makespan"][0] == 17
    out = h.wslide_evaluate(to_gpu(words[:0]))
    torch.cuda.synchronize()
    assert out["makespan"].numel() == 0
    h.set_link_occupancy(True)
    assert_same(run_gpu(h, words), oracle.wslide(prob, words, 8, links=True), "small, links")
    h.set_link_occupancy(False)
    h.set_microbatch_costs(np.repeat(np.asarray(prob.dur)[:, :, None], 2, axis=2))
    with pytest.raises(fp.FpschedError):
        h.wslide_evaluate(to_gpu(words))
    h.close()
    spec = workloads.config(1, 16)
    h = fp.Problem(spec.problem, spec.stride, device=0)
    with pytest.raises(fp.FpschedError):
        h.wslide_evaluate(to_gpu(workloads.generate(spec)))
    h.close()


@pytest.mark.parametrize("links", [False, True])
def test_largest_sizes_and_long_stashes(links):
    from helpers import batch_from_lists, perturb, random_valid_lists
    from workloads.problem import gpipe_lists, one_f_one_b_lists

    def check(prob, words, what):
        h = fp.Problem(prob, words.shape[2], device=0)
        h.set_link_occupancy(links)
        got = run_gpu(h, words)
        assert_same(got, oracle.wslide(prob, words, words.shape[2], threads=8, links=links), what)
        h.close()
        return got

    m = 1024
    prob = chain_problem(2, m, f=1, b=2, w=1, comm=3)
    words = np.stack([pack_lists(gpipe_lists(2, m), stride=3 * m + 8), pack_lists(one_f_one_b_lists(2, m), stride=3 * m + 8)])
    got = check(prob, words, "m=1024")
    assert (got["flags"] == 0).all()
    prob = chain_problem(64, 6, f=2, b=4, w=3, comm=2)
    words = np.stack([pack_lists(gpipe_lists(64, 6), stride=24), pack_lists(one_f_one_b_lists(64, 6), stride=24)])
    check(prob, words, "p=64")
    prob = chain_problem(63, 3, v=4, f=2, b=3, w=1, comm=1)
    rng = np.random.default_rng(252)
    lists = []
    for t in range(6):
        base = random_valid_lists(prob, rng)
        lists += [base, perturb(base, rng, 2)]
    check(prob, batch_from_lists(lists), "S=252")
    # two and four stages per device with stashes deeper than the queue (32 / 16 entries): costs of the W items
    # between "fits most gaps" and "fits none", so that queues overflow, drain and are read back from the rows
    for v, mm in ((2, 96), (4, 40)):
        prob = chain_problem(3, mm, v=v, f=3, b=5, w=2, comm=2)
        S = 3 * v
        lists = []
        for t in range(24):
            base = random_valid_lists(prob, rng)
            lists += [base, perturb(base, rng, 1)]
        words = batch_from_lists(lists)
        for costs in ([40] * S, [1, 60] * (S // 2), [200] * S, list(rng.integers(0, 80, S))):
            p2 = copy.deepcopy(prob)
            p2.dur[3] = costs
            check(p2, words, f"v={v} W costs {costs}")
