"""GPU parity of fpsched_wslide (weight-gradient sliding) against oracle/fpslideoracle.c, through the C ABI."""
import copy

import numpy as np
import pytest
import torch

import oracle
import paper_2510_05112_amd as fp
import workloads
from workloads.problem import B, F, chain_problem, pack_lists

pytestmark = pytest.mark.gpu

NAMES = ("ops", "makespan", "idle", "peak", "flags")


def to_gpu(words):
    return torch.from_numpy(np.ascontiguousarray(words).view(np.int16)).cuda()


def run_gpu(h, words, stride_out):
    out = h.wslide(to_gpu(words), stride_out)
    torch.cuda.synchronize()
    got = {k: v.cpu().numpy() for k, v in out.items()}
    got["ops"] = got["ops"].view(np.uint16)
    return out, got


def assert_same(got, ref, what=""):
    for name in NAMES:
        assert np.array_equal(got[name], ref[name]), (what, name)


@pytest.mark.parametrize("index,n", [(2, 3001), (3, 700), (5, 2000), (4, 130)])
def test_matches_the_oracle_on_the_configurations(index, n):
    spec = workloads.config(index, n)
    words = workloads.generate(spec, threads=16)
    print(f"cfg{index}: {n} candidates", flush=True)
    h = fp.Problem(spec.problem, spec.stride, device=0)
    out, got = run_gpu(h, words, spec.stride)
    ref = oracle.wslide(spec.problem, words, spec.stride, threads=16)
    assert_same(got, ref, f"cfg{index}")
    assert ((ref["flags"] & 3) == 0).sum() > n // 2
    # the new lists, evaluated by the evaluation kernel, give the results the pass reported
    again = h.evaluate(out["ops"])
    torch.cuda.synchronize()
    ok = (ref["flags"] & 3) == 0
    for name in NAMES[1:]:
        assert np.array_equal(again[name].cpu().numpy()[ok], ref[name][ok]), name
    h.close()


def test_lists_without_w_words_short_rows_and_free_items():
    spec = workloads.config(2, 1500)
    prob = spec.problem
    words = workloads.generate(spec, threads=16)
    kinds = words >> 13
    # the same lists with their W words taken out, in a narrower row
    longest = int(((kinds != 0) & (kinds != 3)).sum(2).max())
    stride_in = -(-longest // 8) * 8
    stripped = np.zeros((words.shape[0], words.shape[1], stride_in), np.uint16)
    for c in range(words.shape[0]):
        for d in range(words.shape[1]):
            row = words[c, d]
            keep = row[((row >> 13) != 0) & ((row >> 13) != 3)]
            stripped[c, d, :len(keep)] = keep
    h = fp.Problem(prob, spec.stride, device=0)
    _, got = run_gpu(h, stripped, spec.stride)
    assert_same(got, oracle.wslide(prob, stripped, spec.stride, threads=16), "stripped")
    assert_same(got, oracle.wslide(prob, words, spec.stride, threads=16), "stripped == with W")
    # new rows too short for some candidates: those devices halt
    short = spec.stride - 16
    _, got = run_gpu(h, words, short)
    ref = oracle.wslide(prob, words, short, threads=16)
    assert_same(got, ref, "short rows")
    assert (ref["flags"] == 3).sum() > 0
    h.close()
    # weight-gradient items that cost nothing, and ones longer than any idle time
    for w_cost in (0, 5000):
        p2 = copy.deepcopy(prob)
        p2.dur[3] = w_cost
        h = fp.Problem(p2, spec.stride, device=0)
        _, got = run_gpu(h, words[:600], spec.stride)
        assert_same(got, oracle.wslide(p2, words[:600], spec.stride, threads=16), f"W cost {w_cost}")
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
    _, got = run_gpu(h, words, 8)
    ref = oracle.wslide(prob, words, 8)
    assert_same(got, ref, "small")
    assert list(ref["flags"]) == [0, 1, 3, 2] and ref["makespan"][0] == 17
    # the empty batch is a no-op
    out = h.wslide(to_gpu(words[:0]), 8)
    torch.cuda.synchronize()
    assert out["makespan"].numel() == 0
    # a row stride that is not a multiple of 8 words
    with pytest.raises(fp.FpschedError):
        h.wslide(to_gpu(words), 12)
    h.close()
    # a problem without split backward has no weight-gradient items
    spec = workloads.config(1, 16)
    h = fp.Problem(spec.problem, spec.stride, device=0)
    with pytest.raises(fp.FpschedError):
        h.wslide(to_gpu(workloads.generate(spec)), spec.stride)
    h.close()


@pytest.mark.parametrize("links", [False, True])
def test_largest_sizes_and_long_stashes(links):
    from helpers import batch_from_lists, perturb, random_valid_lists
    from workloads.problem import gpipe_lists, one_f_one_b_lists

    def check(prob, words, stride_out, what):
        h = fp.Problem(prob, max(words.shape[2], stride_out), device=0)
        if links:
            h.set_link_occupancy(True)
        _, got = run_gpu(h, words, stride_out)
        assert_same(got, oracle.wslide(prob, words, stride_out, threads=8, links=links), what)
        h.close()
        return got

    # GPipe order on two devices, 1024 micro-batches: the last device runs all its backward items back to back,
    # so its stash grows to 1024 items (far beyond the kernel's ring of 16) before anything can be placed
    m = 1024
    prob = chain_problem(2, m, f=1, b=2, w=1, comm=3)
    words = np.stack([pack_lists(gpipe_lists(2, m), stride=3 * m + 8), pack_lists(one_f_one_b_lists(2, m), stride=3 * m + 8)])
    got = check(prob, words, 3 * m + 8, "m=1024")
    assert (got["flags"] == 0).all()
    check(prob, words, 3 * m - 8, "m=1024, rows too short")
    # 64 devices; 252 stages on 63 devices
    prob = chain_problem(64, 6, f=2, b=4, w=3, comm=2)
    words = np.stack([pack_lists(gpipe_lists(64, 6), stride=24), pack_lists(one_f_one_b_lists(64, 6), stride=24)])
    check(prob, words, 24, "p=64")
    prob = chain_problem(63, 3, v=4, f=2, b=3, w=1, comm=1)
    rng = np.random.default_rng(252)
    lists = []
    for t in range(6):
        base = random_valid_lists(prob, rng)
        lists += [base, perturb(base, rng, 2)]
    words = batch_from_lists(lists)
    check(prob, words, words.shape[2] + 8, "S=252")


@pytest.mark.parametrize("links", [False, True])
def test_ops_that_wait_longer_than_sixteen_bits_of_time(links):
    # The hand-off between the two kernels carries the low sixteen bits of every start time; an op that waits
    # 2^16 time units or more for its inputs goes through the row's escape list.  Costs of up to 70,000 make
    # such waits common (several per row), next to ordinary ones; strides that are and are not multiples of 16.
    from helpers import batch_from_lists, perturb, random_valid_lists
    rng = np.random.default_rng(31)
    for p, m, v, stride_pad in ((2, 3, 1, 0), (4, 6, 2, 8), (3, 9, 1, 0)):
        prob = chain_problem(p, m, v=v, f=1, b=1, w=1, comm=3)
        S = p * v
        prob.dur[F] = rng.choice([3, 500, 66000, 70000], S)
        prob.dur[B] = rng.choice([7, 900, 66000, 69999], S)
        prob.dur[3] = rng.choice([1, 40, 65536, 30000], S)
        prob.edge_comm[:] = rng.choice([0, 2, 3], S - 1)
        lists = []
        for t in range(40):
            base = random_valid_lists(prob, rng)
            lists += [base, perturb(base, rng, 1 + t % 2)]
        words = batch_from_lists(lists)
        stride = words.shape[2] + stride_pad
        wide = np.zeros(words.shape[:2] + (stride,), np.uint16)
        wide[:, :, :words.shape[2]] = words
        h = fp.Problem(prob, stride, device=0)
        h.set_link_occupancy(links)
        _, got = run_gpu(h, wide, stride)
        ref = oracle.wslide(prob, wide, stride, links=links)
        assert_same(got, ref, f"p{p} m{m} v{v} links={links}")
        ok = (ref["flags"] & 3) == 0
        assert ok.sum() > 20 and ref["makespan"][ok].max() > 6 * 65536
        h.close()
