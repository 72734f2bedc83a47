"""Pins of the weight-gradient sliding oracle (oracle/fpslideoracle.c), CPU only.

The pass has no closed form of its own; it is pinned by what fixes it from outside: the evaluation
oracle applied to its output, the structure its output must have, special cases with a known
answer, and a timeline worked out by hand."""
import copy

import numpy as np
import pytest

import oracle
import workloads
from workloads.problem import B, F, W, chain_problem, one_f_one_b_lists, pack_lists

END = 0


def rows_of(words_one):
    """[(kind, chunk, mb), ...] per device, up to the first END word."""
    out = []
    for row in np.asarray(words_one):
        ops = []
        for w in row:
            if (int(w) >> 13) == END:
                break
            ops.append((int(w) >> 13, (int(w) >> 11) & 3, int(w) & 0x7ff))
        out.append(ops)
    return out


def strip_w(words):
    """The same lists without their W words (END-padded to the same stride)."""
    out = np.zeros_like(words)
    for c in range(words.shape[0]):
        for d, ops in enumerate(rows_of(words[c])):
            keep = [o for o in ops if o[0] != W]
            out[c, d, :len(keep)] = [(k << 13) | (ch << 11) | j for k, ch, j in keep]
    return out


def batch(index, n):
    spec = workloads.config(index, n)
    return spec, workloads.generate(spec, threads=4)


def test_hand_worked_timeline_on_two_devices():
    # stage 0 on device 0: F 2, B 2, W 1; stage 1 on device 1: F 2, B 2, W 3; latency 1 between them.
    # device 0: F0 [0,2] F1 [2,4]; device 1: F0 waits for 2+1: [3,5], B0 [5,7]; its W (3 long) does not
    # fit in front of F1 (device free at 7, F1 ready at 5): F1 [7,9], B1 [9,11], then W0 [11,14], W1 [14,17].
    # device 0: B0 waits for 7+1: [8,10]; B1 waits for 11+1 = 12, the device is free at 10 and W0 (1 long)
    # fits: W0 [10,11], B1 [12,14], at the end W1 [14,15].
    prob = chain_problem(2, 2, v=1, f=2, b=2, w=1, comm=1)
    prob.dur[W] = [1, 3]
    lists = [[(F, 0, 0), (F, 0, 1), (B, 0, 0), (B, 0, 1)], [(F, 0, 0), (B, 0, 0), (F, 0, 1), (B, 0, 1)]]
    r = oracle.wslide(prob, pack_lists(lists, stride=8)[None], 8)
    got = rows_of(r["ops"][0])
    assert got[0] == [(F, 0, 0), (F, 0, 1), (B, 0, 0), (W, 0, 0), (B, 0, 1), (W, 0, 1)]
    assert got[1] == [(F, 0, 0), (B, 0, 0), (F, 0, 1), (B, 0, 1), (W, 0, 0), (W, 0, 1)]
    assert r["makespan"][0] == 17 and r["flags"][0] == 0
    assert list(r["idle"][0]) == [7, 3] and list(r["peak"][0]) == [2, 2]


@pytest.mark.parametrize("index,n", [(2, 300), (3, 40), (5, 200)])
def test_output_evaluates_to_the_reported_results_and_keeps_the_order(index, n):
    spec, words = batch(index, n)
    prob = spec.problem
    r = oracle.wslide(prob, words, spec.stride, threads=4)
    again = oracle.evaluate(prob, r["ops"], threads=4)
    ok = (r["flags"] & 3) == 0
    assert ok.sum() > n // 2
    for name in ("makespan", "idle", "peak", "flags"):
        assert np.array_equal(again[name][ok], r[name][ok]), name
    # failed candidates: sentinels
    assert np.all(r["makespan"][~ok] == oracle.INT64_MAX) and np.all(r["peak"][~ok] == -1)
    # sliding only drops constraints: what deadlocks under it deadlocks as listed, too
    before = oracle.evaluate(prob, words, threads=4)
    assert not np.any(((r["flags"] & 1) != 0) & ((before["flags"] & 1) == 0))
    for c in np.flatnonzero(ok)[:60]:
        old, new = rows_of(words[c]), rows_of(r["ops"][c])
        for d in range(prob.n_devices):
            assert [o for o in new[d] if o[0] != W] == [o for o in old[d] if o[0] != W]
            seen_b, seen_w = set(), set()
            for k, ch, j in new[d]:
                if k == B:
                    seen_b.add((ch, j))
                if k == W:
                    assert (ch, j) in seen_b and (ch, j) not in seen_w   # behind its B, once
                    seen_w.add((ch, j))
            assert seen_b == seen_w
    # where the input's W words stood does not matter
    r2 = oracle.wslide(prob, strip_w(words), spec.stride, threads=4)
    for name in r:
        assert np.array_equal(r[name], r2[name]), name


@pytest.mark.parametrize("index", [2, 5])
def test_items_of_the_list_keep_the_times_of_the_list_without_w(index):
    # a stashed item only runs where it delays nothing, so every other item starts when it would start if
    # there were no W items at all: the traces of the evaluation oracle on the new list and on the list
    # with its W words taken out agree item by item
    spec, words = batch(index, 30)
    prob = spec.problem
    r = oracle.wslide(prob, words, spec.stride, threads=4)
    bare = strip_w(words)
    for c in np.flatnonzero((r["flags"] & 3) == 0)[:12]:
        new, old = oracle.evaluate_trace(prob, r["ops"][c]), oracle.evaluate_trace(prob, bare[c])
        for d in range(prob.n_devices):
            keep = (r["ops"][c, d] >> 13 != 0) & (r["ops"][c, d] >> 13 != W)
            n = int(keep.sum())
            assert np.array_equal(new["start"][d][keep], old["start"][d][:n])
            assert np.array_equal(new["finish"][d][keep], old["finish"][d][:n])


def test_items_of_zero_cost_follow_their_backward_item_at_once():
    spec, words = batch(2, 150)
    prob = copy.deepcopy(spec.problem)
    prob.dur[W] = 0
    r = oracle.wslide(prob, words, spec.stride, threads=4)
    # the expected lists: every B directly followed by its W
    fused = np.zeros_like(words)
    for c in range(words.shape[0]):
        for d, ops in enumerate(rows_of(words[c])):
            new = []
            for k, ch, j in ops:
                if k == W:
                    continue
                new.append((k << 13) | (ch << 11) | j)
                if k == B:
                    new.append((W << 13) | (ch << 11) | j)
            fused[c, d, :len(new)] = new
    ref = oracle.evaluate(prob, fused, threads=4)
    ok = (ref["flags"] & 3) == 0
    assert ok.sum() > 100
    assert np.array_equal(r["ops"][ok], fused[ok])
    for name in ("makespan", "idle", "peak", "flags"):
        assert np.array_equal(r[name][ok], ref[name][ok]), name


def test_one_device_alone_has_no_idle_time_to_fill():
    m = 5
    prob = chain_problem(1, m, v=2, f=3, b=4, w=2, comm=0)
    ops = []
    for j in range(m):
        ops += [(F, 0, j), (F, 1, j), (B, 1, j), (B, 0, j)]
    r = oracle.wslide(prob, pack_lists([ops], stride=32)[None], 32)
    expect = ops + [(W, ch, j) for j in range(m) for ch in (1, 0)]
    assert rows_of(r["ops"][0])[0] == expect
    assert r["makespan"][0] == 2 * m * (3 + 4 + 2) and r["idle"][0][0] == 0 and r["flags"][0] == 0
    assert r["peak"][0][0] == 2 * m   # nothing is freed before the last backward item


@pytest.mark.parametrize("p,m", [(2, 4), (4, 8), (4, 4), (8, 16), (3, 7)])
def test_one_f_one_b_with_unit_costs_reaches_the_known_bubble(p, m):
    # 1F1B order, F = B = W = 1, no latency: sliding leaves the bubble (p - 1)(F + B - W) per device that the
    # zero-bubble literature states for its hand-made schedule of this kind, i.e. makespan 3 m + p - 1;
    # with W fused behind B the same order takes (m + p - 1)(F + B + W)
    prob = chain_problem(p, m, v=1, f=1, b=1, w=1, comm=0)
    words = pack_lists(one_f_one_b_lists(p, m), stride=3 * m + 8)[None]
    r = oracle.wslide(prob, words, 3 * m + 8)
    assert r["flags"][0] == 0 and r["makespan"][0] == 3 * m + p - 1
    assert np.all(r["idle"][0] == p - 1)


def test_a_row_that_is_too_short_keeps_the_head_of_its_list():
    spec, words = batch(2, 40)
    prob = spec.problem
    full = oracle.wslide(prob, words, spec.stride, threads=4)
    longest = max(len(ops) for c in range(40) for ops in rows_of(full["ops"][c]))
    short = (longest - 8) // 8 * 8
    r = oracle.wslide(prob, words, short, threads=4)
    hit = 0
    for c in range(40):
        f_rows, s_rows = rows_of(full["ops"][c]), rows_of(r["ops"][c])
        for a, b in zip(f_rows, s_rows):
            assert b == a[:short]   # every row: the first `short` items of the full row, whatever the others do
        if max(len(x) for x in f_rows) > short:
            hit += 1
            assert r["flags"][c] == 3 and r["makespan"][c] == oracle.INT64_MAX and np.all(r["peak"][c] == -1)
        else:
            for name in ("makespan", "idle", "peak", "flags"):
                assert np.array_equal(r[name][c], full[name][c])
    assert hit > 0


def test_deadlocked_order_and_malformed_words():
    prob = chain_problem(2, 2, v=1, f=1, b=1, w=1, comm=0)
    # device 1 wants micro-batch 1 first, device 0 sends micro-batch 0 first and waits for its backward pass
    lists = [[(F, 0, 0), (B, 0, 0), (F, 0, 1), (B, 0, 1)], [(F, 0, 1), (B, 0, 1), (F, 0, 0), (B, 0, 0)]]
    r = oracle.wslide(prob, pack_lists(lists, stride=8)[None], 8)
    assert r["flags"][0] == 1 and r["makespan"][0] == oracle.INT64_MAX
    assert rows_of(r["ops"][0]) == [[(F, 0, 0)], []]
    # a chunk the device does not have
    lists = [[(F, 0, 0), (F, 1, 0)], [(F, 0, 0), (B, 0, 0)]]
    r = oracle.wslide(prob, pack_lists(lists, stride=8)[None], 8)
    assert r["flags"][0] == 3
    # lists that end early: everything issued, activations unfinished
    lists = [[(F, 0, 0)], [(F, 0, 0)]]
    r = oracle.wslide(prob, pack_lists(lists, stride=8)[None], 8)
    assert r["flags"][0] == 2
    # a problem without split backward is refused
    with pytest.raises(ValueError):
        oracle.wslide(chain_problem(2, 2), pack_lists(lists, stride=8)[None], 8)


# ---- the pass under the link-occupancy variant of the cost model ------------------------------------

def slow_links(prob, seed):
    rng = np.random.default_rng(seed)
    slow = copy.deepcopy(prob)
    slow.edge_comm[:] = rng.integers(0, 2 * int(np.median(np.asarray(prob.dur)[F])) + 2, len(slow.edge_comm))
    return slow


@pytest.mark.parametrize("index,n", [(2, 300), (3, 40), (5, 200)])
def test_links_the_output_evaluates_to_the_reported_results(index, n):
    # the evaluation oracle (another file, another event loop) in its link form on the new lists
    spec, words = batch(index, n)
    prob = slow_links(spec.problem, index)
    r = oracle.wslide(prob, words, spec.stride, threads=4, links=True)
    again = oracle.evaluate(prob, r["ops"], threads=4, links=True)
    ok = (r["flags"] & 3) == 0
    assert ok.sum() > n // 2
    for name in ("makespan", "idle", "peak", "flags"):
        assert np.array_equal(again[name][ok], r[name][ok]), name
    assert np.all(r["makespan"][~ok] == oracle.INT64_MAX)
    # the links matter, and the order of the list items does not depend on the model
    plain = oracle.wslide(prob, words, spec.stride, threads=4)
    assert (r["makespan"][ok] > plain["makespan"][ok]).any()
    for c in np.flatnonzero(ok)[:40]:
        for a, b in zip(rows_of(r["ops"][c]), rows_of(plain["ops"][c])):
            assert [o for o in a if o[0] != W] == [o for o in b if o[0] != W]
    # without latencies the two models are one
    free = copy.deepcopy(prob)
    free.edge_comm[:] = 0
    a, b = oracle.wslide(free, words, spec.stride, threads=4), oracle.wslide(free, words, spec.stride, threads=4, links=True)
    for name in a:
        assert np.array_equal(a[name], b[name]), name


def test_links_items_of_the_list_keep_the_times_of_the_list_without_w():
    spec, words = batch(2, 30)
    prob = slow_links(spec.problem, 11)
    r = oracle.wslide(prob, words, spec.stride, threads=4, links=True)
    bare = strip_w(words)
    for c in np.flatnonzero((r["flags"] & 3) == 0)[:12]:
        new = oracle.evaluate_trace(prob, r["ops"][c], links=True)
        old = oracle.evaluate_trace(prob, bare[c], links=True)
        for d in range(prob.n_devices):
            keep = (r["ops"][c, d] >> 13 != 0) & (r["ops"][c, d] >> 13 != W)
            n = int(keep.sum())
            assert np.array_equal(new["start"][d][keep], old["start"][d][:n])


def test_links_hand_worked_timeline():
    # two stages on two devices, F = B = 1, W = 1, latency 3: the links are the bottleneck (the timeline of
    # tests/test_oracle_links.py); device 0 waits for its gradients from 3 to 9, then for 2 between them
    # device 0: F0 F1 F2 [0,3]; B0 [9,10] B1 [12,13] B2 [15,16]; stash after B0: W0 runs [10,11] (ends before 12),
    # W1 [13,14], W2 at the end [16,17]
    # device 1: F0 [4,5] B0 [5,6] then F1 is ready at 7: W0 [6,7] fits; F1 [7,8] B1 [8,9] W1 [9,10] F2 [10,11]
    # B2 [11,12] W2 [12,13]
    prob = chain_problem(2, 3, f=1, b=1, w=1, comm=3)
    lists = [[(F, 0, 0), (F, 0, 1), (F, 0, 2), (B, 0, 0), (B, 0, 1), (B, 0, 2)],
             [(F, 0, 0), (B, 0, 0), (F, 0, 1), (B, 0, 1), (F, 0, 2), (B, 0, 2)]]
    r = oracle.wslide(prob, pack_lists(lists, stride=16)[None], 16, links=True)
    got = rows_of(r["ops"][0])
    assert got[0] == [(F, 0, 0), (F, 0, 1), (F, 0, 2), (B, 0, 0), (W, 0, 0), (B, 0, 1), (W, 0, 1), (B, 0, 2), (W, 0, 2)]
    assert got[1] == [(F, 0, 0), (B, 0, 0), (W, 0, 0), (F, 0, 1), (B, 0, 1), (W, 0, 1), (F, 0, 2), (B, 0, 2), (W, 0, 2)]
    assert r["makespan"][0] == 17 and r["flags"][0] == 0
