"""Invariants, degenerate inputs, flags/sentinels and top-k of the CPU oracle -- no GPU."""
import numpy as np
import pytest

import oracle
from helpers import batch_from_lists, perturb, random_valid_lists, two_tower_problem
from workloads.problem import (B, F, FD, L, O, R, W, chain_problem, gpipe_lists,
                               one_f_one_b_lists, pack_lists, pack_word)


def _rand_batch(prob, rng, n, pr=0.0, po=0.0):
    return batch_from_lists([random_valid_lists(prob, rng, pr, po) for _ in range(n)])


def test_lower_bounds_and_idle_identity():
    rng = np.random.default_rng(3)
    prob = chain_problem(4, 6, v=2, f=3, b=5, w=2, comm=2)
    words = _rand_batch(prob, rng, 60)
    r = oracle.evaluate(prob, words)
    assert np.all(r["flags"] == 0)
    S, m = prob.n_stages, prob.n_microbatches
    busy = np.zeros(4, np.int64)
    for s in range(S):
        busy[prob.stage_device[s]] += m * (prob.dur[F][s] + prob.dur[B][s] + prob.dur[W][s])
    crit = int(prob.dur[F].sum() + prob.dur[B].sum() + 2 * prob.edge_comm.sum() + prob.dur[W][0])
    assert np.all(r["makespan"] >= busy.max())
    assert np.all(r["makespan"] >= crit)
    assert np.all(r["idle"] >= 0)
    assert np.array_equal(r["idle"].sum(1), 4 * r["makespan"] - busy.sum())
    assert np.array_equal(r["idle"], r["makespan"][:, None] - busy[None, :])
    assert np.all(r["peak"] >= 1) and np.all(r["peak"] <= 2 * m)


def test_monotone_in_durations_and_comm():
    rng = np.random.default_rng(4)
    prob = chain_problem(3, 5, v=2, f=3, b=5, w=2, comm=2)
    words = _rand_batch(prob, rng, 40, pr=0.3)
    base = oracle.evaluate(prob, words)["makespan"]
    for _ in range(10):
        q = chain_problem(3, 5, v=2, f=3, b=5, w=2, comm=2)
        k = int(rng.choice([F, B, W, R, FD]))
        q.dur[k, int(rng.integers(6))] += int(rng.integers(1, 4))
        assert np.all(oracle.evaluate(q, words)["makespan"] >= base)
    q = chain_problem(3, 5, v=2, f=3, b=5, w=2, comm=0)
    assert np.all(oracle.evaluate(q, words)["makespan"] <= base)
    q = chain_problem(3, 5, v=2, f=3, b=5, w=2, comm=5)
    assert np.all(oracle.evaluate(q, words)["makespan"] >= base)


def test_all_forward_first_attains_peak_upper_bound():
    p, m, v = 3, 4, 2
    prob = chain_problem(p, m, v=v, f=1, b=1, w=1, comm=0)
    lists = []
    for d in range(p):
        ops = [(F, c, j) for c in range(v) for j in range(m)]
        ops += [(B, c, j) for c in reversed(range(v)) for j in range(m)]
        ops += [(W, c, j) for c in range(v) for j in range(m)]
        lists.append(ops)
    r = oracle.evaluate_trace(prob, pack_lists(lists))
    assert r["flags"] == 0 and list(r["peak"]) == [m * v] * p


def test_memory_accounting_of_each_kind():
    # one device, one stage, two micro-batches, 3 units per activation
    prob = chain_problem(1, 2, f=2, b=3, w=1, comm=0, r=2)
    prob.mem_units[:] = 3
    prob.dur[O] = 5
    prob.dur[L] = 5
    # F0 (+3) F1 (+3) -> 6 ; O0 (-3 at end) ; FD would not apply here
    lists = [[(F, 0, 0), (F, 0, 1), (O, 0, 0), (L, 0, 0), (B, 0, 0), (W, 0, 0), (B, 0, 1), (W, 0, 1)]]
    r = oracle.evaluate_trace(prob, pack_lists(lists))
    assert r["flags"] == 0 and r["peak"][0] == 6 and r["makespan"] == 2 + 2 + 5 + 5 + 3 + 1 + 3 + 1
    # discarded forward still counts while it runs: FD0 (+3, -3), FD1 (+3, -3) -> peak 3; R0, R1 -> 6
    lists = [[(FD, 0, 0), (FD, 0, 1), (R, 0, 0), (R, 0, 1), (B, 0, 0), (W, 0, 0), (B, 0, 1), (W, 0, 1)]]
    r = oracle.evaluate_trace(prob, pack_lists(lists))
    assert r["flags"] == 0 and r["peak"][0] == 6
    lists = [[(FD, 0, 0), (R, 0, 0), (B, 0, 0), (W, 0, 0), (FD, 0, 1), (R, 0, 1), (B, 0, 1), (W, 0, 1)]]
    r = oracle.evaluate_trace(prob, pack_lists(lists))
    assert r["flags"] == 0 and r["peak"][0] == 3
    # B frees nothing in split mode: F0 B0 F1 B1 W0 W1 -> peak 6; with has_w=0 B frees -> peak 3
    lists = [[(F, 0, 0), (B, 0, 0), (F, 0, 1), (B, 0, 1), (W, 0, 0), (W, 0, 1)]]
    assert oracle.evaluate_trace(prob, pack_lists(lists))["peak"][0] == 6
    q = chain_problem(1, 2, f=2, b=3, comm=0)
    q.mem_units[:] = 3
    lists = [[(F, 0, 0), (B, 0, 0), (F, 0, 1), (B, 0, 1)]]
    assert oracle.evaluate_trace(q, pack_lists(lists))["peak"][0] == 3


def test_flags_and_sentinels():
    prob = chain_problem(2, 2, f=1, b=1, comm=0, mem_cap=1)
    ok = gpipe_lists(2, 2)
    r = oracle.evaluate_trace(prob, pack_lists(ok))
    assert r["flags"] == oracle.FLAG_OVER_CAP and r["makespan"] == 6 and list(r["peak"]) == [2, 2]
    prob = chain_problem(2, 2, f=1, b=1, comm=0, mem_cap=2)
    assert oracle.evaluate_trace(prob, pack_lists(ok))["flags"] == 0

    def sent(lists):
        r = oracle.evaluate_trace(prob, pack_lists(lists))
        if r["flags"] & 3:
            assert r["makespan"] == oracle.INT64_MAX
            assert list(r["idle"]) == [-1, -1] and list(r["peak"]) == [-1, -1]
        return r["flags"]

    # same-device cycle: B before its own F
    assert sent([[(B, 0, 0), (F, 0, 0), (F, 0, 1), (B, 0, 1)], ok[1]]) == oracle.FLAG_DEADLOCK
    # cross-device cycle: F(1,1) <- F(0,1) <- B(0,0) <- B(1,0) <- F(1,1) (list order on device 1)
    assert sent([[(F, 0, 0), (B, 0, 0), (F, 0, 1), (B, 0, 1)],
                 [(F, 0, 1), (F, 0, 0), (B, 0, 1), (B, 0, 0)]]) == oracle.FLAG_DEADLOCK
    # an unusual but valid order (micro-batch 1 drains first)
    assert sent([[(F, 0, 0), (F, 0, 1), (B, 0, 1), (B, 0, 0)],
                 [(F, 0, 0), (F, 0, 1), (B, 0, 1), (B, 0, 0)]]) == 0
    assert sent([[(F, 0, 0), (B, 0, 1), (F, 0, 1), (B, 0, 0)], ok[1]]) == oracle.FLAG_DEADLOCK
    # duplicate op
    assert sent([[(F, 0, 0), (F, 0, 0), (B, 0, 0), (B, 0, 1)], ok[1]]) == oracle.FLAG_DEADLOCK
    # a whole micro-batch missing everywhere -> incomplete, not deadlock
    assert sent([[(F, 0, 0), (B, 0, 0)], [(F, 0, 0), (B, 0, 0)]]) == oracle.FLAG_INCOMPLETE
    # empty candidate -> incomplete
    assert sent([[], []]) == oracle.FLAG_INCOMPLETE
    # malformed words: chunk out of range, micro-batch out of range, W in a non-split problem
    bad = oracle.FLAG_DEADLOCK | oracle.FLAG_INCOMPLETE
    assert sent([[(F, 1, 0)], []]) == bad
    assert sent([[(F, 0, 5)], []]) == bad
    assert sent([ok[0] + [(W, 0, 0)], ok[1]]) == bad
    # a malformed word behind a true deadlock is never reached: plain deadlock
    assert sent([[(B, 0, 0), (F, 1, 0)], ok[1]]) == oracle.FLAG_DEADLOCK
    # words after the first END are ignored
    w = pack_lists(ok, stride=8)
    w[0, 5] = pack_word(F, 3, 77)
    assert oracle.evaluate_trace(prob, w)["flags"] == 0


def test_missing_backward_on_one_device_is_incomplete():
    prob = chain_problem(2, 2, f=1, b=1, comm=0)
    # device 0 lacks B(0,1); nothing waits on it, so every listed op issues
    r = oracle.evaluate_trace(prob, pack_lists([[(F, 0, 0), (F, 0, 1), (B, 0, 0)], gpipe_lists(2, 2)[1]]))
    assert r["flags"] == oracle.FLAG_INCOMPLETE


def test_zero_microbatch_free_devices_and_zero_durations():
    prob = chain_problem(3, 2, f=0, b=0, comm=0)
    r = oracle.evaluate_trace(prob, pack_lists(gpipe_lists(3, 2)))
    assert r["flags"] == 0 and r["makespan"] == 0 and list(r["idle"]) == [0, 0, 0]


def test_sweep_order_independence_via_device_relabelling():
    # reversing the device numbering changes the order in which the event loop visits
    # devices but not the schedule; results must be the mirrored ones
    rng = np.random.default_rng(9)
    p, m = 4, 5
    prob = chain_problem(p, m, f=2, b=3, w=1, comm=1)
    mirror = chain_problem(p, m, f=2, b=3, w=1, comm=1)
    mirror.stage_device[:] = [p - 1 - s for s in range(p)]
    for _ in range(20):
        lists = random_valid_lists(prob, rng)
        a = oracle.evaluate_trace(prob, pack_lists(lists))
        b = oracle.evaluate_trace(mirror, pack_lists(lists[::-1]))
        assert a["makespan"] == b["makespan"]
        assert list(a["idle"]) == list(b["idle"][::-1]) and list(a["peak"]) == list(b["peak"][::-1])


def test_batch_equals_one_by_one_and_threads():
    rng = np.random.default_rng(11)
    prob = two_tower_problem(m=3, has_w=1, comm=1, mem_cap=2)
    lists = [random_valid_lists(prob, rng, 0.2, 0.2) for _ in range(30)]
    lists += [perturb(x, rng, 2) for x in lists[:15]]
    words = batch_from_lists(lists)
    a = oracle.evaluate(prob, words)
    b = oracle.evaluate(prob, words, threads=3)
    for k in a:
        assert np.array_equal(a[k], b[k])
    for i in range(len(words)):
        one = oracle.evaluate_trace(prob, words[i])
        assert one["makespan"] == a["makespan"][i] and one["flags"] == a["flags"][i]
        assert np.array_equal(one["idle"], a["idle"][i]) and np.array_equal(one["peak"], a["peak"][i])


@pytest.mark.parametrize("k", [1, 3, 16, 64])
def test_topk_equals_stable_sort(k):
    rng = np.random.default_rng(k)
    n = 50
    makespan = rng.integers(10, 20, n).astype(np.int64)      # many ties
    flags = rng.choice([0, 0, 0, 1, 2, 4, 5], n).astype(np.uint8)
    makespan[flags & 3 != 0] = oracle.INT64_MAX
    idx, ms, cnt = oracle.topk(makespan, flags, k)
    feas = np.flatnonzero(flags == 0)
    order = feas[np.argsort(makespan[feas], kind="stable")]
    assert cnt == min(k, len(order))
    assert list(idx[:cnt]) == list(order[:cnt]) and list(ms[:cnt]) == list(makespan[order[:cnt]])
    assert np.all(idx[cnt:] == -1) and np.all(ms[cnt:] == oracle.INT64_MAX)


def test_topk_no_feasible_and_empty():
    idx, ms, cnt = oracle.topk(np.array([5, 6], np.int64), np.array([1, 4], np.uint8), 4)
    assert cnt == 0 and np.all(idx == -1)
    idx, ms, cnt = oracle.topk(np.zeros(0, np.int64), np.zeros(0, np.uint8), 2)
    assert cnt == 0 and np.all(idx == -1)


def test_decode_roundtrip():
    rng = np.random.default_rng(0)
    k = rng.integers(0, 8, 500)
    c = rng.integers(0, 4, 500)
    j = rng.integers(0, 2048, 500)
    words = np.array([pack_word(*t) for t in zip(k, c, j)], np.uint16)
    kk, cc, jj = oracle.decode(words)
    assert np.array_equal(kk, k) and np.array_equal(cc, c) and np.array_equal(jj, j)
    # hand-written words
    assert pack_word(F, 0, 0) == 0x2000 and pack_word(FD, 3, 2047) == 0xFFFF and pack_word(W, 1, 5) == 0x6805
    kk, cc, jj = oracle.decode(np.array([0x2000, 0xFFFF, 0x6805, 0x0000], np.uint16))
    assert list(kk) == [F, FD, W, 0] and list(cc) == [0, 3, 1, 0] and list(jj) == [0, 2047, 5, 0]
