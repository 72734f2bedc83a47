"""Pins of the oracle's link-occupancy variant (every ordered pair of devices is a link that carries one
value at a time), CPU only: timelines worked out by hand, closed forms for the two regimes of a GPipe
order, the critical-path checker with one node per transfer, and what ties the variant to the plain model."""
import copy

import numpy as np
import pytest

import checker
import oracle
import workloads
from helpers import perturb, random_valid_lists, two_tower_problem
from workloads.problem import B, F, chain_problem, gpipe_lists, pack_lists


def test_hand_worked_timeline_on_a_link_that_is_the_bottleneck():
    # two stages on two devices, three micro-batches, F = B = 1, latency 3 (longer than any item)
    # device 0: F0 [0,1] F1 [1,2] F2 [2,3]; link 0->1: leaves at 1, 4 (waits for the link), 7: arrives 4, 7, 10
    # device 1 (F0 B0 F1 B1 F2 B2): F0 [4,5] B0 [5,6] F1 [7,8] B1 [8,9] F2 [10,11] B2 [11,12]
    # link 1->0: leaves 6, 9, 12: arrives 9, 12, 15;  device 0: B0 [9,10] B1 [12,13] B2 [15,16]
    prob = chain_problem(2, 3, f=1, b=1, comm=3)
    lists = [[(F, 0, 0), (F, 0, 1), (F, 0, 2), (B, 0, 0), (B, 0, 1), (B, 0, 2)],
             [(F, 0, 0), (B, 0, 0), (F, 0, 1), (B, 0, 1), (F, 0, 2), (B, 0, 2)]]
    words = pack_lists(lists)
    o = oracle.evaluate_trace(prob, words, links=True)
    assert o["makespan"] == 16 and o["flags"] == 0
    assert list(o["start"][0][:6]) == [0, 1, 2, 9, 12, 15]
    assert list(o["start"][1][:6]) == [4, 5, 7, 8, 10, 11]
    assert list(o["idle"]) == [10, 10] and list(o["peak"]) == [3, 1]
    # as a pure latency the same lists take 14: F1 and F2 reach device 1 at 5 and 6
    assert oracle.evaluate_trace(prob, words)["makespan"] == 14


def test_two_stages_of_one_device_share_the_link_to_the_next_device():
    # circular placement, two devices, four stages: 0 and 2 on device 0, 1 and 3 on device 1; one
    # micro-batch, F = 1, B = 1, latency 2.  Forward: F(0) [0,1] -> arrives 3; F(1) [3,4] -> link 1->0,
    # arrives 6; F(2) [6,7] -> link 0->1 (free since 3), arrives 9; F(3) [9,10]; B(3) [10,11] -> link 1->0
    # (free since 6): arrives 13; B(2) [13,14] -> link 0->1: 16; B(1) [16,17] -> 19; B(0) [19,20].
    prob = chain_problem(2, 1, v=2, f=1, b=1, comm=2)
    lists = [[(F, 0, 0), (F, 1, 0), (B, 1, 0), (B, 0, 0)], [(F, 0, 0), (F, 1, 0), (B, 1, 0), (B, 0, 0)]]
    o = oracle.evaluate_trace(prob, pack_lists(lists), links=True)
    assert o["makespan"] == 20
    # with two micro-batches the two stages of device 0 compete for link 0->1:
    # device 0: F(0,0) [0,1] F(0,1) [1,2]: leave at 1 and 3, arrive 3 and 5; device 1: F(1,0) [3,4] F(1,1) [5,6]:
    # leave 4 and 6, arrive 6 and 8; device 0: F(2,0) [6,7] F(2,1) [8,9]: leave 7 and 9, arrive 9 and 11
    prob = chain_problem(2, 2, v=2, f=1, b=1, comm=2)
    lists = [[(F, 0, 0), (F, 0, 1), (F, 1, 0), (F, 1, 1), (B, 1, 0), (B, 1, 1), (B, 0, 0), (B, 0, 1)],
             [(F, 0, 0), (F, 0, 1), (F, 1, 0), (F, 1, 1), (B, 1, 0), (B, 1, 1), (B, 0, 0), (B, 0, 1)]]
    o = oracle.evaluate_trace(prob, pack_lists(lists), links=True)
    assert list(o["start"][0][:4]) == [0, 1, 6, 8] and list(o["start"][1][:4]) == [3, 5, 9, 11]
    c = checker.check(prob, pack_lists(lists), links=True)
    assert c["makespan"] == o["makespan"]


@pytest.mark.parametrize("p,m,f,b,c", [(2, 3, 1, 1, 3), (2, 8, 2, 4, 5), (4, 8, 2, 4, 4), (4, 6, 3, 2, 7), (3, 5, 1, 1, 1)])
def test_gpipe_when_the_links_are_the_bottleneck(p, m, f, b, c):
    # latency >= every item's cost: the first link passes one value every c, every later stage and link keeps
    # that pace without queueing; the last forward item ends at p f + (m + p - 2) c, the backward phase mirrors it:
    #   makespan = p (f + b) + 2 (m + p - 2) c
    assert c >= max(f, b)
    prob = chain_problem(p, m, f=f, b=b, comm=c)
    r = oracle.evaluate(prob, pack_lists(gpipe_lists(p, m))[None], links=True)
    assert r["flags"][0] == 0 and r["makespan"][0] == p * (f + b) + 2 * (m + p - 2) * c
    assert np.all(r["peak"][0] == m)


@pytest.mark.parametrize("p,m,f,b,c", [(2, 4, 3, 5, 3), (4, 8, 2, 4, 2), (4, 8, 2, 4, 1), (6, 5, 4, 4, 3)])
def test_gpipe_when_no_value_ever_waits_for_a_link(p, m, f, b, c):
    # latency <= every item's cost: values leave a device no faster than the link passes them on, so the
    # variant gives the closed form of the pure-latency model, (m + p - 1)(f + b) + 2 (p - 1) c
    assert c <= min(f, b)
    prob = chain_problem(p, m, f=f, b=b, comm=c)
    words = pack_lists(gpipe_lists(p, m))[None]
    r = oracle.evaluate(prob, words, links=True)
    assert r["makespan"][0] == (m + p - 1) * (f + b) + 2 * (p - 1) * c
    plain = oracle.evaluate(prob, words)
    for name in r:
        assert np.array_equal(r[name], plain[name]), name


def _compare(prob, lists):
    words = pack_lists(lists, stride=-(-(max(len(x) for x in lists) + 1) // 8) * 8)
    o = oracle.evaluate_trace(prob, words, links=True)
    c = checker.check(prob, words, links=True)
    if c["deadlock"]:
        assert o["flags"] & oracle.FLAG_DEADLOCK and o["makespan"] == oracle.INT64_MAX
        return "deadlock"
    if c["incomplete"]:
        assert o["flags"] == oracle.FLAG_INCOMPLETE
        return "incomplete"
    assert o["makespan"] == c["makespan"]
    assert list(o["idle"]) == c["idle"] and list(o["peak"]) == c["peak"]
    for (d, i), t in c["finish"].items():
        assert o["finish"][d][i] == t
    return "ok"


@pytest.mark.parametrize("p,m,v,w,pr,po", [(4, 6, 1, None, 0.0, 0.0), (3, 5, 2, 2, 0.4, 0.0),
                                           (3, 4, 1, 2, 0.3, 0.3), (2, 4, 4, 1, 0.2, 0.2), (5, 3, 2, 1, 0.0, 0.0)])
def test_critical_path_checker_with_transfer_nodes(p, m, v, w, pr, po):
    rng = np.random.default_rng(8642 + 100 * p + m)
    S = p * v
    prob = chain_problem(p, m, v=v, f=1, b=1, w=w, comm=0)
    prob.dur[1] = rng.integers(1, 6, S)
    prob.dur[7] = prob.dur[1]
    prob.dur[2] = rng.integers(1, 8, S)
    prob.dur[4] = rng.integers(0, 6, S)
    if w is not None:
        prob.dur[3] = rng.integers(0, 5, S)
    prob.dur[5] = rng.integers(1, 4, S)
    prob.dur[6] = rng.integers(1, 4, S)
    prob.edge_comm[:] = rng.integers(0, 9, len(prob.edge_comm))   # some links slower than the items
    seen = {"ok": 0, "deadlock": 0, "incomplete": 0}
    for t in range(30):
        lists = random_valid_lists(prob, rng, pr, po)
        assert _compare(prob, lists) == "ok"
        seen["ok"] += 1
        seen[_compare(prob, perturb(lists, rng, n_swaps=1 + t % 3))] += 1
    assert seen["ok"] >= 30


@pytest.mark.parametrize("has_w", [0, 1])
def test_checker_on_a_dag_whose_towers_join(has_w):
    rng = np.random.default_rng(31 + has_w)
    prob = two_tower_problem(m=4, has_w=has_w, comm=5)
    outcomes = set()
    for t in range(30):
        lists = random_valid_lists(prob, rng, 0.2, 0.3)
        assert _compare(prob, lists) == "ok"
        outcomes.add(_compare(prob, perturb(lists, rng, 2)))
    assert "deadlock" in outcomes


@pytest.mark.parametrize("index,n", [(2, 200), (3, 30), (5, 100)])
def test_against_the_plain_model_on_the_benchmark_shapes(index, n):
    spec = workloads.config(index, n)
    prob, words = spec.problem, workloads.generate(spec, threads=4)
    plain = oracle.evaluate(prob, words, threads=4)
    linked = oracle.evaluate(prob, words, threads=4, links=True)
    # a link only ever delays a value: same order rules, same memory, no shorter schedule
    assert np.array_equal(linked["flags"] & 3, plain["flags"] & 3)
    assert np.array_equal(linked["peak"], plain["peak"])
    ok = plain["flags"] & 3 == 0
    assert np.all(linked["makespan"][ok] >= plain["makespan"][ok])
    busy = lambda r: r["makespan"][ok, None] - r["idle"][ok]
    assert np.array_equal(busy(linked), busy(plain))
    # without latencies there is nothing to occupy
    free = copy.deepcopy(prob)
    free.edge_comm[:] = 0
    a, b = oracle.evaluate(free, words, threads=4), oracle.evaluate(free, words, threads=4, links=True)
    for name in a:
        assert np.array_equal(a[name], b[name]), name
    # slower links never help
    slow = copy.deepcopy(prob)
    slow.edge_comm[:] = np.asarray(prob.edge_comm) + 3
    slower = oracle.evaluate(slow, words, threads=4, links=True)
    assert np.all(slower["makespan"][ok] >= linked["makespan"][ok])


def test_both_variants_of_the_cost_model_together():
    # costs per micro-batch say what an item costs, links when its result arrives: the checker with per-item
    # weights and transfer nodes, and each variant alone as a special case of the pair
    rng = np.random.default_rng(77)
    prob = chain_problem(3, 5, v=2, f=1, b=1, w=2, comm=0)
    prob.edge_comm[:] = rng.integers(0, 9, len(prob.edge_comm))
    table = rng.integers(0, 9, (8, prob.n_stages, prob.n_microbatches)).astype(np.int32)
    table[7] = table[1]
    constant = np.repeat(np.asarray(prob.dur, np.int32)[:, :, None], prob.n_microbatches, axis=2)
    for t in range(25):
        lists = random_valid_lists(prob, rng, 0.3, 0.2)
        for cand in (lists, perturb(lists, rng, 2)):
            words = pack_lists(cand, stride=-(-(max(len(x) for x in cand) + 1) // 8) * 8)
            o = oracle.evaluate_trace(prob, words, dur_mb=table, links=True)
            c = checker.check(prob, words, dur_mb=table, links=True)
            if c["deadlock"] or c["incomplete"]:
                assert o["makespan"] == oracle.INT64_MAX
                continue
            assert o["makespan"] == c["makespan"] and list(o["idle"]) == c["idle"]
            for (d, i), fin in c["finish"].items():
                assert o["finish"][d][i] == fin
            same = oracle.evaluate_trace(prob, words, dur_mb=constant, links=True)
            alone = oracle.evaluate_trace(prob, words, links=True)
            assert same["makespan"] == alone["makespan"] and np.array_equal(same["finish"], alone["finish"])
    free = copy.deepcopy(prob)
    free.edge_comm[:] = 0
    words = pack_lists(lists, stride=-(-(max(len(x) for x in lists) + 1) // 8) * 8)
    a = oracle.evaluate_trace(free, words, dur_mb=table, links=True)
    b = oracle.evaluate_trace(free, words, dur_mb=table)
    assert a["makespan"] == b["makespan"] and np.array_equal(a["finish"], b["finish"])
