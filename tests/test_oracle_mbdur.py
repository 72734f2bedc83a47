"""Pins of the oracle's per-micro-batch cost variant (dur_mb[kind][stage][micro-batch]), CPU only:
a closed form from flow-shop theory, a timeline worked out by hand, the critical-path checker with
per-item weights, and the plain model as the special case of a constant table."""
import numpy as np
import pytest

import checker
import oracle
import workloads
from helpers import batch_from_lists, perturb, random_valid_lists, two_tower_problem
from workloads.problem import B, F, chain_problem, gpipe_lists, pack_lists

NKINDS = 8


def constant_table(prob):
    return np.repeat(np.asarray(prob.dur, np.int32)[:, :, None], prob.n_microbatches, axis=2)


def random_table(prob, rng, lo=0, hi=12):
    t = rng.integers(lo, hi, (NKINDS, prob.n_stages, prob.n_microbatches)).astype(np.int32)
    t[7] = t[1]   # a forward pass costs the same whether its activation is kept or dropped
    return t


@pytest.mark.parametrize("p,m,c", [(2, 3, 0), (4, 8, 0), (4, 8, 2), (6, 5, 1), (3, 12, 0)])
def test_gpipe_with_proportional_costs_is_a_proportionate_flow_shop(p, m, c):
    # Every stage costs the same for a given micro-batch: f_j forward, b_j backward.  A permutation flow
    # shop whose jobs take the same time on every machine finishes at sum_j p_j + (machines - 1) max_j p_j,
    # whatever the order of the jobs.  The forward phase is such a shop, the backward phase another one in
    # the opposite direction that starts when the last device ends its forward items, and a latency c on
    # each of the p - 1 hops shifts each phase by (p - 1) c:
    #   makespan = sum_j (f_j + b_j) + (p - 1) (max f_j + max b_j + 2 c)
    rng = np.random.default_rng(100 * p + m)
    fj, bj = rng.integers(1, 9, m), rng.integers(1, 13, m)
    prob = chain_problem(p, m, f=1, b=1, comm=c)
    table = np.zeros((NKINDS, p, m), np.int32)
    table[F] = fj[None, :]
    table[B] = bj[None, :]
    r = oracle.evaluate(prob, pack_lists(gpipe_lists(p, m))[None], dur_mb=table)
    expect = int(fj.sum() + bj.sum() + (p - 1) * (fj.max() + bj.max() + 2 * c))
    assert r["flags"][0] == 0 and r["makespan"][0] == expect
    assert np.all(r["idle"][0] == expect - int(fj.sum() + bj.sum())) and np.all(r["peak"][0] == m)
    # equal costs: the uniform closed form (m + p - 1)(f + b) + 2 (p - 1) c
    table[F], table[B] = 3, 5
    r = oracle.evaluate(prob, pack_lists(gpipe_lists(p, m))[None], dur_mb=table)
    assert r["makespan"][0] == (m + p - 1) * 8 + 2 * (p - 1) * c


def test_hand_worked_timeline_with_a_different_cost_for_every_item():
    # two stages on two devices, latency 1, no split backward; every (type, stage, micro-batch) has its own
    # cost, so that any mix-up of the three indices changes the result
    #   F(0,0)=2 F(0,1)=3 F(1,0)=4 F(1,1)=1   B(0,0)=5 B(0,1)=2 B(1,0)=3 B(1,1)=6
    # device 0: F0 [0,2] F1 [2,5];  device 1: F0 ready 2+1: [3,7], B0 [7,10], F1 ready 5+1, free 10: [10,11],
    # B1 [11,17];  device 0: B0 needs 10+1: [11,16], B1 needs 17+1: [18,20]
    prob = chain_problem(2, 2, f=1, b=1, comm=1)
    table = np.zeros((NKINDS, 2, 2), np.int32)
    table[F] = [[2, 3], [4, 1]]
    table[B] = [[5, 2], [3, 6]]
    lists = [[(F, 0, 0), (F, 0, 1), (B, 0, 0), (B, 0, 1)], [(F, 0, 0), (B, 0, 0), (F, 0, 1), (B, 0, 1)]]
    o = oracle.evaluate_trace(prob, pack_lists(lists), dur_mb=table)
    assert o["makespan"] == 20 and o["flags"] == 0
    assert list(o["idle"]) == [8, 6] and list(o["peak"]) == [2, 1]
    assert list(o["start"][0][:4]) == [0, 2, 11, 18] and list(o["finish"][0][:4]) == [2, 5, 16, 20]
    assert list(o["start"][1][:4]) == [3, 7, 10, 11] and list(o["finish"][1][:4]) == [7, 10, 11, 17]


def _compare(prob, lists, table):
    words = pack_lists(lists, stride=-(-(max(len(x) for x in lists) + 1) // 8) * 8)
    o = oracle.evaluate_trace(prob, words, dur_mb=table)
    c = checker.check(prob, words, dur_mb=table)
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
                                           (3, 4, 1, 2, 0.3, 0.3), (2, 4, 4, 1, 0.2, 0.2)])
def test_critical_path_checker_with_per_item_weights(p, m, v, w, pr, po):
    rng = np.random.default_rng(4321 + 100 * p + m)
    prob = chain_problem(p, m, v=v, f=1, b=1, w=w, comm=0)
    prob.edge_comm[:] = rng.integers(0, 5, len(prob.edge_comm))
    table = random_table(prob, rng)
    seen = {"ok": 0, "deadlock": 0, "incomplete": 0}
    for t in range(30):
        lists = random_valid_lists(prob, rng, pr, po)
        assert _compare(prob, lists, table) == "ok"
        seen["ok"] += 1
        seen[_compare(prob, perturb(lists, rng, n_swaps=1 + t % 3), table)] += 1
    assert seen["ok"] >= 30 and seen["ok"] + seen["deadlock"] + seen["incomplete"] == 60


def test_checker_on_a_dag_with_a_join():
    rng = np.random.default_rng(5)
    prob = two_tower_problem(m=4, has_w=1, comm=2)
    table = random_table(prob, rng, 1, 9)
    for _ in range(30):
        assert _compare(prob, random_valid_lists(prob, rng, 0.2, 0.3), table) == "ok"


@pytest.mark.parametrize("index,n", [(2, 200), (3, 30), (4, 20), (5, 100)])
def test_a_constant_table_is_the_plain_model(index, n):
    spec = workloads.config(index, n)
    words = workloads.generate(spec, threads=4)
    plain = oracle.evaluate(spec.problem, words, threads=4)
    same = oracle.evaluate(spec.problem, words, threads=4, dur_mb=constant_table(spec.problem))
    for name in plain:
        assert np.array_equal(plain[name], same[name]), name


def test_the_variants_loop_with_both_switches_off_is_the_plain_definition():
    # fporacle.c holds the plain definition (eval_one) and, written out again with the two switches, the loop
    # of the cost-model variants: with no cost table and no link occupancy the second must repeat the first,
    # results and every op's times, also on lists that deadlock, end early or carry malformed words
    for index, n in ((2, 150), (5, 80)):
        spec = workloads.config(index, n)
        words = workloads.generate(spec, threads=4)
        a = oracle.evaluate(spec.problem, words, threads=4)
        b = oracle.evaluate(spec.problem, words, threads=4, variant_loop=True)
        for name in a:
            assert np.array_equal(a[name], b[name]), name
    rng = np.random.default_rng(77)
    prob = chain_problem(3, 4, v=2, f=2, b=3, w=1, comm=2)
    for trial in range(40):
        lists = random_valid_lists(prob, rng, 0.3, 0.3)
        if trial % 3 == 1:
            lists = perturb(lists, rng, 2)
        if trial % 3 == 2:
            lists = [l[:max(0, len(l) - int(rng.integers(0, 3)))] for l in lists]
        one = batch_from_lists([lists])[0]
        if trial % 10 == 9:
            one[0, 0] = np.uint16((3 << 13) | (3 << 11))   # a chunk the device does not have
        a, b = oracle.evaluate_trace(prob, one), oracle.evaluate_trace(prob, one, variant_loop=True)
        assert a["makespan"] == b["makespan"] and a["flags"] == b["flags"]
        for name in ("idle", "peak", "start", "finish"):
            assert np.array_equal(a[name], b[name]), (trial, name)


def test_raising_one_cost_never_shortens_a_schedule_and_busy_time_follows():
    spec = workloads.config(2, 60)
    prob, words = spec.problem, workloads.generate(spec, threads=4)
    rng = np.random.default_rng(9)
    table = constant_table(prob)
    base = oracle.evaluate(prob, words, threads=4, dur_mb=table)
    ok = base["flags"] & 3 == 0
    dev = np.asarray(prob.stage_device)
    for _ in range(6):
        kind, s, j = int(rng.choice([1, 2, 3] if prob.has_w else [1, 2])), int(rng.integers(prob.n_stages)), int(
            rng.integers(prob.n_microbatches))
        more = table.copy()
        more[kind, s, j] += 7
        if kind == 1:
            more[7, s, j] += 7
        r = oracle.evaluate(prob, words, threads=4, dur_mb=more)
        assert np.array_equal(r["flags"] & 3, base["flags"] & 3) and np.array_equal(r["peak"], base["peak"])
        assert np.all(r["makespan"][ok] >= base["makespan"][ok])
        assert np.all(r["makespan"][ok] <= base["makespan"][ok] + 7)
        # the device of that stage is busy 7 longer, every other device as long as before
        busy_r, busy_b = r["makespan"][ok, None] - r["idle"][ok], base["makespan"][ok, None] - base["idle"][ok]
        delta = np.zeros(prob.n_devices, np.int64)
        delta[dev[s]] = 7
        assert np.array_equal(busy_r - busy_b, np.broadcast_to(delta, busy_r.shape))
