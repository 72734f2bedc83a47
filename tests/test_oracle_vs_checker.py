"""Pins of the CPU oracle against an independent critical-path (Kahn + longest
path) checker on random valid and perturbed candidates -- no GPU."""
import numpy as np
import pytest

import checker
import oracle
from helpers import perturb, random_valid_lists, two_tower_problem
from workloads.problem import (chain_problem, gpipe_lists, one_f_one_b_lists, pack_lists)


def _compare(problem, lists):
    words = pack_lists(lists, stride=-(-(max(len(x) for x in lists) + 1) // 8) * 8)
    o = oracle.evaluate_trace(problem, words)
    c = checker.check(problem, words)
    if c["deadlock"]:
        assert o["flags"] & oracle.FLAG_DEADLOCK
        assert o["makespan"] == oracle.INT64_MAX
        assert all(o["idle"] == -1) and all(o["peak"] == -1)
        return "deadlock"
    assert not (o["flags"] & oracle.FLAG_DEADLOCK)
    if c["incomplete"]:
        assert o["flags"] == oracle.FLAG_INCOMPLETE
        assert o["makespan"] == oracle.INT64_MAX
        return "incomplete"
    assert o["makespan"] == c["makespan"]
    assert list(o["idle"]) == c["idle"]
    assert list(o["peak"]) == c["peak"]
    for (d, i), t in c["finish"].items():
        assert o["finish"][d][i] == t
    over = any(pk > cap for pk, cap in zip(c["peak"], problem.mem_cap))
    assert o["flags"] == (oracle.FLAG_OVER_CAP if over else 0)
    return "ok"


def test_golden_1f1b_rows_by_checker():
    # the 1F1B rows with comm > 0 in tests/golden/closed_forms.txt come from the checker
    for c, ms in [(0, 66), (1, 82), (2, 98)]:
        prob = chain_problem(4, 8, f=2, b=4, comm=c)
        r = checker.check(prob, pack_lists(one_f_one_b_lists(4, 8)))
        assert r["makespan"] == ms and r["peak"] == [4, 3, 2, 1]
    for c, ms in [(0, 66), (1, 72), (2, 78)]:
        prob = chain_problem(4, 8, f=2, b=4, comm=c)
        assert checker.check(prob, pack_lists(gpipe_lists(4, 8)))["makespan"] == ms


CASES = [
    dict(p=4, m=6, v=1, w=None, pr=0.0, po=0.0),
    dict(p=4, m=5, v=2, w=3, pr=0.0, po=0.0),
    dict(p=3, m=5, v=2, w=2, pr=0.4, po=0.0),
    dict(p=3, m=4, v=1, w=2, pr=0.3, po=0.3),
    dict(p=2, m=4, v=4, w=1, pr=0.2, po=0.2),
    dict(p=5, m=3, v=1, w=None, pr=0.5, po=0.5),
]


@pytest.mark.parametrize("case", CASES)
def test_random_valid_and_perturbed_chain(case):
    rng = np.random.default_rng(1234 + case["p"] * 100 + case["m"])
    S = case["p"] * case["v"]
    prob = chain_problem(case["p"], case["m"], v=case["v"], f=1, b=1, w=case["w"], comm=0)
    # heterogeneous integer durations / comm / units / caps
    prob.dur[1] = rng.integers(1, 9, S)
    prob.dur[7] = prob.dur[1]
    prob.dur[4] = rng.integers(0, 9, S)
    prob.dur[2] = rng.integers(1, 15, S)
    if case["w"] is not None:
        prob.dur[3] = rng.integers(0, 7, S)
    prob.dur[5] = rng.integers(1, 6, S)
    prob.dur[6] = rng.integers(1, 6, S)
    prob.edge_comm[:] = rng.integers(0, 5, len(prob.edge_comm))
    prob.mem_units[:] = rng.integers(1, 4, S)
    prob.mem_cap[:] = rng.integers(3, 4 * case["m"] * case["v"], case["p"])
    seen = {"ok": 0, "deadlock": 0, "incomplete": 0}
    for t in range(40):
        lists = random_valid_lists(prob, rng, case["pr"], case["po"])
        assert _compare(prob, lists) == "ok"
        seen["ok"] += 1
        seen[_compare(prob, perturb(lists, rng, n_swaps=1 + t % 3))] += 1
        # drop one op -> incomplete or deadlock
        d = int(rng.integers(case["p"]))
        cut = [list(x) for x in lists]
        if cut[d]:
            cut[d].pop(int(rng.integers(len(cut[d]))))
            seen[_compare(prob, cut)] += 1
    assert seen["deadlock"] > 0 and seen["ok"] > 40


@pytest.mark.parametrize("has_w", [0, 1])
def test_random_two_tower_dag(has_w):
    rng = np.random.default_rng(77 + has_w)
    prob = two_tower_problem(m=4, has_w=has_w, comm=2, mem_cap=3)
    kinds = {"ok": 0, "deadlock": 0, "incomplete": 0}
    for t in range(40):
        lists = random_valid_lists(prob, rng, 0.2, 0.3)
        assert _compare(prob, lists) == "ok"
        kinds[_compare(prob, perturb(lists, rng, 2))] += 1
    assert kinds["deadlock"] > 0


def test_merge_stage_waits_for_both_towers():
    from workloads.problem import B, F, W
    prob = two_tower_problem(m=1, has_w=1, comm=2)
    lists = [[(F, 0, 0), (B, 0, 0), (W, 0, 0)] for _ in range(6)]
    o = oracle.evaluate_trace(prob, pack_lists(lists))
    # tower A: 3+2+3 = 8 -> ready at 10 on device 4; tower B: 2+2+2 = 6 -> ready at 8
    assert o["start"][4][0] == 10
    assert _compare(prob, lists) == "ok"
