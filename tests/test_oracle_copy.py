"""Pins of the copy-engine oracle (oracle/fpcopyoracle.c; CPU only).

The paper does not say how an offload is timed, so the model (offload and reload items on a copy engine
beside the computation, a bounded number of transfers in the engine, memory over time) is pinned by what
mathematics fixes: the plain oracle where no list holds a transfer, timelines worked out by hand, bounds
against the plain model, and an independent checker (topological order + recurrences, sorted events).
"""
import numpy as np
import pytest

import oracle
import workloads
from copy_checker import check
from helpers import batch_from_lists, dag_problem, perturb, random_valid_lists, two_tower_problem
from workloads.problem import B, F, FD, L, O, R, W, chain_problem, make_problem, pack_lists

FIELDS = ("flags", "makespan", "idle", "peak")


@pytest.mark.parametrize("index,n", [(1, 300), (2, 300), (3, 60), (4, 12)])
def test_lists_without_transfers_are_timed_as_in_the_plain_model(index, n):
    spec = workloads.config(index, n)
    words = workloads.generate(spec, threads=4)
    plain = oracle.evaluate(spec.problem, words, threads=4)
    for depth in (1, 4):
        out = oracle.evaluate_copy(spec.problem, words, depth=depth, threads=4)
        for name in FIELDS:
            assert np.array_equal(out[name], plain[name]), (index, depth, name)


def one_device():
    # forward 3, backward 4, offload 5, reload 2; three micro-batches, the first two offloaded
    prob = make_problem(1, 1, 3, 0, [0], [], {F: 3, B: 4, O: 5, L: 2})
    ops = [(F, 0, 0), (O, 0, 0), (F, 0, 1), (O, 0, 1), (F, 0, 2), (L, 0, 0), (L, 0, 1), (B, 0, 0), (B, 0, 1), (B, 0, 2)]
    return prob, pack_lists([ops], 16)


def test_hand_worked_timeline_on_one_device():
    prob, words = one_device()
    # room for four transfers: nothing ever waits for room.
    # compute: F0 0-3, F1 3-6, F2 6-9;  copy: O0 handed over at 3: 3-8, O1 at 6: 8-13, L0 at 9: 13-15,
    # L1 at 9: 15-17;  B0 waits for its reload: 15-19, B1 (reload done at 17): 19-23, B2 23-27.
    t = oracle.evaluate_copy_trace(prob, words, depth=4)
    assert t["flags"] == 0 and t["makespan"] == 27 and list(t["idle"]) == [27 - 21]
    assert list(t["start"][0][:10]) == [0, 3, 3, 8, 6, 13, 15, 15, 19, 23]
    assert list(t["finish"][0][:10]) == [3, 8, 6, 13, 9, 15, 17, 19, 23, 27]
    # memory over time: +1 at 0, 3, 6 (three forward passes), -1 at 8 and 13 (offloads done), +1 at 13 and 15
    # (reloads begin), -1 at 19, 23, 27: never more than three
    assert list(t["peak"]) == [3]
    # room for one transfer: the walk waits in front of O1 until O0 is done (8), so F2 runs 8-11; in front
    # of L0 until O1 is done (13), in front of L1 until L0 is done (15)
    t = oracle.evaluate_copy_trace(prob, words, depth=1)
    assert list(t["start"][0][:10]) == [0, 3, 3, 8, 8, 13, 15, 15, 19, 23]
    assert list(t["finish"][0][:10]) == [3, 8, 6, 13, 11, 15, 17, 19, 23, 27]
    assert t["makespan"] == 27 and list(t["peak"]) == [3]     # F2's +1 at 8 counts before O0's -1 at 8
    # the plain model runs everything on one timeline: 3+5+3+5+3+2+2+4+4+4
    plain = oracle.evaluate_trace(prob, words)
    assert plain["makespan"] == 35 and list(plain["peak"]) == [3]


def test_memory_counts_an_allocation_before_a_release_of_the_copy_engine_at_the_same_time():
    # F0 0-3; O0 3-8; F1 3-8 (cost 5): its successor F2 starts at 8, the moment O0 releases: 1 (F1) + 1 (F0
    # still held until 8) + 1 (F2 allocated at 8, compute first) = 3; with O0 one unit shorter the release
    # comes first: 2
    for o_cost, expect in ((5, 3), (4, 2)):
        prob = make_problem(1, 2, 2, 0, [0, 0], [], {F: [3, 5], B: [1, 1], O: o_cost, L: 1})
        ops = [(F, 0, 0), (O, 0, 0), (F, 1, 0), (F, 1, 1), (B, 1, 0), (B, 1, 1), (L, 0, 0), (B, 0, 0), (F, 0, 1), (B, 0, 1)]
        t = oracle.evaluate_copy_trace(prob, pack_lists([ops], 16), depth=4)
        assert t["flags"] == 0 and list(t["start"][0][:4]) == [0, 3, 3, 8]
        # running sums: F(0,0) 1, F(1,0) 2, then at 8: F(1,1) 3 and the offload's release 2 (or first 1, then 2), ...
        assert list(t["peak"]) == [expect]


def slow_transfers():
    prob = chain_problem(3, 5, v=2, f=2, b=3, w=1, comm=1)
    prob.dur[O], prob.dur[L] = 9, 7          # transfers slower than the computation: the engine fills up
    return prob


PROBLEMS = {
    "chain": slow_transfers,
    "two_tower": lambda: two_tower_problem(m=4, has_w=1, comm=2, mem_cap=3),
    "diamond": lambda: dag_problem([(0, 1), (0, 2), (1, 3), (2, 3)], 4, [0, 1, 2, 0], 3, m=4, has_w=0, seed=3),
}


@pytest.mark.parametrize("name", sorted(PROBLEMS))
def test_against_the_independent_checker_and_the_plain_model(name):
    prob = PROBLEMS[name]()
    rng = np.random.default_rng(13)
    n_ok = n_dead = n_waited = 0
    for t in range(40):
        base = random_valid_lists(prob, rng, 0.25 * (t % 2), 0.5)
        for lists in (base, perturb(base, rng, 1 + t % 3)):
            words = pack_lists(lists, 8 * (-(-max(len(x) for x in lists) // 8) + 1))
            depth = 1 + t % 5
            tr = oracle.evaluate_copy_trace(prob, words, depth=depth)
            ref = check(prob, words, depth)
            assert bool(tr["flags"] & 1) == ref["deadlock"], (name, t)
            if ref["deadlock"]:
                n_dead += 1
                continue
            assert bool(tr["flags"] & 2) == ref["incomplete"]
            if ref["incomplete"]:
                continue
            assert tr["makespan"] == ref["makespan"] and list(tr["idle"]) == ref["idle"], (name, t)
            assert list(tr["peak"]) == ref["peak"], (name, t)
            for (d, i), fin in ref["finish"].items():
                assert tr["finish"][d][i] == fin and tr["start"][d][i] == ref["start"][(d, i)], (name, t, d, i)
            # transfers beside the computation never delay anything: every op ends no later than in the plain
            # model, a deeper engine never delays anything either
            plain = oracle.evaluate_trace(prob, words)
            live = plain["finish"] >= 0
            assert (tr["finish"][live] <= plain["finish"][live]).all() and tr["makespan"] <= plain["makespan"]
            deeper = oracle.evaluate_copy_trace(prob, words, depth=depth + 1)
            assert (deeper["finish"][live] <= tr["finish"][live]).all()
            n_waited += bool((deeper["finish"][live] < tr["finish"][live]).any())
            n_ok += 1
    assert n_ok > 35 and n_dead > 5 and (n_waited > 3 or name != "chain")


def test_batches_of_configuration_five_and_bad_arguments():
    spec = workloads.config(5, 400)
    words = workloads.generate(spec, threads=4)
    plain = oracle.evaluate(spec.problem, words, threads=4)
    out = oracle.evaluate_copy(spec.problem, words, depth=4, threads=4)
    assert np.array_equal(out["flags"] & 3, plain["flags"] & 3)          # who runs at all is a matter of order
    ok = (plain["flags"] & 3) == 0
    assert (out["makespan"][ok] <= plain["makespan"][ok]).all() and (out["makespan"][ok] < plain["makespan"][ok]).any()
    for i in np.flatnonzero(ok)[:25]:
        ref = check(spec.problem, words[i], 4)
        assert out["makespan"][i] == ref["makespan"] and list(out["peak"][i]) == ref["peak"] and list(out["idle"][i]) == ref["idle"]
    with pytest.raises(ValueError):
        oracle.evaluate_copy(spec.problem, words[:2], depth=0)
