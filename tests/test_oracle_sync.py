"""Pins of the oracle for synchronisation stages and dependency pairs (oracle/fpsyncoracle.c; CPU only).

The paper prints no timeline of a schedule with a registered instruction, so the model (Section 4.2:
a registered synchronisation attached to a stage of its own, dependencies given as pairs; Section 2.2:
one synchronisation every few micro-batches) is pinned by what mathematics fixes: the plain oracle where
the new inputs are trivial (two files, two event loops), a pair that doubles a DAG edge, a timeline worked
out by hand, a closed form, an independent critical-path checker, and monotonicity.
"""
import numpy as np
import pytest

import oracle
import workloads
from helpers import (batch_from_lists, dag_problem, perturb, random_sync_lists, random_sync_problem,
                     random_valid_lists, two_tower_problem)
from sync_checker import check
from workloads.problem import B, F, FD, L, O, R, W, chain_problem, gpipe_lists, make_problem, pack_lists, pack_word

FIELDS = ("flags", "makespan", "idle", "peak")


def assert_same(a, b, what=""):
    for name in FIELDS:
        assert np.array_equal(a[name], b[name]), (what, name)


@pytest.mark.parametrize("index,n", [(1, 300), (2, 300), (3, 60), (4, 12), (5, 400)])
def test_group_one_and_no_pairs_is_the_plain_model(index, n):
    spec = workloads.config(index, n)
    words = workloads.generate(spec, threads=4)
    plain = oracle.evaluate(spec.problem, words, threads=4)
    assert_same(oracle.evaluate_sync(spec.problem, words, threads=4), plain, f"cfg{index}")
    if index in (2, 5):
        assert (plain["flags"] & 1).any()      # deadlocking candidates are part of the comparison


def test_plain_model_on_random_lists_with_recompute_offload_and_perturbations():
    rng = np.random.default_rng(7)
    for prob in (two_tower_problem(m=4, has_w=1, comm=2, mem_cap=3), chain_problem(3, 5, v=2, f=2, b=3, w=1, comm=1),
                 dag_problem([(0, 1), (0, 2), (1, 3), (2, 3)], 4, [0, 1, 2, 0], 3, m=4, has_w=0, seed=3)):
        lists = []
        for t in range(60):
            base = random_valid_lists(prob, rng, 0.3 * (t % 2), 0.3 * ((t // 2) % 2))
            lists += [base, perturb(base, rng, 1 + t % 3)]
        words = batch_from_lists(lists)
        assert_same(oracle.evaluate_sync(prob, words), oracle.evaluate(prob, words), prob.name)


def test_pairs_that_double_a_dag_edge_change_nothing_and_pairs_replace_an_edge():
    # edge a -> b of the stage DAG == the pairs ((F, a), (F, b)) and ((B, b), (B, a)) with its latency
    rng = np.random.default_rng(11)
    prob = chain_problem(4, 6, v=2, f=3, b=5, w=2, comm=2)
    lists = [random_valid_lists(prob, rng, 0.2, 0.0) for _ in range(40)]
    lists += [perturb(x, rng, 2) for x in lists]
    words = batch_from_lists(lists)
    plain = oracle.evaluate(prob, words)
    e = 3                                              # stage 3 (device 3) -> stage 4 (device 0)
    a, b, c = int(prob.edge_src[e]), int(prob.edge_dst[e]), int(prob.edge_comm[e])
    doubled = [(F, a, F, b, c), (B, b, B, a, c)]
    assert_same(oracle.evaluate_sync(prob, words, pairs=doubled), plain, "doubled")
    keep = [i for i in range(len(prob.edge_src)) if i != e]
    cut = make_problem(prob.n_devices, prob.n_stages, prob.n_microbatches, prob.has_w, prob.stage_device,
                       [(int(prob.edge_src[i]), int(prob.edge_dst[i]), int(prob.edge_comm[i])) for i in keep],
                       prob.dur, prob.mem_units, prob.mem_cap)
    assert_same(oracle.evaluate_sync(cut, words, pairs=doubled), plain, "replaced")
    # without the pairs the cut problem is a different one (the lists then run two independent chains)
    assert not np.array_equal(oracle.evaluate_sync(cut, words)["makespan"], plain["makespan"])


def sync_example():
    """Two towers of one stage each (stage 0 on device 0, stage 1 on device 1) and a synchronisation
    stage 2 on device 1 that gathers every two micro-batches; no split backward."""
    dur = {F: [2, 3, 1], B: [4, 5, 1]}
    prob = make_problem(2, 3, 2, 0, [0, 1, 1], [(0, 2, 1), (1, 2, 7)], dur, mem_units=[1, 1, 0])
    lists = [[(F, 0, 0), (F, 0, 1), (B, 0, 0), (B, 0, 1)],
             [(F, 0, 0), (F, 0, 1), (F, 1, 0), (B, 1, 0), (B, 0, 0), (B, 0, 1)]]
    return prob, [1, 1, 2], lists


def test_hand_worked_timeline_with_a_synchronisation_every_two_micro_batches():
    # device 0: F(0,0) 0-2, F(0,1) 2-4.  device 1: F(1,0) 0-3, F(1,1) 3-6.  The synchronisation item
    # covers micro-batches 0 and 1: it waits for both forward passes of stage 0 (finish 2 and 4, plus
    # latency 1 = 5) and of stage 1 (3 and 6; same device, the edge's latency 7 does not apply) and for
    # its device (free at 6): 6-7.  Its backward item: 7-8.  Backward of stage 1 (same device): 8-13,
    # 13-18.  Backward of stage 0 waits for 8 + 1 = 9: 9-13, 13-17.  Makespan 18; device 0 works 12 of
    # them, device 1 all 18; two activations at most on either device (the synchronisation holds none).
    prob, group, lists = sync_example()
    words = pack_lists(lists, 8)
    t = oracle.evaluate_sync_trace(prob, words, group=group)
    assert t["flags"] == 0 and t["makespan"] == 18
    assert list(t["idle"]) == [6, 0] and list(t["peak"]) == [2, 2]
    assert list(t["start"][0][:4]) == [0, 2, 9, 13] and list(t["finish"][0][:4]) == [2, 4, 13, 17]
    assert list(t["start"][1][:6]) == [0, 3, 6, 7, 8, 13] and list(t["finish"][1][:6]) == [3, 6, 7, 8, 13, 18]
    # with group 1 the backward pass of micro-batch 1 waits for a second synchronisation item that is in
    # no list
    assert oracle.evaluate_sync(prob, words[None])["flags"][0] == oracle.FLAG_DEADLOCK
    # the synchronisation placed before the second forward pass of its own device can never run
    early = [lists[0], [lists[1][0], lists[1][2], lists[1][1]] + lists[1][3:]]
    assert oracle.evaluate_sync(prob, pack_lists(early, 8)[None], group=group)["flags"][0] == oracle.FLAG_DEADLOCK
    # an item index beyond the stage's item count is a malformed word
    bad = [lists[0], lists[1][:2] + [(F, 1, 1)] + lists[1][3:]]
    assert oracle.evaluate_sync(prob, pack_lists(bad, 8)[None], group=group)["flags"][0] == 3


@pytest.mark.parametrize("p,m,f,b,c,sigma", [(2, 3, 2, 4, 0, 5), (4, 8, 2, 4, 1, 3), (3, 5, 1, 1, 2, 0), (5, 4, 3, 2, 1, 7)])
def test_gpipe_with_one_synchronisation_after_all_forward_passes(p, m, f, b, c, sigma):
    # GPipe order on a chain of p stages; a synchronisation stage on the last device, one item for all m
    # micro-batches, cost sigma, its backward item free: the forward ramp ends at (m + p - 1) f + (p - 1) c,
    # the synchronisation adds sigma, the backward ramp (m + p - 1) b + (p - 1) c.
    edges = [(s, s + 1, c) for s in range(p - 1)] + [(p - 1, p, c)]
    dur = {F: [f] * p + [sigma], B: [b] * p + [0]}
    prob = make_problem(p, p + 1, m, 0, list(range(p)) + [p - 1], edges, dur, mem_units=[1] * p + [0])
    lists = gpipe_lists(p, m)
    lists[p - 1] = lists[p - 1][:m] + [(F, 1, 0), (B, 1, 0)] + lists[p - 1][m:]
    out = oracle.evaluate_sync(prob, pack_lists(lists, 2 * m + 8)[None], group=[1] * p + [m])
    total = (m + p - 1) * (f + b) + 2 * (p - 1) * c + sigma
    assert out["flags"][0] == 0 and out["makespan"][0] == total
    assert list(out["idle"][0]) == [total - m * (f + b)] * (p - 1) + [total - m * (f + b) - sigma]
    assert list(out["peak"][0]) == [m] * p


def test_against_the_critical_path_checker_on_random_problems_groups_and_pairs():
    rng = np.random.default_rng(2024)
    n_checked = n_dead = n_over = n_grouped = n_paired = 0
    for trial in range(70):
        prob, group, pairs = random_sync_problem(rng, trial)
        lists = []
        for t in range(4):
            base = random_sync_lists(prob, group, pairs, rng, 0.25 * (t % 2), 0.25 * (t // 2))
            if base is None:
                break
            lists += [base, perturb(base, rng, 1 + t % 2)]
        if not lists:
            continue
        words = batch_from_lists(lists)
        out = oracle.evaluate_sync(prob, words, group=group, pairs=pairs)
        for i in range(len(words)):
            ref = check(prob, words[i], group, pairs)
            assert bool(out["flags"][i] & 1) == ref["deadlock"], (trial, i)
            if ref["deadlock"]:
                n_dead += 1
                continue
            assert bool(out["flags"][i] & 2) == ref["incomplete"], (trial, i)
            if ref["incomplete"]:
                continue
            assert out["makespan"][i] == ref["makespan"] and list(out["idle"][i]) == ref["idle"], (trial, i)
            assert list(out["peak"][i]) == ref["peak"], (trial, i)
            over = any(p > c for p, c in zip(ref["peak"], prob.mem_cap))
            assert bool(out["flags"][i] & 4) == over
            n_over += over
            n_checked += 1
        assert (out["flags"][::2] & 3 == 0).all()      # the unperturbed lists are valid by construction
        n_grouped += any(g > 1 for g in group)
        n_paired += bool(pairs)
    assert n_checked > 250 and n_dead > 30 and n_over > 5 and n_grouped > 30 and n_paired > 30


def test_op_times_against_the_checker_on_the_two_tower_problem_with_a_synchronisation_stage():
    # configuration-5-like shape: two towers feed a synchronisation stage that gathers every 3 micro-batches
    rng = np.random.default_rng(5)
    edges = [(0, 1, 1), (2, 3, 2), (1, 4, 1), (3, 4, 3)]
    dur = {F: [3, 3, 2, 2, 4], B: [6, 6, 4, 4, 1], W: [3, 3, 2, 2, 0], FD: [3, 3, 2, 2, 4], R: [3, 3, 2, 2, 4], O: 2, L: 2}
    prob = make_problem(4, 5, 7, 1, [0, 1, 2, 3, 3], edges, dur, mem_units=[1, 1, 1, 1, 0], mem_cap=5)
    group = [1, 1, 1, 1, 3]
    pairs = [(W, 0, W, 1, 2)]          # an extra rule: stage 1 computes a weight gradient after stage 0 has
    for t in range(20):
        lists = random_sync_lists(prob, group, pairs, rng, 0.2, 0.2)
        words = pack_lists(lists, 64)
        tr = oracle.evaluate_sync_trace(prob, words, group=group, pairs=pairs)
        ref = check(prob, words, group, pairs)
        assert tr["flags"] & 3 == 0 and tr["makespan"] == ref["makespan"]
        for (d, i), fin in ref["finish"].items():
            assert tr["finish"][d][i] == fin, (t, d, i)


def test_more_constraints_and_longer_latencies_never_shorten_a_schedule():
    rng = np.random.default_rng(9)
    prob = chain_problem(3, 6, v=2, f=2, b=3, w=2, comm=1)
    group = [1, 1, 1, 1, 1, 2]
    lists = [random_sync_lists(prob, group, [(F, 0, B, 5, 1)], rng) for _ in range(40)]
    words = batch_from_lists(lists)
    base = oracle.evaluate_sync(prob, words, group=group)
    one = oracle.evaluate_sync(prob, words, group=group, pairs=[(F, 0, B, 5, 1)])
    slow = oracle.evaluate_sync(prob, words, group=group, pairs=[(F, 0, B, 5, 40)])
    assert not (base["flags"] & 3).any() and not (one["flags"] & 3).any()
    assert (one["makespan"] >= base["makespan"]).all() and (slow["makespan"] >= one["makespan"]).all()
    assert (slow["makespan"] > base["makespan"]).any()
    assert np.array_equal(one["peak"], base["peak"])       # memory follows the order only
    # a pair whose producer always finishes first changes nothing: the forward pass of a stage before its
    # own backward pass (the state machine says so already)
    assert_same(oracle.evaluate_sync(prob, words, group=group, pairs=[(F, 2, B, 2, 0)]), base)
    # a pair against the DAG makes every candidate deadlock: forward of stage 0 after backward of stage 0
    dead = oracle.evaluate_sync(prob, words, group=group, pairs=[(B, 0, F, 0, 0)])
    assert (dead["flags"] == oracle.FLAG_DEADLOCK).all() and (dead["makespan"] == oracle.INT64_MAX).all()


def test_invalid_descriptions_are_refused():
    prob, group, lists = sync_example()
    words = pack_lists(lists, 8)[None]
    for bad_group in ([1, 1, 0], [1, -2, 2]):
        with pytest.raises(ValueError):
            oracle.evaluate_sync(prob, words, group=bad_group)
    for bad_pair in ((R, 0, F, 1, 0), (F, 0, 0, 1, 0), (F, 3, F, 1, 0), (F, 0, F, 1, -1), (F, 0, 8, 1, 0)):
        with pytest.raises(ValueError):
            oracle.evaluate_sync(prob, words, group=group, pairs=[bad_pair])
