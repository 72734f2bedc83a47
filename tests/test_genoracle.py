"""Pins of the schedule-generator oracle (CPU only).

The oracle restates the paper's scheduler (Section 5: instruction pool, reorder queues, step function
of Algorithm 1, Steps 1-5) item by item.  It is pinned by: the two schedules whose order is known in
closed form (1F1B and GPipe, and their 2(m + p - 1) unit steps), an independent counter-based model on
random policies, properties every generated schedule must have, and hand-worked small cases.
"""
import numpy as np
import pytest

import oracle
from gen_checker import simulate
from helpers import two_tower_problem
from workloads.problem import chain_problem, gpipe_lists, interleaved_1f1b_lists, one_f_one_b_lists, pack_lists

NO_LIMIT = 2**31 - 1


def uniform_policy(n, D, cttp, u1=1, u2=1, fdir=0, fint=0, bdir=0, bint=0):
    pol = np.zeros((n, D, 8), np.int32)
    pol[..., 0], pol[..., 1], pol[..., 2] = cttp, u1, u2
    pol[..., 3], pol[..., 4], pol[..., 5], pol[..., 6] = fdir, fint, bdir, bint
    return pol


def stride_for(problem):
    per_dev = np.bincount(problem.stage_device, minlength=problem.n_devices).max()
    n = per_dev * problem.n_microbatches * (3 if problem.has_w else 2)
    return int(-(-(n + 1) // 8) * 8)


@pytest.mark.parametrize("p,m", [(2, 1), (2, 5), (4, 8), (4, 3), (8, 16), (5, 7)])
def test_bwd_first_with_inflight_p_minus_d_is_1f1b_and_fwd_first_is_gpipe(p, m):
    # Section 2.1 / Table of built-in priorities: 1F1B = backward passes first, at most p - d
    # micro-batches in flight on stage d; GPipe = forward passes first, no limit.
    prob = chain_problem(p, m, f=1, b=1, comm=0)
    st = stride_for(prob)
    pol = np.concatenate([uniform_policy(1, p, oracle.CTTP_BWD_FIRST), uniform_policy(1, p, oracle.CTTP_FWD_FIRST)])
    inf = np.full((2, p), NO_LIMIT, np.int32)
    inf[0] = [p - d for d in range(p)]
    out = oracle.generate(prob, pol, inf, st, diagnostics=True)
    assert np.array_equal(out["words"][0], pack_lists(one_f_one_b_lists(p, m), st))
    assert np.array_equal(out["words"][1], pack_lists(gpipe_lists(p, m), st))
    # unit steps = unit-time makespan of both schedules
    assert list(out["steps"]) == [2 * (m + p - 1)] * 2
    assert not out["status"].any() and not out["prefix_violations"].any()
    ev = oracle.evaluate(prob, out["words"])
    assert list(ev["makespan"]) == [2 * (m + p - 1)] * 2 and not ev["flags"].any()


@pytest.mark.parametrize("p,v,m", [(4, 2, 8), (4, 2, 16), (2, 2, 4), (4, 4, 8), (8, 2, 16), (3, 2, 6), (4, 3, 12)])
def test_the_papers_interleaved_setting_reaches_the_interleaved_1f1b_length(p, v, m):
    # The setting the paper gives for its circular-placement example (caption of the figure of the
    # automated scheduling process, Section 5): cttp = interleaved, forward stage traversal
    # (breadth-first, p), backward stage traversal (depth-first, p).  With unit forward and backward
    # times per chunk, interleaved 1F1B over p devices x v chunks (Section 2.1) has the closed-form
    # length 2 v m + 2 (p - 1): all the work of one device plus the (p - 1)-step ramps of one chunk.
    prob = chain_problem(p, m, v=v, f=1, b=1, comm=0)
    st = stride_for(prob)
    pol = uniform_policy(1, p, oracle.CTTP_INTERLEAVED, fdir=0, fint=p, bdir=1, bint=p)
    out = oracle.generate(prob, pol, np.full((1, p * v), NO_LIMIT, np.int32), st)
    assert out["status"][0] == 0 and out["steps"][0] == 2 * v * m + 2 * (p - 1)
    ev = oracle.evaluate(prob, out["words"])
    assert ev["flags"][0] == 0 and ev["makespan"][0] == 2 * v * m + 2 * (p - 1)
    # and it holds fewer activations than running all forward passes first
    gp = oracle.generate(prob, uniform_policy(1, p, oracle.CTTP_FWD_FIRST), np.full((1, p * v), NO_LIMIT, np.int32), st)
    assert ev["peak"][0].max() < oracle.evaluate(prob, gp["words"])["peak"][0].max()


PAPER_INTERLEAVED = dict(cttp=oracle.CTTP_INTERLEAVED, fdir=0, bdir=1)   # intervals = p, set per shape


@pytest.mark.parametrize("p", [2, 3, 4, 5, 6, 8])
@pytest.mark.parametrize("v", [2, 3, 4])
def test_the_papers_interleaved_setting_reproduces_the_published_interleaved_1f1b_order(p, v):
    # An external pin of the interval traversal (Section 5.2, "Stage Traversal Priority") and of the
    # interleaved type priority: on the circular placement the setting of the paper's example --
    # interleaved, forward (breadth-first, p), backward (depth-first, p) -- must give interleaved 1F1B
    # (Section 2.1), whose order is written out from its published definition in
    # workloads.problem.interleaved_1f1b_lists (and is itself pinned below).  One round of p
    # micro-batches: item by item the same op words on every device.
    m = p
    prob = chain_problem(p, m, v=v, f=1, b=1, comm=0)
    st = stride_for(prob)
    pol = uniform_policy(1, p, fint=p, bint=p, **PAPER_INTERLEAVED)
    out = oracle.generate(prob, pol, np.full((1, p * v), NO_LIMIT, np.int32), st)
    assert np.array_equal(out["words"][0], pack_lists(interleaved_1f1b_lists(p, v, m), st))
    assert out["steps"][0] == 2 * v * m + 2 * (p - 1) and out["status"][0] == 0


@pytest.mark.parametrize("p,v,m", [(4, 2, 4), (4, 2, 8), (4, 2, 16), (3, 2, 9), (8, 2, 16), (4, 4, 8), (5, 3, 10)])
def test_the_published_interleaved_order_and_where_the_scheduler_leaves_it(p, v, m):
    # The published order, timed by the evaluation oracle with unit costs, has the closed-form length
    # 2 v m + 2 (p - 1) and holds at most its warm-up depth in activations (this pins the order builder).
    prob = chain_problem(p, m, v=v, f=1, b=1, comm=0)
    st = stride_for(prob)
    lists = interleaved_1f1b_lists(p, v, m)
    ev = oracle.evaluate(prob, pack_lists(lists, st)[None])
    assert ev["flags"][0] == 0 and ev["makespan"][0] == 2 * v * m + 2 * (p - 1)
    assert list(ev["peak"][0]) == [min(2 * (p - d - 1) + (v - 1) * p + 1, m * v) for d in range(p)]
    # With more than one round of micro-batches the fixed order lets a device wait for a forward item
    # of its next chunk where the paper's scheduler, which idles only when nothing at all can be
    # scheduled (Section 5.2, Step 2), takes another item: the orders then differ, the lengths do not.
    pol = uniform_policy(1, p, fint=p, bint=p, **PAPER_INTERLEAVED)
    out = oracle.generate(prob, pol, np.full((1, p * v), NO_LIMIT, np.int32), st)
    assert out["steps"][0] == ev["makespan"][0]
    assert np.array_equal(out["words"][0], pack_lists(lists, st)) == (m == p)


def test_what_the_other_readings_of_the_interval_rule_lead_to():
    # Algorithm 1 as printed moves the position only when `interval` items were scheduled and returns
    # whatever the fetch at the position gives; read a little more kindly, a position whose stage has
    # nothing to offer lets the next type try.  Both readings (modelled in gen_checker.simulate) keep an
    # actor on a stage that cannot move, so a valid problem stops dead:
    prob = chain_problem(2, 2, v=2, f=1, b=1, comm=0)
    none = [NO_LIMIT] * 4
    # (a) a setting of the tuner's own grid (Section 6): forward traversal (depth-first, interval) on the
    # circular placement.  The position starts on the actor's last stage, whose forward items wait for
    # the first stage's: no item is ever scheduled.
    pol = uniform_policy(1, 2, oracle.CTTP_BWD_FIRST, fdir=1, fint=2)[0].tolist()
    for reading in ("strict", "literal"):
        lists, steps, stuck = simulate(prob, pol, none, reading)
        assert stuck and steps == 0 and not any(lists)
    lists, steps, stuck = simulate(prob, pol, none)
    assert not stuck and sum(len(x) for x in lists) == 2 * 4 * 2
    out = oracle.generate(prob, uniform_policy(1, 2, oracle.CTTP_BWD_FIRST, fdir=1, fint=2),
                          np.full((1, 4), NO_LIMIT, np.int32), 16)
    assert out["status"][0] == 0 and np.array_equal(out["words"][0], pack_lists(lists, 16))
    # (b) an interval of two with one micro-batch in flight on the first stage (the case of the next
    # test): after F(0, 0) the position waits on stage 0 for a second item that the limit forbids until
    # the first has come back, which needs the actor's other stage.
    prob = chain_problem(2, 4, v=2, f=1, b=1, comm=0)
    pol = uniform_policy(1, 2, oracle.CTTP_BWD_FIRST, fdir=0, fint=2)[0].tolist()
    for reading in ("strict", "literal"):
        lists, steps, stuck = simulate(prob, pol, [1, NO_LIMIT, NO_LIMIT, NO_LIMIT], reading)
        assert stuck and steps == 2 and [len(x) for x in lists] == [1, 1]
    # (c) on random interval policies without any limit more than half of the processes get stuck
    rng = np.random.default_rng(3)
    pol, inf = random_policies(rng, 60, prob, rng.random(60) < 0.5)
    with_interval = [i for i in range(60) if pol[i][:, 4].any() or pol[i][:, 6].any()]
    stuck = {r: sum(simulate(prob, pol[i].tolist(), [NO_LIMIT] * 4, r)[2] for i in with_interval)
             for r in ("no-idle", "strict", "literal")}
    assert stuck["no-idle"] == 0 and stuck["strict"] > len(with_interval) // 3 and stuck["literal"] >= stuck["strict"]
    # (d) where the paper's example setting is concerned the three readings cannot be told apart: one
    # round of micro-batches gives the published order under each of them
    prob = chain_problem(4, 4, v=2, f=1, b=1, comm=0)
    pol = uniform_policy(1, 4, fint=4, bint=4, **PAPER_INTERLEAVED)[0].tolist()
    for reading in ("no-idle", "strict", "literal"):
        lists, steps, stuck = simulate(prob, pol, [NO_LIMIT] * 8, reading)
        assert not stuck and lists == interleaved_1f1b_lists(4, 2, 4)


def random_policies(rng, n, problem, per_actor):
    D, S, m = problem.n_devices, problem.n_stages, problem.n_microbatches
    pol = np.zeros((n, D, 8), np.int32)
    for i in range(n):
        rows = D if per_actor[i] else 1
        r = np.zeros((rows, 8), np.int32)
        r[:, 0] = rng.integers(0, 3, rows)
        inter = r[:, 0] == 2
        r[:, 1] = np.where(inter, rng.integers(1, 4, rows), 1)
        r[:, 2] = np.where(inter, rng.integers(1, 4, rows), 1)
        r[:, 3] = rng.integers(0, 2, rows)
        r[:, 4] = np.where(rng.random(rows) < 0.5, rng.integers(1, 6, rows), 0)
        r[:, 5] = rng.integers(0, 2, rows)
        r[:, 6] = np.where(rng.random(rows) < 0.5, rng.integers(1, 6, rows), 0)
        pol[i] = r
    inf = np.where(rng.random((n, S)) < 0.3, NO_LIMIT, rng.integers(1, max(2, m), (n, S))).astype(np.int32)
    return pol, inf


PROBLEMS = {
    "chain_v1": lambda: chain_problem(4, 6, f=1, b=1, comm=0),
    "chain_v2_w": lambda: chain_problem(3, 7, v=2, f=1, b=1, w=1, comm=0),
    "chain_v4": lambda: chain_problem(2, 5, v=4, f=1, b=1, comm=0),
    "two_tower_w": lambda: two_tower_problem(m=5, has_w=1),
    "two_tower": lambda: two_tower_problem(m=4, has_w=0),
}


@pytest.mark.parametrize("name", sorted(PROBLEMS))
def test_oracle_equals_the_counter_model_on_random_policies(name):
    prob = PROBLEMS[name]()
    rng = np.random.default_rng(11)
    n = 60
    pol, inf = random_policies(rng, n, prob, rng.random(n) < 0.5)
    st = stride_for(prob)
    out = oracle.generate(prob, pol, inf, st, diagnostics=True)
    assert not out["prefix_violations"].any()
    n_stuck = 0
    for i in range(n):
        lists, steps, stuck = simulate(prob, pol[i].tolist(), inf[i].tolist())
        assert np.array_equal(out["words"][i], pack_lists(lists, st)), (name, i)
        assert out["steps"][i] == steps and bool(out["status"][i] & 1) == stuck, (name, i)
        n_stuck += stuck
    assert n_stuck == 0    # limits >= 1: the oldest unfinished micro-batch can always move


@pytest.mark.parametrize("name", sorted(PROBLEMS))
def test_generated_schedules_are_valid_and_respect_the_limits(name):
    prob = PROBLEMS[name]()
    rng = np.random.default_rng(5)
    n = 80
    pol, inf = random_policies(rng, n, prob, rng.random(n) < 0.5)
    st = stride_for(prob)
    out = oracle.generate(prob, pol, inf, st)
    ev = oracle.evaluate(prob, out["words"])
    kind, chunk, mb = oracle.decode(out["words"])
    stages = [[s for s in range(prob.n_stages) if prob.stage_device[s] == d] for d in range(prob.n_devices)]
    ntypes = 3 if prob.has_w else 2
    for i in range(n):
        complete = out["status"][i] == 0
        # a finished process has scheduled every item once, and the evaluator accepts the schedule
        assert (ev["flags"][i] & 3 == 0) == complete, (name, i, ev["flags"][i])
        n_ops = int((kind[i] != 0).sum())
        assert (n_ops == ntypes * prob.n_stages * prob.n_microbatches) == complete
        # no schedule can take fewer steps than the longest list, nor more than one item per step
        assert out["steps"][i] >= (kind[i] != 0).sum(1).max() and out["steps"][i] <= max(n_ops, 1)
        for d in range(prob.n_devices):
            seen = {}
            live = {s: 0 for s in stages[d]}
            for k, c, j in zip(kind[i, d], chunk[i, d], mb[i, d]):
                if k == 0:
                    break
                s = stages[d][c]
                assert seen.get((k, s), 0) == j      # ascending micro-batches, each once
                seen[(k, s)] = j + 1
                if k == 1:
                    live[s] += 1
                    assert live[s] <= inf[i, s]       # the in-flight rule on every prefix
                if k == 2:
                    live[s] -= 1


def unit_time(problem):
    """The same problem with every duration 1 and no latency: the scheduler's own clock."""
    S = problem.n_stages
    dur = {1: 1, 2: 1, 3: 1, 4: 1, 5: 1, 6: 1, 7: 1}
    edges = [(int(a), int(b), 0) for a, b in zip(problem.edge_src, problem.edge_dst)]
    from workloads.problem import make_problem
    return make_problem(problem.n_devices, S, problem.n_microbatches, problem.has_w,
                        problem.stage_device, edges, dur)


@pytest.mark.parametrize("name", sorted(PROBLEMS))
def test_steps_equal_the_unit_time_makespan_of_the_generated_order(name):
    # Two oracles, one fact.  The scheduler is work-conserving: an actor with an eligible item never
    # idles.  An item is eligible as soon as its dependencies are scheduled (a forward pass held back by
    # the in-flight rule waits for a backward pass of its own actor, which precedes it in that actor's
    # list), so the step in which the scheduler placed an item is the earliest start the evaluator
    # finds for the same per-actor order with unit durations and no latency: steps == makespan.
    prob = PROBLEMS[name]()
    unit = unit_time(prob)
    rng = np.random.default_rng(21)
    n = 60
    pol, inf = random_policies(rng, n, prob, rng.random(n) < 0.5)
    st = stride_for(prob)
    free = oracle.generate(prob, pol, np.full_like(inf, NO_LIMIT), st)
    ev = oracle.evaluate(unit, free["words"])
    assert not ev["flags"].any() and np.array_equal(ev["makespan"], free["steps"])
    tight = oracle.generate(prob, pol, inf, st)
    ev = oracle.evaluate(unit, tight["words"])
    assert not ev["flags"].any() and np.array_equal(ev["makespan"], tight["steps"])
    assert np.any(tight["steps"] > free["steps"])     # the limits do stretch some schedules


def test_hand_worked_interval_traversal():
    # Section 5.2 "Stage Traversal Priority", worked by hand: 2 actors, circular placement of 4 stages
    # (actor 0: stages 0 and 2; actor 1: stages 1 and 3), 2 micro-batches, forward passes first,
    # forward traversal breadth-first with interval 2, backward traversal depth-first, no interval.
    # Fsj / Bsj = stage s, micro-batch j; an item scheduled in step t resolves its successors for t+1.
    #  step:   1    2    3    4    5    6    7    8    9    10
    #  a0:     F00  F01  F20  F21  .    .    B20  B21  B00  B01
    #  a1:     .    F10  F11  F30  F31  B30  B31  B10  B11  .
    # step 3, a0: `stepped` = 2 = interval, so the position moves from stage 0 to stage 2 (F20 was
    # resolved by F10 in step 2); step 4, a1: same move from stage 1 to stage 3 (F30 resolved by F20);
    # steps 5-6, a0: no forward item left and B20 waits for B30 (step 6): two bubbles; step 8, a1:
    # depth-first looks at stage 3 first (exhausted), then stage 1: B10 (resolved by B20 in step 7).
    prob = chain_problem(2, 2, v=2, f=1, b=1, comm=0)
    pol = uniform_policy(1, 2, oracle.CTTP_FWD_FIRST, fdir=0, fint=2, bdir=1, bint=0)
    inf = np.full((1, 4), NO_LIMIT, np.int32)
    out = oracle.generate(prob, pol, inf, 16)
    k, c, j = oracle.decode(out["words"][0])
    seq = [[(int(a), int(b), int(x)) for a, b, x in zip(k[d], c[d], j[d]) if a] for d in range(2)]
    assert seq[0] == [(1, 0, 0), (1, 0, 1), (1, 1, 0), (1, 1, 1), (2, 1, 0), (2, 1, 1), (2, 0, 0), (2, 0, 1)]
    assert seq[1] == [(1, 0, 0), (1, 0, 1), (1, 1, 0), (1, 1, 1), (2, 1, 0), (2, 1, 1), (2, 0, 0), (2, 0, 1)]
    assert out["steps"][0] == 10 and out["status"][0] == 0


def test_an_interval_never_holds_an_actor_on_a_blocked_stage():
    # actor 0 holds stages 0 and 2; with interval 2 it would stay on stage 0 for two forward passes,
    # but the limit of one in-flight micro-batch forbids the second: the traversal moves on to stage 2
    # (Section 5.2, Step 2: an actor idles only when none of its items can be scheduled), and the
    # process completes.  With limits >= 1 nothing ever gets stuck (reading G8).
    prob = chain_problem(2, 4, v=2, f=1, b=1, comm=0)
    pol = uniform_policy(1, 2, oracle.CTTP_BWD_FIRST, fdir=0, fint=2)
    inf = np.full((1, 4), NO_LIMIT, np.int32)
    inf[0, 0] = 1
    out = oracle.generate(prob, pol, inf, 24)
    assert out["status"][0] == 0
    k, c, j = oracle.decode(out["words"][0])
    assert (k != 0).sum() == 2 * 4 * 4
    assert [(int(a), int(b), int(x)) for a, b, x in zip(k[0][:3], c[0][:3], j[0][:3])] == [(1, 0, 0), (1, 1, 0), (2, 1, 0)]


def test_interleaved_units_alternate_runs_of_forward_and_backward():
    # one actor, one stage: interleaved(2, 1) must give F F B F F B ... as far as dependencies allow
    prob = chain_problem(1, 6, f=1, b=1, comm=0)
    pol = uniform_policy(1, 1, oracle.CTTP_INTERLEAVED, u1=2, u2=1)
    out = oracle.generate(prob, pol, np.full((1, 1), NO_LIMIT, np.int32), 16)
    k, _, j = oracle.decode(out["words"][0])
    assert [int(x) for x in k[0][:12]] == [1, 1, 2, 1, 1, 2, 1, 1, 2, 2, 2, 2]
    assert out["steps"][0] == 12


def test_invalid_policies_are_rejected():
    prob = chain_problem(2, 2)
    inf = np.full((1, 2), NO_LIMIT, np.int32)
    for bad in (uniform_policy(1, 2, 3), uniform_policy(1, 2, 0, u1=2), uniform_policy(1, 2, 2, u1=0),
                uniform_policy(1, 2, 0, fdir=2)):
        with pytest.raises(ValueError):
            oracle.generate(prob, bad, inf, 8)
    with pytest.raises(ValueError):
        oracle.generate(prob, uniform_policy(1, 2, 0), np.zeros((1, 2), np.int32), 8)
