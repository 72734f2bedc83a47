"""The tuner's grid (Section 6): rules of the enumeration (CPU) and the GPU search against the oracles."""
import numpy as np
import pytest

import oracle
from paper_2510_05112_amd import tuner
from workloads.problem import make_problem, F, B, W, FD, R


def chain(p, v, m, strategy, has_w=1, seed=0):
    S = p * v
    rng = np.random.default_rng(seed)
    f = rng.integers(8, 13, S)
    dur = {F: f, FD: f, R: f, B: rng.integers(14, 21, S)}
    if has_w:
        dur[W] = rng.integers(6, 11, S)
    edges = [(s, s + 1, int(rng.integers(1, 4))) for s in range(S - 1)]
    return make_problem(p, S, m, has_w, tuner.placement(strategy, p, S), edges, dur, mem_cap=3 * m, name=strategy)


def test_placements():
    assert tuner.placement("one-to-one", 4, 4) == [0, 1, 2, 3]
    assert tuner.placement("circular", 4, 8) == [0, 1, 2, 3, 0, 1, 2, 3]
    assert tuner.placement("v-shape", 4, 8) == [0, 1, 2, 3, 3, 2, 1, 0]
    with pytest.raises(ValueError):
        tuner.placement("one-to-one", 4, 8)
    dev, edges, copy_of = tuner.bidirectional(4)
    assert dev == [0, 1, 2, 3, 3, 2, 1, 0] and copy_of == [0, 1, 2, 3, 0, 1, 2, 3]
    assert edges == [(0, 1), (1, 2), (2, 3), (4, 5), (5, 6), (6, 7)]   # two chains, no edge between them
    dev, edges, copy_of = tuner.bidirectional(3, v_shape=True)
    assert dev == [0, 1, 2, 2, 1, 0, 2, 1, 0, 0, 1, 2] and copy_of == [0, 1, 2, 3, 4, 5] * 2
    assert len(edges) == 10 and (5, 6) not in edges and all(sorted(dev).count(d) == 4 for d in range(3))


def bidirectional_problem(p, m_per_replica, seed=0, v_shape=False):
    rng = np.random.default_rng(seed)
    dev, edges, copy_of = tuner.bidirectional(p, v_shape)
    n = len(dev) // 2
    f, b, w = rng.integers(8, 13, n), rng.integers(14, 21, n), rng.integers(6, 11, n)
    dur = {F: f[copy_of], FD: f[copy_of], R: f[copy_of], B: b[copy_of], W: w[copy_of]}
    return make_problem(p, 2 * n, m_per_replica, 1, dev, [(a, c, 2) for a, c in edges], dur,
                        mem_cap=8 * m_per_replica, name="bidirectional")


def test_bidirectional_schedules_from_the_generator_oracle_are_valid():
    prob = bidirectional_problem(4, 6)
    labels, pol, inf = tuner.grid(prob, circular=False)
    st = tuner.stride_for(prob)
    gen = oracle.generate(prob, pol, inf, st)
    assert np.all(gen["status"] == 0)
    res = oracle.evaluate(prob, gen["words"])
    assert np.all((res["flags"] & 3) == 0)
    # both replicas run at once: the best schedule beats one replica doing all 12 micro-batches alone
    work = int(prob.dur[F][:4].sum() + prob.dur[B][:4].sum() + prob.dur[W][:4].sum())
    one_after_the_other = 12 * max(int(prob.dur[F][s] + prob.dur[B][s] + prob.dur[W][s]) for s in range(4))
    assert work < res["makespan"].min() < one_after_the_other + work


def test_grid_follows_the_papers_rules():
    # Section 6: no interval unless circular; no forward-first unless asked; units 1
    flat = tuner.schedule_types(4, circular=False)
    assert len(flat) == 2 * 2 * 2 and all(t.f_interval == 0 and t.b_interval == 0 for t in flat)
    assert all(t.cttp != tuner.CTTP_FWD_FIRST for t in flat)
    circ = tuner.schedule_types(4, circular=True, forward_first=True)
    assert len(circ) == 3 * 2 * 2 * 2 * 2 and {t.f_interval for t in circ} == {0, 4}
    prob = chain(4, 2, 8, "circular")
    labels, pol, inf = tuner.grid(prob, circular=True)
    assert pol.shape == (len(labels), 4, 8) and inf.shape == (len(labels), 8) and len(set(labels)) == len(labels)
    assert np.all(pol[:, :, 1:3] == 1) and np.all(pol == pol[:, :1])      # units 1, one policy for all actors
    assert np.all(inf >= 1)


@pytest.mark.gpu
def test_gpu_search_with_sliding_and_bidirectional_placement_matches_the_oracles():
    import paper_2510_05112_amd as fp
    for prob, circular in ((chain(4, 2, 12, "circular"), True), (bidirectional_problem(4, 6), False),
                           (bidirectional_problem(3, 5, 1, v_shape=True), False)):
        st = tuner.stride_for(prob)
        h = fp.Problem(prob, st, device=0)
        best = tuner.tune(h, prob, circular, k=7, slide=True)
        labels, pol, inf = tuner.grid(prob, circular)
        words = oracle.generate(prob, pol, inf, st)["words"]
        ref, slid = oracle.evaluate(prob, words), oracle.wslide(prob, words, st)
        ms = np.concatenate([ref["makespan"], slid["makespan"]])
        fl = np.concatenate([ref["flags"], slid["flags"]])
        idx, top_ms, cnt = oracle.topk(ms, fl, 7)
        n = len(labels)
        assert cnt > 0 and [b["makespan"] for b in best] == list(top_ms[:cnt])
        assert [(b["index"], b["slid"]) for b in best] == [(int(i) % n, bool(i >= n)) for i in idx[:cnt]]
        assert all(b["label"].endswith(" +slide") == b["slid"] for b in best)
        h.close()


@pytest.mark.gpu
@pytest.mark.parametrize("strategy,p,v", [("circular", 4, 2), ("v-shape", 4, 2), ("one-to-one", 6, 1)])
def test_gpu_search_over_the_grid_matches_the_oracles(strategy, p, v):
    import paper_2510_05112_amd as fp
    prob = chain(p, v, 12, strategy)
    circular = strategy == "circular"
    st = tuner.stride_for(prob)
    h = fp.Problem(prob, st, device=0)
    best = tuner.tune(h, prob, circular, k=5)
    labels, pol, inf = tuner.grid(prob, circular)
    words = oracle.generate(prob, pol, inf, st)["words"]
    ref = oracle.evaluate(prob, words)
    idx, ms, cnt = oracle.topk(ref["makespan"], ref["flags"], 5)
    assert [b["index"] for b in best] == list(idx[:cnt]) and [b["makespan"] for b in best] == list(ms[:cnt])
    assert cnt > 0 and best[0]["label"] == labels[idx[0]]
    h.close()


@pytest.mark.gpu
@pytest.mark.parametrize("variant", ["costs per micro-batch", "link occupancy"])
def test_gpu_search_under_the_other_cost_models_matches_the_oracles(variant):
    import paper_2510_05112_amd as fp
    import workloads
    prob = chain(4, 2, 12, "circular", seed=3)
    prob.edge_comm[:] = 9   # of the order of an item's cost: a link is often busy
    st = tuner.stride_for(prob)
    h = fp.Problem(prob, st, device=0)
    kwargs = {}
    if variant == "link occupancy":
        h.set_link_occupancy(True)
        kwargs["links"] = True
    else:
        kwargs["dur_mb"] = workloads.microbatch_costs(prob)
        h.set_microbatch_costs(kwargs["dur_mb"])
    best = tuner.tune(h, prob, True, k=5)
    labels, pol, inf = tuner.grid(prob, True)
    words = oracle.generate(prob, pol, inf, st)["words"]
    ref = oracle.evaluate(prob, words, **kwargs)
    idx, ms, cnt = oracle.topk(ref["makespan"], ref["flags"], 5)
    assert cnt > 0 and [b["index"] for b in best] == list(idx[:cnt]) and [b["makespan"] for b in best] == list(ms[:cnt])
    # the model matters for the ranking's makespans
    plain = oracle.evaluate(prob, words)
    assert not np.array_equal(plain["makespan"], ref["makespan"])
    if variant == "link occupancy":
        # the sliding pass follows the link switch: both halves of the ranking against their oracles
        best = tuner.tune(h, prob, True, k=6, slide=True)
        slid = oracle.wslide(prob, words, st, links=True)
        ms = np.concatenate([ref["makespan"], slid["makespan"]])
        fl = np.concatenate([ref["flags"], slid["flags"]])
        idx, top_ms, cnt = oracle.topk(ms, fl, 6)
        n = len(labels)
        assert [(b["index"], b["slid"], b["makespan"]) for b in best] == [(int(i) % n, bool(i >= n), int(t)) for i, t in zip(idx[:cnt], top_ms[:cnt])]
        assert any(b["slid"] for b in best)
    h.close()
