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
        # the fused search with the sliding pass in the kernel finds the same entries and returns their lists
        fused = tuner.tune(h, prob, circular, k=7, slide=True, fused=True)
        assert [(b["index"], b["slid"], b["makespan"]) for b in fused] == [(b["index"], b["slid"], b["makespan"]) for b in best]
        for b in fused:
            want = slid["ops"][b["index"]] if b["slid"] else words[b["index"]]
            assert np.array_equal(b["ops"], want), b["label"]
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
    # the fused search (timed while generated, only the winners' rows written) finds the same schedules
    fused = tuner.tune(h, prob, circular, k=5, fused=True)
    assert [(b["index"], b["makespan"], b["label"]) for b in fused] == [(b["index"], b["makespan"], b["label"]) for b in best]
    assert all(np.array_equal(b["ops"], words[b["index"]]) for b in fused)
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


def shared(p, m_per_replica, seed=0):
    prob = bidirectional_problem(p, m_per_replica, seed)
    _, _, copy_of = tuner.bidirectional(p)
    cost = np.arange(5, 5 + p)
    return (prob, copy_of) + tuner.shared_stage_sync(prob, copy_of, cost)


def append_on_host(words, prob, big):
    """numpy twin of tuner.append_sync_items"""
    S, D = prob.n_stages, prob.n_devices
    dev = list(big.stage_device)
    out = np.zeros(words.shape[:2] + (words.shape[2] + 8,), np.uint16)
    out[:, :, :words.shape[2]] = words
    for d in range(D):
        on_d = [s for s in range(big.n_stages) if dev[s] == d]
        tail = [(k << 13) | (on_d.index(q) << 11) for q in on_d if q >= S for k in (1, 2, 3)]
        for c in range(len(words)):
            n = int((words[c, d] != 0).sum())
            out[c, d, n:n + len(tail)] = tail
    return out


def test_shared_stages_get_a_synchronisation_after_the_last_weight_gradient_of_every_holder():
    p, m = 4, 6
    prob, copy_of, big, group, pairs = shared(p, m)
    # one synchronisation stage per holder, on the holder's device, one item for all micro-batches
    assert big.n_stages == 4 * p and list(big.stage_device[2 * p:]) == [0, 3, 1, 2, 2, 1, 3, 0]
    assert list(group) == [1] * (2 * p) + [m] * (2 * p) and len(pairs) == 4 * p
    assert all(k1 == W and k2 == F and lat == 0 for k1, _, k2, _, lat in pairs)
    assert {(int(a), int(q)) for _, a, _, q, _ in pairs if q == 2 * p} == {(0, 2 * p), (p, 2 * p)}
    assert list(big.dur[F][2 * p:]) == [5, 5, 6, 6, 7, 7, 8, 8] and not big.dur[B][2 * p:].any() and not big.mem_units[2 * p:].any()
    # the timing: schedules of the two-chain problem keep their times, every synchronisation starts when its
    # device is free and the last weight gradient of both holders of its model stage is computed
    labels, pol, inf = tuner.grid(prob, circular=False)
    st = tuner.stride_for(prob)
    words = oracle.generate(prob, pol, inf, st)["words"]
    full = append_on_host(words, prob, big)
    res = oracle.evaluate_sync(big, full, group, pairs)
    assert not (res["flags"] & 3).any()
    for c in (0, 3, len(words) - 1):
        plain = oracle.evaluate_trace(prob, words[c])
        tr = oracle.evaluate_sync_trace(big, full[c], group, pairs)
        k, ch, j = oracle.decode(words[c])
        dev = list(prob.stage_device)
        stages_of = [[s for s in range(prob.n_stages) if dev[s] == d] for d in range(p)]
        last_w = {}
        for d in range(p):
            for i in range(st):
                if k[d, i] == W:
                    s = stages_of[d][ch[d, i]]
                    last_w[copy_of[s]] = max(last_w.get(copy_of[s], 0), int(plain["finish"][d, i]))
        expect = 0
        for d in range(p):
            n = int((words[c, d] != 0).sum())
            assert np.array_equal(tr["finish"][d, :n], plain["finish"][d, :n])
            t = int(plain["finish"][d, :n].max())
            for model_stage in sorted([d, p - 1 - d]):  # its two synchronisation stages, in stage order
                t = max(t, last_w[model_stage]) + 5 + model_stage
            expect = max(expect, t)
        assert tr["makespan"] == expect > plain["makespan"]
    # without the synchronisation items in the lists the model is incomplete, not silently two models
    short = np.zeros_like(full)
    short[:, :, :st] = words
    assert (oracle.evaluate_sync(big, short, group, pairs)["flags"] == oracle.FLAG_INCOMPLETE).all()


@pytest.mark.gpu
def test_gpu_search_with_shared_stages_matches_the_oracles():
    import paper_2510_05112_amd as fp
    import torch
    for p, m in ((4, 6), (3, 5)):
        prob, copy_of, big, group, pairs = shared(p, m, seed=p)
        st = tuner.stride_for(prob)
        gen = fp.Problem(prob, st, device=0)
        ev = fp.Problem(big, st + 8, device=0)
        ev.set_sync(group, pairs)
        best = tuner.tune_shared(gen, ev, prob, big, k=6)
        labels, pol, inf = tuner.grid(prob, circular=False)
        words = oracle.generate(prob, pol, inf, st)["words"]
        ref = oracle.evaluate_sync(big, append_on_host(words, prob, big), group, pairs)
        idx, ms, cnt = oracle.topk(ref["makespan"], ref["flags"], 6)
        assert cnt > 0 and [(b["index"], b["makespan"]) for b in best] == [(int(i), int(t)) for i, t in zip(idx[:cnt], ms[:cnt])]
        # the appended lists on the GPU are the host's
        out = gen.generate(torch.from_numpy(pol).cuda(), torch.from_numpy(inf).cuda(), st)
        ops = tuner.append_sync_items(out["ops"], prob, big)
        torch.cuda.synchronize()
        assert np.array_equal(ops.cpu().numpy().view(np.uint16), append_on_host(words, prob, big))
        gen.close()
        ev.close()
