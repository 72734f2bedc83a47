"""GPU parity of the fused search step: fpsched_generate_evaluate must give, for every parameter set, what
the evaluation oracle gives for the schedule the generator oracle writes for that set (two oracles, each
pinned on its own, composed on the CPU), bit for bit; fpsched_generate_selected must give the rows of the
sets it is asked for."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_05112_amd as fp
import workloads
from helpers import dag_problem, two_tower_problem
from test_genoracle import random_policies, stride_for, uniform_policy

pytestmark = pytest.mark.gpu


def reference(problem, pol, inf, threads=8):
    st = stride_for(problem)
    gen = oracle.generate(problem, pol, inf, st, threads=threads)
    ev = oracle.evaluate(problem, gen["words"], threads=threads)
    return gen, ev


def fused(problem, pol, inf):
    h = fp.Problem(problem, stride_for(problem), device=0)
    res, out = h.generate_evaluate(torch.from_numpy(np.ascontiguousarray(pol, np.int32)).cuda(),
                                   torch.from_numpy(np.ascontiguousarray(inf, np.int32)).cuda())
    torch.cuda.synchronize()
    got = {k: v.cpu().numpy() for k, v in res.items()}
    got.update(steps=out["steps"].cpu().numpy(), status=out["status"].cpu().numpy())
    h.close()
    return got


def check(problem, pol, inf, what):
    gen, ev = reference(problem, pol, inf)
    got = fused(problem, pol, inf)
    for name, ref in (("status", gen["status"]), ("steps", gen["steps"]), ("flags", ev["flags"]),
                      ("makespan", ev["makespan"]), ("idle", ev["idle"]), ("peak", ev["peak"])):
        if not np.array_equal(got[name], ref):
            bad = np.flatnonzero((got[name] != ref).reshape(len(pol), -1).any(1))
            raise AssertionError(f"{what}: {name} differs for {len(bad)} sets, first {bad[:5]}: "
                                 f"{got[name][bad[0]]} vs {ref[bad[0]]}")
    return got, ev


def placed_chain(p, v, m, has_w, seed, circular=True, tight_caps=False):
    """A chain of p v stages with seeded unequal costs and latencies, laid over p devices round after round
    (circular) or down and up again (V-shape, v = 2)."""
    S = p * v
    dev = [s % p for s in range(S)] if circular else [s if s < p else 2 * p - 1 - s for s in range(S)]
    prob = dag_problem([(s, s + 1) for s in range(S - 1)], S, dev, p, m=m, has_w=has_w, seed=seed)
    if tight_caps:
        prob.mem_cap[:] = np.maximum(1, (prob.mem_units.max() * m * v) // 3)
    return prob


@pytest.mark.parametrize("p,v,m,has_w,circular", [(4, 1, 6, 0, True), (3, 2, 7, 1, True), (2, 4, 5, 0, True),
                                                  (5, 2, 9, 1, False), (7, 3, 4, 1, True), (33, 1, 3, 0, True),
                                                  (64, 1, 2, 1, True), (16, 4, 3, 1, True)])
def test_chains_with_unequal_costs(p, v, m, has_w, circular):
    prob = placed_chain(p, v, m, has_w, seed=p * 10 + v, circular=circular, tight_caps=(p % 2 == 1))
    rng = np.random.default_rng(p + m)
    n = 150   # not a multiple of the sets per wavefront
    pol, inf = random_policies(rng, n, prob, rng.random(n) < 0.5)
    got, ev = check(prob, pol, inf, f"p{p} v{v} m{m} w{has_w}")
    if p % 2 == 1:
        assert (ev["flags"] & 4).any()   # some schedules exceed the tightened caps


@pytest.mark.parametrize("has_w", [0, 1])
def test_two_towers_and_a_fork_join_dag(has_w):
    prob = two_tower_problem(m=5, has_w=has_w, comm=2)
    rng = np.random.default_rng(17 + has_w)
    pol, inf = random_policies(rng, 200, prob, rng.random(200) < 0.5)
    check(prob, pol, inf, "two towers")
    edges = [(0, 2), (1, 2), (2, 3), (2, 4), (3, 5), (4, 5)]   # two sources, a fork and a join
    prob = dag_problem(edges, 6, [0, 1, 2, 0, 1, 2], 3, m=6, has_w=has_w, seed=5)
    pol, inf = random_policies(rng, 200, prob, rng.random(200) < 0.5)
    check(prob, pol, inf, "fork and join")


@pytest.mark.parametrize("index,n", [(1, 64), (2, 256), (3, 96), (4, 96), (5, 128)])
def test_benchmark_problems(index, n):
    prob = workloads.config(index, 8).problem
    pol, inf = workloads.policy_sets(prob, n)
    got, ev = check(prob, pol, inf, f"cfg{index}")
    assert (ev["flags"] == 0).any()


def test_bad_policies_empty_batch_and_refusals():
    prob = placed_chain(4, 2, 4, 1, seed=2)
    pol = uniform_policy(6, 4, 0)
    inf = np.full((6, 8), 3, np.int32)
    pol[1, 2, 0] = 7            # unknown computation type priority
    pol[3, 3, 4] = -1           # negative interval
    inf[4, 5] = 0               # limit below 1
    got = fused(prob, pol, inf)   # (the generator oracle refuses bad sets: the good ones are compared)
    good = [0, 2, 5]
    gen, ev = reference(prob, pol[good], inf[good])
    for name in ("makespan", "idle", "peak", "flags"):
        assert np.array_equal(got[name][good], ev[name])
    assert np.array_equal(got["steps"][good], gen["steps"]) and not got["steps"][[1, 3, 4]].any()
    assert list(got["status"]) == [0, 4, 0, 4, 4, 0]
    assert list(got["flags"]) == [0, 2, 0, 2, 2, 0] and got["makespan"][1] == np.iinfo(np.int64).max
    assert (got["idle"][1] == -1).all() and (got["peak"][1] == -1).all()
    h = fp.Problem(prob, stride_for(prob), device=0)
    res, out = h.generate_evaluate(torch.empty((0, 4, 8), dtype=torch.int32, device="cuda"),
                                   torch.empty((0, 8), dtype=torch.int32, device="cuda"))
    assert res["makespan"].numel() == 0
    one = (torch.from_numpy(pol[:1]).cuda(), torch.from_numpy(inf[:1]).cuda())
    h.set_link_occupancy(True)
    with pytest.raises(fp.FpschedError) as e:   # the fused form knows the plain cost model only
        h.generate_evaluate(*one)
    assert e.value.code == -6
    h.set_link_occupancy(False)
    h.generate_evaluate(*one)
    torch.cuda.synchronize()
    h.close()
    # a stage with three inputs: no fused form (the generator itself walks edge lists there)
    wide = dag_problem([(0, 3), (1, 3), (2, 3)], 4, [0, 1, 2, 3], 4, m=3, has_w=0, seed=1)
    h = fp.Problem(wide, stride_for(wide), device=0)
    with pytest.raises(fp.FpschedError) as e:
        h.generate_evaluate(torch.from_numpy(uniform_policy(1, 4, 0)).cuda(),
                            torch.full((1, 4), 9, dtype=torch.int32, device="cuda"))
    assert e.value.code == -6
    h.close()


def test_search_step_and_the_winners_rows():
    # fused search: time while generating, top-k, then only the winners' schedules are written
    spec = workloads.config(4, 8)
    prob = spec.problem
    n, k = 300, 16
    pol, inf = workloads.policy_sets(prob, n)
    st = workloads.generator_stride(prob)
    h = fp.Problem(prob, st, device=0)
    d_pol, d_inf = torch.from_numpy(pol).cuda(), torch.from_numpy(inf).cuda()
    res, _ = h.generate_evaluate(d_pol, d_inf)
    top = h.topk(res, k)
    rows = h.generate_selected(d_pol, d_inf, top["idx"], st)
    torch.cuda.synchronize()
    ref_gen = oracle.generate(prob, pol, inf, st, threads=8)
    ref = oracle.evaluate(prob, ref_gen["words"], threads=8)
    idx, ms, cnt = oracle.topk(ref["makespan"], ref["flags"], k)
    assert int(top["count"].item()) == cnt == k
    assert np.array_equal(top["idx"].cpu().numpy(), idx) and np.array_equal(top["makespan"].cpu().numpy(), ms)
    assert np.array_equal(rows["ops"].cpu().numpy().view(np.uint16), ref_gen["words"][idx])
    assert np.array_equal(rows["steps"].cpu().numpy(), ref_gen["steps"][idx])
    # unused top-k slots (-1) select nothing
    # ... and so do indices beyond the sets that are there
    sel = torch.tensor([5, -1, 0, 299, 300, 2 ** 40], dtype=torch.int64, device="cuda")
    rows = h.generate_selected(d_pol, d_inf, sel, st)
    torch.cuda.synchronize()
    words = rows["ops"].cpu().numpy().view(np.uint16)
    assert np.array_equal(words[[0, 2, 3]], ref_gen["words"][[5, 0, 299]]) and not words[[1, 4, 5]].any()
    assert list(rows["status"].cpu().numpy()) == [0, 4, 0, 0, 4, 4]
    h.close()
