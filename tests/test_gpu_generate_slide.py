"""GPU parity of fpsched_generate_slide_evaluate: for every parameter set, what the sliding oracle reports for the
schedule the generator oracle writes for that set (composed on the CPU), bit for bit."""
import copy

import numpy as np
import pytest
import torch

import oracle
import paper_2510_05112_amd as fp
import workloads
from helpers import dag_problem, two_tower_problem
from test_genoracle import random_policies, stride_for
from test_gpu_generate_evaluate import placed_chain

pytestmark = pytest.mark.gpu


def check_slide(problem, pol, inf, what):
    st = stride_for(problem)
    gen = oracle.generate(problem, pol, inf, st, threads=8)
    ref = oracle.wslide(problem, gen["words"], st, threads=8)
    h = fp.Problem(problem, st, device=0)
    d_pol = torch.from_numpy(np.ascontiguousarray(pol, np.int32)).cuda()
    d_inf = torch.from_numpy(np.ascontiguousarray(inf, np.int32)).cuda()
    res, out = h.generate_evaluate(d_pol, d_inf, slide=True)
    torch.cuda.synchronize()
    got = {k: v.cpu().numpy() for k, v in res.items()}
    got.update(steps=out["steps"].cpu().numpy(), status=out["status"].cpu().numpy())
    for name, want in (("status", gen["status"]), ("steps", gen["steps"]), ("flags", ref["flags"]),
                       ("makespan", ref["makespan"]), ("idle", ref["idle"]), ("peak", ref["peak"])):
        if not np.array_equal(got[name], want):
            bad = np.flatnonzero((got[name] != want).reshape(len(pol), -1).any(1))
            raise AssertionError(f"{what}: {name} differs for {len(bad)} sets, first {bad[:5]}: "
                                 f"{got[name][bad[0]]} vs {want[bad[0]]}")
    # and what the library's own two steps give: generate, then the sliding pass without lists
    rows = h.generate(d_pol, d_inf, st)
    two = h.wslide_evaluate(rows["ops"])
    torch.cuda.synchronize()
    for name in ("makespan", "idle", "peak", "flags"):
        assert np.array_equal(two[name].cpu().numpy(), got[name]), (what, name)
    h.close()
    return got, ref


@pytest.mark.parametrize("p,v,m,circular", [(3, 2, 7, True), (5, 2, 9, False), (7, 3, 4, True), (64, 1, 2, True),
                                            (16, 4, 3, True), (4, 1, 11, True)])
def test_chains_with_unequal_costs(p, v, m, circular):
    prob = placed_chain(p, v, m, 1, seed=p * 10 + v, circular=circular, tight_caps=(p % 2 == 1))
    rng = np.random.default_rng(p + m)
    n = 150
    pol, inf = random_policies(rng, n, prob, rng.random(n) < 0.5)
    got, ref = check_slide(prob, pol, inf, f"p{p} v{v} m{m}")
    assert (ref["flags"] == 0).any()


def test_two_towers_and_a_fork_join_dag():
    prob = two_tower_problem(m=5, has_w=1, comm=2)
    rng = np.random.default_rng(18)
    pol, inf = random_policies(rng, 200, prob, rng.random(200) < 0.5)
    check_slide(prob, pol, inf, "two towers")
    edges = [(0, 2), (1, 2), (2, 3), (2, 4), (3, 5), (4, 5)]
    prob = dag_problem(edges, 6, [0, 1, 2, 0, 1, 2], 3, m=6, has_w=1, seed=5)
    pol, inf = random_policies(rng, 200, prob, rng.random(200) < 0.5)
    check_slide(prob, pol, inf, "fork and join")


@pytest.mark.parametrize("index,n", [(2, 256), (3, 96), (4, 96), (5, 128)])
def test_benchmark_problems(index, n):
    prob = workloads.config(index, 8).problem
    pol, inf = workloads.policy_sets(prob, n)
    got, ref = check_slide(prob, pol, inf, f"cfg{index}")
    assert (ref["flags"] == 0).any()


@pytest.mark.parametrize("v,m", [(2, 48), (4, 20), (1, 70), (2, 100)])
def test_stashes_deeper_than_a_queue_word(v, m):
    # W items from "fit most gaps" to "fit none": the stash of an actor grows to all of its m v backward items (a
    # queue word holds 32 entries at two stages per device, 16 at four), drains and grows again
    base = placed_chain(3, v, m, 1, seed=40 + v)
    rng = np.random.default_rng(v * 100 + m)
    n = 60
    pol, inf = random_policies(rng, n, base, rng.random(n) < 0.5)
    S = 3 * v
    for costs in ([5000] * S, [1, 300] * (S // 2) + [1] * (S % 2), list(rng.integers(0, 60, S)), [0] * S):
        prob = copy.deepcopy(base)
        prob.dur[3] = costs
        check_slide(prob, pol, inf, f"v{v} m{m} W costs {costs}")


def test_refusals():
    prob = placed_chain(4, 2, 4, 0, seed=2)   # no split backward: nothing to slide
    h = fp.Problem(prob, stride_for(prob), device=0)
    rng = np.random.default_rng(1)
    pol, inf = random_policies(rng, 4, prob, np.zeros(4, bool))
    with pytest.raises(fp.FpschedError) as e:
        h.generate_evaluate(torch.from_numpy(pol).cuda(), torch.from_numpy(inf).cuda(), slide=True)
    assert e.value.code == -1
    h.close()
