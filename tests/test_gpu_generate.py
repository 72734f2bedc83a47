"""GPU parity of the schedule generator: fpsched_generate, called through the C ABI, must emit the
same op words, step counts and status as the CPU oracle of the scheduler, bit for bit."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_05112_amd as fp
import workloads
from helpers import dag_problem, two_tower_problem
from test_genoracle import NO_LIMIT, PROBLEMS, random_policies, stride_for, uniform_policy
from workloads.problem import chain_problem, one_f_one_b_lists, pack_lists

pytestmark = pytest.mark.gpu


def gpu_generate(problem, pol, inf, stride):
    h = fp.Problem(problem, stride, device=0)
    out = h.generate(torch.from_numpy(np.ascontiguousarray(pol, np.int32)).cuda(),
                     torch.from_numpy(np.ascontiguousarray(inf, np.int32)).cuda(), stride)
    torch.cuda.synchronize()
    res = dict(words=out["ops"].cpu().numpy().view(np.uint16), steps=out["steps"].cpu().numpy(),
               status=out["status"].cpu().numpy())
    h.close()
    return res


def check(problem, pol, inf, stride, what, threads=8):
    ref = oracle.generate(problem, pol, inf, stride, threads=threads)
    gpu = gpu_generate(problem, pol, inf, stride)
    for name in ("status", "steps", "words"):
        if not np.array_equal(gpu[name], ref[name]):
            bad = np.flatnonzero((gpu[name] != ref[name]).reshape(len(pol), -1).any(1))
            raise AssertionError(f"{what}: {name} differs for {len(bad)} sets, first {bad[:5]}")
    return gpu, ref


@pytest.mark.parametrize("name", sorted(PROBLEMS))
def test_small_problems_random_policies(name):
    prob = PROBLEMS[name]()
    rng = np.random.default_rng(3)
    n = 300
    pol, inf = random_policies(rng, n, prob, rng.random(n) < 0.5)
    check(prob, pol, inf, stride_for(prob), name)


def test_1f1b_and_gpipe_orders():
    p, m = 8, 16
    prob = chain_problem(p, m, f=1, b=1, comm=0)
    st = stride_for(prob)
    pol = np.concatenate([uniform_policy(1, p, 0), uniform_policy(1, p, 1)])
    inf = np.full((2, p), NO_LIMIT, np.int32)
    inf[0] = [p - d for d in range(p)]
    gpu, _ = check(prob, pol, inf, st, "1f1b/gpipe")
    assert np.array_equal(gpu["words"][0], pack_lists(one_f_one_b_lists(p, m), st))
    assert list(gpu["steps"]) == [2 * (m + p - 1)] * 2


@pytest.mark.parametrize("index,n", [(1, 64), (2, 256), (3, 96), (4, 96), (5, 128)])
def test_benchmark_problems(index, n):
    # the five benchmark problems (chains with 1-2 stages per device, the two-tower DAG), seeded sets
    prob = workloads.config(index, 8).problem
    pol, inf = workloads.policy_sets(prob, n)
    gpu, ref = check(prob, pol, inf, workloads.generator_stride(prob), f"cfg{index}")
    assert not ref["status"].any()


@pytest.mark.parametrize("p,m,v,w", [(3, 5, 1, None), (5, 9, 2, 1), (7, 4, 3, 1), (33, 3, 1, None), (64, 2, 1, 1),
                                      (64, 3, 4, 1)])
def test_odd_shapes(p, m, v, w):
    prob = chain_problem(p, m, v=v, f=1, b=1, w=w, comm=0)
    rng = np.random.default_rng(p * 100 + m)
    n = 70   # not a multiple of the sets per wavefront
    pol, inf = random_policies(rng, n, prob, rng.random(n) < 0.5)
    check(prob, pol, inf, stride_for(prob), f"p{p} m{m} v{v}")


def test_wide_dag_and_many_microbatches():
    edges = [(0, 2), (1, 2), (2, 3), (2, 4), (3, 5), (4, 5)]   # two sources, a fork and a join
    prob = dag_problem(edges, 6, [0, 1, 2, 0, 1, 2], 3, m=6, has_w=1)
    rng = np.random.default_rng(8)
    pol, inf = random_policies(rng, 200, prob, rng.random(200) < 0.5)
    check(prob, pol, inf, stride_for(prob), "dag")
    prob = chain_problem(2, 2048, f=1, b=1, comm=0)   # the largest micro-batch count of the word format
    pol = np.concatenate([uniform_policy(1, 2, 0), uniform_policy(1, 2, 2, u1=3, u2=2, fint=5)])
    inf = np.array([[2, 1], [NO_LIMIT, 7]], np.int32)
    gpu, _ = check(prob, pol, inf, stride_for(prob), "m=2048")
    assert gpu["steps"][0] >= 2 * 2048


def test_bad_policies_empty_batch_and_call_errors():
    prob = chain_problem(4, 4, v=2, f=1, b=1, comm=0)
    st = stride_for(prob)
    pol = uniform_policy(6, 4, 0)
    inf = np.full((6, 8), 3, np.int32)
    pol[1, 2, 0] = 7            # unknown computation type priority
    pol[2, 0, 1] = 2            # units other than 1 without interleaving
    pol[3, 3, 4] = -1           # negative interval
    inf[4, 5] = 0               # limit below 1
    gpu = gpu_generate(prob, pol, inf, st)
    assert list(gpu["status"]) == [0, 4, 4, 4, 4, 0]
    assert not gpu["words"][1:5].any() and not gpu["steps"][1:5].any()
    ref = oracle.generate(prob, pol[[0, 5]], inf[[0, 5]], st)
    assert np.array_equal(gpu["words"][[0, 5]], ref["words"])
    h = fp.Problem(prob, st, device=0)
    empty = h.generate(torch.empty((0, 4, 8), dtype=torch.int32, device="cuda"),
                       torch.empty((0, 8), dtype=torch.int32, device="cuda"), st)
    assert empty["ops"].shape[0] == 0
    with pytest.raises(fp.FpschedError) as e:   # the stride cannot hold the longest list
        h.generate(torch.zeros((1, 4, 8), dtype=torch.int32, device="cuda"),
                   torch.ones((1, 8), dtype=torch.int32, device="cuda"), 8)
    assert e.value.code == -1
    h.close()


def test_generate_evaluate_topk_pipeline():
    # the search loop on the GPU: schedules never leave HBM between the three calls
    spec = workloads.config(4, 8)
    prob = spec.problem
    n, k = 192, 16
    pol, inf = workloads.policy_sets(prob, n)
    st = workloads.generator_stride(prob)
    h = fp.Problem(prob, st, device=0)
    out = h.generate(torch.from_numpy(pol).cuda(), torch.from_numpy(inf).cuda(), st)
    res = h.evaluate(out["ops"])
    top = h.topk(res, k)
    torch.cuda.synchronize()
    ref_words = oracle.generate(prob, pol, inf, st, threads=8)["words"]
    ref = oracle.evaluate(prob, ref_words, threads=8)
    idx, ms, cnt = oracle.topk(ref["makespan"], ref["flags"], k)
    assert int(top["count"].item()) == cnt and cnt > 0
    assert np.array_equal(top["idx"].cpu().numpy(), idx) and np.array_equal(top["makespan"].cpu().numpy(), ms)
    for name in ("makespan", "idle", "peak", "flags"):
        assert np.array_equal(res[name].cpu().numpy(), ref[name])
    h.close()
