"""GPU parity of the link-occupancy variant (fpsched_problem_set_link_occupancy + fpsched_evaluate) against
the oracle's variant, bit for bit, on the benchmark shapes with latencies that make links matter and on
random problems, through the C ABI."""
import copy

import numpy as np
import pytest
import torch

import oracle
import paper_2510_05112_amd as fp
import workloads
from gpu_common import assert_same, check_batch
from helpers import batch_from_lists, perturb, random_valid_lists
from test_gpu_fuzz import random_problem
from workloads.problem import chain_problem, gpipe_lists, pack_lists

pytestmark = pytest.mark.gpu


def slow_links(prob, seed):
    """The same problem with latencies of the order of the items' costs (a link is then often busy)."""
    rng = np.random.default_rng(seed)
    slow = copy.deepcopy(prob)
    typical = int(np.median(np.asarray(prob.dur)[1]))
    slow.edge_comm[:] = rng.integers(0, 2 * typical + 2, len(slow.edge_comm))
    return slow


@pytest.mark.parametrize("index,n", [(1, 64), (2, 3000), (3, 700), (4, 900), (5, 2000)])
def test_benchmark_shapes(index, n):
    spec = workloads.config(index, n)
    words = workloads.generate(spec, threads=8)
    # the configuration's own latencies (1: links hardly matter), then slow links
    check_batch(spec.problem, words, k=16, what=f"cfg{index}", links=True)
    prob = slow_links(spec.problem, index)
    gpu, ref = check_batch(prob, words, k=16, what=f"cfg{index} with slow links", links=True)
    plain = oracle.evaluate(prob, words, threads=8)
    ok = ref["flags"] & 3 == 0
    assert ok.sum() > 0 and (ref["makespan"][ok] > plain["makespan"][ok]).any()   # the links matter


@pytest.mark.parametrize("p,m,f,b,c", [(4, 8, 2, 4, 4), (8, 16, 3, 2, 7), (4, 8, 2, 4, 1)])
def test_gpipe_closed_forms_on_the_gpu(p, m, f, b, c):
    prob = chain_problem(p, m, f=f, b=b, comm=c)
    gpu, _ = check_batch(prob, pack_lists(gpipe_lists(p, m))[None], what="gpipe", links=True)
    expect = p * (f + b) + 2 * (m + p - 2) * c if c >= max(f, b) else (m + p - 1) * (f + b) + 2 * (p - 1) * c
    assert gpu["makespan"][0] == expect


@pytest.mark.parametrize("seed", range(8))
def test_random_problems(seed):
    rng = np.random.default_rng(9000 + seed)
    for i in range(10):
        prob = random_problem(rng)
        prob.edge_comm[:] = rng.integers(0, 12, len(prob.edge_comm))
        lists = []
        for t in range(20):
            base = random_valid_lists(prob, rng, 0.3 * (t % 2), 0.3 * ((t // 2) % 2))
            lists.append(base)
            lists.append(perturb(base, rng, 1 + t % 3))
            if t % 6 == 0:
                cut = [list(x) for x in base]
                d = int(rng.integers(prob.n_devices))
                cut[d] = cut[d][: len(cut[d]) // 2]
                lists.append(cut)
        check_batch(prob, batch_from_lists(lists), k=5, what=f"seed {seed} problem {i}", links=True)


def test_switching_the_variant_on_and_off_on_one_handle():
    spec = workloads.config(2, 1500)
    prob = slow_links(spec.problem, 7)
    words = workloads.generate(spec, threads=8)
    ops = torch.from_numpy(words.view(np.int16)).cuda()
    h = fp.Problem(prob, spec.stride, device=0)

    def run():
        res = h.evaluate(ops)
        torch.cuda.synchronize()
        return {n: v.cpu().numpy() for n, v in res.items()}

    plain = oracle.evaluate(prob, words, threads=8)
    linked = oracle.evaluate(prob, words, threads=8, links=True)
    assert_same(run(), plain, "before")
    h.set_link_occupancy(True)
    assert_same(run(), linked, "links on")
    for refused in (lambda: h.wslide(ops), lambda: h.set_microbatch_costs(workloads.microbatch_costs(prob))):
        with pytest.raises(fp.FpschedError) as e:
            refused()
        assert e.value.code == -6
    h.select_kernel("general")
    with pytest.raises(fp.FpschedError) as e:
        h.evaluate(ops)
    assert e.value.code == -6
    h.select_kernel("auto")
    h.set_link_occupancy(False)
    assert_same(run(), plain, "links off")
    h.set_microbatch_costs(workloads.microbatch_costs(prob))
    with pytest.raises(fp.FpschedError) as e:
        h.set_link_occupancy(True)
    assert e.value.code == -6
    h.set_microbatch_costs(None)
    h.set_link_occupancy(True)
    assert_same(run(), linked, "links on again")
    h.close()
