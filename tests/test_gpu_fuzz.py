"""GPU parity on many small random problems: random stage DAGs (in/out degree <= 2), random placements
with 1-4 stages per device, random durations, latencies, units and caps, with valid, perturbed and
truncated candidates.  Both evaluation kernels and the generator, bit for bit against the oracles."""
import numpy as np
import pytest

import oracle
from gpu_common import check_batch
from helpers import batch_from_lists, dag_problem, perturb, random_valid_lists
from test_genoracle import random_policies, stride_for
from test_gpu_generate import check as check_generate

pytestmark = pytest.mark.gpu


def random_dag(rng, S):
    """Edges a -> b with a < b, every stage but the first few has 1-2 predecessors, out-degree <= 2."""
    edges, outdeg = [], [0] * S
    n_sources = int(rng.integers(1, min(3, S) + 1))
    for b in range(n_sources, S):
        cands = [a for a in range(b) if outdeg[a] < 2]
        if not cands:
            continue
        k = min(len(cands), int(rng.integers(1, 3)))
        for a in rng.choice(cands, size=k, replace=False):
            edges.append((int(a), b))
            outdeg[int(a)] += 1
    return edges


def random_problem(rng):
    D = int(rng.integers(1, 9))
    v = int(rng.integers(1, 5))
    S = int(rng.integers(max(1, D), D * v + 1))
    # placement: every device at most 4 stages
    slots = np.repeat(np.arange(D), 4)
    stage_device = np.sort(rng.permutation(slots)[:S]) if rng.random() < 0.5 else rng.permutation(slots)[:S]
    m = int(rng.integers(1, 12))
    has_w = int(rng.integers(0, 2))
    edges = random_dag(rng, S)
    prob = dag_problem(edges, S, [int(x) for x in stage_device], D, m=m, has_w=has_w, seed=int(rng.integers(1 << 30)))
    if rng.random() < 0.5:
        prob.mem_units[:] = rng.integers(1, 4, S) * int(rng.choice([1, 7, 100]))
    prob.mem_cap[:] = rng.integers(1, 6, D) * int(prob.mem_units.max()) * max(1, m // 2)
    return prob


@pytest.mark.parametrize("seed", range(12))
def test_random_problems_evaluation(seed):
    rng = np.random.default_rng(1000 + seed)
    n_problems = 0
    for _ in range(12):
        prob = random_problem(rng)
        lists = []
        for t in range(24):
            base = random_valid_lists(prob, rng, 0.3 * (t % 2), 0.3 * ((t // 2) % 2))
            lists.append(base)
            lists.append(perturb(base, rng, 1 + t % 3))
            if t % 6 == 0:   # a list cut short: incomplete, or a deadlock downstream
                cut = [list(x) for x in base]
                d = int(rng.integers(prob.n_devices))
                cut[d] = cut[d][: len(cut[d]) // 2]
                lists.append(cut)
        check_batch(prob, batch_from_lists(lists), k=7, what=f"seed {seed} problem {n_problems}")
        n_problems += 1


@pytest.mark.parametrize("seed", range(6))
def test_random_problems_generator(seed):
    rng = np.random.default_rng(2000 + seed)
    for i in range(10):
        prob = random_problem(rng)
        n = 40
        pol, inf = random_policies(rng, n, prob, rng.random(n) < 0.5)
        gpu, ref = check_generate(prob, pol, inf, stride_for(prob), f"seed {seed} problem {i}")
        # whatever the scheduler emits, the evaluator accepts
        ev = oracle.evaluate(prob, ref["words"], threads=4)
        assert not (ev["flags"] & 3).any()


@pytest.mark.parametrize("seed", range(8))
def test_random_problems_sliding(seed):
    """fpsched_wslide on random DAGs, placements (1 to 4 stages per device) and lists with recompute and
    offload items, valid, perturbed and cut short; rows that are wide enough and rows that are not."""
    import torch

    import paper_2510_05112_amd as fp
    rng = np.random.default_rng(3000 + seed)
    done = 0
    while done < 8:
        prob = random_problem(rng)
        if not prob.has_w:
            continue
        lists = []
        for t in range(16):
            base = random_valid_lists(prob, rng, 0.3 * (t % 2), 0.3 * ((t // 2) % 2))
            lists.append(base)
            lists.append(perturb(base, rng, 1 + t % 3))
            if t % 5 == 0:
                cut = [list(x) for x in base]
                d = int(rng.integers(prob.n_devices))
                cut[d] = cut[d][: len(cut[d]) // 2]
                lists.append(cut)
        words = batch_from_lists(lists)
        stride = words.shape[2]
        h = fp.Problem(prob, stride + 8, device=0)
        for stride_out in (stride + 8, max(8, (stride // 2) // 8 * 8)):
            out = h.wslide(torch.from_numpy(words.view(np.int16)).cuda(), stride_out)
            torch.cuda.synchronize()
            ref = oracle.wslide(prob, words, stride_out, threads=4)
            what = f"seed {seed} problem {done} stride_out {stride_out}"
            assert np.array_equal(out["ops"].cpu().numpy().view(np.uint16), ref["ops"]), what
            for name in ("makespan", "idle", "peak", "flags"):
                assert np.array_equal(out[name].cpu().numpy(), ref[name]), (what, name)
        # the one-kernel form without lists
        only = h.wslide_evaluate(torch.from_numpy(words.view(np.int16)).cuda())
        torch.cuda.synchronize()
        ref = oracle.wslide(prob, words, stride + 8, threads=4)
        for name in ("makespan", "idle", "peak", "flags"):
            assert np.array_equal(only[name].cpu().numpy(), ref[name]), (f"seed {seed} problem {done} no lists", name)
        h.close()
        done += 1


@pytest.mark.parametrize("seed", range(6))
def test_random_problems_fused_generator(seed):
    # generator and evaluator in one kernel against the two oracles composed on the CPU
    from test_gpu_generate_evaluate import check as check_fused
    from test_gpu_generate_slide import check_slide
    rng = np.random.default_rng(3000 + seed)
    for i in range(10):
        prob = random_problem(rng)
        n = 40
        pol, inf = random_policies(rng, n, prob, rng.random(n) < 0.5)
        check_fused(prob, pol, inf, f"seed {seed} problem {i}")
        if prob.has_w:   # ... and with the sliding pass in the kernel
            check_slide(prob, pol, inf, f"seed {seed} problem {i}, sliding")


@pytest.mark.parametrize("seed", range(6))
def test_random_problems_copy_engine(seed):
    # the copy-engine model on both evaluation kernels against its oracle
    from test_gpu_copy import gpu_copy
    from gpu_common import assert_same
    rng = np.random.default_rng(4000 + seed)
    for i in range(8):
        prob = random_problem(rng)
        depth = int(rng.integers(1, 8))
        lists = []
        for t in range(16):
            base = random_valid_lists(prob, rng, 0.3 * (t % 2), 0.2 + 0.3 * ((t // 2) % 2))
            lists += [base, perturb(base, rng, 1 + t % 3)]
        words = batch_from_lists(lists)
        ref = oracle.evaluate_copy(prob, words, depth=depth, threads=4)
        for kernel in ("auto", "general"):
            out, _ = gpu_copy(prob, words, depth, kernel=kernel)
            assert_same(out, ref, f"seed {seed} problem {i} depth {depth} {kernel}")
