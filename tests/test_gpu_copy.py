"""GPU parity of the copy-engine form of the cost model (fpsched_problem_set_copy_engine + fpsched_evaluate)
against oracle/fpcopyoracle.c, bit for bit, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_05112_amd as fp
import workloads
from gpu_common import assert_same
from helpers import batch_from_lists, dag_problem, perturb, random_valid_lists, two_tower_problem
from workloads.problem import B, F, FD, L, O, R, W, chain_problem, make_problem, pack_lists

pytestmark = pytest.mark.gpu


def gpu_copy(problem, words, depth, k=None, kernel="auto"):
    """kernel: "auto" = the slot kernel's copy-engine form where the problem fits it, "general" = the table
    kernel (eval_sync_kernel<true>)."""
    words = np.ascontiguousarray(words, dtype=np.uint16)
    h = fp.Problem(problem, words.shape[2], device=0)
    if kernel != "auto":
        h.select_kernel(kernel)
    h.set_copy_engine(depth)
    res = h.evaluate(torch.from_numpy(words.view(np.int16)).cuda())
    top = h.topk(res, k) if k else None
    torch.cuda.synchronize()
    out = {n: v.cpu().numpy() for n, v in res.items()}
    if top is not None:
        top = (top["idx"].cpu().numpy(), top["makespan"].cpu().numpy(), int(top["count"].item()))
    h.close()
    return out, top


def test_hand_worked_timelines_on_the_gpu():
    prob = make_problem(1, 1, 3, 0, [0], [], {F: 3, B: 4, O: 5, L: 2})
    ops = [(F, 0, 0), (O, 0, 0), (F, 0, 1), (O, 0, 1), (F, 0, 2), (L, 0, 0), (L, 0, 1), (B, 0, 0), (B, 0, 1), (B, 0, 2)]
    words = pack_lists([ops], 16)[None]
    for kernel in ("auto", "general"):
        for depth in (1, 4, 7):
            out, _ = gpu_copy(prob, words, depth, kernel=kernel)
            assert out["flags"][0] == 0 and out["makespan"][0] == 27 and out["idle"][0, 0] == 6 and out["peak"][0, 0] == 3
            assert_same(out, oracle.evaluate_copy(prob, words, depth=depth), f"depth {depth} {kernel}")
    # an allocation of the compute timeline counts before a release of the copy engine at the same time
    for kernel in ("auto", "general"):
        for o_cost, expect in ((5, 3), (4, 2)):
            prob2 = make_problem(1, 2, 2, 0, [0, 0], [], {F: [3, 5], B: [1, 1], O: o_cost, L: 1})
            ops = [(F, 0, 0), (O, 0, 0), (F, 1, 0), (F, 1, 1), (B, 1, 0), (B, 1, 1), (L, 0, 0), (B, 0, 0), (F, 0, 1), (B, 0, 1)]
            out, _ = gpu_copy(prob2, pack_lists([ops], 16)[None], 4, kernel=kernel)
            assert out["flags"][0] == 0 and out["peak"][0, 0] == expect


def transfer_problems():
    chain = chain_problem(3, 5, v=2, f=2, b=3, w=1, comm=1)
    chain.dur[O], chain.dur[L] = 9, 7
    wide = chain_problem(12, 4, v=1, f=3, b=5, comm=2)
    wide.dur[O], wide.dur[L] = 2, 11
    return [chain, two_tower_problem(m=4, has_w=1, comm=2, mem_cap=3), wide,
            dag_problem([(0, 1), (0, 2), (1, 3), (2, 3)], 4, [0, 1, 2, 0], 3, m=4, has_w=0, seed=3)]


@pytest.mark.parametrize("kernel", ["auto", "general"])
@pytest.mark.parametrize("depth", [1, 2, 4, 7])
def test_random_lists_with_transfers_against_the_oracle(depth, kernel):
    rng = np.random.default_rng(100 + depth)
    for prob in transfer_problems():
        lists = []
        for t in range(50):
            base = random_valid_lists(prob, rng, 0.25 * (t % 2), 0.25 + 0.25 * (t % 3))
            lists += [base, perturb(base, rng, 1 + t % 3)]
        words = batch_from_lists(lists)
        ref = oracle.evaluate_copy(prob, words, depth=depth, threads=4)
        out, top = gpu_copy(prob, words, depth, k=9, kernel=kernel)
        assert_same(out, ref, f"{prob.name} depth {depth}")
        idx, ms, cnt = oracle.topk(ref["makespan"], ref["flags"], 9)
        assert top[2] == cnt and np.array_equal(top[0], idx) and np.array_equal(top[1], ms)
        assert (ref["flags"] & 1).any() and ((ref["flags"] & 3) == 0).any()
        # the transfers do overlap the computation: faster than the plain model somewhere
        plain = oracle.evaluate(prob, words, threads=4)
        ok = (plain["flags"] & 3) == 0
        assert (ref["makespan"][ok] <= plain["makespan"][ok]).all() and (ref["makespan"][ok] < plain["makespan"][ok]).any()


def test_configuration_five_reduced_batch_and_switching():
    spec = workloads.config(5, 3001)
    words = workloads.generate(spec, threads=8)
    prob = spec.problem
    h = fp.Problem(prob, spec.stride, device=0)
    ops = torch.from_numpy(words.view(np.int16)).cuda()

    def run():
        res = h.evaluate(ops)
        torch.cuda.synchronize()
        return {n: v.cpu().numpy() for n, v in res.items()}

    plain = oracle.evaluate(prob, words, threads=8)
    assert_same(run(), plain, "before")
    for depth in (4, 1):
        h.set_copy_engine(depth)
        assert_same(run(), oracle.evaluate_copy(prob, words, depth=depth, threads=8), f"depth {depth}")
    for call in (lambda: h.set_link_occupancy(True), lambda: h.set_microbatch_costs(workloads.microbatch_costs(prob)),
                 lambda: h.wslide(ops, spec.stride), lambda: h.set_sync(pairs=[(F, 0, F, 6, 0)])):
        with pytest.raises(fp.FpschedError) as e:
            call()
        assert e.value.code == -6
    for bad in (-1, 8):
        with pytest.raises(fp.FpschedError) as e:
            h.set_copy_engine(bad)
        assert e.value.code == -1
    assert_same(run(), oracle.evaluate_copy(prob, words, depth=1, threads=8), "after refused settings")
    h.set_copy_engine(0)
    assert_same(run(), plain, "off")
    h.set_sync(pairs=[(F, 0, F, 6, 0)])
    with pytest.raises(fp.FpschedError) as e:
        h.set_copy_engine(2)
    assert e.value.code == -6
    h.close()
    # a problem whose transfers cost nothing is refused: a transfer takes time
    free = fp.Problem(chain_problem(2, 2), 8, device=0)
    with pytest.raises(fp.FpschedError) as e:
        free.set_copy_engine(2)
    assert e.value.code == -1
    free.close()
