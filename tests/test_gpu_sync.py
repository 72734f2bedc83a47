"""GPU parity of the evaluation with synchronisation stages and dependency pairs
(fpsched_problem_set_sync + fpsched_evaluate) against oracle/fpsyncoracle.c, bit for bit, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_05112_amd as fp
import workloads
from gpu_common import assert_same
from helpers import batch_from_lists, perturb, random_slot_sync_problem, random_sync_lists, random_sync_problem
from workloads.problem import B, F, FD, W, make_problem, pack_lists, pack_word

pytestmark = pytest.mark.gpu


def gpu_sync(problem, words, group, pairs, k=None, max_stride=None, kernel="auto", expect_kernel=None):
    """kernel: "auto" = the slot kernel's form of the model where the setting fits it, "general" = the table
    kernel (eval_sync_kernel<false>)."""
    words = np.ascontiguousarray(words, dtype=np.uint16)
    C, D, stride = words.shape
    h = fp.Problem(problem, max_stride or stride, device=0)
    if kernel != "auto":
        h.select_kernel(kernel)
    h.set_sync(group, pairs)
    if expect_kernel:
        assert h.active_kernel() == expect_kernel
    ops = torch.from_numpy(words.view(np.int16)).cuda()
    res = h.evaluate(ops)
    top = h.topk(res, k) if k else None
    torch.cuda.synchronize()
    out = {n: v.cpu().numpy() for n, v in res.items()}
    if top is not None:
        top = (top["idx"].cpu().numpy(), top["makespan"].cpu().numpy(), int(top["count"].item()))
    h.close()
    return out, top


def test_hand_worked_timeline_on_the_gpu():
    dur = {F: [2, 3, 1], B: [4, 5, 1]}
    prob = make_problem(2, 3, 2, 0, [0, 1, 1], [(0, 2, 1), (1, 2, 7)], dur, mem_units=[1, 1, 0])
    lists = [[(F, 0, 0), (F, 0, 1), (B, 0, 0), (B, 0, 1)],
             [(F, 0, 0), (F, 0, 1), (F, 1, 0), (B, 1, 0), (B, 0, 0), (B, 0, 1)]]
    early = [lists[0], [lists[1][0], lists[1][2], lists[1][1]] + lists[1][3:]]
    bad = [lists[0], lists[1][:2] + [(F, 1, 1)] + lists[1][3:]]
    words = batch_from_lists([lists, early, bad], 8)
    for kernel in ("slots", "general"):   # the synchronisation stage's neighbours have one item per micro-batch
        out, _ = gpu_sync(prob, words, [1, 1, 2], None, kernel="auto" if kernel == "slots" else kernel,
                          expect_kernel=kernel)
        assert list(out["flags"]) == [0, 1, 3] and out["makespan"][0] == 18
        assert list(out["idle"][0]) == [6, 0] and list(out["peak"][0]) == [2, 2]
        assert_same(out, oracle.evaluate_sync(prob, words, group=[1, 1, 2]), f"hand-worked {kernel}")


def test_random_problems_groups_and_pairs_against_the_oracle():
    rng = np.random.default_rng(77)
    n_run = n_dead = n_w = 0
    for trial in range(60):
        prob, group, pairs = random_sync_problem(rng, trial)
        lists = []
        for t in range(6):
            base = random_sync_lists(prob, group, pairs, rng, 0.25 * (t % 2), 0.25 * ((t // 2) % 2))
            if base is None:
                break
            cut = [list(x) for x in base]
            d = int(rng.integers(prob.n_devices))
            if cut[d]:
                cut[d].pop(int(rng.integers(len(cut[d]))))
            lists += [base, perturb(base, rng, 1 + t % 3), cut]
        if not lists:
            continue
        words = batch_from_lists(lists)
        # a word whose item index is beyond its stage's item count
        words[-1, 0, 0] = pack_word(F, 0, 2047)
        ref = oracle.evaluate_sync(prob, words, group=group, pairs=pairs)
        out, top = gpu_sync(prob, words, group, pairs, k=5)
        assert_same(out, ref, f"trial {trial}")
        idx, ms, cnt = oracle.topk(ref["makespan"], ref["flags"], 5)
        assert top[2] == cnt and np.array_equal(top[0], idx) and np.array_equal(top[1], ms)
        n_run += 1
        n_dead += int((ref["flags"] & 1).sum())
        n_w += any(int(q[0]) == W for q in pairs)
    assert n_run > 45 and n_dead > 60 and n_w > 3


def test_settings_the_slot_kernel_has_a_form_for():
    # groups in the middle of chains and at joins, forward and backward pairs, two inputs or outputs per stage:
    # the slot kernel's form of the model and the table kernel against the oracle
    rng = np.random.default_rng(91)
    n_grouped = n_pairs = n_deg2 = n_dead = 0
    for trial in range(80):
        prob, group, pairs = random_slot_sync_problem(rng)
        lists = []
        for t in range(6):
            base = random_sync_lists(prob, group, pairs, rng, 0.25 * (t % 2), 0.25 * ((t // 2) % 2))
            if base is None:
                break
            cut = [list(x) for x in base]
            d = int(rng.integers(prob.n_devices))
            if cut[d]:
                cut[d].pop(int(rng.integers(len(cut[d]))))
            lists += [base, perturb(base, rng, 1 + t % 3), cut]
        if not lists:
            continue
        words = batch_from_lists(lists)
        words[-1, 0, 0] = pack_word(F, 0, 2047)   # an item index beyond its stage's item count
        ref = oracle.evaluate_sync(prob, words, group=group, pairs=pairs)
        out, top = gpu_sync(prob, words, group, pairs, k=5, expect_kernel="slots")
        assert_same(out, ref, f"trial {trial} slots")
        idx, ms, cnt = oracle.topk(ref["makespan"], ref["flags"], 5)
        assert top[2] == cnt and np.array_equal(top[0], idx) and np.array_equal(top[1], ms)
        out, _ = gpu_sync(prob, words, group, pairs, kernel="general", expect_kernel="general")
        assert_same(out, ref, f"trial {trial} general")
        n_grouped += any(g > 1 for g in group)
        n_pairs += bool(pairs)
        n_deg2 += max(np.bincount(np.asarray(prob.edge_dst), minlength=1)) > 1
        n_dead += int((ref["flags"] & 1).sum())
    assert n_grouped > 30 and n_pairs > 10 and n_deg2 > 20 and n_dead > 40


@pytest.mark.parametrize("kernel", ["slots", "general"])
@pytest.mark.parametrize("every", [1, 4, 7, 64])
def test_multimodal_workload_reduced_batch(every, kernel):
    spec = workloads.sync_config(3001, sync_every=every)
    words = workloads.generate_sync(spec, threads=8)
    ref = oracle.evaluate_sync(spec.problem, words, spec.group, spec.pairs, threads=8)
    out, top = gpu_sync(spec.problem, words, spec.group, spec.pairs, k=spec.top_k,
                        kernel="auto" if kernel == "slots" else kernel, expect_kernel=kernel)
    assert_same(out, ref, f"sync every {every}")
    idx, ms, cnt = oracle.topk(ref["makespan"], ref["flags"], spec.top_k)
    assert top[2] == cnt and np.array_equal(top[0], idx) and np.array_equal(top[1], ms)
    assert (ref["flags"] & 1).sum() > 0 and (ref["flags"] == 4).sum() > 0
    if every < 12:     # (a synchronisation over more micro-batches than the cap holds keeps every schedule over it)
        assert (ref["flags"] == 0).sum() > 300


def test_switching_the_model_on_and_off_and_what_it_excludes():
    spec = workloads.sync_config(64)
    words = workloads.generate_sync(spec, threads=4)
    prob = spec.problem
    h = fp.Problem(prob, spec.stride, device=0)
    ops = torch.from_numpy(words.view(np.int16)).cuda()

    def run():
        res = h.evaluate(ops)
        torch.cuda.synchronize()
        return {n: v.cpu().numpy() for n, v in res.items()}

    plain = oracle.evaluate(prob, words)                      # group 1 everywhere: most lists are incomplete
    assert_same(run(), plain, "before")
    h.set_sync(spec.group, spec.pairs)
    assert_same(run(), oracle.evaluate_sync(prob, words, spec.group, spec.pairs), "on")
    for call in (lambda: h.set_link_occupancy(True), lambda: h.set_microbatch_costs(workloads.microbatch_costs(prob)),
                 lambda: h.wslide(ops, spec.stride)):
        with pytest.raises(fp.FpschedError) as e:
            call()
        assert e.value.code == -6
    # another setting replaces the first one; pairs alone, with a weight-gradient producer
    pairs = [(W, 5, W, 11, 3), (B, 12, B, 0, 0)]
    h.set_sync(None, pairs)
    assert_same(run(), oracle.evaluate_sync(prob, words, None, pairs), "pairs only")
    h.set_sync()
    assert_same(run(), plain, "off")
    h.set_link_occupancy(True)
    with pytest.raises(fp.FpschedError) as e:
        h.set_sync(spec.group, spec.pairs)
    assert e.value.code == -6
    h.set_link_occupancy(False)
    # the entry point without a workspace follows the switch
    h.set_sync(spec.group, spec.pairs)
    res, top = h.alloc_results(len(words)), dict(idx=torch.empty(8, dtype=torch.int64, device="cuda"),
                                                 makespan=torch.empty(8, dtype=torch.int64, device="cuda"),
                                                 count=torch.empty(1, dtype=torch.int32, device="cuda"))
    h.evaluate_topk_static(ops, 8, res, top)
    torch.cuda.synchronize()
    ref = oracle.evaluate_sync(prob, words, spec.group, spec.pairs)
    idx, ms, cnt = oracle.topk(ref["makespan"], ref["flags"], 8)
    assert np.array_equal(top["idx"].cpu().numpy(), idx) and int(top["count"].item()) == cnt
    for bad in (dict(group=[0] * 13), dict(pairs=[(4, 0, F, 1, 0)]), dict(pairs=[(F, 0, F, 0, 0)]),
                dict(pairs=[(F, 0, F, 13, 0)]), dict(pairs=[(F, 0, B, 1, -1)])):
        with pytest.raises(fp.FpschedError) as e:
            h.set_sync(**bad)
        assert e.value.code == -1
    assert_same(run(), ref, "after refused settings")
    h.close()


def test_large_shapes():
    # tables of 6 KB per kind and candidate, groups of 32 on the second half of the chain, a ragged last group
    rng = np.random.default_rng(3)
    D, S, m = 8, 16, 100
    edges = [(s, s + 1, 1 + s % 3) for s in range(S - 1)]
    dur = {F: rng.integers(1, 9, S), B: rng.integers(1, 9, S), W: rng.integers(0, 5, S)}
    prob = make_problem(D, S, m, 1, [s % D for s in range(S)], edges, dur, mem_cap=4 * m)
    group = [1] * 8 + [32] * 8
    lists = [random_sync_lists(prob, group, [], rng) for _ in range(3)]
    lists.append(perturb(lists[0], rng, 3))
    words = batch_from_lists(lists)
    out, _ = gpu_sync(prob, words, group, None)
    assert_same(out, oracle.evaluate_sync(prob, words, group=group), "large")
    assert (out["flags"][:3] & 3 == 0).all()
