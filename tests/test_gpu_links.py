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
from gpu_common import assert_same, check_batch, gpu_evaluate
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
    # the sliding pass follows the switch
    slid = h.wslide(ops)
    torch.cuda.synchronize()
    ref = oracle.wslide(prob, words, spec.stride, threads=8, links=True)
    for name in ("ops", "makespan", "idle", "peak", "flags"):
        got = slid[name].cpu().numpy()
        assert np.array_equal(got.view(np.uint16) if name == "ops" else got, ref[name]), name
    h.select_kernel("general")
    with pytest.raises(fp.FpschedError) as e:
        h.evaluate(ops)
    assert e.value.code == -6
    h.select_kernel("auto")
    h.set_link_occupancy(False)
    assert_same(run(), plain, "links off")
    # both variants, in either order of the calls, and back to each alone
    table = workloads.microbatch_costs(prob)
    both = oracle.evaluate(prob, words, threads=8, dur_mb=table, links=True)
    h.set_microbatch_costs(table)
    h.set_link_occupancy(True)
    assert_same(run(), both, "costs, then links")
    with pytest.raises(fp.FpschedError) as e:
        h.wslide(ops)
    assert e.value.code == -6
    h.set_microbatch_costs(None)
    assert_same(run(), linked, "links alone again")
    h.set_microbatch_costs(table)
    assert_same(run(), both, "links, then costs")
    h.set_link_occupancy(False)
    assert_same(run(), oracle.evaluate(prob, words, threads=8, dur_mb=table), "costs alone")
    h.close()


@pytest.mark.parametrize("index,n", [(2, 3000), (3, 700), (4, 900), (5, 2000)])
def test_both_variants_on_the_benchmark_shapes(index, n):
    spec = workloads.config(index, n)
    words = workloads.generate(spec, threads=8)
    prob = slow_links(spec.problem, 70 + index)
    check_batch(prob, words, k=16, what=f"cfg{index}", links=True, dur_mb=workloads.microbatch_costs(prob))


@pytest.mark.parametrize("seed", range(6))
def test_both_variants_on_random_problems(seed):
    rng = np.random.default_rng(9800 + seed)
    for i in range(8):
        prob = random_problem(rng)
        prob.edge_comm[:] = rng.integers(0, 12, len(prob.edge_comm))
        table = rng.integers(0, 40 if i % 2 else 2000, (8, prob.n_stages, prob.n_microbatches)).astype(np.int32)
        lists = []
        for t in range(16):
            base = random_valid_lists(prob, rng, 0.3 * (t % 2), 0.3 * ((t // 2) % 2))
            lists.append(base)
            lists.append(perturb(base, rng, 1 + t % 3))
        check_batch(prob, batch_from_lists(lists), k=5, what=f"seed {seed} problem {i}", links=True, dur_mb=table)


def check_slide(prob, words, stride_out, what):
    h = fp.Problem(prob, max(words.shape[2], stride_out), device=0)
    h.set_link_occupancy(True)
    out = h.wslide(torch.from_numpy(words.view(np.int16)).cuda(), stride_out)
    torch.cuda.synchronize()
    ref = oracle.wslide(prob, words, stride_out, threads=8, links=True)
    for name in ("flags", "makespan", "idle", "peak", "ops"):
        got = out[name].cpu().numpy()
        got = got.view(np.uint16) if name == "ops" else got
        if not np.array_equal(got, ref[name]):
            bad = np.flatnonzero((got != ref[name]).reshape(len(got), -1).any(1))
            raise AssertionError(f"{what}: {name} differs for {len(bad)} candidates, first {bad[:5]}")
    h.close()
    return ref


@pytest.mark.parametrize("index,n", [(2, 3000), (3, 700), (4, 600), (5, 2000)])
def test_sliding_pass_under_link_occupancy_on_the_benchmark_shapes(index, n):
    spec = workloads.config(index, n)
    words = workloads.generate(spec, threads=8)
    prob = slow_links(spec.problem, 50 + index)
    ref = check_slide(prob, words, spec.stride, f"cfg{index}")
    plain = oracle.wslide(prob, words, spec.stride, threads=8)
    ok = ref["flags"] & 3 == 0
    assert ok.sum() > 0 and (ref["makespan"][ok] > plain["makespan"][ok]).any()


@pytest.mark.parametrize("seed", range(6))
def test_sliding_pass_under_link_occupancy_on_random_problems(seed):
    rng = np.random.default_rng(9500 + seed)
    done = 0
    while done < 8:
        prob = random_problem(rng)
        if not prob.has_w:
            continue
        prob.edge_comm[:] = rng.integers(0, 12, len(prob.edge_comm))
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
        for stride_out in (stride + 8, max(8, (stride // 2) // 8 * 8)):
            check_slide(prob, words, stride_out, f"seed {seed} problem {done} stride_out {stride_out}")
        done += 1


def test_largest_sizes_under_link_occupancy():
    from workloads.problem import one_f_one_b_lists
    # many micro-batches, a link slower than the items; with the largest count of the word format the
    # link words no longer fit beside the state words, and the call says so
    for m in (512, 2048):
        prob = chain_problem(2, m, f=1, b=2, comm=3)
        words = np.stack([pack_lists(one_f_one_b_lists(2, m), stride=2 * m), pack_lists(gpipe_lists(2, m), stride=2 * m)])
        gpu, _ = gpu_evaluate(prob, words, kernel="slots", links=True)
        if m == 2048 and gpu is None:
            continue
        assert_same(gpu, oracle.evaluate(prob, words, links=True), f"m={m}")
        assert gpu["makespan"][1] == 2 * (1 + 2) + 2 * m * 3        # p (f + b) + 2 (m + p - 2) c
    # 64 devices, and 252 stages on 63 devices (four per device, each sending both ways)
    prob = chain_problem(64, 6, f=2, b=4, comm=5)
    words = np.stack([pack_lists(gpipe_lists(64, 6)), pack_lists(one_f_one_b_lists(64, 6))])
    gpu, _ = check_batch(prob, words, k=2, what="p=64", links=True)
    assert gpu["makespan"][0] == 64 * 6 + 2 * (6 + 64 - 2) * 5
    prob = chain_problem(63, 3, v=4, f=2, b=3, w=1, comm=4)
    rng = np.random.default_rng(63)
    lists = []
    for t in range(6):
        base = random_valid_lists(prob, rng)
        lists += [base, perturb(base, rng, 2)]
    check_batch(prob, batch_from_lists(lists), k=3, what="S=252", links=True)
