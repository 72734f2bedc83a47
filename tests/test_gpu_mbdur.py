"""GPU parity of the per-micro-batch cost variant (fpsched_problem_set_microbatch_costs + fpsched_evaluate)
against the oracle's variant, bit for bit, on the benchmark shapes and on random problems, through both
evaluation kernels."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_05112_amd as fp
import workloads
from gpu_common import assert_same, check_batch
from helpers import batch_from_lists, perturb, random_valid_lists
from test_gpu_fuzz import random_problem

pytestmark = pytest.mark.gpu

NKINDS = 8


def scaled_table(prob, rng):
    """The problem's costs scaled per micro-batch by a factor in [1/2, 3/2): sequences of unequal length."""
    return workloads.microbatch_costs(prob, seed=int(rng.integers(1 << 30)))


@pytest.mark.parametrize("table_in", ["lds", "device memory"])
@pytest.mark.parametrize("index,n", [(1, 64), (2, 3000), (3, 700), (4, 900), (5, 2000)])
def test_benchmark_shapes_with_costs_per_micro_batch(index, n, table_in, monkeypatch):
    # the slot kernel reads the costs from LDS when the table fits there, else from device memory
    # (FPSCHED_MB_GLOBAL forces the latter)
    if table_in != "lds":
        monkeypatch.setenv("FPSCHED_MB_GLOBAL", "1")
    spec = workloads.config(index, n)
    words = workloads.generate(spec, threads=8)
    table = scaled_table(spec.problem, np.random.default_rng(index))
    gpu, ref = check_batch(spec.problem, words, k=16, what=f"cfg{index}", dur_mb=table)
    assert (ref["flags"] == 0).sum() > 0
    # the table matters: the plain costs give other makespans
    plain = oracle.evaluate(spec.problem, words, threads=8)
    assert not np.array_equal(plain["makespan"], ref["makespan"])


@pytest.mark.parametrize("seed", range(6))
def test_random_problems_with_random_tables(seed, monkeypatch):
    if seed % 2:
        monkeypatch.setenv("FPSCHED_MB_GLOBAL", "1")
    rng = np.random.default_rng(7000 + seed)
    for i in range(10):
        prob = random_problem(rng)
        # small values travel as bytes, larger ones as sixteen-bit values
        table = rng.integers(0, 40 if i % 2 else 3000, (NKINDS, prob.n_stages, prob.n_microbatches)).astype(np.int32)
        if i % 3 == 0:
            table[[4, 7]] = table[1]   # kinds with equal costs share their part of the table
            table[[5, 6]] = 0
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
        check_batch(prob, batch_from_lists(lists), k=5, what=f"seed {seed} problem {i}", dur_mb=table)


def test_setting_clearing_and_replacing_the_table_on_one_handle():
    spec = workloads.config(2, 1500)
    prob, words = spec.problem, workloads.generate(spec, threads=8)
    ops = torch.from_numpy(words.view(np.int16)).cuda()
    rng = np.random.default_rng(3)
    first, second = scaled_table(prob, rng), scaled_table(prob, rng)
    constant = np.repeat(np.asarray(prob.dur, np.int32)[:, :, None], prob.n_microbatches, axis=2)
    h = fp.Problem(prob, spec.stride, device=0)

    def run():
        res = h.evaluate(ops)
        torch.cuda.synchronize()
        return {n: v.cpu().numpy() for n, v in res.items()}

    plain = oracle.evaluate(prob, words, threads=8)
    assert_same(run(), plain, "before any table")
    for name, table in (("first", first), ("second", second), ("constant", constant)):
        h.set_microbatch_costs(table)
        ref = plain if name == "constant" else oracle.evaluate(prob, words, threads=8, dur_mb=table)
        assert_same(run(), ref, name)
        # the sliding pass knows one cost per (type, stage) only
        with pytest.raises(fp.FpschedError) as e:
            h.wslide(ops)
        assert e.value.code == -6
    h.set_microbatch_costs(None)
    assert_same(run(), plain, "after clearing")
    out = h.wslide(ops)   # and the sliding pass is back
    torch.cuda.synchronize()
    ref = oracle.wslide(prob, words, spec.stride, threads=8)
    assert np.array_equal(out["makespan"].cpu().numpy(), ref["makespan"])
    # values the time bound refuses, and negative ones
    bad = first.copy()
    bad[1, 0, 0] = -1
    with pytest.raises(fp.FpschedError) as e:
        h.set_microbatch_costs(bad)
    assert e.value.code == -1
    bad[1, 0, 0] = 1 << 30
    with pytest.raises(fp.FpschedError) as e:
        h.set_microbatch_costs(bad)
    assert e.value.code == -4
    assert_same(run(), plain, "a refused table changes nothing")
    h.close()


def test_costs_too_large_for_the_slot_kernel_go_through_the_general_kernel():
    # times beyond 24 bits: the slot kernel keeps them << 8 in 32 bits, so the call falls back
    spec = workloads.config(1, 64)
    prob, words = spec.problem, workloads.generate(spec, threads=2)
    table = np.repeat(np.asarray(prob.dur, np.int32)[:, :, None], prob.n_microbatches, axis=2) * 40000
    table[2, 1, 3] += 12345
    gpu, ref = check_batch(prob, words, k=4, what="large costs", dur_mb=table, kernels=("auto",))
    assert ref["makespan"][ref["flags"] == 0].max() > 1 << 20


def test_largest_sizes_with_costs_per_micro_batch():
    from workloads.problem import gpipe_lists, one_f_one_b_lists, pack_lists, chain_problem
    rng = np.random.default_rng(2048)
    # the largest micro-batch count of the word format (a table of 2 x 2048 values per kind)
    m = 2048
    prob = chain_problem(2, m, f=1, b=2, comm=1)
    table = rng.integers(0, 30, (NKINDS, 2, m)).astype(np.int32)
    words = np.stack([pack_lists(one_f_one_b_lists(2, m), stride=4096), pack_lists(gpipe_lists(2, m), stride=4096)])
    check_batch(prob, words, k=2, what="m=2048", dur_mb=table)
    # 64 devices; 252 stages on 63 devices (the table does not fit LDS beside four chunks of state)
    prob = chain_problem(64, 6, f=2, b=4, comm=1)
    table = rng.integers(1, 300, (NKINDS, 64, 6)).astype(np.int32)
    words = np.stack([pack_lists(gpipe_lists(64, 6)), pack_lists(one_f_one_b_lists(64, 6))])
    check_batch(prob, words, k=2, what="p=64", dur_mb=table)
    prob = chain_problem(63, 3, v=4, f=2, b=3, w=1, comm=1)
    table = rng.integers(0, 20, (NKINDS, 252, 3)).astype(np.int32)
    lists = []
    for t in range(6):
        base = random_valid_lists(prob, rng)
        lists += [base, perturb(base, rng, 2)]
    check_batch(prob, batch_from_lists(lists), k=3, what="S=252", dur_mb=table)


def test_costs_beyond_sixteen_bits_use_the_table_in_device_memory():
    # values that fit the slot kernel's times but not the LDS table's sixteen bits
    from workloads.problem import chain_problem, gpipe_lists, one_f_one_b_lists, pack_lists
    prob = chain_problem(2, 4, f=1, b=1, w=1, comm=1)
    rng = np.random.default_rng(70000)
    table = rng.integers(60000, 90000, (NKINDS, 2, 4)).astype(np.int32)
    lists = [one_f_one_b_lists(2, 4), gpipe_lists(2, 4)]
    with_w = [[[op for x in row for op in ([x, (3, x[1], x[2])] if x[0] == 2 else [x])] for row in l] for l in lists]
    words = np.stack([pack_lists(l, stride=16) for l in with_w])
    gpu, ref = check_batch(prob, words, k=2, what="costs of 17 bits", dur_mb=table)
    assert (ref["flags"] == 0).all() and ref["makespan"].min() > 60000 * 8
