"""GPU parity at the benchmark's full batch sizes, in the launch configuration bench.py times:
every candidate of every configuration against the oracle under each cost model, every candidate of
the sliding pass, 8,192 parameter sets of the generator (its oracle does some 300 per second), plus
properties that hold at any size."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_05112_amd as fp
import workloads

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("index", [1, 2, 5, 4, 3])
def test_full_batch_every_candidate_against_oracle(index):
    spec = workloads.config(index)
    prob = spec.problem
    words = workloads.generate(spec, threads=16)
    C, D, stride = words.shape
    print(f"cfg{index}: {C} candidates, {words.nbytes / 1e9:.2f} GB", flush=True)
    h = fp.Problem(prob, stride, device=0)
    ops = torch.empty((C, D, stride), dtype=torch.int16, device="cuda")
    step = max(1, (256 << 20) // (D * stride * 2))
    for lo in range(0, C, step):
        ops[lo:lo + step].copy_(torch.from_numpy(words[lo:lo + step].view(np.int16)))
    ws = h.alloc_workspace(C, spec.top_k)
    res = h.evaluate(ops, workspace=ws)
    top = h.topk(res, spec.top_k, workspace=ws)
    torch.cuda.synchronize()
    g = {k: v.cpu().numpy() for k, v in res.items()}
    # every candidate of the batch against the oracle (16 host threads: seconds per configuration)
    ref = oracle.evaluate(prob, words, threads=16)
    for name in ("flags", "makespan", "idle", "peak"):
        assert np.array_equal(g[name], ref[name]), name
    r_idx, r_ms, r_cnt = oracle.topk(ref["makespan"], ref["flags"], spec.top_k)
    assert int(top["count"].item()) == r_cnt
    assert np.array_equal(top["idx"].cpu().numpy(), r_idx) and np.array_equal(top["makespan"].cpu().numpy(), r_ms)
    # properties at full size
    fl, ms = g["flags"], g["makespan"]
    assert np.all(np.isin(fl, [0, 1, 3, 2, 4]))
    good = (fl & 3) == 0
    assert np.all(ms[~good] == oracle.INT64_MAX) and np.all(g["idle"][~good] == -1) and np.all(g["peak"][~good] == -1)
    assert np.all(g["idle"][good] >= 0)
    assert np.all(g["idle"][good].max(1) <= ms[good])
    over = (g["peak"] > np.asarray(prob.mem_cap)[None, :]).any(1)
    assert np.array_equal(fl[good] == 4, over[good])
    # every row's busy time is order-independent for configs without optional ops; in all configs
    # idle + busy = makespan means idle differences between devices are makespan-independent
    # top-k: exactly the stable sort of the feasible candidates of the GPU's own results
    feas = np.flatnonzero(fl == 0)
    order = feas[np.argsort(ms[feas], kind="stable")][: spec.top_k]
    assert int(top["count"].item()) == len(order)
    assert np.array_equal(top["idx"].cpu().numpy()[: len(order)], order)
    assert np.array_equal(top["makespan"].cpu().numpy()[: len(order)], ms[order])
    # Pareto front of (makespan, largest peak): the staircase of the GPU's own results
    front = h.pareto(res, 1024)
    torch.cuda.synchronize()
    done = np.flatnonzero(good)
    mp = g["peak"][done].max(1).astype(np.int64)
    expect, best = [], np.iinfo(np.int64).max
    for i in np.lexsort((done, mp, ms[done])):
        if mp[i] < best:
            best = mp[i]
            expect.append((done[i], ms[done[i]], mp[i]))
    cnt = int(front["count"].item())
    assert cnt == min(1024, len(expect)) and cnt >= 1
    got = list(zip(front["idx"].cpu().numpy()[:cnt], front["makespan"].cpu().numpy()[:cnt],
                   front["peak"].cpu().numpy()[:cnt]))
    assert [tuple(int(x) for x in e) for e in got] == [tuple(int(x) for x in e) for e in expect[:cnt]]
    # the same batch under the other cost models (the launches `bench.py --mb-costs`, `--links` and both
    # together time): every candidate
    if index != 1:
        table = workloads.microbatch_costs(prob)
        for dur_mb, links, what in ((table, False, "costs per micro-batch"), (None, True, "link occupancy"),
                                    (table, True, "both variants")):
            h.set_microbatch_costs(dur_mb)
            h.set_link_occupancy(links)
            res = h.evaluate(ops, workspace=ws)
            top = h.topk(res, spec.top_k, workspace=ws)
            torch.cuda.synchronize()
            ref = oracle.evaluate(prob, words, threads=16, dur_mb=dur_mb, links=links)
            for name in ("flags", "makespan", "idle", "peak"):
                assert np.array_equal(res[name].cpu().numpy(), ref[name]), f"{what}: {name}"
            r_idx, r_ms, r_cnt = oracle.topk(ref["makespan"], ref["flags"], spec.top_k)
            assert int(top["count"].item()) == r_cnt and np.array_equal(top["idx"].cpu().numpy(), r_idx), what
            assert np.array_equal(top["makespan"].cpu().numpy(), r_ms), what
            print(f"cfg{index}: {what} ok", flush=True)
    h.close()


def test_generator_full_batch_8192_sets_against_oracle():
    # the generator at the size and launch configuration of `bench.py --mode generate`
    spec = workloads.config(4)
    prob = spec.problem
    n = spec.n_candidates
    pol, inf = workloads.policy_sets(prob, n)
    stride = workloads.generator_stride(prob)
    h = fp.Problem(prob, stride, device=0)
    d_pol, d_inf = torch.from_numpy(pol).cuda(), torch.from_numpy(inf).cuda()
    out = h.generate(d_pol, d_inf, stride)
    fused, fused_out = h.generate_evaluate(d_pol, d_inf)   # the same sets, timed while generated
    torch.cuda.synchronize()
    steps = out["steps"].cpu().numpy()
    status = out["status"].cpu().numpy()
    assert np.array_equal(fused_out["steps"].cpu().numpy(), steps) and not fused_out["status"].any()
    fused = {name: t.cpu().numpy() for name, t in fused.items()}
    rng = np.random.default_rng(4)
    pick = np.unique(np.concatenate([rng.choice(n, 8190, replace=False), [0, n - 1]]))
    for lo in range(0, len(pick), 2048):   # in pieces: the run prints its progress
        part = pick[lo:lo + 2048]
        ref = oracle.generate(prob, pol[part], inf[part], stride, threads=16)
        sel = torch.from_numpy(part).cuda()
        assert np.array_equal(out["ops"][sel].cpu().numpy().view(np.uint16), ref["words"])
        assert np.array_equal(steps[part], ref["steps"]) and np.array_equal(status[part], ref["status"])
        ref_ev = oracle.evaluate(prob, ref["words"], threads=16)
        for name in ("makespan", "idle", "peak", "flags"):
            assert np.array_equal(fused[name][part], ref_ev[name]), name
        print(f"generator: {lo + len(part)} of {len(pick)} sets ok", flush=True)
    # properties at full size: every process completes, every actor schedules each of its items once
    assert not status.any()
    per_dev = 2 * prob.n_microbatches * 3
    assert steps.min() >= per_dev and steps.max() <= 3 * prob.n_stages * prob.n_microbatches
    kinds = (out["ops"].view(torch.int16).to(torch.int32) & 0xffff) >> 13
    assert bool((kinds != 0).sum(dim=2).eq(per_dev).all())
    # and the evaluator accepts all of them
    res = h.evaluate(out["ops"])
    torch.cuda.synchronize()
    assert not bool((res["flags"] & 3).any())
    # ... with the results the fused kernel gave, for every one of the 65,536 sets
    for name in ("makespan", "idle", "peak", "flags"):
        assert np.array_equal(fused[name], res[name].cpu().numpy()), name
    h.close()


@pytest.mark.parametrize("links", [False, True])
def test_wslide_full_batch_every_candidate_against_oracle(links):
    """The sliding pass on configuration 4's full batch, in the launch configuration bench.py times, under
    both readings of a transfer (pure latency; links that carry one value at a time)."""
    spec = workloads.config(4)
    prob = spec.problem
    words = workloads.generate(spec, threads=16)
    C, D, stride = words.shape
    print(f"wslide cfg4: {C} candidates", flush=True)
    h = fp.Problem(prob, stride, device=0)
    h.set_link_occupancy(links)
    ops = torch.empty((C, D, stride), dtype=torch.int16, device="cuda")
    step = max(1, (256 << 20) // (D * stride * 2))
    for lo in range(0, C, step):
        ops[lo:lo + step].copy_(torch.from_numpy(words[lo:lo + step].view(np.int16)))
    out = h.wslide(ops, stride)
    torch.cuda.synchronize()
    # every candidate against the oracle, 8,192 at a time (new lists and their evaluation)
    for lo in range(0, C, 8192):
        ref = oracle.wslide(prob, words[lo:lo + 8192], stride, threads=16, links=links)
        assert np.array_equal(out["ops"][lo:lo + 8192].cpu().numpy().view(np.uint16), ref["ops"]), lo
        for name in ("makespan", "idle", "peak", "flags"):
            assert np.array_equal(out[name][lo:lo + 8192].cpu().numpy(), ref[name]), (name, lo)
        print(f"wslide links={links}: {min(C, lo + 8192)} of {C} candidates ok", flush=True)
    # the one-kernel form (no lists): the same results, for every candidate
    only = h.wslide_evaluate(ops)
    torch.cuda.synchronize()
    for name in ("makespan", "idle", "peak", "flags"):
        assert torch.equal(only[name], out[name]), name
    pick = np.arange(0, C, 1311)
    # at full size: the new lists, timed by the evaluation kernel, give the reported results
    again = h.evaluate(out["ops"])
    torch.cuda.synchronize()
    fl = out["flags"].cpu().numpy()
    ok = torch.from_numpy((fl & 3) == 0).cuda()
    assert int(ok.sum()) > C // 2
    for name in ("makespan", "idle", "peak", "flags"):
        assert torch.equal(again[name][ok], out[name][ok]), name
    # every new row holds the old row's items other than W in their old order
    new = out["ops"].cpu().numpy().view(np.uint16)
    for c in pick[:50]:
        for d in range(D):
            a, b = words[c, d], new[c, d]
            keep_a = a[((a >> 13) != 0) & ((a >> 13) != 3)]
            keep_b = b[((b >> 13) != 0) & ((b >> 13) != 3)]
            if (fl[c] & 3) == 0:
                assert np.array_equal(keep_a, keep_b)
    h.close()


def test_sync_workload_full_batch_every_candidate_against_oracle():
    """The multimodal workload with a registered synchronisation, in the launch `bench.py --mode sync` times."""
    spec = workloads.sync_config()
    words = workloads.generate_sync(spec, threads=16)
    C = len(words)
    h = fp.Problem(spec.problem, spec.stride, device=0)
    h.set_sync(spec.group, spec.pairs)
    ws = h.alloc_workspace(C, spec.top_k)
    res = h.evaluate(torch.from_numpy(words.view(np.int16)).cuda(), workspace=ws)
    top = h.topk(res, spec.top_k, workspace=ws)
    torch.cuda.synchronize()
    ref = oracle.evaluate_sync(spec.problem, words, spec.group, spec.pairs, threads=16)
    for name in ("flags", "makespan", "idle", "peak"):
        assert np.array_equal(res[name].cpu().numpy(), ref[name]), name
    r_idx, r_ms, r_cnt = oracle.topk(ref["makespan"], ref["flags"], spec.top_k)
    assert int(top["count"].item()) == r_cnt and np.array_equal(top["idx"].cpu().numpy(), r_idx)
    assert np.array_equal(top["makespan"].cpu().numpy(), r_ms)
    assert (ref["flags"] == 0).mean() > 0.3 and (ref["flags"] & 1).any()
    h.close()


def test_copy_engine_full_batch_every_candidate_against_oracle():
    """Configuration 5 (offload / reload items) under the copy-engine form, the launch
    `bench.py --config 5 --copy-engine 4` times."""
    spec = workloads.config(5)
    words = workloads.generate(spec, threads=16)
    C = len(words)
    h = fp.Problem(spec.problem, spec.stride, device=0)
    h.set_copy_engine(4)
    ws = h.alloc_workspace(C, spec.top_k)
    res = h.evaluate(torch.from_numpy(words.view(np.int16)).cuda(), workspace=ws)
    top = h.topk(res, spec.top_k, workspace=ws)
    torch.cuda.synchronize()
    ref = oracle.evaluate_copy(spec.problem, words, depth=4, threads=16)
    for name in ("flags", "makespan", "idle", "peak"):
        assert np.array_equal(res[name].cpu().numpy(), ref[name]), name
    r_idx, r_ms, r_cnt = oracle.topk(ref["makespan"], ref["flags"], spec.top_k)
    assert int(top["count"].item()) == r_cnt and np.array_equal(top["idx"].cpu().numpy(), r_idx)
    assert np.array_equal(top["makespan"].cpu().numpy(), r_ms)
    h.close()
