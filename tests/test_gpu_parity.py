"""GPU parity: the HIP path, called through the C ABI, must equal the CPU oracle bit for bit."""
import numpy as np
import pytest

import oracle
import workloads
import paper_2510_05112_amd as fp
import torch
from gpu_common import assert_same, check_batch, gpu_evaluate
from helpers import batch_from_lists, dag_problem, perturb, random_valid_lists, two_tower_problem
from workloads.problem import (B, F, FD, L, O, R, W, chain_problem, gpipe_lists, make_problem,
                               one_f_one_b_lists, pack_lists, pack_word)

pytestmark = pytest.mark.gpu


def test_config1_all_candidates_and_fixed_cases():
    spec = workloads.config(1)
    words = workloads.generate(spec, threads=4)
    assert len(words) == 1026
    gpu, ref = check_batch(spec.problem, words, k=spec.top_k, what="cfg1")
    # the appended textbook orders: GPipe 72, 1F1B 82 at comm 1
    assert gpu["makespan"][1024] == 72 and list(gpu["idle"][1024]) == [24] * 4
    assert gpu["makespan"][1025] == 82 and list(gpu["peak"][1025]) == [4, 3, 2, 1]


@pytest.mark.parametrize("index,n", [(2, 3001), (3, 1027), (4, 300), (5, 2051)])
def test_configs_reduced_batches(index, n):
    spec = workloads.config(index, n)
    words = workloads.generate(spec, threads=8)
    gpu, ref = check_batch(spec.problem, words, k=spec.top_k, what=f"cfg{index}")
    if spec.deadlock_per_mille:
        assert (ref["flags"] & oracle.FLAG_DEADLOCK).sum() > 0
    assert (ref["flags"] == 0).sum() > 0 and (ref["flags"] == oracle.FLAG_OVER_CAP).sum() > 0


@pytest.mark.parametrize("p,m,v,w", [(3, 5, 1, None), (5, 4, 2, 2), (6, 3, 1, 1), (2, 6, 4, 1), (1, 7, 3, 2),
                                     (7, 2, 1, None), (12, 3, 1, 2)])
def test_random_orders_non_power_of_two_devices(p, m, v, w):
    rng = np.random.default_rng(p * 1000 + m * 10 + v)
    S = p * v
    prob = chain_problem(p, m, v=v, f=1, b=1, w=w, comm=0)
    prob.dur[F] = rng.integers(0, 9, S)
    prob.dur[FD] = prob.dur[F]
    prob.dur[R] = rng.integers(0, 9, S)
    prob.dur[B] = rng.integers(1, 15, S)
    prob.dur[O] = rng.integers(1, 6, S)
    prob.dur[L] = rng.integers(1, 6, S)
    if w is not None:
        prob.dur[W] = rng.integers(0, 7, S)
    prob.edge_comm[:] = rng.integers(0, 5, len(prob.edge_comm))
    prob.mem_units[:] = rng.integers(0, 4, S)
    prob.mem_cap[:] = rng.integers(2 * m * v, 8 * m * v, p)
    lists = []
    for t in range(150):
        base = random_valid_lists(prob, rng, 0.3 * (t % 2), 0.3 * ((t // 2) % 2))
        lists.append(base)
        lists.append(perturb(base, rng, 1 + t % 3))
        cut = [list(x) for x in base]
        d = int(rng.integers(p))
        if cut[d]:
            cut[d].pop(int(rng.integers(len(cut[d]))))
        lists.append(cut)
    words = batch_from_lists(lists)
    gpu, ref = check_batch(prob, words, k=7, what=f"random p{p}")
    assert (ref["flags"] & 1).sum() > 0 and ((ref["flags"] & 3) == 0).sum() > 0


def test_random_dag():
    rng = np.random.default_rng(42)
    for has_w in (0, 1):
        prob = two_tower_problem(m=5, has_w=has_w, comm=2, mem_cap=3)
        lists = []
        for t in range(120):
            base = random_valid_lists(prob, rng, 0.2, 0.3)
            lists += [base, perturb(base, rng, 2)]
        check_batch(prob, batch_from_lists(lists), k=33, what="dag")


DAGS = {
    # diamond: one stage feeds two, which merge again (two outputs and two inputs)
    "diamond": dict(edges=[(0, 1), (0, 2), (1, 3), (2, 3), (3, 4)], S=5, dev=[0, 1, 2, 3, 4], D=5),
    # diamond with two stages sharing a device and a chain in front
    "diamond_shared": dict(edges=[(0, 1), (1, 2), (1, 3), (2, 4), (3, 4)], S=5, dev=[0, 1, 2, 2, 0], D=3),
    # two independent pipelines on interleaved devices (two sources, two sinks)
    "two_chains": dict(edges=[(0, 1), (1, 2), (3, 4), (4, 5)], S=6, dev=[0, 1, 2, 2, 1, 0], D=3),
    # three towers into one stage: more inputs than the slot kernel takes -> table kernel only
    "three_towers": dict(edges=[(0, 3), (1, 3), (2, 3), (3, 4)], S=5, dev=[0, 1, 2, 3, 4], D=5),
    # a single stage, no edges
    "single": dict(edges=[], S=1, dev=[0], D=1),
}


@pytest.mark.parametrize("name", sorted(DAGS))
@pytest.mark.parametrize("has_w", [0, 1])
def test_stage_dags(name, has_w):
    g = DAGS[name]
    rng = np.random.default_rng(len(name) * 7 + has_w)
    prob = dag_problem(g["edges"], g["S"], g["dev"], g["D"], m=5, has_w=has_w,
                       mem_cap=rng.integers(4, 30, g["D"]), seed=len(name))
    lists = []
    for t in range(100):
        base = random_valid_lists(prob, rng, 0.25 * (t % 2), 0.25 * ((t // 2) % 2))
        lists += [base, perturb(base, rng, 1 + t % 2)]
    gpu, ref = check_batch(prob, batch_from_lists(lists), k=9, what=name)
    assert ((ref["flags"] & 3) == 0).sum() >= 100


def test_edge_cases_flags_and_sentinels():
    prob = chain_problem(2, 2, f=1, b=1, comm=0, mem_cap=1)
    ok = gpipe_lists(2, 2)
    cases = [
        ok,                                                              # over cap
        [[(B, 0, 0), (F, 0, 0), (F, 0, 1), (B, 0, 1)], ok[1]],           # same-device deadlock
        [[(F, 0, 0), (B, 0, 0), (F, 0, 1), (B, 0, 1)], [(F, 0, 1), (F, 0, 0), (B, 0, 1), (B, 0, 0)]],  # cycle
        [[(F, 0, 0), (F, 0, 0), (B, 0, 0), (B, 0, 1)], ok[1]],           # duplicate
        [[(F, 0, 0), (B, 0, 0)], [(F, 0, 0), (B, 0, 0)]],                # micro-batch missing
        [[], []],                                                        # empty
        [[(F, 1, 0)], []],                                               # bad chunk
        [[(F, 0, 5)], []],                                               # bad micro-batch
        [ok[0] + [(W, 0, 0)], ok[1]],                                    # W without split backward
        [[(B, 0, 0), (F, 1, 0)], ok[1]],                                 # malformed behind a deadlock
        [[(F, 0, 0), (F, 0, 1), (B, 0, 0)], ok[1]],                      # one op missing
        [[(F, 0, 0), (F, 0, 1), (B, 0, 1), (B, 0, 0)]] * 2,              # unusual but valid
    ]
    words = batch_from_lists(cases, stride=8)
    words[0, 0, 5] = pack_word(F, 3, 77)   # behind the END word: ignored
    gpu, ref = check_batch(prob, words, k=4, what="edge")
    assert list(ref["flags"]) == [4, 1, 1, 1, 2, 2, 3, 3, 3, 1, 2, 4]


def test_end_words_with_low_bits_set():
    # kind 0 ends a list whatever its chunk and micro-batch bits say
    p, m = 3, 5
    prob = chain_problem(p, m, f=2, b=3, comm=1)
    base = batch_from_lists([gpipe_lists(p, m), one_f_one_b_lists(p, m)], stride=24)
    words = np.concatenate([base, base, base])
    words[2:4][words[2:4] == 0] = 0x0005          # terminators and padding of kind 0, mb 5
    words[4:6][words[4:6] == 0] = 0x1fff          # kind 0 with every other bit set
    words[5, 1, 3] = 0x0802                       # cuts device 1 short: incomplete, not a deadlock
    gpu, ref = check_batch(prob, words, k=4, what="end words")
    assert list(ref["flags"][:5]) == [0] * 5 and ref["flags"][5] != 0
    assert np.array_equal(ref["makespan"][:2], ref["makespan"][2:4])


@pytest.mark.parametrize("units,slots_fit", [
    ([1000, 3000, 2000], True),      # common divisor 1000
    ([768, 1536, 1536], True),
    ([7, 300, 5], False),            # no common divisor and a unit beyond a byte
    ([255, 1, 17], True),
])
def test_large_memory_units(units, slots_fit):
    # the slot kernel carries units / gcd in a byte; anything else falls to the general kernel
    p, m = 3, 6
    edges = [(s, s + 1, 2) for s in range(p - 1)]
    dur = {F: [2, 3, 2], FD: [2, 3, 2], R: [2, 3, 2], B: [4, 5, 3], W: [1, 2, 1], O: 2, L: 2}
    cap = [int(u * 5.5) for u in units]   # not a multiple of the divisor: the cap rounds down
    prob = make_problem(p, p, m, 1, list(range(p)), edges, dur, mem_units=units, mem_cap=cap, name="units")
    rng = np.random.default_rng(5)
    lists = [random_valid_lists(prob, rng, 0.3 * (t % 2), 0.3 * ((t // 2) % 2)) for t in range(64)]
    words = batch_from_lists(lists)
    g, _ = gpu_evaluate(prob, words, kernel="slots")
    assert (g is not None) == slots_fit
    gpu, ref = check_batch(prob, words, k=5, what=f"units {units}")
    assert (ref["flags"] == 4).any() and (ref["flags"] == 0).any()
    assert ref["peak"].max() > 255


def test_empty_batch_single_candidate_and_ragged_tail():
    spec = workloads.config(2, 64)
    words = workloads.generate(spec, threads=2)
    gpu, top = gpu_evaluate(spec.problem, words[:0], k=5)
    assert top[2] == 0 and np.all(top[0] == -1) and np.all(top[1] == oracle.INT64_MAX)
    for n in (1, 7, 9, 63):
        check_batch(spec.problem, words[:n], k=3, what=f"n={n}")


def test_full_row_without_end_word_and_max_microbatches():
    # every row exactly fills the stride (no END word): the row length bounds the list
    p, m = 2, 4
    prob = chain_problem(p, m, f=2, b=3, comm=1)
    words = pack_lists(gpipe_lists(p, m), stride=8)[None]
    assert np.all(words >> 13 != 0)
    check_batch(prob, words, k=1, what="full row")
    # the largest micro-batch count of the word format on a tiny pipeline
    m = 2048
    prob = chain_problem(2, m, f=1, b=2, comm=1)
    lists = one_f_one_b_lists(2, m)
    words = np.stack([pack_lists(lists, stride=4096), pack_lists(gpipe_lists(2, m), stride=4096)])
    gpu, ref = check_batch(prob, words, k=2, what="m=2048")
    assert gpu["makespan"][1] == (m + 1) * 3 + 2


def test_sixty_four_devices():
    p, m = 64, 6
    prob = chain_problem(p, m, f=2, b=4, comm=1)
    words = np.stack([pack_lists(gpipe_lists(p, m)), pack_lists(one_f_one_b_lists(p, m))])
    gpu, ref = check_batch(prob, words, k=2, what="p=64")
    assert gpu["makespan"][0] == (m + p - 1) * 6 + 2 * (p - 1)


def test_topk_many_ties_and_large_k():
    # config 1 has only a handful of distinct makespans: ties everywhere
    spec = workloads.config(1, 5000)
    words = workloads.generate(spec, threads=4)
    for k in (1, 16, 128, 1000, 1024):
        check_batch(spec.problem, words, k=k, what=f"ties k={k}")


def test_call_errors_streams_and_workspace_reuse():
    import torch

    import paper_2510_05112_amd as fp
    spec = workloads.config(2, 700)
    words = workloads.generate(spec, threads=4)
    ref = oracle.evaluate(spec.problem, words, threads=4)
    h = fp.Problem(spec.problem, spec.stride, device=0)
    ops = torch.from_numpy(words.view(np.int16)).cuda()
    res = h.alloc_results(len(words))
    ws = h.alloc_workspace(len(words), 16)
    lib = fp.load_library()
    R = fp.binding._Results(res["makespan"].data_ptr(), res["idle"].data_ptr(), res["peak"].data_ptr(),
                            res["flags"].data_ptr())
    ev = lambda ops_ptr, n, stride, ws_ptr, ws_bytes: lib.fpsched_evaluate(  # noqa: E731
        h._h, ops_ptr, n, stride, R, ws_ptr, ws_bytes, 0)
    assert ev(ops.data_ptr(), len(words), spec.stride, ws.data_ptr(), 8) == -2          # workspace too small
    assert ev(ops.data_ptr(), len(words), spec.stride, 0, 0) == -1                      # no workspace
    assert ev(ops.data_ptr() + 2, len(words), spec.stride, ws.data_ptr(), ws.numel()) == -1   # misaligned ops
    assert ev(ops.data_ptr(), len(words), spec.stride + 8, ws.data_ptr(), ws.numel()) == -1   # stride > max
    assert ev(ops.data_ptr(), len(words), 12, ws.data_ptr(), ws.numel()) == -1          # stride not a multiple of 8
    assert ev(0, len(words), spec.stride, ws.data_ptr(), ws.numel()) == -1              # null ops
    assert ev(ops.data_ptr(), -1, spec.stride, ws.data_ptr(), ws.numel()) == -1
    out = dict(idx=torch.empty(16, dtype=torch.int64, device="cuda"),
               makespan=torch.empty(16, dtype=torch.int64, device="cuda"),
               count=torch.empty(1, dtype=torch.int32, device="cuda"))
    tk = lambda k, ws_bytes: lib.fpsched_topk(h._h, R, len(words), k, out["idx"].data_ptr(),  # noqa: E731
                                              out["makespan"].data_ptr(), out["count"].data_ptr(),
                                              ws.data_ptr(), ws_bytes, 0)
    assert tk(0, ws.numel()) == -1 and tk(1025, ws.numel()) == -1 and tk(16, 64) == -2
    # a side stream, the same workspace for evaluate and top-k, several times in a row
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    idx, ms, cnt = oracle.topk(ref["makespan"], ref["flags"], 16)
    for rep in range(3):
        for t in res.values():
            t.zero_()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            h.evaluate(ops, res, ws, stream=side)
            top = h.topk(res, 16, ws, out, stream=side)
        side.synchronize()
        for name in ("makespan", "idle", "peak", "flags"):
            assert np.array_equal(res[name].cpu().numpy(), ref[name]), (rep, name)
        assert int(top["count"].item()) == cnt and np.array_equal(top["idx"].cpu().numpy(), idx)
    h.close()


@pytest.mark.parametrize("model", ["plain", "costs per micro-batch", "link occupancy"])
def test_evaluate_and_topk_replayed_from_a_hip_graph(model):
    # the calls enqueue kernels only (the work counter is reset by a kernel, not a memset), so they can
    # be captured once and replayed on new inputs; every replay is checked against the oracle
    import torch

    import paper_2510_05112_amd as fp
    spec = workloads.config(2, 300)
    prob, k = spec.problem, 9
    batches = [workloads.generate(spec, n=300, first=300 * i, threads=2) for i in range(3)]
    h = fp.Problem(prob, spec.stride, device=0)
    variant = {}
    if model == "costs per micro-batch":
        variant["dur_mb"] = workloads.microbatch_costs(prob)
        h.set_microbatch_costs(variant["dur_mb"])
    elif model == "link occupancy":
        variant["links"] = True
        h.set_link_occupancy(True)
    ops = torch.from_numpy(batches[0].view(np.int16)).cuda()
    res, ws = h.alloc_results(300), h.alloc_workspace(300, k)
    top = dict(idx=torch.empty(k, dtype=torch.int64, device="cuda"),
               makespan=torch.empty(k, dtype=torch.int64, device="cuda"),
               count=torch.empty(1, dtype=torch.int32, device="cuda"))
    h.evaluate(ops, res, ws)          # eager once (warm-up outside the capture)
    h.topk(res, k, ws, top)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        h.evaluate(ops, res, ws)
        h.topk(res, k, ws, top)
    for words in batches[::-1] + batches:
        ops.copy_(torch.from_numpy(words.view(np.int16)))
        res["flags"].fill_(255)       # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        ref = oracle.evaluate(prob, words, threads=2, **variant)
        for name in ("makespan", "idle", "peak", "flags"):
            assert np.array_equal(res[name].cpu().numpy(), ref[name]), name
        idx, ms, cnt = oracle.topk(ref["makespan"], ref["flags"], k)
        assert int(top["count"].item()) == cnt and np.array_equal(top["idx"].cpu().numpy(), idx)
    h.close()


@pytest.mark.parametrize("links", [False, True])
def test_generate_slide_and_topk_replayed_from_a_hip_graph(links):
    # the search loop with the sliding pass, captured once and replayed on new parameter sets; every
    # replay is checked against the three oracles
    import torch

    import paper_2510_05112_amd as fp
    spec = workloads.config(2, 8)
    prob, k, n = spec.problem, 5, 160
    st = workloads.generator_stride(prob)
    sets = [workloads.policy_sets(prob, n, seed=77 + i) for i in range(3)]
    h = fp.Problem(prob, st, device=0)
    if links:
        h.set_link_occupancy(True)
    d_pol, d_inf = torch.from_numpy(sets[0][0]).cuda(), torch.from_numpy(sets[0][1]).cuda()
    gen = h.generate(d_pol, d_inf, st)                      # eager once: allocates the outputs
    ws = h.alloc_workspace(n, k)
    slide_ws = torch.empty(int(fp.load_library().fpsched_wslide_workspace_bytes(h._h, n, st)), dtype=torch.uint8,
                           device="cuda")
    slid = h.wslide(gen["ops"], st, workspace=slide_ws)
    top = h.topk(slid, k, ws)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        h.generate(d_pol, d_inf, st, out=gen, workspace=ws)
        h.wslide(gen["ops"], st, out=slid, workspace=slide_ws)
        h.topk(slid, k, ws, top)
    for pol, inf in sets[::-1] + sets:
        d_pol.copy_(torch.from_numpy(pol))
        d_inf.copy_(torch.from_numpy(inf))
        slid["flags"].fill_(255)      # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        ref_gen = oracle.generate(prob, pol, inf, st, threads=2)
        assert np.array_equal(gen["ops"].cpu().numpy().view(np.uint16), ref_gen["words"])
        ref = oracle.wslide(prob, ref_gen["words"], st, threads=2, links=links)
        assert np.array_equal(slid["ops"].cpu().numpy().view(np.uint16), ref["ops"])
        for name in ("makespan", "idle", "peak", "flags"):
            assert np.array_equal(slid[name].cpu().numpy(), ref[name]), name
        idx, ms, cnt = oracle.topk(ref["makespan"], ref["flags"], k)
        assert int(top["count"].item()) == cnt and np.array_equal(top["idx"].cpu().numpy(), idx)
    h.close()


def test_fused_search_step_replayed_from_a_hip_graph():
    # generate-and-time, top-k and the winners' rows, captured once and replayed on new parameter sets;
    # every replay is checked against the two oracles composed on the CPU
    import torch

    import paper_2510_05112_amd as fp
    spec = workloads.config(2, 8)
    prob, k, n = spec.problem, 5, 160
    st = workloads.generator_stride(prob)
    sets = [workloads.policy_sets(prob, n, seed=91 + i) for i in range(3)]
    h = fp.Problem(prob, st, device=0)
    d_pol, d_inf = torch.from_numpy(sets[0][0]).cuda(), torch.from_numpy(sets[0][1]).cuda()
    ws = h.alloc_workspace(n, k)
    res, out = h.generate_evaluate(d_pol, d_inf, workspace=ws)     # eager once: allocates the outputs
    top = h.topk(res, k, ws)
    rows = h.generate_selected(d_pol, d_inf, top["idx"], st, workspace=ws)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        h.generate_evaluate(d_pol, d_inf, results=res, out=out, workspace=ws)
        h.topk(res, k, ws, top)
        h.generate_selected(d_pol, d_inf, top["idx"], st, out=rows, workspace=ws)
    for pol, inf in sets[::-1] + sets:
        d_pol.copy_(torch.from_numpy(pol))
        d_inf.copy_(torch.from_numpy(inf))
        res["flags"].fill_(255)       # eager work between the replays
        rows["ops"].zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        ref_gen = oracle.generate(prob, pol, inf, st, threads=2)
        ref = oracle.evaluate(prob, ref_gen["words"], threads=2)
        for name in ("makespan", "idle", "peak", "flags"):
            assert np.array_equal(res[name].cpu().numpy(), ref[name]), name
        assert np.array_equal(out["steps"].cpu().numpy(), ref_gen["steps"])
        idx, ms, cnt = oracle.topk(ref["makespan"], ref["flags"], k)
        assert int(top["count"].item()) == cnt == k and np.array_equal(top["idx"].cpu().numpy(), idx)
        assert np.array_equal(rows["ops"].cpu().numpy().view(np.uint16), ref_gen["words"][idx])
    h.close()


def test_search_steps_with_the_sliding_pass_replayed_from_a_hip_graph():
    # the one-kernel forms of the sliding pass -- inside the generator kernel, and on generated lists -- with top-k,
    # the winners' rows and their slid lists, captured once and replayed on new parameter sets; every replay is
    # checked against the generator oracle and the sliding oracle composed on the CPU
    import torch

    import paper_2510_05112_amd as fp
    spec = workloads.config(2, 8)
    prob, k, n = spec.problem, 5, 160
    st = workloads.generator_stride(prob)
    sets = [workloads.policy_sets(prob, n, seed=191 + i) for i in range(3)]
    h = fp.Problem(prob, st, device=0)
    d_pol, d_inf = torch.from_numpy(sets[0][0]).cuda(), torch.from_numpy(sets[0][1]).cuda()
    ws = h.alloc_workspace(n, k)
    res, out = h.generate_evaluate(d_pol, d_inf, workspace=ws, slide=True)     # eager once: allocates the outputs
    top = h.topk(res, k, ws)
    rows = h.generate_selected(d_pol, d_inf, top["idx"], st, workspace=ws)
    slide_ws = torch.empty(int(fp.load_library().fpsched_wslide_workspace_bytes(h._h, k, st)), dtype=torch.uint8,
                           device="cuda")
    slid = h.wslide(rows["ops"], st, workspace=slide_ws)
    gen = h.generate(d_pol, d_inf, st, workspace=ws)
    again = h.wslide_evaluate(gen["ops"], workspace=ws)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        h.generate_evaluate(d_pol, d_inf, results=res, out=out, workspace=ws, slide=True)
        h.topk(res, k, ws, top)
        h.generate_selected(d_pol, d_inf, top["idx"], st, out=rows, workspace=ws)
        h.wslide(rows["ops"], st, out=slid, workspace=slide_ws)
        h.generate(d_pol, d_inf, st, out=gen, workspace=ws)
        h.wslide_evaluate(gen["ops"], out=again, workspace=ws)
    for pol, inf in sets[::-1] + sets:
        d_pol.copy_(torch.from_numpy(pol))
        d_inf.copy_(torch.from_numpy(inf))
        res["flags"].fill_(255)       # eager work between the replays
        again["flags"].fill_(255)
        slid["ops"].zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        ref_gen = oracle.generate(prob, pol, inf, st, threads=2)
        ref = oracle.wslide(prob, ref_gen["words"], st, threads=2)
        for name in ("makespan", "idle", "peak", "flags"):
            assert np.array_equal(res[name].cpu().numpy(), ref[name]), name
            assert np.array_equal(again[name].cpu().numpy(), ref[name]), name
        assert np.array_equal(out["steps"].cpu().numpy(), ref_gen["steps"])
        idx, ms, cnt = oracle.topk(ref["makespan"], ref["flags"], k)
        assert int(top["count"].item()) == cnt == k and np.array_equal(top["idx"].cpu().numpy(), idx)
        assert np.array_equal(slid["ops"].cpu().numpy().view(np.uint16), ref["ops"][idx])
        assert np.array_equal(slid["makespan"].cpu().numpy(), ref["makespan"][idx])
    h.close()


def test_copy_engine_evaluation_replayed_from_a_hip_graph():
    import torch

    import paper_2510_05112_amd as fp
    spec = workloads.config(5, 300)
    prob, k = spec.problem, 9
    batches = [workloads.generate(spec, n=300, first=300 * i, threads=2) for i in range(3)]
    h = fp.Problem(prob, spec.stride, device=0)
    h.set_copy_engine(3)
    ops = torch.from_numpy(batches[0].view(np.int16)).cuda()
    res, ws = h.alloc_results(300), h.alloc_workspace(300, k)
    top = h.topk(h.evaluate(ops, res, ws), k, ws)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        h.evaluate(ops, res, ws)
        h.topk(res, k, ws, top)
    for words in batches[::-1] + batches:
        ops.copy_(torch.from_numpy(words.view(np.int16)))
        res["flags"].fill_(255)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        ref = oracle.evaluate_copy(prob, words, depth=3, threads=2)
        for name in ("makespan", "idle", "peak", "flags"):
            assert np.array_equal(res[name].cpu().numpy(), ref[name]), name
        idx, ms, cnt = oracle.topk(ref["makespan"], ref["flags"], k)
        assert int(top["count"].item()) == cnt and np.array_equal(top["idx"].cpu().numpy(), idx)
    h.close()


def test_two_live_handles_with_different_lds_needs():
    # The dynamic-LDS limit of a kernel is one value per process: a handle created later with a smaller
    # need must not take the room of an earlier one (both problems run the same kernel instantiation).
    big, small = workloads.config(4, 64), workloads.config(2, 64)
    w_big, w_small = workloads.generate(big, threads=4), workloads.generate(small, threads=4)
    h_big = fp.Problem(big.problem, big.stride, device=0)
    h_small = fp.Problem(small.problem, small.stride, device=0)       # created second, needs less LDS
    assert h_big.info()["lds_bytes_per_wave"] > h_small.info()["lds_bytes_per_wave"]
    for h, spec, words in ((h_big, big, w_big), (h_small, small, w_small), (h_big, big, w_big)):
        for links in (False, True):
            h.set_link_occupancy(links)
            res = h.evaluate(torch.from_numpy(words.view(np.int16)).cuda())
            torch.cuda.synchronize()
            ref = oracle.evaluate(spec.problem, words, threads=4, links=links)
            assert_same({n: v.cpu().numpy() for n, v in res.items()}, ref, f"{spec.problem.name} links={links}")
    out = h_big.wslide(torch.from_numpy(w_big.view(np.int16)).cuda(), big.stride)   # links still on
    torch.cuda.synchronize()
    ref = oracle.wslide(big.problem, w_big, big.stride, threads=4, links=True)
    assert np.array_equal(out["ops"].cpu().numpy().view(np.uint16), ref["ops"])
    h_big.close()
    h_small.close()


def test_largest_stage_counts():
    # 252 stages (tags up to 251 in the slot kernel) and 256 stages (beyond its 8-bit tags: the
    # general kernel takes over)
    for p, v in ((63, 4), (64, 4)):
        prob = chain_problem(p, 3, v=v, f=2, b=3, w=1, comm=1)
        rng = np.random.default_rng(p)
        lists = []
        for t in range(6):
            base = random_valid_lists(prob, rng)
            lists += [base, perturb(base, rng, 2)]
        words = batch_from_lists(lists)
        g, _ = gpu_evaluate(prob, words, kernel="slots")
        assert (g is not None) == (p * v <= 255)
        check_batch(prob, words, k=3, what=f"S={p * v}")
