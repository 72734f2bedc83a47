"""fpsched_evaluate_topk_static: the entry point for callers that cannot allocate.  It must give what
fpsched_evaluate + fpsched_topk give on the same inputs, bit for bit, on calls in a row that share the
library's static scratch memory (the second on a smaller input), and it must refuse batches beyond it."""
import numpy as np
import pytest
import torch

import paper_2510_05112_amd as fp
import workloads

pytestmark = pytest.mark.gpu


def _top(k):
    return dict(idx=torch.empty(k, dtype=torch.int64, device="cuda"),
                makespan=torch.empty(k, dtype=torch.int64, device="cuda"),
                count=torch.empty(1, dtype=torch.int32, device="cuda"))


def test_static_scratch_entry_point_equals_evaluate_plus_topk_on_two_calls_in_a_row():
    lib = fp.load_library()
    assert lib.fpsched_static_scratch_bytes() == 2 << 20
    # first call: configuration 5 (two-tower DAG, deadlocking candidates), second: a smaller batch of
    # another problem, so that stale keys and a stale counter of the first call would show
    calls = [(5, 6151, 64), (2, 1031, 16), (2, 7, 5)]
    for index, n, k in calls:
        spec = workloads.config(index, n)
        words = workloads.generate(spec, threads=8)
        h = fp.Problem(spec.problem, spec.stride, device=0)
        ops = torch.from_numpy(words.view(np.int16)).cuda()
        # the existing entry points, with a caller's workspace
        ref = h.evaluate(ops)
        ref_top = h.topk(ref, k)
        torch.cuda.synchronize()
        res, top = h.alloc_results(n), _top(k)
        for t in list(res.values()) + list(top.values()):
            t.fill_(-7 if t.dtype != torch.uint8 else 0xaa)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        h.evaluate_topk_static(ops, k, res, top)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        for name in ("makespan", "idle", "peak", "flags"):
            assert torch.equal(res[name], ref[name]), (index, name)
        for name in ("idx", "makespan", "count"):
            assert torch.equal(top[name], ref_top[name]), (index, name)
        assert int(top["count"].item()) > 0
        h.close()


def test_static_scratch_entry_point_refuses_what_does_not_fit_and_bad_arguments():
    lib = fp.load_library()
    spec = workloads.config(1, 16)
    words = workloads.generate(spec, threads=2)
    h = fp.Problem(spec.problem, spec.stride, device=0)
    ops = torch.from_numpy(words.view(np.int16)).cuda()
    res, top = h.alloc_results(len(words)), _top(1024)
    none = fp.binding._Results(0, 0, 0, 0)
    # beyond the array: refused before anything is looked at or enqueued
    assert lib.fpsched_evaluate_topk_static(h._h, 0, 174080, spec.stride, none, 1024, 0, 0, 0, 0) == -7
    assert lib.fpsched_strerror(-7).decode().startswith("batch too large")
    assert lib.fpsched_evaluate_topk_static(h._h, ops.data_ptr(), len(words), spec.stride, none, 4, 1, 1, 1, 0) == -1
    assert lib.fpsched_evaluate_topk_static(h._h, ops.data_ptr(), len(words), spec.stride, h._res_struct(res), 0,
                                            top["idx"].data_ptr(), top["makespan"].data_ptr(),
                                            top["count"].data_ptr(), 0) == -1
    assert lib.fpsched_evaluate_topk_static(None, 0, 1, 8, none, 1, 1, 1, 1, 0) == -1
    host = fp.Problem(spec.problem, spec.stride, device=None)
    assert lib.fpsched_evaluate_topk_static(host._h, 0, 1, spec.stride, none, 1, 1, 1, 1, 0) == -5
    # an empty batch: no candidates, the top-k slots are the unused ones
    empty = torch.empty((0, spec.problem.n_devices, spec.stride), dtype=torch.int16, device="cuda")
    h.evaluate_topk_static(empty, 3, h.alloc_results(0), top)
    torch.cuda.synchronize()
    assert int(top["count"].item()) == 0 and top["idx"][:3].tolist() == [-1, -1, -1]
    # k = 1024 on a small batch still fits
    h.evaluate_topk_static(ops, 1024, res, top)
    ref = h.evaluate(ops)
    ref_top = h.topk(ref, 1024)
    torch.cuda.synchronize()
    assert torch.equal(top["idx"], ref_top["idx"]) and torch.equal(top["makespan"], ref_top["makespan"])
    h.close()
    host.close()
