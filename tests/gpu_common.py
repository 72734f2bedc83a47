"""Shared plumbing of the GPU parity tests: run a batch through the C ABI and fetch numpy results."""
import numpy as np
import torch

import oracle
import paper_2510_05112_amd as fp


KERNELS = ("slots", "general")


def gpu_evaluate(problem, words, k=None, max_stride=None, kernel="auto", dur_mb=None, links=False):
    """words: uint16 [C][D][stride] (numpy).  Returns (results dict of numpy arrays, topk tuple or None).
    dur_mb[8][S][m]: costs per micro-batch, set on the handle before the batch is evaluated; links: the
    link-occupancy variant (a problem or kernel that has no such form gives (None, None))."""
    words = np.ascontiguousarray(words, dtype=np.uint16)
    C, D, stride = words.shape
    h = fp.Problem(problem, max_stride or stride, device=0)
    try:
        h.select_kernel(kernel)
    except fp.FpschedError as e:
        if e.code != -6:   # this kernel's on-chip tables do not fit the problem
            raise
        h.close()
        return None, None
    if dur_mb is not None:
        h.set_microbatch_costs(dur_mb)
    if links:
        try:
            if kernel == "general":
                raise fp.FpschedError(-6, "the general kernel has no link form")
            h.set_link_occupancy(True)
        except fp.FpschedError as e:
            if e.code != -6:
                raise
            h.close()
            return None, None
    ops = torch.from_numpy(words.view(np.int16)).cuda() if C else torch.empty((0, D, stride), dtype=torch.int16, device="cuda")
    res = h.evaluate(ops)
    top = None
    if k is not None:
        t = h.topk(res, k)
        torch.cuda.synchronize()
        top = (t["idx"].cpu().numpy(), t["makespan"].cpu().numpy(), int(t["count"].item()))
    torch.cuda.synchronize()
    out = {n: v.cpu().numpy() for n, v in res.items()}
    h.close()
    return out, top


def assert_same(gpu, ref, what=""):
    for name in ("flags", "makespan", "idle", "peak"):
        a, b = gpu[name], ref[name]
        if not np.array_equal(a, b):
            bad = np.flatnonzero((a != b).reshape(len(a), -1).any(1))
            raise AssertionError(f"{what}: {name} differs for {len(bad)} candidates, first {bad[:5]}: "
                                 f"gpu {a[bad[0]]} oracle {b[bad[0]]}")


def check_batch(problem, words, k=None, what="", threads=8, kernels=KERNELS, dur_mb=None, links=False):
    """Every kernel variant of the library against the oracle, element by element."""
    ref = oracle.evaluate(problem, words, threads=threads, dur_mb=dur_mb, links=links)
    gpu, ran = None, 0
    for kernel in kernels:
        g, top = gpu_evaluate(problem, words, k, kernel=kernel, dur_mb=dur_mb, links=links)
        if g is None:
            continue
        gpu, ran = g, ran + 1
        assert_same(gpu, ref, f"{what} [{kernel}]")
        if k is not None:
            idx, ms, cnt = oracle.topk(ref["makespan"], ref["flags"], k)
            assert top[2] == cnt, what
            assert np.array_equal(top[0], idx), what
            assert np.array_equal(top[1], ms), what
    assert ran > 0, f"{what}: no kernel variant supports this problem"
    return gpu, ref
