"""Host-side checks of libfpsched that need no GPU: the library loads, exports every symbol
the header declares, and its host helpers (create/encode/validate/strerror) behave."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2510_05112_amd as fp
import workloads
from workloads.problem import B, F, FD, R, W, chain_problem, pack_lists, pack_word

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_loads_and_exports_every_declared_symbol():
    lib = fp.load_library()
    header = open(os.path.join(ROOT, "include", "fpsched.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(fpsched_[a-z_]+)\s*\(", header))
    assert {"fpsched_evaluate", "fpsched_topk", "fpsched_problem_create", "fpsched_problem_destroy",
            "fpsched_workspace_bytes", "fpsched_encode", "fpsched_validate", "fpsched_strerror",
            "fpsched_version", "fpsched_problem_info", "fpsched_generate",
            "fpsched_problem_select_kernel", "fpsched_rank", "fpsched_rank_workspace_bytes",
            "fpsched_pareto", "fpsched_pareto_workspace_bytes", "fpsched_apply_caps", "fpsched_wslide", "fpsched_wslide_workspace_bytes",
            "fpsched_wslide_evaluate", "fpsched_generate_slide_evaluate"} <= names
    for n in names:
        assert hasattr(lib, n), n
    assert fp.version() == 100
    assert lib.fpsched_strerror(-4).decode().startswith("time bound")


def test_host_only_handle_and_errors():
    spec = workloads.config(2, 8)
    p = fp.Problem(spec.problem, spec.stride, device=None)
    info = p.info()
    assert info["lanes_per_candidate"] == 8 and info["candidates_per_wave"] == 8
    assert p.workspace_bytes(65536, 16) >= 16 * 16 * 32
    # device calls on a host-only handle are refused, not emulated
    lib = fp.load_library()
    rc = lib.fpsched_evaluate(p._h, 0, 1, spec.stride, fp.binding._Results(0, 0, 0, 0), 0, 0, 0)
    assert rc == -5
    assert lib.fpsched_generate(p._h, 0, 0, 1, 1024, 0, 0, 0, 0, 0, 0) == -5
    assert lib.fpsched_generate_selected(p._h, 0, 0, 4, 1, 1, 1024, 0, 0, 0, 0, 0, 0) == -5
    assert lib.fpsched_generate_evaluate(p._h, 0, 0, 1, fp.binding._Results(0, 0, 0, 0), 0, 0, 0, 0, 0) == -5
    assert lib.fpsched_generate_slide_evaluate(p._h, 0, 0, 1, fp.binding._Results(0, 0, 0, 0), 0, 0, 0, 0, 0) == -5
    assert lib.fpsched_generate_selected(p._h, 0, 0, -1, 1, 1, 1024, 0, 0, 0, 0, 0, 0) == -1   # a negative number of sets
    assert lib.fpsched_generate_selected(p._h, 0, 0, 4, 0, 1, 1024, 0, 0, 0, 0, 0, 0) == -1    # no selection given
    assert lib.fpsched_generate_evaluate(None, 0, 0, 1, fp.binding._Results(0, 0, 0, 0), 0, 0, 0, 0, 0) == -1
    assert lib.fpsched_generate_slide_evaluate(None, 0, 0, 1, fp.binding._Results(0, 0, 0, 0), 0, 0, 0, 0, 0) == -1
    none = fp.binding._Results(0, 0, 0, 0)
    assert lib.fpsched_topk(p._h, none, 1, 1, 1, 1, 1, 0, 0, 0) == -5
    assert lib.fpsched_rank(p._h, none, 1, 1, 0, 0, 1, 1, 1, 0, 0, 0) == -5
    assert lib.fpsched_pareto(p._h, none, 1, 1, 1, 1, 1, 1, 0, 0, 0) == -5
    assert lib.fpsched_apply_caps(p._h, 0, 1, 0, 1, 0, 0) == -5
    assert lib.fpsched_wslide(p._h, 0, 1, spec.stride, 0, spec.stride, none, 0, 0, 0) == -5
    assert lib.fpsched_wslide_evaluate(p._h, 0, 1, spec.stride, none, 0, 0, 0) == -5
    # the workspace sizes are host arithmetic and work without a device
    assert lib.fpsched_wslide_workspace_bytes(p._h, 100, spec.stride) >= 256 + 100 * 8 * spec.stride * 2 + 100 * 8 * 4 + 100
    assert lib.fpsched_pareto_workspace_bytes(p._h, 5000) >= 3 * 2048 * 20
    assert lib.fpsched_rank_workspace_bytes(p._h, 5000, 16) >= lib.fpsched_workspace_bytes(p._h, 5000, 16) + 5000 * 9
    # null handle and nonsense sizes
    assert lib.fpsched_wslide(None, 0, 1, 8, 0, 8, none, 0, 0, 0) == -1
    assert lib.fpsched_wslide_evaluate(None, 0, 1, 8, none, 0, 0, 0) == -1
    assert lib.fpsched_pareto(p._h, none, 1, 0, 1, 1, 1, 1, 0, 0, 0) == -1
    assert lib.fpsched_topk(p._h, none, 1, 2000, 1, 1, 1, 0, 0, 0) == -1
    assert lib.fpsched_pareto(p._h, none, (1 << 24) + 1, 4, 1, 1, 1, 1, 1, 1 << 40, 0) == -1   # more tiles than cursors
    # costs per micro-batch are validated on the host: shape, sign, the int32 time bound
    table = workloads.microbatch_costs(spec.problem)
    p.set_microbatch_costs(table)
    p.set_microbatch_costs(None)
    with pytest.raises(ValueError):
        p.set_microbatch_costs(table[:, :, :-1])
    for value, code in ((-1, -1), (1 << 30, -4)):
        wrong = table.copy()
        wrong[2, -1, -1] = value
        with pytest.raises(fp.FpschedError) as e:
            p.set_microbatch_costs(wrong)
        assert e.value.code == code
    assert lib.fpsched_problem_set_microbatch_costs(None, None) == -1
    # the link switch on a host-only handle is a flag; the two variants combine in either order
    p.set_link_occupancy(True)
    p.set_microbatch_costs(table)
    p.set_link_occupancy(False)
    p.set_link_occupancy(True)
    p.set_microbatch_costs(None)
    p.set_link_occupancy(False)
    assert lib.fpsched_problem_set_link_occupancy(None, 1) == -1
    p.close()
    # bad descriptions
    bad = chain_problem(4, 8)
    bad.stage_device[0] = 9
    with pytest.raises(fp.FpschedError) as e:
        fp.Problem(bad, 64, device=None)
    assert e.value.code == -1
    cyc = chain_problem(3, 2)
    cyc.edge_src = np.array([0, 1, 2], np.int32)
    cyc.edge_dst = np.array([1, 2, 0], np.int32)
    cyc.edge_comm = np.array([0, 0, 0], np.int32)
    with pytest.raises(fp.FpschedError):
        fp.Problem(cyc, 64, device=None)
    big = chain_problem(4, 8, f=1 << 28, b=1)
    with pytest.raises(fp.FpschedError) as e:
        fp.Problem(big, 64, device=None)
    assert e.value.code == -4
    with pytest.raises(fp.FpschedError):
        fp.Problem(chain_problem(4, 8), 60, device=None)   # stride not a multiple of 8
    neg = chain_problem(4, 8)
    neg.mem_cap = np.asarray(neg.mem_cap).copy()
    neg.mem_cap[2] = -1
    with pytest.raises(fp.FpschedError) as e:
        fp.Problem(neg, 64, device=None)                   # a negative memory cap
    assert e.value.code == -1
    five = chain_problem(1, 2, v=5)
    with pytest.raises(fp.FpschedError):
        fp.Problem(five, 64, device=None)                  # more than 4 stages on a device


def test_sync_setting_on_a_host_only_handle():
    # groups and pairs are validated on the host; encode and validate then follow the item counts
    spec = workloads.sync_config(16)
    words = workloads.generate_sync(spec, threads=2)
    p = fp.Problem(spec.problem, spec.stride, device=None)
    assert p.validate(words) == 0            # every item index is below 64 anyway
    p.set_sync(spec.group, spec.pairs)
    assert p.validate(words) == 0
    bad = words.copy()
    bad[3, 11, 5] = pack_word(F, 1, 16)      # the synchronisation stage has 16 items: 0..15
    assert p.validate(bad) == 1
    assert list(p.encode([(F, 12, 15)], device=11)) == [pack_word(F, 1, 15)]
    with pytest.raises(fp.FpschedError):
        p.encode([(F, 12, 16)], device=11)
    for kwargs, code in ((dict(group=[1] * 12 + [0]), -1), (dict(pairs=[(F, 0, F, 0, 0)]), -1),
                         (dict(pairs=[(R, 0, F, 1, 0)]), -1), (dict(pairs=[(F, 0, F, 1, 1 << 30)]), -4)):
        with pytest.raises(fp.FpschedError) as e:
            p.set_sync(**kwargs)
        assert e.value.code == code
    with pytest.raises(ValueError):
        p.set_sync(group=[1, 2])
    p.set_sync()
    assert list(p.encode([(F, 12, 16)], device=11)) == [pack_word(F, 1, 16)]
    assert fp.load_library().fpsched_problem_set_sync(None, None, 0, None) == -1
    p.close()


def test_encode_matches_hand_written_words_and_oracle_decode():
    prob = chain_problem(4, 8, v=2, f=1, b=1, w=1)
    p = fp.Problem(prob, 64, device=None)
    # device 1 hosts stages 1 (chunk 0) and 5 (chunk 1)
    words = p.encode([(F, 1, 0), (FD, 5, 7), (B, 5, 7), (W, 1, 3)], device=1)
    assert list(words) == [0x2000, 0xE807, 0x4807, 0x6003]
    assert list(words) == [pack_word(F, 0, 0), pack_word(FD, 1, 7), pack_word(B, 1, 7), pack_word(W, 0, 3)]
    k, c, j = oracle.decode(words)
    assert list(k) == [F, FD, B, W] and list(c) == [0, 1, 1, 0] and list(j) == [0, 7, 7, 3]
    for item in [(F, 0, 0), (F, 1, 8), (9, 1, 0), (0, 1, 0), (F, 8, 0)]:
        with pytest.raises(fp.FpschedError):
            p.encode([item], device=1)
    nosplit = fp.Problem(chain_problem(2, 2), 8, device=None)
    with pytest.raises(fp.FpschedError):
        nosplit.encode([(W, 0, 0)], device=0)


def test_validate_counts_bad_candidates_like_the_oracle_flags_them():
    spec = workloads.config(1, 64)
    words = workloads.generate(spec, threads=2)
    p = fp.Problem(spec.problem, spec.stride, device=None)
    assert p.validate(words) == 0
    words = words.copy()
    words[3, 1, 4] = pack_word(F, 1, 0)     # chunk 1 does not exist (v=1)
    words[7, 0, 0] = pack_word(B, 0, 9)     # micro-batch 9 >= m
    words[9, 2, 2] = pack_word(W, 0, 0)     # W in a non-split problem
    words[11, 3, 40] = pack_word(F, 3, 99)  # behind the END: ignored
    assert p.validate(words) == 3
    fl = oracle.evaluate(spec.problem, words)["flags"]
    assert set(np.flatnonzero(fl & 2)) <= {3, 7, 9}
