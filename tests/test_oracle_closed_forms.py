"""Pins of the CPU oracle against closed forms (GPipe, 1F1B) -- no GPU."""
import os

import numpy as np
import pytest

import oracle
from workloads.problem import chain_problem, gpipe_lists, one_f_one_b_lists, pack_lists

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "closed_forms.txt")


def _eval(problem, lists):
    return oracle.evaluate_trace(problem, pack_lists(lists))


@pytest.mark.parametrize("p,m,f,b,c", [(4, 8, 2, 4, 0), (4, 8, 2, 4, 1), (2, 1, 1, 1, 0), (8, 32, 3, 5, 2),
                                       (3, 5, 7, 2, 4), (6, 6, 1, 1, 1), (16, 4, 2, 3, 1)])
def test_gpipe_closed_form(p, m, f, b, c):
    r = _eval(chain_problem(p, m, f=f, b=b, comm=c), gpipe_lists(p, m))
    ms = (m + p - 1) * (f + b) + 2 * (p - 1) * c
    assert r["flags"] == 0
    assert r["makespan"] == ms
    assert list(r["idle"]) == [ms - m * (f + b)] * p
    assert list(r["peak"]) == [m] * p


@pytest.mark.parametrize("p,m", [(4, 8), (8, 32), (3, 5), (6, 6), (2, 7), (5, 3)])
@pytest.mark.parametrize("f,b", [(2, 4), (1, 1), (3, 5)])
def test_1f1b_closed_form_zero_comm(p, m, f, b):
    if m < p:
        pytest.skip("the (m+p-1)(f+b) form assumes m >= p")
    r = _eval(chain_problem(p, m, f=f, b=b, comm=0), one_f_one_b_lists(p, m))
    ms = (m + p - 1) * (f + b)
    assert r["flags"] == 0
    assert r["makespan"] == ms
    assert list(r["peak"]) == [min(m, p - d) for d in range(p)]
    # bubble fraction (p-1)/(m+p-1) on every device
    for d in range(p):
        assert r["idle"][d] * (m + p - 1) == ms * (p - 1)


def test_bubble_fraction_gpipe_uniform():
    p, m, f, b = 4, 8, 2, 4
    r = _eval(chain_problem(p, m, f=f, b=b, comm=0), gpipe_lists(p, m))
    assert sum(r["idle"]) * (m + p - 1) == p * r["makespan"] * (p - 1)


def test_golden_rows():
    rows = [ln.split() for ln in open(GOLDEN) if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 6
    for name, p, m, f, b, c, ms, idle, peak in rows:
        p, m, f, b, c, ms = map(int, (p, m, f, b, c, ms))
        lists = gpipe_lists(p, m) if name == "gpipe" else one_f_one_b_lists(p, m)
        r = _eval(chain_problem(p, m, f=f, b=b, comm=c), lists)
        assert r["flags"] == 0
        assert r["makespan"] == ms, (name, c)
        assert list(r["idle"]) == [int(x) for x in idle.split(",")]
        assert list(r["peak"]) == [int(x) for x in peak.split(",")]


def test_1f1b_stage0_peak_is_p():
    for p, m in [(4, 8), (8, 32), (16, 64)]:
        r = _eval(chain_problem(p, m, f=2, b=4, comm=1), one_f_one_b_lists(p, m))
        assert r["peak"][0] == p and r["flags"] == 0


def test_first_op_times_and_comm_only_across_devices():
    # two stages on ONE device (v=2, p=1): the chain edge is same-device, so comm must not be added
    from workloads.problem import B, F
    prob = chain_problem(1, 1, v=2, f=3, b=5, comm=100)
    lists = [[(F, 0, 0), (F, 1, 0), (B, 1, 0), (B, 0, 0)]]
    r = _eval(prob, lists)
    assert r["makespan"] == 16 and list(r["start"][0][:4]) == [0, 3, 6, 11]
    # same stages on two devices: comm added once forward, once backward
    prob = chain_problem(2, 1, f=3, b=5, comm=100)
    r = _eval(prob, [[(F, 0, 0), (B, 0, 0)], [(F, 0, 0), (B, 0, 0)]])
    assert r["makespan"] == 3 + 100 + 3 + 5 + 100 + 5
    assert r["start"][1][0] == 103 and r["start"][0][1] == 211


def test_hand_worked_timeline_with_recompute_offload_and_reload_on_two_devices():
    # Two stages on two devices, two micro-batches, latency 1, split backward.  Costs F/B/W/R/O/L: stage 0
    # 2/3/1/2/4/3 (2 units per activation), stage 1 3/2/2/3/1/1 (5 units).  Worked by hand:
    #  device 0: FD(0,0) 0-2 | F(0,1) 2-4 | O(0,1) 4-8 | R(0,0) 8-10 | B(0,0) waits for B(1,0) (15) + 1: 16-19 |
    #            L(0,1) 19-22 | W(0,0) 22-23 | B(0,1) (its gradient came at 12 + 1) 23-26 | W(0,1) 26-27
    #  device 1: F(1,0) waits for FD(0,0) (2) + 1: 3-6 | F(1,1) (input at 4 + 1, device free at 6) 6-9 |
    #            O(1,0) 9-10 | B(1,1) 10-12 | L(1,0) 12-13 | B(1,0) 13-15 | W(1,1) 15-17 | W(1,0) 17-19
    #  memory, device 0: +2 -2 (discarding forward), +2 (F), -2 (offload done), +2 (recompute), +2 (reload) = 4
    #  at most; device 1: 5, 10 (two forward passes), 5 after the offload, 10 again with the reload.
    from workloads.problem import B, F, FD, L, O, R, W, make_problem
    dur = {F: [2, 3], FD: [2, 3], B: [3, 2], W: [1, 2], R: [2, 3], O: [4, 1], L: [3, 1]}
    prob = make_problem(2, 2, 2, 1, [0, 1], [(0, 1, 1)], dur, mem_units=[2, 5])
    lists = [[(FD, 0, 0), (F, 0, 1), (O, 0, 1), (R, 0, 0), (B, 0, 0), (L, 0, 1), (W, 0, 0), (B, 0, 1), (W, 0, 1)],
             [(F, 0, 0), (F, 0, 1), (O, 0, 0), (B, 0, 1), (L, 0, 0), (B, 0, 0), (W, 0, 1), (W, 0, 0)]]
    r = _eval(prob, lists)
    assert r["flags"] == 0 and r["makespan"] == 27
    assert list(r["start"][0][:9]) == [0, 2, 4, 8, 16, 19, 22, 23, 26]
    assert list(r["start"][1][:8]) == [3, 6, 9, 10, 12, 13, 15, 17]
    assert list(r["finish"][0][:9]) == [2, 4, 8, 10, 19, 22, 23, 26, 27]
    assert list(r["idle"]) == [27 - 21, 27 - 16] and list(r["peak"]) == [4, 10]
    # the backward pass of an offloaded activation cannot run before its reload
    stuck = [list(lists[0]), [(F, 0, 0), (F, 0, 1), (O, 0, 0), (B, 0, 0), (L, 0, 0), (B, 0, 1), (W, 0, 1), (W, 0, 0)]]
    assert _eval(prob, stuck)["flags"] & 1               # B(1,0) while its activation is offloaded: never runs
