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
