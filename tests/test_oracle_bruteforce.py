"""Brute force over ALL per-device order pairs for p=2, m<=3 (F/B only) -- no GPU."""
import itertools

import numpy as np
import pytest

import checker
import oracle
from workloads.problem import B, F, chain_problem, pack_word


def _all_pairs(m):
    ops = [(F, 0, j) for j in range(m)] + [(B, 0, j) for j in range(m)]
    perms = np.array([[pack_word(*o) for o in perm] for perm in itertools.permutations(ops)], np.uint16)
    n = len(perms)
    words = np.zeros((n * n, 2, 8), np.uint16)
    words[:, 0, : 2 * m] = np.repeat(perms, n, axis=0)
    words[:, 1, : 2 * m] = np.tile(perms, (n, 1))
    return words


# deadlock-free count, min makespan and number of minimisers, by (m, f, b, c)
EXPECT_FREE = {1: 1, 2: 26, 3: 3750}


@pytest.mark.parametrize("m", [1, 2, 3])
def test_enumeration_counts(m):
    words = _all_pairs(m)
    prob = chain_problem(2, m, f=2, b=4, comm=0)
    r = oracle.evaluate(prob, words, threads=4)
    free = r["flags"] == 0
    assert int(free.sum()) == EXPECT_FREE[m]
    assert np.all((r["flags"] == 0) | (r["flags"] == oracle.FLAG_DEADLOCK))
    assert int(r["makespan"][free].min()) == {1: 12, 2: 18, 3: 24}[m]
    r1 = oracle.evaluate(chain_problem(2, m, f=2, b=4, comm=1), words, threads=4)
    assert np.array_equal(r1["flags"], r["flags"])
    assert int(r1["makespan"][free].min()) == {1: 14, 2: 20, 3: 26}[m]
    ru = oracle.evaluate(chain_problem(2, m, f=1, b=1, comm=0), words, threads=4)
    assert int(ru["makespan"][free].min()) == {1: 4, 2: 6, 3: 8}[m]
    # number of optimal order pairs (enumeration facts fixed before the oracle existed)
    def n_best(res):
        return int((res["makespan"][free] == res["makespan"][free].min()).sum())
    assert n_best(r) == {1: 1, 2: 6, 3: 114}[m]
    assert n_best(r1) == {1: 1, 2: 6, 3: 108}[m]
    assert n_best(ru) == {1: 1, 2: 6, 3: 138}[m]
    # the optimum is the best over ALL orders, so no feasible candidate may beat the
    # critical path of one micro-batch plus the work of the rest on the bottleneck device
    assert np.all(ru["makespan"][free] >= 2 * m + 2)


@pytest.mark.parametrize("m", [1, 2])
def test_every_pair_against_checker(m):
    words = _all_pairs(m)
    prob = chain_problem(2, m, f=2, b=4, comm=1)
    r = oracle.evaluate(prob, words)
    n_free = 0
    for i in range(len(words)):
        c = checker.check(prob, words[i])
        assert c["deadlock"] == bool(r["flags"][i] & oracle.FLAG_DEADLOCK)
        if not c["deadlock"]:
            n_free += 1
            assert c["makespan"] == r["makespan"][i]
            assert c["idle"] == list(r["idle"][i]) and c["peak"] == list(r["peak"][i])
    assert n_free == EXPECT_FREE[m]


def test_sample_of_m3_against_checker():
    words = _all_pairs(3)
    prob = chain_problem(2, 3, f=2, b=4, comm=1)
    rng = np.random.default_rng(5)
    pick = rng.choice(len(words), 3000, replace=False)
    r = oracle.evaluate(prob, words[pick])
    for n, i in enumerate(pick):
        c = checker.check(prob, words[i])
        assert c["deadlock"] == bool(r["flags"][n] & oracle.FLAG_DEADLOCK)
        if not c["deadlock"]:
            assert c["makespan"] == r["makespan"][n]
