"""Seeded input generator: determinism, structure, and its private clock against the oracle -- no GPU."""
import numpy as np
import pytest

import oracle
import workloads
from workloads.problem import B, F, FD, W


@pytest.mark.parametrize("index,n", [(1, 300), (2, 400), (3, 96), (4, 48), (5, 400)])
def test_generator_clock_equals_oracle_makespan(index, n):
    # the list scheduler's own start/finish bookkeeping is a different algorithm from the oracle's
    # event loop (it builds the order while it advances time); on unperturbed candidates the two
    # must tell the same makespan
    spec = workloads.config(index, n)
    words, clock = workloads.generate(spec, with_generator_clock=True, threads=4)
    r = oracle.evaluate(spec.problem, words, threads=4)
    plain = clock >= 0
    assert plain[:n].sum() > 0.9 * n
    assert np.all((r["flags"][plain] & 3) == 0)
    assert np.array_equal(clock[plain], r["makespan"][plain])


def test_regenerating_a_range_alone_gives_the_same_candidates():
    spec = workloads.config(2, 256)
    full = workloads.generate(spec, threads=3)
    part = workloads.generate(spec, n=40, first=100, threads=2)
    assert np.array_equal(full[100:140], part)
    again = workloads.generate(spec, threads=1)
    assert np.array_equal(full, again)


@pytest.mark.parametrize("index,n", [(2, 3000), (5, 3000)])
def test_deadlock_fraction_and_cap_fraction(index, n):
    spec = workloads.config(index, n)
    words = workloads.generate(spec, threads=4)
    fl = oracle.evaluate(spec.problem, words, threads=4)["flags"]
    dead = float(((fl & 1) != 0).mean())
    assert 0.4 * spec.deadlock_per_mille / 1000 <= dead <= 2.0 * spec.deadlock_per_mille / 1000
    under = float((fl == 0).mean())
    assert 0.3 <= under <= 0.7
    assert np.all((fl == 0) | (fl == 1) | (fl == 4))


def test_unperturbed_streams_ascend_and_lists_are_complete():
    spec = workloads.config(4, 24)
    words, clock = workloads.generate(spec, with_generator_clock=True, threads=4)
    p = spec.problem
    for c in np.flatnonzero(clock >= 0)[:8]:
        n_r = 0
        for d in range(p.n_devices):
            row = words[c, d]
            row = row[: int(np.argmax(row >> 13 == 0))] if (row >> 13 == 0).any() else row
            kind, chunk, mb = row >> 13, (row >> 11) & 3, row & 0x7FF
            for ch in range(2):
                for ks in ((F, FD), (B,), (W,)):
                    sel = np.isin(kind, ks) & (chunk == ch)
                    assert list(mb[sel]) == list(range(p.n_microbatches))
            n_r += int((kind == 4).sum())
            assert (kind == FD).sum() == (kind == 4).sum()
        assert workloads.count_ops(words[c:c + 1]) == 3 * 2 * p.n_microbatches * p.n_devices + n_r


def test_configurations_match_their_description():
    s1, s4, s5 = workloads.config(1), workloads.config(4), workloads.config(5)
    assert (s1.problem.n_devices, s1.problem.n_microbatches, s1.n_candidates, s1.top_k) == (4, 8, 1024, 16)
    assert list(s1.problem.dur[F]) == [2] * 4 and list(s1.problem.dur[B]) == [4] * 4
    assert (s4.problem.n_devices, s4.problem.n_stages, s4.problem.n_microbatches) == (32, 64, 128)
    assert s4.n_candidates == 65536 and s4.top_k == 128 and int(s4.problem.mem_cap[0]) == 24
    assert s4.problem.dur[F].min() >= 20 and s4.problem.dur[B].max() <= 60
    assert list(s4.problem.stage_device[:34]) == list(range(32)) + [0, 1]
    assert s5.problem.n_stages == 16 and len(s5.problem.edge_src) == 15
    assert sorted(s5.problem.edge_dst.tolist()).count(12) == 2      # the fusion stage has two inputs
    s3 = workloads.config(3)
    assert s3.n_candidates == 262144 and s3.problem.dur[F][0] >= 12 and s3.problem.dur[B][-1] >= 29
