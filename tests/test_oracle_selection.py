"""Pins for oracle/selection.py (Alg. 2, selection step: t different chunks of k, uniformly)."""
import itertools
from collections import Counter

import numpy as np
import pytest

from oracle import selection as S


def test_splitmix64_published_vector():
    """First outputs of SplitMix64 from state 1234567, as published with the
    algorithm's reference implementation and reproduced in many test suites."""
    g = S.SplitMix64(1234567)
    assert [g.next() for _ in range(5)] == [
        6457827717110365317, 3203168211198807973, 9817491932198370423,
        4593380528125082431, 16408922859458223821]


def test_bounded_draw_rejects_the_biased_tail():
    class Stub(S.SplitMix64):
        def __init__(self, vals):
            self.vals = list(vals)

        def next(self):
            return self.vals.pop(0)

    # m = 3: floor(2^64/3)*3 = 2^64 - 1, so only the value 2^64-1 is rejected
    assert Stub([2 ** 64 - 1, 5]).below(3) == 2
    assert Stub([2 ** 64 - 2]).below(3) == (2 ** 64 - 2) % 3
    # m = 2^63 + 1: everything from m upwards is rejected
    m = 2 ** 63 + 1
    assert Stub([m, m + 5, 7]).below(m) == 7


@pytest.mark.parametrize("k,t", [(1, 1), (4, 2), (16, 4), (32, 8), (64, 16), (512, 8), (7, 7)])
def test_selection_is_a_valid_descending_subset(k, t):
    for seed in range(50):
        sel = S.select_chunks(seed, seed * 3, k, t)
        assert sel.dtype == np.int32 and sel.shape == (t,)
        assert len(set(sel.tolist())) == t
        assert sel.min() >= 0 and sel.max() < k
        assert (np.diff(sel) < 0).all()
    assert S.select_chunks(5, 0, k, k).tolist() == list(range(k - 1, -1, -1))


def test_selection_depends_on_seed_and_step_and_is_repeatable():
    a = S.select_chunks(1, 0, 64, 8)
    assert (a == S.select_chunks(1, 0, 64, 8)).all()
    assert (a != S.select_chunks(2, 0, 64, 8)).any()
    assert (a != S.select_chunks(1, 1, 64, 8)).any()


def test_inclusion_frequency_and_subset_uniformity():
    k, t, n = 16, 4, 20000
    counts = np.zeros(k)
    for step in range(n):
        counts[S.select_chunks(11, step, k, t)] += 1
    freq = counts / n
    sigma = np.sqrt((t / k) * (1 - t / k) / n)
    assert np.abs(freq - t / k).max() < 5 * sigma
    # every 2-subset of 4 equally likely (chi-square, 5 dof; 0.999 quantile is 20.5)
    n = 12000
    c = Counter(tuple(S.select_chunks(3, step, 4, 2).tolist()) for step in range(n))
    assert set(c) == {tuple(sorted(p, reverse=True)) for p in itertools.combinations(range(4), 2)}
    chi2 = sum((v - n / 6) ** 2 / (n / 6) for v in c.values())
    assert chi2 < 20.5


def test_bad_arguments():
    for k, t in [(4, 0), (4, 5), (0, 0)]:
        with pytest.raises(ValueError):
            S.select_chunks(0, 0, k, t)
