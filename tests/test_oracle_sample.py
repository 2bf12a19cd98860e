"""The sampling oracle (oracle/sample.py) against closed forms: a two-token distribution worked by hand, frequencies on
a grid of draws equal to the renormalised nucleus probabilities, the limits top_p -> 0 and T -> 0 (the greedy token),
top_p = 1 (plain softmax sampling), ties entering together, and the two formulations of the nucleus agreeing."""
import math

import numpy as np
import pytest

from oracle import sample as S
from paper_2603_20661_amd import synth


def test_two_token_example_by_hand():
    lg = np.array([math.log(3.0), 0.0])                       # p = (0.75, 0.25)
    for fast in (False, True):
        _, _, mask, _, _ = S.sample(lg, 1.0, 0.7, 0.5, fast)
        assert mask.tolist() == [True, False]
        _, _, mask, _, _ = S.sample(lg, 1.0, 0.8, 0.5, fast)
        assert mask.tolist() == [True, True]
        assert S.sample(lg, 1.0, 0.8, 0.74, fast)[0] == 0 and S.sample(lg, 1.0, 0.8, 0.76, fast)[0] == 1
        assert S.sample(lg, 1.0, 0.7, 0.99, fast)[0] == 0       # outside the nucleus is never drawn
        # temperature 0.5 squares the odds: p = (0.9, 0.1)
        assert S.sample(lg, 0.5, 1.0, 0.89, fast)[0] == 0 and S.sample(lg, 0.5, 1.0, 0.91, fast)[0] == 1


@pytest.mark.parametrize("top_p", [1.0, 0.9, 0.6])
def test_frequencies_on_a_grid_are_the_renormalised_nucleus_probabilities(top_p):
    lg = synth.normal_f32(4, 1, 12, std=1.5)
    p = np.exp(lg.astype(np.float64) - lg.max()); p /= p.sum()
    order = np.argsort(-p)
    k = int(np.argmax(np.cumsum(p[order]) >= top_p * (1 - 1e-15)))   # textbook: smallest prefix of the sorted list reaching top_p
    members = set(order[:k + 1].tolist())
    want = np.array([p[i] if i in members else 0.0 for i in range(12)]); want /= want.sum()
    N = 20000
    counts = np.zeros(12)
    for m in range(N):
        counts[S.sample(lg, 1.0, top_p, (m + 0.5) / N, fast=False)[0]] += 1
    assert np.abs(counts / N - want).max() <= 1.0 / N + 1e-12
    assert set(np.flatnonzero(counts).tolist()) == members


def test_limits_and_ties():
    lg = synth.normal_f32(5, 1, 500, std=2.0)
    best = int(lg.argmax())
    for u in (0.0, 0.3, 0.999):
        assert S.sample(lg, 1.0, 1e-9, u)[0] == best                       # top_p -> 0: only the maximum is in
        assert S.sample(lg, 1e-3, 0.95, u)[0] == best                      # T -> 0: all mass on the maximum
    _, _, mask, _, _ = S.sample(lg, 1.0, 1.0, 0.5)
    assert mask.all()                                                      # top_p = 1: everything is in
    tied = np.array([1.0, 2.0, 2.0, 0.5, 2.0])
    for top_p in (0.1, 0.5, 0.8):
        _, _, mask, _, _ = S.sample(tied, 1.0, top_p, 0.5)
        assert mask.tolist() == [False, True, True, False, True]            # equal probabilities enter together
    assert [S.sample(tied, 1.0, 0.5, u)[0] for u in (0.0, 0.34, 0.67, 0.99)] == [1, 2, 4, 4]   # index order inside the nucleus


def test_both_formulations_of_the_nucleus_agree():
    for seed, std, top_p in ((1, 1.0, 0.95), (2, 4.0, 0.5), (3, 8.0, 0.9), (4, 0.1, 0.99)):
        lg = synth.normal_f32(seed, 2, 3000, std=std)
        lg[::97] = lg[5]                                                    # some exact ties
        a, b = S.nucleus(lg, 0.8, top_p), S.nucleus_fast(lg, 0.8, top_p)
        assert a[2] == b[2] and np.array_equal(a[1], b[1])
