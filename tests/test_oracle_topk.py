"""Pins for the oracle's top-k anchor selection (keep the ~1 % highest Anchor Scores in FP16)."""
import heapq
import os

import numpy as np
import pytest

from workloads import anchor_count

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_anchor_counts_golden():
    for line in open(os.path.join(GOLD, "anchor_counts.txt")):
        if line.strip() and line[0] != "#":
            n, k = (int(v) for v in line.split()[:2])
            assert anchor_count(n) == k


@pytest.mark.parametrize("N,k", [(1, 1), (10, 3), (257, 41), (1000, 10), (64, 64), (64, 0)])
def test_matches_heap_selection(oracle, N, k):
    rng = np.random.default_rng(N * 7 + k)
    s = rng.random((3, N))
    s[1] = np.round(s[1] * 8) / 8            # many exact ties
    idx = oracle.topk(s, k)
    assert idx.shape == (3, k) and idx.dtype == np.int32
    for r in range(3):
        # heapq.nlargest on (score, -index) keeps the lower index among equal scores
        want = sorted(i for _, i in heapq.nlargest(k, ((s[r, i], -i) for i in range(N))))
        want = sorted(-i for i in want)
        assert idx[r].tolist() == want


def test_all_equal_scores_take_the_first_k(oracle):
    idx = oracle.topk(np.full((2, 50), 3.25), 7)
    assert np.array_equal(idx, np.tile(np.arange(7), (2, 1)))


def test_margin_marks_the_threshold_pair(oracle):
    s = np.array([[5.0, 1.0, 4.0, 3.0, 3.0 - 3e-7, 0.5]])
    idx, margin = oracle.topk(s, 3, want_margin=True)
    assert idx.tolist() == [[0, 2, 3]]
    assert margin[0, 3] < 1e-6 and margin[0, 4] < 1e-6       # swapping 3 and 4 is within the tie band
    assert margin[0, 0] > 0.1 and margin[0, 5] > 0.1
