"""Pins for the oracle's nearest-centroid encode (paper Sec. 3.1)."""
import os

import numpy as np
import pytest
from scipy.cluster.vq import vq
from scipy.spatial.distance import cdist

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape).astype(np.float16)


def test_hand_worked_lattice(oracle):
    rows = [l.split() for l in open(os.path.join(GOLD, "encode_lattice.txt")) if l.strip() and l[0] != "#"]
    x = np.array([[float(v) for v in r[:4]] for r in rows], dtype=np.float16).reshape(1, 1, -1, 4)
    want = np.array([[int(v) for v in r[4:]] for r in rows])
    cb = np.array([[[0, 0], [4, 0], [0, 4], [4, 4]], [[1, 1], [1, 1], [-3, 0], [0, -3]]],
                  dtype=np.float16).reshape(1, 2, 4, 2)
    codes, margin = oracle.encode(x, cb, want_margin=True)
    assert np.array_equal(codes[0, 0], want)
    # exact ties carry zero margin; the clear winners do not
    assert margin[0, 0, 0, 1] == 0.0 and margin[0, 0, 2, 0] == 0.0 and margin[0, 0, 3, 1] == 0.0
    assert margin[0, 0, 1, 0] > 0.1


@pytest.mark.parametrize("d,C", [(4, 256), (8, 256), (16, 256), (8, 7), (32, 4096), (16, 4096)])
def test_matches_scipy_vq(oracle, d, C):
    B, Hkv, n, D = 2, 3, 37, 32
    M = D // d
    x = _rand((B, Hkv, n, D), 1)
    cb = _rand((Hkv, M, C, d), 2)
    codes, margin = oracle.encode(x, cb, want_margin=True)
    for b in range(B):
        for g in range(Hkv):
            for m in range(M):
                obs = x[b, g, :, m * d:(m + 1) * d].astype(np.float64)
                book = cb[g, m].astype(np.float64)
                lib_codes, lib_dist = vq(obs, book)
                clear = margin[b, g, :, m] > 1e-9
                assert np.array_equal(codes[b, g, clear, m], lib_codes[clear])
                # the chosen centroid attains the minimum distance
                dm = cdist(obs, book, "sqeuclidean")
                chosen = dm[np.arange(n), codes[b, g, :, m]]
                assert np.all(chosen <= dm.min(axis=1) * (1 + 1e-12) + 1e-300)
                np.testing.assert_allclose(np.sqrt(chosen), lib_dist, rtol=1e-9, atol=1e-12)


def test_sample_points_encode_to_themselves_lowest_duplicate(oracle):
    # centroids picked from the data (as the workload recipe does) must be hit exactly
    Hkv, M, C, d = 2, 4, 256, 8
    D = M * d
    cb = _rand((Hkv, M, C, d), 3)
    cb[:, :, 200] = cb[:, :, 17]          # plant a duplicate: 17 must win over 200
    pick = np.random.default_rng(4).integers(0, C, size=(Hkv, 50, M))
    x = np.empty((1, Hkv, 50, D), dtype=np.float16)
    for g in range(Hkv):
        for t in range(50):
            for m in range(M):
                x[0, g, t, m * d:(m + 1) * d] = cb[g, m, pick[g, t, m]]
    want = np.where(pick == 200, 17, pick)
    # other accidental duplicates in random fp16 data are astronomically unlikely at d=8
    codes = oracle.encode(x, cb)
    assert np.array_equal(codes[0], want)


def test_each_head_uses_its_own_codebook(oracle):
    # head g's codebook has a centroid at (g+1)*ones at index g; every other entry is far away
    Hkv, M, C, d = 4, 2, 8, 4
    cb = np.full((Hkv, M, C, d), 100.0, dtype=np.float16)
    cb += np.arange(C, dtype=np.float16)[None, None, :, None]
    for g in range(Hkv):
        cb[g, :, g] = g + 1
    x = np.empty((1, Hkv, 3, M * d), dtype=np.float16)
    for g in range(Hkv):
        x[0, g] = g + 1
    codes = oracle.encode(x, cb)
    for g in range(Hkv):
        assert np.all(codes[0, g] == g)


def test_permuting_centroids_permutes_codes(oracle):
    Hkv, M, C, d = 1, 4, 64, 8
    x = _rand((2, Hkv, 40, M * d), 5)
    cb = _rand((Hkv, M, C, d), 6)
    perm = np.random.default_rng(7).permutation(C)
    codes = oracle.encode(x, cb)
    codes_p = oracle.encode(x, cb[:, :, perm])
    assert np.array_equal(perm[codes_p], codes)


def test_translation_invariance(oracle):
    # nearest centroid is unchanged when data and centroids move together (values stay exact in fp16)
    Hkv, M, C, d = 1, 2, 32, 4
    rng = np.random.default_rng(8)
    x = rng.integers(-8, 8, size=(1, Hkv, 64, M * d)).astype(np.float16)
    cb = (rng.integers(-16, 16, size=(Hkv, M, C, d)) / 2).astype(np.float16)
    codes = oracle.encode(x, cb)
    assert np.array_equal(oracle.encode(x + np.float16(3), cb + np.float16(3)), codes)
