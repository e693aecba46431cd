"""Pins for the oracle's token-weighted k-means iteration (paper Sec. 3.1, offline centroid learning).

None of them re-types the update formula: brute-force means over boolean masks, invariances of weighted means
(duplicating a token = doubling its weight; scaling all weights), the descent property of Lloyd's iteration, and a
one-dimensional example worked by hand.
"""
import numpy as np

import oracle
from workloads import make_codebooks, make_qkv


def _data(seed, B, Hkv, n, d):
    _, k, _ = make_qkv(seed, B, Hkv, Hkv, n, 1, 128, want_v=False)
    cb = make_codebooks(seed, k, d, 256, "k", max_sample=min(n, 512))
    rng = np.random.default_rng(seed)
    w = rng.gamma(0.5, 1.0, size=(B, Hkv, n)).astype(np.float32)      # heavy-tailed, like gradient magnitudes
    return k, w, cb


def test_update_equals_masked_weighted_means():
    x, w, cb = _data(1, 2, 2, 300, 8)
    codes = oracle.encode(x, cb)
    new, wsum, _ = oracle.kmeans_update(x, w, codes, cb)
    x64, w64 = x.astype(np.float64), w.astype(np.float64)
    rng = np.random.default_rng(0)
    for _ in range(60):
        g, m, c = int(rng.integers(2)), int(rng.integers(16)), int(rng.integers(256))
        mask = codes[:, g, :, m] == c                                      # [B, n]
        if not mask.any():
            np.testing.assert_array_equal(new[g, m, c], cb[g, m, c].astype(np.float64))
            assert wsum[g, m, c] == 0
            continue
        rows = x64[:, g, :, m * 8:(m + 1) * 8][mask]
        ww = w64[:, g][mask]
        want = np.average(rows, axis=0, weights=ww) if ww.sum() > 0 else cb[g, m, c]
        np.testing.assert_allclose(new[g, m, c], want, rtol=1e-12, atol=1e-14)
        assert np.isclose(wsum[g, m, c], ww.sum(), rtol=1e-13)


def test_doubling_a_weight_equals_duplicating_the_token_and_scale_invariance():
    x, w, cb = _data(2, 1, 1, 200, 16)
    codes = oracle.encode(x, cb)
    base, _, obj = oracle.kmeans_update(x, w, codes, cb)
    scaled, _, obj_s = oracle.kmeans_update(x, 3.5 * w, codes, cb)
    np.testing.assert_allclose(scaled, base, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(obj_s, 3.5 * obj, rtol=1e-12)
    w2 = w.copy(); w2[0, 0, 17] *= 2
    x_dup = np.concatenate([x, x[:, :, 17:18]], axis=2)
    w_dup = np.concatenate([w, w[:, :, 17:18]], axis=2)
    c_dup = np.concatenate([codes, codes[:, :, 17:18]], axis=2)
    a, _, oa = oracle.kmeans_update(x, w2, codes, cb)
    b, _, ob = oracle.kmeans_update(x_dup, w_dup, c_dup, cb)
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(oa, ob, rtol=1e-12)


def test_lloyd_iterations_never_increase_the_weighted_distortion():
    x, w, cb = _data(3, 2, 2, 400, 4)
    cur = cb                                                          # fp16, as the library stores codebooks
    prev_codes = None
    for _ in range(5):
        new, codes, _, obj = oracle.kmeans_step(x, w, cur)
        # obj = distortion right after assigning to `cur`.  Assignment step: it cannot exceed the distortion of
        # the previous assignment against the same centroids.
        if prev_codes is not None:
            _, _, before = oracle.kmeans_update(x, w, prev_codes, cur)
            assert (obj <= before * (1 + 1e-12)).all()
        # Update step: the weighted means cannot raise the distortion of this assignment.
        _, _, after = oracle.kmeans_update(x, w, codes, new)
        assert (after <= obj * (1 + 1e-12)).all()
        assert (after < obj).any()
        prev_codes, cur = codes, new.astype(np.float16)


def test_one_dimensional_example_by_hand():
    # one KV head, D = 128 split in d = 4; only channel 0 carries data, two centroids matter (0 at 0.0, 1 at 10.0)
    x = np.zeros((1, 1, 4, 128), np.float16)
    x[0, 0, :, 0] = [1.0, 2.0, 9.0, 12.0]
    w = np.array([[[1.0, 3.0, 2.0, 2.0]]], np.float32)
    cb = np.full((1, 32, 256, 4), 100.0, np.float16)                 # every other centroid is far away
    cb[0, :, 0] = 0.0
    cb[0, 0, 1] = [10.0, 0.0, 0.0, 0.0]
    new, codes, wsum, obj = oracle.kmeans_step(x, w, cb)
    assert codes[0, 0, :, 0].tolist() == [0, 0, 1, 1]
    assert np.isclose(new[0, 0, 0, 0], (1 * 1.0 + 3 * 2.0) / 4) and np.isclose(new[0, 0, 1, 0], (2 * 9.0 + 2 * 12.0) / 4)
    assert wsum[0, 0, 0] == 4 and wsum[0, 0, 1] == 4 and wsum[0, 0, 2:].sum() == 0
    assert np.isclose(obj[0, 0], 1 * 1 + 3 * 4 + 2 * 1 + 2 * 4)
    assert (new[0, 0, 2:] == 100.0).all()                             # empty clusters keep their centroid
    assert (codes[0, 0, :, 1:] == 0).all() and np.isclose(obj[0, 1:], 0).all()
