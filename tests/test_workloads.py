"""The seeded input generator: deterministic, chunk-order independent, recipe as documented."""
import numpy as np

from workloads import CONFIGS, make_codebooks, make_qkv, normal_fp16, outlier_channels, random_anchor_sets, random_codes


def test_deterministic_and_slice_stable():
    a = normal_fp16(3, "q", (2, 4, 100, 128))
    b = normal_fp16(3, "q", (2, 4, 100, 128))
    assert a.dtype == np.float16 and np.array_equal(a, b)
    assert not np.array_equal(a, normal_fp16(4, "q", (2, 4, 100, 128)))
    assert abs(float(a.astype(np.float64).std()) - 1.0) < 0.02


def test_k_has_four_outlier_channels_per_head():
    q, k, v = make_qkv(0, 1, 8, 2, 2048, 4, 128)
    assert q.shape == (1, 8, 4, 128) and k.shape == (1, 2, 2048, 128) and v.shape == k.shape
    mult = outlier_channels(0, 2, 128)
    assert (mult == 10).sum(axis=1).tolist() == [4, 4]
    std = k.astype(np.float64).std(axis=2)[0]              # [Hkv, D]
    for g in range(2):
        assert np.all(std[g][mult[g] == 10] > 8) and np.all(std[g][mult[g] == 1] < 1.2)


def test_codebooks_are_sample_points():
    _, k, _ = make_qkv(1, 1, 4, 2, 600, 1, 32)
    cb = make_codebooks(1, k, 8, 256, "k")
    assert cb.shape == (2, 4, 256, 8) and cb.dtype == np.float16
    sub = k[0].reshape(2, 600, 4, 8)
    for g in range(2):
        for m in range(4):
            pts = {row.tobytes() for row in sub[g, :, m]}
            assert all(c.tobytes() in pts for c in cb[g, m])
            assert len({c.tobytes() for c in cb[g, m]}) == 256       # D^2 sampling never repeats a point
    assert np.array_equal(cb, make_codebooks(1, k, 8, 256, "k"))


def test_codebook_from_fewer_samples_than_centroids_has_duplicates():
    _, k, _ = make_qkv(2, 1, 1, 1, 40, 1, 16)
    cb = make_codebooks(2, k, 4, 256, "k")
    assert len({c.tobytes() for c in cb[0, 0]}) <= 40


def test_random_cache_tensors():
    c = random_codes(5, "k", 1, 2, 1000, 16)
    assert c.dtype == np.uint8 and c.shape == (1, 2, 1000, 16) and c.max() > 200
    idx = random_anchor_sets(5, "k", 2, 2, 1000, 40)
    assert idx.shape == (2, 2, 40) and np.all(np.diff(idx, axis=-1) > 0) and idx.min() == 0 and idx.max() == 999
    assert random_anchor_sets(5, "k", 1, 1, 10, 10)[0, 0].tolist() == list(range(10))
    assert random_anchor_sets(5, "k", 1, 1, 10, 0).shape == (1, 1, 0)


def test_config_table():
    assert [CONFIGS[f"cfg{i}"].k for i in range(5)] == [41, 328, 1311, 328, 8400]
    assert [CONFIGS[f"cfg{i}"].M for i in range(5)] == [16, 32, 16, 16, 8]
    assert [CONFIGS[f"cfg{i}"].bits_per_element for i in range(5)] == [1.0, 2.0, 1.0, 1.0, 0.5]
