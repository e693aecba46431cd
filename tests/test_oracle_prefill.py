"""Pins for the oracle's prefill attention (paper Sec. 2.1; row statistics of Alg. 1's first step).

Each pin comes from somewhere other than the function under test: a library softmax, a per-row loop written
from the definition, closed forms, and the C oracle's independently written row statistics.
"""
import numpy as np
import scipy.special

import oracle
from workloads import make_qkv


def _inputs(seed, B, Hq, Hkv, N, Nq, D=128):
    q, k, v = make_qkv(seed, B, Hq, Hkv, N, Nq, D)
    return q, k, v


def test_matches_library_softmax_per_row():
    B, Hq, Hkv, N, Nq = 1, 4, 2, 37, 21
    q, k, v = _inputs(3, B, Hq, Hkv, N, Nq)
    scale = 0.11
    out, m, l = oracle.prefill_attn(q, k, v, scale)
    q64, k64, v64 = (a.astype(np.float64) for a in (q, k, v))
    for h in range(Hq):
        for i in range(Nq):
            n_vis = N - Nq + i + 1
            s = scale * (k64[0, h // 2, :n_vis] @ q64[0, h, i])
            a = scipy.special.softmax(s)
            np.testing.assert_allclose(out[0, h, i], a @ v64[0, h // 2, :n_vis], rtol=1e-12, atol=1e-14)
            assert np.isclose(m[0, h, i], s.max(), rtol=0, atol=1e-14)
            assert np.isclose(np.log(l[0, h, i]) + m[0, h, i], scipy.special.logsumexp(s), rtol=1e-13)


def test_first_query_of_a_full_prompt_returns_v0():
    q, k, v = _inputs(5, 2, 4, 4, 16, 16)
    out, m, l = oracle.prefill_attn(q, k, v, 0.3)
    np.testing.assert_allclose(out[:, :, 0], v[:, :, 0].astype(np.float64), rtol=1e-13)
    np.testing.assert_allclose(l[:, :, 0], 1.0, rtol=0, atol=0)


def test_constant_values_come_back_and_zero_queries_average():
    B, Hq, Hkv, N = 1, 2, 1, 12
    q, k, v = _inputs(7, B, Hq, Hkv, N, N)
    vc = np.broadcast_to(v[:, :, :1], v.shape).copy()
    out, _, _ = oracle.prefill_attn(q, k, vc, 0.2)
    np.testing.assert_allclose(out, np.broadcast_to(vc[:, :1].astype(np.float64), out.shape), rtol=1e-13)
    # zero queries: uniform attention, so row i is the mean of the first i+1 values and row_sum = i + 1
    out, m, l = oracle.prefill_attn(np.zeros_like(q), k, v, 0.2)
    v64 = v.astype(np.float64)
    want = np.cumsum(v64[0, 0], axis=0) / np.arange(1, N + 1)[:, None]
    np.testing.assert_allclose(out[0, 0], want, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(l[0, 0], np.arange(1, N + 1), rtol=1e-14)
    assert (m == 0).all()


def test_row_statistics_agree_with_the_anchor_score_oracle():
    # the C oracle computes the same statistics in its own code
    B, Hq, Hkv, N, Nq = 2, 4, 2, 90, 40
    q, k, v = _inputs(11, B, Hq, Hkv, N, Nq)
    _, m, l = oracle.prefill_attn(q, k, v, 0.09)
    _, _, st = oracle.anchor_score(q, k, 0.09, want_stats=True)
    np.testing.assert_allclose(m, st["row_max"], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(l, st["row_sum"], rtol=1e-12)


def test_two_key_closed_form():
    # N = 2, one head, D = 128 with a single non-zero channel: softmax over two scalars
    q = np.zeros((1, 1, 2, 128), np.float16); k = np.zeros((1, 1, 2, 128), np.float16)
    v = np.zeros((1, 1, 2, 128), np.float16)
    q[0, 0, :, 0] = [1.0, 2.0]; k[0, 0, :, 0] = [0.5, -1.5]; v[0, 0, :, 3] = [4.0, -2.0]
    out, m, l = oracle.prefill_attn(q, k, v, 0.5)
    s = 0.5 * 2.0 * np.array([0.5, -1.5])
    w = 1.0 / (1.0 + np.exp(s[1] - s[0]))
    assert np.isclose(out[0, 0, 1, 3], 4.0 * w - 2.0 * (1 - w), rtol=1e-14)
    assert np.isclose(out[0, 0, 0, 3], 4.0)
    assert np.isclose(m[0, 0, 1], s[0]) and np.isclose(l[0, 0, 1], 1 + np.exp(s[1] - s[0]))
