"""Pins for the oracle's Anchor Score (paper Eq. (4), Theorem 3.1 / Eq. (3), Alg. 1)."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F
from scipy.special import softmax as sp_softmax


def _rand(shape, seed, scale=1.0):
    return (np.random.default_rng(seed).standard_normal(shape) * scale).astype(np.float16)


def _mask(N, Nq):
    """Query i sits at position N-Nq+i and sees keys 0..N-Nq+i."""
    i = torch.arange(Nq)[:, None]
    j = torch.arange(N)[None, :]
    return j <= (N - Nq + i)


def _sdpa(q, k, v, scale, N, Nq):
    """Library attention with GQA (query head h reads KV head h // G), fp64."""
    qt, kt, vt = (torch.from_numpy(np.asarray(a, dtype=np.float64)) for a in (q, k, v))
    G = qt.shape[1] // kt.shape[1]
    kt = kt.repeat_interleave(G, dim=1)
    vt = vt.repeat_interleave(G, dim=1)
    return F.scaled_dot_product_attention(qt, kt, vt, attn_mask=_mask(N, Nq), scale=scale)


@pytest.mark.parametrize("B,Hq,Hkv,N,Nq,D", [(1, 4, 2, 19, 19, 16), (2, 8, 2, 33, 7, 32), (1, 2, 2, 12, 1, 8)])
def test_column_sums_of_v_score(oracle, B, Hq, Hkv, N, Nq, D):
    # rows of a softmax sum to one, so the V scores of one KV head sum to Nq * G
    q, k = _rand((B, Hq, Nq, D), 1), _rand((B, Hkv, N, D), 2)
    ans_k, ans_v = oracle.anchor_score(q, k, 1 / math.sqrt(D))
    np.testing.assert_allclose(ans_v.sum(-1), Nq * (Hq // Hkv), rtol=1e-12)
    qn = np.linalg.norm(q.astype(np.float64), axis=-1)           # [B,Hq,Nq]
    bound = 0.25 * qn.reshape(B, Hkv, -1).sum(-1)
    assert np.all(ans_k >= 0) and np.all(ans_k <= bound[..., None] + 1e-12)


def test_v_score_is_the_equality_case_of_eq3(oracle):
    """Eq. (3): ||Attn(Q,K,V+dV) - Attn(Q,K,V)||_L1 <= sum_j AnS(V_j) ||dV_j||_L1, with equality
    when dV >= 0 (the only inequality in the proof is a triangle inequality).  Perturbing one token
    of one KV head isolates a single AnS(V) entry and also checks which query heads feed it."""
    B, Hq, Hkv, N, Nq, D = 2, 6, 3, 21, 9, 16
    scale = 0.3
    q, k, v = _rand((B, Hq, Nq, D), 3), _rand((B, Hkv, N, D), 4), _rand((B, Hkv, N, D), 5)
    _, ans_v = oracle.anchor_score(q, k, scale)
    base = _sdpa(q, k, v, scale, N, Nq)
    rng = np.random.default_rng(6)
    for b, g, j in [(0, 0, 0), (1, 2, 13), (0, 1, 20), (1, 0, 12), (0, 2, 5)]:
        dv = np.zeros((B, Hkv, N, D))
        dv[b, g, j] = rng.random(D)                       # >= 0
        pert = _sdpa(q, k, v.astype(np.float64) + dv, scale, N, Nq)
        lhs = (pert - base).abs().sum().item()
        np.testing.assert_allclose(lhs, ans_v[b, g, j] * dv[b, g, j].sum(), rtol=1e-9)
        # only the G query heads of KV head g move
        moved = (pert - base).abs().sum(dim=(2, 3))[b]
        G = Hq // Hkv
        assert all((moved[h] > 0) == (h // G == g) for h in range(Hq))


def test_k_score_from_finite_differences_of_library_attention(oracle):
    """AnS(K_j) = sum_i A_ij (1 - A_ij) ||Q_i||_2 is the first-order sensitivity of column j of A to a
    perturbation of K_j (paper Sec. 3.2, simplification of Eq. (2)).  With every query parallel to a unit
    vector u and dK_j = eps*u, |dS_ij| = scale*eps*||Q_i||, so sum_i |dA_ij| / (scale*eps) -> AnS(K_j).
    A is read off a library attention call by using V = identity."""
    N, D = 12, 16
    scale = 0.5
    rng = np.random.default_rng(7)
    u = rng.standard_normal(D)
    u /= np.linalg.norm(u)
    coef = rng.uniform(0.5, 2.0, size=N) * rng.choice([-1.0, 1.0], size=N)
    qf = (coef[:, None] * u[None, :])
    q = qf.astype(np.float16)[None, None]                          # [1,1,N,D], fp16-rounded
    k = _rand((1, 1, N, D), 8)
    ans_k, _ = oracle.anchor_score(q, k, scale)
    v = np.zeros((1, 1, N, D))
    v[0, 0, np.arange(N), np.arange(N)] = 1.0                      # O[i, :N] = A[i, :]
    q64 = q.astype(np.float64)
    # direction actually used: the rounded queries are only nearly parallel, so measure |Q_i . u_hat| ~ ||Q_i||
    eps = 1e-6
    for j in (0, 5, 11):
        dk = np.zeros((1, 1, N, D))
        dk[0, 0, j] = eps * u
        ap = _sdpa(q64, k.astype(np.float64) + dk, v, scale, N, N)[0, 0, :, j]
        am = _sdpa(q64, k.astype(np.float64) - dk, v, scale, N, N)[0, 0, :, j]
        fd = ((ap - am).abs().sum() / (2 * eps * scale)).item()
        np.testing.assert_allclose(fd, ans_k[0, 0, j], rtol=2e-3)   # fp16 rounding of q tilts it off u slightly


def test_identical_keys_closed_form(oracle):
    # all keys equal -> A_ij = 1/(p_i+1) for j <= p_i: AnS(V_j) = G * sum_{p>=max(j,N-Nq)} 1/(p+1)
    B, Hq, Hkv, N, Nq, D = 1, 4, 2, 40, 25, 8
    G = Hq // Hkv
    q = _rand((B, Hq, Nq, D), 9)
    k = np.broadcast_to(_rand((1, Hkv, 1, D), 10), (B, Hkv, N, D)).copy()
    ans_k, ans_v = oracle.anchor_score(q, k, 0.7)
    qn = np.linalg.norm(q.astype(np.float64), axis=-1)
    for g in range(Hkv):
        for j in range(N):
            ps = [p for p in range(N - Nq, N) if p >= j]
            want_v = G * sum(1.0 / (p + 1) for p in ps)
            want_k = sum(qn[0, g * G + hh, p - (N - Nq)] * (1.0 / (p + 1)) * (1 - 1.0 / (p + 1))
                         for p in ps for hh in range(G))
            np.testing.assert_allclose(ans_v[0, g, j], want_v, rtol=1e-12)
            np.testing.assert_allclose(ans_k[0, g, j], want_k, rtol=1e-12)


def test_two_keys_sigmoid(oracle):
    # N=2, one query seeing both keys: A_0 = sigmoid(s0 - s1)
    D = 8
    q, k = _rand((1, 1, 1, D), 11), _rand((1, 1, 2, D), 12)
    scale = 0.9
    ans_k, ans_v = oracle.anchor_score(q, k, scale)
    q64, k64 = q.astype(np.float64)[0, 0, 0], k.astype(np.float64)[0, 0]
    sig = 1.0 / (1.0 + math.exp(-scale * float(q64 @ (k64[0] - k64[1]))))
    np.testing.assert_allclose(ans_v[0, 0], [sig, 1 - sig], rtol=1e-12)
    np.testing.assert_allclose(ans_k[0, 0], [sig * (1 - sig) * np.linalg.norm(q64)] * 2, rtol=1e-12)


def test_single_query_is_a_library_softmax_row(oracle):
    B, Hq, Hkv, N, D = 2, 4, 4, 57, 16
    q, k = _rand((B, Hq, 1, D), 13), _rand((B, Hkv, N, D), 14)
    scale = 0.25
    ans_k, ans_v, st = oracle.anchor_score(q, k, scale, want_stats=True)
    s = scale * np.einsum("bhd,bhnd->bhn", q[:, :, 0].astype(np.float64), k.astype(np.float64))
    a = sp_softmax(s, axis=-1)
    qn = np.linalg.norm(q[:, :, 0].astype(np.float64), axis=-1)
    np.testing.assert_allclose(ans_v, a, rtol=1e-12)
    np.testing.assert_allclose(ans_k, a * (1 - a) * qn[..., None], rtol=1e-11)
    np.testing.assert_allclose(st["row_max"][..., 0], s.max(-1), rtol=1e-13)
    np.testing.assert_allclose(st["q_norm"][..., 0], qn, rtol=1e-13)
    np.testing.assert_allclose(st["row_max"][..., 0] + np.log(st["row_sum"][..., 0]),
                               torch.logsumexp(torch.from_numpy(s), -1).numpy(), rtol=1e-12)


@pytest.mark.parametrize("N,Nq", [(31, 31), (48, 5)])
def test_total_k_score_identity(oracle, N, Nq):
    # sum_j AnS(K_j) = sum_i ||Q_i|| (1 - sum_j A_ij^2), with A from a library masked softmax
    B, Hq, Hkv, D = 1, 4, 2, 16
    scale = 0.4
    q, k = _rand((B, Hq, Nq, D), 15), _rand((B, Hkv, N, D), 16, scale=2.0)
    ans_k, ans_v = oracle.anchor_score(q, k, scale)
    qt = torch.from_numpy(q.astype(np.float64))
    kt = torch.from_numpy(k.astype(np.float64)).repeat_interleave(Hq // Hkv, dim=1)
    s = scale * qt @ kt.transpose(-1, -2)
    a = torch.softmax(s.masked_fill(~_mask(N, Nq), -math.inf), dim=-1)      # [B,Hq,Nq,N]
    qn = qt.norm(dim=-1)
    total = (qn * (1 - (a * a).sum(-1))).reshape(B, Hkv, -1).sum(-1)
    np.testing.assert_allclose(ans_k.sum(-1), total.numpy(), rtol=1e-11)
    # and element-wise against the dense matrix (brute force over the full A)
    want_v = a.reshape(B, Hkv, -1, N).sum(2).numpy()
    want_k = (a * (1 - a) * qn[..., None]).reshape(B, Hkv, -1, N).sum(2).numpy()
    np.testing.assert_allclose(ans_v, want_v, rtol=1e-11, atol=1e-15)
    np.testing.assert_allclose(ans_k, want_k, rtol=1e-11, atol=1e-15)


def test_non_causal_flag(oracle):
    q, k = _rand((1, 2, 3, 8), 17), _rand((1, 1, 10, 8), 18)
    _, ans_v = oracle.anchor_score(q, k, 0.5, causal=False)
    a = sp_softmax(0.5 * np.einsum("bhqd,bnd->bhqn", q.astype(np.float64), k[:, 0].astype(np.float64)), axis=-1)
    np.testing.assert_allclose(ans_v[0, 0], a.sum((0, 1, 2)), rtol=1e-12)
