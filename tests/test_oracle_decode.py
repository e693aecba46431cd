"""Pins for the oracle's decode attention over VQ codes + FP16 anchors (paper Sec. 2.1 Attn, Sec. 3 Fig. 2(b))."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F
from scipy.special import softmax as sp_softmax


def _rand(shape, seed, scale=1.0):
    return (np.random.default_rng(seed).standard_normal(shape) * scale).astype(np.float16)


def _sdpa(q, k, v, scale):
    """Library attention, one query row per head, GQA by repeating KV heads (h -> h // G), fp64."""
    qt = torch.from_numpy(np.asarray(q, dtype=np.float64))[:, :, None, :]
    kt, vt = (torch.from_numpy(np.asarray(a, dtype=np.float64)) for a in (k, v))
    G = qt.shape[1] // kt.shape[1]
    o = F.scaled_dot_product_attention(qt, kt.repeat_interleave(G, 1), vt.repeat_interleave(G, 1), scale=scale)
    return o[:, :, 0, :].numpy()


def _dequant(codes, cb):
    """codes [B,Hkv,N,M], cb [Hkv,M,C,d] -> [B,Hkv,N,M*d] by table lookup."""
    B, Hkv, N, M = codes.shape
    out = np.empty((B, Hkv, N, M, cb.shape[-1]), dtype=cb.dtype)
    for g in range(Hkv):
        for m in range(M):
            out[:, g, :, m] = cb[g, m][codes[:, g, :, m]]
    return out.reshape(B, Hkv, N, -1)


def _empty_anchors(B, Hkv, D):
    return np.zeros((B, Hkv, 0), np.int32), np.zeros((B, Hkv, 0, D), np.float16)


def test_identity_codebook_is_plain_attention(oracle):
    # centroid c of every sub-space = token c's sub-vector, code = token index: VQ is lossless
    B, Hq, Hkv, N, D, d = 1, 8, 2, 200, 32, 8
    M = D // d
    q, k, v = _rand((B, Hq, D), 1), _rand((B, Hkv, N, D), 2, 2.0), _rand((B, Hkv, N, D), 3)
    C = 256
    cbk = np.zeros((Hkv, M, C, d), np.float16)
    cbv = np.zeros((Hkv, M, C, d), np.float16)
    cbk[:, :, :N] = k[0].reshape(Hkv, N, M, d).transpose(0, 2, 1, 3)
    cbv[:, :, :N] = v[0].reshape(Hkv, N, M, d).transpose(0, 2, 1, 3)
    codes = np.broadcast_to(np.arange(N, dtype=np.int32)[None, None, :, None], (B, Hkv, N, M))
    ik, rk = _empty_anchors(B, Hkv, D)
    out = oracle.decode_attn(q, codes, codes, cbk, cbv, ik, rk, ik, rk, 1 / math.sqrt(D))
    np.testing.assert_allclose(out, _sdpa(q, k, v, 1 / math.sqrt(D)), rtol=1e-11, atol=1e-13)


def test_all_tokens_anchored_is_plain_attention(oracle):
    # anchor ratio 100 %: codes are ignored entirely
    B, Hq, Hkv, N, D, d = 2, 4, 2, 77, 16, 4
    M = D // d
    q, k, v = _rand((B, Hq, D), 4), _rand((B, Hkv, N, D), 5, 2.0), _rand((B, Hkv, N, D), 6)
    cbk, cbv = _rand((Hkv, M, 256, d), 7), _rand((Hkv, M, 256, d), 8)
    codes_k = np.random.default_rng(9).integers(0, 256, (B, Hkv, N, M)).astype(np.int32)
    codes_v = np.random.default_rng(10).integers(0, 256, (B, Hkv, N, M)).astype(np.int32)
    idx = np.broadcast_to(np.arange(N, dtype=np.int32), (B, Hkv, N))
    out = oracle.decode_attn(q, codes_k, codes_v, cbk, cbv, idx, k, idx, v, 0.3)
    np.testing.assert_allclose(out, _sdpa(q, k, v, 0.3), rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("d,C,D", [(4, 256, 32), (8, 256, 32), (16, 256, 32), (32, 4096, 128), (16, 4096, 128)])
def test_mixed_codes_and_separate_anchor_sets(oracle, d, C, D):
    # K anchors and V anchors are different sets; everything else comes from the code tables
    B, Hq, Hkv, N = 2, 8, 2, 150
    M = D // d
    rng = np.random.default_rng(11 + d)
    q = _rand((B, Hq, D), 12)
    cbk, cbv = _rand((Hkv, M, C, d), 13, 2.0), _rand((Hkv, M, C, d), 14)
    codes_k = rng.integers(0, C, (B, Hkv, N, M)).astype(np.int32)
    codes_v = rng.integers(0, C, (B, Hkv, N, M)).astype(np.int32)
    k_k, k_v = 9, 14
    ik = np.stack([[np.sort(rng.choice(N, k_k, replace=False)) for _ in range(Hkv)] for _ in range(B)]).astype(np.int32)
    iv = np.stack([[np.sort(rng.choice(N, k_v, replace=False)) for _ in range(Hkv)] for _ in range(B)]).astype(np.int32)
    rk, rv = _rand((B, Hkv, k_k, D), 15, 3.0), _rand((B, Hkv, k_v, D), 16)
    keff, veff = _dequant(codes_k, cbk), _dequant(codes_v, cbv)
    for b in range(B):
        for g in range(Hkv):
            keff[b, g, ik[b, g]] = rk[b, g]
            veff[b, g, iv[b, g]] = rv[b, g]
    out, ex = oracle.decode_attn(q, codes_k, codes_v, cbk, cbv, ik, rk, iv, rv, 0.2, want_lse=True, want_ans=True)
    np.testing.assert_allclose(out, _sdpa(q, keff, veff, 0.2), rtol=1e-11, atol=1e-13)
    # log-sum-exp and the decode-time Anchor Score (Eq. (4) with one query row) from a library softmax
    G = Hq // Hkv
    s = 0.2 * np.einsum("bgud,bgnd->bgun", q.astype(np.float64).reshape(B, Hkv, G, D), keff.astype(np.float64))
    a = sp_softmax(s, axis=-1)
    qn = np.linalg.norm(q.astype(np.float64), axis=-1).reshape(B, Hkv, G)
    np.testing.assert_allclose(ex["lse"].reshape(B, Hkv, G), torch.logsumexp(torch.from_numpy(s), -1).numpy(), rtol=1e-12)
    np.testing.assert_allclose(ex["ans_v"], a.sum(2), rtol=1e-11)
    np.testing.assert_allclose(ex["ans_k"], (a * (1 - a) * qn[..., None]).sum(2), rtol=1e-11)
    # ... which must agree with the prefill-form scorer run with a single, unmasked query on K_eff
    ak, av = oracle.anchor_score(q[:, :, None, :], keff, 0.2, causal=False)
    np.testing.assert_allclose(ex["ans_k"], ak, rtol=1e-11)
    np.testing.assert_allclose(ex["ans_v"], av, rtol=1e-11)


def test_token_permutation_invariance(oracle):
    B, Hq, Hkv, N, D, d = 1, 4, 1, 60, 16, 8
    M = D // d
    rng = np.random.default_rng(20)
    q = _rand((B, Hq, D), 21)
    cbk, cbv = _rand((Hkv, M, 256, d), 22), _rand((Hkv, M, 256, d), 23)
    ck = rng.integers(0, 256, (B, Hkv, N, M)).astype(np.int32)
    cv = rng.integers(0, 256, (B, Hkv, N, M)).astype(np.int32)
    ik = np.sort(rng.choice(N, 6, replace=False)).astype(np.int32)[None, None]
    rk, rv = _rand((B, Hkv, 6, D), 24), _rand((B, Hkv, 6, D), 25)
    out = oracle.decode_attn(q, ck, cv, cbk, cbv, ik, rk, ik, rv, 0.25)
    perm = rng.permutation(N)                      # new position p holds old token perm[p]
    inv = np.argsort(perm)
    ik2 = inv[ik[0, 0]]
    order = np.argsort(ik2)
    out2 = oracle.decode_attn(q, ck[:, :, perm], cv[:, :, perm], cbk, cbv,
                              ik2[order].astype(np.int32)[None, None], rk[:, :, order],
                              ik2[order].astype(np.int32)[None, None], rv[:, :, order], 0.25)
    np.testing.assert_allclose(out2, out, rtol=1e-11, atol=1e-14)


def test_halves_merge_by_log_sum_exp(oracle):
    B, Hq, Hkv, N, D, d = 1, 2, 1, 64, 16, 4
    M = D // d
    rng = np.random.default_rng(30)
    q = _rand((B, Hq, D), 31)
    cbk, cbv = _rand((Hkv, M, 256, d), 32, 2.0), _rand((Hkv, M, 256, d), 33)
    ck = rng.integers(0, 256, (B, Hkv, N, M)).astype(np.int32)
    cv = rng.integers(0, 256, (B, Hkv, N, M)).astype(np.int32)
    e_i, e_r = _empty_anchors(B, Hkv, D)
    full = oracle.decode_attn(q, ck, cv, cbk, cbv, e_i, e_r, e_i, e_r, 0.3)
    parts = [oracle.decode_attn(q, ck[:, :, sl], cv[:, :, sl], cbk, cbv, e_i, e_r, e_i, e_r, 0.3, want_lse=True)
             for sl in (slice(0, 20), slice(20, N))]
    l0, l1 = parts[0][1]["lse"], parts[1][1]["lse"]
    w0 = 1 / (1 + np.exp(l1 - l0))
    merged = w0[..., None] * parts[0][0] + (1 - w0)[..., None] * parts[1][0]
    np.testing.assert_allclose(merged, full, rtol=1e-11, atol=1e-14)


def test_rejects_out_of_range_or_unsorted_anchors(oracle):
    B, Hq, Hkv, N, D, d = 1, 1, 1, 8, 8, 8
    q = _rand((B, Hq, D), 40)
    cb = _rand((Hkv, 1, 256, d), 41)
    c = np.zeros((B, Hkv, N, 1), np.int32)
    rows = _rand((B, Hkv, 2, D), 42)
    with pytest.raises(ValueError):
        oracle.decode_attn(q, c, c, cb, cb, np.array([[[3, 1]]], np.int32), rows, np.array([[[1, 3]]], np.int32), rows, 1.0)
    with pytest.raises(RuntimeError):
        oracle.decode_attn(q, c, c, cb, cb, np.array([[[1, 8]]], np.int32), rows, np.array([[[1, 3]]], np.int32), rows, 1.0)
