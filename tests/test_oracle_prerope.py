"""Pins for the oracle's rotary embedding and its decode attention on pre-RoPE keys (paper Sec. 2.1 for RoPE on Q and K,
Sec. 3.3 last paragraph for keys quantised before RoPE)."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F


def _rand(shape, seed, scale=1.0):
    return (np.random.default_rng(seed).standard_normal(shape) * scale).astype(np.float16)


def _rope_complex(x, pos, base, style):
    """The same rotation through complex multiplication: (a + i b) e^{i pos theta}.  Independent of oracle.rope."""
    x = np.asarray(x, np.float64)
    D = x.shape[-1]
    theta = np.array([base ** (-(2 * i) / D) for i in range(D // 2)])
    z = (x[..., 0::2] + 1j * x[..., 1::2]) if style == 0 else (x[..., : D // 2] + 1j * x[..., D // 2:])
    z = z * np.exp(1j * np.asarray(pos, np.float64)[..., None] * theta)
    out = np.empty_like(x)
    if style == 0:
        out[..., 0::2], out[..., 1::2] = z.real, z.imag
    else:
        out[..., : D // 2], out[..., D // 2:] = z.real, z.imag
    return out


def _sdpa(q, k, v, scale):
    qt = torch.from_numpy(np.asarray(q, dtype=np.float64))[:, :, None, :]
    kt, vt = (torch.from_numpy(np.asarray(a, dtype=np.float64)) for a in (k, v))
    G = qt.shape[1] // kt.shape[1]
    o = F.scaled_dot_product_attention(qt, kt.repeat_interleave(G, 1), vt.repeat_interleave(G, 1), scale=scale)
    return o[:, :, 0, :].numpy()


def _identity_cache(k, v, d):
    """Lossless VQ: centroid c of every sub-space = token c's sub-vector, code = token index (N <= 256)."""
    B, Hkv, N, D = k.shape
    M = D // d
    cbk = np.zeros((Hkv, M, 256, d), np.float16)
    cbv = np.zeros((Hkv, M, 256, d), np.float16)
    cbk[:, :, :N] = k[0].reshape(Hkv, N, M, d).transpose(0, 2, 1, 3)
    cbv[:, :, :N] = v[0].reshape(Hkv, N, M, d).transpose(0, 2, 1, 3)
    codes = np.ascontiguousarray(np.broadcast_to(np.arange(N, dtype=np.int32)[None, None, :, None], (B, Hkv, N, M)))
    return cbk, cbv, codes


@pytest.mark.parametrize("style", [0, 1])
def test_rope_position_zero_is_identity_and_norm_is_preserved(oracle, style):
    x = _rand((3, 5, 64), 1).astype(np.float64)
    assert np.array_equal(oracle.rope(x, np.zeros((3, 5), np.int64), 10000.0, style), x)
    pos = np.random.default_rng(2).integers(0, 200000, (3, 5))
    y = oracle.rope(x, pos, 10000.0, style)
    np.testing.assert_allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-13)
    # channel pair 0 turns by exactly pos radians (theta_0 = 1); the last pair by pos * base^(-(D-2)/D)
    a, b = (0, 1) if style == 0 else (0, 32)
    ang = np.arctan2(y[..., b], y[..., a]) - np.arctan2(x[..., b], x[..., a])
    np.testing.assert_allclose(np.mod(ang - pos + np.pi, 2 * np.pi) - np.pi, 0, atol=1e-9)


@pytest.mark.parametrize("style", [0, 1])
def test_rope_matches_complex_rotation_and_relative_position(oracle, style):
    x, y = _rand((4, 7, 128), 3).astype(np.float64), _rand((4, 7, 128), 4).astype(np.float64)
    pos = np.random.default_rng(5).integers(0, 131072, (4, 7))
    np.testing.assert_allclose(oracle.rope(x, pos, 500000.0, style), _rope_complex(x, pos, 500000.0, style), rtol=0, atol=1e-9)
    # q . RoPE_p(k) = RoPE_{-p}(q) . k, and only the distance between the two positions matters
    lhs = np.einsum("...d,...d->...", x, oracle.rope(y, pos, 10000.0, style))
    rhs = np.einsum("...d,...d->...", oracle.rope(x, -pos, 10000.0, style), y)
    np.testing.assert_allclose(lhs, rhs, rtol=1e-10, atol=1e-10)
    shift = 977
    a = np.einsum("...d,...d->...", oracle.rope(x, pos + 3, 10000.0, style), oracle.rope(y, pos, 10000.0, style))
    b = np.einsum("...d,...d->...", oracle.rope(x, pos + 3 + shift, 10000.0, style), oracle.rope(y, pos + shift, 10000.0, style))
    np.testing.assert_allclose(a, b, rtol=1e-9, atol=1e-9)


@pytest.mark.parametrize("style,pos0", [(0, 0), (1, 0), (1, 5000)])
def test_prerope_identity_codebook_is_attention_on_rotated_keys(oracle, style, pos0):
    """Lossless codes: the result must be library attention on keys rotated (by the independent complex form) to their
    positions; a mistake in the sign, the pairing or the position of the rotation inside the oracle fails here."""
    B, Hq, Hkv, N, D, d = 1, 8, 2, 200, 64, 8
    q, k, v = _rand((B, Hq, D), 11), _rand((B, Hkv, N, D), 12, 2.0), _rand((B, Hkv, N, D), 13)
    cbk, cbv, codes = _identity_cache(k, v, d)
    none_i, none_r = np.zeros((B, Hkv, 0), np.int32), np.zeros((B, Hkv, 0, D), np.float16)
    scale = 1 / math.sqrt(D)
    out = oracle.decode_attn_prerope(q, codes, codes, cbk, cbv, none_i, none_r, none_i, none_r, scale, 10000.0, style, pos0)
    k_rot = _rope_complex(k, pos0 + np.arange(N)[None, None, :], 10000.0, style)
    np.testing.assert_allclose(out, _sdpa(q, k_rot, v, scale), rtol=1e-9, atol=1e-11)
    # and it is NOT attention on the unrotated keys (the rotation does something at this size)
    assert np.abs(out - _sdpa(q, k, v, scale)).max() > 1e-3


def test_prerope_anchors_override_codes_before_the_rotation(oracle):
    """Mixed cache: K anchors are FP16 rows stored before RoPE, so they are rotated like every other key; V anchors
    replace the centroids of their token.  Checked against library attention on hand-built K_eff, V_eff."""
    B, Hq, Hkv, N, D, d = 2, 4, 2, 150, 32, 4
    M = D // d
    rng = np.random.default_rng(21)
    q = _rand((B, Hq, D), 22)
    cbk, cbv = _rand((Hkv, M, 256, d), 23, 2.0), _rand((Hkv, M, 256, d), 24)
    ck, cv = rng.integers(0, 256, (B, Hkv, N, M)).astype(np.int32), rng.integers(0, 256, (B, Hkv, N, M)).astype(np.int32)
    ik = np.sort(rng.permuted(np.tile(np.arange(N), (B, Hkv, 1)), axis=-1)[..., :9], axis=-1).astype(np.int32)
    iv = np.sort(rng.permuted(np.tile(np.arange(N), (B, Hkv, 1)), axis=-1)[..., :14], axis=-1).astype(np.int32)
    rk, rv = _rand((B, Hkv, 9, D), 25, 3.0), _rand((B, Hkv, 14, D), 26)
    k_eff = np.empty((B, Hkv, N, D))
    v_eff = np.empty((B, Hkv, N, D))
    for g in range(Hkv):
        for m in range(M):
            k_eff[:, g, :, m * d:(m + 1) * d] = cbk[g, m].astype(np.float64)[ck[:, g, :, m]]
            v_eff[:, g, :, m * d:(m + 1) * d] = cbv[g, m].astype(np.float64)[cv[:, g, :, m]]
    np.put_along_axis(k_eff, ik[..., None].astype(np.int64), rk.astype(np.float64), axis=2)
    np.put_along_axis(v_eff, iv[..., None].astype(np.int64), rv.astype(np.float64), axis=2)
    pos0 = 123
    k_rot = _rope_complex(k_eff, pos0 + np.arange(N)[None, None, :], 10000.0, 1)
    out = oracle.decode_attn_prerope(q, ck, cv, cbk, cbv, ik, rk, iv, rv, 0.2, 10000.0, 1, pos0)
    np.testing.assert_allclose(out, _sdpa(q, k_rot, v_eff, 0.2), rtol=1e-9, atol=1e-11)


def test_prerope_shift_of_all_positions_with_the_query(oracle):
    """Rotating the query by s more and moving every key s positions on leaves the output unchanged."""
    B, Hq, Hkv, N, D, d = 1, 4, 1, 120, 64, 8
    M = D // d
    rng = np.random.default_rng(31)
    q = _rand((B, Hq, D), 32).astype(np.float64)
    cbk, cbv = _rand((Hkv, M, 256, d), 33, 2.0), _rand((Hkv, M, 256, d), 34)
    ck, cv = rng.integers(0, 256, (B, Hkv, N, M)).astype(np.int32), rng.integers(0, 256, (B, Hkv, N, M)).astype(np.int32)
    none_i, none_r = np.zeros((B, Hkv, 0), np.int32), np.zeros((B, Hkv, 0, D), np.float16)
    qa = oracle.rope(q, np.full((B, Hq), N), 10000.0, 0)
    qb = oracle.rope(q, np.full((B, Hq), N + 4000), 10000.0, 0)
    a = oracle.decode_attn_prerope(qa, ck, cv, cbk, cbv, none_i, none_r, none_i, none_r, 0.15, 10000.0, 0, 0)
    b = oracle.decode_attn_prerope(qb, ck, cv, cbk, cbv, none_i, none_r, none_i, none_r, 0.15, 10000.0, 0, 4000)
    np.testing.assert_allclose(a, b, rtol=1e-8, atol=1e-10)
