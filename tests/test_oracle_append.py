"""Pins for the oracle's decode append with an FP16 sliding window (paper Sec. 3.2, last paragraph; Sec. 4: window 32).

The append is checked against things that do not go through the oracle's own routines: nearest centroids by brute
force in numpy, and plain softmax attention over K/V rows assembled by hand (original FP16 rows inside the window and
at the prefill anchors, centroids elsewhere).
"""
import numpy as np
import pytest

from workloads import make_codebooks, make_decode_query, make_qkv, normal_fp16


def _brute_codes(x, cb):
    """x [B,Hkv,D] fp16, cb [Hkv,M,C,d] -> nearest centroid per sub-vector, lowest index on ties (fp64)."""
    B, Hkv, D = x.shape
    _, M, C, d = cb.shape
    xs = x.astype(np.float64).reshape(B, Hkv, M, 1, d)
    dist = ((xs - cb.astype(np.float64)[None]) ** 2).sum(-1)          # [B,Hkv,M,C]
    return dist.argmin(-1)


def _plain_attention(q, k_eff, v_eff, scale, G):
    B, Hq, D = q.shape
    out = np.zeros((B, Hq, D))
    for b in range(B):
        for h in range(Hq):
            s = scale * k_eff[b, h // G].astype(np.float64) @ q[b, h].astype(np.float64)
            p = np.exp(s - s.max())
            out[b, h] = (p / p.sum()) @ v_eff[b, h // G].astype(np.float64)
    return out


def _dequant(codes, cb):
    """codes [B,Hkv,N,M], cb [Hkv,M,C,d] -> rows [B,Hkv,N,M*d]"""
    B, Hkv, N, M = codes.shape
    out = np.zeros((B, Hkv, N, M * cb.shape[-1]), np.float16)
    for g in range(Hkv):
        for m in range(M):
            out[:, g, :, m * cb.shape[-1]:(m + 1) * cb.shape[-1]] = cb[g, m][codes[:, g, :, m]]
    return out


@pytest.mark.parametrize("d,W", [(8, 4), (16, 3), (4, 1), (8, 0)])
def test_append_matches_hand_built_cache(oracle, d, W):
    B, Hq, Hkv, N0, T, k_a = 2, 4, 2, 40, 9, 3
    G = Hq // Hkv
    scale = 1 / np.sqrt(128)
    _, k_all, v_all = make_qkv(5 + d, B, Hq, Hkv, N0 + T, 1, 128)
    cbk, cbv = make_codebooks(5 + d, k_all, d, 256, "k", max_sample=64), make_codebooks(5 + d, v_all, d, 256, "v", max_sample=64)
    M = 128 // d
    N_cap = N0 + T
    codes_k = np.zeros((B, Hkv, N_cap, M), np.int32)
    codes_v = np.zeros((B, Hkv, N_cap, M), np.int32)
    codes_k[:, :, :N0] = oracle.encode(k_all[:, :, :N0], cbk)
    codes_v[:, :, :N0] = oracle.encode(v_all[:, :, :N0], cbv)
    # prefill anchors: the first k_a even positions; the window: the last W prefill tokens
    anchors = np.arange(0, 2 * k_a, 2)
    win = np.arange(N0 - W, N0)
    idx = np.broadcast_to(np.concatenate([anchors, win]), (B, Hkv, k_a + W)).astype(np.int32).copy()
    idx_k, idx_v = idx.copy(), idx.copy()
    rows_k = np.take_along_axis(k_all, idx[..., None].astype(np.int64), axis=2).copy()
    rows_v = np.take_along_axis(v_all, idx[..., None].astype(np.int64), axis=2).copy()
    N = N0
    for t in range(T):
        N = oracle.append_token(k_all[:, :, N0 + t], v_all[:, :, N0 + t], N, W, cbk, cbv, codes_k, codes_v,
                                idx_k, rows_k, idx_v, rows_v)
        assert N == N0 + t + 1
        # the window is the last W positions and holds exactly the rows that were fed
        for idx_x, rows_x, src in ((idx_k, rows_k, k_all), (idx_v, rows_v, v_all)):
            assert (idx_x[..., :k_a] == anchors).all()
            assert (idx_x[..., k_a:] == np.arange(N - W, N)).all()
            assert (rows_x[:, :, k_a:] == src[:, :, N - W:N]).all()
        # every token that left the window (or never was in one) carries its brute-force codes
        for pos in range(N0 - W, N - W):
            assert (codes_k[:, :, pos] == _brute_codes(k_all[:, :, pos], cbk)).all()
            assert (codes_v[:, :, pos] == _brute_codes(v_all[:, :, pos], cbv)).all()
        # decode over the cache == plain attention over hand-assembled rows
        k_eff, v_eff = _dequant(codes_k[:, :, :N], cbk), _dequant(codes_v[:, :, :N], cbv)
        keep = np.concatenate([anchors, np.arange(N - W, N)]).astype(int)
        k_eff[:, :, keep] = k_all[:, :, keep]
        v_eff[:, :, keep] = v_all[:, :, keep]
        q = make_decode_query(100 + t, B, Hq, 128)
        want = _plain_attention(q, k_eff, v_eff, scale, G)
        got = oracle.decode_attn(q, codes_k[:, :, :N], codes_v[:, :, :N], cbk, cbv, idx_k, rows_k, idx_v, rows_v, scale)
        assert np.allclose(got, want, rtol=1e-9, atol=1e-12)
