"""CPU oracle for the AnTKV online path: TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It shares no code with the HIP path and imports nothing from it.

The arithmetic lives in antkv_oracle.c (plain C, fp64); this module marshals numpy
arrays into it and adds the top-k step, which is a stable library sort.

  encode(x, cb)                 paper Sec. 3.1 (sub-vector -> nearest centroid)
  anchor_score(q, k, scale)     paper Eq. (4), causal prefill/window form
  topk(scores, k)               keep the k highest scores (Sec. 3, "anchor tokens")
  decode_attn(...)              Attn (Sec. 2.1) over codes + FP16 anchors, and the
                                decode-time Anchor Score (Sec. 3.2, last paragraph)
  append_token(...)             decode append with an FP16 sliding window (Sec. 3.2, last
                                paragraph; window of 32 in Sec. 4)
  kmeans_update / kmeans_step   one iteration of the offline token-weighted k-means (Sec. 3.1, "Offline
                                Token-Aware Centroids Learning"): nearest-centroid assignment, then weighted means
  prefill_attn(q, k, v, scale)  causal Attn (Sec. 2.1) over the prompt with the softmax row statistics
                                that the Anchor Score pass reuses (Alg. 1, first step)
  rope(x, pos, base, style)     rotary position embedding (Sec. 2.1, the tilde on Q and K)
  decode_attn_prerope(...)      decode attention on a cache whose keys were stored before RoPE (Sec. 3.3, last
                                paragraph: the pre-RoPE strategy): every key is rotated to its position when used
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "antkv_oracle.c")
_LIB = os.path.join(_HERE, "libantkv_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (host code only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-march=x86-64-v3", "-fopenmp", "-fPIC", "-shared", "-Wall",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build()
        lib = ctypes.CDLL(_LIB)
        i64, dbl, vp = ctypes.c_int64, ctypes.c_double, ctypes.c_void_p
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_encode.restype = ctypes.c_int
        lib.oracle_encode.argtypes = [vp, vp, i64, i64, i64, i64, i64, i64, vp, vp]
        lib.oracle_anchor_score.restype = ctypes.c_int
        lib.oracle_anchor_score.argtypes = [vp, vp, i64, i64, i64, i64, i64, i64, dbl, ctypes.c_int,
                                            vp, vp, vp, vp, vp]
        lib.oracle_decode_attn.restype = ctypes.c_int
        lib.oracle_decode_attn.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, vp, vp, i64,
                                           i64, i64, i64, i64, i64, i64, i64, dbl, vp, vp, vp, vp]
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _f32(a) -> np.ndarray:
    """fp16 (or any float) array -> contiguous fp32 holding the same values exactly."""
    a = np.asarray(a)
    if a.dtype == np.float64:
        raise TypeError("oracle inputs are fp16-valued; pass float16 or float32")
    return np.ascontiguousarray(a, dtype=np.float32)


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def encode(x, cb, want_margin: bool = False):
    """x [B,Hkv,n,D], cb [Hkv,M,C,d] -> codes int32 [B,Hkv,n,M] (and margins fp64)."""
    x32, cb32 = _f32(x), _f32(cb)
    B, Hkv, n, D = x32.shape
    Hc, M, C, d = cb32.shape
    assert Hc == Hkv and M * d == D
    codes = np.empty((B, Hkv, n, M), dtype=np.int32)
    margin = np.empty((B, Hkv, n, M), dtype=np.float64) if want_margin else None
    rc = _load().oracle_encode(_ptr(x32), _ptr(cb32), B, Hkv, n, D, d, C, _ptr(codes), _ptr(margin))
    if rc != 0:
        raise RuntimeError(f"oracle_encode failed: {rc}")
    return (codes, margin) if want_margin else codes


def anchor_score(q, k, scale: float, causal: bool = True, want_stats: bool = False):
    """q [B,Hq,Nq,D] = the last Nq positions, k [B,Hkv,N,D] -> (AnS_K, AnS_V) fp64 [B,Hkv,N]."""
    q32, k32 = _f32(q), _f32(k)
    B, Hq, Nq, D = q32.shape
    Bk, Hkv, N, Dk = k32.shape
    assert Bk == B and Dk == D
    ans_k = np.zeros((B, Hkv, N), dtype=np.float64)
    ans_v = np.zeros((B, Hkv, N), dtype=np.float64)
    stats = [np.zeros((B, Hq, Nq), dtype=np.float64) for _ in range(3)] if want_stats else [None] * 3
    rc = _load().oracle_anchor_score(_ptr(q32), _ptr(k32), B, Hq, Hkv, N, Nq, D, float(scale),
                                     1 if causal else 0, _ptr(ans_k), _ptr(ans_v),
                                     _ptr(stats[0]), _ptr(stats[1]), _ptr(stats[2]))
    if rc != 0:
        raise RuntimeError(f"oracle_anchor_score failed: {rc}")
    if want_stats:
        return ans_k, ans_v, {"row_max": stats[0], "row_sum": stats[1], "q_norm": stats[2]}
    return ans_k, ans_v


def topk(scores, k: int, want_margin: bool = False):
    """Indices of the k largest scores per row, ties to the lower index, ascending output.

    scores [..., N] -> idx int32 [..., k].  margin [..., N] is |score - tau| / max(|tau|, 1e-30)
    with tau halfway between the k-th and (k+1)-th largest score (inf if k is 0 or N):
    candidates with a tiny margin are the ones a differently-rounded scorer may swap.
    """
    s = np.asarray(scores, dtype=np.float64)
    N = s.shape[-1]
    assert 0 <= k <= N
    flat = s.reshape(-1, N)
    idx = np.empty((flat.shape[0], k), dtype=np.int32)
    margin = np.full(flat.shape, np.inf) if want_margin else None
    for r in range(flat.shape[0]):
        order = np.argsort(-flat[r], kind="stable")  # descending score, ascending index on ties
        idx[r] = np.sort(order[:k]).astype(np.int32)
        if want_margin and 0 < k < N:
            tau = 0.5 * (flat[r, order[k - 1]] + flat[r, order[k]])
            margin[r] = np.abs(flat[r] - tau) / max(abs(tau), 1e-30)
    idx = idx.reshape(s.shape[:-1] + (k,))
    if want_margin:
        return idx, margin.reshape(s.shape)
    return idx


def decode_attn(q, codes_k, codes_v, cb_k, cb_v, idx_k, rows_k, idx_v, rows_v, scale: float,
                want_lse: bool = False, want_ans: bool = False):
    """Decode attention over codes + anchors.  Returns out fp64 [B,Hq,D] (+ extras dict)."""
    q32, cbk, cbv = _f32(q), _f32(cb_k), _f32(cb_v)
    B, Hq, D = q32.shape
    ck = np.ascontiguousarray(codes_k, dtype=np.int32)
    cv = np.ascontiguousarray(codes_v, dtype=np.int32)
    _, Hkv, N, M = ck.shape
    Hc, Mc, C, d = cbk.shape
    assert Hc == Hkv and Mc == M and M * d == D and cbv.shape == cbk.shape and cv.shape == ck.shape
    ik = np.ascontiguousarray(idx_k, dtype=np.int32).reshape(B, Hkv, -1)
    iv = np.ascontiguousarray(idx_v, dtype=np.int32).reshape(B, Hkv, -1)
    k_k, k_v = ik.shape[-1], iv.shape[-1]
    rk = _f32(rows_k).reshape(B, Hkv, k_k, D)
    rv = _f32(rows_v).reshape(B, Hkv, k_v, D)
    for name, ix in (("idx_k", ik), ("idx_v", iv)):
        if ix.shape[-1] > 1 and not np.all(np.diff(ix, axis=-1) > 0):
            raise ValueError(f"{name} must be strictly ascending")
    out = np.zeros((B, Hq, D), dtype=np.float64)
    lse = np.zeros((B, Hq), dtype=np.float64) if want_lse else None
    ans_k = np.zeros((B, Hkv, N), dtype=np.float64) if want_ans else None
    ans_v = np.zeros((B, Hkv, N), dtype=np.float64) if want_ans else None
    rc = _load().oracle_decode_attn(_ptr(q32), _ptr(ck), _ptr(cv), _ptr(cbk), _ptr(cbv),
                                    _ptr(ik), _ptr(rk), k_k, _ptr(iv), _ptr(rv), k_v,
                                    B, Hq, Hkv, N, D, d, C, float(scale),
                                    _ptr(out), _ptr(lse), _ptr(ans_k), _ptr(ans_v))
    if rc != 0:
        raise RuntimeError(f"oracle_decode_attn failed: {rc}")
    extras = {}
    if want_lse:
        extras["lse"] = lse
    if want_ans:
        extras["ans_k"], extras["ans_v"] = ans_k, ans_v
    return (out, extras) if extras else out


def append_token(k_new, v_new, N: int, W: int, cb_k, cb_v, codes_k, codes_v, idx_k, rows_k, idx_v, rows_v,
                 want_margin: bool = False):
    """One decode append with a sliding window of W full-precision tokens (paper Sec. 3.2, last paragraph).

    The window is the last W entries of both anchor lists (positions N-W .. N-1).  In place: the oldest window
    token is encoded to its codes at position N-W, the window moves one place down, the new rows k_new / v_new
    [B,Hkv,D] become the last entry with position N.  W == 0: the new rows are encoded straight to position N.
    Returns N + 1 (and, if asked, the near-tie margins of the two code rows that were written).
    """
    if W == 0:
        ck, mk = encode(np.asarray(k_new)[:, :, None, :], cb_k, want_margin=True)
        cv, mv = encode(np.asarray(v_new)[:, :, None, :], cb_v, want_margin=True)
        codes_k[:, :, N] = ck[:, :, 0]
        codes_v[:, :, N] = cv[:, :, 0]
        return (N + 1, mk[:, :, 0], mv[:, :, 0]) if want_margin else N + 1
    margins = []
    for codes, cb, idx, rows, new in ((codes_k, cb_k, idx_k, rows_k, k_new), (codes_v, cb_v, idx_v, rows_v, v_new)):
        k = idx.shape[-1]
        first = k - W                                   # the window's oldest entry
        assert (idx[..., first:] == np.arange(N - W, N)).all(), "the window must be the last W positions"
        c, m = encode(rows[:, :, first:first + 1, :], cb, want_margin=True)
        codes[:, :, N - W] = c[:, :, 0]
        margins.append(m[:, :, 0])
        rows[:, :, first:k - 1] = rows[:, :, first + 1:k].copy()
        rows[:, :, k - 1] = new
        idx[..., first:] = np.arange(N - W + 1, N + 1)
    return (N + 1, margins[0], margins[1]) if want_margin else N + 1


def prefill_attn(q, k, v, scale: float):
    """Causal attention over the prompt (paper Sec. 2.1) with the row statistics of Alg. 1's first step.

    q [B,Hq,Nq,D] = the last Nq positions, k and v [B,Hkv,N,D]; query head h reads KV head h // (Hq // Hkv).
    Query row i sits at position N - Nq + i and sees the keys 0 .. N - Nq + i.
    Returns out fp64 [B,Hq,Nq,D], row_max [B,Hq,Nq] = max_j scale*S_ij, row_sum = sum_j exp(scale*S_ij - row_max).
    Written as the definition: the whole score matrix of one head at a time, fp64.
    """
    q64, k64, v64 = (np.asarray(a).astype(np.float64) for a in (q, k, v))
    B, Hq, Nq, D = q64.shape
    _, Hkv, N, _ = k64.shape
    G = Hq // Hkv
    out = np.zeros((B, Hq, Nq, D))
    row_max = np.zeros((B, Hq, Nq))
    row_sum = np.zeros((B, Hq, Nq))
    pos = N - Nq + np.arange(Nq)
    visible = np.arange(N)[None, :] <= pos[:, None]
    for b in range(B):
        for h in range(Hq):
            s = scale * (q64[b, h] @ k64[b, h // G].T)
            s = np.where(visible, s, -np.inf)
            m = s.max(axis=1)
            e = np.exp(s - m[:, None])
            l = e.sum(axis=1)
            out[b, h] = (e / l[:, None]) @ v64[b, h // G]
            row_max[b, h], row_sum[b, h] = m, l
    return out, row_max, row_sum


def kmeans_update(x, w, codes, cb_old):
    """Centroid update of token-weighted k-means (paper Sec. 3.1: clustering of the sub-vectors with one weight per
    token, the weight standing for that token's error-propagation factor).

    x [B,Hkv,n,D], w [B,Hkv,n] >= 0, codes int [B,Hkv,n,M], cb_old [Hkv,M,C,d].  Per (KV head, sub-space):
    centroid c becomes sum_j w_j x_j / sum_j w_j over the tokens j (of all B sequences) assigned to it; a centroid
    whose assigned weight is zero keeps its old value.  Returns (cb_new fp64 [Hkv,M,C,d], wsum fp64 [Hkv,M,C],
    objective fp64 [Hkv,M] = sum_j w_j ||x_j - cb_old[code_j]||^2, the weighted distortion of the assignment).
    """
    x64, w64, cb64 = np.asarray(x).astype(np.float64), np.asarray(w).astype(np.float64), np.asarray(cb_old).astype(np.float64)
    codes = np.asarray(codes).astype(np.int64)
    Hkv, M, C, d = cb64.shape
    cb_new = cb64.copy()
    wsum = np.zeros((Hkv, M, C))
    objective = np.zeros((Hkv, M))
    for g in range(Hkv):
        ws = w64[:, g].reshape(-1)
        for m in range(M):
            xs = x64[:, g, :, m * d:(m + 1) * d].reshape(-1, d)
            cs = codes[:, g, :, m].reshape(-1)
            sums = np.zeros((C, d))
            np.add.at(sums, cs, ws[:, None] * xs)
            tot = np.bincount(cs, weights=ws, minlength=C)
            hit = tot > 0
            cb_new[g, m, hit] = sums[hit] / tot[hit, None]
            wsum[g, m] = tot
            objective[g, m] = (ws * ((xs - cb64[g, m, cs]) ** 2).sum(axis=1)).sum()
    return cb_new, wsum, objective


def kmeans_step(x, w, cb):
    """One Lloyd iteration of the token-weighted k-means: assign every sub-vector to its nearest centroid (the online
    encode, Sec. 3.1), then kmeans_update.  Returns (cb_new, codes, wsum, objective)."""
    codes = encode(x, cb)
    cb_new, wsum, objective = kmeans_update(x, w, codes, cb)
    return cb_new, codes, wsum, objective


def rope(x, pos, base: float = 10000.0, style: int = 0):
    """Rotary position embedding of the rows of x (fp64 [..., D]) at integer positions pos (broadcast over the leading
    axes): channel pair i = 0 .. D/2-1 is rotated by the angle pos * base^(-2 i / D).  style 0 pairs the channels
    (2 i, 2 i + 1), style 1 pairs (i, i + D/2).  Written out as the 2 x 2 rotation of each pair."""
    x = np.asarray(x, dtype=np.float64)
    D = x.shape[-1]
    i = np.arange(D // 2, dtype=np.float64)
    ang = np.asarray(pos, dtype=np.float64)[..., None] * base ** (-2.0 * i / D)
    c, s_ = np.cos(ang), np.sin(ang)
    out = np.empty_like(x)
    if style == 0:
        a, b = x[..., 0::2], x[..., 1::2]
        out[..., 0::2] = a * c - b * s_
        out[..., 1::2] = a * s_ + b * c
    else:
        a, b = x[..., : D // 2], x[..., D // 2:]
        out[..., : D // 2] = a * c - b * s_
        out[..., D // 2:] = a * s_ + b * c
    return out


def decode_attn_prerope(q, codes_k, codes_v, cb_k, cb_v, idx_k, rows_k, idx_v, rows_v, scale: float,
                        rope_base: float = 10000.0, rope_style: int = 0, pos0: int = 0):
    """Decode attention over a cache that holds the keys as they were BEFORE RoPE (coded or, for anchor tokens, as FP16
    rows): K_eff[j] = RoPE_{pos0 + j}(rows_k[slot] if j is a K anchor else the centroids of codes_k[j]); the values and
    the query are used as given (the query already carries its own rotation).  out = softmax_j(scale q . K_eff[j]) V_eff.
    The definition written out in fp64; returns out [B, Hq, D]."""
    q64, cbk, cbv = np.asarray(q, np.float64), np.asarray(cb_k, np.float64), np.asarray(cb_v, np.float64)
    ck, cv = np.asarray(codes_k).astype(np.int64), np.asarray(codes_v).astype(np.int64)
    B, Hq, D = q64.shape
    _, Hkv, N, M = ck.shape
    G = Hq // Hkv
    ik = np.asarray(idx_k).reshape(B, Hkv, -1).astype(np.int64)
    iv = np.asarray(idx_v).reshape(B, Hkv, -1).astype(np.int64)
    rk = np.asarray(rows_k, np.float64).reshape(B, Hkv, ik.shape[-1], D)
    rv = np.asarray(rows_v, np.float64).reshape(B, Hkv, iv.shape[-1], D)
    out = np.zeros((B, Hq, D))
    pos = pos0 + np.arange(N)
    for b in range(B):
        for g in range(Hkv):
            k_eff = np.concatenate([cbk[g, m][ck[b, g, :, m]] for m in range(M)], axis=-1)     # [N, D], before RoPE
            v_eff = np.concatenate([cbv[g, m][cv[b, g, :, m]] for m in range(M)], axis=-1)
            k_eff[ik[b, g]] = rk[b, g]
            v_eff[iv[b, g]] = rv[b, g]
            k_eff = rope(k_eff, pos, rope_base, rope_style)
            for h in range(g * G, (g + 1) * G):
                s_ = scale * (k_eff @ q64[b, h])
                p_ = np.exp(s_ - s_.max())
                out[b, h] = (p_ / p_.sum()) @ v_eff
    return out

