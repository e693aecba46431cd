"""Counter-based seeded tensor generator.

Every tensor is a pure function of (seed, tensor name, shape): element blocks of
2^22 values are drawn from Philox streams keyed by (seed, tensor id, block), so
the result does not depend on thread count or generation order and any slice
can be regenerated alone.

Recipe (stands in for LLaMA-3 / Mistral KV caches, which need model weights):
  * Q, K, V ~ N(0, 1) rounded to fp16.
  * K carries channel outliers: 4 channels per KV head (fixed over tokens and
    batch) are scaled by 10, mimicking the large-magnitude channels of pre-RoPE
    keys (paper App. A).
  * Codebooks are k-means++ seeds (first pick uniform, then D^2-weighted picks,
    no Lloyd iterations) drawn from the sub-vectors of a seeded token sample;
    centroids are the picked fp16 sub-vectors verbatim.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
import os

import numpy as np

_BLOCK = 1 << 22

_TENSOR_ID = {
    "q": 1,
    "k": 2,
    "v": 3,
    "q_decode": 4,
    "outlier": 5,
    "cb_sample_k": 6,
    "cb_sample_v": 7,
    "cb_pick_k": 8,
    "cb_pick_v": 9,
    "codes_k": 10,
    "codes_v": 11,
    "anchor_k": 12,
    "anchor_v": 13,
    "rows_k": 14,
    "rows_v": 15,
    "misc": 16,
    "win_rows_k": 17,
    "win_rows_v": 18,
    "new_k": 19,
    "new_v": 20,
    "cb12_k": 21,
    "cb12_v": 22,
}


def _rng(seed: int, name: str, block: int = 0) -> np.random.Generator:
    tid = _TENSOR_ID[name] if isinstance(name, str) else int(name)
    return np.random.Generator(np.random.Philox(key=[int(seed), (tid << 40) | int(block)]))


def _workers() -> int:
    return max(1, min(16, os.cpu_count() or 1))


def normal_fp16(seed: int, name: str, shape, row_scale: np.ndarray | None = None) -> np.ndarray:
    """N(0,1) tensor of the given shape in fp16.

    row_scale, if given, has shape [shape[-3]... broadcastable to rows]: it must be
    an array of shape (n_rows, shape[-1]) or (shape[-1],) in fp32 that multiplies
    each row before rounding to fp16.
    """
    shape = tuple(int(s) for s in shape)
    n = int(np.prod(shape)) if shape else 1
    out = np.empty(n, dtype=np.float16)
    last = shape[-1] if shape else 1
    assert _BLOCK % last == 0 or n <= _BLOCK, "last dim must divide the block size"
    nblocks = (n + _BLOCK - 1) // _BLOCK

    def fill(bi: int) -> None:
        lo = bi * _BLOCK
        hi = min(n, lo + _BLOCK)
        x = _rng(seed, name, bi).standard_normal(hi - lo, dtype=np.float32)
        if row_scale is not None:
            x = x.reshape(-1, last)
            if row_scale.ndim == 1:
                x = x * row_scale[None, :]
            else:
                r0 = lo // last
                x = x * row_scale[r0:r0 + x.shape[0]]
            x = x.reshape(-1)
        out[lo:hi] = x.astype(np.float16)

    if nblocks <= 1:
        fill(0)
    else:
        with ThreadPoolExecutor(_workers()) as ex:
            list(ex.map(fill, range(nblocks)))
    return out.reshape(shape)


def outlier_channels(seed: int, Hkv: int, D: int, n_out: int = 4, factor: float = 10.0) -> np.ndarray:
    """Per-KV-head channel multipliers [Hkv, D] (fp32): n_out channels get `factor`."""
    mult = np.ones((Hkv, D), dtype=np.float32)
    for g in range(Hkv):
        ch = _rng(seed, "outlier", g).choice(D, size=min(n_out, D), replace=False)
        mult[g, ch] = factor
    return mult


def _k_tensor(seed: int, B: int, Hkv: int, N: int, D: int) -> np.ndarray:
    mult = outlier_channels(seed, Hkv, D)
    n_rows = B * Hkv * N
    if n_rows * D <= (1 << 26):
        head_of_row = (np.arange(n_rows) // N) % Hkv
        return normal_fp16(seed, "k", (B, Hkv, N, D), row_scale=mult[head_of_row])
    # large tensors: generate per (b, g) slab to avoid a huge row-scale array
    out = np.empty((B, Hkv, N, D), dtype=np.float16)
    flat = out.reshape(-1)
    n = flat.size
    nblocks = (n + _BLOCK - 1) // _BLOCK

    def fill(bi: int) -> None:
        lo = bi * _BLOCK
        hi = min(n, lo + _BLOCK)
        x = _rng(seed, "k", bi).standard_normal(hi - lo, dtype=np.float32).reshape(-1, D)
        r0 = lo // D
        heads = ((np.arange(r0, r0 + x.shape[0]) // N) % Hkv)
        x *= mult[heads]
        flat[lo:hi] = x.reshape(-1).astype(np.float16)

    with ThreadPoolExecutor(_workers()) as ex:
        list(ex.map(fill, range(nblocks)))
    return out


def make_qkv(seed: int, B: int, Hq: int, Hkv: int, N: int, Nq: int, D: int,
             want_v: bool = True):
    """Q [B,Hq,Nq,D] (the last Nq positions of the context), K, V [B,Hkv,N,D], all fp16."""
    q = normal_fp16(seed, "q", (B, Hq, Nq, D))
    k = _k_tensor(seed, B, Hkv, N, D)
    v = normal_fp16(seed, "v", (B, Hkv, N, D)) if want_v else None
    return q, k, v


def make_decode_query(seed: int, B: int, Hq: int, D: int) -> np.ndarray:
    """Single decode-step query [B,Hq,D] fp16 ~ N(0,1)."""
    return normal_fp16(seed, "q_decode", (B, Hq, D))


def _kmeanspp_group(points: np.ndarray, C: int, rngs) -> np.ndarray:
    """k-means++ seeding of a group of tables, one random stream per table.

    points: [T, S, d] float64 -> pick indices [T, C].  The result for a table depends
    only on its points and its stream, not on how tables are grouped.
    """
    T, S, _ = points.shape
    picks = np.empty((T, C), dtype=np.int64)
    u = np.empty((T, C))
    for t, rng in enumerate(rngs):
        picks[t, 0] = rng.integers(0, S)
        u[t] = rng.random(C)
    ar = np.arange(T)
    diff = points - points[ar, picks[:, 0]][:, None, :]
    mind = np.einsum("tsd,tsd->ts", diff, diff)
    cum = np.empty_like(mind)
    for c in range(1, C):
        np.cumsum(mind, axis=1, out=cum)
        for t in range(T):
            total = cum[t, -1]
            if total > 0.0:
                picks[t, c] = min(S - 1, int(np.searchsorted(cum[t], u[t, c] * total, side="right")))
            else:  # every sample already coincides with a pick: fall back to uniform
                picks[t, c] = int(u[t, c] * S) % S
        np.subtract(points, points[ar, picks[:, c]][:, None, :], out=diff)
        np.minimum(mind, np.einsum("tsd,tsd->ts", diff, diff), out=mind)
    return picks


def make_codebooks(seed: int, x: np.ndarray, d_sub: int, C: int, which: str,
                   max_sample: int = 16384) -> np.ndarray:
    """Codebook [Hkv, M, C, d_sub] fp16 picked from x [B,Hkv,N,D] (K or V) by k-means++."""
    assert which in ("k", "v")
    B, Hkv, N, D = x.shape
    M = D // d_sub
    total_tok = B * N
    S = min(total_tok, max_sample)
    srng = _rng(seed, "cb_sample_" + which)
    tok = np.sort(srng.choice(total_tok, size=S, replace=False)) if S < total_tok else np.arange(total_tok)
    bsel, tsel = tok // N, tok % N
    sample = x[bsel, :, tsel, :]                       # [S, Hkv, D]
    sample = np.transpose(sample, (1, 0, 2)).reshape(Hkv, S, M, d_sub)
    tables = np.transpose(sample, (0, 2, 1, 3)).reshape(Hkv * M, S, d_sub)
    tables64 = tables.astype(np.float64)

    T = Hkv * M
    groups = np.array_split(np.arange(T), min(T, _workers()))

    def one(ids: np.ndarray) -> np.ndarray:
        return _kmeanspp_group(tables64[ids], C, [_rng(seed, "cb_pick_" + which, int(t)) for t in ids])

    with ThreadPoolExecutor(_workers()) as ex:
        picks = np.concatenate(list(ex.map(one, groups)))
    cb = tables[np.arange(Hkv * M)[:, None], picks]    # [T, C, d] fp16 verbatim
    return np.ascontiguousarray(cb.reshape(Hkv, M, C, d_sub))


def random_codes(seed: int, which: str, B: int, Hkv: int, N: int, M: int, C: int = 256) -> np.ndarray:
    """Uniform random code tensor [B,Hkv,N,M] uint8 (for cache-shaped stress inputs)."""
    n = B * Hkv * N * M
    out = np.empty(n, dtype=np.uint8)
    nblocks = (n + _BLOCK - 1) // _BLOCK

    def fill(bi: int) -> None:
        lo = bi * _BLOCK
        hi = min(n, lo + _BLOCK)
        out[lo:hi] = _rng(seed, "codes_" + which, bi).integers(0, C, size=hi - lo, dtype=np.uint8)

    with ThreadPoolExecutor(_workers()) as ex:
        list(ex.map(fill, range(nblocks)))
    return out.reshape(B, Hkv, N, M)


def random_anchor_sets(seed: int, which: str, B: int, Hkv: int, N: int, k: int,
                       head_frac: float = 0.25, tail_frac: float = 0.25) -> np.ndarray:
    """Anchor index sets [B,Hkv,k] int32, ascending and unique.

    A share of the anchors sits at the head (sink tokens) and tail (recent tokens)
    of the context, the rest is spread uniformly, following the locality the paper
    reports for Anchor Scores (Sec. 3.2, App. D).
    """
    out = np.empty((B, Hkv, k), dtype=np.int32)
    if k == 0:
        return out
    for b in range(B):
        for g in range(Hkv):
            rng = _rng(seed, "anchor_" + which, b * Hkv + g)
            if k >= N:
                out[b, g] = np.arange(N, dtype=np.int32)[:k]
                continue
            n_head = min(int(k * head_frac), N)
            n_tail = min(int(k * tail_frac), N - n_head)
            chosen = set(range(n_head)) | set(range(N - n_tail, N))
            need = k - len(chosen)
            while need > 0:
                cand = rng.integers(0, N, size=2 * need + 8)
                for c in cand:
                    if int(c) not in chosen:
                        chosen.add(int(c))
                        need -= 1
                        if need == 0:
                            break
            out[b, g] = np.sort(np.fromiter(chosen, dtype=np.int64, count=k)).astype(np.int32)
    return out
