"""Helpers shared by the GPU parity tests: device transfer and the comparison rules.

Comparison rules (the bar the HIP path is held to):
  * codes and anchor index sets are bit-exact against the oracle, except for candidates whose oracle
    margin is below 1e-6 (near-ties that fp32 and fp64 arithmetic may legitimately order differently);
    those are counted and reported separately.
  * attention outputs: relative L2 error per (b, head) row <= 2e-3 against the fp64 oracle.
"""
from __future__ import annotations

import numpy as np
import torch

NEAR_TIE = 1e-6
ATTN_TOL = 2e-3


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def rel_l2_rows(got: np.ndarray, want: np.ndarray) -> np.ndarray:
    got = got.astype(np.float64).reshape(-1, got.shape[-1])
    want = want.astype(np.float64).reshape(-1, want.shape[-1])
    den = np.linalg.norm(want, axis=1)
    den[den == 0] = 1.0
    return np.linalg.norm(got - want, axis=1) / den


def check_codes(got: np.ndarray, want: np.ndarray, margin: np.ndarray, what: str = "codes") -> int:
    """Bit-exact outside the near-tie list; returns the number of near-tie disagreements."""
    bad = got.astype(np.int64) != want.astype(np.int64)
    hard = bad & (margin >= NEAR_TIE)
    assert not hard.any(), (f"{what}: {int(hard.sum())} mismatches outside the near-tie list "
                            f"(smallest margin {margin[hard].min():.3e}); {int(bad.sum())} in total")
    return int(bad.sum())


def check_index_sets(got: np.ndarray, want: np.ndarray, margin: np.ndarray, what: str = "indices") -> int:
    """got/want [..., k] ascending index sets, margin [..., N].  Differences must be near-ties."""
    k = want.shape[-1]
    assert got.shape == want.shape, (got.shape, want.shape)
    if k == 0:
        return 0
    g2 = got.reshape(-1, k)
    w2 = want.reshape(-1, k)
    m2 = margin.reshape(g2.shape[0], -1)
    soft = 0
    for r in range(g2.shape[0]):
        assert k == 0 or np.all(np.diff(g2[r]) > 0), f"{what}: row {r} is not strictly ascending"
        diff = np.setxor1d(g2[r], w2[r])
        if diff.size:
            worst = m2[r][diff].max()
            assert worst < NEAR_TIE, (f"{what}: row {r} differs in {diff.size} positions, "
                                      f"largest oracle margin {worst:.3e} >= {NEAR_TIE}")
            soft += diff.size
    return soft


def unpack12(packed: np.ndarray) -> np.ndarray:
    """[..., 3M/2] bytes -> [..., M] codes: the M 12-bit codes of a token packed little-endian (code m at bits
    12 m .. 12 m + 11 of the row, i.e. four codes per six bytes)."""
    b = packed.astype(np.int64)
    assert b.shape[-1] % 6 == 0
    out = []
    for grp in range(b.shape[-1] // 6):
        word = np.zeros(b.shape[:-1], dtype=np.int64)
        for i in range(6):
            word |= b[..., 6 * grp + i] << (8 * i)
        out += [(word >> (12 * m)) & 0xFFF for m in range(4)]
    return np.stack(out, axis=-1).astype(np.int32)


def pack12(codes: np.ndarray) -> np.ndarray:
    """[..., M] codes (< 4096, M a multiple of 4) -> [..., 3M/2] bytes, the inverse of unpack12."""
    c = codes.astype(np.int64)
    assert c.shape[-1] % 4 == 0
    out = []
    for grp in range(c.shape[-1] // 4):
        word = np.zeros(c.shape[:-1], dtype=np.int64)
        for m in range(4):
            word |= c[..., 4 * grp + m] << (12 * m)
        out += [(word >> (8 * i)) & 0xFF for i in range(6)]
    return np.stack(out, axis=-1).astype(np.uint8)


def table_range(q, cb, scale, G):
    """Largest |scale * log2(e) * q_h[m] . cb[g][m][c]| over sub-spaces and codes, per (sequence, query head): the
    magnitude that sets the quantum of the decode kernels' fixed-point q.centroid tables."""
    Hkv, M, C, d = cb.shape
    B, Hq, D = q.shape
    qr = q.astype(np.float64).reshape(B, Hkv, G, M, d)
    lut = np.einsum("bghmd,gmcd->bghmc", qr, cb.astype(np.float64)) * (scale * np.log2(np.e))
    return np.abs(lut).max(axis=(3, 4)).reshape(B, Hq)


def attn_tol_for_range(R, M, levels):
    """Output tolerance as a function of the table range R (per row).  A table entry is rounded to R / levels; a token's
    score is the sum of M entries, so its error has standard deviation (R / levels) sqrt(M / 12) log2-units, i.e.
    ln 2 times that relative to a softmax weight.  Up to 1e-3 this stays inside the 2e-3 tolerance (with the fp16
    rounding of weights and the fp32 sums); beyond that range the bound grows in proportion."""
    r_max = levels * 1e-3 / (np.log(2.0) * np.sqrt(M / 12.0))
    return ATTN_TOL * np.maximum(1.0, np.asarray(R) / r_max)

