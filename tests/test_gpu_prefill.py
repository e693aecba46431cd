"""GPU parity: causal prompt attention with row statistics (antkv_prefill_attn; paper Sec. 2.1 and the first step
of Alg. 1) against the CPU oracle, and its hand-over to the Anchor Score pass."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2506_19505_amd as antkv
from gpu_util import check_index_sets, dev
from workloads import CONFIGS, anchor_count, make_qkv

pytestmark = pytest.mark.gpu

# fp16 probabilities in the value product (2^-11 relative each, averaged over a row) and the fp16 output rounding
OUT_TOL = 2e-3


def _check(oracle, seed, B, Hq, Hkv, N, Nq, scale, q_gain=1.0):
    q, k, v = make_qkv(seed, B, Hq, Hkv, N, Nq, 128)
    q = (q.astype(np.float32) * q_gain).astype(np.float16)
    geom = antkv.Geometry(B, Hq, Hkv, 8)
    out, rm, rs = antkv.prefill_attn(geom, dev(q), dev(k), dev(v), scale)
    torch.cuda.synchronize()
    want, wm, wl = oracle.prefill_attn(q, k, v, scale)
    got = out.cpu().numpy().astype(np.float64)
    err = np.linalg.norm(got - want, axis=-1) / np.maximum(np.linalg.norm(want, axis=-1), 1e-30)
    assert err.max() <= OUT_TOL, f"relative L2 {err.max():.3e}"
    np.testing.assert_allclose(rm.cpu().numpy(), wm, rtol=2e-6, atol=2e-6)
    np.testing.assert_allclose(rs.cpu().numpy(), wl, rtol=1e-4)
    print(f"N={N} Nq={Nq} G={Hq // Hkv}: out rel-L2 max {err.max():.2e}")
    return q, k, v, rm, rs


@pytest.mark.parametrize("B,Hq,Hkv,N,Nq", [(1, 8, 2, 300, 300), (2, 4, 4, 1000, 137), (1, 4, 1, 257, 257),
                                           (1, 4, 2, 64, 64), (1, 2, 2, 1, 1), (1, 8, 2, 2100, 33),
                                           (2, 8, 4, 95, 95)])
def test_prefill_attn_small(oracle, B, Hq, Hkv, N, Nq):
    _check(oracle, 61, B, Hq, Hkv, N, Nq, 1.0 / np.sqrt(128))


def test_prefill_attn_wide_score_range(oracle):
    """Scores spread over a few hundred log2 units: the softmax reference has to move many times per row."""
    _check(oracle, 62, 1, 4, 2, 700, 700, 1.0 / np.sqrt(128), q_gain=12.0)


def test_prefill_attn_feeds_anchor_select(oracle):
    """Alg. 1: the attention pass hands its row statistics to the Anchor Score pass."""
    B, Hq, Hkv, N = 1, 8, 2, 1536
    scale = 1.0 / np.sqrt(128)
    q, k, v, rm, rs = _check(oracle, 63, B, Hq, Hkv, N, N, scale)
    kk = anchor_count(N)
    geom = antkv.Geometry(B, Hq, Hkv, 8)
    idx_k, idx_v, ans_k, ans_v = antkv.anchor_select(geom, dev(q), dev(k), scale, kk, row_max=rm, row_sum=rs)
    ok, ov = oracle.anchor_score(q, k, scale)
    np.testing.assert_allclose(ans_v.cpu().numpy(), ov, rtol=1e-4, atol=1e-9)
    np.testing.assert_allclose(ans_k.cpu().numpy(), ok, rtol=1e-4, atol=1e-9)
    for got, score in ((idx_k, ok), (idx_v, ov)):
        want, margin = oracle.topk(score, kk, want_margin=True)
        check_index_sets(got.cpu().numpy(), want, margin)


def test_prefill_attn_full_prefill_sampled_rows(oracle):
    """Config 3 at full size (N = Nq = 32768, 32 heads): sampled query rows against the oracle's definition,
    computed row by row."""
    w = CONFIGS["cfg3"]
    q, k, v = make_qkv(w.seed, w.B, w.Hq, w.Hkv, w.N, w.N, w.D)
    geom = antkv.Geometry(w.B, w.Hq, w.Hkv, w.d_sub)
    out, rm, rs = antkv.prefill_attn(geom, dev(q), dev(k), dev(v), w.scale)
    torch.cuda.synchronize()
    rng = np.random.default_rng(5)
    G = w.Hq // w.Hkv
    rows = [(0, 0, 0), (0, w.Hq - 1, w.N - 1), (0, 3, 31), (0, 5, 32), (0, 7, 63), (0, 9, 64)]
    rows += [(0, int(rng.integers(w.Hq)), int(rng.integers(w.N))) for _ in range(40)]
    got_all, rm_all, rs_all = out.cpu().numpy(), rm.cpu().numpy(), rs.cpu().numpy()
    worst = 0.0
    for b, h, i in rows:
        # one row through the oracle: the query alone (Nq = 1) over the keys it sees
        want, wm, wl = oracle.prefill_attn(q[b:b + 1, h:h + 1, i:i + 1], k[b:b + 1, h // G:h // G + 1, :i + 1],
                                           v[b:b + 1, h // G:h // G + 1, :i + 1], w.scale)
        got = got_all[b, h, i].astype(np.float64)
        err = np.linalg.norm(got - want[0, 0, 0]) / np.linalg.norm(want[0, 0, 0])
        worst = max(worst, err)
        assert err <= OUT_TOL, f"row {(b, h, i)}: relative L2 {err:.3e}"
        assert abs(rm_all[b, h, i] - wm[0, 0, 0]) <= 2e-6 * (1 + abs(wm[0, 0, 0]))
        assert abs(rs_all[b, h, i] - wl[0, 0, 0]) <= 1e-4 * wl[0, 0, 0]
    print(f"cfg3 sampled rows: out rel-L2 max {worst:.2e}")


def test_prefill_attn_rejects_bad_arguments():
    lib = antkv.load_library()
    g = antkv.Geometry(1, 4, 2, 8).c()
    x = torch.zeros(1, 4, 8, 128, dtype=torch.float16, device="cuda")
    kv = torch.zeros(1, 2, 8, 128, dtype=torch.float16, device="cuda")
    st = torch.zeros(1, 4, 8, dtype=torch.float32, device="cuda")
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    call = lambda **o: lib.antkv_prefill_attn(
        ctypes.byref(g), o.get("q", p(x)), p(kv), p(kv), o.get("N", 8), o.get("Nq", 8), o.get("scale", 0.1), p(x),
        o.get("rm", p(st)), p(st), None)
    assert call(Nq=9) != 0
    assert call(N=0, Nq=0) != 0
    assert call(q=None) != 0
    assert call(rm=None) != 0
    assert call(scale=0.0) != 0
    assert call(q=ctypes.c_void_p(x.data_ptr() + 2)) != 0
    torch.cuda.synchronize()
