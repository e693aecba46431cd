"""GPU parity: Anchor Score (paper Eq. (4)) + selection against the CPU oracle."""
import numpy as np
import pytest
import torch

import paper_2506_19505_amd as antkv
from gpu_util import check_index_sets, dev
from workloads import CONFIGS, anchor_count, make_qkv

pytestmark = pytest.mark.gpu


def _run(oracle, seed, B, Hq, Hkv, N, Nq, k, scale=None, check_scores=True):
    q, kk, _ = make_qkv(seed, B, Hq, Hkv, N, Nq, 128, want_v=False)
    scale = scale or 1.0 / np.sqrt(128)
    geom = antkv.Geometry(B, Hq, Hkv, 8)
    idx_k, idx_v, ans_k, ans_v = antkv.anchor_select(geom, dev(q), dev(kk), scale, k)
    torch.cuda.synchronize()
    ok, ov = oracle.anchor_score(q, kk, scale)
    gk, gv = ans_k.cpu().numpy().astype(np.float64), ans_v.cpu().numpy().astype(np.float64)
    if check_scores:
        # informative tolerance on the scores themselves; the gate is the index sets below
        np.testing.assert_allclose(gv, ov, rtol=2e-5, atol=1e-9)
        np.testing.assert_allclose(gk, ok, rtol=2e-5, atol=1e-9)
    np.testing.assert_allclose(gv.sum(-1), Nq * (Hq // Hkv), rtol=1e-5)      # rows of A sum to one
    soft = 0
    for got, score in ((idx_k, ok), (idx_v, ov)):
        want, margin = oracle.topk(score, k, want_margin=True)
        soft += check_index_sets(got.cpu().numpy(), want, margin)
    rel = max(np.abs(gk - ok).max() / np.abs(ok).max(), np.abs(gv - ov).max() / np.abs(ov).max())
    print(f"N={N} Nq={Nq}: score max-rel-err {rel:.2e}, near-tie index disagreements {soft}")


@pytest.mark.parametrize("B,Hq,Hkv,N,Nq", [(1, 4, 1, 96, 96), (2, 8, 2, 777, 777), (1, 4, 2, 1000, 37),
                                           (1, 2, 2, 300, 1), (2, 4, 4, 65, 64), (1, 4, 1, 5000, 32)])
def test_anchor_select_small(oracle, B, Hq, Hkv, N, Nq):
    _run(oracle, 21, B, Hq, Hkv, N, Nq, anchor_count(N))


def test_anchor_select_k_edges(oracle):
    _run(oracle, 22, 1, 4, 1, 200, 200, 0)
    _run(oracle, 22, 1, 4, 1, 200, 200, 200)


def test_anchor_select_with_supplied_row_stats(oracle):
    """The extended-attention path of Sec. 3.3: row max / row sum come from outside."""
    B, Hq, Hkv, N, Nq, k = 1, 8, 2, 640, 640, 7
    q, kk, _ = make_qkv(23, B, Hq, Hkv, N, Nq, 128, want_v=False)
    scale = 0.1
    ok, ov, st = oracle.anchor_score(q, kk, scale, want_stats=True)
    geom = antkv.Geometry(B, Hq, Hkv, 8)
    rm, rs = dev(st["row_max"].astype(np.float32)), dev(st["row_sum"].astype(np.float32))
    idx_k, idx_v, ans_k, ans_v = antkv.anchor_select(geom, dev(q), dev(kk), scale, k, row_max=rm, row_sum=rs)
    np.testing.assert_allclose(ans_v.cpu().numpy(), ov, rtol=3e-5, atol=1e-9)
    np.testing.assert_allclose(ans_k.cpu().numpy(), ok, rtol=3e-5, atol=1e-9)


def test_anchor_select_tiny_decode_config(oracle):
    """Config 0: 32 query / 8 KV heads, 4096-token prompt scored against itself, 41 anchors."""
    w = CONFIGS["cfg0"]
    _run(oracle, w.seed, w.B, w.Hq, w.Hkv, w.N, w.Nq_select, w.k)


def test_anchor_select_mid_prefill(oracle):
    _run(oracle, 24, 1, 8, 2, 8192, 8192, anchor_count(8192))


def test_anchor_select_long_context_window(oracle):
    """32-query observation window over a 131072-token context (the long-context decode workload)."""
    _run(oracle, 25, 1, 8, 2, 131072, 32, anchor_count(131072))


def test_anchor_select_full_prefill_invariants(oracle):
    """Config 3 at full size (Nq = N = 32768, 32 heads).  All heads: what holds at any size (rows of A sum to one,
    AnS(K) within its bound, ascending unique index sets that pick the largest scores).  One KV head with its four
    query heads: every score and both index sets against the oracle (the oracle needs ~10-20 s for one head)."""
    w = CONFIGS["cfg3"]
    q, kk, _ = make_qkv(w.seed, w.B, w.Hq, w.Hkv, w.N, w.N, w.D, want_v=False)
    geom = antkv.Geometry(w.B, w.Hq, w.Hkv, w.d_sub)
    idx_k, idx_v, ans_k, ans_v = antkv.anchor_select(geom, dev(q), dev(kk), w.scale, w.k)
    gk, gv = ans_k.cpu().numpy().astype(np.float64), ans_v.cpu().numpy().astype(np.float64)
    np.testing.assert_allclose(gv.sum(-1), w.N * w.G, rtol=1e-5)
    qn = np.linalg.norm(q.astype(np.float64), axis=-1).reshape(w.B, w.Hkv, -1).sum(-1)
    assert (gk >= 0).all() and (gk <= 0.25 * qn[..., None]).all()
    for idx, sc in ((idx_k.cpu().numpy(), ans_k.cpu().numpy()), (idx_v.cpu().numpy(), ans_v.cpu().numpy())):
        for b in range(w.B):
            for g in range(w.Hkv):
                sel = idx[b, g]
                assert np.all(np.diff(sel) > 0) and sel.min() >= 0 and sel.max() < w.N
                rest = np.delete(sc[b, g], sel)
                assert sc[b, g][sel].min() >= rest.max()
    g = 5                                                      # a KV head in the middle: non-zero head offsets
    print("oracle on one KV head of cfg3 ...", flush=True)
    ok, ov = oracle.anchor_score(q[:, g * w.G:(g + 1) * w.G], kk[:, g:g + 1], w.scale)
    np.testing.assert_allclose(gv[:, g], ov[:, 0], rtol=3e-5, atol=1e-9)
    np.testing.assert_allclose(gk[:, g], ok[:, 0], rtol=3e-5, atol=1e-9)
    soft = 0
    for got, score in ((idx_k, ok), (idx_v, ov)):
        want, margin = oracle.topk(score, w.k, want_margin=True)
        soft += check_index_sets(got.cpu().numpy()[:, g:g + 1], want, margin)
    print(f"cfg3, KV head {g}: scores within 3e-5, near-tie index disagreements {soft}")
