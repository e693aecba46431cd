"""Run-twice bit comparison.  Codes, Anchor Scores and index sets are the same on every run; the decode output of the
one-byte-code kernel is bit-reproducible in the opt-in fixed-tile-order mode (antkv_set_decode_options), and the
12-bit kernels always are."""
import numpy as np
import pytest
import torch

import paper_2506_19505_amd as antkv
from gpu_util import ATTN_TOL, dev, pack12, rel_l2_rows
from workloads import (anchor_count, make_codebooks, make_decode_query, make_qkv, normal_fp16, random_anchor_sets,
                       random_codes)

pytestmark = pytest.mark.gpu


def test_encode_scores_and_index_sets_repeat_exactly():
    B, Hq, Hkv, N, d = 2, 8, 2, 5000, 8
    qwin, k, _ = make_qkv(400, B, Hq, Hkv, N, 64, 128)
    cb = make_codebooks(400, k, d, 256, "k")
    geom = antkv.Geometry(B, Hq, Hkv, d)
    kd, qd, cbd = dev(k), dev(qwin), dev(cb)
    runs = []
    for _ in range(2):
        codes = antkv.encode(geom, kd, cbd)
        ik, iv, ak, av = antkv.anchor_select(geom, qd, kd, 0.09, anchor_count(N))
        top = antkv.topk(ak.reshape(B * Hkv, N), 77)
        torch.cuda.synchronize()
        runs.append([t.clone() for t in (codes, ik, iv, ak, av, top)])
    for a, b in zip(*runs):
        assert torch.equal(a, b)


@pytest.mark.parametrize("d", [4, 8, 16])
def test_decode_fixed_tile_order_is_bit_reproducible(oracle, d):
    B, Hq, Hkv, N = 4, 32, 8, 30000
    k = anchor_count(N)
    _, ks, vs = make_qkv(410 + d, 1, Hq, Hkv, 2048, 1, 128)
    c = dict(q=make_decode_query(410, B, Hq, 128), ck=random_codes(410, "k", B, Hkv, N, 128 // d),
             cv=random_codes(410, "v", B, Hkv, N, 128 // d), cbk=make_codebooks(410, ks, d, 256, "k"),
             cbv=make_codebooks(410, vs, d, 256, "v"), ik=random_anchor_sets(410, "k", B, Hkv, N, k),
             iv=random_anchor_sets(410, "v", B, Hkv, N, k), rk=normal_fp16(410, "rows_k", (B, Hkv, k, 128)),
             rv=normal_fp16(410, "rows_v", (B, Hkv, k, 128)))
    t = {n: dev(a) for n, a in c.items()}
    geom = antkv.Geometry(B, Hq, Hkv, d)
    ws = antkv.DecodeWorkspace(geom, N, k, k, 0, "cuda")
    outs = torch.empty((6, B, Hq, 128), dtype=torch.float16, device="cuda")
    was = antkv.set_decode_options(antkv.DECODE_FIXED_ORDER)
    try:
        for i in range(6):
            antkv.decode_attn(geom, t["q"], 0.1, t["ck"], t["cv"], t["cbk"], t["cbv"], t["ik"], t["rk"], t["iv"], t["rv"],
                              out=outs[i], workspace=ws)
        torch.cuda.synchronize()
    finally:
        antkv.set_decode_options(was)
    for i in range(1, 6):
        assert torch.equal(outs[i], outs[0]), f"launch {i} differs from launch 0"
    want = oracle.decode_attn(c["q"], c["ck"], c["cv"], c["cbk"], c["cbv"], c["ik"], c["rk"], c["iv"], c["rv"], 0.1)
    err = rel_l2_rows(outs[0].cpu().numpy(), want)
    assert err.max() <= ATTN_TOL, f"relative L2 {err.max():.3e}"


@pytest.mark.parametrize("d", [32, 16])
def test_decode12_is_bit_reproducible(d):
    B, Hq, Hkv, N, C, M = 1, 8, 2, 40000, 4096, 128 // d
    rng = np.random.default_rng(420 + d)
    cbk, cbv = dev(normal_fp16(420, "cb12_k", (Hkv, M, C, d))), dev(normal_fp16(420, "cb12_v", (Hkv, M, C, d)))
    ck = dev(pack12(rng.integers(0, C, (B, Hkv, N, M)).astype(np.int32)))
    cv = dev(pack12(rng.integers(0, C, (B, Hkv, N, M)).astype(np.int32)))
    k = anchor_count(N)
    ik, iv = dev(random_anchor_sets(420, "k", B, Hkv, N, k)), dev(random_anchor_sets(420, "v", B, Hkv, N, k))
    rk, rv = dev(normal_fp16(420, "rows_k", (B, Hkv, k, 128))), dev(normal_fp16(420, "rows_v", (B, Hkv, k, 128)))
    q = dev(make_decode_query(420, B, Hq, 128))
    geom = antkv.Geometry(B, Hq, Hkv, d, n_centroids=C)
    outs = [antkv.decode_attn(geom, q, 0.09, ck, cv, cbk, cbv, ik, rk, iv, rv).clone() for _ in range(4)]
    torch.cuda.synchronize()
    for o in outs[1:]:
        assert torch.equal(o, outs[0])
