"""GPU parity: decode attention on keys stored before RoPE (paper Sec. 3.3, last paragraph) against the oracle's
definition (rotate every key, coded or FP16, to its position; then plain decode attention)."""
import numpy as np
import pytest
import torch

import paper_2506_19505_amd as antkv
from gpu_util import ATTN_TOL, dev, pack12, rel_l2_rows
from workloads import make_codebooks, make_decode_query, make_qkv, normal_fp16, random_anchor_sets, random_codes

pytestmark = pytest.mark.gpu


def _case(oracle, seed, B, Hq, Hkv, N, d, C, k_k, k_v, base, style, pos0, N_cap=None):
    N_cap = N_cap or N
    M = 128 // d
    rng = np.random.default_rng(seed)
    _, k, v = make_qkv(seed, 1, Hq, Hkv, min(max(C, 300), 6000), 1, 128)
    cbk, cbv = make_codebooks(seed, k, d, C, "k", max_sample=6000), make_codebooks(seed, v, d, C, "v", max_sample=6000)
    ck = rng.integers(0, C, (B, Hkv, N_cap, M)).astype(np.int32)
    cv = rng.integers(0, C, (B, Hkv, N_cap, M)).astype(np.int32)
    ik, iv = random_anchor_sets(seed, "k", B, Hkv, N, k_k), random_anchor_sets(seed, "v", B, Hkv, N, k_v)
    rk, rv = normal_fp16(seed, "rows_k", (B, Hkv, k_k, 128)), normal_fp16(seed, "rows_v", (B, Hkv, k_v, 128))
    # the query as a model hands it over: rotated to the position that follows the cache
    q = oracle.rope(make_decode_query(seed, B, Hq, 128).astype(np.float64), np.full((B, Hq), pos0 + N), base, style).astype(np.float16)
    scale = 1 / np.sqrt(128)
    geom = antkv.Geometry(B, Hq, Hkv, d, n_centroids=C)
    to_dev = (lambda c: dev(c.astype(np.uint8))) if C == 256 else (lambda c: dev(pack12(c)))
    out = antkv.decode_attn_prerope(geom, dev(q), scale, to_dev(ck), to_dev(cv), dev(cbk), dev(cbv),
                                    dev(ik) if k_k else None, dev(rk) if k_k else None,
                                    dev(iv) if k_v else None, dev(rv) if k_v else None,
                                    rope_base=base, rope_style=style, pos0=pos0, N=N)
    torch.cuda.synchronize()
    want = oracle.decode_attn_prerope(q, ck[:, :, :N], cv[:, :, :N], cbk, cbv, ik, rk, iv, rv, scale, base, style, pos0)
    err = rel_l2_rows(out.cpu().numpy(), want)
    print(f"pre-RoPE d={d} C={C} N={N} anchors {k_k}/{k_v} style {style} pos0 {pos0}: rel-L2 max {err.max():.2e} mean {err.mean():.2e}")
    assert err.max() <= ATTN_TOL, f"relative L2 {err.max():.3e}"


@pytest.mark.parametrize("d", [4, 8, 16])
@pytest.mark.parametrize("style,pos0", [(0, 0), (1, 100000)])
def test_prerope_byte_codes(oracle, d, style, pos0):
    _case(oracle, 300 + d, 2, 8, 2, 3000, d, 256, 30, 30, 10000.0, style, pos0)


@pytest.mark.parametrize("d", [32, 16])
def test_prerope_12bit_codes(oracle, d):
    _case(oracle, 310 + d, 1, 8, 2, 2500, d, 4096, 25, 25, 500000.0, 1, 4096)
    _case(oracle, 312 + d, 2, 4, 2, 1333, d, 4096, 14, 0, 10000.0, 0, 7)          # the other pairing, two heads per KV head, odd N
    _case(oracle, 314 + d, 1, 2, 2, 70000, d, 4096, 700, 700, 500000.0, 1, 0, N_cap=70100)   # several ranges per KV head


def test_prerope_edge_cases(oracle):
    _case(oracle, 320, 1, 4, 1, 700, 8, 256, 0, 0, 10000.0, 1, 0)                 # no anchors at all
    _case(oracle, 321, 1, 4, 1, 611, 8, 256, 5, 0, 10000.0, 0, 17, N_cap=900)     # N below the capacity, K anchors only
    _case(oracle, 322, 2, 4, 1, 65, 8, 256, 1, 1, 10000.0, 1, 0)                  # one tile and a token
    _case(oracle, 323, 1, 4, 1, 300, 8, 256, 300, 300, 10000.0, 1, 9)             # every token an FP16 anchor in both lists
    _case(oracle, 324, 2, 4, 2, 1500, 16, 256, 20, 10, 10000.0, 0, 3)             # two query heads per KV head
    _case(oracle, 325, 1, 3, 3, 1027, 4, 256, 11, 40, 10000.0, 1, 5)              # one query head per KV head, odd N
    _case(oracle, 326, 1, 4, 1, 40000, 8, 256, 3500, 3300, 10000.0, 1, 2)         # lists too long for the staging areas


def test_prerope_fixed_order_is_reproducible(oracle):
    """With ANTKV_DECODE_FIXED_ORDER the pre-RoPE path too gives the same bits on every launch."""
    B, Hq, Hkv, N, d, k = 2, 8, 2, 40000, 8, 100
    rng = np.random.default_rng(77)
    geom = antkv.Geometry(B, Hq, Hkv, d)
    q = dev(make_decode_query(77, B, Hq, 128))
    ck = dev(rng.integers(0, 256, (B, Hkv, N, 128 // d)).astype(np.uint8))
    cv = dev(rng.integers(0, 256, (B, Hkv, N, 128 // d)).astype(np.uint8))
    cbk, cbv = dev(normal_fp16(77, "cb12_k", (Hkv, 128 // d, 256, d))), dev(normal_fp16(77, "cb12_v", (Hkv, 128 // d, 256, d)))
    ik, iv = dev(random_anchor_sets(77, "k", B, Hkv, N, k)), dev(random_anchor_sets(77, "v", B, Hkv, N, k))
    rk, rv = dev(normal_fp16(77, "rows_k", (B, Hkv, k, 128))), dev(normal_fp16(77, "rows_v", (B, Hkv, k, 128)))
    prev = antkv.set_decode_options(antkv.DECODE_FIXED_ORDER)
    try:
        outs = [antkv.decode_attn_prerope(geom, q, 0.0884, ck, cv, cbk, cbv, ik, rk, iv, rv, rope_base=10000.0, rope_style=1,
                                          pos0=11).clone() for _ in range(3)]
        torch.cuda.synchronize()
    finally:
        antkv.set_decode_options(prev)
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])


def test_prerope_long_context(oracle):
    """131072 positions (angles up to 1.3e5 rad on the fastest pair): the fp64 angle reduction and the fp32 stepping."""
    _case(oracle, 330, 1, 4, 1, 131072, 8, 256, 1311, 1311, 500000.0, 1, 0)


def test_prerope_headline_shape_sampled(oracle):
    """The shape the bench times for this path (4 sequences, 8 KV heads, 131072 tokens, 1311 anchors per list, one launch
    over all of them): two (sequence, KV head) pairs are checked against the oracle, which gets their slices alone."""
    B, Hq, Hkv, N, d, k = 4, 32, 8, 131072, 8, 1311
    M, G, seed, base, style, pos0 = 128 // d, 4, 340, 500000.0, 1, 0
    scale = 1 / np.sqrt(128)
    q = oracle.rope(make_decode_query(seed, B, Hq, 128).astype(np.float64), np.full((B, Hq), pos0 + N), base, style).astype(np.float16)
    ck, cv = random_codes(seed, "k", B, Hkv, N, M), random_codes(seed, "v", B, Hkv, N, M)
    _, kk, vv = make_qkv(seed, 1, Hq, Hkv, 6000, 1, 128)
    cbk, cbv = make_codebooks(seed, kk, d, 256, "k", max_sample=6000), make_codebooks(seed, vv, d, 256, "v", max_sample=6000)
    ik, iv = random_anchor_sets(seed, "k", B, Hkv, N, k), random_anchor_sets(seed, "v", B, Hkv, N, k)
    rk, rv = normal_fp16(seed, "rows_k", (B, Hkv, k, 128)), normal_fp16(seed, "rows_v", (B, Hkv, k, 128))
    geom = antkv.Geometry(B, Hq, Hkv, d)
    out = antkv.decode_attn_prerope(geom, dev(q), scale, dev(ck), dev(cv), dev(cbk), dev(cbv), dev(ik), dev(rk), dev(iv), dev(rv),
                                    rope_base=base, rope_style=style, pos0=pos0)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    for b, g in ((0, 0), (3, 7)):
        hs = slice(g * G, (g + 1) * G)
        want = oracle.decode_attn_prerope(q[b:b + 1, hs], ck[b:b + 1, g:g + 1].astype(np.int32), cv[b:b + 1, g:g + 1].astype(np.int32),
                                          cbk[g:g + 1], cbv[g:g + 1], ik[b:b + 1, g:g + 1], rk[b:b + 1, g:g + 1],
                                          iv[b:b + 1, g:g + 1], rv[b:b + 1, g:g + 1], scale, base, style, pos0)
        err = rel_l2_rows(got[b:b + 1, hs], want)
        print(f"pre-RoPE headline shape, sequence {b} KV head {g}: rel-L2 max {err.max():.2e}")
        assert err.max() <= ATTN_TOL, f"relative L2 {err.max():.3e}"


@pytest.mark.parametrize("d", [32, 16])
def test_prerope_12bit_extreme_context_sampled(oracle, d):
    """The 840000-token shape of the paper's long-context point (Sec. 4.4) with keys stored before RoPE and 12-bit codes:
    one launch over 8 KV heads, one of them checked against the oracle (which gets that head's slices alone)."""
    B, Hq, Hkv, N, k = 1, 32, 8, 840000, 8400
    M, G, seed, base, style, pos0 = 128 // d, 4, 350 + d, 500000.0, 1, 0
    scale = 1 / np.sqrt(128)
    rng = np.random.default_rng(seed)
    q = oracle.rope(make_decode_query(seed, B, Hq, 128).astype(np.float64), np.full((B, Hq), pos0 + N), base, style).astype(np.float16)
    ck = rng.integers(0, 4096, (B, Hkv, N, M)).astype(np.int32)
    cv = rng.integers(0, 4096, (B, Hkv, N, M)).astype(np.int32)
    cbk, cbv = normal_fp16(seed, "cb12_k", (Hkv, M, 4096, d)), normal_fp16(seed, "cb12_v", (Hkv, M, 4096, d))
    ik, iv = random_anchor_sets(seed, "k", B, Hkv, N, k), random_anchor_sets(seed, "v", B, Hkv, N, k)
    rk, rv = normal_fp16(seed, "rows_k", (B, Hkv, k, 128)), normal_fp16(seed, "rows_v", (B, Hkv, k, 128))
    geom = antkv.Geometry(B, Hq, Hkv, d, n_centroids=4096)
    out = antkv.decode_attn_prerope(geom, dev(q), scale, dev(pack12(ck)), dev(pack12(cv)), dev(cbk), dev(cbv), dev(ik), dev(rk),
                                    dev(iv), dev(rv), rope_base=base, rope_style=style, pos0=pos0)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    g = 5
    hs = slice(g * G, (g + 1) * G)
    want = oracle.decode_attn_prerope(q[:, hs], ck[:, g:g + 1], cv[:, g:g + 1], cbk[g:g + 1], cbv[g:g + 1], ik[:, g:g + 1],
                                      rk[:, g:g + 1], iv[:, g:g + 1], rv[:, g:g + 1], scale, base, style, pos0)
    err = rel_l2_rows(got[:, hs], want)
    print(f"pre-RoPE d={d} C=4096 N={N}, KV head {g}: rel-L2 max {err.max():.2e}")
    assert err.max() <= ATTN_TOL, f"relative L2 {err.max():.3e}"
