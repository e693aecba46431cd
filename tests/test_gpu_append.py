"""GPU parity: decode append with an FP16 sliding window (antkv_append_token) followed by decode attention, step by
step against the oracle on the same seeded rows."""
import numpy as np
import pytest
import torch

import paper_2506_19505_amd as antkv
from gpu_util import ATTN_TOL, NEAR_TIE, dev, rel_l2_rows
from workloads import make_codebooks, make_decode_query, make_qkv

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("d,W,B,Hq,Hkv", [(8, 32, 2, 8, 2), (16, 5, 1, 4, 1), (4, 1, 1, 8, 2), (8, 0, 1, 4, 2), (8, 64, 1, 4, 1)])
def test_append_then_decode(oracle, d, W, B, Hq, Hkv):
    N0, T, k_a = 300, 2 * W + 3 if W else 5, 7
    scale = 1 / np.sqrt(128)
    _, k_all, v_all = make_qkv(40 + d + W, B, Hq, Hkv, N0 + T, 1, 128)
    cbk = make_codebooks(40 + d, k_all, d, 256, "k", max_sample=256)
    cbv = make_codebooks(40 + d, v_all, d, 256, "v", max_sample=256)
    M = 128 // d
    N_cap = N0 + T
    codes_k = np.zeros((B, Hkv, N_cap, M), np.int32)
    codes_v = np.zeros((B, Hkv, N_cap, M), np.int32)
    codes_k[:, :, :N0] = oracle.encode(k_all[:, :, :N0], cbk)
    codes_v[:, :, :N0] = oracle.encode(v_all[:, :, :N0], cbv)
    anchors = np.arange(3, 3 + 11 * k_a, 11)
    idx = np.broadcast_to(np.concatenate([anchors, np.arange(N0 - W, N0)]), (B, Hkv, k_a + W)).astype(np.int32).copy()
    idx_k, idx_v = idx.copy(), idx.copy()
    rows_k = np.take_along_axis(k_all, idx[..., None].astype(np.int64), axis=2).copy()
    rows_v = np.take_along_axis(v_all, idx[..., None].astype(np.int64), axis=2).copy()
    geom = antkv.Geometry(B, Hq, Hkv, d)
    g = dict(ck=dev(codes_k.astype(np.uint8)), cv=dev(codes_v.astype(np.uint8)), cbk=dev(cbk), cbv=dev(cbv),
             ik=dev(idx_k), rk=dev(rows_k), iv=dev(idx_v), rv=dev(rows_v))
    N = N0
    for t in range(T):
        kn, vn = k_all[:, :, N0 + t], v_all[:, :, N0 + t]
        N_new, mk, mv = oracle.append_token(kn, vn, N, W, cbk, cbv, codes_k, codes_v, idx_k, rows_k, idx_v, rows_v,
                                            want_margin=True)
        N_gpu = antkv.append_token(geom, dev(kn), dev(vn), N, W, g["cbk"], g["cbv"], g["ck"], g["cv"], g["ik"], g["rk"],
                                   g["iv"], g["rv"])
        torch.cuda.synchronize()
        assert N_gpu == N_new
        pos = N - W                                        # the position whose codes were just written
        for name, got_c, want_c, margin in (("K", g["ck"], codes_k, mk), ("V", g["cv"], codes_v, mv)):
            got = got_c[:, :, pos].cpu().numpy().astype(np.int32)
            bad = got != want_c[:, :, pos]
            assert not (bad & (margin >= NEAR_TIE)).any(), f"step {t}: {name} codes of position {pos} differ"
            got_c[:, :, pos] = dev(want_c[:, :, pos].astype(np.uint8))    # keep both sides on the same codes (near ties)
        assert (g["ik"].cpu().numpy() == idx_k).all() and (g["iv"].cpu().numpy() == idx_v).all(), f"step {t}: lists"
        assert (g["rk"].cpu().numpy() == rows_k).all() and (g["rv"].cpu().numpy() == rows_v).all(), f"step {t}: rows"
        N = N_new
        q = make_decode_query(900 + t, B, Hq, 128)
        out = antkv.decode_attn(geom, dev(q), scale, g["ck"], g["cv"], g["cbk"], g["cbv"], g["ik"], g["rk"], g["iv"],
                                g["rv"], N=N)
        torch.cuda.synchronize()
        want = oracle.decode_attn(q, codes_k[:, :, :N], codes_v[:, :, :N], cbk, cbv, idx_k, rows_k, idx_v, rows_v, scale)
        err = rel_l2_rows(out.cpu().numpy(), want)
        assert err.max() <= ATTN_TOL, f"step {t}: decode relative L2 {err.max():.3e}"
    print(f"d={d} W={W}: {T} appends + decodes ok, last rel-L2 max {err.max():.2e}")


def test_append_rejects_bad_arguments():
    geom = antkv.Geometry(1, 4, 1, 8)
    z16 = lambda *s: torch.zeros(s, dtype=torch.float16, device="cuda")
    codes = torch.zeros((1, 1, 16, 16), dtype=torch.uint8, device="cuda")
    cb = z16(1, 16, 256, 8)
    idx = torch.zeros((1, 1, 4), dtype=torch.int32, device="cuda")
    rows = z16(1, 1, 4, 128)
    with pytest.raises(antkv.AntkvError):      # context already fills the capacity
        antkv.append_token(geom, z16(1, 1, 128), z16(1, 1, 128), 16, 2, cb, cb, codes, codes, idx, rows, idx, rows)
    with pytest.raises(antkv.AntkvError):      # window longer than the lists
        antkv.append_token(geom, z16(1, 1, 128), z16(1, 1, 128), 8, 5, cb, cb, codes, codes, idx, rows, idx, rows)
