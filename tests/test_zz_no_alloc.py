"""GPU check of antkv_decode_attn_static, the decode entry point that takes no workspace and allocates nothing:
its output must equal antkv_decode_attn's (to the attention tolerance) on two calls in a row, the second on a
smaller input."""
import numpy as np
import pytest
import torch

import paper_2506_19505_amd as antkv
from gpu_util import ATTN_TOL, dev, rel_l2_rows
from workloads import make_codebooks, make_decode_query, make_qkv, normal_fp16, random_anchor_sets, random_codes

pytestmark = pytest.mark.gpu


def _inputs(seed, B, Hq, Hkv, N, d, k_k, k_v, C=256):
    M = 128 // d
    _, ks, vs = make_qkv(seed, 1, Hq, Hkv, 2048, 1, 128)
    if C == 256:
        cbk, cbv = make_codebooks(seed, ks, d, 256, "k", max_sample=2048), make_codebooks(seed, vs, d, 256, "v", max_sample=2048)
        ck, cv = random_codes(seed, "k", B, Hkv, N, M), random_codes(seed, "v", B, Hkv, N, M)
    else:
        cbk, cbv = normal_fp16(seed, "cb12_k", (Hkv, M, C, d)), normal_fp16(seed, "cb12_v", (Hkv, M, C, d))
        rng = np.random.default_rng(seed)
        from gpu_util import pack12
        ck = pack12(rng.integers(0, C, (B, Hkv, N, M)))
        cv = pack12(rng.integers(0, C, (B, Hkv, N, M)))
    return dict(q=make_decode_query(seed, B, Hq, 128), ck=ck, cv=cv, cbk=cbk, cbv=cbv,
                ik=random_anchor_sets(seed, "k", B, Hkv, N, k_k), iv=random_anchor_sets(seed, "v", B, Hkv, N, k_v),
                rk=normal_fp16(seed, "rows_k", (B, Hkv, k_k, 128)), rv=normal_fp16(seed, "rows_v", (B, Hkv, k_v, 128)))


@pytest.mark.parametrize("d,C", [(8, 256), (32, 4096)])
def test_static_scratch_matches_workspace_call(oracle, d, C):
    B, Hq, Hkv = 2, 8, 2
    geom = antkv.Geometry(B, Hq, Hkv, d, n_centroids=C)
    scale = 1 / np.sqrt(128)
    # two calls in a row on the library's scratch: a larger input, then a smaller one (fewer workgroups per head)
    for seed, N, k_k, k_v in ((11, 9000, 90, 90), (12, 700, 7, 0)):
        c = _inputs(seed, B, Hq, Hkv, N, d, k_k, k_v, C)
        t = {n: dev(a) for n, a in c.items()}
        out = torch.full((B, Hq, 128), float("nan"), dtype=torch.float16, device="cuda")
        antkv.decode_attn_static(geom, t["q"], scale, t["ck"], t["cv"], t["cbk"], t["cbv"],
                                 t["ik"] if k_k else None, t["rk"] if k_k else None,
                                 t["iv"] if k_v else None, t["rv"] if k_v else None, out)
        torch.cuda.synchronize()
        ref = antkv.decode_attn(geom, t["q"], scale, t["ck"], t["cv"], t["cbk"], t["cbv"],
                                t["ik"] if k_k else None, t["rk"] if k_k else None,
                                t["iv"] if k_v else None, t["rv"] if k_v else None)
        torch.cuda.synchronize()
        err = rel_l2_rows(out.cpu().numpy(), ref.cpu().numpy().astype(np.float64))
        print(f"static scratch vs workspace, d={d} C={C} N={N}: rel-L2 max {err.max():.2e}")
        assert np.isfinite(out.float().cpu().numpy()).all()
        assert err.max() <= ATTN_TOL
        if C == 256:            # and against the oracle itself
            want = oracle.decode_attn(c["q"], c["ck"], c["cv"], c["cbk"], c["cbv"], c["ik"], c["rk"], c["iv"], c["rv"], scale)
            assert rel_l2_rows(out.cpu().numpy(), want).max() <= ATTN_TOL
