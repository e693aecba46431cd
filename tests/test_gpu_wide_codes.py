"""GPU parity for the 12-bit codebooks (paper Sec. 4: 32-channel sub-vectors, 4096 centroids, "0.375 bit"):
encode and decode attention against the CPU oracle, which is generic in the codebook size."""
import numpy as np
import pytest
import torch

import paper_2506_19505_amd as antkv
from gpu_util import check_codes, dev, pack12, unpack12
from workloads import make_codebooks, make_qkv

pytestmark = pytest.mark.gpu

D_SUB, C = 32, 4096


@pytest.fixture(scope="module")
def books():
    """K and V codebooks [2 KV heads][4][4096][32] picked from 6000 synthetic rows."""
    _, k, v = make_qkv(81, 1, 2, 2, 6000, 1, 128)
    return (make_codebooks(81, k, D_SUB, C, "k", max_sample=6000), make_codebooks(81, v, D_SUB, C, "v", max_sample=6000))


def test_pack_unpack_roundtrip():
    rng = np.random.default_rng(0)
    c = rng.integers(0, 4096, size=(3, 5, 4))
    assert np.array_equal(unpack12(pack12(c)), c) and pack12(c).shape == (3, 5, 6)
    assert pack12(np.array([[0x123, 0x456, 0x789, 0xABC]])).tolist() == [[0x23, 0x61, 0x45, 0x89, 0xC7, 0xAB]]


@pytest.mark.parametrize("B,n", [(1, 700), (2, 70), (1, 257)])
def test_encode12_matches_oracle(oracle, books, B, n):
    _, x, _ = make_qkv(82 + n, B, 2, 2, n, 1, 128, want_v=False)
    geom = antkv.Geometry(B, 2, 2, D_SUB, n_centroids=C)
    codes = antkv.encode(geom, dev(x), dev(books[0]))
    torch.cuda.synchronize()
    assert codes.shape == (B, 2, n, 6)
    got = unpack12(codes.cpu().numpy())
    want, margin = oracle.encode(x, books[0], want_margin=True)
    soft = check_codes(got, want, margin)
    print(f"n={n}: near-tie disagreements {soft} of {want.size}")


def test_encode12_duplicate_centroids_and_offsets(oracle, books):
    """Exact ties go to the lower index; token_offset / N_cap place the rows."""
    cb = books[0].copy()
    cb[:, :, 4000:4096] = cb[:, :, 100:196]                   # 96 exact duplicates far apart
    cb[:, :, 33] = cb[:, :, 32]                                 # and one inside a tile
    _, x, _ = make_qkv(83, 1, 2, 2, 300, 1, 128, want_v=False)
    geom = antkv.Geometry(1, 2, 2, D_SUB, n_centroids=C)
    buf = torch.full((1, 2, 400, 6), 0xEE, dtype=torch.uint8, device="cuda")
    antkv.encode(geom, dev(x), dev(cb), codes=buf, token_offset=50)
    got_all = buf.cpu().numpy()
    assert (got_all[:, :, :50] == 0xEE).all() and (got_all[:, :, 350:] == 0xEE).all()
    got = unpack12(got_all[:, :, 50:350])
    want, margin = oracle.encode(x, cb, want_margin=True)
    check_codes(got, want, margin)
    assert not np.isin(got, np.arange(4000, 4096)).any() and not (got == 33).any()
