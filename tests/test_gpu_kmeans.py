"""GPU parity: one iteration of the offline token-weighted k-means (antkv_kmeans_step; paper Sec. 3.1) against the
CPU oracle.  The assignment is held to the code rule (bit-exact outside the 1e-6 near-tie list); the update is then
compared on the assignment the GPU actually used, so that a near-tie cannot leak into the centroid comparison."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2506_19505_amd as antkv
from gpu_util import check_codes, dev
from workloads import CONFIGS, make_codebooks, make_qkv

pytestmark = pytest.mark.gpu


def _weights(seed, shape):
    return np.random.default_rng(seed).gamma(0.5, 1.0, size=shape).astype(np.float32)   # heavy-tailed, like gradients


def _compare(oracle, x, w, cb, d, what=""):
    B, Hkv, n, _ = x.shape
    geom = antkv.Geometry(B, Hkv, Hkv, d)
    new, codes, wsum, obj = antkv.kmeans_step(geom, dev(x), dev(w), dev(cb))
    torch.cuda.synchronize()
    codes_h = codes.cpu().numpy()
    want_codes, margin = oracle.encode(x, cb, want_margin=True)
    soft = check_codes(codes_h, want_codes, margin)
    want, want_w, want_obj = oracle.kmeans_update(x, w, codes_h, cb)
    np.testing.assert_allclose(wsum.cpu().numpy(), want_w, rtol=2e-5, atol=1e-30)
    np.testing.assert_allclose(obj.cpu().numpy(), want_obj, rtol=2e-5)
    got = new.cpu().numpy()
    empty = want_w == 0
    assert np.array_equal(got[empty], cb[empty]), "a centroid without assigned weight must keep its value"
    # fp32 sums rounded once to fp16: within one fp16 spacing of the fp64 mean
    tol = np.abs(want) * 2.0 ** -10 + 2.0 ** -24 + 1e-5 * np.abs(want)
    assert (np.abs(got.astype(np.float64) - want) <= tol).all(), \
        f"centroid error {np.abs(got.astype(np.float64) - want).max():.3e}"
    print(f"{what} d={d}: near-tie codes {soft}, empty centroids {int(empty.sum())}, "
          f"max centroid error {np.abs(got.astype(np.float64) - want).max():.2e}")
    return new


@pytest.mark.parametrize("d", [4, 8, 16])
@pytest.mark.parametrize("B,Hkv,n", [(2, 2, 3000), (1, 3, 70)])
def test_kmeans_step_small(oracle, d, B, Hkv, n):
    _, x, _ = make_qkv(71, B, Hkv, Hkv, n, 1, 128, want_v=False)
    cb = make_codebooks(71, x, d, 256, "k", max_sample=min(n, 1024))
    _compare(oracle, x, _weights(5, (B, Hkv, n)), cb, d)


def test_kmeans_zero_weights_and_no_tokens_keep_the_codebook(oracle):
    _, x, _ = make_qkv(72, 1, 2, 2, 500, 1, 128, want_v=False)
    cb = make_codebooks(72, x, 8, 256, "k", max_sample=500)
    geom = antkv.Geometry(1, 2, 2, 8)
    new, _, wsum, obj = antkv.kmeans_step(geom, dev(x), dev(np.zeros((1, 2, 500), np.float32)), dev(cb))
    assert torch.equal(new.cpu(), torch.from_numpy(cb)) and float(wsum.sum()) == 0 and float(obj.sum()) == 0
    new, _, wsum, _ = antkv.kmeans_step(geom, dev(x[:, :, :0]), dev(np.zeros((1, 2, 0), np.float32)), dev(cb))
    assert torch.equal(new.cpu(), torch.from_numpy(cb)) and float(wsum.sum()) == 0


def test_kmeans_iterations_descend(oracle):
    """Lloyd's iteration on the GPU: the weighted distortion after each assignment never rises (up to the fp16
    rounding of the stored centroids), and it falls overall."""
    _, x, _ = make_qkv(73, 2, 2, 2, 4000, 1, 128, want_v=False)
    w = _weights(6, (2, 2, 4000))
    cb = make_codebooks(73, x, 8, 256, "k", max_sample=512)
    geom = antkv.Geometry(2, 2, 2, 8)
    xd, wd, cur = dev(x), dev(w), dev(cb)
    hist = []
    for _ in range(6):
        cur, _, _, obj = antkv.kmeans_step(geom, xd, wd, cur)
        hist.append(obj.cpu().numpy().sum())
    assert all(b <= a * (1 + 1e-4) for a, b in zip(hist, hist[1:])), hist
    assert hist[-1] < 0.97 * hist[0], hist
    print("distortion per iteration:", [f"{h:.4g}" for h in hist])


def test_kmeans_step_full_prefill_shape(oracle):
    """Config 3's K rows (32768 tokens x 8 KV heads) as the calibration set: whole update against the oracle."""
    w = CONFIGS["cfg3"]
    _, x, _ = make_qkv(w.seed, w.B, w.Hq, w.Hkv, w.N, 1, w.D, want_v=False)
    cb = make_codebooks(w.seed, x, w.d_sub, w.C, "k", max_sample=4096)
    _compare(oracle, x, _weights(7, (w.B, w.Hkv, w.N)), cb, w.d_sub, what="cfg3")


def test_kmeans_rejects_bad_arguments():
    lib = antkv.load_library()
    g = antkv.Geometry(1, 2, 2, 8).c()
    x = torch.zeros(1, 2, 16, 128, dtype=torch.float16, device="cuda")
    wt = torch.ones(1, 2, 16, dtype=torch.float32, device="cuda")
    cb = torch.zeros(2, 16, 256, 8, dtype=torch.float16, device="cuda")
    out = torch.empty_like(cb)
    codes = torch.empty(1, 2, 16, 16, dtype=torch.uint8, device="cuda")
    ws = torch.empty(lib.antkv_kmeans_step_workspace(ctypes.byref(g)) + 256, dtype=torch.uint8, device="cuda")
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    call = lambda **o: lib.antkv_kmeans_step(
        ctypes.byref(g), o.get("x", p(x)), p(wt), o.get("n", 16), p(cb), o.get("out", p(out)), p(codes), None, None,
        p(ws), o.get("ws_bytes", ws.numel()), None)
    assert call() == 0
    assert call(x=None) != 0
    assert call(out=p(cb)) != 0            # in place is not supported
    assert call(n=-1) != 0
    assert call(ws_bytes=16) != 0
    torch.cuda.synchronize()
