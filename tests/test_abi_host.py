"""Host-side checks of the C ABI that need no GPU: exported symbols, argument validation, workspace queries."""
import ctypes
import os
import re

import pytest

import paper_2506_19505_amd as antkv
from paper_2506_19505_amd.binding import EXPORTS, STATIC_SCRATCH_BYTES, _Geom

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OK, EINVAL, EUNSUPPORTED, EWORKSPACE = 0, 1, 2, 3


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(antkv.lib_path()):
        from paper_2506_19505_amd.build import build
        build()
    return antkv.load_library()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "antkv.h")).read()
    declared = set(re.findall(r"\b(antkv_[a-z_]+)\s*\(", header))
    assert declared == set(EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None
    assert lib.antkv_version() >= 1
    assert lib.antkv_strerror(0) == b"ok" and b"workspace" in lib.antkv_strerror(EWORKSPACE)


def _g(B=1, Hq=32, Hkv=8, D=128, d=8, C=256):
    return _Geom(B, Hq, Hkv, D, d, C)


def test_geometry_validation(lib):
    null = None
    enc = lambda g: lib.antkv_encode(ctypes.byref(g), null, 128, 128, 128, 0, null, null, 0, 0, null)
    assert enc(_g()) == OK                                   # n_tok == 0 is a no-op
    assert enc(_g(d=2)) == EUNSUPPORTED
    assert enc(_g(d=32)) == EUNSUPPORTED
    assert enc(_g(C=4096)) == EUNSUPPORTED                   # 4096 centroids go with d_sub 32 or 16 only
    assert enc(_g(d=32, C=4096)) == OK and enc(_g(d=16, C=4096)) == OK
    assert enc(_g(D=64)) == EUNSUPPORTED
    assert enc(_g(Hq=64)) == EUNSUPPORTED                    # group size 8
    assert enc(_g(Hq=30)) == EINVAL                          # Hq not a multiple of Hkv
    assert lib.antkv_encode(None, null, 0, 0, 0, 0, null, null, 0, 0, null) == EINVAL


def test_encode_argument_errors(lib):
    g = _g()
    fake = ctypes.c_void_p(4096)
    call = lambda x, cb, codes, n, cap, off, xs_t=128: lib.antkv_encode(
        ctypes.byref(g), x, 128 * 8 * 64, 128 * 64, xs_t, n, cb, codes, cap, off, None)
    assert call(None, fake, fake, 4, 4, 0) == EINVAL          # null x
    assert call(fake, fake, fake, 4, 3, 0) == EINVAL          # rows do not fit N_cap
    assert call(fake, fake, fake, 4, 8, 5) == EINVAL          # offset + n > N_cap
    assert call(ctypes.c_void_p(4098), fake, fake, 4, 8, 0) == EINVAL   # misaligned
    assert call(fake, fake, fake, 4, 8, 0, xs_t=100) == EINVAL          # token stride < D / unaligned
    assert call(fake, fake, fake, -1, 8, 0) == EINVAL


def test_topk_and_select_argument_errors(lib):
    fake = ctypes.c_void_p(4096)
    assert lib.antkv_topk(fake, 2, 100, 101, fake, fake, 1 << 20, None) == EINVAL   # k > N
    assert lib.antkv_topk(fake, 2, 100, 0, fake, None, 0, None) == OK               # k == 0: nothing to do
    assert lib.antkv_topk(fake, 2, 100, 5, fake, None, 0, None) == EWORKSPACE
    need = lib.antkv_topk_workspace(2, 100, 5)
    assert need > 0 and need % 256 == 0
    assert lib.antkv_topk(fake, 2, 100, 5, fake, fake, need - 1, None) == EWORKSPACE
    g = _g()
    sel = lambda N, Nq, k, rm, rs, ws, wsb: lib.antkv_anchor_select(
        ctypes.byref(g), fake, fake, N, Nq, 0.1, k, rm, rs, None, None, fake, fake, ws, wsb, None)
    assert sel(100, 200, 5, None, None, fake, 1 << 30) == EINVAL      # Nq > N
    assert sel(100, 50, 101, None, None, fake, 1 << 30) == EINVAL     # k > N
    assert sel(100, 50, 5, fake, None, fake, 1 << 30) == EINVAL       # row stats: both or neither
    assert sel(100, 50, 5, None, None, None, 0) == EWORKSPACE
    assert lib.antkv_anchor_select_workspace(ctypes.byref(g), 100, 50, 5) > 0
    assert lib.antkv_anchor_select_workspace(ctypes.byref(g), 100, 200, 5) == 0


def test_decode_argument_errors(lib):
    g = _g()
    fake = ctypes.c_void_p(4096)

    def dec(N=1000, cap=1000, k_k=10, k_v=10, idx_k=fake, rows_k=fake, ans_k=None, ans_v=None, rk=None, k_resel=0,
            ws=fake, wsb=1 << 30, q=fake, scale=0.1):
        return lib.antkv_decode_attn(ctypes.byref(g), q, scale, fake, fake, N, cap, fake, fake, idx_k, rows_k, k_k,
                                     fake, fake, k_v, fake, ans_k, ans_v, rk, None, k_resel, ws, wsb, None)
    assert dec(cap=999) == EINVAL                 # N_cap < N
    assert dec(k_k=1001) == EINVAL                # more anchors than tokens
    assert dec(idx_k=None) == EINVAL              # k_k > 0 needs the index list
    assert dec(q=None) == EINVAL
    assert dec(scale=0.0) == EINVAL
    assert dec(ans_k=fake) == EINVAL              # the two scores come together
    assert dec(rk=fake, k_resel=5) == EINVAL      # re-selection needs the scores
    assert dec(ws=None, wsb=0) == EWORKSPACE
    need = lib.antkv_decode_attn_workspace(ctypes.byref(g), 1000, 10, 10, 0)
    assert need > 0 and need % 256 == 0
    assert dec(wsb=need - 1) == EWORKSPACE
    # more anchors or a re-selection only ever grow the workspace
    assert lib.antkv_decode_attn_workspace(ctypes.byref(g), 1000, 1000, 1000, 50) >= need


def test_binding_refuses_host_tensors():
    import torch
    geom = antkv.Geometry(1, 4, 1, 8)
    with pytest.raises(ValueError):
        antkv.encode(geom, torch.zeros(1, 1, 4, 128, dtype=torch.float16), torch.zeros(1, 16, 256, 8, dtype=torch.float16))


def test_static_scratch_refuses_oversized_shapes(lib):
    """A shape whose scratch need exceeds the built-in array is an error before anything is enqueued."""
    geom = antkv.Geometry(64, 2048, 512, 8)          # 64 x 512 (sequence, KV head) pairs: partials beyond 8 MiB
    g = geom.c()
    need = lib.antkv_decode_attn_workspace(ctypes.byref(g), 4096, 0, 0, 0)
    assert need > STATIC_SCRATCH_BYTES
    fake = ctypes.c_void_p(4096)
    rc = lib.antkv_decode_attn_static(ctypes.byref(g), fake, 0.1, fake, fake, 4096, 4096, fake, fake, None, None, 0,
                                      None, None, 0, fake, None)
    assert rc == 3                                     # ANTKV_EWORKSPACE


def test_decode_options_and_prerope_argument_errors(lib):
    prev = lib.antkv_set_decode_options(3)
    assert lib.antkv_set_decode_options(prev) == 3            # returns the previous mask; unknown bits are dropped
    assert lib.antkv_set_decode_options(0xF0) == prev and lib.antkv_set_decode_options(prev) == 0
    g = _g(B=1)
    fake = ctypes.c_void_p(4096)
    ws_bytes = lib.antkv_decode_attn_prerope_workspace(ctypes.byref(g), 1000, 0)
    # 16 bytes of scores per token (one-byte codes: tokens rounded up to 64) and KV head + the decode kernels' own scratch
    assert ws_bytes >= 8 * 1024 * 16 + lib.antkv_decode_attn_workspace(ctypes.byref(g), 1000, 0, 0, 0)
    g12 = _g(B=1, d=32, C=4096)
    assert lib.antkv_decode_attn_prerope_workspace(ctypes.byref(g12), 1000, 0) >= \
        8 * 1000 * 16 + lib.antkv_decode_attn_workspace(ctypes.byref(g12), 1000, 0, 0, 0)
    assert lib.antkv_decode_attn_prerope_workspace(ctypes.byref(_g(d=2)), 1000, 10) == 0
    call = lambda base, style, pos0, ws=fake, nbytes=1 << 40: lib.antkv_decode_attn_prerope(
        ctypes.byref(g), fake, 0.1, fake, fake, 1000, 1000, fake, fake, None, None, 0, None, None, 0,
        base, style, pos0, fake, ws, nbytes, None)
    assert call(1.0, 0, 0) == EINVAL                          # the base must exceed 1
    assert call(10000.0, 2, 0) == EINVAL                      # pairing 0 or 1
    assert call(10000.0, 1, -1) == EINVAL                     # positions start at pos0 >= 0
    assert call(10000.0, 1, 0, ws=None) == EWORKSPACE
    assert call(10000.0, 1, 0, nbytes=ws_bytes - 1) == EWORKSPACE

