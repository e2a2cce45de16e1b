"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and rejects bad arguments before touching a device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2401_09149_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2401_09149_amd import build
        build.build()
    return binding.load()


def declared_functions():
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(ie_(?:attn|sp|linear)_\w+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported(lib):
    from paper_2401_09149_amd import binding
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for name in names:
        assert getattr(lib, name) is not None


def test_strerror_is_total(lib):
    seen = set()
    for code in range(-8, 2):
        s = lib.ie_attn_strerror(code)
        assert s and len(s) > 0
        seen.add(s)
    assert len(seen) >= 9   # eight statuses + "unknown"


def test_tile_rows_setting(lib):
    f = lib.ie_attn_set_tile_rows
    assert f(0) == 0          # initial setting: chosen per call
    assert f(128) == 0 and f(256) == 128 and f(0) == 256   # returns the previous setting
    assert f(64) == -3 and f(-1) == -3                      # IE_ERR_UNSUPPORTED, setting unchanged
    assert f(0) == 0


def test_workspace_query(lib):
    f = lib.ie_attn_bwd_workspace_bytes
    n = f(1, 32768, 32, 32, 128, 0)
    assert n >= 32768 * 32 * 4 and n % 256 == 0
    assert f(1, 0, 32, 32, 128, 0) == 0          # invalid shapes report 0
    assert f(1, 128, 3, 2, 128, 0) == 0
    assert f(1, 128, 4, 2, 96, 0) == 0


def test_fast_workspace_query(lib):
    """Room for dS only where the dS-storing backward path exists: dense, D = 128, S % 128 == 0."""
    base, fast = lib.ie_attn_bwd_workspace_bytes, lib.ie_attn_bwd_fast_workspace_bytes
    assert fast(1, 32768, 32, 32, 128, 0, 1) == base(1, 32768, 32, 32, 128, 0) + 32 * 32768 * (32768 + 128)
    assert fast(2, 256, 8, 2, 128, 0, 1) == base(2, 256, 8, 2, 128, 0) + 2 * 8 * 256 * 384
    assert fast(1, 4096, 8, 8, 128, 0, 0) == base(1, 4096, 8, 8, 128, 0) + 2 * 8 * 4096 * 4096   # not causal: all blocks
    for args in ((1, 32768, 32, 32, 64, 0, 1),       # head dimension 64
                 (1, 32768 + 64, 32, 32, 128, 0, 1), # ragged
                 (1, 32768, 32, 32, 128, 5, 1),      # packed documents
                 (1, 1 << 23, 1, 1, 128, 0, 1)):     # beyond the 32-bit offsets inside a block
        assert fast(*args) == base(*args[:6])
    assert fast(1, 0, 32, 32, 128, 0, 1) == 0


def test_bad_arguments_fail_before_any_launch(lib):
    one = ctypes.c_void_p(256)   # never dereferenced: validation fails first
    args = dict(B=1, S=128, Hq=4, Hkv=2, D=128, scale=0.1, causal=1)

    def fwd(q=one, k=one, v=one, o=one, lse=one, cu=None, nd=0, **kw):
        a = dict(args, **kw)
        return lib.ie_attn_fwd(q, k, v, o, lse, cu, nd, a["B"], a["S"], a["Hq"], a["Hkv"], a["D"], a["scale"], a["causal"], None)

    assert fwd(q=None) == -1 and fwd(lse=None) == -1
    assert fwd(S=0) == -2 and fwd(Hq=3) == -2 and fwd(B=-1) == -2
    assert fwd(cu=one, nd=3, B=2) == -2 and fwd(cu=one, nd=0) == -2
    assert fwd(D=96) == -3 and fwd(scale=0.0) == -3 and fwd(scale=float("nan")) == -3 and fwd(causal=2) == -3
    assert fwd(S=2 ** 40) == -2

    def bwd(ws=one, ws_bytes=1 << 30, dq=one, **kw):
        a = dict(args, **kw)
        return lib.ie_attn_bwd(one, one, one, one, one, one, dq, one, one, None, 0, a["B"], a["S"], a["Hq"], a["Hkv"],
                               a["D"], a["scale"], a["causal"], ws, ws_bytes, None)

    assert bwd(dq=None) == -1
    assert bwd(ws=None) == -4 and bwd(ws_bytes=16) == -4 and bwd(ws=ctypes.c_void_p(264)) == -4
    assert bwd(D=32) == -3

    def phases(mask, ws_bytes=1 << 30, **kw):
        a = dict(args, **kw)
        return lib.ie_attn_bwd_phases(one, one, one, one, one, one, one, one, one, None, 0, a["B"], a["S"], a["Hq"], a["Hkv"],
                                      a["D"], a["scale"], a["causal"], one, ws_bytes, mask, None)

    assert phases(0) == -3 and phases(8) == -3 and phases(16) == -3 and phases(7 | 32) == -3   # no phase / unknown bits
    assert phases(7 | 16, S=100) == -3                  # the stored-dS path does not exist for this shape
    small = lib.ie_attn_bwd_workspace_bytes(1, 128, 4, 2, 128, 0)
    assert phases(7 | 16, ws_bytes=small) == -4         # it exists, but the workspace has no room for dS

    def static(dq=one, **kw):
        a = dict(args, **kw)
        return lib.ie_attn_bwd_static(one, one, one, one, one, one, dq, one, one, None, 0, a["B"], a["S"], a["Hq"], a["Hkv"],
                                      a["D"], a["scale"], a["causal"], None)

    assert static(dq=None) == -1 and static(D=32) == -3 and static(Hq=3) == -2
    assert static(S=(1 << 21) // 4 + 1) == -4 and static(B=2, S=1 << 20, Hq=2, Hkv=2) == -4   # beyond the static array


    def fwd_sp(x=one, o=one, lse=one, B=1, Sl=256, Hq=8, Hkv=8, D=128, P=4, scale=0.1, causal=1):
        return lib.ie_attn_fwd_sp(x, o, lse, B, Sl, Hq, Hkv, D, P, scale, causal, None)

    assert fwd_sp(x=None) == -1 and fwd_sp(lse=None) == -1
    assert fwd_sp(P=3) == -2 and fwd_sp(P=0) == -2 and fwd_sp(Sl=0) == -2 and fwd_sp(Hkv=6) == -2
    assert fwd_sp(Sl=128) == -3 and fwd_sp(Sl=384) == -3 and fwd_sp(D=96) == -3
    assert fwd_sp(x=ctypes.c_void_p(264)) == -6

    def bwd_sp(ws=one, ws_bytes=1 << 30, dx=one, **kw):
        a = dict(B=1, Sl=256, Hq=8, Hkv=8, D=128, P=4, scale=0.1, causal=1)
        a.update(kw)
        return lib.ie_attn_bwd_sp(one, one, one, one, dx, a["B"], a["Sl"], a["Hq"], a["Hkv"], a["D"], a["P"], a["scale"],
                                  a["causal"], ws, ws_bytes, None)

    assert bwd_sp(dx=None) == -1 and bwd_sp(P=3) == -2 and bwd_sp(Sl=300) == -3
    assert bwd_sp(ws=None) == -4 and bwd_sp(ws_bytes=64) == -4


def test_permute_bad_arguments_fail_before_any_launch(lib):
    one, odd = ctypes.c_void_p(256), ctypes.c_void_p(264)   # never dereferenced
    ok = dict(B=2, Sl=128, Hq=8, Hkv=4, D=128, P=4)

    def qkv(name, *ptrs, **kw):
        a = dict(ok, **kw)
        return getattr(lib, name)(*ptrs, a["B"], a["Sl"], a["Hq"], a["Hkv"], a["D"], a["P"], None)

    def o(name, *ptrs, **kw):
        a = dict(ok, **kw)
        return getattr(lib, name)(*ptrs, a["B"], a["Sl"], a["Hq"], a["D"], a["P"], None)

    for name, n in (("ie_sp_pack_qkv", 2), ("ie_sp_unpack_dqkv", 2), ("ie_sp_unpack_qkv", 4), ("ie_sp_pack_dqkv", 4)):
        for bad in range(n):
            assert qkv(name, *[None if i == bad else one for i in range(n)]) == -1
            assert qkv(name, *[odd if i == bad else one for i in range(n)]) == -6
        ptrs = [one] * n
        assert qkv(name, *ptrs, Sl=0) == -2 and qkv(name, *ptrs, B=-1) == -2 and qkv(name, *ptrs, P=0) == -2
        assert qkv(name, *ptrs, P=3) == -2 and qkv(name, *ptrs, Hkv=2) == -2     # heads not divisible by P
        assert qkv(name, *ptrs, D=12) == -3 and qkv(name, *ptrs, D=0) == -3
        assert qkv(name, *ptrs, Sl=2 ** 40) == -2 and qkv(name, *ptrs, B=40000) == -2
    for name in ("ie_sp_pack_o", "ie_sp_unpack_o", "ie_sp_pack_do", "ie_sp_unpack_do"):
        assert o(name, None, one) == -1 and o(name, one, None) == -1
        assert o(name, odd, one) == -6 and o(name, one, odd) == -6
        assert o(name, one, one, Sl=0) == -2 and o(name, one, one, P=3) == -2 and o(name, one, one, D=4) == -3


def test_linear_bad_arguments_fail_before_any_launch(lib):
    one, odd = ctypes.c_void_p(256), ctypes.c_void_p(264)
    i64 = ctypes.c_int64
    for name, bad_dims in (("ie_linear_fwd", [(128, 64, 96), (128, 60, 128)]),          # K % 64, N % 8
                           ("ie_linear_bwd_input", [(128, 96, 64), (128, 128, 60)]),    # N % 64, K % 8
                           ("ie_linear_bwd_weight", [(96, 64, 64), (128, 60, 64), (128, 64, 60)])):
        f = getattr(lib, name)
        call = lambda a, b, c, M, N, K: f(a, b, c, i64(M), i64(N), i64(K), None)
        assert call(None, one, one, 128, 128, 128) == -1 and call(one, one, None, 128, 128, 128) == -1
        assert call(odd, one, one, 128, 128, 128) == -6 and call(one, one, odd, 128, 128, 128) == -6
        assert call(one, one, one, 0, 128, 128) == -2 and call(one, one, one, 128, -1, 128) == -2
        assert call(one, one, one, 128, 2 ** 22, 128) == -2
        for dims in bad_dims:
            assert call(one, one, one, *dims) == -3
