"""Host-side checks of the C ABI: the library loads, exports every symbol include/modet.h declares,
and rejects bad arguments on the host before any HIP call (so this runs without a GPU)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.environ.get("MODET_LIBRARY") or os.path.join(ROOT, "paper_2403_16526_amd", "libmodet.so")
HDR = os.path.join(ROOT, "include", "modet.h")

OK, E_NULL, E_SHAPE, E_UNSUP, E_ALIGN, E_WS, E_LAUNCH = 0, -1, -2, -3, -4, -5, -6


@pytest.fixture(scope="module")
def lib():
    assert os.path.exists(LIB), "build first: python -m paper_2403_16526_amd.build"
    L = ctypes.CDLL(LIB)
    vp, ci, cf, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
    L.modet_fwd.argtypes = [vp] * 6 + [ci] * 7 + [cf, ci, vp]
    L.modet_bwd.argtypes = [vp] * 10 + [ci] * 7 + [cf, ci, vp, sz, vp]
    L.modet_bwd_static.argtypes = [vp] * 10 + [ci] * 7 + [cf, ci, vp]
    L.modet_warp.argtypes = [vp] * 3 + [ci] * 5 + [ci, ci, vp]
    L.modet_compose.argtypes = [vp] * 3 + [ci] * 5 + [vp]
    L.modet_warp_bwd.argtypes = [vp] * 5 + [ci] * 5 + [ci, ci, vp]
    L.modet_integrate_velocity.argtypes = [vp] * 3 + [ci] * 5 + [vp]
    L.modet_bwd_workspace_bytes.argtypes = [ci] * 9
    L.modet_bwd_workspace_bytes.restype = sz
    L.modet_status_string.argtypes = [ci]
    L.modet_status_string.restype = ctypes.c_char_p
    return L


def declared_functions():
    text = re.sub(r"/\*.*?\*/", "", open(HDR).read(), flags=re.S)
    return sorted(set(re.findall(r"\b(modet_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"modet_fwd", "modet_bwd", "modet_warp", "modet_bwd_workspace_bytes", "modet_status_string",
            "modet_version"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_binding_lists_the_same_names():
    from paper_2403_16526_amd import modet
    assert sorted(modet.EXPORTS) == declared_functions()
    for n in modet.EXPORTS:
        assert callable(getattr(modet, n)), n


P = 0x10000          # fake, 16-byte aligned, never dereferenced: validation fails first
ODD = 0x10004


def fwd(lib, Q=P, K=P, bias=None, phi=P, attn=None, lse=None, B=1, D=4, H=4, W=4, C=8, heads=1, k=3, dt=0):
    return lib.modet_fwd(Q, K, bias, phi, attn, lse, B, D, H, W, C, heads, k, 0.0, dt, None)


def bwd(lib, Q=P, K=P, bias=None, g=P, phi=None, lse=None, dQ=P, dK=P, db=None, B=1, D=4, H=4, W=4, C=8, heads=1,
        k=3, dt=0, ws=None, wsb=0, da=None):
    return lib.modet_bwd(Q, K, bias, g, da, phi, lse, dQ, dK, db, B, D, H, W, C, heads, k, 0.0, dt, ws, wsb, None)


def test_fwd_rejects_bad_arguments(lib):
    assert fwd(lib, Q=None) == E_NULL and fwd(lib, K=None) == E_NULL and fwd(lib, phi=None) == E_NULL
    assert fwd(lib, D=0) == E_SHAPE and fwd(lib, W=-3) == E_SHAPE and fwd(lib, B=0) == E_SHAPE
    assert fwd(lib, C=8, heads=3) == E_SHAPE
    assert fwd(lib, k=4) == E_SHAPE and fwd(lib, k=0) == E_SHAPE and fwd(lib, k=-1) == E_SHAPE
    assert fwd(lib, k=9) == E_UNSUP and fwd(lib, dt=2) == E_UNSUP
    assert fwd(lib, B=64, D=512, H=512, W=512, C=8) == E_UNSUP        # beyond 32-bit indexing
    assert fwd(lib, Q=ODD) == E_ALIGN and fwd(lib, phi=ODD) == E_ALIGN and fwd(lib, attn=ODD) == E_ALIGN


def test_bwd_rejects_bad_arguments(lib):
    assert bwd(lib, g=None) == E_NULL and bwd(lib, dQ=None) == E_NULL and bwd(lib, dK=None) == E_NULL
    assert bwd(lib, phi=P, lse=None) == E_NULL and bwd(lib, phi=None, lse=P) == E_NULL
    assert bwd(lib, H=0) == E_SHAPE and bwd(lib, k=2) == E_SHAPE and bwd(lib, C=6, heads=4) == E_SHAPE
    assert bwd(lib, dK=ODD) == E_ALIGN and bwd(lib, ws=ODD, wsb=1 << 20) == E_ALIGN
    need = lib.modet_bwd_workspace_bytes(1, 4, 4, 4, 8, 1, 3, 0, 0)
    assert need == 64 * 16
    assert lib.modet_bwd_workspace_bytes(1, 4, 4, 4, 8, 1, 3, 0, 1) == 0          # flag 1: phi and lse passed in
    assert lib.modet_bwd_workspace_bytes(1, 4, 4, 4, 8, 3, 3, 0, 0) == 0          # invalid shape
    assert bwd(lib) == E_WS and bwd(lib, ws=P, wsb=need - 1) == E_WS
    # flag 2: the bias gradient is wanted -- 27 fp64 sums (216 bytes, rounded up to 16)
    assert lib.modet_bwd_workspace_bytes(1, 4, 4, 4, 8, 1, 3, 0, 3) == 224
    assert lib.modet_bwd_workspace_bytes(1, 4, 4, 4, 8, 1, 3, 0, 2) == need + 224
    assert bwd(lib, phi=P, lse=P, db=P) == E_WS and bwd(lib, phi=P, lse=P, db=P, ws=P, wsb=223) == E_WS
    assert bwd(lib, db=P, ws=P, wsb=need + 223) == E_WS
    # flag 4: an upstream gradient of the attention weights is passed in -- one float per window
    assert lib.modet_bwd_workspace_bytes(1, 4, 4, 4, 8, 1, 3, 0, 5) == 256
    assert bwd(lib, phi=P, lse=P, da=P) == E_WS and bwd(lib, phi=P, lse=P, da=P, ws=P, wsb=255) == E_WS
    assert bwd(lib, phi=P, lse=P, da=ODD, ws=P, wsb=256) == E_ALIGN


def test_bwd_static_rejects_bad_arguments(lib):
    def sb(Q=P, K=P, bias=None, g=P, phi=None, lse=None, dQ=P, dK=P, db=None, B=1, D=4, H=4, W=4, C=8, heads=1, k=3,
           dt=0):
        return lib.modet_bwd_static(Q, K, bias, g, None, phi, lse, dQ, dK, db, B, D, H, W, C, heads, k, 0.0, dt, None)
    assert sb(g=None) == E_NULL and sb(dK=None) == E_NULL and sb(phi=P) == E_NULL
    assert sb(W=0) == E_SHAPE and sb(k=4) == E_SHAPE and sb(k=9) == E_UNSUP and sb(dQ=ODD) == E_ALIGN
    # the built-in scratch is 8 MiB: statistics of 524288 windows (16 bytes each) fit, one window more does not,
    # and with phi and lse passed in only the bias gradient's sums need scratch
    limit = 8 << 20
    assert lib.modet_bwd_workspace_bytes(1, 64, 64, 128, 8, 1, 3, 0, 0) == limit
    assert sb(D=64, H=64, W=129) == E_WS and sb(D=160, H=192, W=224) == E_WS
    assert sb(D=64, H=64, W=128, db=P) == E_WS                 # the statistics fill it, the sums no longer fit


def test_warp_rejects_bad_arguments(lib):
    w = lambda src=P, f=P, out=P, B=1, D=4, H=4, W=4, C=8, half=0, dt=0: lib.modet_warp(src, f, out, B, D, H, W, C,
                                                                                       half, dt, None)
    assert w(src=None) == E_NULL and w(f=None) == E_NULL and w(out=None) == E_NULL
    assert w(D=0) == E_SHAPE and w(half=1, H=5) == E_SHAPE and w(half=2) == E_SHAPE
    assert w(C=5, dt=1) == E_UNSUP and w(C=260) == E_UNSUP and w(dt=7) == E_UNSUP
    assert w(out=ODD) == E_ALIGN


def test_warp_bwd_rejects_bad_arguments(lib):
    wb = lambda src=P, f=P, g=P, ds=P, df=P, B=1, D=4, H=4, W=4, C=8, half=0, dt=0: lib.modet_warp_bwd(
        src, f, g, ds, df, B, D, H, W, C, half, dt, None)
    assert wb(f=None) == E_NULL and wb(g=None) == E_NULL and wb(ds=None) == E_NULL
    assert wb(src=None) == E_NULL            # the field gradient needs the source values
    assert wb(W=0) == E_SHAPE and wb(half=1, D=5) == E_SHAPE and wb(half=3) == E_SHAPE
    assert wb(C=7, dt=1) == E_UNSUP and wb(C=300) == E_UNSUP and wb(dt=2) == E_UNSUP
    assert wb(df=ODD) == E_ALIGN and wb(g=ODD) == E_ALIGN


def test_field_functions_reject_bad_arguments(lib):
    comp = lambda a=P, b=P, o=P, B=1, D=4, H=4, W=4, half=0: lib.modet_compose(a, b, o, B, D, H, W, half, None)
    assert comp(a=None) == E_NULL and comp(b=None) == E_NULL and comp(o=None) == E_NULL
    assert comp(H=0) == E_SHAPE and comp(o=ODD) == E_ALIGN
    assert comp(half=2) == E_SHAPE and comp(half=1, W=5) == E_SHAPE
    assert comp(B=64, D=512, H=512, W=512) == E_UNSUP
    integ = lambda v=P, o=P, t=P, B=1, D=4, H=4, W=4, T=3: lib.modet_integrate_velocity(v, o, t, B, D, H, W, T, None)
    assert integ(v=None) == E_NULL and integ(o=None) == E_NULL
    assert integ(t=None, T=2) == E_WS and integ(T=-1) == E_SHAPE and integ(T=31) == E_UNSUP
    assert integ(W=0) == E_SHAPE and integ(t=ODD) == E_ALIGN


def test_status_strings(lib):
    seen = set()
    for s in (OK, E_NULL, E_SHAPE, E_UNSUP, E_ALIGN, E_WS, E_LAUNCH):
        t = lib.modet_status_string(s)
        assert t and t not in seen
        seen.add(t)
    assert lib.modet_status_string(-99) == b"unknown status"
    assert lib.modet_version() >= 100


def test_tiled_kernel_coverage(lib):
    """The head counts of the paper's three model sizes (Section 4.4: heads of 6, 8 and 12 channels, up to 32
    heads at the coarsest level of the large model) all run on the LDS-tiled kernels; unusual head sizes and the
    wide windows of fp32 inputs fall to the generic ones."""
    lib.modet_has_tiled_kernels.restype = ctypes.c_int
    lib.modet_has_tiled_kernels.argtypes = [ctypes.c_int] * 4
    for d in (6, 8, 12):
        for heads in (1, 2, 4, 8, 16, 32):
            for dt in (0, 1):
                assert lib.modet_has_tiled_kernels(d * heads, heads, 3, dt) == 3, (d, heads, dt)
    assert lib.modet_has_tiled_kernels(384, 32, 3, 0) == 3
    assert lib.modet_has_tiled_kernels(8, 1, 5, 1) == 3 and lib.modet_has_tiled_kernels(8, 1, 5, 0) == 0
    assert lib.modet_has_tiled_kernels(10, 2, 3, 0) == 0 and lib.modet_has_tiled_kernels(24, 3, 3, 0) == 0
    assert lib.modet_has_tiled_kernels(8, 1, 7, 0) == 0
