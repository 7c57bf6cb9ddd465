"""CPU oracle for the ModeT operator -- TEST INFRASTRUCTURE ONLY.

numpy-facing wrappers around oracle/modet_oracle.cpp (plain fp64 loops written from
Section 3.3.1, Eq. 3-5, and Section 3.1 of the paper).  Only tests, the smoke check and the
benchmark's CPU-baseline leg may import this package; the GPU library never does, and this
package never imports the GPU binding.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from .build_oracle import LIB, build

_lib = None
_DT = {"f32": 0, "bf16": 1, "f64": 2}
_NP = {"f32": np.float32, "bf16": np.uint16, "f64": np.float64}

_c_int = ctypes.c_int
_c_dbl = ctypes.c_double
_vp = ctypes.c_void_p
_i64 = ctypes.c_int64


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build(force=False))
        for name in ("oracle_modet_fwd", "oracle_modet_bwd_scatter", "oracle_modet_bwd_gather",
                     "oracle_modet_fwd_at", "oracle_modet_bwd_at", "oracle_warp", "oracle_warp_bwd",
                     "oracle_upsample2x", "oracle_threads", "oracle_set_threads"):
            getattr(_lib, name).restype = _c_int
    return _lib


def threads() -> int:
    return int(lib().oracle_threads())


def set_threads(n: int) -> int:
    """threads of the oracle's parallel loops from now on; returns the previous number."""
    return int(lib().oracle_set_threads(int(n)))


def _ptr(a):
    return None if a is None else a.ctypes.data_as(_vp)


def _prep(Q, K, dtype):
    Q = np.ascontiguousarray(Q, dtype=_NP[dtype])
    K = np.ascontiguousarray(K, dtype=_NP[dtype])
    assert Q.shape == K.shape and Q.ndim == 5
    return Q, K


def _scale(scale, C, heads):
    return float(scale) if scale is not None and scale > 0 else 1.0 / np.sqrt(C // heads)


def _bias(bias):
    return None if bias is None else np.ascontiguousarray(bias, dtype=np.float64)


def modet_fwd(Q, K, heads, k, scale=None, bias=None, dtype="f32", want_attn=False, want_lse=False):
    """phi[B,D,H,W,heads,3] (float64), optionally attn[...,k^3] and lse[...] (Eq. 3-5)."""
    Q, K = _prep(Q, K, dtype)
    B, D, H, W, C = Q.shape
    bias = _bias(bias)
    phi = np.empty((B, D, H, W, heads, 3), dtype=np.float64)
    attn = np.empty((B, D, H, W, heads, k ** 3), dtype=np.float64) if want_attn else None
    lse = np.empty((B, D, H, W, heads), dtype=np.float64) if want_lse else None
    rc = lib().oracle_modet_fwd(_ptr(Q), _ptr(K), _ptr(bias), B, D, H, W, C, heads, k,
                                _c_dbl(_scale(scale, C, heads)), _DT[dtype], _ptr(phi), _ptr(attn), _ptr(lse))
    assert rc == 0
    out = (phi,)
    if want_attn:
        out += (attn,)
    if want_lse:
        out += (lse,)
    return out if len(out) > 1 else phi


def modet_bwd(Q, K, dphi, heads, k, scale=None, bias=None, dtype="f32", form="gather", want_dbias=False, dattn=None):
    """dQ, dK [B,D,H,W,C] (float64) of L = sum(dphi * phi) (+ sum(dattn * attn) when the attention weights are an
    output with upstream gradient dattn [B,D,H,W,heads,k^3]); form = "scatter" | "gather"."""
    Q, K = _prep(Q, K, dtype)
    B, D, H, W, C = Q.shape
    bias = _bias(bias)
    g = np.ascontiguousarray(dphi, dtype=np.float64)
    assert g.shape == (B, D, H, W, heads, 3)
    da = None if dattn is None else np.ascontiguousarray(dattn, dtype=np.float64)
    assert da is None or da.shape == (B, D, H, W, heads, k ** 3)
    dQ = np.empty(Q.shape, dtype=np.float64)
    dK = np.empty(Q.shape, dtype=np.float64)
    sc = _c_dbl(_scale(scale, C, heads))
    if form == "scatter":
        db = np.empty((heads, k ** 3), dtype=np.float64)
        rc = lib().oracle_modet_bwd_scatter(_ptr(Q), _ptr(K), _ptr(bias), _ptr(g), _ptr(da), B, D, H, W, C, heads, k, sc,
                                            _DT[dtype], _ptr(dQ), _ptr(dK), _ptr(db))
        assert rc == 0
        return (dQ, dK, db) if want_dbias else (dQ, dK)
    assert not want_dbias
    rc = lib().oracle_modet_bwd_gather(_ptr(Q), _ptr(K), _ptr(bias), _ptr(g), _ptr(da), B, D, H, W, C, heads, k, sc,
                                       _DT[dtype], _ptr(dQ), _ptr(dK))
    assert rc == 0
    return dQ, dK


def modet_fwd_at(Q, K, idx, heads, k, scale=None, bias=None, dtype="f32"):
    """phi[n,3], lse[n] at the sampled windows idx (= voxel_linear_index*heads + head)."""
    Q, K = _prep(Q, K, dtype)
    B, D, H, W, C = Q.shape
    bias = _bias(bias)
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    phi = np.empty((idx.size, 3), dtype=np.float64)
    lse = np.empty(idx.size, dtype=np.float64)
    rc = lib().oracle_modet_fwd_at(_ptr(Q), _ptr(K), _ptr(bias), B, D, H, W, C, heads, k,
                                   _c_dbl(_scale(scale, C, heads)), _DT[dtype], _i64(idx.size), _ptr(idx),
                                   _ptr(phi), _ptr(lse))
    assert rc == 0
    return phi, lse


def modet_bwd_at(Q, K, dphi, idx, heads, k, scale=None, bias=None, dtype="f32"):
    """dQ[n,d], dK[n,d]: the head's d channels at the sampled (voxel, head) pairs idx."""
    Q, K = _prep(Q, K, dtype)
    B, D, H, W, C = Q.shape
    bias = _bias(bias)
    g = np.ascontiguousarray(dphi, dtype=np.float64)
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    d = C // heads
    dQ = np.empty((idx.size, d), dtype=np.float64)
    dK = np.empty((idx.size, d), dtype=np.float64)
    rc = lib().oracle_modet_bwd_at(_ptr(Q), _ptr(K), _ptr(bias), _ptr(g), B, D, H, W, C, heads, k,
                                   _c_dbl(_scale(scale, C, heads)), _DT[dtype], _i64(idx.size), _ptr(idx),
                                   _ptr(dQ), _ptr(dK))
    assert rc == 0
    return dQ, dK


def warp(src, field, field_half_res=False, dtype="f32"):
    """out[b,p,:] = trilinear(src[b], p + u(p)), zero outside (Section 3.1); float64 result."""
    src = np.ascontiguousarray(src, dtype=_NP[dtype])
    field = np.ascontiguousarray(field, dtype=np.float32)
    B, D, H, W, C = src.shape
    if field_half_res:
        assert D % 2 == 0 and H % 2 == 0 and W % 2 == 0 and field.shape == (B, D // 2, H // 2, W // 2, 3)
    else:
        assert field.shape == (B, D, H, W, 3)
    out = np.empty(src.shape, dtype=np.float64)
    rc = lib().oracle_warp(_ptr(src), _ptr(field), B, D, H, W, C, int(bool(field_half_res)), _DT[dtype], _ptr(out))
    assert rc == 0
    return out


def warp_bwd(src, field, dout, field_half_res=False, dtype="f32", want_dfield=True):
    """Gradients of L = sum(dout * warp(src, field)): dsrc [B,D,H,W,C] and dfield (shape of field), float64.
    The derivative with respect to a displacement is the one-sided (right) derivative where the sample point
    sits exactly on a voxel."""
    src = np.ascontiguousarray(src, dtype=_NP[dtype])
    field = np.ascontiguousarray(field, dtype=np.float32)
    dout = np.ascontiguousarray(dout, dtype=np.float64)
    B, D, H, W, C = src.shape
    assert dout.shape == src.shape
    if field_half_res:
        assert D % 2 == 0 and H % 2 == 0 and W % 2 == 0 and field.shape == (B, D // 2, H // 2, W // 2, 3)
    else:
        assert field.shape == (B, D, H, W, 3)
    dsrc = np.empty(src.shape, dtype=np.float64)
    dfield = np.empty(field.shape, dtype=np.float64) if want_dfield else None
    rc = lib().oracle_warp_bwd(_ptr(src), _ptr(field), _ptr(dout), B, D, H, W, C, int(bool(field_half_res)),
                               _DT[dtype], _ptr(dsrc), _ptr(dfield))
    assert rc == 0
    return (dsrc, dfield) if want_dfield else dsrc


def upsample2x(coarse):
    """2x upsampled displacement field with values doubled; [B,2Dc,2Hc,2Wc,3] float64."""
    coarse = np.ascontiguousarray(coarse, dtype=np.float32)
    B, Dc, Hc, Wc, _ = coarse.shape
    fine = np.empty((B, 2 * Dc, 2 * Hc, 2 * Wc, 3), dtype=np.float64)
    rc = lib().oracle_upsample2x(_ptr(coarse), B, 2 * Dc, 2 * Hc, 2 * Wc, _ptr(fine))
    assert rc == 0
    return fine


def compose(outer, inner, outer_half_res=False):
    """Displacement of "move by inner, then by outer" (Section 3.1): inner + outer sampled at p + inner(p);
    fields [B,D,H,W,3] (taken as fp32), float64 result.  outer_half_res: outer is the coarser level's field
    [B,D/2,H/2,W/2,3] and is upsampled (2x, values doubled) first, without rounding in between."""
    inner32 = np.ascontiguousarray(inner, dtype=np.float32)
    if outer_half_res:
        return inner32.astype(np.float64) + warp(upsample2x(outer), inner32, dtype="f64")
    return inner32.astype(np.float64) + warp(outer, inner32)


def integrate_velocity(v, T):
    """Scaling and squaring (Section 3.3.2, Eq. 6; the doubling recurrence of the work the paper cites for it):
    phi_0 = v / 2^T, then T times phi <- phi o phi.  Every intermediate field is an fp32 tensor, as it is for
    any caller that composes fields through the fp32 interface; float64 result of the last step."""
    phi = np.ascontiguousarray(v, dtype=np.float32) * np.float32(2.0 ** -T)
    out = phi.astype(np.float64)
    for t in range(T):
        out = compose(phi, phi)
        phi = out.astype(np.float32)
    return out

