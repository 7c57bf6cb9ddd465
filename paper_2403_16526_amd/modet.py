"""ctypes binding of libmodet (include/modet.h): argument marshalling only.

Every function takes torch tensors that already live on the GPU, passes their device
pointers and torch's current HIP stream to the C ABI, and raises on a non-zero status.
No arithmetic of the operator happens in Python, and there is no CPU fallback: if the
shared library is missing the import of this module fails.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("MODET_LIBRARY") or os.path.join(_HERE, "libmodet.so")   # override: another build of libmodet

MODET_F32, MODET_BF16 = 0, 1
MODET_OK = 0

EXPORTS = ("modet_fwd", "modet_bwd", "modet_bwd_static", "modet_bwd_workspace_bytes", "modet_warp", "modet_warp_bwd", "modet_compose",
           "modet_integrate_velocity", "modet_set_kernel_path", "modet_set_math_mode",
           "modet_has_tiled_kernels", "modet_status_string", "modet_version")

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2403_16526_amd.build` "
                      "(there is no fallback path)")
_lib = ctypes.CDLL(LIB_PATH)

_vp, _ci, _cf, _sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
_lib.modet_fwd.argtypes = [_vp] * 6 + [_ci] * 7 + [_cf, _ci, _vp]
_lib.modet_fwd.restype = _ci
_lib.modet_bwd.argtypes = [_vp] * 10 + [_ci] * 7 + [_cf, _ci, _vp, _sz, _vp]
_lib.modet_bwd.restype = _ci
_lib.modet_bwd_static.argtypes = [_vp] * 10 + [_ci] * 7 + [_cf, _ci, _vp]
_lib.modet_bwd_static.restype = _ci
_lib.modet_bwd_workspace_bytes.argtypes = [_ci] * 7 + [_ci, _ci]
_lib.modet_bwd_workspace_bytes.restype = _sz
_lib.modet_warp.argtypes = [_vp] * 3 + [_ci] * 5 + [_ci, _ci, _vp]
_lib.modet_warp_bwd.restype = _ci
_lib.modet_warp_bwd.argtypes = [_vp] * 5 + [_ci] * 5 + [_ci, _ci, _vp]
_lib.modet_compose.restype = _ci
_lib.modet_compose.argtypes = [_vp] * 3 + [_ci] * 5 + [_vp]
_lib.modet_integrate_velocity.restype = _ci
_lib.modet_integrate_velocity.argtypes = [_vp] * 3 + [_ci] * 5 + [_vp]
_lib.modet_warp.restype = _ci
_lib.modet_set_kernel_path.argtypes = [_ci]
_lib.modet_set_kernel_path.restype = _ci
_lib.modet_set_math_mode.argtypes = [_ci]
_lib.modet_set_math_mode.restype = _ci
_lib.modet_has_tiled_kernels.argtypes = [_ci] * 4
_lib.modet_has_tiled_kernels.restype = _ci
_lib.modet_status_string.argtypes = [_ci]
_lib.modet_status_string.restype = ctypes.c_char_p
_lib.modet_version.restype = _ci


class ModetError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"libmodet status {status}: {modet_status_string(status)}")


def modet_status_string(status: int) -> str:
    return _lib.modet_status_string(int(status)).decode()


def modet_version() -> int:
    return int(_lib.modet_version())


def modet_set_kernel_path(path: int) -> int:
    return int(_lib.modet_set_kernel_path(int(path)))


def modet_set_math_mode(mode: int) -> int:
    """0 = fp64 logits for fp32 inputs (default), 1 = fp32 logits (faster, ~1e-6 logit rounding)."""
    return int(_lib.modet_set_math_mode(int(mode)))


def modet_has_tiled_kernels(C: int, heads: int, k: int, dtype: int = MODET_F32) -> int:
    """bit 0: forward, bit 1: backward run on the LDS-tiled kernels."""
    return int(_lib.modet_has_tiled_kernels(C, heads, k, dtype))


def _check(rc: int):
    if rc != MODET_OK:
        raise ModetError(rc)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _in_dtype(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return MODET_F32
    if t.dtype == torch.bfloat16:
        return MODET_BF16
    raise TypeError(f"Q/K/src must be float32 or bfloat16, got {t.dtype}")


def _dev(*ts):
    for t in ts:
        if t is not None and not (t.is_cuda and t.is_contiguous()):
            raise ValueError("libmodet needs contiguous tensors in GPU memory")


def modet_fwd(Q, K, heads: int, k: int, scale: float = 0.0, bias=None, want_attn=False, want_lse=False, out=None):
    """phi [B,D,H,W,heads,3] (+ attn [..,k^3], + lse [B,D,H,W,heads]) for Q, K [B,D,H,W,C].
    `out` = (phi, lse) may be preallocated (then want_lse is implied) for use in timed loops."""
    _dev(Q, K, bias)
    B, D, H, W, C = Q.shape
    if K.shape != Q.shape or K.dtype != Q.dtype:
        raise ValueError("Q and K must have the same shape and dtype")
    f32 = dict(device=Q.device, dtype=torch.float32)
    if out is not None:
        phi, lse = out
        want_lse = True
    else:
        phi = torch.empty((B, D, H, W, heads, 3), **f32)
        lse = torch.empty((B, D, H, W, heads), **f32) if want_lse else None
    attn = torch.empty((B, D, H, W, heads, k ** 3), **f32) if want_attn else None
    _check(_lib.modet_fwd(_ptr(Q), _ptr(K), _ptr(bias), _ptr(phi), _ptr(attn), _ptr(lse), B, D, H, W, C, heads, k,
                          float(scale), _in_dtype(Q), _stream()))
    out = (phi,)
    if want_attn:
        out += (attn,)
    if want_lse:
        out += (lse,)
    return out if len(out) > 1 else phi


MODET_WS_HAVE_STATS, MODET_WS_WANT_DBIAS, MODET_WS_HAVE_DATTN = 1, 2, 4


def modet_bwd_workspace_bytes(B, D, H, W, C, heads, k, dtype=MODET_F32, have_stats=False, want_dbias=False,
                              have_dattn=False) -> int:
    flags = ((MODET_WS_HAVE_STATS if have_stats else 0) | (MODET_WS_WANT_DBIAS if want_dbias else 0) |
             (MODET_WS_HAVE_DATTN if have_dattn else 0))
    return int(_lib.modet_bwd_workspace_bytes(B, D, H, W, C, heads, k, dtype, flags))


def modet_bwd(Q, K, dphi, heads: int, k: int, scale: float = 0.0, bias=None, phi=None, lse=None,
              want_dbias=False, out=None, workspace=None, dattn=None):
    """dQ, dK [B,D,H,W,C] fp32 (+ dbias [heads,k^3]).  `phi`, `lse` are modet_fwd's outputs (optional); `dattn`
    [B,D,H,W,heads,k^3] is the upstream gradient of the attention weights when they were an output too.
    `out` = (dQ, dK) and `workspace` (uint8 tensor) may be preallocated for use in timed loops."""
    _dev(Q, K, dphi, bias, phi, lse, dattn)
    B, D, H, W, C = Q.shape
    f32 = dict(device=Q.device, dtype=torch.float32)
    dQ, dK = out if out is not None else (torch.empty(Q.shape, **f32), torch.empty(Q.shape, **f32))
    dbias = torch.empty((heads, k ** 3), **f32) if want_dbias else None
    need = modet_bwd_workspace_bytes(B, D, H, W, C, heads, k, _in_dtype(Q), phi is not None, want_dbias,
                                     dattn is not None)
    if workspace is None and need:
        workspace = torch.empty(need, device=Q.device, dtype=torch.uint8)
    wbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(_lib.modet_bwd(_ptr(Q), _ptr(K), _ptr(bias), _ptr(dphi), _ptr(dattn), _ptr(phi), _ptr(lse), _ptr(dQ), _ptr(dK),
                          _ptr(dbias), B, D, H, W, C, heads, k, float(scale), _in_dtype(Q), _ptr(workspace),
                          wbytes, _stream()))
    return (dQ, dK, dbias) if want_dbias else (dQ, dK)


MODET_STATIC_SCRATCH_BYTES = 8 << 20


def modet_bwd_static(Q, K, dphi, heads: int, k: int, out, scale: float = 0.0, bias=None, phi=None, lse=None,
                     dbias=None, dattn=None):
    """modet_bwd with the library's built-in scratch: nothing is allocated, here or in the library.  `out` =
    (dQ, dK) and, when the bias gradient is wanted, `dbias` [heads, k^3] are the caller's tensors."""
    _dev(Q, K, dphi, bias, phi, lse, dbias, dattn, *out)
    B, D, H, W, C = Q.shape
    dQ, dK = out
    _check(_lib.modet_bwd_static(_ptr(Q), _ptr(K), _ptr(bias), _ptr(dphi), _ptr(dattn), _ptr(phi), _ptr(lse), _ptr(dQ),
                                 _ptr(dK),
                                 _ptr(dbias), B, D, H, W, C, heads, k, float(scale), _in_dtype(Q), _stream()))
    return (dQ, dK, dbias) if dbias is not None else (dQ, dK)


def modet_warp(src, field, field_half_res: bool = False, out=None):
    """out[b,p,:] = trilinear(src[b], p + u(p)), zero outside; see include/modet.h."""
    _dev(src, field)
    B, D, H, W, C = src.shape
    if out is None:
        out = torch.empty_like(src)
    _check(_lib.modet_warp(_ptr(src), _ptr(field), _ptr(out), B, D, H, W, C, int(bool(field_half_res)),
                           _in_dtype(src), _stream()))
    return out


def modet_warp_bwd(src, field, dout, field_half_res: bool = False, want_dfield: bool = True, out=None):
    """Gradients of sum(dout * modet_warp(src, field)): dsrc [B,D,H,W,C] fp32 (+ dfield, shaped like field)."""
    _dev(src, field, dout)
    B, D, H, W, C = src.shape
    f32 = dict(device=src.device, dtype=torch.float32)
    dsrc = out if out is not None else torch.empty(src.shape, **f32)
    dfield = torch.empty(field.shape, **f32) if want_dfield else None
    _check(_lib.modet_warp_bwd(_ptr(src), _ptr(field), _ptr(dout), _ptr(dsrc), _ptr(dfield), B, D, H, W, C,
                               int(bool(field_half_res)), _in_dtype(src), _stream()))
    return (dsrc, dfield) if want_dfield else dsrc


def modet_compose(outer, inner, outer_half_res: bool = False, out=None):
    """out[b,p,:] = inner[b,p,:] + trilinear(outer[b], p + inner[b,p,:]); fields [B,D,H,W,3] fp32.  With
    outer_half_res, outer is [B,D/2,H/2,W/2,3] and stands for its 2x upsampling (values doubled)."""
    _dev(outer, inner)
    B, D, H, W, _ = inner.shape
    if out is None:
        out = torch.empty_like(inner)
    _check(_lib.modet_compose(_ptr(outer), _ptr(inner), _ptr(out), B, D, H, W, int(bool(outer_half_res)), _stream()))
    return out


def modet_integrate_velocity(v, T: int, out=None, tmp=None):
    """Scaling and squaring: phi_0 = v / 2^T, then T self-compositions; [B,D,H,W,3] fp32."""
    _dev(v)
    B, D, H, W, _ = v.shape
    if out is None:
        out = torch.empty_like(v)
    if tmp is None and T >= 2:
        tmp = torch.empty_like(v)
    _check(_lib.modet_integrate_velocity(_ptr(v), _ptr(out), _ptr(tmp), B, D, H, W, int(T), _stream()))
    return out
