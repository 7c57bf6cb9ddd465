"""Seeded synthetic inputs for the ModeT operator workloads.

This module only *generates inputs* (random features, smooth integer displacement
fields, upstream gradients, bf16 rounding of inputs).  It holds none of the operator's
arithmetic and imports neither the HIP binding nor the CPU oracle, so both sides can be
fed the very same arrays.

Random numbers are counter based: the value of element ``i`` of stream ``t`` under seed
``s`` depends on (s, t, i) only, never on the order or chunking of generation.

The shapes follow the volumes used in the paper's experiments (Section 4.1: brain MRI
160x192x224 / 160x192x160, abdominal CT 160x160x192-like), the five pyramid levels at
1/16 .. 1 resolution (Sections 3.1-3.2) and the window n = 3 (Section 4.4); the features
are unit-variance like LayerNorm outputs (Eq. 2).  No dataset item is reproduced.
"""
from __future__ import annotations

import numpy as np

_G = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 22

BASE_SEED = 240316526

# stream ids
S_Q, S_KNOISE, S_DISP, S_G, S_K, S_FIELD, S_LEVEL0 = 0, 1, 2, 3, 4, 5, 16


def _mix(x: np.ndarray) -> np.ndarray:
    """splitmix64 finaliser on a uint64 array (wrap-around arithmetic)."""
    x = x.copy()
    x ^= x >> np.uint64(30)
    x *= _M1
    x ^= x >> np.uint64(27)
    x *= _M2
    x ^= x >> np.uint64(31)
    return x


def _base(seed: int, stream: int) -> np.uint64:
    with np.errstate(over="ignore"):
        b = np.array([np.uint64(seed)], dtype=np.uint64)
        b = _mix(b + _G)
        b ^= _mix(np.array([np.uint64(stream)], dtype=np.uint64) * _G + _G)
        return _mix(b)[0]


def uniform01(seed: int, stream: int, n: int, which: int = 0, start: int = 0) -> np.ndarray:
    """n doubles in (0,1); `which` (0 or 1) selects one of two values per counter."""
    base = _base(seed, stream)
    out = np.empty(n, dtype=np.float64)
    with np.errstate(over="ignore"):
        for lo in range(0, n, _CHUNK):
            hi = min(n, lo + _CHUNK)
            i = np.arange(start + lo, start + hi, dtype=np.uint64)
            h = _mix(base + (i * np.uint64(2) + np.uint64(which + 1)) * _G)
            out[lo:hi] = ((h >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)
    return out


def normal(seed: int, stream: int, shape, start: int = 0, dtype=np.float32) -> np.ndarray:
    """Standard normal samples (Box-Muller, one value per counter)."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=dtype)
    for lo in range(0, n, _CHUNK):
        hi = min(n, lo + _CHUNK)
        u1 = uniform01(seed, stream, hi - lo, 0, start + lo)
        u2 = uniform01(seed, stream, hi - lo, 1, start + lo)
        out[lo:hi] = (np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)).astype(dtype)
    return out.reshape(shape)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bfloat16 (round-to-nearest-even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def smooth_integer_field(seed: int, stream: int, B: int, D: int, H: int, W: int, m: int) -> np.ndarray:
    """Integer displacement field u[B,D,H,W,3] with entries in [-m, m].

    Per axis: N(0,1) noise, periodic Gaussian blur (sigma = min(D,H,W)/10 voxels, applied as
    a product with the Gaussian's transfer function in the Fourier domain), normalised to
    unit standard deviation, scaled by 0.75*m, rounded to nearest and clamped.
    """
    sigma = min(D, H, W) / 10.0
    fz = np.fft.fftfreq(D)[:, None, None]
    fy = np.fft.fftfreq(H)[None, :, None]
    fx = np.fft.rfftfreq(W)[None, None, :]
    tf = np.exp(-2.0 * (np.pi * sigma) ** 2 * (fz * fz + fy * fy + fx * fx))
    u = np.empty((B, D, H, W, 3), dtype=np.int32)
    n = D * H * W
    for b in range(B):
        for a in range(3):
            noise = normal(seed, stream, (D, H, W), start=(b * 3 + a) * n, dtype=np.float64)
            sm = np.fft.irfftn(np.fft.rfftn(noise) * tf, s=(D, H, W), axes=(0, 1, 2))
            sd = sm.std()
            sm = sm / (sd if sd > 0 else 1.0)
            u[b, ..., a] = np.clip(np.rint(sm * (0.75 * m)), -m, m).astype(np.int32)
    return u


def displaced_keys(Q: np.ndarray, u: np.ndarray, seed: int, noise_std: float = 0.1) -> np.ndarray:
    """K[q] = Q[clamp(q - u(q))] + noise_std * N(0,1): the match of query p sits near p + u."""
    B, D, H, W, C = Q.shape
    K = np.empty_like(Q)
    zz, yy, xx = np.meshgrid(np.arange(D), np.arange(H), np.arange(W), indexing="ij")
    for b in range(B):
        sz = np.clip(zz - u[b, ..., 0], 0, D - 1)
        sy = np.clip(yy - u[b, ..., 1], 0, H - 1)
        sx = np.clip(xx - u[b, ..., 2], 0, W - 1)
        K[b] = Q[b][sz, sy, sx]
    K += noise_std * normal(seed, S_KNOISE, Q.shape)
    return K


# ---------------------------------------------------------------------------------------
# The workloads.  `keys`: "iid" = K independent N(0,1); "displaced" = K is Q moved by a
# smooth integer field in [-m, m] plus N(0, 0.1) noise (attention is peaked).
# ---------------------------------------------------------------------------------------
CONFIGS = {
    1: dict(name="tiny-16^3", B=1, D=16, H=16, W=16, C=8, heads=1, k=3, dtype="f32", keys="iid", m=0),
    2: dict(name="brain-coarse-40x48x56", B=1, D=40, H=48, W=56, C=32, heads=4, k=3, dtype="f32",
            keys="displaced", m=1),
    3: dict(name="brain-full-160x192x224", B=1, D=160, H=192, W=224, C=8, heads=1, k=3, dtype="f32",
            keys="displaced", m=1),
    5: dict(name="abdomen-ct-2x192x160x192-k5-bf16", B=2, D=192, H=160, W=192, C=16, heads=2, k=5,
            dtype="bf16", keys="displaced", m=2),
}

# config 4: the five pyramid levels of a 160x192x224 pair, coarse to fine
PYRAMID_LEVELS = [
    dict(D=10, H=12, W=14, C=64, heads=8),
    dict(D=20, H=24, W=28, C=32, heads=4),
    dict(D=40, H=48, W=56, C=32, heads=4),
    dict(D=80, H=96, W=112, C=16, heads=2),
    dict(D=160, H=192, W=224, C=8, heads=1),
]
PYRAMID_ITERS = 50


def make_case(B, D, H, W, C, heads, k, dtype="f32", keys="iid", m=0, seed=BASE_SEED, **_):
    """Build one operator call's inputs: Q, K (fp32, or bf16 bit patterns), dphi (fp32)."""
    shape = (B, D, H, W, C)
    Q = normal(seed, S_Q, shape)
    u = None
    if keys == "displaced":
        u = smooth_integer_field(seed, S_DISP, B, D, H, W, m)
        K = displaced_keys(Q, u, seed)
    else:
        K = normal(seed, S_K, shape)
    dphi = normal(seed, S_G, (B, D, H, W, heads, 3))
    if dtype == "bf16":
        Q, K = to_bf16_bits(Q), to_bf16_bits(K)
    return dict(Q=Q, K=K, dphi=dphi, u=u, B=B, D=D, H=H, W=W, C=C, heads=heads, k=k, dtype=dtype)


def make_config(no: int, **override):
    cfg = dict(CONFIGS[no])
    cfg.update(override)
    cfg.setdefault("seed", BASE_SEED + no)
    return make_case(**cfg)


def make_pyramid(seed: int = BASE_SEED + 4, levels=None):
    """Config 4: independent N(0,1) features Q_l, K_l per level, one upstream-gradient seed."""
    out = []
    for i, lv in enumerate(levels or PYRAMID_LEVELS):
        shape = (1, lv["D"], lv["H"], lv["W"], lv["C"])
        out.append(dict(Q=normal(seed, S_LEVEL0 + 2 * i, shape), K=normal(seed, S_LEVEL0 + 2 * i + 1, shape),
                        B=1, k=3, dtype="f32", **lv))
    return out


def smooth_real_field(seed: int, B: int, D: int, H: int, W: int, amp: float) -> np.ndarray:
    """Real-valued smooth displacement field [B,D,H,W,3] (voxel units) for the warp workload."""
    sigma = max(1.0, min(D, H, W) / 10.0)
    fz = np.fft.fftfreq(D)[:, None, None]
    fy = np.fft.fftfreq(H)[None, :, None]
    fx = np.fft.rfftfreq(W)[None, None, :]
    tf = np.exp(-2.0 * (np.pi * sigma) ** 2 * (fz * fz + fy * fy + fx * fx))
    f = np.empty((B, D, H, W, 3), dtype=np.float32)
    n = D * H * W
    for b in range(B):
        for a in range(3):
            noise = normal(seed, S_FIELD, (D, H, W), start=(b * 3 + a) * n, dtype=np.float64)
            sm = np.fft.irfftn(np.fft.rfftn(noise) * tf, s=(D, H, W), axes=(0, 1, 2))
            sd = sm.std()
            f[b, ..., a] = (amp * sm / (sd if sd > 0 else 1.0)).astype(np.float32)
    return f
