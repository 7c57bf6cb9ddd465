// Trilinear feature warp between pyramid levels (paper Section 3.1): the moving features of the
// next level are resampled at p + u(p), where u is the total displacement field, either given at
// this resolution or given at half resolution and upsampled x2 (values doubled) on the fly.
// One lane handles VEC consecutive channels of one voxel, so a wavefront reads whole contiguous
// channel rows of each of the 8 corners; the work is pure gather bandwidth.
#include "modet_common.hpp"

namespace modet {
namespace {

constexpr int kThreads = 256;

template <class T, int VEC> struct Vec;
template <> struct Vec<float, 4> {
  static __device__ __forceinline__ void load(const float* p, float* v) {
    float4 t = *reinterpret_cast<const float4*>(p);
    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
  }
  static __device__ __forceinline__ void store(float* p, const float* v) {
    *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  }
};
template <> struct Vec<float, 2> {
  static __device__ __forceinline__ void load(const float* p, float* v) {
    float2 t = *reinterpret_cast<const float2*>(p);
    v[0] = t.x; v[1] = t.y;
  }
  static __device__ __forceinline__ void store(float* p, const float* v) {
    *reinterpret_cast<float2*>(p) = make_float2(v[0], v[1]);
  }
};
template <> struct Vec<float, 1> {
  static __device__ __forceinline__ void load(const float* p, float* v) { v[0] = p[0]; }
  static __device__ __forceinline__ void store(float* p, const float* v) { p[0] = v[0]; }
};
template <> struct Vec<bf16_t, 8> {
  static __device__ __forceinline__ void load(const bf16_t* p, float* v) {
    uint4 t = *reinterpret_cast<const uint4*>(p);
    uint32_t w[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = __uint_as_float(w[i] << 16);
      v[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
    }
  }
  static __device__ __forceinline__ void store(bf16_t* p, const float* v) {
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = (uint32_t)f2bf(v[2 * i]) | ((uint32_t)f2bf(v[2 * i + 1]) << 16);
    *reinterpret_cast<uint4*>(p) = make_uint4(w[0], w[1], w[2], w[3]);
  }
};

template <> struct Vec<bf16_t, 1> {
  static __device__ __forceinline__ void load(const bf16_t* p, float* v) { v[0] = __uint_as_float(((uint32_t)p[0]) << 16); }
  static __device__ __forceinline__ void store(bf16_t* p, const float* v) { p[0] = f2bf(v[0]); }
};
template <> struct Vec<bf16_t, 4> {
  static __device__ __forceinline__ void load(const bf16_t* p, float* v) {
    uint2 t = *reinterpret_cast<const uint2*>(p);
    v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xFFFF0000u);
    v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xFFFF0000u);
  }
  static __device__ __forceinline__ void store(bf16_t* p, const float* v) {
    *reinterpret_cast<uint2*>(p) = make_uint2((uint32_t)f2bf(v[0]) | ((uint32_t)f2bf(v[1]) << 16),
                                              (uint32_t)f2bf(v[2]) | ((uint32_t)f2bf(v[3]) << 16));
  }
};
template <> struct Vec<bf16_t, 2> {
  static __device__ __forceinline__ void load(const bf16_t* p, float* v) {
    const uint32_t t = *reinterpret_cast<const uint32_t*>(p);
    v[0] = __uint_as_float(t << 16); v[1] = __uint_as_float(t & 0xFFFF0000u);
  }
  static __device__ __forceinline__ void store(bf16_t* p, const float* v) {
    *reinterpret_cast<uint32_t*>(p) = (uint32_t)f2bf(v[0]) | ((uint32_t)f2bf(v[1]) << 16);
  }
};

// Half-resolution field: the fine voxel centre i sits at coarse coordinate (i + 0.5)/2 - 0.5 = i/2 - 0.25,
// clamped to the grid, so its lower coarse neighbour is (i - 1) >> 1 (0 for i = 0) and the weight of the
// upper one is 1/4 for odd i, 3/4 for even i >= 2 (0 at i = 0 and wherever the upper neighbour is clamped).
__device__ __forceinline__ int coarse_lo(int i) { return i > 0 ? (i - 1) >> 1 : 0; }

// The coarse voxels a brick of fine voxels needs, staged once per workgroup in LDS: per axis the range
// [coarse_lo(first), coarse_lo(last) + 1], at most extent/2 + 2 values.
constexpr int kMaxTile = 192;     // coarse voxels per workgroup: bricks are at most 16 x 4 x 4 -> 10 x 4 x 4
struct CoarseTile {
  int oz, oy, ox, nz, ny, nx;     // origin and extents (clamped to the coarse grid)
};

// displacement at fine voxel (z,y,x) from the staged tile.  The interpolation runs in fp64: an fp32 result
// would carry ~2e-7 of rounding on a displacement of a few voxels, and the warp multiplies that by the local
// feature gradient.
__device__ __forceinline__ void upsampled_disp(const float* __restrict__ tile, const CoarseTile& ct, int Dc, int Hc,
                                               int Wc, int z, int y, int x, double* u) {
  const int z0 = coarse_lo(z), y0 = coarse_lo(y), x0 = coarse_lo(x);
  const int z1 = min(z0 + 1, Dc - 1), y1 = min(y0 + 1, Hc - 1), x1 = min(x0 + 1, Wc - 1);
  // fractions are multiples of 1/4: exact in fp32; 0 where the coordinate was clamped
  const float tz = (z == 0 || z1 == z0) ? 0.f : ((z & 1) ? 0.25f : 0.75f);
  const float ty = (y == 0 || y1 == y0) ? 0.f : ((y & 1) ? 0.25f : 0.75f);
  const float tx = (x == 0 || x1 == x0) ? 0.f : ((x & 1) ? 0.25f : 0.75f);
  u[0] = u[1] = u[2] = 0.0;
#pragma unroll
  for (int c = 0; c < 8; ++c) {
    const int zi = ((c & 4) ? z1 : z0) - ct.oz, yi = ((c & 2) ? y1 : y0) - ct.oy, xi = ((c & 1) ? x1 : x0) - ct.ox;
    const double w = (double)(((c & 4) ? tz : 1.f - tz) * ((c & 2) ? ty : 1.f - ty) * ((c & 1) ? tx : 1.f - tx));
    const float* p = tile + ((zi * ct.ny + yi) * ct.nx + xi) * 3;
    u[0] = fma(w, (double)p[0], u[0]); u[1] = fma(w, (double)p[1], u[1]); u[2] = fma(w, (double)p[2], u[2]);
  }
  u[0] *= 2.0; u[1] *= 2.0; u[2] *= 2.0;
}

// Work mapping: a workgroup handles a brick of BX x BY x BZ voxels (x fastest, then the channel chunk
// inside a voxel), so the 8 corners of neighbouring voxels are found in the CU's own L1 instead of being
// re-fetched from L2 by another workgroup, and bricks are numbered so that every XCD (own L2) gets one
// contiguous slab of the volume.
struct Brick { int bx, by, bz, nbx, nby, nbz, sc, sx, sy; };   // sc, sx, sy: log2 of nchunk, bx, by (or -1)

inline Brick make_brick(int D, int H, int W, int nchunk) {
  const int vpb = kThreads / nchunk;            // voxels per workgroup (a few lanes idle if it does not divide)
  Brick bk;
  bk.bx = vpb >= 16 ? 16 : vpb;
  bk.by = vpb / bk.bx >= 4 ? 4 : (vpb / bk.bx >= 2 ? 2 : 1);
  bk.bz = vpb / (bk.bx * bk.by);
  if (bk.bz < 1) bk.bz = 1;
  bk.nbx = (W + bk.bx - 1) / bk.bx;
  bk.nby = (H + bk.by - 1) / bk.by;
  bk.nbz = (D + bk.bz - 1) / bk.bz;
  auto lg = [](int n) { int s = 0; while ((1 << s) < n) ++s; return (1 << s) == n ? s : -1; };
  bk.sc = lg(nchunk); bk.sx = lg(bk.bx); bk.sy = lg(bk.by);
  if (bk.sx < 0 || bk.sy < 0) bk.sc = -1;
  return bk;
}


template <class T, int VEC, bool HALF>
__global__ void __launch_bounds__(kThreads)
warp_kernel(const T* __restrict__ src, const float* __restrict__ field, T* __restrict__ out, int B, int D, int H,
            int W, int C, Brick bk) {
  const unsigned nb = gridDim.x, xcd = blockIdx.x & 7u, q = nb >> 3, rem = nb & 7u;
  unsigned blk = xcd * q + (xcd < rem ? xcd : rem) + (blockIdx.x >> 3);
  // per-lane index split with shifts when the channel-chunk count is a power of two (no integer division)
  int chunk, lx, ly, lz;
  if (bk.sc >= 0) {
    int t = threadIdx.x;
    chunk = t & ((1 << bk.sc) - 1); t >>= bk.sc;
    lx = t & (bk.bx - 1); t >>= bk.sx;
    ly = t & (bk.by - 1);
    lz = t >> bk.sy;
  } else {
    const int nchunk = C / VEC;
    chunk = threadIdx.x % nchunk;
    int t = threadIdx.x / nchunk;
    lx = t % bk.bx; t /= bk.bx;
    ly = t % bk.by;
    lz = t / bk.by;
  }
  const int ibx = blk % bk.nbx; blk /= bk.nbx;
  const int iby = blk % bk.nby; blk /= bk.nby;
  const int ibz = blk % bk.nbz;
  const int b = blk / bk.nbz;
  const int x = ibx * bk.bx + lx, y = iby * bk.by + ly, z = ibz * bk.bz + lz;
  const bool live = lz < bk.bz && x < W && y < H && z < D;
  __shared__ float tile[HALF ? kMaxTile * 3 : 1];
  CoarseTile ct = {};
  if (HALF) {
    // stage the coarse voxels this brick needs (every lane helps, also those outside the volume)
    const int Dc = D / 2, Hc = H / 2, Wc = W / 2;
    const int xf = ibx * bk.bx, yf = iby * bk.by, zf = ibz * bk.bz;
    ct.ox = coarse_lo(xf); ct.oy = coarse_lo(yf); ct.oz = coarse_lo(zf);
    ct.nx = min(coarse_lo(min(xf + bk.bx, W) - 1) + 1, Wc - 1) - ct.ox + 1;
    ct.ny = min(coarse_lo(min(yf + bk.by, H) - 1) + 1, Hc - 1) - ct.oy + 1;
    ct.nz = min(coarse_lo(min(zf + bk.bz, D) - 1) + 1, Dc - 1) - ct.oz + 1;
    const float* fc = field + (long long)b * Dc * Hc * Wc * 3;
    const int n = ct.nx * ct.ny * ct.nz;
    for (int e = threadIdx.x; e < n; e += kThreads) {
      const int ex = e % ct.nx, ey = (e / ct.nx) % ct.ny, ez = e / (ct.nx * ct.ny);
      const float* p = fc + (((long long)(ct.oz + ez) * Hc + ct.oy + ey) * Wc + ct.ox + ex) * 3;
      tile[e * 3] = p[0]; tile[e * 3 + 1] = p[1]; tile[e * 3 + 2] = p[2];
    }
    __syncthreads();
  }
  if (!live) return;
  const long long v = (((long long)b * D + z) * H + y) * W + x;
  double u[3];
  if (HALF) {
    upsampled_disp(tile, ct, D / 2, H / 2, W / 2, z, y, x, u);
  } else {
    u[0] = field[v * 3]; u[1] = field[v * 3 + 1]; u[2] = field[v * 3 + 2];
  }
  // split u into integer and fractional parts first: the fraction of an fp32 displacement is then exact
  const double fz = floor(u[0]), fy = floor(u[1]), fx = floor(u[2]);
  const float tz = (float)(u[0] - fz), ty = (float)(u[1] - fy), tx = (float)(u[2] - fx);
  // clamp the integer part far outside the volume so z + fz cannot overflow an int
  const int z0 = z + (int)fmin(fmax(fz, -1.0e6), 1.0e6);
  const int y0 = y + (int)fmin(fmax(fy, -1.0e6), 1.0e6);
  const int x0 = x + (int)fmin(fmax(fx, -1.0e6), 1.0e6);
  const T* sb = src + (long long)b * D * H * W * C + chunk * VEC;
  // all 8 corner loads are issued before any is consumed (addresses clamped into the volume, values of
  // corners outside it replaced by zero afterwards): one memory round trip per lane instead of eight
  float val[8][VEC];
  bool in[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) {
    const int zi = z0 + ((c >> 2) & 1), yi = y0 + ((c >> 1) & 1), xi = x0 + (c & 1);
    in[c] = (unsigned)zi < (unsigned)D && (unsigned)yi < (unsigned)H && (unsigned)xi < (unsigned)W;
    const int zc = min(max(zi, 0), D - 1), yc = min(max(yi, 0), H - 1), xc = min(max(xi, 0), W - 1);
    Vec<T, VEC>::load(sb + (((long long)zc * H + yc) * W + xc) * C, val[c]);
  }
  float acc[VEC];
#pragma unroll
  for (int i = 0; i < VEC; ++i) acc[i] = 0.f;
#pragma unroll
  for (int c = 0; c < 8; ++c) {
    const float w = ((c & 4) ? tz : 1.f - tz) * ((c & 2) ? ty : 1.f - ty) * ((c & 1) ? tx : 1.f - tx);
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = fmaf(w, in[c] ? val[c][i] : 0.f, acc[i]);
  }
  Vec<T, VEC>::store(out + v * C + chunk * VEC, acc);
}

template <class T, int VEC>
hipError_t launch_t(const void* src, const float* field, void* out, int B, int D, int H, int W, int C, int half,
                    hipStream_t st) {
  const Brick bk = make_brick(D, H, W, C / VEC);
  dim3 grid((unsigned)((long long)bk.nbx * bk.nby * bk.nbz * B)), block(kThreads);
  if (half)
    hipLaunchKernelGGL((warp_kernel<T, VEC, true>), grid, block, 0, st, (const T*)src, field, (T*)out, B, D, H, W,
                       C, bk);
  else
    hipLaunchKernelGGL((warp_kernel<T, VEC, false>), grid, block, 0, st, (const T*)src, field, (T*)out, B, D, H, W,
                       C, bk);
  return hipGetLastError();
}

// ---- adjoint of the warp --------------------------------------------------------------------------
// Gradients of L = sum(dout * warp(src, field)).  Same work mapping as the warp: one lane per (voxel, channel
// chunk).  The source gradient is the transpose of the gather, a scatter: each lane adds weight * dout to the
// eight corners it would have read, with hardware fp32 atomics (the order of the additions, hence the last
// bits of the result, is not fixed).  The field gradient differentiates the corner weights: per corner the dot
// product of dout with the source values, signed by the side of the corner along the axis; the lanes of one
// voxel are summed by lane shuffles when they form an aligned power-of-two group, and one of them writes
// (full resolution) or scatters through the 2x upsampling weights (half resolution).
__global__ void zero_kernel(float* p, long long n) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0.f;
}

template <class T, int VEC, bool HALF, bool FIELD>
__global__ void __launch_bounds__(kThreads)
warp_bwd_kernel(const T* __restrict__ src, const float* __restrict__ field, const float* __restrict__ dout,
                float* __restrict__ dsrc, float* __restrict__ dfield, int B, int D, int H, int W, int C, Brick bk) {
  const unsigned nb = gridDim.x, xcd = blockIdx.x & 7u, q = nb >> 3, rem = nb & 7u;
  unsigned blk = xcd * q + (xcd < rem ? xcd : rem) + (blockIdx.x >> 3);
  int chunk, lx, ly, lz;
  if (bk.sc >= 0) {
    int t = threadIdx.x;
    chunk = t & ((1 << bk.sc) - 1); t >>= bk.sc;
    lx = t & (bk.bx - 1); t >>= bk.sx;
    ly = t & (bk.by - 1);
    lz = t >> bk.sy;
  } else {
    const int nchunk = C / VEC;
    chunk = threadIdx.x % nchunk;
    int t = threadIdx.x / nchunk;
    lx = t % bk.bx; t /= bk.bx;
    ly = t % bk.by;
    lz = t / bk.by;
  }
  const int ibx = blk % bk.nbx; blk /= bk.nbx;
  const int iby = blk % bk.nby; blk /= bk.nby;
  const int ibz = blk % bk.nbz;
  const int b = blk / bk.nbz;
  const int x = ibx * bk.bx + lx, y = iby * bk.by + ly, z = ibz * bk.bz + lz;
  const bool live = lz < bk.bz && x < W && y < H && z < D;
  __shared__ float tile[HALF ? kMaxTile * 3 : 1];
  __shared__ float dtile[(HALF && FIELD) ? kMaxTile * 3 : 1];      // gradient of the staged coarse voxels
  CoarseTile ct = {};
  const int Dc = D / 2, Hc = H / 2, Wc = W / 2;
  if (HALF) {
    const int xf = ibx * bk.bx, yf = iby * bk.by, zf = ibz * bk.bz;
    ct.ox = coarse_lo(xf); ct.oy = coarse_lo(yf); ct.oz = coarse_lo(zf);
    ct.nx = min(coarse_lo(min(xf + bk.bx, W) - 1) + 1, Wc - 1) - ct.ox + 1;
    ct.ny = min(coarse_lo(min(yf + bk.by, H) - 1) + 1, Hc - 1) - ct.oy + 1;
    ct.nz = min(coarse_lo(min(zf + bk.bz, D) - 1) + 1, Dc - 1) - ct.oz + 1;
    const float* fc = field + (long long)b * Dc * Hc * Wc * 3;
    const int n = ct.nx * ct.ny * ct.nz;
    for (int e = threadIdx.x; e < n; e += kThreads) {
      const int ex = e % ct.nx, ey = (e / ct.nx) % ct.ny, ez = e / (ct.nx * ct.ny);
      const float* p = fc + (((long long)(ct.oz + ez) * Hc + ct.oy + ey) * Wc + ct.ox + ex) * 3;
      tile[e * 3] = p[0]; tile[e * 3 + 1] = p[1]; tile[e * 3 + 2] = p[2];
      if (FIELD) { dtile[e * 3] = 0.f; dtile[e * 3 + 1] = 0.f; dtile[e * 3 + 2] = 0.f; }
    }
    __syncthreads();
  }
  // (nobody leaves early: the scatter below moves values between neighbouring lanes, and with a half-resolution
  // field gradient everybody meets again at a barrier)
  float du[3] = {0.f, 0.f, 0.f};
  bool writer = false;       // does this lane hold the voxel's whole sum?
  bool single = false;
  int z0 = 0, y0 = 0, x0 = 0;
  float tz = 0.f, ty = 0.f, tx = 0.f;
  float g[VEC];
#pragma unroll
  for (int i = 0; i < VEC; ++i) g[i] = 0.f;
  const long long vol = (long long)b * D * H * W * C + chunk * VEC;
  if (live) {
    const long long v = (((long long)b * D + z) * H + y) * W + x;
    double u[3];
    if (HALF) {
      upsampled_disp(tile, ct, Dc, Hc, Wc, z, y, x, u);
    } else {
      u[0] = field[v * 3]; u[1] = field[v * 3 + 1]; u[2] = field[v * 3 + 2];
    }
    const double fz = floor(u[0]), fy = floor(u[1]), fx = floor(u[2]);
    tz = (float)(u[0] - fz); ty = (float)(u[1] - fy); tx = (float)(u[2] - fx);
    z0 = z + (int)fmin(fmax(fz, -1.0e6), 1.0e6);
    y0 = y + (int)fmin(fmax(fy, -1.0e6), 1.0e6);
    x0 = x + (int)fmin(fmax(fx, -1.0e6), 1.0e6);
    Vec<float, VEC>::load(dout + v * C + chunk * VEC, g);
    if (FIELD) {
      float val[8][VEC];
      bool in[8];
#pragma unroll
      for (int c = 0; c < 8; ++c) {     // all corner loads first, from clamped addresses
        const int zi = z0 + ((c >> 2) & 1), yi = y0 + ((c >> 1) & 1), xi = x0 + (c & 1);
        in[c] = (unsigned)zi < (unsigned)D && (unsigned)yi < (unsigned)H && (unsigned)xi < (unsigned)W;
        const int zc = min(max(zi, 0), D - 1), yc = min(max(yi, 0), H - 1), xc = min(max(xi, 0), W - 1);
        Vec<T, VEC>::load(src + vol + (((long long)zc * H + yc) * W + xc) * C, val[c]);
      }
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        const float wz = (c & 4) ? tz : 1.f - tz, wy = (c & 2) ? ty : 1.f - ty, wx = (c & 1) ? tx : 1.f - tx;
        if (in[c]) {
          float dot = 0.f;
#pragma unroll
          for (int i = 0; i < VEC; ++i) dot = fmaf(g[i], val[c][i], dot);
          du[0] = fmaf(((c & 4) ? wy : -wy) * wx, dot, du[0]);
          du[1] = fmaf(((c & 2) ? wz : -wz) * wx, dot, du[1]);
          du[2] = fmaf(((c & 1) ? wz : -wz) * wy, dot, du[2]);
        }
      }
      writer = true;
      if (bk.sc >= 0) {        // (uniform) the voxel's lanes are an aligned group of 2^sc lanes
        for (int m = 1; m < (1 << bk.sc); m <<= 1) {
          du[0] += __shfl_xor(du[0], m); du[1] += __shfl_xor(du[1], m); du[2] += __shfl_xor(du[2], m);
        }
        writer = chunk == 0;
        single = true;
      }
      if (!HALF && writer) {
        float* o = dfield + v * 3;
        if (single) {          // the only writer of this voxel's entry
          o[0] = du[0]; o[1] = du[1]; o[2] = du[2];
        } else {
          unsafeAtomicAdd(o, du[0]); unsafeAtomicAdd(o + 1, du[1]); unsafeAtomicAdd(o + 2, du[2]);
        }
      }
    }
  }
  // ---- the scatter: weight * dout to the eight corners.  The upper-x corner of a voxel is the lower-x corner
  // of its x-neighbour whenever both have the same integer displacement, which a smooth field gives almost
  // always: the neighbour's lane (2^sc lanes up, when the voxel's lanes are such an aligned group) then takes
  // the contribution over and adds both with one atomic, which nearly halves the cache lines the atomic units
  // have to work through.
  const bool comb = bk.sc >= 0;                 // uniform
  const int nch = comb ? 1 << bk.sc : 1;
  const int lane = threadIdx.x & 63;
  bool same_prev = false, next_same = false;
  if (comb) {
    const int pz = __shfl_up(z0, nch), py = __shfl_up(y0, nch), px = __shfl_up(x0, nch);
    const int pl = __shfl_up((int)live, nch);
    same_prev = live && pl != 0 && lane >= nch && lx > 0 && pz == z0 && py == y0 && px + 1 == x0;
    next_same = __shfl_down((int)same_prev, nch) != 0 && lane + nch < 64;
  }
#pragma unroll
  for (int r = 0; r < 4; ++r) {                 // the four (z, y) corner rows
    const float wzy = ((r & 2) ? tz : 1.f - tz) * ((r & 1) ? ty : 1.f - ty);
    float lo[VEC], hi[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) { lo[i] = wzy * (1.f - tx) * g[i]; hi[i] = wzy * tx * g[i]; }
    if (comb) {
#pragma unroll
      for (int i = 0; i < VEC; ++i) {
        const float from_prev = __shfl_up(hi[i], nch);
        if (same_prev) lo[i] += from_prev;
      }
    }
    const int zi = z0 + (r >> 1), yi = y0 + (r & 1);
    if (live && (unsigned)zi < (unsigned)D && (unsigned)yi < (unsigned)H) {
      float* row = dsrc + vol + ((long long)zi * H + yi) * W * C;
      if ((unsigned)x0 < (unsigned)W) {
#pragma unroll
        for (int i = 0; i < VEC; ++i) unsafeAtomicAdd(row + (long long)x0 * C + i, lo[i]);
      }
      if (!next_same && (unsigned)(x0 + 1) < (unsigned)W) {
#pragma unroll
        for (int i = 0; i < VEC; ++i) unsafeAtomicAdd(row + (long long)(x0 + 1) * C + i, hi[i]);
      }
    }
  }
  if (!(HALF && FIELD)) return;
  // Half resolution: u = 2 * sum of weight * coarse value over the (clamped) coarse corners of a voxel, and up to
  // 64 fine voxels share a coarse one.  The workgroup first sums into its LDS copy of the coarse tile, then adds
  // every tile entry to the global gradient once.
  if (live && writer) {
    const int cz0 = coarse_lo(z), cy0 = coarse_lo(y), cx0 = coarse_lo(x);
    const int cz1 = min(cz0 + 1, Dc - 1), cy1 = min(cy0 + 1, Hc - 1), cx1 = min(cx0 + 1, Wc - 1);
    const float sz = (z == 0 || cz1 == cz0) ? 0.f : ((z & 1) ? 0.25f : 0.75f);
    const float sy = (y == 0 || cy1 == cy0) ? 0.f : ((y & 1) ? 0.25f : 0.75f);
    const float sx = (x == 0 || cx1 == cx0) ? 0.f : ((x & 1) ? 0.25f : 0.75f);
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      const float w = 2.f * ((c & 4) ? sz : 1.f - sz) * ((c & 2) ? sy : 1.f - sy) * ((c & 1) ? sx : 1.f - sx);
      if (w == 0.f) continue;
      const int zi = ((c & 4) ? cz1 : cz0) - ct.oz, yi = ((c & 2) ? cy1 : cy0) - ct.oy, xi = ((c & 1) ? cx1 : cx0) - ct.ox;
      float* o = dtile + ((zi * ct.ny + yi) * ct.nx + xi) * 3;
#pragma unroll
      for (int a = 0; a < 3; ++a)
        __hip_atomic_fetch_add(o + a, w * du[a], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
  }
  __syncthreads();
  float* dc = dfield + (long long)b * Dc * Hc * Wc * 3;
  const int n = ct.nx * ct.ny * ct.nz;
  for (int e = threadIdx.x; e < n; e += kThreads) {
    const int ex = e % ct.nx, ey = (e / ct.nx) % ct.ny, ez = e / (ct.nx * ct.ny);
    float* o = dc + (((long long)(ct.oz + ez) * Hc + ct.oy + ey) * Wc + ct.ox + ex) * 3;
    unsafeAtomicAdd(o, dtile[e * 3]); unsafeAtomicAdd(o + 1, dtile[e * 3 + 1]); unsafeAtomicAdd(o + 2, dtile[e * 3 + 2]);
  }
}


template <class T, int VEC>
hipError_t launch_bwd_t(const void* src, const float* field, const float* dout, float* dsrc, float* dfield, int B,
                        int D, int H, int W, int C, int half, hipStream_t st) {
  const Brick bk = make_brick(D, H, W, C / VEC);
  const long long n = (long long)B * D * H * W * C;
  hipLaunchKernelGGL(zero_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, dsrc, n);
  // the field gradient is accumulated with atomics unless every entry has exactly one writer
  if (dfield && (half || bk.sc < 0)) {
    const long long nf = half ? (long long)B * (D / 2) * (H / 2) * (W / 2) * 3 : (long long)B * D * H * W * 3;
    hipLaunchKernelGGL(zero_kernel, dim3((unsigned)((nf + 255) / 256)), dim3(256), 0, st, dfield, nf);
  }
  dim3 grid((unsigned)((long long)bk.nbx * bk.nby * bk.nbz * B)), block(kThreads);
#define MODET_WB(HALF_, FIELD_)                                                                                      \
  hipLaunchKernelGGL((warp_bwd_kernel<T, VEC, HALF_, FIELD_>), grid, block, 0, st, (const T*)src, field, dout, dsrc, \
                     dfield, B, D, H, W, C, bk)
  if (half) { if (dfield) MODET_WB(true, true); else MODET_WB(true, false); }
  else { if (dfield) MODET_WB(false, true); else MODET_WB(false, false); }
#undef MODET_WB
  return hipGetLastError();
}

// ---- composition of displacement fields --------------------------------------------------------------
// out[p] = s * (inner[p] + trilinear(outer, p + s * inner[p])), zero outside the volume, one lane per voxel
// (three channels share the corner weights).  s = 1 is the composition of Section 3.1 (a level's residual
// field with the upsampled total field of the level below); s = 2^-T folds the scaling of a velocity
// field into the first squaring step of the integration of Eq. 6 (scaling by a power of two is exact).
struct Disp { float z, y, x; };      // one voxel of a field: a single 12-byte load or store

__global__ void __launch_bounds__(kThreads)
compose_kernel(const float* __restrict__ outer, const float* __restrict__ inner, float* __restrict__ out, int B,
               int D, int H, int W, float s) {
  // (32-bit indices: the host has checked that the field has fewer than 2^31 elements)
  const int nvox = B * D * H * W;
  const int v = blockIdx.x * kThreads + threadIdx.x;
  if (v >= nvox) return;
  int t = v;
  const int x = t % W; t /= W;
  const int y = t % H; t /= H;
  const int z = t % D;
  const int b = t / D;
  const Disp iv = *reinterpret_cast<const Disp*>(inner + v * 3);
  const float i0 = iv.z, i1 = iv.y, i2 = iv.x;
  const float u0 = s * i0, u1 = s * i1, u2 = s * i2;      // exact: s is a power of two
  // integer and fractional parts as in the warp kernel; both are exact in fp32 for an fp32 displacement
  const float fz = floorf(u0), fy = floorf(u1), fx = floorf(u2);
  const float tz = u0 - fz, ty = u1 - fy, tx = u2 - fx;
  const int z0 = z + (int)fminf(fmaxf(fz, -1.0e6f), 1.0e6f);
  const int y0 = y + (int)fminf(fmaxf(fy, -1.0e6f), 1.0e6f);
  const int x0 = x + (int)fminf(fmaxf(fx, -1.0e6f), 1.0e6f);
  const float* ob = outer + b * (D * H * W * 3);
  float val[8][3];
  bool in[8];
  // per axis: is the lower / upper corner inside, and its clamped index
  const bool zin[2] = {(unsigned)z0 < (unsigned)D, (unsigned)(z0 + 1) < (unsigned)D};
  const bool yin[2] = {(unsigned)y0 < (unsigned)H, (unsigned)(y0 + 1) < (unsigned)H};
  const bool xin[2] = {(unsigned)x0 < (unsigned)W, (unsigned)(x0 + 1) < (unsigned)W};
  const int zc[2] = {min(max(z0, 0), D - 1) * H, min(max(z0 + 1, 0), D - 1) * H};
  const int yc[2] = {min(max(y0, 0), H - 1), min(max(y0 + 1, 0), H - 1)};
  const int xc[2] = {min(max(x0, 0), W - 1), min(max(x0 + 1, 0), W - 1)};
#pragma unroll
  for (int c = 0; c < 8; ++c) {     // all corner loads first, from clamped addresses
    in[c] = zin[(c >> 2) & 1] && yin[(c >> 1) & 1] && xin[c & 1];
    const Disp q = *reinterpret_cast<const Disp*>(ob + ((zc[(c >> 2) & 1] + yc[(c >> 1) & 1]) * W + xc[c & 1]) * 3);
    val[c][0] = q.z; val[c][1] = q.y; val[c][2] = q.x;
  }
  float acc[3] = {0.f, 0.f, 0.f};
#pragma unroll
  for (int c = 0; c < 8; ++c) {
    const float w = ((c & 4) ? tz : 1.f - tz) * ((c & 2) ? ty : 1.f - ty) * ((c & 1) ? tx : 1.f - tx);
#pragma unroll
    for (int i = 0; i < 3; ++i) acc[i] = fmaf(w, in[c] ? val[c][i] : 0.f, acc[i]);
  }
  Disp r;
  r.z = s * (i0 + acc[0]); r.y = s * (i1 + acc[1]); r.x = s * (i2 + acc[2]);
  *reinterpret_cast<Disp*>(out + v * 3) = r;
}

// The same with the outer field given at half resolution [B, D/2, H/2, W/2, 3]: the value of the 2x upsampled
// field (values doubled) at each of the eight fine corners around p + inner(p) is itself a trilinear mix of
// coarse voxels, and per axis the two fine corners together touch at most three consecutive coarse voxels.  The
// two interpolations are folded into one table of three weights per axis (fp64: the factors are exact, the
// result is rounded once) over a 3 x 3 x 3 coarse neighbourhood, so the upsampled field is never materialised.
// Fine corners outside the volume contribute nothing (zero padding of the fine field); inside, the upsampling
// clamps its coarse coordinates like the warp's.
__device__ __forceinline__ void axis_table(int i0, float t, int N, int& base, double (&w)[3]) {
  const int Nc = N >> 1;
  w[0] = w[1] = w[2] = 0.0;
  base = -1;
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int i = i0 + j;
    if ((unsigned)i >= (unsigned)N) continue;                    // this fine corner is outside: weight 0
    const double cw = j ? (double)t : 1.0 - (double)t;
    const int lo = coarse_lo(i), hi = min(lo + 1, Nc - 1);
    const double f = (i == 0 || hi == lo) ? 0.0 : ((i & 1) ? 0.25 : 0.75);
    if (base < 0) base = lo;
    w[lo - base] += cw * (1.0 - f);
    w[hi - base] += cw * f;
  }
  if (base < 0) base = 0;
}

__global__ void __launch_bounds__(kThreads)
compose_up_kernel(const float* __restrict__ outer_c, const float* __restrict__ inner, float* __restrict__ out, int B,
                  int D, int H, int W) {
  const int nvox = B * D * H * W;
  const int v = blockIdx.x * kThreads + threadIdx.x;
  if (v >= nvox) return;
  int t = v;
  const int x = t % W; t /= W;
  const int y = t % H; t /= H;
  const int z = t % D;
  const int b = t / D;
  const Disp iv = *reinterpret_cast<const Disp*>(inner + v * 3);
  const float fz = floorf(iv.z), fy = floorf(iv.y), fx = floorf(iv.x);
  const float tz = iv.z - fz, ty = iv.y - fy, tx = iv.x - fx;
  const int z0 = z + (int)fminf(fmaxf(fz, -1.0e6f), 1.0e6f);
  const int y0 = y + (int)fminf(fmaxf(fy, -1.0e6f), 1.0e6f);
  const int x0 = x + (int)fminf(fmaxf(fx, -1.0e6f), 1.0e6f);
  int bz, by, bx;
  double wz[3], wy[3], wx[3];
  axis_table(z0, tz, D, bz, wz);
  axis_table(y0, ty, H, by, wy);
  axis_table(x0, tx, W, bx, wx);
  const int Dc = D >> 1, Hc = H >> 1, Wc = W >> 1;
  const float* ob = outer_c + b * (Dc * Hc * Wc * 3);
  Disp val[27];
#pragma unroll
  for (int c = 0; c < 27; ++c) {      // all loads first, from clamped addresses (a clamped one has weight 0)
    const int zi = min(bz + c / 9, Dc - 1), yi = min(by + (c / 3) % 3, Hc - 1), xi = min(bx + c % 3, Wc - 1);
    val[c] = *reinterpret_cast<const Disp*>(ob + ((zi * Hc + yi) * Wc + xi) * 3);
  }
  double acc[3] = {0.0, 0.0, 0.0};
#pragma unroll
  for (int c = 0; c < 27; ++c) {
    const double w = wz[c / 9] * wy[(c / 3) % 3] * wx[c % 3];
    acc[0] = fma(w, (double)val[c].z, acc[0]);
    acc[1] = fma(w, (double)val[c].y, acc[1]);
    acc[2] = fma(w, (double)val[c].x, acc[2]);
  }
  Disp r;
  r.z = (float)((double)iv.z + 2.0 * acc[0]); r.y = (float)((double)iv.y + 2.0 * acc[1]);
  r.x = (float)((double)iv.x + 2.0 * acc[2]);
  *reinterpret_cast<Disp*>(out + v * 3) = r;
}

}  // namespace

hipError_t launch_compose(const float* outer, const float* inner, float* out, int B, int D, int H, int W, float s,
                          int outer_half_res, hipStream_t st) {
  const long long nvox = (long long)B * D * H * W;
  const dim3 grid((unsigned)((nvox + kThreads - 1) / kThreads)), block(kThreads);
  if (outer_half_res) hipLaunchKernelGGL(compose_up_kernel, grid, block, 0, st, outer, inner, out, B, D, H, W);
  else hipLaunchKernelGGL(compose_kernel, grid, block, 0, st, outer, inner, out, B, D, H, W, s);
  return hipGetLastError();
}

hipError_t launch_warp_bwd(const void* src, const float* field, const float* dout, float* dsrc, float* dfield, int B,
                           int D, int H, int W, int C, int half, int dtype, hipStream_t st) {
  // One channel per lane: the atomic units work through one 64-byte line per clock and XCD, so what counts is
  // how few lines a wave-wide atomic touches.  With one channel per lane it covers the contiguous channels of 64/C
  // neighbouring voxels (4-5 lines at C = 8); with a 16-byte chunk per lane, the same channel of 32 voxels, 16
  // lines (measured at 160x192x224, C = 8: 1.8 ms against 6.9 ms).
  if (dtype == 1) return launch_bwd_t<bf16_t, 1>(src, field, dout, dsrc, dfield, B, D, H, W, C, half, st);
  return launch_bwd_t<float, 1>(src, field, dout, dsrc, dfield, B, D, H, W, C, half, st);
}

hipError_t launch_warp(const void* src, const float* field, void* out, int B, int D, int H, int W, int C,
                       int half, int dtype, hipStream_t st) {
  // the widest vector that divides the channel count (6 and 12 channels per head give C = 6, 12, 24, ...)
  if (dtype == 1) {
    if (C % 8 == 0) return launch_t<bf16_t, 8>(src, field, out, B, D, H, W, C, half, st);
    if (C % 4 == 0) return launch_t<bf16_t, 4>(src, field, out, B, D, H, W, C, half, st);
    return launch_t<bf16_t, 2>(src, field, out, B, D, H, W, C, half, st);
  }
  if (C % 4 == 0) return launch_t<float, 4>(src, field, out, B, D, H, W, C, half, st);
  if (C % 2 == 0) return launch_t<float, 2>(src, field, out, B, D, H, W, C, half, st);
  return launch_t<float, 1>(src, field, out, B, D, H, W, C, half, st);
}

}  // namespace modet
