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
// weight of coarse voxel c (of n) in the upsampled value at fine voxel i
__device__ __forceinline__ float up_weight(int i, int c, int n) {
  const int lo = coarse_lo(i), hi = min(lo + 1, n - 1);
  const float t = (i == 0 || hi == lo) ? 0.f : ((i & 1) ? 0.25f : 0.75f);
  return (c == lo ? 1.f - t : 0.f) + (c == hi ? t : 0.f);
}

// The coarse voxels a brick of fine voxels needs, staged once per workgroup in LDS: per axis the range
// [coarse_lo(first), coarse_lo(last) + 1], at most extent/2 + 2 values.
constexpr int kMaxTile = 192;     // coarse voxels per workgroup: bricks are at most 16 x 4 x 4 -> 10 x 4 x 4
struct CoarseTile {
  int oz, oy, ox, nz, ny, nx;     // origin and extents (clamped to the coarse grid)
};

// Displacement of the 2x upsampled field at fine voxel (z,y,x); at(zi, yi, xi) points at a coarse voxel's three
// values.  The interpolation runs in fp64: an fp32 result would carry ~2e-7 of rounding on a displacement of a few
// voxels, and the warp multiplies that by the local feature gradient.  Every caller goes through this one function,
// so kernels that classify a voxel by its displacement agree bit for bit.
template <class At>
__device__ __forceinline__ void upsample_mix(int Dc, int Hc, int Wc, int z, int y, int x, double* u, At at) {
  const int z0 = coarse_lo(z), y0 = coarse_lo(y), x0 = coarse_lo(x);
  const int z1 = min(z0 + 1, Dc - 1), y1 = min(y0 + 1, Hc - 1), x1 = min(x0 + 1, Wc - 1);
  // fractions are multiples of 1/4: exact in fp32; 0 where the coordinate was clamped
  const float tz = (z == 0 || z1 == z0) ? 0.f : ((z & 1) ? 0.25f : 0.75f);
  const float ty = (y == 0 || y1 == y0) ? 0.f : ((y & 1) ? 0.25f : 0.75f);
  const float tx = (x == 0 || x1 == x0) ? 0.f : ((x & 1) ? 0.25f : 0.75f);
  u[0] = u[1] = u[2] = 0.0;
#pragma unroll
  for (int c = 0; c < 8; ++c) {
    const double w = (double)(((c & 4) ? tz : 1.f - tz) * ((c & 2) ? ty : 1.f - ty) * ((c & 1) ? tx : 1.f - tx));
    const float* p = at((c & 4) ? z1 : z0, (c & 2) ? y1 : y0, (c & 1) ? x1 : x0);
    u[0] = fma(w, (double)p[0], u[0]); u[1] = fma(w, (double)p[1], u[1]); u[2] = fma(w, (double)p[2], u[2]);
  }
  u[0] *= 2.0; u[1] *= 2.0; u[2] *= 2.0;
}

// from the tile staged in LDS
__device__ __forceinline__ void upsampled_disp(const float* __restrict__ tile, const CoarseTile& ct, int Dc, int Hc,
                                               int Wc, int z, int y, int x, double* u) {
  upsample_mix(Dc, Hc, Wc, z, y, x, u, [&](int zi, int yi, int xi) {
    return tile + (((zi - ct.oz) * ct.ny + yi - ct.oy) * ct.nx + xi - ct.ox) * 3;
  });
}

// straight from the coarse field of one batch item in global memory
__device__ __forceinline__ void upsampled_disp_global(const float* __restrict__ fc, int Dc, int Hc, int Wc, int z,
                                                      int y, int x, double* u) {
  upsample_mix(Dc, Hc, Wc, z, y, x, u, [&](int zi, int yi, int xi) {
    return fc + (((long long)zi * Hc + yi) * Wc + xi) * 3;
  });
}

// A displacement split into whole voxels and the fraction in [0, 1) (the fraction of an fp32 value is exact in
// fp64; the integer part is clamped far outside any volume so that adding a coordinate cannot overflow).
struct Split { int fz, fy, fx; float tz, ty, tx; };
__device__ __forceinline__ Split split_disp(const double* u) {
  const double fz = floor(u[0]), fy = floor(u[1]), fx = floor(u[2]);
  Split s;
  s.tz = (float)(u[0] - fz); s.ty = (float)(u[1] - fy); s.tx = (float)(u[2] - fx);
  s.fz = (int)fmin(fmax(fz, -1.0e6), 1.0e6);
  s.fy = (int)fmin(fmax(fy, -1.0e6), 1.0e6);
  s.fx = (int)fmin(fmax(fx, -1.0e6), 1.0e6);
  return s;
}

// The adjoint of the warp splits dsrc into boxes of kBoxXY x kBoxXY voxels in (y, x) and 2^lshift planes in z.
// Every box has a whole-voxel offset c: the displacement at its centre voxel, rounded to the nearest integer.  A
// smooth field moves the voxels that land in a box by about that much, so the box's owner looks for them around
// (box - c).  One function computes c for everybody, so that all kernels agree on it bit for bit.
constexpr int kBoxXY = 16;
constexpr int kNear = 3;        // a contribution p -> t is "near" if |(t - p) - c(box of t)| <= kNear on every axis
template <bool HALF>
__device__ __forceinline__ void box_offset(const float* __restrict__ fb, int D, int H, int W, int lshift, int bz,
                                           int by, int bx, int* c) {
  const int zc = min((bz << lshift) + ((1 << lshift) >> 1), D - 1);
  const int yc = min(by * kBoxXY + kBoxXY / 2, H - 1), xc = min(bx * kBoxXY + kBoxXY / 2, W - 1);
  // (half resolution: twice the coarse voxel under the centre; c only has to be close to the displacements
  // around the box, and the same for everybody)
  const float* f = HALF ? fb + (((long long)(zc >> 1) * (H / 2) + (yc >> 1)) * (W / 2) + (xc >> 1)) * 3
                        : fb + (((long long)zc * H + yc) * W + xc) * 3;
  const double s = HALF ? 2.0 : 1.0;
#pragma unroll
  for (int a = 0; a < 3; ++a) c[a] = (int)fmin(fmax(floor(s * (double)f[a] + 0.5), -1.0e6), 1.0e6);
}
__device__ __forceinline__ bool within(int o, int c) { return o - c >= -kNear && o - c <= kNear; }

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
  if (bk.sx < 0 || bk.sy < 0 || nchunk > 64) bk.sc = -1;      // (a voxel's lanes must sit in one wavefront)
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
// Gradients of L = sum(dout * warp(src, field)).  The source gradient is the transpose of the gather, a scatter:
// every voxel p adds weight * dout[p] to the eight corners t it would have read.  It runs in two passes.
//
// Pass 1 (warp_adj_near_kernel) turns the scatter into owner-computes for the near contributions (see box_offset
// above).  A workgroup owns one box of dsrc and walks the planes of the source voxels that can reach it near-ly:
// its (y, x) footprint shifted by -c and widened by kNear, planes za - cz - kNear ... zb - 1 - cz + kNear.  The
// 2 kNear + 1 target planes that the current source plane can touch live in LDS.  Per source plane: (a) one lane
// per voxel of the widened plane splits its displacement and, if a near corner lands in the box, appends a
// record (source index, LDS target, validity of the six corner coordinates, fractions) to a list in LDS; (b) the
// lanes load the records' dout values and add the weighted copies to the planes in LDS; (c) the
// target plane that no later source plane can reach is written to dsrc with plain, coalesced stores and its LDS
// slot cleared.  Every element of dsrc is written exactly once here: no zero-fill pass, no global atomic.
//
// LDS float atomics run at a few lanes per clock on this chip (measured: ~190 clocks per wave-wide ds_add_f32,
// against ~8 for a read, an add and a write), so the adds of step (b) are plain read-modify-writes made safe by
// ownership: wavefront w alone touches the target rows [w kAdjRows, (w + 1) kAdjRows) of every plane in the
// ring.  Step (a) files each record under the wave that owns both of its corner rows (list from the front of the
// wave's bin: eight corners each) or, row by row, under the two waves that own one each (list from the back: four
// corners each).  In step (b) a wave works through its own bin, 64 / (lanes per entry) entries per instruction, a
// lane taking four channels (or all, if fewer).  LDS operations of one wave execute in order, so two lanes can
// only collide inside one instruction, and only (see adj_adds) if their entries' first adds go to the same (row,
// column): step (a) numbers the entries of a step that share one (an LDS counter per row and column), and an
// instruction applies its entries in turns, one number at a time.
//
// Pass 2 (warp_adj_far_kernel, one lane per voxel) finds the contributions that are not near and adds them with
// hardware fp32 atomics on top: for every voxel that has any, the whole wave takes one (corner, channel) pair per
// lane, so that an atomic covers the contiguous channels of a corner.  Both passes decide from the same arithmetic
// (split_disp of the same fp64 displacement, box_offset of the same box), so each contribution is added exactly
// once.  The order of the additions to one element, hence the last bits of the result, is not fixed.
//
// The field gradient (warp_dfield_kernel, one lane per voxel and channel) differentiates the corner weights: per
// corner the dot product of dout with the source values, signed by the side of the corner along the axis; the
// lanes of one voxel are summed by lane shuffles when they form an aligned power-of-two group, through LDS
// otherwise, and one lane writes (full resolution); at half resolution the coarse voxels collect from the fine
// ones through the 2x upsampling weights.
constexpr int kAdjThreads = 512, kAdjWaves = kAdjThreads / 64, kAdjRows = kBoxXY / kAdjWaves;
constexpr int kAdjCols = kBoxXY + 2;               // columns a lower corner can have: -1 ... kBoxXY
constexpr int kAdjLastTurn = 63;                   // (a column can collect (2 kNear + 1)^2 = 49 entries per step: a safeguard)

struct AdjRec {
  int vox;            // source voxel, index inside its batch item
  unsigned bits;      // [0,6) x0 - box_x + 1, [6,12) y0 - box_y + 1, [12,16) ring slot of z0, [16,20) of z0 + 1,
                      // [20,26) this corner coordinate is near and inside the box: z0, z0+1, y0, y0+1, x0, x0+1
  float tz, ty, tx;
};
struct AdjGrid { int nbx, nby, nbz, lshift, nch; };   // boxes along x, y, z, log2 of their depth, channel chunks

// Step (b) for a wave's bin.  An entry is a record index (9 bits), for the back list the corner row (bit 9), and
// its turn (bits 10-15).  Front list: both corner rows, eight adds; back list: four adds.  Two entries of one
// instruction whose first adds go to different (row, column) pairs can only meet where the upper-x corner of one
// is the lower-x corner of the other, so the lower-x adds of all lanes go first, as one batch of independent
// read-modify-writes (all reads, then all writes), and the upper-x adds follow as a second batch.  Entries that
// share (row, column) have different turns; those past the last turn number are applied one entry at a time.
template <int CC, bool VEC4>
struct AdjFetch {                                  // one round of one list, fetched ahead of its adds
  static constexpr int VW = CC >= 4 ? 4 : CC;      // channels per lane
  unsigned ent;                                    // bit 16: there is an entry
  AdjRec r;
  float g[VW];
  __device__ __forceinline__ void entry(const unsigned short* __restrict__ list, int i, int n, bool back) {
    ent = i < n ? (unsigned)list[back ? -i : i] | 0x10000u : 0u;
  }
  __device__ __forceinline__ void value(const float* __restrict__ dbase, int C, int chb, int cleft) {
    const float* gp = dbase + (long long)r.vox * C + chb;
#pragma unroll
    for (int j = 0; j < VW; ++j) g[j] = 0.f;
    if (ent >> 16) {
      if (VEC4) {                                  // (C is a multiple of 4: a lane's channels exist together)
        if (chb < cleft) Vec<float, VW>::load(gp, g);
      } else {
#pragma unroll
        for (int j = 0; j < VW; ++j)
          if (chb + j < cleft) g[j] = gp[j];
      }
    }
  }
};

template <int CC, bool ROW, bool VEC4, int PLANE>
__device__ __forceinline__ void adj_adds(float* __restrict__ ring, const AdjFetch<CC, VEC4>& f, int lane) {
  constexpr int T = kBoxXY;
  constexpr int VW = CC >= 4 ? 4 : CC, LPE = CC / VW;
  constexpr int NB = ROW ? 2 : 4;                  // adds per batch: (plane) or (plane, row) pairs
  const int chb = (lane % LPE) * VW;
  const bool any = (f.ent >> 16) != 0u;
  const unsigned bits = f.r.bits;
  const unsigned up = ROW ? (f.ent >> 9) & 1u : 0u;
  const int turn = (int)((f.ent >> 10) & 63u);
  const int row = (int)((bits >> 6) & 63u) - 1 + (int)up;                // of the first add
  const int a0 = (row * T + (int)(bits & 63u) - 1) * CC + chb;
  const int sl[2] = {(int)((bits >> 12) & 15u) * PLANE, (int)((bits >> 16) & 15u) * PLANE};
  const float wy1 = up ? f.r.ty : 1.f - f.r.ty;
  auto batches = [&](bool on) {
#pragma unroll
    for (int kx = 0; kx < 2; ++kx) {
      const float wx = kx ? f.r.tx : 1.f - f.r.tx;
      const bool okx = on && ((bits >> (24 + kx)) & 1u) != 0u;
      int addr[NB];
      bool ok[NB];
      float val[NB][VW];
#pragma unroll
      for (int c = 0; c < NB; ++c) {
        const int kz = ROW ? c : c >> 1, ky = ROW ? 0 : c & 1;
        ok[c] = okx && ((bits >> (20 + kz)) & 1u) != 0u && (ROW || ((bits >> (22 + ky)) & 1u) != 0u);
        addr[c] = sl[kz] + a0 + (ky * T + kx) * CC;
        if (ok[c]) Vec<float, VW>::load(ring + addr[c], val[c]);
      }
#pragma unroll
      for (int c = 0; c < NB; ++c) {
        const int kz = ROW ? c : c >> 1, ky = ROW ? 0 : c & 1;
        const float wy = ROW ? wy1 : (ky ? f.r.ty : 1.f - f.r.ty);
        const float w = (kz ? f.r.tz : 1.f - f.r.tz) * wy * wx;
        if (ok[c]) {
#pragma unroll
          for (int j = 0; j < VW; ++j) val[c][j] = fmaf(w, f.g[j], val[c][j]);
          Vec<float, VW>::store(ring + addr[c], val[c]);
        }
      }
      asm volatile("" ::: "memory");               // the next batch's reads stay behind these writes
    }
  };
  for (int rd = 0; rd < kAdjLastTurn && __ballot(any && turn >= rd) != 0ull; ++rd) batches(any && turn == rd);
  // (rare) entries past the last turn number, one at a time
  for (unsigned long long m = __ballot(any && turn == kAdjLastTurn); m != 0ull;) {
    const int l = __ffsll((long long)m) - 1;
    batches(any && turn == kAdjLastTurn && lane / LPE == l / LPE);
    m &= ~(((1ull << LPE) - 1ull) << (l / LPE * LPE));
  }
}

// nf entries from `front` upwards, nb entries from `back` downwards.  The first two rounds of each list (all of it,
// usually) are fetched together, before the first add: one wait for memory per step.
template <int CC, bool VEC4, int PLANE>
__device__ __forceinline__ void adj_apply(float* __restrict__ ring, const AdjRec* __restrict__ rec,
                                          const unsigned short* __restrict__ front, int nf,
                                          const unsigned short* __restrict__ back, int nb,
                                          const float* __restrict__ dbase, int C, int cleft, int lane) {
  constexpr int VW = CC >= 4 ? 4 : CC, LPE = CC / VW, EPI = 64 / LPE;    // lanes per entry, entries per instruction
  const int slot = lane / LPE, chb = (lane % LPE) * VW;
  AdjFetch<CC, VEC4> f[4];                         // rounds 0, 1 of the front list, rounds 0, 1 of the back list
  for (int i0 = 0; i0 < nf || i0 < nb; i0 += 2 * EPI) {
#pragma unroll
    for (int k = 0; k < 4; ++k) f[k].entry(k < 2 ? front : back, i0 + (k & 1) * EPI + slot, k < 2 ? nf : nb, k >= 2);
#pragma unroll
    for (int k = 0; k < 4; ++k) f[k].r = rec[f[k].ent & 511u];
#pragma unroll
    for (int k = 0; k < 4; ++k) f[k].value(dbase, C, chb, cleft);
#pragma unroll
    for (int k = 0; k < 2; ++k)
      if (i0 + k * EPI < nf) adj_adds<CC, false, VEC4, PLANE>(ring, f[k], lane);       // (uniform)
#pragma unroll
    for (int k = 0; k < 2; ++k)
      if (i0 + k * EPI < nb) adj_adds<CC, true, VEC4, PLANE>(ring, f[2 + k], lane);
  }
}

template <int CC, bool HALF, bool VEC4>
__global__ void __launch_bounds__(kAdjThreads)
warp_adj_near_kernel(const float* __restrict__ field, const float* __restrict__ dout, float* __restrict__ dsrc,
                     int B, int D, int H, int W, int C, AdjGrid gr) {
  constexpr int M = kNear, T = kBoxXY;
  constexpr int NR = 2 * M + 1;                                    // target planes alive at a time
  constexpr int DX = T + 2 * M;                                    // the widened plane of source voxels
  constexpr int NREC = DX * DX;
  constexpr int PLANE = T * T * CC;
  constexpr int SC = CC == 8 ? 3 : CC == 4 ? 2 : CC == 2 ? 1 : 0;
  constexpr int NOCC = (kAdjWaves + T) * kAdjCols;                 // counters of the front keys, then of the back keys
  static_assert((1 << SC) == CC && NR <= 15 && T + 1 < 64 && NREC <= kAdjThreads && NREC <= 512 &&
                NOCC <= kAdjThreads, "layout");
  __shared__ __align__(16) float ring[NR * PLANE];
  __shared__ AdjRec rec[NREC];
  __shared__ unsigned short bin[kAdjWaves][NREC];    // entries: front list from [0] upwards, back list from the end
  __shared__ int cnt[2][2 * kAdjWaves + 1];          // per parity of the step: front and back entries per wave, records
  __shared__ int occ[2][NOCC];                       // per parity: entries so far per (row pair or row, column)

  const unsigned nb = gridDim.x, xcd = blockIdx.x & 7u, q = nb >> 3, rem = nb & 7u;
  unsigned blk = xcd * q + (xcd < rem ? xcd : rem) + (blockIdx.x >> 3);
  const int ibx = blk % gr.nbx; blk /= gr.nbx;
  const int iby = blk % gr.nby; blk /= gr.nby;
  const int ibz = blk % gr.nbz; blk /= gr.nbz;
  const int ich = blk % gr.nch;
  const int b = blk / gr.nch;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int tx0 = ibx * T, ty0 = iby * T, za = ibz << gr.lshift, zb = min(za + (1 << gr.lshift), D);
  const int tw = min(T, W - tx0), th = min(T, H - ty0);
  const int c0 = ich * CC;
  const long long vb = (long long)b * D * H * W;
  const int Dc = D / 2, Hc = H / 2, Wc = W / 2;
  const float* fb = HALF ? field + (long long)b * Dc * Hc * Wc * 3 : field + vb * 3;
  int cb[3];
  box_offset<HALF>(fb, D, H, W, gr.lshift, ibz, iby, ibx, cb);
  const int cz = cb[0], cy = cb[1], cx = cb[2];

  for (int i = tid; i < NR * PLANE; i += kAdjThreads) ring[i] = 0.f;
  if (tid < 2 * (2 * kAdjWaves + 1)) (&cnt[0][0])[tid] = 0;
  if (tid < NOCC) { occ[0][tid] = 0; occ[1][tid] = 0; }
  __syncthreads();

  // this lane's voxel of the widened plane
  const int yy = tid / DX, xx = tid - yy * DX;
  const int y = ty0 - cy - M + yy, x = tx0 - cx - M + xx;
  const bool mine = tid < NREC && (unsigned)y < (unsigned)H && (unsigned)x < (unsigned)W;
  const float* dbase = dout + vb * C + c0;

  // source planes that reach [za, zb) near-ly; the last 2 M steps of the walk only flush.  (Clipped: a step below
  // plane 0, or 2 M and more beyond the last plane, has neither sources nor anything to flush but zeros.)
  const int zs0 = max(za - cz - M, 0), zs1 = min(zb - cz + M, D + 2 * M);
  float fu[3] = {0.f, 0.f, 0.f};                   // (full-resolution field) the displacement, one plane ahead
  if (!HALF && mine && zs0 < D) {
    const float* f = fb + ((long long)(zs0 * H + y) * W + x) * 3;
    fu[0] = f[0]; fu[1] = f[1]; fu[2] = f[2];
  }
  for (int z = zs0; z < zs1; ++z) {
    const bool have = z < D;                       // (uniform) is there a plane of source voxels at z?
    const int par = (z - zs0) & 1;
    if (have) {
      // (a) the records of this plane
      bool hit = false;
      AdjRec r = {};
      int w0 = -1, w1 = -1;                        // the waves that own the rows of its lower and upper corners
      int ly = 0, lx = 0;
      if (mine) {
        const int v = (z * H + y) * W + x;
        double u[3];
        if (HALF) upsampled_disp_global(fb, Dc, Hc, Wc, z, y, x, u);
        else { u[0] = fu[0]; u[1] = fu[1]; u[2] = fu[2]; }
        const Split sp = split_disp(u);
        const int z0 = z + sp.fz;                  // lower corner; ly, lx: box-relative
        ly = y + sp.fy - ty0;
        lx = x + sp.fx - tx0;
        const unsigned vz0 = within(sp.fz, cz) && z0 >= za && z0 < zb;
        const unsigned vz1 = within(sp.fz + 1, cz) && z0 + 1 >= za && z0 + 1 < zb;
        const unsigned vy0 = within(sp.fy, cy) && (unsigned)ly < (unsigned)th;
        const unsigned vy1 = within(sp.fy + 1, cy) && (unsigned)(ly + 1) < (unsigned)th;
        const unsigned vx0 = within(sp.fx, cx) && (unsigned)lx < (unsigned)tw;
        const unsigned vx1 = within(sp.fx + 1, cx) && (unsigned)(lx + 1) < (unsigned)tw;
        hit = (vz0 | vz1) && (vy0 | vy1) && (vx0 | vx1);
        if (hit) {       // (then z0 - za >= -1, ly >= -1, lx >= -1)
          const unsigned s0 = (unsigned)(z0 - za + NR) % NR, s1 = s0 + 1 == NR ? 0u : s0 + 1;
          r.vox = v;
          r.bits = (unsigned)(lx + 1) | ((unsigned)(ly + 1) << 6) | (s0 << 12) | (s1 << 16) | (vz0 << 20) |
                   (vz1 << 21) | (vy0 << 22) | (vy1 << 23) | (vx0 << 24) | (vx1 << 25);
          r.tz = sp.tz; r.ty = sp.ty; r.tx = sp.tx;
          if (vy0) w0 = ly / kAdjRows;
          if (vy1) w1 = (ly + 1) / kAdjRows;
        }
      }
      const unsigned long long m = __ballot(hit);
      int at = 0;
      if (lane == 0 && m) at = atomicAdd(&cnt[par][2 * kAdjWaves], __popcll(m));
      at = __shfl(at, 0);
      if (hit) {
        const unsigned ri = (unsigned)(at + __popcll(m & ((1ull << lane) - 1ull)));
        rec[ri] = r;
        int* oc = &occ[par][0];
        if (w0 == w1) {
          const unsigned t = (unsigned)min(atomicAdd(oc + w0 * kAdjCols + lx + 1, 1), kAdjLastTurn);
          bin[w0][atomicAdd(&cnt[par][2 * w0], 1)] = (unsigned short)(ri | (t << 10));
        } else {
          oc += kAdjWaves * kAdjCols;
          if (w0 >= 0) {
            const unsigned t = (unsigned)min(atomicAdd(oc + ly * kAdjCols + lx + 1, 1), kAdjLastTurn);
            bin[w0][NREC - 1 - atomicAdd(&cnt[par][2 * w0 + 1], 1)] = (unsigned short)(ri | (t << 10));
          }
          if (w1 >= 0) {
            const unsigned t = (unsigned)min(atomicAdd(oc + (ly + 1) * kAdjCols + lx + 1, 1), kAdjLastTurn);
            bin[w1][NREC - 1 - atomicAdd(&cnt[par][2 * w1 + 1], 1)] = (unsigned short)(ri | (1u << 9) | (t << 10));
          }
        }
      }
    }
    __syncthreads();
    if (have) {
      if (!HALF && mine && z + 1 < D) {            // the next plane's displacements arrive during step (b)
        const float* f = fb + ((long long)((z + 1) * H + y) * W + x) * 3;
        fu[0] = f[0]; fu[1] = f[1]; fu[2] = f[2];
      }
      // (b) this wave's bin
      if (tid <= 2 * kAdjWaves) cnt[par ^ 1][tid] = 0;
      if (tid < NOCC) occ[par ^ 1][tid] = 0;
      adj_apply<CC, VEC4, PLANE>(ring, rec, &bin[wv][0], cnt[par][2 * wv], &bin[wv][NREC - 1], cnt[par][2 * wv + 1],
                                 dbase, C, C - c0, lane);
    }
    __syncthreads();
    // (c) target plane z + cz - M is complete: no source plane above z reaches it
    const int zt = z + cz - M;
    if (zt >= za && zt < zb) {
      float* slot = ring + ((unsigned)(zt - za + NR) % NR) * PLANE;
      float* o = dsrc + (vb + ((long long)zt * H + ty0) * W + tx0) * C + c0;
      if (VEC4) {
        constexpr int Q4 = CC / 4;
        for (int e = tid; e < PLANE / 4; e += kAdjThreads) {
          const int c4 = e % Q4, ex = (e / Q4) % T, ey = e / (Q4 * T);
          const float4 val = *reinterpret_cast<const float4*>(slot + e * 4);
          *reinterpret_cast<float4*>(slot + e * 4) = make_float4(0.f, 0.f, 0.f, 0.f);
          if (ey < th && ex < tw && c0 + c4 * 4 < C)
            *reinterpret_cast<float4*>(o + ((long long)ey * W + ex) * C + c4 * 4) = val;
        }
      } else {
        for (int e = tid; e < PLANE; e += kAdjThreads) {
          const int c = e & (CC - 1), ex = (e >> SC) % T, ey = (e >> SC) / T;
          const float val = slot[e];
          slot[e] = 0.f;
          if (ey < th && ex < tw && c0 + c < C) o[((long long)ey * W + ex) * C + c] = val;
        }
      }
    }
  }
  // target planes that no existing source plane precedes by cz - M (a box offset that points out of the volume)
  // have received nothing and are still to be written
  for (int zt = za; zt < zb; ++zt) {
    const int z = zt - cz + M;                     // the source plane whose step flushes zt
    if (z >= zs0 && z < zs1) continue;
    float* o = dsrc + (vb + ((long long)zt * H + ty0) * W + tx0) * C + c0;
    for (int e = tid; e < PLANE; e += kAdjThreads) {
      const int c = e & (CC - 1), ex = (e >> SC) % T, ey = (e >> SC) / T;
      if (ey < th && ex < tw && c0 + c < C) o[((long long)ey * W + ex) * C + c] = 0.f;
    }
  }
}

// Pass 2: one lane per voxel decides which of its corners are not near; the wave then scatters them together.
template <bool HALF>
__global__ void __launch_bounds__(kThreads)
warp_adj_far_kernel(const float* __restrict__ field, const float* __restrict__ dout, float* __restrict__ dsrc, int B,
                    int D, int H, int W, int C, int lshift) {
  const unsigned nvox = (unsigned)B * D * H * W;  // (the host checks that B D H W C fits 31 bits)
  const unsigned v = blockIdx.x * kThreads + threadIdx.x;
  const int lane = threadIdx.x & 63;
  unsigned far = 0u;
  int z0 = 0, y0 = 0, x0 = 0;
  float tz = 0.f, ty = 0.f, tx = 0.f;
  if (v < nvox) {
    const unsigned row = v / (unsigned)W, pl = row / (unsigned)H;
    const int x = (int)(v - row * W), y = (int)(row - pl * H), b = (int)(pl / (unsigned)D), z = (int)(pl - b * D);
    const float* fb = HALF ? field + (long long)b * (D / 2) * (H / 2) * (W / 2) * 3
                           : field + (long long)b * D * H * W * 3;
    double u[3];
    if (HALF) {
      upsampled_disp_global(fb, D / 2, H / 2, W / 2, z, y, x, u);
    } else {
      const float* f = field + (long long)v * 3;
      u[0] = f[0]; u[1] = f[1]; u[2] = f[2];
    }
    const Split sp = split_disp(u);
    tz = sp.tz; ty = sp.ty; tx = sp.tx;
    z0 = z + sp.fz; y0 = y + sp.fy; x0 = x + sp.fx;
    int cb[3] = {0, 0, 0};
    const int z1 = z0 + 1, y1 = y0 + 1, x1 = x0 + 1;
    const bool inside = z0 >= 0 && z1 < D && y0 >= 0 && y1 < H && x0 >= 0 && x1 < W;
    if (inside && (z0 >> lshift) == (z1 >> lshift) && y0 / kBoxXY == y1 / kBoxXY && x0 / kBoxXY == x1 / kBoxXY) {
      // (most voxels) all eight corners in one box: one offset, two tests per axis
      box_offset<HALF>(fb, D, H, W, lshift, z0 >> lshift, y0 / kBoxXY, x0 / kBoxXY, cb);
      const unsigned nz = (within(sp.fz, cb[0]) ? 0x0Fu : 0u) | (within(sp.fz + 1, cb[0]) ? 0xF0u : 0u);
      const unsigned ny = (within(sp.fy, cb[1]) ? 0x33u : 0u) | (within(sp.fy + 1, cb[1]) ? 0xCCu : 0u);
      const unsigned nx = (within(sp.fx, cb[2]) ? 0x55u : 0u) | (within(sp.fx + 1, cb[2]) ? 0xAAu : 0u);
      far = ~(nz & ny & nx) & 0xFFu;
    } else {
      int lbz = -1, lby = -1, lbx = -1;              // the box whose offset is at hand
      for (int c = 0; c < 8; ++c) {
        const int oz = sp.fz + ((c >> 2) & 1), oy = sp.fy + ((c >> 1) & 1), ox = sp.fx + (c & 1);
        const int zt = z + oz, yt = y + oy, xt = x + ox;
        if ((unsigned)zt < (unsigned)D && (unsigned)yt < (unsigned)H && (unsigned)xt < (unsigned)W) {
          const int bz = zt >> lshift, by = yt / kBoxXY, bx = xt / kBoxXY;
          if (bz != lbz || by != lby || bx != lbx) {
            box_offset<HALF>(fb, D, H, W, lshift, bz, by, bx, cb);
            lbz = bz; lby = by; lbx = bx;
          }
          if (!(within(oz, cb[0]) && within(oy, cb[1]) && within(ox, cb[2]))) far |= 1u << c;
        }
      }
    }
  }
  // the voxels of this wave that have something to add, one after the other: lane = (corner, channel mod 8)
  const int c = lane >> 3;
  for (unsigned long long pend = __ballot(far != 0u); pend != 0ull; pend &= pend - 1ull) {
    const int l = __builtin_amdgcn_readfirstlane(__ffsll((long long)pend) - 1);
    const unsigned lfar = (unsigned)__shfl((int)far, l);
    const int zi = __shfl(z0, l) + ((c >> 2) & 1), yi = __shfl(y0, l) + ((c >> 1) & 1), xi = __shfl(x0, l) + (c & 1);
    const float lz = __shfl(tz, l), ly = __shfl(ty, l), lx = __shfl(tx, l);
    if (!((lfar >> c) & 1u)) continue;             // (far corners lie inside the volume)
    const unsigned lv = (v - lane) + l;            // the voxel of lane l
    const long long bv = (long long)(lv / ((unsigned)W * H * D)) * ((long long)W * H * D);
    const float w = ((c & 4) ? lz : 1.f - lz) * ((c & 2) ? ly : 1.f - ly) * ((c & 1) ? lx : 1.f - lx);
    float* o = dsrc + (bv + ((long long)zi * H + yi) * W + xi) * C;
    const float* g = dout + (long long)lv * C;
    for (int ch = lane & 7; ch < C; ch += 8) unsafeAtomicAdd(o + ch, w * g[ch]);
  }
}

__global__ void zero_kernel(float* p, long long n) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0.f;
}

// A workgroup works through my x mz bricks, one after the other (a super-brick; 1 x 1 at full resolution): at half
// resolution the coarse voxels it touches are staged once, and each collects from all of those bricks before
// it is added to the global gradient.
template <class T, int VEC, bool HALF>
__global__ void __launch_bounds__(kThreads)
warp_dfield_kernel(const T* __restrict__ src, const float* __restrict__ field, const float* __restrict__ dout,
                   float* __restrict__ dfield, int B, int D, int H, int W, int C, Brick bk, int my, int mz) {
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
  const int nsy = (bk.nby + my - 1) / my, nsz = (bk.nbz + mz - 1) / mz;
  const int ibx = blk % bk.nbx; blk /= bk.nbx;
  const int isy = blk % nsy; blk /= nsy;
  const int isz = blk % nsz;
  const int b = blk / nsz;
  __shared__ float tile[HALF ? kMaxTile * 3 : 1];
  __shared__ float dus[kThreads * 3];                   // every lane's sums, to be collected per (coarse) voxel
  CoarseTile ct = {};
  const int Dc = D / 2, Hc = H / 2, Wc = W / 2;
  if (HALF) {
    // the coarse voxels of the whole super-brick (the host keeps them within kMaxTile)
    const int xf = ibx * bk.bx, yf = isy * my * bk.by, zf = isz * mz * bk.bz;
    ct.ox = coarse_lo(xf); ct.oy = coarse_lo(min(yf, H - 1)); ct.oz = coarse_lo(min(zf, D - 1));
    ct.nx = min(coarse_lo(min(xf + bk.bx, W) - 1) + 1, Wc - 1) - ct.ox + 1;
    ct.ny = min(coarse_lo(max(min(yf + my * bk.by, H), 1) - 1) + 1, Hc - 1) - ct.oy + 1;
    ct.nz = min(coarse_lo(max(min(zf + mz * bk.bz, D), 1) - 1) + 1, Dc - 1) - ct.oz + 1;
    const float* fc = field + (long long)b * Dc * Hc * Wc * 3;
    const int n = ct.nx * ct.ny * ct.nz;
    for (int e = threadIdx.x; e < n; e += kThreads) {
      const int ex = e % ct.nx, ey = (e / ct.nx) % ct.ny, ez = e / (ct.nx * ct.ny);
      const float* p = fc + (((long long)(ct.oz + ez) * Hc + ct.oy + ey) * Wc + ct.ox + ex) * 3;
      tile[e * 3] = p[0]; tile[e * 3 + 1] = p[1]; tile[e * 3 + 2] = p[2];
    }
    __syncthreads();
  }
  // half resolution: this lane's coarse voxel (one per lane) and what it has collected so far
  const int ncoarse = HALF ? ct.nx * ct.ny * ct.nz : 0;
  const int ce = threadIdx.x;
  const int cx = ct.ox + ce % max(ct.nx, 1), cy = ct.oy + (ce / max(ct.nx, 1)) % max(ct.ny, 1);
  const int cz = ct.oz + ce / max(ct.nx * ct.ny, 1);
  float acc[3] = {0.f, 0.f, 0.f};
  // (nobody leaves the loop early: everybody meets at its barriers)
  for (int sub = 0; sub < my * mz; ++sub) {
    const int iby = isy * my + sub % my, ibz = isz * mz + sub / my;
    const int x = ibx * bk.bx + lx, y = iby * bk.by + ly, z = ibz * bk.bz + lz;
    const bool live = lz < bk.bz && x < W && y < H && z < D;
    float du[3] = {0.f, 0.f, 0.f};
    bool writer = false;       // does this lane hold the voxel's whole sum?
    if (live) {
      const long long vol = (long long)b * D * H * W * C + chunk * VEC;
      const long long v = (((long long)b * D + z) * H + y) * W + x;
      double u[3];
      if (HALF) {
        upsampled_disp(tile, ct, Dc, Hc, Wc, z, y, x, u);
      } else {
        u[0] = field[v * 3]; u[1] = field[v * 3 + 1]; u[2] = field[v * 3 + 2];
      }
      const Split sp = split_disp(u);
      const float tz = sp.tz, ty = sp.ty, tx = sp.tx;
      const int z0 = z + sp.fz, y0 = y + sp.fy, x0 = x + sp.fx;
      float g[VEC];
      Vec<float, VEC>::load(dout + v * C + chunk * VEC, g);
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
        if (!HALF && writer) {     // the only writer of this voxel's entry
          float* o = dfield + v * 3;
          o[0] = du[0]; o[1] = du[1]; o[2] = du[2];
        }
      }
    }
    if (!HALF && bk.sc >= 0) return;               // (uniform; full resolution runs one brick per workgroup)
    // the lanes park their sums in LDS
#pragma unroll
    for (int a = 0; a < 3; ++a) dus[threadIdx.x * 3 + a] = writer ? du[a] : 0.f;
    __syncthreads();
    if (!HALF) {
      // a voxel's lanes are no lane group (its channel count is no power of two): one lane per voxel adds their
      // parts up and writes
      const int nchunk = C / VEC, t = threadIdx.x;
      const int vx = ibx * bk.bx + t % bk.bx, vy = iby * bk.by + (t / bk.bx) % bk.by, vz = ibz * bk.bz + t / (bk.bx * bk.by);
      if (t < kThreads / nchunk && t / (bk.bx * bk.by) < bk.bz && vx < W && vy < H && vz < D) {
        float sum[3] = {0.f, 0.f, 0.f};
        for (int j = 0; j < nchunk; ++j) {
          const float* d = dus + (t * nchunk + j) * 3;
          sum[0] += d[0]; sum[1] += d[1]; sum[2] += d[2];
        }
        float* o = dfield + ((((long long)b * D + vz) * H + vy) * W + vx) * 3;
        o[0] = sum[0]; o[1] = sum[1]; o[2] = sum[2];
      }
      return;
    }
    // Half resolution: u = 2 * sum of weight * coarse value over the (clamped) coarse corners of a voxel, and up
    // to 64 fine voxels share a coarse one: every staged coarse voxel collects, through the upsampling weights,
    // what this brick's fine voxels owe it (along each axis the fine voxels 2c - 1 ... 2c + 2 touch coarse voxel c).
    if (ce < ncoarse) {
      const int nlane = bk.sc >= 0 ? 1 : C / VEC;      // lanes of a voxel that hold a part of its sum
      const int vstride = bk.sc >= 0 ? 1 << bk.sc : C / VEC;
      const int xf = ibx * bk.bx, yf = iby * bk.by, zf = ibz * bk.bz;
      const int xe = min(xf + bk.bx, W), ye = min(yf + bk.by, H), ze = min(zf + bk.bz, D);
      for (int fz = max(2 * cz - 1, zf); fz <= min(2 * cz + 2, ze - 1); ++fz) {
        const float wz = up_weight(fz, cz, Dc);
        for (int fy = max(2 * cy - 1, yf); fy <= min(2 * cy + 2, ye - 1); ++fy) {
          const float wzy = wz * up_weight(fy, cy, Hc);
          for (int fx = max(2 * cx - 1, xf); fx <= min(2 * cx + 2, xe - 1); ++fx) {
            const float w = 2.f * wzy * up_weight(fx, cx, Wc);
            const int first = (((fz - zf) * bk.by + fy - yf) * bk.bx + fx - xf) * vstride;
            for (int j = 0; j < nlane; ++j) {
              const float* d = dus + (first + j) * 3;
              acc[0] = fmaf(w, d[0], acc[0]); acc[1] = fmaf(w, d[1], acc[1]); acc[2] = fmaf(w, d[2], acc[2]);
            }
          }
        }
      }
    }
    __syncthreads();                               // (the next brick parks its sums in the same place)
  }
  if (HALF && ce < ncoarse) {                      // one addition per coarse voxel and workgroup
    float* o = dfield + (long long)b * Dc * Hc * Wc * 3 + (((long long)cz * Hc + cy) * Wc + cx) * 3;
    unsafeAtomicAdd(o, acc[0]); unsafeAtomicAdd(o + 1, acc[1]); unsafeAtomicAdd(o + 2, acc[2]);
  }
}

template <int CC, bool HALF, bool VEC4>
void launch_adj_near(const float* field, const float* dout, float* dsrc, int B, int D, int H, int W, int C,
                     int lshift, hipStream_t st) {
  AdjGrid gr;
  gr.nbx = (W + kBoxXY - 1) / kBoxXY;
  gr.nby = (H + kBoxXY - 1) / kBoxXY;
  gr.lshift = lshift;
  gr.nbz = (D + (1 << lshift) - 1) >> lshift;
  gr.nch = (C + CC - 1) / CC;
  const long long boxes = (long long)gr.nbx * gr.nby * gr.nbz * gr.nch * B;
  hipLaunchKernelGGL((warp_adj_near_kernel<CC, HALF, VEC4>), dim3((unsigned)boxes), dim3(kAdjThreads), 0, st, field,
                     dout, dsrc, B, D, H, W, C, gr);
}

template <class T, int VEC>
hipError_t launch_bwd_t(const void* src, const float* field, const float* dout, float* dsrc, float* dfield, int B,
                        int D, int H, int W, int C, int half, hipStream_t st) {
  // boxes of 16 planes (8 for shallow volumes): a deeper box strays further from its centre's displacement, a
  // shallower one spends more of its walk on the 2 kNear planes beyond its ends
  const int lshift = D > 8 ? 4 : 3;
  // pass 1: every element of dsrc, from the near contributions (channels in chunks of up to 8: a power of two,
  // the last chunk masked)
  const bool v4 = C % 4 == 0;
#define MODET_ADJ(CC_, V4_)                                                                              \
  do {                                                                                                   \
    if (half) launch_adj_near<CC_, true, V4_>(field, dout, dsrc, B, D, H, W, C, lshift, st);              \
    else launch_adj_near<CC_, false, V4_>(field, dout, dsrc, B, D, H, W, C, lshift, st);                  \
  } while (0)
  if (C >= 5) { if (v4) MODET_ADJ(8, true); else MODET_ADJ(8, false); }
  else if (C >= 3) { if (v4) MODET_ADJ(4, true); else MODET_ADJ(4, false); }
  else if (C == 2) MODET_ADJ(2, false);
  else MODET_ADJ(1, false);
#undef MODET_ADJ
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  // pass 2: what is not near
  const long long nvox = (long long)B * D * H * W;
  const dim3 fgrid((unsigned)((nvox + kThreads - 1) / kThreads)), block(kThreads);
  if (half) hipLaunchKernelGGL((warp_adj_far_kernel<true>), fgrid, block, 0, st, field, dout, dsrc, B, D, H, W, C, lshift);
  else hipLaunchKernelGGL((warp_adj_far_kernel<false>), fgrid, block, 0, st, field, dout, dsrc, B, D, H, W, C, lshift);
  if (!dfield) return hipGetLastError();
  // the half-resolution field gradient is accumulated with atomics (a coarse voxel collects from several bricks)
  const Brick bk = make_brick(D, H, W, C / VEC);
  if (half) {
    const long long nf = (long long)B * (D / 2) * (H / 2) * (W / 2) * 3;
    hipLaunchKernelGGL(zero_kernel, dim3((unsigned)((nf + 255) / 256)), dim3(256), 0, st, dfield, nf);
  }
  // half resolution: bricks per workgroup, as many (up to 2 x 4 in y, z) as keep the staged coarse voxels, at
  // most n/2 + 2 per axis, within kMaxTile
  int my = 1, mz = 1;
  if (half) {
    auto staged = [&](int a, int c) { return (bk.bx / 2 + 2) * (bk.by * a / 2 + 2) * (bk.bz * c / 2 + 2); };
    while (mz < 4 && staged(my, mz * 2) <= kMaxTile) mz *= 2;
    while (my < 2 && staged(my * 2, mz) <= kMaxTile) my *= 2;
  }
  dim3 grid((unsigned)((long long)bk.nbx * ((bk.nby + my - 1) / my) * ((bk.nbz + mz - 1) / mz) * B));
  if (half)
    hipLaunchKernelGGL((warp_dfield_kernel<T, VEC, true>), grid, block, 0, st, (const T*)src, field, dout, dfield, B, D,
                       H, W, C, bk, my, mz);
  else
    hipLaunchKernelGGL((warp_dfield_kernel<T, VEC, false>), grid, block, 0, st, (const T*)src, field, dout, dfield, B,
                       D, H, W, C, bk, my, mz);
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
// two interpolations are folded into one table of three weights per axis (built in fp64: the factors are exact)
// over a 3 x 3 x 3 coarse neighbourhood, so the upsampled field is never materialised.
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
  // the 27-term sum itself runs in fp32, x innermost (its rounding, ~3e-7 of the displacement, is far inside the
  // tolerance of a field; the fp64 of the tables keeps the weights of clamped and outside corners exact)
  float fwz[3], fwy[3], fwx[3];
#pragma unroll
  for (int j = 0; j < 3; ++j) { fwz[j] = (float)wz[j]; fwy[j] = (float)wy[j]; fwx[j] = (float)wx[j]; }
  float acc[3] = {0.f, 0.f, 0.f};
#pragma unroll
  for (int zy = 0; zy < 9; ++zy) {
    float row[3] = {0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < 3; ++j) {
      const Disp& d = val[zy * 3 + j];
      row[0] = fmaf(fwx[j], d.z, row[0]); row[1] = fmaf(fwx[j], d.y, row[1]); row[2] = fmaf(fwx[j], d.x, row[2]);
    }
    const float w = fwz[zy / 3] * fwy[zy % 3];
    acc[0] = fmaf(w, row[0], acc[0]); acc[1] = fmaf(w, row[1], acc[1]); acc[2] = fmaf(w, row[2], acc[2]);
  }
  Disp r;
  r.z = fmaf(2.f, acc[0], iv.z); r.y = fmaf(2.f, acc[1], iv.y); r.x = fmaf(2.f, acc[2], iv.x);
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
