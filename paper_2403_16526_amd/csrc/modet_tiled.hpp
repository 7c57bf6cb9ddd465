// LDS-tiled ModeT kernels (gfx950): heads of 8 channels, of 6 (padded to 8 on chip) and of 12 (two half-heads).
//
// Paper: Section 3.3.1, Eq. 3 (neighbourhood scores + softmax, with the bias B) and Eq. 4-5 (attention-weighted
// offset grid), and their derivatives with respect to Q, K and B.
//
// Work decomposition
//   * The head axis is folded into W: a voxel row [W][heads][8] is a row of Wh = W*heads "fused columns" of 8
//     contiguous channels; the W-neighbour of fused column xs is xs +- heads (the kernels' HS).
//   * A group of 256 lanes owns a TX x TY = 32 x 8 patch of (fused column, H row) and marches along D over a
//     chunk of planes.  One plane of the *other* operand (patch + halo, zero filled outside the volume, so the
//     inner loops are branch free) lives in LDS at a time, double buffered; the next plane is fetched into
//     registers while the current one is consumed.
//   * Register blocking along D: a lane keeps the k planes of its own operand that can see the current LDS plane
//     in flight ("roles"), so every vector read from LDS is used for k windows.
//   * forward (FwdPolicy): lane owns a query column, K planes in LDS; softmax sums against one fixed reference per
//     query (no running maximum, nothing rescaled); no logit or weight is ever stored.
//   * backward: w = exp(l - lse) with the forward's lse.  k = 3 with one or two heads: bwd_fused_kernel, a
//     512-lane workgroup whose query half (DqPolicy) computes every logit once and hands dl to its key half
//     through LDS, which gathers dK; k = 3 with more heads: bwd_shared_kernel, the dQ and dK marches (DqPolicy,
//     DkPolicy) side by side on shared staged planes; k = 5: march_pair_kernel, the two marches as neighbouring
//     workgroups.  dK is always a gather over the queries that see a key: no atomics, fixed summation order.
//   * The gradient of the bias is a by-product of the backward kernels (sums of dl, folded in fp64).
//   * Logits are accumulated in fp64 for fp32 inputs (template parameter LT): an fp32 sum of eight products
//     leaves ~1e-6 of rounding on a logit of magnitude ~10, which the softmax turns into a 1e-6 relative error of
//     the weights.  An fp64 FMA issues at the rate of an unpacked fp32 one on this chip; fp64 is confined to the
//     dot product, the subtraction of the softmax reference and the softmax sums of the forward, everything else
//     is fp32.  Logits are kept in log2 units (the in-flight operand is pre-multiplied by scale*log2(e)).
#pragma once
#include "modet_common.hpp"
#include <type_traits>

namespace modet {
namespace {

constexpr int TX = 32, TY = 8, NT = TX * TY;
constexpr float kLog2e = 1.4426950408889634f, kLn2 = 0.6931471805599453f;

__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float log2_fast(float x) { return __builtin_amdgcn_logf(x); }

struct TiledParams {
  const void* Q; const void* K;
  const float* bias;                                              // [heads, k^3] or NULL (zeros)
  const float* dphi; const float* phi_in; const float* lse_in;   // backward only
  double* dbias_acc;                                              // backward, optional: [heads, k^3] sums of dl
  float* phi; float* lse;                                         // forward outputs
  float* out;                                                     // dQ or dK
  int B, D, H, Wh;          // Wh = W * HS fused columns of one head group (what a launch's tiles cover)
  // Head groups: a kernel handles at most 8 fused columns per voxel (its HS).  With more (16 or 32 heads, or more
  // than 4 heads of twelve channels) the columns of a voxel are split into ngrp groups of HS = 1 << hs_shift, a
  // group is one more grid axis, and only the addresses know: local column xl of group g is global column
  // (xl >> hs_shift) * HSg + g * HS + (xl & (HS - 1)) of a row of Whg = W * HSg columns.  Heads never interact,
  // so nothing else changes.  One group: HSg = HS, Whg = Wh, the mapping is the identity.
  int Whg, HSg, hs_shift, ngrp;
  int ch;                   // channels per fused column in memory (8, or 6: see Mem)
  int ZC, ntx, nty, nzc;    // planes per chunk; tiles along Wh, H; chunks along D
  float qscale;             // scale * log2(e)
  float scale;
};

// workgroups are dealt round-robin to the 8 XCDs (each with its own L2); give every XCD one
// contiguous range of logical tiles so that tiles sharing a halo share an L2.
__device__ __forceinline__ unsigned xcd_remap(unsigned id, unsigned n) {
  const unsigned xcd = id & 7u, k = id >> 3, q = n >> 3, rem = n & 7u;
  return xcd * q + (xcd < rem ? xcd : rem) + k;
}

struct Tile {
  int b, z0, z1, y0, xs0, tx, ty, xs, y;
  int gofs;                // first global column (inside a voxel) of this workgroup's head group
  bool lane_ok;
  long long plane_elems;   // H * Whg * channels per column
  long long col;           // global column index of (b, z=0, y, xs): + z*H*Whg
};

// local fused column of a head group -> global fused column of the row
__device__ __forceinline__ int gcol(const TiledParams& p, int gofs, int xl) {
  return (xl >> p.hs_shift) * p.HSg + gofs + (xl & ((1 << p.hs_shift) - 1));
}

__device__ __forceinline__ Tile make_tile(const TiledParams& p, unsigned id, int lane = -1) {
  Tile t;
  if (lane < 0) lane = threadIdx.x;
  const int txi = id % p.ntx; id /= p.ntx;
  const int tyi = id % p.nty; id /= p.nty;
  const int zc = id % p.nzc; id /= p.nzc;
  t.b = id % p.B;
  t.gofs = (id / p.B) << p.hs_shift;
  t.tx = lane % TX; t.ty = lane / TX;
  t.xs0 = txi * TX; t.y0 = tyi * TY;
  t.z0 = zc * p.ZC; t.z1 = min(p.D, t.z0 + p.ZC);
  t.xs = t.xs0 + t.tx; t.y = t.y0 + t.ty;
  t.lane_ok = t.xs < p.Wh && t.y < p.H;
  t.plane_elems = (long long)p.H * p.Whg * p.ch;
  t.col = (long long)t.b * p.D * p.H * p.Whg + (long long)t.y * p.Whg + gcol(p, t.gofs, min(t.xs, p.Wh - 1));
  return t;
}

// ---- plane staging -----------------------------------------------------------------------------
// LDS holds, per position of the haloed patch, the 8 channels split into 16-byte chunks that are stored in
// separate arrays: chunk c of position pos sits at [c*NPOS + pos], so lane-consecutive 16-byte reads are
// bank-conflict free.  The element type is fp32 (2 chunks) or fp64 (4 chunks, converted once when staged).
template <int KW, int HS>
struct Patch {
  static constexpr int R = KW / 2;
  static constexpr int PC = TX + 2 * R * HS, PR = TY + 2 * R, NPOS = PC * PR;
  static constexpr int NV = 2 * NPOS;                 // 4-channel loads per plane
  static constexpr int NL = (NV + NT - 1) / NT;       // 4-channel loads per lane per plane
  static constexpr int NS = (NPOS + NT - 1) / NT;     // positions per lane per plane (statistics)
};

template <class ET> struct Lds;
template <> struct Lds<float> {
  typedef float4 chunk;
  static constexpr int CH = 2;     // chunks per position
  static __device__ __forceinline__ void put4(chunk* buf, int npos, int pos, int hv, const float4& v) {
    buf[hv * npos + pos] = v;
  }
  static __device__ __forceinline__ void get8(const chunk* buf, int npos, int pos, float (&v)[8]) {
    const float4 a = buf[pos], b = buf[npos + pos];
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
};
template <> struct Lds<double> {
  typedef double2 chunk;
  static constexpr int CH = 4;
  static __device__ __forceinline__ void put4(chunk* buf, int npos, int pos, int hv, const float4& v) {
    buf[(2 * hv) * npos + pos] = make_double2((double)v.x, (double)v.y);
    buf[(2 * hv + 1) * npos + pos] = make_double2((double)v.z, (double)v.w);
  }
  static __device__ __forceinline__ void get8(const chunk* buf, int npos, int pos, double (&v)[8]) {
    const double2 a = buf[pos], b = buf[npos + pos], c = buf[2 * npos + pos], d = buf[3 * npos + pos];
    v[0] = a.x; v[1] = a.y; v[2] = b.x; v[3] = b.y; v[4] = c.x; v[5] = c.y; v[6] = d.x; v[7] = d.y;
  }
};

template <class E> struct Ld;
template <> struct Ld<float> {
  static __device__ __forceinline__ float4 vec4(const float* p) { return *reinterpret_cast<const float4*>(p); }
  static __device__ __forceinline__ float2 vec2(const float* p) { return *reinterpret_cast<const float2*>(p); }
  static __device__ __forceinline__ float one(const float* p) { return *p; }
};
template <> struct Ld<bf16_t> {
  static __device__ __forceinline__ float4 vec4(const bf16_t* p) {
    uint2 t = *reinterpret_cast<const uint2*>(p);
    return make_float4(__uint_as_float(t.x << 16), __uint_as_float(t.x & 0xFFFF0000u),
                       __uint_as_float(t.y << 16), __uint_as_float(t.y & 0xFFFF0000u));
  }
  static __device__ __forceinline__ float2 vec2(const bf16_t* p) {
    const uint32_t t = *reinterpret_cast<const uint32_t*>(p);
    return make_float2(__uint_as_float(t << 16), __uint_as_float(t & 0xFFFF0000u));
  }
  static __device__ __forceinline__ float one(const bf16_t* p) { return __uint_as_float(((uint32_t)*p) << 16); }
};

// The input type T of a kernel names the element type AND the number of channels of a head in memory.  Heads
// of six channels (the paper's small model, Section 4.4) are padded to eight in registers and in LDS: only
// the loads from and the stores to global memory know about it, the two extra channels are zeros that take
// part in the arithmetic.
//
// Heads of twelve channels (the paper's large model) are two six-channel HALF-HEADS in neighbouring fused
// columns, hence in neighbouring lanes (even lane = channels 0..5): Wh = 2 * W * heads columns, the W-neighbour
// of a column is 2 * heads columns away (that is the kernels' HS).  Each lane forms the dot product of its half
// and adds its partner's (one cross-lane move); from there on both lanes of a pair compute the same numbers
// and each keeps the gradient of its own six channels.  What is indexed by window (phi, lse, dphi, the bias's
// head) uses the column index shifted right by SH = 1.
struct f32x6_t;
struct bf16x6_t;
struct f32x12_t;
struct bf16x12_t;
template <class T> struct Mem { typedef T E; static constexpr int CH = 8; static constexpr bool PAIR = false; };
template <> struct Mem<f32x6_t> { typedef float E; static constexpr int CH = 6; static constexpr bool PAIR = false; };
template <> struct Mem<bf16x6_t> { typedef bf16_t E; static constexpr int CH = 6; static constexpr bool PAIR = false; };
template <> struct Mem<f32x12_t> { typedef float E; static constexpr int CH = 6; static constexpr bool PAIR = true; };
template <> struct Mem<bf16x12_t> { typedef bf16_t E; static constexpr int CH = 6; static constexpr bool PAIR = true; };
template <class T> struct Win {       // column index -> window index, and the share of a logit's additive terms
  static constexpr int SH = Mem<T>::PAIR ? 1 : 0;                 // (reference, lse, bias) a lane's partial sum
  static constexpr float kShare = Mem<T>::PAIR ? 0.5f : 1.0f;     // starts from: the two halves add up to the whole
};

// the value the other lane of a pair (lane ^ 1) holds; all lanes of the wave execute it together
__device__ __forceinline__ float partner(float x) {
  return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(x), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
}
__device__ __forceinline__ double partner(double x) {
  const int lo = __builtin_amdgcn_mov_dpp(__double2loint(x), 0xB1, 0xF, 0xF, true);
  const int hi = __builtin_amdgcn_mov_dpp(__double2hiint(x), 0xB1, 0xF, 0xF, true);
  return __hiloint2double(hi, lo);
}
// a logit from this lane's partial sum
template <class T, class LT>
__device__ __forceinline__ LT whole_logit(LT part) {
  if constexpr (Mem<T>::PAIR) return part + partner(part);
  else return part;
}

// stages one haloed plane of an [.., H, Wh, 8] tensor: global -> registers (fetch), registers -> LDS (commit).
// The loads are unconditional (slots outside the volume read a clamped, valid address and are zeroed when
// committed): a load under a branch makes the compiler wait for it at the end of the branch, which would
// expose the whole memory latency in every step.
template <int KW, int HS, class T, class ET>
struct Stager {
  typedef Patch<KW, HS> P;
  typedef typename Mem<T>::E E;
  static constexpr int CH = Mem<T>::CH;
  int goff[P::NL];      // element offset inside a plane (clamped into the plane)
  int loff[P::NL];      // (position << 2 | half << 1 | inside-the-volume) inside the patch, or -1 when unused
  float4 v[P::NL];
  bool plane_ok;

  __device__ __forceinline__ void init(int tid, int y0, int xs0, int H, int Wh, const TiledParams& p, int gofs) {
#pragma unroll
    for (int i = 0; i < P::NL; ++i) {
      const int e = tid + i * NT;
      const int pos = e >> 1, hv = e & 1;
      const int pr = pos / P::PC, pc = pos - pr * P::PC;
      const int gy = y0 - P::R + pr, gx = xs0 - P::R * HS + pc;
      const bool used = e < P::NV;
      const bool in = used && gy >= 0 && gy < H && gx >= 0 && gx < Wh;
      const int cy = min(max(gy, 0), H - 1), cx = min(max(gx, 0), Wh - 1);
      goff[i] = (cy * p.Whg + gcol(p, gofs, cx)) * CH + hv * 4;
      loff[i] = used ? (pos << 2 | hv << 1 | (in ? 1 : 0)) : -1;
    }
    plane_ok = false;
  }
  // `plane` must point at a plane inside the tensor; ok = false: the wanted plane lies outside the volume
  // (zero padding) and the loaded values are discarded
  __device__ __forceinline__ float4 load_slot(const E* plane, int i) const {
    if constexpr (CH == 8) {
      return Ld<E>::vec4(plane + goff[i]);
    } else {
      // six channels: the first half of a column is channels 0..3, the second channels 4, 5 and two zeros
      // (the second load of a second half re-reads the same address: always valid, then discarded)
      const bool second = (loff[i] >> 1) & 1;
      const float2 a = Ld<E>::vec2(plane + goff[i]);
      const float2 b = Ld<E>::vec2(plane + goff[i] + (second ? 0 : 2));
      return make_float4(a.x, a.y, second ? 0.f : b.x, second ? 0.f : b.y);
    }
  }
  __device__ __forceinline__ void fetch(const E* plane, bool ok) {
#pragma unroll
    for (int i = 0; i < P::NL; ++i) v[i] = load_slot(plane, i);
    plane_ok = ok;
  }
  // a second plane staged with the same patch geometry keeps only its values: `vals` and `ok` live with the caller
  __device__ __forceinline__ void fetch_into(float4 (&vals)[P::NL], const E* plane) const {
#pragma unroll
    for (int i = 0; i < P::NL; ++i) vals[i] = load_slot(plane, i);
  }
  __device__ __forceinline__ void commit_from(const float4 (&vals)[P::NL], bool ok, typename Lds<ET>::chunk* buf) const {
    if (ok) {      // (uniform)
#pragma unroll
      for (int i = 0; i < P::NL; ++i)
        if (loff[i] >= 0 && (loff[i] & 1)) Lds<ET>::put4(buf, P::NPOS, loff[i] >> 2, (loff[i] >> 1) & 1, vals[i]);
    } else {
#pragma unroll
      for (int i = 0; i < P::NL; ++i)
        if (loff[i] >= 0 && (loff[i] & 1))
          Lds<ET>::put4(buf, P::NPOS, loff[i] >> 2, (loff[i] >> 1) & 1, make_float4(0.f, 0.f, 0.f, 0.f));
    }
  }
  // Patch slots outside the volume (in H, W) never change: they are zeroed once per LDS buffer, and commit
  // writes the others only; a plane outside the volume (in D) is a uniform case, so nothing is selected per
  // lane and component.
  __device__ __forceinline__ void zero_outside(typename Lds<ET>::chunk* buf) const {
#pragma unroll
    for (int i = 0; i < P::NL; ++i)
      if (loff[i] >= 0 && !(loff[i] & 1))
        Lds<ET>::put4(buf, P::NPOS, loff[i] >> 2, (loff[i] >> 1) & 1, make_float4(0.f, 0.f, 0.f, 0.f));
  }
  __device__ __forceinline__ void commit(typename Lds<ET>::chunk* buf) const {
    if (plane_ok) {
#pragma unroll
      for (int i = 0; i < P::NL; ++i)
        if (loff[i] >= 0 && (loff[i] & 1)) Lds<ET>::put4(buf, P::NPOS, loff[i] >> 2, (loff[i] >> 1) & 1, v[i]);
    } else {
#pragma unroll
      for (int i = 0; i < P::NL; ++i)
        if (loff[i] >= 0 && (loff[i] & 1))
          Lds<ET>::put4(buf, P::NPOS, loff[i] >> 2, (loff[i] >> 1) & 1, make_float4(0.f, 0.f, 0.f, 0.f));
    }
  }
};

// per-query statistics of a haloed patch: (-lse*log2e, g_D, g_H, g_W) and -g.phi; zeros outside the volume.
// Loads are unconditional from clamped addresses, like the Stager's.
template <int KW, int HS>
struct StatStager {
  typedef Patch<KW, HS> P;
  int goff[P::NS];   // window index inside a plane (clamped)
  int loff[P::NS];   // (position << 1 | inside-the-volume), or -1
  float lse[P::NS], g[P::NS][3], f[P::NS][3];
  bool plane_ok;
  int sh;            // column index -> window index (1 for half-head columns)
  float nshare;      // -log2(e) * the share of lse a lane's partial logit starts from

  __device__ __forceinline__ void init(int tid, int y0, int xs0, int H, int Wh, const TiledParams& p, int gofs,
                                       int sh_ = 0) {
    sh = sh_;
    nshare = sh_ ? -0.5f * kLog2e : -kLog2e;
#pragma unroll
    for (int i = 0; i < P::NS; ++i) {
      const int pos = tid + i * NT;
      const int pr = pos / P::PC, pc = pos - pr * P::PC;
      const int gy = y0 - P::R + pr, gx = xs0 - P::R * HS + pc;
      const bool used = pos < P::NPOS;
      const bool in = used && gy >= 0 && gy < H && gx >= 0 && gx < Wh;
      const int cy = min(max(gy, 0), H - 1), cx = min(max(gx, 0), Wh - 1);
      goff[i] = cy * p.Whg + gcol(p, gofs, cx);
      loff[i] = used ? (pos << 1 | (in ? 1 : 0)) : -1;
    }
    plane_ok = false;
  }
  // base = window index of (b, z, 0, 0) of a plane inside the volume; ok as in Stager::fetch
  __device__ __forceinline__ void fetch(const TiledParams& p, long long base, bool ok) {
#pragma unroll
    for (int i = 0; i < P::NS; ++i) {
      const long long w = (base + goff[i]) >> sh;
      const float* gp = p.dphi + w * 3;
      const float* fp = p.phi_in + w * 3;
      lse[i] = p.lse_in[w];
      g[i][0] = gp[0]; g[i][1] = gp[1]; g[i][2] = gp[2];
      f[i][0] = fp[0]; f[i][1] = fp[1]; f[i][2] = fp[2];
    }
    plane_ok = ok;
  }
  __device__ __forceinline__ void zero_outside(float4* sa, float* sc) const {
#pragma unroll
    for (int i = 0; i < P::NS; ++i)
      if (loff[i] >= 0 && !(loff[i] & 1)) {
        sa[loff[i] >> 1] = make_float4(0.f, 0.f, 0.f, 0.f);
        sc[loff[i] >> 1] = 0.f;
      }
  }
  __device__ __forceinline__ void commit(float4* sa, float* sc) const {
    if (plane_ok) {
#pragma unroll
      for (int i = 0; i < P::NS; ++i)
        if (loff[i] >= 0 && (loff[i] & 1)) {
          sa[loff[i] >> 1] = make_float4(lse[i] * nshare, g[i][0], g[i][1], g[i][2]);
          sc[loff[i] >> 1] = -(g[i][0] * f[i][0] + g[i][1] * f[i][1] + g[i][2] * f[i][2]);
        }
    } else {
#pragma unroll
      for (int i = 0; i < P::NS; ++i)
        if (loff[i] >= 0 && (loff[i] & 1)) {
          sa[loff[i] >> 1] = make_float4(0.f, 0.f, 0.f, 0.f);
          sc[loff[i] >> 1] = 0.f;
        }
    }
  }
};

// Makes the compiler treat x as read and rewritten here, so a load into x is waited for at this point of the
// program and nowhere later.
__device__ __forceinline__ void pin(float& x) { asm volatile("" : "+v"(x)); }
__device__ __forceinline__ void pin(float (&x)[8]) {
#pragma unroll
  for (int i = 0; i < 8; ++i) pin(x[i]);
}

// unconditional (see Stager): p must be a valid address; the caller discards the values where they are not wanted
template <class T>
__device__ __forceinline__ void load8(const typename Mem<T>::E* p, float (&q)[8]) {
  typedef typename Mem<T>::E E;
  if constexpr (Mem<T>::CH == 8) {
    const float4 a = Ld<E>::vec4(p), b = Ld<E>::vec4(p + 4);
    q[0] = a.x; q[1] = a.y; q[2] = a.z; q[3] = a.w; q[4] = b.x; q[5] = b.y; q[6] = b.z; q[7] = b.w;
  } else {
    const float2 a = Ld<E>::vec2(p), b = Ld<E>::vec2(p + 2), c = Ld<E>::vec2(p + 4);
    q[0] = a.x; q[1] = a.y; q[2] = b.x; q[3] = b.y; q[4] = c.x; q[5] = c.y; q[6] = 0.f; q[7] = 0.f;
  }
}

// sum_c q[c] * v[c] (+ init), accumulated in LT
template <class LT>
__device__ __forceinline__ LT dot8(const LT (&q)[8], const LT (&v)[8]) {
  LT acc = q[0] * v[0];
#pragma unroll
  for (int c = 1; c < 8; ++c) acc = fma(q[c], v[c], acc);
  return acc;
}
template <class LT>
__device__ __forceinline__ LT dot8(const LT (&q)[8], const LT (&v)[8], LT init) {
  LT acc = init;
#pragma unroll
  for (int c = 0; c < 8; ++c) acc = fma(q[c], v[c], acc);
  return acc;
}

__device__ __forceinline__ void axpy8(float (&acc)[8], float a, const float (&v)[8]) {
#pragma unroll
  for (int c = 0; c < 8; ++c) acc[c] = fmaf(a, v[c], acc[c]);
}

template <class LT, class ET>
__device__ __forceinline__ void widen8(const ET (&v)[8], LT (&w)[8]) {
#pragma unroll
  for (int c = 0; c < 8; ++c) w[c] = (LT)v[c];
}

// column w of a [.., CH] fp32 gradient tensor
template <int CH>
__device__ __forceinline__ void store_col_scaled(float* out, long long w, const float (&acc)[8], float sc) {
  float* o = out + w * CH;
  if constexpr (CH == 8) {
    *reinterpret_cast<float4*>(o) = make_float4(acc[0] * sc, acc[1] * sc, acc[2] * sc, acc[3] * sc);
    *reinterpret_cast<float4*>(o + 4) = make_float4(acc[4] * sc, acc[5] * sc, acc[6] * sc, acc[7] * sc);
  } else {
#pragma unroll
    for (int c = 0; c < CH; c += 2) *reinterpret_cast<float2*>(o + c) = make_float2(acc[c] * sc, acc[c + 1] * sc);
  }
}

// The bias B[s, o] of Eq. 3 lives in LDS as bt[o * HS + s], in the units and type of the logits (times log2 e).
// A lane's head is its fused column modulo HS, so it reads through bt + head at the compile-time offset o * HS,
// o = ((a+R)*KW + b+R)*KW + c+R.  A NULL bias is all zeros (its gradient may still be wanted).
template <class T, class LT, int KW, int HS>
__device__ __forceinline__ void fill_bias_table(LT* bt, const float* bias, int tid, int nthreads, int gofs = 0) {
  constexpr int K3 = KW * KW * KW;
  for (int i = tid; i < K3 * HS; i += nthreads) {
    const int j = i / HS, h = (gofs + i - j * HS) >> Win<T>::SH;      // (gofs: first column of the head group)
    bt[i] = bias ? (LT)bias[h * K3 + j] * (LT)kLog2e * (LT)Win<T>::kShare : (LT)0;
  }
}
template <class LT, int KW, int HS, bool BIAS> struct BiasTable { LT v[KW * KW * KW * HS]; };
template <class LT, int KW, int HS> struct BiasTable<LT, KW, HS, false> {};

template <int KW>
__device__ __forceinline__ unsigned active_roles(int s, int z0, int z1) {
  constexpr int R = KW / 2;
  unsigned active = 0;
#pragma unroll
  for (int i = 0; i < KW; ++i) {
    const int z = s - R + i;
    if (z >= z0 && z < z1) active |= 1u << i;
  }
  return active;
}

// =================================================================================================
// Policies.  A policy names the operand staged in LDS, the per-lane state of one in-flight plane (one
// "role"), and the arithmetic of one step.  Role i (state slot (i+PH)%KW) is the in-flight plane
// z = s - R + i while LDS plane s is current; it is complete after step z + R.
// =================================================================================================

// ---- forward: lane owns a query column; K planes in LDS (in LT); softmax sums against a fixed reference ----
// The weights of a query are exp2(l - ref) with ONE reference per query, the largest logit of the first
// window row it meets: no running maximum is maintained, nothing is rescaled from row to row, and the inner
// loop has no branches.  phi = S / Z does not depend on the reference.  A logit more than ~2^7 above the
// reference (far outside what normalised features produce) overflows fp32 and makes Z non-finite; such a
// query is recomputed on its own with a two-pass softmax when it is stored.

// Eq. 3-4 for one query straight from global memory, all in fp64 (the rare path of the above).
template <int KW, int HS, class T>
__device__ void fwd_query_two_pass(const TiledParams& p, long long w) {
  constexpr int R = KW / 2;
  long long r = w;
  const int xs = (int)(r % p.Whg); r /= p.Whg;      // (global columns: w is a global column index)
  const int y = (int)(r % p.H); r /= p.H;
  const int z = (int)(r % p.D);
  typedef typename Mem<T>::E E;
  constexpr int CH = Mem<T>::CH, SH = Win<T>::SH;
  constexpr int CHW = CH << SH;            // channels of the whole head (w is the even column of a pair)
  const E* Qp = (const E*)p.Q + w * CH;    // re-read per offset: this path is rare, keep it small in registers
  double mx = -INFINITY, Z = 0.0, S0 = 0.0, S1 = 0.0, S2 = 0.0;
#pragma unroll 1
  for (int pass = 0; pass < 2; ++pass)
#pragma unroll 1
    for (int j = 0; j < KW * KW * KW; ++j) {
      const int a = j / (KW * KW) - R, bb = (j / KW) % KW - R, cc = j % KW - R;
      const int zz = z + a, yy = y + bb, xx = xs + cc * p.HSg;
      double l = 0.0;      // a neighbour outside the volume is a zero key
      if (zz >= 0 && zz < p.D && yy >= 0 && yy < p.H && xx >= 0 && xx < p.Whg) {
        const E* Kp = (const E*)p.K + (w + ((long long)a * p.H + bb) * p.Whg + cc * p.HSg) * CH;
#pragma unroll 1
        for (int c = 0; c < CHW; ++c) l = fma((double)Ld<E>::one(Qp + c), (double)Ld<E>::one(Kp + c), l);
        l *= (double)p.qscale;
      }
      if (p.bias) l += (double)p.bias[((xs % p.HSg) >> SH) * (KW * KW * KW) + j] * (double)kLog2e;
      if (pass == 0) {
        mx = fmax(mx, l);
      } else {
        const double e = (double)exp2_fast((float)(l - mx));
        Z += e; S0 += a * e; S1 += bb * e; S2 += cc * e;
      }
    }
  float* ph = p.phi + (w >> SH) * 3;
  ph[0] = (float)(S0 / Z); ph[1] = (float)(S1 / Z); ph[2] = (float)(S2 / Z);
  if (p.lse) p.lse[w >> SH] = (float)((mx + (double)log2_fast((float)Z)) * (double)kLn2);
}

template <int KW_, int HS_, class T_, class LT, bool BIAS = false>
struct FwdPolicy {
  static constexpr int KW = KW_, HS = HS_, R = KW_ / 2;
  static constexpr bool kBias = BIAS;
  typedef T_ T;
  typedef typename Mem<T_>::E E;
  typedef LT Logit;
  typedef LT ET;                           // LDS element type: no conversions in the inner loop
  typedef Patch<KW, HS> P;
  static constexpr bool kStats = false;
  static constexpr bool kWaveSums = false;
  struct State {
    LT q[8];            // Q * scale * log2e
    LT nref;            // minus the reference (log2 units) times Win<T>::kShare; the dot products start from it
    LT Z, S0, S1, S2;   // sum of weights and of weight*offset, relative to the reference.  Kept in LT: phi
  };                    // feeds the backward, where its error is multiplied by the upstream gradient
  struct Pre { float q[8]; };
  static __device__ __forceinline__ void arrived(Pre& a) { pin(a.q); }

  static __device__ __forceinline__ const E* lds_operand(const TiledParams& p) { return (const E*)p.K; }
  static __device__ __forceinline__ const E* own_operand(const TiledParams& p) { return (const E*)p.Q; }

  static __device__ __forceinline__ void reset(State& s) {
#pragma unroll
    for (int c = 0; c < 8; ++c) s.q[c] = (LT)0;
    s.nref = (LT)0; s.Z = (LT)0; s.S0 = (LT)0; s.S1 = (LT)0; s.S2 = (LT)0;
  }
  static __device__ __forceinline__ void prefetch(const TiledParams&, const E* own, long long, Pre& pre) {
    load8<T>(own, pre.q);
  }
  static __device__ __forceinline__ void refill(State& s, const Pre& pre, const TiledParams& p) {
#pragma unroll
    for (int c = 0; c < 8; ++c) s.q[c] = (LT)pre.q[c] * (LT)p.qscale;
    s.nref = (LT)0; s.Z = (LT)0; s.S0 = (LT)0; s.S1 = (LT)0; s.S2 = (LT)0;
  }
  // Fold one window row (in-plane row offset b) into the sums.  l holds the logits MINUS the reference (the dot
  // products started from nref); FIRST: the first row this query meets, whose l is relative to zero and which
  // fixes the reference.  The row sum goes to `plane` (the caller adds the plane's total to Z and S0 once).
  template <bool FIRST>
  static __device__ __forceinline__ void fold_row(State& s, LT (&l)[KW], LT& plane, int b) {
    if (FIRST) {
      float mx = (float)l[0];
#pragma unroll
      for (int c = 1; c < KW; ++c) mx = fmaxf(mx, (float)l[c]);
      s.nref = -(LT)mx * (LT)Win<T>::kShare;
#pragma unroll
      for (int c = 0; c < KW; ++c) l[c] -= (LT)mx;
    }
    float rs = 0.f, ws = 0.f;
#pragma unroll
    for (int c = 0; c < KW; ++c) {
      const float e = exp2_fast((float)l[c]);
      rs = c == 0 ? e : rs + e;
      if (c != R) ws = (c == 0) ? (float)(c - R) * e : fmaf((float)(c - R), e, ws);
    }
    const LT rr = (LT)rs;
    plane += rr;
    if (b != 0) s.S1 = fma((LT)b, rr, s.S1);
    s.S2 += (LT)ws;
  }
  template <int PH, bool FULL>
  static __device__ __forceinline__ void step(State (&st)[KW], const typename Lds<ET>::chunk* kb, const float4*,
                                              const float*, int lbase, unsigned active, const LT* bl) {
    LT plane[KW];      // per role: sum of the weights of this plane of its window
#pragma unroll
    for (int i = 0; i < KW; ++i) plane[i] = (LT)0;
#pragma unroll
    for (int b = 0; b < KW; ++b) {
      LT l[KW][KW];   // [role][col] of this window row
#pragma unroll
      for (int c = 0; c < KW; ++c) {
        LT kv[8];
        Lds<ET>::get8(kb, P::NPOS, lbase + b * P::PC + c * HS, kv);
#pragma unroll
        for (int i = 0; i < KW; ++i)
          if (FULL || (active & (1u << i))) {
            // role i sees this plane under the plane offset a = R - i
            LT init = st[(i + PH) % KW].nref;
            if (BIAS) init += bl[(((KW - 1 - i) * KW + b) * KW + c) * HS];
            l[i][c] = whole_logit<T, LT>(dot8<LT>(st[(i + PH) % KW].q, kv, init));
          }
      }
      // role KW-1 is the plane that entered last: this step shows it the first plane of its window
#pragma unroll
      for (int i = 0; i < KW; ++i)
        if (FULL || (active & (1u << i))) {
          if (i == KW - 1 && b == 0) fold_row<true>(st[(i + PH) % KW], l[i], plane[i], b - R);
          else fold_row<false>(st[(i + PH) % KW], l[i], plane[i], b - R);
        }
    }
#pragma unroll
    for (int i = 0; i < KW; ++i)
      if (FULL || (active & (1u << i))) {
        State& s = st[(i + PH) % KW];
        s.Z += plane[i];
        if (R - i != 0) s.S0 = fma((LT)(R - i), plane[i], s.S0);
      }
  }
  static __device__ __forceinline__ void store(const State& s, const TiledParams& p, long long w) {
    if (Mem<T>::PAIR && (w & 1)) return;      // the even lane of a pair stores for both
    const float zf = (float)s.Z;
    if (!(zf >= 1e-30f && zf <= 1e30f)) {     // overflowed, all underflowed, or NaN: this query alone, safely
      fwd_query_two_pass<KW, HS, T>(p, w);
      return;
    }
    LT inv = (LT)__builtin_amdgcn_rcpf(zf);
    inv = inv * ((LT)2 - s.Z * inv);          // one Newton step: relative error ~1e-14 in fp64
    float* ph = p.phi + (w >> Win<T>::SH) * 3;
    ph[0] = (float)(s.S0 * inv); ph[1] = (float)(s.S1 * inv); ph[2] = (float)(s.S2 * inv);
    if (p.lse)
      p.lse[w >> Win<T>::SH] = (float)(((LT)log2_fast(zf) - s.nref * (LT)(1.0f / Win<T>::kShare)) * (LT)kLn2);
  }
};

// ---- backward, dQ: lane owns a query column; K planes in LDS (fp32); w = exp(l - lse) ----------------
template <int KW_, int HS_, class T_, class LT, bool BIAS = false, bool SUMS = false>
struct DqPolicy {
  static constexpr int KW = KW_, HS = HS_, R = KW_ / 2;
  static constexpr bool kBias = BIAS;
  typedef T_ T;
  typedef typename Mem<T_>::E E;
  typedef LT Logit;
  typedef float ET;                        // the fp32 copy is needed for the fp32 accumulation anyway
  typedef Patch<KW, HS> P;
  static constexpr bool kStats = false;
  static constexpr bool kWaveSums = SUMS;      // this march also sums dl for the bias gradient: see WaveSumSink
  static_assert(!SUMS || (BIAS && !Mem<T_>::PAIR), "the sums come with the bias variant, one lane per window");
  struct State {
    LT q[8];          // Q * scale * log2e
    LT nlse;          // -lse * log2e * Win<T>::kShare
    float g0, g1, g2, ngphi;
    float acc[8];
  };
  struct Pre { float q[8]; float lse, g0, g1, g2, f0, f1, f2; };
  static __device__ __forceinline__ void arrived(Pre& a) {
    pin(a.q);
    pin(a.lse); pin(a.g0); pin(a.g1); pin(a.g2); pin(a.f0); pin(a.f1); pin(a.f2);
  }

  static __device__ __forceinline__ const E* lds_operand(const TiledParams& p) { return (const E*)p.K; }
  static __device__ __forceinline__ const E* own_operand(const TiledParams& p) { return (const E*)p.Q; }

  static __device__ __forceinline__ void reset(State& s) {
#pragma unroll
    for (int c = 0; c < 8; ++c) { s.q[c] = (LT)0; s.acc[c] = 0.f; }
    s.nlse = (LT)0; s.g0 = s.g1 = s.g2 = s.ngphi = 0.f;
  }
  static __device__ __forceinline__ void prefetch(const TiledParams& p, const E* own, long long w, Pre& a) {
    load8<T>(own, a.q);
    const long long ww = w >> Win<T>::SH;
    a.lse = p.lse_in[ww];
    const float* g = p.dphi + ww * 3;
    const float* f = p.phi_in + ww * 3;
    a.g0 = g[0]; a.g1 = g[1]; a.g2 = g[2]; a.f0 = f[0]; a.f1 = f[1]; a.f2 = f[2];
  }
  static __device__ __forceinline__ void refill(State& s, const Pre& a, const TiledParams& p) {
#pragma unroll
    for (int c = 0; c < 8; ++c) { s.q[c] = (LT)a.q[c] * (LT)p.qscale; s.acc[c] = 0.f; }
    s.nlse = -(LT)a.lse * (LT)kLog2e * (LT)Win<T>::kShare;
    s.g0 = a.g0; s.g1 = a.g1; s.g2 = a.g2;
    s.ngphi = -(a.g0 * a.f0 + a.g1 * a.f1 + a.g2 * a.f2);
  }
  // the same from LDS: the query's features at patch position pos of a staged Q plane, its statistics from the
  // (-lse*log2e, g) / -g.phi arrays the dK half of the workgroup keeps
  static __device__ __forceinline__ void refill_lds(State& s, const float4* own, int pos, const float4* sa,
                                                    const float* sc, const TiledParams& p) {
    float qf[8];
    Lds<float>::get8(own, P::NPOS, pos, qf);
#pragma unroll
    for (int c = 0; c < 8; ++c) { s.q[c] = (LT)qf[c] * (LT)p.qscale; s.acc[c] = 0.f; }
    const float4 a4 = sa[pos];
    s.nlse = (LT)a4.x;
    s.g0 = a4.y; s.g1 = a4.z; s.g2 = a4.w;
    s.ngphi = sc[pos];
  }
  // One step: for every in-plane offset (b, c) the K vector is read once and every active role i (plane
  // offset a = R - i) gets its pair: w = exp2(logit - lse), dl = w * (g.o - g.phi), dQ += dl * K.  What else
  // happens to dl is the sink's business: sink.begin(b, c) runs before the dot products of an in-plane offset,
  // sink.pair(i, b, c, dl) after each of them, sink.idle(i, b, c) for a role that is not active, sink.end_row(b)
  // after the last in-plane offset of row b.
  struct NoSink {
    static constexpr bool kRolledRows = false;
    __device__ __forceinline__ void begin(int, int) {}
    __device__ __forceinline__ void pair(int, int, int, float) {}
    __device__ __forceinline__ void idle(int, int, int) {}
    __device__ __forceinline__ void end_row(int) {}
  };
  template <int PH, bool FULL, class Sink>
  static __device__ __forceinline__ void pairs(State (&st)[KW], const typename Lds<ET>::chunk* kb, int lbase,
                                               unsigned active, const LT* bl, Sink& sink) {
    if constexpr (Sink::kRolledRows) {      // one copy of a row's code, run KW times (b is a run-time value then)
#pragma unroll 1
      for (int b = 0; b < KW; ++b) pairs_of_row<PH, FULL>(st, kb, lbase, active, bl, sink, b);
    } else {
#pragma unroll
      for (int b = 0; b < KW; ++b) pairs_of_row<PH, FULL>(st, kb, lbase, active, bl, sink, b);
    }
  }
  template <int PH, bool FULL, class Sink>
  static __device__ __forceinline__ void pairs_of_row(State (&st)[KW], const typename Lds<ET>::chunk* kb, int lbase,
                                                      unsigned active, const LT* bl, Sink& sink, int b) {
#pragma unroll
      for (int c = 0; c < KW; ++c) {
        float kf[8];
        Lds<ET>::get8(kb, P::NPOS, lbase + b * P::PC + c * HS, kf);
        LT kv[8];
        widen8<LT, float>(kf, kv);
        sink.begin(b, c);
#pragma unroll
        for (int i = 0; i < KW; ++i) {
          if (FULL || (active & (1u << i))) {
            State& s = st[(i + PH) % KW];
            LT init = s.nlse;
            if (BIAS) init += bl[(((KW - 1 - i) * KW + b) * KW + c) * HS];
            const float w = exp2_fast((float)whole_logit<T, LT>(dot8<LT>(s.q, kv, init)));
            // t = g.o - g.phi with o = (R - i, b - R, c - R)
            float tt = s.ngphi;
            if (R - i != 0) tt = fmaf((float)(R - i), s.g0, tt);
            if (b - R != 0) tt = fmaf((float)(b - R), s.g1, tt);
            if (c - R != 0) tt = fmaf((float)(c - R), s.g2, tt);
            const float dl = w * tt;
            axpy8(s.acc, dl, kf);
            sink.pair(i, b, c, dl);
          } else {
            sink.idle(i, b, c);
          }
        }
        if (c == KW - 1) sink.end_row(b);
      }
  }
  template <int PH, bool FULL>
  static __device__ __forceinline__ void step(State (&st)[KW], const typename Lds<ET>::chunk* kb, const float4*,
                                              const float*, int lbase, unsigned active, const LT* bl) {
    NoSink sink;
    pairs<PH, FULL>(st, kb, lbase, active, bl, sink);
  }
  // The same step, also adding dl of every (role, offset) to this lane's running sums for the bias gradient:
  // sums[(((a+R)*KW + b+R)*KW + c+R) * NT] is a lane-private column of an LDS array: a plain read, add and
  // write (nobody else touches the address; LDS atomics are an order of magnitude slower).  The sums of an
  // in-plane offset are read before its dot products and written after them.
  struct SumSink {
    static constexpr bool kRolledRows = false;
    float* sums;
    float run[KW];
    __device__ __forceinline__ void begin(int b, int c) {
#pragma unroll
      for (int i = 0; i < KW; ++i) run[i] = sums[(((KW - 1 - i) * KW + b) * KW + c) * NT];
    }
    __device__ __forceinline__ void pair(int i, int b, int c, float dl) {
      sums[(((KW - 1 - i) * KW + b) * KW + c) * NT] = run[i] + dl;
    }
    __device__ __forceinline__ void idle(int, int, int) {}
    __device__ __forceinline__ void end_row(int) {}
  };
  template <int PH, bool FULL>
  static __device__ __forceinline__ void step_sum(State (&st)[KW], const typename Lds<ET>::chunk* kb, int lbase,
                                                  unsigned active, const LT* bl, float* sums) {
    SumSink sink;
    sink.sums = sums;
    pairs<PH, FULL>(st, kb, lbase, active, bl, sink);
  }
  // The same step for a march that has no room for per-lane sums (k = 5: 125 offsets).  The wave transposes
  // through its own LDS staging area: for one window row b every lane writes its KW * KW values of dl (role i,
  // column c) to stage[(i * KW + c) * 64 + slot]; then lane 2e + part adds up one half (32 lanes' values, 8 vector
  // reads rotated by e against bank conflicts) of entry e = i * KW + c into its accumulator of row b.  With two
  // heads the lanes of a wave alternate heads and `slot` sorts them by head, so a half is a head; with one head
  // the two halves are added across the lane pair.  Only the wave itself touches its staging area: the fences
  // order its own LDS writes and reads.  `keep` is false for lanes that compute on a clamped column outside the
  // volume.
  struct WaveSumSink {
    static constexpr bool kRolledRows = true;      // (unrolled over the rows as well, this variant spills)
    float* acc;        // this lane's KW running sums, one per row b: acc[b * 64], in the wave's LDS area
    float* stage;      // this wave's KW * KW rows of 64 floats
    int lane, slot;
    bool keep;
    static_assert(HS <= 2 && 2 * KW * KW <= 64, "one or two heads; an adding lane per entry and half");
    __device__ __forceinline__ void begin(int, int) {}
    __device__ __forceinline__ void pair(int i, int, int c, float dl) { stage[(i * KW + c) * 64 + slot] = keep ? dl : 0.f; }
    __device__ __forceinline__ void idle(int i, int, int c) { stage[(i * KW + c) * 64 + slot] = 0.f; }
    __device__ __forceinline__ void end_row(int b) {
      __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
      const int e = min(lane >> 1, KW * KW - 1);      // (lanes beyond the last entry repeat it; their sums are not used)
      const float4* src = reinterpret_cast<const float4*>(stage + e * 64 + (lane & 1) * 32);
      float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 2
      for (int j = 0; j < 8; ++j) {
        const float4 v = src[(j + e) & 7];
        t.x += v.x; t.y += v.y; t.z += v.z; t.w += v.w;
      }
      float sum = (t.x + t.y) + (t.z + t.w);
      if (HS == 1) sum += partner(sum);
      acc[b * 64] += sum;
      __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    }
    // bias entry (offset o, head) this lane's accumulator of row b belongs to, or -1
    static __device__ __forceinline__ int entry(int lane, int b) {
      const int e = lane >> 1, part = lane & 1;
      if (e >= KW * KW || (HS == 1 && part != 0)) return -1;
      const int o = ((KW - 1 - e / KW) * KW + b) * KW + e % KW;
      return HS == 1 ? o : o * 2 + part;
    }
  };
  template <int PH, bool FULL>
  static __device__ __forceinline__ void step_wavesum(State (&st)[KW], const typename Lds<ET>::chunk* kb, int lbase,
                                                      unsigned active, const LT* bl, float* wave_area, bool keep) {
    const int lane = threadIdx.x & 63;
    WaveSumSink sink = {wave_area + KW * KW * 64 + lane, wave_area, lane,
                        HS == 1 ? lane : (lane & 1) * 32 + (lane >> 1), keep};
    pairs<PH, FULL>(st, kb, lbase, active, bl, sink);
  }
  // The same step, also handing dl of every (role, offset) to the key side:
  // dl_out[(a+R) * DLA + ((b+R)*KW + c+R) * NT + li], a = R - i the plane offset of role i; roles that are not
  // active emit 0.
  template <int DLA>
  struct EmitSink {
    static constexpr bool kRolledRows = false;
    float* out;      // dl_out + li
    __device__ __forceinline__ void begin(int, int) {}
    __device__ __forceinline__ void pair(int i, int b, int c, float dl) {
      out[(KW - 1 - i) * DLA + (b * KW + c) * NT] = dl;      // a + R = R - i + R = KW - 1 - i
    }
    __device__ __forceinline__ void idle(int i, int b, int c) { out[(KW - 1 - i) * DLA + (b * KW + c) * NT] = 0.f; }
    __device__ __forceinline__ void end_row(int) {}
  };
  template <int PH, bool FULL, int DLA>
  static __device__ __forceinline__ void step_emit(State (&st)[KW], const typename Lds<ET>::chunk* kb, int lbase,
                                                   unsigned active, float* dl_out, int li, const LT* bl) {
    EmitSink<DLA> sink;
    sink.out = dl_out + li;
    pairs<PH, FULL>(st, kb, lbase, active, bl, sink);
  }
  static __device__ __forceinline__ void store(const State& s, const TiledParams& p, long long w) {
    store_col_scaled<Mem<T>::CH>(p.out, w, s.acc, p.scale);
  }
};

// ---- backward, dK: lane owns a key column; Q planes (fp32) + per-query statistics in LDS ----------------
// The query at patch position (row, col) = (ty + r, tx + cc*HS) sees this lane's key of role i under the
// offset (a, b, c) = (i - R, R - r, R - cc).
template <int KW_, int HS_, class T_, class LT, bool BIAS = false>
struct DkPolicy {
  static constexpr int KW = KW_, HS = HS_, R = KW_ / 2;
  static constexpr bool kBias = BIAS;
  typedef T_ T;
  typedef typename Mem<T_>::E E;
  typedef LT Logit;
  typedef float ET;
  typedef Patch<KW, HS> P;
  static constexpr bool kStats = true;
  static constexpr bool kWaveSums = false;
  struct State {
    LT k[8];          // K * scale * log2e
    float acc[8];
  };
  struct Pre { float k[8]; };
  static __device__ __forceinline__ void arrived(Pre& a) { pin(a.k); }

  static __device__ __forceinline__ const E* lds_operand(const TiledParams& p) { return (const E*)p.Q; }
  static __device__ __forceinline__ const E* own_operand(const TiledParams& p) { return (const E*)p.K; }

  static __device__ __forceinline__ void reset(State& s) {
#pragma unroll
    for (int c = 0; c < 8; ++c) { s.k[c] = (LT)0; s.acc[c] = 0.f; }
  }
  static __device__ __forceinline__ void prefetch(const TiledParams&, const E* own, long long, Pre& pre) {
    load8<T>(own, pre.k);
  }
  static __device__ __forceinline__ void refill(State& s, const Pre& pre, const TiledParams& p) {
#pragma unroll
    for (int c = 0; c < 8; ++c) { s.k[c] = (LT)pre.k[c] * (LT)p.qscale; s.acc[c] = 0.f; }
  }
  static __device__ __forceinline__ void refill_lds(State& s, const float4* own, int pos, const float4*, const float*,
                                                    const TiledParams& p) {
    float kf[8];
    Lds<float>::get8(own, P::NPOS, pos, kf);
#pragma unroll
    for (int c = 0; c < 8; ++c) { s.k[c] = (LT)kf[c] * (LT)p.qscale; s.acc[c] = 0.f; }
  }
  template <int PH, bool FULL>
  static __device__ __forceinline__ void step(State (&st)[KW], const typename Lds<ET>::chunk* qb, const float4* sa,
                                              const float* sc, int lbase, unsigned active, const LT* bl) {
#pragma unroll
    for (int r = 0; r < KW; ++r)
#pragma unroll
      for (int cc = 0; cc < KW; ++cc) {
        const int idx = lbase + r * P::PC + cc * HS;
        float qf[8];
        Lds<ET>::get8(qb, P::NPOS, idx, qf);
        LT qv[8];
        widen8<LT, float>(qf, qv);
        const float4 a4 = sa[idx];     // (-lse*log2e, g_D, g_H, g_W) of that query
        float tb = sc[idx];            // -g.phi
        if (R - r != 0) tb = fmaf((float)(R - r), a4.z, tb);
        if (R - cc != 0) tb = fmaf((float)(R - cc), a4.w, tb);
        const LT nlse = (LT)a4.x;
#pragma unroll
        for (int i = 0; i < KW; ++i)
          if (FULL || (active & (1u << i))) {
            State& s = st[(i + PH) % KW];
            LT init = nlse;
            if (BIAS) init += bl[((i * KW + (KW - 1 - r)) * KW + (KW - 1 - cc)) * HS];
            const float w = exp2_fast((float)whole_logit<T, LT>(dot8<LT>(s.k, qv, init)));
            const float tt = (i - R != 0) ? fmaf((float)(i - R), a4.y, tb) : tb;
            axpy8(s.acc, w * tt, qf);
          }
      }
  }
  static __device__ __forceinline__ void store(const State& s, const TiledParams& p, long long w) {
    store_col_scaled<Mem<T>::CH>(p.out, w, s.acc, p.scale);
  }
};

// ---- the marching kernel ---------------------------------------------------------------------------
template <class Pol, bool STATS> struct SharedPlanes;
template <class Pol> struct SharedPlanes<Pol, false> {
  typename Lds<typename Pol::ET>::chunk main[2][Lds<typename Pol::ET>::CH * Pol::P::NPOS];
  BiasTable<typename Pol::Logit, Pol::KW, Pol::HS, Pol::kBias> bias;
  // per wave: sums of dl per (window offset, head), for the bias gradient of a dQ march (WaveSumSink)
  float wsum[Pol::kWaveSums ? (NT / 64) * Pol::KW * Pol::KW * Pol::KW * Pol::HS : 1];
  // per wave: KW * KW staging rows of 64 floats, then KW rows of per-lane running sums
  alignas(16) float wstage[Pol::kWaveSums ? (NT / 64) * (Pol::KW * Pol::KW + Pol::KW) * 64 : 4];
};
template <class Pol> struct SharedPlanes<Pol, true> {
  typename Lds<typename Pol::ET>::chunk main[2][Lds<typename Pol::ET>::CH * Pol::P::NPOS];
  float4 sa[2][Pol::P::NPOS];
  float sc[2][Pol::P::NPOS];
  BiasTable<typename Pol::Logit, Pol::KW, Pol::HS, Pol::kBias> bias;
};
// this lane's view of the bias table (NULL for a policy without bias)
template <class Pol, class Sh>
__device__ __forceinline__ const typename Pol::Logit* lane_bias(const Sh& sh, int xs) {
  if constexpr (Pol::kBias) return sh.bias.v + xs % Pol::HS;
  else return nullptr;
}

template <class Pol, int PH, class Sh, class Stg, class SStg>
__device__ __forceinline__ void march_body(typename Pol::State (&st)[Pol::KW], const TiledParams& p, const Tile& t,
                                           Sh& sh, int cur, int lbase, int s, typename Pol::Pre& pre,
                                           bool have_next, bool commit_next, const Stg& stg, const SStg& sst) {
  constexpr int KW = Pol::KW, R = KW / 2;
  const unsigned active = active_roles<KW>(s, t.z0, t.z1);
  const float4* sa = nullptr;
  const float* sc = nullptr;
  if constexpr (Pol::kStats) { sa = sh.sa[cur]; sc = sh.sc[cur]; }
  const typename Pol::Logit* bl = lane_bias<Pol>(sh, t.xs);
  if constexpr (Pol::kWaveSums) {      // a dQ march that also sums its dl for the bias gradient
    if (active == (1u << KW) - 1u)
      Pol::template step_wavesum<PH, true>(st, sh.main[cur], lbase, active, bl,
                                           sh.wstage + (threadIdx.x >> 6) * (KW * KW + KW) * 64, t.lane_ok);
    else
      Pol::template step_wavesum<PH, false>(st, sh.main[cur], lbase, active, bl,
                                            sh.wstage + (threadIdx.x >> 6) * (KW * KW + KW) * 64, t.lane_ok);
  } else {
    if (active == (1u << KW) - 1u) Pol::template step<PH, true>(st, sh.main[cur], sa, sc, lbase, active, bl);
    else Pol::template step<PH, false>(st, sh.main[cur], sa, sc, lbase, active, bl);
  }
  // the staged plane goes to LDS before the results are stored: the wait for its loads would otherwise
  // also wait for those stores (one counter covers loads and stores on this chip)
  if (commit_next) {
    stg.commit(sh.main[cur ^ 1]);
    if constexpr (Pol::kStats) sst.commit(sh.sa[cur ^ 1], sh.sc[cur ^ 1]);
  }
  // All loads of this step end here, before the stores are issued: a wait placed after the stores (or at the
  // top of the next step, when the refill below is skipped) would wait for the stores as well.
  Pol::arrived(pre);
  typename Pol::State& done = st[PH % KW];     // role 0 is complete: it has seen planes z-R .. z+R
  if ((active & 1u) && t.lane_ok) Pol::store(done, p, t.col + (long long)(s - R) * p.H * p.Whg);
  if (have_next) Pol::refill(done, pre, p);     // the freed slot takes the plane s + R + 1
}

struct NoStats {
  __device__ __forceinline__ void init(int, int, int, int, int, const TiledParams&, int, int = 0) {}
  __device__ __forceinline__ void fetch(const TiledParams&, long long, bool) {}
  __device__ __forceinline__ void zero_outside(float4*, float*) const {}
};

__device__ __forceinline__ int clampi(int v, int lo, int hi) { return min(max(v, lo), hi); }
// a valid column for a lane right of the volume; a half-head column keeps its parity, so that the two lanes of
// a pair still hold the two halves of one head
template <class T>
__device__ __forceinline__ int clamp_column(int xs, int Wh) {
  if (xs < Wh) return xs;
  return Mem<T>::PAIR ? Wh - 2 + (xs & 1) : Wh - 1;
}

// Workgroups that share a CU compete for its vector units, and the hardware prefers the older wave: left alone,
// the first workgroup on a CU runs at nearly full speed, the second one on what is left, and finishes the
// last third of its march alone, when a single wave per SIMD cannot keep the vector unit busy.  Each wave
// therefore lowers its own priority as it advances, in a sawtooth over four steps: whichever workgroup is (up to
// three steps) behind wins the arbitration, the workgroups of a CU advance together and finish together.
__device__ __forceinline__ void step_priority(int n) {
  switch (n & 3) {
    case 0: __builtin_amdgcn_s_setprio(3); break;
    case 1: __builtin_amdgcn_s_setprio(2); break;
    case 2: __builtin_amdgcn_s_setprio(1); break;
    default: __builtin_amdgcn_s_setprio(0); break;
  }
}

// One workgroup's march over its chunk.  id: logical tile index (after the XCD remap); smem: the workgroup's LDS.
template <class Pol>
__device__ __forceinline__ void march(const TiledParams& p, unsigned id, void* smem) {
  typedef typename Pol::P P;
  typedef typename Pol::T T;
  typedef typename Pol::E E;
  constexpr int KW = Pol::KW, HS = Pol::HS, R = KW / 2;
  constexpr bool ROT = (KW == 3);
  SharedPlanes<Pol, Pol::kStats>& sh = *reinterpret_cast<SharedPlanes<Pol, Pol::kStats>*>(smem);

  const Tile t = make_tile(p, id);
  const E* Lb = Pol::lds_operand(p) + (long long)t.b * p.D * t.plane_elems;
  // lanes outside the volume compute on a clamped (valid) column and never store
  const int cy = min(t.y, p.H - 1), cxs = gcol(p, t.gofs, clamp_column<T>(t.xs, p.Wh));
  const E* Ob = Pol::own_operand(p) + (long long)t.b * p.D * t.plane_elems +
                ((long long)cy * p.Whg + cxs) * Mem<T>::CH;
  const long long ccol = (long long)t.b * p.D * p.H * p.Whg + (long long)cy * p.Whg + cxs;
  const long long pw = (long long)p.H * p.Whg;
  const long long wb = (long long)t.b * p.D * pw;    // window index of (b, 0, 0, 0)
  const int lbase = t.ty * P::PC + t.tx;             // patch position of the window corner of this lane

  Stager<KW, HS, T, typename Pol::ET> stg;
  stg.init(threadIdx.x, t.y0, t.xs0, p.H, p.Wh, p, t.gofs);
  typename std::conditional<Pol::kStats, StatStager<KW, HS>, NoStats>::type sst;
  sst.init(threadIdx.x, t.y0, t.xs0, p.H, p.Wh, p, t.gofs, Win<T>::SH);
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    stg.zero_outside(sh.main[j]);
    if constexpr (Pol::kStats) sst.zero_outside(sh.sa[j], sh.sc[j]);
  }
  if constexpr (Pol::kBias) fill_bias_table<T, typename Pol::Logit, KW, HS>(sh.bias.v, p.bias, threadIdx.x, NT, t.gofs);
  if constexpr (Pol::kWaveSums) {      // every lane's running sums start at zero (its own slots: no barrier needed)
#pragma unroll
    for (int b = 0; b < KW; ++b)
      sh.wstage[(threadIdx.x >> 6) * (KW * KW + KW) * 64 + (KW * KW + b) * 64 + (threadIdx.x & 63)] = 0.f;
  }

  typename Pol::State st[KW];
#pragma unroll
  for (int i = 0; i < KW; ++i) Pol::reset(st[i]);
  {
    typename Pol::Pre pre;
    Pol::prefetch(p, Ob + (long long)t.z0 * t.plane_elems, ccol + t.z0 * pw, pre);
    Pol::refill(st[KW - 1], pre, p);
  }
  const int s_first = t.z0 - R, s_last = t.z1 - 1 + R;
  // Loads run one step ahead of their use and are issued at the END of a step, right after the registers
  // they land in were consumed: they are in flight across the barrier and the whole next step.  All of them
  // are unconditional and read clamped (valid) planes; what lies outside the volume or is not wanted is
  // discarded where it is consumed.
  typename Pol::Pre pre;
  auto issue_loads = [&](int s) {    // for step s: the plane s + 1 to stage and the plane s + R + 1 to refill
    const int sn = s + 1;
    const int zs = clampi(sn, 0, p.D - 1);
    stg.fetch(Lb + (long long)zs * t.plane_elems, sn >= 0 && sn < p.D);
    sst.fetch(p, wb + (long long)zs * pw, sn >= 0 && sn < p.D);
    const int zo = min(s + R + 1, p.D - 1);
    Pol::prefetch(p, Ob + (long long)zo * t.plane_elems, ccol + zo * pw, pre);
  };
  {
    const bool ok = s_first >= 0;
    const int zc = clampi(s_first, 0, p.D - 1);
    stg.fetch(Lb + (long long)zc * t.plane_elems, ok);
    sst.fetch(p, wb + (long long)zc * pw, ok);
    stg.commit(sh.main[0]);
    if constexpr (Pol::kStats) sst.commit(sh.sa[0], sh.sc[0]);
  }
  issue_loads(s_first);
  __syncthreads();

  // one step with the role -> register-slot phase PH fixed at compile time
  auto one_step = [&](auto PHc, int s) __attribute__((always_inline)) {
    constexpr int PH = decltype(PHc)::value;
    const int cur = (s - s_first) & 1;
    const bool commit_next = s + 1 <= s_last;
    const bool have_next = s + R + 1 < t.z1;
    step_priority(s - s_first);
    march_body<Pol, PH>(st, p, t, sh, cur, lbase, s, pre, have_next, commit_next, stg, sst);
    if (!ROT) {
      // rotate by moving: role i+1 becomes role i, the refilled slot 0 becomes role KW-1
      typename Pol::State tmp = st[0];
#pragma unroll
      for (int i = 0; i + 1 < KW; ++i) st[i] = st[i + 1];
      st[KW - 1] = tmp;
    }
    issue_loads(s + 1);
    __syncthreads();
  };
  if (ROT) {
    // the three phases are unrolled in sequence (not selected by a switch): the state stays in the same
    // registers from phase to phase and nothing has to be moved where the branches would meet
    int s = s_first;
    while (true) {
      one_step(std::integral_constant<int, 0>(), s); if (++s > s_last) break;
      one_step(std::integral_constant<int, 1 % KW>(), s); if (++s > s_last) break;
      one_step(std::integral_constant<int, 2 % KW>(), s); if (++s > s_last) break;
    }
  } else {
    for (int s = s_first; s <= s_last; ++s) one_step(std::integral_constant<int, 0>(), s);
  }
  if constexpr (Pol::kWaveSums) {      // every wave's totals go to its row of the LDS table, then the rows are folded
    constexpr int K3 = KW * KW * KW;
#pragma unroll
    for (int b = 0; b < KW; ++b) {
      const int e = Pol::WaveSumSink::entry(threadIdx.x & 63, b);
      if (e >= 0)
        sh.wsum[(threadIdx.x >> 6) * K3 * HS + e] =
            sh.wstage[(threadIdx.x >> 6) * (KW * KW + KW) * 64 + (KW * KW + b) * 64 + (threadIdx.x & 63)];
    }
    __syncthreads();
    for (int i = threadIdx.x; i < K3 * HS; i += NT) {
      double v = 0.0;
#pragma unroll
      for (int w = 0; w < NT / 64; ++w) v += (double)sh.wsum[w * K3 * HS + i];
      atomicAdd(p.dbias_acc + (i % HS) * K3 + i / HS, v);
    }
  }
}

template <class Pol, int WAVES>
__global__ void __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(WAVES)))
march_kernel(TiledParams p) {
  __shared__ __align__(16) unsigned char smem[sizeof(SharedPlanes<Pol, Pol::kStats>)];
  march<Pol>(p, xcd_remap(blockIdx.x, gridDim.x), smem);
}

// Two marches over the same tiles in one grid: even logical ids run PolA, odd ones PolB, writing outA / outB.
// The two workgroups of a tile are neighbours in dispatch order and land on the same XCD, so what one of
// them has just read from HBM (Q, K and the per-query statistics are inputs of both) is still in the caches
// in front of HBM when the other asks for it; run one after the other, each pass re-reads everything.
template <class PolA, class PolB, int WAVES>
__global__ void __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(WAVES)))
march_pair_kernel(TiledParams p, float* outA, float* outB) {
  constexpr size_t kA = sizeof(SharedPlanes<PolA, PolA::kStats>), kB = sizeof(SharedPlanes<PolB, PolB::kStats>);
  __shared__ __align__(16) unsigned char smem[kA > kB ? kA : kB];
  const unsigned id = xcd_remap(blockIdx.x, gridDim.x);
  if (id & 1u) {
    p.out = outB;
    march<PolB>(p, id >> 1, smem);
  } else {
    p.out = outA;
    march<PolA>(p, id >> 1, smem);
  }
}

// Adds a workgroup's per-lane sums of dl (dlsum[o * NT + lane], lane = column of the patch) to the fp64 sums
// of the bias gradient: lane = (window offset o, 32-lane segment) adds up its segment by the columns' position
// in a group of HS columns (position >> SH is the head; of a pair of half-head columns, which hold the same dl,
// only the even one counts), the 8 segments are folded across lanes, and one lane per offset issues the atomics.
// Called by NT lanes, tid = 0..NT-1, all of them.
template <class T, int KW, int HS>
__device__ __forceinline__ void reduce_dl_sums(const float* dlsum, int tid, double* acc, int gofs = 0) {
  static_assert(KW == 3 && HS <= 8 && NT == 256, "27 offsets x 8 segments of 32 lanes");
  constexpr int SH = Win<T>::SH, NH = HS >> SH;
  const int row = tid >> 3, seg = tid & 7;
  const bool on = row < 27;
  double cls[8];              // by (column mod 8)
#pragma unroll
  for (int c = 0; c < 8; ++c) cls[c] = 0.0;
  if (on) {
    const float4* src = reinterpret_cast<const float4*>(dlsum + row * NT + seg * 32);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float4 v = src[i];
      cls[4 * (i & 1) + 0] += (double)v.x; cls[4 * (i & 1) + 1] += (double)v.y;
      cls[4 * (i & 1) + 2] += (double)v.z; cls[4 * (i & 1) + 3] += (double)v.w;
    }
  }
#pragma unroll
  for (int h = 0; h < NH; ++h) {
    double v = 0.0;
#pragma unroll
    for (int c = h << SH; c < 8; c += HS) v += cls[c];
#pragma unroll
    for (int m = 1; m < 8; m <<= 1) v += __shfl_xor(v, m);
    if (on && seg == 0) atomicAdd(acc + ((gofs >> SH) + h) * 27 + row, v);
  }
}

// ---- backward with both operands staged once --------------------------------------------------------
// A 512-lane workgroup owns one tile: lanes 0..255 run the dQ march, lanes 256..511 the dK march, in the same
// steps.  The dQ half stages the haloed K planes, the dK half the haloed Q planes and query statistics, into
// rings of RING planes in LDS; what a half needs of the OTHER operand (the features of its own column, for the
// plane that enters its window next) it reads from the other half's ring instead of from memory.  Every
// input is read once per tile (plus halo) for both gradients.
template <int KW, int HS>
struct BwdRings {
  typedef Patch<KW, HS> P;
  static constexpr int RING = KW / 2 + 2;      // planes s .. s+R in use during step s, one more being written
  float4 k[RING][2 * P::NPOS];
  float4 q[RING][2 * P::NPOS];
  float4 sa[RING][P::NPOS];
  float sc[RING][P::NPOS];
};
template <int KW, int HS, class LT, bool BIAS>
struct BwdRingsB : BwdRings<KW, HS> {
  BiasTable<LT, KW, HS, BIAS> bias;
  alignas(16) float dlsum[BIAS ? KW * KW * KW * NT : 4];   // per query lane: running sums of dl per window offset
};

// the part of a step after the arithmetic, for one half; OTHER = the ring this half refills from
template <class Pol, int PH, class Commit>
__device__ __forceinline__ void shared_step(typename Pol::State (&st)[Pol::KW], const TiledParams& p, const Tile& t,
                                            const float4* lds_cur, const float4* sa_cur, const float* sc_cur,
                                            const float4* own_new, const float4* sa_new, const float* sc_new,
                                            int lbase, int s, bool fill_new, const Commit& commit_staged,
                                            const typename Pol::Logit* bl, float* sums) {
  constexpr int KW = Pol::KW, R = KW / 2;
  typedef typename Pol::P P;
  // the plane s + R enters the window of the newest role: its slot was freed by the store of the last step
  if (fill_new) Pol::refill_lds(st[(KW - 1 + PH) % KW], own_new, lbase + R * P::PC + R * Pol::HS, sa_new, sc_new, p);
  const unsigned active = active_roles<KW>(s, t.z0, t.z1);
  bool summed = false;
  if constexpr (Pol::kBias && !Pol::kStats) {      // (the dQ half, when the bias gradient is wanted: uniform)
    if (sums != nullptr) {
      if (active == (1u << KW) - 1u) Pol::template step_sum<PH, true>(st, lds_cur, lbase, active, bl, sums);
      else Pol::template step_sum<PH, false>(st, lds_cur, lbase, active, bl, sums);
      summed = true;
    }
  }
  if (!summed) {
    if (active == (1u << KW) - 1u) Pol::template step<PH, true>(st, lds_cur, sa_cur, sc_cur, lbase, active, bl);
    else Pol::template step<PH, false>(st, lds_cur, sa_cur, sc_cur, lbase, active, bl);
  }
  commit_staged();       // before the stores: its wait for the loads must not cover them
  if ((active & 1u) && t.lane_ok)          // role 0 has seen its whole window
    Pol::store(st[PH % KW], p, t.col + (long long)(s - R) * p.H * p.Whg);
}

template <class Pol, bool IS_DK, class Rings>
__device__ __forceinline__ void shared_march(const TiledParams& p, const Tile& t, Rings& sh, int tid) {
  typedef typename Pol::P P;
  typedef typename Pol::T T;
  typedef typename Pol::E E;
  constexpr int KW = Pol::KW, HS = Pol::HS, R = KW / 2, RING = Rings::RING;
  static_assert(KW == 3, "phase rotation below is written for k = 3");
  const E* Lb = Pol::lds_operand(p) + (long long)t.b * p.D * t.plane_elems;
  const long long pw = (long long)p.H * p.Whg;
  const long long wb = (long long)t.b * p.D * pw;
  const int lbase = t.ty * P::PC + t.tx;
  float4 (*mine)[2 * P::NPOS] = IS_DK ? sh.q : sh.k;        // the ring this half fills and marches over
  float4 (*other)[2 * P::NPOS] = IS_DK ? sh.k : sh.q;       // the ring it takes its own column from

  Stager<KW, HS, T, float> stg;
  stg.init(tid, t.y0, t.xs0, p.H, p.Wh, p, t.gofs);
  typename std::conditional<IS_DK, StatStager<KW, HS>, NoStats>::type sst;
  sst.init(tid, t.y0, t.xs0, p.H, p.Wh, p, t.gofs, Win<T>::SH);
#pragma unroll
  for (int j = 0; j < RING; ++j) {
    stg.zero_outside(mine[j]);
    if constexpr (IS_DK) sst.zero_outside(sh.sa[j], sh.sc[j]);
  }
  auto fetch = [&](int z) {
    const int zc = clampi(z, 0, p.D - 1);
    const bool ok = z >= 0 && z < p.D;
    stg.fetch(Lb + (long long)zc * t.plane_elems, ok);
    sst.fetch(p, wb + (long long)zc * pw, ok);
  };
  auto commit = [&](int slot) {
    stg.commit(mine[slot]);
    if constexpr (IS_DK) sst.commit(sh.sa[slot], sh.sc[slot]);
  };

  typename Pol::State st[KW];
#pragma unroll
  for (int i = 0; i < KW; ++i) Pol::reset(st[i]);
  const int s_first = t.z0 - R, s_last = t.z1 - 1 + R;
#pragma unroll
  for (int j = 0; j <= R; ++j) { fetch(s_first + j); commit(j); }
  fetch(s_first + R + 1);
  if constexpr (Pol::kBias && !IS_DK) fill_bias_table<T, typename Pol::Logit, KW, HS>(sh.bias.v, p.bias, tid, NT, t.gofs);
  const typename Pol::Logit* bl = lane_bias<Pol>(sh, t.xs);
  float* sums = nullptr;      // the dQ half's sums of dl, when the bias gradient is wanted
  if constexpr (Pol::kBias && !IS_DK) {
    if (p.dbias_acc != nullptr) {
      sums = sh.dlsum + tid;
#pragma unroll
      for (int j = 0; j < KW * KW * KW; ++j) sums[j * NT] = 0.f;
    }
  }
  __syncthreads();

  int cur = 0;                               // cur = (s - s_first) % RING
  auto one_step = [&](auto PHc, int s) __attribute__((always_inline)) {
    constexpr int PH = decltype(PHc)::value;
    const int nw = cur + R >= RING ? cur + R - RING : cur + R;               // slot of the plane s + R
    const int wr = nw + 1 >= RING ? nw + 1 - RING : nw + 1;                  // slot the staged plane goes to
    const bool fill_new = s + R < t.z1;
    // the staged plane s + R + 1 replaces the plane s - 1, which nobody reads any more
    auto commit_staged = [&]() { if (s + R + 1 <= s_last) commit(wr); };
    shared_step<Pol, PH>(st, p, t, mine[cur], sh.sa[cur], sh.sc[cur], other[nw], sh.sa[nw], sh.sc[nw], lbase, s,
                         fill_new, commit_staged, bl, sums);
    fetch(s + R + 2);
    cur = cur + 1 == RING ? 0 : cur + 1;
    __syncthreads();
  };
  // (here the phases are selected by a switch: unrolled in sequence, this kernel's two bodies spill)
  int ph = 0;
  for (int s = s_first; s <= s_last; ++s) {
    switch (ph) {
      case 0: one_step(std::integral_constant<int, 0>(), s); break;
      case 1: one_step(std::integral_constant<int, 1>(), s); break;
      default: one_step(std::integral_constant<int, 2>(), s); break;
    }
    ph = ph == KW - 1 ? 0 : ph + 1;
  }
  if constexpr (Pol::kBias && !IS_DK) {
    if (sums != nullptr)      // (uniform; the last step ended with a barrier, so every lane's sums are visible)
      reduce_dl_sums<T, KW, HS>(sh.dlsum, tid, p.dbias_acc, t.gofs);
  }
}

template <int KW, int HS, class T, class LT, bool BIAS>
__global__ void __launch_bounds__(2 * NT) __attribute__((amdgpu_waves_per_eu(2)))
bwd_shared_kernel(TiledParams p, float* dQ, float* dK) {
  __shared__ BwdRingsB<KW, HS, LT, BIAS> sh;
  const int tid = threadIdx.x & (NT - 1);
  Tile t = make_tile(p, xcd_remap(blockIdx.x, gridDim.x), tid);
  if (threadIdx.x < NT) {
    p.out = dQ;
    shared_march<DqPolicy<KW, HS, T, LT, BIAS>, false>(p, t, sh, tid);
  } else {
    p.out = dK;
    shared_march<DkPolicy<KW, HS, T, LT, BIAS>, true>(p, t, sh, tid);
  }
}

// ---- backward with every logit computed once (k = 3, one or two heads) --------------------------------
// 512 lanes per tile.  Lanes 0..255 ("query half") run the dQ march and hand dl of each of their 27 (query,
// key) pairs to lanes 256..511 ("key half") through LDS; a key lane sums dl * Q over the 27 queries that see
// its key of the current plane: dK needs no logits of its own.  Queries in the one-voxel ring around the
// patch belong to neighbouring tiles; the key half recomputes dl for the pairs of those queries that point
// into the patch (about 10 % of all pairs with one head), one or two ring queries per lane.  The ring is one
// row above and below and HS fused columns (one voxel) left and right.  The key half also stages all planes.
//   step s (K plane s current), one barrier B(s):
//     query half:  [refill newest role] [dl, dQ of 27 pairs -> DL[s&1]] [store dQ of plane s-1]   B(s)
//     key half:    B(s)   [gather plane s from DL[s&1]] [ring queries of step s+1 -> DL[(s+1)&1]]
//                  [commit K plane s+2, Q / ring statistics plane s+3] [store dK] [issue loads for K s+3, Q s+4]
// so the gather of step s overlaps the query half's arithmetic of step s+1, and the staged loads have a
// whole step to arrive.
template <class T, class LT, int HS_, bool BIAS>
struct FusedBwd {
  static constexpr int KW = 3, HS = HS_, R = 1;
  typedef Patch<KW, HS> P;
  typedef DqPolicy<KW, HS, T, LT, BIAS> Dq;
  static constexpr int NRP = 2 * P::PC + 2 * HS * TY;   // ring positions: top row, bottom row, left, right columns
  static constexpr int NRC = 3 * NRP;                // (ring position, inward offset) combinations per plane
  static constexpr int DLA = 9 * NT + NRC;           // floats per plane offset a: 9 in-plane offsets of the patch
  static constexpr int DLN = 3 * DLA;                //   lanes, then the ring combinations; one DL buffer
  static constexpr int QR = 5;                       // Q planes s-1 .. s+2 readable, one being written
  struct Lds {
    float4 k[2][2 * P::NPOS];
    float4 q[QR][2 * P::NPOS];
    float4 sa[QR][NRP];      // (-lse*log2e, g) of the ring queries
    float sc[QR][NRP];       // -g.phi
    float dl[2][DLN];
    BiasTable<LT, KW, HS, BIAS> bias;
  };
  // ring position -> patch row / column
  static __device__ __forceinline__ void ring_rc(int rp, int& pr, int& pc) {
    if (rp < P::PC) { pr = 0; pc = rp; }
    else if (rp < 2 * P::PC) { pr = P::PR - 1; pc = rp - P::PC; }
    else if (rp < 2 * P::PC + HS * TY) { const int e = rp - 2 * P::PC; pr = e / HS + 1; pc = e % HS; }
    else { const int e = rp - 2 * P::PC - HS * TY; pr = e / HS + 1; pc = HS + TX + e % HS; }
  }
  // the inverse, for a patch position outside the interior
  static __device__ __forceinline__ int ring_index(int pr, int pc) {
    if (pr == 0) return pc;
    if (pr == P::PR - 1) return P::PC + pc;
    if (pc < HS) return 2 * P::PC + (pr - 1) * HS + pc;
    return 2 * P::PC + HS * TY + (pr - 1) * HS + (pc - HS - TX);
  }
  // offset (b, c) number t = 0..2 of a ring query towards the patch; false if it points outside
  static __device__ __forceinline__ bool ring_offset(int pr, int pc, int t, int& b, int& c) {
    if (pr == 0 || pr == P::PR - 1) { b = pr == 0 ? 1 : -1; c = t - 1; }
    else { c = pc < HS ? 1 : -1; b = t - 1; }
    const int kr = pr + b, kc = pc + c * HS;
    return kr >= 1 && kr <= TY && kc >= HS && kc < HS + TX;
  }
};

template <class T, class LT, int HS, bool BIAS, int PH>
__device__ __forceinline__ void fused_query_step(typename DqPolicy<3, HS, T, LT, BIAS>::State (&st)[3],
                                                 typename DqPolicy<3, HS, T, LT, BIAS>::Pre& pre, const TiledParams& p,
                                                 const Tile& t, const typename Mem<T>::E* Ob, long long ccol,
                                                 const float4* kcur,
                                                 float* dl, int lbase, int tid, int s, bool fill_new, unsigned active,
                                                 bool store_old, long long w_old, const LT* bl) {
  typedef DqPolicy<3, HS, T, LT, BIAS> Dq;
  constexpr int KW = 3;
  if (fill_new) Dq::refill(st[(KW - 1 + PH) % KW], pre, p);
  {   // own features and statistics of the plane that enters next, one step ahead
    const int zc = clampi(s + 2, 0, p.D - 1);
    Dq::prefetch(p, Ob + (long long)zc * t.plane_elems, ccol + (long long)zc * p.H * p.Wh, pre);
  }
  constexpr int DLA = FusedBwd<T, LT, HS, BIAS>::DLA;
  if (active == 7u) Dq::template step_emit<PH, true, DLA>(st, kcur, lbase, active, dl, tid, bl);
  else Dq::template step_emit<PH, false, DLA>(st, kcur, lbase, active, dl, tid, bl);
  // the prefetched registers are pinned here, before the store: a wait for them at the top of the next step
  // would wait for the store as well
  Dq::arrived(pre);
  if (!t.lane_ok) {      // no such query: its dl must be zero for the keys next to it
    pre.g0 = pre.g1 = pre.g2 = 0.f;
    pre.f0 = pre.f1 = pre.f2 = 0.f;
  }
  if (store_old) Dq::store(st[PH % KW], p, w_old);
}

template <class T, class LT, int HS, bool BIAS>
__device__ __forceinline__ void fused_query_half(TiledParams p, const Tile& t,
                                                 typename FusedBwd<T, LT, HS, BIAS>::Lds& sh, int tid) {
  typedef FusedBwd<T, LT, HS, BIAS> F;
  typedef typename F::Dq Dq;
  typedef typename F::P P;
  constexpr int KW = 3, R = 1;
  const int cy = min(t.y, p.H - 1), cxs = clamp_column<T>(t.xs, p.Wh);
  const long long pw = (long long)p.H * p.Wh;
  typedef typename Mem<T>::E E;
  const E* Ob = (const E*)p.Q + (long long)t.b * p.D * t.plane_elems + ((long long)cy * p.Wh + cxs) * Mem<T>::CH;
  const long long ccol = (long long)t.b * p.D * pw + (long long)cy * p.Wh + cxs;
  const int lbase = t.ty * P::PC + t.tx;
  const int s_lo = t.z0 - 1, s_hi = t.z1;
  const int zlo = max(t.z0 - 1, 0), zhi = min(t.z1 + 1, p.D);     // planes whose dl is wanted

  typename Dq::State st[KW];
#pragma unroll
  for (int i = 0; i < KW; ++i) Dq::reset(st[i]);
  typename Dq::Pre pre;
  auto prefetch = [&](int z) {
    const int zc = clampi(z, 0, p.D - 1);
    Dq::prefetch(p, Ob + (long long)zc * t.plane_elems, ccol + zc * pw, pre);
  };
  // at the first step the roles are the planes s_lo-1, s_lo, s_lo+1: the middle one is filled here, the
  // newest at the top of the loop like in every step
  if (s_lo >= zlo) {
    prefetch(s_lo);
    Dq::arrived(pre);
    if (!t.lane_ok) { pre.g0 = pre.g1 = pre.g2 = 0.f; pre.f0 = pre.f1 = pre.f2 = 0.f; }
    Dq::refill(st[1], pre, p);
  }
  prefetch(s_lo + 1);
  Dq::arrived(pre);
  if (!t.lane_ok) { pre.g0 = pre.g1 = pre.g2 = 0.f; pre.f0 = pre.f1 = pre.f2 = 0.f; }
  if constexpr (BIAS) fill_bias_table<T, LT, KW, HS>(sh.bias.v, p.bias, tid, NT);
  const LT* bl = lane_bias<Dq>(sh, t.xs);
  __syncthreads();          // the key half has staged the first planes

  auto one_step = [&](auto PHc, int s) __attribute__((always_inline)) {
    constexpr int PH = decltype(PHc)::value;
    const float4* kcur = sh.k[(s - s_lo) & 1];
    float* dl = sh.dl[(s - s_lo) & 1];
    const bool fill_new = s + 1 >= zlo && s + 1 < zhi;
    const unsigned active = active_roles<KW>(s, zlo, zhi);
    const bool store_old = s - 1 >= t.z0 && s - 1 < t.z1 && t.lane_ok;
    const long long w_old = t.col + (long long)(s - 1) * pw;
    fused_query_step<T, LT, HS, BIAS, PH>(st, pre, p, t, Ob, ccol, kcur, dl, lbase, tid, s, fill_new, active,
                                          store_old, w_old, bl);
    __syncthreads();        // B(s)
  };
  if (sizeof(LT) == 8) {
    int s = s_lo;           // the three phases in sequence: the state never changes registers
    while (true) {
      one_step(std::integral_constant<int, 0>(), s); if (++s > s_hi) break;
      one_step(std::integral_constant<int, 1>(), s); if (++s > s_hi) break;
      one_step(std::integral_constant<int, 2>(), s); if (++s > s_hi) break;
    }
  } else {                  // (measured: the all-fp32 variant is 2 % faster with the phases under a switch)
    int ph = 0;
    for (int s = s_lo; s <= s_hi; ++s) {
      switch (ph) {
        case 0: one_step(std::integral_constant<int, 0>(), s); break;
        case 1: one_step(std::integral_constant<int, 1>(), s); break;
        default: one_step(std::integral_constant<int, 2>(), s); break;
      }
      ph = ph == KW - 1 ? 0 : ph + 1;
    }
  }
}

template <class T, class LT, int HS, bool BIAS>
__device__ __forceinline__ void fused_key_half(TiledParams p, const Tile& t,
                                               typename FusedBwd<T, LT, HS, BIAS>::Lds& sh, int tid) {
  typedef FusedBwd<T, LT, HS, BIAS> F;
  typedef typename F::P P;
  constexpr int KW = 3, QR = F::QR, NRP = F::NRP, NRC = F::NRC;
  constexpr int NRQ = 3 * NRP, RPL = (NRQ + NT - 1) / NT;      // ring queries per step; per lane (1 or 2)
  const long long pw = (long long)p.H * p.Wh;
  const long long wb = (long long)t.b * p.D * pw;
  typedef typename Mem<T>::E E;
  const E* Kb = (const E*)p.K + (long long)t.b * p.D * t.plane_elems;
  const E* Qb = (const E*)p.Q + (long long)t.b * p.D * t.plane_elems;
  const int s_lo = t.z0 - 1, s_hi = t.z1;

  // ---- staging: K and Q planes (whole haloed patch), statistics of the ring queries (lanes < NRP)
  Stager<KW, HS, T, float> stk, stq;
  stk.init(tid, t.y0, t.xs0, p.H, p.Wh, p, t.gofs);
  stq.init(tid, t.y0, t.xs0, p.H, p.Wh, p, t.gofs);
  stk.zero_outside(sh.k[0]);
  stk.zero_outside(sh.k[1]);
#pragma unroll
  for (int j = 0; j < QR; ++j) stq.zero_outside(sh.q[j]);
  int rpr, rpc;
  F::ring_rc(min(tid, NRP - 1), rpr, rpc);
  const int rgy = t.y0 - 1 + rpr, rgx = t.xs0 - HS + rpc;
  const bool ring_in = tid < NRP && rgy >= 0 && rgy < p.H && rgx >= 0 && rgx < p.Wh;
  const long long ring_w = (long long)min(max(rgy, 0), p.H - 1) * p.Wh + min(max(rgx, 0), p.Wh - 1);
  float r_lse, r_g[3], r_f[3];
  bool r_ok = false;
  auto fetch_k = [&](int z) {
    stk.fetch(Kb + (long long)clampi(z, 0, p.D - 1) * t.plane_elems, z >= 0 && z < p.D);
  };
  auto fetch_q = [&](int z) {
    const int zc = clampi(z, 0, p.D - 1);
    stq.fetch(Qb + (long long)zc * t.plane_elems, z >= 0 && z < p.D);
    const long long w = (wb + (long long)zc * pw + ring_w) >> Win<T>::SH;
    r_lse = p.lse_in[w];
    r_g[0] = p.dphi[w * 3]; r_g[1] = p.dphi[w * 3 + 1]; r_g[2] = p.dphi[w * 3 + 2];
    r_f[0] = p.phi_in[w * 3]; r_f[1] = p.phi_in[w * 3 + 1]; r_f[2] = p.phi_in[w * 3 + 2];
    r_ok = ring_in && z >= 0 && z < p.D;
  };
  auto commit_q = [&](int slot) {
    stq.commit(sh.q[slot]);
    if (tid < NRP) {
      const float g0 = r_ok ? r_g[0] : 0.f, g1 = r_ok ? r_g[1] : 0.f, g2 = r_ok ? r_g[2] : 0.f;
      sh.sa[slot][tid] = make_float4(r_ok ? -r_lse * kLog2e * Win<T>::kShare : 0.f, g0, g1, g2);
      sh.sc[slot][tid] = -(g0 * r_f[0] + g1 * r_f[1] + g2 * r_f[2]);
    }
  };
  // K slot of plane z: (z - s_lo) & 1;  Q slot: (z - s_lo) mod QR, kept as running counters below
  fetch_k(s_lo); stk.commit(sh.k[0]);
  fetch_k(s_lo + 1); stk.commit(sh.k[1]);
#pragma unroll
  for (int j = 0; j < 3; ++j) { fetch_q(s_lo + j); commit_q(j); }
  fetch_k(s_lo + 2);
  fetch_q(s_lo + 3);

  // ---- this lane's ring queries (number i: ring query tid + i * NT): plane offset a = ra - 1 (query plane
  // s - a), ring position rq
  int ra[RPL], rq[RPL], qr_[RPL], qc_[RPL], ring_pos[RPL];
  bool has_ring[RPL];
#pragma unroll
  for (int i = 0; i < RPL; ++i) {
    const int e = tid + i * NT;
    has_ring[i] = e < NRQ;
    ra[i] = has_ring[i] ? e / NRP : 0;
    rq[i] = has_ring[i] ? e - ra[i] * NRP : 0;
    F::ring_rc(rq[i], qr_[i], qc_[i]);
    ring_pos[i] = qr_[i] * P::PC + qc_[i];
  }
  // ---- gather addresses: the query of offset (b, c) sits at patch position (kr - b, kc - c * HS)
  const int kr = t.ty + 1, kc = t.tx + HS;
  int gidx[9];
#pragma unroll
  for (int bc = 0; bc < 9; ++bc) {
    const int b = bc / 3 - 1, c = bc % 3 - 1;
    const int qr = kr - b, qc = kc - c * HS;
    const bool inside = qr >= 1 && qr <= TY && qc >= HS && qc < HS + TX;
    const bool row = qr == 0 || qr == P::PR - 1;      // ring rows number their offsets by c, ring columns by b
    gidx[bc] = inside ? (bc * NT + (qr - 1) * TX + (qc - HS))
                      : (9 * NT + F::ring_index(qr, qc) * 3 + (row ? c + 1 : b + 1));
  }
  // ---- gradient of the bias: this half also sums dl over the patch's queries.  Lane = (row, segment):
  // row = (plane offset, in-plane offset) of the DL buffer, segment = 32 of its 256 lanes; the four components
  // of the vector reads are columns of fixed parity, hence of a fixed head.  The reads of a lane are rotated
  // by its row so that the rows of a wave fall into different banks.
  const int db_row = tid >> 3, db_seg = tid & 7;
  const bool db_on = BIAS && p.dbias_acc != nullptr && db_row < 27;
  double db_sum[4] = {0.0, 0.0, 0.0, 0.0};
  __syncthreads();          // first planes staged

  int qs = 0;               // Q slot of plane s (s = s_lo: 0)
  for (int s = s_lo; s <= s_hi; ++s) {
    const int kslot = (s - s_lo) & 1;
    float* dl = sh.dl[kslot];
    const bool key_plane = s >= t.z0 && s < t.z1;
    auto qslot = [&](int d) { int v = qs + d; v += v < 0 ? QR : 0; v -= v >= QR ? QR : 0; return v; };
    __syncthreads();        // B(s)
    // ---- gather: dK of this lane's key in plane s
    float acc[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[c] = 0.f;
    if (key_plane) {
      // 27 (dl, Q vector) pairs in nine groups of three (one window row each).  The reads of a group are issued
      // one group ahead of its arithmetic and the order is pinned: left to itself the scheduler hoists all 27
      // vector reads (and spills) when the loop is unrolled, and exposes the LDS latency once per plane offset
      // when it is not.
      const float4* qpl[3] = {sh.q[qslot(1)], sh.q[qslot(0)], sh.q[qslot(-1)]};   // query plane s - (a - 1)
      float gd[2][3];
      float4 gq[2][3][2];
      auto read_group = [&](int g, int buf) __attribute__((always_inline)) {
        const int a = g / 3, b = g % 3 - 1;
#pragma unroll
        for (int ci = 0; ci < 3; ++ci) {
          const int c = ci - 1, pos = (kr - b) * P::PC + kc - c * HS;
          gd[buf][ci] = dl[a * F::DLA + gidx[(b + 1) * 3 + ci]];
          gq[buf][ci][0] = qpl[a][pos];
          gq[buf][ci][1] = qpl[a][P::NPOS + pos];
        }
      };
      read_group(0, 0);
#pragma unroll
      for (int g = 0; g < 9; ++g) {
        if (g + 1 < 9) read_group(g + 1, (g + 1) & 1);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ci = 0; ci < 3; ++ci) {
          const float d = gd[g & 1][ci];
          const float4 u = gq[g & 1][ci][0], v = gq[g & 1][ci][1];
          acc[0] = fmaf(d, u.x, acc[0]); acc[1] = fmaf(d, u.y, acc[1]);
          acc[2] = fmaf(d, u.z, acc[2]); acc[3] = fmaf(d, u.w, acc[3]);
          acc[4] = fmaf(d, v.x, acc[4]); acc[5] = fmaf(d, v.y, acc[5]);
          acc[6] = fmaf(d, v.z, acc[6]); acc[7] = fmaf(d, v.w, acc[7]);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    if constexpr (BIAS) {
      // pairs of step s whose query plane z = s + 1 - (a + 1) this workgroup owns (the halo planes' pairs are
      // counted by the workgroups that own them)
      const int da = db_row / 9, zq = s + 1 - da;
      if (db_on && zq >= t.z0 && zq < t.z1) {
        const float4* src = reinterpret_cast<const float4*>(dl + da * F::DLA + (db_row - da * 9) * NT + db_seg * 32);
        float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float4 v = src[(i + db_row) & 7];
          sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
        }
        db_sum[0] += (double)sum.x; db_sum[1] += (double)sum.y; db_sum[2] += (double)sum.z; db_sum[3] += (double)sum.w;
      }
    }
    // ---- ring queries of the NEXT step (their K and Q planes are already in LDS): ahead of the barrier that
    // hands them to the gather, and ahead of the commit below, whose loads thereby get a whole step to arrive
    if (s + 1 >= t.z0 && s + 1 < t.z1) {
      float* dln = sh.dl[kslot ^ 1];
#pragma unroll
      for (int i = 0; i < RPL; ++i) {
        if (!has_ring[i]) continue;
        const int sl = qslot(2 - ra[i]);              // query plane z = (s + 1) - a, a = ra - 1
        float qf[8];
        Lds<float>::get8(sh.q[sl], P::NPOS, ring_pos[i], qf);
        LT qv[8];
        widen8<LT, float>(qf, qv);
        const float4 a4 = sh.sa[sl][rq[i]];
        const float base = fmaf((float)(ra[i] - 1), a4.y, sh.sc[sl][rq[i]]);
#pragma unroll
        for (int tt = 0; tt < 3; ++tt) {
          int b, c;
          const bool valid = F::ring_offset(qr_[i], qc_[i], tt, b, c);
          const int kpos = valid ? (qr_[i] + b) * P::PC + qc_[i] + c * HS : ring_pos[i];
          float kf[8];
          Lds<float>::get8(sh.k[kslot ^ 1], P::NPOS, kpos, kf);
          LT kv[8];
          widen8<LT, float>(kf, kv);
          LT l = fma(dot8<LT>(qv, kv), (LT)p.qscale, (LT)a4.x);
          if constexpr (BIAS) l += sh.bias.v[((ra[i] * 3 + b + 1) * 3 + c + 1) * HS + qc_[i] % HS];
          l = whole_logit<T, LT>(l);      // (ring queries of a pair sit in neighbouring lanes: NRP is even)
          const float tq = fmaf((float)b, a4.z, fmaf((float)c, a4.w, base));
          dln[ra[i] * F::DLA + 9 * NT + rq[i] * 3 + tt] = valid ? exp2_fast((float)l) * tq : 0.f;
        }
      }
    }
    // the staged planes go to LDS last: K plane s + 2 replaces plane s, Q plane s + 3 replaces plane s - 2
    stk.commit(sh.k[kslot]);
    commit_q(qslot(3));
    // (the store after the commit: the commit's wait for its loads must not cover it)
    if (key_plane && t.lane_ok) store_col_scaled<Mem<T>::CH>(p.out, t.col + (long long)s * pw, acc, p.scale);
    fetch_k(s + 3);
    fetch_q(s + 4);
    qs = qs + 1 == QR ? 0 : qs + 1;
  }
  if constexpr (BIAS) {
    if (p.dbias_acc != nullptr) {      // (uniform) fold the components into heads, the 8 segments into one lane
      // a component's columns have a fixed position in the group of HS columns; of a pair of half-head
      // columns (which hold the same dl) only the even one counts
      constexpr int SH = Win<T>::SH, NH = HS >> SH;
      double hsum[NH];
#pragma unroll
      for (int h = 0; h < NH; ++h) {
        double v = 0.0;
#pragma unroll
        for (int c = h << SH; c < 4; c += HS) v += db_sum[c];
#pragma unroll
        for (int m = 1; m < 8; m <<= 1) v += __shfl_xor(v, m);
        hsum[h] = v;
      }
      if (db_on && db_seg == 0) {
#pragma unroll
        for (int h = 0; h < NH; ++h) atomicAdd(p.dbias_acc + h * 27 + db_row, hsum[h]);
      }
    }
  }
}

template <class T, class LT, int HS, bool BIAS>
__global__ void __launch_bounds__(2 * NT) __attribute__((amdgpu_waves_per_eu(2)))
bwd_fused_kernel(TiledParams p, float* dQ, float* dK) {
  __shared__ typename FusedBwd<T, LT, HS, BIAS>::Lds sh;
  const int tid = threadIdx.x & (NT - 1);
  const Tile t = make_tile(p, xcd_remap(blockIdx.x, gridDim.x), tid);
  if (threadIdx.x < NT) {
    p.out = dQ;
    fused_query_half<T, LT, HS, BIAS>(p, t, sh, tid);
  } else {
    // every SIMD holds one wave of each half; the key half's step is the longer one (the query half waits for it
    // at the barrier), so its waves win the arbitration for the vector unit and the query wave fills the gaps
    __builtin_amdgcn_s_setprio(3);
    p.out = dK;
    fused_key_half<T, LT, HS, BIAS>(p, t, sh, tid);
  }
}

// ---- backward with every logit computed once, one 256-lane workgroup per tile (k = 3, one head) -----------
// The same arithmetic as bwd_fused_kernel, but the lanes that compute dl for a query column (phase A) afterwards
// gather dK for the key of the same column (phase B), and two such workgroups share a CU.  In the 512-lane
// kernel the query wave and the key wave of a SIMD meet at a barrier every step, so a step lasts as long as the
// slower of the two, each of them alone on its SIMD for part of it, and a single wave cannot issue fast enough to
// keep the vector unit busy.  Here the two waves of a SIMD belong to different workgroups and run freely against
// each other: whenever one waits (barrier, LDS, memory) the other has arithmetic to issue.  What makes two
// workgroups fit: one K plane (not two: the next one is committed in phase B, when nobody reads it), a ring of
// three Q planes (plane s+1 is committed in phase A, when nobody gathers), one dl buffer: 79 KB.
//   step s (K plane s in LDS; roles = query planes s-1, s, s+1):
//     phase A  [refill newest role from registers] [commit Q plane s+1 and its ring statistics] [dl, dQ of 27
//              pairs -> dl] [issue loads: own column of plane s+2, K plane s+1] [store dQ of plane s-1]   barrier
//     phase R  [ring queries of this step -> dl]  (they read Q plane s+1, committed in phase A)            barrier
//     phase B  [gather dK of plane s] [commit K plane s+1] [store dK] [issue loads: Q plane s+2]           barrier
template <class T, class LT, int HS_, bool BIAS>
struct SymBwd {
  typedef FusedBwd<T, LT, HS_, BIAS> F;
  typedef typename F::P P;
  static constexpr int QR = 3;
  struct Lds {
    float4 k[2 * P::NPOS];
    float4 q[QR][2 * P::NPOS];
    float4 sa[QR][F::NRP];
    float sc[QR][F::NRP];
    float dl[F::DLN];
    BiasTable<LT, 3, HS_, BIAS> bias;
  };
};

template <class T, class LT, int HS, bool BIAS>
__global__ void __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(2)))
bwd_sym_kernel(TiledParams p, float* dQ, float* dK) {
  typedef SymBwd<T, LT, HS, BIAS> S;
  typedef typename S::F F;
  typedef typename F::Dq Dq;
  typedef typename F::P P;
  typedef typename Mem<T>::E E;
  constexpr int KW = 3, NRP = F::NRP, NRQ = 3 * NRP, RPL = (NRQ + NT - 1) / NT;
  __shared__ typename S::Lds sh;
  const int tid = threadIdx.x;
  const Tile t = make_tile(p, xcd_remap(blockIdx.x, gridDim.x));
  const long long pw = (long long)p.H * p.Wh;
  const long long wb = (long long)t.b * p.D * pw;
  const E* Kb = (const E*)p.K + (long long)t.b * p.D * t.plane_elems;
  const E* Qb = (const E*)p.Q + (long long)t.b * p.D * t.plane_elems;
  const int cy = min(t.y, p.H - 1), cxs = clamp_column<T>(t.xs, p.Wh);
  const E* Ob = Qb + ((long long)cy * p.Wh + cxs) * Mem<T>::CH;            // own query column
  const long long ccol = wb + (long long)cy * p.Wh + cxs;
  const int lbase = t.ty * P::PC + t.tx;
  const int s_lo = t.z0 - 1, s_hi = t.z1;
  const int zlo = max(t.z0 - 1, 0), zhi = min(t.z1 + 1, p.D);              // query planes whose dl is wanted

  // ---- staging: the K plane in the stager's own registers, the Q plane (same patch geometry) in qv
  Stager<KW, HS, T, float> stg;
  stg.init(tid, t.y0, t.xs0, p.H, p.Wh, p, t.gofs);
  stg.zero_outside(sh.k);
#pragma unroll
  for (int j = 0; j < S::QR; ++j) stg.zero_outside(sh.q[j]);
  float4 qv[P::NL];
  bool q_ok = false;
  int rpr, rpc;
  F::ring_rc(min(tid, NRP - 1), rpr, rpc);
  const int rgy = t.y0 - 1 + rpr, rgx = t.xs0 - HS + rpc;
  const bool ring_in = tid < NRP && rgy >= 0 && rgy < p.H && rgx >= 0 && rgx < p.Wh;
  const long long ring_w = (long long)min(max(rgy, 0), p.H - 1) * p.Wh + min(max(rgx, 0), p.Wh - 1);
  float r_lse, r_g[3], r_f[3];       // statistics of ring position `tid` of the Q plane fetched last
  auto fetch_k = [&](int z) {
    stg.fetch(Kb + (long long)clampi(z, 0, p.D - 1) * t.plane_elems, z >= 0 && z < p.D);
  };
  auto fetch_q = [&](int z) {
    const int zc = clampi(z, 0, p.D - 1);
    stg.fetch_into(qv, Qb + (long long)zc * t.plane_elems);
    const long long w = (wb + (long long)zc * pw + ring_w) >> Win<T>::SH;
    r_lse = p.lse_in[w];
    r_g[0] = p.dphi[w * 3]; r_g[1] = p.dphi[w * 3 + 1]; r_g[2] = p.dphi[w * 3 + 2];
    r_f[0] = p.phi_in[w * 3]; r_f[1] = p.phi_in[w * 3 + 1]; r_f[2] = p.phi_in[w * 3 + 2];
    q_ok = z >= 0 && z < p.D;
  };
  auto commit_q = [&](int slot) {
    stg.commit_from(qv, q_ok, sh.q[slot]);
    if (tid < NRP) {
      const bool ok = ring_in && q_ok;
      const float g0 = ok ? r_g[0] : 0.f, g1 = ok ? r_g[1] : 0.f, g2 = ok ? r_g[2] : 0.f;
      sh.sa[slot][tid] = make_float4(ok ? -r_lse * kLog2e * Win<T>::kShare : 0.f, g0, g1, g2);
      sh.sc[slot][tid] = -(g0 * r_f[0] + g1 * r_f[1] + g2 * r_f[2]);
    }
  };
  // Q slot of plane s - 1 + j in phase PH: (PH + j) % 3
  fetch_q(s_lo - 1); commit_q(0);
  fetch_q(s_lo); commit_q(1);
  fetch_k(s_lo); stg.commit(sh.k);
  fetch_q(s_lo + 1);

  // ---- this lane's ring queries, packed: [0] = ring position | rq << 9 | ra << 16 | ring row << 18 | negative
  // fixed offset component << 19 | valid(tt) << 20.. | used << 31;  [1] = key position of tt = 0, 1, 2 (10 bits each)
  unsigned rdesc[RPL][2];
#pragma unroll
  for (int i = 0; i < RPL; ++i) {
    const int e = tid + i * NT;
    const bool used = e < NRQ;
    const int ra = used ? e / NRP : 1, rq = used ? e - ra * NRP : 0;
    int qr_, qc_;
    F::ring_rc(rq, qr_, qc_);
    const int ring_pos = qr_ * P::PC + qc_;
    const bool rowq = qr_ == 0 || qr_ == P::PR - 1;
    const bool neg = rowq ? qr_ != 0 : qc_ >= HS;      // row 0 looks down (b = +1), the left columns look right (c = +1)
    unsigned da = (unsigned)ring_pos | (unsigned)rq << 9 | (unsigned)ra << 16 | (rowq ? 1u << 18 : 0u) |
                  (neg ? 1u << 19 : 0u) | (used ? 1u << 31 : 0u), db = 0;
#pragma unroll
    for (int tt = 0; tt < 3; ++tt) {
      int b, c;
      const bool valid = F::ring_offset(qr_, qc_, tt, b, c);
      const int kpos = valid ? (qr_ + b) * P::PC + qc_ + c * HS : ring_pos;
      da |= valid ? 1u << (20 + tt) : 0u;
      db |= (unsigned)kpos << (10 * tt);
    }
    rdesc[i][0] = da; rdesc[i][1] = db;
  }
  // ---- gather addresses: the query of offset (b, c) sits at patch position (kr - b, kc - c * HS)
  const int kr = t.ty + 1, kc = t.tx + HS;
  int gidx[9];
#pragma unroll
  for (int bc = 0; bc < 9; ++bc) {
    const int b = bc / 3 - 1, c = bc % 3 - 1;
    const int qr = kr - b, qc = kc - c * HS;
    const bool inside = qr >= 1 && qr <= TY && qc >= HS && qc < HS + TX;
    const bool row = qr == 0 || qr == P::PR - 1;
    gidx[bc] = inside ? (bc * NT + (qr - 1) * TX + (qc - HS))
                      : (9 * NT + F::ring_index(qr, qc) * 3 + (row ? c + 1 : b + 1));
  }
  const int db_row = tid >> 3, db_seg = tid & 7;      // bias gradient: see bwd_fused_kernel
  const bool db_on = BIAS && p.dbias_acc != nullptr && db_row < 27;
  double db_sum[4] = {0.0, 0.0, 0.0, 0.0};

  // ---- the query roles
  typename Dq::State st[KW];
#pragma unroll
  for (int i = 0; i < KW; ++i) Dq::reset(st[i]);
  typename Dq::Pre pre;
  auto prefetch = [&](int z) {
    const int zc = clampi(z, 0, p.D - 1);
    Dq::prefetch(p, Ob + (long long)zc * t.plane_elems, ccol + zc * pw, pre);
  };
  auto no_query = [&]() {      // a lane without a query: its dl must be zero for the keys next to it
    if (!t.lane_ok) { pre.g0 = pre.g1 = pre.g2 = 0.f; pre.f0 = pre.f1 = pre.f2 = 0.f; }
  };
  if (s_lo >= zlo) {
    prefetch(s_lo);
    Dq::arrived(pre);
    no_query();
    Dq::refill(st[1], pre, p);
  }
  prefetch(s_lo + 1);
  if constexpr (BIAS) fill_bias_table<T, LT, KW, HS>(sh.bias.v, p.bias, tid, NT);
  const LT* bl = lane_bias<Dq>(sh, t.xs);
  __syncthreads();

  auto one_step = [&](auto PHc, int s) __attribute__((always_inline)) {
    constexpr int PH = decltype(PHc)::value;
    constexpr int Q0 = PH % 3, Q1 = (PH + 1) % 3, Q2 = (PH + 2) % 3;      // Q slots of the planes s - 1, s, s + 1
    const bool fill_new = s + 1 >= zlo && s + 1 < zhi;
    const unsigned active = active_roles<KW>(s, zlo, zhi);
    const bool store_old = s - 1 >= t.z0 && s - 1 < t.z1 && t.lane_ok;
    const bool key_plane = s >= t.z0 && s < t.z1;
    step_priority(s - s_lo);
    // ================= phase A
    Dq::arrived(pre);
    no_query();
    if (fill_new) Dq::refill(st[(KW - 1 + PH) % KW], pre, p);
    commit_q(Q2);      // Q plane s + 1 replaces plane s - 2
    if (active == 7u) Dq::template step_emit<PH, true, F::DLA>(st, sh.k, lbase, active, sh.dl, tid, bl);
    else Dq::template step_emit<PH, false, F::DLA>(st, sh.k, lbase, active, sh.dl, tid, bl);
    prefetch(s + 2);
    fetch_k(s + 1);
    if (store_old) store_col_scaled<Mem<T>::CH>(dQ, t.col + (long long)(s - 1) * pw, st[PH % KW].acc, p.scale);
    __syncthreads();
    // ================= phase R: the pairs of the ring queries that point into the patch.  A lane's ring query
    // (number e = tid + i * NT: plane offset index ra = e / NRP, query plane s + 1 - ra, ring position rq) and its
    // three key positions are fixed for the whole march and packed into rdesc; all LDS reads are issued before
    // the three dot products, which advance together.
    if (key_plane) {
#pragma unroll
      for (int i = 0; i < RPL; ++i) {
        unsigned da = rdesc[i][0], db = rdesc[i][1];
        asm volatile("" : "+v"(da), "+v"(db));      // unpacked here, in every step: hoisted out of the loop, the
        if (!(da >> 31)) continue;                   // addresses derived from them would occupy (and spill) registers
        const int ring_pos = da & 511, rq = (da >> 9) & 127, ra = (da >> 16) & 3;
        const bool rowq = (da >> 18) & 1;             // ring row: its offsets differ in c; ring column: in b
        const float sgn = (da & (1u << 19)) ? -1.f : 1.f;   // the fixed component of the offset
        const int sl = ra == 0 ? Q2 : (ra == 1 ? Q1 : Q0);
        float qf[8], kf[3][8];
        Lds<float>::get8(sh.q[sl], P::NPOS, ring_pos, qf);
        const float4 a4 = sh.sa[sl][rq];
        const float c4 = sh.sc[sl][rq];
#pragma unroll
        for (int tt = 0; tt < 3; ++tt) Lds<float>::get8(sh.k, P::NPOS, (db >> (10 * tt)) & 1023, kf[tt]);
        LT qd[8];
        widen8<LT, float>(qf, qd);
        // t = g.o - g.phi with o = (ra - 1, b, c): u + (tt - 1) * v
        const float base = fmaf((float)(ra - 1), a4.y, c4);
        const float u = fmaf(sgn, rowq ? a4.z : a4.w, base), v = rowq ? a4.w : a4.z;
        LT l[3];
#pragma unroll
        for (int tt = 0; tt < 3; ++tt) {
          LT kd[8];
          widen8<LT, float>(kf[tt], kd);
          l[tt] = fma(dot8<LT>(qd, kd), (LT)p.qscale, (LT)a4.x);
        }
#pragma unroll
        for (int tt = 0; tt < 3; ++tt) {
          if constexpr (BIAS) {
            const int b = rowq ? (sgn > 0.f ? 1 : -1) : tt - 1, c = rowq ? tt - 1 : (sgn > 0.f ? 1 : -1);
            l[tt] += sh.bias.v[((ra * 3 + b + 1) * 3 + c + 1) * HS + (ring_pos % P::PC) % HS];
          }
          const LT lw = whole_logit<T, LT>(l[tt]);
          const float tq = fmaf((float)(tt - 1), v, u);
          const bool valid = (da >> (20 + tt)) & 1;
          sh.dl[ra * F::DLA + 9 * NT + rq * 3 + tt] = valid ? exp2_fast((float)lw) * tq : 0.f;
        }
      }
    }
    __syncthreads();
    // ================= phase B
    float acc[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[c] = 0.f;
    if (key_plane) {
      // 27 (dl, Q vector) pairs in nine groups of three (one window row each); the reads of a group are issued
      // one group ahead of its arithmetic and the order is pinned
      const float4* qpl[3] = {sh.q[Q2], sh.q[Q1], sh.q[Q0]};      // a = 0, 1, 2: query plane s + 1 - a
      float gd[2][3];
      float4 gq[2][3][2];
      auto read_group = [&](int g, int buf) __attribute__((always_inline)) {
        const int a = g / 3, b = g % 3 - 1;
#pragma unroll
        for (int ci = 0; ci < 3; ++ci) {
          const int c = ci - 1, pos = (kr - b) * P::PC + kc - c * HS;
          gd[buf][ci] = sh.dl[a * F::DLA + gidx[(b + 1) * 3 + ci]];
          gq[buf][ci][0] = qpl[a][pos];
          gq[buf][ci][1] = qpl[a][P::NPOS + pos];
        }
      };
      read_group(0, 0);
#pragma unroll
      for (int g = 0; g < 9; ++g) {
        if (g + 1 < 9) read_group(g + 1, (g + 1) & 1);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ci = 0; ci < 3; ++ci) {
          const float d = gd[g & 1][ci];
          const float4 u = gq[g & 1][ci][0], v = gq[g & 1][ci][1];
          acc[0] = fmaf(d, u.x, acc[0]); acc[1] = fmaf(d, u.y, acc[1]);
          acc[2] = fmaf(d, u.z, acc[2]); acc[3] = fmaf(d, u.w, acc[3]);
          acc[4] = fmaf(d, v.x, acc[4]); acc[5] = fmaf(d, v.y, acc[5]);
          acc[6] = fmaf(d, v.z, acc[6]); acc[7] = fmaf(d, v.w, acc[7]);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    if constexpr (BIAS) {
      const int da = db_row / 9, zq = s + 1 - da;
      if (db_on && zq >= t.z0 && zq < t.z1) {
        const float4* src = reinterpret_cast<const float4*>(sh.dl + da * F::DLA + (db_row - da * 9) * NT + db_seg * 32);
        float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float4 v = src[(i + db_row) & 7];
          sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
        }
        db_sum[0] += (double)sum.x; db_sum[1] += (double)sum.y; db_sum[2] += (double)sum.z; db_sum[3] += (double)sum.w;
      }
    }
    stg.commit(sh.k);      // K plane s + 1 (nobody reads the K plane in this phase)
    if (key_plane && t.lane_ok) store_col_scaled<Mem<T>::CH>(dK, t.col + (long long)s * pw, acc, p.scale);
    fetch_q(s + 2);
    __syncthreads();
  };
  {
    int s = s_lo;      // the three phases in sequence: the state never changes registers
    while (true) {
      one_step(std::integral_constant<int, 0>(), s); if (++s > s_hi) break;
      one_step(std::integral_constant<int, 1>(), s); if (++s > s_hi) break;
      one_step(std::integral_constant<int, 2>(), s); if (++s > s_hi) break;
    }
  }
  if constexpr (BIAS) {
    if (p.dbias_acc != nullptr) {
      constexpr int SH = Win<T>::SH, NH = HS >> SH;
      double hsum[NH];
#pragma unroll
      for (int h = 0; h < NH; ++h) {
        double v = 0.0;
#pragma unroll
        for (int c = h << SH; c < 4; c += HS) v += db_sum[c];
#pragma unroll
        for (int m = 1; m < 8; m <<= 1) v += __shfl_xor(v, m);
        hsum[h] = v;
      }
      if (db_on && db_seg == 0) {
#pragma unroll
        for (int h = 0; h < NH; ++h) atomicAdd(p.dbias_acc + h * 27 + db_row, hsum[h]);
      }
    }
  }
}

// ---- launch ------------------------------------------------------------------------------------------

int compute_units() {
  static int n = 0;
  if (n == 0) {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
      n = v;
    else
      n = 256;
  }
  return n;
}

// Chunk length along D.  A workgroup marches through zc + k - 1 planes, and `slots` workgroups are resident at a
// time (compute units x the workgroups of this kernel that fit one CU).  The cost of a split is the number of
// steps the busiest slot runs: full rounds of resident workgroups plus a last, partly filled one.  A round in
// which every workgroup has a CU to itself counts half when the kernel normally shares the CU (a workgroup alone
// steps almost twice as fast; a kernel that fills the CU with one workgroup gains nothing).  Small volumes thus
// get short chunks -- the machine is empty and only the length of one march counts -- large ones long chunks,
// because every chunk re-reads and re-computes k - 1 planes.
int chunk_length(long long tiles, int D, int k, int wgs_per_cu) {
  const int cus = compute_units();
  const long long slots = (long long)cus * wgs_per_cu;
  int best_zc = D;
  double best = 1e30;
  for (int nz = 1; nz <= D; ++nz) {
    const int zc = (D + nz - 1) / nz;
    if ((D + zc - 1) / zc != nz) continue;      // the same split as a smaller nz
    const long long wgs = tiles * nz, full = wgs / slots, rem = wgs % slots;
    const int steps = zc + k - 1;
    const double last = rem == 0 ? 0.0 : ((rem <= cus && wgs_per_cu >= 2) ? 0.5 : 1.0) * steps;
    const double cost = (double)full * steps + last;
    if (cost < best - 1e-9) { best = cost; best_zc = zc; }
  }
  return best_zc;
}

// hs: fused columns per voxel the kernel handles (its HS); more columns than that are split into head groups
TiledParams make_params(const Geo& g, int wgs_per_cu, int wgs_per_tile = 1, int hs = 0) {
  TiledParams p = {};
  p.B = g.B; p.D = g.D; p.H = g.H;
  p.HSg = g.heads * (g.d == 12 ? 2 : 1);           // twelve channels: two half-head columns per head
  p.Whg = g.W * p.HSg;
  if (hs <= 0 || hs > p.HSg) hs = p.HSg;
  p.ngrp = p.HSg / hs;
  p.hs_shift = 0;
  while ((1 << p.hs_shift) < hs) ++p.hs_shift;
  p.Wh = g.W * hs;
  p.ntx = (p.Wh + TX - 1) / TX;
  p.nty = (g.H + TY - 1) / TY;
  int zc = chunk_length((long long)p.ntx * p.nty * g.B * p.ngrp * wgs_per_tile, g.D, g.k, wgs_per_cu);
  if (zc > g.D) zc = g.D;
  if (zc < 1) zc = 1;
  p.ZC = zc;
  p.nzc = (g.D + zc - 1) / zc;
  p.scale = g.scale;
  p.qscale = g.scale * kLog2e;
  p.ch = g.d == 12 ? 6 : g.d;
  return p;
}

inline unsigned nblocks(const TiledParams& p) { return (unsigned)((long long)p.ntx * p.nty * p.B * p.nzc * p.ngrp); }

// waves per SIMD the register allocator is asked to make room for: the fp64 state of the fp32-input
// kernels and the five in-flight planes of k = 5 fit two, the all-fp32 state of k = 3 fits three
template <class LT, int KW> struct Waves { static constexpr int value = 2; };
template <> struct Waves<float, 3> { static constexpr int value = 3; };

// workgroups of one kernel instantiation that are resident on a CU (registers and LDS decide)
template <class Pol, int WAVES>
int resident_workgroups() {
  static int n = 0;
  if (n == 0) {
    int v = 0;
    n = (hipOccupancyMaxActiveBlocksPerMultiprocessor(&v, march_kernel<Pol, WAVES>, NT, 0) == hipSuccess && v > 0)
            ? v : WAVES;
  }
  return n;
}

template <class Pol, int WAVES>
void launch_march(const Geo& g, TiledParams io, hipStream_t st) {
  TiledParams p = make_params(g, resident_workgroups<Pol, WAVES>(), 1, Pol::HS);
  p.Q = io.Q; p.K = io.K; p.bias = io.bias; p.phi = io.phi; p.lse = io.lse;
  p.dphi = io.dphi; p.phi_in = io.phi_in; p.lse_in = io.lse_in; p.out = io.out;
  hipLaunchKernelGGL((march_kernel<Pol, WAVES>), dim3(nblocks(p)), dim3(NT), 0, st, p);
}

}  // namespace
}  // namespace modet

// calls CALL(KW, HS, T, LT) for the instantiation that covers (g.k, g.heads, dtype, fast_logits); the two halves
// (one or two heads and k = 5; four or eight heads) can be instantiated in different translation units
#define MODET_DISPATCH_FEW(CALL)                                                 \
  if (g.k == 3 && dtype == 0 && fast_logits) {                                   \
    switch (g.heads) {                                                           \
      case 1: return CALL(3, 1, float, float);                                   \
      case 2: return CALL(3, 2, float, float);                                   \
    }                                                                            \
  } else if (g.k == 3 && dtype == 0) {                                           \
    switch (g.heads) {                                                           \
      case 1: return CALL(3, 1, float, double);                                  \
      case 2: return CALL(3, 2, float, double);                                  \
    }                                                                            \
  } else if (g.k == 3) {                                                         \
    switch (g.heads) {                                                           \
      case 1: return CALL(3, 1, bf16_t, float);                                  \
      case 2: return CALL(3, 2, bf16_t, float);                                  \
    }                                                                            \
  } else if (g.k == 5 && dtype == 1) {                                           \
    switch (g.heads) {                                                           \
      case 1: return CALL(5, 1, bf16_t, float);                                  \
      case 2: return CALL(5, 2, bf16_t, float);                                  \
    }                                                                            \
  }
#define MODET_DISPATCH_MANY(CALL)                                                \
  if (g.k == 3 && dtype == 0 && fast_logits) {                                   \
    switch (g.heads) {                                                           \
      case 4: return CALL(3, 4, float, float);                                   \
      case 8: case 16: case 32: return CALL(3, 8, float, float);                 \
    }                                                                            \
  } else if (g.k == 3 && dtype == 0) {                                           \
    switch (g.heads) {                                                           \
      case 4: return CALL(3, 4, float, double);                                  \
      case 8: case 16: case 32: return CALL(3, 8, float, double);                \
    }                                                                            \
  } else if (g.k == 3) {                                                         \
    switch (g.heads) {                                                           \
      case 4: return CALL(3, 4, bf16_t, float);                                  \
      case 8: case 16: case 32: return CALL(3, 8, bf16_t, float);                \
    }                                                                            \
  }
#define MODET_DISPATCH(CALL)                                                     \
  MODET_DISPATCH_FEW(CALL)                                                       \
  MODET_DISPATCH_MANY(CALL)                                                      \
  return hipErrorNotSupported;

// the same for heads of six channels (k = 3; fp64 logits for fp32 inputs whatever the math mode)
#define MODET_DISPATCH_D6(CALL)                                                               \
  if (g.k == 3) {                                                                             \
    switch (g.heads) {                                                                        \
      case 1: return dtype == 0 ? CALL(3, 1, f32x6_t, double) : CALL(3, 1, bf16x6_t, float);  \
      case 2: return dtype == 0 ? CALL(3, 2, f32x6_t, double) : CALL(3, 2, bf16x6_t, float);  \
      case 4: return dtype == 0 ? CALL(3, 4, f32x6_t, double) : CALL(3, 4, bf16x6_t, float);  \
      case 8: case 16: case 32:                                                               \
        return dtype == 0 ? CALL(3, 8, f32x6_t, double) : CALL(3, 8, bf16x6_t, float);        \
    }                                                                                         \
  }                                                                                           \
  return hipErrorNotSupported;

// heads of twelve channels as pairs of half-heads: the kernels' HS is twice the number of heads
#define MODET_DISPATCH_D12(CALL)                                                                \
  if (g.k == 3) {                                                                               \
    switch (g.heads) {                                                                          \
      case 1: return dtype == 0 ? CALL(3, 2, f32x12_t, double) : CALL(3, 2, bf16x12_t, float);  \
      case 2: return dtype == 0 ? CALL(3, 4, f32x12_t, double) : CALL(3, 4, bf16x12_t, float);  \
      case 4: case 8: case 16: case 32:                                                         \
        return dtype == 0 ? CALL(3, 8, f32x12_t, double) : CALL(3, 8, bf16x12_t, float);        \
    }                                                                                           \
  }                                                                                             \
  return hipErrorNotSupported;
