// LDS-tiled ModeT kernels for head size d = 8 (gfx950).
//
// Paper: Section 3.3.1, Eq. 3 (neighbourhood scores + softmax) and Eq. 4-5 (attention-weighted
// offset grid), and their derivatives with respect to Q and K.
//
// Work decomposition (all three kernels)
//   * The head axis is folded into W: a voxel row [W][heads][8] is a row of Wh = W*heads
//     "fused columns" of 8 contiguous channels; the W-neighbour of fused column xs is xs +- heads.
//   * A workgroup of 256 lanes owns a TX x TY = 32 x 8 patch of (fused column, H row) and marches
//     along D over a chunk of planes.  One plane of the *other* operand (patch + halo, zero filled
//     outside the volume, so the inner loops are branch free) lives in LDS at a time, double
//     buffered; the next plane is fetched into registers while the current one is consumed.
//   * Register blocking along D: a lane keeps the k planes of its own operand that can see the
//     current LDS plane in flight, so every vector read from LDS is used for k windows.
//   * forward : lane owns a query column, K planes in LDS, online softmax (running maximum), no
//               logit or weight is ever stored.
//   * dQ      : lane owns a query column, K planes in LDS, weights from w = exp(l - lse).
//   * dK      : lane owns a key column, Q planes and per-query statistics (lse, g, g.phi) in LDS;
//               it gathers over the queries that see the key, so no atomics and a fixed summation
//               order (bit-reproducible).
//   * Logits are accumulated in fp64 for fp32 inputs (template parameter LT): an fp32 sum of eight
//     products leaves ~1e-6 of rounding on a logit of magnitude ~10, which the softmax turns into a
//     1e-6 relative error of the weights.  An fp64 FMA costs two fp32 issue slots on this chip, so fp64
//     is confined to the dot product, the subtraction of the softmax reference and the running softmax
//     sums of the forward; everything else is fp32.  Logits are kept in log2 units (the in-flight
//     operand is pre-multiplied by scale*log2(e)).
#include "modet_common.hpp"
#include <type_traits>
#ifdef MODET_TUNING_ENV
#include <stdlib.h>
#endif

namespace modet {
namespace {

#ifndef MODET_TX
#define MODET_TX 32
#endif
#ifndef MODET_TY
#define MODET_TY 8
#endif
constexpr int TX = MODET_TX, TY = MODET_TY, NT = TX * TY;
constexpr float kLog2e = 1.4426950408889634f, kLn2 = 0.6931471805599453f;

__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float log2_fast(float x) { return __builtin_amdgcn_logf(x); }

struct TiledParams {
  const void* Q; const void* K;
  const float* dphi; const float* phi_in; const float* lse_in;   // backward only
  float* phi; float* lse;                                         // forward outputs
  float* out;                                                     // dQ or dK
  int B, D, H, Wh;          // Wh = W * heads fused columns
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
  bool lane_ok;
  long long plane_elems;   // H * Wh * 8
  long long col;           // window index of (b, z=0, y, xs): + z*H*Wh
};

__device__ __forceinline__ Tile make_tile(const TiledParams& p) {
  Tile t;
  unsigned id = xcd_remap(blockIdx.x, gridDim.x);
  const int txi = id % p.ntx; id /= p.ntx;
  const int tyi = id % p.nty; id /= p.nty;
  const int zc = id % p.nzc;
  t.b = id / p.nzc;
  t.tx = threadIdx.x % TX; t.ty = threadIdx.x / TX;
  t.xs0 = txi * TX; t.y0 = tyi * TY;
  t.z0 = zc * p.ZC; t.z1 = min(p.D, t.z0 + p.ZC);
  t.xs = t.xs0 + t.tx; t.y = t.y0 + t.ty;
  t.lane_ok = t.xs < p.Wh && t.y < p.H;
  t.plane_elems = (long long)p.H * p.Wh * 8;
  t.col = (long long)t.b * p.D * p.H * p.Wh + (long long)t.y * p.Wh + t.xs;
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

template <class T> struct Ld;
template <> struct Ld<float> {
  static __device__ __forceinline__ float4 vec4(const float* p) { return *reinterpret_cast<const float4*>(p); }
};
template <> struct Ld<bf16_t> {
  static __device__ __forceinline__ float4 vec4(const bf16_t* p) {
    uint2 t = *reinterpret_cast<const uint2*>(p);
    return make_float4(__uint_as_float(t.x << 16), __uint_as_float(t.x & 0xFFFF0000u),
                       __uint_as_float(t.y << 16), __uint_as_float(t.y & 0xFFFF0000u));
  }
};

// stages one haloed plane of an [.., H, Wh, 8] tensor: global -> registers (fetch), registers -> LDS (commit)
template <int KW, int HS, class T, class ET>
struct Stager {
  typedef Patch<KW, HS> P;
  int goff[P::NL];      // element offset inside a plane, or -1: outside the volume / unused slot
  int loff[P::NL];      // (position << 1 | half) inside the patch, or -1 when unused
  float4 v[P::NL];

  __device__ __forceinline__ void init(int tid, int y0, int xs0, int H, int Wh) {
#pragma unroll
    for (int i = 0; i < P::NL; ++i) {
      const int e = tid + i * NT;
      const int pos = e >> 1, hv = e & 1;
      const int pr = pos / P::PC, pc = pos - pr * P::PC;
      const int gy = y0 - P::R + pr, gx = xs0 - P::R * HS + pc;
      const bool used = e < P::NV;
      const bool in = used && gy >= 0 && gy < H && gx >= 0 && gx < Wh;
      goff[i] = in ? (gy * Wh + gx) * 8 + hv * 4 : -1;
      loff[i] = used ? (pos << 1 | hv) : -1;
    }
  }
  // plane == nullptr: the plane lies outside the volume (zero padding)
  __device__ __forceinline__ void fetch(const T* plane) {
#pragma unroll
    for (int i = 0; i < P::NL; ++i)
      v[i] = (plane && goff[i] >= 0) ? Ld<T>::vec4(plane + goff[i]) : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  __device__ __forceinline__ void commit(typename Lds<ET>::chunk* buf) const {
#pragma unroll
    for (int i = 0; i < P::NL; ++i)
      if (loff[i] >= 0) Lds<ET>::put4(buf, P::NPOS, loff[i] >> 1, loff[i] & 1, v[i]);
  }
};

// per-query statistics of a haloed patch: (-lse*log2e, g_D, g_H, g_W) and -g.phi; zeros outside the volume
template <int KW, int HS>
struct StatStager {
  typedef Patch<KW, HS> P;
  int goff[P::NS];   // window index inside a plane, or -1
  int loff[P::NS];
  float4 a[P::NS];
  float c[P::NS];

  __device__ __forceinline__ void init(int tid, int y0, int xs0, int H, int Wh) {
#pragma unroll
    for (int i = 0; i < P::NS; ++i) {
      const int pos = tid + i * NT;
      const int pr = pos / P::PC, pc = pos - pr * P::PC;
      const int gy = y0 - P::R + pr, gx = xs0 - P::R * HS + pc;
      const bool used = pos < P::NPOS;
      const bool in = used && gy >= 0 && gy < H && gx >= 0 && gx < Wh;
      goff[i] = in ? gy * Wh + gx : -1;
      loff[i] = used ? pos : -1;
    }
  }
  // base = window index of (b, z, 0, 0); pass ok = false for planes outside the volume
  __device__ __forceinline__ void fetch(const TiledParams& p, long long base, bool ok) {
#pragma unroll
    for (int i = 0; i < P::NS; ++i) {
      if (ok && goff[i] >= 0) {
        const long long w = base + goff[i];
        const float* g = p.dphi + w * 3;
        const float* f = p.phi_in + w * 3;
        const float g0 = g[0], g1 = g[1], g2 = g[2];
        a[i] = make_float4(-p.lse_in[w] * kLog2e, g0, g1, g2);
        c[i] = -(g0 * f[0] + g1 * f[1] + g2 * f[2]);
      } else {
        a[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        c[i] = 0.f;
      }
    }
  }
  __device__ __forceinline__ void commit(float4* sa, float* sc) const {
#pragma unroll
    for (int i = 0; i < P::NS; ++i)
      if (loff[i] >= 0) { sa[loff[i]] = a[i]; sc[loff[i]] = c[i]; }
  }
};

template <class T>
__device__ __forceinline__ void load8(const T* p, bool ok, float (&q)[8]) {
  if (ok) {
    float4 a = Ld<T>::vec4(p), b = Ld<T>::vec4(p + 4);
    q[0] = a.x; q[1] = a.y; q[2] = a.z; q[3] = a.w; q[4] = b.x; q[5] = b.y; q[6] = b.z; q[7] = b.w;
  } else {
#pragma unroll
    for (int c = 0; c < 8; ++c) q[c] = 0.f;
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

__device__ __forceinline__ void store8_scaled(float* o, const float (&acc)[8], float sc) {
  *reinterpret_cast<float4*>(o) = make_float4(acc[0] * sc, acc[1] * sc, acc[2] * sc, acc[3] * sc);
  *reinterpret_cast<float4*>(o + 4) = make_float4(acc[4] * sc, acc[5] * sc, acc[6] * sc, acc[7] * sc);
}

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

// ---- forward: lane owns a query column; K planes in LDS (in LT); online softmax per window row --------
template <int KW_, int HS_, class T_, class LT>
struct FwdPolicy {
  static constexpr int KW = KW_, HS = HS_, R = KW_ / 2;
  typedef T_ T;
  typedef LT ET;                           // LDS element type: no conversions in the inner loop
  typedef Patch<KW, HS> P;
  static constexpr bool kStats = false;
  struct State {
    LT q[8];            // Q * scale * log2e
    float m;            // running maximum (log2 units)
    LT Z, S0, S1, S2;   // sum of weights and of weight*offset, relative to m.  Kept in LT: phi feeds the
  };                    // backward, where its error is multiplied by the upstream gradient
  struct Pre { float q[8]; };

  static __device__ __forceinline__ const T* lds_operand(const TiledParams& p) { return (const T*)p.K; }
  static __device__ __forceinline__ const T* own_operand(const TiledParams& p) { return (const T*)p.Q; }

  static __device__ __forceinline__ void reset(State& s) {
#pragma unroll
    for (int c = 0; c < 8; ++c) s.q[c] = (LT)0;
    s.m = -INFINITY; s.Z = (LT)0; s.S0 = (LT)0; s.S1 = (LT)0; s.S2 = (LT)0;
  }
  static __device__ __forceinline__ void prefetch(const TiledParams&, const T* own, long long, bool ok, Pre& pre) {
    load8<T>(own, ok, pre.q);
  }
  static __device__ __forceinline__ void refill(State& s, const Pre& pre, const TiledParams& p) {
#pragma unroll
    for (int c = 0; c < 8; ++c) s.q[c] = (LT)pre.q[c] * (LT)p.qscale;
    s.m = -INFINITY; s.Z = (LT)0; s.S0 = (LT)0; s.S1 = (LT)0; s.S2 = (LT)0;
  }
  // fold one window row (in-plane offsets (b, -R..R), plane offset a) into the running softmax
  static __device__ __forceinline__ void fold_row(State& s, const LT (&l)[KW], int a, int b) {
    float mx = s.m;
#pragma unroll
    for (int c = 0; c < KW; ++c) mx = fmaxf(mx, (float)l[c]);
    const float alpha = exp2_fast(s.m - mx);
    float rs = 0.f, ws = 0.f;
#pragma unroll
    for (int c = 0; c < KW; ++c) {
      const float e = exp2_fast((float)(l[c] - (LT)mx));
      rs += e;
      if (c != R) ws = fmaf((float)(c - R), e, ws);
    }
    const LT al = (LT)alpha, rr = (LT)rs;
    s.Z = fma(s.Z, al, rr);
    s.S0 = a == 0 ? s.S0 * al : fma(s.S0, al, (LT)a * rr);
    s.S1 = b == 0 ? s.S1 * al : fma(s.S1, al, (LT)b * rr);
    s.S2 = fma(s.S2, al, (LT)ws);
    s.m = mx;
  }
  template <int PH, bool FULL, class Sh>
  static __device__ __forceinline__ void step(State (&st)[KW], const Sh& sh, int cur, int lbase, unsigned active) {
    const typename Lds<ET>::chunk* kb = sh.main[cur];
#pragma unroll
    for (int b = 0; b < KW; ++b) {
      LT l[KW][KW];   // [role][col] of this window row
#pragma unroll
      for (int c = 0; c < KW; ++c) {
        LT kv[8];
        Lds<ET>::get8(kb, P::NPOS, lbase + b * P::PC + c * HS, kv);
#pragma unroll
        for (int i = 0; i < KW; ++i)
          if (FULL || (active & (1u << i))) l[i][c] = dot8<LT>(st[(i + PH) % KW].q, kv);
      }
#pragma unroll
      for (int i = 0; i < KW; ++i)
        if (FULL || (active & (1u << i))) fold_row(st[(i + PH) % KW], l[i], R - i, b - R);
    }
  }
  static __device__ __forceinline__ void store(const State& s, const TiledParams& p, long long w) {
    LT inv = (LT)__builtin_amdgcn_rcpf((float)s.Z);
    inv = inv * ((LT)2 - s.Z * inv);          // one Newton step: relative error ~1e-14 in fp64
    float* ph = p.phi + w * 3;
    ph[0] = (float)(s.S0 * inv); ph[1] = (float)(s.S1 * inv); ph[2] = (float)(s.S2 * inv);
    if (p.lse) p.lse[w] = (s.m + log2_fast((float)s.Z)) * kLn2;
  }
};

// ---- backward, dQ: lane owns a query column; K planes in LDS (fp32); w = exp(l - lse) ----------------
template <int KW_, int HS_, class T_, class LT>
struct DqPolicy {
  static constexpr int KW = KW_, HS = HS_, R = KW_ / 2;
  typedef T_ T;
  typedef float ET;                        // the fp32 copy is needed for the fp32 accumulation anyway
  typedef Patch<KW, HS> P;
  static constexpr bool kStats = false;
  struct State {
    LT q[8];          // Q * scale * log2e
    LT nlse;          // -lse * log2e
    float g0, g1, g2, ngphi;
    float acc[8];
  };
  struct Pre { float q[8]; float lse, g0, g1, g2, f0, f1, f2; };

  static __device__ __forceinline__ const T* lds_operand(const TiledParams& p) { return (const T*)p.K; }
  static __device__ __forceinline__ const T* own_operand(const TiledParams& p) { return (const T*)p.Q; }

  static __device__ __forceinline__ void reset(State& s) {
#pragma unroll
    for (int c = 0; c < 8; ++c) { s.q[c] = (LT)0; s.acc[c] = 0.f; }
    s.nlse = (LT)0; s.g0 = s.g1 = s.g2 = s.ngphi = 0.f;
  }
  static __device__ __forceinline__ void prefetch(const TiledParams& p, const T* own, long long w, bool ok,
                                                  Pre& a) {
    load8<T>(own, ok, a.q);
    if (ok) {
      a.lse = p.lse_in[w];
      const float* g = p.dphi + w * 3;
      const float* f = p.phi_in + w * 3;
      a.g0 = g[0]; a.g1 = g[1]; a.g2 = g[2]; a.f0 = f[0]; a.f1 = f[1]; a.f2 = f[2];
    } else {
      a.lse = a.g0 = a.g1 = a.g2 = a.f0 = a.f1 = a.f2 = 0.f;
    }
  }
  static __device__ __forceinline__ void refill(State& s, const Pre& a, const TiledParams& p) {
#pragma unroll
    for (int c = 0; c < 8; ++c) { s.q[c] = (LT)a.q[c] * (LT)p.qscale; s.acc[c] = 0.f; }
    s.nlse = -(LT)a.lse * (LT)kLog2e;
    s.g0 = a.g0; s.g1 = a.g1; s.g2 = a.g2;
    s.ngphi = -(a.g0 * a.f0 + a.g1 * a.f1 + a.g2 * a.f2);
  }
  template <int PH, bool FULL, class Sh>
  static __device__ __forceinline__ void step(State (&st)[KW], const Sh& sh, int cur, int lbase, unsigned active) {
    const typename Lds<ET>::chunk* kb = sh.main[cur];
#pragma unroll
    for (int b = 0; b < KW; ++b)
#pragma unroll
      for (int c = 0; c < KW; ++c) {
        float kf[8];
        Lds<ET>::get8(kb, P::NPOS, lbase + b * P::PC + c * HS, kf);
        LT kv[8];
        widen8<LT, float>(kf, kv);
#pragma unroll
        for (int i = 0; i < KW; ++i)
          if (FULL || (active & (1u << i))) {
            State& s = st[(i + PH) % KW];
            const float w = exp2_fast((float)dot8<LT>(s.q, kv, s.nlse));
            // t = g.o - g.phi with o = (R - i, b - R, c - R)
            float tt = s.ngphi;
            if (R - i != 0) tt = fmaf((float)(R - i), s.g0, tt);
            if (b - R != 0) tt = fmaf((float)(b - R), s.g1, tt);
            if (c - R != 0) tt = fmaf((float)(c - R), s.g2, tt);
            axpy8(s.acc, w * tt, kf);
          }
      }
  }
  static __device__ __forceinline__ void store(const State& s, const TiledParams& p, long long w) {
    store8_scaled(p.out + w * 8, s.acc, p.scale);
  }
};

// ---- backward, dK: lane owns a key column; Q planes (fp32) + per-query statistics in LDS ----------------
// The query at patch position (row, col) = (ty + r, tx + cc*HS) sees this lane's key of role i under the
// offset (a, b, c) = (i - R, R - r, R - cc).
template <int KW_, int HS_, class T_, class LT>
struct DkPolicy {
  static constexpr int KW = KW_, HS = HS_, R = KW_ / 2;
  typedef T_ T;
  typedef float ET;
  typedef Patch<KW, HS> P;
  static constexpr bool kStats = true;
  struct State {
    LT k[8];          // K * scale * log2e
    float acc[8];
  };
  struct Pre { float k[8]; };

  static __device__ __forceinline__ const T* lds_operand(const TiledParams& p) { return (const T*)p.Q; }
  static __device__ __forceinline__ const T* own_operand(const TiledParams& p) { return (const T*)p.K; }

  static __device__ __forceinline__ void reset(State& s) {
#pragma unroll
    for (int c = 0; c < 8; ++c) { s.k[c] = (LT)0; s.acc[c] = 0.f; }
  }
  static __device__ __forceinline__ void prefetch(const TiledParams&, const T* own, long long, bool ok, Pre& pre) {
    load8<T>(own, ok, pre.k);
  }
  static __device__ __forceinline__ void refill(State& s, const Pre& pre, const TiledParams& p) {
#pragma unroll
    for (int c = 0; c < 8; ++c) { s.k[c] = (LT)pre.k[c] * (LT)p.qscale; s.acc[c] = 0.f; }
  }
  template <int PH, bool FULL, class Sh>
  static __device__ __forceinline__ void step(State (&st)[KW], const Sh& sh, int cur, int lbase, unsigned active) {
    const typename Lds<ET>::chunk* qb = sh.main[cur];
    const float4* sa = sh.sa[cur];
    const float* sc = sh.sc[cur];
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
            const float w = exp2_fast((float)dot8<LT>(s.k, qv, nlse));
            const float tt = (i - R != 0) ? fmaf((float)(i - R), a4.y, tb) : tb;
            axpy8(s.acc, w * tt, qf);
          }
      }
  }
  static __device__ __forceinline__ void store(const State& s, const TiledParams& p, long long w) {
    store8_scaled(p.out + w * 8, s.acc, p.scale);
  }
};

// ---- the marching kernel ---------------------------------------------------------------------------
template <class Pol, bool STATS> struct SharedPlanes;
template <class Pol> struct SharedPlanes<Pol, false> {
  typename Lds<typename Pol::ET>::chunk main[2][Lds<typename Pol::ET>::CH * Pol::P::NPOS];
};
template <class Pol> struct SharedPlanes<Pol, true> {
  typename Lds<typename Pol::ET>::chunk main[2][Lds<typename Pol::ET>::CH * Pol::P::NPOS];
  float4 sa[2][Pol::P::NPOS];
  float sc[2][Pol::P::NPOS];
};

template <class Pol, int PH, class Sh, class Stg, class SStg>
__device__ __forceinline__ void march_body(typename Pol::State (&st)[Pol::KW], const TiledParams& p, const Tile& t,
                                           Sh& sh, int cur, int lbase, int s, const typename Pol::Pre& pre,
                                           bool have_next, bool commit_next, const Stg& stg, const SStg& sst) {
  constexpr int KW = Pol::KW, R = KW / 2;
  const unsigned active = active_roles<KW>(s, t.z0, t.z1);
  if (active == (1u << KW) - 1u) Pol::template step<PH, true>(st, sh, cur, lbase, active);
  else Pol::template step<PH, false>(st, sh, cur, lbase, active);
  // the staged plane goes to LDS before the results are stored: the wait for its loads would otherwise
  // also wait for those stores (one counter covers loads and stores on this chip)
  if (commit_next) {
    stg.commit(sh.main[cur ^ 1]);
    if constexpr (Pol::kStats) sst.commit(sh.sa[cur ^ 1], sh.sc[cur ^ 1]);
  }
  typename Pol::State& done = st[PH % KW];     // role 0 is complete: it has seen planes z-R .. z+R
  if ((active & 1u) && t.lane_ok) Pol::store(done, p, t.col + (long long)(s - R) * p.H * p.Wh);
  if (have_next) Pol::refill(done, pre, p);     // the freed slot takes the plane s + R + 1
}

struct NoStats {
  __device__ __forceinline__ void init(int, int, int, int, int) {}
  __device__ __forceinline__ void fetch(const TiledParams&, long long, bool) {}
};

template <class Pol, int WAVES>
__global__ void __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(WAVES)))
march_kernel(TiledParams p) {
  typedef typename Pol::P P;
  typedef typename Pol::T T;
  constexpr int KW = Pol::KW, HS = Pol::HS, R = KW / 2;
#ifdef MODET_NOROT
  constexpr bool ROT = false;
#else
  constexpr bool ROT = (KW == 3);
#endif
  __shared__ SharedPlanes<Pol, Pol::kStats> sh;

  const Tile t = make_tile(p);
  const T* Lb = Pol::lds_operand(p) + (long long)t.b * p.D * t.plane_elems;
  const T* Ob = Pol::own_operand(p) + (long long)t.b * p.D * t.plane_elems + ((long long)t.y * p.Wh + t.xs) * 8;
  const long long pw = (long long)p.H * p.Wh;
  const long long wb = (long long)t.b * p.D * pw;    // window index of (b, 0, 0, 0)
  const int lbase = t.ty * P::PC + t.tx;             // patch position of the window corner of this lane

  Stager<KW, HS, T, typename Pol::ET> stg;
  stg.init(threadIdx.x, t.y0, t.xs0, p.H, p.Wh);
  typename std::conditional<Pol::kStats, StatStager<KW, HS>, NoStats>::type sst;
  sst.init(threadIdx.x, t.y0, t.xs0, p.H, p.Wh);

  typename Pol::State st[KW];
#pragma unroll
  for (int i = 0; i < KW; ++i) Pol::reset(st[i]);
  {
    typename Pol::Pre pre;
    Pol::prefetch(p, Ob + (long long)t.z0 * t.plane_elems, t.col + t.z0 * pw, t.lane_ok, pre);
    Pol::refill(st[KW - 1], pre, p);
  }
  const int s_first = t.z0 - R, s_last = t.z1 - 1 + R;
  {
    const bool ok = s_first >= 0;
    stg.fetch(ok ? Lb + (long long)s_first * t.plane_elems : nullptr);
    sst.fetch(p, wb + (long long)s_first * pw, ok);
    stg.commit(sh.main[0]);
    if constexpr (Pol::kStats) sst.commit(sh.sa[0], sh.sc[0]);
  }
  __syncthreads();

  int ph = 0;
  for (int s = s_first; s <= s_last; ++s) {
    const int cur = (s - s_first) & 1;
    const int sn = s + 1;
    const bool commit_next = sn <= s_last;
    if (commit_next) {
      const bool ok = sn >= 0 && sn < p.D;
      stg.fetch(ok ? Lb + (long long)sn * t.plane_elems : nullptr);
      sst.fetch(p, wb + (long long)sn * pw, ok);
    }
    const int zn = s + R + 1;
    const bool have_next = zn < t.z1;
    typename Pol::Pre pre;
    Pol::prefetch(p, Ob + (long long)zn * t.plane_elems, t.col + zn * pw, t.lane_ok && have_next, pre);

    if (ROT) {
      switch (ph) {
        case 0: march_body<Pol, 0>(st, p, t, sh, cur, lbase, s, pre, have_next, commit_next, stg, sst); break;
        case 1: march_body<Pol, 1 % KW>(st, p, t, sh, cur, lbase, s, pre, have_next, commit_next, stg, sst); break;
        default: march_body<Pol, 2 % KW>(st, p, t, sh, cur, lbase, s, pre, have_next, commit_next, stg, sst); break;
      }
      ph = ph == KW - 1 ? 0 : ph + 1;
    } else {
      march_body<Pol, 0>(st, p, t, sh, cur, lbase, s, pre, have_next, commit_next, stg, sst);
      // rotate by moving: role i+1 becomes role i, the refilled slot 0 becomes role KW-1
      typename Pol::State tmp = st[0];
#pragma unroll
      for (int i = 0; i + 1 < KW; ++i) st[i] = st[i + 1];
      st[KW - 1] = tmp;
    }
    __syncthreads();
  }
}

// ---- launch ------------------------------------------------------------------------------------------
#ifndef MODET_WAVES
#define MODET_WAVES 2
#endif

TiledParams make_params(const Geo& g) {
  TiledParams p = {};
  p.B = g.B; p.D = g.D; p.H = g.H; p.Wh = g.W * g.heads;
  p.ntx = (p.Wh + TX - 1) / TX;
  p.nty = (g.H + TY - 1) / TY;
  // enough chunks along D to give every CU several workgroups (4 per CU on 256 CUs), but not so short
  // that the k-1 extra planes per chunk dominate
  const long long tiles = (long long)p.ntx * p.nty * g.B;
  int zc = 16;
  while (zc > 4 && tiles * ((g.D + zc - 1) / zc) < 1024) zc >>= 1;
#ifdef MODET_TUNING_ENV
  if (const char* e = getenv("MODET_ZC")) zc = atoi(e);
#endif
  if (zc > g.D) zc = g.D;
  p.ZC = zc;
  p.nzc = (g.D + zc - 1) / zc;
  p.scale = g.scale;
  p.qscale = g.scale * kLog2e;
  return p;
}

inline unsigned nblocks(const TiledParams& p) { return (unsigned)((long long)p.ntx * p.nty * p.B * p.nzc); }

// waves per SIMD the register allocator is asked to make room for: the fp64 state of the fp32-input
// kernels and the five in-flight planes of k = 5 fit two, the all-fp32 state of k = 3 fits three
template <class LT, int KW> struct Waves { static constexpr int value = MODET_WAVES; };
template <> struct Waves<float, 3> { static constexpr int value = 3; };

template <int KW, int HS, class T, class LT>
hipError_t launch_fwd_t(const Geo& g, const void* Q, const void* K, float* phi, float* lse, hipStream_t st) {
  TiledParams p = make_params(g);
  p.Q = Q; p.K = K; p.phi = phi; p.lse = lse;
  hipLaunchKernelGGL((march_kernel<FwdPolicy<KW, HS, T, LT>, Waves<LT, KW>::value>), dim3(nblocks(p)), dim3(NT), 0,
                     st, p);
  return hipGetLastError();
}

template <int KW, int HS, class T, class LT>
hipError_t launch_bwd_t(const Geo& g, const void* Q, const void* K, const float* dphi, const float* phi,
                        const float* lse, float* dQ, float* dK, hipStream_t st) {
  TiledParams p = make_params(g);
  p.Q = Q; p.K = K; p.dphi = dphi; p.phi_in = phi; p.lse_in = lse;
  p.out = dQ;
  hipLaunchKernelGGL((march_kernel<DqPolicy<KW, HS, T, LT>, Waves<LT, KW>::value>), dim3(nblocks(p)), dim3(NT), 0, st,
                     p);
  p.out = dK;
  hipLaunchKernelGGL((march_kernel<DkPolicy<KW, HS, T, LT>, Waves<LT, KW>::value>), dim3(nblocks(p)), dim3(NT), 0, st,
                     p);
  return hipGetLastError();
}

}  // namespace

// Covered: head size 8, no bias;  k = 3: 1/2/4/8 heads, fp32 inputs (fp64 logits) and bf16 inputs (fp32
// logits: the bf16 tolerance leaves room);  k = 5: 1/2 heads, bf16 inputs.
bool tiled_fwd_supported(int d, int heads, int k, int dtype, bool has_bias) {
  if (d != 8 || has_bias) return false;
  if (k == 3) return heads == 1 || heads == 2 || heads == 4 || heads == 8;
  if (k == 5) return dtype == 1 && (heads == 1 || heads == 2);
  return false;
}

bool tiled_bwd_supported(int d, int heads, int k, int dtype, bool has_bias) {
  return tiled_fwd_supported(d, heads, k, dtype, has_bias);
}

#define MODET_DISPATCH(CALL)                                                     \
  if (g.k == 3 && dtype == 0 && fast_logits) {                                   \
    switch (g.heads) {                                                           \
      case 1: return CALL(3, 1, float, float);                                   \
      case 2: return CALL(3, 2, float, float);                                   \
      case 4: return CALL(3, 4, float, float);                                   \
      case 8: return CALL(3, 8, float, float);                                   \
    }                                                                            \
  } else if (g.k == 3 && dtype == 0) {                                           \
    switch (g.heads) {                                                           \
      case 1: return CALL(3, 1, float, double);                                  \
      case 2: return CALL(3, 2, float, double);                                  \
      case 4: return CALL(3, 4, float, double);                                  \
      case 8: return CALL(3, 8, float, double);                                  \
    }                                                                            \
  } else if (g.k == 3) {                                                         \
    switch (g.heads) {                                                           \
      case 1: return CALL(3, 1, bf16_t, float);                                  \
      case 2: return CALL(3, 2, bf16_t, float);                                  \
      case 4: return CALL(3, 4, bf16_t, float);                                  \
      case 8: return CALL(3, 8, bf16_t, float);                                  \
    }                                                                            \
  } else if (g.k == 5 && dtype == 1) {                                           \
    switch (g.heads) {                                                           \
      case 1: return CALL(5, 1, bf16_t, float);                                  \
      case 2: return CALL(5, 2, bf16_t, float);                                  \
    }                                                                            \
  }                                                                              \
  return hipErrorNotSupported;

hipError_t launch_fwd_tiled(const Geo& g, int dtype, bool fast_logits, const void* Q, const void* K,
                            const float* bias, float* phi, float* lse, hipStream_t st) {
  (void)bias;
#define MODET_FWD(KW, HS, T, LT) launch_fwd_t<KW, HS, T, LT>(g, Q, K, phi, lse, st)
  MODET_DISPATCH(MODET_FWD)
#undef MODET_FWD
}

hipError_t launch_bwd_tiled(const Geo& g, int dtype, bool fast_logits, const void* Q, const void* K,
                            const float* bias, const float* dphi, const float* phi, const float* lse, float* dQ,
                            float* dK, hipStream_t st) {
  (void)bias;
#define MODET_BWD(KW, HS, T, LT) launch_bwd_t<KW, HS, T, LT>(g, Q, K, dphi, phi, lse, dQ, dK, st)
  MODET_DISPATCH(MODET_BWD)
#undef MODET_BWD
}

}  // namespace modet
