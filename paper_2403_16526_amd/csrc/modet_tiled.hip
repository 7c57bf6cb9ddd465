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
//   * Logits are accumulated in fp64 (template parameter LT): an fp32 sum of eight products leaves
//     ~1e-6 of rounding on a logit of magnitude ~10, which the softmax turns into a 1e-6 relative
//     error of the weights; fp64 FMAs issue at the rate of unpacked fp32 ones on this chip.
//     Logits are kept in log2 units (Q is pre-multiplied by scale*log2(e)).
#include "modet_common.hpp"

namespace modet {
namespace {

constexpr int TX = 32, TY = 8, NT = TX * TY;
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
// LDS holds, per position of the haloed patch, the 8 channels split in two float4 halves stored in
// separate arrays (lane-consecutive 16-byte reads are then bank-conflict free).
template <int KW, int HS>
struct Patch {
  static constexpr int R = KW / 2;
  static constexpr int PC = TX + 2 * R * HS, PR = TY + 2 * R, NPOS = PC * PR;
  static constexpr int NV = 2 * NPOS;                 // float4 slots per plane
  static constexpr int NL = (NV + NT - 1) / NT;       // float4 loads per lane per plane
  static constexpr int NS = (NPOS + NT - 1) / NT;     // positions per lane per plane (statistics)
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

template <int KW, int HS, class T>
struct Stager {
  typedef Patch<KW, HS> P;
  int goff[P::NL];      // element offset inside a plane, or -1: outside the volume / unused slot
  int loff[P::NL];      // float4 index inside an LDS plane buffer, or -1 when unused
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
      loff[i] = used ? hv * P::NPOS + pos : -1;
    }
  }
  // plane == nullptr: the plane lies outside the volume (zero padding)
  __device__ __forceinline__ void fetch(const T* plane) {
#pragma unroll
    for (int i = 0; i < P::NL; ++i)
      v[i] = (plane && goff[i] >= 0) ? Ld<T>::vec4(plane + goff[i]) : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  __device__ __forceinline__ void commit(float4* buf) const {
#pragma unroll
    for (int i = 0; i < P::NL; ++i)
      if (loff[i] >= 0) buf[loff[i]] = v[i];
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

// init + sum_c q[c] * v[c], accumulated in LT
template <class LT>
__device__ __forceinline__ LT dot8(const LT (&q)[8], const float4& lo, const float4& hi, LT init) {
  LT acc = init;
  acc = fma(q[0], (LT)lo.x, acc); acc = fma(q[1], (LT)lo.y, acc);
  acc = fma(q[2], (LT)lo.z, acc); acc = fma(q[3], (LT)lo.w, acc);
  acc = fma(q[4], (LT)hi.x, acc); acc = fma(q[5], (LT)hi.y, acc);
  acc = fma(q[6], (LT)hi.z, acc); acc = fma(q[7], (LT)hi.w, acc);
  return acc;
}

// acc += a * v, accumulated in AT.  The gradients are sums of k^3 terms of either sign whose magnitude
// follows the upstream gradient; in fp32 the 5-sigma tail of a 55M-element volume collects ~1e-6 of
// rounding, so the accumulators are fp64 as well (same issue rate as fp32 FMAs, one conversion per pair).
template <class AT>
__device__ __forceinline__ void axpy8(AT (&acc)[8], float a, const float4& lo, const float4& hi) {
  const AT aa = (AT)a;
  acc[0] = fma(aa, (AT)lo.x, acc[0]); acc[1] = fma(aa, (AT)lo.y, acc[1]);
  acc[2] = fma(aa, (AT)lo.z, acc[2]); acc[3] = fma(aa, (AT)lo.w, acc[3]);
  acc[4] = fma(aa, (AT)hi.x, acc[4]); acc[5] = fma(aa, (AT)hi.y, acc[5]);
  acc[6] = fma(aa, (AT)hi.z, acc[6]); acc[7] = fma(aa, (AT)hi.w, acc[7]);
}

template <class AT>
__device__ __forceinline__ void store8_scaled(float* o, const AT (&acc)[8], float sc) {
  const AT s = (AT)sc;
  *reinterpret_cast<float4*>(o) = make_float4((float)(acc[0] * s), (float)(acc[1] * s), (float)(acc[2] * s),
                                              (float)(acc[3] * s));
  *reinterpret_cast<float4*>(o + 4) = make_float4((float)(acc[4] * s), (float)(acc[5] * s), (float)(acc[6] * s),
                                                  (float)(acc[7] * s));
}

// ---- forward -----------------------------------------------------------------------------------
template <class LT>
struct QState {
  LT q[8];
  float m;            // running maximum (log2 units)
  LT Z, S0, S1, S2;   // sum of weights and of weight*offset, relative to m
};

template <class LT>
__device__ __forceinline__ void qstate_reset(QState<LT>& s) {
  s.m = -INFINITY; s.Z = (LT)0; s.S0 = (LT)0; s.S1 = (LT)0; s.S2 = (LT)0;
}

// fold NB rows x KW columns of logits (window rows b0.., plane offset a) into the running softmax state.
// The sums run in LT as well: phi feeds the backward pass, where its error is multiplied by the
// upstream gradient, so it has to be good to fp32 rounding rather than to a few 1e-7.
template <int KW, int NB, class LT>
__device__ __forceinline__ void fold(QState<LT>& s, const LT (&l)[NB][KW], int a, int b0) {
  constexpr int R = KW / 2;
  float mx = s.m;
#pragma unroll
  for (int b = 0; b < NB; ++b)
#pragma unroll
    for (int c = 0; c < KW; ++c) mx = fmaxf(mx, (float)l[b][c]);
  const LT alpha = (LT)exp2_fast(s.m - mx);
  LT P = (LT)0, Hs = (LT)0, Ws = (LT)0;
#pragma unroll
  for (int b = 0; b < NB; ++b) {
    LT rs = (LT)0;
#pragma unroll
    for (int c = 0; c < KW; ++c) {
      const LT e = (LT)exp2_fast((float)(l[b][c] - (LT)mx));
      rs += e;
      if (c != R) Ws = fma((LT)(c - R), e, Ws);
    }
    P += rs;
    if (b0 + b != 0) Hs = fma((LT)(b0 + b), rs, Hs);
  }
  s.Z = fma(s.Z, alpha, P);
  s.S0 = a == 0 ? s.S0 * alpha : fma(s.S0, alpha, (LT)a * P);
  s.S1 = fma(s.S1, alpha, Hs);
  s.S2 = fma(s.S2, alpha, Ws);
  s.m = mx;
}

// One K plane against the KW query planes in flight.  Role i (slot (i+PH)%KW) is the query plane
// zq = s - R + i, which sees key plane s under the D offset a = R - i.
template <int KW, int HS, int PH, int NB, class LT>
__device__ __forceinline__ void fwd_step(QState<LT> (&st)[KW], const float4* __restrict__ kb, int lbase,
                                         unsigned active) {
  typedef Patch<KW, HS> P;
  constexpr int R = KW / 2;
  LT l[KW][NB][KW];   // [role][row][col]; only NB rows are live at a time
#pragma unroll
  for (int b = 0; b < KW; ++b) {
#pragma unroll
    for (int c = 0; c < KW; ++c) {
      const int idx = lbase + b * P::PC + c * HS;
      const float4 lo = kb[idx], hi = kb[P::NPOS + idx];
#pragma unroll
      for (int i = 0; i < KW; ++i)
        if (active & (1u << i)) l[i][b % NB][c] = dot8<LT>(st[(i + PH) % KW].q, lo, hi, (LT)0);
    }
    if ((b + 1) % NB == 0) {
#pragma unroll
      for (int i = 0; i < KW; ++i)
        if (active & (1u << i)) fold<KW, NB, LT>(st[(i + PH) % KW], l[i], R - i, b + 1 - NB - R);
    }
  }
}

template <int KW, int HS, class T, class LT, int PH>
__device__ __forceinline__ void fwd_body(QState<LT> (&st)[KW], const TiledParams& p, const Tile& t,
                                         const float4* kb, int lbase, int s, float (&qn)[8], bool have_next) {
  constexpr int R = KW / 2;
  unsigned active = 0;
#pragma unroll
  for (int i = 0; i < KW; ++i) {
    const int zq = s - R + i;
    if (zq >= t.z0 && zq < t.z1) active |= 1u << i;
  }
  fwd_step<KW, HS, PH, (KW == 3 ? 3 : 1), LT>(st, kb, lbase, active);
  QState<LT>& done = st[PH % KW];              // role 0: query plane s - R has now seen all its key planes
  if ((active & 1u) && t.lane_ok) {
    const long long o = t.col + (long long)(s - R) * p.H * p.Wh;
    const LT inv = (LT)1 / done.Z;
    float* ph = p.phi + o * 3;
    ph[0] = (float)(done.S0 * inv); ph[1] = (float)(done.S1 * inv); ph[2] = (float)(done.S2 * inv);
    if (p.lse) p.lse[o] = (done.m + log2_fast((float)done.Z)) * kLn2;
  }
  if (have_next) {                             // the freed slot takes the query plane s + R + 1
#pragma unroll
    for (int c = 0; c < 8; ++c) done.q[c] = (LT)qn[c] * (LT)p.qscale;
    qstate_reset(done);
  }
}

template <int KW, int HS, class T, class LT>
__global__ void __launch_bounds__(NT)
fwd_tiled_kernel(TiledParams p) {
  typedef Patch<KW, HS> P;
  constexpr int R = KW / 2;
  constexpr bool ROT = (KW == 3);
  __shared__ float4 kbuf[2][P::NV];

  const Tile t = make_tile(p);
  const T* Kb = (const T*)p.K + (long long)t.b * p.D * t.plane_elems;
  const T* Qb = (const T*)p.Q + (long long)t.b * p.D * t.plane_elems + ((long long)t.y * p.Wh + t.xs) * 8;
  const int lbase = t.ty * P::PC + t.tx;      // window corner (b = c = -R) of this lane inside the patch

  Stager<KW, HS, T> stg;
  stg.init(threadIdx.x, t.y0, t.xs0, p.H, p.Wh);

  QState<LT> st[KW];
#pragma unroll
  for (int i = 0; i < KW; ++i) {
#pragma unroll
    for (int c = 0; c < 8; ++c) st[i].q[c] = (LT)0;
    qstate_reset(st[i]);
  }
  {
    float q0[8];
    load8<T>(Qb + (long long)t.z0 * t.plane_elems, t.lane_ok, q0);
#pragma unroll
    for (int c = 0; c < 8; ++c) st[KW - 1].q[c] = (LT)q0[c] * (LT)p.qscale;
  }
  const int s_first = t.z0 - R, s_last = t.z1 - 1 + R;
  stg.fetch(s_first >= 0 ? Kb + (long long)s_first * t.plane_elems : nullptr);
  stg.commit(kbuf[0]);
  __syncthreads();

  int ph = 0;
  for (int s = s_first; s <= s_last; ++s) {
    const int cur = (s - s_first) & 1;
    const int sn = s + 1;
    if (sn <= s_last) stg.fetch((sn >= 0 && sn < p.D) ? Kb + (long long)sn * t.plane_elems : nullptr);
    const int zn = s + R + 1;
    const bool have_next = zn < t.z1;
    float qn[8];
    load8<T>(Qb + (long long)zn * t.plane_elems, t.lane_ok && have_next, qn);

    if (ROT) {
      switch (ph) {
        case 0: fwd_body<KW, HS, T, LT, 0>(st, p, t, kbuf[cur], lbase, s, qn, have_next); break;
        case 1: fwd_body<KW, HS, T, LT, 1>(st, p, t, kbuf[cur], lbase, s, qn, have_next); break;
        default: fwd_body<KW, HS, T, LT, 2 % KW>(st, p, t, kbuf[cur], lbase, s, qn, have_next); break;
      }
      ph = ph == KW - 1 ? 0 : ph + 1;
    } else {
      fwd_body<KW, HS, T, LT, 0>(st, p, t, kbuf[cur], lbase, s, qn, have_next);
      // rotate by moving: role i+1 becomes role i, the refilled slot 0 becomes role KW-1
      QState<LT> tmp = st[0];
#pragma unroll
      for (int i = 0; i + 1 < KW; ++i) st[i] = st[i + 1];
      st[KW - 1] = tmp;
    }
    if (sn <= s_last) stg.commit(kbuf[cur ^ 1]);
    __syncthreads();
  }
}

// ---- backward, dQ: lane owns a query column, K planes in LDS -----------------------------------------
template <class LT>
struct DQState {
  LT q[8];          // Q * scale * log2e
  LT nlse;          // -lse * log2e
  float g0, g1, g2, ngphi;
  LT acc[8];        // accumulated in the logit type
};

template <int KW, int HS, int PH, class LT>
__device__ __forceinline__ void dq_step(DQState<LT> (&st)[KW], const float4* __restrict__ kb, int lbase,
                                        unsigned active) {
  typedef Patch<KW, HS> P;
  constexpr int R = KW / 2;
#pragma unroll
  for (int b = 0; b < KW; ++b)
#pragma unroll
    for (int c = 0; c < KW; ++c) {
      const int idx = lbase + b * P::PC + c * HS;
      const float4 lo = kb[idx], hi = kb[P::NPOS + idx];
#pragma unroll
      for (int i = 0; i < KW; ++i)
        if (active & (1u << i)) {
          DQState<LT>& s = st[(i + PH) % KW];
          const float w = exp2_fast((float)dot8<LT>(s.q, lo, hi, s.nlse));
          // t = g.o - g.phi with o = (R - i, b - R, c - R)
          float tt = s.ngphi;
          if (R - i != 0) tt = fmaf((float)(R - i), s.g0, tt);
          if (b - R != 0) tt = fmaf((float)(b - R), s.g1, tt);
          if (c - R != 0) tt = fmaf((float)(c - R), s.g2, tt);
          axpy8<LT>(s.acc, w * tt, lo, hi);
        }
    }
}

struct QueryAux { float q[8]; float lse, g0, g1, g2, f0, f1, f2; };

template <class T>
__device__ __forceinline__ void load_query_aux(const TiledParams& p, const T* qptr, long long w, bool ok,
                                               QueryAux& a) {
  load8<T>(qptr, ok, a.q);
  if (ok) {
    a.lse = p.lse_in[w];
    const float* g = p.dphi + w * 3;
    const float* f = p.phi_in + w * 3;
    a.g0 = g[0]; a.g1 = g[1]; a.g2 = g[2]; a.f0 = f[0]; a.f1 = f[1]; a.f2 = f[2];
  } else {
    a.lse = a.g0 = a.g1 = a.g2 = a.f0 = a.f1 = a.f2 = 0.f;
  }
}

template <class LT>
__device__ __forceinline__ void dq_refill(DQState<LT>& s, const QueryAux& a, float qscale) {
#pragma unroll
  for (int c = 0; c < 8; ++c) { s.q[c] = (LT)a.q[c] * (LT)qscale; s.acc[c] = (LT)0; }
  s.nlse = -(LT)a.lse * (LT)kLog2e;
  s.g0 = a.g0; s.g1 = a.g1; s.g2 = a.g2;
  s.ngphi = -(a.g0 * a.f0 + a.g1 * a.f1 + a.g2 * a.f2);
}

template <int KW, int HS, class T, class LT, int PH>
__device__ __forceinline__ void dq_body(DQState<LT> (&st)[KW], const TiledParams& p, const Tile& t,
                                        const float4* kb, int lbase, int s, const QueryAux& nx, bool have_next) {
  constexpr int R = KW / 2;
  unsigned active = 0;
#pragma unroll
  for (int i = 0; i < KW; ++i) {
    const int zq = s - R + i;
    if (zq >= t.z0 && zq < t.z1) active |= 1u << i;
  }
  dq_step<KW, HS, PH, LT>(st, kb, lbase, active);
  DQState<LT>& done = st[PH % KW];
  if ((active & 1u) && t.lane_ok) {
    store8_scaled<LT>(p.out + (t.col + (long long)(s - R) * p.H * p.Wh) * 8, done.acc, p.scale);
  }
  if (have_next) dq_refill<LT>(done, nx, p.qscale);
}

template <int KW, int HS, class T, class LT>
__global__ void __launch_bounds__(NT)
dq_tiled_kernel(TiledParams p) {
  typedef Patch<KW, HS> P;
  constexpr int R = KW / 2;
  constexpr bool ROT = (KW == 3);
  __shared__ float4 kbuf[2][P::NV];

  const Tile t = make_tile(p);
  const T* Kb = (const T*)p.K + (long long)t.b * p.D * t.plane_elems;
  const T* Qb = (const T*)p.Q + (long long)t.b * p.D * t.plane_elems + ((long long)t.y * p.Wh + t.xs) * 8;
  const long long pw = (long long)p.H * p.Wh;
  const int lbase = t.ty * P::PC + t.tx;

  Stager<KW, HS, T> stg;
  stg.init(threadIdx.x, t.y0, t.xs0, p.H, p.Wh);

  DQState<LT> st[KW];
  {
    QueryAux zero;
    load_query_aux<T>(p, Qb, 0, false, zero);
#pragma unroll
    for (int i = 0; i < KW; ++i) dq_refill<LT>(st[i], zero, p.qscale);
    QueryAux a0;
    load_query_aux<T>(p, Qb + (long long)t.z0 * t.plane_elems, t.col + t.z0 * pw, t.lane_ok, a0);
    dq_refill<LT>(st[KW - 1], a0, p.qscale);
  }
  const int s_first = t.z0 - R, s_last = t.z1 - 1 + R;
  stg.fetch(s_first >= 0 ? Kb + (long long)s_first * t.plane_elems : nullptr);
  stg.commit(kbuf[0]);
  __syncthreads();

  int ph = 0;
  for (int s = s_first; s <= s_last; ++s) {
    const int cur = (s - s_first) & 1;
    const int sn = s + 1;
    if (sn <= s_last) stg.fetch((sn >= 0 && sn < p.D) ? Kb + (long long)sn * t.plane_elems : nullptr);
    const int zn = s + R + 1;
    const bool have_next = zn < t.z1;
    QueryAux nx;
    load_query_aux<T>(p, Qb + (long long)zn * t.plane_elems, t.col + zn * pw, t.lane_ok && have_next, nx);

    if (ROT) {
      switch (ph) {
        case 0: dq_body<KW, HS, T, LT, 0>(st, p, t, kbuf[cur], lbase, s, nx, have_next); break;
        case 1: dq_body<KW, HS, T, LT, 1>(st, p, t, kbuf[cur], lbase, s, nx, have_next); break;
        default: dq_body<KW, HS, T, LT, 2 % KW>(st, p, t, kbuf[cur], lbase, s, nx, have_next); break;
      }
      ph = ph == KW - 1 ? 0 : ph + 1;
    } else {
      dq_body<KW, HS, T, LT, 0>(st, p, t, kbuf[cur], lbase, s, nx, have_next);
      DQState<LT> tmp = st[0];
#pragma unroll
      for (int i = 0; i + 1 < KW; ++i) st[i] = st[i + 1];
      st[KW - 1] = tmp;
    }
    if (sn <= s_last) stg.commit(kbuf[cur ^ 1]);
    __syncthreads();
  }
}

// ---- backward, dK: lane owns a key column; Q planes + per-query statistics in LDS --------------------
template <class LT>
struct DKState {
  LT k[8];
  LT acc[8];
};

// One query plane s against the KW key planes in flight.  Role i is the key plane zk = s - R + i, which
// the queries of plane s see under the D offset a = i - R.  The query at patch position (row, col) =
// (ty + r, tx + cc*HS) sees this lane's key under the in-plane offset (b, c) = (R - r, R - cc).
template <int KW, int HS, int PH, class LT>
__device__ __forceinline__ void dk_step(DKState<LT> (&st)[KW], const float4* __restrict__ qb,
                                        const float4* __restrict__ sa, const float* __restrict__ sc, int lbase,
                                        unsigned active) {
  typedef Patch<KW, HS> P;
  constexpr int R = KW / 2;
#pragma unroll
  for (int r = 0; r < KW; ++r)
#pragma unroll
    for (int cc = 0; cc < KW; ++cc) {
      const int idx = lbase + r * P::PC + cc * HS;
      const float4 lo = qb[idx], hi = qb[P::NPOS + idx];
      const float4 a4 = sa[idx];     // (-lse*log2e, g_D, g_H, g_W) of that query
      float tb = sc[idx];            // -g.phi
      if (R - r != 0) tb = fmaf((float)(R - r), a4.z, tb);
      if (R - cc != 0) tb = fmaf((float)(R - cc), a4.w, tb);
#pragma unroll
      for (int i = 0; i < KW; ++i)
        if (active & (1u << i)) {
          DKState<LT>& s = st[(i + PH) % KW];
          const float w = exp2_fast((float)dot8<LT>(s.k, lo, hi, (LT)a4.x));
          const float tt = (i - R != 0) ? fmaf((float)(i - R), a4.y, tb) : tb;
          axpy8<LT>(s.acc, w * tt, lo, hi);
        }
    }
}

template <int KW, int HS, class T, class LT, int PH>
__device__ __forceinline__ void dk_body(DKState<LT> (&st)[KW], const TiledParams& p, const Tile& t,
                                        const float4* qb, const float4* sa, const float* sc, int lbase, int s,
                                        const float (&kn)[8], bool have_next) {
  constexpr int R = KW / 2;
  unsigned active = 0;
#pragma unroll
  for (int i = 0; i < KW; ++i) {
    const int zk = s - R + i;
    if (zk >= t.z0 && zk < t.z1) active |= 1u << i;
  }
  dk_step<KW, HS, PH, LT>(st, qb, sa, sc, lbase, active);
  DKState<LT>& done = st[PH % KW];
  if ((active & 1u) && t.lane_ok) {
    store8_scaled<LT>(p.out + (t.col + (long long)(s - R) * p.H * p.Wh) * 8, done.acc, p.scale);
  }
  if (have_next) {     // the in-flight copy of K carries the factor scale*log2e (applied in LT precision)
#pragma unroll
    for (int c = 0; c < 8; ++c) { done.k[c] = (LT)kn[c] * (LT)p.qscale; done.acc[c] = (LT)0; }
  }
}

template <int KW, int HS, class T, class LT>
__global__ void __launch_bounds__(NT)
dk_tiled_kernel(TiledParams p) {
  typedef Patch<KW, HS> P;
  constexpr int R = KW / 2;
  constexpr bool ROT = (KW == 3);
  __shared__ float4 qbuf[2][P::NV];
  __shared__ float4 sabuf[2][P::NPOS];
  __shared__ float scbuf[2][P::NPOS];

  const Tile t = make_tile(p);
  const T* Qb = (const T*)p.Q + (long long)t.b * p.D * t.plane_elems;
  const T* Kb = (const T*)p.K + (long long)t.b * p.D * t.plane_elems + ((long long)t.y * p.Wh + t.xs) * 8;
  const long long pw = (long long)p.H * p.Wh;
  const long long wb = (long long)t.b * p.D * pw;    // window index of (b, 0, 0, 0)
  const int lbase = t.ty * P::PC + t.tx;

  Stager<KW, HS, T> stg;
  stg.init(threadIdx.x, t.y0, t.xs0, p.H, p.Wh);
  StatStager<KW, HS> sst;
  sst.init(threadIdx.x, t.y0, t.xs0, p.H, p.Wh);

  DKState<LT> st[KW];
#pragma unroll
  for (int i = 0; i < KW; ++i)
#pragma unroll
    for (int c = 0; c < 8; ++c) { st[i].k[c] = (LT)0; st[i].acc[c] = (LT)0; }
  {
    float k0[8];
    load8<T>(Kb + (long long)t.z0 * t.plane_elems, t.lane_ok, k0);
#pragma unroll
    for (int c = 0; c < 8; ++c) st[KW - 1].k[c] = (LT)k0[c] * (LT)p.qscale;
  }
  const int s_first = t.z0 - R, s_last = t.z1 - 1 + R;
  {
    const bool ok = s_first >= 0;
    stg.fetch(ok ? Qb + (long long)s_first * t.plane_elems : nullptr);
    sst.fetch(p, wb + (long long)s_first * pw, ok);
    stg.commit(qbuf[0]);
    sst.commit(sabuf[0], scbuf[0]);
  }
  __syncthreads();

  int ph = 0;
  for (int s = s_first; s <= s_last; ++s) {
    const int cur = (s - s_first) & 1;
    const int sn = s + 1;
    if (sn <= s_last) {
      const bool ok = sn >= 0 && sn < p.D;
      stg.fetch(ok ? Qb + (long long)sn * t.plane_elems : nullptr);
      sst.fetch(p, wb + (long long)sn * pw, ok);
    }
    const int zn = s + R + 1;
    const bool have_next = zn < t.z1;
    float kn[8];
    load8<T>(Kb + (long long)zn * t.plane_elems, t.lane_ok && have_next, kn);

    if (ROT) {
      switch (ph) {
        case 0: dk_body<KW, HS, T, LT, 0>(st, p, t, qbuf[cur], sabuf[cur], scbuf[cur], lbase, s, kn, have_next); break;
        case 1: dk_body<KW, HS, T, LT, 1>(st, p, t, qbuf[cur], sabuf[cur], scbuf[cur], lbase, s, kn, have_next); break;
        default: dk_body<KW, HS, T, LT, 2 % KW>(st, p, t, qbuf[cur], sabuf[cur], scbuf[cur], lbase, s, kn, have_next); break;
      }
      ph = ph == KW - 1 ? 0 : ph + 1;
    } else {
      dk_body<KW, HS, T, LT, 0>(st, p, t, qbuf[cur], sabuf[cur], scbuf[cur], lbase, s, kn, have_next);
      DKState<LT> tmp = st[0];
#pragma unroll
      for (int i = 0; i + 1 < KW; ++i) st[i] = st[i + 1];
      st[KW - 1] = tmp;
    }
    if (sn <= s_last) {
      stg.commit(qbuf[cur ^ 1]);
      sst.commit(sabuf[cur ^ 1], scbuf[cur ^ 1]);
    }
    __syncthreads();
  }
}

// ---- launch ------------------------------------------------------------------------------------------
#ifndef MODET_LOGIT_T
#define MODET_LOGIT_T double
#endif
typedef MODET_LOGIT_T logit_t;    // accumulation type of the logits (see the note at the top of the file)

TiledParams make_params(const Geo& g) {
  TiledParams p = {};
  p.B = g.B; p.D = g.D; p.H = g.H; p.Wh = g.W * g.heads;
  p.ntx = (p.Wh + TX - 1) / TX;
  p.nty = (g.H + TY - 1) / TY;
  // enough chunks along D to give every CU several workgroups, but not so short that the
  // k-1 extra planes per chunk dominate
  const long long tiles = (long long)p.ntx * p.nty * g.B;
  int zc = 16;
  while (zc > 4 && tiles * ((g.D + zc - 1) / zc) < 2048) zc >>= 1;
  if (zc > g.D) zc = g.D;
  p.ZC = zc;
  p.nzc = (g.D + zc - 1) / zc;
  p.scale = g.scale;
  p.qscale = g.scale * kLog2e;
  return p;
}

inline unsigned nblocks(const TiledParams& p) { return (unsigned)((long long)p.ntx * p.nty * p.B * p.nzc); }

template <int KW, int HS, class T>
hipError_t launch_fwd_t(const Geo& g, const void* Q, const void* K, float* phi, float* lse, hipStream_t st) {
  TiledParams p = make_params(g);
  p.Q = Q; p.K = K; p.phi = phi; p.lse = lse;
  hipLaunchKernelGGL((fwd_tiled_kernel<KW, HS, T, logit_t>), dim3(nblocks(p)), dim3(NT), 0, st, p);
  return hipGetLastError();
}

template <int KW, int HS, class T>
hipError_t launch_bwd_t(const Geo& g, const void* Q, const void* K, const float* dphi, const float* phi,
                        const float* lse, float* dQ, float* dK, hipStream_t st) {
  TiledParams p = make_params(g);
  p.Q = Q; p.K = K; p.dphi = dphi; p.phi_in = phi; p.lse_in = lse;
  p.out = dQ;
  hipLaunchKernelGGL((dq_tiled_kernel<KW, HS, T, logit_t>), dim3(nblocks(p)), dim3(NT), 0, st, p);
  p.out = dK;
  hipLaunchKernelGGL((dk_tiled_kernel<KW, HS, T, logit_t>), dim3(nblocks(p)), dim3(NT), 0, st, p);
  return hipGetLastError();
}

}  // namespace

bool tiled_fwd_supported(int d, int heads, int k, int dtype, bool has_bias) {
  if (d != 8 || has_bias) return false;
  if (k == 3) return dtype == 0 && (heads == 1 || heads == 2 || heads == 4 || heads == 8);
  return false;
}

bool tiled_bwd_supported(int d, int heads, int k, int dtype, bool has_bias) {
  return tiled_fwd_supported(d, heads, k, dtype, has_bias);
}

hipError_t launch_fwd_tiled(const Geo& g, int dtype, const void* Q, const void* K, const float* bias,
                            float* phi, float* lse, hipStream_t st) {
  (void)bias; (void)dtype;
  switch (g.heads) {
    case 1: return launch_fwd_t<3, 1, float>(g, Q, K, phi, lse, st);
    case 2: return launch_fwd_t<3, 2, float>(g, Q, K, phi, lse, st);
    case 4: return launch_fwd_t<3, 4, float>(g, Q, K, phi, lse, st);
    case 8: return launch_fwd_t<3, 8, float>(g, Q, K, phi, lse, st);
    default: return hipErrorNotSupported;
  }
}

hipError_t launch_bwd_tiled(const Geo& g, int dtype, const void* Q, const void* K, const float* bias,
                            const float* dphi, const float* phi, const float* lse, float* dQ, float* dK,
                            hipStream_t st) {
  (void)bias; (void)dtype;
  switch (g.heads) {
    case 1: return launch_bwd_t<3, 1, float>(g, Q, K, dphi, phi, lse, dQ, dK, st);
    case 2: return launch_bwd_t<3, 2, float>(g, Q, K, dphi, phi, lse, dQ, dK, st);
    case 4: return launch_bwd_t<3, 4, float>(g, Q, K, dphi, phi, lse, dQ, dK, st);
    case 8: return launch_bwd_t<3, 8, float>(g, Q, K, dphi, phi, lse, dQ, dK, st);
    default: return hipErrorNotSupported;
  }
}

}  // namespace modet
