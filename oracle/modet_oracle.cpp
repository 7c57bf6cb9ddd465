// CPU oracle for the ModeT motion-decomposition operator.
//
// TEST INFRASTRUCTURE ONLY.  Plain, slow, fp64 loops written from the paper's definition:
// windowed scores and softmax (Section 3.3.1, Eq. 3), the attention-weighted sum of the
// integer offset grid V (Eq. 4-5), the derivatives of those two equations with respect to
// Q and K (and the bias B), and the trilinear feature warp / 2x field upsampling used
// between pyramid levels (Section 3.1).  It shares no code with the GPU library and is
// called only by the tests, by the smoke check and by the benchmark's CPU-baseline leg.
//
// Layout: Q, K, src, out are [B, D, H, W, C] (channels last, head s owns channels
// [s*d, (s+1)*d) with d = C / heads); phi, dphi are [B, D, H, W, heads, 3] with component
// order (D, H, W); attn is [B, D, H, W, heads, k^3]; bias is [heads, k^3]; window offsets
// are enumerated row-major with the D offset slowest: j = ((a+r)*k + (b+r))*k + (c+r).
//
// Readings of the paper that are built in here:
//  * the moving (key) map is zero padded and a padded neighbour still takes part in the
//    softmax with logit 0 (+ bias)  (Section 3.3.1, sentence after Eq. 3);
//  * V_x = x - x_c, i.e. integer offsets -r..r per axis, r = (k-1)/2  (text after Eq. 4);
//  * Eq. 3 prints no scale; `scale` multiplies the dot product (scale = 1 is Eq. 3 as
//    printed, 1/sqrt(d) is the usual attention scaling).
//
// All inputs are widened exactly to double; every sum, exp and division is done in double.

#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>
#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

enum { IN_F32 = 0, IN_BF16 = 1, IN_F64 = 2 };

struct Geo {
  int B, D, H, W, C, heads, k, r, d, k3;
};

Geo make_geo(int B, int D, int H, int W, int C, int heads, int k) {
  Geo g;
  g.B = B; g.D = D; g.H = H; g.W = W; g.C = C; g.heads = heads; g.k = k;
  g.r = (k - 1) / 2; g.d = C / heads; g.k3 = k * k * k;
  return g;
}

inline double widen(float v) { return (double)v; }
inline double widen(double v) { return v; }
struct bf16 { uint16_t bits; };
inline double widen(bf16 v) {
  uint32_t u = (uint32_t)v.bits << 16;
  float f;
  std::memcpy(&f, &u, sizeof f);
  return (double)f;
}

inline int64_t vox(const Geo& g, int b, int z, int y, int x) {
  return (((int64_t)b * g.D + z) * g.H + y) * g.W + x;
}
inline bool inside(const Geo& g, int z, int y, int x) {
  return z >= 0 && z < g.D && y >= 0 && y < g.H && x >= 0 && x < g.W;
}

// Eq. 3, the argument of the softmax: l[j] for the k^3 neighbours of voxel (b,z,y,x), head s.
template <class T>
void logits(const Geo& g, const T* Q, const T* K, const double* bias, double scale,
            int b, int z, int y, int x, int s, double* l) {
  const T* q = Q + vox(g, b, z, y, x) * g.C + s * g.d;
  int j = 0;
  for (int a = -g.r; a <= g.r; ++a)
    for (int bb = -g.r; bb <= g.r; ++bb)
      for (int c = -g.r; c <= g.r; ++c, ++j) {
        double v = bias ? bias[s * g.k3 + j] : 0.0;
        if (inside(g, z + a, y + bb, x + c)) {
          const T* kk = K + vox(g, b, z + a, y + bb, x + c) * g.C + s * g.d;
          double dot = 0.0;
          for (int ch = 0; ch < g.d; ++ch) dot += widen(q[ch]) * widen(kk[ch]);
          v += scale * dot;
        }
        l[j] = v;
      }
}

// softmax over n values; returns log(sum(exp(l))).
double softmax(const double* l, int n, double* w) {
  double m = l[0];
  for (int j = 1; j < n; ++j) m = l[j] > m ? l[j] : m;
  double Z = 0.0;
  for (int j = 0; j < n; ++j) { w[j] = std::exp(l[j] - m); Z += w[j]; }
  for (int j = 0; j < n; ++j) w[j] /= Z;
  return m + std::log(Z);
}

// Eq. 4: phi = sum_j w[j] * V[j],  V[j] = (a, b, c).
void weighted_offsets(const Geo& g, const double* w, double* phi) {
  phi[0] = phi[1] = phi[2] = 0.0;
  int j = 0;
  for (int a = -g.r; a <= g.r; ++a)
    for (int bb = -g.r; bb <= g.r; ++bb)
      for (int c = -g.r; c <= g.r; ++c, ++j) {
        phi[0] += w[j] * a; phi[1] += w[j] * bb; phi[2] += w[j] * c;
      }
}

// derivative of L = sum g.phi (+ sum da.w when the attention weights of Eq. 3 are an output with upstream
// gradient da) with respect to the logits of one window: the softmax Jacobian applied to
// t[j] = g.V[j] (+ da[j]):  dl[j] = w[j] * (t[j] - sum_i w[i] t[i]),  and sum_i w[i] g.V[i] = g.phi.
void dlogits(const Geo& g, const double* w, const double* phi, const double* gr, const double* da, double* dl) {
  double mean = gr[0] * phi[0] + gr[1] * phi[1] + gr[2] * phi[2];
  if (da)
    for (int j = 0; j < g.k3; ++j) mean += w[j] * da[j];
  int j = 0;
  for (int a = -g.r; a <= g.r; ++a)
    for (int bb = -g.r; bb <= g.r; ++bb)
      for (int c = -g.r; c <= g.r; ++c, ++j) {
        double t = gr[0] * a + gr[1] * bb + gr[2] * c + (da ? da[j] : 0.0);
        dl[j] = w[j] * (t - mean);
      }
}

template <class T>
void fwd_impl(const Geo& g, const T* Q, const T* K, const double* bias, double scale,
              double* phi, double* attn, double* lse) {
#pragma omp parallel
  {
    std::vector<double> l(g.k3), w(g.k3);
#pragma omp for collapse(2) schedule(static)
    for (int b = 0; b < g.B; ++b)
      for (int z = 0; z < g.D; ++z)
        for (int y = 0; y < g.H; ++y)
          for (int x = 0; x < g.W; ++x)
            for (int s = 0; s < g.heads; ++s) {
              int64_t vn = vox(g, b, z, y, x) * g.heads + s;
              logits(g, Q, K, bias, scale, b, z, y, x, s, l.data());
              double ls = softmax(l.data(), g.k3, w.data());
              weighted_offsets(g, w.data(), phi + vn * 3);
              if (attn) std::memcpy(attn + vn * g.k3, w.data(), sizeof(double) * g.k3);
              if (lse) lse[vn] = ls;
            }
  }
}

// literal, serial: every (query, neighbour) pair adds into dQ[query] and dK[neighbour].
template <class T>
void bwd_scatter_impl(const Geo& g, const T* Q, const T* K, const double* bias, double scale,
                      const double* dphi, const double* dattn, double* dQ, double* dK, double* dbias) {
  int64_t n = (int64_t)g.B * g.D * g.H * g.W * g.C;
  for (int64_t i = 0; i < n; ++i) dQ[i] = dK[i] = 0.0;
  if (dbias) for (int i = 0; i < g.heads * g.k3; ++i) dbias[i] = 0.0;
  std::vector<double> l(g.k3), w(g.k3), dl(g.k3);
  for (int b = 0; b < g.B; ++b)
    for (int z = 0; z < g.D; ++z)
      for (int y = 0; y < g.H; ++y)
        for (int x = 0; x < g.W; ++x)
          for (int s = 0; s < g.heads; ++s) {
            int64_t p = vox(g, b, z, y, x);
            double phi[3];
            logits(g, Q, K, bias, scale, b, z, y, x, s, l.data());
            softmax(l.data(), g.k3, w.data());
            weighted_offsets(g, w.data(), phi);
            dlogits(g, w.data(), phi, dphi + (p * g.heads + s) * 3,
                    dattn ? dattn + (p * g.heads + s) * g.k3 : nullptr, dl.data());
            int j = 0;
            for (int a = -g.r; a <= g.r; ++a)
              for (int bb = -g.r; bb <= g.r; ++bb)
                for (int c = -g.r; c <= g.r; ++c, ++j) {
                  if (dbias) dbias[s * g.k3 + j] += dl[j];
                  if (!inside(g, z + a, y + bb, x + c)) continue;   // padding has no gradient
                  int64_t q = vox(g, b, z + a, y + bb, x + c);
                  for (int ch = 0; ch < g.d; ++ch) {
                    int64_t ip = p * g.C + s * g.d + ch, iq = q * g.C + s * g.d + ch;
                    dQ[ip] += scale * dl[j] * widen(K[iq]);
                    dK[iq] += scale * dl[j] * widen(Q[ip]);
                  }
                }
          }
}

// second derivation: first dl for every window, then each output element collects its terms.
template <class T>
void bwd_gather_impl(const Geo& g, const T* Q, const T* K, const double* bias, double scale,
                     const double* dphi, const double* dattn, double* dQ, double* dK) {
  int64_t nvn = (int64_t)g.B * g.D * g.H * g.W * g.heads;
  std::vector<double> DL((size_t)nvn * g.k3);
#pragma omp parallel
  {
    std::vector<double> l(g.k3), w(g.k3);
#pragma omp for collapse(2) schedule(static)
    for (int b = 0; b < g.B; ++b)
      for (int z = 0; z < g.D; ++z)
        for (int y = 0; y < g.H; ++y)
          for (int x = 0; x < g.W; ++x)
            for (int s = 0; s < g.heads; ++s) {
              int64_t vn = vox(g, b, z, y, x) * g.heads + s;
              double phi[3];
              logits(g, Q, K, bias, scale, b, z, y, x, s, l.data());
              softmax(l.data(), g.k3, w.data());
              weighted_offsets(g, w.data(), phi);
              dlogits(g, w.data(), phi, dphi + vn * 3, dattn ? dattn + vn * g.k3 : nullptr, DL.data() + vn * g.k3);
            }
#pragma omp for collapse(2) schedule(static)
    for (int b = 0; b < g.B; ++b)
      for (int z = 0; z < g.D; ++z)
        for (int y = 0; y < g.H; ++y)
          for (int x = 0; x < g.W; ++x)
            for (int s = 0; s < g.heads; ++s) {
              int64_t p = vox(g, b, z, y, x);
              for (int ch = 0; ch < g.d; ++ch) {
                double aq = 0.0, ak = 0.0;
                int j = 0;
                for (int a = -g.r; a <= g.r; ++a)
                  for (int bb = -g.r; bb <= g.r; ++bb)
                    for (int c = -g.r; c <= g.r; ++c, ++j) {
                      // dQ[p]: neighbour p + o
                      if (inside(g, z + a, y + bb, x + c))
                        aq += DL[(size_t)(p * g.heads + s) * g.k3 + j] *
                              widen(K[vox(g, b, z + a, y + bb, x + c) * g.C + s * g.d + ch]);
                      // dK[p]: the query p - o sees this key under offset o
                      if (inside(g, z - a, y - bb, x - c)) {
                        int64_t qv = vox(g, b, z - a, y - bb, x - c);
                        ak += DL[(size_t)(qv * g.heads + s) * g.k3 + j] * widen(Q[qv * g.C + s * g.d + ch]);
                      }
                    }
                dQ[p * g.C + s * g.d + ch] = scale * aq;
                dK[p * g.C + s * g.d + ch] = scale * ak;
              }
            }
  }
}

void decode_vn(const Geo& g, int64_t vn, int& b, int& z, int& y, int& x, int& s) {
  s = (int)(vn % g.heads); vn /= g.heads;
  x = (int)(vn % g.W); vn /= g.W;
  y = (int)(vn % g.H); vn /= g.H;
  z = (int)(vn % g.D); vn /= g.D;
  b = (int)vn;
}

template <class T>
void fwd_at_impl(const Geo& g, const T* Q, const T* K, const double* bias, double scale,
                 int64_t n, const int64_t* idx, double* phi, double* lse) {
#pragma omp parallel
  {
    std::vector<double> l(g.k3), w(g.k3);
#pragma omp for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
      int b, z, y, x, s;
      decode_vn(g, idx[i], b, z, y, x, s);
      logits(g, Q, K, bias, scale, b, z, y, x, s, l.data());
      double ls = softmax(l.data(), g.k3, w.data());
      weighted_offsets(g, w.data(), phi + i * 3);
      if (lse) lse[i] = ls;
    }
  }
}

// dQ and dK for the d channels of head s at the sampled voxels idx[i] (voxel*heads + s).
template <class T>
void bwd_at_impl(const Geo& g, const T* Q, const T* K, const double* bias, double scale,
                 const double* dphi, int64_t n, const int64_t* idx, double* dQ, double* dK) {
#pragma omp parallel
  {
    std::vector<double> l(g.k3), w(g.k3), dl(g.k3);
#pragma omp for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
      int b, z, y, x, s;
      decode_vn(g, idx[i], b, z, y, x, s);
      double phi[3];
      // dQ at (b,z,y,x,s): its own window
      logits(g, Q, K, bias, scale, b, z, y, x, s, l.data());
      softmax(l.data(), g.k3, w.data());
      weighted_offsets(g, w.data(), phi);
      dlogits(g, w.data(), phi, dphi + idx[i] * 3, nullptr, dl.data());
      for (int ch = 0; ch < g.d; ++ch) dQ[i * g.d + ch] = dK[i * g.d + ch] = 0.0;
      int j = 0;
      for (int a = -g.r; a <= g.r; ++a)
        for (int bb = -g.r; bb <= g.r; ++bb)
          for (int c = -g.r; c <= g.r; ++c, ++j)
            if (inside(g, z + a, y + bb, x + c))
              for (int ch = 0; ch < g.d; ++ch)
                dQ[i * g.d + ch] += scale * dl[j] * widen(K[vox(g, b, z + a, y + bb, x + c) * g.C + s * g.d + ch]);
      // dK at (b,z,y,x,s): every query p = q - o that has this key in its window
      j = 0;
      for (int a = -g.r; a <= g.r; ++a)
        for (int bb = -g.r; bb <= g.r; ++bb)
          for (int c = -g.r; c <= g.r; ++c, ++j) {
            int pz = z - a, py = y - bb, px = x - c;
            if (!inside(g, pz, py, px)) continue;
            int64_t pv = vox(g, b, pz, py, px);
            logits(g, Q, K, bias, scale, b, pz, py, px, s, l.data());
            softmax(l.data(), g.k3, w.data());
            weighted_offsets(g, w.data(), phi);
            dlogits(g, w.data(), phi, dphi + (pv * g.heads + s) * 3, nullptr, dl.data());
            for (int ch = 0; ch < g.d; ++ch)
              dK[i * g.d + ch] += scale * dl[j] * widen(Q[pv * g.C + s * g.d + ch]);
          }
    }
  }
}

// trilinear sample of a [D,H,W,C] volume (one batch item) at real coordinates, zero outside.
template <class T>
void sample_zero(const T* vol, int D, int H, int W, int C, double cz, double cy, double cx, double* out) {
  double fz = std::floor(cz), fy = std::floor(cy), fx = std::floor(cx);
  double tz = cz - fz, ty = cy - fy, tx = cx - fx;
  for (int c = 0; c < C; ++c) out[c] = 0.0;
  for (int dz = 0; dz < 2; ++dz)
    for (int dy = 0; dy < 2; ++dy)
      for (int dx = 0; dx < 2; ++dx) {
        double z = fz + dz, y = fy + dy, x = fx + dx;
        if (z < 0 || z > D - 1 || y < 0 || y > H - 1 || x < 0 || x > W - 1) continue;
        double wgt = (dz ? tz : 1.0 - tz) * (dy ? ty : 1.0 - ty) * (dx ? tx : 1.0 - tx);
        const T* v = vol + (((int64_t)z * H + (int64_t)y) * W + (int64_t)x) * C;
        for (int c = 0; c < C; ++c) out[c] += wgt * widen(v[c]);
      }
}

inline double clampd(double v, double lo, double hi) { return v < lo ? lo : (v > hi ? hi : v); }

// displacement (fine-grid voxel units) at fine voxel (z,y,x) from a half-resolution field:
// the coarse voxel i covers fine voxels 2i and 2i+1 (2x average pooling geometry), so the fine
// centre z sits at coarse coordinate (z + 0.5)/2 - 0.5, clamped to the coarse grid; values x2.
void upsampled_disp(const float* fc, int Dc, int Hc, int Wc, int z, int y, int x, double* u) {
  double cz = clampd((z + 0.5) / 2.0 - 0.5, 0.0, Dc - 1.0);
  double cy = clampd((y + 0.5) / 2.0 - 0.5, 0.0, Hc - 1.0);
  double cx = clampd((x + 0.5) / 2.0 - 0.5, 0.0, Wc - 1.0);
  sample_zero(fc, Dc, Hc, Wc, 3, cz, cy, cx, u);
  u[0] *= 2.0; u[1] *= 2.0; u[2] *= 2.0;
}

template <class T>
void warp_impl(const T* src, const float* field, int B, int D, int H, int W, int C, int half, double* out) {
  int Dc = D / 2, Hc = H / 2, Wc = W / 2;
#pragma omp parallel for collapse(2) schedule(static)
  for (int b = 0; b < B; ++b)
    for (int z = 0; z < D; ++z)
      for (int y = 0; y < H; ++y)
        for (int x = 0; x < W; ++x) {
          double u[3];
          int64_t p = (((int64_t)b * D + z) * H + y) * W + x;
          if (half) {
            upsampled_disp(field + (int64_t)b * Dc * Hc * Wc * 3, Dc, Hc, Wc, z, y, x, u);
          } else {
            for (int a = 0; a < 3; ++a) u[a] = (double)field[p * 3 + a];
          }
          sample_zero(src + (int64_t)b * D * H * W * C, D, H, W, C, z + u[0], y + u[1], x + u[2], out + p * C);
        }
}

// Adjoint of the warp (derivative of L = sum(dout * warp(src, field)) with respect to src and to the field),
// written as the transpose of sample_zero: every output voxel hands dout back to the corners it read, with
// the weights it read them with; the derivative with respect to a displacement component differentiates
// the weights (d/dt of t is +1 on the upper corner, of 1-t is -1 on the lower one).  A half-resolution field
// receives the gradient of the displacement it was upsampled to, through the upsampling weights (x2).
template <class T>
void warp_bwd_impl(const T* src, const float* field, const double* dout, int B, int D, int H, int W, int C,
                   int half, double* dsrc, double* dfield) {
  int Dc = D / 2, Hc = H / 2, Wc = W / 2;
  for (int64_t i = 0; i < (int64_t)B * D * H * W * C; ++i) dsrc[i] = 0.0;
  if (dfield) {
    int64_t n = half ? (int64_t)B * Dc * Hc * Wc * 3 : (int64_t)B * D * H * W * 3;
    for (int64_t i = 0; i < n; ++i) dfield[i] = 0.0;
  }
  for (int b = 0; b < B; ++b)
    for (int z = 0; z < D; ++z)
      for (int y = 0; y < H; ++y)
        for (int x = 0; x < W; ++x) {
          double u[3];
          int64_t p = (((int64_t)b * D + z) * H + y) * W + x;
          const float* fc = field + (int64_t)b * Dc * Hc * Wc * 3;
          if (half) upsampled_disp(fc, Dc, Hc, Wc, z, y, x, u);
          else for (int a = 0; a < 3; ++a) u[a] = (double)field[p * 3 + a];
          double cz = z + u[0], cy = y + u[1], cx = x + u[2];
          double fz = std::floor(cz), fy = std::floor(cy), fx = std::floor(cx);
          double tz = cz - fz, ty = cy - fy, tx = cx - fx;
          double du[3] = {0.0, 0.0, 0.0};
          const T* sb = src + (int64_t)b * D * H * W * C;
          double* db = dsrc + (int64_t)b * D * H * W * C;
          for (int dz = 0; dz < 2; ++dz)
            for (int dy = 0; dy < 2; ++dy)
              for (int dx = 0; dx < 2; ++dx) {
                double zz = fz + dz, yy = fy + dy, xx = fx + dx;
                if (zz < 0 || zz > D - 1 || yy < 0 || yy > H - 1 || xx < 0 || xx > W - 1) continue;
                double wz = dz ? tz : 1.0 - tz, wy = dy ? ty : 1.0 - ty, wx = dx ? tx : 1.0 - tx;
                int64_t q = (((int64_t)zz * H + (int64_t)yy) * W + (int64_t)xx) * C;
                double dot = 0.0;
                for (int c = 0; c < C; ++c) {
                  db[q + c] += wz * wy * wx * dout[p * C + c];
                  dot += dout[p * C + c] * widen(sb[q + c]);
                }
                du[0] += (dz ? 1.0 : -1.0) * wy * wx * dot;
                du[1] += wz * (dy ? 1.0 : -1.0) * wx * dot;
                du[2] += wz * wy * (dx ? 1.0 : -1.0) * dot;
              }
          if (!dfield) continue;
          if (!half) {
            for (int a = 0; a < 3; ++a) dfield[p * 3 + a] = du[a];
            continue;
          }
          // u = 2 * sum_corners W * fc[corner] at the clamped coarse coordinate of this fine voxel
          double gz = clampd((z + 0.5) / 2.0 - 0.5, 0.0, Dc - 1.0), gy = clampd((y + 0.5) / 2.0 - 0.5, 0.0, Hc - 1.0);
          double gx = clampd((x + 0.5) / 2.0 - 0.5, 0.0, Wc - 1.0);
          double ez = std::floor(gz), ey = std::floor(gy), ex = std::floor(gx);
          double sz = gz - ez, sy = gy - ey, sx = gx - ex;
          double* dc = dfield + (int64_t)b * Dc * Hc * Wc * 3;
          for (int dz = 0; dz < 2; ++dz)
            for (int dy = 0; dy < 2; ++dy)
              for (int dx = 0; dx < 2; ++dx) {
                double zz = ez + dz, yy = ey + dy, xx = ex + dx;
                if (zz > Dc - 1 || yy > Hc - 1 || xx > Wc - 1) continue;
                double wgt = (dz ? sz : 1.0 - sz) * (dy ? sy : 1.0 - sy) * (dx ? sx : 1.0 - sx);
                int64_t q = (((int64_t)zz * Hc + (int64_t)yy) * Wc + (int64_t)xx) * 3;
                for (int a = 0; a < 3; ++a) dc[q + a] += 2.0 * wgt * du[a];
              }
        }
}

}  // namespace

#define DISPATCH(dtype, CALL)                                            \
  switch (dtype) {                                                       \
    case IN_F32: { typedef float T; CALL; return 0; }                    \
    case IN_BF16: { typedef bf16 T; CALL; return 0; }                    \
    case IN_F64: { typedef double T; CALL; return 0; }                   \
    default: return -1;                                                  \
  }

extern "C" {

int oracle_modet_fwd(const void* Q, const void* K, const double* bias, int B, int D, int H, int W, int C,
                     int heads, int k, double scale, int dtype, double* phi, double* attn, double* lse) {
  Geo g = make_geo(B, D, H, W, C, heads, k);
  DISPATCH(dtype, fwd_impl<T>(g, (const T*)Q, (const T*)K, bias, scale, phi, attn, lse));
}

// dattn (nullable): upstream gradient of the attention weights [B, D, H, W, heads, k^3]
int oracle_modet_bwd_scatter(const void* Q, const void* K, const double* bias, const double* dphi,
                             const double* dattn, int B, int D, int H, int W, int C, int heads, int k, double scale,
                             int dtype, double* dQ, double* dK, double* dbias) {
  Geo g = make_geo(B, D, H, W, C, heads, k);
  DISPATCH(dtype, bwd_scatter_impl<T>(g, (const T*)Q, (const T*)K, bias, scale, dphi, dattn, dQ, dK, dbias));
}

int oracle_modet_bwd_gather(const void* Q, const void* K, const double* bias, const double* dphi,
                            const double* dattn, int B, int D, int H, int W, int C, int heads, int k, double scale,
                            int dtype, double* dQ, double* dK) {
  Geo g = make_geo(B, D, H, W, C, heads, k);
  DISPATCH(dtype, bwd_gather_impl<T>(g, (const T*)Q, (const T*)K, bias, scale, dphi, dattn, dQ, dK));
}

int oracle_modet_fwd_at(const void* Q, const void* K, const double* bias, int B, int D, int H, int W, int C,
                        int heads, int k, double scale, int dtype, int64_t n, const int64_t* idx, double* phi,
                        double* lse) {
  Geo g = make_geo(B, D, H, W, C, heads, k);
  DISPATCH(dtype, fwd_at_impl<T>(g, (const T*)Q, (const T*)K, bias, scale, n, idx, phi, lse));
}

int oracle_modet_bwd_at(const void* Q, const void* K, const double* bias, const double* dphi, int B, int D, int H,
                        int W, int C, int heads, int k, double scale, int dtype, int64_t n, const int64_t* idx,
                        double* dQ, double* dK) {
  Geo g = make_geo(B, D, H, W, C, heads, k);
  DISPATCH(dtype, bwd_at_impl<T>(g, (const T*)Q, (const T*)K, bias, scale, dphi, n, idx, dQ, dK));
}

int oracle_warp(const void* src, const float* field, int B, int D, int H, int W, int C, int field_half_res,
                int dtype, double* out) {
  DISPATCH(dtype, warp_impl<T>((const T*)src, field, B, D, H, W, C, field_half_res, out));
}

int oracle_warp_bwd(const void* src, const float* field, const double* dout, int B, int D, int H, int W, int C,
                    int field_half_res, int dtype, double* dsrc, double* dfield) {
  DISPATCH(dtype, warp_bwd_impl<T>((const T*)src, field, dout, B, D, H, W, C, field_half_res, dsrc, dfield));
}

// the 2x upsampled, x2 scaled field on its own: fine [B,D,H,W,3] from coarse [B,D/2,H/2,W/2,3].
int oracle_upsample2x(const float* coarse, int B, int D, int H, int W, double* fine) {
  int Dc = D / 2, Hc = H / 2, Wc = W / 2;
  for (int b = 0; b < B; ++b)
    for (int z = 0; z < D; ++z)
      for (int y = 0; y < H; ++y)
        for (int x = 0; x < W; ++x)
          upsampled_disp(coarse + (int64_t)b * Dc * Hc * Wc * 3, Dc, Hc, Wc, z, y, x,
                         fine + ((((int64_t)b * D + z) * H + y) * W + x) * 3);
  return 0;
}

int oracle_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

// number of threads the parallel loops use from now on (for timing the oracle on one core); returns the old value
int oracle_set_threads(int n) {
#ifdef _OPENMP
  const int old = omp_get_max_threads();
  if (n >= 1) omp_set_num_threads(n);
  return old;
#else
  (void)n;
  return 1;
#endif
}

}  // extern "C"
