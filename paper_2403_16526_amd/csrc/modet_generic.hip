// Generic ModeT kernels: one lane per (voxel, head) window, keys read straight from global
// memory.  They cover every head size, k in {1,3,5,7} and both input types, produce the
// optional attention map, and serve as the fallback for shapes the LDS-tiled kernels do
// not cover.  Paper: Section 3.3.1, Eq. 3 (scores + softmax) and Eq. 4-5 (weighted offsets);
// the backward is the derivative of those two equations.
#include "modet_common.hpp"

namespace modet {
namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ void decode_vn(const Geo& g, long long vn, int& b, int& z, int& y, int& x, int& s,
                                          long long& v) {
  s = (int)(vn % g.heads);
  v = vn / g.heads;
  long long t = v;
  x = (int)(t % g.W); t /= g.W;
  y = (int)(t % g.H); t /= g.H;
  z = (int)(t % g.D);
  b = (int)(t / g.D);
}

__device__ __forceinline__ bool inside(const Geo& g, int z, int y, int x) {
  return (unsigned)z < (unsigned)g.D && (unsigned)y < (unsigned)g.H && (unsigned)x < (unsigned)g.W;
}

// The dot product is accumulated in fp64: a logit of magnitude ~10 carries ~1e-6 of rounding when summed
// in fp32, which the softmax turns into a 1e-6 relative error of every weight; fp64 FMAs issue at the
// same rate as unpacked fp32 ones on this chip.
template <class T>
__device__ __forceinline__ double dot_d(const T* q, const T* kk, int d) {
  double acc = 0.0;
  for (int c = 0; c < d; ++c) acc = fma((double)ldf(q, c), (double)ldf(kk, c), acc);
  return acc;
}

// Eq. 3 + Eq. 4 for one window per lane; online softmax (running max) so no logit is stored.
template <class T>
__global__ void __launch_bounds__(kThreads)
fwd_generic_kernel(Geo g, const T* __restrict__ Q, const T* __restrict__ K, const float* __restrict__ bias,
                   float* __restrict__ phi, float* __restrict__ attn, float* __restrict__ lse) {
  long long vn = (long long)blockIdx.x * kThreads + threadIdx.x;
  if (vn >= g.nvn) return;
  int b, z, y, x, s; long long v;
  decode_vn(g, vn, b, z, y, x, s, v);
  const T* q = Q + v * g.C + s * g.d;
  const int r = g.r;
  double m = -INFINITY;          // running maximum, kept in fp64 like the logits
  double Z = 0.0, S0 = 0.0, S1 = 0.0, S2 = 0.0;   // fp64 sums: phi must be good to fp32 rounding for the backward
  int j = 0;
  for (int a = -r; a <= r; ++a)
    for (int bb = -r; bb <= r; ++bb)
      for (int c = -r; c <= r; ++c, ++j) {
        double l = bias ? (double)bias[s * g.k3 + j] : 0.0;
        if (inside(g, z + a, y + bb, x + c)) {
          long long nb = v + ((long long)a * g.H + bb) * g.W + c;
          l = fma((double)g.scale, dot_d(q, K + nb * g.C + s * g.d, g.d), l);
        }
        if (l > m) {
          double al = (double)expf((float)(m - l));
          Z *= al; S0 *= al; S1 *= al; S2 *= al;
          m = l;
        }
        double e = (double)expf((float)(l - m));
        Z += e; S0 = fma(e, (double)a, S0); S1 = fma(e, (double)bb, S1); S2 = fma(e, (double)c, S2);
      }
  double inv = 1.0 / Z;
  phi[vn * 3 + 0] = (float)(S0 * inv);
  phi[vn * 3 + 1] = (float)(S1 * inv);
  phi[vn * 3 + 2] = (float)(S2 * inv);
  if (lse) lse[vn] = (float)(m + (double)logf((float)Z));
  if (attn) {
    j = 0;
    for (int a = -r; a <= r; ++a)
      for (int bb = -r; bb <= r; ++bb)
        for (int c = -r; c <= r; ++c, ++j) {
          double l = bias ? (double)bias[s * g.k3 + j] : 0.0;
          if (inside(g, z + a, y + bb, x + c)) {
            long long nb = v + ((long long)a * g.H + bb) * g.W + c;
            l = fma((double)g.scale, dot_d(q, K + nb * g.C + s * g.d, g.d), l);
          }
          attn[vn * g.k3 + j] = (float)((double)expf((float)(l - m)) * inv);
        }
  }
}

// dQ (KEYSIDE = false): lane owns CH channels of one head of query voxel p and walks its window.
// dK (KEYSIDE = true) : lane owns CH channels of key voxel q and walks the queries p = q - o that
//                       see it under offset o.  Weights come from w = exp(l - lse[p]).
// When the attention weights are an output with upstream gradient dattn, the softmax Jacobian is applied to
// t_o = g.o + dattn_o:  dl_o = w_o * (t_o - g.phi - adot),  adot = sum_o w_o dattn_o  (one value per window,
// computed by attn_dot_kernel before the gradient kernels run).
template <class T>
__global__ void __launch_bounds__(kThreads)
attn_dot_kernel(Geo g, const T* __restrict__ Q, const T* __restrict__ K, const float* __restrict__ bias,
                const float* __restrict__ lse, const float* __restrict__ dattn, float* __restrict__ adot) {
  const long long vn = (long long)blockIdx.x * kThreads + threadIdx.x;
  if (vn >= g.nvn) return;
  int b, z, y, x, s; long long v;
  decode_vn(g, vn, b, z, y, x, s, v);
  const int r = g.r;
  const T* q = Q + v * g.C + s * g.d;
  const double ls = (double)lse[vn];
  // The weights exp(l - lse) inherit the fp32 rounding of lse as a common factor 1 + eps.  In dl that factor is
  // harmless (a relative error of the whole gradient), but in this mean it would be an absolute error of every
  // dl of the window: divide by the weights' own sum instead of trusting it to be one.
  double acc = 0.0, Z = 0.0;
  int j = 0;
  for (int a = -r; a <= r; ++a)
    for (int bb = -r; bb <= r; ++bb)
      for (int c = -r; c <= r; ++c, ++j) {
        double l = bias ? (double)bias[s * g.k3 + j] : 0.0;
        if (inside(g, z + a, y + bb, x + c))
          l = fma((double)g.scale, dot_d(q, K + (v + ((long long)a * g.H + bb) * g.W + c) * g.C + s * g.d, g.d), l);
        const double w = (double)expf((float)(l - ls));
        Z += w;
        acc = fma(w, (double)dattn[vn * g.k3 + j], acc);
      }
  adot[vn] = (float)(acc / Z);
}

template <class T, int CH, bool KEYSIDE>
__global__ void __launch_bounds__(kThreads)
grad_generic_kernel(Geo g, const T* __restrict__ Q, const T* __restrict__ K, const float* __restrict__ bias,
                    const float* __restrict__ dphi, const float* __restrict__ phi,
                    const float* __restrict__ lse, const float* __restrict__ dattn,
                    const float* __restrict__ adot, float* __restrict__ out) {
  const int nchunk = g.d / CH;
  long long idx = (long long)blockIdx.x * kThreads + threadIdx.x;
  if (idx >= g.nvn * nchunk) return;
  const int chunk = (int)(idx % nchunk);
  const long long vn = idx / nchunk;
  int b, z, y, x, s; long long v;
  decode_vn(g, vn, b, z, y, x, s, v);
  const int r = g.r, c0 = s * g.d + chunk * CH;
  // (sums in fp64: with a gradient through the attention weights the terms are several times larger than those
  // of the displacement alone, and their fp32 sum would sit at the tolerance)
  double acc[CH];
#pragma unroll
  for (int i = 0; i < CH; ++i) acc[i] = 0.0;
  float g0 = 0.f, g1 = 0.f, g2 = 0.f, ls = 0.f;
  double gphi = 0.0;
  if (!KEYSIDE) {
    g0 = dphi[vn * 3]; g1 = dphi[vn * 3 + 1]; g2 = dphi[vn * 3 + 2];
    gphi = (double)(g0 * phi[vn * 3] + g1 * phi[vn * 3 + 1] + g2 * phi[vn * 3 + 2]);
    if (dattn) gphi += (double)adot[vn];
    ls = lse[vn];
  }
  int j = 0;
  for (int a = -r; a <= r; ++a)
    for (int bb = -r; bb <= r; ++bb)
      for (int c = -r; c <= r; ++c, ++j) {
        const int oz = KEYSIDE ? z - a : z + a, oy = KEYSIDE ? y - bb : y + bb, ox = KEYSIDE ? x - c : x + c;
        if (!inside(g, oz, oy, ox)) continue;   // a padded key has no gradient and feeds none
        const long long ov = v + (KEYSIDE ? -1 : 1) * (((long long)a * g.H + bb) * g.W + c);
        const long long pv = KEYSIDE ? ov : v;    // query voxel of the pair
        const long long qv = KEYSIDE ? v : ov;    // key voxel of the pair
        const long long pvn = pv * g.heads + s;
        if (KEYSIDE) {
          g0 = dphi[pvn * 3]; g1 = dphi[pvn * 3 + 1]; g2 = dphi[pvn * 3 + 2];
          gphi = (double)(g0 * phi[pvn * 3] + g1 * phi[pvn * 3 + 1] + g2 * phi[pvn * 3 + 2]);
          if (dattn) gphi += (double)adot[pvn];
          ls = lse[pvn];
        }
        const double l = fma((double)g.scale, dot_d(Q + pv * g.C + s * g.d, K + qv * g.C + s * g.d, g.d),
                             bias ? (double)bias[s * g.k3 + j] : 0.0);
        const float w = expf((float)(l - (double)ls));
        double t = (double)(g0 * (float)a + g1 * (float)bb + g2 * (float)c);
        if (dattn) t += (double)dattn[pvn * g.k3 + j];
        const double dl = (double)w * (t - gphi);
        const T* other = KEYSIDE ? Q + pv * g.C + c0 : K + qv * g.C + c0;
#pragma unroll
        for (int i = 0; i < CH; ++i) acc[i] = fma(dl, (double)ldf(other, i), acc[i]);
      }
#pragma unroll
  for (int i = 0; i < CH; ++i) out[v * g.C + c0 + i] = (float)((double)g.scale * acc[i]);
}

__global__ void fill_zero_kernel(double* p, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0.0;
}

__global__ void round_to_float_kernel(const double* a, float* o, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) o[i] = (float)a[i];
}

// acc[s, j] += sum over voxels of dl_j(p, s): per-block partial sums in LDS, then one global atomic per entry
// and block, all in fp64 (the terms cancel: a sum over millions of voxels is far smaller than the sum of their
// magnitudes).  The order of the additions is not fixed; in fp64 that leaves the rounded fp32 result unchanged
// in practice.
template <class T>
__global__ void __launch_bounds__(kThreads)
dbias_kernel(Geo g, const T* __restrict__ Q, const T* __restrict__ K, const float* __restrict__ bias,
             const float* __restrict__ dphi, const float* __restrict__ phi, const float* __restrict__ lse,
             const float* __restrict__ dattn, const float* __restrict__ adot, double* __restrict__ acc,
             long long per_block) {
  extern __shared__ double part[];
  const int nent = g.heads * g.k3;
  for (int i = threadIdx.x; i < nent; i += kThreads) part[i] = 0.0;
  __syncthreads();
  const long long lo = (long long)blockIdx.x * per_block;
  const long long hi = lo + per_block < g.nvn ? lo + per_block : g.nvn;
  const int r = g.r;
  for (long long vn = lo + threadIdx.x; vn < hi; vn += kThreads) {
    int b, z, y, x, s; long long v;
    decode_vn(g, vn, b, z, y, x, s, v);
    const float g0 = dphi[vn * 3], g1 = dphi[vn * 3 + 1], g2 = dphi[vn * 3 + 2];
    float gphi = g0 * phi[vn * 3] + g1 * phi[vn * 3 + 1] + g2 * phi[vn * 3 + 2];
    if (dattn) gphi += adot[vn];
    const float ls = lse[vn];
    const T* q = Q + v * g.C + s * g.d;
    int j = 0;
    for (int a = -r; a <= r; ++a)
      for (int bb = -r; bb <= r; ++bb)
        for (int c = -r; c <= r; ++c, ++j) {
          double l = bias ? (double)bias[s * g.k3 + j] : 0.0;
          if (inside(g, z + a, y + bb, x + c)) {
            long long nb = v + ((long long)a * g.H + bb) * g.W + c;
            l = fma((double)g.scale, dot_d(q, K + nb * g.C + s * g.d, g.d), l);
          }
          float t = g0 * (float)a + g1 * (float)bb + g2 * (float)c;
          if (dattn) t += dattn[vn * g.k3 + j];
          const float dl = expf((float)(l - (double)ls)) * (t - gphi);
          atomicAdd(&part[s * g.k3 + j], (double)dl);
        }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < nent; i += kThreads) atomicAdd(&acc[i], part[i]);
}

inline unsigned blocks_for(long long n) { return (unsigned)((n + kThreads - 1) / kThreads); }

template <class T, bool KEYSIDE>
void launch_grad(const Geo& g, const T* Q, const T* K, const float* bias, const float* dphi, const float* phi,
                 const float* lse, const float* dattn, const float* adot, float* out, hipStream_t st) {
  int ch = 1;
  for (int c : {8, 6, 4, 3, 2}) if (g.d % c == 0) { ch = c; break; }
  const long long n = g.nvn * (g.d / ch);
  dim3 grid(blocks_for(n)), block(kThreads);
#define MODET_GRAD(CH_) \
  hipLaunchKernelGGL((grad_generic_kernel<T, CH_, KEYSIDE>), grid, block, 0, st, g, Q, K, bias, dphi, phi, lse, dattn, \
                     adot, out)
  switch (ch) {
    case 8: MODET_GRAD(8); break;
    case 6: MODET_GRAD(6); break;
    case 4: MODET_GRAD(4); break;
    case 3: MODET_GRAD(3); break;
    case 2: MODET_GRAD(2); break;
    default: MODET_GRAD(1); break;
  }
#undef MODET_GRAD
}

}  // namespace

hipError_t launch_fwd_generic(const Geo& g, int dtype, const void* Q, const void* K, const float* bias,
                              float* phi, float* attn, float* lse, hipStream_t st) {
  dim3 grid(blocks_for(g.nvn)), block(kThreads);
  if (dtype == 0)
    hipLaunchKernelGGL((fwd_generic_kernel<float>), grid, block, 0, st, g, (const float*)Q, (const float*)K, bias,
                       phi, attn, lse);
  else
    hipLaunchKernelGGL((fwd_generic_kernel<bf16_t>), grid, block, 0, st, g, (const bf16_t*)Q, (const bf16_t*)K,
                       bias, phi, attn, lse);
  return hipGetLastError();
}

hipError_t launch_bwd_generic(const Geo& g, int dtype, const void* Q, const void* K, const float* bias,
                              const float* dphi, const float* phi, const float* lse, const float* dattn,
                              float* adot, float* dQ, float* dK, hipStream_t st) {
  dim3 grid(blocks_for(g.nvn)), block(kThreads);
  if (dtype == 0) {
    if (dattn)
      hipLaunchKernelGGL((attn_dot_kernel<float>), grid, block, 0, st, g, (const float*)Q, (const float*)K, bias, lse,
                         dattn, adot);
    launch_grad<float, false>(g, (const float*)Q, (const float*)K, bias, dphi, phi, lse, dattn, adot, dQ, st);
    launch_grad<float, true>(g, (const float*)Q, (const float*)K, bias, dphi, phi, lse, dattn, adot, dK, st);
  } else {
    if (dattn)
      hipLaunchKernelGGL((attn_dot_kernel<bf16_t>), grid, block, 0, st, g, (const bf16_t*)Q, (const bf16_t*)K, bias,
                         lse, dattn, adot);
    launch_grad<bf16_t, false>(g, (const bf16_t*)Q, (const bf16_t*)K, bias, dphi, phi, lse, dattn, adot, dQ, st);
    launch_grad<bf16_t, true>(g, (const bf16_t*)Q, (const bf16_t*)K, bias, dphi, phi, lse, dattn, adot, dK, st);
  }
  return hipGetLastError();
}

hipError_t launch_dbias_begin(const Geo& g, double* acc, hipStream_t st) {
  const int nent = g.heads * g.k3;
  hipLaunchKernelGGL(fill_zero_kernel, dim3((nent + 255) / 256), dim3(256), 0, st, acc, nent);
  return hipGetLastError();
}

hipError_t launch_dbias_end(const Geo& g, const double* acc, float* dbias, hipStream_t st) {
  const int nent = g.heads * g.k3;
  hipLaunchKernelGGL(round_to_float_kernel, dim3((nent + 255) / 256), dim3(256), 0, st, acc, dbias, nent);
  return hipGetLastError();
}

hipError_t launch_dbias_generic(const Geo& g, int dtype, const void* Q, const void* K, const float* bias,
                                const float* dphi, const float* phi, const float* lse, const float* dattn,
                                const float* adot, double* acc, hipStream_t st) {
  const int nent = g.heads * g.k3;
  long long per_block = 8192;
  unsigned nblk = (unsigned)((g.nvn + per_block - 1) / per_block);
  size_t shm = sizeof(double) * (size_t)nent;
  if (dtype == 0)
    hipLaunchKernelGGL((dbias_kernel<float>), dim3(nblk), dim3(kThreads), shm, st, g, (const float*)Q,
                       (const float*)K, bias, dphi, phi, lse, dattn, adot, acc, per_block);
  else
    hipLaunchKernelGGL((dbias_kernel<bf16_t>), dim3(nblk), dim3(kThreads), shm, st, g, (const bf16_t*)Q,
                       (const bf16_t*)K, bias, dphi, phi, lse, dattn, adot, acc, per_block);
  return hipGetLastError();
}

}  // namespace modet
