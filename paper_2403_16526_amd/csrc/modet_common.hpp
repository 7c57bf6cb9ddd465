// Shared declarations of the libmodet HIP sources (kernels + C ABI).  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace modet {

struct Geo {
  int B, D, H, W, C, heads, k, r, d, k3;
  long long nvox;   // B*D*H*W
  long long nvn;    // nvox*heads
  float scale;      // multiplies the dot product (natural-log units)
};

typedef uint16_t bf16_t;   // bfloat16 bit pattern

__device__ __forceinline__ float ldf(const float* p, long long i) { return p[i]; }
__device__ __forceinline__ float ldf(const bf16_t* p, long long i) {
  return __uint_as_float(((uint32_t)p[i]) << 16);
}

// fp32 -> bf16 bits, round to nearest even (finite inputs)
__device__ __forceinline__ bf16_t f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

// ---- launchers (each returns hipGetLastError() of its launches) ------------------------
// generic kernels: any head size, k in {1,3,5,7}, fp32 / bf16 inputs
hipError_t launch_fwd_generic(const Geo& g, int dtype, const void* Q, const void* K, const float* bias,
                              float* phi, float* attn, float* lse, hipStream_t st);
// dattn (nullable): upstream gradient of the attention weights; adot: one float per window of scratch for it
hipError_t launch_bwd_generic(const Geo& g, int dtype, const void* Q, const void* K, const float* bias,
                              const float* dphi, const float* phi, const float* lse, const float* dattn,
                              float* adot, float* dQ, float* dK, hipStream_t st);
// Gradient of the bias.  The sums over all voxels are accumulated in fp64 in `acc` ([heads, k^3] doubles of the
// caller's workspace): _begin zeroes it, any number of kernels add to it, _end rounds it into dbias.
hipError_t launch_dbias_begin(const Geo& g, double* acc, hipStream_t st);
hipError_t launch_dbias_generic(const Geo& g, int dtype, const void* Q, const void* K, const float* bias,
                                const float* dphi, const float* phi, const float* lse, const float* dattn,
                                const float* adot, double* acc, hipStream_t st);
hipError_t launch_dbias_end(const Geo& g, const double* acc, float* dbias, hipStream_t st);
hipError_t launch_warp(const void* src, const float* field, void* out, int B, int D, int H, int W, int C,
                       int half, int dtype, hipStream_t st);
// gradients of sum(dout * warp(src, field)): dsrc [B, D, H, W, C] fp32, dfield (nullable) in the shape of field
hipError_t launch_warp_bwd(const void* src, const float* field, const float* dout, float* dsrc, float* dfield, int B,
                           int D, int H, int W, int C, int half, int dtype, hipStream_t st);
// out = s * (inner + trilinear(outer, p + s * inner)); fields [B, D, H, W, 3] fp32.  outer_half_res (with s = 1):
// outer is [B, D/2, H/2, W/2, 3] and is upsampled 2x (values doubled) on the fly
hipError_t launch_compose(const float* outer, const float* inner, float* out, int B, int D, int H, int W, float s,
                          int outer_half_res, hipStream_t st);

// LDS-tiled kernels (heads of 8, 6 or 12 channels)
bool tiled_fwd_supported(int d, int heads, int k, int dtype);
bool tiled_bwd_supported(int d, int heads, int k, int dtype);
// fast_logits: fp32 instead of fp64 dot products for fp32 inputs (logits good to ~1e-6 only)
hipError_t launch_fwd_tiled(const Geo& g, int dtype, bool fast_logits, const void* Q, const void* K,
                            const float* bias, float* phi, float* lse, hipStream_t st);
struct BwdTensors {
  const void* Q; const void* K;
  const float* bias;          // nullable
  const float* dphi; const float* phi; const float* lse;
  float* dQ; float* dK;
  double* dbias_acc;          // nullable: where the sums of dl go if the kernel can provide them
};
// *dbias_done: the launched kernel adds the bias gradient's sums to io.dbias_acc
hipError_t launch_bwd_tiled(const Geo& g, int dtype, bool fast_logits, const BwdTensors& io, hipStream_t st,
                            bool* dbias_done);
hipError_t launch_bwd_tiled_plain(const Geo& g, int dtype, bool fast_logits, const BwdTensors& io, hipStream_t st,
                                  bool* dbias_done);
hipError_t launch_bwd_tiled_biased(const Geo& g, int dtype, bool fast_logits, const BwdTensors& io, hipStream_t st,
                                   bool* dbias_done);
hipError_t launch_bwd_tiled_biased_many(const Geo& g, int dtype, bool fast_logits, const BwdTensors& io,
                                        hipStream_t st, bool* dbias_done);
// heads of six channels
hipError_t launch_fwd_tiled_d6(const Geo& g, int dtype, const void* Q, const void* K, const float* bias,
                               float* phi, float* lse, hipStream_t st);
hipError_t launch_bwd_tiled_d6(const Geo& g, int dtype, const BwdTensors& io, hipStream_t st, bool* dbias_done);
// heads of twelve channels
hipError_t launch_fwd_tiled_d12(const Geo& g, int dtype, const void* Q, const void* K, const float* bias,
                                float* phi, float* lse, hipStream_t st);
hipError_t launch_bwd_tiled_d12(const Geo& g, int dtype, const BwdTensors& io, hipStream_t st, bool* dbias_done);

}  // namespace modet
