// Forward entry of the LDS-tiled kernels (Section 3.3.1, Eq. 3-5): instantiations and dispatch.
#include "modet_tiled.hpp"

namespace modet {
namespace {

template <int KW, int HS, class T, class LT, bool BIAS>
hipError_t launch_fwd_t(const Geo& g, const void* Q, const void* K, const float* bias, float* phi, float* lse,
                        hipStream_t st) {
  TiledParams io = {};
  io.Q = Q; io.K = K; io.bias = bias; io.phi = phi; io.lse = lse;
  launch_march<FwdPolicy<KW, HS, T, LT, BIAS>, Waves<LT, KW>::value>(g, io, st);
  return hipGetLastError();
}

hipError_t launch_fwd_plain(const Geo& g, int dtype, bool fast_logits, const void* Q, const void* K, float* phi,
                            float* lse, hipStream_t st) {
#define MODET_FWD(KW, HS, T, LT) launch_fwd_t<KW, HS, T, LT, false>(g, Q, K, nullptr, phi, lse, st)
  MODET_DISPATCH(MODET_FWD)
#undef MODET_FWD
}

hipError_t launch_fwd_biased(const Geo& g, int dtype, bool fast_logits, const void* Q, const void* K,
                             const float* bias, float* phi, float* lse, hipStream_t st) {
#define MODET_FWD(KW, HS, T, LT) launch_fwd_t<KW, HS, T, LT, true>(g, Q, K, bias, phi, lse, st)
  MODET_DISPATCH(MODET_FWD)
#undef MODET_FWD
}

}  // namespace

// Covered, with or without bias.  Head size 8:  k = 3: 1/2/4/8/16/32 heads, fp32 inputs (fp64 logits) and bf16
// inputs (fp32 logits: the bf16 tolerance leaves room);  k = 5: 1/2 heads, bf16 inputs.  Head sizes 6 and 12
// (the paper's small and large model, Section 4.4): k = 3, 1/2/4/8/16/32 heads, both input types.
bool tiled_fwd_supported(int d, int heads, int k, int dtype) {
  const bool pow2 = heads == 1 || heads == 2 || heads == 4 || heads == 8 || heads == 16 || heads == 32;
  if (d == 6) return k == 3 && pow2;      // (more than 8 fused columns per voxel run as head groups of 8)
  if (d == 12) return k == 3 && pow2;
  if (d != 8) return false;
  if (k == 3) return pow2;
  if (k == 5) return dtype == 1 && (heads == 1 || heads == 2);
  return false;
}

hipError_t launch_fwd_tiled(const Geo& g, int dtype, bool fast_logits, const void* Q, const void* K,
                            const float* bias, float* phi, float* lse, hipStream_t st) {
  if (g.d == 6) return launch_fwd_tiled_d6(g, dtype, Q, K, bias, phi, lse, st);
  if (g.d == 12) return launch_fwd_tiled_d12(g, dtype, Q, K, bias, phi, lse, st);
  if (bias) return launch_fwd_biased(g, dtype, fast_logits, Q, K, bias, phi, lse, st);
  return launch_fwd_plain(g, dtype, fast_logits, Q, K, phi, lse, st);
}

}  // namespace modet
