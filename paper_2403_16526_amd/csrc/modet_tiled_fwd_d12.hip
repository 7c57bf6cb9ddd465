// Forward of the LDS-tiled kernels for heads of twelve channels (the paper's large model, Section 4.4):
// Eq. 3-5 with a head split into two half-heads in neighbouring lanes.
#include "modet_tiled.hpp"

namespace modet {
namespace {

template <int KW, int HS, class T, class LT>
hipError_t launch_fwd_d12_t(const Geo& g, const void* Q, const void* K, const float* bias, float* phi, float* lse,
                           hipStream_t st) {
  TiledParams io = {};
  io.Q = Q; io.K = K; io.bias = bias; io.phi = phi; io.lse = lse;
  launch_march<FwdPolicy<KW, HS, T, LT, true>, Waves<LT, KW>::value>(g, io, st);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_fwd_tiled_d12(const Geo& g, int dtype, const void* Q, const void* K, const float* bias,
                               float* phi, float* lse, hipStream_t st) {
#define MODET_FWD(KW, HS, T, LT) launch_fwd_d12_t<KW, HS, T, LT>(g, Q, K, bias, phi, lse, st)
  MODET_DISPATCH_D12(MODET_FWD)
#undef MODET_FWD
}

}  // namespace modet
