// LDS-tiled ModeT kernels (placeholder until the tiled path lands).
#include "modet_common.hpp"
namespace modet {
bool tiled_supported(int, int, int) { return false; }
hipError_t launch_fwd_tiled(const Geo&, int, const void*, const void*, const float*, float*, float*, hipStream_t) {
  return hipErrorNotSupported;
}
hipError_t launch_bwd_tiled(const Geo&, int, const void*, const void*, const float*, const float*, const float*,
                            const float*, float*, float*, hipStream_t) {
  return hipErrorNotSupported;
}
}  // namespace modet
