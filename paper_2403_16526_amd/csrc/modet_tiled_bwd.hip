// Backward entry of the LDS-tiled kernels (derivatives of Eq. 3-4 with respect to Q and K): the kernels
// without bias, and the choice between the two variants.
#define MODET_BWD_VARIANT 0
#include "modet_tiled_bwd.inc"

namespace modet {

bool tiled_bwd_supported(int d, int heads, int k, int dtype) { return tiled_fwd_supported(d, heads, k, dtype); }

// The variant with the bias table also serves a NULL bias whose gradient is wanted.  *dbias_done tells whether
// the kernel that ran has added its sums of dl to io.dbias_acc (only the kernel that hands dl through LDS does).
hipError_t launch_bwd_tiled(const Geo& g, int dtype, bool fast_logits, const BwdTensors& io, hipStream_t st,
                            bool* dbias_done) {
  *dbias_done = false;
  if (g.d == 6) return launch_bwd_tiled_d6(g, dtype, io, st, dbias_done);
  if (g.d == 12) return launch_bwd_tiled_d12(g, dtype, io, st, dbias_done);
  if (io.bias || io.dbias_acc) return launch_bwd_tiled_biased(g, dtype, fast_logits, io, st, dbias_done);
  return launch_bwd_tiled_plain(g, dtype, fast_logits, io, st, dbias_done);
}

}  // namespace modet
