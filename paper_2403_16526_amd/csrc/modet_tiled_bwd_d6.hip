// Backward of the LDS-tiled kernels for heads of six channels (the paper's small model, Section 4.4).
#define MODET_BWD_VARIANT 2
#include "modet_tiled_bwd.inc"
