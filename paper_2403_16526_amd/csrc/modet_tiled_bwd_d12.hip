// Backward of the LDS-tiled kernels for heads of twelve channels (the paper's large model, Section 4.4).
#define MODET_BWD_VARIANT 3
#include "modet_tiled_bwd.inc"
