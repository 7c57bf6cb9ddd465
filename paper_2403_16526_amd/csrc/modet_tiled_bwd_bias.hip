// Backward of the LDS-tiled kernels with the bias B of Eq. 3 in the logits (and its gradient): one and two
// heads, and k = 5.
#define MODET_BWD_VARIANT 1
#include "modet_tiled_bwd.inc"
