// Backward of the LDS-tiled kernels with the bias B of Eq. 3, four and eight heads.
#define MODET_BWD_VARIANT 4
#include "modet_tiled_bwd.inc"
