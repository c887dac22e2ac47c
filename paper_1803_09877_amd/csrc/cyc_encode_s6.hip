// Cyclic encoder kernels for s = 6 (window of 13 gradients).
#define DRACO_S 6
#include "cyc_encode_s.inc"
