// Cyclic encoder kernels for s = 8 (window of 17 gradients).
#define DRACO_S 8
#include "cyc_encode_s.inc"
