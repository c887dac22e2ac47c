// Cyclic encoder kernels for s = 3 (window of 7 gradients).
#define DRACO_S 3
#include "cyc_encode_s.inc"
