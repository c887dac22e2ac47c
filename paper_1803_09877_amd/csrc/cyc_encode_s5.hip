// Cyclic encoder kernels for s = 5 (window of 11 gradients).
#define DRACO_S 5
#include "cyc_encode_s.inc"
