// Cyclic encoder kernels for s = 0 (window of 1 gradients).
#define DRACO_S 0
#include "cyc_encode_s.inc"
