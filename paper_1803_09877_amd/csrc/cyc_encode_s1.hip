// Cyclic encoder kernels for s = 1 (window of 3 gradients).
#define DRACO_S 1
#include "cyc_encode_s.inc"
