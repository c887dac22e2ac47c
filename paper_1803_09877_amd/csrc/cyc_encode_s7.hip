// Cyclic encoder kernels for s = 7 (window of 15 gradients).
#define DRACO_S 7
#include "cyc_encode_s.inc"
