// Cyclic encoder kernels for s = 2 (window of 5 gradients).
#define DRACO_S 2
#include "cyc_encode_s.inc"
