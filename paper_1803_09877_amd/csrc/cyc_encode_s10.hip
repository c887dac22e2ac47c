// Cyclic encoder kernels for s = 10 (window of 21 gradients).
#define DRACO_S 10
#include "cyc_encode_s.inc"
