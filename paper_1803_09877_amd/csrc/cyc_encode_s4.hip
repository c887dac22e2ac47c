// Cyclic encoder kernels for s = 4 (window of 9 gradients).
#define DRACO_S 4
#include "cyc_encode_s.inc"
