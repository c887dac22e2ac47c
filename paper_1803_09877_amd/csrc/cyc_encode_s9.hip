// Cyclic encoder kernels for s = 9 (window of 19 gradients).
#define DRACO_S 9
#include "cyc_encode_s.inc"
