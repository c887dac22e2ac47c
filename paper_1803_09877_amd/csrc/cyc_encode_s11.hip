// Cyclic encoder kernels for s = 11 (wide windows: one complex coordinate per lane).
#define DRACO_S 11
#include "cyc_encode_narrow_s.inc"
