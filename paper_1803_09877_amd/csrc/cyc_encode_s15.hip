// Cyclic encoder kernels for s = 15 (wide windows: one complex coordinate per lane).
#define DRACO_S 15
#include "cyc_encode_narrow_s.inc"
