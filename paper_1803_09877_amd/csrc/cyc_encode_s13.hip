// Cyclic encoder kernels for s = 13 (wide windows: one complex coordinate per lane).
#define DRACO_S 13
#include "cyc_encode_narrow_s.inc"
