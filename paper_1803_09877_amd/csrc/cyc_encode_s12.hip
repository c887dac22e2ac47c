// Cyclic encoder kernels for s = 12 (wide windows: one complex coordinate per lane).
#define DRACO_S 12
#include "cyc_encode_narrow_s.inc"
