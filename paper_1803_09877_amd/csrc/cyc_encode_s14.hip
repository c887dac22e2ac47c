// Cyclic encoder kernels for s = 14 (wide windows: one complex coordinate per lane).
#define DRACO_S 14
#include "cyc_encode_narrow_s.inc"
