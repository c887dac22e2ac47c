// Cyclic encoder kernels for s = 16 (wide windows: one complex coordinate per lane).
#define DRACO_S 16
#include "cyc_encode_narrow_s.inc"
