// Counter-based generator of phi's random vector f ~ N(1, I) (Sec. 3, phi step 1): entry i
// depends on (seed, i) only, so the projection kernel makes the entries it needs on the fly
// instead of reading a stored vector, and any host can reproduce them.
//
//   z  = splitmix64 finaliser of  seed + (i+1) * 0x9E3779B97F4A7C15
//   u1 = (top 24 bits of z + 1/2) / 2^24,   u2 = (bits 16..39 of z + 1/2) / 2^24
//   f  = fp32( 1 + sqrt(-2 ln u1) * cos(2 pi u2) )          (Box-Muller, evaluated in fp64)
#pragma once

#include <cmath>
#include <cstdint>

namespace draco {

__host__ __device__ inline float projection_entry(uint64_t seed, uint64_t i) {
    uint64_t z = seed + (i + 1) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    z ^= z >> 31;
    const double u1 = ((double)(z >> 40) + 0.5) * (1.0 / 16777216.0);
    const double u2 = ((double)((z >> 16) & 0xFFFFFFull) + 0.5) * (1.0 / 16777216.0);
#if defined(__HIP_DEVICE_COMPILE__)
    const double c = cospi(2.0 * u2);
#else
    const double c = std::cos(6.283185307179586476925286766559 * u2);
#endif
    return (float)(1.0 + std::sqrt(-2.0 * std::log(u1)) * c);
}

}  // namespace draco
