// Host-side algebra of the cyclic code (Sec. 3, "Cyclic Code"): the encoding
// matrix W, the locator phi's small linear algebra and the recombination
// vector b.  Everything here is O(P s + s^3) work on P <= 256 numbers and runs
// in extended precision (x87 long double, 64-bit mantissa) because W and b
// cancel over four to five decimal orders at P = 45.
#pragma once

#include <complex>
#include <cstdint>
#include <vector>

namespace draco {

using real_t = long double;
using cplx_t = std::complex<real_t>;

// exp(2 pi i k / P), argument reduced first.
cplx_t root_of_unity(int P, long long k);

struct CyclicCode {
    int P = 0, s = 0;
    // Z = G W with W[k][k-t] = rot[k] * taps[t], t = 0..2s (all other entries 0):
    // node j's message is sum_t taps[t] * (rot[j+t] * g_{j+t}).
    std::vector<cplx_t> taps;  // 2s+1
    std::vector<cplx_t> rot;   // P, unimodular
    // The same weights with REAL taps: W[j+t][j] = node_phase[j] * real_taps[t] * row_phase[j+t],
    // row_phase indexed by the unwrapped row j + t < P + 2s (its half-angle phase is not
    // P-periodic).  This is the form W() returns and the packed encoders compute with.
    std::vector<real_t> real_taps;    // 2s+1
    std::vector<cplx_t> node_phase;   // P, unimodular
    std::vector<cplx_t> row_phase;    // P + 2s, unimodular
    void build(int P_, int s_);
    cplx_t W(int k, int j) const;  // weight of gradient k in node j's message
};

// Relative size below which a syndrome counts as zero (in units of the median
// |projection|): 32 ulps of the fp32 wire.
constexpr double kTauH = 32.0 / 16777216.0;
// The same for the two-word wire, whose messages carry 48 bits: clean syndromes sit
// near 1e-14 (the fp64 projection's own rounding); 2^-36 leaves three decimal orders.
constexpr double kTauHWide = 1.0 / 68719476736.0;
// Two-word wire with a bfloat16 second word: 32 bits of the message, so 32 of ITS ulps.
constexpr double kTauHBf16 = 32.0 / 8589934592.0;
// And with an 8-bit second word (the residual in 254ths of the first word's spacing).
constexpr double kTauHI8 = 32.0 / 4294967296.0;

// A projection more than kEnormous times the median projection in size: its fp64 rounding,
// times the error growth of the s-error locator, comes within reach of the zero thresholds
// (see cyclic_locate).  Lies of a hundred times an honest message stay below it.
constexpr double kEnormous = 1024.0;
// A node that phi HAS located is set aside only when the rounding of its projection (2^-53 of it,
// summed over up to 256 nodes) could pass for a syndrome: beyond tau * kLocatedEnormousOverTau
// times the median (and kEnormous times it).
constexpr double kLocatedEnormousOverTau = 17592186044416.0;   // 2^44

// phi steps 2-4 on the projections gamma (length P); tau: relative zero threshold (kTauH...).  mask[j] = 1 for located
// nodes; t (length P) receives the reconstructed error projections.  Returns
// true on success, false when no set of at most s nodes accounts for the
// syndromes (mask then holds the s largest |t_j|).  Nodes whose projection is
// not finite are flagged outright and enter the algebra with projection 0.
bool cyclic_locate(int P, int s, double tau, const std::complex<double>* gamma, std::vector<uint8_t>& mask,
                   std::vector<std::complex<double>>& t);

// Minimum-norm b with C_L[:, U] b_U = e_last, U = {j : mask[j] == 0}; needs
// |V| <= 2s.  b[j] = 0 on masked nodes.  Returns false if |V| > 2s.
bool cyclic_recombination_vector(int P, int s, const std::vector<uint8_t>& mask,
                                 std::vector<cplx_t>& b);

}  // namespace draco
