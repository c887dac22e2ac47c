// Launchers of the gfx950 kernels behind the C ABI.  All pointers are device
// pointers; every launcher only enqueues work on `stream` and returns the HIP
// error of the launch.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace draco {

constexpr int kBlock = 256;           // threads per workgroup (4 wavefronts of 64)
constexpr int kMaxS = 7;              // repetition kernels are specialised for r = 2s+1 <= 15; larger r takes the generic path
constexpr int kMaxCycS = 10;          // cyclic encoder: two complex per lane up to r = 21, one per lane up to r = 33, an LDS ring beyond
constexpr int kProjectLoads = 8;      // float4 loads per lane per message row in the projection kernel
constexpr int kMaxNodes = 256;        // DRACO_MAX_NODES
constexpr int kMaskWords = 4;         // 64-bit words of node flags (kMaxNodes / 64)
constexpr int kLocateMaxS = 16;       // largest s the on-device locator handles

// Which kernel families spread a workgroup's wavefronts over a 128 KiB window of each row
// (device_util.hpp, "workgroup footprint"); chosen per family by measurement.
constexpr bool kSpreadEncodeCyc = true;
constexpr bool kSpreadEncodeRep = true;
constexpr bool kSpreadVote = true;
constexpr bool kSpreadRecombine = true;
constexpr bool kSpreadUpdate = true;

// Complex numbers in device tables: (re, im) as double2.

// ---- repetition code ----
hipError_t launch_encode_rep(const float* G, int64_t ldg, float* Z, int64_t ldm, int P, int s,
                             int64_t d, hipStream_t stream);
hipError_t launch_encode_rep_node(const float* Gn, int64_t ldg, float* z, int s, int64_t d,
                                  hipStream_t stream);
// ORs node flags into flags[kMaskWords] (must be zero on entry).
hipError_t launch_decode_rep_vote(const float* R, int64_t ldm, float* u, uint64_t* flags, int P,
                                  int s, int64_t d, hipStream_t stream);
// mask_out <- flags; status_out <- NO_MAJORITY if a group has more than s flags; flags <- 0.
hipError_t launch_decode_rep_finish(uint64_t* flags, uint64_t* mask_out, int32_t* status_out,
                                    int P, int s, hipStream_t stream);
// The vote and its finish on flag words held in a device array of the library itself (one per
// GPU, shared by every call on that GPU): no allocation anywhere.
hipError_t launch_decode_rep_static(const float* R, int64_t ldm, float* u, uint64_t* mask_out,
                                    int32_t* status_out, int P, int s, int64_t d, hipStream_t stream);

// B > P: the gradient slab holds m = B/P per-sample rows per unit gradient (rows k*m .. k*m+m-1).
hipError_t launch_encode_rep_samples(const float* G, int64_t ldg, int m, float* Z, int64_t ldm, int P,
                                     int s, int64_t d, hipStream_t stream);

// ---- cyclic code ----
// coef[n*(2s+1) + t] = W[(n+t) mod P][n]: the weight node n gives its t-th assigned gradient
// (used by the unpacked wire).  The packed encoders take W factored, W[(n+t) mod P][n] =
// rotA[n] * rho[t] * rotB[n+t] with real rho[2s+1], unit rotA[P] and unit rotB[P+2s] (indexed by
// the unwrapped row n + t): device pointers.
struct CycTaps {
    const double* rho;
    const double2* rotA;
    const double2* rotB;
};
// Zlo / zlo / Rlo below: second word of the two-word wire (message = hi + lo), or nullptr;
// lo names its format: kSecondWordF32 (a float slab), kSecondWordBf16 (a bfloat16 slab) or
// kSecondWordI8 (a slab of 8-bit residual codes), each with the same row stride counted in
// ELEMENTS.  Ignored when the pointer is null.
constexpr int kSecondWordF32 = 1, kSecondWordBf16 = 2, kSecondWordI8 = 3;
// B > P on the cyclic code (rows as for launch_encode_rep_samples).
hipError_t launch_encode_cyc_samples(const float* G, int64_t ldg, int m, float* Z, float* Zlo, int lo,
                                     int64_t ldm, const CycTaps& tab, int P, int s, int64_t d, hipStream_t stream);
hipError_t launch_encode_cyc(const float* G, int64_t ldg, float* Z, float* Zlo, int lo, int64_t ldm,
                             const CycTaps& tab, int P, int s, int64_t d, hipStream_t stream);
// Unpacked wire: real gradients [P][d] in, messages of d complex entries (2d floats) out.
hipError_t launch_encode_cyc_real(const float* G, int64_t ldg, float* Z, int64_t ldm, const double2* coef,
                                  int P, int s, int64_t d, hipStream_t stream);
// Gn holds only the node's 2s+1 gradients, in assignment order.
hipError_t launch_encode_cyc_real_node(const float* Gn, int64_t ldg, float* z, const double2* coef, int node,
                                       int P, int s, int64_t d, hipStream_t stream);
hipError_t launch_encode_cyc_node(const float* Gn, int64_t ldg, float* z, float* zlo, int lo,
                                  const CycTaps& tab, int node, int P, int s, int64_t d, hipStream_t stream);
// Number of workgroups (= rows of `partial`) the projection uses for gradient length d.
int64_t project_tiles(int64_t d);
// partial[tile][P] <- per-tile sums of f_i * R[j][i]; gamma[P] <- their sum in tile order.
// b0[P]: recombination vector for "no adversary"; u: output written speculatively when
// spec_state[0] != 0 (spec_state: two device words, see cyc_decode.hip; nullptr = never).
// f == nullptr: the entries of f are generated from f_seed (projection_rng.hpp).
// d is the number of floats a message carries (odd d: one more, zero); realout (unpacked
// wire, messages of d/2 complex entries): u receives only the real parts, d/2 floats.
hipError_t launch_cyc_project(const float* R, const float* Rlo, int lo, int64_t ldm, const float* f,
                              uint64_t f_seed, double2* partial, double2* gamma, const double2* b0,
                              float* u, bool realout, int32_t* spec_state, int P, int64_t d,
                              hipStream_t stream);
// phi steps 2-4 and the recombination vector on the device (one wavefront, fp64; s <= kLocateMaxS):
// gamma[P] -> mask words, status, and the honest nodes' (idx, b) compacted in ascending order with
// their count in *nu_out.  roots[k] = exp(2 pi i k / P), k < P.  tau: relative zero threshold for syndromes.
// With no located node the coefficients are copied from b0 (bit-identical to the speculative pass);
// spec_state[0] <- 1 if this decode was clean (the next call speculates), else 0.
hipError_t launch_cyc_locate(const double2* gamma, const double2* roots, int P, int s, double tau, const double2* b0,
                             uint64_t* mask_out, int32_t* status_out, double2* b_out, int32_t* idx_out,
                             int32_t* nu_out, int32_t* spec_state, hipStream_t stream);
// u <- unpack( sum_{q < *nu} b[q] * R[idx[q]] ); nu is read from device memory.
hipError_t launch_cyc_recombine(const float* R, const float* Rlo, int lo, int64_t ldm, const double2* b,
                                const int32_t* idx, const int32_t* nu, const int32_t* spec_state, int P,
                                float* u, bool realout, int64_t d, hipStream_t stream);

// params[i] <- params[i] - scale * sum[i], i < d (the model update of mini-batch SGD).
hipError_t launch_apply_update(float* params, const float* sum, float scale, int64_t d, hipStream_t stream);

// dst[j][0..row_len) <- src[j][0..row_len) for j < rows, row_len a multiple of 4 floats
// (bandwidth / counter calibration).
hipError_t launch_copy_probe(const float* src, float* dst, int rows, int64_t row_len, int64_t ld,
                             hipStream_t stream);

}  // namespace draco
