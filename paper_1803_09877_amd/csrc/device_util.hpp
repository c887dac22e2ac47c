// Shared device helpers and launch helpers of the streaming kernels.
//
// Every kernel of the library is a streaming pass over [node][coordinate] fp32 slabs and
// is bound by HBM bandwidth: one lane owns 4 consecutive floats (one 16-byte load per
// row), a wavefront therefore reads 1 KiB of each row per step, and the loop over the
// rows runs inside the lane so each input byte is read from HBM exactly once.
// Workgroups are 256 lanes (4 wavefronts).  There is no reuse between workgroups; which
// part of a row a workgroup takes is chosen for the memory system alone (see "workgroup
// footprint" below).
#pragma once

#include "kernels.hpp"

namespace draco {
namespace {


// Slabs are streamed: every byte is used once, so 16-byte accesses carry the
// non-temporal hint (measured on MI355X: +10% on read-dominated passes).
typedef float vfloat4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 ld4(const float* p) {
    const vfloat4 v = __builtin_nontemporal_load(reinterpret_cast<const vfloat4*>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void st4(float* p, float4 v) {
    vfloat4 w;
    w.x = v.x;
    w.y = v.y;
    w.z = v.z;
    w.w = v.w;
    __builtin_nontemporal_store(w, reinterpret_cast<vfloat4*>(p));
}

typedef float vfloat2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float2 ld2(const float* p) {
    const vfloat2 v = __builtin_nontemporal_load(reinterpret_cast<const vfloat2*>(p));
    return make_float2(v.x, v.y);
}
__device__ __forceinline__ void st2(float* p, float2 v) {
    vfloat2 w;
    w.x = v.x;
    w.y = v.y;
    __builtin_nontemporal_store(w, reinterpret_cast<vfloat2*>(p));
}
// Guarded load of up to 2 floats; missing ones read as 0.
__device__ __forceinline__ float2 ld2_partial(const float* p, int n) {
    float2 v = make_float2(0.f, 0.f);
    if (n > 0) v.x = p[0];
    if (n > 1) v.y = p[1];
    return v;
}

// Guarded load of up to 4 floats; missing ones read as 0.
__device__ __forceinline__ float4 ld4_partial(const float* p, int n) {
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (n > 0) v.x = p[0];
    if (n > 1) v.y = p[1];
    if (n > 2) v.z = p[2];
    if (n > 3) v.w = p[3];
    return v;
}
__device__ __forceinline__ void st4_partial(float* p, float4 v, int n) {
    if (n > 0) p[0] = v.x;
    if (n > 1) p[1] = v.y;
    if (n > 2) p[2] = v.z;
    if (n > 3) p[3] = v.w;
}

__device__ __forceinline__ int clamp4(int64_t n) { return n >= 4 ? 4 : (n <= 0 ? 0 : (int)n); }

// Every workgroup but the last of a launch covers whole 16-byte vectors only;
// the kernels branch ONCE, uniformly, on that, so the common path has no
// per-access bounds checks (FULL) and the ragged tail takes the guarded path.
template <bool FULL>
__device__ __forceinline__ float4 ldx(const float* p, int n) {
    if constexpr (FULL) return ld4(p);
    else return ld4_partial(p, n);
}
template <bool FULL>
__device__ __forceinline__ void stx(float* p, float4 v, int n) {
    if constexpr (FULL) st4(p, v);
    else st4_partial(p, v, n);
}

// --- second word of the two-word wire ------------------------------------------
// A message of the two-word wire is hi + lo, hi = fp32(z) and lo the rounding residual
// z - hi.  lo travels as fp32 (kLoF32: the pair carries z to 48 bits), as bfloat16
// (kLoBf16: 32 bits of z at 1.5 words per value), or as an 8-bit fixed-point code in
// units of hi's spacing (kLoI8: 32 bits at 1.25 words); kLoNone is the one-word wire.
// A second-word slab has the element layout of the fp32 one (row stride ldm ELEMENTS,
// same column index), so the kernels address both with the same offsets; the pointer is
// typed float* either way and reinterpreted here.
enum : int { kLoNone = 0, kLoF32 = kSecondWordF32, kLoBf16 = kSecondWordBf16, kLoI8 = kSecondWordI8 };
typedef __bf16 vbf4 __attribute__((ext_vector_type(4)));
typedef __bf16 vbf2 __attribute__((ext_vector_type(2)));

// The 8-bit code.  With E the exponent field of hi, u = 2^(max(E, 24) - 150) is the spacing of
// fp32 numbers at hi (numbers below 2^-103 share the spacing 2^-126: their residuals do not
// matter) and |z - hi| <= u / 2.  Code q = rint(lo / u * 254) in [-127, 127], computed in fp32:
// lo * 254 rounds once, the scaling by 1 / u is exact.  Value of a code: q * u / 254.  Next to a
// non-finite hi the code is arbitrary (hi + anything stays non-finite).
__device__ __forceinline__ int lo8_field(float hi) {
    const int e = (int)((__float_as_uint(hi) >> 23) & 0xFFu);
    return e < 24 ? 24 : e;
}
// The code in the low byte of the result (upper bytes: junk).  Adding 1.5 * 2^23 rounds to the
// nearest integer, ties to even, and leaves it in the low mantissa bits in two's complement.
__device__ __forceinline__ unsigned lo8_code(float hi, float lo) {
    const float t = ldexpf(lo * 254.0f, 150 - lo8_field(hi));
    return __float_as_uint(t + 12582912.0f);
}
__device__ __forceinline__ float lo8_value(float hi, int q) {
    return ldexpf((float)q * (1.0f / 254.0f), lo8_field(hi) - 150);
}

// What one lane holds of the second word for its 4 values, as loaded.
template <int LO> struct lo_raw { typedef float4 type; };
template <> struct lo_raw<kLoBf16> { typedef vbf4 type; };
template <> struct lo_raw<kLoI8> { typedef unsigned type; };
template <int LO> using lo_raw_t = typename lo_raw<LO>::type;

template <bool FULL, int LO>
__device__ __forceinline__ void st_lo(float* base, int64_t off, float4 hi, float4 v, int n) {
    static_assert(LO == kLoF32 || LO == kLoBf16 || LO == kLoI8, "a second word has a format");
    if constexpr (LO == kLoF32) {
        stx<FULL>(base + off, v, n);
    } else if constexpr (LO == kLoBf16) {
        __bf16* p = reinterpret_cast<__bf16*>(base) + off;
        vfloat4 w;
        w.x = v.x;
        w.y = v.y;
        w.z = v.z;
        w.w = v.w;
        const vbf4 b = __builtin_convertvector(w, vbf4);   // round to nearest even
        if constexpr (FULL) {
            __builtin_nontemporal_store(b, reinterpret_cast<vbf4*>(p));
        } else {
            if (n > 0) p[0] = b.x;
            if (n > 1) p[1] = b.y;
            if (n > 2) p[2] = b.z;
            if (n > 3) p[3] = b.w;
        }
    } else {
        signed char* p = reinterpret_cast<signed char*>(base) + off;
        const unsigned q0 = lo8_code(hi.x, v.x), q1 = lo8_code(hi.y, v.y), q2 = lo8_code(hi.z, v.z),
                       q3 = lo8_code(hi.w, v.w);
        if constexpr (FULL) {
            const unsigned w = (q0 & 0xFFu) | ((q1 & 0xFFu) << 8) | ((q2 & 0xFFu) << 16) | (q3 << 24);
            __builtin_nontemporal_store(w, reinterpret_cast<unsigned*>(p));
        } else {
            if (n > 0) p[0] = (signed char)q0;
            if (n > 1) p[1] = (signed char)q1;
            if (n > 2) p[2] = (signed char)q2;
            if (n > 3) p[3] = (signed char)q3;
        }
    }
}
// Load of a lane's 4 second words, unconverted (missing ones read as zero).
template <bool FULL, int LO>
__device__ __forceinline__ lo_raw_t<LO> ld_lo(const float* base, int64_t off, int n) {
    static_assert(LO == kLoF32 || LO == kLoBf16 || LO == kLoI8, "a second word has a format");
    if constexpr (LO == kLoF32) {
        return ldx<FULL>(base + off, n);
    } else if constexpr (LO == kLoBf16) {
        const __bf16* p = reinterpret_cast<const __bf16*>(base) + off;
        if constexpr (FULL) {
            return __builtin_nontemporal_load(reinterpret_cast<const vbf4*>(p));
        } else {
            vbf4 b = {(__bf16)0.0f, (__bf16)0.0f, (__bf16)0.0f, (__bf16)0.0f};
            if (n > 0) b.x = p[0];
            if (n > 1) b.y = p[1];
            if (n > 2) b.z = p[2];
            if (n > 3) b.w = p[3];
            return b;
        }
    } else {
        const unsigned char* p = reinterpret_cast<const unsigned char*>(base) + off;
        if constexpr (FULL) {
            return __builtin_nontemporal_load(reinterpret_cast<const unsigned*>(p));
        } else {
            unsigned w = 0;
            if (n > 0) w |= (unsigned)p[0];
            if (n > 1) w |= (unsigned)p[1] << 8;
            if (n > 2) w |= (unsigned)p[2] << 16;
            if (n > 3) w |= (unsigned)p[3] << 24;
            return w;
        }
    }
}
// The values a lane's 4 second words stand for, next to their first words.
template <int LO>
__device__ __forceinline__ float4 lo_values(lo_raw_t<LO> raw, float4 hi) {
    if constexpr (LO == kLoF32) {
        return raw;
    } else if constexpr (LO == kLoBf16) {
        return make_float4((float)raw.x, (float)raw.y, (float)raw.z, (float)raw.w);
    } else {
        const int w = (int)raw;
        return make_float4(lo8_value(hi.x, (w << 24) >> 24), lo8_value(hi.y, (w << 16) >> 24),
                           lo8_value(hi.z, (w << 8) >> 24), lo8_value(hi.w, w >> 24));
    }
}
// Stores with the format chosen at run time (kernels off the hot path).
template <bool FULL>
__device__ __forceinline__ void st_lo_rt(float* base, int64_t off, float4 hi, float4 v, int n, int lo) {
    if (lo == kLoBf16) st_lo<FULL, kLoBf16>(base, off, hi, v, n);
    else if (lo == kLoI8) st_lo<FULL, kLoI8>(base, off, hi, v, n);
    else st_lo<FULL, kLoF32>(base, off, hi, v, n);
}
// Two values (one complex coordinate) of the second word.
__device__ __forceinline__ void st_lo2_rt(float* base, int64_t off, float2 hi, float2 v, int lo) {
    if (lo == kLoBf16) {
        vfloat2 w;
        w.x = v.x;
        w.y = v.y;
        __builtin_nontemporal_store(__builtin_convertvector(w, vbf2),
                                    reinterpret_cast<vbf2*>(reinterpret_cast<__bf16*>(base) + off));
    } else if (lo == kLoI8) {
        const unsigned short w = (unsigned short)((lo8_code(hi.x, v.x) & 0xFFu) | ((lo8_code(hi.y, v.y) & 0xFFu) << 8));
        __builtin_nontemporal_store(w, reinterpret_cast<unsigned short*>(reinterpret_cast<signed char*>(base) + off));
    } else {
        st2(base + off, v);
    }
}

// --- workgroup footprint ------------------------------------------------------
// Which 4 KiB of a row a workgroup touches.  Contiguous (SPREAD = false): workgroup t owns
// floats [1024 t, 1024 t + 1024).  Spread: the row is cut into windows of 128 KiB; workgroup
// t = 32 w + k owns, in window w, one 1 KiB piece per wavefront, 32 KiB apart:
// floats 32768 w + 8192 v + 256 k + [0, 256) for wavefront v = 0..3.  Every load and store
// instruction of a wavefront still covers 1 KiB contiguously, and the 32 workgroups of a
// window together cover it exactly once.
// Measured on MI355X: a compute unit that walks down many rows sustains more bandwidth when
// what it has in flight at one time is spread over address bits 15 and 16 than when it sits
// in one 4 KiB block -- the cyclic encoder at (P, s, d) = (45, 3, 25.6 M) runs at 5.9 TB/s
// with this footprint against 5.65 contiguous, its two-word form at 5.9 against 5.1; piece
// distances of 16, 32 and 64 KiB help, 128 KiB and more do not (the same channel again).
constexpr int64_t kWindow = 32768;             // floats per footprint window (128 KiB)
constexpr int64_t kWaveStride = kWindow / 4;   // floats between a workgroup's wavefronts (32 KiB)
constexpr int64_t kTilesPerWindow = kWaveStride / 256;

// First float of the window piece this workgroup's wavefront 0 owns.
__device__ __forceinline__ int64_t spread_base() {
    const int64_t tile = blockIdx.x;
    return (tile / kTilesPerWindow) * kWindow + (tile % kTilesPerWindow) * 256;
}
// Column (float index within a row) of this lane's 4 floats.
template <bool SPREAD>
__device__ __forceinline__ int64_t lane_column() {
    if constexpr (SPREAD)
        return spread_base() + (int64_t)(threadIdx.x >> 6) * kWaveStride + (threadIdx.x & 63) * 4;
    else
        return ((int64_t)blockIdx.x * kBlock + threadIdx.x) * 4;
}
// True when every lane of the workgroup has its 4 floats inside [0, len).
template <bool SPREAD>
__device__ __forceinline__ bool block_is_full(int64_t len) {
    if constexpr (SPREAD) return spread_base() + 3 * kWaveStride + 256 <= len;
    else return (int64_t)(blockIdx.x + 1) * (kBlock * 4) <= len;
}


// acc += (tr + i ti) * (x + i y): one instruction sequence wherever it is used
__device__ __forceinline__ void cmac(double tr, double ti, double x, double y, double& are, double& aim) {
    are = fma(tr, x, are);
    are = fma(-ti, y, are);
    aim = fma(tr, y, aim);
    aim = fma(ti, x, aim);
}


// (hr + i hi) = (br + i bi) * (x + i y): one instruction sequence wherever it is used
__device__ __forceinline__ void cmul(double br, double bi, double x, double y, double& hr, double& hi) {
    hr = fma(-bi, y, br * x);
    hi = fma(bi, x, br * y);
}


// ---------------------------------------------------------------------------
// Launch helpers (host)
// ---------------------------------------------------------------------------

inline unsigned grid_for(int64_t units_of_4_floats) {
    return (unsigned)((units_of_4_floats + kBlock - 1) / kBlock);
}
// Workgroups that cover a row of len floats with the footprint lane_column<SPREAD>() describes.
template <bool SPREAD>
inline unsigned grid_cols(int64_t len) {
    if constexpr (SPREAD) return (unsigned)((len + kWindow - 1) / kWindow * kTilesPerWindow);
    else return grid_for((len + 3) / 4);
}

// --- occupancy throttle -----------------------------------------------------
// HBM throughput on MI355X peaks when a CU has roughly 24-48 KiB of loads in
// flight (measured: a [45][25.6M] copy runs at 5.3 TB/s with 32 resident
// wavefronts per CU and at 5.9 TB/s with 4; a read-only pass at 6.1 vs 6.7).
// The streaming kernels therefore ask for more LDS than they use, so that only
// `blocks_per_cu` workgroups fit on a CU at a time.
inline size_t lds_per_cu() {
    static const size_t v = [] {
        int dev = 0, val = 0;
        if (hipGetDevice(&dev) != hipSuccess) return (size_t)65536;
        if (hipDeviceGetAttribute(&val, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, dev) != hipSuccess || val <= 0)
            return (size_t)65536;
        return (size_t)val;
    }();
    return v;
}

// Dynamic LDS bytes to request so that at most blocks_per_cu workgroups are
// resident per CU (0 = no limit), given the kernel's static LDS use and the
// dynamic bytes it really needs.
inline size_t throttle_lds(int blocks_per_cu, size_t static_bytes, size_t needed) {
    if (blocks_per_cu <= 0) return needed;
    size_t per = lds_per_cu() / (size_t)blocks_per_cu;
    per = per / 1024 * 1024;
    const size_t dyn = per > static_bytes ? per - static_bytes : 0;
    return dyn > needed ? dyn : needed;
}

// Opt a kernel in to workgroups with more than 64 KiB of dynamic LDS (once);
// static_bytes is what the kernel declares itself.
template <auto Kernel>
void allow_large_lds(size_t static_bytes = 0) {
    static const hipError_t e =
        hipFuncSetAttribute(reinterpret_cast<const void*>(Kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)(lds_per_cu() - static_bytes));
    if (e != hipSuccess) (void)hipGetLastError();  // the launch itself reports a request that does not fit
}


}  // namespace
}  // namespace draco
