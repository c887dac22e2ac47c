// Cyclic encoder E^Cyc (Sec. 3, "Cyclic Code") for wide windows, 11 <= s <= 16: with r = 2s+1
// up to 33 taps per output the pass is bound by fp64 multiply-adds (2 r + 8 per complex
// coordinate on the packed wire, where W's taps are real; 4 r on the unpacked wire), not by
// HBM, so a lane owns ONE complex coordinate (8-byte accesses) and keeps the whole window
// g_n .. g_{n+2s} of it in registers as doubles (on the packed wire: rotated by the row
// phase as it enters).  The window is a shift register: U = 4 outputs are formed per step
// from positions i .. i+2s, then everything moves down by U; the taps of the
// U outputs are interleaved, which keeps 2U independent accumulator chains in flight.  The
// first 2s unit gradients are parked in LDS for the wrap-around; the next U rows are fetched
// while the current outputs are computed.  One kernel covers the packed wire (one or two words), the
// unpacked wire (REAL: a lane owns two real coordinates and writes two complex entries) and
// B > P (MULTI: a unit gradient is the fp64 sum of its m rows, formed as it enters the window).
// Same taps in the same order as the one-node kernels: identical bits.
#pragma once

#include <type_traits>

#include "device_util.hpp"

namespace draco {

template <int S, bool REAL, bool MULTI, bool FULL>
__device__ __forceinline__ void encode_cyc_narrow_body(const float* __restrict__ G, int64_t ldg, int m,
                                                       float* __restrict__ Z, float* __restrict__ Zlo, int lo,
                                                       int64_t ldm, const double2* __restrict__ coef,
                                                       const CycTaps tab, int P, int64_t d) {
    constexpr int R = 2 * S + 1;
    constexpr int U = 4;
    // unit gradients 0 .. 2s-1 of this lane's pair, parked for the wrap-around: the fp64 sums
    // when a unit is a sum of rows, else the raw floats (half the LDS: two workgroups per CU)
    using parked_t = typename std::conditional<MULTI, double2, float2>::type;
    extern __shared__ unsigned char parked_raw[];
    parked_t* parked = reinterpret_cast<parked_t*>(parked_raw);   // [2S][kBlock]
    const int64_t c0 = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * 2;   // first float of the lane's pair
    const int64_t len = REAL ? d : 2 * ((d + 1) / 2);                       // floats of a row that carry lanes
    if (!FULL && c0 >= len) return;
    // gradient floats of the pair that exist (odd d: the pad reads 0); FULL: the whole workgroup has both
    const int nin = FULL ? 2 : (d - c0 >= 2 ? 2 : (d - c0 <= 0 ? 0 : 1));

    auto load_row = [&](int64_t row) -> float2 {
        const float* p = G + row * ldg + c0;
        if constexpr (FULL) return ld2(p);
        else return ld2_partial(p, nin);
    };
    auto widen = [](float2 x) { return make_double2((double)x.x, (double)x.y); };
    // a unit gradient as it enters the window: on the packed wire rotated by B of its unwrapped
    // row index (see tap_sum in cyc_encode_kernels.hpp), on the unpacked wire as it is
    auto enter = [&](double2 v, int kappa) -> double2 {
        if constexpr (REAL) {
            return v;
        } else {
            const double2 B = tab.rotB[kappa];
            double2 h;
            cmul(B.x, B.y, v.x, v.y, h.x, h.y);
            return h;
        }
    };
    auto unit_sum = [&](int k) -> double2 {   // MULTI: unit gradient k < P, the fp64 sum of its m rows, ascending
        double2 acc = make_double2(0.0, 0.0);
        const int64_t first = (int64_t)k * m;
        for (int i0 = 0; i0 < m; i0 += 4) {
            float2 x[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (i0 + i < m) x[i] = load_row(first + i0 + i);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (i0 + i < m) {
                    acc.x += (double)x[i].x;
                    acc.y += (double)x[i].y;
                }
            }
        }
        return acc;
    };
    // U outputs n0 .. n0+U-1 from window positions i .. i+2s; the taps of the U outputs are
    // interleaved so that 2U (4U on the unpacked wire) independent accumulators are in flight
    auto outputs = [&](int n0, const double2 (&w)[2 * S + U], int count) {
        if constexpr (REAL) {
            const double2* cn = coef + (int64_t)n0 * R;
            double re0[U], im0[U], re1[U], im1[U];
#pragma unroll
            for (int i = 0; i < U; ++i) re0[i] = im0[i] = re1[i] = im1[i] = 0.0;
#pragma unroll
            for (int t = 0; t < R; ++t) {
#pragma unroll
                for (int i = 0; i < U; ++i) {
                    if (i < count) {
                        const double cr = cn[i * R + t].x, ci = cn[i * R + t].y;
                        re0[i] = fma(cr, w[i + t].x, re0[i]);
                        im0[i] = fma(ci, w[i + t].x, im0[i]);
                        re1[i] = fma(cr, w[i + t].y, re1[i]);
                        im1[i] = fma(ci, w[i + t].y, im1[i]);
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < U; ++i) {
                if (i < count) {
                    float* dst = Z + (int64_t)(n0 + i) * ldm + 2 * c0;
                    const float4 out = make_float4((float)re0[i], (float)im0[i], (float)re1[i], (float)im1[i]);
                    if (FULL || nin == 2) st4(dst, out);
                    else st4_partial(dst, out, 2 * nin);
                }
            }
        } else {
            double sr[U], si[U], are[U], aim[U];
#pragma unroll
            for (int i = 0; i < U; ++i) sr[i] = si[i] = 0.0;
#pragma unroll
            for (int t = 0; t < R; ++t) {
                const double r = tab.rho[t];
#pragma unroll
                for (int i = 0; i < U; ++i) {
                    if (i < count) {
                        sr[i] = fma(r, w[i + t].x, sr[i]);
                        si[i] = fma(r, w[i + t].y, si[i]);
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < U; ++i) {
                if (i < count) {
                    const double2 A = tab.rotA[n0 + i];
                    cmul(A.x, A.y, sr[i], si[i], are[i], aim[i]);
                    const float hr = (float)are[i], hi = (float)aim[i];
                    st2(Z + (int64_t)(n0 + i) * ldm + c0, make_float2(hr, hi));
                    if (Zlo != nullptr)   // second word of the wide wire: what the first rounding lost
                        st_lo2_rt(Zlo, (int64_t)(n0 + i) * ldm + c0, make_float2(hr, hi),
                                  make_float2((float)(are[i] - (double)hr), (float)(aim[i] - (double)hi)), lo);
                }
            }
        }
    };

    double2 w[2 * S + U];   // position t holds unit gradient n0 + t
    if constexpr (MULTI) {
#pragma unroll
        for (int k = 0; k < 2 * S; ++k) {
            const double2 v = unit_sum(k);
            parked[k * kBlock + threadIdx.x] = v;
            w[k] = enter(v, k);
        }
    } else {   // all 2s loads in flight before the first is parked
        float2 x[2 * S];
#pragma unroll
        for (int k = 0; k < 2 * S; ++k) x[k] = load_row(k);
#pragma unroll
        for (int k = 0; k < 2 * S; ++k) {
            parked[k * kBlock + threadIdx.x] = x[k];
            w[k] = enter(widen(x[k]), k);
        }
    }
    float2 pre[MULTI ? 1 : U];   // rows 2s + i of the coming step, in flight (plain rows only)
    if constexpr (!MULTI) {
#pragma unroll
        for (int i = 0; i < U; ++i) pre[i] = load_row(2 * S + i < P ? 2 * S + i : P - 1);
    }
    int n0 = 0;
    // steps whose U outputs bring only rows below P into the window: no guards
    for (; n0 + U + 2 * S <= P; n0 += U) {
#pragma unroll
        for (int i = 0; i < U; ++i) {
            if constexpr (MULTI) w[2 * S + i] = enter(unit_sum(n0 + i + 2 * S), n0 + i + 2 * S);
            else w[2 * S + i] = enter(widen(pre[i]), n0 + i + 2 * S);
        }
        if constexpr (!MULTI) {
#pragma unroll
            for (int i = 0; i < U; ++i) {
                const int k = n0 + U + i + 2 * S;
                pre[i] = load_row(k < P ? k : P - 1);   // past the last row: a harmless repeat, never used
            }
        }
        outputs(n0, w, U);
#pragma unroll
        for (int t = 0; t < 2 * S; ++t) w[t] = w[t + U];
    }
    // the last steps: rows wrap around to the parked ones, the final step may be short
    for (; n0 < P; n0 += U) {
        const int count = P - n0 < U ? P - n0 : U;
#pragma unroll
        for (int i = 0; i < U; ++i) {
            const int k = n0 + i + 2 * S;
            if (i < count) {
                if (k >= P) {
                    if constexpr (MULTI) w[2 * S + i] = enter(parked[(k - P) * kBlock + threadIdx.x], k);
                    else w[2 * S + i] = enter(widen(parked[(k - P) * kBlock + threadIdx.x]), k);
                } else {
                    if constexpr (MULTI) w[2 * S + i] = enter(unit_sum(k), k);
                    else w[2 * S + i] = enter(widen(pre[i]), k);
                }
            }
        }
        if constexpr (!MULTI) {
#pragma unroll
            for (int i = 0; i < U; ++i) {
                const int k = n0 + U + i + 2 * S;
                if (k < P) pre[i] = load_row(k);
            }
        }
        if (count == U) outputs(n0, w, U);   // a constant count folds the guards away: the taps interleave
        else outputs(n0, w, count);
#pragma unroll
        for (int t = 0; t < 2 * S; ++t) w[t] = w[t + U];
    }
}

template <int S, bool REAL, bool MULTI>
__global__ __launch_bounds__(kBlock) void encode_cyc_narrow_kernel(const float* __restrict__ G, int64_t ldg, int m,
                                                                   float* __restrict__ Z, float* __restrict__ Zlo,
                                                                   int lo, int64_t ldm,
                                                                   const double2* __restrict__ coef,
                                                                   const CycTaps tab, int P, int64_t d) {
    // every lane of the workgroup has both floats of its pair inside the gradient
    if ((int64_t)(blockIdx.x + 1) * (kBlock * 2) <= d) encode_cyc_narrow_body<S, REAL, MULTI, true>(G, ldg, m, Z, Zlo, lo, ldm, coef, tab, P, d);
    else encode_cyc_narrow_body<S, REAL, MULTI, false>(G, ldg, m, Z, Zlo, lo, ldm, coef, tab, P, d);
}

// Launch for one s (defined in the translation unit of that s).
template <int S>
hipError_t launch_encode_cyc_narrow_s(bool real, hipStream_t stream, const float* G, int64_t ldg, int m, float* Z,
                                      float* Zlo, int lo, int64_t ldm, const double2* coef, const CycTaps& tab, int P,
                                      int64_t d);

}  // namespace draco
