// Kernel templates of the cyclic encoder E^Cyc (Sec. 3, "Cyclic Code"), shared by the
// per-window-width translation units (one per s, so they compile in parallel).
#pragma once

#include <type_traits>

#include "device_util.hpp"

namespace draco {

// E^Cyc for all nodes: z_n = sum_{t=0}^{2s} W[(n+t) mod P][n] * g_{(n+t) mod P} on packed
// complex coordinates in fp64, W in the factored form described at tap_sum below.  A lane
// keeps the window g_n .. g_{n+2s} of its two complex coordinates in registers
// and slides it down the P rows, so every gradient row is read from HBM once;
// rows 0..2s-1, needed again by the last 2s nodes, are parked in LDS (each lane
// reads back only what it wrote: no barrier).  Rows are fetched NB-1 rounds of
// R = 2s+1 ahead of the arithmetic (a ring of NB register buffers).
// W factors as W[k][j] = A_j * rho_t * B_k for k = j + t (t = 0..2s), with REAL taps rho_t: the
// nodes that do not hold gradient k are consecutive on the circle, so every factor
// w^j - w^m of W's closed form is a unit phase times a sine.  A message is therefore
//   z_j = A_j * sum_t rho_t * (B_{j+t} g_{j+t}),
// one complex rotation per gradient row as it enters the window, 2 real multiply-adds per tap and
// complex coordinate (instead of 4), one rotation per output.  B is indexed by the UNWRAPPED row
// j + t < P + 2s (its half-angle phase is not P-periodic).  Every packed encoder below forms
// these products in this order, so their messages agree bit for bit.
// Window entry of unwrapped gradient row kappa for a lane's two complex coordinates.
__device__ __forceinline__ void rotate_in(const CycTaps& tab, int kappa, double x, double y, double z, double w,
                                          double (&re)[2], double (&im)[2]) {
    const double2 B = tab.rotB[kappa];
    cmul(B.x, B.y, x, y, re[0], im[0]);
    cmul(B.x, B.y, z, w, re[1], im[1]);
}
// Node n's two message entries from the window: taps on slots (first + t) mod R, then A_n.
template <int R>
__device__ __forceinline__ void tap_sum(const CycTaps& tab, int n, const double (&wre)[R][2], const double (&wim)[R][2],
                                        int first, double& are0, double& aim0, double& are1, double& aim1) {
    double sr0 = 0.0, si0 = 0.0, sr1 = 0.0, si1 = 0.0;
#pragma unroll
    for (int t = 0; t < R; ++t) {
        const int slot = (first + t) % R;
        const double r = tab.rho[t];
        sr0 = fma(r, wre[slot][0], sr0);
        si0 = fma(r, wim[slot][0], si0);
        sr1 = fma(r, wre[slot][1], sr1);
        si1 = fma(r, wim[slot][1], si1);
    }
    const double2 A = tab.rotA[n];
    cmul(A.x, A.y, sr0, si0, are0, aim0);
    cmul(A.x, A.y, sr1, si1, are1, aim1);
}

template <int S, int NB, bool FULL, int LO>
__device__ __forceinline__ void encode_cyc_body(const float* __restrict__ G, int64_t ldg, float* __restrict__ Z,
                                                float* __restrict__ Zlo, int64_t ldm,
                                                const CycTaps tab, int P, int64_t d,
                                                float4* head /* LDS [2S][kBlock] */) {
    constexpr int R = 2 * S + 1;
    const int64_t c0 = lane_column<kSpreadEncodeCyc>();
    const int64_t mlen = 2 * ((d + 1) / 2);
    if (!FULL && c0 >= mlen) return;
    const int nin = FULL ? 4 : clamp4(d - c0);      // gradient floats that exist (the pad of an odd d reads as 0)
    const int nout = FULL ? 4 : clamp4(mlen - c0);  // message floats to write

    double wre[R][2], wim[R][2];  // window slot = row index mod R

    auto put = [&](int slot, const float4& raw, int kappa) {
        rotate_in(tab, kappa, (double)raw.x, (double)raw.y, (double)raw.z, (double)raw.w, wre[slot], wim[slot]);
    };
    // fetch the rows that nodes n0 .. n0+R-1 bring into the window
    auto issue = [&](int n0, float4 (&buf)[R]) {
#pragma unroll
        for (int uu = 0; uu < R; ++uu) {
            const int kk = n0 + uu + 2 * S;
            if (n0 + uu < P) {
                if (kk < P) buf[uu] = ldx<FULL>(G + (int64_t)kk * ldg + c0, nin);
                else buf[uu] = head[(kk - P) * kBlock + threadIdx.x];
            }
        }
    };
    auto consume = [&](int n0, const float4 (&buf)[R]) {
#pragma unroll
        for (int uu = 0; uu < R; ++uu) {
            const int n = n0 + uu;
            if (n < P) {
                put((uu + 2 * S) % R, buf[uu], n + 2 * S);
                double are0, aim0, are1, aim1;
                tap_sum<R>(tab, n, wre, wim, uu % R, are0, aim0, are1, aim1);
                const float4 hi = make_float4((float)are0, (float)aim0, (float)are1, (float)aim1);
                stx<FULL>(Z + (int64_t)n * ldm + c0, hi, nout);
                if constexpr (LO != kLoNone) {  // second word of the wide wire: what the first rounding lost
                    const float4 lo = make_float4((float)(are0 - (double)hi.x), (float)(aim0 - (double)hi.y),
                                                  (float)(are1 - (double)hi.z), (float)(aim1 - (double)hi.w));
                    st_lo<FULL, LO>(Zlo, (int64_t)n * ldm + c0, hi, lo, nout);
                }
            }
        }
    };

#pragma unroll
    for (int k = 0; k < 2 * S; ++k) {
        const float4 raw = ldx<FULL>(G + (int64_t)k * ldg + c0, nin);
        head[k * kBlock + threadIdx.x] = raw;
        put(k, raw, k);
    }
    float4 buf[NB][R];
#pragma unroll
    for (int b = 0; b < NB - 1; ++b)
        if (b * R < P) issue(b * R, buf[b]);
    for (int n0 = 0; n0 < P; n0 += NB * R) {
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int cur = n0 + b * R;
            if (cur < P) {
                const int nxt = cur + (NB - 1) * R;
                if (nxt < P) issue(nxt, buf[(b + NB - 1) % NB]);
                consume(cur, buf[b]);
            }
        }
    }
}

template <int S, int NB, int LO>
__global__ __launch_bounds__(kBlock) void encode_cyc_kernel(const float* __restrict__ G, int64_t ldg,
                                                            float* __restrict__ Z, float* __restrict__ Zlo,
                                                            int64_t ldm, const CycTaps tab, int P,
                                                            int64_t d) {
    extern __shared__ float4 head[];  // [2S][kBlock]
    if (block_is_full<kSpreadEncodeCyc>(d)) encode_cyc_body<S, NB, true, LO>(G, ldg, Z, Zlo, ldm, tab, P, d, head);
    else encode_cyc_body<S, NB, false, LO>(G, ldg, Z, Zlo, ldm, tab, P, d, head);
}

// The same encoder with a wider lane: a lane owns C float4 of every row (its wavefront's C
// pieces of 1 KiB) and a workgroup's 4C pieces are spread evenly over the 128 KiB footprint
// window -- wavefront v, piece q at (v + 4q) * (32 KiB / C) -- so a compute unit has more
// distinct channels in flight at a time.  One row of loads is issued per finished row, D
// rows ahead (a ring of raw rows whose slot is the row index mod the unroll length).  Same
// taps in the same order as encode_cyc_body: identical bits.  Registers hold the window of
// C lanes' worth (R*C*8 doubles), so this form is for narrow windows.
// Measured at (P, s, d) = (45, 3, 25.6 M), one word per float: C = 4, D = 2 runs at 6.1 TB/s
// against 5.9 for encode_cyc_body on the same footprint window (and 5.65 contiguous); with an
// 8-bit second word 1750 us against 1770; with a 16- or 32-bit second word it gains nothing.
template <int S, int C, int D, bool FULL, int LO>
__device__ __forceinline__ void encode_cyc_strip_body(const float* __restrict__ G, int64_t ldg,
                                                      float* __restrict__ Z, float* __restrict__ Zlo, int64_t ldm,
                                                      const CycTaps tab, int P, int64_t d,
                                                      float4* head /* LDS [2S][C][kBlock] */,
                                                      const int64_t (&cq)[C]) {
    constexpr int R = 2 * S + 1;
    constexpr int U = R * ((D + R - 1) / R);  // unroll length and ring size: a multiple of R that holds D rows
    const int64_t mlen = 2 * ((d + 1) / 2);
    int nin[C], nout[C];
#pragma unroll
    for (int q = 0; q < C; ++q) {
        nin[q] = FULL ? 4 : clamp4(d - cq[q]);
        nout[q] = FULL ? 4 : clamp4(mlen - cq[q]);
    }
    double wre[C][R][2], wim[C][R][2];  // [piece][window slot = row index mod R]
    auto put = [&](int slot, const float4 (&raw)[C], int kappa) {
#pragma unroll
        for (int q = 0; q < C; ++q)
            rotate_in(tab, kappa, (double)raw[q].x, (double)raw[q].y, (double)raw[q].z, (double)raw[q].w,
                      wre[q][slot], wim[q][slot]);
    };
    auto fetch = [&](int k, float4 (&dst)[C]) {  // row k; k >= P wraps to the rows parked in LDS
        if (k < P) {
#pragma unroll
            for (int q = 0; q < C; ++q)
                if (FULL || nout[q] > 0) dst[q] = ldx<FULL>(G + (int64_t)k * ldg + cq[q], nin[q]);
        } else {
#pragma unroll
            for (int q = 0; q < C; ++q) dst[q] = head[((k - P) * C + q) * kBlock + threadIdx.x];
        }
    };
    float4 ring[U][C];
    {
        float4 row[C];
#pragma unroll
        for (int k = 0; k < 2 * S; ++k) {
            fetch(k, row);
#pragma unroll
            for (int q = 0; q < C; ++q) head[(k * C + q) * kBlock + threadIdx.x] = row[q];
            put(k, row, k);
        }
    }
#pragma unroll
    for (int i = 0; i < D; ++i)
        if (i < P) fetch(i + 2 * S, ring[i]);
    for (int n0 = 0; n0 < P; n0 += U) {
#pragma unroll
        for (int uu = 0; uu < U; ++uu) {
            const int n = n0 + uu;
            if (n < P) {
                put((uu + 2 * S) % R, ring[uu], n + 2 * S);
                if (n + D < P) fetch(n + D + 2 * S, ring[(uu + D) % U]);
#pragma unroll
                for (int q = 0; q < C; ++q) {
                    double are0, aim0, are1, aim1;
                    tap_sum<R>(tab, n, wre[q], wim[q], uu % R, are0, aim0, are1, aim1);
                    if (FULL || nout[q] > 0) {
                        const float4 hi = make_float4((float)are0, (float)aim0, (float)are1, (float)aim1);
                        stx<FULL>(Z + (int64_t)n * ldm + cq[q], hi, nout[q]);
                        if constexpr (LO != kLoNone) {
                            const float4 lo = make_float4((float)(are0 - (double)hi.x), (float)(aim0 - (double)hi.y),
                                                          (float)(are1 - (double)hi.z), (float)(aim1 - (double)hi.w));
                            st_lo<FULL, LO>(Zlo, (int64_t)n * ldm + cq[q], hi, lo, nout[q]);
                        }
                    }
                }
            }
        }
    }
}

template <int S, int C, int D, int LO>
__global__ __launch_bounds__(kBlock) void encode_cyc_strip_kernel(const float* __restrict__ G, int64_t ldg,
                                                                  float* __restrict__ Z, float* __restrict__ Zlo,
                                                                  int64_t ldm,
                                                                  const CycTaps tab, int P,
                                                                  int64_t d) {
    extern __shared__ float4 head[];  // [2S][C][kBlock]
    constexpr int64_t u = kWindow / (4 * C);   // floats between neighbouring pieces of the workgroup
    constexpr int64_t per = u / 256;           // workgroups per window
    const int64_t base = ((int64_t)blockIdx.x / per) * kWindow + ((int64_t)blockIdx.x % per) * 256;
    int64_t cq[C];
#pragma unroll
    for (int q = 0; q < C; ++q) cq[q] = base + ((threadIdx.x >> 6) + 4 * q) * u + (threadIdx.x & 63) * 4;
    if (base + (4 * C - 1) * u + 256 <= d) encode_cyc_strip_body<S, C, D, true, LO>(G, ldg, Z, Zlo, ldm, tab, P, d, head, cq);
    else encode_cyc_strip_body<S, C, D, false, LO>(G, ldg, Z, Zlo, ldm, tab, P, d, head, cq);
}
// Workgroups of encode_cyc_strip_kernel<S, C, D> for messages of mlen floats.
template <int C>
inline unsigned strip_grid(int64_t mlen) {
    return (unsigned)((mlen + kWindow - 1) / kWindow * (kWindow / (4 * C) / 256));
}

// E^Cyc on the real gradients as Sec. 3 states it, without the packing remark that closes
// the section: z_n = sum_t coef[n][t] * g_{(n+t) mod P} with real g, so a message has d
// complex entries (2d floats, re/im interleaved).  Same sliding window and prefetch ring
// as above, on four reals per lane instead of two complex numbers (two FMAs per tap and
// coordinate).  A message row is twice as long as a gradient row, so a lane owns two PAIRS
// of real coordinates half a wavefront span apart (8-byte loads): their complex outputs
// are 16 bytes each and every store instruction of a wavefront writes 1 KiB contiguously.
template <int S, int NB, bool FULL>
__device__ __forceinline__ void encode_cyc_real_body(const float* __restrict__ G, int64_t ldg,
                                                     float* __restrict__ Z, int64_t ldm,
                                                     const double2* __restrict__ coef, int P, int64_t d,
                                                     float4* head /* LDS [2S][kBlock] */) {
    constexpr int R = 2 * S + 1;
    // the wavefront covers 256 consecutive real coordinates; mine are cA, cA+1, cA+128, cA+129
    const int64_t cA = lane_column<kSpreadEncodeCyc>() - (threadIdx.x & 63) * 2;
    const int64_t cB = cA + 128;
    if (!FULL && cA >= d) return;
    const int nA = FULL ? 2 : (d - cA >= 2 ? 2 : (int)(d - cA));
    const int nB = FULL ? 2 : (d - cB >= 2 ? 2 : (d - cB <= 0 ? 0 : (int)(d - cB)));

    auto fetch = [&](int row) -> float4 {
        const float* p = G + (int64_t)row * ldg;
        float2 a, b;
        if constexpr (FULL) {
            a = ld2(p + cA);
            b = ld2(p + cB);
        } else {
            a = ld2_partial(p + cA, nA);
            b = ld2_partial(p + cB, nB);
        }
        return make_float4(a.x, a.y, b.x, b.y);
    };

    double w[R][4];  // window slot = row index mod R
    auto put = [&](int slot, const float4& raw) {
        w[slot][0] = (double)raw.x;
        w[slot][1] = (double)raw.y;
        w[slot][2] = (double)raw.z;
        w[slot][3] = (double)raw.w;
    };
    auto issue = [&](int n0, float4 (&buf)[R]) {
#pragma unroll
        for (int uu = 0; uu < R; ++uu) {
            const int kk = n0 + uu + 2 * S;
            if (n0 + uu < P) {
                if (kk < P) buf[uu] = fetch(kk);
                else buf[uu] = head[(kk - P) * kBlock + threadIdx.x];
            }
        }
    };
    auto consume = [&](int n0, const float4 (&buf)[R]) {
#pragma unroll
        for (int uu = 0; uu < R; ++uu) {
            const int n = n0 + uu;
            if (n < P) {
                put((uu + 2 * S) % R, buf[uu]);
                const double2* cn = coef + (int64_t)n * R;
                double re[4] = {0.0, 0.0, 0.0, 0.0}, im[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
                for (int t = 0; t < R; ++t) {
                    const int slot = (uu + t) % R;
                    const double cr = cn[t].x, ci = cn[t].y;
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        re[c] = fma(cr, w[slot][c], re[c]);
                        im[c] = fma(ci, w[slot][c], im[c]);
                    }
                }
                float* dst = Z + (int64_t)n * ldm;
                stx<FULL>(dst + 2 * cA, make_float4((float)re[0], (float)im[0], (float)re[1], (float)im[1]), 2 * nA);
                stx<FULL>(dst + 2 * cB, make_float4((float)re[2], (float)im[2], (float)re[3], (float)im[3]), 2 * nB);
            }
        }
    };

#pragma unroll
    for (int k = 0; k < 2 * S; ++k) {
        const float4 raw = fetch(k);
        head[k * kBlock + threadIdx.x] = raw;
        put(k, raw);
    }
    float4 buf[NB][R];
#pragma unroll
    for (int b = 0; b < NB - 1; ++b)
        if (b * R < P) issue(b * R, buf[b]);
    for (int n0 = 0; n0 < P; n0 += NB * R) {
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int cur = n0 + b * R;
            if (cur < P) {
                const int nxt = cur + (NB - 1) * R;
                if (nxt < P) issue(nxt, buf[(b + NB - 1) % NB]);
                consume(cur, buf[b]);
            }
        }
    }
}

template <int S, int NB>
__global__ __launch_bounds__(kBlock) void encode_cyc_real_kernel(const float* __restrict__ G, int64_t ldg,
                                                                 float* __restrict__ Z, int64_t ldm,
                                                                 const double2* __restrict__ coef, int P,
                                                                 int64_t d) {
    extern __shared__ float4 head[];  // [2S][kBlock]
    if (block_is_full<kSpreadEncodeCyc>(d)) encode_cyc_real_body<S, NB, true>(G, ldg, Z, ldm, coef, P, d, head);
    else encode_cyc_real_body<S, NB, false>(G, ldg, Z, ldm, coef, P, d, head);
}

// E^Cyc when every unit gradient is the sum of m = B/P per-sample gradients (rows k*m ..
// k*m+m-1 of the sample slab): the same sliding window, but a window entry is the fp64
// sum of m rows, formed as the rows arrive; the first 2s unit sums are parked in LDS in
// fp64 for the wrap-around.  Units are fetched one round ahead.
template <int S, bool FULL, int LO>
__device__ __forceinline__ void encode_cyc_multi_body(const float* __restrict__ G, int64_t ldg, int m,
                                                      float* __restrict__ Z, float* __restrict__ Zlo, int64_t ldm,
                                                      const CycTaps tab, int P, int64_t d,
                                                      double4* head /* LDS [2S][kBlock] */) {
    constexpr int R = 2 * S + 1;
    constexpr int UN = 4;
    const int64_t c0 = lane_column<kSpreadEncodeCyc>();
    const int64_t mlen = 2 * ((d + 1) / 2);
    if (!FULL && c0 >= mlen) return;
    const int nin = FULL ? 4 : clamp4(d - c0);
    const int nout = FULL ? 4 : clamp4(mlen - c0);

    double wre[R][2], wim[R][2];
    auto put = [&](int slot, const double4& v, int kappa) {
        rotate_in(tab, kappa, v.x, v.y, v.z, v.w, wre[slot], wim[slot]);
    };
    auto unit_sum = [&](int k) -> double4 {  // g_k = sum of its m sample rows, ascending, in fp64
        double4 acc = make_double4(0.0, 0.0, 0.0, 0.0);
        const float* src = G + (int64_t)k * m * ldg + c0;
        for (int i0 = 0; i0 < m; i0 += UN) {
            float4 x[UN];
#pragma unroll
            for (int i = 0; i < UN; ++i)
                if (i0 + i < m) x[i] = ldx<FULL>(src + (int64_t)(i0 + i) * ldg, nin);
#pragma unroll
            for (int i = 0; i < UN; ++i) {
                if (i0 + i < m) {
                    acc.x += (double)x[i].x;
                    acc.y += (double)x[i].y;
                    acc.z += (double)x[i].z;
                    acc.w += (double)x[i].w;
                }
            }
        }
        return acc;
    };
    auto issue = [&](int n0, double4 (&buf)[R]) {
#pragma unroll
        for (int uu = 0; uu < R; ++uu) {
            const int kk = n0 + uu + 2 * S;
            if (n0 + uu < P) {
                if (kk < P) buf[uu] = unit_sum(kk);
                else buf[uu] = head[(kk - P) * kBlock + threadIdx.x];
            }
        }
    };
    auto consume = [&](int n0, const double4 (&buf)[R]) {
#pragma unroll
        for (int uu = 0; uu < R; ++uu) {
            const int n = n0 + uu;
            if (n < P) {
                put((uu + 2 * S) % R, buf[uu], n + 2 * S);
                double are0, aim0, are1, aim1;
                tap_sum<R>(tab, n, wre, wim, uu % R, are0, aim0, are1, aim1);
                const float4 hi = make_float4((float)are0, (float)aim0, (float)are1, (float)aim1);
                stx<FULL>(Z + (int64_t)n * ldm + c0, hi, nout);
                if constexpr (LO != kLoNone) {
                    const float4 lo = make_float4((float)(are0 - (double)hi.x), (float)(aim0 - (double)hi.y),
                                                  (float)(are1 - (double)hi.z), (float)(aim1 - (double)hi.w));
                    st_lo<FULL, LO>(Zlo, (int64_t)n * ldm + c0, hi, lo, nout);
                }
            }
        }
    };
#pragma unroll
    for (int k = 0; k < 2 * S; ++k) {
        const double4 v = unit_sum(k);
        head[k * kBlock + threadIdx.x] = v;
        put(k, v, k);
    }
    double4 bufA[R], bufB[R];
    issue(0, bufA);
    for (int n0 = 0; n0 < P; n0 += 2 * R) {
        if (n0 + R < P) issue(n0 + R, bufB);
        consume(n0, bufA);
        if (n0 + R < P) {
            if (n0 + 2 * R < P) issue(n0 + 2 * R, bufA);
            consume(n0 + R, bufB);
        }
    }
}

// The same when m is a multiple of D: the B = m P sample rows are consumed in one linear
// walk with the next D rows always in flight (a ring of D raw rows whose slot is the row
// index mod D, static because m is a multiple of D), so the loads of the next unit overlap
// the sums of this one.  Same additions in the same order as above: identical bits.
template <int S, int D, bool FULL, int LO>
__device__ __forceinline__ void encode_cyc_multi_ring_body(const float* __restrict__ G, int64_t ldg, int m,
                                                           float* __restrict__ Z, float* __restrict__ Zlo,
                                                           int64_t ldm, const CycTaps tab, int P,
                                                           int64_t d, double4* head /* LDS [2S][kBlock] */) {
    constexpr int R = 2 * S + 1;
    const int64_t c0 = lane_column<kSpreadEncodeCyc>();
    const int64_t mlen = 2 * ((d + 1) / 2);
    if (!FULL && c0 >= mlen) return;
    const int nin = FULL ? 4 : clamp4(d - c0);
    const int nout = FULL ? 4 : clamp4(mlen - c0);
    const int64_t rows = (int64_t)P * m;

    float4 ring[D];
    int64_t next = 0;  // next sample row to fetch
    const float* src = G + c0;
#pragma unroll
    for (int t = 0; t < D; ++t) {
        ring[t] = ldx<FULL>(src + next * ldg, nin);
        ++next;
    }
    auto unit_sum = [&]() -> double4 {  // the next unit gradient: its m rows, ascending, in fp64
        double4 acc = make_double4(0.0, 0.0, 0.0, 0.0);
        for (int t0 = 0; t0 < m; t0 += D) {
#pragma unroll
            for (int t = 0; t < D; ++t) {
                const float4 x = ring[t];
                if (next < rows) ring[t] = ldx<FULL>(src + next * ldg, nin);
                ++next;
                acc.x += (double)x.x;
                acc.y += (double)x.y;
                acc.z += (double)x.z;
                acc.w += (double)x.w;
            }
        }
        return acc;
    };
    double wre[R][2], wim[R][2];
    auto put = [&](int slot, const double4& v, int kappa) {
        rotate_in(tab, kappa, v.x, v.y, v.z, v.w, wre[slot], wim[slot]);
    };
#pragma unroll
    for (int k = 0; k < 2 * S; ++k) {
        const double4 v = unit_sum();
        head[k * kBlock + threadIdx.x] = v;
        put(k, v, k);
    }
    for (int n0 = 0; n0 < P; n0 += R) {
#pragma unroll
        for (int uu = 0; uu < R; ++uu) {
            const int n = n0 + uu;
            if (n < P) {
                const int kk = n + 2 * S;
                const double4 v = kk < P ? unit_sum() : head[(kk - P) * kBlock + threadIdx.x];
                put((uu + 2 * S) % R, v, kk);
                double are0, aim0, are1, aim1;
                tap_sum<R>(tab, n, wre, wim, uu % R, are0, aim0, are1, aim1);
                const float4 hi = make_float4((float)are0, (float)aim0, (float)are1, (float)aim1);
                stx<FULL>(Z + (int64_t)n * ldm + c0, hi, nout);
                if constexpr (LO != kLoNone) {
                    const float4 lo = make_float4((float)(are0 - (double)hi.x), (float)(aim0 - (double)hi.y),
                                                  (float)(are1 - (double)hi.z), (float)(aim1 - (double)hi.w));
                    st_lo<FULL, LO>(Zlo, (int64_t)n * ldm + c0, hi, lo, nout);
                }
            }
        }
    }
}

// m = 4 (the paper's B = 180 on P = 45): two units, eight rows, in flight.  Row i sits in ring
// slot i mod 8 = 4 (k mod 2) + t for row t of unit k, so the half a unit reads is fixed by the
// parity of k; the node loop is unrolled over 2R nodes to make that parity static.
template <int S, bool FULL, int LO>
__device__ __forceinline__ void encode_cyc_multi_four_body(const float* __restrict__ G, int64_t ldg,
                                                           float* __restrict__ Z, float* __restrict__ Zlo,
                                                           int64_t ldm, const CycTaps tab, int P,
                                                           int64_t d, double4* head /* LDS [2S][kBlock] */) {
    constexpr int R = 2 * S + 1;
    const int64_t c0 = lane_column<kSpreadEncodeCyc>();
    const int64_t mlen = 2 * ((d + 1) / 2);
    if (!FULL && c0 >= mlen) return;
    const int nin = FULL ? 4 : clamp4(d - c0);
    const int nout = FULL ? 4 : clamp4(mlen - c0);
    const int64_t rows = (int64_t)P * 4;

    float4 ring[8];
    int64_t next = 0;  // next sample row to fetch
    const float* src = G + c0;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        if (next < rows) ring[t] = ldx<FULL>(src + next * ldg, nin);
        ++next;
    }
    auto unit_sum = [&](auto parity) -> double4 {  // the next unit gradient: its 4 rows, ascending, in fp64
        constexpr int H = 4 * decltype(parity)::value;
        double4 acc = make_double4(0.0, 0.0, 0.0, 0.0);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const float4 x = ring[H + t];
            if (next < rows) ring[H + t] = ldx<FULL>(src + next * ldg, nin);
            ++next;
            acc.x += (double)x.x;
            acc.y += (double)x.y;
            acc.z += (double)x.z;
            acc.w += (double)x.w;
        }
        return acc;
    };
    double wre[R][2], wim[R][2];
    auto put = [&](int slot, const double4& v, int kappa) {
        rotate_in(tab, kappa, v.x, v.y, v.z, v.w, wre[slot], wim[slot]);
    };
#pragma unroll
    for (int k = 0; k < 2 * S; ++k) {
        double4 v;
        if (k % 2 == 0) v = unit_sum(std::integral_constant<int, 0>());
        else v = unit_sum(std::integral_constant<int, 1>());
        head[k * kBlock + threadIdx.x] = v;
        put(k, v, k);
    }
    for (int n0 = 0; n0 < P; n0 += 2 * R) {
#pragma unroll
        for (int uu = 0; uu < 2 * R; ++uu) {
            const int n = n0 + uu;
            if (n < P) {
                const int kk = n + 2 * S;   // same parity as uu: n0 and 2S are even
                double4 v;
                if (kk >= P) v = head[(kk - P) * kBlock + threadIdx.x];
                else if (uu % 2 == 0) v = unit_sum(std::integral_constant<int, 0>());
                else v = unit_sum(std::integral_constant<int, 1>());
                put((uu + 2 * S) % R, v, kk);
                double are0, aim0, are1, aim1;
                tap_sum<R>(tab, n, wre, wim, uu % R, are0, aim0, are1, aim1);
                const float4 hi = make_float4((float)are0, (float)aim0, (float)are1, (float)aim1);
                stx<FULL>(Z + (int64_t)n * ldm + c0, hi, nout);
                if constexpr (LO != kLoNone) {
                    const float4 lo = make_float4((float)(are0 - (double)hi.x), (float)(aim0 - (double)hi.y),
                                                  (float)(are1 - (double)hi.z), (float)(aim1 - (double)hi.w));
                    st_lo<FULL, LO>(Zlo, (int64_t)n * ldm + c0, hi, lo, nout);
                }
            }
        }
    }
}

template <int S, int LO>
__global__ __launch_bounds__(kBlock) void encode_cyc_multi_four_kernel(const float* __restrict__ G, int64_t ldg,
                                                                       float* __restrict__ Z, float* __restrict__ Zlo,
                                                                       int64_t ldm, const CycTaps tab,
                                                                       int P, int64_t d) {
    extern __shared__ double4 head_sums[];  // [2S][kBlock]
    if (block_is_full<kSpreadEncodeCyc>(d))
        encode_cyc_multi_four_body<S, true, LO>(G, ldg, Z, Zlo, ldm, tab, P, d, head_sums);
    else
        encode_cyc_multi_four_body<S, false, LO>(G, ldg, Z, Zlo, ldm, tab, P, d, head_sums);
}

template <int S, int D, int LO>
__global__ __launch_bounds__(kBlock) void encode_cyc_multi_ring_kernel(const float* __restrict__ G, int64_t ldg, int m,
                                                                       float* __restrict__ Z, float* __restrict__ Zlo,
                                                                       int64_t ldm, const CycTaps tab,
                                                                       int P, int64_t d) {
    extern __shared__ double4 head_sums[];  // [2S][kBlock]
    if (block_is_full<kSpreadEncodeCyc>(d))
        encode_cyc_multi_ring_body<S, D, true, LO>(G, ldg, m, Z, Zlo, ldm, tab, P, d, head_sums);
    else
        encode_cyc_multi_ring_body<S, D, false, LO>(G, ldg, m, Z, Zlo, ldm, tab, P, d, head_sums);
}

template <int S, int LO>
__global__ __launch_bounds__(kBlock) void encode_cyc_multi_kernel(const float* __restrict__ G, int64_t ldg, int m,
                                                                  float* __restrict__ Z, float* __restrict__ Zlo,
                                                                  int64_t ldm, const CycTaps tab,
                                                                  int P, int64_t d) {
    extern __shared__ double4 head_sums[];  // [2S][kBlock]
    if (block_is_full<kSpreadEncodeCyc>(d)) encode_cyc_multi_body<S, true, LO>(G, ldg, m, Z, Zlo, ldm, tab, P, d, head_sums);
    else encode_cyc_multi_body<S, false, LO>(G, ldg, m, Z, Zlo, ldm, tab, P, d, head_sums);
}


// Launch of the all-node encoder for one s (defined in the translation unit of that s).
// one_per_cu selects the launch shape: one workgroup per CU with deep prefetch, or two.
// lo: format of the second word (kLoF32 / kLoBf16) when Zlo is not null.
template <int S>
hipError_t launch_encode_cyc_s(bool one_per_cu, dim3 grid, hipStream_t stream, const float* G, int64_t ldg, float* Z,
                               float* Zlo, int lo, int64_t ldm, const CycTaps& tab, int P, int64_t d);
// Same for the unpacked wire (real gradients in, d complex entries out).
template <int S>
hipError_t launch_encode_cyc_real_s(bool one_per_cu, dim3 grid, hipStream_t stream, const float* G, int64_t ldg,
                                    float* Z, int64_t ldm, const double2* coef, int P, int64_t d);
// Same for the B > P form (m per-sample rows per unit gradient).
template <int S>
hipError_t launch_encode_cyc_multi_s(dim3 grid, hipStream_t stream, const float* G, int64_t ldg, int m, float* Z,
                                     float* Zlo, int lo, int64_t ldm, const CycTaps& tab, int P, int64_t d);

}  // namespace draco
