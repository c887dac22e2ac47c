// Cyclic code (Sec. 3, "Cyclic Code"): dispatch of the encoder E^Cyc, z_j = G W_{.,j},
// over the window width, and the one-node / any-width kernel.
#include "cyc_encode_kernels.hpp"
#include "cyc_encode_narrow.hpp"

namespace draco {

namespace {

// Windows of 23 to 33 gradients (11 <= s <= 16): the one-complex-per-lane kernel.
hipError_t launch_narrow(int s, bool real, hipStream_t stream, const float* G, int64_t ldg, int m, float* Z, float* Zlo,
                         int lo, int64_t ldm, const double2* coef, const CycTaps& tab, int P, int64_t d) {
    switch (s) {
        case 11: return launch_encode_cyc_narrow_s<11>(real, stream, G, ldg, m, Z, Zlo, lo, ldm, coef, tab, P, d);
        case 12: return launch_encode_cyc_narrow_s<12>(real, stream, G, ldg, m, Z, Zlo, lo, ldm, coef, tab, P, d);
        case 13: return launch_encode_cyc_narrow_s<13>(real, stream, G, ldg, m, Z, Zlo, lo, ldm, coef, tab, P, d);
        case 14: return launch_encode_cyc_narrow_s<14>(real, stream, G, ldg, m, Z, Zlo, lo, ldm, coef, tab, P, d);
        case 15: return launch_encode_cyc_narrow_s<15>(real, stream, G, ldg, m, Z, Zlo, lo, ldm, coef, tab, P, d);
        case 16: return launch_encode_cyc_narrow_s<16>(real, stream, G, ldg, m, Z, Zlo, lo, ldm, coef, tab, P, d);
        default: return hipErrorInvalidValue;
    }
}
constexpr int kMaxNarrowS = 16;

}  // namespace

// One node: z = A_node * sum_t rho_t * (B_{node+t} g_t), W in the factored form the all-node
// kernels use (tap_sum in cyc_encode_kernels.hpp); each tap rotates its row as it reads it.  With
// wrap_rows == 0, Gn holds only the node's r gradients in assignment order;
// with wrap_rows == P it is the full [P][ldg] slab and row (node+t) mod P is
// used (the all-node path for r > 2*kMaxCycS+1).  Same operation order as the
// all-node kernel, so results are bit-identical.  The second word, if any, goes to
// element lo_off + column of the slab zlo, in the format lo.
__global__ __launch_bounds__(kBlock) void encode_cyc_node_kernel(const float* __restrict__ Gn, int64_t ldg,
                                                                 float* __restrict__ z, float* __restrict__ zlo,
                                                                 int64_t lo_off, int lo,
                                                                 const CycTaps tab, int node, int P,
                                                                 int r, int wrap_rows, int m, int64_t d) {
    const int64_t c0 = lane_column<kSpreadEncodeCyc>();
    const int64_t mlen = 2 * ((d + 1) / 2);
    if (c0 >= mlen) return;
    const int nin = clamp4(d - c0);
    const int nout = clamp4(mlen - c0);
    double sr0 = 0.0, si0 = 0.0, sr1 = 0.0, si1 = 0.0;
    for (int t = 0; t < r; ++t) {
        int k = node + t;
        if (k >= P) k -= P;
        const float* p = Gn + (int64_t)(wrap_rows ? k : t) * m * ldg + c0;
        double gx = 0.0, gy = 0.0, gz = 0.0, gw = 0.0;  // the unit gradient: sum of its m sample rows
        for (int i = 0; i < m; ++i) {
            const float4 raw = (nin == 4) ? ld4(p + (int64_t)i * ldg) : ld4_partial(p + (int64_t)i * ldg, nin);
            gx += (double)raw.x;
            gy += (double)raw.y;
            gz += (double)raw.z;
            gw += (double)raw.w;
        }
        double re[2], im[2];
        rotate_in(tab, node + t, gx, gy, gz, gw, re, im);
        const double rho = tab.rho[t];
        sr0 = fma(rho, re[0], sr0);
        si0 = fma(rho, im[0], si0);
        sr1 = fma(rho, re[1], sr1);
        si1 = fma(rho, im[1], si1);
    }
    double are0, aim0, are1, aim1;
    const double2 A = tab.rotA[node];
    cmul(A.x, A.y, sr0, si0, are0, aim0);
    cmul(A.x, A.y, sr1, si1, are1, aim1);
    const float4 out = make_float4((float)are0, (float)aim0, (float)are1, (float)aim1);
    if (nout == 4) st4(z + c0, out);
    else st4_partial(z + c0, out, nout);
    if (zlo != nullptr) {
        const float4 lo4 = make_float4((float)(are0 - (double)out.x), (float)(aim0 - (double)out.y),
                                       (float)(are1 - (double)out.z), (float)(aim1 - (double)out.w));
        if (nout == 4) st_lo_rt<true>(zlo, lo_off + c0, out, lo4, nout, lo);
        else st_lo_rt<false>(zlo, lo_off + c0, out, lo4, nout, lo);
    }
}



// All nodes for any window width r = 2s+1 (used beyond s = 16, where no register-window
// kernel is instantiated): the window lives in LDS as a ring of r raw rows per lane (each lane reads back
// only what it wrote: no barrier), rows are fetched Q ahead into registers, and the last
// 2s nodes re-read rows 0..2s-1 from memory (2s/P more reads than the register kernels).
// Same operation order as the one-node kernel: results are bit-identical to it.
template <int TB, bool FULL>
__device__ __forceinline__ void encode_cyc_ring_body(const float* __restrict__ G, int64_t ldg,
                                                     float* __restrict__ Z, float* __restrict__ Zlo, int lo, int64_t ldm,
                                                     const CycTaps tab, int P, int r, int64_t d,
                                                     float4* ring /* LDS [r][TB] */) {
    constexpr int Q = 4;
    const int64_t c0 = ((int64_t)blockIdx.x * TB + threadIdx.x) * 4;
    const int64_t mlen = 2 * ((d + 1) / 2);
    if (!FULL && c0 >= mlen) return;
    const int nin = FULL ? 4 : clamp4(d - c0);
    const int nout = FULL ? 4 : clamp4(mlen - c0);
    float4* mine = ring + threadIdx.x;
    auto fetch = [&](int row) -> float4 {  // row index may run past P: the circle wraps
        if (row >= P) row -= P;
        return ldx<FULL>(G + (int64_t)row * ldg + c0, nin);
    };
    for (int k = 0; k < r - 1; ++k) mine[k * TB] = fetch(k);
    float4 ahead[Q];  // rows n+r-1 .. n+r-1+Q-1 for the current n
#pragma unroll
    for (int q = 0; q < Q; ++q) ahead[q] = fetch(r - 1 + q);
    int first = 0;      // ring slot of row n
    int last = r - 1;   // ring slot that receives row n+r-1
    for (int n0 = 0; n0 < P; n0 += Q) {
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            const int n = n0 + q;
            if (n < P) {
                mine[last * TB] = ahead[q];
                if (n + Q < P) ahead[q] = fetch(n + Q + r - 1);
                double sr0 = 0.0, si0 = 0.0, sr1 = 0.0, si1 = 0.0;
                int slot = first;
                for (int t = 0; t < r; ++t) {
                    const float4 x = mine[slot * TB];
                    double re[2], im[2];
                    rotate_in(tab, n + t, (double)x.x, (double)x.y, (double)x.z, (double)x.w, re, im);
                    const double rho = tab.rho[t];
                    sr0 = fma(rho, re[0], sr0);
                    si0 = fma(rho, im[0], si0);
                    sr1 = fma(rho, re[1], sr1);
                    si1 = fma(rho, im[1], si1);
                    if (++slot == r) slot = 0;
                }
                double are0, aim0, are1, aim1;
                const double2 A = tab.rotA[n];
                cmul(A.x, A.y, sr0, si0, are0, aim0);
                cmul(A.x, A.y, sr1, si1, are1, aim1);
                const float4 hi = make_float4((float)are0, (float)aim0, (float)are1, (float)aim1);
                stx<FULL>(Z + (int64_t)n * ldm + c0, hi, nout);
                if (Zlo != nullptr) {
                    const float4 lo4 = make_float4((float)(are0 - (double)hi.x), (float)(aim0 - (double)hi.y),
                                                   (float)(are1 - (double)hi.z), (float)(aim1 - (double)hi.w));
                    st_lo_rt<FULL>(Zlo, (int64_t)n * ldm + c0, hi, lo4, nout, lo);
                }
                if (++first == r) first = 0;
                if (++last == r) last = 0;
            }
        }
    }
}

template <int TB>
__global__ __launch_bounds__(TB) void encode_cyc_ring_kernel(const float* __restrict__ G, int64_t ldg,
                                                                 float* __restrict__ Z, float* __restrict__ Zlo,
                                                                 int lo, int64_t ldm,
                                                                 const CycTaps tab, int P, int r,
                                                                 int64_t d) {
    extern __shared__ float4 ring[];  // [r][TB]
    if ((int64_t)(blockIdx.x + 1) * (TB * 4) <= d) encode_cyc_ring_body<TB, true>(G, ldg, Z, Zlo, lo, ldm, tab, P, r, d, ring);
    else encode_cyc_ring_body<TB, false>(G, ldg, Z, Zlo, lo, ldm, tab, P, r, d, ring);
}

// One node on the unpacked wire (real gradients, d complex entries out), any window width:
// with wrap_rows == 0 Gn holds only the node's r gradients in assignment order, with
// wrap_rows == P it is the full slab (the all-node path for r > 2*kMaxCycS+1).  Same operation order as the windowed kernel.
__global__ __launch_bounds__(kBlock) void encode_cyc_real_node_kernel(const float* __restrict__ G, int64_t ldg,
                                                                      float* __restrict__ z,
                                                                      const double2* __restrict__ cn, int node,
                                                                      int P, int r, int wrap_rows, int64_t d) {
    const int64_t c0 = lane_column<kSpreadEncodeCyc>();
    if (c0 >= d) return;
    const int nin = clamp4(d - c0);
    double re[4] = {0.0, 0.0, 0.0, 0.0}, im[4] = {0.0, 0.0, 0.0, 0.0};
    for (int t = 0; t < r; ++t) {
        int k = node + t;
        if (k >= P) k -= P;
        const float* p = G + (int64_t)(wrap_rows ? k : t) * ldg + c0;
        const float4 raw = (nin == 4) ? ld4(p) : ld4_partial(p, nin);
        const double g[4] = {(double)raw.x, (double)raw.y, (double)raw.z, (double)raw.w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            re[c] = fma(cn[t].x, g[c], re[c]);
            im[c] = fma(cn[t].y, g[c], im[c]);
        }
    }
    float* dst = z + 2 * c0;
    st4_partial(dst, make_float4((float)re[0], (float)im[0], (float)re[1], (float)im[1]), clamp4(2 * (int64_t)nin));
    st4_partial(dst + 4, make_float4((float)re[2], (float)im[2], (float)re[3], (float)im[3]),
                clamp4(2 * (int64_t)nin - 4));
}


// ---------------------------------------------------------------------------
// Launchers
// ---------------------------------------------------------------------------

hipError_t launch_encode_cyc(const float* G, int64_t ldg, float* Z, float* Zlo, int lo, int64_t ldm, const CycTaps& tab,
                             int P, int s, int64_t d, hipStream_t stream) {
    const int64_t mlen = 2 * ((d + 1) / 2);
    const dim3 grid(grid_cols<kSpreadEncodeCyc>(mlen)), block(kBlock);
    const int r = 2 * s + 1;
    const bool one_per_cu = s <= 3 && P >= 32;
    if (s > kMaxCycS && s <= kMaxNarrowS) return launch_narrow(s, false, stream, G, ldg, 1, Z, Zlo, lo, ldm, nullptr, tab, P, d);
#define DRACO_CASE(S) \
    case S: return launch_encode_cyc_s<S>(one_per_cu, grid, stream, G, ldg, Z, Zlo, lo, ldm, tab, P, d);
    switch (s) {
        DRACO_CASE(0) DRACO_CASE(1) DRACO_CASE(2) DRACO_CASE(3) DRACO_CASE(4) DRACO_CASE(5) DRACO_CASE(6) DRACO_CASE(7)
        DRACO_CASE(8) DRACO_CASE(9) DRACO_CASE(10)
        default: {
            // one wavefront per workgroup: the ring is r KiB, so a CU holds 160/r of them and
            // has that many wavefronts to hide the LDS and scalar-load latency of the tap loop
            constexpr int TB = 64;
            const size_t ring_bytes = (size_t)r * TB * sizeof(float4);
            if (ring_bytes <= lds_per_cu()) {
                allow_large_lds<encode_cyc_ring_kernel<TB>>();
                const dim3 g64((unsigned)(((mlen + 3) / 4 + TB - 1) / TB));
                hipLaunchKernelGGL(encode_cyc_ring_kernel<TB>, g64, dim3(TB), ring_bytes, stream, G, ldg, Z, Zlo, lo,
                                   ldm, tab, P, r, d);
            } else {  // windows too wide for LDS: one launch per node
                for (int j = 0; j < P; ++j)
                    hipLaunchKernelGGL(encode_cyc_node_kernel, grid, block, 0, stream, G, ldg, Z + (int64_t)j * ldm,
                                       Zlo, (int64_t)j * ldm, lo, tab, j, P, r, P, 1, d);
            }
        }
    }
#undef DRACO_CASE
    return hipGetLastError();
}

hipError_t launch_encode_cyc_real(const float* G, int64_t ldg, float* Z, int64_t ldm, const double2* coef, int P,
                                  int s, int64_t d, hipStream_t stream) {
    const dim3 grid(grid_cols<kSpreadEncodeCyc>(d)), block(kBlock);
    const int r = 2 * s + 1;
    const bool one_per_cu = s <= 3 && P >= 32;
    if (s > kMaxCycS && s <= kMaxNarrowS) return launch_narrow(s, true, stream, G, ldg, 1, Z, nullptr, kLoNone, ldm, coef, CycTaps{nullptr, nullptr, nullptr}, P, d);
#define DRACO_CASE(S) \
    case S: return launch_encode_cyc_real_s<S>(one_per_cu, grid, stream, G, ldg, Z, ldm, coef, P, d);
    switch (s) {
        DRACO_CASE(0) DRACO_CASE(1) DRACO_CASE(2) DRACO_CASE(3) DRACO_CASE(4) DRACO_CASE(5) DRACO_CASE(6) DRACO_CASE(7)
        DRACO_CASE(8) DRACO_CASE(9) DRACO_CASE(10)
        default:
            for (int j = 0; j < P; ++j)
                hipLaunchKernelGGL(encode_cyc_real_node_kernel, grid, block, 0, stream, G, ldg, Z + (int64_t)j * ldm,
                                   coef + (int64_t)j * r, j, P, r, P, d);
    }
#undef DRACO_CASE
    return hipGetLastError();
}

hipError_t launch_encode_cyc_samples(const float* G, int64_t ldg, int m, float* Z, float* Zlo, int lo, int64_t ldm,
                                     const CycTaps& tab, int P, int s, int64_t d, hipStream_t stream) {
    const int64_t mlen = 2 * ((d + 1) / 2);
    const dim3 grid(grid_cols<kSpreadEncodeCyc>(mlen)), block(kBlock);
    const int r = 2 * s + 1;
    if (s > kMaxCycS && s <= kMaxNarrowS) return launch_narrow(s, false, stream, G, ldg, m, Z, Zlo, lo, ldm, nullptr, tab, P, d);
#define DRACO_CASE(S) \
    case S: return launch_encode_cyc_multi_s<S>(grid, stream, G, ldg, m, Z, Zlo, lo, ldm, tab, P, d);
    switch (s) {
        DRACO_CASE(0) DRACO_CASE(1) DRACO_CASE(2) DRACO_CASE(3) DRACO_CASE(4) DRACO_CASE(5) DRACO_CASE(6) DRACO_CASE(7)
        DRACO_CASE(8) DRACO_CASE(9) DRACO_CASE(10)
        default:
            for (int j = 0; j < P; ++j)
                hipLaunchKernelGGL(encode_cyc_node_kernel, grid, block, 0, stream, G, ldg, Z + (int64_t)j * ldm,
                                   Zlo, (int64_t)j * ldm, lo, tab, j, P, r, P, m, d);
    }
#undef DRACO_CASE
    return hipGetLastError();
}

hipError_t launch_encode_cyc_real_node(const float* Gn, int64_t ldg, float* z, const double2* coef, int node, int P,
                                       int s, int64_t d, hipStream_t stream) {
    const dim3 grid(grid_cols<kSpreadEncodeCyc>(d)), block(kBlock);
    const int r = 2 * s + 1;
    hipLaunchKernelGGL(encode_cyc_real_node_kernel, grid, block, 0, stream, Gn, ldg, z, coef + (int64_t)node * r, node,
                       P, r, 0, d);
    return hipGetLastError();
}

hipError_t launch_encode_cyc_node(const float* Gn, int64_t ldg, float* z, float* zlo, int lo, const CycTaps& tab,
                                  int node, int P, int s, int64_t d, hipStream_t stream) {
    const int64_t mlen = 2 * ((d + 1) / 2);
    const dim3 grid(grid_cols<kSpreadEncodeCyc>(mlen)), block(kBlock);
    const int r = 2 * s + 1;
    hipLaunchKernelGGL(encode_cyc_node_kernel, grid, block, 0, stream, Gn, ldg, z, zlo, (int64_t)0, lo,
                       tab, node, P, r, 0, 1, d);
    return hipGetLastError();
}

}  // namespace draco
