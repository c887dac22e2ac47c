// Cyclic code: the two streaming passes of the decoder D^Cyc (Algorithm 1) -- the
// projection f R of phi and the recombination R_{.,U} b -- and the plain copy kernel
// used for calibration.
#include "device_util.hpp"
#include "projection_rng.hpp"

namespace draco {

// phi step 1: gamma'_j = sum_i f_i * r_j[i].  A workgroup owns a tile of
// kBlock*kProjectLoads float4 (two complex numbers each) of every row, keeps
// its slice of f in registers, and for each row forms a per-wavefront sum in
// fp64; the four wavefront sums are added in fixed order and stored per tile.
//
// Speculation (SPEC): while a row is in registers the kernel also accumulates
// u0 = sum_j b0_j r_j with b0 the recombination vector for "no adversary", and writes it to
// the output.  If the locator then finds no adversary -- the usual case in training -- u0 IS
// the decoded sum (same coefficients, same order, same instruction sequence as the
// recombination kernel) and the second pass over the messages is skipped.
template <int LO, bool SPEC>
__device__ __forceinline__ void cyc_project_body(const float* __restrict__ Rm, const float* __restrict__ Rlo,
                                                 int64_t ldm, const float* __restrict__ f, uint64_t f_seed,
                                                 double2* __restrict__ partial, const double2* __restrict__ b0,
                                                 float* __restrict__ u, bool realout, int P, int64_t d,
                                                 double2 (*wsum)[kMaxNodes]) {
    constexpr int K = kProjectLoads;
    const int64_t h = (d + 1) / 2;                                   // complex numbers per row
    const int64_t q0 = (int64_t)blockIdx.x * (kBlock * K) + threadIdx.x;  // my first float4
    const bool tile_full = ((int64_t)(blockIdx.x + 1) * (kBlock * K)) * 2 <= h;
    double f0[K], f1[K];
    int nflt[K];  // message floats that exist in my k-th float4 (4, 2 or 0)
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int64_t q = q0 + (int64_t)k * kBlock;
        const int64_t c = 2 * q;  // first complex index
        if (f != nullptr) {
            f0[k] = (c < h) ? (double)f[c] : 0.0;
            f1[k] = (c + 1 < h) ? (double)f[c + 1] : 0.0;
        } else {  // no stored vector: make the two entries (once per tile, reused for all P rows)
            f0[k] = (c < h) ? (double)projection_entry(f_seed, (uint64_t)c) : 0.0;
            f1[k] = (c + 1 < h) ? (double)projection_entry(f_seed, (uint64_t)(c + 1)) : 0.0;
        }
        nflt[k] = (c + 1 < h) ? 4 : (c < h ? 2 : 0);
    }
    double ure0[SPEC ? K : 1], uim0[SPEC ? K : 1], ure1[SPEC ? K : 1], uim1[SPEC ? K : 1];
    if constexpr (SPEC) {
#pragma unroll
        for (int k = 0; k < K; ++k) ure0[k] = uim0[k] = ure1[k] = uim1[k] = 0.0;
    }
    const int wave = threadIdx.x >> 6;
    for (int j = 0; j < P; ++j) {
        const float* row = Rm + (int64_t)j * ldm + q0 * 4;
        float4 x[K];
        if (tile_full) {
#pragma unroll
            for (int k = 0; k < K; ++k) x[k] = ld4(row + (int64_t)k * kBlock * 4);
        } else {
#pragma unroll
            for (int k = 0; k < K; ++k) x[k] = ld4_partial(row + (int64_t)k * kBlock * 4, nflt[k]);
        }
        double xr0[K], xi0[K], xr1[K], xi1[K];  // the wire values in fp64 (hi + lo is exact)
        if constexpr (LO != kLoNone) {
            const int64_t rowl = (int64_t)j * ldm + q0 * 4;
            lo_raw_t<LO> xl[K];
            if (tile_full) {
#pragma unroll
                for (int k = 0; k < K; ++k) xl[k] = ld_lo<true, LO>(Rlo, rowl + (int64_t)k * kBlock * 4, 4);
            } else {
#pragma unroll
                for (int k = 0; k < K; ++k) xl[k] = ld_lo<false, LO>(Rlo, rowl + (int64_t)k * kBlock * 4, nflt[k]);
            }
#pragma unroll
            for (int k = 0; k < K; ++k) {
                const float4 l = lo_values<LO>(xl[k], x[k]);
                xr0[k] = (double)x[k].x + (double)l.x;
                xi0[k] = (double)x[k].y + (double)l.y;
                xr1[k] = (double)x[k].z + (double)l.z;
                xi1[k] = (double)x[k].w + (double)l.w;
            }
        } else {
#pragma unroll
            for (int k = 0; k < K; ++k) {
                xr0[k] = (double)x[k].x;
                xi0[k] = (double)x[k].y;
                xr1[k] = (double)x[k].z;
                xi1[k] = (double)x[k].w;
            }
        }
        double are = 0.0, aim = 0.0;
#pragma unroll
        for (int k = 0; k < K; ++k) {
            are = fma(f0[k], xr0[k], are);
            aim = fma(f0[k], xi0[k], aim);
            are = fma(f1[k], xr1[k], are);
            aim = fma(f1[k], xi1[k], aim);
        }
        if constexpr (SPEC) {
            const double br = b0[j].x, bi = b0[j].y;
#pragma unroll
            for (int k = 0; k < K; ++k) {
                cmac(br, bi, xr0[k], xi0[k], ure0[k], uim0[k]);
                cmac(br, bi, xr1[k], xi1[k], ure1[k], uim1[k]);
            }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            are += __shfl_xor(are, off);
            aim += __shfl_xor(aim, off);
        }
        if ((threadIdx.x & 63) == 0) wsum[wave][j] = make_double2(are, aim);
    }
    if constexpr (SPEC) {
#pragma unroll
        for (int k = 0; k < K; ++k) {
            const int64_t c0 = (q0 + (int64_t)k * kBlock) * 4;
            if (realout) {  // unpacked wire: the sum is the real part, one float per complex entry
                const int64_t c = c0 / 2;
                if (c < h) u[c] = (float)ure0[k];
                if (c + 1 < h) u[c + 1] = (float)ure1[k];
            } else {
                const int nout = clamp4(d - c0);
                const float4 out = make_float4((float)ure0[k], (float)uim0[k], (float)ure1[k], (float)uim1[k]);
                if (nout == 4) st4(u + c0, out);
                else st4_partial(u + c0, out, nout);
            }
        }
    }
    __syncthreads();
    if ((int)threadIdx.x < P) {
        double2 a = wsum[0][threadIdx.x];
#pragma unroll
        for (int w = 1; w < kBlock / 64; ++w) {
            a.x += wsum[w][threadIdx.x].x;
            a.y += wsum[w][threadIdx.x].y;
        }
        partial[(int64_t)blockIdx.x * P + threadIdx.x] = a;
    }
}

// spec_state[0]: speculate in this call (set by the previous call's locator: 1 if that decode was
// clean); spec_state[1]: whether this call speculated (read by the recombination kernel).
// spec_state == nullptr: never speculate.
template <int LO>
__global__ __launch_bounds__(kBlock) void cyc_project_kernel(const float* __restrict__ Rm,
                                                             const float* __restrict__ Rlo, int64_t ldm,
                                                             const float* __restrict__ f, uint64_t f_seed,
                                                             double2* __restrict__ partial,
                                                             const double2* __restrict__ b0, float* __restrict__ u,
                                                             int realout, int32_t* __restrict__ spec_state, int P,
                                                             int64_t d) {
    __shared__ double2 wsum[kBlock / 64][kMaxNodes];
    const bool spec = spec_state != nullptr && spec_state[0] != 0;
    if (blockIdx.x == 0 && threadIdx.x == 0 && spec_state != nullptr) spec_state[1] = spec ? 1 : 0;
    if (spec) cyc_project_body<LO, true>(Rm, Rlo, ldm, f, f_seed, partial, b0, u, realout != 0, P, d, wsum);
    else cyc_project_body<LO, false>(Rm, Rlo, ldm, f, f_seed, partial, b0, u, false, P, d, wsum);
}

// gamma[j] = sum over tiles of partial[tile][j], in a fixed order.
__global__ __launch_bounds__(kBlock) void cyc_project_reduce_kernel(const double2* __restrict__ partial,
                                                                    double2* __restrict__ gamma, int P,
                                                                    int64_t tiles) {
    __shared__ double2 sm[kBlock];
    const int j = blockIdx.x;
    double2 a = make_double2(0.0, 0.0);
    for (int64_t t = threadIdx.x; t < tiles; t += kBlock) {
        const double2 p = partial[t * P + j];
        a.x += p.x;
        a.y += p.y;
    }
    sm[threadIdx.x] = a;
    __syncthreads();
    for (int off = kBlock / 2; off >= 1; off >>= 1) {
        if ((int)threadIdx.x < off) {
            sm[threadIdx.x].x += sm[threadIdx.x + off].x;
            sm[threadIdx.x].y += sm[threadIdx.x + off].y;
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) gamma[j] = sm[0];
}

constexpr int kRecombineRows = 6;      // message rows a lane has in flight (one word per float)
constexpr int kRecombineRowsWide = 3;  // the same on the two-word wire (two loads per row)
constexpr int kRecombineRowsBf16 = 3;  // and with a bfloat16 second word (a 16- and an 8-byte load per row)
constexpr int kRecombineRowsI8 = 2;    // and with an 8-bit one (a 16- and a 4-byte load per row)

// u = R_{.,U} b on packed complex messages, unpacked to reals: honest rows in
// ascending node order, fp64 accumulation, one rounding to fp32.
template <bool FULL, int LO, int UN>
__device__ __forceinline__ void cyc_recombine_body(const float* __restrict__ Rm, const float* __restrict__ Rlo,
                                                   int64_t ldm,
                                                   const double2* __restrict__ b, const int32_t* __restrict__ idx,
                                                   const int32_t* __restrict__ nu_ptr, float* __restrict__ u,
                                                   bool realout, int64_t d) {
    const int nu = *nu_ptr;  // honest nodes; written by the locator (device) or copied in by the host path
    const int64_t c0 = lane_column<kSpreadRecombine>();
    if (!FULL && c0 >= d) return;
    const int64_t mlen = 2 * ((d + 1) / 2);
    const int nin = FULL ? 4 : clamp4(mlen - c0);
    const int nout = FULL ? 4 : clamp4(d - c0);
    double are0 = 0.0, aim0 = 0.0, are1 = 0.0, aim1 = 0.0;
    for (int q0 = 0; q0 < nu; q0 += UN) {
        float4 x[UN];
        lo_raw_t<LO> xl[LO != kLoNone ? UN : 1];
#pragma unroll
        for (int i = 0; i < UN; ++i) {
            if (q0 + i < nu) {
                x[i] = ldx<FULL>(Rm + (int64_t)idx[q0 + i] * ldm + c0, nin);
                if constexpr (LO != kLoNone) xl[i] = ld_lo<FULL, LO>(Rlo, (int64_t)idx[q0 + i] * ldm + c0, nin);
            }
        }
#pragma unroll
        for (int i = 0; i < UN; ++i) {
            if (q0 + i < nu) {
                const double br = b[q0 + i].x, bi = b[q0 + i].y;
                if constexpr (LO != kLoNone) {
                    const float4 l = lo_values<LO>(xl[i], x[i]);
                    cmac(br, bi, (double)x[i].x + (double)l.x, (double)x[i].y + (double)l.y, are0, aim0);
                    cmac(br, bi, (double)x[i].z + (double)l.z, (double)x[i].w + (double)l.w, are1, aim1);
                } else {
                    cmac(br, bi, (double)x[i].x, (double)x[i].y, are0, aim0);
                    cmac(br, bi, (double)x[i].z, (double)x[i].w, are1, aim1);
                }
            }
        }
    }
    if (realout) {  // unpacked wire: the sum is the real part, one float per complex entry
        const int64_t c = c0 / 2;
        if (FULL || 2 * c < d) u[c] = (float)are0;
        if (FULL || 2 * c + 2 < d) u[c + 1] = (float)are1;
    } else {
        stx<FULL>(u + c0, make_float4((float)are0, (float)aim0, (float)are1, (float)aim1), nout);
    }
}

// If the projection pass speculated (spec_state[1]) and every node turned out honest
// (*nu == P), the output already holds the answer: nothing to do.
template <int LO, int UN>
__global__ __launch_bounds__(kBlock) void cyc_recombine_kernel(const float* __restrict__ Rm,
                                                               const float* __restrict__ Rlo, int64_t ldm,
                                                               const double2* __restrict__ b,
                                                               const int32_t* __restrict__ idx,
                                                               const int32_t* __restrict__ nu,
                                                               const int32_t* __restrict__ spec_state, int P,
                                                               float* __restrict__ u, int realout, int64_t d) {
    if (spec_state != nullptr && spec_state[1] != 0 && *nu == P) return;
    if (block_is_full<kSpreadRecombine>(d)) cyc_recombine_body<true, LO, UN>(Rm, Rlo, ldm, b, idx, nu, u, realout != 0, d);
    else cyc_recombine_body<false, LO, UN>(Rm, Rlo, ldm, b, idx, nu, u, realout != 0, d);
}

// Plain copy of a [rows][row_len] slab (row stride ld): the fastest copy of a row-major
// slab found on MI355X.  A workgroup moves one 4 KiB piece of one row and ends; column
// tiles vary fastest across the grid, so at any moment the chip streams one or two rows.
// Calibration kernel for bandwidth figures and for scaling hardware byte counters.
__global__ __launch_bounds__(kBlock) void copy_probe_kernel(const float* __restrict__ src, float* __restrict__ dst,
                                                            int rows, int64_t row_len, int64_t ld) {
    const int64_t c0 = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * 4;
    if (c0 + 4 > row_len || (int)blockIdx.y >= rows) return;
    const int64_t off = (int64_t)blockIdx.y * ld + c0;
    st4(dst + off, ld4(src + off));
}


// ---------------------------------------------------------------------------
// Launchers
// ---------------------------------------------------------------------------

int64_t project_tiles(int64_t d) {
    const int64_t h = (d + 1) / 2;
    const int64_t nvec = (h + 1) / 2;
    const int64_t per = (int64_t)kBlock * kProjectLoads;
    return (nvec + per - 1) / per;
}

hipError_t launch_cyc_project(const float* R, const float* Rlo, int lo, int64_t ldm, const float* f, uint64_t f_seed,
                              double2* partial, double2* gamma, const double2* b0, float* u, bool realout,
                              int32_t* spec_state, int P, int64_t d, hipStream_t stream) {
    const int64_t tiles = project_tiles(d);
    if (Rlo == nullptr)
        hipLaunchKernelGGL(cyc_project_kernel<kLoNone>, dim3((unsigned)tiles), dim3(kBlock), 0, stream, R, Rlo, ldm, f,
                           f_seed, partial, b0, u, realout ? 1 : 0, spec_state, P, d);
    else if (lo == kLoBf16)
        hipLaunchKernelGGL(cyc_project_kernel<kLoBf16>, dim3((unsigned)tiles), dim3(kBlock), 0, stream, R, Rlo, ldm, f,
                           f_seed, partial, b0, u, realout ? 1 : 0, spec_state, P, d);
    else if (lo == kLoI8)
        hipLaunchKernelGGL(cyc_project_kernel<kLoI8>, dim3((unsigned)tiles), dim3(kBlock), 0, stream, R, Rlo, ldm, f,
                           f_seed, partial, b0, u, realout ? 1 : 0, spec_state, P, d);
    else
        hipLaunchKernelGGL(cyc_project_kernel<kLoF32>, dim3((unsigned)tiles), dim3(kBlock), 0, stream, R, Rlo, ldm, f,
                           f_seed, partial, b0, u, realout ? 1 : 0, spec_state, P, d);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(cyc_project_reduce_kernel, dim3((unsigned)P), dim3(kBlock), 0, stream, partial, gamma, P, tiles);
    return hipGetLastError();
}

hipError_t launch_copy_probe(const float* src, float* dst, int rows, int64_t row_len, int64_t ld,
                             hipStream_t stream) {
    hipLaunchKernelGGL(copy_probe_kernel, dim3(grid_for(row_len / 4), (unsigned)rows), dim3(kBlock), 0, stream, src,
                       dst, rows, row_len, ld);
    return hipGetLastError();
}

hipError_t launch_cyc_recombine(const float* R, const float* Rlo, int lo, int64_t ldm, const double2* b, const int32_t* idx,
                                const int32_t* nu, const int32_t* spec_state, int P, float* u, bool realout,
                                int64_t d, hipStream_t stream) {
    const dim3 grid(grid_cols<kSpreadRecombine>(d)), block(kBlock);
    const size_t lds = throttle_lds(2, 0, 0);
    if (Rlo == nullptr) {
        allow_large_lds<cyc_recombine_kernel<kLoNone, kRecombineRows>>();
        hipLaunchKernelGGL((cyc_recombine_kernel<kLoNone, kRecombineRows>), grid, block, lds, stream, R, Rlo, ldm, b, idx,
                           nu, spec_state, P, u, realout ? 1 : 0, d);
    } else if (lo == kLoBf16) {
        // the 8-byte loads of the 16-bit slab want more wavefronts per CU: four workgroups run
        // at 0.82 of the HBM peak at (P, s, d) = (45, 3, 25.6 M), two at 0.69-0.76
        allow_large_lds<cyc_recombine_kernel<kLoBf16, kRecombineRowsBf16>>();
        hipLaunchKernelGGL((cyc_recombine_kernel<kLoBf16, kRecombineRowsBf16>), grid, block, throttle_lds(4, 0, 0), stream,
                           R, Rlo, ldm, b, idx, nu, spec_state, P, u, realout ? 1 : 0, d);
    } else if (lo == kLoI8) {
        // sweep at (45, 3, 25.6 M): 0.81 of the HBM peak with 4 workgroups x 2 rows (also 2 x 6 and 6 x 1)
        allow_large_lds<cyc_recombine_kernel<kLoI8, kRecombineRowsI8>>();
        hipLaunchKernelGGL((cyc_recombine_kernel<kLoI8, kRecombineRowsI8>), grid, block, throttle_lds(4, 0, 0), stream,
                           R, Rlo, ldm, b, idx, nu, spec_state, P, u, realout ? 1 : 0, d);
    } else {
        allow_large_lds<cyc_recombine_kernel<kLoF32, kRecombineRowsWide>>();
        hipLaunchKernelGGL((cyc_recombine_kernel<kLoF32, kRecombineRowsWide>), grid, block, lds, stream, R, Rlo, ldm, b,
                           idx, nu, spec_state, P, u, realout ? 1 : 0, d);
    }
    return hipGetLastError();
}


}  // namespace draco
