// Device-side phi and recombination vector of the cyclic code (Sec. 3, phi;
// Algorithm 1, lines 1-3): the same steps as host_math.cpp, run by ONE
// wavefront in fp64 so that a cyclic decode needs no host round trip.
//
//   gamma[P] (projections f R)  ->  mask words, status, and the honest nodes'
//   indices and coefficients b (compacted, ascending) for the recombination.
//
// Work distribution: a lane owns node j (j = lane, lane+64, ...) in the O(P)
// and O(P^2) loops, and owns one matrix row in the small dense algebra (the
// s x s system for beta, the 2s x |V| least-squares fits), whose inner
// products are wavefront reductions.  Limits: P <= 256, s <= kLocateMaxS.
#include "kernels.hpp"

namespace draco {

namespace {

constexpr int kW = 64;  // one wavefront

// Butterfly reductions over aligned groups of N lanes (every lane of a group gets the
// group's result).  The dense algebra only populates lanes < 2s <= 32 (or < s <= 16),
// so it reduces over 32 (or 16) lanes; lanes outside contribute zeros to their own group.
template <int N = kW>
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int off = N / 2; off >= 1; off >>= 1) v += __shfl_xor(v, off);
    return v;
}
template <int N = kW>
__device__ __forceinline__ double wave_max(double v) {
#pragma unroll
    for (int off = N / 2; off >= 1; off >>= 1) v = fmax(v, __shfl_xor(v, off));
    return v;
}
constexpr int kRowLanes = 2 * kLocateMaxS;  // lanes that can hold a row of a (2s) x a matrix
constexpr int kColLanes = kLocateMaxS;      // lanes that can hold a row of the s x s system
__device__ __forceinline__ double2 cmul(double2 a, double2 b) {
    return make_double2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x);
}
__device__ __forceinline__ double2 cconj(double2 a) { return make_double2(a.x, -a.y); }
__device__ __forceinline__ double2 cadd(double2 a, double2 b) { return make_double2(a.x + b.x, a.y + b.y); }
__device__ __forceinline__ double2 csub(double2 a, double2 b) { return make_double2(a.x - b.x, a.y - b.y); }
__device__ __forceinline__ double cnorm2(double2 a) { return a.x * a.x + a.y * a.y; }
__device__ __forceinline__ double2 cscale(double2 a, double s) { return make_double2(a.x * s, a.y * s); }

struct Smem {
    double2 root[kMaxNodes];  // exp(2 pi i k / P)
    double2 gam[kMaxNodes];
    double2 h[kMaxNodes];
    double mag[kMaxNodes];
    double2 A[kLocateMaxS * kLocateMaxS];      // column-major s x s
    double2 V[kLocateMaxS * kLocateMaxS];
    double2 Q[2 * kLocateMaxS * kLocateMaxS];   // column-major, leading dimension 2*kLocateMaxS, <= s columns
    double2 Rr[2 * kLocateMaxS * kLocateMaxS];  // upper triangular factor, same indexing
    double2 hk[2 * kLocateMaxS];
    double2 res[2 * kLocateMaxS];
    double2 rhs[2 * kLocateMaxS];
    double2 beta[kLocateMaxS];
    double2 y[2 * kLocateMaxS];
    double2 Bv[2 * kLocateMaxS];
    int order[kLocateMaxS];
    int vlist[2 * kLocateMaxS];
    unsigned char mask[kMaxNodes];
    double lo, hi;
    int nv;
};

// Append column `col` (already stored in Q[:, c]) to the thin QR held in
// (Q[:, 0..c-1], Rr): modified Gram-Schmidt with a second pass; lane = row.
__device__ __forceinline__ void mgs_append(Smem& sm, int rows, int c, int lane) {
    const int ldq = 2 * kLocateMaxS;
    for (int pass = 0; pass < 2; ++pass) {
        for (int i = 0; i < c; ++i) {
            double2 prod = make_double2(0.0, 0.0);
            if (lane < rows) prod = cmul(cconj(sm.Q[i * ldq + lane]), sm.Q[c * ldq + lane]);
            const double2 dot = make_double2(wave_sum<kRowLanes>(prod.x), wave_sum<kRowLanes>(prod.y));
            if (lane < rows) sm.Q[c * ldq + lane] = csub(sm.Q[c * ldq + lane], cmul(dot, sm.Q[i * ldq + lane]));
            if (lane == 0) sm.Rr[c * ldq + i] = pass == 0 ? dot : cadd(sm.Rr[c * ldq + i], dot);
            __syncthreads();
        }
    }
    double n2 = 0.0;
    if (lane < rows) n2 = cnorm2(sm.Q[c * ldq + lane]);
    const double nrm = sqrt(wave_sum<kRowLanes>(n2));
    if (lane < rows) sm.Q[c * ldq + lane] = cscale(sm.Q[c * ldq + lane], 1.0 / nrm);
    if (lane == 0) sm.Rr[c * ldq + c] = make_double2(nrm, 0.0);
    __syncthreads();
}

}  // namespace

__global__ __launch_bounds__(kW) void cyc_locate_kernel(const double2* __restrict__ gamma, int P, int s, double tau,
                                                        const double2* __restrict__ b0,
                                                        int32_t* __restrict__ spec_state,
                                                        uint64_t* __restrict__ mask_out,
                                                        int32_t* __restrict__ status_out,
                                                        double2* __restrict__ b_out, int32_t* __restrict__ idx_out,
                                                        int32_t* __restrict__ nu_out) {
    __shared__ Smem sm;
    const int lane = threadIdx.x;
    const int n = P - 2 * s;  // rows of C_L
    const int ldq = 2 * kLocateMaxS;
    const double isq = 1.0 / sqrt((double)P);
    int status = 0;

    // A message with NaN or Inf entries is no vector of R^d: its node is flagged outright and
    // its projection taken as 0, which leaves an ordinary error at a known node.
    int my_broken = 0;
    for (int j = lane; j < P; j += kW) {
        double2 g = gamma[j];
        const bool ok = isfinite(g.x) && isfinite(g.y);
        if (!ok) g = make_double2(0.0, 0.0);
        my_broken += ok ? 0 : 1;
        sm.gam[j] = g;
        double sn, cs;
        sincospi(2.0 * (double)j / (double)P, &sn, &cs);
        sm.root[j] = make_double2(cs, sn);
        sm.mag[j] = hypot(g.x, g.y);
        sm.mask[j] = ok ? 0 : 1;
    }
    if (lane == 0) sm.nv = 0;
    __syncthreads();
    const int broken = (int)wave_sum<kW>((double)my_broken);

    if (broken > s) status = 2;  // DRACO_LOCATE_FAILED: more broken messages than tolerated
    if (s > 0 && broken <= s) {
        // rho = median |gamma_j| by rank counting
        for (int j = lane; j < P; j += kW) {
            const double mj = sm.mag[j];
            int rank = 0;
            for (int i = 0; i < P; ++i) rank += (sm.mag[i] < mj) || (sm.mag[i] == mj && i < j);
            if (rank == (P - 1) / 2) sm.lo = mj;
            if (rank == P / 2) sm.hi = mj;
        }
        __syncthreads();
        const double rho = 0.5 * (sm.lo + sm.hi);
        const double zero = tau * rho;

        // syndromes h_m = (1/sqrt P) sum_j gamma_j w^{-m j}, m = n .. P-1
        for (int j = lane; j < P; j += kW) sm.h[j] = make_double2(0.0, 0.0);
        __syncthreads();
        double mymax = 0.0;
        for (int mp = lane; mp < 2 * s; mp += kW) {
            const int m = n + mp;
            double2 acc = make_double2(0.0, 0.0);
            int e = 0;
            for (int j = 0; j < P; ++j) {
                acc = cadd(acc, cmul(sm.gam[j], cconj(sm.root[e])));
                e += m;
                e %= P;
            }
            acc = cscale(acc, isq);
            sm.hk[mp] = acc;
            sm.h[m] = acc;
            mymax = fmax(mymax, hypot(acc.x, acc.y));
        }
        __syncthreads();
        const double hmax = wave_max(mymax);

        if (hmax > zero) {
            // ---- beta: least squares on the s x s system, singular values <= zero dropped
            // (one-sided Jacobi; lane i owns row i of A and of V)
            for (int k = 0; k < s; ++k) {
                if (lane < s) {
                    sm.A[k * kLocateMaxS + lane] = sm.h[P - s - (lane + 1) + k];   // row i = lane+1
                    sm.V[k * kLocateMaxS + lane] = make_double2(lane == k ? 1.0 : 0.0, 0.0);
                }
            }
            if (lane < s) sm.rhs[lane] = sm.h[P - (lane + 1)];
            __syncthreads();
            for (int sweep = 0; sweep < 60; ++sweep) {
                bool rotated = false;
                for (int p = 0; p < s - 1; ++p) {
                    for (int q = p + 1; q < s; ++q) {
                        double2 ap = make_double2(0.0, 0.0), aq = ap;
                        if (lane < s) {
                            ap = sm.A[p * kLocateMaxS + lane];
                            aq = sm.A[q * kLocateMaxS + lane];
                        }
                        // lanes >= kColLanes form their own (all-zero) groups: they skip every
                        // rotation and never touch A or V, so only group 0's decisions matter
                        const double alpha = wave_sum<kColLanes>(cnorm2(ap));
                        const double bet = wave_sum<kColLanes>(cnorm2(aq));
                        const double2 gp = cmul(cconj(ap), aq);
                        const double2 g = make_double2(wave_sum<kColLanes>(gp.x), wave_sum<kColLanes>(gp.y));
                        const double ag = hypot(g.x, g.y);
                        // columns that both end below the cutoff are dropped from the solution: no need
                        // to make them orthogonal to each other
                        const bool skip = ag == 0.0 || ag <= 1e-10 * sqrt(alpha * bet) ||
                                          (alpha <= zero * zero && bet <= zero * zero);
                        if (__shfl(skip ? 1 : 0, 0) != 0) continue;   // lane 0's decision, uniform
                        rotated = true;
                        const double2 ph = make_double2(g.x / ag, -g.y / ag);
                        const double zeta = (bet - alpha) / (2.0 * ag);
                        const double t = (zeta >= 0.0 ? 1.0 : -1.0) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
                        const double c = 1.0 / sqrt(1.0 + t * t), sn = c * t;
                        if (lane < s) {
                            const double2 aqr = cmul(aq, ph);
                            sm.A[p * kLocateMaxS + lane] = csub(cscale(ap, c), cscale(aqr, sn));
                            sm.A[q * kLocateMaxS + lane] = cadd(cscale(ap, sn), cscale(aqr, c));
                            const double2 vp = sm.V[p * kLocateMaxS + lane];
                            const double2 vq = cmul(sm.V[q * kLocateMaxS + lane], ph);
                            sm.V[p * kLocateMaxS + lane] = csub(cscale(vp, c), cscale(vq, sn));
                            sm.V[q * kLocateMaxS + lane] = cadd(cscale(vp, sn), cscale(vq, c));
                        }
                        __syncthreads();
                    }
                }
                if (__shfl(rotated ? 1 : 0, 0) == 0) break;
            }
            // beta_k = sum_i V[k][i] (a_i^H rhs) / |a_i|^2 over columns with |a_i| > zero
            double2 bk = make_double2(0.0, 0.0);
            for (int i = 0; i < s; ++i) {
                double2 ai = make_double2(0.0, 0.0), ri = ai;
                if (lane < s) {
                    ai = sm.A[i * kLocateMaxS + lane];
                    ri = sm.rhs[lane];
                }
                const double s2 = wave_sum<kColLanes>(cnorm2(ai));
                const double2 dp = cmul(cconj(ai), ri);
                const double2 dot = make_double2(wave_sum<kColLanes>(dp.x), wave_sum<kColLanes>(dp.y));
                if (sqrt(s2) > zero && lane < s)
                    bk = cadd(bk, cmul(cscale(dot, 1.0 / s2), sm.V[i * kLocateMaxS + lane]));
            }
            if (lane < s) sm.beta[lane] = bk;
            __syncthreads();

            // ---- recurrence h_l = sum_u beta_u h_{l+u-s}, l = 0 .. n-1: inherently serial, so one
            // lane runs it out of LDS (a wavefront's LDS accesses complete in order)
            if (lane == 0) {
                for (int l = 0; l < n; ++l) {
                    double2 acc = make_double2(0.0, 0.0);
                    for (int u = 0; u < s; ++u) {
                        int e = l + u - s;
                        if (e < 0) e += P;
                        acc = cadd(acc, cmul(sm.beta[u], sm.h[e]));
                    }
                    sm.h[l] = acc;
                }
            }
            __syncthreads();
            // ---- t = C h, ranking by |t_j| (descending, ties to the lower index)
            for (int j = lane; j < P; j += kW) {
                double2 acc = make_double2(0.0, 0.0);
                int e = 0;
                for (int m = 0; m < P; ++m) {
                    acc = cadd(acc, cmul(sm.h[m], sm.root[e]));
                    e += j;
                    if (e >= P) e -= P;
                }
                sm.mag[j] = hypot(acc.x * isq, acc.y * isq);
            }
            __syncthreads();
            for (int j = lane; j < P; j += kW) {
                const double mj = sm.mag[j];
                int rank = 0;
                for (int i = 0; i < P; ++i) rank += (sm.mag[i] > mj) || (sm.mag[i] == mj && i < j);
                if (rank < s) sm.order[rank] = j;
            }
            __syncthreads();
            // ---- shortest leading part of the ranking whose errors account for the syndromes
            int found = 0;
            for (int a = 1; a <= s; ++a) {
                const int v = sm.order[a - 1];
                if (lane < 2 * s) sm.Q[(a - 1) * ldq + lane] = cscale(cconj(sm.root[((n + lane) * v) % P]), isq);
                __syncthreads();
                mgs_append(sm, 2 * s, a - 1, lane);
                if (lane < 2 * s) sm.res[lane] = sm.hk[lane];
                __syncthreads();
                for (int pass = 0; pass < 2; ++pass) {
                    for (int c = 0; c < a; ++c) {
                        double2 prod = make_double2(0.0, 0.0);
                        if (lane < 2 * s) prod = cmul(cconj(sm.Q[c * ldq + lane]), sm.res[lane]);
                        const double2 dot = make_double2(wave_sum<kRowLanes>(prod.x), wave_sum<kRowLanes>(prod.y));
                        if (lane < 2 * s) sm.res[lane] = csub(sm.res[lane], cmul(dot, sm.Q[c * ldq + lane]));
                        __syncthreads();
                    }
                }
                double r = 0.0;
                if (lane < 2 * s) r = hypot(sm.res[lane].x, sm.res[lane].y);
                if (__shfl(wave_max<kRowLanes>(r), 0) <= zero) {
                    found = a;
                    break;
                }
            }
            const int take = found ? found : s;
            if (!found) status = 2;
            if (lane < take) sm.mask[sm.order[lane]] = 1;
            __syncthreads();
            int mine = 0;
            for (int j = lane; j < P; j += kW) mine += sm.mask[j];
            if ((int)wave_sum<kW>((double)mine) > s) status = 2;
        }
    }
    // ---- b: minimum-norm solution of C_L[:, U] b_U = e_last (see host_math.cpp)
    if (lane == 0) {
        int a = 0;
        for (int j = 0; j < P; ++j)
            if (sm.mask[j]) {  // a failed decode can flag any number of nodes; the list keeps the first 2s
                if (a < 2 * kLocateMaxS) sm.vlist[a] = j;
                ++a;
            }
        sm.nv = a;
    }
    __syncthreads();
    // more than s flagged nodes only happens with status LOCATE_FAILED; the factorisation
    // below has room for s columns, so a failed decode takes the first s of them
    const int a = sm.nv <= s ? sm.nv : s;
    if (sm.nv > s) status = 2;
    if (lane < 2 * s) sm.Bv[lane] = make_double2(0.0, 0.0);
    __syncthreads();
    if (a > 0) {
        for (int v = 0; v < a; ++v) {
            const int node = sm.vlist[v];
            if (lane < 2 * s) sm.Q[v * ldq + lane] = cscale(sm.root[((n + lane) * node) % P], isq);
            if (lane == 0) sm.rhs[v] = cscale(cconj(sm.root[((n - 1) * node) % P]), -isq);
            __syncthreads();
            mgs_append(sm, 2 * s, v, lane);
        }
        if (lane == 0) {  // R^H y = rhs, forward substitution
            for (int i = 0; i < a; ++i) {
                double2 acc = sm.rhs[i];
                for (int k = 0; k < i; ++k) acc = csub(acc, cmul(cconj(sm.Rr[i * ldq + k]), sm.y[k]));
                const double rii = sm.Rr[i * ldq + i].x;
                sm.y[i] = cscale(acc, 1.0 / rii);
            }
        }
        __syncthreads();
        if (lane < 2 * s) {
            double2 acc = make_double2(0.0, 0.0);
            for (int v = 0; v < a; ++v) acc = cadd(acc, cmul(sm.Q[v * ldq + lane], sm.y[v]));
            sm.Bv[lane] = acc;
        }
        __syncthreads();
    }
    for (int j = lane; j < P; j += kW) {
        double2 acc = make_double2(0.0, 0.0);
        if (!sm.mask[j]) {
            if (sm.nv == 0) {
                acc = b0[j];  // the table the speculative pass used: identical results either way
            } else {
                acc = cconj(sm.root[((n - 1) * j) % P]);
                for (int m = 0; m < 2 * s; ++m) acc = cadd(acc, cmul(cconj(sm.root[((n + m) * j) % P]), sm.Bv[m]));
                acc = cscale(acc, isq);
            }
        }
        sm.h[j] = acc;  // reuse: b_j
    }
    __syncthreads();
    if (lane == 0) {
        uint64_t words[kMaskWords] = {0, 0, 0, 0};
        int nu = 0;
        for (int j = 0; j < P; ++j) {
            if (sm.mask[j]) {
                words[j >> 6] |= 1ull << (j & 63);
            } else {
                idx_out[nu] = j;
                b_out[nu] = sm.h[j];
                ++nu;
            }
        }
        *nu_out = nu;
        if (spec_state != nullptr) spec_state[0] = (nu == P && status == 0) ? 1 : 0;
        for (int w = 0; w < (P + 63) / 64; ++w) mask_out[w] = words[w];
        *status_out = status;
    }
}

hipError_t launch_cyc_locate(const double2* gamma, int P, int s, double tau, const double2* b0, uint64_t* mask_out,
                             int32_t* status_out, double2* b_out, int32_t* idx_out, int32_t* nu_out,
                             int32_t* spec_state, hipStream_t stream) {
    hipLaunchKernelGGL(cyc_locate_kernel, dim3(1), dim3(kW), 0, stream, gamma, P, s, tau, b0, spec_state, mask_out,
                       status_out, b_out, idx_out, nu_out);
    return hipGetLastError();
}

}  // namespace draco
