// Device-side phi and recombination vector of the cyclic code (Sec. 3, phi;
// Algorithm 1, lines 1-3): the same steps as host_math.cpp, run by ONE
// wavefront in fp64 so that a cyclic decode needs no host round trip.
//
//   gamma[P] (projections f R)  ->  mask words, status, and the honest nodes'
//   indices and coefficients b (compacted, ascending) for the recombination.
//
// The kernel is a chain of small dependent steps, so its time is latency, not
// throughput.  What keeps it short:
//   * a lane owns node j (j = lane, lane+64, ...) in the O(P) and O(P^2) loops and one
//     matrix row in the small dense algebra (the s x s system for beta, the 2s x |V|
//     least-squares fits); inner products are sums over 16 or 32 lanes done with DPP
//     row operations (a few cycles each) instead of LDS-routed shuffles;
//   * the 2s syndromes are split over all 64 lanes (a lane sums a slice of the nodes);
//   * the recurrence for the remaining h_l, serial by nature, runs out of registers
//     (the window of the last s values never goes through LDS);
//   * the residual of the syndromes is updated by one projection per candidate node
//     instead of being recomputed against every column so far;
//   * indices into the table of roots advance by addition and a conditional
//     subtraction, never by an integer division;
//   * the honest nodes are compacted with wavefront ballots.
// Limits: P <= 256, s <= kLocateMaxS.
#include "host_math.hpp"
#include "kernels.hpp"

namespace draco {

namespace {

constexpr int kW = 64;  // one wavefront

// ---- sums and maxima over aligned groups of N lanes -----------------------------
// Every lane of a group receives the group's result, bit-identical across the group
// (each step combines the same two numbers in both partners).  Must be called with all
// 64 lanes active.
template <int CTRL>
__device__ __forceinline__ double dpp_read(double v) {
    int lo = __double2loint(v), hi = __double2hiint(v);
    lo = __builtin_amdgcn_update_dpp(lo, lo, CTRL, 0xF, 0xF, false);
    hi = __builtin_amdgcn_update_dpp(hi, hi, CTRL, 0xF, 0xF, false);
    return __hiloint2double(hi, lo);
}
constexpr int kDppXor1 = 0xB1;         // quad_perm [1, 0, 3, 2]
constexpr int kDppXor2 = 0x4E;         // quad_perm [2, 3, 0, 1]
constexpr int kDppHalfMirror = 0x141;  // lane i <-> 7 - i within each 8 lanes
constexpr int kDppMirror = 0x140;      // lane i <-> 15 - i within each 16 lanes

template <int N = kW>
__device__ __forceinline__ double group_sum(double v) {
    v += dpp_read<kDppXor1>(v);
    if constexpr (N >= 4) v += dpp_read<kDppXor2>(v);
    if constexpr (N >= 8) v += dpp_read<kDppHalfMirror>(v);   // quads are uniform by now: pairs quad q with quad q^1
    if constexpr (N >= 16) v += dpp_read<kDppMirror>(v);
    if constexpr (N >= 32) v += __shfl_xor(v, 16);
    if constexpr (N >= 64) v += __shfl_xor(v, 32);
    return v;
}
template <int N = kW>
__device__ __forceinline__ double group_max(double v) {
    v = fmax(v, dpp_read<kDppXor1>(v));
    if constexpr (N >= 4) v = fmax(v, dpp_read<kDppXor2>(v));
    if constexpr (N >= 8) v = fmax(v, dpp_read<kDppHalfMirror>(v));
    if constexpr (N >= 16) v = fmax(v, dpp_read<kDppMirror>(v));
    if constexpr (N >= 32) v = fmax(v, __shfl_xor(v, 16));
    if constexpr (N >= 64) v = fmax(v, __shfl_xor(v, 32));
    return v;
}
// Sum over aligned groups of n lanes, n a power of two <= 32 known only at run time
// (the same n in every lane).
__device__ __forceinline__ double group_sum_n(double v, int n) {
    if (n > 1) v += dpp_read<kDppXor1>(v);
    if (n > 2) v += dpp_read<kDppXor2>(v);
    if (n > 4) v += dpp_read<kDppHalfMirror>(v);
    if (n > 8) v += dpp_read<kDppMirror>(v);
    if (n > 16) v += __shfl_xor(v, 16);
    return v;
}
__device__ __forceinline__ bool lane0_says(bool b) { return __builtin_amdgcn_readfirstlane(b ? 1 : 0) != 0; }

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
// acc + a * b with fused multiply-adds (two deep per component)
__device__ __forceinline__ double2 cfma(double2 a, double2 b, double2 acc) {
    return make_double2(fma(-a.y, b.y, fma(a.x, b.x, acc.x)), fma(a.y, b.x, fma(a.x, b.y, acc.y)));
}
// 1/sqrt(x) and 1/x for positive, finite, normal x: the hardware's estimate refined by two
// Newton steps (the library forms cost three to four times the latency, and this kernel is
// a chain of dependent scalars)
__device__ __forceinline__ double rsqrt_pos(double x) {
    double r = __builtin_amdgcn_rsq(x);
    const double hx = 0.5 * x;
    r = r * fma(-hx * r, r, 1.5);
    r = r * fma(-hx * r, r, 1.5);
    return r;
}
__device__ __forceinline__ double rcp_pos(double x) {
    double r = __builtin_amdgcn_rcp(x);
    r = r * fma(-x, r, 2.0);
    r = r * fma(-x, r, 2.0);
    return r;
}
// (a + b) mod P for 0 <= a, b < P
__device__ __forceinline__ int addmod(int a, int b, int P) {
    const int c = a + b;
    return c >= P ? c - P : c;
}
__device__ __forceinline__ int mulmod(int a, int b, int P) { return (int)(((long long)a * b) % P); }

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

// Append the column stored in Q[:, c] to the thin QR held in (Q[:, 0..c-1], Rr): modified
// Gram-Schmidt with a second pass; lane = row.  Returns this lane's entry of the new
// orthonormal column (0 outside the rows).
__device__ __forceinline__ double2 mgs_append(Smem& sm, int rows, int c, int lane) {
    const int ldq = 2 * kLocateMaxS;
    double2 mine = lane < rows ? sm.Q[c * ldq + lane] : make_double2(0.0, 0.0);
    for (int pass = 0; pass < 2; ++pass) {
        for (int i = 0; i < c; ++i) {
            const double2 qi = lane < rows ? sm.Q[i * ldq + lane] : make_double2(0.0, 0.0);
            const double2 prod = cmul(cconj(qi), mine);
            const double2 dot = make_double2(group_sum<kRowLanes>(prod.x), group_sum<kRowLanes>(prod.y));
            mine = csub(mine, cmul(dot, qi));
            if (lane == 0) sm.Rr[c * ldq + i] = pass == 0 ? dot : cadd(sm.Rr[c * ldq + i], dot);
        }
    }
    const double n2 = group_sum<kRowLanes>(cnorm2(mine));
    const double inv = rsqrt_pos(n2);
    mine = cscale(mine, inv);
    if (lane < rows) sm.Q[c * ldq + lane] = mine;
    if (lane == 0) sm.Rr[c * ldq + c] = make_double2(n2 * inv, 0.0);
    __syncthreads();
    return mine;
}

// phi step 3: h_l = sum_u beta_u h_{l+u-s} for l = 0 .. n-1 (indices mod P).  Serial by
// nature; every lane runs it redundantly with beta and the window of the last S values in
// registers, lane 0 records the results.  Slot k of the window holds h_{l-s} when
// l = k (mod S), so entry u of the sum sits in slot (k + u) mod S.
template <int S>
__device__ __forceinline__ void recurrence(Smem& sm, int n, int P, int lane) {
    double2 beta[S], win[S];
#pragma unroll
    for (int u = 0; u < S; ++u) {
        beta[u] = sm.beta[u];
        win[u] = sm.h[P - S + u];
    }
    for (int l0 = 0; l0 < n; l0 += S) {
#pragma unroll
        for (int k = 0; k < S; ++k) {
            const int l = l0 + k;
            if (l < n) {
                double2 acc = make_double2(0.0, 0.0);
#pragma unroll
                for (int u = 0; u < S; ++u) acc = cfma(beta[u], win[(k + u) % S], acc);   // the newest value enters last
                win[k] = acc;
                if (lane == 0) sm.h[l] = acc;
            }
        }
    }
}
// The same out of LDS, for windows too long to unroll.
__device__ __forceinline__ void recurrence_lds(Smem& sm, int n, int P, int s, int lane) {
    if (lane == 0) {
        for (int l = 0; l < n; ++l) {
            double2 acc = make_double2(0.0, 0.0);
            int e = l - s;
            if (e < 0) e += P;
            for (int u = 0; u < s; ++u) {
                acc = cadd(acc, cmul(sm.beta[u], sm.h[e]));
                e = addmod(e, 1, P);
            }
            sm.h[l] = acc;
        }
    }
}

}  // namespace

__global__ __launch_bounds__(kW) void cyc_locate_kernel(const double2* __restrict__ gamma,
                                                        const double2* __restrict__ roots, int P, int s, double tau,
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
    int fitted = 0;  // columns of the syndrome fit left in (Q, Rr) by the locator: the located nodes, in ranking order

    // A message with NaN or Inf entries is no vector of R^d: its node is flagged outright and
    // its projection taken as 0, which leaves an ordinary error at a known node.
    int my_broken = 0;
    for (int j = lane; j < P; j += kW) {
        double2 g = gamma[j];
        const bool ok = isfinite(g.x) && isfinite(g.y);
        if (!ok) g = make_double2(0.0, 0.0);
        my_broken += ok ? 0 : 1;
        sm.gam[j] = g;
        sm.root[j] = roots[j];
        sm.mask[j] = ok ? 0 : 1;
    }
    if (lane == 0) sm.nv = 0;
    __syncthreads();
    const int broken = (int)group_sum<kW>((double)my_broken);

    if (broken > s) status = 2;  // DRACO_LOCATE_FAILED: more broken messages than tolerated
    // Passes of phi.  A projection more than kEnormous * rho in size is "enormous": its fp64
    // rounding can reach the zero threshold or swallow a smaller lie whole (an adversary may send
    // 1e30).  After a pass the located nodes whose projection is enormous and large enough for its
    // rounding to pass for a syndrome (kLocatedEnormousOverTau) -- or, if it found no set, the top
    // layer of the enormous nodes (within a factor kEnormous of the largest) -- are set aside like
    // broken ones and phi runs again, provided the flagged nodes stay within s; the
    // first pass that sets nothing aside is the last.  Every other pass flags at least one more node, so there are at
    // most s + 1.  Every branch below is taken by all 64 lanes together.
    int aside = broken;  // nodes flagged outright so far
    for (int pass = 0; pass <= s && s > 0 && broken <= s; ++pass) {
        for (int j = lane; j < P; j += kW) sm.mag[j] = sqrt(cnorm2(sm.gam[j]));
        __syncthreads();
        // rho = median |gamma_j| by rank counting
        for (int j = lane; j < P; j += kW) {
            const double mj = sm.mag[j];
            int rank = 0;
            for (int i = 0; i < P; ++i) rank += (sm.mag[i] < mj) || (sm.mag[i] == mj && i < j);
            if (rank == (P - 1) / 2) sm.lo = mj;
            if (rank == P / 2) sm.hi = mj;
        }
        for (int j = lane; j < P; j += kW) sm.h[j] = make_double2(0.0, 0.0);
        __syncthreads();
        const double rho = 0.5 * (sm.lo + sm.hi);
        const double zero = tau * rho;
        const double zero2 = zero * zero;

        // syndromes h_m = (1/sqrt P) sum_j gamma_j w^{-m j}, m = n .. P-1: `parts` lanes share a
        // syndrome, each summing the nodes j = part, part + parts, ...
        int parts = 1;
        while (2 * parts * 2 * s <= kW && parts < 32) parts *= 2;
        double mymax = 0.0;
        {
            const int mp = lane / parts, part = lane % parts;
            const bool live = mp < 2 * s;
            const int m = n + (live ? mp : 0);
            double2 acc = make_double2(0.0, 0.0);
            if (live) {
                int e = mulmod(m, part, P);
                const int step = mulmod(m, parts, P);
                for (int j = part; j < P; j += parts) {
                    acc = cadd(acc, cmul(sm.gam[j], cconj(sm.root[e])));
                    e = addmod(e, step, P);
                }
            }
            acc = make_double2(group_sum_n(acc.x, parts), group_sum_n(acc.y, parts));
            acc = cscale(acc, isq);
            if (live && part == 0) {
                sm.hk[mp] = acc;
                sm.h[m] = acc;
            }
            if (live) mymax = cnorm2(acc);
        }
        __syncthreads();
        const double hmax2 = group_max<kW>(mymax);

        int found = 0;      // length of the leading part of the ranking that accounts for the syndromes
        bool located = true;
        fitted = 0;
        if (hmax2 > zero2) {
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
                        // lanes >= kColLanes form their own (all-zero) groups: they never touch A or V,
                        // and only lane 0's decision counts
                        const double alpha = group_sum<kColLanes>(cnorm2(ap));
                        const double bet = group_sum<kColLanes>(cnorm2(aq));
                        const double2 gp = cmul(cconj(ap), aq);
                        const double2 g = make_double2(group_sum<kColLanes>(gp.x), group_sum<kColLanes>(gp.y));
                        const double ag2 = cnorm2(g);
                        // columns that both end below the cutoff are dropped from the solution: no need
                        // to make them orthogonal to each other
                        const bool skip = ag2 == 0.0 || ag2 <= 1e-20 * (alpha * bet) || (alpha <= zero2 && bet <= zero2);
                        if (lane0_says(skip)) continue;
                        rotated = true;
                        // rotation that makes the two columns orthogonal: with zeta = (bet - alpha) / (2 |g|),
                        // t = sign(zeta) / (|zeta| + sqrt(1 + zeta^2)), c = 1 / sqrt(1 + t^2), sn = c t
                        const double inv_ag = rsqrt_pos(ag2);
                        const double2 ph = make_double2(g.x * inv_ag, -g.y * inv_ag);
                        const double zeta = (bet - alpha) * (0.5 * inv_ag);
                        const double w2 = fma(zeta, zeta, 1.0);
                        const double t = (zeta >= 0.0 ? 1.0 : -1.0) * rcp_pos(fabs(zeta) + w2 * rsqrt_pos(w2));
                        const double c = rsqrt_pos(fma(t, t, 1.0)), sn = c * t;
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
                if (!lane0_says(rotated)) break;
            }
            // beta_k = sum_i V[k][i] (a_i^H rhs) / |a_i|^2 over columns with |a_i| > zero
            double2 bk = make_double2(0.0, 0.0);
            for (int i = 0; i < s; ++i) {
                double2 ai = make_double2(0.0, 0.0), ri = ai;
                if (lane < s) {
                    ai = sm.A[i * kLocateMaxS + lane];
                    ri = sm.rhs[lane];
                }
                const double s2 = group_sum<kColLanes>(cnorm2(ai));
                const double2 dp = cmul(cconj(ai), ri);
                const double2 dot = make_double2(group_sum<kColLanes>(dp.x), group_sum<kColLanes>(dp.y));
                if (s2 > zero2 && lane < s) bk = cadd(bk, cmul(cscale(dot, 1.0 / s2), sm.V[i * kLocateMaxS + lane]));
            }
            if (lane < s) sm.beta[lane] = bk;
            __syncthreads();

            // ---- recurrence h_l = sum_u beta_u h_{l+u-s}, l = 0 .. n-1
            switch (s) {
                case 1: recurrence<1>(sm, n, P, lane); break;
                case 2: recurrence<2>(sm, n, P, lane); break;
                case 3: recurrence<3>(sm, n, P, lane); break;
                case 4: recurrence<4>(sm, n, P, lane); break;
                case 5: recurrence<5>(sm, n, P, lane); break;
                case 6: recurrence<6>(sm, n, P, lane); break;
                case 7: recurrence<7>(sm, n, P, lane); break;
                case 8: recurrence<8>(sm, n, P, lane); break;
                default: recurrence_lds(sm, n, P, s, lane);
            }
            __syncthreads();
            // ---- t = C h, ranking by |t_j| (descending, ties to the lower index)
            for (int j = lane; j < P; j += kW) {
                double2 acc0 = make_double2(0.0, 0.0), acc1 = acc0;   // even and odd m: two independent chains
                int e = 0;
                const int j2 = addmod(j, j, P);
                int m = 0;
                for (; m + 1 < P; m += 2) {
                    const int e1 = addmod(e, j, P);
                    acc0 = cfma(sm.h[m], sm.root[e], acc0);
                    acc1 = cfma(sm.h[m + 1], sm.root[e1], acc1);
                    e = addmod(e, j2, P);
                }
                if (m < P) acc0 = cfma(sm.h[m], sm.root[e], acc0);
                sm.mag[j] = cnorm2(cadd(acc0, acc1));   // P |t_j|^2: the ranking needs no more
            }
            __syncthreads();
            for (int j = lane; j < P; j += kW) {
                const double mj = sm.mag[j];
                int rank = 0;
                for (int i = 0; i < P; ++i) rank += (sm.mag[i] > mj) || (sm.mag[i] == mj && i < j);
                if (rank < s) sm.order[rank] = j;
            }
            __syncthreads();
            // ---- shortest leading part of the ranking whose errors account for the syndromes: the
            // residual of the syndromes loses its component along each new orthonormal column
            double2 res = lane < 2 * s ? sm.hk[lane] : make_double2(0.0, 0.0);
            for (int a = 1; a <= s; ++a) {
                const int v = sm.order[a - 1];
                if (lane < 2 * s) sm.Q[(a - 1) * ldq + lane] = cscale(cconj(sm.root[mulmod(n + lane, v, P)]), isq);
                __syncthreads();
                const double2 qa = mgs_append(sm, 2 * s, a - 1, lane);
                {   // qa is orthogonal to the earlier columns, so is res: one projection removes the new component
                    const double2 prod = cmul(cconj(qa), res);
                    const double2 dot = make_double2(group_sum<kRowLanes>(prod.x), group_sum<kRowLanes>(prod.y));
                    res = csub(res, cmul(dot, qa));
                }
                // largest |residual| against the zero threshold, on squares
                const double r2 = lane < 2 * s ? cnorm2(res) : 0.0;
                if (lane0_says(group_max<kRowLanes>(r2) <= zero2)) {
                    found = a;
                    break;
                }
            }
            located = found != 0;
            fitted = found;
        }
        bool last = pass == s;   // (never reached with something left to set aside: aside <= s)
        if (!last) {
            const double limit = kEnormous * rho;
            const double located_limit = fmax(limit, kLocatedEnormousOverTau * tau * rho);
            double top = 0.0;   // the largest enormous projection not flagged yet
            for (int j = lane; j < P; j += kW) {
                const double size = sqrt(cnorm2(sm.gam[j]));
                if (sm.mask[j] == 0 && size > limit) top = fmax(top, size);
            }
            top = group_max<kW>(top);
            auto set_aside = [&](int j) {   // enormous, not flagged yet; located, or else in the top layer
                const double size = sqrt(cnorm2(sm.gam[j]));
                if (sm.mask[j] != 0 || !(size > limit)) return false;
                if (!located) return size * kEnormous > top;
                if (!(size > located_limit)) return false;
                for (int i = 0; i < found; ++i)
                    if (sm.order[i] == j) return true;
                return false;
            };
            int mine = 0;
            for (int j = lane; j < P; j += kW) mine += set_aside(j) ? 1 : 0;
            const int huge = (int)group_sum<kW>((double)mine);
            if (huge == 0 || aside + huge > s) {
                last = true;   // nothing to set aside, or too many: this pass stands
            } else {
                bool go[(kMaxNodes + kW - 1) / kW];
                for (int j = lane, k = 0; j < P; j += kW, ++k) go[k] = set_aside(j);
                for (int j = lane, k = 0; j < P; j += kW, ++k) {
                    if (go[k]) {
                        sm.gam[j] = make_double2(0.0, 0.0);
                        sm.mask[j] = 1;
                    }
                }
                aside += huge;
                __syncthreads();
            }
        }
        if (last) {
            const int take = located ? found : s;   // a failed decode flags the s largest |t_j|
            if (!located) status = 2;
            if (hmax2 > zero2 && lane < take) sm.mask[sm.order[lane]] = 1;
            __syncthreads();
            int mine = 0;
            for (int j = lane; j < P; j += kW) mine += sm.mask[j];
            if ((int)group_sum<kW>((double)mine) > s) status = 2;
            break;
        }
    }

    // ---- b: minimum-norm solution of C_L[:, U] b_U = e_last (see host_math.cpp)
    {   // flagged nodes in ascending order; a failed decode can flag any number, the list keeps the first 2s
        int count = 0;
        for (int c = 0; c < P; c += kW) {
            const int j = c + lane;
            const bool flagged = j < P && sm.mask[j] != 0;
            const unsigned long long bal = __ballot(flagged);
            const int pos = count + __popcll(bal & ((1ull << lane) - 1ull));
            if (flagged && pos < 2 * kLocateMaxS) sm.vlist[pos] = j;
            count += __popcll(bal);
        }
        if (lane == 0) sm.nv = count;
    }
    if (lane < 2 * s) sm.Bv[lane] = make_double2(0.0, 0.0);
    __syncthreads();
    // more than s flagged nodes only happens with status LOCATE_FAILED; the factorisation
    // below has room for s columns, so a failed decode takes the first s of them
    const int nv = sm.nv;
    const int a = nv <= s ? nv : s;
    if (nv > s) status = 2;
    if (a > 0) {
        // The columns needed here, (1/sqrt P) w^{(n+row) v} for the flagged nodes v, are the complex
        // conjugates of the columns the locator fitted the syndromes with.  When the flagged nodes
        // are exactly the located ones, that factorisation is reused (conjugate Q and R; the order
        // of the columns does not change the minimum-norm solution); else it is built afresh.
        const bool reuse = fitted == nv && fitted > 0;
        if (!reuse) {
            for (int v = 0; v < a; ++v) {
                const int node = sm.vlist[v];
                if (lane < 2 * s) sm.Q[v * ldq + lane] = cscale(sm.root[mulmod(n + lane, node, P)], isq);
                __syncthreads();
                mgs_append(sm, 2 * s, v, lane);
            }
        }
        if (lane == 0) {  // R^H y = rhs, forward substitution
            for (int i = 0; i < a; ++i) {
                const int node = reuse ? sm.order[i] : sm.vlist[i];
                double2 acc = cscale(cconj(sm.root[mulmod(n - 1, node, P)]), -isq);
                for (int k = 0; k < i; ++k) {
                    const double2 rki = sm.Rr[i * ldq + k];   // R[k][i] of the factorisation in LDS
                    acc = csub(acc, cmul(reuse ? rki : cconj(rki), sm.y[k]));
                }
                sm.y[i] = cscale(acc, 1.0 / sm.Rr[i * ldq + i].x);
            }
        }
        __syncthreads();
        if (lane < 2 * s) {
            double2 acc = make_double2(0.0, 0.0);
            for (int v = 0; v < a; ++v) {
                const double2 qv = sm.Q[v * ldq + lane];
                acc = cadd(acc, cmul(reuse ? cconj(qv) : qv, sm.y[v]));
            }
            sm.Bv[lane] = acc;
        }
        __syncthreads();
    }
    // b_j = (1/sqrt P) (conj w^{(n-1) j} + sum_m conj w^{(n+m) j} Bv_m) on honest nodes, written
    // one behind the other in ascending node order; mask words by ballot
    int nu = 0;
    for (int c = 0; c < P; c += kW) {
        const int j = c + lane;
        const bool inside = j < P;
        const bool honest = inside && sm.mask[j] == 0;
        double2 acc = make_double2(0.0, 0.0);
        if (honest) {
            if (nv == 0) {
                acc = b0[j];  // the table the speculative pass used: identical results either way
            } else {
                int e = mulmod(n - 1, j, P);
                acc = cconj(sm.root[e]);
                for (int m = 0; m < 2 * s; ++m) {
                    e = addmod(e, j, P);
                    acc = cadd(acc, cmul(cconj(sm.root[e]), sm.Bv[m]));
                }
                acc = cscale(acc, isq);
            }
        }
        const unsigned long long bal = __ballot(honest);
        const unsigned long long flagged = __ballot(inside && !honest);
        if (honest) {
            const int pos = nu + __popcll(bal & ((1ull << lane) - 1ull));
            idx_out[pos] = j;
            b_out[pos] = acc;
        }
        if (lane == 0) mask_out[c / kW] = flagged;
        nu += __popcll(bal);
    }
    if (lane == 0) {
        *nu_out = nu;
        if (spec_state != nullptr) spec_state[0] = (nu == P && status == 0) ? 1 : 0;
        *status_out = status;
    }
}

hipError_t launch_cyc_locate(const double2* gamma, const double2* roots, int P, int s, double tau, const double2* b0,
                             uint64_t* mask_out, int32_t* status_out, double2* b_out, int32_t* idx_out,
                             int32_t* nu_out, int32_t* spec_state, hipStream_t stream) {
    hipLaunchKernelGGL(cyc_locate_kernel, dim3(1), dim3(kW), 0, stream, gamma, roots, P, s, tau, b0, spec_state,
                       mask_out, status_out, b_out, idx_out, nu_out);
    return hipGetLastError();
}

}  // namespace draco
