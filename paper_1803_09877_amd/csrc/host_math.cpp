// Host-side algebra of the cyclic code; see host_math.hpp.
#include "host_math.hpp"

#include <algorithm>
#include <cmath>
#include <numeric>

namespace draco {

namespace {

const real_t kPi = 3.14159265358979323846264338327950288L;

real_t norm2(const cplx_t& z) { return z.real() * z.real() + z.imag() * z.imag(); }

// Column-major dense complex matrix, tiny.
struct Mat {
    int m = 0, n = 0;
    std::vector<cplx_t> a;
    Mat(int m_, int n_) : m(m_), n(n_), a((size_t)m_ * n_) {}
    cplx_t& operator()(int i, int j) { return a[(size_t)j * m + i]; }
    const cplx_t& operator()(int i, int j) const { return a[(size_t)j * m + i]; }
};

// Thin QR by modified Gram-Schmidt with one re-orthogonalisation pass:
// X (m x n, m >= n, full column rank) = Q R.
void qr_mgs(const Mat& X, Mat& Q, Mat& R) {
    const int m = X.m, n = X.n;
    Q = X;
    R = Mat(n, n);
    for (int j = 0; j < n; ++j) {
        for (int pass = 0; pass < 2; ++pass) {
            for (int i = 0; i < j; ++i) {
                cplx_t dot = 0;
                for (int k = 0; k < m; ++k) dot += std::conj(Q(k, i)) * Q(k, j);
                for (int k = 0; k < m; ++k) Q(k, j) -= dot * Q(k, i);
                R(i, j) += dot;
            }
        }
        real_t nrm = 0;
        for (int k = 0; k < m; ++k) nrm += norm2(Q(k, j));
        nrm = std::sqrt(nrm);
        R(j, j) = nrm;
        for (int k = 0; k < m; ++k) Q(k, j) /= nrm;
    }
}

// Least-squares solution of H x = rhs that ignores singular directions with
// singular value <= cutoff (one-sided Jacobi SVD, H is n x n).
std::vector<cplx_t> solve_truncated(const Mat& H, const std::vector<cplx_t>& rhs, real_t cutoff) {
    const int n = H.n, m = H.m;
    Mat A = H;
    Mat V(n, n);
    for (int i = 0; i < n; ++i) V(i, i) = 1;
    const real_t eps = 1e-19L;
    for (int sweep = 0; sweep < 80; ++sweep) {
        bool rotated = false;
        for (int p = 0; p < n - 1; ++p) {
            for (int q = p + 1; q < n; ++q) {
                real_t alpha = 0, beta = 0;
                cplx_t g = 0;
                for (int i = 0; i < m; ++i) {
                    alpha += norm2(A(i, p));
                    beta += norm2(A(i, q));
                    g += std::conj(A(i, p)) * A(i, q);
                }
                const real_t ag = std::abs(g);
                if (ag == 0 || ag <= eps * std::sqrt(alpha * beta)) continue;
                // columns that both end below the cutoff are dropped from the solution
                if (alpha <= cutoff * cutoff && beta <= cutoff * cutoff) continue;
                rotated = true;
                const cplx_t ph = std::conj(g / ag);  // turns column q so that <a_p, a_q> is real >= 0
                const real_t zeta = (beta - alpha) / (2 * ag);
                const real_t t = (zeta >= 0 ? 1 : -1) / (std::fabs(zeta) + std::sqrt(1 + zeta * zeta));
                const real_t c = 1 / std::sqrt(1 + t * t), sn = c * t;
                for (int i = 0; i < m; ++i) {
                    const cplx_t ap = A(i, p), aq = A(i, q) * ph;
                    A(i, p) = c * ap - sn * aq;
                    A(i, q) = sn * ap + c * aq;
                }
                for (int i = 0; i < n; ++i) {
                    const cplx_t vp = V(i, p), vq = V(i, q) * ph;
                    V(i, p) = c * vp - sn * vq;
                    V(i, q) = sn * vp + c * vq;
                }
            }
        }
        if (!rotated) break;
    }
    // H = U S V^H with U S = A.  x = sum_i v_i (a_i^H rhs) / sigma_i^2 over kept i.
    std::vector<cplx_t> x(n, cplx_t(0));
    for (int i = 0; i < n; ++i) {
        real_t s2 = 0;
        for (int k = 0; k < m; ++k) s2 += norm2(A(k, i));
        if (std::sqrt(s2) <= cutoff) continue;
        cplx_t dot = 0;
        for (int k = 0; k < m; ++k) dot += std::conj(A(k, i)) * rhs[k];
        const cplx_t coef = dot / s2;
        for (int k = 0; k < n; ++k) x[k] += coef * V(k, i);
    }
    return x;
}

// Largest |syndrome| left once errors on the nodes V are fitted out:
// syndromes of an error vector e are h_m = (1/sqrt P) sum_j e_j w^{-m j}.
real_t unexplained(int P, int s, const std::vector<cplx_t>& hk, const std::vector<int>& V) {
    std::vector<cplx_t> r = hk;
    const int a = (int)V.size();
    if (a > 0) {
        Mat M(2 * s, a);
        const real_t isq = 1 / std::sqrt((real_t)P);
        for (int v = 0; v < a; ++v)
            for (int mp = 0; mp < 2 * s; ++mp)
                M(mp, v) = isq * root_of_unity(P, -(long long)(P - 2 * s + mp) * V[v]);
        Mat Q(0, 0), R(0, 0);
        qr_mgs(M, Q, R);
        for (int pass = 0; pass < 2; ++pass)
            for (int v = 0; v < a; ++v) {
                cplx_t dot = 0;
                for (int k = 0; k < 2 * s; ++k) dot += std::conj(Q(k, v)) * r[k];
                for (int k = 0; k < 2 * s; ++k) r[k] -= dot * Q(k, v);
            }
    }
    real_t mx = 0;
    for (const auto& z : r) mx = std::max(mx, std::abs(z));
    return mx;
}

}  // namespace

cplx_t root_of_unity(int P, long long k) {
    // One table per P (P <= 256), built on first use: the decoder asks for
    // O(P^2) roots per call and long-double trigonometry is slow.
    struct Table {
        std::vector<cplx_t> w;
    };
    thread_local Table tables[257];
    k %= P;
    if (k < 0) k += P;
    if (P <= 256) {
        Table& t = tables[P];
        if (t.w.empty()) {
            t.w.resize(P);
            for (int i = 0; i < P; ++i) {
                const real_t ang = 2 * kPi * (real_t)i / (real_t)P;
                t.w[i] = cplx_t(std::cos(ang), std::sin(ang));
            }
        }
        return t.w[(size_t)k];
    }
    const real_t ang = 2 * kPi * (real_t)k / (real_t)P;
    return cplx_t(std::cos(ang), std::sin(ang));
}

void CyclicCode::build(int P_, int s_) {
    P = P_;
    s = s_;
    const int r = 2 * s + 1;
    const int D = P - r;  // degree of the monic polynomial behind each row of W
    taps.assign(r, cplx_t(0));
    rot.assign(P, cplx_t(0));
    const real_t isq = 1 / std::sqrt((real_t)P);
    // Row k of W, as a function of the node j, is (1/sqrt P) * prod over the
    // non-holders m of gradient k of (w^j - w^m).  With j = k - t and m = k - u
    // the factor w^k comes out D times: W[k][k-t] = w^{kD} * taps[t].
    for (int t = 0; t < r; ++t) {
        cplx_t prod = isq;
        for (int u = r; u < P; ++u) prod *= root_of_unity(P, -t) - root_of_unity(P, -u);
        taps[t] = prod;
    }
    for (int k = 0; k < P; ++k) rot[k] = root_of_unity(P, (long long)k * D);
    // The non-holders are consecutive on the circle, so each factor above is a unit phase times a
    // sine: w^a - w^b = e^{i pi (a+b)/P} * 2i sin(pi (a-b)/P).  Collecting the phases,
    // taps[t] = c * e^{-i pi D t / P} * rho[t] with rho real and c one constant phase, hence
    // W[j+t][j] = rot[j+t] * taps[t] = (c e^{i pi D j / P}) * rho[t] * e^{i pi D (j+t) / P}.
    const cplx_t c = taps[0] / std::abs(taps[0]);
    real_taps.assign(r, 0);
    node_phase.assign(P, cplx_t(0));
    row_phase.assign(P + 2 * s, cplx_t(0));
    for (int t = 0; t < r; ++t)
        real_taps[t] = (taps[t] * std::conj(c) * root_of_unity(2 * P, (long long)D * t)).real();
    for (int j = 0; j < P; ++j) node_phase[j] = c * root_of_unity(2 * P, (long long)D * j);
    for (int k = 0; k < P + 2 * s; ++k) row_phase[k] = root_of_unity(2 * P, (long long)D * k);
}

cplx_t CyclicCode::W(int k, int j) const {
    const int t = ((k - j) % P + P) % P;
    if (t > 2 * s) return cplx_t(0);
    return node_phase[j] * real_taps[t] * row_phase[j + t];
}

namespace {

double median_size(int P, const std::complex<double>* gamma) {
    std::vector<double> mags(P);
    for (int j = 0; j < P; ++j) mags[j] = std::abs(gamma[j]);
    std::sort(mags.begin(), mags.end());
    return (P % 2) ? mags[P / 2] : (double)(((real_t)mags[P / 2 - 1] + (real_t)mags[P / 2]) / 2);
}

// One pass of phi's steps 2-4 over finite projections: flags the located nodes in `mask` (on
// failure: the s largest |t_j|), fills t_out, returns whether a set of at most s nodes accounts
// for the syndromes.
bool locate_attempt(int P, int s, double tau, const std::complex<double>* gamma, std::vector<uint8_t>& mask,
                    std::vector<std::complex<double>>& t_out);

}  // namespace

bool cyclic_locate(int P, int s, double tau, const std::complex<double>* gamma_in, std::vector<uint8_t>& mask,
                   std::vector<std::complex<double>>& t_out) {
    mask.assign(P, 0);
    t_out.assign(P, std::complex<double>(0, 0));
    // A message with NaN or Inf entries is no vector of R^d: its node is flagged outright and
    // its projection taken as 0, which leaves an ordinary error at a known node.
    std::vector<std::complex<double>> clean(gamma_in, gamma_in + P);
    int broken = 0;
    for (int j = 0; j < P; ++j) {
        if (!std::isfinite(clean[j].real()) || !std::isfinite(clean[j].imag())) {
            clean[j] = 0;
            mask[j] = 1;
            ++broken;
        }
    }
    if (s == 0) return broken == 0;
    if (broken > s) return false;
    std::vector<uint8_t> located;
    bool found = false;
    // A finite projection can be so large that its own fp64 rounding drowns the zero threshold
    // or swallows a smaller lie whole (an adversary may send 1e30): "enormous" is more than
    // kEnormous times the median.  After a pass of phi the located nodes whose projection is
    // enormous and large enough for its rounding to pass for a syndrome (kLocatedEnormousOverTau)
    // -- or, if it found no set, the top layer of the enormous nodes (within a factor kEnormous of
    // the largest) -- are set aside like broken ones and phi runs again, provided the flagged nodes
    // stay within s; the result of the first pass that sets nothing aside stands (at most s + 1
    // passes).  Nodes phi did not locate are never set aside while it succeeds: heavy-tailed honest
    // batches flag nobody.
    for (;;) {
        found = locate_attempt(P, s, tau, clean.data(), located, t_out);
        const double rho = median_size(P, clean.data());
        const double limit = kEnormous * rho;
        const double located_limit = std::max(limit, kLocatedEnormousOverTau * tau * rho);
        double top = 0.0;
        for (int j = 0; j < P; ++j)
            if (!mask[j] && std::abs(clean[j]) > limit) top = std::max(top, std::abs(clean[j]));
        std::vector<uint8_t> aside(P, 0);
        int count = 0;
        for (int j = 0; j < P; ++j) {
            const double size = std::abs(clean[j]);
            aside[j] = (!mask[j] && size > limit &&
                        (found ? (located[j] != 0 && size > located_limit) : size * kEnormous > top)) ? 1 : 0;
            count += aside[j];
        }
        if (count == 0 || broken + count > s) break;
        for (int j = 0; j < P; ++j) {
            if (aside[j]) {
                clean[j] = 0;
                mask[j] = 1;
            }
        }
        broken += count;
    }
    int total = 0;
    for (int j = 0; j < P; ++j) {
        mask[j] = (mask[j] || located[j]) ? 1 : 0;
        total += mask[j];
    }
    return found && total <= s;
}

namespace {

bool locate_attempt(int P, int s, double tau, const std::complex<double>* gamma, std::vector<uint8_t>& mask,
                    std::vector<std::complex<double>>& t_out) {
    mask.assign(P, 0);
    t_out.assign(P, std::complex<double>(0, 0));
    const real_t rho = (real_t)median_size(P, gamma);
    const real_t zero = (real_t)tau * rho;
    const real_t isq = 1 / std::sqrt((real_t)P);

    // [h_{P-2s}, ..., h_{P-1}] = (f R) C_R^dagger
    std::vector<cplx_t> h(P, cplx_t(0)), hk(2 * s);
    for (int m = P - 2 * s; m < P; ++m) {
        cplx_t acc = 0;
        for (int j = 0; j < P; ++j)
            acc += cplx_t(gamma[j].real(), gamma[j].imag()) * root_of_unity(P, -(long long)m * j);
        h[m] = acc * isq;
        hk[m - (P - 2 * s)] = h[m];
    }
    if (unexplained(P, s, hk, {}) <= zero) return true;

    // s x s system for beta: row i (1..s): sum_k beta_k h_{P-s-i+k} = h_{P-i}
    Mat H(s, s);
    std::vector<cplx_t> rhs(s);
    for (int i = 1; i <= s; ++i) {
        for (int k = 0; k < s; ++k) H(i - 1, k) = h[P - s - i + k];
        rhs[i - 1] = h[P - i];
    }
    const std::vector<cplx_t> beta = solve_truncated(H, rhs, zero);

    // remaining syndromes by the recurrence h_l = sum_u beta_u h_{l+u-s}
    for (int l = 0; l < P - 2 * s; ++l) {
        cplx_t acc = 0;
        for (int u = 0; u < s; ++u) acc += beta[u] * h[((l + u - s) % P + P) % P];
        h[l] = acc;
    }
    // t = C h.  t only ranks the nodes (the decision is the residual test below), so
    // plain doubles are enough here and keep this O(P^2) loop cheap.
    std::vector<std::complex<double>> hd(P), wd(P);
    for (int m = 0; m < P; ++m) {
        hd[m] = std::complex<double>((double)h[m].real(), (double)h[m].imag());
        const cplx_t w = root_of_unity(P, m);
        wd[m] = std::complex<double>((double)w.real(), (double)w.imag());
    }
    const double isqd = (double)isq;
    std::vector<double> tmag(P);
    for (int j = 0; j < P; ++j) {
        double ar = 0.0, ai = 0.0;
        int e = 0;  // (m * j) mod P
        for (int m = 0; m < P; ++m) {
            ar += hd[m].real() * wd[e].real() - hd[m].imag() * wd[e].imag();
            ai += hd[m].real() * wd[e].imag() + hd[m].imag() * wd[e].real();
            e += j;
            if (e >= P) e -= P;
        }
        t_out[j] = std::complex<double>(ar * isqd, ai * isqd);
        tmag[j] = std::abs(t_out[j]);
    }
    std::vector<int> order(P);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return tmag[a] > tmag[b]; });
    order.resize(s);
    for (int a = 1; a <= s; ++a) {
        std::vector<int> V(order.begin(), order.begin() + a);
        if (unexplained(P, s, hk, V) <= zero) {
            for (int j : V) mask[j] = 1;
            return true;
        }
    }
    for (int j : order) mask[j] = 1;
    return false;
}

}  // namespace

bool cyclic_recombination_vector(int P, int s, const std::vector<uint8_t>& mask,
                                 std::vector<cplx_t>& b) {
    std::vector<int> V;
    for (int j = 0; j < P; ++j)
        if (mask[j]) V.push_back(j);
    const int a = (int)V.size();
    if (a > 2 * s) return false;
    const int n = P - 2 * s;
    const real_t isq = 1 / std::sqrt((real_t)P);
    // b = C^H [e_last ; B] for free B in C^{2s} (C is unitary, so |b| = |[e;B]|):
    // the smallest b that vanishes on V takes the smallest B with
    //   conj(C[n-1][v]) + sum_m conj(C_R[m][v]) B_m = 0   for v in V.
    std::vector<cplx_t> B(2 * s, cplx_t(0));
    if (a > 0) {
        Mat X(2 * s, a);  // X = C_R[:, V]
        std::vector<cplx_t> rhs(a);
        for (int v = 0; v < a; ++v) {
            for (int m = 0; m < 2 * s; ++m) X(m, v) = isq * root_of_unity(P, (long long)(n + m) * V[v]);
            rhs[v] = -isq * root_of_unity(P, -(long long)(n - 1) * V[v]);
        }
        // X^H B = rhs, minimum norm: X = Q R, B = Q y with R^H y = rhs
        Mat Q(0, 0), R(0, 0);
        qr_mgs(X, Q, R);
        std::vector<cplx_t> y(a);
        for (int i = 0; i < a; ++i) {
            cplx_t acc = rhs[i];
            for (int k = 0; k < i; ++k) acc -= std::conj(R(k, i)) * y[k];
            y[i] = acc / std::conj(R(i, i));
        }
        for (int m = 0; m < 2 * s; ++m) {
            cplx_t acc = 0;
            for (int v = 0; v < a; ++v) acc += Q(m, v) * y[v];
            B[m] = acc;
        }
    }
    b.assign(P, cplx_t(0));
    for (int j = 0; j < P; ++j) {
        if (mask[j]) continue;
        cplx_t acc = isq * root_of_unity(P, -(long long)(n - 1) * j);
        for (int m = 0; m < 2 * s; ++m) acc += isq * root_of_unity(P, -(long long)(n + m) * j) * B[m];
        b[j] = acc;
    }
    return true;
}

}  // namespace draco
