// C ABI of the library (see include/draco.h): argument checks, the plan object
// with its device tables and scratch, and the sequencing of kernels and host
// algebra for each entry point.
#include "../../include/draco.h"
#include "../../include/draco_bench.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <complex>
#include <cstdio>
#include <cstring>
#include <map>
#include <mutex>
#include <new>
#include <random>
#include <tuple>
#include <vector>

#include "host_math.hpp"
#include "kernels.hpp"
#include "projection_rng.hpp"

using namespace draco;

namespace {

enum Kind { kEncode = 0, kVote = 1, kProject = 2, kRecombine = 3, kLocateKind = 4, kKinds = 5 };

// Ring of HIP event pairs bracketing the kernels of one kind.
struct Timer {
    std::vector<hipEvent_t> start, stop;
    int used = 0;
};

}  // namespace

struct draco_plan {
    int code = 0, P = 0, s = 0;
    int64_t d = 0;
    CyclicCode cyc;

    // device side (valid once prepared)
    bool prepared = false;
    int device = -1;
    double2* coef_dev = nullptr;     // P*(2s+1): W[(n+t) mod P][n]
    double* taps_dev = nullptr;      // the factored W: rho[2s+1] (padded to even), rotA[P], rotB[P+2s]
    CycTaps taps{nullptr, nullptr, nullptr};
    double2* partial_dev = nullptr;  // project_tiles(d) * P
    double2* gamma_dev = nullptr;    // P
    double2* b_dev = nullptr;        // P
    double2* b0_dev = nullptr;       // P: recombination vector when no node is flagged
    double2* root_dev = nullptr;     // P: exp(2 pi i k / P)
    int32_t* spec_dev = nullptr;     // 2 words: speculate next / speculated now (see cyc_decode.hip)
    bool speculation = true;
    uint64_t f_seed = 0;             // base seed of the generated projection vector (f_dev == NULL)
    uint64_t f_calls = 0;            // decodes that generated f since the base seed was set
    uint64_t f_last = 0;             // seed the last such decode used
    int wire = DRACO_WIRE_PACKED;    // cyclic code: packed (ceil(d/2) complex) or unpacked (d complex)
    int second_word = DRACO_SECOND_WORD_F32;   // two-word wire: format of the second word
    int32_t* idx_dev = nullptr;      // P, then one more word: the number of honest nodes
    uint64_t* flags_dev = nullptr;   // kMaskWords, zero between calls
    // pinned host staging
    double* gamma_pin = nullptr;     // 2P
    double* b_pin = nullptr;         // 2P
    int32_t* idx_pin = nullptr;      // P
    uint64_t* mask_pin = nullptr;    // pinned, device-mapped: kMaskWords + 1 (status in the last word)
    uint64_t* mask_pin_dev = nullptr;  // the same memory as the device addresses it

    Timer timers[kKinds];
};

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_slab(const void* p, int64_t ld, int64_t row_len) {
    if (p == nullptr) return DRACO_EINVAL;
    if (!aligned16(p) || (ld & 3) != 0 || ld < row_len) return DRACO_EALIGN;
    return DRACO_OK;
}

bool unpacked(const draco_plan* p) { return p->wire == DRACO_WIRE_UNPACKED; }

// Second-word format as the launchers name it, and the locator's zero threshold for a wire.
int lo_format(const draco_plan* p) {
    return p->second_word == DRACO_SECOND_WORD_BF16 ? kSecondWordBf16
           : p->second_word == DRACO_SECOND_WORD_I8 ? kSecondWordI8 : kSecondWordF32;
}
double tau_of(const draco_plan* p, bool wide) {
    if (!wide) return kTauH;
    return p->second_word == DRACO_SECOND_WORD_BF16 ? kTauHBf16
           : p->second_word == DRACO_SECOND_WORD_I8 ? kTauHI8 : kTauHWide;
}

int64_t message_len(const draco_plan* p) {
    if (p->code == DRACO_CODE_REPETITION) return p->d;
    return unpacked(p) ? 2 * p->d : 2 * ((p->d + 1) / 2);
}

// Seed of the generated projection vector for the next decode: the base seed itself for the
// first decode after it was set, then splitmix64's finaliser on base + k * golden ratio for
// the k-th one, so that no two decodes project on the same f.
uint64_t next_projection_seed(draco_plan* p) {
    uint64_t z = p->f_seed + p->f_calls * 0x9E3779B97F4A7C15ull;
    if (p->f_calls != 0) {
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        z ^= z >> 31;
    }
    ++p->f_calls;
    p->f_last = z;
    return z;
}

// Cyclic code: how many floats of a message the decode kernels treat as packed pairs
// (they see the unpacked wire as the packed wire of a gradient twice as long).
int64_t paired_len(const draco_plan* p) { return unpacked(p) ? 2 * p->d : p->d; }

// Text of the last HIP failure seen by this thread (for draco_last_hip_error).
thread_local char g_hip_detail[256] = "";

#define HIP_TRY(expr)                                                                          \
    do {                                                                                       \
        const hipError_t hip_try_e = (expr);                                                   \
        if (hip_try_e != hipSuccess) {                                                         \
            std::snprintf(g_hip_detail, sizeof(g_hip_detail), "%s (line %d): %s", #expr, __LINE__, \
                          hipGetErrorString(hip_try_e));                                       \
            (void)hipGetLastError();                                                           \
            return DRACO_EHIP;                                                                 \
        }                                                                                      \
    } while (0)

int prepare(draco_plan* p) {
    if (p->prepared) {  // a plan stays with the device that was current when it was prepared
        int dev = -1;
        HIP_TRY(hipGetDevice(&dev));
        return dev == p->device ? DRACO_OK : DRACO_EINVAL;
    }
    HIP_TRY(hipGetDevice(&p->device));
    const int P = p->P, r = 2 * p->s + 1;
    HIP_TRY(hipMalloc(&p->flags_dev, kMaskWords * sizeof(uint64_t)));
    HIP_TRY(hipMemset(p->flags_dev, 0, kMaskWords * sizeof(uint64_t)));
    // The synchronous decoders let the last kernel write mask and status straight into
    // mapped host memory: the host reads them after the stream wait, no copy commands.
    HIP_TRY(hipHostMalloc(&p->mask_pin, (kMaskWords + 1) * sizeof(uint64_t), hipHostMallocMapped));
    HIP_TRY(hipHostGetDevicePointer(reinterpret_cast<void**>(&p->mask_pin_dev), p->mask_pin, 0));
    if (p->code == DRACO_CODE_CYCLIC) {
        HIP_TRY(hipMalloc(&p->coef_dev, (size_t)P * r * sizeof(double2)));
        HIP_TRY(hipMalloc(&p->partial_dev, (size_t)project_tiles(paired_len(p)) * P * sizeof(double2)));
        HIP_TRY(hipMalloc(&p->gamma_dev, P * sizeof(double2)));
        HIP_TRY(hipMalloc(&p->b_dev, P * sizeof(double2)));
        HIP_TRY(hipMalloc(&p->b0_dev, P * sizeof(double2)));
        HIP_TRY(hipMalloc(&p->spec_dev, 2 * sizeof(int32_t)));
        {
            std::vector<uint8_t> none(P, 0);
            std::vector<cplx_t> b0;
            cyclic_recombination_vector(P, p->s, none, b0);
            std::vector<double> t0(2 * P);
            for (int j = 0; j < P; ++j) {
                t0[2 * j] = (double)b0[j].real();
                t0[2 * j + 1] = (double)b0[j].imag();
            }
            HIP_TRY(hipMemcpy(p->b0_dev, t0.data(), P * sizeof(double2), hipMemcpyHostToDevice));
            for (int k = 0; k < P; ++k) {
                const cplx_t w = root_of_unity(P, k);
                t0[2 * k] = (double)w.real();
                t0[2 * k + 1] = (double)w.imag();
            }
            HIP_TRY(hipMalloc(&p->root_dev, P * sizeof(double2)));
            HIP_TRY(hipMemcpy(p->root_dev, t0.data(), P * sizeof(double2), hipMemcpyHostToDevice));
            const int32_t init[2] = {1, 0};  // optimistic: the first decode speculates
            HIP_TRY(hipMemcpy(p->spec_dev, init, sizeof(init), hipMemcpyHostToDevice));
        }
        HIP_TRY(hipMalloc(&p->idx_dev, (P + 1) * sizeof(int32_t)));
        HIP_TRY(hipHostMalloc(&p->gamma_pin, 2 * P * sizeof(double), hipHostMallocDefault));
        HIP_TRY(hipHostMalloc(&p->b_pin, 2 * P * sizeof(double), hipHostMallocDefault));
        HIP_TRY(hipHostMalloc(&p->idx_pin, (P + 1) * sizeof(int32_t), hipHostMallocDefault));
        std::vector<double> tmp((size_t)2 * P * r);
        for (int n = 0; n < P; ++n)
            for (int t = 0; t < r; ++t) {
                const cplx_t w = p->cyc.W((n + t) % P, n);
                tmp[2 * ((size_t)n * r + t)] = (double)w.real();
                tmp[2 * ((size_t)n * r + t) + 1] = (double)w.imag();
            }
        HIP_TRY(hipMemcpy(p->coef_dev, tmp.data(), tmp.size() * sizeof(double), hipMemcpyHostToDevice));
        // the factored form for the packed encoders: real taps, then the two tables of unit phases
        const int nrho = (r + 1) / 2 * 2, nB = P + 2 * p->s;   // rho padded so the phases stay 16-byte aligned
        std::vector<double> fac((size_t)nrho + 2 * P + 2 * nB, 0.0);
        for (int t = 0; t < r; ++t) fac[t] = (double)p->cyc.real_taps[t];
        for (int j = 0; j < P; ++j) {
            fac[nrho + 2 * j] = (double)p->cyc.node_phase[j].real();
            fac[nrho + 2 * j + 1] = (double)p->cyc.node_phase[j].imag();
        }
        for (int k = 0; k < nB; ++k) {
            fac[nrho + 2 * P + 2 * k] = (double)p->cyc.row_phase[k].real();
            fac[nrho + 2 * P + 2 * k + 1] = (double)p->cyc.row_phase[k].imag();
        }
        HIP_TRY(hipMalloc(&p->taps_dev, fac.size() * sizeof(double)));
        HIP_TRY(hipMemcpy(p->taps_dev, fac.data(), fac.size() * sizeof(double), hipMemcpyHostToDevice));
        p->taps.rho = p->taps_dev;
        p->taps.rotA = reinterpret_cast<const double2*>(p->taps_dev + nrho);
        p->taps.rotB = reinterpret_cast<const double2*>(p->taps_dev + nrho + 2 * P);
    }
    p->prepared = true;
    return DRACO_OK;
}

// Brackets the kernels launched in its scope with the next free event pair.
struct Timed {
    Timer* t;
    hipStream_t st;
    bool on;
    Timed(draco_plan* plan, Kind k, hipStream_t stream) : t(&plan->timers[k]), st(stream) {
        on = t->used < (int)t->start.size();
        if (on) (void)hipEventRecord(t->start[t->used], st);
    }
    ~Timed() {
        if (on) {
            (void)hipEventRecord(t->stop[t->used], st);
            ++t->used;
        }
    }
};

void words_from_mask(const std::vector<uint8_t>& mask, uint64_t* words, int P) {
    for (int w = 0; w < (P + 63) / 64; ++w) words[w] = 0;
    for (int j = 0; j < P; ++j)
        if (mask[j]) words[j >> 6] |= 1ull << (j & 63);
}

}  // namespace

extern "C" {

int draco_plan_create(draco_plan** out, int code, int P, int s, int64_t d) {
    if (out == nullptr) return DRACO_EINVAL;
    if (code != DRACO_CODE_REPETITION && code != DRACO_CODE_CYCLIC) return DRACO_EINVAL;
    if (P < 1 || P > DRACO_MAX_NODES || s < 0 || d < 1 || d > DRACO_MAX_DIM) return DRACO_EINVAL;
    if (2 * (int64_t)s + 1 > P) return DRACO_EINVAL;                               // corollary to Theorem 1
    if (code == DRACO_CODE_REPETITION && P % (2 * s + 1) != 0) return DRACO_EINVAL; // "Suppose 2s+1 divides P"
    draco_plan* p = new (std::nothrow) draco_plan();
    if (p == nullptr) return DRACO_ENOMEM;
    p->code = code;
    p->P = P;
    p->s = s;
    p->d = d;
    if (code == DRACO_CODE_CYCLIC) {
        p->cyc.build(P, s);
        // phi draws f afresh for every decode (Lemma 3 needs f unknown to the adversaries):
        // the base seed comes from the system's entropy source unless the caller sets one
        std::random_device rd;
        p->f_seed = ((uint64_t)rd() << 32) ^ (uint64_t)rd();
    }
    *out = p;
    return DRACO_OK;
}

int draco_plan_prepare(draco_plan* plan) {
    if (plan == nullptr) return DRACO_EINVAL;
    return prepare(plan);
}

void draco_plan_destroy(draco_plan* p) {
    if (p == nullptr) return;
    if (p->device >= 0) {
        (void)hipDeviceSynchronize();
        (void)hipFree(p->coef_dev);
        (void)hipFree(p->taps_dev);
        (void)hipFree(p->partial_dev);
        (void)hipFree(p->gamma_dev);
        (void)hipFree(p->b_dev);
        (void)hipFree(p->b0_dev);
        (void)hipFree(p->root_dev);
        (void)hipFree(p->spec_dev);
        (void)hipFree(p->idx_dev);
        (void)hipFree(p->flags_dev);
        (void)hipHostFree(p->gamma_pin);
        (void)hipHostFree(p->b_pin);
        (void)hipHostFree(p->idx_pin);
        (void)hipHostFree(p->mask_pin);
        for (auto& t : p->timers) {
            for (hipEvent_t e : t.start) (void)hipEventDestroy(e);
            for (hipEvent_t e : t.stop) (void)hipEventDestroy(e);
        }
    }
    delete p;
}

int64_t draco_message_len(const draco_plan* plan) {
    if (plan == nullptr) return DRACO_EINVAL;
    return message_len(plan);
}

int draco_plan_assign(const draco_plan* p, uint8_t* A) {
    if (p == nullptr || A == nullptr) return DRACO_EINVAL;
    const int P = p->P, r = 2 * p->s + 1;
    std::memset(A, 0, (size_t)P * P);
    for (int j = 0; j < P; ++j)
        for (int t = 0; t < r; ++t) {
            const int k = (p->code == DRACO_CODE_REPETITION) ? (j / r) * r + t : (j + t) % P;
            A[(size_t)j * P + k] = 1;
        }
    return DRACO_OK;
}

int draco_plan_weights(const draco_plan* p, double* W) {
    if (p == nullptr || W == nullptr) return DRACO_EINVAL;
    const int P = p->P, r = 2 * p->s + 1;
    for (int k = 0; k < P; ++k)
        for (int j = 0; j < P; ++j) {
            double re = 0.0, im = 0.0;
            if (p->code == DRACO_CODE_REPETITION) {
                re = (k / r == j / r) ? 1.0 : 0.0;
            } else {
                const cplx_t w = p->cyc.W(k, j);
                re = (double)w.real();
                im = (double)w.imag();
            }
            W[((size_t)k * P + j) * 2] = re;
            W[((size_t)k * P + j) * 2 + 1] = im;
        }
    return DRACO_OK;
}

namespace {

int encode_impl(draco_plan* p, const float* grads_dev, int64_t ld_g, float* hi_dev, float* lo_dev, bool wide,
                int64_t ld_m, void* stream) {
    if (p == nullptr) return DRACO_EINVAL;
    if (wide && (p->code != DRACO_CODE_CYCLIC || unpacked(p))) return DRACO_EINVAL;
    int rc = check_slab(grads_dev, ld_g, p->d);
    if (rc != DRACO_OK) return rc;
    rc = check_slab(hi_dev, ld_m, message_len(p));
    if (rc != DRACO_OK) return rc;
    if (wide) {
        rc = check_slab(lo_dev, ld_m, message_len(p));
        if (rc != DRACO_OK) return rc;
    }
    rc = prepare(p);
    if (rc != DRACO_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    Timed timed(p, kEncode, st);
    if (p->code == DRACO_CODE_REPETITION)
        HIP_TRY(launch_encode_rep(grads_dev, ld_g, hi_dev, ld_m, p->P, p->s, p->d, st));
    else if (unpacked(p))
        HIP_TRY(launch_encode_cyc_real(grads_dev, ld_g, hi_dev, ld_m, p->coef_dev, p->P, p->s, p->d, st));
    else
        HIP_TRY(launch_encode_cyc(grads_dev, ld_g, hi_dev, wide ? lo_dev : nullptr, lo_format(p), ld_m, p->taps,
                                  p->P, p->s, p->d, st));
    return DRACO_OK;
}

}  // namespace

int draco_encode(draco_plan* p, const float* grads_dev, int64_t ld_g, float* messages_dev, int64_t ld_m,
                 void* stream) {
    return encode_impl(p, grads_dev, ld_g, messages_dev, nullptr, false, ld_m, stream);
}

int draco_encode_wide(draco_plan* p, const float* grads_dev, int64_t ld_g, float* messages_hi_dev,
                      void* messages_lo_dev, int64_t ld_m, void* stream) {
    return encode_impl(p, grads_dev, ld_g, messages_hi_dev, static_cast<float*>(messages_lo_dev), true, ld_m, stream);
}

namespace {

int encode_samples_impl(draco_plan* p, const float* samples_dev, int64_t B, int64_t ld_g, float* messages_dev,
                        float* lo_dev, bool wide, int64_t ld_m, void* stream) {
    if (p == nullptr || B < p->P || B % p->P != 0 || B / p->P > (1 << 20)) return DRACO_EINVAL;
    if (unpacked(p) && B != p->P) return DRACO_EINVAL;
    if (wide && (p->code != DRACO_CODE_CYCLIC || unpacked(p))) return DRACO_EINVAL;
    const int m = (int)(B / p->P);
    if (m == 1) return encode_impl(p, samples_dev, ld_g, messages_dev, lo_dev, wide, ld_m, stream);
    int rc = check_slab(samples_dev, ld_g, p->d);
    if (rc != DRACO_OK) return rc;
    rc = check_slab(messages_dev, ld_m, message_len(p));
    if (rc != DRACO_OK) return rc;
    if (wide) {
        rc = check_slab(lo_dev, ld_m, message_len(p));
        if (rc != DRACO_OK) return rc;
    }
    rc = prepare(p);
    if (rc != DRACO_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    Timed timed(p, kEncode, st);
    if (p->code == DRACO_CODE_REPETITION)
        HIP_TRY(launch_encode_rep_samples(samples_dev, ld_g, m, messages_dev, ld_m, p->P, p->s, p->d, st));
    else
        HIP_TRY(launch_encode_cyc_samples(samples_dev, ld_g, m, messages_dev, wide ? lo_dev : nullptr, lo_format(p), ld_m, p->taps,
                                          p->P, p->s, p->d, st));
    return DRACO_OK;
}

}  // namespace

int draco_encode_samples(draco_plan* p, const float* samples_dev, int64_t B, int64_t ld_g, float* messages_dev,
                         int64_t ld_m, void* stream) {
    return encode_samples_impl(p, samples_dev, B, ld_g, messages_dev, nullptr, false, ld_m, stream);
}

int draco_encode_samples_wide(draco_plan* p, const float* samples_dev, int64_t B, int64_t ld_g,
                              float* messages_hi_dev, void* messages_lo_dev, int64_t ld_m, void* stream) {
    return encode_samples_impl(p, samples_dev, B, ld_g, messages_hi_dev, static_cast<float*>(messages_lo_dev), true, ld_m, stream);
}

namespace {

int encode_node_impl(draco_plan* p, int node, const float* node_grads_dev, int64_t ld_g, float* message_dev,
                     float* lo_dev, bool wide, void* stream) {
    if (p == nullptr || node < 0 || node >= p->P) return DRACO_EINVAL;
    if (wide && (p->code != DRACO_CODE_CYCLIC || unpacked(p) || lo_dev == nullptr)) return DRACO_EINVAL;
    int rc = check_slab(node_grads_dev, ld_g, p->d);
    if (rc != DRACO_OK) return rc;
    if (message_dev == nullptr) return DRACO_EINVAL;
    if (!aligned16(message_dev) || (wide && !aligned16(lo_dev))) return DRACO_EALIGN;
    rc = prepare(p);
    if (rc != DRACO_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    Timed timed(p, kEncode, st);
    if (p->code == DRACO_CODE_REPETITION)
        HIP_TRY(launch_encode_rep_node(node_grads_dev, ld_g, message_dev, p->s, p->d, st));
    else if (unpacked(p))
        HIP_TRY(launch_encode_cyc_real_node(node_grads_dev, ld_g, message_dev, p->coef_dev, node, p->P, p->s, p->d, st));
    else
        HIP_TRY(launch_encode_cyc_node(node_grads_dev, ld_g, message_dev, wide ? lo_dev : nullptr, lo_format(p), p->taps,
                                       node, p->P, p->s, p->d, st));
    return DRACO_OK;
}

}  // namespace

int draco_encode_node(draco_plan* p, int node, const float* node_grads_dev, int64_t ld_g, float* message_dev,
                      void* stream) {
    return encode_node_impl(p, node, node_grads_dev, ld_g, message_dev, nullptr, false, stream);
}

int draco_encode_node_wide(draco_plan* p, int node, const float* node_grads_dev, int64_t ld_g,
                           float* message_hi_dev, void* message_lo_dev, void* stream) {
    return encode_node_impl(p, node, node_grads_dev, ld_g, message_hi_dev, static_cast<float*>(message_lo_dev), true,
                            stream);
}

int draco_decode_repetition_async(draco_plan* p, const float* messages_dev, int64_t ld_m, float* sum_dev,
                                  uint64_t* mask_dev, int32_t* status_dev, void* stream) {
    if (p == nullptr || p->code != DRACO_CODE_REPETITION) return DRACO_EINVAL;
    if (sum_dev == nullptr || mask_dev == nullptr || status_dev == nullptr) return DRACO_EINVAL;
    int rc = check_slab(messages_dev, ld_m, p->d);
    if (rc != DRACO_OK) return rc;
    if (!aligned16(sum_dev)) return DRACO_EALIGN;
    rc = prepare(p);
    if (rc != DRACO_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    {
        Timed timed(p, kVote, st);
        HIP_TRY(launch_decode_rep_vote(messages_dev, ld_m, sum_dev, p->flags_dev, p->P, p->s, p->d, st));
    }
    HIP_TRY(launch_decode_rep_finish(p->flags_dev, mask_dev, status_dev, p->P, p->s, st));
    return DRACO_OK;
}

int draco_decode_repetition(draco_plan* p, const float* messages_dev, int64_t ld_m, float* sum_dev,
                            uint64_t* mask_host, void* stream) {
    if (p == nullptr || mask_host == nullptr) return DRACO_EINVAL;
    int rc = prepare(p);
    if (rc != DRACO_OK) return rc;
    rc = draco_decode_repetition_async(p, messages_dev, ld_m, sum_dev, p->mask_pin_dev,
                                       reinterpret_cast<int32_t*>(p->mask_pin_dev + kMaskWords), stream);
    if (rc != DRACO_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int words = (p->P + 63) / 64;
    HIP_TRY(hipStreamSynchronize(st));
    for (int w = 0; w < words; ++w) mask_host[w] = p->mask_pin[w];
    int32_t status;
    std::memcpy(&status, p->mask_pin + kMaskWords, sizeof(status));
    return status;
}

int draco_decode_repetition_static(int P, int s, int64_t d, const float* messages_dev, int64_t ld_m, float* sum_dev,
                                   uint64_t* mask_dev, int32_t* status_dev, void* stream) {
    if (P < 1 || P > DRACO_MAX_NODES || s < 0 || d < 1 || d > DRACO_MAX_DIM) return DRACO_EINVAL;
    if (2 * (int64_t)s + 1 > P || P % (2 * s + 1) != 0) return DRACO_EINVAL;
    if (sum_dev == nullptr || mask_dev == nullptr || status_dev == nullptr) return DRACO_EINVAL;
    const int rc = check_slab(messages_dev, ld_m, d);
    if (rc != DRACO_OK) return rc;
    if (!aligned16(sum_dev)) return DRACO_EALIGN;
    HIP_TRY(launch_decode_rep_static(messages_dev, ld_m, sum_dev, mask_dev, status_dev, P, s, d,
                                     static_cast<hipStream_t>(stream)));
    return DRACO_OK;
}

namespace {

int check_cyclic_args(draco_plan* p, const float* hi_dev, const float* lo_dev, bool wide, int64_t ld_m,
                      const float* f_dev, float* sum_dev) {
    if (p == nullptr || p->code != DRACO_CODE_CYCLIC) return DRACO_EINVAL;
    if (sum_dev == nullptr || (wide && unpacked(p))) return DRACO_EINVAL;
    int rc = check_slab(hi_dev, ld_m, message_len(p));
    if (rc != DRACO_OK) return rc;
    if (wide) {
        rc = check_slab(lo_dev, ld_m, message_len(p));
        if (rc != DRACO_OK) return rc;
    }
    if (!aligned16(sum_dev) || (reinterpret_cast<uintptr_t>(f_dev) & 3u) != 0) return DRACO_EALIGN;
    return prepare(p);
}

int decode_cyclic_async_impl(draco_plan* p, const float* hi_dev, const float* lo_dev, bool wide, int64_t ld_m,
                             const float* f_dev, float* sum_dev, uint64_t* mask_dev, int32_t* status_dev,
                             void* stream) {
    if (mask_dev == nullptr || status_dev == nullptr) return DRACO_EINVAL;
    int rc = check_cyclic_args(p, hi_dev, lo_dev, wide, ld_m, f_dev, sum_dev);
    if (rc != DRACO_OK) return rc;
    if (p->s > kLocateMaxS) return DRACO_EINVAL;
    const float* lo = wide ? lo_dev : nullptr;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int P = p->P;
    int32_t* spec = p->speculation ? p->spec_dev : nullptr;
    const uint64_t seed = f_dev == nullptr ? next_projection_seed(p) : 0;
    {
        Timed timed(p, kProject, st);
        HIP_TRY(launch_cyc_project(hi_dev, lo, lo_format(p), ld_m, f_dev, seed, p->partial_dev, p->gamma_dev, p->b0_dev,
                                   sum_dev, unpacked(p), spec, P, paired_len(p), st));
    }
    {
        Timed timed(p, kLocateKind, st);
        HIP_TRY(launch_cyc_locate(p->gamma_dev, p->root_dev, P, p->s, tau_of(p, wide), p->b0_dev, mask_dev, status_dev,
                                  p->b_dev, p->idx_dev, p->idx_dev + P, spec, st));
    }
    {
        Timed timed(p, kRecombine, st);
        HIP_TRY(launch_cyc_recombine(hi_dev, lo, lo_format(p), ld_m, p->b_dev, p->idx_dev, p->idx_dev + P, spec, P, sum_dev,
                                     unpacked(p), paired_len(p), st));
    }
    return DRACO_OK;
}

int decode_cyclic_hostphi_impl(draco_plan* p, const float* hi_dev, const float* lo_dev, bool wide, int64_t ld_m,
                               const float* f_dev, float* sum_dev, uint64_t* mask_host, void* stream) {
    if (mask_host == nullptr) return DRACO_EINVAL;
    int rc = check_cyclic_args(p, hi_dev, lo_dev, wide, ld_m, f_dev, sum_dev);
    if (rc != DRACO_OK) return rc;
    const float* lo = wide ? lo_dev : nullptr;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int P = p->P, s = p->s;
    const uint64_t seed = f_dev == nullptr ? next_projection_seed(p) : 0;
    {
        Timed timed(p, kProject, st);
        HIP_TRY(launch_cyc_project(hi_dev, lo, lo_format(p), ld_m, f_dev, seed, p->partial_dev, p->gamma_dev, p->b0_dev,
                                   sum_dev, unpacked(p), nullptr, P, paired_len(p), st));
    }
    HIP_TRY(hipMemcpyAsync(p->gamma_pin, p->gamma_dev, P * sizeof(double2), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));

    std::vector<std::complex<double>> gamma(P), t;
    for (int j = 0; j < P; ++j) gamma[j] = std::complex<double>(p->gamma_pin[2 * j], p->gamma_pin[2 * j + 1]);
    std::vector<uint8_t> mask;
    const bool located = cyclic_locate(P, s, tau_of(p, wide), gamma.data(), mask, t);
    words_from_mask(mask, mask_host, P);
    std::vector<cplx_t> b;
    if (!cyclic_recombination_vector(P, s, mask, b)) return DRACO_LOCATE_FAILED;
    int nu = 0;
    for (int j = 0; j < P; ++j) {
        if (mask[j]) continue;
        p->idx_pin[nu] = j;
        p->b_pin[2 * nu] = (double)b[j].real();
        p->b_pin[2 * nu + 1] = (double)b[j].imag();
        ++nu;
    }
    p->idx_pin[P] = nu;
    HIP_TRY(hipMemcpyAsync(p->b_dev, p->b_pin, nu * sizeof(double2), hipMemcpyHostToDevice, st));
    HIP_TRY(hipMemcpyAsync(p->idx_dev, p->idx_pin, (P + 1) * sizeof(int32_t), hipMemcpyHostToDevice, st));
    {
        Timed timed(p, kRecombine, st);
        HIP_TRY(launch_cyc_recombine(hi_dev, lo, lo_format(p), ld_m, p->b_dev, p->idx_dev, p->idx_dev + P, nullptr, P, sum_dev,
                                     unpacked(p), paired_len(p), st));
    }
    HIP_TRY(hipStreamSynchronize(st));
    return located ? DRACO_OK : DRACO_LOCATE_FAILED;
}

int decode_cyclic_impl(draco_plan* p, const float* hi_dev, const float* lo_dev, bool wide, int64_t ld_m,
                       const float* f_dev, float* sum_dev, uint64_t* mask_host, void* stream) {
    if (p == nullptr || mask_host == nullptr) return DRACO_EINVAL;
    if (p->s > kLocateMaxS)
        return decode_cyclic_hostphi_impl(p, hi_dev, lo_dev, wide, ld_m, f_dev, sum_dev, mask_host, stream);
    int rc = prepare(p);
    if (rc != DRACO_OK) return rc;
    rc = decode_cyclic_async_impl(p, hi_dev, lo_dev, wide, ld_m, f_dev, sum_dev, p->mask_pin_dev,
                                  reinterpret_cast<int32_t*>(p->mask_pin_dev + kMaskWords), stream);
    if (rc != DRACO_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int words = (p->P + 63) / 64;
    HIP_TRY(hipStreamSynchronize(st));
    for (int w = 0; w < words; ++w) mask_host[w] = p->mask_pin[w];
    int32_t status;
    std::memcpy(&status, p->mask_pin + kMaskWords, sizeof(status));
    return status;
}

}  // namespace

int draco_decode_cyclic(draco_plan* p, const float* messages_dev, int64_t ld_m, const float* f_dev, float* sum_dev,
                        uint64_t* mask_host, void* stream) {
    return decode_cyclic_impl(p, messages_dev, nullptr, false, ld_m, f_dev, sum_dev, mask_host, stream);
}

int draco_decode_cyclic_async(draco_plan* p, const float* messages_dev, int64_t ld_m, const float* f_dev,
                              float* sum_dev, uint64_t* mask_dev, int32_t* status_dev, void* stream) {
    return decode_cyclic_async_impl(p, messages_dev, nullptr, false, ld_m, f_dev, sum_dev, mask_dev, status_dev,
                                    stream);
}

int draco_decode_cyclic_hostphi(draco_plan* p, const float* messages_dev, int64_t ld_m, const float* f_dev,
                                float* sum_dev, uint64_t* mask_host, void* stream) {
    return decode_cyclic_hostphi_impl(p, messages_dev, nullptr, false, ld_m, f_dev, sum_dev, mask_host, stream);
}

int draco_decode_cyclic_wide(draco_plan* p, const float* messages_hi_dev, const void* messages_lo_dev, int64_t ld_m,
                             const float* f_dev, float* sum_dev, uint64_t* mask_host, void* stream) {
    return decode_cyclic_impl(p, messages_hi_dev, static_cast<const float*>(messages_lo_dev), true, ld_m, f_dev, sum_dev, mask_host, stream);
}

int draco_decode_cyclic_wide_async(draco_plan* p, const float* messages_hi_dev, const void* messages_lo_dev,
                                   int64_t ld_m, const float* f_dev, float* sum_dev, uint64_t* mask_dev,
                                   int32_t* status_dev, void* stream) {
    return decode_cyclic_async_impl(p, messages_hi_dev, static_cast<const float*>(messages_lo_dev), true, ld_m, f_dev, sum_dev, mask_dev,
                                    status_dev, stream);
}

int draco_cyclic_locate(const draco_plan* p, const double* gamma_host, uint64_t* mask_host, double* t_host) {
    return draco_cyclic_locate_tol(p, gamma_host, kTauH, mask_host, t_host);
}

int draco_cyclic_locate_tol(const draco_plan* p, const double* gamma_host, double tau, uint64_t* mask_host,
                            double* t_host) {
    if (p == nullptr || p->code != DRACO_CODE_CYCLIC || gamma_host == nullptr || mask_host == nullptr)
        return DRACO_EINVAL;
    if (!(tau > 0.0 && tau < 1.0)) return DRACO_EINVAL;
    const int P = p->P;
    std::vector<std::complex<double>> gamma(P), t;
    for (int j = 0; j < P; ++j) gamma[j] = std::complex<double>(gamma_host[2 * j], gamma_host[2 * j + 1]);
    std::vector<uint8_t> mask;
    const bool ok = cyclic_locate(P, p->s, tau, gamma.data(), mask, t);
    words_from_mask(mask, mask_host, P);
    if (t_host != nullptr)
        for (int j = 0; j < P; ++j) {
            t_host[2 * j] = t[j].real();
            t_host[2 * j + 1] = t[j].imag();
        }
    return ok ? DRACO_OK : DRACO_LOCATE_FAILED;
}

int draco_cyclic_recombination_vector(const draco_plan* p, const uint64_t* mask_host, double* b_host) {
    if (p == nullptr || p->code != DRACO_CODE_CYCLIC || mask_host == nullptr || b_host == nullptr)
        return DRACO_EINVAL;
    const int P = p->P;
    std::vector<uint8_t> mask(P);
    for (int j = 0; j < P; ++j) mask[j] = (uint8_t)((mask_host[j >> 6] >> (j & 63)) & 1ull);
    std::vector<cplx_t> b;
    if (!cyclic_recombination_vector(P, p->s, mask, b)) return DRACO_EINVAL;
    for (int j = 0; j < P; ++j) {
        b_host[2 * j] = (double)b[j].real();
        b_host[2 * j + 1] = (double)b[j].imag();
    }
    return DRACO_OK;
}

const char* draco_strerror(int status) {
    switch (status) {
        case DRACO_OK: return "ok";
        case DRACO_NO_MAJORITY: return "repetition code: a group has more than s nodes that differ from its vote";
        case DRACO_LOCATE_FAILED: return "cyclic code: no set of at most s nodes accounts for the syndromes";
        case DRACO_EINVAL: return "invalid argument";
        case DRACO_EALIGN: return "pointer not 16-byte aligned or stride not a multiple of 4 floats / too short";
        case DRACO_EHIP: return "HIP runtime error";
        case DRACO_ENOMEM: return "out of host memory";
        default: return "unknown status";
    }
}

const char* draco_last_hip_error(void) { return g_hip_detail; }

int draco_plan_set_wire(draco_plan* p, int wire) {
    if (p == nullptr || p->code != DRACO_CODE_CYCLIC || p->prepared) return DRACO_EINVAL;
    if (wire != DRACO_WIRE_PACKED && wire != DRACO_WIRE_UNPACKED) return DRACO_EINVAL;
    p->wire = wire;
    return DRACO_OK;
}

int draco_plan_set_second_word(draco_plan* p, int format) {
    if (p == nullptr || p->code != DRACO_CODE_CYCLIC || unpacked(p)) return DRACO_EINVAL;
    if (format != DRACO_SECOND_WORD_F32 && format != DRACO_SECOND_WORD_BF16 && format != DRACO_SECOND_WORD_I8)
        return DRACO_EINVAL;
    p->second_word = format;
    return DRACO_OK;
}

int draco_plan_set_projection_seed(draco_plan* p, uint64_t seed) {
    if (p == nullptr || p->code != DRACO_CODE_CYCLIC) return DRACO_EINVAL;
    p->f_seed = seed;
    p->f_calls = 0;
    return DRACO_OK;
}

int draco_plan_last_projection_seed(const draco_plan* p, uint64_t* seed) {
    if (p == nullptr || seed == nullptr || p->code != DRACO_CODE_CYCLIC || p->f_calls == 0) return DRACO_EINVAL;
    *seed = p->f_last;
    return DRACO_OK;
}

int draco_projection_vector(const draco_plan* p, uint64_t seed, float* f_host) {
    if (p == nullptr || p->code != DRACO_CODE_CYCLIC || f_host == nullptr) return DRACO_EINVAL;
    const int64_t h = message_len(p) / 2;
    for (int64_t i = 0; i < h; ++i) f_host[i] = projection_entry(seed, (uint64_t)i);
    return DRACO_OK;
}

int draco_plan_set_speculation(draco_plan* p, int enabled) {
    if (p == nullptr) return DRACO_EINVAL;
    p->speculation = enabled != 0;
    return DRACO_OK;
}

int draco_copy_probe(const float* src_dev, float* dst_dev, int rows, int64_t row_len, int64_t ld, void* stream) {
    if (src_dev == nullptr || dst_dev == nullptr || rows < 1 || rows > 65535 || row_len < 4) return DRACO_EINVAL;
    if (!aligned16(src_dev) || !aligned16(dst_dev) || (row_len & 3) != 0 || (ld & 3) != 0 || ld < row_len)
        return DRACO_EALIGN;
    HIP_TRY(launch_copy_probe(src_dev, dst_dev, rows, row_len, ld, static_cast<hipStream_t>(stream)));
    return DRACO_OK;
}

int draco_plan_set_timing(draco_plan* p, int max_records) {
    if (p == nullptr || max_records < 0 || max_records > 65536) return DRACO_EINVAL;
    int rc = prepare(p);
    if (rc != DRACO_OK) return rc;
    for (auto& t : p->timers) {
        while ((int)t.start.size() > max_records) {
            (void)hipEventDestroy(t.start.back());
            (void)hipEventDestroy(t.stop.back());
            t.start.pop_back();
            t.stop.pop_back();
        }
        while ((int)t.start.size() < max_records) {
            hipEvent_t a = nullptr, b = nullptr;
            HIP_TRY(hipEventCreate(&a));
            if (hipEventCreate(&b) != hipSuccess) {
                (void)hipEventDestroy(a);
                return DRACO_EHIP;
            }
            t.start.push_back(a);
            t.stop.push_back(b);
        }
        t.used = 0;
    }
    return DRACO_OK;
}

int draco_plan_kernel_time(draco_plan* p, int kind, double* total_ms, int* launches) {
    if (p == nullptr || kind < 0 || kind >= kKinds || total_ms == nullptr || launches == nullptr) return DRACO_EINVAL;
    Timer& t = p->timers[kind];
    double sum = 0.0;
    for (int i = 0; i < t.used; ++i) {
        HIP_TRY(hipEventSynchronize(t.stop[i]));
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, t.start[i], t.stop[i]));
        sum += (double)ms;
    }
    *total_ms = sum;
    *launches = t.used;
    t.used = 0;
    return DRACO_OK;
}

int draco_plan_kernel_times(draco_plan* p, int kind, double* ms_host, int capacity, int* launches) {
    if (p == nullptr || kind < 0 || kind >= kKinds || launches == nullptr || capacity < 0) return DRACO_EINVAL;
    if (capacity > 0 && ms_host == nullptr) return DRACO_EINVAL;
    Timer& t = p->timers[kind];
    for (int i = 0; i < t.used; ++i) {
        HIP_TRY(hipEventSynchronize(t.stop[i]));
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, t.start[i], t.stop[i]));
        if (i < capacity) ms_host[i] = (double)ms;
    }
    *launches = t.used;
    t.used = 0;
    return DRACO_OK;
}

int draco_apply_update(float* params_dev, const float* sum_dev, int64_t d, float scale, void* stream) {
    if (params_dev == nullptr || sum_dev == nullptr || d < 1 || d > DRACO_MAX_DIM) return DRACO_EINVAL;
    if (!aligned16(params_dev) || !aligned16(sum_dev)) return DRACO_EALIGN;
    HIP_TRY(launch_apply_update(params_dev, sum_dev, scale, d, static_cast<hipStream_t>(stream)));
    return DRACO_OK;
}

}  // extern "C"

// ---------------------------------------------------------------------------
// Plan-free forms: (code, P, s, d) in, a cached plan per parameter set and device inside.
// ---------------------------------------------------------------------------
namespace {

struct CachedPlan {
    draco_plan* plan = nullptr;
    std::mutex busy;  // a plan's scratch serves one call at a time
};
using CacheKey = std::tuple<int, int, int, int64_t, int>;  // code, P, s, d, device

std::mutex g_cache_mutex;
// never destroyed: plans hold device memory, and the HIP runtime may be gone by the time
// static destructors run; draco_cache_clear() is the way to release them
std::map<CacheKey, CachedPlan*>* g_cache = nullptr;

int cached_plan(int code, int P, int s, int64_t d, CachedPlan** out) {
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lock(g_cache_mutex);
    if (g_cache == nullptr) g_cache = new (std::nothrow) std::map<CacheKey, CachedPlan*>();
    if (g_cache == nullptr) return DRACO_ENOMEM;
    const CacheKey key(code, P, s, d, dev);
    auto it = g_cache->find(key);
    if (it == g_cache->end()) {
        draco_plan* plan = nullptr;
        int rc = draco_plan_create(&plan, code, P, s, d);
        if (rc != DRACO_OK) return rc;
        rc = prepare(plan);
        if (rc != DRACO_OK) {
            draco_plan_destroy(plan);
            return rc;
        }
        CachedPlan* c = new (std::nothrow) CachedPlan();
        if (c == nullptr) {
            draco_plan_destroy(plan);
            return DRACO_ENOMEM;
        }
        c->plan = plan;
        it = g_cache->emplace(key, c).first;
    }
    *out = it->second;
    return DRACO_OK;
}

}  // namespace

extern "C" {

int draco_encode_oneshot(const uint8_t* assign_host, int code, int P, int64_t d, const float* samples_dev, int64_t B,
                         int64_t ld_g, float* messages_dev, int64_t ld_m, void* stream) {
    if (assign_host == nullptr || P < 1 || P > DRACO_MAX_NODES) return DRACO_EINVAL;
    // the assignment matrix names the code: every node holds r = 2s+1 gradients
    int r = 0;
    for (int k = 0; k < P; ++k) r += assign_host[k] != 0;
    if (r < 1 || (r & 1) == 0) return DRACO_EINVAL;
    const int s = (r - 1) / 2;
    CachedPlan* c = nullptr;
    int rc = cached_plan(code, P, s, d, &c);
    if (rc != DRACO_OK) return rc;
    std::vector<uint8_t> A((size_t)P * P);
    rc = draco_plan_assign(c->plan, A.data());
    if (rc != DRACO_OK) return rc;
    for (size_t i = 0; i < A.size(); ++i)
        if ((assign_host[i] != 0) != (A[i] != 0)) return DRACO_EINVAL;  // not this code's allocation matrix
    std::lock_guard<std::mutex> lock(c->busy);
    return draco_encode_samples(c->plan, samples_dev, B, ld_g, messages_dev, ld_m, stream);
}

int draco_decode_repetition_oneshot(const float* messages_dev, int64_t ld_m, int P, int s, int64_t d, float* sum_dev,
                                    uint64_t* mask_host, void* stream) {
    CachedPlan* c = nullptr;
    const int rc = cached_plan(DRACO_CODE_REPETITION, P, s, d, &c);
    if (rc != DRACO_OK) return rc;
    std::lock_guard<std::mutex> lock(c->busy);
    return draco_decode_repetition(c->plan, messages_dev, ld_m, sum_dev, mask_host, stream);
}

int draco_decode_cyclic_oneshot(const float* messages_dev, int64_t ld_m, int P, int s, int64_t d, float* sum_dev,
                                uint64_t* mask_host, void* stream) {
    CachedPlan* c = nullptr;
    const int rc = cached_plan(DRACO_CODE_CYCLIC, P, s, d, &c);
    if (rc != DRACO_OK) return rc;
    std::lock_guard<std::mutex> lock(c->busy);
    return draco_decode_cyclic(c->plan, messages_dev, ld_m, nullptr, sum_dev, mask_host, stream);
}

void draco_cache_clear(void) {
    std::lock_guard<std::mutex> lock(g_cache_mutex);
    if (g_cache == nullptr) return;
    for (auto& kv : *g_cache) {
        draco_plan_destroy(kv.second->plan);
        delete kv.second;
    }
    g_cache->clear();
}

}  // extern "C"
