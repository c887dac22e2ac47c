/* Plain C99 client of the three plan-free calls -- encode(assign, grads) -> messages,
 * decode_repetition(messages, P, s) -> (sum, mask), decode_cyclic(messages, P, s) ->
 * (sum, mask) -- on a GPU, with device memory from the HIP runtime's C API.  One node
 * lies; the decoded sum must be the plain sum of the gradients (Definition 2) and the
 * mask must name the liar.  Prints "ok" and exits 0 when every check holds. */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>

#include "draco.h"

#define CHECK(cond)                                                           \
    do {                                                                      \
        if (!(cond)) {                                                        \
            fprintf(stderr, "check failed: %s (line %d)\n", #cond, __LINE__); \
            return 1;                                                         \
        }                                                                     \
    } while (0)

enum { P = 9, S = 1, D = 1001, LD = 1004, LIAR = 5 };

static int run(int code) {
    const int r = 2 * S + 1;
    const int64_t mlen = code == DRACO_CODE_REPETITION ? D : 2 * ((D + 1) / 2);
    const int64_t ldm = (mlen + 3) / 4 * 4;
    uint8_t A[P * P];
    memset(A, 0, sizeof(A));
    for (int j = 0; j < P; ++j)
        for (int t = 0; t < r; ++t) A[j * P + (code == DRACO_CODE_REPETITION ? (j / r) * r + t : (j + t) % P)] = 1;

    float* G = (float*)calloc((size_t)P * LD, sizeof(float));
    double* want = (double*)calloc(D, sizeof(double));
    float* Z = (float*)calloc((size_t)P * ldm, sizeof(float));
    float* u = (float*)calloc(LD, sizeof(float));
    CHECK(G && want && Z && u);
    unsigned x = 12345u + (unsigned)code;
    for (int k = 0; k < P; ++k)
        for (int i = 0; i < D; ++i) {
            x = x * 1664525u + 1013904223u;
            G[k * LD + i] = (float)((int)(x >> 8) % 2001 - 1000) / 512.0f;
            want[i] += (double)G[k * LD + i];
        }

    float *Gd = NULL, *Zd = NULL, *ud = NULL;
    CHECK(hipMalloc((void**)&Gd, (size_t)P * LD * sizeof(float)) == hipSuccess);
    CHECK(hipMalloc((void**)&Zd, (size_t)P * ldm * sizeof(float)) == hipSuccess);
    CHECK(hipMalloc((void**)&ud, LD * sizeof(float)) == hipSuccess);
    CHECK(hipMemcpy(Gd, G, (size_t)P * LD * sizeof(float), hipMemcpyHostToDevice) == hipSuccess);

    CHECK(draco_encode_oneshot(A, code, P, D, Gd, P, LD, Zd, ldm, NULL) == DRACO_OK);
    CHECK(hipDeviceSynchronize() == hipSuccess);
    CHECK(hipMemcpy(Z, Zd, (size_t)P * ldm * sizeof(float), hipMemcpyDeviceToHost) == hipSuccess);
    for (int64_t i = 0; i < mlen; ++i) Z[LIAR * ldm + i] *= -100.0f;     /* the reversed-gradient attack */
    CHECK(hipMemcpy(Zd, Z, (size_t)P * ldm * sizeof(float), hipMemcpyHostToDevice) == hipSuccess);

    uint64_t mask[4] = {0, 0, 0, 0};
    int st;
    if (code == DRACO_CODE_REPETITION) st = draco_decode_repetition_oneshot(Zd, ldm, P, S, D, ud, mask, NULL);
    else st = draco_decode_cyclic_oneshot(Zd, ldm, P, S, D, ud, mask, NULL);
    CHECK(st == DRACO_OK);
    CHECK(mask[0] == (1ull << LIAR));
    CHECK(hipMemcpy(u, ud, LD * sizeof(float), hipMemcpyDeviceToHost) == hipSuccess);
    double num = 0.0, den = 0.0;
    for (int i = 0; i < D; ++i) {
        num += ((double)u[i] - want[i]) * ((double)u[i] - want[i]);
        den += want[i] * want[i];
    }
    CHECK(sqrt(num / den) <= (code == DRACO_CODE_REPETITION ? 1e-5 : 1e-4));

    A[0] = 0;                                                            /* no longer the code's matrix */
    CHECK(draco_encode_oneshot(A, code, P, D, Gd, P, LD, Zd, ldm, NULL) == DRACO_EINVAL);
    CHECK(hipFree(Gd) == hipSuccess && hipFree(Zd) == hipSuccess && hipFree(ud) == hipSuccess);
    free(G); free(want); free(Z); free(u);
    return 0;
}

int main(void) {
    if (run(DRACO_CODE_REPETITION) != 0) return 1;
    if (run(DRACO_CODE_CYCLIC) != 0) return 1;
    draco_cache_clear();
    puts("ok");
    return 0;
}
