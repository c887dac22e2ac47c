/* Plain C99 client of the library's host-only entry points: proves that
 * include/draco.h is a C header and that the ABI can be used without C++ or
 * Python.  Prints "ok" and exits 0 when every check holds. */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "draco.h"

#define CHECK(cond)                                                   \
    do {                                                              \
        if (!(cond)) {                                                \
            fprintf(stderr, "check failed: %s (line %d)\n", #cond, __LINE__); \
            return 1;                                                 \
        }                                                             \
    } while (0)

int main(void) {
    draco_plan* plan = NULL;
    const int P = 7, s = 2;
    CHECK(draco_plan_create(&plan, DRACO_CODE_CYCLIC, P, s, 10) == DRACO_OK);
    CHECK(draco_message_len(plan) == 10);
    CHECK(draco_plan_set_wire(plan, DRACO_WIRE_UNPACKED) == DRACO_OK);
    CHECK(draco_message_len(plan) == 20);
    CHECK(draco_plan_set_wire(plan, DRACO_WIRE_PACKED) == DRACO_OK);

    uint8_t A[49];
    CHECK(draco_plan_assign(plan, A) == DRACO_OK);
    for (int j = 0; j < P; ++j) {
        int row = 0;
        for (int k = 0; k < P; ++k) row += A[j * P + k];
        CHECK(row == 2 * s + 1);                 /* every node holds 2s+1 gradients */
        CHECK(A[j * P + j] == 1 && A[j * P + (j + 2 * s) % P] == 1);
    }

    double W[2 * 49];
    CHECK(draco_plan_weights(plan, W) == DRACO_OK);
    for (int k = 0; k < P; ++k)
        for (int j = 0; j < P; ++j) {
            const double mag = hypot(W[(k * P + j) * 2], W[(k * P + j) * 2 + 1]);
            CHECK((A[j * P + k] != 0) == (mag > 1e-12));   /* W vanishes exactly where A does (Lemma 1) */
        }

    /* clean projections have zero syndromes: the locator flags nobody, and b sums the
     * columns of W to the all-ones vector */
    double gamma[14], t[14], b[14];
    uint64_t mask[4] = {0, 0, 0, 0};
    for (int j = 0; j < P; ++j) {                /* gamma = (row vector of ones) * W: node j's message for g = 1 */
        gamma[2 * j] = gamma[2 * j + 1] = 0.0;
        for (int k = 0; k < P; ++k) {
            gamma[2 * j] += W[(k * P + j) * 2];
            gamma[2 * j + 1] += W[(k * P + j) * 2 + 1];
        }
    }
    CHECK(draco_cyclic_locate(plan, gamma, mask, t) == DRACO_OK);
    CHECK(mask[0] == 0);
    gamma[2 * 3] += 5.0;                         /* node 3 lies */
    CHECK(draco_cyclic_locate(plan, gamma, mask, t) == DRACO_OK);
    CHECK(mask[0] == (1ull << 3));
    CHECK(fabs(t[2 * 3] - 5.0) < 1e-9 && fabs(t[2 * 3 + 1]) < 1e-9);
    CHECK(draco_cyclic_recombination_vector(plan, mask, b) == DRACO_OK);
    CHECK(b[2 * 3] == 0.0 && b[2 * 3 + 1] == 0.0);
    for (int k = 0; k < P; ++k) {
        double re = 0.0, im = 0.0;
        for (int j = 0; j < P; ++j) {
            const double wr = W[(k * P + j) * 2], wi = W[(k * P + j) * 2 + 1];
            re += wr * b[2 * j] - wi * b[2 * j + 1];
            im += wr * b[2 * j + 1] + wi * b[2 * j];
        }
        CHECK(fabs(re - 1.0) < 1e-10 && fabs(im) < 1e-10);   /* W_{.,U} b = 1_P */
    }

    float f[5];
    CHECK(draco_projection_vector(plan, 0, f) == DRACO_OK);
    CHECK(f[0] == f[0] && f[0] != f[1]);
    CHECK(strcmp(draco_strerror(DRACO_OK), "ok") == 0);
    draco_plan_destroy(plan);

    plan = NULL;
    CHECK(draco_plan_create(&plan, DRACO_CODE_REPETITION, 10, 1, 8) == DRACO_EINVAL && plan == NULL);
    CHECK(draco_plan_create(&plan, DRACO_CODE_REPETITION, 9, 1, 8) == DRACO_OK);
    CHECK(draco_message_len(plan) == 8);
    CHECK(draco_plan_set_wire(plan, DRACO_WIRE_UNPACKED) == DRACO_EINVAL);
    draco_plan_destroy(plan);
    puts("ok");
    return 0;
}
