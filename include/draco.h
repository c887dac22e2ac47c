/*
 * draco.h -- C ABI of the MI355X (gfx950) implementation of DRACO's
 * data-parallel hot path (arXiv 1803.09877): the node-side encoder and the
 * parameter-server decoder, for the repetition code and the cyclic code.
 *
 * The P compute nodes of the paper are simulated on ONE GPU: a "slab" is a
 * row-major fp32 matrix in device memory with one row per node (messages) or
 * per unit gradient (inputs; B = P as in Sec. 3), coordinates contiguous.
 *
 * Conventions for every entry point
 *   - Pointers named *_dev are DEVICE pointers owned by the caller; pointers
 *     named *_host are HOST pointers owned by the caller.  The library keeps
 *     none of them after the call returns.
 *   - `ld*` is a row stride in floats.  Every slab base pointer must be
 *     16-byte aligned and every stride a multiple of 4 floats and at least
 *     the row length; otherwise DRACO_EALIGN is returned.  For full speed
 *     make strides multiples of 32 floats (rows 128-byte aligned): rows that
 *     are only 16-byte aligned cost up to 11 % of the bandwidth.
 *   - `stream` is a hipStream_t (NULL = the null stream).  Kernels are
 *     enqueued on it.  Entry points that return data to the host
 *     (draco_decode_repetition, draco_decode_cyclic) wait for `stream`
 *     before returning; the *_async forms and draco_encode* do not wait.
 *   - Return value 0 (DRACO_OK) on success.  Negative values are caller or
 *     runtime errors and leave the outputs untouched or unspecified.
 *     Positive values mean the decoder ran but the input violated the
 *     method's contract (more than s adversaries): the sum is then not to be
 *     trusted and the mask is a best effort.
 *   - No exceptions cross the boundary.  Calls on distinct plans may run
 *     concurrently; calls on ONE plan must not overlap (a plan owns scratch
 *     memory that its decode calls reuse).
 *   - The device that is current when a plan first touches the GPU
 *     (draco_plan_prepare or the first encode/decode) owns the plan; calling
 *     it with another device current returns DRACO_EINVAL.
 */
#ifndef DRACO_H
#define DRACO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct draco_plan draco_plan;

enum draco_code {
    DRACO_CODE_REPETITION = 0, /* Sec. 3, "Fractional Repetition Code" */
    DRACO_CODE_CYCLIC = 1      /* Sec. 3, "Cyclic Code" */
};

enum draco_wire {
    DRACO_WIRE_PACKED = 0,   /* ceil(d/2) complex entries per message (remark closing Sec. 3); default */
    DRACO_WIRE_UNPACKED = 1  /* d complex entries per message: Z = G W on the real gradients, as Sec. 3 defines E^Cyc */
};

enum draco_status {
    DRACO_OK = 0,
    DRACO_NO_MAJORITY = 1,   /* repetition: a group has more than s nodes that differ from its vote */
    DRACO_LOCATE_FAILED = 2, /* cyclic: no set of at most s nodes accounts for the syndromes */
    DRACO_EINVAL = -1,       /* null pointer, P < 1, s < 0, 2s+1 > P, (2s+1) does not divide P (repetition), d < 1, P > DRACO_MAX_NODES, d > DRACO_MAX_DIM, wrong code for the call */
    DRACO_EALIGN = -2,       /* pointer or stride alignment (see above) */
    DRACO_EHIP = -3,         /* a HIP runtime call failed (no device, out of memory, launch failure) */
    DRACO_ENOMEM = -4        /* host allocation failed */
};

#define DRACO_MAX_NODES 256
/* Largest gradient dimension accepted.  The kernels index rows with 64-bit
 * offsets (tested beyond 2^31); the limit keeps every launch below 2^32 lanes. */
#define DRACO_MAX_DIM 4294963200LL

/* ---- plan ------------------------------------------------------------- */

/* Build the code for P nodes tolerating s adversaries on d-dimensional
 * gradients: the allocation matrix A (A^Rep: P/r all-ones r x r diagonal
 * blocks, r = 2s+1; A^Cyc: node j holds gradients j..j+2s mod P) and, for the
 * cyclic code, the encoding matrix W = [Q 1] C_L of Sec. 3 (computed in
 * closed form on the host in extended precision).  Conditions checked:
 * Theorem 1's corollary 2s+1 <= P, and (2s+1) | P for the repetition code.
 * Host-only: works without a GPU.  *out is set only on success. */
int draco_plan_create(draco_plan** out, int code, int P, int s, int64_t d);

/* Cyclic code: choose what a message carries, before the plan is prepared
 * (DRACO_EINVAL afterwards, for the repetition code, or for an unknown value).
 * DRACO_WIRE_PACKED (default): pairs of real coordinates ride in one complex
 * number, 2*ceil(d/2) floats per message.
 * DRACO_WIRE_UNPACKED: the encoder multiplies the real gradients by W directly,
 * a message is d complex numbers (2d floats, re/im interleaved) -- the form in
 * which Sec. 3 states the code and proves Theorem 5, at twice the bytes.  The
 * decoder is the same (projection on f with one entry per complex coordinate,
 * i.e. d entries; locate; recombine) and writes the real part of R_{.,U} b to
 * sum_dev[d].  In this mode draco_encode, every draco_decode_cyclic* form and
 * draco_encode_node work as documented below with draco_message_len() = 2d;
 * the wide wire and draco_encode_samples with B > P return DRACO_EINVAL. */
int draco_plan_set_wire(draco_plan* plan, int wire);

/* Cyclic code, two-word wire (draco_encode_wide and the other *_wide entry
 * points): the format in which the second word of a message travels.  Sec. 3
 * defines the code over the complex numbers and leaves the number format of a
 * message open; this picks it.
 * DRACO_SECOND_WORD_F32 (default): lo = fp32(z - hi); hi + lo carries 48 bits
 * of the fp64 message z, at 8 bytes per value.
 * DRACO_SECOND_WORD_BF16: lo = bfloat16(z - hi), rounded to nearest even;
 * hi + lo carries 32 bits of z at 6 bytes per value -- the decoded sum stays
 * within about 1e-6 of the true one at P = 45 (one fp32 word: 3e-4), and
 * every pass over the messages moves a quarter fewer bytes.  messages_lo_dev
 * then points at [P][ld_m] 16-bit values: SAME ld_m and column index as the
 * first word, counted in elements, so its rows are half as long in bytes.
 * DRACO_SECOND_WORD_I8: lo is an 8-bit signed code q of the residual in units
 * of the spacing u of fp32 numbers at hi: with E the exponent field of hi,
 * u = 2^(max(E, 24) - 150), q = (z - hi) / u * 254 rounded to nearest even,
 * -127 <= q <= 127 (unspecified next to a hi that is not finite); it stands
 * for q * u / 254, and the decoder accepts any byte.
 * hi + lo is within u / 508 <= 2^-32 |z| of z at 5 bytes per value: the
 * decoded sum stays within about 1e-6 of the true one at (P, s) = (45, 3)
 * and 5e-6 at (45, 5).  messages_lo_dev then points at [P][ld_m] bytes,
 * same ld_m and column index, rows a quarter as long in bytes.
 * May be changed at any time; encoder and decoder must agree.  DRACO_EINVAL
 * for the repetition code, the unpacked wire, or an unknown value. */
enum {
    DRACO_SECOND_WORD_F32 = 0,
    DRACO_SECOND_WORD_BF16 = 1,
    DRACO_SECOND_WORD_I8 = 2
};
int draco_plan_set_second_word(draco_plan* plan, int format);

/* Allocate the plan's device-side tables and scratch on the current device
 * (a few MB: per-node coefficients, per-wave partial projections, flag
 * words).  Called implicitly by the first encode/decode if omitted; after it
 * no entry point allocates device memory. */
int draco_plan_prepare(draco_plan* plan);

/* Free the plan and everything it owns (waits for the device if prepared). */
void draco_plan_destroy(draco_plan* plan);

/* Floats per message row: d for the repetition code; 2*ceil(d/2) for the
 * cyclic code (ceil(d/2) complex numbers, real and imaginary part interleaved;
 * complex coordinate i packs real coordinates 2i and 2i+1 -- the packing at
 * the end of Sec. 3 with adjacent instead of half-apart pairs), or 2*d on
 * the unpacked wire (draco_plan_set_wire).  < 0 on a null plan. */
int64_t draco_message_len(const draco_plan* plan);

/* A_host[j*P + k] = 1 if node j is assigned gradient k, else 0 (P*P bytes). */
int draco_plan_assign(const draco_plan* plan, uint8_t* A_host);

/* W_host[(k*P + j)*2 + {0,1}] = real, imaginary part of W[k][j]: the weight of
 * gradient k in node j's message (Z = G W).  Repetition code: A^T as 0/1. */
int draco_plan_weights(const draco_plan* plan, double* W_host);

/* ---- encoder (node side) ---------------------------------------------- */

/* All P nodes at once: messages[j] = E_j(Y_j).
 * Repetition (E^Rep): z_j = sum of the r gradients of node j's group, added in
 * ascending k in fp32; computed once per group and stored r times, so the r
 * copies are bit-identical.
 * Cyclic (E^Cyc): z_j = sum_{k in S_j} W[k][j] * g^_k on packed complex
 * gradients, accumulated in fp64 and rounded once to fp32.
 *   grads_dev     [P][ld_g]  fp32, row k = gradient k, first d floats used
 *                  (cyclic with odd d: coordinate d is taken as 0, it need not
 *                  be stored as 0)
 *   messages_dev  [P][ld_m]  fp32, first draco_message_len() floats written
 * Asynchronous on `stream`. */
int draco_encode(draco_plan* plan, const float* grads_dev, int64_t ld_g,
                 float* messages_dev, int64_t ld_m, void* stream);

/* B > P (Sec. 1: "each compute node processes rB/P gradients"; the experiments
 * use B = 180 or 720 on P = 45): samples_dev is [B][ld_g] with B a multiple of
 * P, and unit gradient k of Sec. 3 is the sum of rows k*(B/P) .. (k+1)*(B/P)-1.
 * The sums are formed inside the encoder pass (fp32, ascending, for the
 * repetition code; fp64 for the cyclic code), so every per-sample row is read
 * from HBM once and no [P][d] intermediate is written.  B = P is draco_encode. */
int draco_encode_samples(draco_plan* plan, const float* samples_dev, int64_t B, int64_t ld_g,
                         float* messages_dev, int64_t ld_m, void* stream);

/* Cyclic code with the WIDE wire: every message is sent as two fp32 words per
 * float, messages_hi = fp32(z) and messages_lo = fp32(z - hi) with z the fp64
 * value, so that hi + lo carries 48 bits of z.  The entries of W grow like
 * 1e4-1e5 at P = 45 and the decoder cancels them back to O(1); rounding z to
 * one fp32 word then leaves a relative error near 3e-4 in the decoded sum,
 * the wide wire leaves about 1e-9, at twice the message bytes.  Same layout
 * and conditions as draco_encode for each of the two slabs (one ld_m).
 * draco_plan_set_second_word selects a 16-bit second word instead; the
 * pointer is untyped for that reason.  DRACO_EINVAL for the repetition code. */
int draco_encode_wide(draco_plan* plan, const float* grads_dev, int64_t ld_g,
                      float* messages_hi_dev, void* messages_lo_dev, int64_t ld_m, void* stream);

/* draco_encode_samples on the wide wire (B a multiple of P; B = P is
 * draco_encode_wide).  DRACO_EINVAL for the repetition code or the unpacked wire. */
int draco_encode_samples_wide(draco_plan* plan, const float* samples_dev, int64_t B, int64_t ld_g,
                              float* messages_hi_dev, void* messages_lo_dev, int64_t ld_m,
                              void* stream);

/* One node, as a real compute node would run it: node_grads_dev holds ONLY
 * that node's r = 2s+1 assigned gradients, [r][ld_g], in assignment order
 * (repetition: ascending k within the group; cyclic: k = node, node+1, ...,
 * node+2s mod P).  Writes one message row.  Same arithmetic and order as
 * draco_encode, so the result is bit-identical to row `node` of it. */
int draco_encode_node(draco_plan* plan, int node, const float* node_grads_dev,
                      int64_t ld_g, float* message_dev, void* stream);

/* The same on the two-word wire: one row of each word (message_lo_dev in the
 * format draco_plan_set_second_word selected, 16-byte aligned), bit-identical
 * to row `node` of what draco_encode_wide writes.  DRACO_EINVAL for the
 * repetition code or the unpacked wire. */
int draco_encode_node_wide(draco_plan* plan, int node, const float* node_grads_dev,
                           int64_t ld_g, float* message_hi_dev, void* message_lo_dev,
                           void* stream);

/* ---- decoder (parameter server) --------------------------------------- */

/* D^Rep: per group of r consecutive nodes, majority vote (Algorithm 2, the
 * streaming vote, applied per coordinate on bit patterns, then a count), sum
 * of the P/r winners in ascending group order in fp32.
 *   messages_dev [P][ld_m] fp32 as received (R = Z + N)
 *   sum_dev      [d]       fp32 out: u = G 1_P
 *   mask_host    [ceil(P/64)] out: bit (j%64) of word j/64 set iff node j's
 *                message differs from its group's vote in any coordinate
 * Returns DRACO_NO_MAJORITY if some group has more than s such nodes.
 * Waits for `stream`. */
int draco_decode_repetition(draco_plan* plan, const float* messages_dev, int64_t ld_m,
                            float* sum_dev, uint64_t* mask_host, void* stream);

/* Same, stream-ordered: mask_dev [ceil(P/64)] and status_dev [1] (a
 * draco_status value) are DEVICE outputs valid once `stream` reaches the end
 * of the call.  Does not wait. */
int draco_decode_repetition_async(draco_plan* plan, const float* messages_dev, int64_t ld_m,
                                  float* sum_dev, uint64_t* mask_dev, int32_t* status_dev,
                                  void* stream);

/* For callers that cannot allocate device memory -- code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc: draco_decode_repetition_async without a
 * plan and without any allocation, by the library or the HIP runtime on its behalf.  The
 * node-flag words the vote needs (DRACO_MAX_NODES bits = 32 bytes) live in a device array
 * inside the library's code object: every GPU the library runs on holds one copy until the
 * process ends, and EVERY call on a GPU uses that GPU's copy, so two calls that overlap on
 * one GPU (different streams, or graphs replayed concurrently) race on it and must be
 * ordered by the caller.  The array is cleared by a small kernel at the start of each
 * call.  The first call on a device looks up the array's address (no stream work): make
 * that call outside stream capture.
 *   P, s, d       the code, as for draco_plan_create with DRACO_CODE_REPETITION:
 *                 1 <= P <= DRACO_MAX_NODES (the array's size: more nodes are rejected),
 *                 (2s+1) | P, 1 <= d <= DRACO_MAX_DIM; otherwise DRACO_EINVAL, nothing runs
 *   messages_dev, ld_m, sum_dev, mask_dev, status_dev, stream
 *                 as draco_decode_repetition_async; results are bit-identical to it
 * Does not wait. */
int draco_decode_repetition_static(int P, int s, int64_t d, const float* messages_dev, int64_t ld_m,
                                   float* sum_dev, uint64_t* mask_dev, int32_t* status_dev,
                                   void* stream);

/* D^Cyc (Algorithm 1): V = phi(R) (random projection f R, syndromes
 * f R C_R^dagger, the s x s system for beta, the recurrence for the remaining
 * h_l, IDFT), U = complement, b with W_{.,U} b = 1_P (minimum-norm), and
 * u = R_{.,U} b, unpacked to d reals.
 *   messages_dev [P][ld_m] fp32, complex interleaved (see draco_message_len)
 *   f_dev        [ceil(d/2)] fp32: the random vector f ~ N(1, I) of phi, one
 *                entry per complex coordinate, drawn by the caller; or NULL:
 *                the projection kernel then makes the entries on the fly from
 *                a seed that changes with every decode (see
 *                draco_plan_set_projection_seed) and no vector is read from memory
 *   sum_dev      [d] fp32 out
 *   mask_host    as above: the located set V
 * A node whose message holds NaN or Inf is flagged outright (it is one of the
 * at most s adversaries) and the sum is still recovered.  So is a node whose
 * projection is enormous (an adversary may send 1e30, and the fp64 rounding
 * of such a value would drown the syndromes of everything else): a located
 * node beyond max(1024, tau * 2^44) times the median projection, or, when phi
 * finds no set, the largest nodes beyond 1024 times the median.  phi then runs
 * again without such nodes, layer by layer, so a smaller lie cannot hide in
 * the rounding of an enormous one.
 * Returns DRACO_LOCATE_FAILED if no set of at most s nodes explains the
 * syndromes.  For s <= 16 the small linear
 * algebra of phi and b runs in one fp64 wavefront between the two streaming
 * kernels, so the whole call is stream-ordered and waits for `stream` only
 * once, at the end, to fetch mask and status; for larger s it is
 * draco_decode_cyclic_hostphi. */
int draco_decode_cyclic(draco_plan* plan, const float* messages_dev, int64_t ld_m,
                        const float* f_dev, float* sum_dev, uint64_t* mask_host,
                        void* stream);

/* The generated projection vector (f_dev == NULL).  Entry i is a counter-based
 * function of (seed, i): splitmix64's finaliser on seed + (i+1)*0x9E3779B97F4A7C15
 * gives two 24-bit uniforms u1 (top bits) and u2 (bits 16..39), and
 * f_i = fp32(1 + sqrt(-2 ln u1) cos(2 pi u2)).
 * phi needs an f the adversaries cannot know in advance (Lemma 3), so every
 * decode of a plan uses another seed: a plan starts from a base seed taken from
 * the system's entropy source when it is created; the k-th decode (k = 0, 1, ...)
 * after the base was set uses seed_0 = base and, for k > 0, seed_k = splitmix64's
 * finaliser on base + k*0x9E3779B97F4A7C15.  draco_plan_set_projection_seed sets
 * the base (and restarts k at 0), which makes a run reproducible;
 * draco_plan_last_projection_seed reports the seed the most recent such decode
 * used (DRACO_EINVAL before the first).  The seed travels as a kernel argument:
 * a captured HIP graph replays the seed it was captured with (pass f_dev,
 * refreshed by the caller, to vary f there).
 * draco_projection_vector writes the entries for a seed (draco_message_len()/2
 * of them) to host memory (inspection, tests). */
int draco_plan_set_projection_seed(draco_plan* plan, uint64_t seed);
int draco_plan_last_projection_seed(const draco_plan* plan, uint64_t* seed);
int draco_projection_vector(const draco_plan* plan, uint64_t seed, float* f_host);

/* Speculative single-pass decode (cyclic code, s <= 16; on by default).  While
 * the projection pass of draco_decode_cyclic* has a row in registers it can also
 * accumulate the recombination for "no adversary" and write it to sum_dev; if
 * phi then flags nobody -- the usual case in training -- that is the decoded sum
 * (bit-identical to what the second pass would give) and the second pass over
 * the messages is skipped, which halves the decode.  A plan speculates in a
 * call when its previous decode was clean (the first call does), so a run with
 * persistent adversaries pays for one wasted speculation only.  0 switches it off. */
int draco_plan_set_speculation(draco_plan* plan, int enabled);

/* Same, stream-ordered (s <= 16 only, else DRACO_EINVAL): mask_dev
 * [ceil(P/64)] and status_dev [1] are DEVICE outputs valid once `stream`
 * reaches the end of the call.  Does not wait, allocates nothing. */
int draco_decode_cyclic_async(draco_plan* plan, const float* messages_dev, int64_t ld_m,
                              const float* f_dev, float* sum_dev, uint64_t* mask_dev,
                              int32_t* status_dev, void* stream);

/* Same result with phi and b computed on the HOST in extended precision
 * between the projection and the recombination kernel: waits for `stream`
 * twice (after the projection and at the end).  Any s. */
int draco_decode_cyclic_hostphi(draco_plan* plan, const float* messages_dev, int64_t ld_m,
                                const float* f_dev, float* sum_dev, uint64_t* mask_host,
                                void* stream);

/* D^Cyc on the wide wire of draco_encode_wide: the received message of node j
 * is messages_hi[j] + messages_lo[j] (added exactly in fp64).  Otherwise as
 * draco_decode_cyclic / draco_decode_cyclic_async, except that the locator
 * counts a syndrome as zero below DRACO_TAU_WIDE (instead of DRACO_TAU) times
 * the median projection: the wide wire's clean syndromes sit near 1e-14, so
 * much smaller lies can be told from rounding.  With a bfloat16 second word
 * (draco_plan_set_second_word) the threshold is DRACO_TAU_BF16, with an 8-bit
 * one DRACO_TAU_I8. */
int draco_decode_cyclic_wide(draco_plan* plan, const float* messages_hi_dev,
                             const void* messages_lo_dev, int64_t ld_m, const float* f_dev,
                             float* sum_dev, uint64_t* mask_host, void* stream);
int draco_decode_cyclic_wide_async(draco_plan* plan, const float* messages_hi_dev,
                                   const void* messages_lo_dev, int64_t ld_m, const float* f_dev,
                                   float* sum_dev, uint64_t* mask_dev, int32_t* status_dev,
                                   void* stream);

/* ---- host-side pieces of D^Cyc, exposed for inspection and testing ----- */

/* phi, steps 2-4, on the P projections gamma'_j = f . r_j given as
 * gamma_host[2j], gamma_host[2j+1] (re, im).  Writes the mask words and, if
 * t_host != NULL, the vector t (2P doubles).  Returns DRACO_OK or
 * DRACO_LOCATE_FAILED.  Host-only. */
int draco_cyclic_locate(const draco_plan* plan, const double* gamma_host,
                        uint64_t* mask_host, double* t_host);
/* Same with the relative zero threshold of the syndromes given (0 < tau < 1):
 * DRACO_TAU is what the one-word decoders use, DRACO_TAU_WIDE the wide ones,
 * DRACO_TAU_BF16 / DRACO_TAU_I8 the wide ones with a bfloat16 / 8-bit second word. */
#define DRACO_TAU (32.0 / 16777216.0)        /* 32 ulps of an fp32 wire */
#define DRACO_TAU_WIDE (1.0 / 68719476736.0) /* 2^-36 */
#define DRACO_TAU_BF16 (32.0 / 8589934592.0) /* 32 ulps of the 32-bit fp32 + bfloat16 wire */
#define DRACO_TAU_I8 (32.0 / 4294967296.0)   /* 32 ulps of the fp32 + 8-bit wire */
int draco_cyclic_locate_tol(const draco_plan* plan, const double* gamma_host, double tau,
                            uint64_t* mask_host, double* t_host);

/* The minimum-norm b with C_L[:, U] b_U = e_last (proof of Lemma 1) for
 * U = nodes whose mask bit is clear; b_host[2j], b_host[2j+1] = re, im of b_j,
 * zero on masked nodes.  Needs at most 2s masked nodes.  Host-only. */
int draco_cyclic_recombination_vector(const draco_plan* plan, const uint64_t* mask_host,
                                      double* b_host);

/* ---- the three calls without a plan ------------------------------------ */

/* encode(assign, grads_per_sample) -> messages.  assign_host is the P x P 0/1
 * allocation matrix A (row j = node j, as draco_plan_assign writes it); it must
 * be A^Rep or A^Cyc of Sec. 3 for `code` (every row holds r = 2s+1 ones, which
 * fixes s), otherwise DRACO_EINVAL.  samples_dev is [B][ld_g] with B a multiple
 * of P (B = P: one unit gradient per row), as for draco_encode_samples; the
 * cyclic code uses the packed wire with ONE fp32 word per message float (these
 * calls take a single message slab): rounding the messages to fp32 leaves the
 * decoded sum about 5e-7 from the true one at P = 15 but 3e-4 at P = 45 -- use
 * the plan forms with a two-word wire (draco_encode_wide) where that matters.
 * The library keeps one plan per
 * (code, P, s, d, device) behind these calls and prepares it on first use (that
 * call allocates; later ones do not).  Calls with the same parameters take
 * turns.  Asynchronous on `stream`. */
int draco_encode_oneshot(const uint8_t* assign_host, int code, int P, int64_t d,
                         const float* samples_dev, int64_t B, int64_t ld_g,
                         float* messages_dev, int64_t ld_m, void* stream);

/* decode_repetition(messages, P, s) -> (sum, adversary_mask) and
 * decode_cyclic(messages, P, s) -> (sum, adversary_mask): draco_decode_repetition
 * / draco_decode_cyclic on the cached plan for (P, s, d).  The cyclic form draws
 * f inside the library (f_dev = NULL: a fresh seed per call).  Return values,
 * outputs and waiting as for the plan forms. */
int draco_decode_repetition_oneshot(const float* messages_dev, int64_t ld_m, int P, int s,
                                    int64_t d, float* sum_dev, uint64_t* mask_host, void* stream);
int draco_decode_cyclic_oneshot(const float* messages_dev, int64_t ld_m, int P, int s,
                                int64_t d, float* sum_dev, uint64_t* mask_host, void* stream);

/* Destroy every cached plan (waits for the device).  Not to be called while a
 * plan-free call is running. */
void draco_cache_clear(void);

/* ---- parameter server: the model update -------------------------------- */

/* Mini-batch SGD's update with the decoded sum (Sec. 2, "Distributed Training":
 * w_k = w_{k-1} - (gamma/|S_k|) * sum of the batch's gradients):
 * params[i] <- params[i] - scale * sum[i] for i < d, in fp32 with one fused
 * multiply-add per parameter (scale = learning rate / B).  One read of the sum,
 * one read-modify-write of the parameters.  Both pointers 16-byte aligned.
 * Asynchronous on `stream`. */
int draco_apply_update(float* params_dev, const float* sum_dev, int64_t d, float scale,
                       void* stream);

/* ---- misc -------------------------------------------------------------- */

/* Static, NUL-terminated description of a status value. */
const char* draco_strerror(int status);

/* Text describing the last HIP runtime failure behind a DRACO_EHIP return on the
 * calling thread (the failing call and HIP's error string); "" if none. */
const char* draco_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* DRACO_H */
