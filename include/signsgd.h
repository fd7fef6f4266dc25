/*
 * signsgd.h - C ABI of the MI355X (gfx950) library for the per-step hot path
 * of signSGD / Signum with majority vote (arxiv 1802.04434, Algorithms 1-3).
 *
 * One step over a d-coordinate model held by M data-parallel workers:
 *
 *   m_w <- beta m_w + (1-beta) g_w          Algorithm 2 (Signum), per worker
 *   s_w  = sign(m_w)   (sign(g_w) without momentum: Algorithm 1)
 *   one bit per coordinate per worker       Table 1: 1 bit up, 1 bit down
 *   v    = sign( sum_w s_w )                Algorithm 3, server ("(best)", Section 4)
 *   x   <- x - delta v                      Algorithm 3, worker
 *
 * On one GPU the M workers are M device buffers.
 *
 * CONVENTIONS (the paper leaves these open; they are part of this ABI)
 *   sign(v)    -1 if v < 0, otherwise +1.  +0.0 and -0.0 are "+".  The same
 *              rule is applied to the integer vote sum: an even-M tie is "+".
 *   bits       bit = 1 means sign = -1.  Coordinate i is bit (i mod 32),
 *              least significant first, of the uint32 word (i div 32).  A
 *              packed buffer holds ss_packed_bytes(d) bytes: ceil(d/32) words
 *              rounded up to a multiple of 16 bytes.  Every routine that
 *              writes a packed buffer writes ALL of those bytes; bits at and
 *              beyond coordinate d are written as 0.
 *   arithmetic fp32, round to nearest even, subnormals kept, no fused
 *              multiply-add:  m <- fl( fl(beta*m) + fl(omb*g) ) with
 *              omb = fl(1 - beta) computed once;  x <- fl(x - delta) or
 *              fl(x + delta).  bf16 gradients are widened to fp32 exactly.
 *              NaN / Inf inputs follow these rules literally (a NaN is not
 *              < 0, hence "+"); they are not an error.
 *   momentum   with M > 1 every worker owns its momentum buffer and votes
 *              with sign(m_w).
 *
 * MEMORY      Every data pointer (g, m, x, packed, voted) is DEVICE memory,
 *             owned by the caller and 16-byte aligned.  A buffer that a call
 *             writes (m, x, packed, voted, sums, ...) may not share a byte with
 *             any other buffer of that call: SS_ERR_ARG, nothing launched.
 *             Buffers that are only read may coincide.  Arrays OF pointers
 *             (g[], m[], packed[]) are HOST arrays of M device pointers; they
 *             are copied into the kernel arguments during the call and may be
 *             freed on return.  The library allocates nothing and keeps no
 *             state between calls (one exception, stated there: the fixed
 *             scratch array of ss_density_static).
 * STREAMS     hip_stream is a hipStream_t passed as void* (NULL: the default
 *             stream).  Work is enqueued and the call returns without
 *             synchronising.  Calls are thread safe.
 * ERRORS      Every call returns SS_OK or a negative ss_status and never
 *             aborts.  Arguments are validated before anything is enqueued:
 *             on an argument error nothing has been launched.  d == 0 is
 *             SS_OK and launches nothing.
 */
#ifndef SIGNSGD_H
#define SIGNSGD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SS_OK = 0,
    SS_ERR_NULL = -1,  /* a required pointer (or an entry of a pointer array) is NULL */
    SS_ERR_BAD_M = -2, /* M < 1 or M > SS_MAX_WORKERS */
    SS_ERR_ALIGN = -3, /* a data pointer is not 16-byte aligned */
    SS_ERR_DTYPE = -4, /* unknown gradient dtype */
    SS_ERR_ARG = -5,   /* any other invalid argument (d too large, overlapping buffers, ...) */
    SS_ERR_HIP = -6,   /* the HIP runtime refused a launch; see ss_last_hip_error */
    SS_ERR_RANGE = -7  /* the arguments are valid but the answer lies beyond a documented limit */
} ss_status;

/* gradient element type; momentum and parameters are always fp32 */
typedef enum { SS_F32 = 0, SS_BF16 = 1 } ss_dtype;

#define SS_MAX_WORKERS 64

/* ceil(d/32): words that carry payload bits */
size_t ss_packed_words(size_t d);
/* bytes a packed / voted buffer for d coordinates must hold (multiple of 16) */
size_t ss_packed_bytes(size_t d);

/*
 * One worker's half of a step.  Algorithm 2: m <- beta m + (1-beta) g, then
 * packed <- bits of sign(m).  With m == NULL, Algorithm 1: packed <- bits of
 * sign(g), beta ignored.
 *   g       in   d elements of type gdt
 *   m       i/o  d x fp32, or NULL
 *   packed  out  ss_packed_bytes(d) bytes
 */
int ss_signum_pack(const void *g, ss_dtype gdt, float *m, float beta,
                   uint32_t *packed, size_t d, void *hip_stream);

/*
 * Algorithm 3, server side: voted <- bits of sign( sum_w sign_w ), where
 * packed[w] holds worker w's sign bits.  "-" wins at a coordinate iff more
 * than M/2 workers are "-".
 *   packed  in   host array of M device pointers, ss_packed_bytes(d) bytes each
 *   voted   out  ss_packed_bytes(d) bytes
 */
int ss_majority_vote(const uint32_t *const *packed, int M, uint32_t *voted,
                     size_t d, void *hip_stream);

/*
 * Algorithm 1 / Algorithm 3, worker side: x_i <- x_i - delta * s_i with
 * s_i = -1 where bit i of `bits` is set, +1 otherwise.  `bits` is a voted
 * buffer, or a single worker's packed buffer.
 *   x     i/o  d x fp32
 *   bits  in   ss_packed_bytes(d) bytes (only the first ceil(d/32) words are read)
 */
int ss_sign_apply(float *x, const uint32_t *bits, float delta, size_t d,
                  void *hip_stream);

/*
 * The whole step in one pass over memory: for every worker the momentum
 * update and sign (Algorithm 2), the vote and the parameter update
 * (Algorithm 3).  Identical results, bit for bit, to M calls of
 * ss_signum_pack, one ss_majority_vote and one ss_sign_apply.
 *   g           in   host array of M device pointers, d elements of gdt each
 *   m           i/o  host array of M device pointers, d x fp32 each; NULL = no
 *                    momentum (Algorithm 1 + 3: vote on sign(g_w), beta ignored)
 *   x           i/o  d x fp32
 *   voted       out  ss_packed_bytes(d) bytes: the bits that were applied
 *   packed_out  out  NULL, or host array of M device pointers that receive
 *                    every worker's sign bits (ss_packed_bytes(d) bytes each)
 * Normally one kernel launch.  When packed_out is given, d >= 2^24 and there
 * are two workers or more, the call enqueues M + 2 launches that hand the signs
 * over through packed_out, which is as fast or faster there; the results are
 * the same.  Should the runtime refuse one of those launches
 * (SS_ERR_HIP), the launches before it stay enqueued: some momentum buffers
 * have then been advanced by this step and x has not.
 */
int ss_signum_vote_step(const void *const *g, ss_dtype gdt, float *const *m,
                        int M, float beta, float delta, float *x,
                        uint32_t *voted, uint32_t *const *packed_out, size_t d,
                        void *hip_stream);

/* ---- variants of the step that the paper describes besides Algorithms 1-3 ---- */

typedef enum {
    SS_STEP_DEFAULT = 0,
    SS_STEP_WARMUP = 1,    /* Theorem 3: during the first C(beta) iterations every worker votes with
                              sign(g_w) while its momentum is still updated as in Algorithm 2 */
    SS_STEP_SUM_UPDATE = 2 /* Section 4, scheme "(good)": x <- x - delta * sum_w s_w (rounded as
                              fl(x - fl(delta * S)), S converted to fp32 exactly) instead of
                              x <- x - delta * sign(sum_w s_w) */
} ss_step_flags;

/*
 * Theorem 3's warm-up length: the smallest positive integer C with
 * (C/2) beta^C <= 1/((1 - beta^2)(C + 1)) and beta^(C+1) <= 1/2, evaluated in
 * double precision (beta^C by repeated multiplication).  Host only, launches
 * nothing.  54 for beta = 0.9.  SS_ERR_ARG unless 0 < beta < 1.  The search is
 * linear in C and stops at SS_WARMUP_MAX (about 20 ms of host time): a beta so
 * close to 1 that C would be larger (beta above roughly 1 - 2e-6) gives
 * SS_ERR_RANGE.
 */
#define SS_WARMUP_MAX 10000000L
long ss_warmup_length(float beta);

/*
 * One worker's half of a warm-up iteration (Theorem 3): m <- beta m + (1-beta) g
 * as in ss_signum_pack, but packed <- bits of sign(g).  m == NULL: same as
 * ss_signum_pack without momentum.  Arguments as for ss_signum_pack.
 */
int ss_signum_pack_warmup(const void *g, ss_dtype gdt, float *m, float beta,
                          uint32_t *packed, size_t d, void *hip_stream);

/*
 * Section 4 "(good)", server side: sums_i <- sum_w s_w,i (each s = +-1, so
 * |sums_i| <= M and sums_i = M mod 2).
 *   packed  in   host array of M device pointers, ss_packed_bytes(d) bytes each
 *   sums    out  d x int8, 16-byte aligned
 */
int ss_vote_sum(const uint32_t *const *packed, int M, int8_t *sums, size_t d,
                void *hip_stream);

/*
 * Section 4 "(good)", worker side: x_i <- fl(x_i - fl(delta * sums_i)).
 *   x     i/o  d x fp32
 *   sums  in   d x int8, 16-byte aligned
 */
int ss_sum_apply(float *x, const int8_t *sums, float delta, size_t d,
                 void *hip_stream);

/*
 * ss_signum_vote_step with the variants selected by `flags` (an OR of
 * ss_step_flags; unknown bits: SS_ERR_ARG).  `voted` always receives the bits of
 * sign(sum_w s_w).
 *   sums_out  out  NULL, or d x int8 (16-byte aligned): sum_w s_w per coordinate
 * Everything else as for ss_signum_vote_step, which is this call with
 * flags = SS_STEP_DEFAULT and sums_out = NULL.
 */
int ss_signum_vote_step_ex(const void *const *g, ss_dtype gdt, float *const *m,
                           int M, float beta, float delta, float *x,
                           uint32_t *voted, uint32_t *const *packed_out,
                           int8_t *sums_out, size_t d, unsigned flags,
                           void *hip_stream);

/* ---- majority vote with abstention (Section 6, Discussion) ----
 *
 * The paper only sketches this extension: workers send their vote unless they
 * are very unsure about the sign, in which case they send zero; the server
 * sends zero back when no quorum is reached.  It gives neither the workers'
 * criterion nor the quorum rule, so the rule below is THIS LIBRARY'S READING
 * (parity with the paper is unpinned; parity with the CPU oracle is exact):
 *   worker   abstains at coordinate i when |v_i| < tau, v = m (g without
 *            momentum), tau >= 0; otherwise votes sign(v_i) as in Algorithm 3
 *   server   S_i = (#plus) - (#minus); answer sign(S_i) if |S_i| >= quorum,
 *            otherwise 0 (quorum >= 1)
 *   update   x_i <- x_i - delta * answer_i (x_i untouched where the answer is 0)
 * A ternary vector is two packed bit planes with the layout of CONVENTIONS:
 * `neg` (bit set: -1) and `zero` (bit set: 0); never both set in what the
 * library writes; where both are set in an input, `zero` wins.  With tau = 0,
 * quorum = 1 and odd M this is exactly Algorithm 3.
 */

/* worker: momentum update as in ss_signum_pack (m may be NULL), then the ternary
 * vote of this worker.  neg, zero: out, ss_packed_bytes(d) bytes each. */
int ss_signum_pack_ternary(const void *g, ss_dtype gdt, float *m, float beta,
                           float tau, uint32_t *neg, uint32_t *zero, size_t d,
                           void *hip_stream);

/* server: neg, zero = host arrays of M device pointers (the workers' planes);
 * voted_neg, voted_zero: out, ss_packed_bytes(d) bytes each. */
int ss_quorum_vote(const uint32_t *const *neg, const uint32_t *const *zero,
                   int M, int quorum, uint32_t *voted_neg, uint32_t *voted_zero,
                   size_t d, void *hip_stream);

/* worker: x <- x - delta * answer, the answer given by its two planes */
int ss_ternary_apply(float *x, const uint32_t *neg, const uint32_t *zero,
                     float delta, size_t d, void *hip_stream);

/* the three in one pass; arguments as for ss_signum_vote_step */
int ss_signum_vote_step_ternary(const void *const *g, ss_dtype gdt,
                                float *const *m, int M, float beta, float tau,
                                int quorum, float delta, float *x,
                                uint32_t *voted_neg, uint32_t *voted_zero,
                                size_t d, void *hip_stream);

/* ---- gradient statistics (Section 3: equation (1) and Figure 1) ---- */

/*
 * Welford's single-pass mean / variance over a sequence of stochastic
 * gradients, one call per gradient.  Per coordinate, in fp32, every operation
 * rounded once (division correctly rounded):
 *     delta = g - mean;  mean <- mean + delta / n;  m2 <- m2 + delta * (g - mean)
 *   g     in   d elements of type gdt (bf16 widened exactly): the n-th gradient
 *   mean  i/o  d x fp32, running mean (all zero before the first call)
 *   m2    i/o  d x fp32, running sum of squared deviations (all zero before the first call)
 *   n     1-based index of this gradient, at most 2^24 (so that it is exact in fp32)
 */
int ss_welford_update(const void *g, ss_dtype gdt, float *mean, float *m2,
                      uint64_t n, size_t d, void *hip_stream);

/* sigma_i <- sqrt(m2_i / n): the standard deviation over the n gradients seen
 * (division and square root correctly rounded).  m2, sigma: d x fp32. */
int ss_welford_sigma(const float *m2, uint64_t n, float *sigma, size_t d,
                     void *hip_stream);

/*
 * Equation (1): the density phi(v) = |v|_1^2 / (d |v|_2^2) of a vector
 * (1 for a fully dense vector, 1/d for a one-hot one).
 *   v          in   d x fp32
 *   out        out  3 doubles in DEVICE memory, 16-byte aligned:
 *                   out[0] = |v|_1, out[1] = |v|_2^2, out[2] = phi(v) (0 for the zero vector)
 *   workspace  i/o  ss_density_workspace_bytes() bytes of DEVICE memory, 16-byte
 *                   aligned, owned by the caller.  It must be all zero bytes before
 *                   the first call that uses it; every call that runs to completion
 *                   leaves it ready for the next one (no clearing in between).  Two
 *                   calls that may run at the same time need two workspaces.
 * Both sums are accumulated in fp64 (every term is exact) in an order that
 * depends on d alone: the same input gives the same bits on every run.  One
 * kernel launch; the blocks leave partial sums in the workspace and the block
 * that finishes last adds them up.
 */
size_t ss_density_workspace_bytes(void);
int ss_density(const float *v, size_t d, double *out, void *workspace, void *hip_stream);

/*
 * ss_density for callers that cannot allocate device memory or hand in a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same kernel, same results bit for bit as ss_density; the
 * partial sums live in a fixed array inside the library instead
 * (ss_density_workspace_bytes() bytes = 4,160, one copy per device, held until
 * the process ends).  The call allocates and frees nothing.
 *   v, out  as for ss_density
 *   d       at most SS_DENSITY_STATIC_MAX_D coordinates, else SS_ERR_RANGE
 * The device that is current when the call is made must be the one v and out
 * live on.  All calls on one device share that device's array: calls that may
 * overlap in time on one device (two streams, two threads) race - serialise
 * them, or give each its own workspace through ss_density.  The first call on a
 * device looks up the array's address (a host-side runtime query, no stream
 * operation); make that first call outside of graph capture.  A call that is
 * killed half-way can leave the array's counter non-zero; the process cannot
 * repair that (ss_density with a fresh workspace still works).
 */
#define SS_DENSITY_STATIC_MAX_D ((size_t)1 << 36)
int ss_density_static(const float *v, size_t d, double *out, void *hip_stream);

/* the hipError_t (as int) behind this thread's most recent SS_ERR_HIP; 0 if none */
int ss_last_hip_error(void);

/*
 * Measurement aid, not part of the method: dst <- src, nbytes (multiple of 16,
 * both 16-byte aligned, device memory), with the same 128-bit streaming
 * accesses the step kernels use.  Gives the copy bandwidth of the machine and
 * a known byte count against which hardware traffic counters are scaled.
 */
int ss_stream_copy(void *dst, const void *src, size_t nbytes, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SIGNSGD_H */
