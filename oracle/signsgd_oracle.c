/*
 * CPU oracle for the signSGD / Signum + majority-vote step.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It exists so that the HIP
 * library can be checked bit for bit against something a reader can verify
 * against the paper by eye.  Only the tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it.  It shares no code with the HIP
 * path and is deliberately plain: one scalar loop per definition, no
 * blocking, no bit tricks, no vector intrinsics.
 *
 * What each routine follows (arxiv 1802.04434):
 *   sso_signum_pack   Algorithm 2 (Signum), momentum line and the sign that
 *                     the next line takes; with m == NULL, Algorithm 1's
 *                     sign(g).  One bit per coordinate as in Table 1.
 *   sso_majority_vote Algorithm 3, server side: sign[ sum_m sign(g_m) ]
 *                     (the "(best)" update of Section 4).
 *   sso_sign_apply    Algorithm 1 / Algorithm 3, worker side:
 *                     x <- x - delta * sign(...).
 *   sso_signum_vote_step  the three above in sequence over M workers.
 *   sso_vote_sum      the integer sum_m sign(g_m) of Section 4's "(good)".
 *   sso_sum_apply     Section 4 "(good)": x <- x - delta * sum_m sign(g_m).
 *   sso_warmup_length Theorem 3's warm-up length C(beta).
 *   sso_signum_pack_warmup  Theorem 3's warm-up iteration: momentum is
 *                     accumulated as usual, the sign is taken from the gradient.
 *   sso_signum_vote_step_ex  the whole step with either or both variants.
 *   sso_*_ternary, sso_quorum_vote  "majority vote with abstention" sketched in
 *                     Section 6 (Discussion): workers may send 0, the server
 *                     sends 0 unless a quorum agrees.  PARITY UNPINNED as far
 *                     as the paper goes: it gives neither the workers'
 *                     criterion nor the quorum rule.  The reading below is
 *                     this build's; under it the arithmetic is exact and the
 *                     routines are pinned by brute force like the others.
 *   sso_density       equation (1): phi(v) = |v|_1^2 / (d |v|_2^2).
 *   sso_welford_update, sso_welford_sigma  the single-pass mean / variance of a
 *                     sequence of stochastic gradients that Section 3 uses to
 *                     measure gradient and noise density (Welford's algorithm).
 *
 * Readings the paper leaves open, fixed here:
 *   sign(v) = -1 if v < 0, else +1.  Zero (either sign of zero) is "+".
 *     The same rule is applied to the integer vote sum, so an even-M tie
 *     votes "+".  (One bit in each direction leaves no code for 0, and the
 *     analysis of Theorem 1 moves every coordinate by exactly delta.)
 *   bit = 1 means sign = -1; coordinate i is bit (i mod 32), least
 *     significant first, of 32-bit word (i div 32); unused bits are 0, and
 *     zero words are appended until the byte length is a multiple of 16.
 *   momentum is fp32: fl(fl(beta*m) + fl((1-beta)*g)), (1-beta) rounded once,
 *     no fused multiply-add (build with -ffp-contract=off), subnormals kept.
 *   with momentum and M workers, every worker keeps its own m and votes
 *     with sign(m_m).
 *   bf16 gradients are widened to fp32 exactly before use.
 *   "(good)" update: x <- fl(x - fl(delta * S)) with the integer sum S
 *     converted to fp32 exactly; with momentum, S sums sign(m_m).
 *   density: every term (|v_i|, v_i^2) is exact in double; the two sums are
 *     accumulated in long double, so the oracle's own rounding is negligible
 *     next to the tolerance the GPU's fp64 sums are held to.
 *   Welford, per coordinate and in fp32, n = index of this gradient (1-based):
 *     delta = g - mean; mean <- mean + delta / n; m2 <- m2 + delta * (g - mean)
 *     each operation rounded once (division and square root correctly
 *     rounded), n converted to fp32 (exact below 2^24);
 *     sigma = sqrt(m2 / n): the population standard deviation over the pass.
 *   abstention (reading, not the paper's): a worker abstains at a coordinate
 *     when |v| < tau, v = m (or g without momentum), tau >= 0 given by the
 *     caller; otherwise it votes sign(v).  The server sums the votes
 *     S = (#plus) - (#minus) and answers sign(S) if |S| >= Q, else 0, with the
 *     quorum Q >= 1 given by the caller.  x moves by -delta * answer, not at
 *     all where the answer is 0.  A ternary vector is two bit planes with the
 *     usual layout: "negative" bits and "zero" bits (never both set).  With
 *     tau = 0, Q = 1 and odd M this is exactly Algorithm 3.
 *   C(beta) is evaluated in double precision with beta^C built by repeated
 *     multiplication; the smallest positive integer meeting both conditions
 *     of Theorem 3 is returned, exactly as the theorem states it.
 *
 * Parity pins: tests/test_oracle_*.py (brute force on small sizes, exact
 * rational rounding, closed forms and invariants).
 */
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define SSO_OK 0
#define SSO_ERR_NULL (-1)
#define SSO_ERR_BAD_M (-2)
#define SSO_ERR_DTYPE (-4)
#define SSO_ERR_ARG (-5)

#define SSO_F32 0
#define SSO_BF16 1

size_t sso_packed_words(size_t d) { return d / 32 + (d % 32 != 0); }

size_t sso_packed_bytes(size_t d)
{
    size_t bytes = 4 * sso_packed_words(d);
    while (bytes % 16 != 0) bytes += 4;
    return bytes;
}

/* gradient element i as an fp32 value */
static float grad_at(const void *g, int gdt, size_t i)
{
    if (gdt == SSO_F32) return ((const float *)g)[i];
    /* bf16 is the upper half of an fp32 */
    uint32_t bits = (uint32_t)((const uint16_t *)g)[i] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return f;
}

static int bit_at(const uint32_t *bits, size_t i)
{
    return (int)((bits[i / 32] >> (i % 32)) & 1u);
}

static void set_bit(uint32_t *bits, size_t i)
{
    bits[i / 32] |= (uint32_t)1 << (i % 32);
}

/* Algorithm 2: m <- beta m + (1-beta) g ; bit_i <- [sign(m_i) = -1].
 * m == NULL: Algorithm 1, bit_i <- [sign(g_i) = -1]. */
int sso_signum_pack(const void *g, int gdt, float *m, float beta,
                    uint32_t *packed, size_t d)
{
    if (gdt != SSO_F32 && gdt != SSO_BF16) return SSO_ERR_DTYPE;
    if (d == 0) return SSO_OK;
    if (!g || !packed) return SSO_ERR_NULL;
    memset(packed, 0, sso_packed_bytes(d));
    const float one_minus_beta = 1.0f - beta;
    for (size_t i = 0; i < d; ++i) {
        float gi = grad_at(g, gdt, i);
        float v;
        if (m) {
            float t1 = beta * m[i];
            float t2 = one_minus_beta * gi;
            m[i] = t1 + t2;
            v = m[i];
        } else {
            v = gi;
        }
        if (v < 0.0f) set_bit(packed, i);
    }
    return SSO_OK;
}

/* the +-1 value a packed bit stands for */
int sso_unpack(const uint32_t *bits, size_t d, int8_t *out)
{
    if (d == 0) return SSO_OK;
    if (!bits || !out) return SSO_ERR_NULL;
    for (size_t i = 0; i < d; ++i) out[i] = bit_at(bits, i) ? -1 : +1;
    return SSO_OK;
}

/* Section 4 "(good)": out_i = sum_m sign_m,i */
int sso_vote_sum(const uint32_t *const *packed, int M, size_t d, int32_t *out)
{
    if (M < 1) return SSO_ERR_BAD_M;
    if (d == 0) return SSO_OK;
    if (!packed || !out) return SSO_ERR_NULL;
    for (int w = 0; w < M; ++w)
        if (!packed[w]) return SSO_ERR_NULL;
    for (size_t i = 0; i < d; ++i) {
        int32_t s = 0;
        for (int w = 0; w < M; ++w) s += bit_at(packed[w], i) ? -1 : +1;
        out[i] = s;
    }
    return SSO_OK;
}

/* Algorithm 3, server: voted bit_i <- [ sign( sum_m sign_m,i ) = -1 ] */
int sso_majority_vote(const uint32_t *const *packed, int M, uint32_t *voted,
                      size_t d)
{
    if (M < 1) return SSO_ERR_BAD_M;
    if (d == 0) return SSO_OK;
    if (!packed || !voted) return SSO_ERR_NULL;
    for (int w = 0; w < M; ++w)
        if (!packed[w]) return SSO_ERR_NULL;
    memset(voted, 0, sso_packed_bytes(d));
    for (size_t i = 0; i < d; ++i) {
        int sum = 0;
        for (int w = 0; w < M; ++w) sum += bit_at(packed[w], i) ? -1 : +1;
        if (sum < 0) set_bit(voted, i);
    }
    return SSO_OK;
}

/* Algorithm 1 / Algorithm 3, worker: x_i <- x_i - delta * s_i, s_i = +-1 */
int sso_sign_apply(float *x, const uint32_t *bits, float delta, size_t d)
{
    if (d == 0) return SSO_OK;
    if (!x || !bits) return SSO_ERR_NULL;
    for (size_t i = 0; i < d; ++i) {
        if (bit_at(bits, i))
            x[i] = x[i] + delta; /* s = -1 */
        else
            x[i] = x[i] - delta; /* s = +1 */
    }
    return SSO_OK;
}

/* One whole step over M workers: Algorithm 2 on every worker, then
 * Algorithm 3.  g, m: arrays of M host pointers (m == NULL: no momentum).
 * packed_out: NULL, or M buffers that receive every worker's sign bits. */
int sso_signum_vote_step(const void *const *g, int gdt, float *const *m, int M,
                         float beta, float delta, float *x, uint32_t *voted,
                         uint32_t *const *packed_out, size_t d)
{
    if (M < 1) return SSO_ERR_BAD_M;
    if (gdt != SSO_F32 && gdt != SSO_BF16) return SSO_ERR_DTYPE;
    if (d == 0) return SSO_OK;
    if (!g || !x || !voted) return SSO_ERR_NULL;

    size_t bytes = sso_packed_bytes(d);
    uint32_t **signs = malloc((size_t)M * sizeof *signs);
    uint32_t *own = NULL;
    if (!signs) return SSO_ERR_ARG;
    if (!packed_out) {
        own = malloc((size_t)M * bytes);
        if (!own) {
            free(signs);
            return SSO_ERR_ARG;
        }
    }
    int rc = SSO_OK;
    for (int w = 0; w < M && rc == SSO_OK; ++w) {
        signs[w] = packed_out ? packed_out[w] : own + (size_t)w * (bytes / 4);
        rc = sso_signum_pack(g[w], gdt, m ? m[w] : NULL, beta, signs[w], d);
    }
    if (rc == SSO_OK)
        rc = sso_majority_vote((const uint32_t *const *)signs, M, voted, d);
    if (rc == SSO_OK) rc = sso_sign_apply(x, voted, delta, d);
    free(own);
    free(signs);
    return rc;
}

/* The same step with the coordinate range cut into `nthreads` contiguous
 * pieces whose boundaries are multiples of 32 (whole packed words), each
 * piece handed to sso_signum_vote_step on its own thread.  Coordinates do
 * not interact, so this is the same result; it only exists so that the
 * benchmark can time the oracle on all host cores as well as on one. */
int sso_signum_vote_step_mt(const void *const *g, int gdt, float *const *m,
                            int M, float beta, float delta, float *x,
                            uint32_t *voted, uint32_t *const *packed_out,
                            size_t d, int nthreads)
{
    if (nthreads < 1) return SSO_ERR_ARG;
    if (M < 1) return SSO_ERR_BAD_M;
    if (gdt != SSO_F32 && gdt != SSO_BF16) return SSO_ERR_DTYPE;
    if (d == 0) return SSO_OK;
    if (!g || !x || !voted) return SSO_ERR_NULL;

    /* piece length: multiple of 128 coordinates, so that every piece's
     * packed range starts on a 16-byte boundary and pad words of one piece
     * never land in the next */
    size_t per = (d + (size_t)nthreads - 1) / (size_t)nthreads;
    per = (per + 127) / 128 * 128;
    int pieces = (int)((d + per - 1) / per);
    size_t gsize = gdt == SSO_F32 ? 4 : 2;
    int rc_all = SSO_OK;

#pragma omp parallel for num_threads(nthreads) schedule(static, 1)
    for (int p = 0; p < pieces; ++p) {
        size_t lo = (size_t)p * per;
        size_t n = d - lo < per ? d - lo : per;
        const void **gp = malloc((size_t)M * sizeof *gp);
        float **mp = malloc((size_t)M * sizeof *mp);
        uint32_t **pp = malloc((size_t)M * sizeof *pp);
        int rc = SSO_ERR_ARG;
        if (gp && mp && pp) {
            for (int w = 0; w < M; ++w) {
                gp[w] = (const char *)g[w] + lo * gsize;
                mp[w] = m ? m[w] + lo : NULL;
                pp[w] = packed_out ? packed_out[w] + lo / 32 : NULL;
            }
            rc = sso_signum_vote_step(gp, gdt, m ? mp : NULL, M, beta, delta,
                                      x + lo, voted + lo / 32,
                                      packed_out ? pp : NULL, n);
        }
        free(gp);
        free(mp);
        free(pp);
        if (rc != SSO_OK) {
#pragma omp critical
            rc_all = rc;
        }
    }
    return rc_all;
}

/* ---- variants: Theorem 3's warm-up and Section 4's "(good)" update ---- */

#define SSO_STEP_WARMUP 1
#define SSO_STEP_SUM_UPDATE 2

/* Theorem 3: C(beta) = min C in Z+ with
 *   (C/2) beta^C <= 1/(1-beta^2) * 1/(C+1)   and   beta^(C+1) <= 1/2      */
long sso_warmup_length(float beta_f)
{
    double beta = (double)beta_f;
    if (!(beta > 0.0 && beta < 1.0)) return SSO_ERR_ARG;
    double pow_c = 1.0; /* beta^C */
    for (long C = 1; C <= 1000000000L; ++C) {
        pow_c *= beta;
        double lhs = (double)C / 2.0 * pow_c;
        double rhs = 1.0 / (1.0 - beta * beta) * (1.0 / ((double)C + 1.0));
        if (lhs <= rhs && pow_c * beta <= 0.5) return C;
    }
    return SSO_ERR_ARG;
}

/* Theorem 3, one of the first C(beta) iterations on one worker:
 * m <- beta m + (1-beta) g as in Algorithm 2, but bit_i <- [sign(g_i) = -1] */
int sso_signum_pack_warmup(const void *g, int gdt, float *m, float beta,
                           uint32_t *packed, size_t d)
{
    if (gdt != SSO_F32 && gdt != SSO_BF16) return SSO_ERR_DTYPE;
    if (d == 0) return SSO_OK;
    if (!g || !packed) return SSO_ERR_NULL;
    if (m) {
        /* the momentum line of Algorithm 2; its sign bits are not used */
        int rc = sso_signum_pack(g, gdt, m, beta, packed, d);
        if (rc != SSO_OK) return rc;
    }
    return sso_signum_pack(g, gdt, NULL, beta, packed, d);
}

/* Section 4 "(good)": x_i <- x_i - delta * S_i, S_i = sum_m sign_m,i */
int sso_sum_apply(float *x, const int8_t *sums, float delta, size_t d)
{
    if (d == 0) return SSO_OK;
    if (!x || !sums) return SSO_ERR_NULL;
    for (size_t i = 0; i < d; ++i) {
        float t = delta * (float)sums[i];
        x[i] = x[i] - t;
    }
    return SSO_OK;
}

/* One whole step with the variants selected by flags:
 *   SSO_STEP_WARMUP      every worker votes with sign(g_m) while its momentum
 *                        is still updated (Theorem 3)
 *   SSO_STEP_SUM_UPDATE  x <- x - delta * sum_m sign (Section 4 "(good)")
 *                        instead of x <- x - delta * sign(sum)
 * voted always receives the bits of sign(sum); sums_out (NULL or d bytes)
 * receives the sums. */
int sso_signum_vote_step_ex(const void *const *g, int gdt, float *const *m,
                            int M, float beta, float delta, float *x,
                            uint32_t *voted, uint32_t *const *packed_out,
                            int8_t *sums_out, size_t d, unsigned flags)
{
    if (M < 1 || M > 127) return SSO_ERR_BAD_M;
    if (gdt != SSO_F32 && gdt != SSO_BF16) return SSO_ERR_DTYPE;
    if (flags & ~(unsigned)(SSO_STEP_WARMUP | SSO_STEP_SUM_UPDATE)) return SSO_ERR_ARG;
    if (d == 0) return SSO_OK;
    if (!g || !x || !voted) return SSO_ERR_NULL;

    size_t bytes = sso_packed_bytes(d);
    uint32_t **signs = malloc((size_t)M * sizeof *signs);
    uint32_t *own = packed_out ? NULL : malloc((size_t)M * bytes);
    int32_t *sums = malloc(d * sizeof *sums);
    int8_t *sums8 = sums_out ? sums_out : malloc(d);
    int rc = (signs && (packed_out || own) && sums && sums8) ? SSO_OK : SSO_ERR_ARG;
    for (int w = 0; w < M && rc == SSO_OK; ++w) {
        signs[w] = packed_out ? packed_out[w] : own + (size_t)w * (bytes / 4);
        if (flags & SSO_STEP_WARMUP)
            rc = sso_signum_pack_warmup(g[w], gdt, m ? m[w] : NULL, beta, signs[w], d);
        else
            rc = sso_signum_pack(g[w], gdt, m ? m[w] : NULL, beta, signs[w], d);
    }
    if (rc == SSO_OK)
        rc = sso_majority_vote((const uint32_t *const *)signs, M, voted, d);
    if (rc == SSO_OK)
        rc = sso_vote_sum((const uint32_t *const *)signs, M, d, sums);
    if (rc == SSO_OK) {
        for (size_t i = 0; i < d; ++i) sums8[i] = (int8_t)sums[i];
        if (flags & SSO_STEP_SUM_UPDATE)
            rc = sso_sum_apply(x, sums8, delta, d);
        else
            rc = sso_sign_apply(x, voted, delta, d);
    }
    if (!sums_out) free(sums8);
    free(sums);
    free(own);
    free(signs);
    return rc;
}

/* ---- gradient statistics (Section 3, equation (1) and Figure 1) ---- */

/* out[0] = |v|_1, out[1] = |v|_2^2, out[2] = phi(v) = |v|_1^2 / (d |v|_2^2) */
int sso_density(const float *v, size_t d, double *out)
{
    if (!out) return SSO_ERR_NULL;
    if (d == 0) {
        out[0] = out[1] = 0.0;
        out[2] = 0.0;
        return SSO_OK;
    }
    if (!v) return SSO_ERR_NULL;
    long double l1 = 0.0L, l2sq = 0.0L;
    for (size_t i = 0; i < d; ++i) {
        double a = v[i] < 0.0f ? -(double)v[i] : (double)v[i];
        l1 += a;
        l2sq += a * a; /* exact: 24-bit significands */
    }
    out[0] = (double)l1;
    out[1] = (double)l2sq;
    out[2] = l2sq > 0.0L ? (double)(l1 * l1 / ((long double)d * l2sq)) : 0.0;
    return SSO_OK;
}

/* Welford's update with the n-th gradient (n >= 1) */
int sso_welford_update(const void *g, int gdt, float *mean, float *m2,
                       uint64_t n, size_t d)
{
    if (gdt != SSO_F32 && gdt != SSO_BF16) return SSO_ERR_DTYPE;
    if (n < 1) return SSO_ERR_ARG;
    if (d == 0) return SSO_OK;
    if (!g || !mean || !m2) return SSO_ERR_NULL;
    const float nf = (float)n;
    for (size_t i = 0; i < d; ++i) {
        float gi = grad_at(g, gdt, i);
        float delta = gi - mean[i];
        float q = delta / nf;
        mean[i] = mean[i] + q;
        float delta2 = gi - mean[i];
        float p = delta * delta2;
        m2[i] = m2[i] + p;
    }
    return SSO_OK;
}

/* sigma_i = sqrt(m2_i / n) */
int sso_welford_sigma(const float *m2, uint64_t n, float *sigma, size_t d)
{
    if (n < 1) return SSO_ERR_ARG;
    if (d == 0) return SSO_OK;
    if (!m2 || !sigma) return SSO_ERR_NULL;
    const float nf = (float)n;
    for (size_t i = 0; i < d; ++i) {
        float var = m2[i] / nf;
        sigma[i] = __builtin_sqrtf(var);
    }
    return SSO_OK;
}

/* ---- majority vote with abstention (Section 6, Discussion; reading above) ---- */

/* worker: momentum as in Algorithm 2 (m may be NULL), then a ternary vote */
int sso_signum_pack_ternary(const void *g, int gdt, float *m, float beta,
                            float tau, uint32_t *neg, uint32_t *zero, size_t d)
{
    if (gdt != SSO_F32 && gdt != SSO_BF16) return SSO_ERR_DTYPE;
    if (!(tau >= 0.0f)) return SSO_ERR_ARG;
    if (d == 0) return SSO_OK;
    if (!g || !neg || !zero) return SSO_ERR_NULL;
    memset(neg, 0, sso_packed_bytes(d));
    memset(zero, 0, sso_packed_bytes(d));
    const float one_minus_beta = 1.0f - beta;
    for (size_t i = 0; i < d; ++i) {
        float gi = grad_at(g, gdt, i);
        float v = gi;
        if (m) {
            float t1 = beta * m[i];
            float t2 = one_minus_beta * gi;
            m[i] = t1 + t2;
            v = m[i];
        }
        float mag = v < 0.0f ? -v : v;
        if (mag < tau)
            set_bit(zero, i); /* abstain */
        else if (v < 0.0f)
            set_bit(neg, i);
    }
    return SSO_OK;
}

/* server: answer_i = sign(S_i) if |S_i| >= quorum else 0 */
int sso_quorum_vote(const uint32_t *const *neg, const uint32_t *const *zero,
                    int M, int quorum, uint32_t *voted_neg,
                    uint32_t *voted_zero, size_t d)
{
    if (M < 1) return SSO_ERR_BAD_M;
    if (quorum < 1) return SSO_ERR_ARG;
    if (d == 0) return SSO_OK;
    if (!neg || !zero || !voted_neg || !voted_zero) return SSO_ERR_NULL;
    memset(voted_neg, 0, sso_packed_bytes(d));
    memset(voted_zero, 0, sso_packed_bytes(d));
    for (size_t i = 0; i < d; ++i) {
        int sum = 0;
        for (int w = 0; w < M; ++w) {
            if (bit_at(zero[w], i)) continue; /* abstained */
            sum += bit_at(neg[w], i) ? -1 : +1;
        }
        if (sum <= -quorum)
            set_bit(voted_neg, i);
        else if (sum < quorum)
            set_bit(voted_zero, i);
    }
    return SSO_OK;
}

/* worker: x_i <- x_i - delta * answer_i */
int sso_ternary_apply(float *x, const uint32_t *neg, const uint32_t *zero,
                      float delta, size_t d)
{
    if (d == 0) return SSO_OK;
    if (!x || !neg || !zero) return SSO_ERR_NULL;
    for (size_t i = 0; i < d; ++i) {
        if (bit_at(zero, i)) continue;
        if (bit_at(neg, i))
            x[i] = x[i] + delta;
        else
            x[i] = x[i] - delta;
    }
    return SSO_OK;
}

/* the three in sequence over M workers */
int sso_signum_vote_step_ternary(const void *const *g, int gdt, float *const *m,
                                 int M, float beta, float tau, int quorum,
                                 float delta, float *x, uint32_t *voted_neg,
                                 uint32_t *voted_zero, size_t d)
{
    if (M < 1) return SSO_ERR_BAD_M;
    if (d == 0) return SSO_OK;
    if (!g || !x || !voted_neg || !voted_zero) return SSO_ERR_NULL;
    size_t words = sso_packed_bytes(d) / 4;
    uint32_t *store = malloc(2 * (size_t)M * words * 4);
    const uint32_t **negs = malloc((size_t)M * sizeof *negs);
    const uint32_t **zeros = malloc((size_t)M * sizeof *zeros);
    int rc = (store && negs && zeros) ? SSO_OK : SSO_ERR_ARG;
    for (int w = 0; w < M && rc == SSO_OK; ++w) {
        uint32_t *n = store + (size_t)(2 * w) * words, *z = n + words;
        negs[w] = n;
        zeros[w] = z;
        rc = sso_signum_pack_ternary(g[w], gdt, m ? m[w] : NULL, beta, tau, n, z, d);
    }
    if (rc == SSO_OK) rc = sso_quorum_vote(negs, zeros, M, quorum, voted_neg, voted_zero, d);
    if (rc == SSO_OK) rc = sso_ternary_apply(x, voted_neg, voted_zero, delta, d);
    free(store);
    free(negs);
    free(zeros);
    return rc;
}
