/*
 * Memory-safety self-check of the CPU oracle (test infrastructure): every
 * routine is run over ragged sizes with buffers allocated at exactly the
 * documented size, so that AddressSanitizer / UBSan (the test builds this file
 * together with signsgd_oracle.c under -fsanitize=address,undefined) see any
 * access outside them.  Prints "selfcheck ok" and returns 0.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

size_t sso_packed_bytes(size_t d);
int sso_signum_pack(const void *, int, float *, float, uint32_t *, size_t);
int sso_signum_pack_warmup(const void *, int, float *, float, uint32_t *, size_t);
int sso_unpack(const uint32_t *, size_t, int8_t *);
int sso_vote_sum(const uint32_t *const *, int, size_t, int32_t *);
int sso_majority_vote(const uint32_t *const *, int, uint32_t *, size_t);
int sso_sign_apply(float *, const uint32_t *, float, size_t);
int sso_sum_apply(float *, const int8_t *, float, size_t);
int sso_signum_vote_step(const void *const *, int, float *const *, int, float, float, float *, uint32_t *,
                         uint32_t *const *, size_t);
int sso_signum_vote_step_mt(const void *const *, int, float *const *, int, float, float, float *, uint32_t *,
                            uint32_t *const *, size_t, int);
int sso_signum_vote_step_ex(const void *const *, int, float *const *, int, float, float, float *, uint32_t *,
                            uint32_t *const *, int8_t *, size_t, unsigned);
int sso_signum_vote_step_ternary(const void *const *, int, float *const *, int, float, float, int, float, float *,
                                 uint32_t *, uint32_t *, size_t);
int sso_density(const float *, size_t, double *);
int sso_welford_update(const void *, int, float *, float *, uint64_t, size_t);
int sso_welford_sigma(const float *, uint64_t, float *, size_t);
long sso_warmup_length(float);

static uint32_t rng_state = 12345u;
static float next_float(void)
{
    rng_state = rng_state * 1664525u + 1013904223u;
    return (float)((int32_t)rng_state) / 2147483648.0f;
}

#define MUST(call)                                          \
    do {                                                    \
        if ((call) != 0) {                                  \
            fprintf(stderr, "failed: %s\n", #call);         \
            return 1;                                       \
        }                                                   \
    } while (0)

int main(void)
{
    const size_t sizes[] = {1, 31, 32, 33, 127, 128, 129, 1000, 4099};
    for (size_t si = 0; si < sizeof sizes / sizeof sizes[0]; ++si) {
        const size_t d = sizes[si];
        for (int M = 1; M <= 5; M += 2) {
            for (int gdt = 0; gdt < 2; ++gdt) {
                const size_t gsz = gdt ? 2 : 4, pb = sso_packed_bytes(d);
                void *g[5];
                float *m[5];
                uint32_t *packed[5];
                for (int w = 0; w < M; ++w) {
                    g[w] = malloc(d * gsz);
                    m[w] = malloc(d * 4);
                    packed[w] = malloc(pb);
                    for (size_t i = 0; i < d; ++i) {
                        float v = next_float();
                        m[w][i] = next_float();
                        if (gdt) {
                            uint32_t b;
                            memcpy(&b, &v, 4);
                            ((uint16_t *)g[w])[i] = (uint16_t)(b >> 16);
                        } else {
                            ((float *)g[w])[i] = v;
                        }
                    }
                }
                float *x = malloc(d * 4), *sigma = malloc(d * 4);
                uint32_t *voted = malloc(pb), *zero = malloc(pb);
                int8_t *sums = malloc(d), *signs = malloc(d);
                int32_t *sums32 = malloc(d * 4);
                double phi[3];
                for (size_t i = 0; i < d; ++i) x[i] = next_float();
                MUST(sso_signum_pack(g[0], gdt, m[0], 0.9f, packed[0], d));
                MUST(sso_signum_pack(g[0], gdt, NULL, 0.9f, packed[0], d));
                MUST(sso_signum_pack_warmup(g[0], gdt, m[0], 0.9f, packed[0], d));
                MUST(sso_unpack(packed[0], d, signs));
                MUST(sso_signum_vote_step((const void *const *)g, gdt, m, M, 0.9f, 1e-3f, x, voted, packed, d));
                MUST(sso_signum_vote_step((const void *const *)g, gdt, NULL, M, 0.9f, 1e-3f, x, voted, NULL, d));
                MUST(sso_signum_vote_step_mt((const void *const *)g, gdt, m, M, 0.9f, 1e-3f, x, voted, packed, d, 3));
                MUST(sso_vote_sum((const uint32_t *const *)packed, M, d, sums32));
                MUST(sso_majority_vote((const uint32_t *const *)packed, M, voted, d));
                MUST(sso_sign_apply(x, voted, 1e-3f, d));
                MUST(sso_signum_vote_step_ex((const void *const *)g, gdt, m, M, 0.9f, 1e-3f, x, voted, packed, sums, d, 3u));
                MUST(sso_signum_vote_step_ex((const void *const *)g, gdt, m, M, 0.9f, 1e-3f, x, voted, NULL, NULL, d, 0u));
                MUST(sso_sum_apply(x, sums, 1e-3f, d));
                MUST(sso_signum_vote_step_ternary((const void *const *)g, gdt, m, M, 0.9f, 0.2f, 2, 1e-3f, x, voted, zero, d));
                MUST(sso_welford_update(g[0], gdt, m[0], x, 3, d));
                MUST(sso_welford_sigma(m[0], 3, sigma, d));
                MUST(sso_density(x, d, phi));
                for (int w = 0; w < M; ++w) {
                    free(g[w]);
                    free(m[w]);
                    free(packed[w]);
                }
                free(x);
                free(sigma);
                free(voted);
                free(zero);
                free(sums);
                free(signs);
                free(sums32);
            }
        }
    }
    if (sso_warmup_length(0.9f) != 54) return 1;
    printf("selfcheck ok\n");
    return 0;
}
