// "Majority vote with abstention", the ternary extension sketched in the
// Discussion (Section 6) of arxiv 1802.04434: a worker that is unsure about a
// coordinate sends 0 instead of a sign, and the server sends 0 back unless a
// quorum agrees.
//
// The paper gives no criterion, so this is a READING, stated in the header of
// the library: a worker abstains where |v| < tau (v = its momentum, or its
// gradient when there is none); the server sums the votes S = #plus - #minus
// and answers sign(S) if |S| >= Q, otherwise 0; x moves by -delta * answer.
// A ternary vector travels as two bit planes in the usual packed layout,
// "negative" and "zero" (never both set).
//
// The kernels mirror the binary ones: a streaming kernel for the worker's pack
// and for the fused step (one worker at a time, same lane geometry, optional
// cap on resident blocks at launch), a small server kernel and an apply kernel.
#pragma once
#include "step_kernels.hpp"
#include "vote_apply_kernels.hpp"

namespace ss {

struct TernaryStepArgs {
    const void *g[64];
    float *m[64];          // all NULL without momentum
    uint32_t *neg_out;     // pack only: this worker's planes
    uint32_t *zero_out;
    float *x;              // fused only
    uint32_t *voted_neg;
    uint32_t *voted_zero;
    float beta, omb, delta, tau;
    int M;
    int quorum;
    size_t d;
    size_t n_tiles;
    size_t words_total;
};

// answer for one coordinate from its counts: bit 0 = negative, bit 1 = zero
__device__ __forceinline__ uint32_t quorum_answer(int n_neg, int n_zero, int M, int Q) {
    const int S = M - n_zero - 2 * n_neg;
    return S <= -Q ? 1u : (S < Q ? 2u : 0u);
}

__device__ __forceinline__ float step_ternary(float x, float delta, uint32_t answer) {
    return (answer & 2u) ? x : ((answer & 1u) ? x + delta : x - delta);
}

template <int R, bool HAS_M, bool VOTE, typename G>
__global__ __launch_bounds__(kBlock) void ternary_step_kernel(const TernaryStepArgs a) {
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int M = a.M;
    const size_t tile = blockIdx.x;

    if (tile < a.n_tiles) {
        size_t q[R];
        uint32_t n_neg[R], n_zero[R];
        f32x4 xv[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            q[r] = (tile * R + r) * kBlock + tid;
            n_neg[r] = 0;
            n_zero[r] = 0;
            if (VOTE) xv[r] = ld_stream(reinterpret_cast<const f32x4 *>(a.x) + q[r]);
        }
        for (int w = 0; w < M; ++w) {
            f32x4 gv[R], mv[R];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                gv[r] = G::load4(a.g[w], q[r]);
                if (HAS_M) mv[r] = ld_stream(reinterpret_cast<const f32x4 *>(a.m[w]) + q[r]);
            }
#pragma unroll
            for (int r = 0; r < R; ++r) {
                f32x4 v = gv[r];
                if (HAS_M) {
                    v.x = momentum(a.beta, a.omb, mv[r].x, v.x);
                    v.y = momentum(a.beta, a.omb, mv[r].y, v.y);
                    v.z = momentum(a.beta, a.omb, mv[r].z, v.z);
                    v.w = momentum(a.beta, a.omb, mv[r].w, v.w);
                    st_stream(reinterpret_cast<f32x4 *>(a.m[w]) + q[r], v);
                }
                uint32_t zero_nib = 0, neg_nib = 0;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const bool abstain = __builtin_fabsf(v[c]) < a.tau;
                    zero_nib |= (abstain ? 1u : 0u) << c;
                    neg_nib |= ((!abstain && v[c] < 0.0f) ? 1u : 0u) << c;
                }
                if (VOTE) {
                    n_neg[r] += spread_nibble(neg_nib);
                    n_zero[r] += spread_nibble(zero_nib);
                } else {
                    const uint32_t nw = combine8(neg_nib, lane);
                    const uint32_t zw = combine8(zero_nib, lane);
                    if ((lane & 7) == 0) {
                        a.neg_out[q[r] >> 3] = nw;
                        a.zero_out[q[r] >> 3] = zw;
                    }
                }
            }
        }
        if (VOTE) {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                uint32_t neg_nib = 0, zero_nib = 0;
                f32x4 v = xv[r];
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const uint32_t ans = quorum_answer((int)((n_neg[r] >> (8 * c)) & 0xFFu),
                                                       (int)((n_zero[r] >> (8 * c)) & 0xFFu), M, a.quorum);
                    neg_nib |= (ans & 1u) << c;
                    zero_nib |= ((ans >> 1) & 1u) << c;
                    v[c] = step_ternary(v[c], a.delta, ans);
                }
                st_stream(reinterpret_cast<f32x4 *>(a.x) + q[r], v);
                const uint32_t nw = combine8(neg_nib, lane);
                const uint32_t zw = combine8(zero_nib, lane);
                if ((lane & 7) == 0) {
                    a.voted_neg[q[r] >> 3] = nw;
                    a.voted_zero[q[r] >> 3] = zw;
                }
            }
        }
        return;
    }

    // scalar path: what does not fill a tile, and the zero padding words
    const size_t i = a.n_tiles * (size_t)(R * kRowCoords) + (tile - a.n_tiles) * kBlock + tid;
    const bool in = i < a.d;
    const size_t word = i >> 5;
    const bool writes_word = (lane & 31) == 0 && word < a.words_total;
    int n_neg = 0, n_zero = 0;
    for (int w = 0; w < M; ++w) {
        float v = 0.0f;
        if (in) {
            v = G::load1(a.g[w], i);
            if (HAS_M) {
                v = momentum(a.beta, a.omb, a.m[w][i], v);
                a.m[w][i] = v;
            }
        }
        const bool abstain = in && __builtin_fabsf(v) < a.tau;
        const bool neg = in && !abstain && v < 0.0f;
        n_neg += neg ? 1 : 0;
        n_zero += abstain ? 1 : 0;
        if (!VOTE) {
            const uint64_t nmask = __builtin_amdgcn_ballot_w64(neg);
            const uint64_t zmask = __builtin_amdgcn_ballot_w64(abstain);
            if (writes_word) {
                a.neg_out[word] = (uint32_t)(lane == 0 ? nmask : nmask >> 32);
                a.zero_out[word] = (uint32_t)(lane == 0 ? zmask : zmask >> 32);
            }
        }
    }
    if (VOTE) {
        const uint32_t ans = in ? quorum_answer(n_neg, n_zero, M, a.quorum) : 0u;
        if (in) a.x[i] = step_ternary(a.x[i], a.delta, ans);
        const uint64_t nmask = __builtin_amdgcn_ballot_w64((ans & 1u) != 0);
        const uint64_t zmask = __builtin_amdgcn_ballot_w64((ans & 2u) != 0);
        if (writes_word) {
            a.voted_neg[word] = (uint32_t)(lane == 0 ? nmask : nmask >> 32);
            a.voted_zero[word] = (uint32_t)(lane == 0 ? zmask : zmask >> 32);
        }
    }
}

// ----------------------------------------------------------- server ----

struct QuorumVoteArgs {
    const uint32_t *neg[64];
    const uint32_t *zero[64];
    uint32_t *voted_neg;
    uint32_t *voted_zero;
    int M;
    int quorum;
    size_t d;
    size_t words_total;
};

// one lane per packed word: counts of "-" and of abstentions for its 32
// coordinates sit in byte lanes of 2 x 8 registers
__global__ __launch_bounds__(kBlock) void quorum_vote_kernel(const QuorumVoteArgs a) {
    const size_t wi = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (wi >= a.words_total) return;
    uint32_t n_neg[8], n_zero[8];
#pragma unroll
    for (int n = 0; n < 8; ++n) n_neg[n] = n_zero[n] = 0;
    for (int w = 0; w < a.M; ++w) {
        const uint32_t zw = a.zero[w][wi];
        const uint32_t nw = a.neg[w][wi] & ~zw;   // an abstention is not a vote, whatever the other plane says
#pragma unroll
        for (int n = 0; n < 8; ++n) {
            n_neg[n] += spread_nibble((nw >> (4 * n)) & 0xFu);
            n_zero[n] += spread_nibble((zw >> (4 * n)) & 0xFu);
        }
    }
    uint32_t out_neg = 0, out_zero = 0;
#pragma unroll
    for (int n = 0; n < 8; ++n) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint32_t ans = quorum_answer((int)((n_neg[n] >> (8 * c)) & 0xFFu),
                                               (int)((n_zero[n] >> (8 * c)) & 0xFFu), a.M, a.quorum);
            out_neg |= (ans & 1u) << (4 * n + c);
            out_zero |= ((ans >> 1) & 1u) << (4 * n + c);
        }
    }
    const uint32_t live = live_mask(wi, a.d);
    a.voted_neg[wi] = out_neg & live;
    a.voted_zero[wi] = out_zero & live;
}

// ------------------------------------------------------------ apply ----

struct TernaryApplyArgs {
    float *x;
    const uint32_t *neg;
    const uint32_t *zero;
    float delta;
    size_t d;
    size_t n_tiles;
};

template <int R>
__global__ __launch_bounds__(kBlock) void ternary_apply_kernel(const TernaryApplyArgs a) {
    const int tid = threadIdx.x;
    const size_t tile = blockIdx.x;
    if (tile < a.n_tiles) {
        size_t q[R];
        f32x4 xv[R];
        uint32_t nw[R], zw[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            q[r] = (tile * R + r) * kBlock + tid;
            xv[r] = ld_stream(reinterpret_cast<const f32x4 *>(a.x) + q[r]);
            nw[r] = a.neg[q[r] >> 3];
            zw[r] = a.zero[q[r] >> 3];
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const uint32_t nn = nw[r] >> ((tid & 7) * 4), zn = zw[r] >> ((tid & 7) * 4);
            f32x4 v = xv[r];
#pragma unroll
            for (int c = 0; c < 4; ++c) v[c] = step_ternary(v[c], a.delta, ((nn >> c) & 1u) | (((zn >> c) & 1u) << 1));
            st_stream(reinterpret_cast<f32x4 *>(a.x) + q[r], v);
        }
        return;
    }
    const size_t i = a.n_tiles * (size_t)(R * kRowCoords) + (tile - a.n_tiles) * kBlock + tid;
    if (i < a.d) {
        const uint32_t ans = ((a.neg[i >> 5] >> (i & 31)) & 1u) | (((a.zero[i >> 5] >> (i & 31)) & 1u) << 1);
        a.x[i] = step_ternary(a.x[i], a.delta, ans);
    }
}

}  // namespace ss
