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
// cap on resident blocks through an LDS reservation), a small server kernel and an apply kernel.
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

// One stage of the vector path: NW consecutive workers starting at w0, R rows (as step_stage
// of the binary kernel: with LOADS_FIRST every load of the stage is out before the first wait)
template <int NW, int R, bool LOADS_FIRST, bool HAS_M, bool VOTE, typename G>
__device__ __forceinline__ void ternary_stage(const TernaryStepArgs &a, int w0, const size_t (&q)[R],
                                              uint32_t (&n_neg)[R], uint32_t (&n_zero)[R], int lane) {
    f32x4 gv[R][NW], mv[R][NW];
#pragma unroll
    for (int j = 0; j < NW; ++j) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            gv[r][j] = G::load4(a.g[w0 + j], q[r]);
            if (HAS_M) mv[r][j] = ld_stream(reinterpret_cast<const f32x4 *>(a.m[w0 + j]) + q[r]);
        }
    }
    if (LOADS_FIRST) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < NW; ++j) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            f32x4 v = gv[r][j];
            if (HAS_M) {
                const f32x4 m0 = mv[r][j];
                v.x = momentum(a.beta, a.omb, m0.x, v.x);
                v.y = momentum(a.beta, a.omb, m0.y, v.y);
                v.z = momentum(a.beta, a.omb, m0.z, v.z);
                v.w = momentum(a.beta, a.omb, m0.w, v.w);
                st_stream(reinterpret_cast<f32x4 *>(a.m[w0 + j]) + q[r], v);
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
    if (LOADS_FIRST) __builtin_amdgcn_sched_barrier(0);
}

// BLOCK threads per block, BW workers per stage (what M leaves over goes one at a time), R rows
// per block, HOLD_KB of LDS reserved to cap the blocks per compute unit, LOADS_FIRST as in the
// binary step kernel
template <int BLOCK, int BW, int R, int HOLD_KB, bool LOADS_FIRST, bool HAS_M, bool VOTE, typename G>
__global__ __launch_bounds__(BLOCK) void ternary_step_kernel(const TernaryStepArgs a) {
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int M = a.M;
    const size_t tile = blockIdx.x;
    reserve_lds<HOLD_KB>(a.d == ~(size_t)0 /* the host rejects such a d */, VOTE ? a.voted_neg : a.neg_out);

    if (tile < a.n_tiles) {
        size_t q[R];
        uint32_t n_neg[R], n_zero[R];
        f32x4 xv[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            q[r] = (tile * R + r) * BLOCK + tid;
            n_neg[r] = 0;
            n_zero[r] = 0;
            if (VOTE) xv[r] = ld_stream(reinterpret_cast<const f32x4 *>(a.x) + q[r]);
        }
        int w0 = 0;
        if constexpr (BW > 1) {
            for (; w0 + BW <= M; w0 += BW) ternary_stage<BW, R, LOADS_FIRST, HAS_M, VOTE, G>(a, w0, q, n_neg, n_zero, lane);
        }
        for (; w0 < M; ++w0) ternary_stage<1, R, LOADS_FIRST, HAS_M, VOTE, G>(a, w0, q, n_neg, n_zero, lane);
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
    const size_t i = a.n_tiles * (size_t)(R * BLOCK * kQuad) + (tile - a.n_tiles) * BLOCK + tid;
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
    size_t n_vec;     // 128-bit groups of words, padding included
};

// Bit-sliced, like the binary vote: a lane holds 128 coordinates (four words)
// of every plane.  The numbers of "-" votes (n) and of abstentions (z) are
// counted into binary planes with a ripple of half adders per worker; then
// t = 2 n + z is formed plane by plane, and since S = #plus - #minus = M - t,
//     answer "-"  iff  S <= -Q  iff  t >= M + Q
//     answer  0   iff  |S| < Q  iff  M - Q < t < M + Q
// which are two comparisons of t with constants, done from the lowest plane up.
constexpr int kQuorumBatch = 4;    // workers (two planes each) whose words are loaded together

__device__ __forceinline__ u32x4 splat(uint32_t v) { return u32x4{v, v, v, v}; }

// planes of (t >= c) for a constant c, t given by its N binary planes
template <int N>
__device__ __forceinline__ u32x4 planes_ge(const u32x4 (&t)[N], int c) {
    if (c <= 0) return splat(0xFFFFFFFFu);
    if (c >= (1 << N)) return splat(0u);
    u32x4 ge = splat(0xFFFFFFFFu);
#pragma unroll
    for (int k = 0; k < N; ++k) ge = ((c >> k) & 1) ? (t[k] & ge) : (t[k] | ge);
    return ge;
}

// NB workers' planes loaded together (no test between the loads), then counted
template <int P, int NB>
__device__ __forceinline__ void quorum_batch(const uint32_t *const *neg, const uint32_t *const *zero, size_t u,
                                             u32x4 (&n)[P], u32x4 (&z)[P]) {
    u32x4 nw[NB], zw[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        nw[j] = ld_stream(reinterpret_cast<const u32x4 *>(neg[j]) + u);
        zw[j] = ld_stream(reinterpret_cast<const u32x4 *>(zero[j]) + u);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        u32x4 cz = zw[j];
        u32x4 cn = nw[j] & ~zw[j];   // an abstention is not a vote, whatever the other plane says
#pragma unroll
        for (int k = 0; k < P; ++k) {
            const u32x4 tn = n[k] & cn, tz = z[k] & cz;
            n[k] ^= cn;
            z[k] ^= cz;
            cn = tn;
            cz = tz;
        }
    }
}

// P = number of binary planes of n and z (M < 2^P); t = 2 n + z <= 2 M needs one more.
// HOLD_KB: LDS reserved to cap the blocks per compute unit.
template <int P, int HOLD_KB>
__global__ __launch_bounds__(kBlock) void quorum_vote_kernel(const QuorumVoteArgs a) {
    reserve_lds<HOLD_KB>(a.d == ~(size_t)0, a.voted_neg);
    constexpr int kCountPlanes = P;
    constexpr int kTotalPlanes = P + 1;
    static_assert(kQuorumBatch == 4, "the remainder switch below lists 1 .. 3");
    const size_t u = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (u >= a.n_vec) return;
    u32x4 n[kCountPlanes], z[kCountPlanes];
#pragma unroll
    for (int k = 0; k < kCountPlanes; ++k) n[k] = z[k] = splat(0u);
    int w0 = 0;
    for (; w0 + kQuorumBatch <= a.M; w0 += kQuorumBatch) quorum_batch<P, kQuorumBatch>(a.neg + w0, a.zero + w0, u, n, z);
    switch (a.M - w0) {
        case 1: quorum_batch<P, 1>(a.neg + w0, a.zero + w0, u, n, z); break;
        case 2: quorum_batch<P, 2>(a.neg + w0, a.zero + w0, u, n, z); break;
        case 3: quorum_batch<P, 3>(a.neg + w0, a.zero + w0, u, n, z); break;
        default: break;
    }
    // t = 2 n + z
    u32x4 t[kTotalPlanes];
    t[0] = z[0];
    u32x4 carry = splat(0u);
#pragma unroll
    for (int k = 1; k < kTotalPlanes; ++k) {
        const u32x4 x = k - 1 < kCountPlanes ? n[k - 1] : splat(0u);
        const u32x4 y = k < kCountPlanes ? z[k] : splat(0u);
        const u32x4 xy = x ^ y;
        t[k] = xy ^ carry;
        carry = (x & y) | (xy & carry);
    }
    const u32x4 is_neg = planes_ge(t, a.M + a.quorum);
    const u32x4 not_plus = planes_ge(t, a.M - a.quorum + 1);
    u32x4 live;
    live.x = live_mask(4 * u + 0, a.d);
    live.y = live_mask(4 * u + 1, a.d);
    live.z = live_mask(4 * u + 2, a.d);
    live.w = live_mask(4 * u + 3, a.d);
    st_stream(reinterpret_cast<u32x4 *>(a.voted_neg) + u, is_neg & live);
    st_stream(reinterpret_cast<u32x4 *>(a.voted_zero) + u, not_plus & ~is_neg & live);
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

template <int R, int HOLD_KB, bool LOADS_FIRST>
__global__ __launch_bounds__(kBlock) void ternary_apply_kernel(const TernaryApplyArgs a) {
    reserve_lds<HOLD_KB>(a.d == ~(size_t)0, reinterpret_cast<uint32_t *>(a.x));
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
        if (LOADS_FIRST) __builtin_amdgcn_sched_barrier(0);
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
