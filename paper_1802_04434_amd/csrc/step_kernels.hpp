// The streaming kernel behind ss_signum_vote_step and ss_signum_pack.
//
// One template covers both: per worker the momentum update and sign of
// Algorithm 2 (or the plain sign of Algorithm 1), the optional per-worker
// packed bits, and - when VOTE is set - the majority vote and parameter
// update of Algorithm 3, all while each gradient, momentum and parameter
// element is read once and written once (arxiv 1802.04434).
//
// The path is bound by HBM traffic (12 bytes per worker and coordinate plus
// 8 for x, against a handful of ALU operations).  What decides how close to
// the DRAM's rate it runs, all measured on MI355X:
//
//  * The loads of a stage (BW workers x R rows, gradient and momentum) are
//    issued into registers before the first dependent operation or store: a
//    store to one worker's momentum could alias (as far as the compiler knows)
//    the next worker's loads and would otherwise serialise them.
//  * The amount of traffic in flight.  16-24 KB of outstanding loads per compute
//    unit (4-6 MB over the chip, the bandwidth-delay product) saturate HBM; more
//    only lengthens the memory system's queues and mixes more DRAM rows into
//    them, and the rate drops by 3-10 % - the more streams (workers) the worse.
//    For large d the kernel therefore takes one or two workers per stage and
//    the block reserves LDS that it never uses (HOLD_KB), which caps the blocks
//    that share a compute unit: e.g. 96 KB leaves room for one 512-thread block
//    in a unit's 160 KB, 64 KB for two 256-thread blocks, 40 KB for four of 128.
//    The host picks the shape (launch_step_m in api.hip).
//  * A tile costs (number of stages) x (one memory latency); the x load goes out
//    with the first stage's loads and the x store overlaps the next tile.
//    Small d is latency bound instead: there all M workers' loads go out
//    together (BW = M) and nothing is held back.
#pragma once
#include "common.hpp"

namespace ss {

template <int NPTR>
struct StepArgs {
    PtrTable<NPTR> p;
    float *x;            // VOTE only
    uint32_t *voted;     // VOTE only
    float beta, omb, delta;
    int M;               // number of workers in use (<= NPTR)
    int write_packed;    // per-worker bits wanted
    int warmup;          // Theorem 3 warm-up: signs come from g while m is still updated
    int sum_update;      // Section 4 "(good)": x <- x - delta * (sum of signs) instead of its sign
    int8_t *sums;        // VOTE only, may be NULL: per-coordinate sum of signs
    size_t d;            // coordinates
    size_t n_tiles;      // blocks on the vector path (R rows of kRowCoords coordinates each)
    size_t words_total;  // words of a packed buffer including zero padding
};

// byte-wise counters: bit k of a nibble -> +1 in byte k
__device__ __forceinline__ uint32_t spread_nibble(uint32_t nib) {
    return (nib * 0x00204081u) & 0x01010101u;
}

// bits of the vote: byte k of `counts` holds how many workers are "-" at
// coordinate k of the quad; "-" wins iff that count reaches T = floor(M/2)+1
__device__ __forceinline__ uint32_t vote_nibble(uint32_t counts, int T) {
    uint32_t nib = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) nib |= (((counts >> (8 * k)) & 0xFFu) >= (uint32_t)T ? 1u : 0u) << k;
    return nib;
}

// the four sums of signs of a quad, S = M - 2 * (count of "-"), as four int8
// in one word.  Biasing every byte by 128 keeps each byte's arithmetic inside
// the byte; flipping bit 7 afterwards removes the bias modulo 256.
__device__ __forceinline__ uint32_t sums_word(uint32_t counts, int M) {
    return ((0x80808080u + (uint32_t)M * 0x01010101u) - 2u * counts) ^ 0x80808080u;
}

// Section 4 "(good)" for one coordinate: x - delta * S, product and
// difference each rounded (the file is compiled with contraction off)
__device__ __forceinline__ float step_sum(float x, float delta, int S) {
    const float t = delta * (float)S;
    return x - t;
}

__device__ __forceinline__ int sum_at(uint32_t counts, int k, int M) {
    return M - 2 * (int)((counts >> (8 * k)) & 0xFFu);
}

// One stage of the vector path: NW consecutive workers starting at w0, R rows.  With
// LOADS_FIRST every load of the stage is issued before anything waits for one of them;
// without it the compiler interleaves (for two rows it starts the second row's loads
// when the first row's momentum has arrived, which keeps fewer bytes in flight).
template <int NW, int R, int BLOCK, bool LOADS_FIRST, bool HAS_M, typename G, int NPTR>
__device__ __forceinline__ void step_stage(const StepArgs<NPTR> &a, int w0, const size_t (&q)[R],
                                           uint32_t (&counts)[R], int lane) {
    f32x4 gv[R][NW], mv[R][NW];
#pragma unroll
    for (int j = 0; j < NW; ++j) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            gv[r][j] = G::load4(a.p.g[w0 + j], q[r]);
            if (HAS_M) mv[r][j] = ld_stream(reinterpret_cast<const f32x4 *>(a.p.m[w0 + j]) + q[r]);
        }
    }
    if (LOADS_FIRST) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < NW; ++j) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            f32x4 v = gv[r][j];
            if (HAS_M) {
                f32x4 m0 = mv[r][j];
                v.x = momentum(a.beta, a.omb, m0.x, v.x);
                v.y = momentum(a.beta, a.omb, m0.y, v.y);
                v.z = momentum(a.beta, a.omb, m0.z, v.z);
                v.w = momentum(a.beta, a.omb, m0.w, v.w);
                st_stream(reinterpret_cast<f32x4 *>(a.p.m[w0 + j]) + q[r], v);
            }
            // Algorithm 2 votes with sign(m); a warm-up iteration with sign(g)
            const uint32_t nib = neg_nibble((HAS_M && a.warmup) ? gv[r][j] : v);
            counts[r] += spread_nibble(nib);
            if (a.write_packed) {
                const uint32_t word = combine8(nib, lane);
                if ((lane & 7) == 0) a.p.packed[w0 + j][q[r] >> 3] = word;
            }
        }
    }
    if (LOADS_FIRST) __builtin_amdgcn_sched_barrier(0);
}

// MT  > 0: number of workers known at compile time (M == MT)
// MT == 0: a.M workers, looped at run time
// BLOCK  : threads per block (a row is BLOCK * 4 coordinates)
// BW     : workers per stage (whose loads are issued together); what M leaves
//          over after the full stages goes one worker at a time
// R      : rows per block
// HOLD_KB: kilobytes of LDS the block reserves and never uses, which caps how
//          many blocks share a compute unit (0: no cap)
template <int MT, int NPTR, int BLOCK, int BW, int R, int HOLD_KB, bool LOADS_FIRST, bool HAS_M, bool VOTE, typename G>
__global__ __launch_bounds__(BLOCK) void step_kernel(const StepArgs<NPTR> a) {
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int M = MT > 0 ? MT : a.M;
    const int T = M / 2 + 1;
    const size_t tile = blockIdx.x;
    reserve_lds<HOLD_KB>(a.d == ~(size_t)0 /* the host rejects such a d */, a.p.packed[0]);

    if (tile < a.n_tiles) {
        size_t q[R];
        uint32_t counts[R];
        f32x4 xv[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            q[r] = (tile * R + r) * BLOCK + tid;
            counts[r] = 0;
            if (VOTE) xv[r] = ld_stream(reinterpret_cast<const f32x4 *>(a.x) + q[r]);
        }
        int w0 = 0;
        if constexpr (BW > 1) {
            for (; w0 + BW <= M; w0 += BW) step_stage<BW, R, BLOCK, LOADS_FIRST, HAS_M, G>(a, w0, q, counts, lane);
        }
        for (; w0 < M; ++w0) step_stage<1, R, BLOCK, LOADS_FIRST, HAS_M, G>(a, w0, q, counts, lane);
        if (VOTE) {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const uint32_t nib = vote_nibble(counts[r], T);
                f32x4 v = xv[r];
                if (a.sum_update) {
                    v.x = step_sum(v.x, a.delta, sum_at(counts[r], 0, M));
                    v.y = step_sum(v.y, a.delta, sum_at(counts[r], 1, M));
                    v.z = step_sum(v.z, a.delta, sum_at(counts[r], 2, M));
                    v.w = step_sum(v.w, a.delta, sum_at(counts[r], 3, M));
                } else {
                    v.x = step(v.x, a.delta, nib & 1u);
                    v.y = step(v.y, a.delta, nib & 2u);
                    v.z = step(v.z, a.delta, nib & 4u);
                    v.w = step(v.w, a.delta, nib & 8u);
                }
                st_stream(reinterpret_cast<f32x4 *>(a.x) + q[r], v);
                if (a.sums) reinterpret_cast<uint32_t *>(a.sums)[q[r]] = sums_word(counts[r], M);
                const uint32_t word = combine8(nib, lane);
                if ((lane & 7) == 0) a.voted[q[r] >> 3] = word;
            }
        }
        return;
    }

    // Scalar path for what does not fill a tile: one coordinate per lane, so
    // the 64-bit wave ballot is two packed words in order.  It also writes
    // the zero padding words.
    const size_t i = a.n_tiles * (size_t)(R * BLOCK * kQuad) + (tile - a.n_tiles) * BLOCK + tid;
    const bool in = i < a.d;
    const size_t word = i >> 5;   // for lanes 0 and 32: the word this half-wave fills
    const bool writes_word = (lane & 31) == 0 && word < a.words_total;
    int count = 0;
    for (int w = 0; w < M; ++w) {
        float v = 0.0f;
        if (in) {
            const float gi = G::load1(a.p.g[w], i);
            v = gi;
            if (HAS_M) {
                v = momentum(a.beta, a.omb, a.p.m[w][i], gi);
                a.p.m[w][i] = v;
                if (a.warmup) v = gi;
            }
        }
        const bool neg = in && v < 0.0f;
        count += neg ? 1 : 0;
        if (a.write_packed) {
            const uint64_t mask = __builtin_amdgcn_ballot_w64(neg);
            if (writes_word) a.p.packed[w][word] = (uint32_t)(lane == 0 ? mask : mask >> 32);
        }
    }
    if (VOTE) {
        const bool vneg = in && count >= T;
        if (in) {
            a.x[i] = a.sum_update ? step_sum(a.x[i], a.delta, M - 2 * count) : step(a.x[i], a.delta, vneg);
            if (a.sums) a.sums[i] = (int8_t)(M - 2 * count);
        }
        const uint64_t mask = __builtin_amdgcn_ballot_w64(vneg);
        if (writes_word) a.voted[word] = (uint32_t)(lane == 0 ? mask : mask >> 32);
    }
}

}  // namespace ss
