// Stand-alone kernels of the three-call path: the server's majority vote over
// packed sign words and the worker's parameter update from packed bits
// (arxiv 1802.04434, Algorithm 3; Algorithm 1 when the bits are one worker's).
#pragma once
#include "step_kernels.hpp"

namespace ss {

// ---------------------------------------------------------------- vote ----
// Bit-sliced: a 32-bit word holds 32 coordinates of one worker; the M
// workers' words for the same coordinates are added "vertically" with
// carry-save adders into the binary planes of the per-coordinate count of "-"
// votes, and the count is compared with the constant threshold
// T = floor(M/2)+1 plane by plane.  32 coordinates per ALU lane-operation.

struct Sum2 { uint32_t sum, carry; };
__device__ __forceinline__ Sum2 full_add(uint32_t a, uint32_t b, uint32_t c) {
    const uint32_t ab = a ^ b;
    return {ab ^ c, (a & b) | (ab & c)};
}
__device__ __forceinline__ Sum2 half_add(uint32_t a, uint32_t b) { return {a ^ b, a & b}; }

// count >= T decided from the least significant plane upwards:
// ge_k = plane_k > T_k, or equal and ge_(k-1)
__device__ __forceinline__ uint32_t ge_step(uint32_t ge, uint32_t plane, int T, int k) {
    return ((T >> k) & 1) ? (plane & ge) : (plane | ge);
}

// N words of weight 2^K: reduce to one word (plane K) and N/2 carries of
// weight 2^(K+1), fold plane K into the comparison, recurse on the carries.
template <int N, int K, int T>
struct CsaLevel {
    static __device__ __forceinline__ uint32_t run(const uint32_t (&w)[N], uint32_t ge) {
        constexpr int kFull = (N - 1) / 2;
        constexpr int kNext = N / 2;
        uint32_t next[kNext > 0 ? kNext : 1];
        uint32_t acc = w[0];
#pragma unroll
        for (int j = 0; j < kFull; ++j) {
            const Sum2 s = full_add(acc, w[1 + 2 * j], w[2 + 2 * j]);
            acc = s.sum;
            next[j] = s.carry;
        }
        if constexpr (N % 2 == 0) {
            const Sum2 s = half_add(acc, w[N - 1]);
            acc = s.sum;
            next[kFull] = s.carry;
        }
        ge = ge_step(ge, acc, T, K);
        if constexpr (kNext > 0) {
            return CsaLevel<kNext, K + 1, T>::run(next, ge);
        } else {
            return ge;
        }
    }
};

// bit set where at least floor(M/2)+1 of the M words have it set
template <int M>
__device__ __forceinline__ uint32_t majority_word(const uint32_t (&w)[M]) {
    return CsaLevel<M, 0, M / 2 + 1>::run(w, 0xFFFFFFFFu);
}

template <int NPTR>
struct VoteArgs {
    const uint32_t *packed[NPTR];
    uint32_t *voted;
    int M;
    size_t d;
    size_t n_vec;   // 128-bit groups of words, padding included
};

// bits of word `wi` that lie below coordinate d
__device__ __forceinline__ uint32_t live_mask(size_t wi, size_t d) {
    const size_t lo = wi * 32;
    if (lo + 32 <= d) return 0xFFFFFFFFu;
    if (lo >= d) return 0u;
    return (1u << (unsigned)(d - lo)) - 1u;
}

template <int M, int HOLD_KB>
__global__ __launch_bounds__(kBlock) void vote_kernel(const VoteArgs<M> a) {
    reserve_lds<HOLD_KB>(a.d == ~(size_t)0, a.voted);
    const size_t u = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (u >= a.n_vec) return;
    u32x4 in[M];
#pragma unroll
    for (int w = 0; w < M; ++w) in[w] = ld_stream(reinterpret_cast<const u32x4 *>(a.packed[w]) + u);
    uint32_t col[M];
    u32x4 out;
#pragma unroll
    for (int w = 0; w < M; ++w) col[w] = in[w].x;
    out.x = majority_word<M>(col) & live_mask(4 * u + 0, a.d);
#pragma unroll
    for (int w = 0; w < M; ++w) col[w] = in[w].y;
    out.y = majority_word<M>(col) & live_mask(4 * u + 1, a.d);
#pragma unroll
    for (int w = 0; w < M; ++w) col[w] = in[w].z;
    out.z = majority_word<M>(col) & live_mask(4 * u + 2, a.d);
#pragma unroll
    for (int w = 0; w < M; ++w) col[w] = in[w].w;
    out.w = majority_word<M>(col) & live_mask(4 * u + 3, a.d);
    st_stream(reinterpret_cast<u32x4 *>(a.voted) + u, out);
}

// Any M up to SS_MAX_WORKERS: the count planes are kept in seven registers
// and every word is added with a ripple of half adders.
constexpr int kPlanes = 7;   // counts up to 64 < 2^7

// NB workers' 128-bit groups loaded together (no test between the loads: all NB are in flight
// before the first is used), then rippled into the P count planes with half adders
template <int P, int NB>
__device__ __forceinline__ void ripple_batch(const uint32_t *const *packed, size_t u, u32x4 (&plane)[P]) {
    u32x4 in[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) in[j] = ld_stream(reinterpret_cast<const u32x4 *>(packed[j]) + u);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        u32x4 carry = in[j];
#pragma unroll
        for (int k = 0; k < P; ++k) {
            const u32x4 t = plane[k] & carry;
            plane[k] ^= carry;
            carry = t;
        }
    }
}

// all M workers: full batches of NB, then the remaining 1 .. NB-1 as one batch of exactly that size
template <int P, int NB>
__device__ __forceinline__ void ripple_all(const uint32_t *const *packed, int M, size_t u, u32x4 (&plane)[P]) {
    static_assert(NB == 8, "the remainder switch below lists 1 .. 7");
    int w0 = 0;
    for (; w0 + NB <= M; w0 += NB) ripple_batch<P, NB>(packed + w0, u, plane);
    switch (M - w0) {
        case 1: ripple_batch<P, 1>(packed + w0, u, plane); break;
        case 2: ripple_batch<P, 2>(packed + w0, u, plane); break;
        case 3: ripple_batch<P, 3>(packed + w0, u, plane); break;
        case 4: ripple_batch<P, 4>(packed + w0, u, plane); break;
        case 5: ripple_batch<P, 5>(packed + w0, u, plane); break;
        case 6: ripple_batch<P, 6>(packed + w0, u, plane); break;
        case 7: ripple_batch<P, 7>(packed + w0, u, plane); break;
        default: break;
    }
}

template <int HOLD_KB>
__global__ __launch_bounds__(kBlock) void vote_kernel_any(const VoteArgs<64> a) {
    reserve_lds<HOLD_KB>(a.d == ~(size_t)0, a.voted);
    const size_t u = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (u >= a.n_vec) return;
    const int T = a.M / 2 + 1;
    u32x4 plane[kPlanes];
#pragma unroll
    for (int k = 0; k < kPlanes; ++k) plane[k] = u32x4{0, 0, 0, 0};
    ripple_all<kPlanes, 8>(a.packed, a.M, u, plane);
    u32x4 ge = u32x4{0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu};
#pragma unroll
    for (int k = 0; k < kPlanes; ++k) ge = ((T >> k) & 1) ? (plane[k] & ge) : (plane[k] | ge);
    ge.x &= live_mask(4 * u + 0, a.d);
    ge.y &= live_mask(4 * u + 1, a.d);
    ge.z &= live_mask(4 * u + 2, a.d);
    ge.w &= live_mask(4 * u + 3, a.d);
    st_stream(reinterpret_cast<u32x4 *>(a.voted) + u, ge);
}

// --------------------------------------------------------------- apply ----

struct ApplyArgs {
    float *x;
    const uint32_t *bits;
    float delta;
    size_t d;
    size_t n_tiles;   // blocks on the vector path, R rows each
};

// R rows per block, HOLD_KB of LDS reserved (caps the blocks per compute unit), LOADS_FIRST: every
// load of the block is issued before the first result is waited for
template <int R, int HOLD_KB, bool LOADS_FIRST>
__global__ __launch_bounds__(kBlock) void apply_kernel(const ApplyArgs a) {
    reserve_lds<HOLD_KB>(a.d == ~(size_t)0, reinterpret_cast<uint32_t *>(a.x));
    const int tid = threadIdx.x;
    const size_t tile = blockIdx.x;
    if (tile < a.n_tiles) {
        size_t q[R];
        f32x4 xv[R];
        uint32_t word[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            q[r] = (tile * R + r) * kBlock + tid;
            xv[r] = ld_stream(reinterpret_cast<const f32x4 *>(a.x) + q[r]);
            word[r] = a.bits[q[r] >> 3];   // 8 lanes share a word
        }
        if (LOADS_FIRST) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const uint32_t nib = word[r] >> ((tid & 7) * 4);
            f32x4 v = xv[r];
            v.x = step(v.x, a.delta, nib & 1u);
            v.y = step(v.y, a.delta, nib & 2u);
            v.z = step(v.z, a.delta, nib & 4u);
            v.w = step(v.w, a.delta, nib & 8u);
            st_stream(reinterpret_cast<f32x4 *>(a.x) + q[r], v);
        }
        return;
    }
    const size_t i = a.n_tiles * (size_t)(R * kRowCoords) + (tile - a.n_tiles) * kBlock + tid;
    if (i < a.d) {
        const bool neg = (a.bits[i >> 5] >> (i & 31)) & 1u;
        a.x[i] = step(a.x[i], a.delta, neg);
    }
}

// ------------------------------------------------ "(good)": vote sums ----
// Section 4's first scheme sends back the sum of the workers' signs instead of
// its sign.  Bit-sliced like the vote: a lane loads 128 coordinates (four words)
// of every worker with one 128-bit load and ripples them into the binary planes
// of the count of "-" votes; only at the end are the planes turned into one
// int8 per coordinate.  A lane's 128 sums are contiguous in memory, so the block
// passes them through LDS and stores them in coordinate order (a wave's store is
// 1024 contiguous bytes).

struct VoteSumArgs {
    const uint32_t *packed[64];
    int8_t *sums;
    int M;
    size_t d;
    size_t n_vec;      // 128-bit groups of packed words, padding included
};

constexpr int kVoteSumBatch = 8;           // workers whose words are loaded together
constexpr int kVoteSumLaneBytes = 128;     // a lane's 128 coordinates give 128 int8 sums
constexpr int kVoteSumLdsStride = 144;     // ... kept 144 bytes apart in LDS (spreads the banks)

// P = number of binary planes of the count of "-" votes: counts up to M < 2^P
template <int P, int HOLD_KB>
__global__ __launch_bounds__(kBlock) void vote_sum_kernel(const VoteSumArgs a) {
    reserve_lds<HOLD_KB>(a.d == ~(size_t)0, reinterpret_cast<uint32_t *>(a.sums));   // on top of the tile below
    __shared__ __align__(16) unsigned char tile[kBlock * kVoteSumLdsStride];
    const int tid = threadIdx.x;
    const size_t u = (size_t)blockIdx.x * kBlock + tid;
    // lanes beyond the last group (last block only) re-read the last group: their coordinates
    // lie at or beyond d and are never stored
    const size_t ul = u < a.n_vec ? u : a.n_vec - 1;
    u32x4 plane[P];
#pragma unroll
    for (int k = 0; k < P; ++k) plane[k] = u32x4{0, 0, 0, 0};
    ripple_all<P, kVoteSumBatch>(a.packed, a.M, ul, plane);
    // planes -> one int8 sum per coordinate: the lane's 128 sums go to LDS as eight 16-byte pieces
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        u32x4 piece;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int shift = 4 * ((q & 1) * 4 + e);     // nibble of word q / 2
            uint32_t counts = 0;
#pragma unroll
            for (int k = 0; k < P; ++k) counts += spread_nibble((plane[k][q >> 1] >> shift) & 0xFu) << k;
            piece[e] = sums_word(counts, a.M);
        }
        *reinterpret_cast<u32x4 *>(tile + tid * kVoteSumLdsStride + 16 * q) = piece;
    }
    __syncthreads();
    // ... and leave in the order of the coordinates: a wave's store is 1024 contiguous bytes
    const size_t base = (size_t)blockIdx.x * (kBlock * kVoteSumLaneBytes);
    if (base + (size_t)kBlock * kVoteSumLaneBytes <= a.d) {      // every block but the last: no test per store
        u32x4 piece[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int c = j * kBlock + tid;              // 16-byte piece within the block's output
            piece[j] = *reinterpret_cast<const u32x4 *>(tile + (c >> 3) * kVoteSumLdsStride + 16 * (c & 7));
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
            st_stream(reinterpret_cast<u32x4 *>(a.sums + base + 16 * (size_t)(j * kBlock + tid)), piece[j]);
        return;
    }
#pragma unroll 1
    for (int j = 0; j < 8; ++j) {
        const int c = j * kBlock + tid;
        const u32x4 piece = *reinterpret_cast<const u32x4 *>(tile + (c >> 3) * kVoteSumLdsStride + 16 * (c & 7));
        const size_t first = base + 16 * (size_t)c;
        if (first + 16 <= a.d) {
            st_stream(reinterpret_cast<u32x4 *>(a.sums + first), piece);
        } else if (first < a.d) {
            const uint32_t words[4] = {piece.x, piece.y, piece.z, piece.w};
            for (size_t i = first; i < a.d; ++i)
                a.sums[i] = (int8_t)(words[(i - first) >> 2] >> (8 * ((i - first) & 3)));
        }
    }
}

struct SumApplyArgs {
    float *x;
    const int8_t *sums;
    float delta;
    size_t d;
    size_t n_tiles;
};

template <int R, int HOLD_KB, bool LOADS_FIRST>
__global__ __launch_bounds__(kBlock) void sum_apply_kernel(const SumApplyArgs a) {
    reserve_lds<HOLD_KB>(a.d == ~(size_t)0, reinterpret_cast<uint32_t *>(a.x));
    const int tid = threadIdx.x;
    const size_t tile = blockIdx.x;
    if (tile < a.n_tiles) {
        size_t q[R];
        f32x4 xv[R];
        uint32_t sw[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            q[r] = (tile * R + r) * kBlock + tid;
            xv[r] = ld_stream(reinterpret_cast<const f32x4 *>(a.x) + q[r]);
            sw[r] = ld_stream(reinterpret_cast<const uint32_t *>(a.sums) + q[r]);
        }
        if (LOADS_FIRST) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int r = 0; r < R; ++r) {
            f32x4 v = xv[r];
            v.x = step_sum(v.x, a.delta, (int)(int8_t)(sw[r] & 0xFFu));
            v.y = step_sum(v.y, a.delta, (int)(int8_t)((sw[r] >> 8) & 0xFFu));
            v.z = step_sum(v.z, a.delta, (int)(int8_t)((sw[r] >> 16) & 0xFFu));
            v.w = step_sum(v.w, a.delta, (int)(int8_t)(sw[r] >> 24));
            st_stream(reinterpret_cast<f32x4 *>(a.x) + q[r], v);
        }
        return;
    }
    const size_t i = a.n_tiles * (size_t)(R * kRowCoords) + (tile - a.n_tiles) * kBlock + tid;
    if (i < a.d) a.x[i] = step_sum(a.x[i], a.delta, (int)a.sums[i]);
}

// ---------------------------------------------------------------- copy ----

struct CopyArgs {
    f32x4 *dst;
    const f32x4 *src;
    size_t n_vec;
};

template <int R, int HOLD_KB>
__global__ __launch_bounds__(kBlock) void copy_kernel(const CopyArgs a) {
    reserve_lds<HOLD_KB>(a.n_vec == ~(size_t)0, reinterpret_cast<uint32_t *>(a.dst));
    const size_t base = (size_t)blockIdx.x * (kBlock * R) + threadIdx.x;
    f32x4 v[R];
#pragma unroll
    for (int r = 0; r < R; ++r)
        if (base + r * kBlock < a.n_vec) v[r] = ld_stream(a.src + base + r * kBlock);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int r = 0; r < R; ++r)
        if (base + r * kBlock < a.n_vec) st_stream(a.dst + base + r * kBlock, v[r]);
}

}  // namespace ss
