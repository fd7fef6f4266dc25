// Gradient statistics of Section 3 (arxiv 1802.04434): Welford's single-pass
// mean / variance over a sequence of stochastic gradients, and the density
// measure phi(v) = |v|_1^2 / (d |v|_2^2) of equation (1), with which the paper
// compares how dense gradient and noise are (Figure 1).
//
// Welford is pointwise and streams like the step kernels (20 bytes per
// coordinate: read g, mean, m2; write mean, m2).  The density is two sums over
// d elements: every term is exact in fp64, each lane accumulates its share in
// fp64, waves and blocks reduce through shuffles and LDS, each block leaves
// its pair of sums in a scratch slot and the last block to finish adds the
// slots.  Every addition happens in an order that depends on d alone, so the
// result is the same bits on every run.
#pragma once
#include "common.hpp"

namespace ss {

struct WelfordArgs {
    const void *g;
    float *mean;
    float *m2;
    float n;          // index of this gradient, 1-based, as fp32
    size_t d;
    size_t n_tiles;
};

// delta = g - mean; mean <- mean + delta / n; m2 <- m2 + delta * (g - mean)
__device__ __forceinline__ void welford1(float g, float n, float &mean, float &m2) {
    const float delta = g - mean;
    const float q = delta / n;
    mean = mean + q;
    const float delta2 = g - mean;
    const float p = delta * delta2;
    m2 = m2 + p;
}

template <int R, int HOLD_KB, bool LOADS_FIRST, typename G>
__global__ __launch_bounds__(kBlock) void welford_update_kernel(const WelfordArgs a) {
    reserve_lds<HOLD_KB>(a.d == ~(size_t)0, reinterpret_cast<uint32_t *>(a.mean));
    const int tid = threadIdx.x;
    const size_t tile = blockIdx.x;
    if (tile < a.n_tiles) {
        size_t q[R];
        f32x4 gv[R], mean[R], m2[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            q[r] = (tile * R + r) * kBlock + tid;
            gv[r] = G::load4(a.g, q[r]);
            mean[r] = ld_stream(reinterpret_cast<const f32x4 *>(a.mean) + q[r]);
            m2[r] = ld_stream(reinterpret_cast<const f32x4 *>(a.m2) + q[r]);
        }
        if (LOADS_FIRST) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int r = 0; r < R; ++r) {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                float mean_c = mean[r][c], m2_c = m2[r][c];
                welford1(gv[r][c], a.n, mean_c, m2_c);
                mean[r][c] = mean_c;
                m2[r][c] = m2_c;
            }
            st_stream(reinterpret_cast<f32x4 *>(a.mean) + q[r], mean[r]);
            st_stream(reinterpret_cast<f32x4 *>(a.m2) + q[r], m2[r]);
        }
        return;
    }
    const size_t i = a.n_tiles * (size_t)(R * kRowCoords) + (tile - a.n_tiles) * kBlock + tid;
    if (i < a.d) {
        float mean = a.mean[i], m2 = a.m2[i];
        welford1(G::load1(a.g, i), a.n, mean, m2);
        a.mean[i] = mean;
        a.m2[i] = m2;
    }
}

struct SigmaArgs {
    const float *m2;
    float *sigma;
    float n;
    size_t d;
    size_t n_tiles;
};

__device__ __forceinline__ float sigma1(float m2, float n) {
    const float var = m2 / n;
    return __builtin_sqrtf(var);
}

template <int R, int HOLD_KB, bool LOADS_FIRST>
__global__ __launch_bounds__(kBlock) void welford_sigma_kernel(const SigmaArgs a) {
    reserve_lds<HOLD_KB>(a.d == ~(size_t)0, reinterpret_cast<uint32_t *>(a.sigma));
    const int tid = threadIdx.x;
    const size_t tile = blockIdx.x;
    if (tile < a.n_tiles) {
        f32x4 v[R];
#pragma unroll
        for (int r = 0; r < R; ++r)
            v[r] = ld_stream(reinterpret_cast<const f32x4 *>(a.m2) + (tile * R + r) * kBlock + tid);
        if (LOADS_FIRST) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int r = 0; r < R; ++r) {
            f32x4 s;
            s.x = sigma1(v[r].x, a.n);
            s.y = sigma1(v[r].y, a.n);
            s.z = sigma1(v[r].z, a.n);
            s.w = sigma1(v[r].w, a.n);
            st_stream(reinterpret_cast<f32x4 *>(a.sigma) + (tile * R + r) * kBlock + tid, s);
        }
        return;
    }
    const size_t i = a.n_tiles * (size_t)(R * kRowCoords) + (tile - a.n_tiles) * kBlock + tid;
    if (i < a.d) a.sigma[i] = sigma1(a.m2[i], a.n);
}

// ------------------------------------------------------------- density ----
// One launch, fixed summation order.  Block b owns tiles b, b + G, b + 2G, ...
// (G = gridDim.x <= kDensityMaxBlocks, a function of d alone); each lane adds its elements in that
// order in fp64, lanes combine through a shuffle tree, waves through LDS, and
// the block's two sums go to slot b of a scratch array.  The block that takes
// the last ticket adds the G slots in a fixed order (whichever block it is),
// writes the result and puts the ticket back to zero for the next call.

// Few, large blocks: the tickets are atomics on one address and cost about 11 ns each, one after
// the other, at the very end of the launch (measured: 780 blocks of 256 threads 25 us at
// d = 25.6 M, 223 blocks of 512 threads 18 us; a plain read of the same bytes 16 us).
constexpr int kDensityMaxBlocks = 256;
constexpr int kDensityThreads = 512;
constexpr int kDensityRows = 8;          // rows of kDensityThreads * 4 coordinates per tile

// layout of the scratch area: ticket counter, then one pair of sums per block
struct DensityScratch {
    unsigned long long ticket;           // zero between calls
    unsigned long long pad[7];
    double partial[kDensityMaxBlocks][2];
};

struct DensityArgs {
    const float *v;
    double *out;       // out[0] = |v|_1, out[1] = |v|_2^2, out[2] = phi
    DensityScratch *scratch;
    size_t d;
    size_t n_tiles;    // tiles of kDensityRows rows
};

__device__ __forceinline__ void accumulate(float v, double &l1, double &l2sq) {
    const double a = (double)__builtin_fabsf(v);
    l1 += a;
    l2sq += a * a;     // exact product of two 24-bit significands
}

// sum over the block of each lane's (s1, s2), in a fixed order; valid in thread 0
__device__ __forceinline__ void block_sum(double &s1, double &s2, double (*part)[kDensityThreads / 64]) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        s1 += __shfl_down(s1, off, 64);
        s2 += __shfl_down(s2, off, 64);
    }
    const int tid = threadIdx.x;
    if ((tid & 63) == 0) {
        part[0][tid >> 6] = s1;
        part[1][tid >> 6] = s2;
    }
    __syncthreads();
    if (tid == 0) {
        s1 = part[0][0];
        s2 = part[1][0];
#pragma unroll
        for (int w = 1; w < kDensityThreads / 64; ++w) {
            s1 += part[0][w];
            s2 += part[1][w];
        }
    }
    __syncthreads();
}

__global__ __launch_bounds__(kDensityThreads) void density_kernel(const DensityArgs a) {
    constexpr int R = kDensityRows;
    constexpr int B = kDensityThreads;
    __shared__ double part[2][B / 64];
    __shared__ int is_last;
    const int tid = threadIdx.x;
    const unsigned G = gridDim.x;
    double l1 = 0.0, l2sq = 0.0;
    for (size_t tile = blockIdx.x; tile < a.n_tiles; tile += G) {
        f32x4 v[R];
#pragma unroll
        for (int r = 0; r < R; ++r)
            v[r] = ld_stream(reinterpret_cast<const f32x4 *>(a.v) + (tile * R + r) * B + tid);
        // a tile's 32 elements first, then the tile into the running sums: the longest chain of
        // additions is 32 + (tiles per block), not their product
        double t1 = 0.0, t2 = 0.0;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            accumulate(v[r].x, t1, t2);
            accumulate(v[r].y, t1, t2);
            accumulate(v[r].z, t1, t2);
            accumulate(v[r].w, t1, t2);
        }
        l1 += t1;
        l2sq += t2;
    }
    // what does not fill a tile: spread over the whole grid, one element per thread and turn
    const size_t done = a.n_tiles * (size_t)(R * B * kQuad);
    for (size_t i = done + (size_t)blockIdx.x * B + tid; i < a.d; i += (size_t)G * B)
        accumulate(a.v[i], l1, l2sq);
    block_sum(l1, l2sq, part);
    if (tid == 0) {
        // Publish the slot, then take a ticket.  The slot is written with device-scope stores
        // (they go through to where every compute die sees them) and the wave waits until they
        // have been performed before it issues the ticket's atomic; a device-wide release fence
        // would do the same but writes back the whole L2 once per block (measured: 30 us of a
        // 50 us launch).
        __hip_atomic_store(&a.scratch->partial[blockIdx.x][0], l1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&a.scratch->partial[blockIdx.x][1], l2sq, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        is_last = __hip_atomic_fetch_add(&a.scratch->ticket, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) ==
                  (unsigned long long)G - 1;
    }
    __syncthreads();
    if (!is_last) return;
    // every other block's slot was performed before its ticket, and this block's loads below are
    // device-scope loads issued after the last ticket came back
    double s1 = 0.0, s2 = 0.0;
    for (unsigned b = tid; b < G; b += B) {
        s1 += __hip_atomic_load(&a.scratch->partial[b][0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s2 += __hip_atomic_load(&a.scratch->partial[b][1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    block_sum(s1, s2, part);
    if (tid == 0) {
        a.out[0] = s1;
        a.out[1] = s2;
        a.out[2] = s2 > 0.0 ? s1 * s1 / ((double)a.d * s2) : 0.0;
        __hip_atomic_store(&a.scratch->ticket, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

}  // namespace ss
