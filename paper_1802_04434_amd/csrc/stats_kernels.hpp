// Gradient statistics of Section 3 (arxiv 1802.04434): Welford's single-pass
// mean / variance over a sequence of stochastic gradients, and the density
// measure phi(v) = |v|_1^2 / (d |v|_2^2) of equation (1), with which the paper
// compares how dense gradient and noise are (Figure 1).
//
// Welford is pointwise and streams like the step kernels (20 bytes per
// coordinate: read g, mean, m2; write mean, m2).  The density is two sums over
// d elements: every term is exact in fp64, each lane accumulates its share in
// fp64, waves and blocks reduce through shuffles and LDS, and one hardware
// fp64 atomic per block and sum lands in the caller's result.  The
// order of those atomics is not fixed, so the two sums can differ from run to
// run in the last bits (relative error below 1e-12; see the tests).
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

template <int R, typename G>
__global__ __launch_bounds__(kBlock) void welford_update_kernel(const WelfordArgs a) {
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

template <int R>
__global__ __launch_bounds__(kBlock) void welford_sigma_kernel(const SigmaArgs a) {
    const int tid = threadIdx.x;
    const size_t tile = blockIdx.x;
    if (tile < a.n_tiles) {
        f32x4 v[R];
#pragma unroll
        for (int r = 0; r < R; ++r)
            v[r] = ld_stream(reinterpret_cast<const f32x4 *>(a.m2) + (tile * R + r) * kBlock + tid);
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

struct DensityArgs {
    const float *v;
    double *out;       // out[0] = |v|_1, out[1] = |v|_2^2, out[2] = phi
    size_t d;
    size_t n_tiles;    // tiles of R rows; block b takes tiles b, b + gridDim.x, ...
};

__global__ void density_clear_kernel(double *out) {
    if (threadIdx.x < 3) out[threadIdx.x] = 0.0;
}

__device__ __forceinline__ void accumulate(float v, double &l1, double &l2sq) {
    const double a = (double)__builtin_fabsf(v);
    l1 += a;
    l2sq += a * a;     // exact product of two 24-bit significands
}

template <int R>
__global__ __launch_bounds__(kBlock) void density_kernel(const DensityArgs a) {
    __shared__ double part[2][kBlock / 64];
    const int tid = threadIdx.x;
    double l1 = 0.0, l2sq = 0.0;
    for (size_t tile = blockIdx.x; tile < a.n_tiles; tile += gridDim.x) {
        f32x4 v[R];
#pragma unroll
        for (int r = 0; r < R; ++r)
            v[r] = ld_stream(reinterpret_cast<const f32x4 *>(a.v) + (tile * R + r) * kBlock + tid);
#pragma unroll
        for (int r = 0; r < R; ++r) {
            accumulate(v[r].x, l1, l2sq);
            accumulate(v[r].y, l1, l2sq);
            accumulate(v[r].z, l1, l2sq);
            accumulate(v[r].w, l1, l2sq);
        }
    }
    // what does not fill a tile: spread over the whole grid, one element per thread and turn
    const size_t done = a.n_tiles * (size_t)(R * kRowCoords);
    for (size_t i = done + (size_t)blockIdx.x * kBlock + tid; i < a.d; i += (size_t)gridDim.x * kBlock)
        accumulate(a.v[i], l1, l2sq);
    // wave, then block, then one atomic per block and sum
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        l1 += __shfl_down(l1, off, 64);
        l2sq += __shfl_down(l2sq, off, 64);
    }
    if ((tid & 63) == 0) {
        part[0][tid >> 6] = l1;
        part[1][tid >> 6] = l2sq;
    }
    __syncthreads();
    if (tid == 0) {
        double s1 = 0.0, s2 = 0.0;
#pragma unroll
        for (int w = 0; w < kBlock / 64; ++w) {
            s1 += part[0][w];
            s2 += part[1][w];
        }
        unsafeAtomicAdd(&a.out[0], s1);
        unsafeAtomicAdd(&a.out[1], s2);
        // The block that finishes last turns the two sums into phi.  Until
        // then out[2] (cleared to all-zero bits before this kernel) serves as
        // the count of finished blocks.
        __threadfence();
        unsigned long long *ticket = reinterpret_cast<unsigned long long *>(&a.out[2]);
        if (atomicAdd(ticket, 1ull) == (unsigned long long)gridDim.x - 1) {
            __threadfence();
            const double l1 = __hip_atomic_load(&a.out[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const double l2sq = __hip_atomic_load(&a.out[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            a.out[2] = l2sq > 0.0 ? l1 * l1 / ((double)a.d * l2sq) : 0.0;
        }
    }
}

}  // namespace ss
