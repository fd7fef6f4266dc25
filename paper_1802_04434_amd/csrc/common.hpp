// Shared device helpers for the gfx950 kernels of the signSGD / Signum
// majority-vote step (arxiv 1802.04434, Algorithms 1-3).
//
// Geometry used by every streaming kernel here
//   lane      owns 4 consecutive coordinates ("quad" q = coordinates 4q..4q+3):
//             one 128-bit access per fp32 buffer, one 64-bit access for bf16
//   8 lanes   own 32 consecutive coordinates = one packed word
//   wave      64 lanes = 256 coordinates = 8 packed words
//   block     B threads = 4 B coordinates per row, R rows per block (B = 256 = kBlock
//             everywhere but in the step kernel's streaming shapes, which use 128-512)
// The coordinates that do not fill a whole tile go through a scalar path in
// extra blocks at the end of the same grid (one coordinate per lane; there a
// wave ballot is already in packed-word order).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#pragma clang fp contract(off)

namespace ss {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint16_t u16x4 __attribute__((ext_vector_type(4)));

constexpr int kBlock = 256;          // threads per block unless a kernel is launched with its own
constexpr int kQuad = 4;             // coordinates per lane per row
constexpr int kRowCoords = kBlock * kQuad;   // 1024

// Streaming accesses: every byte is touched once per step, so mark them
// non-temporal and keep them out of the way of anything cached.
template <typename T>
__device__ __forceinline__ T ld_stream(const T *p) {
    return __builtin_nontemporal_load(p);
}
template <typename T>
__device__ __forceinline__ void st_stream(T *p, T v) {
    __builtin_nontemporal_store(v, p);
}

// bf16 -> fp32 is exact: the bf16 pattern is the upper half of the fp32
__device__ __forceinline__ float widen_bf16(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

struct F32Grad {
    typedef float elem;
    static __device__ __forceinline__ f32x4 load4(const void *base, size_t quad) {
        return ld_stream(reinterpret_cast<const f32x4 *>(base) + quad);
    }
    static __device__ __forceinline__ float load1(const void *base, size_t i) {
        return reinterpret_cast<const float *>(base)[i];
    }
};

struct Bf16Grad {
    typedef uint16_t elem;
    static __device__ __forceinline__ f32x4 load4(const void *base, size_t quad) {
        u16x4 r = ld_stream(reinterpret_cast<const u16x4 *>(base) + quad);
        f32x4 o;
        o.x = widen_bf16(r.x); o.y = widen_bf16(r.y); o.z = widen_bf16(r.z); o.w = widen_bf16(r.w);
        return o;
    }
    static __device__ __forceinline__ float load1(const void *base, size_t i) {
        return widen_bf16(reinterpret_cast<const uint16_t *>(base)[i]);
    }
};

// Algorithm 2's momentum line in fp32 with three roundings (two products, one
// sum); the file is compiled with contraction off so no FMA is formed.
__device__ __forceinline__ float momentum(float beta, float omb, float m, float g) {
    float t1 = beta * m;
    float t2 = omb * g;
    return t1 + t2;
}

// sign(v) = -1 exactly when v < 0 (zeros of either sign and NaN are "+")
__device__ __forceinline__ uint32_t neg_bit(float v) { return v < 0.0f ? 1u : 0u; }

__device__ __forceinline__ uint32_t neg_nibble(f32x4 v) {
    return neg_bit(v.x) | (neg_bit(v.y) << 1) | (neg_bit(v.z) << 2) | (neg_bit(v.w) << 3);
}

// Algorithm 3's worker update for one coordinate: s = -1 where `neg`
__device__ __forceinline__ float step(float x, float delta, bool neg) {
    return neg ? x + delta : x - delta;
}

// OR-combine the 4-bit sign nibbles of 8 neighbouring lanes (lane & 7 = 0..7)
// into the 32-bit packed word of their 32 coordinates; every one of the 8
// lanes ends up holding the word.  Three DPP moves inside a row of 16 lanes:
// swap lanes within pairs, swap pairs within a quad, then mirror each group of
// 8 (lane i <-> 7-i), which after the first two steps brings in the other
// quad's value whichever lane it comes from.
__device__ __forceinline__ uint32_t combine8(uint32_t nibble, int lane) {
    uint32_t v = nibble << ((lane & 7) * 4);
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1 /* quad_perm [1,0,3,2] */, 0xF, 0xF, false);
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E /* quad_perm [2,3,0,1] */, 0xF, 0xF, false);
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141 /* row_half_mirror */, 0xF, 0xF, false);
    return v;
}

// Reserves HOLD_KB kilobytes of LDS in the kernel that calls it and never uses them: the only
// effect is that fewer blocks fit into a compute unit's LDS, i.e. a cap on the traffic a unit
// keeps in flight (see step_kernels.hpp for why that matters).  `never` must be false at run
// time; the dead store through `sink` only keeps the compiler from dropping the array.
template <int HOLD_KB>
__device__ __forceinline__ void reserve_lds(bool never, uint32_t *sink) {
    if constexpr (HOLD_KB > 0) {
        __shared__ uint32_t hold[HOLD_KB * 256];
        if (never) {
            hold[threadIdx.x] = threadIdx.x;
            sink[threadIdx.x] = hold[threadIdx.x ^ 1];
        }
    }
}

// kernel argument block: M device pointers by value (no table in memory)
template <int N>
struct PtrTable {
    const void *g[N];
    float *m[N];           // all NULL when there is no momentum
    uint32_t *packed[N];   // all NULL when per-worker bits are not wanted
};

}  // namespace ss
