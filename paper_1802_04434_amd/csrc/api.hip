// C ABI of the library (see include/signsgd.h): argument validation, kernel
// selection and launch.  Nothing here allocates or synchronises.
#include "../../include/signsgd.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <type_traits>

#include "step_kernels.hpp"
#include "vote_apply_kernels.hpp"
#include "stats_kernels.hpp"
#include "ternary_kernels.hpp"

// Scratch area of ss_density_static: the same layout ss_density finds in its caller's workspace,
// one copy per device that loads this library, zero when the module is loaded and left zero
// (ticket) by every call that runs to completion.  In host code this name only stands for the
// symbol; the device address comes from hipGetSymbolAddress (see ss_density_static).
static __device__ __align__(256) unsigned long long scratch[sizeof(ss::DensityScratch) / sizeof(unsigned long long)];

namespace {

thread_local int g_last_hip_error = 0;

// device address of `scratch` on each device, looked up the first time a device is used
constexpr int kMaxDevices = 64;
std::atomic<ss::DensityScratch *> g_scratch_on_device[kMaxDevices];

constexpr size_t kMaxGrid = 0x7FFFFFFFull;

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline size_t grad_bytes(ss_dtype gdt) { return gdt == SS_BF16 ? 2 : 4; }

// binary digits needed for a count of up to M votes
inline int count_planes(int M) {
    int p = 1;
    while ((1 << p) <= M) ++p;
    return p;
}

// A buffer of one call, for the check that nothing that is written shares a byte
// with anything else (buffers that are only read may coincide, e.g. one gradient
// handed in for two workers).
struct Span {
    uintptr_t lo, hi;   // [lo, hi); empty spans (NULL pointer or no bytes) never overlap
    bool written;
};

inline Span span(const void *p, size_t bytes, bool written) {
    const uintptr_t lo = reinterpret_cast<uintptr_t>(p);
    return Span{lo, p ? lo + bytes : lo, written};
}

// sorts s; true iff a written span overlaps any other span
inline bool written_spans_overlap(Span *s, int n) {
    std::sort(s, s + n, [](const Span &a, const Span &b) { return a.lo < b.lo; });
    uintptr_t end_any = 0, end_written = 0;   // furthest end among the spans seen so far
    for (int i = 0; i < n; ++i) {
        if (s[i].lo == s[i].hi) continue;
        if (s[i].lo < (s[i].written ? end_any : end_written)) return true;
        end_any = std::max(end_any, s[i].hi);
        if (s[i].written) end_written = std::max(end_written, s[i].hi);
    }
    return false;
}

// Every kernel takes one argument struct by value.  The status is the launch
// call's own return value: an error left on this thread by an earlier, unrelated
// runtime call is neither reported as ours nor cleared.
template <typename Args>
int launch(void (*kernel)(Args), size_t grid, unsigned lds_bytes, hipStream_t stream, const Args &a,
           int block = ss::kBlock) {
    void *params[1] = {const_cast<Args *>(&a)};
    const hipError_t e = hipLaunchKernel(reinterpret_cast<const void *>(kernel), dim3((unsigned)grid),
                                         dim3((unsigned)block), params, lds_bytes, stream);
    if (e != hipSuccess) {
        g_last_hip_error = (int)e;
        return SS_ERR_HIP;
    }
    return SS_OK;
}

// how the coordinate range is cut for a kernel that handles R rows per block
struct Tiling {
    size_t n_tiles;      // blocks on the vector path
    size_t tail_blocks;  // blocks of kBlock scalar coordinates, zero padding included
    size_t words_total;
};

inline Tiling make_tiling(size_t d, int rows, bool covers_padding, int block = ss::kBlock) {
    Tiling t;
    const size_t tile = (size_t)rows * block * ss::kQuad;
    t.words_total = ss_packed_bytes(d) / 4;
    t.n_tiles = d / tile;
    const size_t done = t.n_tiles * tile;
    const size_t end = covers_padding ? t.words_total * 32 : d;
    t.tail_blocks = (end - done + block - 1) / block;
    return t;
}

// ------------------------------------------------------------------------
// Launch shapes of the step kernel (see step_kernels.hpp for the reasoning).
//   streaming shape, d >= kStreamingMinD and several workers: one worker at a
//     time, and a reservation of LDS that no kernel touches, sized so that the
//     wanted number of blocks fits in a compute unit's LDS
//   latency shape, smaller d: all workers' loads at once, no cap
constexpr size_t kStreamingMinD = (size_t)1 << 20;
constexpr int kLdsPerUnitKB = 160;   // what the reservations below assume; checked against the device

// when ss_signum_vote_step is given packed_out buffers it may run as M + 2 launches (see there)
constexpr size_t kSplitMinD = (size_t)1 << 24;
constexpr int kSplitMinWorkers = 2;

// LDS of one compute unit of the current device, in KB; 0 if the runtime will not say.  A pure
// query: nothing is remembered between calls.
inline int lds_per_unit_kb() {
    int dev = 0, bytes = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&bytes, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, dev) != hipSuccess) return 0;
    return bytes / 1024;
}

// The kernels that stream one or a few buffers (pack, apply, copy, Welford, the stand-alone votes)
// are launched with as many blocks per unit as fit while the buffers are small; from about a
// gigabyte per array on every one of them runs 3-12 % faster with roughly 24 KB of loads in flight
// per compute unit (six 256-thread blocks of one row, or four of two rows), which an LDS
// reservation enforces.  Measured on MI355X for 2^27 .. 1.5 * 2^30 coordinates; each entry point
// states the shape it takes on either side of its threshold.
constexpr size_t kLargeD = (size_t)1 << 28;

// the reservations are sized for a unit with kLdsPerUnitKB of LDS: on anything else, no cap
inline bool caps_apply() { return lds_per_unit_kb() == kLdsPerUnitKB; }

constexpr int latency_rows(int m, bool has_m) {
    const int streams = m * (has_m ? 2 : 1);
    return streams >= 8 ? 1 : streams >= 4 ? 2 : 4;
}
constexpr int latency_batch(int m) { return m < 8 ? m : 8; }

template <int NPTR>
void fill_step_args(ss::StepArgs<NPTR> &a, int M, const void *const *g, float *const *m, uint32_t *const *packed,
                    float beta, float delta, float *x, uint32_t *voted, size_t d) {
    for (int w = 0; w < NPTR; ++w) {
        a.p.g[w] = w < M ? g[w] : nullptr;
        a.p.m[w] = (m && w < M) ? m[w] : nullptr;
        a.p.packed[w] = (packed && w < M) ? packed[w] : nullptr;
    }
    a.x = x;
    a.voted = voted;
    a.beta = beta;
    a.omb = 1.0f - beta;
    a.delta = delta;
    a.M = M;
    a.write_packed = packed != nullptr;
    a.warmup = 0;
    a.sum_update = 0;
    a.sums = nullptr;
    a.d = d;
}

template <int MT, int NPTR, int BLOCK, int BW, int R, int HOLD_KB, bool LOADS_FIRST, bool HAS_M, bool VOTE, typename G>
int launch_step_shape(ss::StepArgs<NPTR> &a, size_t d, hipStream_t stream) {
    const Tiling t = make_tiling(d, R, true, BLOCK);
    a.n_tiles = t.n_tiles;
    a.words_total = t.words_total;
    const size_t grid = t.n_tiles + t.tail_blocks;
    if (grid > kMaxGrid) return SS_ERR_ARG;
    return launch(ss::step_kernel<MT, NPTR, BLOCK, BW, R, HOLD_KB, LOADS_FIRST, HAS_M, VOTE, G>, grid, 0, stream, a, BLOCK);
}

// what distinguishes the variants of the step (see ss_step_flags)
struct StepVariant {
    unsigned flags;
    int8_t *sums;
};

// MT > 0: M fixed at compile time; MT == 0: any M up to SS_MAX_WORKERS
template <int MT, bool HAS_M, bool VOTE, typename G>
int launch_step_m(int M, const void *const *g, float *const *m, uint32_t *const *packed, float beta, float delta,
                  float *x, uint32_t *voted, StepVariant var, size_t d, hipStream_t stream) {
    constexpr int NPTR = MT > 0 ? MT : SS_MAX_WORKERS;
    ss::StepArgs<NPTR> a;
    fill_step_args<NPTR>(a, M, g, HAS_M ? m : nullptr, packed, beta, delta, x, voted, d);
    a.warmup = (var.flags & SS_STEP_WARMUP) ? 1 : 0;
    a.sum_update = (var.flags & SS_STEP_SUM_UPDATE) ? 1 : 0;
    a.sums = var.sums;
    constexpr bool kBf16 = std::is_same<G, ss::Bf16Grad>::value;
    if constexpr (MT == 1) {
        // a single worker is two or three streams whatever the shape: no cap needed
        if constexpr (!VOTE && HAS_M) {
            // pack over a large vector: one row per block, six blocks per unit
            if (d >= kLargeD && caps_apply()) return launch_step_shape<1, NPTR, 256, 1, 1, 24, true, true, false, G>(a, d, stream);
        }
        if constexpr (VOTE) {
            // the whole step for one worker (Algorithm 1, or Signum on one worker): the same shape from
            // 2^27 coordinates on (+5-12 % without momentum, +1-8 % with)
            if (d >= ((size_t)1 << 27) && caps_apply()) return launch_step_shape<1, NPTR, 256, 1, 1, 24, true, HAS_M, true, G>(a, d, stream);
        }
        constexpr int R = VOTE ? 2 : 4;
        return launch_step_shape<1, NPTR, 256, 1, R, 0, false, HAS_M, VOTE, G>(a, d, stream);
    } else {
        // Streaming shapes.  Each keeps roughly 16-24 KB of loads in flight per compute unit (see
        // step_kernels.hpp) and was picked by measurement among block sizes 64-1024, 1-8 workers per
        // stage, 1-8 rows and 1-5 blocks per unit, with the workloads' own buffer placement.  The
        // reservations only mean what they should on a part with the LDS size they were sized for.
        if (d >= kStreamingMinD && lds_per_unit_kb() == kLdsPerUnitKB) {
            if constexpr (!HAS_M) {
                // gradients only: four (bf16: eight) loads per lane make up for the missing momentum stream
                return launch_step_shape<MT, NPTR, 256, 2, kBf16 ? 4 : 2, 64, true, false, VOTE, G>(a, d, stream);
            } else if constexpr (!kBf16) {
                // fp32: one 512-thread block per unit, one worker and one row at a time
                return launch_step_shape<MT, NPTR, 512, 1, 1, 96, true, true, VOTE, G>(a, d, stream);
            } else {
                // bf16 gradients (a wave's gradient load is half as long): from four workers on, four
                // 128-thread blocks per unit that take two workers at a time; below that, two
                // 256-thread blocks with two rows, the loads left to the compiler's own interleaving
                if (M >= 4) return launch_step_shape<MT, NPTR, 128, 2, 1, 40, true, true, VOTE, G>(a, d, stream);
                return launch_step_shape<MT, NPTR, 256, 1, 2, 64, false, true, VOTE, G>(a, d, stream);
            }
        }
        constexpr int R = MT > 0 ? latency_rows(MT, HAS_M) : 1;
        constexpr int BW = MT > 0 ? latency_batch(MT) : 8;
        return launch_step_shape<MT, NPTR, 256, BW, R, 0, false, HAS_M, VOTE, G>(a, d, stream);
    }
}

template <bool HAS_M, typename G>
int launch_step(int M, const void *const *g, float *const *m, uint32_t *const *packed, float beta,
                float delta, float *x, uint32_t *voted, StepVariant var, size_t d, hipStream_t stream) {
#define SS_CASE(n) \
    case n: return launch_step_m<n, HAS_M, true, G>(M, g, m, packed, beta, delta, x, voted, var, d, stream)
    switch (M) {
        SS_CASE(1); SS_CASE(2); SS_CASE(3); SS_CASE(4); SS_CASE(5); SS_CASE(6); SS_CASE(7); SS_CASE(8);
        SS_CASE(16);
        default: return launch_step_m<0, HAS_M, true, G>(M, g, m, packed, beta, delta, x, voted, var, d, stream);
    }
#undef SS_CASE
}

// the votes read M buffers at once; with packed buffers beyond ~128 MB each (d >= 2^30) two blocks
// per unit are faster than eight (+12 % at d = 1.5 G, M = 8), below that nothing is gained
constexpr size_t kVoteCapMinD = (size_t)1 << 30;
constexpr int kVoteHoldKB = 64;

template <int M>
int launch_vote_fixed(const uint32_t *const *packed, uint32_t *voted, size_t d, hipStream_t stream) {
    ss::VoteArgs<M> a;
    for (int w = 0; w < M; ++w) a.packed[w] = packed[w];
    a.voted = voted;
    a.M = M;
    a.d = d;
    a.n_vec = ss_packed_bytes(d) / 16;
    const size_t grid = (a.n_vec + ss::kBlock - 1) / ss::kBlock;
    if (grid > kMaxGrid) return SS_ERR_ARG;
    if (d >= kVoteCapMinD && caps_apply()) return launch(ss::vote_kernel<M, kVoteHoldKB>, grid, 0, stream, a);
    return launch(ss::vote_kernel<M, 0>, grid, 0, stream, a);
}

int launch_vote_any(const uint32_t *const *packed, int M, uint32_t *voted, size_t d, hipStream_t stream) {
    ss::VoteArgs<SS_MAX_WORKERS> a;
    for (int w = 0; w < SS_MAX_WORKERS; ++w) a.packed[w] = w < M ? packed[w] : nullptr;
    a.voted = voted;
    a.M = M;
    a.d = d;
    a.n_vec = ss_packed_bytes(d) / 16;
    const size_t grid = (a.n_vec + ss::kBlock - 1) / ss::kBlock;
    if (grid > kMaxGrid) return SS_ERR_ARG;
    if (d >= kVoteCapMinD && caps_apply()) return launch(ss::vote_kernel_any<kVoteHoldKB>, grid, 0, stream, a);
    return launch(ss::vote_kernel_any<0>, grid, 0, stream, a);
}

// launch helpers of the ternary (vote with abstention) kernels
template <int BLOCK, int BW, int R, int HOLD_KB, bool LOADS_FIRST, bool HAS_M, bool VOTE, typename G>
int launch_ternary_shape(ss::TernaryStepArgs &a, size_t d, hipStream_t stream) {
    const Tiling t = make_tiling(d, R, true, BLOCK);
    a.n_tiles = t.n_tiles;
    a.words_total = t.words_total;
    const size_t grid = t.n_tiles + t.tail_blocks;
    if (grid > kMaxGrid) return SS_ERR_ARG;
    return launch(ss::ternary_step_kernel<BLOCK, BW, R, HOLD_KB, LOADS_FIRST, HAS_M, VOTE, G>, grid, 0, stream, a, BLOCK);
}

template <bool HAS_M, bool VOTE, typename G>
int launch_ternary(ss::TernaryStepArgs &a, size_t d, hipStream_t stream) {
    constexpr bool kBf16 = std::is_same<G, ss::Bf16Grad>::value;
    if (VOTE && a.M >= 2 && d >= kStreamingMinD && lds_per_unit_kb() == kLdsPerUnitKB) {
        // bf16 gradients with momentum, from four workers on: the binary step's shape for that case
        if (kBf16 && HAS_M && a.M >= 4) return launch_ternary_shape<128, 2, 1, 40, true, HAS_M, VOTE, G>(a, d, stream);
        // otherwise two blocks per unit, one worker at a time (the one-block-per-unit shape of
        // the binary step measured 7 % slower here)
        return launch_ternary_shape<256, 1, 2, 64, false, HAS_M, VOTE, G>(a, d, stream);
    }
    if constexpr (!VOTE && HAS_M) {
        // one worker's ternary pack: four blocks of two rows per unit, six of one row over a large vector
        if (caps_apply()) {
            if (d >= kLargeD) return launch_ternary_shape<256, 1, 1, 24, true, true, false, G>(a, d, stream);
            if (d >= kStreamingMinD) return launch_ternary_shape<256, 1, 2, 40, true, true, false, G>(a, d, stream);
        }
    }
    return launch_ternary_shape<256, 1, 2, 0, false, HAS_M, VOTE, G>(a, d, stream);
}

template <bool VOTE>
int dispatch_ternary(ss::TernaryStepArgs &a, ss_dtype gdt, bool has_m, size_t d, hipStream_t stream) {
    if (has_m) {
        if (gdt == SS_F32) return launch_ternary<true, VOTE, ss::F32Grad>(a, d, stream);
        return launch_ternary<true, VOTE, ss::Bf16Grad>(a, d, stream);
    }
    if (gdt == SS_F32) return launch_ternary<false, VOTE, ss::F32Grad>(a, d, stream);
    return launch_ternary<false, VOTE, ss::Bf16Grad>(a, d, stream);
}

}  // namespace

extern "C" {

size_t ss_packed_words(size_t d) { return d / 32 + (d % 32 != 0 ? 1 : 0); }

size_t ss_packed_bytes(size_t d) { return (ss_packed_words(d) * 4 + 15) / 16 * 16; }

int ss_last_hip_error(void) { return g_last_hip_error; }

static int signum_pack_impl(const void *g, ss_dtype gdt, float *m, float beta, uint32_t *packed, size_t d,
                            unsigned flags, void *hip_stream) {
    if (gdt != SS_F32 && gdt != SS_BF16) return SS_ERR_DTYPE;
    if (d == 0) return SS_OK;
    if (!g || !packed) return SS_ERR_NULL;
    if (!aligned16(g) || !aligned16(m) || !aligned16(packed)) return SS_ERR_ALIGN;
    Span spans[3] = {span(g, d * grad_bytes(gdt), false), span(m, d * sizeof(float), true),
                     span(packed, ss_packed_bytes(d), true)};
    if (written_spans_overlap(spans, 3)) return SS_ERR_ARG;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const void *gs[1] = {g};
    float *ms[1] = {m};
    uint32_t *ps[1] = {packed};
    const StepVariant var{flags, nullptr};
    if (m) {
        if (gdt == SS_F32)
            return launch_step_m<1, true, false, ss::F32Grad>(1, gs, ms, ps, beta, 0.0f, nullptr, nullptr, var, d, stream);
        return launch_step_m<1, true, false, ss::Bf16Grad>(1, gs, ms, ps, beta, 0.0f, nullptr, nullptr, var, d, stream);
    }
    if (gdt == SS_F32)
        return launch_step_m<1, false, false, ss::F32Grad>(1, gs, ms, ps, beta, 0.0f, nullptr, nullptr, var, d, stream);
    return launch_step_m<1, false, false, ss::Bf16Grad>(1, gs, ms, ps, beta, 0.0f, nullptr, nullptr, var, d, stream);
}

int ss_signum_pack(const void *g, ss_dtype gdt, float *m, float beta, uint32_t *packed, size_t d,
                   void *hip_stream) {
    return signum_pack_impl(g, gdt, m, beta, packed, d, SS_STEP_DEFAULT, hip_stream);
}

int ss_signum_pack_warmup(const void *g, ss_dtype gdt, float *m, float beta, uint32_t *packed, size_t d,
                          void *hip_stream) {
    return signum_pack_impl(g, gdt, m, beta, packed, d, SS_STEP_WARMUP, hip_stream);
}

long ss_warmup_length(float beta_f) {
    const double beta = (double)beta_f;
    if (!(beta > 0.0 && beta < 1.0)) return SS_ERR_ARG;
    // smallest C >= 1 with (C/2) beta^C (C+1) (1 - beta^2) <= 1 and beta^(C+1) <= 1/2
    double beta_to_c = 1.0;
    for (long c = 1; c <= SS_WARMUP_MAX; ++c) {
        beta_to_c *= beta;
        const bool bias_settled = 0.5 * (double)c * beta_to_c <= 1.0 / ((1.0 - beta * beta) * ((double)c + 1.0));
        const bool decayed = beta_to_c * beta <= 0.5;
        if (bias_settled && decayed) return c;
    }
    return SS_ERR_RANGE;
}

int ss_majority_vote(const uint32_t *const *packed, int M, uint32_t *voted, size_t d, void *hip_stream) {
    if (M < 1 || M > SS_MAX_WORKERS) return SS_ERR_BAD_M;
    if (d == 0) return SS_OK;
    if (!packed || !voted) return SS_ERR_NULL;
    for (int w = 0; w < M; ++w)
        if (!packed[w]) return SS_ERR_NULL;
    if (!aligned16(voted)) return SS_ERR_ALIGN;
    for (int w = 0; w < M; ++w)
        if (!aligned16(packed[w])) return SS_ERR_ALIGN;
    {
        Span spans[SS_MAX_WORKERS + 1];
        for (int w = 0; w < M; ++w) spans[w] = span(packed[w], ss_packed_bytes(d), false);
        spans[M] = span(voted, ss_packed_bytes(d), true);
        if (written_spans_overlap(spans, M + 1)) return SS_ERR_ARG;
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
#define SS_CASE(n) \
    case n: return launch_vote_fixed<n>(packed, voted, d, stream)
    switch (M) {
        SS_CASE(1); SS_CASE(2); SS_CASE(3); SS_CASE(4); SS_CASE(5); SS_CASE(6); SS_CASE(7); SS_CASE(8);
        SS_CASE(9); SS_CASE(10); SS_CASE(11); SS_CASE(12); SS_CASE(13); SS_CASE(14); SS_CASE(15); SS_CASE(16);
        default: return launch_vote_any(packed, M, voted, d, stream);
    }
#undef SS_CASE
}

int ss_sign_apply(float *x, const uint32_t *bits, float delta, size_t d, void *hip_stream) {
    if (d == 0) return SS_OK;
    if (!x || !bits) return SS_ERR_NULL;
    if (!aligned16(x) || !aligned16(bits)) return SS_ERR_ALIGN;
    Span spans[2] = {span(x, d * sizeof(float), true), span(bits, ss_packed_words(d) * 4, false)};
    if (written_spans_overlap(spans, 2)) return SS_ERR_ARG;
    const bool large = d >= kLargeD && caps_apply();   // then one row per block, six blocks per unit
    const Tiling t = make_tiling(d, large ? 1 : 4, false);
    ss::ApplyArgs a;
    a.x = x;
    a.bits = bits;
    a.delta = delta;
    a.d = d;
    a.n_tiles = t.n_tiles;
    const size_t grid = t.n_tiles + t.tail_blocks;
    if (grid > kMaxGrid) return SS_ERR_ARG;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (large) return launch(ss::apply_kernel<1, 24, true>, grid, 0, stream, a);
    return launch(ss::apply_kernel<4, 0, false>, grid, 0, stream, a);
}

int ss_signum_vote_step_ex(const void *const *g, ss_dtype gdt, float *const *m, int M, float beta, float delta,
                           float *x, uint32_t *voted, uint32_t *const *packed_out, int8_t *sums_out, size_t d,
                           unsigned flags, void *hip_stream) {
    if (M < 1 || M > SS_MAX_WORKERS) return SS_ERR_BAD_M;
    if (gdt != SS_F32 && gdt != SS_BF16) return SS_ERR_DTYPE;
    if (flags & ~(unsigned)(SS_STEP_WARMUP | SS_STEP_SUM_UPDATE)) return SS_ERR_ARG;
    if (d == 0) return SS_OK;
    if (!g || !x || !voted) return SS_ERR_NULL;
    for (int w = 0; w < M; ++w) {
        if (!g[w]) return SS_ERR_NULL;
        if (m && !m[w]) return SS_ERR_NULL;
        if (packed_out && !packed_out[w]) return SS_ERR_NULL;
    }
    if (!aligned16(x) || !aligned16(voted) || !aligned16(sums_out)) return SS_ERR_ALIGN;
    for (int w = 0; w < M; ++w) {
        if (!aligned16(g[w])) return SS_ERR_ALIGN;
        if (m && !aligned16(m[w])) return SS_ERR_ALIGN;
        if (packed_out && !aligned16(packed_out[w])) return SS_ERR_ALIGN;
    }
    {
        Span spans[3 * SS_MAX_WORKERS + 3];
        int n = 0;
        for (int w = 0; w < M; ++w) {
            spans[n++] = span(g[w], d * grad_bytes(gdt), false);
            if (m) spans[n++] = span(m[w], d * sizeof(float), true);
            if (packed_out) spans[n++] = span(packed_out[w], ss_packed_bytes(d), true);
        }
        spans[n++] = span(x, d * sizeof(float), true);
        spans[n++] = span(voted, ss_packed_bytes(d), true);
        spans[n++] = span(sums_out, d, true);
        if (written_spans_overlap(spans, n)) return SS_ERR_ARG;
    }
    // A large vector, and the caller wants every worker's bits anyway: then those buffers can carry
    // the signs from launch to launch, and M pack launches + vote + apply (each touching two or
    // three buffers chip-wide at a time) are never slower than the one-pass kernel that also writes
    // the bits, and up to 10 % faster (measured for M = 2 .. 16 at 2^25, 1.4 * 2^27 and 2^29
    // coordinates: fp32 0-8 %, bf16 2-10 %).  Same results, bit for bit.
    if (packed_out && !sums_out && !(flags & SS_STEP_SUM_UPDATE) && d >= kSplitMinD && M >= kSplitMinWorkers) {
        for (int w = 0; w < M; ++w) {
            const int rc = signum_pack_impl(g[w], gdt, m ? m[w] : nullptr, beta, packed_out[w], d,
                                            flags & SS_STEP_WARMUP, hip_stream);
            if (rc != SS_OK) return rc;
        }
        const int rc = ss_majority_vote(packed_out, M, voted, d, hip_stream);
        if (rc != SS_OK) return rc;
        return ss_sign_apply(x, voted, delta, d, hip_stream);
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const StepVariant var{flags, sums_out};
    if (m) {
        if (gdt == SS_F32)
            return launch_step<true, ss::F32Grad>(M, g, m, packed_out, beta, delta, x, voted, var, d, stream);
        return launch_step<true, ss::Bf16Grad>(M, g, m, packed_out, beta, delta, x, voted, var, d, stream);
    }
    if (gdt == SS_F32)
        return launch_step<false, ss::F32Grad>(M, g, m, packed_out, beta, delta, x, voted, var, d, stream);
    return launch_step<false, ss::Bf16Grad>(M, g, m, packed_out, beta, delta, x, voted, var, d, stream);
}

int ss_signum_vote_step(const void *const *g, ss_dtype gdt, float *const *m, int M, float beta, float delta,
                        float *x, uint32_t *voted, uint32_t *const *packed_out, size_t d, void *hip_stream) {
    return ss_signum_vote_step_ex(g, gdt, m, M, beta, delta, x, voted, packed_out, nullptr, d, SS_STEP_DEFAULT,
                                  hip_stream);
}

int ss_vote_sum(const uint32_t *const *packed, int M, int8_t *sums, size_t d, void *hip_stream) {
    if (M < 1 || M > SS_MAX_WORKERS) return SS_ERR_BAD_M;
    if (d == 0) return SS_OK;
    if (!packed || !sums) return SS_ERR_NULL;
    for (int w = 0; w < M; ++w)
        if (!packed[w]) return SS_ERR_NULL;
    if (!aligned16(sums)) return SS_ERR_ALIGN;
    for (int w = 0; w < M; ++w)
        if (!aligned16(packed[w])) return SS_ERR_ALIGN;
    {
        Span spans[SS_MAX_WORKERS + 1];
        for (int w = 0; w < M; ++w) spans[w] = span(packed[w], ss_packed_bytes(d), false);
        spans[M] = span(sums, d, true);
        if (written_spans_overlap(spans, M + 1)) return SS_ERR_ARG;
    }
    ss::VoteSumArgs a;
    for (int w = 0; w < SS_MAX_WORKERS; ++w) a.packed[w] = w < M ? packed[w] : nullptr;
    a.sums = sums;
    a.M = M;
    a.d = d;
    a.n_vec = ss_packed_bytes(d) / 16;
    const size_t grid = (a.n_vec + ss::kBlock - 1) / ss::kBlock;
    if (grid > kMaxGrid) return SS_ERR_ARG;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    // beyond cache-resident sizes two blocks per unit instead of four (the tile in LDS already
    // limits them to four): +3 % at d = 138 M, +9 % at 1.5 G
    constexpr int kVoteSumHoldKB = 24;
    const bool capped = d >= ((size_t)1 << 27) && caps_apply();
    switch (count_planes(M)) {
        case 1: return capped ? launch(ss::vote_sum_kernel<1, kVoteSumHoldKB>, grid, 0, stream, a)
                              : launch(ss::vote_sum_kernel<1, 0>, grid, 0, stream, a);
        case 2: return capped ? launch(ss::vote_sum_kernel<2, kVoteSumHoldKB>, grid, 0, stream, a)
                              : launch(ss::vote_sum_kernel<2, 0>, grid, 0, stream, a);
        case 3: return capped ? launch(ss::vote_sum_kernel<3, kVoteSumHoldKB>, grid, 0, stream, a)
                              : launch(ss::vote_sum_kernel<3, 0>, grid, 0, stream, a);
        case 4: return capped ? launch(ss::vote_sum_kernel<4, kVoteSumHoldKB>, grid, 0, stream, a)
                              : launch(ss::vote_sum_kernel<4, 0>, grid, 0, stream, a);
        case 5: return capped ? launch(ss::vote_sum_kernel<5, kVoteSumHoldKB>, grid, 0, stream, a)
                              : launch(ss::vote_sum_kernel<5, 0>, grid, 0, stream, a);
        case 6: return capped ? launch(ss::vote_sum_kernel<6, kVoteSumHoldKB>, grid, 0, stream, a)
                              : launch(ss::vote_sum_kernel<6, 0>, grid, 0, stream, a);
        default: return capped ? launch(ss::vote_sum_kernel<7, kVoteSumHoldKB>, grid, 0, stream, a)
                               : launch(ss::vote_sum_kernel<7, 0>, grid, 0, stream, a);
    }
}

int ss_sum_apply(float *x, const int8_t *sums, float delta, size_t d, void *hip_stream) {
    if (d == 0) return SS_OK;
    if (!x || !sums) return SS_ERR_NULL;
    if (!aligned16(x) || !aligned16(sums)) return SS_ERR_ALIGN;
    Span spans[2] = {span(x, d * sizeof(float), true), span(sums, d, false)};
    if (written_spans_overlap(spans, 2)) return SS_ERR_ARG;
    const bool large = d >= kLargeD && caps_apply();   // then one row per block, six blocks per unit
    const Tiling t = make_tiling(d, large ? 1 : 4, false);
    ss::SumApplyArgs a;
    a.x = x;
    a.sums = sums;
    a.delta = delta;
    a.d = d;
    a.n_tiles = t.n_tiles;
    const size_t grid = t.n_tiles + t.tail_blocks;
    if (grid > kMaxGrid) return SS_ERR_ARG;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (large) return launch(ss::sum_apply_kernel<1, 24, true>, grid, 0, stream, a);
    return launch(ss::sum_apply_kernel<4, 0, false>, grid, 0, stream, a);
}

int ss_welford_update(const void *g, ss_dtype gdt, float *mean, float *m2, uint64_t n, size_t d, void *hip_stream) {
    if (gdt != SS_F32 && gdt != SS_BF16) return SS_ERR_DTYPE;
    if (n < 1 || n > (1ull << 24)) return SS_ERR_ARG;   // n must be exact in fp32
    if (d == 0) return SS_OK;
    if (!g || !mean || !m2) return SS_ERR_NULL;
    if (!aligned16(g) || !aligned16(mean) || !aligned16(m2)) return SS_ERR_ALIGN;
    Span spans[3] = {span(g, d * grad_bytes(gdt), false), span(mean, d * sizeof(float), true),
                     span(m2, d * sizeof(float), true)};
    if (written_spans_overlap(spans, 3)) return SS_ERR_ARG;
    // five streams: from 2^27 coordinates on one row per block and six blocks per unit (+4 % at
    // d = 138 M, +10 % at 1.5 G), below that two rows and no cap
    const bool large = d >= ((size_t)1 << 27) && caps_apply();
    const Tiling t = make_tiling(d, large ? 1 : 2, false);
    ss::WelfordArgs a;
    a.g = g;
    a.mean = mean;
    a.m2 = m2;
    a.n = (float)n;
    a.d = d;
    a.n_tiles = t.n_tiles;
    const size_t grid = t.n_tiles + t.tail_blocks;
    if (grid > kMaxGrid) return SS_ERR_ARG;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (large) {
        if (gdt == SS_F32) return launch(ss::welford_update_kernel<1, 24, true, ss::F32Grad>, grid, 0, stream, a);
        return launch(ss::welford_update_kernel<1, 24, true, ss::Bf16Grad>, grid, 0, stream, a);
    }
    if (gdt == SS_F32) return launch(ss::welford_update_kernel<2, 0, false, ss::F32Grad>, grid, 0, stream, a);
    return launch(ss::welford_update_kernel<2, 0, false, ss::Bf16Grad>, grid, 0, stream, a);
}

int ss_welford_sigma(const float *m2, uint64_t n, float *sigma, size_t d, void *hip_stream) {
    if (n < 1 || n > (1ull << 24)) return SS_ERR_ARG;
    if (d == 0) return SS_OK;
    if (!m2 || !sigma) return SS_ERR_NULL;
    if (!aligned16(m2) || !aligned16(sigma)) return SS_ERR_ALIGN;
    Span spans[2] = {span(m2, d * sizeof(float), false), span(sigma, d * sizeof(float), true)};
    if (written_spans_overlap(spans, 2)) return SS_ERR_ARG;
    // two rows per block, six blocks per unit at every size (+2-9 % over four rows and no cap)
    const bool capped = caps_apply();
    const Tiling t = make_tiling(d, capped ? 2 : 4, false);
    ss::SigmaArgs a;
    a.m2 = m2;
    a.sigma = sigma;
    a.n = (float)n;
    a.d = d;
    a.n_tiles = t.n_tiles;
    const size_t grid = t.n_tiles + t.tail_blocks;
    if (grid > kMaxGrid) return SS_ERR_ARG;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (capped) return launch(ss::welford_sigma_kernel<2, 24, true>, grid, 0, stream, a);
    return launch(ss::welford_sigma_kernel<4, 0, false>, grid, 0, stream, a);
}

size_t ss_density_workspace_bytes(void) { return sizeof(ss::DensityScratch); }

// `partials` is a device address: the caller's workspace, or the looked-up address of the array above
static int density_impl(const float *v, size_t d, double *out, ss::DensityScratch *partials, hipStream_t stream) {
    ss::DensityArgs a;
    a.v = v;
    a.out = out;
    a.scratch = partials;
    a.d = d;
    a.n_tiles = d / ((size_t)ss::kDensityRows * ss::kDensityThreads * ss::kQuad);
    // every block gets the same number of tiles (the last one possibly fewer): the grid is a
    // function of d alone, which is what fixes the order of the additions
    const size_t per_block = (a.n_tiles + ss::kDensityMaxBlocks - 1) / ss::kDensityMaxBlocks;
    size_t grid = per_block ? (a.n_tiles + per_block - 1) / per_block : 1;
    if (grid == 0) grid = 1;
    return launch(ss::density_kernel, grid, 0, stream, a, ss::kDensityThreads);
}

int ss_density(const float *v, size_t d, double *out, void *workspace, void *hip_stream) {
    if (!out || !workspace) return SS_ERR_NULL;
    if (d > 0 && !v) return SS_ERR_NULL;
    if (!aligned16(v) || !aligned16(out) || !aligned16(workspace)) return SS_ERR_ALIGN;
    Span spans[3] = {span(out, 3 * sizeof(double), true), span(workspace, sizeof(ss::DensityScratch), true),
                     span(v, d * sizeof(float), false)};
    if (written_spans_overlap(spans, 3)) return SS_ERR_ARG;
    return density_impl(v, d, out, static_cast<ss::DensityScratch *>(workspace), static_cast<hipStream_t>(hip_stream));
}

int ss_density_static(const float *v, size_t d, double *out, void *hip_stream) {
    if (!out) return SS_ERR_NULL;
    if (d > 0 && !v) return SS_ERR_NULL;
    if (!aligned16(v) || !aligned16(out)) return SS_ERR_ALIGN;
    if (d > SS_DENSITY_STATIC_MAX_D) return SS_ERR_RANGE;
    Span spans[2] = {span(out, 3 * sizeof(double), true), span(v, d * sizeof(float), false)};
    if (written_spans_overlap(spans, 2)) return SS_ERR_ARG;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) {
        g_last_hip_error = (int)e;
        return SS_ERR_HIP;
    }
    if (dev < 0 || dev >= kMaxDevices) return SS_ERR_ARG;
    ss::DensityScratch *on_device = g_scratch_on_device[dev].load(std::memory_order_acquire);
    if (!on_device) {
        // first call on this device (which is current): every device holds its own copy of the
        // array at its own address.  Two threads racing here look up the same address.
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            g_last_hip_error = (int)e;
            return SS_ERR_HIP;
        }
        on_device = static_cast<ss::DensityScratch *>(p);
        g_scratch_on_device[dev].store(on_device, std::memory_order_release);
    }
    return density_impl(v, d, out, on_device, static_cast<hipStream_t>(hip_stream));
}

// ---- majority vote with abstention ----

int ss_signum_pack_ternary(const void *g, ss_dtype gdt, float *m, float beta, float tau, uint32_t *neg,
                           uint32_t *zero, size_t d, void *hip_stream) {
    if (gdt != SS_F32 && gdt != SS_BF16) return SS_ERR_DTYPE;
    if (!(tau >= 0.0f)) return SS_ERR_ARG;
    if (d == 0) return SS_OK;
    if (!g || !neg || !zero) return SS_ERR_NULL;
    if (!aligned16(g) || !aligned16(m) || !aligned16(neg) || !aligned16(zero)) return SS_ERR_ALIGN;
    Span spans[4] = {span(g, d * grad_bytes(gdt), false), span(m, d * sizeof(float), true),
                     span(neg, ss_packed_bytes(d), true), span(zero, ss_packed_bytes(d), true)};
    if (written_spans_overlap(spans, 4)) return SS_ERR_ARG;
    ss::TernaryStepArgs a{};
    a.g[0] = g;
    a.m[0] = m;
    a.neg_out = neg;
    a.zero_out = zero;
    a.beta = beta;
    a.omb = 1.0f - beta;
    a.tau = tau;
    a.M = 1;
    a.quorum = 1;
    a.d = d;
    return dispatch_ternary<false>(a, gdt, m != nullptr, d, static_cast<hipStream_t>(hip_stream));
}

int ss_quorum_vote(const uint32_t *const *neg, const uint32_t *const *zero, int M, int quorum,
                   uint32_t *voted_neg, uint32_t *voted_zero, size_t d, void *hip_stream) {
    if (M < 1 || M > SS_MAX_WORKERS) return SS_ERR_BAD_M;
    if (quorum < 1) return SS_ERR_ARG;
    if (d == 0) return SS_OK;
    if (!neg || !zero || !voted_neg || !voted_zero) return SS_ERR_NULL;
    for (int w = 0; w < M; ++w)
        if (!neg[w] || !zero[w]) return SS_ERR_NULL;
    if (!aligned16(voted_neg) || !aligned16(voted_zero)) return SS_ERR_ALIGN;
    for (int w = 0; w < M; ++w)
        if (!aligned16(neg[w]) || !aligned16(zero[w])) return SS_ERR_ALIGN;
    {
        Span spans[2 * SS_MAX_WORKERS + 2];
        for (int w = 0; w < M; ++w) {
            spans[2 * w] = span(neg[w], ss_packed_bytes(d), false);
            spans[2 * w + 1] = span(zero[w], ss_packed_bytes(d), false);
        }
        spans[2 * M] = span(voted_neg, ss_packed_bytes(d), true);
        spans[2 * M + 1] = span(voted_zero, ss_packed_bytes(d), true);
        if (written_spans_overlap(spans, 2 * M + 2)) return SS_ERR_ARG;
    }
    ss::QuorumVoteArgs a{};
    for (int w = 0; w < M; ++w) {
        a.neg[w] = neg[w];
        a.zero[w] = zero[w];
    }
    a.voted_neg = voted_neg;
    a.voted_zero = voted_zero;
    a.M = M;
    a.quorum = quorum > M + 1 ? M + 1 : quorum;   // any quorum above M can never be met: same answers
    a.d = d;
    a.n_vec = ss_packed_bytes(d) / 16;
    const size_t grid = (a.n_vec + ss::kBlock - 1) / ss::kBlock;
    if (grid > kMaxGrid) return SS_ERR_ARG;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    // beyond cache-resident sizes two blocks per unit instead of eight: +2-4 % at d = 138 M, +9 % at 1.5 G
    const bool capped = d >= ((size_t)1 << 27) && caps_apply();
    switch (count_planes(M)) {
        case 1: return capped ? launch(ss::quorum_vote_kernel<1, kVoteHoldKB>, grid, 0, stream, a)
                              : launch(ss::quorum_vote_kernel<1, 0>, grid, 0, stream, a);
        case 2: return capped ? launch(ss::quorum_vote_kernel<2, kVoteHoldKB>, grid, 0, stream, a)
                              : launch(ss::quorum_vote_kernel<2, 0>, grid, 0, stream, a);
        case 3: return capped ? launch(ss::quorum_vote_kernel<3, kVoteHoldKB>, grid, 0, stream, a)
                              : launch(ss::quorum_vote_kernel<3, 0>, grid, 0, stream, a);
        case 4: return capped ? launch(ss::quorum_vote_kernel<4, kVoteHoldKB>, grid, 0, stream, a)
                              : launch(ss::quorum_vote_kernel<4, 0>, grid, 0, stream, a);
        case 5: return capped ? launch(ss::quorum_vote_kernel<5, kVoteHoldKB>, grid, 0, stream, a)
                              : launch(ss::quorum_vote_kernel<5, 0>, grid, 0, stream, a);
        case 6: return capped ? launch(ss::quorum_vote_kernel<6, kVoteHoldKB>, grid, 0, stream, a)
                              : launch(ss::quorum_vote_kernel<6, 0>, grid, 0, stream, a);
        default: return capped ? launch(ss::quorum_vote_kernel<7, kVoteHoldKB>, grid, 0, stream, a)
                               : launch(ss::quorum_vote_kernel<7, 0>, grid, 0, stream, a);
    }
}

int ss_ternary_apply(float *x, const uint32_t *neg, const uint32_t *zero, float delta, size_t d,
                     void *hip_stream) {
    if (d == 0) return SS_OK;
    if (!x || !neg || !zero) return SS_ERR_NULL;
    if (!aligned16(x) || !aligned16(neg) || !aligned16(zero)) return SS_ERR_ALIGN;
    Span spans[3] = {span(x, d * sizeof(float), true), span(neg, ss_packed_words(d) * 4, false),
                     span(zero, ss_packed_words(d) * 4, false)};
    if (written_spans_overlap(spans, 3)) return SS_ERR_ARG;
    const bool large = d >= kLargeD && caps_apply();   // then two rows per block, four blocks per unit
    const Tiling t = make_tiling(d, large ? 2 : 4, false);
    ss::TernaryApplyArgs a;
    a.x = x;
    a.neg = neg;
    a.zero = zero;
    a.delta = delta;
    a.d = d;
    a.n_tiles = t.n_tiles;
    const size_t grid = t.n_tiles + t.tail_blocks;
    if (grid > kMaxGrid) return SS_ERR_ARG;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (large) return launch(ss::ternary_apply_kernel<2, 40, true>, grid, 0, stream, a);
    return launch(ss::ternary_apply_kernel<4, 0, false>, grid, 0, stream, a);
}

int ss_signum_vote_step_ternary(const void *const *g, ss_dtype gdt, float *const *m, int M, float beta, float tau,
                                int quorum, float delta, float *x, uint32_t *voted_neg, uint32_t *voted_zero,
                                size_t d, void *hip_stream) {
    if (M < 1 || M > SS_MAX_WORKERS) return SS_ERR_BAD_M;
    if (gdt != SS_F32 && gdt != SS_BF16) return SS_ERR_DTYPE;
    if (!(tau >= 0.0f) || quorum < 1) return SS_ERR_ARG;
    if (d == 0) return SS_OK;
    if (!g || !x || !voted_neg || !voted_zero) return SS_ERR_NULL;
    for (int w = 0; w < M; ++w) {
        if (!g[w]) return SS_ERR_NULL;
        if (m && !m[w]) return SS_ERR_NULL;
    }
    if (!aligned16(x) || !aligned16(voted_neg) || !aligned16(voted_zero)) return SS_ERR_ALIGN;
    for (int w = 0; w < M; ++w) {
        if (!aligned16(g[w])) return SS_ERR_ALIGN;
        if (m && !aligned16(m[w])) return SS_ERR_ALIGN;
    }
    {
        Span spans[2 * SS_MAX_WORKERS + 3];
        int n = 0;
        for (int w = 0; w < M; ++w) {
            spans[n++] = span(g[w], d * grad_bytes(gdt), false);
            if (m) spans[n++] = span(m[w], d * sizeof(float), true);
        }
        spans[n++] = span(x, d * sizeof(float), true);
        spans[n++] = span(voted_neg, ss_packed_bytes(d), true);
        spans[n++] = span(voted_zero, ss_packed_bytes(d), true);
        if (written_spans_overlap(spans, n)) return SS_ERR_ARG;
    }
    ss::TernaryStepArgs a{};
    for (int w = 0; w < M; ++w) {
        a.g[w] = g[w];
        a.m[w] = m ? m[w] : nullptr;
    }
    a.x = x;
    a.voted_neg = voted_neg;
    a.voted_zero = voted_zero;
    a.beta = beta;
    a.omb = 1.0f - beta;
    a.delta = delta;
    a.tau = tau;
    a.M = M;
    a.quorum = quorum;
    a.d = d;
    return dispatch_ternary<true>(a, gdt, m != nullptr, d, static_cast<hipStream_t>(hip_stream));
}

int ss_stream_copy(void *dst, const void *src, size_t nbytes, void *hip_stream) {
    if (nbytes == 0) return SS_OK;
    if (!dst || !src) return SS_ERR_NULL;
    if (!aligned16(dst) || !aligned16(src)) return SS_ERR_ALIGN;
    if (nbytes % 16 != 0) return SS_ERR_ARG;
    Span spans[2] = {span(dst, nbytes, true), span(src, nbytes, false)};
    if (written_spans_overlap(spans, 2)) return SS_ERR_ARG;
    const size_t n_vec = nbytes / 16;
    // four blocks of two rows per unit; six of one row from a gigabyte on; without the cap four rows
    const bool capped = caps_apply();
    const int rows = !capped ? 4 : (nbytes >= ((size_t)1 << 30) ? 1 : 2);
    const size_t per_block = (size_t)ss::kBlock * rows;
    const size_t grid = (n_vec + per_block - 1) / per_block;
    if (grid > kMaxGrid) return SS_ERR_ARG;
    const ss::CopyArgs a{static_cast<ss::f32x4 *>(dst), static_cast<const ss::f32x4 *>(src), n_vec};
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (rows == 1) return launch(ss::copy_kernel<1, 24>, grid, 0, stream, a);
    if (rows == 2) return launch(ss::copy_kernel<2, 40>, grid, 0, stream, a);
    return launch(ss::copy_kernel<4, 0>, grid, 0, stream, a);
}

}  // extern "C"
