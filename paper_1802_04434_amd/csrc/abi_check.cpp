// Stand-alone host program that drives the library through its C ABI only
// (include/signsgd.h), with plain hipMalloc / hipMemcpy and no Python or
// torch: the check that the boundary is usable on its own.
//
//   abi_check <in.bin> <out.bin>
//
// in.bin : header {uint64 d; int32 M; int32 bf16; float beta; float delta},
//          then M gradients (d x fp32, or d x uint16 when bf16), M momentum
//          buffers (d x fp32), x (d x fp32)
// out.bin: voted words, M packed buffers, M momentum buffers, x - as the
//          fused ss_signum_vote_step leaves them
// The caller compares out.bin with whatever reference it trusts.
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include <vector>

#include "../../include/signsgd.h"

#define CHECK_HIP(call)                                                             \
    do {                                                                            \
        hipError_t e_ = (call);                                                     \
        if (e_ != hipSuccess) {                                                     \
            fprintf(stderr, "%s failed: %s\n", #call, hipGetErrorString(e_));       \
            return 2;                                                               \
        }                                                                           \
    } while (0)

struct Header {
    uint64_t d;
    int32_t M;
    int32_t bf16;
    float beta;
    float delta;
};

int main(int argc, char **argv) {
    if (argc != 3) {
        fprintf(stderr, "usage: %s in.bin out.bin\n", argv[0]);
        return 1;
    }
    FILE *in = fopen(argv[1], "rb");
    if (!in) return 1;
    Header h;
    if (fread(&h, sizeof h, 1, in) != 1 || h.M < 1 || h.M > SS_MAX_WORKERS) return 1;
    const size_t d = (size_t)h.d, gsize = h.bf16 ? 2 : 4;
    const size_t pbytes = ss_packed_bytes(d);
    std::vector<char> host(d * 4 > pbytes ? d * 4 : pbytes);
    std::vector<void *> g(h.M), m(h.M), packed(h.M);
    void *x = nullptr, *voted = nullptr;
    for (int w = 0; w < h.M; ++w) {
        CHECK_HIP(hipMalloc(&g[w], d * gsize));
        if (fread(host.data(), gsize, d, in) != d) return 1;
        CHECK_HIP(hipMemcpy(g[w], host.data(), d * gsize, hipMemcpyHostToDevice));
    }
    for (int w = 0; w < h.M; ++w) {
        CHECK_HIP(hipMalloc(&m[w], d * 4));
        if (fread(host.data(), 4, d, in) != d) return 1;
        CHECK_HIP(hipMemcpy(m[w], host.data(), d * 4, hipMemcpyHostToDevice));
        CHECK_HIP(hipMalloc(&packed[w], pbytes));
        CHECK_HIP(hipMemset(packed[w], 0xFF, pbytes));
    }
    CHECK_HIP(hipMalloc(&x, d * 4));
    if (fread(host.data(), 4, d, in) != d) return 1;
    CHECK_HIP(hipMemcpy(x, host.data(), d * 4, hipMemcpyHostToDevice));
    CHECK_HIP(hipMalloc(&voted, pbytes));
    CHECK_HIP(hipMemset(voted, 0xFF, pbytes));
    fclose(in);

    hipStream_t stream;
    CHECK_HIP(hipStreamCreate(&stream));
    const int rc = ss_signum_vote_step((const void *const *)g.data(), h.bf16 ? SS_BF16 : SS_F32,
                                       (float *const *)m.data(), h.M, h.beta, h.delta, (float *)x,
                                       (uint32_t *)voted, (uint32_t *const *)packed.data(), d, stream);
    if (rc != SS_OK) {
        fprintf(stderr, "ss_signum_vote_step returned %d (hip error %d)\n", rc, ss_last_hip_error());
        return 3;
    }
    CHECK_HIP(hipStreamSynchronize(stream));

    FILE *out = fopen(argv[2], "wb");
    if (!out) return 1;
    CHECK_HIP(hipMemcpy(host.data(), voted, pbytes, hipMemcpyDeviceToHost));
    fwrite(host.data(), 1, pbytes, out);
    for (int w = 0; w < h.M; ++w) {
        CHECK_HIP(hipMemcpy(host.data(), packed[w], pbytes, hipMemcpyDeviceToHost));
        fwrite(host.data(), 1, pbytes, out);
    }
    for (int w = 0; w < h.M; ++w) {
        CHECK_HIP(hipMemcpy(host.data(), m[w], d * 4, hipMemcpyDeviceToHost));
        fwrite(host.data(), 4, d, out);
    }
    CHECK_HIP(hipMemcpy(host.data(), x, d * 4, hipMemcpyDeviceToHost));
    fwrite(host.data(), 4, d, out);
    fclose(out);
    for (int w = 0; w < h.M; ++w) {
        CHECK_HIP(hipFree(g[w]));
        CHECK_HIP(hipFree(m[w]));
        CHECK_HIP(hipFree(packed[w]));
    }
    CHECK_HIP(hipFree(x));
    CHECK_HIP(hipFree(voted));
    CHECK_HIP(hipStreamDestroy(stream));
    printf("abi_check ok: d=%zu M=%d\n", d, h.M);
    return 0;
}
