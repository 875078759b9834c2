/* Driver for a host-sanitizer build of mpo_adam_step_noalloc (see test_sanitizers.py): its validation, layer
 * ordering and chunk layout run in fixed-size stack storage and are walked here without a GPU.  Every call is
 * refused before anything would be launched, or fails at the first HIP call (there is no device): the kernel
 * launchers are stubs that must never be reached. */
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include <hip/hip_runtime_api.h>

#include "mpo.h"
#include "mpo_internal.h"

namespace mpo {
static void unreachable(const char *what)
{
    std::fprintf(stderr, "launcher reached: %s\n", what);
    std::abort();
}
hipError_t launch_step_adam(const StepLaunch &) { unreachable("step"); return hipSuccess; }
hipError_t launch_step_adam_ov(const StepLaunch &) { unreachable("step"); return hipSuccess; }
hipError_t launch_step_sgd(const StepLaunch &) { unreachable("step"); return hipSuccess; }
hipError_t launch_step_sgd_ov(const StepLaunch &) { unreachable("step"); return hipSuccess; }
hipError_t launch_split(const float *, uint16_t *, void *, uint64_t, int, int, int, int, uint64_t, uint32_t, hipStream_t)
{
    unreachable("split");
    return hipSuccess;
}
hipError_t launch_merge(const uint16_t *, const void *, float *, uint64_t, int, int, int, int, hipStream_t)
{
    unreachable("merge");
    return hipSuccess;
}
} // namespace mpo

static uint32_t lcg(uint32_t *s) { *s = *s * 1664525u + 1013904223u; return *s; }

#define CHECK(cond) do { if (!(cond)) { std::fprintf(stderr, "line %d: %s\n", __LINE__, #cond); return 1; } } while (0)

int main()
{
    int devices = 0;
    if (hipGetDeviceCount(&devices) == hipSuccess && devices > 0) {
        std::printf("a GPU is present: this driver is for machines without one\n0 lists\n");
        return 0;
    }
    (void)hipGetLastError();
    const mpo_adam_cfg a = {1e-3, 0.9, 0.999, 1e-8, 0.01, 1, 1.0, MPO_BF16, MPO_BF16, MPO_ROUND_TRUNC, 0, 0.0};
    uint32_t seed = 11;
    int lists = 0;
    for (int round = 0; round < 30; ++round) {
        const uint64_t nt = 1 + lcg(&seed) % MPO_NOALLOC_MAX_TENSORS;          /* up to the maximum */
        const int packed = round % 5 == 4, bits = packed ? 1 + (int)(lcg(&seed) % 15) : (round % 3 ? 0 : 8);
        std::vector<mpo_tensor> ts(nt);
        uintptr_t at = 0x100000;
        for (uint64_t i = 0; i < nt; ++i) {
            mpo_tensor &t = ts[i];
            t.n = (lcg(&seed) % 7 == 0) ? 0 : 1 + lcg(&seed) % 20000;
            if (round % 4 == 1 && i == nt / 2) t.n = (1ull << 26) + lcg(&seed) % 10000;     /* a layer with long chunks */
            t.layer = (int32_t)(lcg(&seed) % 9);
            t.res_bits = bits;
            t.res_packed = packed;
            auto take = [&](uint64_t bytes) { void *p = (void *)at; at += (bytes + 255) / 256 * 256 + 256; return p; };
            t.hi = (uint16_t *)take(t.n * 2);
            t.res = take(mpo_res_bytes(t.n, bits, packed));
            t.grad = (const uint16_t *)take(t.n * 2);
            t.m = (float *)take(t.n * 4);
            t.v = (float *)take(t.n * 4);
        }
        /* a valid list gets as far as the first HIP call, which fails without a device */
        const mpo_status s = mpo_adam_step_noalloc(ts.data(), nt, &a, 1, nullptr);
        bool any = false;
        for (const mpo_tensor &t : ts) any |= t.n != 0;
        CHECK(s == (any ? MPO_ERR_HIP : MPO_OK));
        if (any) CHECK(mpo_last_hip_error() != 0);
        /* an overlap anywhere in the list is found */
        if (nt >= 2 && ts[0].n && ts[nt - 1].n) {
            std::vector<mpo_tensor> bad = ts;
            bad[nt - 1].m = (float *)((char *)bad[0].hi + 1);
            CHECK(mpo_adam_step_noalloc(bad.data(), nt, &a, 1, nullptr) == MPO_ERR_ALIAS);
        }
        /* a tensor without a gradient, or without v, is refused */
        if (ts[0].n) {
            std::vector<mpo_tensor> bad = ts;
            bad[0].grad = nullptr;
            CHECK(mpo_adam_step_noalloc(bad.data(), nt, &a, 1, nullptr) == MPO_ERR_INVALID_ARG);
            bad = ts;
            bad[0].v = nullptr;
            CHECK(mpo_adam_step_noalloc(bad.data(), nt, &a, 1, nullptr) == MPO_ERR_INVALID_ARG);
        }
        ++lists;
    }
    /* limits: one tensor too many; one chunk too many (sizes alone decide, the addresses are never used) */
    std::vector<mpo_tensor> many(MPO_NOALLOC_MAX_TENSORS + 1);
    for (mpo_tensor &t : many) t = mpo_tensor{nullptr, nullptr, nullptr, nullptr, nullptr, 0, 0, 0, 0};
    CHECK(mpo_adam_step_noalloc(many.data(), many.size(), &a, 1, nullptr) == MPO_ERR_TOO_LARGE);
    CHECK(mpo_adam_step_noalloc(many.data(), many.size() - 1, &a, 1, nullptr) == MPO_OK);
    const uint64_t big = ((uint64_t)MPO_NOALLOC_MAX_CHUNKS + 1) * 4096;
    const uintptr_t base = (uintptr_t)1 << 44;
    mpo_tensor huge = {(uint16_t *)base, (void *)(base + ((uintptr_t)1 << 40)), (const uint16_t *)(base + ((uintptr_t)2 << 40)),
                       (float *)(base + ((uintptr_t)3 << 40)), (float *)(base + ((uintptr_t)4 << 40)), big, 0, 0, 0};
    CHECK(mpo_adam_step_noalloc(&huge, 1, &a, 1, nullptr) == MPO_ERR_TOO_LARGE);
    huge.n = big - 4096;                      /* exactly the maximum: passes the limits, then needs a device */
    CHECK(mpo_adam_step_noalloc(&huge, 1, &a, 1, nullptr) == MPO_ERR_HIP);
    CHECK(mpo_adam_step_noalloc(nullptr, 1, &a, 1, nullptr) == MPO_ERR_INVALID_ARG);
    CHECK(mpo_adam_step_noalloc(&huge, 1, &a, 0, nullptr) == MPO_ERR_INVALID_ARG);
    CHECK(mpo_adam_step_noalloc(&huge, 1, nullptr, 1, nullptr) == MPO_ERR_INVALID_ARG);
    std::printf("%d lists\n", lists);
    return 0;
}
