/* Driver for a sanitizer build of the library's host side (see test_sanitizers.py): plan building,
 * overlap detection, layer and chunk queries and every argument check, without a GPU.  The kernel
 * launchers are replaced by stubs that must never be reached: every call below is either a
 * host-only call or is refused before anything would be launched. */
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
    uint32_t seed = 7;
    int plans = 0;
    /* lists of many tensors at made-up, disjoint addresses (a host plan never touches them) */
    for (int round = 0; round < 40; ++round) {
        const uint64_t nt = lcg(&seed) % 300;
        const int packed = round % 5 == 4, bits = packed ? 1 + (int)(lcg(&seed) % 15) : (round % 3 ? 0 : 8);
        std::vector<mpo_tensor> ts(nt);
        uintptr_t at = 0x100000;
        uint64_t total = 0, chunks = 0;
        uint64_t per_layer[9] = {0};
        for (uint64_t i = 0; i < nt; ++i) {
            mpo_tensor &t = ts[i];
            t.n = (lcg(&seed) % 7 == 0) ? 0 : 1 + lcg(&seed) % 20000;
            t.layer = (int32_t)(lcg(&seed) % 9);
            /* now and then one tensor long enough to give its layer the long chunks */
            if (round % 4 == 1 && i == nt / 2) t.n = (1ull << 26) + lcg(&seed) % 10000;
            per_layer[t.layer] += t.n;
            t.res_bits = bits;
            t.res_packed = packed;
            auto take = [&](uint64_t bytes) { void *p = (void *)at; at += (bytes + 255) / 256 * 256 + 256; return p; };
            t.hi = (uint16_t *)take(t.n * 2);
            t.res = take(mpo_res_bytes(t.n, bits, packed));
            t.grad = (i % 2) ? (const uint16_t *)take(t.n * 2) : nullptr;
            t.m = (float *)take(t.n * 4);
            t.v = (i % 3) ? (float *)take(t.n * 4) : nullptr;
            total += t.n;
        }
        for (uint64_t i = 0; i < nt; ++i) {
            const uint64_t ce = per_layer[ts[i].layer] >= (1ull << 26) ? 4096 : 1024;
            chunks += (ts[i].n + ce - 1) / ce;
        }
        mpo_plan *p = nullptr;
        const mpo_plan_opts mixed = {1ull << 26, 1};        /* host only; long chunks from 2^26 parameters on */
        CHECK(mpo_plan_create_opts(ts.data(), nt, &mixed, &p) == MPO_OK && p);
        CHECK(mpo_plan_num_params(p) == total && mpo_plan_num_chunks(p) == chunks);
        uint64_t seen = 0, covered = 0;
        for (uint64_t c = 0; c < chunks; ++c) {
            uint64_t tensor, first, count;
            CHECK(mpo_plan_get_chunk(p, c, &tensor, &first, &count) == MPO_OK && tensor < nt);
            CHECK(count >= 1 && first + count <= ts[tensor].n);
            covered += count;
            ++seen;
        }
        uint64_t tensor, first, count;
        CHECK(mpo_plan_get_chunk(p, chunks, &tensor, &first, &count) == MPO_ERR_INVALID_ARG);
        uint64_t by_layer = 0;
        for (int32_t l = 0; l < 9; ++l) {
            uint64_t fc, nc, ntl, np, ce;
            if (mpo_plan_layer_info(p, l, &fc, &nc, &ntl, &np, &ce) == MPO_OK) {
                CHECK(fc + nc <= chunks);
                CHECK(ce == (per_layer[l] >= (1ull << 26) ? 4096u : 1024u));
                by_layer += np;
            }
        }
        CHECK(by_layer == total && seen == chunks && covered == total);
        /* a host plan cannot be stepped */
        mpo_adam_cfg a = {1e-3, 0.9, 0.999, 1e-8, 0.0, 1, 1.0, MPO_BF16, MPO_BF16, MPO_ROUND_TRUNC, 0, 0.0};
        CHECK(mpo_adam_step(p, &a, 1, nullptr) == MPO_ERR_INVALID_ARG);
        CHECK(mpo_step_layer(p, 0, nullptr, 0, MPO_OPT_ADAM, &a, 1, nullptr) == MPO_ERR_INVALID_ARG);
        /* an overlap anywhere in the list is found */
        if (nt >= 2 && ts[0].n && ts[nt - 1].n) {
            std::vector<mpo_tensor> bad = ts;
            bad[nt - 1].m = (float *)((char *)bad[0].hi + 1);
            mpo_plan *q = nullptr;
            CHECK(mpo_plan_create_host(bad.data(), nt, &q) == MPO_ERR_ALIAS && !q);
        }
        CHECK(mpo_plan_destroy(p) == MPO_OK);
        ++plans;
    }
    /* argument checks of split / merge: refused before any launch */
    float *w = (float *)0x1000;
    uint16_t *hi = (uint16_t *)0x100000;
    void *res = (void *)0x200000;
    CHECK(mpo_split(w, hi, res, 10, (mpo_fmt)7, 0, 0, MPO_ROUND_TRUNC, 0, 0, nullptr) == MPO_ERR_INVALID_ARG);
    CHECK(mpo_split(w, hi, res, 10, MPO_FP16, 14, 0, MPO_ROUND_TRUNC, 0, 0, nullptr) == MPO_ERR_INVALID_ARG);
    CHECK(mpo_split(w, hi, res, 10, MPO_BF16, 16, 1, MPO_ROUND_TRUNC, 0, 0, nullptr) == MPO_ERR_INVALID_ARG);
    CHECK(mpo_split(w, hi, (char *)res + 4, 10, MPO_BF16, 12, 1, MPO_ROUND_TRUNC, 0, 0, nullptr) == MPO_ERR_INVALID_ARG);
    CHECK(mpo_split(w, (uint16_t *)w, res, 10, MPO_BF16, 0, 0, MPO_ROUND_TRUNC, 0, 0, nullptr) == MPO_ERR_ALIAS);
    CHECK(mpo_merge(hi, res, (float *)hi, 10, MPO_BF16, 0, 0, MPO_ROUND_TRUNC, nullptr) == MPO_ERR_ALIAS);
    CHECK(mpo_merge(hi, res, w, 10, MPO_BF16, 1, 1, MPO_ROUND_STOCHASTIC, nullptr) == MPO_ERR_INVALID_ARG);
    CHECK(mpo_split(nullptr, nullptr, nullptr, 0, MPO_BF16, 0, 0, MPO_ROUND_TRUNC, 0, 0, nullptr) == MPO_OK);
    CHECK(mpo_plan_destroy(nullptr) == MPO_OK);
    std::printf("%d plans\n", plans);
    return 0;
}
