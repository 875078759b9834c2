/*
 * mpo_place_second: where to put res, v and the gradient buffer in the device memory, given hi
 * and m, decided by measurement with the bandwidth probe (see include/mpo_probe.h).  The native
 * counterpart of placement.py, for callers of the C interface; part of libmpo_probe.so.
 */
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>

#include "mpo_probe.h"

namespace {

constexpr uint64_t kGiB = 1ull << 30;
constexpr uint64_t kTestParams = 1ull << 26;      /* parameters per probe launch: 1.75 GB of traffic, about 0.3 ms */
constexpr uint64_t kN2 = 2 * kTestParams;         /* bytes of a window of a 16-bit array */
constexpr uint64_t kN4 = 4 * kTestParams;         /* bytes of a window of an fp32 array  */
constexpr uint64_t kStride = 16 * kGiB;           /* successive candidates start at least this far apart */
constexpr uint64_t kReserve = 4 * kGiB;           /* never take the last of the device memory */
constexpr int kMaxTries = 8;
constexpr int kPositions = 4;
constexpr double kGain = 1.07, kFloor = 1.04;

/* byte offset of a window of `len` bytes at relative position k / (kPositions - 1) of an array of `total` bytes */
uint64_t window(uint64_t total, uint64_t len, int k)
{
    return ((total - len) / (kPositions - 1) * (uint64_t)k) & ~4095ull;
}

/* GB/s of the probe over five windows: median of 3 timed launches after one untimed; < 0: a HIP error (in *err) */
double rate(void *hi, void *res, const void *grad, void *m, void *v, hipStream_t s, hipEvent_t e0, hipEvent_t e1, int *err)
{
    int rc = mpo_probe_stream(hi, res, grad, m, v, (long long)kTestParams, s);
    if (rc != 0) { *err = rc; return -1.0; }
    double r[3];
    for (int i = 0; i < 3; ++i) {
        hipError_t e = hipEventRecord(e0, s);
        if (e == hipSuccess) {
            rc = mpo_probe_stream(hi, res, grad, m, v, (long long)kTestParams, s);
            if (rc != 0) { *err = rc; return -1.0; }
            e = hipEventRecord(e1, s);
        }
        if (e == hipSuccess) e = hipEventSynchronize(e1);
        float ms = 0.0f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
        if (e != hipSuccess) { *err = (int)e; return -1.0; }
        r[i] = 26.0 * (double)kTestParams / ((double)ms * 1e6);
    }
    std::sort(r, r + 3);
    return r[1];
}

bool good(const double *r, const double *ref)
{
    double sr = 0.0, sref = 0.0;
    for (int k = 0; k < kPositions; ++k) {
        if (r[k] < kFloor * ref[k]) return false;
        sr += r[k];
        sref += ref[k];
    }
    return sr >= kGain * sref;
}

} // namespace

extern "C" int mpo_place_free(void *block)
{
    return block ? (int)hipFree(block) : 0;
}

extern "C" int mpo_place_second(void *hi, uint64_t hi_bytes, void *m, uint64_t m_bytes, uint64_t res_bytes, uint64_t v_bytes,
                                uint64_t grad_bytes, uint64_t max_transient_bytes, int keep_hi, void **block,
                                mpo_place_report *report, void *stream)
{
    if (!block || !report || !hi || !m || res_bytes == 0 || v_bytes == 0) return -1;
    if (res_bytes > (1ull << 46) || v_bytes > (1ull << 46) || grad_bytes > (1ull << 46)) return -1;
    *block = nullptr;
    std::memset(report, 0, sizeof *report);
    const uint64_t v_off = (res_bytes + 255) / 256 * 256, g_off = v_off + (v_bytes + 255) / 256 * 256;
    const uint64_t need_bytes = g_off + grad_bytes;
    report->v_offset = v_off;
    report->grad_offset = g_off;
    report->block_bytes = need_bytes;
    hipStream_t s = static_cast<hipStream_t>(stream);
    size_t free0 = 0, total = 0;
    hipError_t e = hipMemGetInfo(&free0, &total);
    if (e != hipSuccess) return (int)e;
    if (max_transient_bytes == 0) max_transient_bytes = free0 / 2;
    report->max_transient_bytes = max_transient_bytes;

    if (hi_bytes < kN2 || m_bytes < 6 * kN2 || res_bytes < kN2 || v_bytes < kN4) {
        /* too small to probe: a plain allocation */
        e = hipMalloc(block, need_bytes);
        report->candidates = e == hipSuccess ? 1 : 0;
        return (int)e;
    }

    char *const hi_c = static_cast<char *>(hi), *const m_c = static_cast<char *>(m);
    void *cand[kMaxTries] = {}, *filler[kMaxTries] = {};
    double rates[kMaxTries][kPositions] = {};
    void *saved = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int err = 0, n = 0;
    uint64_t held = 0;

    e = hipEventCreate(&e0);
    if (e == hipSuccess) e = hipEventCreate(&e1);
    if (e == hipSuccess && keep_hi) {
        e = hipMalloc(&saved, kPositions * kN2);
        for (int k = 0; e == hipSuccess && k < kPositions; ++k)
            e = hipMemcpyAsync(static_cast<char *>(saved) + k * kN2, hi_c + window(hi_bytes, kN2, k), kN2, hipMemcpyDeviceToDevice, s);
    }
    if (e != hipSuccess) err = (int)e;

    /* reference: the same hi windows the candidates are measured with, everything else inside m, that is
     * certainly close together (hi and m are taken to lie in one region) */
    for (int k = 0; !err && k < kPositions; ++k) {
        char *w = m_c + window(m_bytes, 6 * kN2, k);
        report->one_region_GBps[k] = rate(hi_c + window(hi_bytes, kN2, k), w, w + kN2, w + 2 * kN2, w + 2 * kN2 + kN4, s, e0, e1, &err);
    }

    while (!err && n < kMaxTries) {
        const uint64_t gap = (n > 0 && need_bytes < kStride) ? kStride - need_bytes : 0;
        size_t fr = 0;
        e = hipMemGetInfo(&fr, &total);
        if (e != hipSuccess) { err = (int)e; break; }
        if (fr < need_bytes + gap + kReserve) break;
        if (n > 0 && held + gap > max_transient_bytes) break;      /* one more candidate would hold too much */
        if (gap) {
            e = hipMalloc(&filler[n], gap);
            if (e != hipSuccess) { (void)hipGetLastError(); filler[n] = nullptr; break; }
        }
        e = hipMalloc(&cand[n], need_bytes);
        if (e != hipSuccess) { (void)hipGetLastError(); cand[n] = nullptr; break; }
        held += need_bytes + gap;
        char *b = static_cast<char *>(cand[n]);
        for (int k = 0; !err && k < kPositions; ++k) {
            /* no gradient part to read from: a part of m away from the m window (reading the res window twice
             * would save a sixth of the reads and make every candidate look better than it is) */
            const char *g = grad_bytes >= kN2 ? b + g_off : m_c + window(m_bytes, kN2, (k + 2) % kPositions);
            rates[n][k] = rate(hi_c + window(hi_bytes, kN2, k), b + window(res_bytes, kN2, k), g, m_c + window(m_bytes, kN4, k),
                               b + v_off + window(v_bytes, kN4, k), s, e0, e1, &err);
        }
        ++n;
        if (!err && good(rates[n - 1], report->one_region_GBps)) break;
    }

    int best = -1;
    if (!err && n > 0) {
        double top = -1.0;
        for (int i = 0; i < n; ++i) {
            double sum = 0.0;
            for (int k = 0; k < kPositions; ++k) sum += rates[i][k];
            if (sum > top) { top = sum; best = i; }
        }
    }
    if (saved) {
        for (int k = 0; k < kPositions; ++k)
            (void)hipMemcpyAsync(hi_c + window(hi_bytes, kN2, k), static_cast<char *>(saved) + k * kN2, kN2, hipMemcpyDeviceToDevice, s);
    }
    (void)hipStreamSynchronize(s);
    for (int i = 0; i < kMaxTries; ++i) {
        if (cand[i] && i != best) (void)hipFree(cand[i]);
        if (filler[i]) (void)hipFree(filler[i]);
    }
    if (saved) (void)hipFree(saved);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (err) {
        if (best >= 0) (void)hipFree(cand[best]);
        return err;
    }
    if (best < 0) {
        /* no memory to search with: a plain allocation, or its error */
        e = hipMalloc(block, need_bytes);
        report->candidates = e == hipSuccess ? 1 : 0;
        return (int)e;
    }
    *block = cand[best];
    report->candidates = n;
    report->chosen = best;
    report->split = good(rates[best], report->one_region_GBps) ? 1 : 0;
    for (int k = 0; k < kPositions; ++k) report->chosen_GBps[k] = rates[best][k];
    report->peak_transient_bytes = held - need_bytes;
    return 0;
}
