/*
 * Bandwidth probe: the memory traffic of the split-precision step with the
 * arithmetic taken out.  A measuring aid for bench.py, not part of the method
 * and not part of libmpo.so.
 *
 * Per parameter it reads three 16-bit values and two fp32 values and writes two
 * 16-bit values and two fp32 values, in place, like the Adam step (26 bytes;
 * without `v`: 18 bytes, like SGD with momentum), with the same launch shape:
 * 256 lanes per 4096 consecutive parameters, each wavefront on a contiguous
 * quarter, 4 parameters per lane per row, all rows loaded before the first
 * store, non-temporal accesses.  What it reaches on a given GPU is the
 * practical ceiling for this access pattern there; the step kernel is judged
 * against it as well as against the published HBM peak.
 *
 * The values it writes are a cheap function of what it read, so that no load
 * or store can be dropped.  It overwrites the arrays it is given.
 */
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

#define PROBE_GLOBAL __attribute__((address_space(1)))
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kLanes = 256;
constexpr int kChunk = 4096;
constexpr int kRows = 4;

template <typename T> __device__ __forceinline__ T ld(const void *base, uint64_t byte_off)
{
    return __builtin_nontemporal_load((const PROBE_GLOBAL T *)((const PROBE_GLOBAL char *)base + byte_off));
}
template <typename T> __device__ __forceinline__ void st(void *base, uint64_t byte_off, T x)
{
    __builtin_nontemporal_store(x, (PROBE_GLOBAL T *)((PROBE_GLOBAL char *)base + byte_off));
}

template <bool WITH_V>
__global__ __launch_bounds__(kLanes) void probe_kernel(void *hi, void *res, const void *grad, void *m, void *v)
{
    const uint32_t t = threadIdx.x;
    const uint64_t chunk0 = static_cast<uint64_t>(blockIdx.x) * kChunk;
    u32x2 h[kRows], r[kRows], g[kRows];
    f32x4 a[kRows], b[kRows];
#pragma unroll
    for (int k = 0; k < kRows; ++k) {
        const uint64_t e = chunk0 + (t / 64) * 1024 + k * 256 + (t % 64) * 4;
        h[k] = ld<u32x2>(hi, e * 2);
        r[k] = ld<u32x2>(res, e * 2);
        g[k] = ld<u32x2>(grad, e * 2);
        a[k] = ld<f32x4>(m, e * 4);
        if (WITH_V) b[k] = ld<f32x4>(v, e * 4);
    }
#pragma unroll
    for (int k = 0; k < kRows; ++k) {
        const uint64_t e = chunk0 + (t / 64) * 1024 + k * 256 + (t % 64) * 4;
        st<u32x2>(hi, e * 2, h[k] ^ g[k]);
        st<u32x2>(res, e * 2, ~(r[k] ^ g[k]));
        st<f32x4>(m, e * 4, a[k] + 1.0f);
        if (WITH_V) st<f32x4>(v, e * 4, b[k] + 2.0f);
    }
}

} // namespace

/* Runs the probe over the first n - n % 4096 parameters of the arrays (device
 * pointers, 16-byte aligned; hi, res, grad: 2 bytes per parameter; m, v: 4).
 * v may be null: then the SGD-shaped traffic (18 bytes per parameter).  Returns
 * 0, or -1 for a bad argument, or the hipError_t of a failed launch.  The launch
 * is asynchronous on `stream` (a hipStream_t, may be null). */
extern "C" int mpo_probe_stream(void *hi, void *res, const void *grad, void *m, void *v, long long n, void *stream)
{
    if (!hi || !res || !grad || !m || n < 0) return -1;
    const uintptr_t bits = reinterpret_cast<uintptr_t>(hi) | reinterpret_cast<uintptr_t>(res) |
                           reinterpret_cast<uintptr_t>(grad) | reinterpret_cast<uintptr_t>(m) |
                           reinterpret_cast<uintptr_t>(v);
    if (bits & 15) return -1;
    const long long chunks = n / kChunk;
    if (chunks == 0) return 0;
    if (chunks > 0x7fffffffLL) return -1;
    hipStream_t s = static_cast<hipStream_t>(stream);
    (void)hipGetLastError(); /* an error an earlier, unrelated runtime call left on this thread is not ours */
    if (v)
        hipLaunchKernelGGL(probe_kernel<true>, dim3(static_cast<unsigned>(chunks)), dim3(kLanes), 0, s, hi, res, grad, m, v);
    else
        hipLaunchKernelGGL(probe_kernel<false>, dim3(static_cast<unsigned>(chunks)), dim3(kLanes), 0, s, hi, res, grad, m, v);
    return static_cast<int>(hipGetLastError());
}
