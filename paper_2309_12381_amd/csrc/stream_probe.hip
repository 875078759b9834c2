/*
 * Bandwidth probe: the memory traffic of the split-precision step with the
 * arithmetic taken out, and plain read / write streams.  A measuring aid for
 * bench.py and for the placement of the state arrays, not part of the method
 * and not part of libmpo.so.
 *
 * mpo_probe_stream  Per parameter it reads three 16-bit values and two fp32
 *   values and writes two 16-bit values and two fp32 values, in place, like the
 *   Adam step (26 bytes; without `v`: 18 bytes, like SGD with momentum), with the
 *   same launch shape: 256 lanes per 4096 consecutive parameters, each wavefront
 *   on a contiguous quarter, 4 parameters per lane per row, all rows loaded
 *   before the first store, non-temporal accesses.  What it reaches on a given
 *   GPU is the practical ceiling for this access pattern there; the step kernel
 *   is judged against it as well as against the published HBM peak.
 * mpo_probe_variant  The same traffic with ONE choice of the launch shape changed
 *   (lane width, cache policy, rows in flight, chunk length, row order, persistent
 *   workgroups, software pipelining, workgroup size, chunk order): the measurements
 *   behind the shape the step kernel has.
 * mpo_probe_plain   k equal arrays walked in lock step, read only, written only,
 *   or read and written back in place: what the memory system gives each kind of
 *   traffic, for arrays placed in one or in several parts of the device memory.
 *
 * The values written are a cheap function of what was read, so that no load or
 * store can be dropped.  The probes overwrite the arrays they are given.
 */
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mpo_probe.h"

namespace {

#define PROBE_GLOBAL __attribute__((address_space(1)))
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kLanes = 256;
constexpr int kChunk = 4096;
constexpr int kRows = 4;

template <bool NT = true, typename T> __device__ __forceinline__ T ldp(const void *base, uint64_t byte_off)
{
    const PROBE_GLOBAL T *p = (const PROBE_GLOBAL T *)((const PROBE_GLOBAL char *)base + byte_off);
    return NT ? __builtin_nontemporal_load(p) : *p;
}
template <bool NT = true, typename T> __device__ __forceinline__ void stp(void *base, uint64_t byte_off, T x)
{
    PROBE_GLOBAL T *p = (PROBE_GLOBAL T *)((PROBE_GLOBAL char *)base + byte_off);
    if (NT) __builtin_nontemporal_store(x, p);
    else *p = x;
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
        h[k] = ldp<true, u32x2>(hi, e * 2);
        r[k] = ldp<true, u32x2>(res, e * 2);
        g[k] = ldp<true, u32x2>(grad, e * 2);
        a[k] = ldp<true, f32x4>(m, e * 4);
        if (WITH_V) b[k] = ldp<true, f32x4>(v, e * 4);
    }
#pragma unroll
    for (int k = 0; k < kRows; ++k) {
        const uint64_t e = chunk0 + (t / 64) * 1024 + k * 256 + (t % 64) * 4;
        stp<true, u32x2>(hi, e * 2, h[k] ^ g[k]);
        stp<true, u32x2>(res, e * 2, ~(r[k] ^ g[k]));
        stp<true, f32x4>(m, e * 4, a[k] + 1.0f);
        if (WITH_V) stp<true, f32x4>(v, e * 4, b[k] + 2.0f);
    }
}

/* ---- variants of the launch shape ------------------------------------------------------------
 * BLK lanes; a chunk is BLK * 4 * ROWS parameters (EPL = 4) or BLK * 8 * ROWS (EPL = 8); FLY rows are
 * requested before the first is stored; WAVEC: each wavefront owns a contiguous share of the chunk
 * (else rows are interleaved over the wavefronts); PERSIST: gridDim workgroups stride over the chunks;
 * PIPE: the next chunk's first rows are requested before this chunk's last stores (persistent walk over
 * PIPE adjacent chunks per workgroup); XCD: workgroup b takes chunk (b % 8) * (n / 8) + b / 8, so that
 * each of the 8 dies walks an eighth of the arrays of its own. */
struct Row4 { u32x2 h, r, g; f32x4 a, b; };
struct Row8 { u32x4 h, r, g; f32x4 a0, a1, b0, b1; };

template <bool NTL> __device__ __forceinline__ void load_row(Row4 &x, const void *hi, const void *res, const void *grad,
                                                            const void *m, const void *v, uint64_t e)
{
    x.h = ldp<NTL, u32x2>(hi, e * 2); x.r = ldp<NTL, u32x2>(res, e * 2); x.g = ldp<NTL, u32x2>(grad, e * 2);
    x.a = ldp<NTL, f32x4>(m, e * 4); x.b = ldp<NTL, f32x4>(v, e * 4);
}
template <bool NTS, bool NTHI> __device__ __forceinline__ void store_row(const Row4 &x, void *hi, void *res, void *m, void *v, uint64_t e)
{
    stp<NTHI, u32x2>(hi, e * 2, x.h ^ x.g); stp<NTS, u32x2>(res, e * 2, ~(x.r ^ x.g));
    stp<NTS, f32x4>(m, e * 4, x.a + 1.0f); stp<NTS, f32x4>(v, e * 4, x.b + 2.0f);
}
template <bool NTL> __device__ __forceinline__ void load_row(Row8 &x, const void *hi, const void *res, const void *grad,
                                                            const void *m, const void *v, uint64_t e)
{
    x.h = ldp<NTL, u32x4>(hi, e * 2); x.r = ldp<NTL, u32x4>(res, e * 2); x.g = ldp<NTL, u32x4>(grad, e * 2);
    x.a0 = ldp<NTL, f32x4>(m, e * 4); x.a1 = ldp<NTL, f32x4>(m, e * 4 + 16);
    x.b0 = ldp<NTL, f32x4>(v, e * 4); x.b1 = ldp<NTL, f32x4>(v, e * 4 + 16);
}
template <bool NTS, bool NTHI> __device__ __forceinline__ void store_row(const Row8 &x, void *hi, void *res, void *m, void *v, uint64_t e)
{
    stp<NTHI, u32x4>(hi, e * 2, x.h ^ x.g); stp<NTS, u32x4>(res, e * 2, ~(x.r ^ x.g));
    stp<NTS, f32x4>(m, e * 4, x.a0 + 1.0f); stp<NTS, f32x4>(m, e * 4 + 16, x.a1 + 1.0f);
    stp<NTS, f32x4>(v, e * 4, x.b0 + 2.0f); stp<NTS, f32x4>(v, e * 4 + 16, x.b1 + 2.0f);
}
template <int EPL> struct RowOf { typedef Row4 T; };
template <> struct RowOf<8> { typedef Row8 T; };

template <int BLK, int EPL, int ROWS, int FLY, bool NTL, bool NTS, bool NTHI, bool WAVEC, bool PERSIST, int PIPE, bool XCD>
__global__ __launch_bounds__(BLK) void variant_kernel(void *hi, void *res, const void *grad, void *m, void *v, uint64_t nchunks)
{
    typedef typename RowOf<EPL>::T Row;
    constexpr uint32_t CH = BLK * EPL * ROWS;
    static_assert(ROWS % FLY == 0, "rows go in batches");
    const uint32_t t = threadIdx.x;
    auto eoff = [&](uint64_t chunk, int r) -> uint64_t {
        const uint32_t in = WAVEC ? (t / 64) * (CH / (BLK / 64)) + r * (64 * EPL) + (t % 64) * EPL : (r * BLK + t) * EPL;
        return chunk * CH + in;
    };
    if (PIPE > 1) {
        /* PIPE adjacent chunks per workgroup, two row buffers: chunk c+1 is requested before chunk c is stored */
        static_assert(PIPE == 1 || (ROWS == FLY), "pipelining keeps whole chunks in flight");
        Row x[2][ROWS];
        const uint64_t c0 = static_cast<uint64_t>(blockIdx.x) * PIPE;
#pragma unroll
        for (int r = 0; r < ROWS; ++r) load_row<NTL>(x[0][r], hi, res, grad, m, v, eoff(c0, r));
#pragma unroll
        for (int c = 0; c < PIPE; ++c) {
            if (c + 1 < PIPE) {
#pragma unroll
                for (int r = 0; r < ROWS; ++r) load_row<NTL>(x[(c + 1) & 1][r], hi, res, grad, m, v, eoff(c0 + c + 1, r));
            }
#pragma unroll
            for (int r = 0; r < ROWS; ++r) store_row<NTS, NTHI>(x[c & 1][r], hi, res, m, v, eoff(c0 + c, r));
        }
        return;
    }
    for (uint64_t b = blockIdx.x; b < nchunks; b += PERSIST ? gridDim.x : nchunks) {
        uint64_t chunk = b;
        if (XCD) {
            const uint64_t per = nchunks / 8;
            if (b < per * 8) chunk = (b % 8) * per + b / 8;
        }
#pragma unroll 1
        for (int r0 = 0; r0 < ROWS; r0 += FLY) {
            Row x[FLY];
#pragma unroll
            for (int r = 0; r < FLY; ++r) load_row<NTL>(x[r], hi, res, grad, m, v, eoff(chunk, r0 + r));
#pragma unroll
            for (int r = 0; r < FLY; ++r) store_row<NTS, NTHI>(x[r], hi, res, m, v, eoff(chunk, r0 + r));
        }
    }
}

struct Variant {
    const char *name;
    uint32_t chunk;      /* parameters per chunk                                     */
    uint32_t per_group;  /* chunks per workgroup (pipelined), else 1                 */
    uint32_t block;
    int persist;         /* workgroups per compute unit of a persistent grid, else 0 */
    void (*kernel)(void *, void *, const void *, void *, void *, uint64_t);
};

#define V(BLK, EPL, ROWS, FLY, NTL, NTS, NTHI, WAVEC, PERSIST, PIPE, XCD) \
    (BLK) * (EPL) * (ROWS), (PIPE), (BLK), ((PERSIST) ? 8 : 0), variant_kernel<BLK, EPL, ROWS, FLY, NTL, NTS, NTHI, WAVEC, PERSIST, PIPE, XCD>

const Variant kVariants[] = {
    {"256 lanes, 4 parameters per lane, chunk of 4096 parameters with its 4 rows in flight, wavefront-contiguous, non-temporal",
     V(256, 4, 4, 4, true, true, true, true, false, 1, false)},
    {"8 parameters per lane (128-bit 16-bit accesses, two 128-bit fp32 accesses 32 bytes apart)",
     V(256, 8, 2, 2, true, true, true, true, false, 1, false)},
    {"default cache policy for loads and stores", V(256, 4, 4, 4, false, false, false, true, false, 1, false)},
    {"default cache policy for stores only", V(256, 4, 4, 4, true, false, false, true, false, 1, false)},
    {"default cache policy for loads only", V(256, 4, 4, 4, false, true, true, true, false, 1, false)},
    {"default cache policy for the stores of hi only", V(256, 4, 4, 4, true, true, false, true, false, 1, false)},
    {"chunk of 4096 parameters, one row in flight (the step kernel's long chunks)", V(256, 4, 4, 1, true, true, true, true, false, 1, false)},
    {"two rows in flight", V(256, 4, 4, 2, true, true, true, true, false, 1, false)},
    {"chunk of 1024 parameters, one row (the step kernel's default)", V(256, 4, 1, 1, true, true, true, true, false, 1, false)},
    {"chunk of 2048 parameters", V(256, 4, 2, 2, true, true, true, true, false, 1, false)},
    {"chunk of 16384 parameters, 4 rows in flight", V(256, 4, 16, 4, true, true, true, true, false, 1, false)},
    {"rows interleaved over the four wavefronts", V(256, 4, 4, 4, true, true, true, false, false, 1, false)},
    {"persistent workgroups (8 per compute unit) striding over the chunks", V(256, 4, 4, 4, true, true, true, true, true, 1, false)},
    {"two adjacent chunks per workgroup, software pipelined", V(256, 4, 4, 4, true, true, true, true, false, 2, false)},
    {"four adjacent chunks per workgroup, software pipelined", V(256, 4, 4, 4, true, true, true, true, false, 4, false)},
    {"512 lanes per workgroup (chunk of 8192)", V(512, 4, 4, 4, true, true, true, true, false, 1, false)},
    {"1024 lanes per workgroup (chunk of 16384)", V(1024, 4, 4, 4, true, true, true, true, false, 1, false)},
    {"64 lanes per workgroup (chunk of 1024)", V(64, 4, 4, 4, true, true, true, true, false, 1, false)},
    {"each of the 8 dies walks a contiguous eighth of the arrays", V(256, 4, 4, 4, true, true, true, true, false, 1, true)},
};
#undef V
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);

/* ---- plain streams: K arrays in lock step ---------------------------------------------------- */
constexpr int kMaxPlain = 8;
struct PlainArgs { void *p[kMaxPlain]; };

/* MODE 0: read, 1: write, 2: read and write back.  A workgroup handles 16 KiB of each array. */
template <int MODE>
__global__ __launch_bounds__(kLanes) void plain_kernel(PlainArgs a, int k, float *sink)
{
    const uint32_t t = threadIdx.x;
    const uint64_t base = static_cast<uint64_t>(blockIdx.x) * 16384;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int j = 0; j < k; ++j) {
        f32x4 x[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const uint64_t off = base + (t / 64) * 4096 + r * 1024 + (t % 64) * 16;
            if (MODE != 1) x[r] = ldp<true, f32x4>(a.p[j], off);
            else x[r] = f32x4{1.f, 2.f, 3.f, (float)r};
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const uint64_t off = base + (t / 64) * 4096 + r * 1024 + (t % 64) * 16;
            if (MODE != 0) stp<true, f32x4>(a.p[j], off, x[r] + 1.0f);
            else acc += x[r];
        }
    }
    if (MODE == 0 && acc[0] + acc[1] + acc[2] + acc[3] == 123.456f) *sink = 1.0f;   /* keeps the loads */
}

inline bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

} // namespace

/* Runs the probe over the first n - n % 4096 parameters of the arrays (device
 * pointers, 16-byte aligned; hi, res, grad: 2 bytes per parameter; m, v: 4).
 * v may be null: then the SGD-shaped traffic (18 bytes per parameter).  Returns
 * 0, or -1 for a bad argument, or the hipError_t of a failed launch.  The launch
 * is asynchronous on `stream` (a hipStream_t, may be null). */
extern "C" int mpo_probe_stream(void *hi, void *res, const void *grad, void *m, void *v, long long n, void *stream)
{
    if (!hi || !res || !grad || !m || n < 0) return -1;
    if (misaligned(hi) || misaligned(res) || misaligned(grad) || misaligned(m) || misaligned(v)) return -1;
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

extern "C" int mpo_probe_num_variants(void) { return kNumVariants; }
extern "C" const char *mpo_probe_variant_name(int variant)
{
    return (variant >= 0 && variant < kNumVariants) ? kVariants[variant].name : nullptr;
}

/* The Adam-shaped traffic (all five arrays required) in variant `variant` of the launch shape over the first
 * n - n % 131072 parameters (every variant's chunk and group size divides that, and so does 8 times it).
 * `compute_units` sizes the grid of the persistent variant.  Same return values as mpo_probe_stream. */
extern "C" int mpo_probe_variant(int variant, void *hi, void *res, const void *grad, void *m, void *v, long long n,
                                 int compute_units, void *stream)
{
    if (variant < 0 || variant >= kNumVariants || !hi || !res || !grad || !m || !v || n < 0 || compute_units < 1) return -1;
    if (misaligned(hi) || misaligned(res) || misaligned(grad) || misaligned(m) || misaligned(v)) return -1;
    const Variant &q = kVariants[variant];
    const uint64_t use = static_cast<uint64_t>(n) / 131072u * 131072u;
    const uint64_t nchunks = use / q.chunk;
    if (nchunks == 0) return 0;
    uint64_t grid = nchunks / q.per_group;
    if (q.persist) grid = static_cast<uint64_t>(q.persist) * compute_units < nchunks ? static_cast<uint64_t>(q.persist) * compute_units : nchunks;
    if (grid > 0x7fffffffULL) return -1;
    (void)hipGetLastError();
    hipLaunchKernelGGL(q.kernel, dim3(static_cast<unsigned>(grid)), dim3(q.block), 0, static_cast<hipStream_t>(stream), hi, res,
                       grad, m, v, nchunks);
    return static_cast<int>(hipGetLastError());
}

/* k (1..8) arrays of `bytes` bytes each (the first bytes - bytes % 16384 are used), walked in lock step:
 * mode 0 reads them, 1 writes them, 2 reads them and writes them back.  `sink`: 4 bytes of device memory
 * (only written if the data happen to add up to one particular value).  Same return values as above. */
extern "C" int mpo_probe_plain(int mode, void *const *arrays, int k, unsigned long long bytes, void *sink, void *stream)
{
    if (mode < 0 || mode > 2 || !arrays || k < 1 || k > kMaxPlain || !sink) return -1;
    PlainArgs a;
    for (int j = 0; j < kMaxPlain; ++j) a.p[j] = j < k ? arrays[j] : nullptr;
    for (int j = 0; j < k; ++j)
        if (!a.p[j] || misaligned(a.p[j])) return -1;
    const unsigned long long groups = bytes / 16384u;
    if (groups == 0) return 0;
    if (groups > 0x7fffffffULL) return -1;
    hipStream_t s = static_cast<hipStream_t>(stream);
    (void)hipGetLastError();
    if (mode == 0) hipLaunchKernelGGL(plain_kernel<0>, dim3((unsigned)groups), dim3(kLanes), 0, s, a, k, (float *)sink);
    else if (mode == 1) hipLaunchKernelGGL(plain_kernel<1>, dim3((unsigned)groups), dim3(kLanes), 0, s, a, k, (float *)sink);
    else hipLaunchKernelGGL(plain_kernel<2>, dim3((unsigned)groups), dim3(kLanes), 0, s, a, k, (float *)sink);
    return static_cast<int>(hipGetLastError());
}
