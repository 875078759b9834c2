/*
 * mpo_adam_step_noalloc: the multi-tensor Adam step for callers that cannot allocate device
 * memory (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).
 *
 * mpo_adam_step reads a chunk table and tensor descriptors that mpo_plan_create put into device
 * memory it allocated.  Here the same table is built, on every call, by a small kernel into a
 * fixed array in the library's own device image (`scratch` below, 16 MiB + 64 KiB per GPU, held
 * until the process ends), from descriptors that travel in kernel arguments; then the same step
 * kernel runs over it.  Nothing is allocated or freed, on the host or on the device, and there is
 * no copy: the call only enqueues kernels on the caller's stream.
 *
 * All calls on one GPU share that GPU's array: two calls whose kernels may overlap in time (two
 * streams, two threads) race on it.  A call rewrites every entry it uses, so nothing needs
 * clearing between calls.
 */
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstring>

#include "mpo_internal.h"

namespace mpo {
namespace {

constexpr uint64_t kDescBytes = (uint64_t)MPO_NOALLOC_MAX_TENSORS * sizeof(TensorDesc);
constexpr uint64_t kScratchBytes = kDescBytes + (uint64_t)MPO_NOALLOC_MAX_CHUNKS * sizeof(Chunk);
static_assert(kDescBytes % 256 == 0, "the chunk table starts on a 256-byte boundary");

/* Descriptors, then the chunk table.  In host code this name is only a handle for
 * hipGetSymbolAddress: the device address is looked up once per device (scratch_of). */
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];

/* Address of `scratch` on the current device. */
hipError_t scratch_of(int device, void **out)
{
    void *p = g_scratch_ptr[device].load(std::memory_order_acquire);
    if (!p) {
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        g_scratch_ptr[device].store(p, std::memory_order_release); /* every thread finds the same address */
    }
    *out = p;
    return hipSuccess;
}

/* One batch of descriptors with the places of their chunks: at most 4 KiB of kernel arguments. */
constexpr uint32_t kBatch = 32;
struct TableBatch {
    TensorDesc desc[kBatch];
    uint32_t ragged_pos[kBatch];
    uint32_t full_pos[kBatch];
    uint32_t first;  /* index of desc[0] in the descriptor array */
    uint32_t count;
};
static_assert(sizeof(TableBatch) <= 4096 - 64, "fits the kernel argument segment beside the two pointers");

/* Workgroup b writes descriptor b of the batch and that tensor's chunk table entries: the ragged
 * chunk (if any) at ragged_pos, the full chunks from full_pos (same order as mpo_plan_create). */
__global__ void __launch_bounds__(256) build_table_kernel(TensorDesc *descs, Chunk *chunks, TableBatch b)
{
    const uint32_t j = blockIdx.x;
    if (j >= b.count) return;
    const TensorDesc d = b.desc[j];
    const uint32_t k = b.first + j;
    if (threadIdx.x == 0) descs[k] = d;
    const uint32_t rl = d.pad;                                   /* log2 of the rows per chunk */
    const uint64_t celems = (uint64_t)kRowElems << rl;
    const uint64_t num_full = d.n / celems;
    if (threadIdx.x == 0 && d.n % celems != 0) {
        Chunk c;
        c.tensor = k;
        c.where = (uint32_t)(num_full * celems / kRowElems) | (rl << kChunkStartBits);
        chunks[b.ragged_pos[j]] = c;
    }
    for (uint64_t i = threadIdx.x; i < num_full; i += blockDim.x) {
        Chunk c;
        c.tensor = k;
        c.where = (uint32_t)(i * celems / kRowElems) | (rl << kChunkStartBits);
        chunks[b.full_pos[j] + i] = c;
    }
}

} // namespace
} // namespace mpo

using namespace mpo;

extern "C" mpo_status mpo_adam_step_noalloc(const mpo_tensor *tensors, uint64_t nt, const mpo_adam_cfg *cfg,
                                            uint64_t step, void *hip_stream)
{
    StepLaunch L;
    mpo_status s = adam_scalars(cfg, step, L);
    if (s != MPO_OK) return s;
    if (nt > 0 && !tensors) return MPO_ERR_INVALID_ARG;
    if (nt > MPO_NOALLOC_MAX_TENSORS) return MPO_ERR_TOO_LARGE;

    /* validation as in mpo_plan_create, in fixed-size storage on the stack */
    Range ranges[5 * MPO_NOALLOC_MAX_TENSORS];
    uint64_t nr = 0;
    uint32_t res_slot = 0, max_bits = 0, min_bits = 16;
    bool any_bits = false;
    for (uint64_t i = 0; i < nt; ++i) {
        const mpo_tensor &t = tensors[i];
        s = check_tensor(t, res_slot, ranges, &nr);
        if (s != MPO_OK) return s;
        if (t.n == 0) continue;
        if (!t.grad || !t.m || !t.v) return MPO_ERR_INVALID_ARG;
        if (t.res_bits) {
            any_bits = true;
            max_bits = std::max(max_bits, (uint32_t)t.res_bits);
            min_bits = std::min(min_bits, (uint32_t)t.res_bits);
        }
    }
    if (has_conflict(ranges, nr)) return MPO_ERR_ALIAS;
    s = check_res_mode(res_slot, any_bits, min_bits, max_bits, L);
    if (s != MPO_OK) return s;

    /* layer order (stable): sort keys of (layer, position in the list) */
    uint64_t key[MPO_NOALLOC_MAX_TENSORS];
    for (uint64_t i = 0; i < nt; ++i) key[i] = ((uint64_t)(uint32_t)tensors[i].layer << 32) | i;
    std::sort(key, key + nt);
    TensorDesc descs[MPO_NOALLOC_MAX_TENSORS];
    int32_t layer[MPO_NOALLOC_MAX_TENSORS];
    TensorLayout lay[MPO_NOALLOC_MAX_TENSORS];
    for (uint64_t k = 0; k < nt; ++k) {
        const uint32_t i = (uint32_t)key[k];
        descs[k] = make_desc(tensors[i], i);
        layer[k] = tensors[i].layer;
    }
    const uint64_t total = layout_chunks(descs, layer, nt, kNoallocSmallLayerParams, lay);
    if (total == UINT64_MAX) return MPO_ERR_INVALID_ARG;
    if (total > MPO_NOALLOC_MAX_CHUNKS) return MPO_ERR_TOO_LARGE;
    if (total == 0) return MPO_OK;

    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev < 0 || dev >= kMaxDevices) return MPO_ERR_UNSUPPORTED;
    void *base = nullptr;
    e = scratch_of(dev, &base);
    if (e != hipSuccess) return hip_fail(e);
    TensorDesc *d_descs = static_cast<TensorDesc *>(base);
    Chunk *d_chunks = reinterpret_cast<Chunk *>(static_cast<unsigned char *>(base) + kDescBytes);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);

    for (uint64_t k0 = 0; k0 < nt; k0 += kBatch) {
        TableBatch b;
        std::memset(&b, 0, sizeof b);
        b.first = (uint32_t)k0;
        b.count = (uint32_t)std::min<uint64_t>(kBatch, nt - k0);
        for (uint32_t j = 0; j < b.count; ++j) {
            b.desc[j] = descs[k0 + j];
            b.desc[j].pad = lay[k0 + j].rows_log2;
            b.ragged_pos[j] = (uint32_t)lay[k0 + j].ragged_pos;
            b.full_pos[j] = (uint32_t)lay[k0 + j].full_pos;
        }
        (void)hipGetLastError();
        build_table_kernel<<<dim3(b.count), dim3(256), 0, stream>>>(d_descs, d_chunks, b);
        e = hipGetLastError();
        if (e != hipSuccess) return hip_fail(e);
    }
    L.descs = d_descs;
    L.chunks = d_chunks;
    L.first_chunk = 0;
    L.num_chunks = total;
    L.stream = stream;
    e = launch_step(L);
    return e == hipSuccess ? MPO_OK : hip_fail(e);
}
