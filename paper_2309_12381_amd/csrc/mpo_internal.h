/* Shared between the host side (mpo_host.cpp) and the kernels (mpo_kernels.hip)
 * of libmpo.  Not part of the public interface (see include/mpo.h). */
#ifndef MPO_INTERNAL_H
#define MPO_INTERNAL_H

#include <hip/hip_runtime_api.h>
#include <stdint.h>

#include "mpo.h"

namespace mpo {

/* One workgroup (256 lanes = 4 wavefronts of 64) owns one chunk.  A chunk is 1, 2 or 4 "rows" of
 * 1024 consecutive parameters (4 per lane).  Measured on MI355X, one row per workgroup is the
 * faster cut for 16-bit and byte residuals: +5 % on a list of 25.6 M parameters (four times as
 * many workgroups to fill 256 compute units), and on layers of 2 * 10^8 parameters it measures the
 * same as 4 rows walked one after the other by one workgroup (27.20 against 27.25 ms per step of
 * the 7B-shaped set), at the price of a chunk table of 8 bytes per 1024 parameters instead of per
 * 4096.  The length is chosen per layer by a threshold the caller may set.  A row is requested,
 * updated and stored before the next is touched: with one row in flight per wavefront every
 * variant of the kernel fits 7 or 8 wavefronts per SIMD, which hide the latency. */
constexpr uint32_t kBlock = 256;
constexpr uint32_t kRowElems = 1024;                 /* kBlock lanes x 4 parameters               */
constexpr uint32_t kChunkElems = 4096;               /* the longest chunk: 4 rows                 */
constexpr uint64_t kSmallLayerParams = UINT64_MAX;   /* plans: layers below this are cut into single rows (default: all) */
constexpr uint64_t kPlanesSmallLayerParams = 1ull << 26; /* packed planes: the per-workgroup set-up (four plane addresses) and the
                                                           * sub-dword accesses weigh more, and long chunks measured 3 % (fp16, 13
                                                           * bits) faster on large layers, at -1.7 % for bf16 with 12 bits */
constexpr uint64_t kNoallocSmallLayerParams = 1ull << 26; /* the fixed table of mpo_adam_step_noalloc: long chunks
                                                            * for large layers, so that 2^21 entries go further */

/* Bits of TensorDesc::flags. */
constexpr uint32_t kStateAligned = 1u; /* hi, res, m, v all 16-byte aligned          */
constexpr uint32_t kGradAligned = 2u;  /* the plan's own grad pointer 16-byte aligned */

struct TensorDesc {
    uint16_t *hi;
    void *res;           /* uint8_t per parameter when 1 <= res_bits <= 8, else uint16_t */
    const uint16_t *grad;
    float *m;
    float *v;
    uint64_t n;
    uint32_t flags;
    uint32_t res_bits;   /* extra bits kept, 0 = all (Section 3.1) */
    uint32_t tensor_id;  /* index in the caller's list: selects the random stream */
    uint32_t pad;
};
static_assert(sizeof(TensorDesc) == 64, "descriptor layout is read by the kernels");

/* Chunk table entry: which tensor (index into the layer-ordered descriptor array) and which part
 * of it.  `where` holds the chunk's first parameter in units of kRowElems in its low 30 bits and
 * log2 of the chunk's length in rows in its top 2 bits. */
struct Chunk {
    uint32_t tensor;
    uint32_t where;
};
constexpr uint32_t kChunkStartBits = 30;
constexpr uint32_t kChunkStartMask = (1u << kChunkStartBits) - 1u;
constexpr uint64_t kMaxTensorElems = (uint64_t)kRowElems << kChunkStartBits; /* 2^40 */

inline uint32_t chunk_where(uint64_t first_elem, uint32_t rows_log2)
{
    return (uint32_t)(first_elem / kRowElems) | (rows_log2 << kChunkStartBits);
}

/* How one layer's tensors are cut (Section 3.1, "Fused" optimizer: one launch over many tensors).
 * All chunks of a layer have the same length; in the table the layer's ragged chunks (the last,
 * shorter chunk of a tensor) come first, so that they run beside full chunks instead of at the
 * end of the launch, then the full chunks tensor by tensor. */
inline uint32_t layer_rows_log2(uint64_t layer_params, uint64_t small_layer_params)
{
    return layer_params < small_layer_params ? 0u : 2u;
}

/* Scalars of one step, already rounded to fp32 on the host (Section 3.1:
 * the classic optimizers).  Adam uses all but LR/MU; SGD uses LR, MU, WD, IS. */
struct StepScalars {
    float B1, B2, O1, O2; /* beta1, beta2, 1-beta1, 1-beta2                      */
    float SS, SQ, EPS;    /* lr/(1-beta1^t), sqrt(1-beta2^t), eps                */
    float DEC, WD, IS;    /* 1-lr*wd, wd, 1/loss_scale                           */
    float LR, MU;         /* SGD learning rate and momentum                      */
    float CLIP;           /* gradient clamp bound, +infinity when off (Section 4.1) */
    /* rounding of the 16-bit value (Section 3.1, last paragraph) */
    uint32_t round;       /* mpo_round                                           */
    uint32_t seed_lo, seed_hi, step32;
};

/* Per-call gradient pointers for one layer (Section 3.2), passed by value to the kernels that are
 * compiled for them; launches that use the plan's own pointers carry NoOverride instead. */
struct GradOverride {
    const uint16_t *ptr[MPO_MAX_LAYER_GRADS];
    uint64_t misaligned; /* bit i set: ptr[i] is not 16-byte aligned            */
    uint32_t first;      /* descriptor index of the layer's first tensor        */
    uint32_t pad;
};
struct NoOverride {
    uint32_t unused;
};

enum Decay { kNoDecay = 0, kDecoupled = 1, kL2 = 2 };

/* How the residual is stored (Section 3.1: all extra bits, or only the leading E). */
enum ResMode {
    kResFull = 0,    /* uint16_t, every extra bit kept: no shifting                  */
    kResPartial = 1, /* uint16_t, some tensor keeps fewer bits: shift per descriptor  */
    kResByte = 2,    /* uint8_t (1..8 bits kept)                                      */
    kResPlanes = 3   /* packed bit planes of 8, 4, 2 and 1 bits (Figure 1)             */
};

inline uint64_t round16(uint64_t x) { return (x + 15u) / 16u * 16u; }

/* Bytes of the residual buffer of one tensor. */
inline uint64_t res_bytes(uint64_t n, int res_bits, int packed)
{
    if (!packed) return n * ((res_bits >= 1 && res_bits <= 8) ? 1u : 2u);
    uint64_t b = 0;
    if (res_bits & 8) b += round16(n);
    if (res_bits & 4) b += round16((n + 1) / 2);
    if (res_bits & 2) b += round16((n + 3) / 4);
    if (res_bits & 1) b += round16((n + 7) / 8);
    return b;
}

inline int full_res_bits(int fmt) { return fmt == MPO_FP16 ? 13 : 16; }

struct StepLaunch {
    const TensorDesc *descs; /* device */
    const Chunk *chunks;     /* device */
    uint64_t first_chunk, num_chunks;
    int opt;      /* mpo_opt */
    int wfmt;     /* mpo_fmt of hi   */
    int gfmt;     /* mpo_fmt of grad */
    int decay;    /* Decay           */
    int momentum; /* SGD: momentum != 0 */
    int rmode;    /* ResMode         */
    StepScalars s;
    bool use_ov;  /* gradients come from `ov` (mpo_step_layer with per-call pointers) */
    GradOverride ov;
    hipStream_t stream;
};

/* Where one tensor's chunks sit in the chunk table (see layer_rows_log2). */
struct TensorLayout {
    uint32_t rows_log2;   /* chunk length of the tensor's layer: 2^rows_log2 rows            */
    uint32_t has_ragged;  /* the tensor ends in a shorter chunk                               */
    uint64_t ragged_pos;  /* table index of that chunk                                        */
    uint64_t full_pos;    /* table index of the tensor's first full chunk                     */
    uint64_t num_full;    /* number of full chunks                                            */
};

/* Host-side pieces shared by the plan (mpo_host.cpp) and the entry point that allocates nothing
 * (mpo_noalloc.hip).  None of them allocates. */
struct Range {
    uintptr_t lo, hi; /* [lo, hi) in bytes */
    bool written;
};
bool has_conflict(Range *r, uint64_t count);                 /* sorts r in place */
/* Validates one list entry and appends its ranges (at most 5) to r[*count...]. */
mpo_status check_tensor(const mpo_tensor &t, uint32_t &res_slot, Range *r, uint64_t *count);
TensorDesc make_desc(const mpo_tensor &t, uint32_t tensor_id);
/* descs[0..nt) in layer order, layer[k] the layer id of descs[k]: fills lay[0..nt), returns the
 * number of chunks, or UINT64_MAX if a tensor is too long for the table's encoding. */
uint64_t layout_chunks(const TensorDesc *descs, const int32_t *layer, uint64_t nt, uint64_t small_layer_params,
                       TensorLayout *lay);
mpo_status adam_scalars(const mpo_adam_cfg *c, uint64_t step, StepLaunch &L);
mpo_status sgd_scalars(const mpo_sgd_cfg *c, uint64_t step, StepLaunch &L);
/* Residual storage of a list against the format and rounding mode of a step: fills L.rmode. */
mpo_status check_res_mode(uint32_t res_slot, bool any_explicit_bits, uint32_t min_res_bits, uint32_t max_res_bits,
                          StepLaunch &L);
mpo_status hip_fail(hipError_t e);

hipError_t launch_step(const StepLaunch &L);
/* the four parts of launch_step, one object file each (mpo_step.hip) */
hipError_t launch_step_adam(const StepLaunch &L);
hipError_t launch_step_adam_ov(const StepLaunch &L);
hipError_t launch_step_sgd(const StepLaunch &L);
hipError_t launch_step_sgd_ov(const StepLaunch &L);
hipError_t launch_split(const float *w32, uint16_t *hi, void *res, uint64_t n, int fmt, int res_bits, int packed,
                        int round, uint64_t seed, uint32_t tensor_id, hipStream_t stream);
hipError_t launch_merge(const uint16_t *hi, const void *res, float *w32, uint64_t n, int fmt, int res_bits, int packed,
                        int round, hipStream_t stream);

/* Extra bits actually kept: an explicit count, else all of them; stochastic rounding of bf16
 * keeps 15 so that the flag fits the 16-bit slot.  In packed planes res_bits counts the stored
 * bits, and with stochastic rounding the leading one of them is the flag. */
inline int kept_res_bits(int fmt, int res_bits, int round, int packed)
{
    if (packed) return res_bits - (round == MPO_ROUND_STOCHASTIC ? 1 : 0);
    if (res_bits) return res_bits;
    return (round == MPO_ROUND_STOCHASTIC && fmt == MPO_BF16) ? 15 : full_res_bits(fmt);
}

} // namespace mpo
#endif
