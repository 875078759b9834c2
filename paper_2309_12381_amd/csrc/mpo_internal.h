/* Shared between the host side (mpo_host.cpp) and the kernels (mpo_kernels.hip)
 * of libmpo.  Not part of the public interface (see include/mpo.h). */
#ifndef MPO_INTERNAL_H
#define MPO_INTERNAL_H

#include <hip/hip_runtime_api.h>
#include <stdint.h>

#include "mpo.h"

namespace mpo {

/* One workgroup (256 lanes = 4 wavefronts of 64) owns one chunk.  The chunk length can be set at
 * build time (a multiple of 1024) for measurements: 1024, 2048 and 4096 give the same throughput on
 * the large parameter sets; 4096 keeps the chunk table smallest. */
constexpr uint32_t kBlock = 256;
#ifndef MPO_CHUNK_ELEMS
#define MPO_CHUNK_ELEMS 4096
#endif
constexpr uint32_t kChunkElems = MPO_CHUNK_ELEMS;
static_assert(kChunkElems % 1024 == 0 && kChunkElems >= 1024, "a chunk is a whole number of rows of 4 wavefronts");

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

/* Chunk table entry: which tensor (index into the plan's layer-ordered
 * descriptor array) and which chunk of it. */
struct Chunk {
    uint32_t tensor;
    uint32_t index;
};

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

/* Per-call gradient pointers for one layer (Section 3.2), passed by value. */
struct GradOverride {
    const uint16_t *ptr[MPO_MAX_LAYER_GRADS];
    uint64_t misaligned; /* bit i set: ptr[i] is not 16-byte aligned            */
    uint32_t first;      /* descriptor index of the layer's first tensor        */
    uint32_t enabled;
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
    GradOverride ov;
    hipStream_t stream;
};

hipError_t launch_step(const StepLaunch &L);
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
