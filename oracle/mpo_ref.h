/*
 * mpo_ref — CPU oracle for the split-precision optimizer step.
 *
 * TEST INFRASTRUCTURE ONLY.  This is the slow, plain definition of what the
 * GPU library must compute.  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg may use it; the product path never does.  It shares no
 * code with the GPU library.
 *
 * What it follows (arXiv 2309.12381):
 *   - Table 1           : field widths of fp32 / bf16 / fp16.
 *   - Section 3.1       : a weight is kept as a 16-bit float plus the
 *                         significand bits that an fp32 copy would have kept
 *                         (16 for bf16, 13 for fp16); keeping only the leading
 *                         part of the significand is a round-toward-zero; the
 *                         update is carried out in full (fp32) precision and
 *                         both parts are written back; Adam and SGD are the
 *                         classic ones.
 *   - Section 3.2, 4.1  : the step runs per parameter as soon as its gradient
 *                         exists; gradient scaling is applied inside the step.
 *
 * All arithmetic is fp32, one IEEE round-to-nearest-even operation at a time
 * (no fused multiply-add, denormals kept).  Every pointer is a host pointer.
 * Parity status: every function here is pinned by tests/test_oracle_*.py.
 */
#ifndef MPO_REF_H
#define MPO_REF_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { MPO_REF_BF16 = 0, MPO_REF_FP16 = 1 };

/* Section 3.1 also allows keeping only some of those bits: res_bits = E keeps the E
 * leading bits of the dropped significand bits (E = 8 is the paper's fp16+8 /
 * bf16+8).  0 means all of them (16 for bf16, 13 for fp16).  The residual array
 * has one uint8_t per element when 1 <= E <= 8, else one uint16_t; the E bits
 * are right-aligned in it. */

/* Section 3.1, last paragraph: how the 16-bit value is rounded.
 *   TRUNC      hi = the leading bits (round toward zero): the method's base mode.
 *   NEAREST    hi is rounded up in magnitude when the dropped bits are at least
 *              half a unit; the leading dropped bit tells whether that happened,
 *              so no extra storage is needed to undo it.
 *   STOCHASTIC hi is rounded up in magnitude with probability (dropped bits) /
 *              2^full; one more bit, stored just above the kept residual bits,
 *              records it so that the value can be "un-rounded" before the update.
 * In every mode merge gives back the same fp32 value as TRUNC would: only the
 * 16-bit value seen by forward / backward differs.  STOCHASTIC never rounds a
 * value up out of the finite range; NEAREST, like IEEE rounding, turns a value
 * within half a unit of overflow into infinity (merge still undoes it), and never
 * touches a NaN pattern (a NaN stays a NaN in hi; its payload is not preserved
 * when the fp32 NaN has its payload in the dropped bits only).
 * In STOCHASTIC mode res_bits = 0 means 15 kept bits
 * for bf16 (15 + 1 flag fill the 16-bit slot) and 13 for fp16; at most 7 kept
 * bits fit a byte slot and 15 a 16-bit slot.
 * Random numbers: Philox4x32-10 (Salmon et al., SC'11), key = the 64-bit seed,
 * counter = (i/4 low, i/4 high, step low 32 bits, tensor_id); element i uses
 * word i%4, its top `full` bits.  The initial split uses step 0. */
enum { MPO_REF_TRUNC = 0, MPO_REF_NEAREST = 1, MPO_REF_STOCHASTIC = 2 };

/* Packed storage (Section 3.1, Figure 1: the extra bits of many values packed without
 * padding).  With res_packed != 0 the residual is stored in bit planes instead of one slot per
 * value, and res_bits = S in 1..15 is the number of bits stored per value: the E = S kept bits
 * in TRUNC and NEAREST mode; in STOCHASTIC mode E = S - 1 kept bits below the flag, which is the
 * leading stored bit.  The S bits are cut, from the top, into the pieces of 8, 4, 2 and 1 bits
 * that the binary form of S contains; each piece has its own dense array ("plane") in which
 * value i occupies bits [w*i, w*i + w) (w = 8, 4, 2, 1; little-endian within a byte).  The
 * planes follow each other in the residual buffer in that order, each starting at a multiple
 * of 16 bytes: sizes round16(n), round16(ceil(n/2)), round16(ceil(n/4)), round16(ceil(n/8)).
 * S bits per value, nothing wasted: 12 extra bits take 1.5 bytes, the 13 of fp16 take 13 bits. */
uint64_t mpo_ref_res_bytes(uint64_t n, int fmt, int res_bits, int res_packed);

typedef struct {
    double lr, beta1, beta2, eps, weight_decay;
    int32_t decoupled_wd; /* 1: AdamW (w *= 1-lr*wd), 0: L2 (g += wd*w)      */
    double loss_scale;    /* gradients arrive multiplied by this              */
    int32_t weight_fmt;   /* format of hi                                     */
    int32_t grad_fmt;     /* format of grad                                   */
    int32_t res_bits;     /* extra bits kept, 0 = all                         */
    int32_t res_packed;   /* residual stored in bit planes                    */
    int32_t round;        /* MPO_REF_TRUNC / NEAREST / STOCHASTIC             */
    uint64_t seed;        /* STOCHASTIC only                                  */
    double grad_clip;     /* Section 4.1: clamp the un-scaled gradient to [-c, c]; 0 = off */
} mpo_ref_adam_cfg;

typedef struct {
    double lr, momentum, weight_decay; /* weight decay is L2 (added to g)     */
    double loss_scale;
    int32_t weight_fmt, grad_fmt;
    int32_t res_bits;
    int32_t res_packed;
    int32_t round;
    uint64_t seed;
    double grad_clip;
} mpo_ref_sgd_cfg;

/* `first_index` (split and the steps): the arrays given hold elements first_index ..
 * first_index + n - 1 of their tensor.  It matters to STOCHASTIC rounding only, whose random
 * stream is indexed by an element's position in its tensor: a slice of a tensor handled with its
 * first_index gives the same bits as the same elements handled as part of the whole tensor.
 * Must be 0 with res_packed (where a plane starts depends on the tensor's length). */

/* Section 3.1, Table 1: fp32 -> (16-bit float, extra bits), truncation. */
void mpo_ref_split(const float *w32, uint16_t *hi, void *res, uint64_t n, int fmt, int res_bits, int res_packed,
                   int round, uint64_t seed, uint32_t tensor_id, uint64_t first_index);
/* Section 3.1: (16-bit float, extra bits) -> fp32. */
void mpo_ref_merge(const uint16_t *hi, const void *res, float *w32, uint64_t n, int fmt, int res_bits, int res_packed,
                   int round);

/* Section 3.1 (the usual optimizers): bias-corrected Adam / AdamW on one tensor. */
void mpo_ref_adam_step(uint16_t *hi, void *res, const uint16_t *grad, float *m, float *v,
                       uint64_t n, const mpo_ref_adam_cfg *cfg, uint64_t step, uint32_t tensor_id,
                       uint64_t first_index);
/* Section 3.1 (the usual optimizers): SGD with momentum (dampening 0, no Nesterov).
 * momentum == 0 leaves buf untouched (it may then be NULL). */
void mpo_ref_sgd_step(uint16_t *hi, void *res, const uint16_t *grad, float *buf,
                      uint64_t n, const mpo_ref_sgd_cfg *cfg, uint64_t step, uint32_t tensor_id,
                      uint64_t first_index);

/* One Philox4x32-10 block: out = philox(counter, key). */
void mpo_ref_philox4x32_10(const uint32_t counter[4], const uint32_t key[2], uint32_t out[4]);

/* Exact conversion of one 16-bit float to fp32 (used for gradients). */
float mpo_ref_cvt16(uint16_t x, int fmt);

#ifdef __cplusplus
}
#endif
#endif
