/*
 * mpo — split-precision optimizer step for AMD MI355X (gfx950).
 *
 * Method: arXiv 2309.12381, "Memory Efficient Mixed Precision Optimizers".
 * A weight is stored as a 16-bit float `hi` (bf16 or fp16: what forward and
 * backward use) plus a 16-bit residual `res` holding the significand bits an
 * fp32 master copy would have kept (Section 3.1; field widths in Table 1).
 * The optimizer step rebuilds the fp32 weight from (hi, res), applies Adam or
 * SGD in fp32 with fp32 moments, and splits the result again; no fp32 copy of
 * the weights exists.  The step can be run per layer as soon as that layer's
 * gradient exists, so a gradient is consumed and never kept (Section 3.2).
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers on the current HIP device, owned by
 *     the caller.  Arrays are dense, element i of every array of a tensor
 *     belongs to parameter i.  `hi` and `grad` are uint16_t bit patterns, `res`
 *     is uint16_t or, with at most 8 extra bits kept, uint8_t (see res_bits).
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = default stream).
 *     Calls only enqueue work on that stream and return; they never wait for
 *     the device.  Only mpo_plan_create allocates (host and device memory, freed
 *     by mpo_plan_destroy); split, merge and the step entry points allocate
 *     nothing, on the host or on the device.
 *   - Pointers need no particular alignment: 16-byte aligned tensors take the
 *     128-bit path, others a slower element-wise path with identical results.
 *   - Errors are reported by return code only and nothing is enqueued when a
 *     call fails validation.  n == 0 and empty lists are legal no-ops.
 *   - All arithmetic is IEEE binary32, one rounding per operation (no fused
 *     multiply-add, correctly rounded division and square root, denormals
 *     kept), so results are reproducible bit for bit.
 */
#ifndef MPO_H
#define MPO_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MPO_OK = 0,
    MPO_ERR_INVALID_ARG = 1, /* null pointer with n > 0, step == 0, unknown enum, bad size   */
    MPO_ERR_UNSUPPORTED = 2, /* a combination that is not built (mixed residual widths, ...)  */
    MPO_ERR_ALIAS = 3,       /* buffers that are written overlap each other or an input      */
    MPO_ERR_HIP = 4,         /* a HIP runtime call failed (see mpo_last_hip_error)           */
    MPO_ERR_NOMEM = 5,       /* host or device allocation for a plan failed                  */
    MPO_ERR_TOO_LARGE = 6    /* more tensors or chunks than mpo_adam_step_noalloc has room for */
} mpo_status;

/* Format of a 16-bit float array (Table 1): bf16 = 1+8+7 bits, 16 extra bits;
 * fp16 = 1+5+10 bits, 13 extra bits right-aligned in the 16-bit residual (its
 * top three bits are written as zero and ignored when read). */
typedef enum { MPO_BF16 = 0, MPO_FP16 = 1 } mpo_fmt;

/* How `hi` is derived from the fp32 value (Section 3.1, last paragraph).
 *   MPO_ROUND_TRUNC       hi = the leading bits, a round-toward-zero: the method's base mode.
 *   MPO_ROUND_STOCHASTIC  hi is moved to the next 16-bit value away from zero with probability
 *                         (dropped bits) / 2^full; one more bit, stored just above the kept
 *                         residual bits, records it, and the step un-rounds hi before the
 *                         update.  Never rounds out of the finite range.  When res_bits is 0,
 *                         bf16 keeps 15 extra bits (15 + flag fill the 16-bit slot), fp16 13.
 *                         At most 7 kept bits fit a byte slot and 15 a 16-bit slot, else
 *                         MPO_ERR_INVALID_ARG.
 *   MPO_ROUND_NEAREST     the deterministic counterpart: up when the dropped bits are at least
 *                         half a unit (ties away from zero; like IEEE rounding a value within
 *                         half a unit of overflow becomes infinity; a NaN pattern is left as
 *                         it is, so a NaN weight stays a NaN in hi).  The leading dropped bit
 *                         tells the step to undo it; nothing extra is stored.
 * In every mode the fp32 value held by (hi, res), and therefore the whole fp32 trajectory of a
 * training run, is the same as with MPO_ROUND_TRUNC; only the 16-bit value that forward and
 * backward see differs.  The mode is a property of the stored data: use the same one in
 * mpo_split, every step and mpo_merge.
 * Random numbers: Philox4x32-10 (Salmon et al., SC'11), key = the 64-bit seed, counter =
 * (i/4 low, i/4 high, low 32 bits of step, index of the tensor in its list); parameter i takes
 * word i%4, its top `full` bits.  mpo_split draws with step 0. */
typedef enum { MPO_ROUND_TRUNC = 0, MPO_ROUND_NEAREST = 1, MPO_ROUND_STOCHASTIC = 2 } mpo_round;

typedef enum { MPO_OPT_ADAM = 0, MPO_OPT_SGD = 1 } mpo_opt;

/* ---- how many extra bits are kept (Section 3.1) ---------------------------
 *
 * `res_bits` = E, the number of leading dropped significand bits that the
 * residual keeps.  0 means all of them (16 for bf16, 13 for fp16): the pair
 * is then as precise as fp32.  1 <= E < all keeps only part of them (the
 * paper's fp16+8 / bf16+8 is E = 8): the fp32 value is cut toward zero to
 * 16 + E bits.  Storage: one uint8_t per parameter when 1 <= E <= 8, else one
 * uint16_t; the E bits are right-aligned in it.  E above the format's full
 * count is MPO_ERR_INVALID_ARG.
 *
 * `res_packed` != 0 stores the bits without padding (Section 3.1, Figure 1).
 * `res_bits` = S, 1 to 15, is then the number of bits STORED per parameter:
 * the E = S kept bits with MPO_ROUND_TRUNC and MPO_ROUND_NEAREST; with
 * MPO_ROUND_STOCHASTIC the flag is the leading stored bit and E = S - 1 (so
 * S >= 2).  E above the format's full count is MPO_ERR_INVALID_ARG (the 13
 * extra bits of fp16 with the flag are S = 14).  The layout is planar rather
 * than one bit string, so that lanes read and write whole bytes: the S bits
 * are cut, from the top, into the pieces of 8, 4, 2 and 1 bits that the binary
 * form of S contains; each piece has its own dense plane in which value i
 * occupies bits [w*i, w*i + w) (w = 8, 4, 2, 1; little-endian in a byte); the
 * planes follow each other in `res` in that order, each starting at a
 * multiple of 16 bytes (sizes round16(n), round16(ceil(n/2)),
 * round16(ceil(n/4)), round16(ceil(n/8))).  `res` must then be 16-byte
 * aligned and hold mpo_res_bytes() bytes: 12 extra bits take 1.5 bytes per
 * parameter.  Bits of the last bytes that belong to no parameter are written
 * as zero by mpo_split and kept by the steps.
 */
uint64_t mpo_res_bytes(uint64_t n, int32_t res_bits, int32_t res_packed);

/* ---- split / merge (Section 3.1, Table 1) --------------------------------
 *
 * mpo_split: w32[i] -> (hi[i], res[i]).  bf16: hi = upper, res = lower half of
 * the fp32 pattern (a bijection on all 2^32 patterns).  fp16: exact for
 * 2^-14 <= |x| < 65536 and for multiples of 2^-37 below that; other values are
 * cut toward zero to the 2^-37 grid, finite values of 65536 or more saturate
 * at the largest finite pair, +-inf and NaN map to fp16 +-inf / NaN.
 * mpo_merge: the inverse, (hi[i], res[i]) -> w32[i] (cut bits read as zero).
 * w32 must not overlap hi or res (MPO_ERR_ALIAS); n is a number of elements.
 * `seed` and `tensor_id` select the random stream (MPO_ROUND_STOCHASTIC only):
 * give mpo_split the seed of the optimizer configuration and the index the
 * tensor has in the list passed to mpo_plan_create.
 */
mpo_status mpo_split(const float *w32, uint16_t *hi, void *res, uint64_t n,
                     mpo_fmt fmt, int32_t res_bits, int32_t res_packed, mpo_round round, uint64_t seed,
                     uint32_t tensor_id, void *hip_stream);
mpo_status mpo_merge(const uint16_t *hi, const void *res, float *w32, uint64_t n,
                     mpo_fmt fmt, int32_t res_bits, int32_t res_packed, mpo_round round, void *hip_stream);

/* ---- parameter list -------------------------------------------------------
 *
 * One entry per parameter tensor.  `grad` may be NULL if gradients are only
 * ever supplied per call (mpo_step_layer).  `v` may be NULL for a list that is
 * only stepped with SGD, `m` (the momentum buffer) too if momentum is 0.
 * `layer` (>= 0) groups tensors whose gradients become available together.
 * `res_bits` is the number of extra bits this tensor's residual keeps (see
 * above; with `res_packed` it fixes whether `res` is a uint8_t array, a uint16_t
 * array or packed planes).  All tensors of one list must use the same kind of
 * residual storage, else MPO_ERR_UNSUPPORTED.
 * Gradient buffers may overlap each other (one reused buffer for all layers);
 * nothing may overlap hi, res, m or v.
 * Alignment: arrays that are all 16-byte aligned take the vector path (any
 * alignment gives the same results, more slowly).  For full speed start every
 * array on a 128-byte boundary: rows of a tensor that starts inside a memory
 * line straddle lines, which costs about 14 % on lists of many small tensors.
 * Placement: on MI355X (288 GiB) the device memory behaves as three regions
 * of 96 GiB, and a step whose written arrays (hi, res, m, v) all lie in one
 * region runs about 14 % slower than one whose written arrays are divided
 * between two (measured; arrays allocated one after the other in a fresh
 * process all land in the first region).  The library takes the pointers it
 * is given; mpo_place_second (mpo_probe.h, libmpo_probe.so) finds a block in
 * another region by measurement, and the Python package's
 * placement.allocate_state does the same on torch tensors.
 */
typedef struct {
    uint16_t *hi;
    void *res;
    const uint16_t *grad;
    float *m;
    float *v;
    uint64_t n;
    int32_t layer;
    int32_t res_bits;
    int32_t res_packed;
} mpo_tensor;

/* Adam / AdamW (Section 3.1: the classic optimizer, hyper-parameters
 * unchanged): bias-corrected moments, eps added to sqrt(v_hat); step size,
 * corrections and decay factor are formed in double on the host and rounded to
 * fp32 once.  decoupled_wd != 0: w *= 1 - lr*wd before the update (AdamW);
 * else g += wd*w (L2).  Gradients arrive multiplied by loss_scale and are
 * divided by it inside the step (Section 4.1); loss_scale must be finite, > 0.
 * grad_clip > 0 clamps every un-scaled gradient element to [-grad_clip,
 * grad_clip] inside the step (Section 4.1: with the step fused into backward,
 * clipping has to happen there); 0 switches it off; NaN stays NaN.
 */
typedef struct {
    double lr, beta1, beta2, eps, weight_decay;
    int32_t decoupled_wd;
    double loss_scale;
    int32_t weight_fmt; /* mpo_fmt of hi   */
    int32_t grad_fmt;   /* mpo_fmt of grad */
    int32_t round;      /* mpo_round       */
    uint64_t seed;      /* random stream of MPO_ROUND_STOCHASTIC */
    double grad_clip;   /* element-wise clamp of the gradient, 0 = off */
} mpo_adam_cfg;

/* SGD with momentum (dampening 0, no Nesterov), L2 weight decay.
 * momentum == 0 leaves m untouched. */
typedef struct {
    double lr, momentum, weight_decay;
    double loss_scale;
    int32_t weight_fmt, grad_fmt, round;
    uint64_t seed;
    double grad_clip;
} mpo_sgd_cfg;

typedef struct mpo_plan mpo_plan;

/* Section 3.1 ("Fused" optimizer: all parameters handled as one stream so one
 * launch covers many tensors).  Validates the list, rejects overlaps, orders
 * tensors by layer (stable), cuts them into fixed-size chunks and uploads the
 * chunk table and tensor descriptors to the current device once.  The plan
 * owns only that table (a few MB); free it with mpo_plan_destroy.  The list is
 * copied: `tensors` may be freed after the call.  nt == 0 gives a valid empty
 * plan.  mpo_plan_destroy(NULL) is a no-op.  A plan belongs to the device that
 * was current when it was created: stepping it with another device current is
 * MPO_ERR_INVALID_ARG.  Step calls are plain kernel launches and may be
 * captured into a HIP graph (the step number is then fixed in the graph). */
mpo_status mpo_plan_create(const mpo_tensor *tensors, uint64_t nt, mpo_plan **out);
mpo_status mpo_plan_destroy(mpo_plan *plan);

/* Same validation and layout, kept on the host only (no HIP call at all): for
 * inspecting the layout and for tests on machines without a GPU.  Step calls
 * on such a plan return MPO_ERR_INVALID_ARG. */
mpo_status mpo_plan_create_host(const mpo_tensor *tensors, uint64_t nt, mpo_plan **out);

/* mpo_plan_create with options; opts == NULL or a zero field means the default.
 *   small_layer_params  layers with fewer parameters than this are cut into chunks of 1024
 *                       parameters instead of 4096.  0 = the default: short chunks everywhere
 *                       for 16-bit and byte residuals, 2^26 for packed planes (what measured
 *                       fastest on MI355X); 1 = long chunks everywhere (a chunk table a
 *                       quarter the size); UINT64_MAX = short chunks everywhere.  A tuning
 *                       knob: results do not depend on it.
 *   host_only           != 0: as mpo_plan_create_host. */
typedef struct {
    uint64_t small_layer_params;
    int32_t host_only;
} mpo_plan_opts;
mpo_status mpo_plan_create_opts(const mpo_tensor *tensors, uint64_t nt, const mpo_plan_opts *opts, mpo_plan **out);

/* Layout queries (host side, no HIP call).  One workgroup handles one chunk.  All
 * chunks of a layer have the same length: 1024 parameters, or 4096 (what
 * mpo_plan_chunk_elems returns, the longest) in layers of at least
 * mpo_plan_opts.small_layer_params parameters (by default: never, except with packed
 * planes from 2^26 parameters on).  Chunks are numbered in launch order:
 * layer by layer; within a layer first every tensor's last, shorter chunk (if its
 * length is not a multiple of the chunk length), then the full chunks tensor by
 * tensor.  Chunk i covers `count` elements from element `first` of tensor `tensor`
 * (an index into the list given at creation). */
uint64_t mpo_plan_chunk_elems(const mpo_plan *plan);
uint64_t mpo_plan_num_chunks(const mpo_plan *plan);
uint64_t mpo_plan_num_params(const mpo_plan *plan);
mpo_status mpo_plan_get_chunk(const mpo_plan *plan, uint64_t i, uint64_t *tensor, uint64_t *first, uint64_t *count);
/* Chunk range, tensor and parameter count and chunk length of one layer (any output may be
 * NULL); an unknown layer is MPO_ERR_INVALID_ARG. */
mpo_status mpo_plan_layer_info(const mpo_plan *plan, int32_t layer, uint64_t *first_chunk,
                               uint64_t *num_chunks, uint64_t *num_tensors, uint64_t *num_params,
                               uint64_t *chunk_elems);

/* One optimizer step over every tensor of the plan in ONE kernel launch
 * (Section 3.1).  `step` counts from 1 and is shared by all tensors.  Every
 * tensor needs grad and m (and v for Adam) from plan creation. */
mpo_status mpo_adam_step(mpo_plan *plan, const mpo_adam_cfg *cfg, uint64_t step, void *hip_stream);
mpo_status mpo_sgd_step(mpo_plan *plan, const mpo_sgd_cfg *cfg, uint64_t step, void *hip_stream);

/* Section 3.2: the step of ONE layer, to be called as soon as that layer's
 * gradients exist, in one launch; the caller may reuse the gradient memory as
 * soon as later work on the same stream is enqueued.  `cfg` points to an
 * mpo_adam_cfg (opt == MPO_OPT_ADAM) or an mpo_sgd_cfg (MPO_OPT_SGD).
 * `grads` is NULL to use the gradient pointers given at plan creation, else
 * `ngrads` device pointers, one per tensor of that layer in the order the
 * tensors were listed at creation (ngrads must equal the layer's tensor count
 * and be at most MPO_MAX_LAYER_GRADS).  Stepping every layer once with the
 * same `step` is bit-identical to one mpo_adam_step / mpo_sgd_step. */
#define MPO_MAX_LAYER_GRADS 64
mpo_status mpo_step_layer(mpo_plan *plan, int32_t layer, const void *const *grads, uint64_t ngrads,
                          mpo_opt opt, const void *cfg, uint64_t step, void *hip_stream);

/* For callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  The same step as mpo_adam_step (one
 * launch over the whole list, same results bit for bit) without a plan: the list is given
 * on every call, and the chunk table and descriptors that a plan would hold in allocated
 * memory are rebuilt, by a small kernel on `hip_stream`, in a fixed array inside the
 * library's device image (16 MiB + 64 KiB per GPU, held until the process ends).  Nothing
 * is allocated, freed or copied, on the host or on the device; the call only enqueues
 * kernels (1 + ceil(nt / 32) of them).
 * Every tensor needs grad, m and v.  Limits: at most MPO_NOALLOC_MAX_TENSORS tensors and
 * MPO_NOALLOC_MAX_CHUNKS chunks (here layers of 2^26 parameters or more get the long
 * chunks: about 8.6e9 parameters in such layers), else MPO_ERR_TOO_LARGE and nothing is
 * enqueued.
 * All calls on one GPU share that GPU's array: calls whose kernels may overlap in time
 * (different streams or threads) race on it and must be ordered by the caller.  The first
 * call on a device looks the array's address up and must not run under stream capture;
 * later calls may be captured.  The validation works in fixed-size arrays on the calling
 * thread's stack, about 256 KiB of it. */
#define MPO_NOALLOC_MAX_TENSORS 1024
#define MPO_NOALLOC_MAX_CHUNKS (1u << 21)
mpo_status mpo_adam_step_noalloc(const mpo_tensor *tensors, uint64_t nt, const mpo_adam_cfg *cfg, uint64_t step,
                                 void *hip_stream);

const char *mpo_status_string(mpo_status s);
/* hipError_t (as int) of the most recent failing HIP call on this thread, 0 if none. */
int mpo_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* MPO_H */
