/*
 * mpo_ref — CPU oracle (see mpo_ref.h).  TEST INFRASTRUCTURE ONLY.
 *
 * Build: gcc -O2 -std=c11 -ffp-contract=off -fno-fast-math -fPIC -shared
 * One element at a time, one rounded fp32 operation per line.
 */
#include "mpo_ref.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

/* ---- bit views ---------------------------------------------------------- */

static uint32_t bits_of(float x) { uint32_t b; memcpy(&b, &x, 4); return b; }
static float float_of(uint32_t b) { float x; memcpy(&x, &b, 4); return x; }

/* ---- bf16: 1 + 8 + 7 bits (Table 1); 16 significand bits dropped (Sec. 3.1) */

static void split_bf16(float x, uint16_t *hi, uint16_t *res)
{
    uint32_t b = bits_of(x);
    *hi = (uint16_t)(b >> 16);      /* sign, exponent, leading 7 fraction bits */
    *res = (uint16_t)(b & 0xFFFFu); /* the 16 fraction bits bf16 cannot hold   */
}

static float merge_bf16(uint16_t hi, uint16_t res)
{
    return float_of(((uint32_t)hi << 16) | (uint32_t)res);
}

/* ---- fp16: 1 + 5 + 10 bits (Table 1); 13 significand bits dropped (Sec. 3.1)
 *
 * The 13 extra bits sit right-aligned in the 16-bit residual; its top three
 * bits are written as zero and ignored on merge.
 * fp16 keeps its subnormals (Sec. 1.1): below 2^-14 the pair (hi, res) is a
 * 23-bit fixed-point number in units of 2^-37.  Values the pair cannot hold are
 * truncated toward zero, in line with the round-toward-zero reading of Sec. 3.1:
 * finite magnitudes of 65536 or more saturate at the largest finite pair.
 */

static void split_fp16(float x, uint16_t *hi, uint16_t *res)
{
    uint32_t b = bits_of(x);
    uint16_t s = (uint16_t)((b >> 31) << 15);
    uint32_t E = (b >> 23) & 0xFFu;
    uint32_t M = b & 0x7FFFFFu;

    if (E == 255u) {                       /* infinity or NaN */
        *hi = (uint16_t)(s | (M == 0 ? 0x7C00u : 0x7E00u));
        *res = 0;
        return;
    }
    if (E == 0u) {                         /* fp32 zero or subnormal: below 2^-37 */
        *hi = s;
        *res = 0;
        return;
    }
    int e = (int)E - 127;
    if (e > 15) {                          /* too large: largest finite pair */
        *hi = (uint16_t)(s | 0x7BFFu);
        *res = 0x1FFFu;
        return;
    }
    if (e >= -14) {                        /* fp16 normal range: re-bias the exponent */
        *hi = (uint16_t)(s | ((uint32_t)(e + 15) << 10) | (M >> 13));
        *res = (uint16_t)(M & 0x1FFFu);
        return;
    }
    /* fp16 subnormal range: shift the 24-bit significand down to the 2^-37 grid */
    int shift = -14 - e;
    uint32_t F = shift >= 24 ? 0u : ((1u << 23) | M) >> shift;
    *hi = (uint16_t)(s | (F >> 13));
    *res = (uint16_t)(F & 0x1FFFu);
}

static float merge_fp16(uint16_t hi, uint16_t res)
{
    uint32_t s = (uint32_t)(hi >> 15) << 31;
    uint32_t E = (hi >> 10) & 0x1Fu;
    uint32_t k = hi & 0x3FFu;
    uint32_t r = res & 0x1FFFu;

    if (E == 31u)                          /* infinity, or a quiet NaN */
        return float_of(s | 0x7F800000u | (k == 0 ? 0u : (0x00400000u | (k << 13))));
    if (E == 0u) {                         /* subnormal: (k, r) counts units of 2^-37 */
        float mag = ldexpf((float)((k << 13) | r), -37);   /* exact: integer < 2^23 */
        return s ? -mag : mag;
    }
    return float_of(s | ((E + 112u) << 23) | (k << 13) | r);
}

static void split_one(float x, uint16_t *hi, uint16_t *res, int fmt)
{
    if (fmt == MPO_REF_FP16) split_fp16(x, hi, res); else split_bf16(x, hi, res);
}

static float merge_one(uint16_t hi, uint16_t res, int fmt)
{
    return fmt == MPO_REF_FP16 ? merge_fp16(hi, res) : merge_bf16(hi, res);
}

/* ---- Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as
 * easy as 1, 2, 3", SC'11): ten rounds of two 32x32->64 multiplications. ---- */

void mpo_ref_philox4x32_10(const uint32_t counter[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = counter[0], c1 = counter[1], c2 = counter[2], c3 = counter[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        if (round > 0) {
            k0 += 0x9E3779B9u;             /* golden ratio   */
            k1 += 0xBB67AE85u;             /* sqrt(3) - 1    */
        }
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* ---- residual storage, rounding of the 16-bit value (Sec. 3.1) -------------
 * The stored residual is the full one with its trailing bits cut off (E kept
 * bits, right-aligned); on merge the cut bits read as zero: the fp32 value is
 * truncated toward zero to 16 + E bits.  NEAREST / STOCHASTIC add one to the
 * 16-bit pattern of hi (the next value away from zero) and remember it. */

typedef struct {
    int fmt, round;
    int full;      /* dropped bits of the format: 16 (bf16) or 13 (fp16) */
    int kept;      /* E: bits of them that are stored                    */
    int byte_slot; /* residual array is uint8_t                          */
    int packed;    /* residual stored in bit planes (Figure 1)           */
    int stored;    /* packed: bits per value in the planes (E, plus the flag of STOCHASTIC) */
    uint64_t n;    /* number of values: fixes where each plane starts    */
    uint64_t first; /* index, within its tensor, of element 0 of the arrays given */
    uint64_t seed;
    uint32_t tensor_id, step32;
} res_layout;

static uint64_t round16(uint64_t x) { return (x + 15u) / 16u * 16u; }

/* Packed storage: value i of a plane of width w (8, 4, 2 or 1 bits) */
static uint32_t plane_get(const uint8_t *plane, uint64_t i, int w)
{
    uint64_t bit = i * (uint64_t)w;
    return (plane[bit / 8] >> (bit % 8)) & ((1u << w) - 1u);
}

static void plane_put(uint8_t *plane, uint64_t i, int w, uint32_t x)
{
    uint64_t bit = i * (uint64_t)w;
    uint8_t mask = (uint8_t)(((1u << w) - 1u) << (bit % 8));
    plane[bit / 8] = (uint8_t)((plane[bit / 8] & ~mask) | ((x << (bit % 8)) & mask));
}

/* The S stored bits of value i, assembled from / distributed to the planes: S is cut from the
 * top into the pieces of 8, 4, 2 and 1 bits its binary form contains; the 8-bit piece holds the
 * leading bits, then the 4-bit piece, the 2-bit piece, the 1-bit piece. */
static uint16_t packed_get(const uint8_t *base, uint64_t n, uint64_t i, int S)
{
    uint32_t r = 0;
    const uint8_t *plane = base;
    if (S & 8) { r = (r << 8) | plane_get(plane, i, 8); plane += round16(n); }
    if (S & 4) { r = (r << 4) | plane_get(plane, i, 4); plane += round16((n + 1) / 2); }
    if (S & 2) { r = (r << 2) | plane_get(plane, i, 2); plane += round16((n + 3) / 4); }
    if (S & 1) { r = (r << 1) | plane_get(plane, i, 1); }
    return (uint16_t)r;
}

static void packed_put(uint8_t *base, uint64_t n, uint64_t i, int S, uint16_t r)
{
    uint8_t *plane = base;
    int left = S;
    if (S & 8) { left -= 8; plane_put(plane, i, 8, (r >> left) & 0xFFu); plane += round16(n); }
    if (S & 4) { left -= 4; plane_put(plane, i, 4, (r >> left) & 0xFu); plane += round16((n + 1) / 2); }
    if (S & 2) { left -= 2; plane_put(plane, i, 2, (r >> left) & 0x3u); plane += round16((n + 3) / 4); }
    if (S & 1) { left -= 1; plane_put(plane, i, 1, (r >> left) & 0x1u); }
}

/* Packed: res_bits counts the bits stored per value (with STOCHASTIC one of them is the flag). */
uint64_t mpo_ref_res_bytes(uint64_t n, int fmt, int res_bits, int res_packed)
{
    (void)fmt;
    if (!res_packed) return n * (uint64_t)((res_bits >= 1 && res_bits <= 8) ? 1 : 2);
    uint64_t b = 0;
    if (res_bits & 8) b += round16(n);
    if (res_bits & 4) b += round16((n + 1) / 2);
    if (res_bits & 2) b += round16((n + 3) / 4);
    if (res_bits & 1) b += round16((n + 7) / 8);
    return b;
}

static res_layout make_layout(int fmt, int res_bits, int packed, uint64_t n, int round, uint64_t seed,
                              uint32_t tensor_id, uint64_t step, uint64_t first_index)
{
    res_layout L;
    /* the planes of a packed residual start at places fixed by the tensor's length: a slice of
     * such a tensor cannot be handled on its own */
    if (packed && first_index != 0) abort();
    L.packed = packed;
    L.n = n;
    L.first = first_index;
    L.fmt = fmt;
    L.round = round;
    L.full = fmt == MPO_REF_FP16 ? 13 : 16;
    L.kept = res_bits != 0 ? res_bits : (round == MPO_REF_STOCHASTIC && L.full == 16 ? 15 : L.full);
    L.stored = res_bits;
    /* in the planes the flag of STOCHASTIC is one of the res_bits stored bits, the leading one */
    if (packed && round == MPO_REF_STOCHASTIC) L.kept = res_bits - 1;
    L.byte_slot = res_bits >= 1 && res_bits <= 8;
    L.seed = seed;
    L.tensor_id = tensor_id;
    L.step32 = (uint32_t)step;
    return L;
}

static uint16_t max_finite_hi(int fmt) { return fmt == MPO_REF_FP16 ? 0x7BFFu : 0x7F7Fu; }

/* A 16-bit pattern above that of infinity (sign aside) is a NaN. */
static int is_nan16(uint16_t h, int fmt) { return (uint16_t)(h & 0x7FFFu) > (fmt == MPO_REF_FP16 ? 0x7C00u : 0x7F80u); }

/* Uniform integer in [0, 2^full) for element i of the arrays at this step: the stream is
 * indexed by the element's position in its tensor. */
static uint32_t draw(const res_layout *L, uint64_t i)
{
    i += L->first;
    uint64_t block = i / 4;
    uint32_t counter[4] = { (uint32_t)block, (uint32_t)(block >> 32), L->step32, L->tensor_id };
    uint32_t key[2] = { (uint32_t)L->seed, (uint32_t)(L->seed >> 32) };
    uint32_t out[4];
    mpo_ref_philox4x32_10(counter, key, out);
    return out[i % 4] >> (32 - L->full);
}

/* (hi, res) as stored -> the truncated 16-bit value and the full residual. */
static void load_pair(const uint16_t *hi, const void *res, uint64_t i, const res_layout *L,
                      uint16_t *hi_trunc, uint16_t *res_full)
{
    uint16_t stored = L->packed ? packed_get((const uint8_t *)res, L->n, i, L->stored)
                    : L->byte_slot ? ((const uint8_t *)res)[i] : ((const uint16_t *)res)[i];
    uint16_t kept = (uint16_t)(stored & ((1u << L->kept) - 1u));
    uint16_t full = (uint16_t)(kept << (L->full - L->kept));
    int was_rounded_up = 0;
    if (L->round == MPO_REF_STOCHASTIC) was_rounded_up = (stored >> L->kept) & 1;
    /* NEAREST leaves NaN patterns alone (see store_pair), so there is nothing to undo on one */
    if (L->round == MPO_REF_NEAREST) was_rounded_up = !is_nan16(hi[i], L->fmt) && ((full >> (L->full - 1)) & 1);
    *hi_trunc = (uint16_t)(hi[i] - was_rounded_up);     /* un-round */
    *res_full = full;
}

/* the truncated 16-bit value and the full residual -> (hi, res) as stored */
static void store_pair(uint16_t *hi, void *res, uint64_t i, const res_layout *L, uint16_t hi_trunc, uint16_t res_full)
{
    int up = 0;
    /* NEAREST: the leading dropped bit decides (it is also what tells merge to undo it); like
     * IEEE rounding, a value within half a unit of overflow becomes infinity.  A NaN pattern is
     * never rounded: adding one to the all-ones pattern would wrap around to a zero, and the
     * 16-bit weight must stay a NaN when the fp32 value is one. */
    if (L->round == MPO_REF_NEAREST) up = !is_nan16(hi_trunc, L->fmt) && ((res_full >> (L->full - 1)) & 1);
    /* STOCHASTIC: up with probability res_full / 2^full, but never out of the finite range
     * (the stored flag keeps this invertible) */
    if (L->round == MPO_REF_STOCHASTIC)
        up = (uint16_t)(hi_trunc & 0x7FFFu) < max_finite_hi(L->fmt) && draw(L, i) < res_full;
    uint16_t kept = (uint16_t)(res_full >> (L->full - L->kept));
    if (L->round == MPO_REF_STOCHASTIC) kept = (uint16_t)(kept | (up << L->kept));
    hi[i] = (uint16_t)(hi_trunc + up);
    if (L->packed) packed_put((uint8_t *)res, L->n, i, L->stored, kept);
    else if (L->byte_slot) ((uint8_t *)res)[i] = (uint8_t)kept;
    else ((uint16_t *)res)[i] = kept;
}

/* A 16-bit float read as fp32: every bf16 and fp16 value is an fp32 value. */
float mpo_ref_cvt16(uint16_t x, int fmt)
{
    return fmt == MPO_REF_FP16 ? merge_fp16(x, 0) : merge_bf16(x, 0);
}

void mpo_ref_split(const float *w32, uint16_t *hi, void *res, uint64_t n, int fmt, int res_bits, int res_packed,
                   int round, uint64_t seed, uint32_t tensor_id, uint64_t first_index)
{
    res_layout L = make_layout(fmt, res_bits, res_packed, n, round, seed, tensor_id, 0, first_index);
    for (uint64_t i = 0; i < n; ++i) {
        uint16_t h, full;
        split_one(w32[i], &h, &full, fmt);
        store_pair(hi, res, i, &L, h, full);
    }
}

void mpo_ref_merge(const uint16_t *hi, const void *res, float *w32, uint64_t n, int fmt, int res_bits, int res_packed,
                   int round)
{
    res_layout L = make_layout(fmt, res_bits, res_packed, n, round, 0, 0, 0, 0);
    for (uint64_t i = 0; i < n; ++i) {
        uint16_t h, full;
        load_pair(hi, res, i, &L, &h, &full);
        w32[i] = merge_one(h, full, fmt);
    }
}

/* ---- Adam (Sec. 3.1: the classic optimizer, hyper-parameters unchanged) ----
 *
 * Kingma & Ba's Adam with bias correction; epsilon is added to the
 * bias-corrected root of v; decoupled decay (AdamW) scales the weight by
 * 1 - lr*wd before the update, L2 decay adds wd*w to the gradient.
 * Scalars are formed in double and rounded to fp32 once.  Per element every
 * line below is one rounded fp32 operation.
 */
void mpo_ref_adam_step(uint16_t *hi, void *res, const uint16_t *grad, float *m, float *v,
                       uint64_t n, const mpo_ref_adam_cfg *cfg, uint64_t step, uint32_t tensor_id, uint64_t first_index)
{
    const res_layout L = make_layout(cfg->weight_fmt, cfg->res_bits, cfg->res_packed, n, cfg->round, cfg->seed, tensor_id, step,
                                     first_index);
    const double t = (double)step;
    const float B1 = (float)cfg->beta1;
    const float B2 = (float)cfg->beta2;
    const float O1 = (float)(1.0 - cfg->beta1);
    const float O2 = (float)(1.0 - cfg->beta2);
    const float SS = (float)(cfg->lr / (1.0 - pow(cfg->beta1, t)));  /* lr / bias_correction1   */
    const float SQ = (float)sqrt(1.0 - pow(cfg->beta2, t));          /* sqrt(bias_correction2)  */
    const float EPS = (float)cfg->eps;
    const float DEC = (float)(1.0 - cfg->lr * cfg->weight_decay);
    const float WD = (float)cfg->weight_decay;
    const float IS = (float)(1.0 / cfg->loss_scale);
    const float CLIP = (float)cfg->grad_clip;
    const int has_clip = cfg->grad_clip != 0.0;
    const int has_wd = cfg->weight_decay != 0.0;

    for (uint64_t i = 0; i < n; ++i) {
        uint16_t h16, full;
        load_pair(hi, res, i, &L, &h16, &full);
        float w = merge_one(h16, full, cfg->weight_fmt);
        float g = mpo_ref_cvt16(grad[i], cfg->grad_fmt);
        g = g * IS;
        if (has_clip) {                    /* Sec. 4.1: element-wise clipping inside the step */
            if (g > CLIP) g = CLIP;
            if (g < -CLIP) g = -CLIP;
        }
        if (has_wd) {
            if (cfg->decoupled_wd) {
                w = w * DEC;
            } else {
                float wdw = WD * w;
                g = g + wdw;
            }
        }
        float b1m = B1 * m[i];
        float o1g = O1 * g;
        float m1 = b1m + o1g;
        float b2v = B2 * v[i];
        float o2g = O2 * g;
        float o2gg = o2g * g;
        float v1 = b2v + o2gg;
        float root = sqrtf(v1);
        float rootc = root / SQ;
        float d = rootc + EPS;
        float q = m1 / d;
        float upd = SS * q;
        float w1 = w - upd;
        m[i] = m1;
        v[i] = v1;
        split_one(w1, &h16, &full, cfg->weight_fmt);
        store_pair(hi, res, i, &L, h16, full);
    }
}

/* ---- SGD with momentum (Sec. 3.1; appendix: SGD with momentum, weight decay) */
void mpo_ref_sgd_step(uint16_t *hi, void *res, const uint16_t *grad, float *buf,
                      uint64_t n, const mpo_ref_sgd_cfg *cfg, uint64_t step, uint32_t tensor_id, uint64_t first_index)
{
    /* momentum buffers start at zero, so step 1 needs no special case */
    const res_layout L = make_layout(cfg->weight_fmt, cfg->res_bits, cfg->res_packed, n, cfg->round, cfg->seed, tensor_id, step,
                                     first_index);
    const float LR = (float)cfg->lr;
    const float MU = (float)cfg->momentum;
    const float WD = (float)cfg->weight_decay;
    const float IS = (float)(1.0 / cfg->loss_scale);
    const float CLIP = (float)cfg->grad_clip;
    const int has_clip = cfg->grad_clip != 0.0;
    const int has_wd = cfg->weight_decay != 0.0;
    const int has_mu = cfg->momentum != 0.0;

    for (uint64_t i = 0; i < n; ++i) {
        uint16_t h16, full;
        load_pair(hi, res, i, &L, &h16, &full);
        float w = merge_one(h16, full, cfg->weight_fmt);
        float g = mpo_ref_cvt16(grad[i], cfg->grad_fmt);
        g = g * IS;
        if (has_clip) {                    /* Sec. 4.1: element-wise clipping inside the step */
            if (g > CLIP) g = CLIP;
            if (g < -CLIP) g = -CLIP;
        }
        if (has_wd) {
            float wdw = WD * w;
            g = g + wdw;
        }
        float b = g;
        if (has_mu) {
            float mub = MU * buf[i];
            b = mub + g;
            buf[i] = b;
        }
        float upd = LR * b;
        float w1 = w - upd;
        split_one(w1, &h16, &full, cfg->weight_fmt);
        store_pair(hi, res, i, &L, h16, full);
    }
}
