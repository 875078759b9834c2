/*
 * mpo device code for gfx950 (MI355X), shared by the kernel files (mpo_step.hip,
 * mpo_split_merge.hip): formats, residual storage, rounding and the fused optimizer step.
 *
 * arXiv 2309.12381, Section 3.1: each weight is a 16-bit float plus the
 * significand bits an fp32 copy would have kept; the update runs in fp32 and
 * both parts are written back.  Here the whole step (merge, un-scale, clamp,
 * decay, moments, update, split) is ONE pass over memory: per parameter it
 * reads hi, res, grad (2 B each) and m, v (4 B each) and writes hi, res, m, v:
 * 26 B for Adam, 18 B for SGD with momentum.  Nothing is a contraction, so
 * there is no MFMA; the work is bounded by HBM bandwidth (replacing the
 * arithmetic by a copy does not change the measured time).
 *
 * Mapping: one workgroup of 256 lanes (4 wavefronts of 64) per chunk of 1024
 * (optionally 4096) consecutive parameters of one tensor; the chunk table lets one
 * launch cover every tensor of a list (Section 3.1, "Fused" optimizer).
 *   - A lane owns 4 consecutive parameters per row: 64-bit accesses to the
 *     16-bit arrays and 128-bit accesses to the fp32 arrays, so EVERY load and
 *     store instruction of a wavefront covers one dense span (512 B or 1 KiB)
 *     and no cache line is touched by two instructions.  (8 parameters per lane,
 *     i.e. 128-bit accesses to the 16-bit arrays and two 32-byte-strided
 *     accesses to the fp32 arrays, measured 10 % slower on MI355X.)
 *   - In a long chunk each wavefront owns a contiguous quarter and walks it row
 *     by row.
 *   - One row is in flight per wavefront (5 requests per lane): 44 to 70 vector
 *     registers in every variant, so 7 or 8 wavefronts per SIMD hide the latency.
 *     Requesting all 4 rows of a long chunk first measured the same or slower
 *     (the memory system's queues are full either way) and cost the heavier
 *     variants half their occupancy.
 *   - All accesses carry the non-temporal hint: every byte is used once per step,
 *     and streaming past the caches measured 3-5 % faster than the default policy.
 *
 * Built with -ffp-contract=off and correctly rounded division / square root:
 * every line of arithmetic below is one IEEE binary32 operation.
 */
#ifndef MPO_DEVICE_H
#define MPO_DEVICE_H
#include <hip/hip_runtime.h>

#include "mpo_internal.h"

namespace mpo {
namespace {

constexpr int EPL = 4;                                /* parameters per lane per row   */
constexpr int ROWS = kChunkElems / (kBlock * EPL);    /* rows of the longest chunk */
static_assert(ROWS * kBlock * EPL == kChunkElems, "a chunk is a whole number of rows");
static_assert(kBlock * EPL == kRowElems, "a row is one access of every lane of the workgroup");

/* Every parameter array lives in device (global) memory.  Saying so lets the
 * compiler emit global_load/global_store instead of flat accesses for pointers
 * that were read from a descriptor. */
#define MPO_GLOBAL __attribute__((address_space(1)))
typedef MPO_GLOBAL uint16_t *gu16p;
typedef const MPO_GLOBAL uint16_t *gcu16p;
typedef MPO_GLOBAL uint8_t *gu8p;
typedef const MPO_GLOBAL uint8_t *gcu8p;
typedef MPO_GLOBAL float *gf32p;
typedef const MPO_GLOBAL float *gcf32p;

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

/* Vector accesses of the fast path: non-temporal (streaming) loads and stores. */
template <typename T> __device__ __forceinline__ T ld_stream(const MPO_GLOBAL T *p) { return __builtin_nontemporal_load(p); }
template <typename T> __device__ __forceinline__ void st_stream(MPO_GLOBAL T *p, T x) { __builtin_nontemporal_store(x, p); }

/* 4 x 16 bit = 2 dwords in one access */
__device__ __forceinline__ void load16(gcu16p p, uint32_t (&out)[EPL / 2])
{
    const u32x2 x = ld_stream(reinterpret_cast<const MPO_GLOBAL u32x2 *>(p));
    out[0] = x[0];
    out[1] = x[1];
}
__device__ __forceinline__ void store16(gu16p p, const uint32_t (&in)[EPL / 2])
{
    u32x2 x;
    x[0] = in[0];
    x[1] = in[1];
    st_stream(reinterpret_cast<MPO_GLOBAL u32x2 *>(p), x);
}

/* 4 x 8 bit (byte residuals) = 1 dword; the second register of the pair is unused */
__device__ __forceinline__ void load8(gcu8p p, uint32_t (&out)[EPL / 2])
{
    out[0] = ld_stream(reinterpret_cast<const MPO_GLOBAL uint32_t *>(p));
    out[1] = 0u;
}
__device__ __forceinline__ void store8(gu8p p, const uint32_t (&in)[EPL / 2])
{
    st_stream(reinterpret_cast<MPO_GLOBAL uint32_t *>(p), in[0]);
}

/* 4 x fp32 in one 128-bit access */
__device__ __forceinline__ void load32(gcf32p p, float (&out)[EPL])
{
    const f32x4 x = ld_stream(reinterpret_cast<const MPO_GLOBAL f32x4 *>(p));
#pragma unroll
    for (int i = 0; i < 4; ++i) out[i] = x[i];
}
__device__ __forceinline__ void store32(gf32p p, const float (&in)[EPL])
{
    f32x4 x;
#pragma unroll
    for (int i = 0; i < 4; ++i) x[i] = in[i];
    st_stream(reinterpret_cast<MPO_GLOBAL f32x4 *>(p), x);
}

/* ---- formats (Table 1; Section 3.1) --------------------------------------
 * Both 16-bit values travel in the low half of a dword. */

template <int FMT> __device__ __forceinline__ float merge16(uint32_t hi, uint32_t res);
template <int FMT> __device__ __forceinline__ void split32(float w, uint32_t &hi, uint32_t &res);
template <int FMT> __device__ __forceinline__ float cvt16(uint32_t x);

/* bf16 is the upper half of an fp32 pattern, the residual the lower half. */
template <> __device__ __forceinline__ float merge16<MPO_BF16>(uint32_t hi, uint32_t res)
{
    return __uint_as_float((hi << 16) | res);
}
template <> __device__ __forceinline__ void split32<MPO_BF16>(float w, uint32_t &hi, uint32_t &res)
{
    const uint32_t b = __float_as_uint(w);
    hi = b >> 16;
    res = b & 0xFFFFu;
}
template <> __device__ __forceinline__ float cvt16<MPO_BF16>(uint32_t x)
{
    return __uint_as_float(x << 16);
}

/* fp16 + 13 extra bits.  P = (hi without sign) << 13 | res is a 28-bit payload:
 * 5 exponent bits above a 23-bit fraction, i.e. an fp32 magnitude with the
 * exponent re-biased by 112.  Exponent 0 holds fp16 subnormals: P then counts
 * units of 2^-37.  Exponent 31 is infinity / NaN. */
template <> __device__ __forceinline__ float merge16<MPO_FP16>(uint32_t hi, uint32_t res)
{
    const uint32_t sign = (hi & 0x8000u) << 16;
    const uint32_t P = ((hi & 0x7FFFu) << 13) | (res & 0x1FFFu);
    const uint32_t E = (hi >> 10) & 31u;
    const uint32_t k = hi & 0x3FFu;
    const uint32_t normal = P + 0x38000000u;                  /* exponent + 112 */
    const float sub = (float)P * 0x1p-37f;                    /* exact: P < 2^23 when E == 0 */
    const uint32_t nonfinite = 0x7F800000u | (k ? (0x00400000u | (k << 13)) : 0u);
    uint32_t mag = normal;
    mag = (E == 0u) ? __float_as_uint(sub) : mag;
    mag = (E == 31u) ? nonfinite : mag;
    return __uint_as_float(sign | mag);
}
template <> __device__ __forceinline__ void split32<MPO_FP16>(float w, uint32_t &hi, uint32_t &res)
{
    const uint32_t b = __float_as_uint(w);
    const uint32_t sign = (b >> 16) & 0x8000u;
    const uint32_t a = b & 0x7FFFFFFFu;
    const uint32_t E = a >> 23;
    /* below 2^-14: shift the 24-bit significand down to the 2^-37 grid, toward zero */
    const uint32_t sh = 113u - E;
    const uint32_t sig = (a & 0x7FFFFFu) | 0x800000u;
    const uint32_t F = (E == 0u || sh >= 24u) ? 0u : (sig >> (sh & 31u));
    uint32_t P = (a >= 0x38800000u) ? (a - 0x38000000u) : F;  /* 2^-14 and up: re-bias */
    P = (a >= 0x47800000u) ? 0x0F7FFFFFu : P;                 /* 65536 and up: largest finite pair */
    P = (a == 0x7F800000u) ? 0x0F800000u : P;                 /* infinity */
    P = (a > 0x7F800000u) ? 0x0FC00000u : P;                  /* NaN */
    hi = sign | (P >> 13);
    res = P & 0x1FFFu;
}
template <> __device__ __forceinline__ float cvt16<MPO_FP16>(uint32_t x)
{
    /* every fp16 value is an fp32 value: the hardware conversion is exact (subnormals included;
     * a NaN comes out quiet with its payload, as merge16 builds it) */
    return (float)__builtin_bit_cast(_Float16, (uint16_t)x);
}

/* ---- the update of one parameter (Section 3.1) ---------------------------
 * One IEEE operation per line; the order is part of the definition. */

template <int OPT, int WFMT, int GFMT, int DECAY, bool MOM>
__device__ __forceinline__ void step_one(uint32_t &hi, uint32_t &res, uint32_t g16, float &m, float &v,
                                         const StepScalars &s)
{
    float w = merge16<WFMT>(hi, res);
    float g = cvt16<GFMT>(g16);
    g = g * s.IS;
    /* Section 4.1: element-wise clipping inside the step; the bound is +infinity when off,
     * and a NaN gradient stays NaN */
    g = g > s.CLIP ? s.CLIP : g;
    g = g < -s.CLIP ? -s.CLIP : g;
    if (OPT == MPO_OPT_ADAM) {
        if (DECAY == kDecoupled) {
            w = w * s.DEC;
        } else if (DECAY == kL2) {
            const float wdw = s.WD * w;
            g = g + wdw;
        }
        const float b1m = s.B1 * m;
        const float o1g = s.O1 * g;
        m = b1m + o1g;
        const float b2v = s.B2 * v;
        const float o2g = s.O2 * g;
        const float o2gg = o2g * g;
        v = b2v + o2gg;
        const float root = __builtin_sqrtf(v);
        const float rootc = root / s.SQ;
        const float d = rootc + s.EPS;
        const float q = m / d;
        const float upd = s.SS * q;
        w = w - upd;
    } else {
        if (DECAY == kL2) {
            const float wdw = s.WD * w;
            g = g + wdw;
        }
        float b = g;
        if (MOM) {
            const float mub = s.MU * m;
            b = mub + g;
            m = b;
        }
        const float upd = s.LR * b;
        w = w - upd;
    }
    split32<WFMT>(w, hi, res);
}

/* ---- residual storage (Section 3.1: all extra bits, or only the leading E) --
 * kResFull: 16-bit slots, every bit kept.  kResPartial: 16-bit slots, the kept
 * bits right-aligned, `sh` = number of cut bits.  kResByte: 8-bit slots.
 * In registers the residual of element k of a row sits in x.r[] exactly as in
 * memory; res_get widens it to the full residual (cut bits zero), res_put cuts. */
template <int RMODE> __device__ __forceinline__ uint32_t res_get(const uint32_t *r, int k, uint32_t sh)
{
    if (RMODE == kResByte) return ((r[k / 4] >> (8 * (k % 4))) & 0xFFu) << sh;
    const uint32_t x = (k & 1) ? (r[k / 2] >> 16) : (r[k / 2] & 0xFFFFu);
    return RMODE == kResPartial ? (x << sh) : x;
}
template <int RMODE> __device__ __forceinline__ void res_put(uint32_t *r, int k, uint32_t full, uint32_t sh)
{
    /* r[] is cleared by the caller before the first put of a row */
    if (RMODE == kResByte) r[k / 4] |= ((full >> sh) & 0xFFu) << (8 * (k % 4));
    else r[k / 2] |= (RMODE == kResPartial ? ((full >> sh) & 0xFFFFu) : full) << (16 * (k & 1));
}
template <int RMODE> struct ResElem { typedef uint16_t T; };
template <> struct ResElem<kResByte> { typedef uint8_t T; };

/* ---- packed planes (Section 3.1, Figure 1: extra bits stored without padding) --
 * The S stored bits (the kept bits, plus the flag of stochastic rounding) are cut from the
 * top into the pieces of 8, 4, 2 and 1 bits that S contains, each in a dense plane of its
 * own.  The EPL values of a lane occupy whole bytes of the 8-, 4- and 2-bit planes: no byte
 * is shared between lanes.  In the 1-bit plane two neighbouring lanes share a byte: both
 * load it, and on the way back the even lane fetches its neighbour's four bits with one
 * cross-lane move and stores the byte.  Outside the fast path a lane walks groups of 8
 * values and owns whole bytes of every plane.  In registers the stored bits are held as in
 * a cut 16-bit slot (kResPartial), so the arithmetic path is shared. */
constexpr int reg_mode(int rmode) { return rmode == kResPlanes ? kResPartial : rmode; }

struct ResRef {
    MPO_GLOBAL void *slots;                /* slot storage at the chunk's first parameter  */
    MPO_GLOBAL uint8_t *p8, *p4, *p2, *p1; /* planes at the chunk's first parameter        */
    uint32_t S;                            /* bits stored per value (planes)               */
};

/* base: start of the tensor's residual buffer, n: its length, off: first parameter of the chunk */
template <int RMODE>
__device__ __forceinline__ ResRef res_ref(void *base, uint64_t n, uint64_t off, uint32_t S)
{
    ResRef R;
    R.S = S;
    R.slots = nullptr;
    R.p8 = R.p4 = R.p2 = R.p1 = nullptr;
    if (RMODE == kResPlanes) {
        MPO_GLOBAL uint8_t *b = (MPO_GLOBAL uint8_t *)base;
        R.p8 = b + off;
        if (S & 8u) b += (n + 15u) / 16u * 16u;
        R.p4 = b + off / 2;
        if (S & 4u) b += ((n + 1u) / 2u + 15u) / 16u * 16u;
        R.p2 = b + off / 4;
        if (S & 2u) b += ((n + 3u) / 4u + 15u) / 16u * 16u;
        R.p1 = b + off / 8;
    } else {
        R.slots = (MPO_GLOBAL void *)(static_cast<char *>(base) + off * sizeof(typename ResElem<RMODE>::T));
    }
    return R;
}

/* 1, 2 or 4 bytes of a plane: everything a lane owns of one plane fits a dword.  Where a
 * wavefront covers whole 128-byte lines (2 and 4 bytes per lane) the accesses are streaming
 * like those of the other arrays; single bytes (a wavefront then writes a part of a line, the
 * rest comes from its neighbours) go through the cache with the default policy: measured
 * 2-3 % faster than streaming them. */
template <int NBYTES> __device__ __forceinline__ uint32_t ld_bytes(const MPO_GLOBAL uint8_t *p)
{
    static_assert(NBYTES == 1 || NBYTES == 2 || NBYTES == 4, "a lane owns 4, 2 or 1 bytes of a plane");
    if (NBYTES == 1) return *p;
    if (NBYTES == 2) return ld_stream(reinterpret_cast<const MPO_GLOBAL uint16_t *>(p));
    return ld_stream(reinterpret_cast<const MPO_GLOBAL uint32_t *>(p));
}
template <int NBYTES> __device__ __forceinline__ void st_bytes(MPO_GLOBAL uint8_t *p, uint32_t x)
{
    if (NBYTES == 1) *p = (uint8_t)x;
    else if (NBYTES == 2) st_stream(reinterpret_cast<MPO_GLOBAL uint16_t *>(p), (uint16_t)x);
    else st_stream(reinterpret_cast<MPO_GLOBAL uint32_t *>(p), x);
}

/* The EPL values that start at chunk-local parameter e (a multiple of EPL): the 8-, 4- and
 * 2-bit planes plus `ones`, their EPL bits of the 1-bit plane -> 16-bit pairs. */
__device__ __forceinline__ void planes_unpack(const ResRef &R, uint32_t e, uint32_t ones, uint32_t (&r)[EPL / 2])
{
    const uint32_t b8 = (R.S & 8u) ? ld_bytes<EPL>(R.p8 + e) : 0u;
    const uint32_t b4 = (R.S & 4u) ? ld_bytes<EPL / 2>(R.p4 + e / 2) : 0u;
    const uint32_t b2 = (R.S & 2u) ? ld_bytes<EPL / 4>(R.p2 + e / 4) : 0u;
    /* width of each piece, 0 when S does not contain it (its bits above are then 0 as well): the
     * pieces are joined by shifts by these uniform widths, with no selection per value */
    const uint32_t w4 = R.S & 4u, w2 = R.S & 2u, w1 = R.S & 1u;
#pragma unroll
    for (int j = 0; j < EPL / 2; ++j) r[j] = 0u;
#pragma unroll
    for (int k = 0; k < EPL; ++k) {
        uint32_t x = (b8 >> (8 * k)) & 0xFFu;
        x = (x << w4) | ((b4 >> (4 * k)) & 0xFu);
        x = (x << w2) | ((b2 >> (2 * k)) & 0x3u);
        x = (x << w1) | ((ones >> k) & 1u);
        r[k / 2] |= x << (16 * (k & 1));
    }
}

/* The reverse: stores this lane's bytes of the 8-, 4- and 2-bit planes and returns its EPL
 * bits of the 1-bit plane. */
__device__ __forceinline__ uint32_t planes_pack(const ResRef &R, uint32_t e, const uint32_t (&r)[EPL / 2])
{
    /* width and position (from the low end of the S bits) of each piece; a bit field of width 0 is 0 */
    const uint32_t w8 = R.S & 8u, w4 = R.S & 4u, w2 = R.S & 2u, w1 = R.S & 1u;
    const uint32_t o8 = R.S - w8, o4 = o8 - w4, o2 = o4 - w2;
    uint32_t b8 = 0u, b4 = 0u, b2 = 0u, ones = 0u;
#pragma unroll
    for (int k = 0; k < EPL; ++k) {
        const uint32_t x = (r[k / 2] >> (16 * (k & 1))) & 0xFFFFu;
        b8 |= __builtin_amdgcn_ubfe(x, o8, w8) << (8 * k);
        b4 |= __builtin_amdgcn_ubfe(x, o4, w4) << (4 * k);
        b2 |= __builtin_amdgcn_ubfe(x, o2, w2) << (2 * k);
        ones |= (x & w1) << k;
    }
    if (R.S & 8u) st_bytes<EPL>(R.p8 + e, b8);
    if (R.S & 4u) st_bytes<EPL / 2>(R.p4 + e / 2, b4);
    if (R.S & 2u) st_bytes<EPL / 4>(R.p2 + e / 4, b2);
    return ones;
}

static_assert(EPL == 4, "two lanes share a byte of the 1-bit plane");

/* Fast path, every lane of the wavefront active, lane t at e = ... + 4 * (t % 64): the byte of
 * the 1-bit plane is shared by lanes 2k and 2k+1. */
__device__ __forceinline__ void planes_load(const ResRef &R, uint32_t e, uint32_t (&r)[EPL / 2])
{
    const uint32_t ones = (R.S & 1u) ? (ld_bytes<1>(R.p1 + e / 8) >> (e & 4u)) & 0xFu : 0u;
    planes_unpack(R, e, ones, r);
}

__device__ __forceinline__ void planes_store(const ResRef &R, uint32_t e, const uint32_t (&r)[EPL / 2])
{
    const uint32_t ones = planes_pack(R, e, r);
    if (R.S & 1u) {
        const uint32_t other = (uint32_t)__shfl_xor((int)ones, 1);
        if (!(e & 4u)) st_bytes<1>(R.p1 + e / 8, ones | (other << 4));
    }
}

template <int WFMT> struct FullBits { static constexpr uint32_t value = (WFMT == MPO_FP16) ? 13u : 16u; };
/* 16-bit pattern of infinity without the sign: everything above it is a NaN */
template <int WFMT> struct InfBits { static constexpr uint32_t value = (WFMT == MPO_FP16) ? 0x7C00u : 0x7F80u; };

/* ---- rounding of the 16-bit value (Section 3.1, last paragraph) -------------
 * Philox4x32-10 (Salmon et al., SC'11): counter-based, so every lane computes
 * the four words of its own four parameters and nothing is stored. */
struct Rng {
    uint32_t seed_lo, seed_hi, step32, tensor_id;
};

/* a ^ b ^ c in one instruction (the three-input bit operation of gfx950, truth table 0x96) */
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c)
{
    return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                              uint32_t k1, uint32_t (&out)[4])
{
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        if (round > 0) {
            k0 += 0x9E3779B9u;
            k1 += 0xBB67AE85u;
        }
        /* one 32 x 32 -> 64 bit product per multiplier: both halves from one instruction */
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t h0 = (uint32_t)(p0 >> 32), l0 = (uint32_t)p0;
        const uint32_t h1 = (uint32_t)(p1 >> 32), l1 = (uint32_t)p1;
        const uint32_t n0 = xor3(h1, c1, k0), n2 = xor3(h0, c3, k1);
        c0 = n0; c1 = l1; c2 = n2; c3 = l0;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The four draws of parameters 4*block .. 4*block+3 of a tensor, each in [0, 2^FULL). */
template <uint32_t FULL>
__device__ __forceinline__ void draw4(const Rng &g, uint64_t block, uint32_t (&u)[4])
{
    philox4x32_10((uint32_t)block, (uint32_t)(block >> 32), g.step32, g.tensor_id, g.seed_lo, g.seed_hi, u);
#pragma unroll
    for (int j = 0; j < 4; ++j) u[j] >>= (32u - FULL);
}

/* What a stored (hi, slot) pair means: the truncated 16-bit value and the full residual. */
template <int WFMT>
__device__ __forceinline__ void unround(uint32_t &hi, uint32_t slot, uint32_t &res_full, uint32_t kept, uint32_t sh,
                                        uint32_t round)
{
    constexpr uint32_t FULL = FullBits<WFMT>::value;
    res_full = (slot & ((1u << kept) - 1u)) << sh;
    /* round-to-nearest never touches a NaN pattern: a NaN stays a NaN in what forward sees */
    const uint32_t is_nan = ((hi & 0x7FFFu) > InfBits<WFMT>::value) ? 1u : 0u;
    const uint32_t flag = (round == MPO_ROUND_STOCHASTIC) ? ((slot >> kept) & 1u)
                        : (round == MPO_ROUND_NEAREST)    ? (((res_full >> (FULL - 1u)) & 1u) & ~is_nan) : 0u;
    hi = (hi - flag) & 0xFFFFu;
}

/* The reverse: round the truncated value and build the slot.  `u` is this parameter's draw. */
template <int WFMT>
__device__ __forceinline__ uint32_t reround(uint32_t &hi, uint32_t res_full, uint32_t kept, uint32_t sh, uint32_t round,
                                            uint32_t u)
{
    constexpr uint32_t FULL = FullBits<WFMT>::value;
    constexpr uint32_t MAXFIN = (WFMT == MPO_FP16) ? 0x7BFFu : 0x7F7Fu;
    uint32_t up = 0u;
    if (round == MPO_ROUND_NEAREST) up = ((hi & 0x7FFFu) > InfBits<WFMT>::value) ? 0u : ((res_full >> (FULL - 1u)) & 1u);
    if (round == MPO_ROUND_STOCHASTIC) up = ((hi & 0x7FFFu) < MAXFIN && u < res_full) ? 1u : 0u;
    hi = (hi + up) & 0xFFFFu;
    uint32_t slot = res_full >> sh;
    if (round == MPO_ROUND_STOCHASTIC) slot |= up << kept;
    return slot;
}

/* raw slot k of a row as it sits in registers / memory */
template <int RMODE> __device__ __forceinline__ uint32_t slot_get(const uint32_t *r, int k)
{
    if (RMODE == kResByte) return (r[k / 4] >> (8 * (k % 4))) & 0xFFu;
    return (k & 1) ? (r[k / 2] >> 16) : (r[k / 2] & 0xFFFFu);
}
template <int RMODE> __device__ __forceinline__ void slot_put(uint32_t *r, int k, uint32_t slot)
{
    if (RMODE == kResByte) r[k / 4] |= (slot & 0xFFu) << (8 * (k % 4));
    else r[k / 2] |= (slot & 0xFFFFu) << (16 * (k & 1));
}

template <int OPT, bool MOM> struct Uses {
    static constexpr bool m = (OPT == MPO_OPT_ADAM) || MOM;
    static constexpr bool v = (OPT == MPO_OPT_ADAM);
};

/* First parameter (within the chunk) of row r for lane t.  Each wavefront owns one
 * contiguous quarter of the chunk and walks it row by row, so the rows one wavefront
 * requests from a stream are adjacent in memory (measured ~5 % faster than rows
 * interleaved across the four wavefronts). */
__device__ __forceinline__ uint32_t row_elem(uint32_t r, uint32_t t, uint32_t span = kChunkElems / (kBlock / 64))
{
    /* span: the wavefront's share of the chunk (a quarter of its length) */
    return (t / 64) * span + r * (64 * EPL) + (t % 64) * EPL;
}

struct Row {
    uint32_t h[EPL / 2], r[EPL / 2], g[EPL / 2];
    float m[EPL], v[EPL];
};

template <int OPT, bool MOM, int RMODE>
__device__ __forceinline__ void load_row(Row &x, gcu16p hi, const ResRef &R, gcu16p grad, gcf32p m, gcf32p v, uint32_t e)
{
    load16(hi + e, x.h);
    if (RMODE == kResPlanes) planes_load(R, e, x.r);
    else if (RMODE == kResByte) load8(static_cast<gcu8p>(R.slots) + e, x.r);
    else load16(static_cast<gcu16p>(R.slots) + e, x.r);
    load16(grad + e, x.g);
    if (Uses<OPT, MOM>::m) load32(m + e, x.m);
    if (Uses<OPT, MOM>::v) load32(v + e, x.v);
}

/* The same with the 16-bit value rounded to nearest or stochastically: un-round, update,
 * round again with this step's draws.  `first` is the tensor-relative index of the row's
 * first parameter (a multiple of 4). */
template <int OPT, int WFMT, int GFMT, int DECAY, bool MOM, int RMODE>
__device__ __forceinline__ void compute_row_rounded(Row &x, const StepScalars &s, uint32_t kept, uint32_t sh,
                                                    const Rng &g, uint64_t first, uint32_t round)
{
    uint32_t rin[EPL / 2];
#pragma unroll
    for (int j = 0; j < EPL / 2; ++j) { rin[j] = x.r[j]; x.r[j] = 0u; }
#pragma unroll
    for (int q = 0; q < EPL / 4; ++q) {
        uint32_t u[4] = {0u, 0u, 0u, 0u};
        if (round == MPO_ROUND_STOCHASTIC) draw4<FullBits<WFMT>::value>(g, first / 4 + q, u);
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            const int j = 2 * q + jj;
            uint32_t h0 = x.h[j] & 0xFFFFu, h1 = x.h[j] >> 16, r0, r1;
            unround<WFMT>(h0, slot_get<RMODE>(rin, 2 * j), r0, kept, sh, round);
            unround<WFMT>(h1, slot_get<RMODE>(rin, 2 * j + 1), r1, kept, sh, round);
            step_one<OPT, WFMT, GFMT, DECAY, MOM>(h0, r0, x.g[j] & 0xFFFFu, x.m[2 * j], x.v[2 * j], s);
            step_one<OPT, WFMT, GFMT, DECAY, MOM>(h1, r1, x.g[j] >> 16, x.m[2 * j + 1], x.v[2 * j + 1], s);
            const uint32_t s0 = reround<WFMT>(h0, r0, kept, sh, round, u[2 * jj]);
            const uint32_t s1 = reround<WFMT>(h1, r1, kept, sh, round, u[2 * jj + 1]);
            x.h[j] = h0 | (h1 << 16);
            slot_put<RMODE>(x.r, 2 * j, s0);
            slot_put<RMODE>(x.r, 2 * j + 1, s1);
        }
    }
}

template <int OPT, int WFMT, int GFMT, int DECAY, bool MOM, int RMODE>
__device__ __forceinline__ void compute_row(Row &x, const StepScalars &s, uint32_t sh)
{
    uint32_t rin[EPL / 2];
#pragma unroll
    for (int j = 0; j < EPL / 2; ++j) { rin[j] = x.r[j]; x.r[j] = 0u; }
#pragma unroll
    for (int j = 0; j < EPL / 2; ++j) {
        uint32_t h0 = x.h[j] & 0xFFFFu, h1 = x.h[j] >> 16;
        uint32_t r0 = res_get<RMODE>(rin, 2 * j, sh), r1 = res_get<RMODE>(rin, 2 * j + 1, sh);
        step_one<OPT, WFMT, GFMT, DECAY, MOM>(h0, r0, x.g[j] & 0xFFFFu, x.m[2 * j], x.v[2 * j], s);
        step_one<OPT, WFMT, GFMT, DECAY, MOM>(h1, r1, x.g[j] >> 16, x.m[2 * j + 1], x.v[2 * j + 1], s);
        x.h[j] = h0 | (h1 << 16);
        res_put<RMODE>(x.r, 2 * j, r0, sh);
        res_put<RMODE>(x.r, 2 * j + 1, r1, sh);
    }
}

template <int OPT, bool MOM, int RMODE>
__device__ __forceinline__ void store_row(const Row &x, gu16p hi, const ResRef &R, gf32p m, gf32p v, uint32_t e)
{
    store16(hi + e, x.h);
    if (RMODE == kResPlanes) planes_store(R, e, x.r);
    else if (RMODE == kResByte) store8(static_cast<gu8p>(R.slots) + e, x.r);
    else store16(static_cast<gu16p>(R.slots) + e, x.r);
    if (Uses<OPT, MOM>::m) store32(m + e, x.m);
    if (Uses<OPT, MOM>::v) store32(v + e, x.v);
}

/* Parameters [e0, e1) one at a time: ragged tails and tensors that are not
 * 16-byte aligned.  Same arithmetic, 16- and 32-bit accesses. */
template <int OPT, int WFMT, int GFMT, int DECAY, bool MOM, int RMODE>
__device__ __forceinline__ void step_scalar(gu16p hi, MPO_GLOBAL void *res_, gcu16p grad, gf32p m, gf32p v, uint32_t e,
                                            const StepScalars &s, uint32_t sh)
{
    MPO_GLOBAL typename ResElem<RMODE>::T *res = static_cast<MPO_GLOBAL typename ResElem<RMODE>::T *>(res_);
    uint32_t h = hi[e], r = (uint32_t)res[e] << sh;
    float mm = Uses<OPT, MOM>::m ? m[e] : 0.0f;
    float vv = Uses<OPT, MOM>::v ? v[e] : 0.0f;
    step_one<OPT, WFMT, GFMT, DECAY, MOM>(h, r, grad[e], mm, vv, s);
    hi[e] = (uint16_t)h;
    res[e] = (typename ResElem<RMODE>::T)(r >> sh);
    if (Uses<OPT, MOM>::m) m[e] = mm;
    if (Uses<OPT, MOM>::v) v[e] = vv;
}

/* Packed planes outside the fast path: the (up to) 8 parameters that start at chunk-local
 * parameter e (a multiple of 8), one at a time: ragged ends and tensors whose other arrays are
 * not 16-byte aligned.  The lane owns whole bytes of every plane (the planes are padded to 16
 * bytes); bits of positions past the end are written back as they were read. */
template <int OPT, int WFMT, int GFMT, int DECAY, bool MOM, bool RND>
__device__ __forceinline__ void step_group_planes(gu16p hi, const ResRef &R, gcu16p grad, gf32p m, gf32p v, uint32_t e,
                                                  uint32_t len, const StepScalars &s, uint32_t kept, uint32_t sh,
                                                  const Rng &g, uint64_t off, uint32_t round)
{
    uint32_t ones = (R.S & 1u) ? R.p1[e / 8] : 0u;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        const uint32_t eh = e + 4u * half;
        if (eh < len) {
            uint32_t r[EPL / 2];
            planes_unpack(R, eh, (ones >> (4 * half)) & 0xFu, r);
            uint32_t u[4] = {0u, 0u, 0u, 0u};
            if (RND && round == MPO_ROUND_STOCHASTIC) draw4<FullBits<WFMT>::value>(g, (off + eh) / 4, u);
#pragma unroll
            for (int k = 0; k < EPL; ++k) {
                if (eh + k < len) {
                    uint32_t h = hi[eh + k], rr;
                    uint32_t slot = (r[k / 2] >> (16 * (k & 1))) & 0xFFFFu;
                    if (RND) unround<WFMT>(h, slot, rr, kept, sh, round);
                    else rr = slot << sh;
                    float mm = Uses<OPT, MOM>::m ? m[eh + k] : 0.0f;
                    float vv = Uses<OPT, MOM>::v ? v[eh + k] : 0.0f;
                    step_one<OPT, WFMT, GFMT, DECAY, MOM>(h, rr, grad[eh + k], mm, vv, s);
                    if (RND) slot = reround<WFMT>(h, rr, kept, sh, round, u[k]);
                    else slot = rr >> sh;
                    hi[eh + k] = (uint16_t)h;
                    if (Uses<OPT, MOM>::m) m[eh + k] = mm;
                    if (Uses<OPT, MOM>::v) v[eh + k] = vv;
                    r[k / 2] = (r[k / 2] & ~(0xFFFFu << (16 * (k & 1)))) | ((slot & 0xFFFFu) << (16 * (k & 1)));
                }
            }
            const uint32_t out = planes_pack(R, eh, r);
            ones = (ones & ~(0xFu << (4 * half))) | (out << (4 * half));
        }
    }
    if (R.S & 1u) R.p1[e / 8] = (uint8_t)ones;
}

template <int OPT, int WFMT, int GFMT, int DECAY, bool MOM, int RMODE>
__device__ __forceinline__ void step_scalar_rounded(gu16p hi, MPO_GLOBAL void *res_, gcu16p grad, gf32p m, gf32p v,
                                                    uint32_t e, const StepScalars &s, uint32_t kept, uint32_t sh,
                                                    const Rng &g, uint64_t index, uint32_t round)
{
    MPO_GLOBAL typename ResElem<RMODE>::T *res = static_cast<MPO_GLOBAL typename ResElem<RMODE>::T *>(res_);
    uint32_t h = hi[e], r;
    unround<WFMT>(h, (uint32_t)res[e], r, kept, sh, round);
    float mm = Uses<OPT, MOM>::m ? m[e] : 0.0f;
    float vv = Uses<OPT, MOM>::v ? v[e] : 0.0f;
    step_one<OPT, WFMT, GFMT, DECAY, MOM>(h, r, grad[e], mm, vv, s);
    uint32_t u[4] = {0u, 0u, 0u, 0u};
    if (round == MPO_ROUND_STOCHASTIC) draw4<FullBits<WFMT>::value>(g, index / 4, u);
    const uint32_t slot = reround<WFMT>(h, r, kept, sh, round, u[index % 4]);
    hi[e] = (uint16_t)h;
    res[e] = (typename ResElem<RMODE>::T)slot;
    if (Uses<OPT, MOM>::m) m[e] = mm;
    if (Uses<OPT, MOM>::v) v[e] = vv;
}

/* How a launch gets its gradient pointers: from the descriptors, or (Section 3.2, per-call
 * pointers of one layer) from the kernel arguments. */
template <bool OV> struct OvArg { typedef NoOverride T; };
template <> struct OvArg<true> { typedef GradOverride T; };

/* One chunk per workgroup.  ROUND is the rounding mode as a constant (the kernel branches on
 * the uniform s.round once, so the loops hold the code of one mode only). */
template <int OPT, int WFMT, int GFMT, int DECAY, bool MOM, int RMODE, bool RND, bool OV, uint32_t ROUND>
__device__ __forceinline__ void step_chunk(const TensorDesc *__restrict__ descs, const Chunk *__restrict__ chunks,
                                           uint64_t first_chunk, const StepScalars &s, const typename OvArg<OV>::T &ov)
{
    constexpr uint32_t round = ROUND;
    /* Uniform per workgroup: scalar loads. */
    const Chunk c = chunks[first_chunk + blockIdx.x];
    const TensorDesc d = descs[c.tensor];
    const uint16_t *gbase = d.grad;
    bool aligned = (d.flags & (kStateAligned | kGradAligned)) == (kStateAligned | kGradAligned);
    if constexpr (OV) {
        const uint32_t k = c.tensor - ov.first;
        gbase = ov.ptr[k];
        aligned = (d.flags & kStateAligned) && !((ov.misaligned >> k) & 1ull);
    }
    const uint32_t rows = 1u << (c.where >> kChunkStartBits);      /* 1, 2 or 4 */
    const uint32_t celems = rows * kRowElems;
    const uint32_t span = celems / (kBlock / 64);                  /* a wavefront's contiguous share */
    const uint64_t off = (uint64_t)(c.where & kChunkStartMask) * kRowElems;
    const uint64_t left = d.n - off;
    const uint32_t len = left < celems ? (uint32_t)left : celems;

    /* cut bits of this tensor's residual (uniform); a full residual has none */
    const uint32_t all = (RND && round == MPO_ROUND_STOCHASTIC && WFMT == MPO_BF16) ? 15u : FullBits<WFMT>::value;
    const uint32_t stored = d.res_bits ? d.res_bits : all;
    /* in the planes the flag of stochastic rounding is the leading one of the stored bits */
    const uint32_t kept = (RMODE == kResPlanes && RND && round == MPO_ROUND_STOCHASTIC) ? stored - 1u : stored;
    const uint32_t sh = (RMODE == kResFull && !RND) ? 0u : FullBits<WFMT>::value - kept;
    const Rng rng = {s.seed_lo, s.seed_hi, s.step32, d.tensor_id};
    gu16p hi = (gu16p)(d.hi + off);
    const ResRef R = res_ref<RMODE>(d.res, d.n, off, stored);
    MPO_GLOBAL void *res = R.slots;
    constexpr int RREG = reg_mode(RMODE);          /* how the kept bits sit in registers */
    gcu16p grad = (gcu16p)(gbase + off);
    gf32p m = Uses<OPT, MOM>::m ? (gf32p)(d.m + off) : (gf32p) nullptr;
    gf32p v = Uses<OPT, MOM>::v ? (gf32p)(d.v + off) : (gf32p) nullptr;
    const uint32_t t = threadIdx.x;

    if (aligned && len == celems) {
        /* whole chunk: row by row, every lane active, no bounds checks.  One row in flight per
         * wavefront keeps the register count low enough for 8 wavefronts per SIMD in every
         * variant of the kernel, and they hide the latency: measured the same as, or faster
         * than, requesting all rows of a long chunk before the first is used. */
#pragma unroll 1
        for (uint32_t r = 0; r < rows; ++r) {
            const uint32_t e = row_elem(r, t, span);
            Row x;
            load_row<OPT, MOM, RMODE>(x, hi, R, grad, m, v, e);
            if (RND) compute_row_rounded<OPT, WFMT, GFMT, DECAY, MOM, RREG>(x, s, kept, sh, rng, off + e, round);
            else compute_row<OPT, WFMT, GFMT, DECAY, MOM, RREG>(x, s, sh);
            store_row<OPT, MOM, RMODE>(x, hi, R, m, v, e);
        }
    } else if (RMODE == kResPlanes) {
        /* packed planes outside the fast path: every lane walks whole groups of 8 parameters */
        for (uint32_t e = t * 8u; e < len; e += kBlock * 8u)
            step_group_planes<OPT, WFMT, GFMT, DECAY, MOM, RND>(hi, R, grad, m, v, e, len, s, kept, sh, rng, off, round);
    } else if (aligned) {
        /* last chunk of a tensor: full vectors, then one lane finishes the ragged end */
#pragma unroll 1
        for (uint32_t r = 0; r < rows; ++r) {
            const uint32_t e = row_elem(r, t, span);
            if (e + EPL <= len) {
                Row x;
                load_row<OPT, MOM, RMODE>(x, hi, R, grad, m, v, e);
                if (RND) compute_row_rounded<OPT, WFMT, GFMT, DECAY, MOM, RREG>(x, s, kept, sh, rng, off + e, round);
                else compute_row<OPT, WFMT, GFMT, DECAY, MOM, RREG>(x, s, sh);
                store_row<OPT, MOM, RMODE>(x, hi, R, m, v, e);
            } else if (e < len) {
                for (uint32_t i = e; i < len; ++i) {
                    if (RND) step_scalar_rounded<OPT, WFMT, GFMT, DECAY, MOM, RMODE>(hi, res, grad, m, v, i, s, kept, sh, rng, off + i, round);
                    else step_scalar<OPT, WFMT, GFMT, DECAY, MOM, RMODE>(hi, res, grad, m, v, i, s, sh);
                }
            }
        }
    } else {
        for (uint32_t i = t; i < len; i += kBlock) {
            if (RND) step_scalar_rounded<OPT, WFMT, GFMT, DECAY, MOM, RMODE>(hi, res, grad, m, v, i, s, kept, sh, rng, off + i, round);
            else step_scalar<OPT, WFMT, GFMT, DECAY, MOM, RMODE>(hi, res, grad, m, v, i, s, sh);
        }
    }
}

template <int OPT, int WFMT, int GFMT, int DECAY, bool MOM, int RMODE, bool RND, bool OV>
__global__ void __launch_bounds__(kBlock)
step_kernel(const TensorDesc *__restrict__ descs, const Chunk *__restrict__ chunks, uint64_t first_chunk,
            StepScalars s, typename OvArg<OV>::T ov)
{
    if (!RND)
        step_chunk<OPT, WFMT, GFMT, DECAY, MOM, RMODE, RND, OV, MPO_ROUND_TRUNC>(descs, chunks, first_chunk, s, ov);
    else if (s.round == MPO_ROUND_STOCHASTIC)
        step_chunk<OPT, WFMT, GFMT, DECAY, MOM, RMODE, RND, OV, MPO_ROUND_STOCHASTIC>(descs, chunks, first_chunk, s, ov);
    else
        step_chunk<OPT, WFMT, GFMT, DECAY, MOM, RMODE, RND, OV, MPO_ROUND_NEAREST>(descs, chunks, first_chunk, s, ov);
}

/* Grids are limited to 2^31-1 workgroups: longer lists go out in slices. */
constexpr uint64_t kMaxGrid = 0x7FFFFFFFull;

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

} // namespace
} // namespace mpo
#endif /* MPO_DEVICE_H */
