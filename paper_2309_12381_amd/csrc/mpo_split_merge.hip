/*
 * Split and merge kernels of libmpo (arXiv 2309.12381, Section 3.1, Table 1): fp32 <-> (16-bit
 * float, extra bits), 8 bytes per parameter (7 with byte residuals).  Same row layout as the
 * step kernel (mpo_device.h): 256 lanes per 4096 parameters, 4 parameters per lane per row,
 * each wavefront on a contiguous quarter, non-temporal accesses.
 */
#include <hip/hip_runtime.h>

#include "mpo_device.h"

namespace mpo {
namespace {

/* ---- split / merge: 8 B per parameter (7 B with byte residuals) ------------
 * RND: the 16-bit value is rounded to nearest or stochastically (split) and
 * un-rounded (merge); `rs` carries mode, seed and tensor id, step32 is 0. */

struct RoundArgs {
    uint32_t round, seed_lo, seed_hi, tensor_id;
};

/* split32 with the usual case of fp16 decided for the whole wavefront: when every active lane holds
 * 2^-14 <= |w| < 65536 the payload is the fp32 magnitude with its exponent re-biased and nothing
 * else has to be looked at.  Worth it here, where 8 bytes per parameter leave the vector ALUs a
 * third of the time per parameter that the optimizer step has (with stochastic rounding the
 * fp16 split is bound by them); the step kernel measured faster without the branch. */
template <int FMT> __device__ __forceinline__ void split32_wave(float w, uint32_t &hi, uint32_t &res)
{
    if (FMT == MPO_FP16) {
        const uint32_t b = __float_as_uint(w);
        const uint32_t a = b & 0x7FFFFFFFu;
        if (__all((a - 0x38800000u) < 0x0F000000u)) {
            const uint32_t P = a - 0x38000000u;
            hi = ((b >> 16) & 0x8000u) | (P >> 13);
            res = P & 0x1FFFu;
            return;
        }
    }
    split32<FMT>(w, hi, res);
}

template <int FMT, int RMODE, bool RND>
__device__ __forceinline__ void split_store_one(float w, uint32_t &h, uint32_t &slot, uint32_t kept, uint32_t sh,
                                                uint32_t round, uint32_t u)
{
    uint32_t r;
    split32_wave<FMT>(w, h, r);
    if (RND) slot = reround<FMT>(h, r, kept, sh, round, u);
    else slot = r >> sh;
}

/* w32, hi, res point at the tensor's first parameter; this launch covers chunks from `first`. */
template <int FMT, int RMODE, bool RND, uint32_t ROUND>
__device__ __forceinline__ void split_chunk(const float *__restrict__ w32_, uint16_t *__restrict__ hi_, void *__restrict__ res_,
                                            uint64_t n, uint64_t first, int aligned, uint32_t kept, uint32_t sh,
                                            uint32_t stored, const RoundArgs &rs)
{
    constexpr uint32_t round = ROUND;      /* the rounding mode as a constant: the kernel branches on it once */
    typedef typename ResElem<RMODE>::T R;
    constexpr int RREG = reg_mode(RMODE);
    const uint64_t off = first + (uint64_t)blockIdx.x * kChunkElems;   /* tensor-relative */
    const uint64_t left = n - off;
    const uint32_t len = left < kChunkElems ? (uint32_t)left : kChunkElems;
    gcf32p w32 = (gcf32p)(w32_ + off);
    gu16p hi = (gu16p)(hi_ + off);
    const ResRef ref = res_ref<RMODE>(res_, n, off, stored);
    MPO_GLOBAL R *res = (MPO_GLOBAL R *)ref.slots;
    const Rng rng = {rs.seed_lo, rs.seed_hi, 0u, rs.tensor_id};
    const uint32_t t = threadIdx.x;
    auto one = [&](uint32_t i, uint32_t &h, uint32_t &slot) {
        uint32_t u[4] = {0u, 0u, 0u, 0u};
        if (RND && round == MPO_ROUND_STOCHASTIC) draw4<FullBits<FMT>::value>(rng, (off + i) / 4, u);
        split_store_one<FMT, RREG, RND>(w32[i], h, slot, kept, sh, round, u[(off + i) % 4]);
    };
    if (RMODE == kResPlanes && !(aligned && len == kChunkElems)) {
        /* whole groups of 8 parameters per lane, one parameter at a time; positions past the
         * end are written as zero bits */
        for (uint32_t e = t * 8u; e < len; e += kBlock * 8u) {
            uint32_t ones = 0u;
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const uint32_t eh = e + 4u * half;
                if (eh < len) {
                    uint32_t q[EPL / 2];
#pragma unroll
                    for (int j = 0; j < EPL / 2; ++j) q[j] = 0u;
#pragma unroll
                    for (int k = 0; k < EPL; ++k) {
                        if (eh + k < len) {
                            uint32_t h, slot;
                            one(eh + k, h, slot);
                            hi[eh + k] = (uint16_t)h;
                            q[k / 2] |= (slot & 0xFFFFu) << (16 * (k & 1));
                        }
                    }
                    ones |= planes_pack(ref, eh, q) << (4 * half);
                }
            }
            if (ref.S & 1u) ref.p1[e / 8] = (uint8_t)ones;
        }
        return;
    }
    if (!aligned) {
        for (uint32_t i = t; i < len; i += kBlock) {
            uint32_t h, slot;
            one(i, h, slot);
            hi[i] = (uint16_t)h;
            res[i] = (R)slot;
        }
        return;
    }
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        const uint32_t e = row_elem(r, t);
        if (e + EPL <= len) {
            float w[EPL];
            uint32_t h[EPL / 2], q[EPL / 2];
            load32(w32 + e, w);
#pragma unroll
            for (int j = 0; j < EPL / 2; ++j) q[j] = 0u;
#pragma unroll
            for (int g4 = 0; g4 < EPL / 4; ++g4) {
                uint32_t u[4] = {0u, 0u, 0u, 0u};
                if (RND && round == MPO_ROUND_STOCHASTIC) draw4<FullBits<FMT>::value>(rng, (off + e) / 4 + g4, u);
#pragma unroll
                for (int jj = 0; jj < 2; ++jj) {
                    const int j = 2 * g4 + jj;
                    uint32_t h0, s0, h1, s1;
                    split_store_one<FMT, RREG, RND>(w[2 * j], h0, s0, kept, sh, round, u[2 * jj]);
                    split_store_one<FMT, RREG, RND>(w[2 * j + 1], h1, s1, kept, sh, round, u[2 * jj + 1]);
                    h[j] = h0 | (h1 << 16);
                    slot_put<RREG>(q, 2 * j, s0);
                    slot_put<RREG>(q, 2 * j + 1, s1);
                }
            }
            store16(hi + e, h);
            if (RMODE == kResPlanes) planes_store(ref, e, q);
            else if (RMODE == kResByte) store8((gu8p)res + e, q);
            else store16((gu16p)res + e, q);
        } else if (e < len) {
            for (uint32_t i = e; i < len; ++i) {
                uint32_t h, slot;
                one(i, h, slot);
                hi[i] = (uint16_t)h;
                res[i] = (R)slot;
            }
        }
    }
}

template <int FMT, int RMODE, bool RND>
__global__ void __launch_bounds__(kBlock)
split_kernel(const float *__restrict__ w32, uint16_t *__restrict__ hi, void *__restrict__ res, uint64_t n,
             uint64_t first, int aligned, uint32_t kept, uint32_t sh, uint32_t stored, RoundArgs rs)
{
    if (!RND) split_chunk<FMT, RMODE, RND, MPO_ROUND_TRUNC>(w32, hi, res, n, first, aligned, kept, sh, stored, rs);
    else if (rs.round == MPO_ROUND_STOCHASTIC)
        split_chunk<FMT, RMODE, RND, MPO_ROUND_STOCHASTIC>(w32, hi, res, n, first, aligned, kept, sh, stored, rs);
    else split_chunk<FMT, RMODE, RND, MPO_ROUND_NEAREST>(w32, hi, res, n, first, aligned, kept, sh, stored, rs);
}

template <int FMT, int RMODE, bool RND>
__device__ __forceinline__ float merge_load_one(uint32_t h, uint32_t slot, uint32_t kept, uint32_t sh, uint32_t round)
{
    uint32_t r;
    if (RND) unround<FMT>(h, slot, r, kept, sh, round);
    else r = slot << sh;
    return merge16<FMT>(h, r);
}

template <int FMT, int RMODE, bool RND>
__global__ void __launch_bounds__(kBlock)
merge_kernel(const uint16_t *__restrict__ hi_, const void *__restrict__ res_, float *__restrict__ w32_, uint64_t n,
             uint64_t first, int aligned, uint32_t kept, uint32_t sh, uint32_t stored, uint32_t round)
{
    typedef typename ResElem<RMODE>::T R;
    constexpr int RREG = reg_mode(RMODE);
    const uint64_t off = first + (uint64_t)blockIdx.x * kChunkElems;
    const uint64_t left = n - off;
    const uint32_t len = left < kChunkElems ? (uint32_t)left : kChunkElems;
    gf32p w32 = (gf32p)(w32_ + off);
    gcu16p hi = (gcu16p)(hi_ + off);
    const ResRef ref = res_ref<RMODE>(const_cast<void *>(res_), n, off, stored);
    const MPO_GLOBAL R *res = (const MPO_GLOBAL R *)ref.slots;
    const uint32_t t = threadIdx.x;
    if (RMODE == kResPlanes && !(aligned && len == kChunkElems)) {
        for (uint32_t e = t * 8u; e < len; e += kBlock * 8u) {
            const uint32_t ones = (ref.S & 1u) ? ref.p1[e / 8] : 0u;
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const uint32_t eh = e + 4u * half;
                if (eh < len) {
                    uint32_t q[EPL / 2];
                    planes_unpack(ref, eh, (ones >> (4 * half)) & 0xFu, q);
#pragma unroll
                    for (int k = 0; k < EPL; ++k)
                        if (eh + k < len)
                            w32[eh + k] = merge_load_one<FMT, RREG, RND>(hi[eh + k], slot_get<RREG>(q, k), kept, sh, round);
                }
            }
        }
        return;
    }
    if (!aligned) {
        for (uint32_t i = t; i < len; i += kBlock)
            w32[i] = merge_load_one<FMT, RREG, RND>(hi[i], (uint32_t)res[i], kept, sh, round);
        return;
    }
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        const uint32_t e = row_elem(r, t);
        if (e + EPL <= len) {
            float w[EPL];
            uint32_t h[EPL / 2], q[EPL / 2];
            load16(hi + e, h);
            if (RMODE == kResPlanes) planes_load(ref, e, q);
            else if (RMODE == kResByte) load8((gcu8p)res + e, q);
            else load16((gcu16p)res + e, q);
#pragma unroll
            for (int j = 0; j < EPL / 2; ++j) {
                w[2 * j] = merge_load_one<FMT, RREG, RND>(h[j] & 0xFFFFu, slot_get<RREG>(q, 2 * j), kept, sh, round);
                w[2 * j + 1] = merge_load_one<FMT, RREG, RND>(h[j] >> 16, slot_get<RREG>(q, 2 * j + 1), kept, sh, round);
            }
            store32(w32 + e, w);
        } else if (e < len) {
            for (uint32_t i = e; i < len; ++i)
                w32[i] = merge_load_one<FMT, RREG, RND>(hi[i], (uint32_t)res[i], kept, sh, round);
        }
    }
}

struct SplitMergeArgs {
    const float *w32_in;
    float *w32_out;
    uint16_t *hi;
    void *res;
    uint64_t n;
    int al;
    uint32_t kept, sh, stored;
    RoundArgs rs;
    hipStream_t stream;
};

template <int FMT, int RMODE, bool RND>
hipError_t launch_split_t(const SplitMergeArgs &a)
{
    uint64_t done = 0;
    const uint64_t blocks = (a.n + kChunkElems - 1) / kChunkElems;
    while (done < blocks) {
        const uint64_t now = (blocks - done < kMaxGrid) ? (blocks - done) : kMaxGrid;
        const uint64_t e0 = done * kChunkElems;
        (void)hipGetLastError();
        split_kernel<FMT, RMODE, RND><<<dim3((uint32_t)now), dim3(kBlock), 0, a.stream>>>(
            a.w32_in, a.hi, a.res, a.n, e0, a.al, a.kept, a.sh, a.stored, a.rs);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        done += now;
    }
    return hipSuccess;
}

template <int FMT, int RMODE, bool RND>
hipError_t launch_merge_t(const SplitMergeArgs &a)
{
    uint64_t done = 0;
    const uint64_t blocks = (a.n + kChunkElems - 1) / kChunkElems;
    while (done < blocks) {
        const uint64_t now = (blocks - done < kMaxGrid) ? (blocks - done) : kMaxGrid;
        const uint64_t e0 = done * kChunkElems;
        (void)hipGetLastError();
        merge_kernel<FMT, RMODE, RND><<<dim3((uint32_t)now), dim3(kBlock), 0, a.stream>>>(
            a.hi, a.res, a.w32_out, a.n, e0, a.al, a.kept, a.sh, a.stored, a.rs.round);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        done += now;
    }
    return hipSuccess;
}

template <int FMT, bool SPLIT>
hipError_t launch_sm(const SplitMergeArgs &a, int rmode)
{
    const bool rnd = a.rs.round != MPO_ROUND_TRUNC;
    if (rnd && rmode == kResFull) rmode = kResPartial;     /* rounded modes: general residual path */
#define MPO_SM(RM, RN) (SPLIT ? launch_split_t<FMT, RM, RN>(a) : launch_merge_t<FMT, RM, RN>(a))
    if (rnd) return rmode == kResByte ? MPO_SM(kResByte, true) : rmode == kResPlanes ? MPO_SM(kResPlanes, true) : MPO_SM(kResPartial, true);
    if (rmode == kResPlanes) return MPO_SM(kResPlanes, false);
    if (rmode == kResByte) return MPO_SM(kResByte, false);
    if (rmode == kResPartial) return MPO_SM(kResPartial, false);
    return MPO_SM(kResFull, false);
#undef MPO_SM
}

/* Storage mode, kept bits and number of cut bits for a single-tensor call. */
inline void res_layout(int fmt, int res_bits, int packed, int round, int &rmode, uint32_t &kept, uint32_t &sh,
                       uint32_t &stored)
{
    const int full = full_res_bits(fmt);
    const int k = kept_res_bits(fmt, res_bits, round, packed);
    kept = (uint32_t)k;
    sh = (uint32_t)(full - k);
    stored = packed ? (uint32_t)res_bits : kept;
    rmode = packed ? kResPlanes : (res_bits >= 1 && res_bits <= 8) ? kResByte : (k == full ? kResFull : kResPartial);
}

} // namespace

hipError_t launch_split(const float *w32, uint16_t *hi, void *res, uint64_t n, int fmt, int res_bits, int packed,
                        int round, uint64_t seed, uint32_t tensor_id, hipStream_t stream)
{
    SplitMergeArgs a;
    a.w32_in = w32; a.w32_out = nullptr; a.hi = hi; a.res = res; a.n = n;
    a.al = aligned16(w32) && aligned16(hi) && aligned16(res);
    int rmode;
    res_layout(fmt, res_bits, packed, round, rmode, a.kept, a.sh, a.stored);
    a.rs = RoundArgs{(uint32_t)round, (uint32_t)seed, (uint32_t)(seed >> 32), tensor_id};
    a.stream = stream;
    return fmt == MPO_BF16 ? launch_sm<MPO_BF16, true>(a, rmode) : launch_sm<MPO_FP16, true>(a, rmode);
}

hipError_t launch_merge(const uint16_t *hi, const void *res, float *w32, uint64_t n, int fmt, int res_bits, int packed,
                        int round, hipStream_t stream)
{
    SplitMergeArgs a;
    a.w32_in = nullptr; a.w32_out = w32; a.hi = const_cast<uint16_t *>(hi); a.res = const_cast<void *>(res); a.n = n;
    a.al = aligned16(w32) && aligned16(hi) && aligned16(res);
    int rmode;
    res_layout(fmt, res_bits, packed, round, rmode, a.kept, a.sh, a.stored);
    a.rs = RoundArgs{(uint32_t)round, 0u, 0u, 0u};
    a.stream = stream;
    return fmt == MPO_BF16 ? launch_sm<MPO_BF16, false>(a, rmode) : launch_sm<MPO_FP16, false>(a, rmode);
}

} // namespace mpo
