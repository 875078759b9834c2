/*
 * Host side of libmpo: the C entry points declared in include/mpo.h.
 * Argument validation, overlap detection, the multi-tensor plan (layer order,
 * chunk table, descriptors) and the per-step scalars.  No arithmetic on
 * parameters happens here; every step of the method runs in the kernels
 * (mpo_device.h).  Only plan creation allocates; the step, split and merge
 * entry points use fixed-size stack storage.
 */
#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <vector>

#include <hip/hip_runtime_api.h>

#include "mpo_internal.h"

namespace mpo {

namespace {

thread_local int g_last_hip_error = 0;

bool valid_fmt(int f) { return f == MPO_BF16 || f == MPO_FP16; }

mpo_status check_round(int r)
{
    return (r == MPO_ROUND_TRUNC || r == MPO_ROUND_NEAREST || r == MPO_ROUND_STOCHASTIC) ? MPO_OK : MPO_ERR_INVALID_ARG;
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

/* Section 3.1, partial extra bits: at most 8 kept bits live in a byte, more in 16 bits. */
inline uint32_t res_slot_bytes(int res_bits) { return (res_bits >= 1 && res_bits <= 8) ? 1u : 2u; }

/* Packed planes: 1 to 15 stored bits per value (Figure 1 of the paper has 12). */
inline bool valid_packed_bits(int res_bits) { return res_bits >= 1 && res_bits <= 15; }

/* Packed planes with a format and a rounding mode: at least one kept bit, at most all of them. */
inline bool valid_packed_mode(int res_bits, int fmt, int round)
{
    const int kept = kept_res_bits(fmt, res_bits, round, 1);
    return valid_packed_bits(res_bits) && kept >= 1 && kept <= full_res_bits(fmt);
}

/* Kind of residual storage: 1 = bytes, 2 = 16-bit slots, 3 = packed planes. */
inline uint32_t res_kind(int res_bits, int packed) { return packed ? 3u : res_slot_bytes(res_bits); }

/* Slots: 0 means all; otherwise 1..full for the format.  Stochastic rounding stores one flag
 * above the kept bits: they must leave room for it in the slot. */
inline bool valid_res_bits(int res_bits, int fmt, int round)
{
    if (res_bits < 0 || res_bits > full_res_bits(fmt)) return false;
    if (round != MPO_ROUND_STOCHASTIC) return true;
    return kept_res_bits(fmt, res_bits, round, 0) + 1 <= 8 * (int)res_slot_bytes(res_bits);
}

bool finite_pos(double x) { return std::isfinite(x) && x > 0.0; }

} // namespace

mpo_status hip_fail(hipError_t e)
{
    g_last_hip_error = (int)e;
    return e == hipErrorOutOfMemory ? MPO_ERR_NOMEM : MPO_ERR_HIP;
}

/* True if some written range overlaps any other range.  Read-only ranges
 * (gradients) may overlap each other: one buffer reused for every layer. */
bool has_conflict(Range *r, uint64_t count)
{
    std::sort(r, r + count, [](const Range &a, const Range &b) { return a.lo < b.lo; });
    /* sweep: furthest end seen so far among all ranges and among written ranges */
    uintptr_t end_any = 0, end_written = 0;
    bool first = true;
    for (uint64_t i = 0; i < count; ++i) {
        const Range &x = r[i];
        if (x.lo == x.hi) continue;
        if (!first) {
            if (x.written && x.lo < end_any) return true;
            if (!x.written && x.lo < end_written) return true;
        }
        first = false;
        end_any = std::max(end_any, x.hi);
        if (x.written) end_written = std::max(end_written, x.hi);
    }
    return false;
}

mpo_status check_tensor(const mpo_tensor &t, uint32_t &res_slot, Range *r, uint64_t *count)
{
    if (t.layer < 0) return MPO_ERR_INVALID_ARG;
    if (t.n >= kMaxTensorElems) return MPO_ERR_INVALID_ARG;
    if (t.res_bits < 0 || t.res_bits > 16) return MPO_ERR_INVALID_ARG;
    if (t.res_packed && !valid_packed_bits(t.res_bits)) return MPO_ERR_INVALID_ARG;
    if (t.n == 0) return MPO_OK;
    if (!t.hi || !t.res) return MPO_ERR_INVALID_ARG;
    if (t.res_packed && !aligned16(t.res)) return MPO_ERR_INVALID_ARG;
    const uint32_t slot = res_kind(t.res_bits, t.res_packed);
    if (res_slot == 0) res_slot = slot;
    else if (res_slot != slot) return MPO_ERR_UNSUPPORTED;
    auto add = [&](const void *p, uint64_t bytes, bool written) {
        const uintptr_t lo = reinterpret_cast<uintptr_t>(p);
        r[(*count)++] = Range{lo, lo + bytes, written};
    };
    add(t.hi, t.n * 2, true);
    add(t.res, res_bytes(t.n, t.res_bits, t.res_packed), true);
    if (t.grad) add(t.grad, t.n * 2, false);
    if (t.m) add(t.m, t.n * 4, true);
    if (t.v) add(t.v, t.n * 4, true);
    return MPO_OK;
}

TensorDesc make_desc(const mpo_tensor &t, uint32_t tensor_id)
{
    TensorDesc d;
    std::memset(&d, 0, sizeof d);
    d.hi = t.hi; d.res = t.res; d.grad = t.grad; d.m = t.m; d.v = t.v; d.n = t.n;
    d.res_bits = (uint32_t)t.res_bits;
    d.tensor_id = tensor_id;
    if (aligned16(t.hi) && aligned16(t.res) && aligned16(t.m) && aligned16(t.v)) d.flags |= kStateAligned;
    if (t.grad && aligned16(t.grad)) d.flags |= kGradAligned;
    return d;
}

uint64_t layout_chunks(const TensorDesc *descs, const int32_t *layer, uint64_t nt, uint64_t small_layer_params,
                       TensorLayout *lay)
{
    uint64_t pos = 0;
    for (uint64_t k0 = 0; k0 < nt;) {
        uint64_t k1 = k0, params = 0;
        while (k1 < nt && layer[k1] == layer[k0]) params += descs[k1++].n;
        const uint32_t rl = layer_rows_log2(params, small_layer_params);
        const uint64_t celems = (uint64_t)kRowElems << rl;
        /* the layer's ragged chunks first, then the full chunks tensor by tensor */
        for (uint64_t k = k0; k < k1; ++k) {
            if (descs[k].n >= kMaxTensorElems) return UINT64_MAX;
            lay[k].rows_log2 = rl;
            lay[k].num_full = descs[k].n / celems;
            lay[k].has_ragged = descs[k].n % celems != 0;
            lay[k].ragged_pos = pos;
            pos += lay[k].has_ragged;
        }
        for (uint64_t k = k0; k < k1; ++k) {
            lay[k].full_pos = pos;
            pos += lay[k].num_full;
        }
        k0 = k1;
    }
    return pos;
}

/* Adam scalars: formed in double, rounded to fp32 once (Section 3.1: classic Adam). */
mpo_status adam_scalars(const mpo_adam_cfg *c, uint64_t step, StepLaunch &L)
{
    if (!c || step == 0) return MPO_ERR_INVALID_ARG;
    if (!valid_fmt(c->weight_fmt) || !valid_fmt(c->grad_fmt)) return MPO_ERR_INVALID_ARG;
    const mpo_status rs = check_round(c->round);
    if (rs != MPO_OK) return rs;
    if (!std::isfinite(c->lr) || !std::isfinite(c->eps) || !std::isfinite(c->weight_decay)) return MPO_ERR_INVALID_ARG;
    if (!(c->beta1 >= 0.0 && c->beta1 < 1.0) || !(c->beta2 >= 0.0 && c->beta2 < 1.0)) return MPO_ERR_INVALID_ARG;
    if (!finite_pos(c->loss_scale)) return MPO_ERR_INVALID_ARG;
    if (!(c->grad_clip >= 0.0) || !std::isfinite(c->grad_clip)) return MPO_ERR_INVALID_ARG;
    const double t = (double)step;
    const double bc1 = 1.0 - std::pow(c->beta1, t);
    const double bc2 = 1.0 - std::pow(c->beta2, t);
    StepScalars &s = L.s;
    std::memset(&s, 0, sizeof s);
    s.B1 = (float)c->beta1;
    s.B2 = (float)c->beta2;
    s.O1 = (float)(1.0 - c->beta1);
    s.O2 = (float)(1.0 - c->beta2);
    s.SS = (float)(c->lr / bc1);
    s.SQ = (float)std::sqrt(bc2);
    s.EPS = (float)c->eps;
    s.DEC = (float)(1.0 - c->lr * c->weight_decay);
    s.WD = (float)c->weight_decay;
    s.IS = (float)(1.0 / c->loss_scale);
    s.CLIP = c->grad_clip != 0.0 ? (float)c->grad_clip : INFINITY;
    s.round = (uint32_t)c->round;
    s.seed_lo = (uint32_t)c->seed;
    s.seed_hi = (uint32_t)(c->seed >> 32);
    s.step32 = (uint32_t)step;
    L.opt = MPO_OPT_ADAM;
    L.wfmt = c->weight_fmt;
    L.gfmt = c->grad_fmt;
    L.decay = c->weight_decay == 0.0 ? kNoDecay : (c->decoupled_wd ? kDecoupled : kL2);
    L.momentum = 1;
    L.use_ov = false;
    return MPO_OK;
}

mpo_status sgd_scalars(const mpo_sgd_cfg *c, uint64_t step, StepLaunch &L)
{
    if (!c || step == 0) return MPO_ERR_INVALID_ARG;
    if (!valid_fmt(c->weight_fmt) || !valid_fmt(c->grad_fmt)) return MPO_ERR_INVALID_ARG;
    const mpo_status rs = check_round(c->round);
    if (rs != MPO_OK) return rs;
    if (!std::isfinite(c->lr) || !std::isfinite(c->momentum) || !std::isfinite(c->weight_decay)) return MPO_ERR_INVALID_ARG;
    if (!finite_pos(c->loss_scale)) return MPO_ERR_INVALID_ARG;
    if (!(c->grad_clip >= 0.0) || !std::isfinite(c->grad_clip)) return MPO_ERR_INVALID_ARG;
    StepScalars &s = L.s;
    std::memset(&s, 0, sizeof s);
    s.LR = (float)c->lr;
    s.MU = (float)c->momentum;
    s.WD = (float)c->weight_decay;
    s.IS = (float)(1.0 / c->loss_scale);
    s.CLIP = c->grad_clip != 0.0 ? (float)c->grad_clip : INFINITY;
    s.round = (uint32_t)c->round;
    s.seed_lo = (uint32_t)c->seed;
    s.seed_hi = (uint32_t)(c->seed >> 32);
    s.step32 = (uint32_t)step;
    L.opt = MPO_OPT_SGD;
    L.wfmt = c->weight_fmt;
    L.gfmt = c->grad_fmt;
    L.decay = c->weight_decay == 0.0 ? kNoDecay : kL2;
    L.momentum = c->momentum != 0.0;
    L.use_ov = false;
    return MPO_OK;
}

mpo_status check_res_mode(uint32_t res_slot, bool any_explicit_bits, uint32_t min_res_bits, uint32_t max_res_bits,
                          StepLaunch &L)
{
    if (res_slot == 3) {
        /* packed planes: every tensor's stored bits must suit this format and rounding mode */
        if (any_explicit_bits && (!valid_packed_mode((int)max_res_bits, L.wfmt, (int)L.s.round) ||
                                  !valid_packed_mode((int)min_res_bits, L.wfmt, (int)L.s.round)))
            return MPO_ERR_INVALID_ARG;
    } else {
        if ((int)max_res_bits > full_res_bits(L.wfmt)) return MPO_ERR_INVALID_ARG;
        if (L.s.round == MPO_ROUND_STOCHASTIC && max_res_bits > (res_slot == 1 ? 7u : 15u)) return MPO_ERR_INVALID_ARG;
    }
    L.rmode = res_slot == 3 ? kResPlanes : res_slot == 1 ? kResByte : (any_explicit_bits ? kResPartial : kResFull);
    return MPO_OK;
}

hipError_t launch_step(const StepLaunch &L)
{
    if (L.num_chunks == 0) return hipSuccess;
    if (L.opt == MPO_OPT_ADAM) return L.use_ov ? launch_step_adam_ov(L) : launch_step_adam(L);
    return L.use_ov ? launch_step_sgd_ov(L) : launch_step_sgd(L);
}

namespace {

struct LayerInfo {
    int32_t id;
    uint64_t first_tensor, num_tensors; /* in layer order */
    uint64_t first_chunk, num_chunks;
    uint64_t num_params;
    uint32_t rows_log2;
};

} // namespace
} // namespace mpo

using namespace mpo;

struct mpo_plan {
    std::vector<TensorDesc> descs;      /* layer order */
    std::vector<uint64_t> caller_index; /* layer order -> index in the caller's list */
    std::vector<Chunk> chunks;
    std::vector<LayerInfo> layers;      /* sorted by id */
    uint64_t num_params = 0;
    uint32_t res_slot = 0;       /* residual storage: 1 bytes, 2 16-bit slots, 3 packed planes; 0 = no elements yet */
    uint32_t max_res_bits = 0;   /* largest explicit res_bits in the list                       */
    uint32_t min_res_bits = 16;  /* smallest explicit res_bits in the list                      */
    bool any_explicit_bits = false;
    bool on_device = false;
    int device = -1;
    TensorDesc *d_descs = nullptr;
    Chunk *d_chunks = nullptr;
};

namespace {

mpo_status build_plan(const mpo_tensor *tensors, uint64_t nt, uint64_t small_layer_params, mpo_plan **out)
{
    if (!out) return MPO_ERR_INVALID_ARG;
    *out = nullptr;
    if (nt > 0 && !tensors) return MPO_ERR_INVALID_ARG;
    if (nt > 0xFFFFFFFFull) return MPO_ERR_INVALID_ARG;

    mpo_plan *p = new (std::nothrow) mpo_plan;
    if (!p) return MPO_ERR_NOMEM;
    try {
        std::vector<Range> ranges(nt * 5);
        uint64_t nr = 0;
        for (uint64_t i = 0; i < nt; ++i) {
            const mpo_status s = check_tensor(tensors[i], p->res_slot, ranges.data(), &nr);
            if (s != MPO_OK) { delete p; return s; }
        }
        if (has_conflict(ranges.data(), nr)) { delete p; return MPO_ERR_ALIAS; }

        /* stable order by layer: a layer's tensors and chunks are contiguous */
        std::vector<uint64_t> order(nt);
        for (uint64_t i = 0; i < nt; ++i) order[i] = i;
        std::stable_sort(order.begin(), order.end(),
                         [&](uint64_t a, uint64_t b) { return tensors[a].layer < tensors[b].layer; });
        p->descs.reserve(nt);
        p->caller_index = order;
        std::vector<int32_t> layer(nt);
        for (uint64_t k = 0; k < nt; ++k) {
            const mpo_tensor &t = tensors[order[k]];
            p->descs.push_back(make_desc(t, (uint32_t)order[k]));
            layer[k] = t.layer;
            if (t.n && t.res_bits) {
                p->any_explicit_bits = true;
                p->max_res_bits = std::max(p->max_res_bits, (uint32_t)t.res_bits);
                p->min_res_bits = std::min(p->min_res_bits, (uint32_t)t.res_bits);
            }
            p->num_params += t.n;
        }
        /* default cut: by the kind of residual storage (see kSmallLayerParams) */
        if (small_layer_params == 0) small_layer_params = p->res_slot == 3 ? kPlanesSmallLayerParams : kSmallLayerParams;
        std::vector<TensorLayout> lay(nt);
        const uint64_t total = layout_chunks(p->descs.data(), layer.data(), nt, small_layer_params, lay.data());
        if (total == UINT64_MAX) { delete p; return MPO_ERR_INVALID_ARG; }
        p->chunks.resize(total);
        for (uint64_t k = 0; k < nt; ++k) {
            const TensorLayout &y = lay[k];
            const uint64_t celems = (uint64_t)kRowElems << y.rows_log2;
            if (y.has_ragged) p->chunks[y.ragged_pos] = Chunk{(uint32_t)k, chunk_where(y.num_full * celems, y.rows_log2)};
            for (uint64_t c = 0; c < y.num_full; ++c)
                p->chunks[y.full_pos + c] = Chunk{(uint32_t)k, chunk_where(c * celems, y.rows_log2)};
            if (p->layers.empty() || p->layers.back().id != layer[k])
                p->layers.push_back(LayerInfo{layer[k], k, 0, y.ragged_pos, 0, 0, y.rows_log2});
            LayerInfo &L = p->layers.back();
            L.num_tensors += 1;
            L.num_chunks += y.num_full + y.has_ragged;
            L.num_params += p->descs[k].n;
        }
    } catch (const std::bad_alloc &) {
        delete p;
        return MPO_ERR_NOMEM;
    }
    *out = p;
    return MPO_OK;
}

const LayerInfo *find_layer(const mpo_plan *p, int32_t layer)
{
    auto it = std::lower_bound(p->layers.begin(), p->layers.end(), layer,
                               [](const LayerInfo &L, int32_t id) { return L.id < id; });
    return (it != p->layers.end() && it->id == layer) ? &*it : nullptr;
}

/* Buffers the chosen optimizer needs, over tensors [k0, k0+nk) in layer order. */
bool state_present(const TensorDesc *descs, uint64_t k0, uint64_t nk, const StepLaunch &L, bool need_plan_grad)
{
    const bool need_m = L.opt == MPO_OPT_ADAM || L.momentum;
    const bool need_v = L.opt == MPO_OPT_ADAM;
    for (uint64_t k = k0; k < k0 + nk; ++k) {
        const TensorDesc &d = descs[k];
        if (d.n == 0) continue;
        if (need_m && !d.m) return false;
        if (need_v && !d.v) return false;
        if (need_plan_grad && !d.grad) return false;
    }
    return true;
}

mpo_status run(mpo_plan *p, StepLaunch &L, void *stream)
{
    /* the table and the descriptors live on the device the plan was created on */
    int dev = -1;
    const hipError_t de = hipGetDevice(&dev);
    if (de != hipSuccess) return hip_fail(de);
    if (dev != p->device) return MPO_ERR_INVALID_ARG;
    const mpo_status ms = check_res_mode(p->res_slot, p->any_explicit_bits, p->min_res_bits, p->max_res_bits, L);
    if (ms != MPO_OK) return ms;
    L.descs = p->d_descs;
    L.chunks = p->d_chunks;
    L.stream = static_cast<hipStream_t>(stream);
    const hipError_t e = launch_step(L);
    return e == hipSuccess ? MPO_OK : hip_fail(e);
}

mpo_status step_all(mpo_plan *p, StepLaunch &L, void *stream)
{
    if (!p || !p->on_device) return MPO_ERR_INVALID_ARG;
    if (!state_present(p->descs.data(), 0, p->descs.size(), L, true)) return MPO_ERR_INVALID_ARG;
    L.first_chunk = 0;
    L.num_chunks = p->chunks.size();
    return run(p, L, stream);
}

mpo_status split_merge_args(const void *w32, const void *hi, const void *res, uint64_t n, int fmt, int res_bits,
                            int res_packed, int round, bool w32_written)
{
    if (!valid_fmt(fmt) || check_round(round) != MPO_OK) return MPO_ERR_INVALID_ARG;
    if (res_packed ? !valid_packed_mode(res_bits, fmt, round) : !valid_res_bits(res_bits, fmt, round)) return MPO_ERR_INVALID_ARG;
    if (res_packed && n > 0 && !aligned16(res)) return MPO_ERR_INVALID_ARG;
    if (n >= kMaxTensorElems) return MPO_ERR_INVALID_ARG;
    if (n == 0) return MPO_OK;
    if (!w32 || !hi || !res) return MPO_ERR_INVALID_ARG;
    const uintptr_t a = (uintptr_t)w32, b = (uintptr_t)hi, c = (uintptr_t)res;
    Range r[3] = {Range{a, a + n * 4, w32_written}, Range{b, b + n * 2, !w32_written},
                  Range{c, c + res_bytes(n, res_bits, res_packed), !w32_written}};
    return has_conflict(r, 3) ? MPO_ERR_ALIAS : MPO_OK;
}

} // namespace

extern "C" {

mpo_status mpo_split(const float *w32, uint16_t *hi, void *res, uint64_t n, mpo_fmt fmt, int32_t res_bits,
                     int32_t res_packed, mpo_round round, uint64_t seed, uint32_t tensor_id, void *hip_stream)
{
    const mpo_status s = split_merge_args(w32, hi, res, n, fmt, res_bits, res_packed, round, false);
    if (s != MPO_OK || n == 0) return s;
    const hipError_t e = launch_split(w32, hi, res, n, fmt, res_bits, res_packed, round, seed, tensor_id,
                                      static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MPO_OK : hip_fail(e);
}

mpo_status mpo_merge(const uint16_t *hi, const void *res, float *w32, uint64_t n, mpo_fmt fmt, int32_t res_bits,
                     int32_t res_packed, mpo_round round, void *hip_stream)
{
    const mpo_status s = split_merge_args(w32, hi, res, n, fmt, res_bits, res_packed, round, true);
    if (s != MPO_OK || n == 0) return s;
    const hipError_t e = launch_merge(hi, res, w32, n, fmt, res_bits, res_packed, round,
                                      static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MPO_OK : hip_fail(e);
}

mpo_status mpo_plan_create_host(const mpo_tensor *tensors, uint64_t nt, mpo_plan **out)
{
    return build_plan(tensors, nt, 0, out);
}

mpo_status mpo_plan_create(const mpo_tensor *tensors, uint64_t nt, mpo_plan **out)
{
    return mpo_plan_create_opts(tensors, nt, nullptr, out);
}

mpo_status mpo_plan_create_opts(const mpo_tensor *tensors, uint64_t nt, const mpo_plan_opts *opts, mpo_plan **out)
{
    mpo_plan *p = nullptr;
    const uint64_t small = opts ? opts->small_layer_params : 0;   /* 0: the default for the storage kind */
    const mpo_status s = build_plan(tensors, nt, small, &p);
    if (s != MPO_OK) return s;
    if (opts && opts->host_only) {
        *out = p;
        return MPO_OK;
    }
    hipError_t e = hipGetDevice(&p->device);
    if (e == hipSuccess && !p->descs.empty())
        e = hipMalloc(reinterpret_cast<void **>(&p->d_descs), p->descs.size() * sizeof(TensorDesc));
    if (e == hipSuccess && !p->chunks.empty())
        e = hipMalloc(reinterpret_cast<void **>(&p->d_chunks), p->chunks.size() * sizeof(Chunk));
    if (e == hipSuccess && !p->descs.empty())
        e = hipMemcpy(p->d_descs, p->descs.data(), p->descs.size() * sizeof(TensorDesc), hipMemcpyHostToDevice);
    if (e == hipSuccess && !p->chunks.empty())
        e = hipMemcpy(p->d_chunks, p->chunks.data(), p->chunks.size() * sizeof(Chunk), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        if (p->d_descs) (void)hipFree(p->d_descs);
        if (p->d_chunks) (void)hipFree(p->d_chunks);
        delete p;
        *out = nullptr;
        return hip_fail(e);
    }
    p->on_device = true;
    *out = p;
    return MPO_OK;
}

mpo_status mpo_plan_destroy(mpo_plan *p)
{
    if (!p) return MPO_OK;
    mpo_status s = MPO_OK;
    if (p->d_descs) { const hipError_t e = hipFree(p->d_descs); if (e != hipSuccess) s = hip_fail(e); }
    if (p->d_chunks) { const hipError_t e = hipFree(p->d_chunks); if (e != hipSuccess) s = hip_fail(e); }
    delete p;
    return s;
}

uint64_t mpo_res_bytes(uint64_t n, int32_t res_bits, int32_t res_packed) { return res_bytes(n, res_bits, res_packed); }

uint64_t mpo_plan_chunk_elems(const mpo_plan *) { return kChunkElems; }
uint64_t mpo_plan_num_chunks(const mpo_plan *p) { return p ? p->chunks.size() : 0; }
uint64_t mpo_plan_num_params(const mpo_plan *p) { return p ? p->num_params : 0; }

mpo_status mpo_plan_get_chunk(const mpo_plan *p, uint64_t i, uint64_t *tensor, uint64_t *first, uint64_t *count)
{
    if (!p || !tensor || !first || !count || i >= p->chunks.size()) return MPO_ERR_INVALID_ARG;
    const Chunk &c = p->chunks[i];
    const uint64_t celems = (uint64_t)kRowElems << (c.where >> kChunkStartBits);
    *tensor = p->caller_index[c.tensor];
    *first = (uint64_t)(c.where & kChunkStartMask) * kRowElems;
    *count = std::min(celems, p->descs[c.tensor].n - *first);
    return MPO_OK;
}

mpo_status mpo_plan_layer_info(const mpo_plan *p, int32_t layer, uint64_t *first_chunk, uint64_t *num_chunks,
                               uint64_t *num_tensors, uint64_t *num_params, uint64_t *chunk_elems)
{
    if (!p) return MPO_ERR_INVALID_ARG;
    const LayerInfo *L = find_layer(p, layer);
    if (!L) return MPO_ERR_INVALID_ARG;
    if (first_chunk) *first_chunk = L->first_chunk;
    if (num_chunks) *num_chunks = L->num_chunks;
    if (num_tensors) *num_tensors = L->num_tensors;
    if (num_params) *num_params = L->num_params;
    if (chunk_elems) *chunk_elems = (uint64_t)kRowElems << L->rows_log2;
    return MPO_OK;
}

mpo_status mpo_adam_step(mpo_plan *p, const mpo_adam_cfg *cfg, uint64_t step, void *hip_stream)
{
    StepLaunch L;
    const mpo_status s = adam_scalars(cfg, step, L);
    if (s != MPO_OK) return s;
    return step_all(p, L, hip_stream);
}

mpo_status mpo_sgd_step(mpo_plan *p, const mpo_sgd_cfg *cfg, uint64_t step, void *hip_stream)
{
    StepLaunch L;
    const mpo_status s = sgd_scalars(cfg, step, L);
    if (s != MPO_OK) return s;
    return step_all(p, L, hip_stream);
}

mpo_status mpo_step_layer(mpo_plan *p, int32_t layer, const void *const *grads, uint64_t ngrads, mpo_opt opt,
                          const void *cfg, uint64_t step, void *hip_stream)
{
    StepLaunch L;
    mpo_status s;
    if (opt == MPO_OPT_ADAM) s = adam_scalars(static_cast<const mpo_adam_cfg *>(cfg), step, L);
    else if (opt == MPO_OPT_SGD) s = sgd_scalars(static_cast<const mpo_sgd_cfg *>(cfg), step, L);
    else return MPO_ERR_INVALID_ARG;
    if (s != MPO_OK) return s;
    if (!p || !p->on_device) return MPO_ERR_INVALID_ARG;
    const LayerInfo *info = find_layer(p, layer);
    if (!info) return MPO_ERR_INVALID_ARG;
    if (grads) {
        if (ngrads != info->num_tensors) return MPO_ERR_INVALID_ARG;
        if (ngrads > MPO_MAX_LAYER_GRADS) return MPO_ERR_UNSUPPORTED;
        /* per-call gradients must not overlap anything this layer writes */
        Range r[5 * MPO_MAX_LAYER_GRADS];
        uint64_t nr = 0;
        std::memset(&L.ov, 0, sizeof L.ov);
        for (uint64_t k = 0; k < ngrads; ++k) {
            const TensorDesc &d = p->descs[info->first_tensor + k];
            if (d.n == 0) continue;
            if (!grads[k]) return MPO_ERR_INVALID_ARG;
            const uintptr_t g = (uintptr_t)grads[k];
            r[nr++] = Range{g, g + d.n * 2, false};
            r[nr++] = Range{(uintptr_t)d.hi, (uintptr_t)d.hi + d.n * 2, true};
            r[nr++] = Range{(uintptr_t)d.res, (uintptr_t)d.res + res_bytes(d.n, (int)d.res_bits, p->res_slot == 3), true};
            if (d.m) r[nr++] = Range{(uintptr_t)d.m, (uintptr_t)d.m + d.n * 4, true};
            if (d.v) r[nr++] = Range{(uintptr_t)d.v, (uintptr_t)d.v + d.n * 4, true};
            L.ov.ptr[k] = static_cast<const uint16_t *>(grads[k]);
            if (!aligned16(grads[k])) L.ov.misaligned |= 1ull << k;
        }
        if (has_conflict(r, nr)) return MPO_ERR_ALIAS;
        L.ov.first = (uint32_t)info->first_tensor;
        L.use_ov = true;
    }
    if (!state_present(p->descs.data(), info->first_tensor, info->num_tensors, L, grads == nullptr)) return MPO_ERR_INVALID_ARG;
    L.first_chunk = info->first_chunk;
    L.num_chunks = info->num_chunks;
    return run(p, L, hip_stream);
}

const char *mpo_status_string(mpo_status s)
{
    switch (s) {
    case MPO_OK: return "ok";
    case MPO_ERR_INVALID_ARG: return "invalid argument";
    case MPO_ERR_UNSUPPORTED: return "mode declared but not built";
    case MPO_ERR_ALIAS: return "buffers overlap";
    case MPO_ERR_HIP: return "HIP runtime error";
    case MPO_ERR_NOMEM: return "out of memory";
    case MPO_ERR_TOO_LARGE: return "list too large for the entry point that allocates nothing";
    }
    return "unknown status";
}

int mpo_last_hip_error(void) { return g_last_hip_error; }

} // extern "C"
