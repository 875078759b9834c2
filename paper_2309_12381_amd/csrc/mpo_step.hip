/*
 * The fused optimizer step kernels of libmpo (arXiv 2309.12381, Sections 3.1 and 3.2), compiled
 * in four parts so that the parts build side by side: MPO_PART_OPT selects Adam (0) or SGD (1),
 * MPO_PART_OV whether the gradient pointers come from the descriptors (0) or, for the per-layer
 * step with per-call gradients, from the kernel arguments (1).  The device code itself is in
 * mpo_device.h; this file only instantiates it and picks the instantiation of a launch.
 */
#include <hip/hip_runtime.h>

#include "mpo_device.h"

#if !defined(MPO_PART_OPT) || !defined(MPO_PART_OV)
#error "compile with -DMPO_PART_OPT=0|1 -DMPO_PART_OV=0|1"
#endif

namespace mpo {
namespace {

constexpr bool kOv = MPO_PART_OV != 0;

[[maybe_unused]] inline void set_ov(GradOverride &o, const StepLaunch &L) { o = L.ov; }
[[maybe_unused]] inline void set_ov(NoOverride &o, const StepLaunch &) { o.unused = 0u; }

template <int OPT, int WFMT, int GFMT, int DECAY, bool MOM, int RMODE, bool RND>
hipError_t launch_step_t(const StepLaunch &L)
{
    typename OvArg<kOv>::T ov;
    set_ov(ov, L);
    uint64_t done = 0;
    while (done < L.num_chunks) {
        const uint64_t now = (L.num_chunks - done < kMaxGrid) ? (L.num_chunks - done) : kMaxGrid;
        (void)hipGetLastError(); /* an error an earlier, unrelated runtime call left on this thread is not ours */
        step_kernel<OPT, WFMT, GFMT, DECAY, MOM, RMODE, RND, kOv><<<dim3((uint32_t)now), dim3(kBlock), 0, L.stream>>>(
            L.descs, L.chunks, L.first_chunk + done, L.s, ov);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        done += now;
    }
    return hipSuccess;
}

template <int OPT, int WFMT, int GFMT, int DECAY, bool MOM>
hipError_t launch_step_res(const StepLaunch &L)
{
    if (L.s.round != MPO_ROUND_TRUNC) {
        /* rounded modes always go through the general residual path */
        return L.rmode == kResByte     ? launch_step_t<OPT, WFMT, GFMT, DECAY, MOM, kResByte, true>(L)
               : L.rmode == kResPlanes ? launch_step_t<OPT, WFMT, GFMT, DECAY, MOM, kResPlanes, true>(L)
                                       : launch_step_t<OPT, WFMT, GFMT, DECAY, MOM, kResPartial, true>(L);
    }
    switch (L.rmode) {
    case kResFull: return launch_step_t<OPT, WFMT, GFMT, DECAY, MOM, kResFull, false>(L);
    case kResPartial: return launch_step_t<OPT, WFMT, GFMT, DECAY, MOM, kResPartial, false>(L);
    case kResPlanes: return launch_step_t<OPT, WFMT, GFMT, DECAY, MOM, kResPlanes, false>(L);
    default: return launch_step_t<OPT, WFMT, GFMT, DECAY, MOM, kResByte, false>(L);
    }
}

template <int OPT, int DECAY, bool MOM>
hipError_t launch_step_fmt(const StepLaunch &L)
{
    if (L.wfmt == MPO_BF16)
        return L.gfmt == MPO_BF16 ? launch_step_res<OPT, MPO_BF16, MPO_BF16, DECAY, MOM>(L)
                                  : launch_step_res<OPT, MPO_BF16, MPO_FP16, DECAY, MOM>(L);
    return L.gfmt == MPO_BF16 ? launch_step_res<OPT, MPO_FP16, MPO_BF16, DECAY, MOM>(L)
                              : launch_step_res<OPT, MPO_FP16, MPO_FP16, DECAY, MOM>(L);
}

} // namespace

#if MPO_PART_OPT == 0
#if MPO_PART_OV
hipError_t launch_step_adam_ov(const StepLaunch &L)
#else
hipError_t launch_step_adam(const StepLaunch &L)
#endif
{
    switch (L.decay) {
    case kNoDecay: return launch_step_fmt<MPO_OPT_ADAM, kNoDecay, true>(L);
    case kDecoupled: return launch_step_fmt<MPO_OPT_ADAM, kDecoupled, true>(L);
    default: return launch_step_fmt<MPO_OPT_ADAM, kL2, true>(L);
    }
}
#else
#if MPO_PART_OV
hipError_t launch_step_sgd_ov(const StepLaunch &L)
#else
hipError_t launch_step_sgd(const StepLaunch &L)
#endif
{
    if (L.momentum)
        return L.decay == kL2 ? launch_step_fmt<MPO_OPT_SGD, kL2, true>(L)
                              : launch_step_fmt<MPO_OPT_SGD, kNoDecay, true>(L);
    return L.decay == kL2 ? launch_step_fmt<MPO_OPT_SGD, kL2, false>(L)
                          : launch_step_fmt<MPO_OPT_SGD, kNoDecay, false>(L);
}
#endif

} // namespace mpo
