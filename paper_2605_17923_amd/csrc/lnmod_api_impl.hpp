// lnmod_api_impl.hpp -- argument validation and hand-over to the launchers, shared by the operator
// library (lnmod_api.cpp: include/lnmod.h) and the measurement library (lnmod_tools_api.cpp:
// include/lnmod_tools.h).  Validation comes before any HIP call, so that it can be exercised on a
// host without a GPU.
#pragma once
#include <cmath>

#include "lnmod.h"
#include "lnmod_launch.hpp"

namespace lnmod {
namespace api {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline int check_shape(int64_t nseg, int64_t S_or_T, int64_t D, float eps, int dtype, int64_t total) {
    if (nseg < 0 || nseg >= (int64_t(1) << 24) || S_or_T < 0 || D < 0) return LNMOD_EINVAL;
    if (!(std::isfinite(eps) && eps > 0.0f)) return LNMOD_EINVAL;
    if (dtype != LNMOD_BF16 && dtype != LNMOD_F32) return LNMOD_EINVAL;
    if (total < 0 || total >= (int64_t(1) << 31)) return LNMOD_EINVAL;
    const int64_t vec = dtype == LNMOD_BF16 ? 8 : 4;
    if (D < 8 || D > kMaxD || D % vec != 0) return LNMOD_EUNSUPPORTED;
    return LNMOD_OK;
}

// total tokens of a fixed-length batch, or -1 on overflow
inline int64_t total_tokens(int64_t B, int64_t S) {
    if (B < 0 || S < 0) return -1;
    if (B == 0 || S == 0) return 0;
    if (B > (int64_t(1) << 31) / S) return -1;
    return B * S;
}

inline size_t workspace_bytes(int64_t nseg, int64_t T, int64_t D, const Shape* force = nullptr) {
    // partial-sum slots of the plan with the most of them (neither the dtype nor whether the
    // statistics will be recomputed is an argument of the query)
    int64_t slots = 0;
    for (int v = 0; v < 4; ++v) {
        const int dtype = v & 1;
        if (D % (dtype == 0 ? 8 : 4) != 0) continue;
        const RowPlan pl = bwd_plan(T, nseg, D, dtype, (v & 2) != 0, force);
        const int64_t s = bwd_slots(pl, nseg);
        if (s > slots) slots = s;
    }
    return static_cast<size_t>(slots) * 2u * static_cast<size_t>(D) * sizeof(float);
}

inline int forward_impl(const void* x, const void* shift, const void* scale, const int32_t* cu,
                        bool varlen, int64_t nseg, int64_t S, int64_t T, int64_t D, float eps,
                        void* stream, void* y, float* mean, float* rstd, int dtype, int mod,
                        const Shape* force = nullptr) {
    if (mod != LNMOD_PER_SAMPLE && mod != LNMOD_PER_TOKEN) return LNMOD_EINVAL;
    const int st = check_shape(nseg, varlen ? T : S, D, eps, dtype, T);
    if (st != LNMOD_OK) return st;
    if (T == 0) return LNMOD_OK;
    if (nseg == 0) return LNMOD_EINVAL;           // tokens that belong to no segment
    if (!x || !shift || !scale || !y || (varlen && !cu)) return LNMOD_EINVAL;
    if ((mean == nullptr) != (rstd == nullptr)) return LNMOD_EINVAL;    // both, or neither (not stored)
    if (!aligned16(x) || !aligned16(shift) || !aligned16(scale) || !aligned16(y)) return LNMOD_EALIGN;
    const Problem p{dtype, varlen ? cu : nullptr, nseg, S, T, D, eps, force};
    const hipStream_t hs = static_cast<hipStream_t>(stream);
    const hipError_t e = (mod == LNMOD_PER_TOKEN)
                             ? launch_fwd_tok(p, x, shift, scale, y, mean, rstd, hs)
                             : launch_fwd_seg(p, x, shift, scale, y, mean, rstd, hs);
    return e == hipSuccess ? LNMOD_OK : LNMOD_ELAUNCH;
}

inline int backward_impl(const void* dy, const void* x, const void* scale, const int32_t* cu, bool varlen,
                         int64_t nseg, int64_t S, int64_t T, int64_t D, float eps, void* stream,
                         const float* mean, const float* rstd, void* dx, void* dshift, void* dscale,
                         void* workspace, size_t workspace_size, int dtype, int mod,
                         const Shape* force = nullptr, bool exact_workspace = false) {
    if (mod != LNMOD_PER_SAMPLE && mod != LNMOD_PER_TOKEN) return LNMOD_EINVAL;
    const int st = check_shape(nseg, varlen ? T : S, D, eps, dtype, T);
    if (st != LNMOD_OK) return st;
    const hipStream_t hs = static_cast<hipStream_t>(stream);
    if (T == 0) {
        if (mod == LNMOD_PER_SAMPLE && nseg > 0) {      // empty sums are zeros
            if (!dshift || !dscale) return LNMOD_EINVAL;
            if (!aligned16(dshift) || !aligned16(dscale)) return LNMOD_EALIGN;
            hipError_t e = launch_zero_f32(static_cast<float*>(dshift), nseg * D, hs);
            if (e == hipSuccess) e = launch_zero_f32(static_cast<float*>(dscale), nseg * D, hs);
            return e == hipSuccess ? LNMOD_OK : LNMOD_ELAUNCH;
        }
        return LNMOD_OK;
    }
    if (nseg == 0) return LNMOD_EINVAL;
    if (!dy || !x || !scale || !dx || !dshift || !dscale || (varlen && !cu)) return LNMOD_EINVAL;
    if ((mean == nullptr) != (rstd == nullptr)) return LNMOD_EINVAL;    // both, or neither (recompute)
    if (!aligned16(dy) || !aligned16(x) || !aligned16(scale) || !aligned16(dx) ||
        !aligned16(dshift) || !aligned16(dscale))
        return LNMOD_EALIGN;
    const Problem p{dtype, varlen ? cu : nullptr, nseg, S, T, D, eps, force};
    hipError_t e;
    if (mod == LNMOD_PER_TOKEN) {
        e = launch_bwd_tok(p, dy, x, scale, mean, rstd, dx, dshift, dscale, hs);
    } else {
        // exact_workspace: the caller has sized the workspace for this very plan (element type,
        // statistics recomputed or not) instead of the query's bound over all plans
        const size_t need =
            exact_workspace ? static_cast<size_t>(bwd_slots(bwd_plan(T, nseg, D, dtype, mean == nullptr, force), nseg)) *
                                  2u * static_cast<size_t>(D) * sizeof(float)
                            : workspace_bytes(nseg, T, D, force);
        if (!workspace || workspace_size < need) return LNMOD_EWORKSPACE;
        if (!aligned16(workspace)) return LNMOD_EALIGN;
        e = launch_bwd_seg(p, dy, x, scale, mean, rstd, dx, static_cast<float*>(dshift),
                                  static_cast<float*>(dscale), static_cast<float*>(workspace), hs);
    }
    return e == hipSuccess ? LNMOD_OK : LNMOD_ELAUNCH;
}

}  // namespace api
}  // namespace lnmod
