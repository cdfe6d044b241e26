// lnmod_api.cpp -- the C ABI declared in include/lnmod.h: the operator entry points, nothing else.
// The library keeps no mutable state: a call's result depends on its arguments alone.
#include "lnmod_api_impl.hpp"

static_assert(LNMOD_STATIC_WORKSPACE_BYTES == lnmod::kStaticWorkspaceBytes, "header and library disagree");

namespace {

using lnmod::Problem;
using namespace lnmod::api;

size_t gated_workspace_bytes(int64_t nseg, int64_t T, int64_t D) {
    int64_t slots = 0;
    for (int dtype = 0; dtype < 2; ++dtype) {
        if (D % (dtype == 0 ? 8 : 4) != 0) continue;
        const lnmod::RowPlan pl = lnmod::gated_bwd_plan(T, nseg, D, dtype);
        const int64_t s = lnmod::bwd_slots(pl, nseg);
        if (s > slots) slots = s;
    }
    return static_cast<size_t>(slots) * 3u * static_cast<size_t>(D) * sizeof(float);
}

size_t qknorm_workspace_bytes(int64_t N, int64_t D) {
    int64_t nb = 0;
    for (int dtype = 0; dtype < 2; ++dtype) {
        if (D % (dtype == 0 ? 8 : 4) != 0) continue;
        const int64_t b = lnmod::qknorm_bwd_blocks(N, D, dtype);
        if (b > nb) nb = b;
    }
    return static_cast<size_t>(2 * nb) * static_cast<size_t>(D) * sizeof(float);
}

// (segments, tokens per sample, total tokens) of a gated call, or false on overflow
bool gated_shape(const int32_t* cu, int64_t B_or_nseg, int64_t S_or_T, int64_t* S, int64_t* T) {
    if (cu) {
        *S = 0;
        *T = S_or_T;
        return true;
    }
    *S = S_or_T;
    *T = total_tokens(B_or_nseg, S_or_T);
    return *T >= 0;
}

}  // namespace

extern "C" {

int lnmod_forward(const void* x, const void* shift, const void* scale, int64_t B, int64_t S,
                  int64_t D, float eps, void* stream, void* y, float* mean, float* rstd,
                  int dtype, int mod) {
    const int64_t T = total_tokens(B, S);
    if (T < 0) return LNMOD_EINVAL;
    return forward_impl(x, shift, scale, nullptr, false, B, S, T, D, eps, stream, y, mean, rstd,
                        dtype, mod);
}

int lnmod_backward(const void* dy, const void* x, const void* shift, const void* scale, int64_t B,
                   int64_t S, int64_t D, float eps, void* stream, const float* mean,
                   const float* rstd, void* dx, void* dshift, void* dscale, void* workspace,
                   size_t workspace_size, int dtype, int mod) {
    (void)shift;
    const int64_t T = total_tokens(B, S);
    if (T < 0) return LNMOD_EINVAL;
    return backward_impl(dy, x, scale, nullptr, false, B, S, T, D, eps, stream, mean, rstd, dx,
                         dshift, dscale, workspace, workspace_size, dtype, mod);
}

int lnmod_forward_varlen(const void* x, const void* shift, const void* scale,
                         const int32_t* cu_seqlens, int64_t nseg, int64_t T, int64_t D, float eps,
                         void* stream, void* y, float* mean, float* rstd, int dtype) {
    return forward_impl(x, shift, scale, cu_seqlens, true, nseg, 0, T, D, eps, stream, y, mean,
                        rstd, dtype, LNMOD_PER_SAMPLE);
}

int lnmod_backward_varlen(const void* dy, const void* x, const void* shift, const void* scale,
                          const int32_t* cu_seqlens, int64_t nseg, int64_t T, int64_t D, float eps,
                          void* stream, const float* mean, const float* rstd, void* dx,
                          void* dshift, void* dscale, void* workspace, size_t workspace_size,
                          int dtype) {
    (void)shift;
    return backward_impl(dy, x, scale, cu_seqlens, true, nseg, 0, T, D, eps, stream, mean, rstd,
                         dx, dshift, dscale, workspace, workspace_size, dtype, LNMOD_PER_SAMPLE);
}

int lnmod_backward_static(const void* dy, const void* x, const void* shift, const void* scale,
                          int64_t B, int64_t S, int64_t D, float eps, void* stream,
                          const float* mean, const float* rstd, void* dx, void* dshift,
                          void* dscale, int dtype, int mod) {
    (void)shift;
    const int64_t T = total_tokens(B, S);
    if (T < 0) return LNMOD_EINVAL;
    if (mod != LNMOD_PER_SAMPLE && mod != LNMOD_PER_TOKEN) return LNMOD_EINVAL;
    const int st = check_shape(B, S, D, eps, dtype, T);
    if (st != LNMOD_OK) return st;
    void* ws = nullptr;
    size_t ws_bytes = 0;
    if (mod == LNMOD_PER_SAMPLE && T > 0 && B > 0) {
        // the slots of exactly this call's plan (element type and whether the statistics are
        // recomputed are known here), not the query's upper bound over all plans
        if ((mean == nullptr) != (rstd == nullptr)) return LNMOD_EINVAL;
        const lnmod::RowPlan pl = lnmod::bwd_plan(T, B, D, dtype, mean == nullptr);
        const size_t need = static_cast<size_t>(lnmod::bwd_slots(pl, B)) * 2u * static_cast<size_t>(D) * sizeof(float);
        if (need > lnmod::kStaticWorkspaceBytes) return LNMOD_EWORKSPACE;
        // every other argument is checked before the first HIP call
        if (!dy || !x || !scale || !dx || !dshift || !dscale) return LNMOD_EINVAL;
        if (!aligned16(dy) || !aligned16(x) || !aligned16(scale) || !aligned16(dx) ||
            !aligned16(dshift) || !aligned16(dscale))
            return LNMOD_EALIGN;
        float* p = nullptr;
        if (lnmod::static_workspace(&p) != hipSuccess) return LNMOD_ELAUNCH;
        ws = p;
        ws_bytes = lnmod::kStaticWorkspaceBytes;
    }
    return backward_impl(dy, x, scale, nullptr, false, B, S, T, D, eps, stream, mean, rstd, dx,
                         dshift, dscale, ws, ws_bytes, dtype, mod, nullptr, /*exact_workspace=*/true);
}

size_t lnmod_backward_workspace_bytes(int64_t B_or_nseg, int64_t total, int64_t D, int mod) {
    if (mod != LNMOD_PER_SAMPLE) return 0;
    if (B_or_nseg < 0 || total < 0 || total >= (int64_t(1) << 31)) return 0;
    if (D < 8 || D > lnmod::kMaxD || D % 4 != 0) return 0;
    return workspace_bytes(B_or_nseg, total, D);
}

const char* lnmod_status_string(int status) {
    switch (status) {
        case LNMOD_OK: return "ok";
        case LNMOD_EINVAL: return "invalid argument";
        case LNMOD_EUNSUPPORTED: return "unsupported hidden size";
        case LNMOD_EALIGN: return "pointer not 16-byte aligned";
        case LNMOD_EWORKSPACE: return "workspace missing or too small";
        case LNMOD_ELAUNCH: return "kernel launch failed";
        default: return "unknown status";
    }
}

int lnmod_gated_forward(const void* x, const void* u, const void* gate, const void* shift,
                        const void* scale, const int32_t* cu_seqlens, int64_t B_or_nseg,
                        int64_t S_or_T, int64_t D, float eps, void* stream, void* h, void* y,
                        float* mean, float* rstd, int dtype) {
    int64_t S, T;
    if (!gated_shape(cu_seqlens, B_or_nseg, S_or_T, &S, &T)) return LNMOD_EINVAL;
    const int st = check_shape(B_or_nseg, S_or_T, D, eps, dtype, T);
    if (st != LNMOD_OK) return st;
    if (T == 0) return LNMOD_OK;
    if (B_or_nseg == 0) return LNMOD_EINVAL;
    if (!x || !u || !gate || !shift || !scale || !h || !y || !mean || !rstd) return LNMOD_EINVAL;
    if (!aligned16(x) || !aligned16(u) || !aligned16(gate) || !aligned16(shift) || !aligned16(scale) ||
        !aligned16(h) || !aligned16(y))
        return LNMOD_EALIGN;
    const Problem p{dtype, cu_seqlens, B_or_nseg, S, T, D, eps};
    const hipError_t e = lnmod::launch_gated_fwd(p, x, u, gate, shift, scale, h, y, mean, rstd,
                                                 static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LNMOD_OK : LNMOD_ELAUNCH;
}

int lnmod_gated_backward(const void* dy, const void* dh, const void* h, const void* u,
                         const void* gate, const void* scale, const int32_t* cu_seqlens,
                         int64_t B_or_nseg, int64_t S_or_T, int64_t D, float eps, void* stream,
                         const float* mean, const float* rstd, void* dx, void* du, float* dgate,
                         float* dshift, float* dscale, void* workspace, size_t workspace_size,
                         int dtype) {
    int64_t S, T;
    if (!gated_shape(cu_seqlens, B_or_nseg, S_or_T, &S, &T)) return LNMOD_EINVAL;
    const int st = check_shape(B_or_nseg, S_or_T, D, eps, dtype, T);
    if (st != LNMOD_OK) return st;
    const hipStream_t hs = static_cast<hipStream_t>(stream);
    if (T == 0) {
        if (B_or_nseg > 0) {                                  // empty sums are zeros
            if (!dgate || !dshift || !dscale) return LNMOD_EINVAL;
            hipError_t e = lnmod::launch_zero_f32(dgate, B_or_nseg * D, hs);
            if (e == hipSuccess) e = lnmod::launch_zero_f32(dshift, B_or_nseg * D, hs);
            if (e == hipSuccess) e = lnmod::launch_zero_f32(dscale, B_or_nseg * D, hs);
            return e == hipSuccess ? LNMOD_OK : LNMOD_ELAUNCH;
        }
        return LNMOD_OK;
    }
    if (B_or_nseg == 0) return LNMOD_EINVAL;
    if (!dy || !dh || !h || !u || !gate || !scale || !mean || !rstd || !dx || !du || !dgate ||
        !dshift || !dscale)
        return LNMOD_EINVAL;
    if (!aligned16(dy) || !aligned16(dh) || !aligned16(h) || !aligned16(u) || !aligned16(gate) ||
        !aligned16(scale) || !aligned16(dx) || !aligned16(du) || !aligned16(dgate) ||
        !aligned16(dshift) || !aligned16(dscale))
        return LNMOD_EALIGN;
    if (!workspace || workspace_size < gated_workspace_bytes(B_or_nseg, T, D)) return LNMOD_EWORKSPACE;
    if (!aligned16(workspace)) return LNMOD_EALIGN;
    const Problem p{dtype, cu_seqlens, B_or_nseg, S, T, D, eps};
    const hipError_t e = lnmod::launch_gated_bwd(p, dy, dh, h, u, gate, scale, mean, rstd, dx, du,
                                                 dgate, dshift, dscale,
                                                 static_cast<float*>(workspace), hs);
    return e == hipSuccess ? LNMOD_OK : LNMOD_ELAUNCH;
}

size_t lnmod_gated_backward_workspace_bytes(int64_t B_or_nseg, int64_t total, int64_t D) {
    if (B_or_nseg < 0 || total < 0 || total >= (int64_t(1) << 31)) return 0;
    if (D < 8 || D > lnmod::kMaxD || D % 4 != 0) return 0;
    return gated_workspace_bytes(B_or_nseg, total, D);
}

int lnmod_qknorm_forward(const void* q, const void* k, const void* wq, const void* wk, int64_t N,
                         int64_t D, float eps, void* stream, void* q_out, void* k_out,
                         float* rstd_q, float* rstd_k, int dtype) {
    const int st = check_shape(1, N, D, eps, dtype, N);
    if (st != LNMOD_OK) return st;
    if (N == 0) return LNMOD_OK;
    if (!q || !k || !wq || !wk || !q_out || !k_out || !rstd_q || !rstd_k) return LNMOD_EINVAL;
    if (!aligned16(q) || !aligned16(k) || !aligned16(wq) || !aligned16(wk) || !aligned16(q_out) ||
        !aligned16(k_out))
        return LNMOD_EALIGN;
    const hipError_t e = lnmod::launch_qknorm_fwd(dtype, q, k, wq, wk, N, D, eps, q_out, k_out, rstd_q,
                                                  rstd_k, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LNMOD_OK : LNMOD_ELAUNCH;
}

int lnmod_qknorm_backward(const void* dq_out, const void* dk_out, const void* q, const void* k,
                          const void* wq, const void* wk, int64_t N, int64_t D, float eps,
                          void* stream, const float* rstd_q, const float* rstd_k, void* dq, void* dk,
                          float* dwq, float* dwk, void* workspace, size_t workspace_size, int dtype) {
    const int st = check_shape(1, N, D, eps, dtype, N);
    if (st != LNMOD_OK) return st;
    const hipStream_t hs = static_cast<hipStream_t>(stream);
    if (N == 0) {                                             // empty sums are zeros
        if (!dwq || !dwk) return LNMOD_EINVAL;
        hipError_t e = lnmod::launch_zero_f32(dwq, D, hs);
        if (e == hipSuccess) e = lnmod::launch_zero_f32(dwk, D, hs);
        return e == hipSuccess ? LNMOD_OK : LNMOD_ELAUNCH;
    }
    if (!dq_out || !dk_out || !q || !k || !wq || !wk || !rstd_q || !rstd_k || !dq || !dk || !dwq || !dwk)
        return LNMOD_EINVAL;
    if (!aligned16(dq_out) || !aligned16(dk_out) || !aligned16(q) || !aligned16(k) || !aligned16(wq) ||
        !aligned16(wk) || !aligned16(dq) || !aligned16(dk))
        return LNMOD_EALIGN;
    if (!workspace || workspace_size < qknorm_workspace_bytes(N, D)) return LNMOD_EWORKSPACE;
    if (!aligned16(workspace)) return LNMOD_EALIGN;
    const hipError_t e = lnmod::launch_qknorm_bwd(dtype, dq_out, dk_out, q, k, wq, wk, N, D, rstd_q,
                                                  rstd_k, dq, dk, dwq, dwk,
                                                  static_cast<float*>(workspace), hs);
    return e == hipSuccess ? LNMOD_OK : LNMOD_ELAUNCH;
}

size_t lnmod_qknorm_backward_workspace_bytes(int64_t N, int64_t D) {
    if (N < 0 || N >= (int64_t(1) << 31)) return 0;
    if (D < 8 || D > lnmod::kMaxD || D % 4 != 0) return 0;
    return qknorm_workspace_bytes(N, D);
}

}  // extern "C"
