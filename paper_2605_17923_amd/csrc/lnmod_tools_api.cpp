// lnmod_tools_api.cpp -- the C ABI declared in include/lnmod_tools.h: bandwidth references, the
// comparators of the fused-against-unfused measurement, and forms of the operator calls that take
// their launch shape as an argument.  Built into liblnmod_tools.so, not into the operator library.
#include "lnmod_tools.h"

#include "lnmod_api_impl.hpp"

namespace {

using lnmod::Problem;
using lnmod::Shape;
using namespace lnmod::api;

// shape == NULL: the table's entry.  false for values outside the documented ranges.
bool read_shape(const int* shape, Shape* out, const Shape** force) {
    *force = nullptr;
    if (!shape) return true;
    if (shape[0] < 1 || shape[0] > 16 || shape[1] < 1 || shape[1] > 6 || shape[2] < 1 || shape[2] > 2 ||
        shape[3] < 1 || shape[3] > 16)
        return false;
    if (shape[4] < 0 || shape[4] > 256 || (shape[5] != 0 && shape[5] != 1) || shape[6] < 0 || shape[6] > 2) return false;
    *out = Shape{shape[0], shape[1], shape[2], shape[3], shape[4], shape[5], shape[6]};
    *force = out;
    return true;
}

// (segments, tokens per sample, total tokens) of a call that is packed when cu != NULL
bool batch_shape(bool varlen, int64_t B_or_nseg, int64_t S_or_T, int64_t* S, int64_t* T) {
    if (varlen) {
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

int lnmod_copy(const void* src, void* dst, size_t bytes, void* stream) {
    if (bytes == 0) return LNMOD_OK;
    if (!src || !dst || bytes % 16 != 0) return LNMOD_EINVAL;
    if (!aligned16(src) || !aligned16(dst)) return LNMOD_EALIGN;
    const hipError_t e = lnmod::launch_copy(src, dst, bytes, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LNMOD_OK : LNMOD_ELAUNCH;
}

int lnmod_stream_probe(const void* const* in, int reads, void* const* out, int writes, size_t bytes,
                       int blocks, int waves, int vecs, void* stream) {
    if (reads < 0 || writes < 0 || !lnmod::probe_mixture_supported(reads, writes)) return LNMOD_EINVAL;
    if (bytes % 16 != 0 || !out || (reads > 0 && !in)) return LNMOD_EINVAL;
    const bool dflt = blocks == 0 && waves == 0 && vecs == 0;
    if (!dflt && (blocks < 1 || blocks > 65536 || waves < 1 || waves > 8 ||
                  (vecs != 1 && vecs != 2 && vecs != 4 && vecs != 8)))
        return LNMOD_EINVAL;
    if (bytes == 0) return LNMOD_OK;
    if (writes == 0 && bytes < 1024) return LNMOD_EINVAL;              // out[0] must hold 1 KB
    for (int i = 0; i < reads; ++i) {
        if (!in[i]) return LNMOD_EINVAL;
        if (!aligned16(in[i])) return LNMOD_EALIGN;
    }
    for (int j = 0; j < (writes > 0 ? writes : 1); ++j) {
        if (!out[j]) return LNMOD_EINVAL;
        if (!aligned16(out[j])) return LNMOD_EALIGN;
    }
    const hipError_t e = lnmod::launch_stream_probe(in, reads, out, writes, bytes, blocks, waves, vecs,
                                                    static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LNMOD_OK : LNMOD_ELAUNCH;
}

int lnmod_unfused_forward(const void* x, const void* shift, const void* scale, int64_t B, int64_t S,
                          int64_t D, float eps, void* stream, void* xhat_tmp, void* y, float* mean,
                          float* rstd, int dtype) {
    const int64_t T = total_tokens(B, S);
    if (T < 0) return LNMOD_EINVAL;
    const int st = check_shape(B, S, D, eps, dtype, T);
    if (st != LNMOD_OK) return st;
    if (T == 0) return LNMOD_OK;
    if (!x || !shift || !scale || !xhat_tmp || !y || !mean || !rstd) return LNMOD_EINVAL;
    if (!aligned16(x) || !aligned16(shift) || !aligned16(scale) || !aligned16(xhat_tmp) || !aligned16(y))
        return LNMOD_EALIGN;
    const Problem p{dtype, nullptr, B, S, T, D, eps};
    const hipError_t e = lnmod::launch_unfused(p, x, shift, scale, xhat_tmp, y, mean, rstd,
                                               static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LNMOD_OK : LNMOD_ELAUNCH;
}

int lnmod_gate_residual(const void* x, const void* u, const void* gate, int64_t B, int64_t S,
                        int64_t D, void* stream, void* h, int dtype) {
    const int64_t T = total_tokens(B, S);
    if (T < 0) return LNMOD_EINVAL;
    const int st = check_shape(B, S, D, 1.0f, dtype, T);
    if (st != LNMOD_OK) return st;
    if (T == 0) return LNMOD_OK;
    if (!x || !u || !gate || !h) return LNMOD_EINVAL;
    if (!aligned16(x) || !aligned16(u) || !aligned16(gate) || !aligned16(h)) return LNMOD_EALIGN;
    const Problem p{dtype, nullptr, B, S, T, D, 1.0f};
    const hipError_t e = lnmod::launch_gate_residual(p, x, u, gate, h, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LNMOD_OK : LNMOD_ELAUNCH;
}

int lnmod_table_shape(int family, int64_t D, int dtype, int64_t tokens, int* out) {
    if (family < LNMOD_FAMILY_FORWARD || family > LNMOD_FAMILY_QKNORM_BACKWARD || !out) return LNMOD_EINVAL;
    if (dtype != LNMOD_BF16 && dtype != LNMOD_F32) return LNMOD_EINVAL;
    const int64_t vec = dtype == LNMOD_BF16 ? 8 : 4;
    if (D < 8 || D > lnmod::kMaxD || D % vec != 0) return LNMOD_EUNSUPPORTED;
    const int nchunks = static_cast<int>(D / vec);
    Shape sh{};
    switch (family) {
        case LNMOD_FAMILY_FORWARD: sh = lnmod::fwd_shape(nchunks, dtype, tokens < 0 ? 0 : tokens); break;
        case LNMOD_FAMILY_BACKWARD: sh = lnmod::bwd_shape(nchunks, dtype); break;
        case LNMOD_FAMILY_BACKWARD_RECOMPUTE: sh = lnmod::rc_bwd_shape(nchunks, dtype); break;
        case LNMOD_FAMILY_TOKEN_FORWARD: sh = lnmod::tok_fwd_shape(nchunks, dtype); break;
        case LNMOD_FAMILY_TOKEN_BACKWARD: sh = lnmod::tok_bwd_shape(nchunks, dtype); break;
        case LNMOD_FAMILY_GATED_FORWARD: sh = lnmod::gated_fwd_table_shape(nchunks, dtype); break;
        case LNMOD_FAMILY_GATED_BACKWARD: sh = lnmod::gated_bwd_table_shape(nchunks, dtype); break;
        case LNMOD_FAMILY_QKNORM_FORWARD: sh = lnmod::qknorm_table_shape(nchunks, dtype, false); break;
        default: sh = lnmod::qknorm_table_shape(nchunks, dtype, true); break;
    }
    out[0] = sh.K;
    out[1] = sh.VPL;
    out[2] = sh.R;
    out[3] = sh.per_cu;
    return LNMOD_OK;
}

int lnmod_forward_shaped(const int* shape, const void* x, const void* shift, const void* scale,
                         const int32_t* cu_seqlens, int64_t B_or_nseg, int64_t S_or_T, int64_t D,
                         float eps, void* stream, void* y, float* mean, float* rstd, int dtype,
                         int mod) {
    Shape sh;
    const Shape* force;
    if (!read_shape(shape, &sh, &force)) return LNMOD_EINVAL;
    const bool varlen = cu_seqlens != nullptr;
    if (varlen && mod != LNMOD_PER_SAMPLE) return LNMOD_EINVAL;
    int64_t S, T;
    if (!batch_shape(varlen, B_or_nseg, S_or_T, &S, &T)) return LNMOD_EINVAL;
    return forward_impl(x, shift, scale, cu_seqlens, varlen, B_or_nseg, S, T, D, eps, stream, y, mean,
                        rstd, dtype, mod, force);
}

int lnmod_backward_shaped(const int* shape, const void* dy, const void* x, const void* scale,
                          const int32_t* cu_seqlens, int64_t B_or_nseg, int64_t S_or_T, int64_t D,
                          float eps, void* stream, const float* mean, const float* rstd, void* dx,
                          void* dshift, void* dscale, void* workspace, size_t workspace_size,
                          int dtype, int mod) {
    Shape sh;
    const Shape* force;
    if (!read_shape(shape, &sh, &force)) return LNMOD_EINVAL;
    const bool varlen = cu_seqlens != nullptr;
    if (varlen && mod != LNMOD_PER_SAMPLE) return LNMOD_EINVAL;
    int64_t S, T;
    if (!batch_shape(varlen, B_or_nseg, S_or_T, &S, &T)) return LNMOD_EINVAL;
    return backward_impl(dy, x, scale, cu_seqlens, varlen, B_or_nseg, S, T, D, eps, stream, mean, rstd,
                         dx, dshift, dscale, workspace, workspace_size, dtype, mod, force);
}

size_t lnmod_backward_workspace_bytes_shaped(const int* shape, int64_t B_or_nseg, int64_t total,
                                             int64_t D, int mod) {
    Shape sh;
    const Shape* force;
    if (!read_shape(shape, &sh, &force)) return 0;
    if (mod != LNMOD_PER_SAMPLE) return 0;
    if (B_or_nseg < 0 || total < 0 || total >= (int64_t(1) << 31)) return 0;
    if (D < 8 || D > lnmod::kMaxD || D % 4 != 0) return 0;
    return workspace_bytes(B_or_nseg, total, D, force);
}

int lnmod_describe_launch(int backward, const int* shape, int64_t B_or_nseg, int64_t S_or_T,
                          int varlen, int64_t D, int dtype, int mod, int recompute, char* buf,
                          size_t n) {
    if (!buf || n == 0) return 0;
    buf[0] = '\0';
    Shape sh;
    const Shape* force;
    if (!read_shape(shape, &sh, &force)) return 0;
    if (mod != LNMOD_PER_SAMPLE && mod != LNMOD_PER_TOKEN) return 0;
    int64_t S, T;
    if (!batch_shape(varlen != 0, B_or_nseg, S_or_T, &S, &T)) return 0;
    if (check_shape(B_or_nseg, S_or_T, D, 1.0f, dtype, T) != LNMOD_OK || T == 0 || B_or_nseg == 0) return 0;
    // the plans look at the segment count and the totals, never at the table's contents
    const Problem p{dtype, nullptr, B_or_nseg, S, T, D, 1.0f, force};
    const int k = backward ? lnmod::describe_bwd(p, mod == LNMOD_PER_TOKEN, recompute != 0, buf, n)
                           : lnmod::describe_fwd(p, mod == LNMOD_PER_TOKEN, buf, n);
    if (k < 0) return 0;
    return static_cast<size_t>(k) < n ? k : static_cast<int>(n - 1);
}

}  // extern "C"
