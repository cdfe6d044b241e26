// lnmod_gated_fwd.hip -- instantiation and launch of the gated residual + LayerNorm-Modulate
// forward, and of the residual-only kernel that serves as the unfused comparator's first half.
#include "lnmod_gated_kernels.hpp"
#include "lnmod_launch.hpp"

namespace lnmod {
namespace {

// Launch shape (see Shape in lnmod_launch.hpp).  The rule: the split of choose_split, two rows per
// step, about five waves per CU.  The widths where a sweep of every compiled shape (multiples of
// 512 features, 774 MB per tensor, both element types) beat the rule override it; the winners
// again are multiples of the four SIMDs of a CU or one block of five waves.
int blocks_per_cu(int K) {
    if (K == 1) return 4;
    if (K == 3) return 2;              // three waves alone leave a CU short
    const int b = 5 / K;
    return b < 1 ? 1 : b;
}

Shape gated_fwd_shape(int nchunks, int dtype, bool ln) {
    const Split sp = choose_split(nchunks, dtype);
    Shape sh{sp.K, sp.VPL, 2, blocks_per_cu(sp.K)};
    if (dtype == 0 && ln) {
        const int cols = (nchunks + kWave - 1) / kWave;
        switch (cols) {
            case 2: sh = {2, 2, 1, 4}; break;       // D = 1024: 523 against 549 us for one wave
            case 3:                                 // D = 1536: 524 against 542 us for one wave x 3
            case 4: sh = {2, 2, 1, 3}; break;
            case 5:
            case 6: sh = {3, 2, 1, 2}; break;
            case 7: sh = {4, 2, 2, 1}; break;       // D = 3584: 531 against 557 us for five waves
            case 8: sh = {4, 3, 1, 1}; break;       // D = 4096: 515 against 521 us for five waves x 2
            case 9: sh = {5, 2, 2, 1}; break;       // D = 4608: 517 against 546 us for four waves x 3
            case 10:
            case 11:
            case 12: sh = {4, 3, 1, 1}; break;      // D = 5120: 537 against 560 us for five waves x 2
            case 13:
            case 14: sh = {8, 2, 2, 1}; break;      // D = 6656, 7168: 530 against 583 us for one row, two blocks
            case 15: sh = {8, 2, 1, 1}; break;      // D = 7680: 541 against 582 us for two blocks
            default:                                // D = 8192: 527 against 572 us for two rows, one block
                if (cols >= 16) sh = {8, 2, 1, 2};
                break;
        }
    }
    if (dtype == 1 && ln) {
        // fp32, per 512 features (128 chunks): the widths where the sweep beat the rule by 2 % or more
        switch ((nchunks + 127) / 128) {
            case 1: sh = {1, nchunks <= 64 ? 1 : 4, 2, 4}; break;    // D = 512: 515 against 535 us
            case 3: sh = {2, 4, 1, 2}; break;                        // D = 1536: 556 against 576 us
            case 4: sh = {3, 4, 2, 2}; break;                        // D = 2048: 527 against 541 us
            case 6: sh = {5, 4, 2, 1}; break;                        // D = 3072: 538 against 565 us
            case 8: sh = {5, 4, 1, 3}; break;                        // D = 4096: 528 against 555 us
            case 16: sh = {8, 4, 2, 2}; break;                       // D = 8192: 568 against 592 us
            default: break;
        }
    }
    if (dtype == 0 && !ln) {
        // the residual-only kernel (first half of the unfused comparator) at the two model widths:
        // D = 1536: 366 against 393 us, D = 5120: 385 against 401 us on 774 MB per tensor
        const int cols = (nchunks + kWave - 1) / kWave;
        if (cols == 3) sh = {3, 2, 2, 2};
        if (cols >= 9 && cols <= 12) sh = {4, 3, 2, 1};
    }
    return sh;
}

template <typename Tag, int VPL, int K, int R, bool LN>
void go_r(const GatedFwdArgs& a, int64_t blocks, hipStream_t st) {
    const dim3 grid(static_cast<unsigned>(blocks)), block(K * kWave);
    if (a.nchunks == K * VPL * kWave)
        hipLaunchKernelGGL((gated_fwd_kernel<Tag, VPL, K, R, true, LN>), grid, block, 0, st, a);
    else
        hipLaunchKernelGGL((gated_fwd_kernel<Tag, VPL, K, R, false, LN>), grid, block, 0, st, a);
}

template <typename Tag, int VPL, int K, bool LN>
void go(const GatedFwdArgs& a, int R, int64_t blocks, hipStream_t st) {
    if constexpr (LN && IO<Tag>::E == 8) {               // only the bf16 table asks for one row
        if (R == 1) {
            go_r<Tag, VPL, K, 1, LN>(a, blocks, st);
            return;
        }
    }
    go_r<Tag, VPL, K, 2, LN>(a, blocks, st);
}

template <typename Tag, bool LN>
bool dispatch(const GatedFwdArgs& a, Shape sh, int64_t blocks, hipStream_t st) {
    switch (sh.VPL * 100 + sh.K) {
        case 101: go<Tag, 1, 1, LN>(a, sh.R, blocks, st); return true;
        case 201: go<Tag, 2, 1, LN>(a, sh.R, blocks, st); return true;
        case 301: go<Tag, 3, 1, LN>(a, sh.R, blocks, st); return true;
        default: break;
    }
    if constexpr (IO<Tag>::E == 8) {
        switch (sh.VPL * 100 + sh.K) {
            case 202: go<Tag, 2, 2, LN>(a, sh.R, blocks, st); return true;
            case 203: go<Tag, 2, 3, LN>(a, sh.R, blocks, st); return true;
            case 204: go<Tag, 2, 4, LN>(a, sh.R, blocks, st); return true;
            case 205: go<Tag, 2, 5, LN>(a, sh.R, blocks, st); return true;
            case 206: go<Tag, 2, 6, LN>(a, sh.R, blocks, st); return true;
            case 208: go<Tag, 2, 8, LN>(a, sh.R, blocks, st); return true;
            case 304: go<Tag, 3, 4, LN>(a, sh.R, blocks, st); return true;
            default: break;
        }
    } else {
        switch (sh.VPL * 100 + sh.K) {
            case 401: go<Tag, 4, 1, LN>(a, sh.R, blocks, st); return true;
            case 601: go<Tag, 6, 1, LN>(a, sh.R, blocks, st); return true;
            case 402: go<Tag, 4, 2, LN>(a, sh.R, blocks, st); return true;
            case 403: go<Tag, 4, 3, LN>(a, sh.R, blocks, st); return true;
            case 404: go<Tag, 4, 4, LN>(a, sh.R, blocks, st); return true;
            case 405: go<Tag, 4, 5, LN>(a, sh.R, blocks, st); return true;
            case 406: go<Tag, 4, 6, LN>(a, sh.R, blocks, st); return true;
            case 408: go<Tag, 4, 8, LN>(a, sh.R, blocks, st); return true;
            default: break;
        }
    }
    return false;
}

template <bool LN>
hipError_t launch(const Problem& p, const void* x, const void* u, const void* gate, const void* shift,
                  const void* scale, void* h, void* y, float* mean, float* rstd, hipStream_t st) {
    const int E = p.dtype == 0 ? 8 : 4;
    GatedFwdArgs a;
    a.x = x;
    a.u = u;
    a.gate = gate;
    a.shift = shift;
    a.scale = scale;
    a.h = h;
    a.y = y;
    a.mean = mean;
    a.rstd = rstd;
    a.seg = Segments{p.cu, p.S, p.nseg};
    a.T = p.T;
    a.D = static_cast<int32_t>(p.D);
    a.nchunks = static_cast<int32_t>(p.D / E);
    a.eps = p.eps;
    a.inv_D = 1.0f / static_cast<float>(p.D);
    const Shape sh = gated_fwd_shape(a.nchunks, p.dtype, LN);
    if (!covers(sh, a.nchunks)) return hipErrorInvalidConfiguration;
    // bytes of x, u, h and y at 6 TB/s
    const double stream_us = static_cast<double>(p.T) * static_cast<double>(p.D) * (p.dtype == 0 ? 8.0 : 16.0) / 6.0e6;
    const RowPlan pl = plan_rows_clusters(p.T, p.nseg, static_cast<int64_t>(kNumCU) * sh.per_cu, sh.R,
                                          pick_clusters(stream_us, p.nseg));
    a.rows_per_cluster = pl.rows_per_cluster;
    a.nb = pl.nb;
    const bool ok = p.dtype == 0 ? dispatch<bf16_io, LN>(a, sh, pl.blocks, st)
                                 : dispatch<f32_io, LN>(a, sh, pl.blocks, st);
    return ok ? hipGetLastError() : hipErrorInvalidConfiguration;
}

}  // namespace

Shape gated_fwd_table_shape(int nchunks, int dtype) { return gated_fwd_shape(nchunks, dtype, true); }

hipError_t launch_gated_fwd(const Problem& p, const void* x, const void* u, const void* gate,
                            const void* shift, const void* scale, void* h, void* y, float* mean,
                            float* rstd, hipStream_t st) {
    return launch<true>(p, x, u, gate, shift, scale, h, y, mean, rstd, st);
}

hipError_t launch_gate_residual(const Problem& p, const void* x, const void* u, const void* gate,
                                void* h, hipStream_t st) {
    return launch<false>(p, x, u, gate, nullptr, nullptr, h, nullptr, nullptr, nullptr, st);
}

}  // namespace lnmod
