// lnmod_gated_fwd.hip -- instantiation and launch of the gated residual + LayerNorm-Modulate
// forward, and of the residual-only kernel that serves as the unfused comparator's first half.
#include "lnmod_gated_kernels.hpp"
#include "lnmod_launch.hpp"

namespace lnmod {
namespace {

constexpr int kRows = 2;           // rows per block and step

// Two input and two output streams per row: the waves per CU that stream best for the plain
// forward (one input, one output) carry twice the bytes here, so the same counts are kept.
int blocks_per_cu(int K) {
    if (K == 1) return 4;
    if (K == 3) return 2;              // three waves alone leave a CU short
    const int b = 5 / K;
    return b < 1 ? 1 : b;
}

// bf16 rows of 9 to 12 times 512 features (D = 4608 .. 6144) go to 4 waves with 3 chunks per
// lane and one row per step: one wave per SIMD keeps the four SIMDs of a CU evenly loaded, where
// five waves put two on one of them (D = 5120: 537 against 560 us).
constexpr bool balanced4(int VPL, int K) { return VPL == 3 && K == 4; }

Split gated_fwd_split(int nchunks, int dtype) {
    if (dtype == 0) {
        const int need = (nchunks + kWave - 1) / kWave;
        if (need >= 9 && need <= 12) return {4, 3};
    }
    return choose_split(nchunks, dtype);
}

int rows_per_step(Split sp) { return balanced4(sp.VPL, sp.K) ? 1 : kRows; }

template <typename Tag, int VPL, int K, bool LN>
void go(const GatedFwdArgs& a, int64_t blocks, hipStream_t st) {
    constexpr int R = balanced4(VPL, K) ? 1 : kRows;
    const dim3 grid(static_cast<unsigned>(blocks)), block(K * kWave);
    if (a.nchunks == K * VPL * kWave)
        hipLaunchKernelGGL((gated_fwd_kernel<Tag, VPL, K, R, true, LN>), grid, block, 0, st, a);
    else
        hipLaunchKernelGGL((gated_fwd_kernel<Tag, VPL, K, R, false, LN>), grid, block, 0, st, a);
}

template <typename Tag, int VPL_WIDE, bool LN>
void dispatch(const GatedFwdArgs& a, Split sp, int64_t blocks, hipStream_t st) {
    if (sp.K == 1) {
        switch (sp.VPL) {
            case 1: go<Tag, 1, 1, LN>(a, blocks, st); break;
            case 2: go<Tag, 2, 1, LN>(a, blocks, st); break;
            case 3: go<Tag, 3, 1, LN>(a, blocks, st); break;
            default:                             // 4 and 6 chunks per lane: fp32 rows only
                if constexpr (IO<Tag>::E == 4) {
                    if (sp.VPL == 4) go<Tag, 4, 1, LN>(a, blocks, st);
                    else go<Tag, 6, 1, LN>(a, blocks, st);
                }
                break;
        }
        return;
    }
    if (balanced4(sp.VPL, sp.K)) {
        go<Tag, 3, 4, LN>(a, blocks, st);
        return;
    }
    switch (sp.K) {
        case 2: go<Tag, VPL_WIDE, 2, LN>(a, blocks, st); break;
        case 3: go<Tag, VPL_WIDE, 3, LN>(a, blocks, st); break;
        case 4: go<Tag, VPL_WIDE, 4, LN>(a, blocks, st); break;
        case 5: go<Tag, VPL_WIDE, 5, LN>(a, blocks, st); break;
        case 6: go<Tag, VPL_WIDE, 6, LN>(a, blocks, st); break;
        default: go<Tag, VPL_WIDE, 8, LN>(a, blocks, st); break;
    }
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
    const Split sp = LN ? gated_fwd_split(a.nchunks, p.dtype) : choose_split(a.nchunks, p.dtype);
    const RowPlan pl = plan_rows(p.T, p.nseg, static_cast<int64_t>(kNumCU) * blocks_per_cu(sp.K),
                                 rows_per_step(sp), 20);
    a.rows_per_cluster = pl.rows_per_cluster;
    a.nb = pl.nb;
    if (p.dtype == 0) dispatch<bf16_io, 2, LN>(a, sp, pl.blocks, st);
    else dispatch<f32_io, 4, LN>(a, sp, pl.blocks, st);
    return hipGetLastError();
}

}  // namespace

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
