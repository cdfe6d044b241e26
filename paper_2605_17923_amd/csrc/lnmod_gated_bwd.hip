// lnmod_gated_bwd.hip -- instantiation and launch of the gated residual + LayerNorm-Modulate
// backward (dx, du, and the per-sample / per-segment dgate, dshift, dscale) and of its second,
// fixed-order reduction pass.
#include "lnmod_gated_kernels.hpp"
#include "lnmod_launch.hpp"

namespace lnmod {
namespace {

// A lane holds 8 features of a row (one bf16 chunk, two fp32 chunks): with five fp32 values per
// feature living in registers (1+scale, gate, three running sums) and four packed input streams
// prefetched one step ahead, that is what fits without spilling, and it streams better than 16
// features per lane on half the waves (819 against 870 us on 75600 x 5120 bf16).
constexpr int kWaveCounts[] = {1, 2, 3, 4, 5, 6, 8, 10, 12, 16};

// Exception: bf16 rows of 9 to 16 times 512 features take 8 waves with two chunks per lane (two
// waves on every SIMD of the CU) rather than 10 to 16 waves with one (D = 5120: 798 against
// 819 us; at D = 8192 sixteen waves would also halve the registers a wave may use).
Split gated_split(int nchunks, int dtype) {
    if (dtype == 0) {
        const int cols = (nchunks + kWave - 1) / kWave;
        if (cols >= 9 && cols <= 16) return {8, 2};
    }
    const int vpl = dtype == 0 ? 1 : 2;
    const int need = (nchunks + kWave * vpl - 1) / (kWave * vpl);
    for (int k : kWaveCounts)
        if (k >= need) return {k, vpl};
    return {16, vpl};                        // not reached: D <= 8192 needs at most 16 waves
}

int blocks_per_cu(int K) {
    const int b = 6 / K;
    return b < 1 ? 1 : b;
}

// Four input streams per row: one row per step already gives a wave as many bytes in flight as
// two rows give the plain backward; short rows take two.
int rows_per_step(int64_t row_bytes) { return row_bytes < 4096 ? 2 : 1; }

template <typename Tag, int VPL, int K, int R>
void go_r(const GatedBwdArgs& a, int64_t blocks, hipStream_t st) {
    const dim3 grid(static_cast<unsigned>(blocks)), block(K * kWave);
    if (a.nchunks == K * VPL * kWave)
        hipLaunchKernelGGL((gated_bwd_kernel<Tag, VPL, K, R, true>), grid, block, 0, st, a);
    else
        hipLaunchKernelGGL((gated_bwd_kernel<Tag, VPL, K, R, false>), grid, block, 0, st, a);
}

template <typename Tag, int VPL, int K>
void go(const GatedBwdArgs& a, int R, int64_t blocks, hipStream_t st) {
    if constexpr (K <= 4) {                  // rows shorter than 4 KB never need more waves
        if (R == 2) {
            go_r<Tag, VPL, K, 2>(a, blocks, st);
            return;
        }
    }
    go_r<Tag, VPL, K, 1>(a, blocks, st);
}

template <typename Tag, int VPL>
void dispatch(const GatedBwdArgs& a, Split sp, int R, int64_t blocks, hipStream_t st) {
    if (sp.VPL != VPL) {                     // the 8-wave, two-chunk split of wide bf16 rows
        go<Tag, 2, 8>(a, R, blocks, st);
        return;
    }
    switch (sp.K) {
        case 1: go<Tag, VPL, 1>(a, R, blocks, st); break;
        case 2: go<Tag, VPL, 2>(a, R, blocks, st); break;
        case 3: go<Tag, VPL, 3>(a, R, blocks, st); break;
        case 4: go<Tag, VPL, 4>(a, R, blocks, st); break;
        case 5: go<Tag, VPL, 5>(a, R, blocks, st); break;
        case 6: go<Tag, VPL, 6>(a, R, blocks, st); break;
        case 8: go<Tag, VPL, 8>(a, R, blocks, st); break;
        case 10: go<Tag, VPL, 10>(a, R, blocks, st); break;
        case 12: go<Tag, VPL, 12>(a, R, blocks, st); break;
        default: go<Tag, VPL, 16>(a, R, blocks, st); break;
    }
}

}  // namespace

RowPlan gated_bwd_plan(int64_t T, int64_t nseg, int64_t D, int dtype) {
    const int E = dtype == 0 ? 8 : 4;
    const Split sp = gated_split(static_cast<int>(D / E), dtype);
    const int R = rows_per_step(D * (dtype == 0 ? 2 : 4));
    return plan_rows(T, nseg, static_cast<int64_t>(kNumCU) * blocks_per_cu(sp.K), R, 90);
}

hipError_t launch_gated_bwd(const Problem& p, const void* dy, const void* dh, const void* h,
                            const void* u, const void* gate, const void* scale, const float* mean,
                            const float* rstd, void* dx, void* du, float* dgate, float* dshift,
                            float* dscale, float* ws, hipStream_t st) {
    const int E = p.dtype == 0 ? 8 : 4;
    GatedBwdArgs a;
    a.dy = dy;
    a.dh = dh;
    a.h = h;
    a.u = u;
    a.gate = gate;
    a.scale = scale;
    a.mean = mean;
    a.rstd = rstd;
    a.dx = dx;
    a.du = du;
    a.ws = ws;
    a.seg = Segments{p.cu, p.S, p.nseg};
    a.T = p.T;
    a.D = static_cast<int32_t>(p.D);
    a.nchunks = static_cast<int32_t>(p.D / E);
    a.inv_D = 1.0f / static_cast<float>(p.D);
    const Split sp = gated_split(a.nchunks, p.dtype);
    const RowPlan pl = gated_bwd_plan(p.T, p.nseg, p.D, p.dtype);
    a.rows_per_cluster = pl.rows_per_cluster;
    a.nb = pl.nb;
    const int R = rows_per_step(p.D * (p.dtype == 0 ? 2 : 4));
    if (p.dtype == 0) dispatch<bf16_io, 1>(a, sp, R, pl.blocks, st);
    else dispatch<f32_io, 2>(a, sp, R, pl.blocks, st);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;

    GatedReduceArgs r;
    r.ws = ws;
    r.out[0] = dshift;
    r.out[1] = dscale;
    r.out[2] = dgate;
    r.seg = a.seg;
    r.T = p.T;
    r.rows_per_cluster = a.rows_per_cluster;
    r.nb = a.nb;
    r.D = a.D;
    r.dblocks = static_cast<int32_t>((p.D + kWave - 1) / kWave);
    const dim3 grid(static_cast<unsigned>(p.nseg * 3 * r.dblocks));
    hipLaunchKernelGGL(gated_reduce_kernel<0>, grid, dim3(kReduceWaves * kWave), 0, st, r);
    return hipGetLastError();
}

}  // namespace lnmod
