// lnmod_gated_bwd.hip -- instantiation and launch of the gated residual + LayerNorm-Modulate
// backward (dx, du, and the per-sample / per-segment dgate, dshift, dscale) and of its second,
// fixed-order reduction pass.
#include "lnmod_gated_kernels.hpp"
#include "lnmod_launch.hpp"

namespace lnmod {
namespace {

// Launch shape (see Shape in lnmod_launch.hpp).  A lane holds 8 features of a row (one bf16 chunk,
// two fp32 chunks): with five fp32 values per feature living in registers (1+scale, gate, three
// running sums) and four packed input streams prefetched one step ahead, that is what fits
// without spilling.  bf16 rows of 9 to 16 times 512 features take two chunks per lane on 6 or 8
// waves instead (whole multiples of the four SIMDs; D = 5120: 798 against 819 us, and sixteen
// waves would halve the registers a wave may use).  One block per CU once a row needs three
// waves; two rows per step for rows up to 8 KB.  Timed like the other tables (D = 1536 ... 8192).
constexpr int kWaveCounts[] = {1, 2, 3, 4, 5, 6, 8, 10, 12, 16};

Shape gated_bwd_shape(int nchunks, int dtype, int64_t row_bytes) {
    const int vpl = dtype == 0 ? 1 : 2;
    const int need = (nchunks + kWave * vpl - 1) / (kWave * vpl);
    int K = 16;
    for (int k : kWaveCounts)
        if (k >= need) {
            K = k;
            break;
        }
    int per_cu = 6 / K;
    if (per_cu < 1 || K >= 3) per_cu = 1;
    Shape sh{K, vpl, row_bytes <= 8192 ? 2 : 1, per_cu};
    if (dtype == 0) {
        const int cols = (nchunks + kWave - 1) / kWave;
        if (cols == 1) sh = {1, 1, 2, 3};                // D = 512: 800 against 880 us for six blocks per CU
        if (cols == 2) sh = {2, 1, 1, 2};                // D = 1024: 809 against 856 us
        if (cols == 4) sh.R = 1;                         // D = 2048: 5.97 against 5.6 TB/s
        if (cols == 5) sh = {5, 1, 1, 1};                // D = 2560: 773 against 801 us for two rows
        if (cols == 6) sh = {8, 1, 1, 1};                // D = 3072: 768 against 805 us for six waves
        if (cols >= 9 && cols <= 10) sh = {8, 2, 1, 1};
        if (cols >= 11 && cols <= 12) sh = {6, 2, 1, 1};
        if (cols >= 13) sh = {8, 2, 1, 1};
    }
    if (dtype == 1) {
        // fp32, per 512 features: D = 512: 774 against 880 us, D = 1024: 783 against 863 us,
        // D = 3584: 819 against 857 us
        const int cols = (nchunks + 127) / 128;
        if (cols == 1) sh = {1, 2, 1, 3};
        if (cols == 2) sh = {3, 2, 1, 2};
        if (cols == 7) sh = {8, 2, 2, 1};
    }
    return sh;
}

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
    // two rows per step only for rows up to 8 KB: at most 8 waves of 8 features per lane
    if constexpr (K <= 8 && (VPL == 1 || IO<Tag>::E == 4)) {
        if (R == 2) {
            go_r<Tag, VPL, K, 2>(a, blocks, st);
            return;
        }
    }
    go_r<Tag, VPL, K, 1>(a, blocks, st);
}

template <typename Tag, int VPL>
bool dispatch(const GatedBwdArgs& a, Shape sh, int64_t blocks, hipStream_t st) {
    if (sh.VPL != VPL) {                     // the two-chunk shapes of wide bf16 rows
        if (sh.VPL != 2) return false;
        if (sh.K == 8) go<Tag, 2, 8>(a, sh.R, blocks, st);
        else if (sh.K == 6) go<Tag, 2, 6>(a, sh.R, blocks, st);
        else return false;
        return true;
    }
    switch (sh.K) {
        case 1: go<Tag, VPL, 1>(a, sh.R, blocks, st); return true;
        case 2: go<Tag, VPL, 2>(a, sh.R, blocks, st); return true;
        case 3: go<Tag, VPL, 3>(a, sh.R, blocks, st); return true;
        case 4: go<Tag, VPL, 4>(a, sh.R, blocks, st); return true;
        case 5: go<Tag, VPL, 5>(a, sh.R, blocks, st); return true;
        case 6: go<Tag, VPL, 6>(a, sh.R, blocks, st); return true;
        case 8: go<Tag, VPL, 8>(a, sh.R, blocks, st); return true;
        case 10: go<Tag, VPL, 10>(a, sh.R, blocks, st); return true;
        case 12: go<Tag, VPL, 12>(a, sh.R, blocks, st); return true;
        case 16: go<Tag, VPL, 16>(a, sh.R, blocks, st); return true;
        default: return false;
    }
}

}  // namespace

Shape gated_bwd_table_shape(int nchunks, int dtype) {
    return gated_bwd_shape(nchunks, dtype, static_cast<int64_t>(nchunks) * 16);
}

RowPlan gated_bwd_plan(int64_t T, int64_t nseg, int64_t D, int dtype) {
    const int E = dtype == 0 ? 8 : 4;
    const Shape sh = gated_bwd_shape(static_cast<int>(D / E), dtype, D * (dtype == 0 ? 2 : 4));
    // a row moves 6 D elements (dy, dh, h, u, dx, du), a slot 3 D floats written and read back
    const double elem = dtype == 0 ? 2.0 : 4.0;
    const double stream_us = static_cast<double>(T) * static_cast<double>(D) * 6.0 * elem / 5.8e6;
    return plan_rows_slots(T, nseg, static_cast<int64_t>(kNumCU) * sh.per_cu, sh.R, stream_us,
                           24.0 / (6.0 * elem));
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
    const Shape sh = gated_bwd_shape(a.nchunks, p.dtype, p.D * (p.dtype == 0 ? 2 : 4));
    if (!covers(sh, a.nchunks)) return hipErrorInvalidConfiguration;
    const RowPlan pl = gated_bwd_plan(p.T, p.nseg, p.D, p.dtype);
    a.rows_per_cluster = pl.rows_per_cluster;
    a.nb = pl.nb;
    const bool ok = p.dtype == 0 ? dispatch<bf16_io, 1>(a, sh, pl.blocks, st)
                                 : dispatch<f32_io, 2>(a, sh, pl.blocks, st);
    if (!ok) return hipErrorInvalidConfiguration;
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;

    ReduceArgs r;
    r.ws = ws;
    r.out[0] = dshift;
    r.out[1] = dscale;
    r.out[2] = dgate;
    r.seg = a.seg;
    r.T = p.T;
    r.rows_per_cluster = a.rows_per_cluster;
    r.nb = a.nb;
    r.D = a.D;
    r.nsum = 3;
    return launch_reduce(r, pl.clusters, st);
}

}  // namespace lnmod
