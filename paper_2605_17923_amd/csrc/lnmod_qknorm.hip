// lnmod_qknorm.hip -- instantiation and launch of the fused Q-Norm + K-Norm kernels (forward,
// backward and the fixed-order second pass of the weight gradients).
#include "lnmod_qknorm_kernels.hpp"
#include "lnmod_launch.hpp"

namespace lnmod {
namespace {

constexpr int kRows = 2;           // rows per block and step

// Resident blocks per CU over both tensors together; each tensor gets half of them.
int fwd_blocks_per_cu(int K) {
    if (K == 1) return 4;
    if (K == 3) return 2;              // three waves alone leave a CU short
    const int b = 5 / K;
    return b < 1 ? 1 : b;
}
int bwd_blocks_per_cu(int K) {
    if (K == 1) return 4;
    const int b = 6 / K;
    return b < 1 ? 1 : b;
}

// Launch shape of the wide-row kernels: the split of choose_split, two rows per step, and the
// blocks per CU above (R is fixed by the instantiations).
Shape wide_table_shape(int nchunks, int dtype, bool backward) {
    const Split sp = choose_split(nchunks, dtype);
    Shape sh{sp.K, sp.VPL, kRows, backward ? bwd_blocks_per_cu(sp.K) : fwd_blocks_per_cu(sp.K)};
    if (dtype == 0) {
        // widths where the sweep of every compiled shape (D = 512 ... 8192, 774 MB per tensor) beat
        // the rule by 3 % or more
        const int cols = (nchunks + kWave - 1) / kWave;
        if (!backward) {
            if (cols == 1) sh.per_cu = 8;                    // D = 512: 555 against 670 us
            if (cols == 3) sh = {1, 3, kRows, 3};            // D = 1536: 516 against 560 us
            if (cols == 8) sh = {4, 3, kRows, 1};            // D = 4096: 527 against 562 us for 4 waves x 2
        } else {
            if (cols == 1) sh.per_cu = 6;                    // D = 512: 776 against 810 us
            if (cols == 2) sh = {1, 2, kRows, 3};            // D = 1024: 760 against 833 us
            if (cols == 3) sh = {2, 2, kRows, 3};            // D = 1536: 784 against 838 us
            if (cols == 6) sh = {3, 2, kRows, 1};            // D = 3072: 750 against 807 us
            if (cols == 7) sh = {4, 2, kRows, 2};            // D = 3584: 827 against 850 us
            if (cols == 8) sh = {5, 2, kRows, 2};            // D = 4096: 778 against 805 us
        }
    }
    if (dtype == 1 && !backward) {
        const int cols = (nchunks + 127) / 128;              // fp32, per 512 features
        if (cols == 3) sh = {2, 4, kRows, 2};                // D = 1536: 518 against 535 us
        if (cols == 6) sh = {3, 4, kRows, 1};                // D = 3072: 520 against 560 us
        if (cols == 8) sh = {5, 4, kRows, 2};                // D = 4096: 551 against 576 us
    }
    return sh;
}

// The table's shape; ok is false for a shape these kernels are not compiled for or that does not
// cover the row (a mistake in the table then fails the launch instead of computing on part of a row).
Shape wide_shape(int nchunks, int dtype, bool backward, bool* ok) {
    const Shape sh = wide_table_shape(nchunks, dtype, backward);
    const int wide = dtype == 0 ? 2 : 4;
    bool compiled;
    if (sh.K == 1) compiled = sh.VPL >= 1 && (sh.VPL <= 3 || (dtype == 1 && (sh.VPL == 4 || sh.VPL == 6)));
    else compiled = (sh.VPL == wide && (sh.K <= 6 || sh.K == 8)) || (dtype == 0 && sh.VPL == 3 && sh.K == 4);
    *ok = compiled && sh.R == kRows && covers(sh, nchunks);
    return sh;
}

int32_t blocks_per_tensor(int64_t N, int per_cu) {
    int64_t nb = static_cast<int64_t>(kNumCU) * per_cu / 2;
    const int64_t need = (N + kRows - 1) / kRows;
    if (nb > need) nb = need;
    return static_cast<int32_t>(nb < 1 ? 1 : nb);
}

template <typename Tag, int VPL, int K>
void go_fwd(const QkFwdArgs& a, hipStream_t st) {
    const dim3 grid(static_cast<unsigned>(2 * a.nb)), block(K * kWave);
    if (a.nchunks == K * VPL * kWave)
        hipLaunchKernelGGL((qknorm_fwd_kernel<Tag, VPL, K, kRows, true>), grid, block, 0, st, a);
    else
        hipLaunchKernelGGL((qknorm_fwd_kernel<Tag, VPL, K, kRows, false>), grid, block, 0, st, a);
}

template <typename Tag, int VPL, int K>
void go_bwd(const QkBwdArgs& a, hipStream_t st) {
    const dim3 grid(static_cast<unsigned>(2 * a.nb)), block(K * kWave);
    if (a.nchunks == K * VPL * kWave)
        hipLaunchKernelGGL((qknorm_bwd_kernel<Tag, VPL, K, kRows, true>), grid, block, 0, st, a);
    else
        hipLaunchKernelGGL((qknorm_bwd_kernel<Tag, VPL, K, kRows, false>), grid, block, 0, st, a);
}

// calls f.template operator()<VPL, K>() for the split; VPL_WIDE as in the other launchers
template <typename Tag, int VPL_WIDE, typename F>
void for_split(Split sp, F&& f) {
    if constexpr (IO<Tag>::E == 8) {             // bf16: three chunks per lane on four waves
        if (sp.VPL == 3 && sp.K == 4) {
            f.template operator()<3, 4>();
            return;
        }
    }
    if (sp.K == 1) {
        switch (sp.VPL) {
            case 1: f.template operator()<1, 1>(); break;
            case 2: f.template operator()<2, 1>(); break;
            case 3: f.template operator()<3, 1>(); break;
            default:                             // 4 and 6 chunks per lane: fp32 rows only
                if constexpr (IO<Tag>::E == 4) {
                    if (sp.VPL == 4) f.template operator()<4, 1>();
                    else f.template operator()<6, 1>();
                }
                break;
        }
        return;
    }
    switch (sp.K) {
        case 2: f.template operator()<VPL_WIDE, 2>(); break;
        case 3: f.template operator()<VPL_WIDE, 3>(); break;
        case 4: f.template operator()<VPL_WIDE, 4>(); break;
        case 5: f.template operator()<VPL_WIDE, 5>(); break;
        case 6: f.template operator()<VPL_WIDE, 6>(); break;
        default: f.template operator()<VPL_WIDE, 8>(); break;
    }
}

template <typename Tag>
struct FwdGo {
    const QkFwdArgs& a;
    hipStream_t st;
    template <int VPL, int K> void operator()() const { go_fwd<Tag, VPL, K>(a, st); }
};
template <typename Tag>
struct BwdGo {
    const QkBwdArgs& a;
    hipStream_t st;
    template <int VPL, int K> void operator()() const { go_bwd<Tag, VPL, K>(a, st); }
};

// Short rows (at most 32 chunks, e.g. one head's width): 16 lanes per row, four rows per wave.
constexpr int kShortMaxChunks = 32;
constexpr int kShortFwdBlocksPerCu = 8;              // blocks of 4 waves, over both tensors
constexpr int kShortBwdBlocksPerCu = 2;

// rows per wave and step = 4 * R: about 8 KB of loads per wave and step
template <int VPL> constexpr int short_fwd_r() { return VPL == 1 ? 8 : 4; }
template <int VPL> constexpr int short_bwd_r() { return VPL == 1 ? 4 : 2; }

int32_t short_blocks_per_tensor(int64_t N, int rows_per_piece, int per_cu) {
    int64_t nb = static_cast<int64_t>(kNumCU) * per_cu / 2;
    const int64_t pieces = (N + rows_per_piece - 1) / rows_per_piece;
    const int64_t need = (pieces + kShortWaves - 1) / kShortWaves;
    if (nb > need) nb = need;
    return static_cast<int32_t>(nb < 1 ? 1 : nb);
}

}  // namespace

int32_t qknorm_bwd_blocks(int64_t N, int64_t D, int dtype) {
    const int E = dtype == 0 ? 8 : 4;
    const int nchunks = static_cast<int>(D / E);
    if (nchunks <= kShortMaxChunks) {                // one slot per wave
        const int r = nchunks <= 16 ? short_bwd_r<1>() : short_bwd_r<2>();
        return short_blocks_per_tensor(N, 4 * r, kShortBwdBlocksPerCu) * kShortWaves;
    }
    bool ok;
    const Shape sh = wide_shape(nchunks, dtype, true, &ok);
    return blocks_per_tensor(N, sh.per_cu);
}

Shape qknorm_table_shape(int nchunks, int dtype, bool backward) { return wide_table_shape(nchunks, dtype, backward); }

hipError_t launch_qknorm_fwd(int dtype, const void* q, const void* k, const void* wq, const void* wk,
                             int64_t N, int64_t D, float eps, void* q_out, void* k_out,
                             float* rstd_q, float* rstd_k, hipStream_t st) {
    const int E = dtype == 0 ? 8 : 4;
    QkFwdArgs a;
    a.x[0] = q; a.x[1] = k;
    a.w[0] = wq; a.w[1] = wk;
    a.y[0] = q_out; a.y[1] = k_out;
    a.rstd[0] = rstd_q; a.rstd[1] = rstd_k;
    a.N = N;
    a.D = static_cast<int32_t>(D);
    a.nchunks = static_cast<int32_t>(D / E);
    a.eps = eps;
    a.inv_D = 1.0f / static_cast<float>(D);
    if (a.nchunks <= kShortMaxChunks) {
        const bool one = a.nchunks <= 16;
        a.nb = short_blocks_per_tensor(N, 4 * (one ? short_fwd_r<1>() : short_fwd_r<2>()), kShortFwdBlocksPerCu);
        const dim3 grid(static_cast<unsigned>(2 * a.nb)), block(kShortWaves * kWave);
        if (dtype == 0) {
            if (one) hipLaunchKernelGGL((qknorm_short_fwd_kernel<bf16_io, 1, short_fwd_r<1>()>), grid, block, 0, st, a);
            else hipLaunchKernelGGL((qknorm_short_fwd_kernel<bf16_io, 2, short_fwd_r<2>()>), grid, block, 0, st, a);
        } else {
            if (one) hipLaunchKernelGGL((qknorm_short_fwd_kernel<f32_io, 1, short_fwd_r<1>()>), grid, block, 0, st, a);
            else hipLaunchKernelGGL((qknorm_short_fwd_kernel<f32_io, 2, short_fwd_r<2>()>), grid, block, 0, st, a);
        }
        return hipGetLastError();
    }
    bool ok;
    const Shape sh = wide_shape(a.nchunks, dtype, false, &ok);
    if (!ok) return hipErrorInvalidConfiguration;
    const Split sp{sh.K, sh.VPL};
    a.nb = blocks_per_tensor(N, sh.per_cu);
    if (dtype == 0) for_split<bf16_io, 2>(sp, FwdGo<bf16_io>{a, st});
    else for_split<f32_io, 4>(sp, FwdGo<f32_io>{a, st});
    return hipGetLastError();
}

hipError_t launch_qknorm_bwd(int dtype, const void* dq_out, const void* dk_out, const void* q,
                             const void* k, const void* wq, const void* wk, int64_t N, int64_t D,
                             const float* rstd_q, const float* rstd_k, void* dq, void* dk,
                             float* dwq, float* dwk, float* ws, hipStream_t st) {
    const int E = dtype == 0 ? 8 : 4;
    QkBwdArgs a;
    a.dy[0] = dq_out; a.dy[1] = dk_out;
    a.x[0] = q; a.x[1] = k;
    a.w[0] = wq; a.w[1] = wk;
    a.rstd[0] = rstd_q; a.rstd[1] = rstd_k;
    a.dx[0] = dq; a.dx[1] = dk;
    a.ws = ws;
    a.N = N;
    a.D = static_cast<int32_t>(D);
    a.nchunks = static_cast<int32_t>(D / E);
    a.inv_D = 1.0f / static_cast<float>(D);
    int32_t slots = qknorm_bwd_blocks(N, D, dtype);              // per tensor
    if (a.nchunks <= kShortMaxChunks) {
        const bool one = a.nchunks <= 16;
        a.nb = slots / kShortWaves;
        const dim3 grid(static_cast<unsigned>(2 * a.nb)), block(kShortWaves * kWave);
        if (dtype == 0) {
            if (one) hipLaunchKernelGGL((qknorm_short_bwd_kernel<bf16_io, 1, short_bwd_r<1>()>), grid, block, 0, st, a);
            else hipLaunchKernelGGL((qknorm_short_bwd_kernel<bf16_io, 2, short_bwd_r<2>()>), grid, block, 0, st, a);
        } else {
            if (one) hipLaunchKernelGGL((qknorm_short_bwd_kernel<f32_io, 1, short_bwd_r<1>()>), grid, block, 0, st, a);
            else hipLaunchKernelGGL((qknorm_short_bwd_kernel<f32_io, 2, short_bwd_r<2>()>), grid, block, 0, st, a);
        }
    } else {
        bool ok;
        const Shape sh = wide_shape(a.nchunks, dtype, true, &ok);
        if (!ok) return hipErrorInvalidConfiguration;
        const Split sp{sh.K, sh.VPL};
        a.nb = slots;
        if (dtype == 0) for_split<bf16_io, 2>(sp, BwdGo<bf16_io>{a, st});
        else for_split<f32_io, 4>(sp, BwdGo<f32_io>{a, st});
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;

    QkReduceArgs r;
    r.ws = ws;
    r.dw[0] = dwq;
    r.dw[1] = dwk;
    r.nb = slots;
    r.D = a.D;
    r.dblocks = static_cast<int32_t>((D + kWave - 1) / kWave);
    hipLaunchKernelGGL(qknorm_reduce_kernel<0>, dim3(static_cast<unsigned>(2 * r.dblocks)),
                       dim3(kReduceWaves * kWave), 0, st, r);
    return hipGetLastError();
}

}  // namespace lnmod
