// lnmod_fwd.hip -- instantiation and launch of the forward kernels (per-sample / per-segment
// modulation through LDS, and per-token modulation streamed with x).
#include "lnmod_kernels.hpp"
#include "lnmod_launch.hpp"

namespace lnmod {
namespace {

constexpr int kFwdWaves = 4;                    // waves (= rows in flight) per block
constexpr size_t kLdsPerCU = 160 * 1024;

// Resident blocks per CU: 8 waves per CU stream best whatever the row length (more concurrent
// waves lower the achieved HBM bandwidth), so 2 blocks of 4 waves, LDS permitting.
int fwd_blocks_per_cu(size_t lds_bytes) {
    int bpc = 2;
    if (lds_bytes) {
        const int fit = static_cast<int>((kLdsPerCU - 8 * 1024) / lds_bytes);
        if (bpc > fit) bpc = fit;
    }
    return bpc < 1 ? 1 : bpc;
}

FwdArgs make_args(const Problem& p, const void* x, const void* shift, const void* scale, void* y,
                  float* mean, float* rstd, int E) {
    FwdArgs a;
    a.x = x;
    a.shift = shift;
    a.scale = scale;
    a.y = y;
    a.mean = mean;
    a.rstd = rstd;
    a.seg = Segments{p.cu, p.S, p.nseg};
    a.T = p.T;
    a.rows_per_cluster = 0;
    a.nb = 1;
    a.D = static_cast<int32_t>(p.D);
    a.nchunks = static_cast<int32_t>(p.D / E);
    a.eps = p.eps;
    a.inv_D = 1.0f / static_cast<float>(p.D);
    return a;
}

template <typename Tag, int VPL>
void go_seg(FwdArgs a, hipStream_t st) {
    constexpr int E = IO<Tag>::E;
    const size_t lds = static_cast<size_t>(2) * VPL * kWave * E * sizeof(float);
    const int bpc = fwd_blocks_per_cu(lds);
    const RowPlan pl = plan_rows(a.T, a.seg.nseg, static_cast<int64_t>(kNumCU) * bpc, kFwdWaves, 20);
    a.rows_per_cluster = pl.rows_per_cluster;
    a.nb = pl.nb;
    const dim3 grid(static_cast<unsigned>(pl.blocks)), block(kFwdWaves * kWave);
    if (a.nchunks == VPL * kWave)
        hipLaunchKernelGGL((fwd_seg_kernel<Tag, VPL, kFwdWaves, true>), grid, block, lds, st, a);
    else
        hipLaunchKernelGGL((fwd_seg_kernel<Tag, VPL, kFwdWaves, false>), grid, block, lds, st, a);
}

template <typename Tag, int VPL>
void go_tok(FwdArgs a, hipStream_t st) {
    const int bpc = fwd_blocks_per_cu(0);
    int64_t blocks = (a.T + kFwdWaves - 1) / kFwdWaves;
    if (blocks > static_cast<int64_t>(kNumCU) * bpc) blocks = static_cast<int64_t>(kNumCU) * bpc;
    const dim3 grid(static_cast<unsigned>(blocks)), block(kFwdWaves * kWave);
    if (a.nchunks == VPL * kWave)
        hipLaunchKernelGGL((fwd_tok_kernel<Tag, VPL, kFwdWaves, true>), grid, block, 0, st, a);
    else
        hipLaunchKernelGGL((fwd_tok_kernel<Tag, VPL, kFwdWaves, false>), grid, block, 0, st, a);
}

// chunks per lane: the smallest instantiated count that covers the row
#define LNMOD_FWD_DISPATCH(GO, TAG, NEED, ...)                                   \
    do {                                                                         \
        if ((NEED) <= 1) GO<TAG, 1>(__VA_ARGS__);                                \
        else if ((NEED) <= 2) GO<TAG, 2>(__VA_ARGS__);                           \
        else if ((NEED) <= 3) GO<TAG, 3>(__VA_ARGS__);                           \
        else if ((NEED) <= 4) GO<TAG, 4>(__VA_ARGS__);                           \
        else if ((NEED) <= 5) GO<TAG, 5>(__VA_ARGS__);                           \
        else if ((NEED) <= 6) GO<TAG, 6>(__VA_ARGS__);                           \
        else if ((NEED) <= 8) GO<TAG, 8>(__VA_ARGS__);                           \
        else if ((NEED) <= 10) GO<TAG, 10>(__VA_ARGS__);                         \
        else if ((NEED) <= 12) GO<TAG, 12>(__VA_ARGS__);                         \
        else GO<TAG, 16>(__VA_ARGS__);                                           \
    } while (0)

// fp32 rows have twice the chunks: up to 32 per lane at D = 8192
#define LNMOD_FWD_DISPATCH_WIDE(GO, TAG, NEED, ...)                              \
    do {                                                                         \
        if ((NEED) <= 16) LNMOD_FWD_DISPATCH(GO, TAG, NEED, __VA_ARGS__);        \
        else if ((NEED) <= 20) GO<TAG, 20>(__VA_ARGS__);                         \
        else if ((NEED) <= 24) GO<TAG, 24>(__VA_ARGS__);                         \
        else GO<TAG, 32>(__VA_ARGS__);                                           \
    } while (0)

}  // namespace

hipError_t launch_fwd_seg(const Problem& p, const void* x, const void* shift, const void* scale,
                          void* y, float* mean, float* rstd, hipStream_t st) {
    if (p.dtype == 0) {
        const FwdArgs a = make_args(p, x, shift, scale, y, mean, rstd, 8);
        const int need = (a.nchunks + kWave - 1) / kWave;      // <= 16 for D <= 8192
        LNMOD_FWD_DISPATCH(go_seg, bf16_io, need, a, st);
    } else {
        const FwdArgs a = make_args(p, x, shift, scale, y, mean, rstd, 4);
        const int need = (a.nchunks + kWave - 1) / kWave;      // <= 32
        LNMOD_FWD_DISPATCH_WIDE(go_seg, f32_io, need, a, st);
    }
    return hipGetLastError();
}

hipError_t launch_fwd_tok(const Problem& p, const void* x, const void* shift, const void* scale,
                          void* y, float* mean, float* rstd, hipStream_t st) {
    if (p.dtype == 0) {
        const FwdArgs a = make_args(p, x, shift, scale, y, mean, rstd, 8);
        const int need = (a.nchunks + kWave - 1) / kWave;
        LNMOD_FWD_DISPATCH(go_tok, bf16_io, need, a, st);
    } else {
        const FwdArgs a = make_args(p, x, shift, scale, y, mean, rstd, 4);
        const int need = (a.nchunks + kWave - 1) / kWave;
        LNMOD_FWD_DISPATCH_WIDE(go_tok, f32_io, need, a, st);
    }
    return hipGetLastError();
}

}  // namespace lnmod
