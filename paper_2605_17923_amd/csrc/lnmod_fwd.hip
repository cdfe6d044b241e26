// lnmod_fwd.hip -- instantiation and launch of the forward kernels (per-sample / per-segment
// modulation kept in registers by K waves per row, and per-token modulation streamed with x).
#include "lnmod_kernels.hpp"
#include "lnmod_launch.hpp"

namespace lnmod {
namespace {

constexpr int kFwdRows = 2;        // rows per block and step, one modulation row per segment
constexpr int kTokRows = 1;        // rows per block and step, modulation streamed per token

// About 4 or 5 waves per CU, each with its chunks of the current step in registers and those of
// the next step in flight, stream best.
int fwd_blocks_per_cu(int K) {
    if (K == 1) return 4;
    if (K == 3) return 2;              // three waves alone leave a CU short (D = 3072: 5.3 against 4.5 TB/s)
    const int b = 5 / K;
    return b < 1 ? 1 : b;
}

// Per-token modulation streams three inputs per row and takes one row per step: twice the waves.
int tok_blocks_per_cu(int K) {
    if (K == 1) return 8;
    const int b = 10 / K;
    return b < 1 ? 1 : b;
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

// fp32 rows shared by several waves carry twice the bytes per wave of bf16 rows: one row per
// step and twice the blocks stream better there (266 against 287 us on 37800 x 5120).
constexpr bool wide_fp32(int elems_per_chunk, int K) { return elems_per_chunk == 4 && K > 1; }

int seg_rows(int dtype, int K) { return wide_fp32(dtype == 0 ? 8 : 4, K) ? 1 : kFwdRows; }

template <typename Tag, int VPL, int K, int MODE>
void go_split(const FwdArgs& a, int64_t blocks, hipStream_t st) {
    constexpr int R = MODE == kModToken ? kTokRows : wide_fp32(IO<Tag>::E, K) ? 1 : kFwdRows;
    const dim3 grid(static_cast<unsigned>(blocks)), block(K * kWave);
    if (a.nchunks == K * VPL * kWave)
        hipLaunchKernelGGL((fwd_split_kernel<Tag, VPL, K, R, true, MODE>), grid, block, 0, st, a);
    else
        hipLaunchKernelGGL((fwd_split_kernel<Tag, VPL, K, R, false, MODE>), grid, block, 0, st, a);
}

// VPL_WIDE: chunks per lane when several waves share a row (fixed by the dtype)
template <typename Tag, int VPL_WIDE, int MODE>
void dispatch_split(const FwdArgs& a, Split sp, int64_t blocks, hipStream_t st) {
    if (sp.K == 1) {
        switch (sp.VPL) {
            case 1: go_split<Tag, 1, 1, MODE>(a, blocks, st); break;
            case 2: go_split<Tag, 2, 1, MODE>(a, blocks, st); break;
            case 3: go_split<Tag, 3, 1, MODE>(a, blocks, st); break;
            case 4: go_split<Tag, 4, 1, MODE>(a, blocks, st); break;
            default: go_split<Tag, 6, 1, MODE>(a, blocks, st); break;
        }
        return;
    }
    switch (sp.K) {
        case 2: go_split<Tag, VPL_WIDE, 2, MODE>(a, blocks, st); break;
        case 3: go_split<Tag, VPL_WIDE, 3, MODE>(a, blocks, st); break;
        case 4: go_split<Tag, VPL_WIDE, 4, MODE>(a, blocks, st); break;
        case 5: go_split<Tag, VPL_WIDE, 5, MODE>(a, blocks, st); break;
        case 6: go_split<Tag, VPL_WIDE, 6, MODE>(a, blocks, st); break;
        default: go_split<Tag, VPL_WIDE, 8, MODE>(a, blocks, st); break;
    }
}

template <int MODE>
hipError_t launch_mode(const Problem& p, const void* x, const void* shift, const void* scale, void* y,
                       float* mean, float* rstd, hipStream_t st) {
    const int E = p.dtype == 0 ? 8 : 4;
    FwdArgs a = make_args(p, x, shift, scale, y, mean, rstd, E);
    const Split sp = choose_split(a.nchunks, p.dtype);
    const bool per_segment = MODE == kModSegment || MODE == kModOnly;
    const int rows = MODE == kModToken ? kTokRows : seg_rows(p.dtype, sp.K);
    const int per_cu = MODE == kModToken ? tok_blocks_per_cu(sp.K)
                                         : fwd_blocks_per_cu(sp.K) * (kFwdRows / rows);
    const RowPlan pl = plan_rows(p.T, per_segment ? p.nseg : 1, static_cast<int64_t>(kNumCU) * per_cu, rows, 20);
    a.rows_per_cluster = pl.rows_per_cluster;
    a.nb = pl.nb;
    if (p.dtype == 0) dispatch_split<bf16_io, 2, MODE>(a, sp, pl.blocks, st);
    else dispatch_split<f32_io, 4, MODE>(a, sp, pl.blocks, st);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_fwd_seg(const Problem& p, const void* x, const void* shift, const void* scale,
                          void* y, float* mean, float* rstd, hipStream_t st) {
    return launch_mode<kModSegment>(p, x, shift, scale, y, mean, rstd, st);
}

hipError_t launch_fwd_tok(const Problem& p, const void* x, const void* shift, const void* scale,
                          void* y, float* mean, float* rstd, hipStream_t st) {
    return launch_mode<kModToken>(p, x, shift, scale, y, mean, rstd, st);
}

// The unfused comparator: LayerNorm to xhat (I/O dtype) in HBM, then the modulation of xhat.
hipError_t launch_unfused(const Problem& p, const void* x, const void* shift, const void* scale,
                          void* xhat, void* y, float* mean, float* rstd, hipStream_t st) {
    const hipError_t e = launch_mode<kLnOnly>(p, x, nullptr, nullptr, xhat, mean, rstd, st);
    if (e != hipSuccess) return e;
    return launch_mode<kModOnly>(p, xhat, shift, scale, y, nullptr, nullptr, st);
}

}  // namespace lnmod
