// lnmod_bwd.hip -- instantiation and launch of the backward kernels: the fused
// dx + dshift/dscale-partials kernel with its fixed-order second pass, and the per-token kernel.
#include "lnmod_kernels.hpp"
#include "lnmod_launch.hpp"

namespace lnmod {
namespace {

constexpr int kTokWaves = 4;

// How a row of `nchunks` 16-byte chunks is split: K waves per row, VPL chunks per lane, R rows
// per block and step.  A lane keeps about 16 features (up to 24 when one wave can take the
// whole row, which needs no barrier at all); longer rows are shared by more waves.
struct Split {
    int K;
    int VPL;
};

Split choose_split(int nchunks, int dtype) {
    const int per_feat16 = dtype == 0 ? 2 : 4;          // chunks holding 16 features
    const int solo_max = dtype == 0 ? 3 : 6;            // chunks per lane a single wave may take
    const int need = (nchunks + kWave - 1) / kWave;
    if (need <= solo_max) {
        int vpl = need;
        if (dtype == 1 && vpl == 5) vpl = 6;            // instantiated: 1, 2, 3, 4, 6
        return {1, vpl};
    }
    int k = (nchunks + per_feat16 * kWave - 1) / (per_feat16 * kWave);
    if (k == 7) k = 8;
    return {k, per_feat16};
}

// With the software pipeline about 5 or 6 waves per CU, each with 20 to 40 KB of loads in
// flight, reach the highest HBM bandwidth; more concurrent waves lower it.
int blocks_per_cu(int K) {
    if (K == 1) return 4;
    const int b = 6 / K;
    return b < 1 ? 1 : b;
}

// Rows per block and step: one row when a row is long enough to fill the pipeline by itself.
int rows_per_step(int K, int64_t row_bytes) { return (K > 1 && row_bytes >= 8192) ? 1 : 2; }

template <typename Tag, int VPL, int K, int R>
void go_seg_r(const BwdArgs& a, int64_t blocks, hipStream_t st) {
    const dim3 grid(static_cast<unsigned>(blocks)), block(K * kWave);
    if (a.nchunks == K * VPL * kWave)
        hipLaunchKernelGGL((bwd_seg_kernel<Tag, VPL, K, R, true>), grid, block, 0, st, a);
    else
        hipLaunchKernelGGL((bwd_seg_kernel<Tag, VPL, K, R, false>), grid, block, 0, st, a);
}

template <typename Tag, int VPL, int K>
void go_seg(const BwdArgs& a, int R, int64_t blocks, hipStream_t st) {
    if (K > 1 && R == 1) go_seg_r<Tag, VPL, K, 1>(a, blocks, st);
    else go_seg_r<Tag, VPL, K, 2>(a, blocks, st);
}

// rows wider than one wave: VPL is fixed by the dtype, K varies
template <typename Tag, int VPL>
void go_seg_k(const BwdArgs& a, int K, int R, int64_t blocks, hipStream_t st) {
    switch (K) {
        case 2: go_seg<Tag, VPL, 2>(a, R, blocks, st); break;
        case 3: go_seg<Tag, VPL, 3>(a, R, blocks, st); break;
        case 4: go_seg<Tag, VPL, 4>(a, R, blocks, st); break;
        case 5: go_seg<Tag, VPL, 5>(a, R, blocks, st); break;
        case 6: go_seg<Tag, VPL, 6>(a, R, blocks, st); break;
        default: go_seg<Tag, VPL, 8>(a, R, blocks, st); break;
    }
}

// rows one wave takes alone (two rows per step)
template <typename Tag>
void go_seg_solo(const BwdArgs& a, int VPL, int64_t blocks, hipStream_t st) {
    switch (VPL) {
        case 1: go_seg<Tag, 1, 1>(a, 2, blocks, st); break;
        case 2: go_seg<Tag, 2, 1>(a, 2, blocks, st); break;
        case 3: go_seg<Tag, 3, 1>(a, 2, blocks, st); break;
        case 4: go_seg<Tag, 4, 1>(a, 2, blocks, st); break;
        default: go_seg<Tag, 6, 1>(a, 2, blocks, st); break;
    }
}

template <typename Tag, int VPL>
void go_tok(BwdArgs a, hipStream_t st) {
    int64_t blocks = (a.T + kTokWaves - 1) / kTokWaves;
    const int64_t cap = static_cast<int64_t>(kNumCU) * (a.nchunks >= 384 ? 2 : 4);
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    const dim3 grid(static_cast<unsigned>(blocks)), block(kTokWaves * kWave);
    if (a.nchunks == VPL * kWave)
        hipLaunchKernelGGL((bwd_tok_kernel<Tag, VPL, kTokWaves, true>), grid, block, 0, st, a);
    else
        hipLaunchKernelGGL((bwd_tok_kernel<Tag, VPL, kTokWaves, false>), grid, block, 0, st, a);
}

#define LNMOD_TOK_DISPATCH(TAG, NEED, ...)                                       \
    do {                                                                         \
        if ((NEED) <= 1) go_tok<TAG, 1>(__VA_ARGS__);                            \
        else if ((NEED) <= 2) go_tok<TAG, 2>(__VA_ARGS__);                       \
        else if ((NEED) <= 3) go_tok<TAG, 3>(__VA_ARGS__);                       \
        else if ((NEED) <= 4) go_tok<TAG, 4>(__VA_ARGS__);                       \
        else if ((NEED) <= 5) go_tok<TAG, 5>(__VA_ARGS__);                       \
        else if ((NEED) <= 6) go_tok<TAG, 6>(__VA_ARGS__);                       \
        else if ((NEED) <= 8) go_tok<TAG, 8>(__VA_ARGS__);                       \
        else if ((NEED) <= 10) go_tok<TAG, 10>(__VA_ARGS__);                     \
        else if ((NEED) <= 12) go_tok<TAG, 12>(__VA_ARGS__);                     \
        else go_tok<TAG, 16>(__VA_ARGS__);                                       \
    } while (0)

BwdArgs make_args(const Problem& p, const void* dy, const void* x, const void* scale,
                  const float* mean, const float* rstd, void* dx, void* dshift, void* dscale,
                  float* ws, int E) {
    BwdArgs a;
    a.dy = dy;
    a.x = x;
    a.scale = scale;
    a.mean = mean;
    a.rstd = rstd;
    a.dx = dx;
    a.dshift = dshift;
    a.dscale = dscale;
    a.ws = ws;
    a.seg = Segments{p.cu, p.S, p.nseg};
    a.T = p.T;
    a.rows_per_cluster = 0;
    a.nb = 1;
    a.D = static_cast<int32_t>(p.D);
    a.nchunks = static_cast<int32_t>(p.D / E);
    a.inv_D = 1.0f / static_cast<float>(p.D);
    return a;
}

__global__ __launch_bounds__(256) void zero_f32_kernel(float* p, int64_t n) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += stride)
        p[i] = 0.0f;
}

}  // namespace

RowPlan bwd_plan(int64_t T, int64_t nseg, int64_t D, int dtype) {
    const int E = dtype == 0 ? 8 : 4;
    const Split sp = choose_split(static_cast<int>(D / E), dtype);
    const int R = rows_per_step(sp.K, D * (dtype == 0 ? 2 : 4));
    return plan_rows(T, nseg, static_cast<int64_t>(kNumCU) * blocks_per_cu(sp.K), R, 90);
}

hipError_t launch_bwd_seg(const Problem& p, const void* dy, const void* x, const void* scale,
                          const float* mean, const float* rstd, void* dx, float* dshift,
                          float* dscale, float* ws, hipStream_t st) {
    const int E = p.dtype == 0 ? 8 : 4;
    BwdArgs a = make_args(p, dy, x, scale, mean, rstd, dx, nullptr, nullptr, ws, E);
    const Split sp = choose_split(a.nchunks, p.dtype);
    const RowPlan pl = bwd_plan(p.T, p.nseg, p.D, p.dtype);
    const int64_t blocks = pl.blocks;
    a.rows_per_cluster = pl.rows_per_cluster;
    a.nb = pl.nb;
    const int R = rows_per_step(sp.K, p.D * (p.dtype == 0 ? 2 : 4));
    if (p.dtype == 0) {
        if (sp.K == 1) go_seg_solo<bf16_io>(a, sp.VPL, blocks, st);
        else go_seg_k<bf16_io, 2>(a, sp.K, R, blocks, st);
    } else {
        if (sp.K == 1) go_seg_solo<f32_io>(a, sp.VPL, blocks, st);
        else go_seg_k<f32_io, 4>(a, sp.K, R, blocks, st);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;

    ReduceArgs r;
    r.ws = ws;
    r.dshift = dshift;
    r.dscale = dscale;
    r.seg = a.seg;
    r.T = p.T;
    r.rows_per_cluster = a.rows_per_cluster;
    r.nb = a.nb;
    r.D = a.D;
    r.dblocks = static_cast<int32_t>((p.D + kWave - 1) / kWave);
    const dim3 grid(static_cast<unsigned>(p.nseg * 2 * r.dblocks));
    hipLaunchKernelGGL(bwd_reduce_kernel<0>, grid, dim3(kReduceWaves * kWave), 0, st, r);
    return hipGetLastError();
}

hipError_t launch_bwd_tok(const Problem& p, const void* dy, const void* x, const void* scale,
                          const float* mean, const float* rstd, void* dx, void* dshift,
                          void* dscale, hipStream_t st) {
    const int E = p.dtype == 0 ? 8 : 4;
    const BwdArgs a = make_args(p, dy, x, scale, mean, rstd, dx, dshift, dscale, nullptr, E);
    const int need = (a.nchunks + kWave - 1) / kWave;
    if (p.dtype == 0) {
        LNMOD_TOK_DISPATCH(bf16_io, need, a, st);
    } else {
        if (need <= 16) LNMOD_TOK_DISPATCH(f32_io, need, a, st);
        else if (need <= 20) go_tok<f32_io, 20>(a, st);
        else if (need <= 24) go_tok<f32_io, 24>(a, st);
        else go_tok<f32_io, 32>(a, st);
    }
    return hipGetLastError();
}

hipError_t launch_zero_f32(float* p, int64_t n, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    int64_t blocks = (n + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(zero_f32_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, st, p, n);
    return hipGetLastError();
}

}  // namespace lnmod
