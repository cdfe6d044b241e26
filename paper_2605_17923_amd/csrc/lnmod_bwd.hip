// lnmod_bwd.hip -- instantiation and launch of the backward kernels: the fused
// dx + dshift/dscale-partials kernel with its fixed-order second pass, and the per-token kernel.
#include "lnmod_kernels.hpp"
#include "lnmod_launch.hpp"

namespace lnmod {
namespace {

constexpr int kTokWaves = 4;

// How a row of `nchunks` 16-byte chunks is split: K waves per row, VPL chunks per lane.
struct Split {
    int K;
    int VPL;
};

// bf16: 2 chunks (16 features) per lane; fp32: 4 chunks (16 features) per lane; as many waves
// as the row needs.  Small rows use fewer chunks per lane instead of idle lanes.
Split choose_split(int nchunks, int dtype) {
    const int vpl_full = dtype == 0 ? 2 : 4;
    int vpl = vpl_full;
    while (vpl > 1 && nchunks <= (vpl / 2) * kWave) vpl /= 2;
    int k = (nchunks + vpl * kWave - 1) / (vpl * kWave);
    if (k == 7) k = 8;
    return {k, vpl};
}

// Blocks per CU so that about 16 waves share a CU.
int blocks_per_cu(int K) {
    int b = 16 / K;
    return b < 1 ? 1 : b;
}

template <typename Tag, int VPL, int K>
void go_seg(BwdArgs a, int64_t blocks, hipStream_t st) {
    constexpr int R = 2;
    const dim3 grid(static_cast<unsigned>(blocks)), block(K * kWave);
    if (a.nchunks == K * VPL * kWave)
        hipLaunchKernelGGL((bwd_seg_kernel<Tag, VPL, K, R, true>), grid, block, 0, st, a);
    else
        hipLaunchKernelGGL((bwd_seg_kernel<Tag, VPL, K, R, false>), grid, block, 0, st, a);
}

template <typename Tag, int VPL>
void go_seg_k(const BwdArgs& a, int K, int64_t blocks, hipStream_t st) {
    switch (K) {
        case 1: go_seg<Tag, VPL, 1>(a, blocks, st); break;
        case 2: go_seg<Tag, VPL, 2>(a, blocks, st); break;
        case 3: go_seg<Tag, VPL, 3>(a, blocks, st); break;
        case 4: go_seg<Tag, VPL, 4>(a, blocks, st); break;
        case 5: go_seg<Tag, VPL, 5>(a, blocks, st); break;
        case 6: go_seg<Tag, VPL, 6>(a, blocks, st); break;
        default: go_seg<Tag, VPL, 8>(a, blocks, st); break;
    }
}

template <typename Tag, int VPL>
void go_tok(BwdArgs a, hipStream_t st) {
    int64_t blocks = (a.T + kTokWaves - 1) / kTokWaves;
    const int64_t cap = static_cast<int64_t>(kNumCU) * 8;
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    a.rows_per_block = (a.T + blocks - 1) / blocks;
    blocks = (a.T + a.rows_per_block - 1) / a.rows_per_block;
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
    a.rows_per_block = 0;
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

int64_t bwd_num_blocks(int64_t T, int64_t D, int dtype) {
    if (T <= 0) return 0;
    const int E = dtype == 0 ? 8 : 4;
    const Split sp = choose_split(static_cast<int>(D / E), dtype);
    int64_t blocks = static_cast<int64_t>(kNumCU) * blocks_per_cu(sp.K);
    if (blocks > kMaxBwdBlocks) blocks = kMaxBwdBlocks;
    if (blocks > T) blocks = T;
    const int64_t rpb = (T + blocks - 1) / blocks;
    return (T + rpb - 1) / rpb;
}

int64_t bwd_rows_per_block(int64_t T, int64_t D, int dtype) {
    const int64_t blocks = bwd_num_blocks(T, D, dtype);
    return blocks > 0 ? (T + blocks - 1) / blocks : 1;
}

hipError_t launch_bwd_seg(const Problem& p, const void* dy, const void* x, const void* scale,
                          const float* mean, const float* rstd, void* dx, float* dshift,
                          float* dscale, float* ws, hipStream_t st) {
    const int E = p.dtype == 0 ? 8 : 4;
    BwdArgs a = make_args(p, dy, x, scale, mean, rstd, dx, nullptr, nullptr, ws, E);
    const Split sp = choose_split(a.nchunks, p.dtype);
    const int64_t blocks = bwd_num_blocks(p.T, p.D, p.dtype);
    a.rows_per_block = bwd_rows_per_block(p.T, p.D, p.dtype);
    if (p.dtype == 0) {
        if (sp.VPL == 1) go_seg_k<bf16_io, 1>(a, sp.K, blocks, st);
        else go_seg_k<bf16_io, 2>(a, sp.K, blocks, st);
    } else {
        if (sp.VPL == 1) go_seg_k<f32_io, 1>(a, sp.K, blocks, st);
        else if (sp.VPL == 2) go_seg_k<f32_io, 2>(a, sp.K, blocks, st);
        else go_seg_k<f32_io, 4>(a, sp.K, blocks, st);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;

    ReduceArgs r;
    r.ws = ws;
    r.dshift = dshift;
    r.dscale = dscale;
    r.seg = a.seg;
    r.T = p.T;
    r.rows_per_block = a.rows_per_block;
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
