// lnmod_bwd.hip -- instantiation and launch of the backward: the fused dx + dshift/dscale
// partial-sum kernel with its fixed-order second pass, and its per-token form.
#include "lnmod_kernels.hpp"
#include "lnmod_launch.hpp"

#include <cstdio>

namespace lnmod {
namespace {

template <typename Tag, int VPL, int K, int R, bool TOK, bool RC>
void go_seg_rc(const BwdArgs& a, int64_t blocks, hipStream_t st) {
    const dim3 grid(static_cast<unsigned>(blocks)), block(K * kWave);
    if (a.nchunks == K * VPL * kWave)
        hipLaunchKernelGGL((bwd_seg_kernel<Tag, VPL, K, R, true, TOK, true, RC>), grid, block, 0, st, a);
    else
        hipLaunchKernelGGL((bwd_seg_kernel<Tag, VPL, K, R, false, TOK, true, RC>), grid, block, 0, st, a);
}

// The statistics are recomputed when the caller passed none.
template <typename Tag, int VPL, int K, bool TOK>
void go_seg(const BwdArgs& a, int R, int64_t blocks, hipStream_t st) {
    const bool rc = a.mean == nullptr;
    if (R == 1) {
        if (rc) go_seg_rc<Tag, VPL, K, 1, TOK, true>(a, blocks, st);
        else go_seg_rc<Tag, VPL, K, 1, TOK, false>(a, blocks, st);
    } else {
        if (rc) go_seg_rc<Tag, VPL, K, 2, TOK, true>(a, blocks, st);
        else go_seg_rc<Tag, VPL, K, 2, TOK, false>(a, blocks, st);
    }
}

// Every (VPL, K) the shape table, the fp32 rule and the per-token rule can ask for.
template <typename Tag, bool TOK>
bool dispatch_seg(const BwdArgs& a, int VPL, int K, int R, int64_t blocks, hipStream_t st) {
    switch (VPL * 100 + K) {
        case 101: go_seg<Tag, 1, 1, TOK>(a, R, blocks, st); return true;
        case 201: go_seg<Tag, 2, 1, TOK>(a, R, blocks, st); return true;
        case 301: go_seg<Tag, 3, 1, TOK>(a, R, blocks, st); return true;
        default: break;
    }
    if constexpr (IO<Tag>::E == 8) {                     // bf16 rule: two chunks per lane when shared
        switch (VPL * 100 + K) {
            case 202: go_seg<Tag, 2, 2, TOK>(a, R, blocks, st); return true;
            case 203: go_seg<Tag, 2, 3, TOK>(a, R, blocks, st); return true;
            case 204: go_seg<Tag, 2, 4, TOK>(a, R, blocks, st); return true;
            case 205: go_seg<Tag, 2, 5, TOK>(a, R, blocks, st); return true;
            case 206: go_seg<Tag, 2, 6, TOK>(a, R, blocks, st); return true;
            case 208: go_seg<Tag, 2, 8, TOK>(a, R, blocks, st); return true;
            default: break;
        }
    }
    if constexpr (IO<Tag>::E == 8 && !TOK) {             // bf16 shape table only
        switch (VPL * 100 + K) {
            case 103: go_seg<Tag, 1, 3, TOK>(a, R, blocks, st); return true;
            case 104: go_seg<Tag, 1, 4, TOK>(a, R, blocks, st); return true;
            case 105: go_seg<Tag, 1, 5, TOK>(a, R, blocks, st); return true;
            case 106: go_seg<Tag, 1, 6, TOK>(a, R, blocks, st); return true;
            case 304: go_seg<Tag, 3, 4, TOK>(a, R, blocks, st); return true;
            case 306: go_seg<Tag, 3, 6, TOK>(a, R, blocks, st); return true;
            default: break;
        }
    }
    if constexpr (IO<Tag>::E == 4) {                     // fp32 rule: up to 6 chunks alone, else 4 per lane
        switch (VPL * 100 + K) {
            case 401: go_seg<Tag, 4, 1, TOK>(a, R, blocks, st); return true;
            case 601: go_seg<Tag, 6, 1, TOK>(a, R, blocks, st); return true;
            case 402: go_seg<Tag, 4, 2, TOK>(a, R, blocks, st); return true;
            case 403: go_seg<Tag, 4, 3, TOK>(a, R, blocks, st); return true;
            case 404: go_seg<Tag, 4, 4, TOK>(a, R, blocks, st); return true;
            case 405: go_seg<Tag, 4, 5, TOK>(a, R, blocks, st); return true;
            case 406: go_seg<Tag, 4, 6, TOK>(a, R, blocks, st); return true;
            case 408: go_seg<Tag, 4, 8, TOK>(a, R, blocks, st); return true;
            default: break;
        }
    }
    return false;                                        // no such instantiation
}

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
    a.interleave = 0;
    a.D = static_cast<int32_t>(p.D);
    a.nchunks = static_cast<int32_t>(p.D / E);
    a.inv_D = 1.0f / static_cast<float>(p.D);
    a.eps = p.eps;
    return a;
}

__global__ __launch_bounds__(256) void zero_f32_kernel(float* p, int64_t n) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += stride)
        p[i] = 0.0f;
}

}  // namespace

// Grid of the second pass: one block per (segment, sum, feature block) triple, at most
// kReduceMaxGrid blocks; beyond that the blocks walk the triples with a stride of the grid.
constexpr int64_t kReduceMaxGrid = int64_t(1) << 20;

hipError_t launch_reduce(ReduceArgs r, int64_t clusters, hipStream_t st) {
    const ReduceShape sh = reduce_shape(r.seg.nseg, r.nsum, r.D, clusters, r.nb);
    const int V = sh.V, W = sh.W, G = sh.G;
    const int per_block = kWave / G * V;
    r.dblocks = static_cast<int32_t>((r.D + per_block - 1) / per_block);
    r.total = r.seg.nseg * r.nsum * r.dblocks;
    const int64_t g = r.total < kReduceMaxGrid ? r.total : kReduceMaxGrid;
    const dim3 grid(static_cast<unsigned>(g)), block(W * kWave);
    if (G == 4) hipLaunchKernelGGL((bwd_reduce_kernel<4, 4>), grid, block, 0, st, r);
    else if (G == 2) hipLaunchKernelGGL((bwd_reduce_kernel<4, 2>), grid, block, 0, st, r);
    else if (V == 4) hipLaunchKernelGGL((bwd_reduce_kernel<4, 1>), grid, block, 0, st, r);
    else if (V == 2) hipLaunchKernelGGL((bwd_reduce_kernel<2, 1>), grid, block, 0, st, r);
    else hipLaunchKernelGGL((bwd_reduce_kernel<1, 1>), grid, block, 0, st, r);
    return hipGetLastError();
}

namespace {

// Shape and row plan of a backward launch: what the launcher uses, what sizes the workspace and
// what describe_bwd() reports.
struct BwdLaunch {
    Shape sh;
    RowPlan pl;
    int nchunks;
};

BwdLaunch plan_bwd(int64_t T, int64_t nseg, int64_t D, int dtype, bool per_token, bool recompute,
                   const Shape* force) {
    BwdLaunch L;
    const int E = dtype == 0 ? 8 : 4;
    L.nchunks = static_cast<int>(D / E);
    if (per_token) {
        L.sh = pick_shape(force, tok_bwd_shape(L.nchunks, dtype));
        L.pl = plan_rows(T, static_cast<int64_t>(kNumCU) * L.sh.per_cu, L.sh.R);
        return L;
    }
    L.sh = pick_shape(force, recompute ? rc_bwd_shape(L.nchunks, dtype) : bwd_shape(L.nchunks, dtype));
    // a row moves 3 D elements (dy, x, dx), a slot 2 D floats that are written and read back
    const double elem = dtype == 0 ? 2.0 : 4.0;
    const double stream_us = static_cast<double>(T) * static_cast<double>(D) * 3.0 * elem / 5.8e6;
    L.pl = plan_rows_slots(T, nseg, static_cast<int64_t>(kNumCU) * L.sh.per_cu, L.sh.R, stream_us,
                           16.0 / (3.0 * elem), L.sh.clusters);
    return L;
}

}  // namespace

RowPlan bwd_plan(int64_t T, int64_t nseg, int64_t D, int dtype, bool recompute, const Shape* force) {
    return plan_bwd(T, nseg, D, dtype, false, recompute, force).pl;
}

hipError_t launch_bwd_seg(const Problem& p, const void* dy, const void* x, const void* scale,
                          const float* mean, const float* rstd, void* dx, float* dshift,
                          float* dscale, float* ws, hipStream_t st) {
    const int E = p.dtype == 0 ? 8 : 4;
    BwdArgs a = make_args(p, dy, x, scale, mean, rstd, dx, nullptr, nullptr, ws, E);
    const bool rc = mean == nullptr;
    const BwdLaunch L = plan_bwd(p.T, p.nseg, p.D, p.dtype, false, rc, p.force);
    const Shape sh = L.sh;
    const RowPlan pl = L.pl;
    if (!covers(sh, a.nchunks)) return hipErrorInvalidConfiguration;
    a.rows_per_cluster = pl.rows_per_cluster;
    a.nb = pl.nb;
    a.interleave = cluster_interleave(p.force, pl);
    const bool ok = p.dtype == 0 ? dispatch_seg<bf16_io, false>(a, sh.VPL, sh.K, sh.R, pl.blocks, st)
                                 : dispatch_seg<f32_io, false>(a, sh.VPL, sh.K, sh.R, pl.blocks, st);
    if (!ok) return hipErrorInvalidConfiguration;
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;

    ReduceArgs r;
    r.ws = ws;
    r.out[0] = dshift;
    r.out[1] = dscale;
    r.out[2] = nullptr;
    r.seg = a.seg;
    r.T = p.T;
    r.rows_per_cluster = a.rows_per_cluster;
    r.nb = a.nb;
    r.D = a.D;
    r.nsum = 2;
    return launch_reduce(r, pl.clusters, st);
}

hipError_t launch_bwd_tok(const Problem& p, const void* dy, const void* x, const void* scale,
                          const float* mean, const float* rstd, void* dx, void* dshift,
                          void* dscale, hipStream_t st) {
    const int E = p.dtype == 0 ? 8 : 4;
    BwdArgs a = make_args(p, dy, x, scale, mean, rstd, dx, dshift, dscale, nullptr, E);
    const BwdLaunch L = plan_bwd(p.T, p.nseg, p.D, p.dtype, true, mean == nullptr, p.force);
    const Shape sh = L.sh;
    const RowPlan pl = L.pl;
    if (!covers(sh, a.nchunks)) return hipErrorInvalidConfiguration;
    a.rows_per_cluster = pl.rows_per_cluster;
    a.nb = pl.nb;
    const bool ok = p.dtype == 0 ? dispatch_seg<bf16_io, true>(a, sh.VPL, sh.K, sh.R, pl.blocks, st)
                                 : dispatch_seg<f32_io, true>(a, sh.VPL, sh.K, sh.R, pl.blocks, st);
    return ok ? hipGetLastError() : hipErrorInvalidConfiguration;
}

// Text that names the kernel instantiations and grids a backward call with these arguments launches
// (template arguments in the order of bwd_seg_kernel's parameter list).
int describe_bwd(const Problem& p, bool per_token, bool recompute, char* buf, size_t n) {
    const BwdLaunch L = plan_bwd(p.T, p.nseg, p.D, p.dtype, per_token, recompute, p.force);
    const bool exact = L.nchunks == L.sh.K * L.sh.VPL * kWave;
    int k = std::snprintf(buf, n, "bwd_seg_kernel<%s, %d, %d, %d, %s, %s, true, %s> grid=%lld block=%d clusters=%lld",
                          p.dtype == 0 ? "bf16_io" : "f32_io", L.sh.VPL, L.sh.K, L.sh.R, exact ? "true" : "false",
                          per_token ? "true" : "false", recompute ? "true" : "false",
                          static_cast<long long>(L.pl.blocks), L.sh.K * kWave,
                          static_cast<long long>(L.pl.clusters));
    if (!per_token && k > 0 && static_cast<size_t>(k) < n) {
        const ReduceShape rs = reduce_shape(p.nseg, 2, p.D, L.pl.clusters, L.pl.nb);
        const int64_t per_block = kWave / rs.G * rs.V;
        const int64_t dblocks = (p.D + per_block - 1) / per_block;
        k += std::snprintf(buf + k, n - k, " + bwd_reduce_kernel<%d, %d> grid=%lld block=%d slots=%lld", rs.V, rs.G,
                           static_cast<long long>(p.nseg * 2 * dblocks), rs.W * kWave,
                           static_cast<long long>(bwd_slots(L.pl, p.nseg)));
    }
    return k;
}

hipError_t launch_zero_f32(float* p, int64_t n, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    int64_t blocks = (n + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(zero_f32_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, st, p, n);
    return hipGetLastError();
}

}  // namespace lnmod
