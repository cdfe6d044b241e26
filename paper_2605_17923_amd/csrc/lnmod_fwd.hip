// lnmod_fwd.hip -- instantiation and launch of the forward kernels (per-sample / per-segment
// modulation kept in registers by K waves per row, and per-token modulation streamed with x).
#include "lnmod_kernels.hpp"
#include "lnmod_launch.hpp"

#include <cstdio>

namespace lnmod {
namespace {

constexpr int E_bytes(int dtype) { return dtype == 0 ? 2 : 4; }

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
    a.interleave = 0;
    a.D = static_cast<int32_t>(p.D);
    a.nchunks = static_cast<int32_t>(p.D / E);
    a.eps = p.eps;
    a.inv_D = 1.0f / static_cast<float>(p.D);
    return a;
}

template <typename Tag, int VPL, int K, int R, int MODE>
void go_r(const FwdArgs& a, int64_t blocks, hipStream_t st) {
    const dim3 grid(static_cast<unsigned>(blocks)), block(K * kWave);
    if (a.nchunks == K * VPL * kWave)
        hipLaunchKernelGGL((fwd_split_kernel<Tag, VPL, K, R, true, MODE>), grid, block, 0, st, a);
    else
        hipLaunchKernelGGL((fwd_split_kernel<Tag, VPL, K, R, false, MODE>), grid, block, 0, st, a);
}

template <typename Tag, int VPL, int K, int MODE>
void go(const FwdArgs& a, int R, int64_t blocks, hipStream_t st) {
    if (R == 1) go_r<Tag, VPL, K, 1, MODE>(a, blocks, st);
    else go_r<Tag, VPL, K, 2, MODE>(a, blocks, st);
}

// Every (VPL, K) the shape table, the fp32 rule and the per-token rule can ask for.
template <typename Tag, int MODE>
bool dispatch(const FwdArgs& a, int VPL, int K, int R, int64_t blocks, hipStream_t st) {
    switch (VPL * 100 + K) {
        case 101: go<Tag, 1, 1, MODE>(a, R, blocks, st); return true;
        case 201: go<Tag, 2, 1, MODE>(a, R, blocks, st); return true;
        case 301: go<Tag, 3, 1, MODE>(a, R, blocks, st); return true;
        default: break;
    }
    if constexpr (IO<Tag>::E == 8) {                     // bf16
        switch (VPL * 100 + K) {
            case 202: go<Tag, 2, 2, MODE>(a, R, blocks, st); return true;
            case 204: go<Tag, 2, 4, MODE>(a, R, blocks, st); return true;
            case 205: go<Tag, 2, 5, MODE>(a, R, blocks, st); return true;
            default: break;
        }
        if constexpr (MODE == kModToken) {               // rule-based split of the per-token kernels
            switch (VPL * 100 + K) {
                case 203: go<Tag, 2, 3, MODE>(a, R, blocks, st); return true;
                case 206: go<Tag, 2, 6, MODE>(a, R, blocks, st); return true;
                case 208: go<Tag, 2, 8, MODE>(a, R, blocks, st); return true;
                case 502:                                    // compiled for one row per step only
                    if (R != 1) return false;
                    go_r<Tag, 5, 2, 1, MODE>(a, blocks, st);
                    return true;
                default: break;
            }
        } else {                                         // shape table
            switch (VPL * 100 + K) {
                case 302: go<Tag, 3, 2, MODE>(a, R, blocks, st); return true;
                case 304: go<Tag, 3, 4, MODE>(a, R, blocks, st); return true;
                case 306: go<Tag, 3, 6, MODE>(a, R, blocks, st); return true;
                default: break;
            }
        }
    } else {                                             // fp32 rule: up to 6 chunks alone, else 4 per lane
        switch (VPL * 100 + K) {
            case 401: go<Tag, 4, 1, MODE>(a, R, blocks, st); return true;
            case 601: go<Tag, 6, 1, MODE>(a, R, blocks, st); return true;
            case 402: go<Tag, 4, 2, MODE>(a, R, blocks, st); return true;
            case 403: go<Tag, 4, 3, MODE>(a, R, blocks, st); return true;
            case 404: go<Tag, 4, 4, MODE>(a, R, blocks, st); return true;
            case 405: go<Tag, 4, 5, MODE>(a, R, blocks, st); return true;
            case 406: go<Tag, 4, 6, MODE>(a, R, blocks, st); return true;
            case 408: go<Tag, 4, 8, MODE>(a, R, blocks, st); return true;
            default: break;
        }
    }
    return false;                                        // no such instantiation
}

// Whether a forward with one modulation row per sample / segment runs one loop over all rows of a
// block's region (kModFlat) or one loop per segment (kModSegment).  With several segments the flat
// loop wins wherever few blocks share a CU, because a block that drains its pipeline at a segment's
// end leaves the CU idle: bf16 rows shared by three or more waves (D >= 2560) and D = 1536 gained 1
// to 11 % on 8 to 480 segments (D = 5120, 24 mixed segments: 514 against 530 us; 3 x 75 600 rows: 766
// against 819; D = 1536, 24 mixed: 159 against 178, 480 x 312: 170 against 244); D = 1024 and 2048
// lost 2 to 9 % on 96 segments and fp32 was mixed, so those keep the loop per segment.
bool fwd_flat(const Problem& p, const Shape& table) {
    if (p.force && p.force->flat != 0) return p.force->flat == 1;
    if (p.nseg <= 1 || p.dtype != 0) return false;
    return table.K >= 3 || p.D == 1536;
}

// Clusters of a flat launch: every block reloads its modulation registers once per segment of its
// cluster's region (about 0.3 us each, the next rows being already in flight), and every further
// window costs bandwidth, so the count is the smallest power of two that leaves a block at most 32
// segments, between 2 and 32 (D = 5120: 2, 4, 8 clusters best on 24, 96, 480 segments; D = 1536:
// 2, 4, 16).
int64_t flat_clusters(int64_t nseg) {
    int64_t c = 2;
    while (c < 32 && nseg > 32 * c) c *= 2;
    return c;
}

// Shape and row plan of a forward launch: what the launcher uses and what describe_fwd() reports.
struct FwdLaunch {
    Shape sh;
    RowPlan pl;
    int nchunks;
};

FwdLaunch plan_fwd(const Problem& p, int mode) {
    FwdLaunch L;
    const int E = p.dtype == 0 ? 8 : 4;
    L.nchunks = static_cast<int>(p.D / E);
    Shape sh = fwd_shape(L.nchunks, p.dtype);                      // the comparators' starting point
    if (mode == kModToken) sh = pick_shape(p.force, tok_fwd_shape(L.nchunks, p.dtype));
    if (mode == kModSegment || mode == kModFlat) {
        Shape tab = fwd_shape(L.nchunks, p.dtype, p.T);
        // D = 1536, flat: four blocks per CU at every token count (24 mixed segments, 152 880 rows:
        // 159 us against 182 with three)
        if (mode == kModFlat && L.nchunks == 192 && p.dtype == 0) tab.per_cu = 4;
        sh = pick_shape(p.force, tab);
    }
    if ((mode == kLnOnly || mode == kModOnly) && p.dtype == 0) {
        // the two kernels of the unfused comparator get the shape that makes their chain fastest at
        // the two model widths (D = 5120: 540 against 609 us, D = 1536: 528 against 559 us on 774 MB)
        const int cols = (L.nchunks + kWave - 1) / kWave;
        if (cols == 3) sh = {1, 3, 1, 8};
        if (cols >= 9 && cols <= 10) sh = {5, 2, 1, 3};
    }
    const bool per_segment = mode == kModSegment || mode == kModOnly;
    // bytes of x and y at 6 TB/s
    const double stream_us = static_cast<double>(p.T) * static_cast<double>(p.D) * (2.0 * E_bytes(p.dtype)) / 6.0e6;
    L.sh = sh;
    if (mode == kModFlat)
        L.pl = plan_rows_clusters(p.T, p.nseg, static_cast<int64_t>(kNumCU) * sh.per_cu, sh.R,
                                  flat_clusters(p.nseg), sh.clusters);
    else
        L.pl = plan_rows_clusters(p.T, per_segment ? p.nseg : 1, static_cast<int64_t>(kNumCU) * sh.per_cu,
                                  sh.R, per_segment ? pick_clusters(stream_us, p.nseg) : 1,
                                  per_segment ? sh.clusters : 0);
    return L;
}

template <int MODE>
hipError_t launch_mode(const Problem& p, const void* x, const void* shift, const void* scale, void* y,
                       float* mean, float* rstd, hipStream_t st) {
    const int E = p.dtype == 0 ? 8 : 4;
    FwdArgs a = make_args(p, x, shift, scale, y, mean, rstd, E);
    const FwdLaunch L = plan_fwd(p, MODE);
    const Shape sh = L.sh;
    const RowPlan pl = L.pl;
    a.rows_per_cluster = pl.rows_per_cluster;
    a.nb = pl.nb;
    a.interleave = cluster_interleave(p.force, pl);
    if (!covers(sh, a.nchunks)) return hipErrorInvalidConfiguration;
    const bool ok = p.dtype == 0 ? dispatch<bf16_io, MODE>(a, sh.VPL, sh.K, sh.R, pl.blocks, st)
                                 : dispatch<f32_io, MODE>(a, sh.VPL, sh.K, sh.R, pl.blocks, st);
    return ok ? hipGetLastError() : hipErrorInvalidConfiguration;
}

}  // namespace

hipError_t launch_fwd_seg(const Problem& p, const void* x, const void* shift, const void* scale,
                          void* y, float* mean, float* rstd, hipStream_t st) {
    if (fwd_flat(p, fwd_shape(static_cast<int>(p.D / (p.dtype == 0 ? 8 : 4)), p.dtype, p.T)))
        return launch_mode<kModFlat>(p, x, shift, scale, y, mean, rstd, st);
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

// Text that names the kernel instantiation and grid a forward call with these arguments launches
// (template arguments in the order of fwd_split_kernel's parameter list).
int describe_fwd(const Problem& p, bool per_token, char* buf, size_t n) {
    const Shape tab = fwd_shape(static_cast<int>(p.D / (p.dtype == 0 ? 8 : 4)), p.dtype, p.T);
    const int mode = per_token ? kModToken : fwd_flat(p, tab) ? kModFlat : kModSegment;
    const FwdLaunch L = plan_fwd(p, mode);
    const bool exact = L.nchunks == L.sh.K * L.sh.VPL * kWave;
    return std::snprintf(buf, n, "fwd_split_kernel<%s, %d, %d, %d, %s, %d, true> grid=%lld block=%d clusters=%lld",
                         p.dtype == 0 ? "bf16_io" : "f32_io", L.sh.VPL, L.sh.K, L.sh.R, exact ? "true" : "false",
                         mode, static_cast<long long>(L.pl.blocks), L.sh.K * kWave,
                         static_cast<long long>(L.pl.clusters));
}

}  // namespace lnmod
