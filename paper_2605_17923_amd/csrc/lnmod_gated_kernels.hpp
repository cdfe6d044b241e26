// lnmod_gated_kernels.hpp -- gfx950 device code of the gated residual + LayerNorm-Modulate fusion.
//
// The paper lists "Gate + Norm" among its fused operator chains (Sec. 4.4) without a definition.
// This is the chain a DiT block with adaptive LayerNorm has around every LayerNorm-Modulate
// (Sec. 3.3): the branch output u, scaled by the conditioned gate, joins the residual stream, and
// the sum is normalised and modulated at once:
//
//   h = x + gate[m]*u      one fp32 fused multiply-add, rounded once to the I/O type and stored
//   y = LN(h)*(1 + scale[m]) + shift[m]      statistics from h exactly as stored
//
// and backwards, with dy the gradient of y and dh the gradient reaching h along the residual
// stream:  dx = dh + rstd*(g - c1 - hhat*c2),  du = gate*dx,  dgate = sum_n u*dx,
// dshift = sum_n dy, dscale = sum_n dy*hhat  (g = dy*(1+scale), c1 = mean_d g, c2 = mean_d g*hhat).
//
// Same design as the LayerNorm-Modulate kernels (lnmod_kernels.hpp, whose helpers are used
// here): K waves share a row, a lane owns fixed features, so gate, 1+scale, shift and the three
// running gradient sums live in registers; rows stay packed in registers and are unpacked per
// pass; the next step's rows are requested before the current step is computed; clusters of
// blocks walk consecutive rows; per-block partial sums go to slots that a second kernel adds in
// a fixed order.  Fusing saves the second read of h in the forward (4 streams instead of 5) and,
// in the backward, the write and re-read of the LayerNorm's dx (6 streams instead of 8).
#pragma once
#include "lnmod_kernels.hpp"

namespace lnmod {

struct GatedFwdArgs {
    const void* x;
    const void* u;
    const void* gate;
    const void* shift;
    const void* scale;
    void* h;
    void* y;
    float* mean;
    float* rstd;
    Segments seg;
    int64_t T;
    int64_t rows_per_cluster;
    int32_t nb;
    int32_t D;
    int32_t nchunks;
    float eps;
    float inv_D;
};

constexpr int gated_fwd_waves_per_eu(int vpl, int elems, int rows, bool ln) {
    // per lane and chunk: gate (and 1+scale, shift) in fp32, two packed copies of x and u per row
    const int regs = vpl * ((ln ? 3 : 1) * elems + 16 * rows) + 64;
    const int w = 512 / regs;
    return w > LNMOD_MAX_WAVES_PER_EU ? LNMOD_MAX_WAVES_PER_EU : w < 1 ? 1 : w;
}

// LN = false: only h = x + gate*u is produced (the first kernel of the unfused comparator).
template <typename Tag, int VPL, int K, int R, bool EXACT, bool LN = true>
__global__ __launch_bounds__(K* kWave)
LNMOD_OCCUPANCY(gated_fwd_waves_per_eu(VPL, IO<Tag>::E, R, LN))
void gated_fwd_kernel(const GatedFwdArgs a) {
    using io = IO<Tag>;
    constexpr int E = io::E;
    __shared__ float part[2][R][K][2];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t row_bytes = static_cast<int64_t>(a.D) * io::kBytes;

    int chunk[VPL];
    bool ok[VPL];
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
        chunk[i] = (i * K + wave) * kWave + lane;
        ok[i] = EXACT || chunk[i] < a.nchunks;
    }
    float cnt[K];
#pragma unroll
    for (int w = 0; w < K; ++w) {
        int n = 0;
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            int left = a.nchunks - (i * K + w) * kWave;
            left = left < 0 ? 0 : left > kWave ? kWave : left;
            n += left;
        }
        cnt[w] = static_cast<float>(n * E);
    }
    float my_cnt = cnt[0];
#pragma unroll
    for (int w = 1; w < K; ++w) my_cnt = wave == w ? cnt[w] : my_cnt;
    const float inv_my_cnt = my_cnt > 0.0f ? 1.0f / my_cnt : 0.0f;

    const int64_t cluster = blockIdx.x / a.nb;
    const int64_t member = blockIdx.x - cluster * a.nb;
    int64_t r0 = cluster * a.rows_per_cluster;
    int64_t r1 = r0 + a.rows_per_cluster;
    if (r1 > a.T) r1 = a.T;
    int buf = 0;
    uint32_t turn = 0;                       // see take_turn

    while (r0 < r1) {
        int64_t m = find_segment(a.seg, r0);
        int64_t stop = seg_begin(a.seg, m + 1);
        if (stop > r1) stop = r1;
        if (stop <= r0) stop = r0 + 1;          // malformed table: still make progress

        float G[VPL][E], A[VPL][E], B[VPL][E];
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            u32x4 rg = u32x4{0u, 0u, 0u, 0u}, rsc = rg, rsh = rg;
            if (ok[i]) {
                const uint32_t lo = static_cast<uint32_t>(chunk[i]) * 16u;
                rg = load16_cached(a.gate, m * row_bytes, lo);
                if (LN) {
                    rsc = load16_cached(a.scale, m * row_bytes, lo);
                    rsh = load16_cached(a.shift, m * row_bytes, lo);
                }
            }
            io::unpack(rg, G[i]);
            io::unpack(rsc, A[i]);
            io::unpack(rsh, B[i]);
#pragma unroll
            for (int e = 0; e < E; ++e) A[i][e] += 1.0f;
        }

        // q[s][j][i]: s = 0 x, 1 u; rows at or beyond `stop` read as zeros
        auto fetch = [&](int64_t base, u32x4 (&q)[2][R][VPL]) {
#pragma unroll
            for (int j = 0; j < R; ++j) {
                const int64_t row = base + j;
#pragma unroll
                for (int i = 0; i < VPL; ++i) {
                    if (row < stop && ok[i]) {
                        const uint32_t lo = static_cast<uint32_t>(chunk[i]) * 16u;
                        q[0][j][i] = load16_u(a.x, row * row_bytes, lo);
                        q[1][j][i] = load16_u(a.u, row * row_bytes, lo);
                    } else {
                        q[0][j][i] = u32x4{0u, 0u, 0u, 0u};
                        q[1][j][i] = u32x4{0u, 0u, 0u, 0u};
                    }
                }
            }
        };
        const int64_t step = static_cast<int64_t>(a.nb) * R;
        u32x4 raw[2][R][VPL];
        const int64_t first = take_turn<R>(turn, r0, stop, member, a.nb);
        fetch(first, raw);

        for (int64_t base = first; base < stop; base += step) {
            u32x4 nxt[2][R][VPL];
            fetch(base + step, nxt);
            __builtin_amdgcn_sched_barrier(0);               // keep the requests up here

            // h = x + gate*u: one fused multiply-add, one rounding to the I/O type.  The packed
            // result replaces x in the registers, so the LayerNorm below sees what memory holds.
#pragma unroll
            for (int j = 0; j < R; ++j) {
                const int64_t row = base + j;
#pragma unroll
                for (int i = 0; i < VPL; ++i) {
                    float xv[E], uv[E], hv[E];
                    io::unpack(raw[0][j][i], xv);
                    io::unpack(raw[1][j][i], uv);
#pragma unroll
                    for (int e = 0; e < E; ++e) hv[e] = __builtin_fmaf(G[i][e], uv[e], xv[e]);
                    raw[0][j][i] = io::pack(hv);
                    if (row < stop && ok[i])
                        store16_u(a.h, row * row_bytes, static_cast<uint32_t>(chunk[i]) * 16u, raw[0][j][i]);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }

            if (LN) {
                float mu[R], rs[R];
                float pm[R], pq[R];
#pragma unroll
                for (int j = 0; j < R; ++j) {
                    float s = 0.0f;
#pragma unroll
                    for (int i = 0; i < VPL; ++i) {
                        float v[E];
                        io::unpack(raw[0][j][i], v);
#pragma unroll
                        for (int e = 0; e < E; ++e) s += v[e];
                    }
                    pm[j] = wave_sum(s) * inv_my_cnt;
                    float q2 = 0.0f;
#pragma unroll
                    for (int i = 0; i < VPL; ++i) {
                        if (ok[i]) {
                            float v[E];
                            io::unpack(raw[0][j][i], v);
#pragma unroll
                            for (int e = 0; e < E; ++e) q2 += (v[e] - pm[j]) * (v[e] - pm[j]);
                        }
                    }
                    pq[j] = wave_sum(q2);
                }
                if (K > 1) {
                    if (lane == 0) {
#pragma unroll
                        for (int j = 0; j < R; ++j) {
                            part[buf][j][wave][0] = pm[j];
                            part[buf][j][wave][1] = pq[j];
                        }
                    }
                    __syncthreads();
#pragma unroll
                    for (int j = 0; j < R; ++j) {
                        float wsum = 0.0f;
#pragma unroll
                        for (int w = 0; w < K; ++w) wsum += cnt[w] * part[buf][j][w][0];
                        const float mean = wsum / static_cast<float>(a.D);
                        float m2 = 0.0f;
#pragma unroll
                        for (int w = 0; w < K; ++w) {
                            const float d = part[buf][j][w][0] - mean;
                            m2 += part[buf][j][w][1] + cnt[w] * d * d;
                        }
                        mu[j] = mean;
                        rs[j] = 1.0f / sqrtf(m2 * a.inv_D + a.eps);
                    }
                    buf ^= 1;
                } else {
#pragma unroll
                    for (int j = 0; j < R; ++j) {
                        mu[j] = pm[j];
                        rs[j] = 1.0f / sqrtf(pq[j] * a.inv_D + a.eps);
                    }
                }
                // opaque packed registers: the fp32 values are rebuilt below, not carried across
                // the barrier
#pragma unroll
                for (int j = 0; j < R; ++j) {
#pragma unroll
                    for (int i = 0; i < VPL; ++i) asm volatile("" : "+v"(raw[0][j][i]));
                }
#pragma unroll
                for (int j = 0; j < R; ++j) {
                    const int64_t row = base + j;
                    if (row < stop) {
                        if (wave == 0 && lane == 0) {
                            a.mean[row] = mu[j];
                            a.rstd[row] = rs[j];
                        }
#pragma unroll
                        for (int i = 0; i < VPL; ++i) {
                            if (ok[i]) {
                                float v[E], o[E];
                                io::unpack(raw[0][j][i], v);
#pragma unroll
                                for (int e = 0; e < E; ++e) o[e] = ((v[e] - mu[j]) * rs[j]) * A[i][e] + B[i][e];
                                store16_u(a.y, row * row_bytes, static_cast<uint32_t>(chunk[i]) * 16u, io::pack(o));
                            }
                            __builtin_amdgcn_sched_barrier(0);
                        }
                    }
                }
            }
#pragma unroll
            for (int t = 0; t < 2; ++t) {
#pragma unroll
                for (int j = 0; j < R; ++j) {
#pragma unroll
                    for (int i = 0; i < VPL; ++i) raw[t][j][i] = nxt[t][j][i];
                }
            }
        }
        r0 = stop;
    }
}

// =============================================================================================
// Backward
// =============================================================================================
struct GatedBwdArgs {
    const void* dy;
    const void* dh;
    const void* h;
    const void* u;
    const void* gate;
    const void* scale;
    const float* mean;
    const float* rstd;
    void* dx;
    void* du;
    float* ws;               // [nslots][3][D] fp32 partial sums: dshift, dscale, dgate
    Segments seg;
    int64_t T;
    int64_t rows_per_cluster;
    int32_t nb;
    int32_t D;
    int32_t nchunks;
    float inv_D;
};

constexpr int gated_bwd_waves_per_eu(int vpl, int elems, int rows) {
    // per lane and chunk: 1+scale, gate and three running sums in fp32; two packed copies of
    // four streams per row
    const int regs = vpl * (5 * elems + 32 * rows) + 40;
    const int w = 512 / regs;
    return w > LNMOD_MAX_WAVES_PER_EU ? LNMOD_MAX_WAVES_PER_EU : w < 1 ? 1 : w;
}

template <typename Tag, int VPL, int K, int R, bool EXACT>
__global__ __launch_bounds__(K* kWave)
LNMOD_OCCUPANCY(gated_bwd_waves_per_eu(VPL, IO<Tag>::E, R))
void gated_bwd_kernel(const GatedBwdArgs a) {
    using io = IO<Tag>;
    constexpr int E = io::E;
    constexpr int NS = 4;                      // streamed inputs per row: dy, h, dh, u
    __shared__ float part[2][R][K][2];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t row_bytes = static_cast<int64_t>(a.D) * io::kBytes;

    int chunk[VPL];
    bool ok[VPL];
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
        chunk[i] = (i * K + wave) * kWave + lane;
        ok[i] = EXACT || chunk[i] < a.nchunks;
    }

    const int64_t cluster = blockIdx.x / a.nb;
    const int64_t member = blockIdx.x - cluster * a.nb;
    int64_t r0 = cluster * a.rows_per_cluster;
    int64_t r1 = r0 + a.rows_per_cluster;
    if (r1 > a.T) r1 = a.T;
    int buf = 0;
    uint32_t turn = 0;                       // see take_turn

    while (r0 < r1) {
        const int64_t m = find_segment(a.seg, r0);
        int64_t stop = seg_begin(a.seg, m + 1);
        if (stop > r1) stop = r1;
        if (stop <= r0) stop = r0 + 1;          // malformed table: still make progress

        float A[VPL][E], G[VPL][E], acc_s[VPL][E], acc_c[VPL][E], acc_g[VPL][E];
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            u32x4 rsc = u32x4{0u, 0u, 0u, 0u}, rg = rsc;
            if (ok[i]) {
                const uint32_t lo = static_cast<uint32_t>(chunk[i]) * 16u;
                rsc = load16_cached(a.scale, m * row_bytes, lo);
                rg = load16_cached(a.gate, m * row_bytes, lo);
            }
            io::unpack(rsc, A[i]);
            io::unpack(rg, G[i]);
#pragma unroll
            for (int e = 0; e < E; ++e) {
                A[i][e] += 1.0f;
                acc_s[i][e] = 0.0f;
                acc_c[i][e] = 0.0f;
                acc_g[i][e] = 0.0f;
            }
        }

        // q[s][j][i]: s = 0 dy, 1 h, 2 dh, 3 u; rows at or beyond `stop` read as zeros
        auto fetch = [&](int64_t base, u32x4 (&q)[NS][R][VPL], float (&qmu)[R], float (&qrs)[R]) {
#pragma unroll
            for (int j = 0; j < R; ++j) {
                const int64_t row = base + j;
                const bool live = row < stop;
                qmu[j] = live ? a.mean[row] : 0.0f;
                qrs[j] = live ? a.rstd[row] : 0.0f;
#pragma unroll
                for (int i = 0; i < VPL; ++i) {
                    if (live && ok[i]) {
                        const uint32_t lo = static_cast<uint32_t>(chunk[i]) * 16u;
                        q[0][j][i] = load16_u(a.dy, row * row_bytes, lo);
                        q[1][j][i] = load16_u(a.h, row * row_bytes, lo);
                        q[2][j][i] = load16_u(a.dh, row * row_bytes, lo);
                        q[3][j][i] = load16_u(a.u, row * row_bytes, lo);
                    } else {
#pragma unroll
                        for (int t = 0; t < NS; ++t) q[t][j][i] = u32x4{0u, 0u, 0u, 0u};
                    }
                }
            }
        };
        const int64_t step = static_cast<int64_t>(a.nb) * R;
        u32x4 raw[NS][R][VPL];
        float mu[R], rs[R];
        const int64_t first = take_turn<R>(turn, r0, stop, member, a.nb);
        fetch(first, raw, mu, rs);

        for (int64_t base = first; base < stop; base += step) {
            u32x4 nxt[NS][R][VPL];
            float nmu[R], nrs[R];
            fetch(base + step, nxt, nmu, nrs);
            __builtin_amdgcn_sched_barrier(0);               // keep the requests up here

            // pass 1: the two row sums of the LayerNorm backward and the running dshift/dscale
            float c1[R], c2[R];
#pragma unroll
            for (int j = 0; j < R; ++j) {
                float p1 = 0.0f, p2 = 0.0f;
#pragma unroll
                for (int i = 0; i < VPL; ++i) {
                    float dyv[E], hv[E];
                    io::unpack(raw[0][j][i], dyv);
                    io::unpack(raw[1][j][i], hv);
#pragma unroll
                    for (int e = 0; e < E; ++e) {
                        const float hh = (hv[e] - mu[j]) * rs[j];
                        const float gg = dyv[e] * A[i][e];
                        p1 += gg;
                        p2 += gg * hh;
                        acc_s[i][e] += dyv[e];
                        acc_c[i][e] += dyv[e] * hh;
                    }
                    // pin the running sums here, or the optimiser sinks the adds below the barrier
                    // and keeps every unpacked value alive until then
#pragma unroll
                    for (int e = 0; e < E; ++e) asm volatile("" : "+v"(acc_s[i][e]), "+v"(acc_c[i][e]));
                    __builtin_amdgcn_sched_barrier(0);
                }
                c1[j] = wave_sum(p1);
                c2[j] = wave_sum(p2);
            }
            if (K > 1) {
                if (lane == 0) {
#pragma unroll
                    for (int j = 0; j < R; ++j) {
                        part[buf][j][wave][0] = c1[j];
                        part[buf][j][wave][1] = c2[j];
                    }
                }
                __syncthreads();
#pragma unroll
                for (int j = 0; j < R; ++j) {
                    float t1 = 0.0f, t2 = 0.0f;
#pragma unroll
                    for (int w = 0; w < K; ++w) {
                        t1 += part[buf][j][w][0];
                        t2 += part[buf][j][w][1];
                    }
                    c1[j] = t1;
                    c2[j] = t2;
                }
                buf ^= 1;
            }
            // pass 2: dx = dh + rstd*(g - c1 - hhat*c2), du = gate*dx, dgate += u*dx (fp32 dx).
            // The empty asm makes the packed registers opaque so that pass 1's fp32 values are
            // rebuilt here instead of being carried across the barrier.
#pragma unroll
            for (int t = 0; t < NS; ++t) {
#pragma unroll
                for (int j = 0; j < R; ++j) {
#pragma unroll
                    for (int i = 0; i < VPL; ++i) asm volatile("" : "+v"(raw[t][j][i]));
                }
            }
#pragma unroll
            for (int j = 0; j < R; ++j) {
                const int64_t row = base + j;
                if (row < stop) {
                    const float k1 = rs[j] * (c1[j] * a.inv_D), k2 = rs[j] * (c2[j] * a.inv_D);
#pragma unroll
                    for (int i = 0; i < VPL; ++i) {
                        if (ok[i]) {
                            float dyv[E], hv[E], dhv[E], uv[E], o[E], ou[E];
                            io::unpack(raw[0][j][i], dyv);
                            io::unpack(raw[1][j][i], hv);
                            io::unpack(raw[2][j][i], dhv);
                            io::unpack(raw[3][j][i], uv);
#pragma unroll
                            for (int e = 0; e < E; ++e) {
                                const float hh = (hv[e] - mu[j]) * rs[j];
                                o[e] = dhv[e] + ((dyv[e] * A[i][e]) * rs[j] - k1 - hh * k2);
                                ou[e] = G[i][e] * o[e];
                                acc_g[i][e] += uv[e] * o[e];
                            }
#pragma unroll
                            for (int e = 0; e < E; ++e) asm volatile("" : "+v"(acc_g[i][e]));
                            const uint32_t lo = static_cast<uint32_t>(chunk[i]) * 16u;
                            store16_u(a.dx, row * row_bytes, lo, io::pack(o));
                            store16_u(a.du, row * row_bytes, lo, io::pack(ou));
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
#pragma unroll
            for (int j = 0; j < R; ++j) {
                mu[j] = nmu[j];
                rs[j] = nrs[j];
#pragma unroll
                for (int t = 0; t < NS; ++t) {
#pragma unroll
                    for (int i = 0; i < VPL; ++i) raw[t][j][i] = nxt[t][j][i];
                }
            }
        }

        // this block's partial sums for segment m (zeros if it had no row of it)
        float* slot = a.ws + ((cluster + m) * a.nb + member) * 3 * a.D;
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            if (ok[i]) {
                f32x4* ps = reinterpret_cast<f32x4*>(slot + static_cast<int64_t>(chunk[i]) * E);
                f32x4* pc = reinterpret_cast<f32x4*>(slot + a.D + static_cast<int64_t>(chunk[i]) * E);
                f32x4* pg = reinterpret_cast<f32x4*>(slot + 2 * a.D + static_cast<int64_t>(chunk[i]) * E);
#pragma unroll
                for (int q = 0; q < E / 4; ++q) {
                    ps[q] = f32x4{acc_s[i][4 * q], acc_s[i][4 * q + 1], acc_s[i][4 * q + 2], acc_s[i][4 * q + 3]};
                    pc[q] = f32x4{acc_c[i][4 * q], acc_c[i][4 * q + 1], acc_c[i][4 * q + 2], acc_c[i][4 * q + 3]};
                    pg[q] = f32x4{acc_g[i][4 * q], acc_g[i][4 * q + 1], acc_g[i][4 * q + 2], acc_g[i][4 * q + 3]};
                }
            }
        }
        r0 = stop;
    }
}

// The second pass is bwd_reduce_kernel with three sums per slot.

}  // namespace lnmod
