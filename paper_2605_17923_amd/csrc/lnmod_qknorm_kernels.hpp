// lnmod_qknorm_kernels.hpp -- gfx950 device code of the fused Q-Norm + K-Norm operator.
//
// The paper lists "Q-Norm + K-Norm" among its fused operator chains (Sec. 4.4) without a
// definition.  This is the query/key normalisation of MMDiT-style attention blocks: for each of
// the two tensors, x [N, D] with a learned weight w [D],
//
//   rstd_n = 1/sqrt((1/D) sum_d x[n,d]^2 + eps)      y[n,d] = (x[n,d]*rstd_n) * w[d]
//   g = dy*w   c_n = (1/D) sum_d g*xhat   dx = rstd_n*(g - xhat*c_n)   dw[d] = sum_n dy[n,d]*xhat[n,d]
//
// Both tensors are handled by one launch ("two norms, one launch"): the first half of the grid
// takes the query rows, the second half the key rows.  Inside a half the design is that of the
// LayerNorm-Modulate kernels (lnmod_kernels.hpp, whose helpers are used here): K waves share a
// row, a lane owns fixed features, so the weight and the running dw sums live in registers; rows
// stay packed in registers and are unpacked per pass; the next step's rows are requested before
// the current step is computed; the blocks of a half take consecutive rows; per-block partial dw
// sums go to slots that a second kernel adds in a fixed order (no float atomics).
#pragma once
#include "lnmod_kernels.hpp"

namespace lnmod {

struct QkFwdArgs {
    const void* x[2];        // q, k
    const void* w[2];
    void* y[2];
    float* rstd[2];
    int64_t N;               // rows of each tensor
    int32_t nb;              // blocks per tensor (grid = 2 * nb)
    int32_t D;
    int32_t nchunks;
    float eps;
    float inv_D;
};

constexpr int qk_waves_per_eu(int vpl, int elems, int feat_regs, int packed_rows) {
    const int regs = vpl * (feat_regs * elems + 5 * packed_rows) + 28;
    const int w = 512 / regs;
    return w > LNMOD_MAX_WAVES_PER_EU ? LNMOD_MAX_WAVES_PER_EU : w < 1 ? 1 : w;
}

template <typename Tag, int VPL, int K, int R, bool EXACT>
__global__ __launch_bounds__(K* kWave)
LNMOD_OCCUPANCY(qk_waves_per_eu(VPL, IO<Tag>::E, 1, 2 * R))
void qknorm_fwd_kernel(const QkFwdArgs a) {
    using io = IO<Tag>;
    constexpr int E = io::E;
    __shared__ float part[2][R][K];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t row_bytes = static_cast<int64_t>(a.D) * io::kBytes;
    const int t = blockIdx.x >= static_cast<unsigned>(a.nb) ? 1 : 0;          // which tensor
    const int64_t member = static_cast<int64_t>(blockIdx.x) - static_cast<int64_t>(t) * a.nb;
    const void* x = t ? a.x[1] : a.x[0];
    const void* wgt = t ? a.w[1] : a.w[0];
    void* y = t ? a.y[1] : a.y[0];
    float* rstd = t ? a.rstd[1] : a.rstd[0];

    int chunk[VPL];
    bool ok[VPL];
    float W[VPL][E];
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
        chunk[i] = (i * K + wave) * kWave + lane;
        ok[i] = EXACT || chunk[i] < a.nchunks;
        u32x4 rw = u32x4{0u, 0u, 0u, 0u};
        if (ok[i]) rw = load16_cached(wgt, 0, static_cast<uint32_t>(chunk[i]) * 16u);
        io::unpack(rw, W[i]);
    }

    const int64_t stop = a.N;
    auto fetch = [&](int64_t base, u32x4 (&q)[R][VPL]) {
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const int64_t row = base + j;
#pragma unroll
            for (int i = 0; i < VPL; ++i) {
                if (row < stop && ok[i]) q[j][i] = load16_u(x, row * row_bytes, static_cast<uint32_t>(chunk[i]) * 16u);
                else q[j][i] = u32x4{0u, 0u, 0u, 0u};
            }
        }
    };
    const int64_t step = static_cast<int64_t>(a.nb) * R;
    int buf = 0;
    u32x4 raw[R][VPL];
    fetch(member * R, raw);

    for (int64_t base = member * R; base < stop; base += step) {
        u32x4 nxt[R][VPL];
        fetch(base + step, nxt);
        __builtin_amdgcn_sched_barrier(0);                   // keep the requests up here

        float rs[R];
#pragma unroll
        for (int j = 0; j < R; ++j) {
            float s = 0.0f;
#pragma unroll
            for (int i = 0; i < VPL; ++i) {
                float v[E];
                io::unpack(raw[j][i], v);
#pragma unroll
                for (int e = 0; e < E; ++e) s += v[e] * v[e];
            }
            rs[j] = wave_sum(s);
        }
        if (K > 1) {
            if (lane == 0) {
#pragma unroll
                for (int j = 0; j < R; ++j) part[buf][j][wave] = rs[j];
            }
            __syncthreads();
#pragma unroll
            for (int j = 0; j < R; ++j) {
                float tsum = 0.0f;
#pragma unroll
                for (int w = 0; w < K; ++w) tsum += part[buf][j][w];
                rs[j] = tsum;
            }
            buf ^= 1;
        }
#pragma unroll
        for (int j = 0; j < R; ++j) rs[j] = 1.0f / sqrtf(rs[j] * a.inv_D + a.eps);
        // opaque packed registers: the fp32 values are rebuilt below, not carried across the barrier
#pragma unroll
        for (int j = 0; j < R; ++j) {
#pragma unroll
            for (int i = 0; i < VPL; ++i) asm volatile("" : "+v"(raw[j][i]));
        }
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const int64_t row = base + j;
            if (row < stop) {
                if (wave == 0 && lane == 0) rstd[row] = rs[j];
#pragma unroll
                for (int i = 0; i < VPL; ++i) {
                    if (ok[i]) {
                        float v[E], o[E];
                        io::unpack(raw[j][i], v);
#pragma unroll
                        for (int e = 0; e < E; ++e) o[e] = (v[e] * rs[j]) * W[i][e];
                        store16_u(y, row * row_bytes, static_cast<uint32_t>(chunk[i]) * 16u, io::pack(o));
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
#pragma unroll
        for (int j = 0; j < R; ++j) {
#pragma unroll
            for (int i = 0; i < VPL; ++i) raw[j][i] = nxt[j][i];
        }
    }
}

// =============================================================================================
// Backward
// =============================================================================================
struct QkBwdArgs {
    const void* dy[2];       // gradients of the normalised q, k
    const void* x[2];
    const void* w[2];
    const float* rstd[2];
    void* dx[2];
    float* ws;               // [2][nb][D] fp32 partial dw sums
    int64_t N;
    int32_t nb;
    int32_t D;
    int32_t nchunks;
    float inv_D;
};

template <typename Tag, int VPL, int K, int R, bool EXACT>
__global__ __launch_bounds__(K* kWave)
LNMOD_OCCUPANCY(qk_waves_per_eu(VPL, IO<Tag>::E, 2, 4 * R))
void qknorm_bwd_kernel(const QkBwdArgs a) {
    using io = IO<Tag>;
    constexpr int E = io::E;
    __shared__ float part[2][R][K];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t row_bytes = static_cast<int64_t>(a.D) * io::kBytes;
    const int t = blockIdx.x >= static_cast<unsigned>(a.nb) ? 1 : 0;
    const int64_t member = static_cast<int64_t>(blockIdx.x) - static_cast<int64_t>(t) * a.nb;
    const void* dy = t ? a.dy[1] : a.dy[0];
    const void* x = t ? a.x[1] : a.x[0];
    const void* wgt = t ? a.w[1] : a.w[0];
    const float* rstd = t ? a.rstd[1] : a.rstd[0];
    void* dx = t ? a.dx[1] : a.dx[0];

    int chunk[VPL];
    bool ok[VPL];
    float W[VPL][E], acc[VPL][E];
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
        chunk[i] = (i * K + wave) * kWave + lane;
        ok[i] = EXACT || chunk[i] < a.nchunks;
        u32x4 rw = u32x4{0u, 0u, 0u, 0u};
        if (ok[i]) rw = load16_cached(wgt, 0, static_cast<uint32_t>(chunk[i]) * 16u);
        io::unpack(rw, W[i]);
#pragma unroll
        for (int e = 0; e < E; ++e) acc[i][e] = 0.0f;
    }

    const int64_t stop = a.N;
    // q[s][j][i]: s = 0 dy, 1 x; rows at or beyond `stop` read as zeros
    auto fetch = [&](int64_t base, u32x4 (&q)[2][R][VPL], float (&qrs)[R]) {
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const int64_t row = base + j;
            const bool live = row < stop;
            qrs[j] = live ? rstd[row] : 0.0f;
#pragma unroll
            for (int i = 0; i < VPL; ++i) {
                if (live && ok[i]) {
                    const uint32_t lo = static_cast<uint32_t>(chunk[i]) * 16u;
                    q[0][j][i] = load16_u(dy, row * row_bytes, lo);
                    q[1][j][i] = load16_u(x, row * row_bytes, lo);
                } else {
                    q[0][j][i] = u32x4{0u, 0u, 0u, 0u};
                    q[1][j][i] = u32x4{0u, 0u, 0u, 0u};
                }
            }
        }
    };
    const int64_t step = static_cast<int64_t>(a.nb) * R;
    int buf = 0;
    u32x4 raw[2][R][VPL];
    float rs[R];
    fetch(member * R, raw, rs);

    for (int64_t base = member * R; base < stop; base += step) {
        u32x4 nxt[2][R][VPL];
        float nrs[R];
        fetch(base + step, nxt, nrs);
        __builtin_amdgcn_sched_barrier(0);                   // keep the requests up here

        // pass 1: row sum of g*xhat and the running dw sums
        float c[R];
#pragma unroll
        for (int j = 0; j < R; ++j) {
            float p = 0.0f;
#pragma unroll
            for (int i = 0; i < VPL; ++i) {
                float dyv[E], xv[E];
                io::unpack(raw[0][j][i], dyv);
                io::unpack(raw[1][j][i], xv);
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    const float h = xv[e] * rs[j];
                    p += (dyv[e] * W[i][e]) * h;
                    acc[i][e] += dyv[e] * h;
                }
                // pin the running sums here, or the optimiser sinks the adds below the barrier
#pragma unroll
                for (int e = 0; e < E; ++e) asm volatile("" : "+v"(acc[i][e]));
                __builtin_amdgcn_sched_barrier(0);
            }
            c[j] = wave_sum(p);
        }
        if (K > 1) {
            if (lane == 0) {
#pragma unroll
                for (int j = 0; j < R; ++j) part[buf][j][wave] = c[j];
            }
            __syncthreads();
#pragma unroll
            for (int j = 0; j < R; ++j) {
                float tsum = 0.0f;
#pragma unroll
                for (int w = 0; w < K; ++w) tsum += part[buf][j][w];
                c[j] = tsum;
            }
            buf ^= 1;
        }
        // pass 2: dx = rstd*(g - xhat*c), from the packed registers again
#pragma unroll
        for (int s = 0; s < 2; ++s) {
#pragma unroll
            for (int j = 0; j < R; ++j) {
#pragma unroll
                for (int i = 0; i < VPL; ++i) asm volatile("" : "+v"(raw[s][j][i]));
            }
        }
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const int64_t row = base + j;
            if (row < stop) {
                const float k2 = rs[j] * (c[j] * a.inv_D);
#pragma unroll
                for (int i = 0; i < VPL; ++i) {
                    if (ok[i]) {
                        float dyv[E], xv[E], o[E];
                        io::unpack(raw[0][j][i], dyv);
                        io::unpack(raw[1][j][i], xv);
#pragma unroll
                        for (int e = 0; e < E; ++e) o[e] = (dyv[e] * W[i][e]) * rs[j] - (xv[e] * rs[j]) * k2;
                        store16_u(dx, row * row_bytes, static_cast<uint32_t>(chunk[i]) * 16u, io::pack(o));
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
#pragma unroll
        for (int j = 0; j < R; ++j) {
            rs[j] = nrs[j];
#pragma unroll
            for (int s = 0; s < 2; ++s) {
#pragma unroll
                for (int i = 0; i < VPL; ++i) raw[s][j][i] = nxt[s][j][i];
            }
        }
    }

    // this block's partial dw (zeros if it had no row)
    float* slot = a.ws + (static_cast<int64_t>(t) * a.nb + member) * a.D;
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
        if (ok[i]) {
            f32x4* ps = reinterpret_cast<f32x4*>(slot + static_cast<int64_t>(chunk[i]) * E);
#pragma unroll
            for (int q = 0; q < E / 4; ++q)
                ps[q] = f32x4{acc[i][4 * q], acc[i][4 * q + 1], acc[i][4 * q + 2], acc[i][4 * q + 3]};
        }
    }
}

// =============================================================================================
// Short rows (one head's width as the normalised dimension): a row of at most 16*VPL chunks is
// held by 16 lanes, so a wave works on four consecutive rows at once and reduces inside each
// group of 16 lanes with the DPP steps alone (no cross-row step, no LDS, no barrier).  A wave
// takes R such groups of four rows per step (consecutive rows, so its loads are contiguous), the
// waves of a tensor's half of the grid take consecutive pieces, and the next piece is requested
// before the current one is computed.
// =============================================================================================
__device__ inline float row16_sum(float v) {
    v = dpp_add<0xB1>(v);    // quad_perm [1,0,3,2]
    v = dpp_add<0x4E>(v);    // quad_perm [2,3,0,1]
    v = dpp_add<0x141>(v);   // row_half_mirror
    v = dpp_add<0x140>(v);   // row_mirror
    return v;                // every lane of the 16 holds the sum of its group
}

constexpr int kShortWaves = 4;               // waves per block (independent of each other)

template <typename Tag, int VPL, int R>
__global__ __launch_bounds__(kShortWaves* kWave)
void qknorm_short_fwd_kernel(const QkFwdArgs a) {
    using io = IO<Tag>;
    constexpr int E = io::E;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int group = lane >> 4, gl = lane & 15;
    const uint32_t row_bytes = static_cast<uint32_t>(a.D) * io::kBytes;
    const int t = blockIdx.x >= static_cast<unsigned>(a.nb) ? 1 : 0;
    const int64_t member = static_cast<int64_t>(blockIdx.x) - static_cast<int64_t>(t) * a.nb;
    const char* x = static_cast<const char*>(t ? a.x[1] : a.x[0]);
    const void* wgt = t ? a.w[1] : a.w[0];
    char* y = static_cast<char*>(t ? a.y[1] : a.y[0]);
    float* rstd = t ? a.rstd[1] : a.rstd[0];

    bool ok[VPL];
    uint32_t off[VPL];
    float W[VPL][E];
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
        const int chunk = i * 16 + gl;
        ok[i] = chunk < a.nchunks;
        off[i] = static_cast<uint32_t>(chunk) * 16u;
        u32x4 rw = u32x4{0u, 0u, 0u, 0u};
        if (ok[i]) rw = load16_cached(wgt, 0, off[i]);
        io::unpack(rw, W[i]);
    }

    constexpr int64_t kPieceRows = 4 * R;                                   // rows per wave and step
    const int64_t pieces = (a.N + kPieceRows - 1) / kPieceRows;
    const int64_t stride = static_cast<int64_t>(a.nb) * kShortWaves;
    auto fetch = [&](int64_t piece, u32x4 (&q)[R][VPL]) {
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const int64_t row = piece * kPieceRows + j * 4 + group;
#pragma unroll
            for (int i = 0; i < VPL; ++i) {
                if (piece < pieces && row < a.N && ok[i])
                    q[j][i] = load16(x, uniform64(piece * kPieceRows * row_bytes), (j * 4 + group) * row_bytes + off[i]);
                else
                    q[j][i] = u32x4{0u, 0u, 0u, 0u};
            }
        }
    };
    int64_t piece = member * kShortWaves + wave;
    u32x4 raw[R][VPL];
    fetch(piece, raw);
    for (; piece < pieces; piece += stride) {
        u32x4 nxt[R][VPL];
        fetch(piece + stride, nxt);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const int64_t row = piece * kPieceRows + j * 4 + group;
            float s = 0.0f;
#pragma unroll
            for (int i = 0; i < VPL; ++i) {
                float v[E];
                io::unpack(raw[j][i], v);
#pragma unroll
                for (int e = 0; e < E; ++e) s += v[e] * v[e];
            }
            const float rs = 1.0f / sqrtf(row16_sum(s) * a.inv_D + a.eps);
            if (row < a.N) {
                if (gl == 0) rstd[row] = rs;
#pragma unroll
                for (int i = 0; i < VPL; ++i) {
                    if (ok[i]) {
                        float v[E], o[E];
                        io::unpack(raw[j][i], v);
#pragma unroll
                        for (int e = 0; e < E; ++e) o[e] = (v[e] * rs) * W[i][e];
                        store16(y, uniform64(piece * kPieceRows * row_bytes), (j * 4 + group) * row_bytes + off[i], io::pack(o));
                    }
                }
            }
        }
#pragma unroll
        for (int j = 0; j < R; ++j) {
#pragma unroll
            for (int i = 0; i < VPL; ++i) raw[j][i] = nxt[j][i];
        }
    }
}

// One partial-sum slot per wave: slot (t*nb + member)*kShortWaves + wave of a.ws.
template <typename Tag, int VPL, int R>
__global__ __launch_bounds__(kShortWaves* kWave)
void qknorm_short_bwd_kernel(const QkBwdArgs a) {
    using io = IO<Tag>;
    constexpr int E = io::E;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int group = lane >> 4, gl = lane & 15;
    const uint32_t row_bytes = static_cast<uint32_t>(a.D) * io::kBytes;
    const int t = blockIdx.x >= static_cast<unsigned>(a.nb) ? 1 : 0;
    const int64_t member = static_cast<int64_t>(blockIdx.x) - static_cast<int64_t>(t) * a.nb;
    const char* dy = static_cast<const char*>(t ? a.dy[1] : a.dy[0]);
    const char* x = static_cast<const char*>(t ? a.x[1] : a.x[0]);
    const void* wgt = t ? a.w[1] : a.w[0];
    const float* rstd = t ? a.rstd[1] : a.rstd[0];
    char* dx = static_cast<char*>(t ? a.dx[1] : a.dx[0]);

    bool ok[VPL];
    uint32_t off[VPL];
    float W[VPL][E], acc[VPL][E];
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
        const int chunk = i * 16 + gl;
        ok[i] = chunk < a.nchunks;
        off[i] = static_cast<uint32_t>(chunk) * 16u;
        u32x4 rw = u32x4{0u, 0u, 0u, 0u};
        if (ok[i]) rw = load16_cached(wgt, 0, off[i]);
        io::unpack(rw, W[i]);
#pragma unroll
        for (int e = 0; e < E; ++e) acc[i][e] = 0.0f;
    }

    constexpr int64_t kPieceRows = 4 * R;
    const int64_t pieces = (a.N + kPieceRows - 1) / kPieceRows;
    const int64_t stride = static_cast<int64_t>(a.nb) * kShortWaves;
    auto fetch = [&](int64_t piece, u32x4 (&q)[2][R][VPL], float (&qrs)[R]) {
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const int64_t row = piece * kPieceRows + j * 4 + group;
            const bool live = piece < pieces && row < a.N;
            qrs[j] = live ? rstd[row] : 0.0f;
#pragma unroll
            for (int i = 0; i < VPL; ++i) {
                if (live && ok[i]) {
                    const int64_t base = uniform64(piece * kPieceRows * row_bytes);
                    const uint32_t lo = (j * 4 + group) * row_bytes + off[i];
                    q[0][j][i] = load16(dy, base, lo);
                    q[1][j][i] = load16(x, base, lo);
                } else {
                    q[0][j][i] = u32x4{0u, 0u, 0u, 0u};
                    q[1][j][i] = u32x4{0u, 0u, 0u, 0u};
                }
            }
        }
    };
    int64_t piece = member * kShortWaves + wave;
    u32x4 raw[2][R][VPL];
    float rs[R];
    fetch(piece, raw, rs);
    for (; piece < pieces; piece += stride) {
        u32x4 nxt[2][R][VPL];
        float nrs[R];
        fetch(piece + stride, nxt, nrs);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const int64_t row = piece * kPieceRows + j * 4 + group;
            float dyv[VPL][E], hv[VPL][E];
            float p = 0.0f;
#pragma unroll
            for (int i = 0; i < VPL; ++i) {
                float xv[E];
                io::unpack(raw[0][j][i], dyv[i]);
                io::unpack(raw[1][j][i], xv);
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    hv[i][e] = xv[e] * rs[j];
                    p += (dyv[i][e] * W[i][e]) * hv[i][e];
                    acc[i][e] += dyv[i][e] * hv[i][e];
                }
            }
            const float k2 = rs[j] * (row16_sum(p) * a.inv_D);
            if (row < a.N) {
#pragma unroll
                for (int i = 0; i < VPL; ++i) {
                    if (ok[i]) {
                        float o[E];
#pragma unroll
                        for (int e = 0; e < E; ++e) o[e] = (dyv[i][e] * W[i][e]) * rs[j] - hv[i][e] * k2;
                        store16(dx, uniform64(piece * kPieceRows * row_bytes), (j * 4 + group) * row_bytes + off[i], io::pack(o));
                    }
                }
            }
        }
#pragma unroll
        for (int j = 0; j < R; ++j) {
            rs[j] = nrs[j];
#pragma unroll
            for (int s = 0; s < 2; ++s) {
#pragma unroll
                for (int i = 0; i < VPL; ++i) raw[s][j][i] = nxt[s][j][i];
            }
        }
    }

    // add the four groups of the wave (lanes l, l+16, l+32, l+48 hold the same features), then
    // the first group writes the wave's slot
    float* slot = a.ws + ((static_cast<int64_t>(t) * a.nb + member) * kShortWaves + wave) * a.D;
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
#pragma unroll
        for (int e = 0; e < E; ++e) {
            float v = acc[i][e];
            v += __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(((lane ^ 16) << 2), __builtin_bit_cast(int, v)));
            v += __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(((lane ^ 32) << 2), __builtin_bit_cast(int, v)));
            acc[i][e] = v;
        }
        if (ok[i] && group == 0) {
            f32x4* ps = reinterpret_cast<f32x4*>(slot + (i * 16 + gl) * E);
#pragma unroll
            for (int q = 0; q < E / 4; ++q)
                ps[q] = f32x4{acc[i][4 * q], acc[i][4 * q + 1], acc[i][4 * q + 2], acc[i][4 * q + 3]};
        }
    }
}

// Second pass: dw[t][d] = sum of the nb slots of tensor t, slots in ascending order split over 16
// waves, the 16 wave sums then added in wave order.  grid.x = 2 * dblocks.
struct QkReduceArgs {
    const float* ws;
    float* dw[2];
    int32_t nb;
    int32_t D;
    int32_t dblocks;
};

template <int kUnused = 0>
__global__ __launch_bounds__(kReduceWaves* kWave) void qknorm_reduce_kernel(const QkReduceArgs a) {
    __shared__ float red[kReduceWaves][kWave];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int d = static_cast<int>(blockIdx.x % a.dblocks) * kWave + lane;
    const int t = static_cast<int>(blockIdx.x / a.dblocks);
    float acc = 0.0f;
    if (d < a.D) {
        // eight slots requested before the first is added (a wave may have 64 of them: short rows
        // give one slot per wave of the main kernel); the additions keep slot order
        const float* base = a.ws + static_cast<int64_t>(t) * a.nb * a.D + d;
        for (int64_t sl = wave; sl < a.nb; sl += 8 * kReduceWaves) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int64_t su = sl + static_cast<int64_t>(u) * kReduceWaves;
                v[u] = su < a.nb ? base[su * a.D] : 0.0f;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) acc += v[u];
        }
    }
    red[wave][lane] = acc;
    __syncthreads();
    if (wave == 0 && d < a.D) {
        float s = 0.0f;
#pragma unroll
        for (int w = 0; w < kReduceWaves; ++w) s += red[w][lane];
        (t ? a.dw[1] : a.dw[0])[d] = s;
    }
}

}  // namespace lnmod
