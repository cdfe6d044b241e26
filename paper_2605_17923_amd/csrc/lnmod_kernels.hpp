// lnmod_kernels.hpp -- gfx950 (MI355X, CDNA4) device code of the fused LayerNorm-Modulate operator.
//
// The operator (paper Sec. 3.3): per token row, mean and biased variance over the hidden
// dimension D in fp32, xhat = (x - mean) * rstd with rstd = 1/sqrt(var + eps), then
// y = xhat * (1 + scale) + shift; mean and rstd are saved for the backward.  The backward
// computes dx per row and the modulation gradients dshift = sum_n dy, dscale = sum_n dy*xhat
// along the token axis of each sample / packed segment (or per token, without a sum).
//
// Design for CDNA4 (64-wide wavefronts, no tensor-core work here: the path is bound by HBM):
//   * a token row is read once with 128-bit loads, lane l of a wave owns the 16-byte chunks
//     l, l+64, ... of the row, and the row stays in registers for all three uses
//     (sum, centred sum of squares, output), so x crosses HBM exactly once;
//   * row reductions use DPP adds inside a wave (no LDS, no ds_bpermute) and v_readlane for
//     the four 16-lane rows; only the backward, where several waves share a row so that the
//     per-lane dshift/dscale accumulators stay small, crosses waves through a few LDS floats;
//   * the forward keeps the sample's (1+scale, shift) rows in LDS as fp32, laid out by chunk
//     so that the ds_read_b128 of consecutive lanes hit consecutive banks;
//   * the backward fixes lane <-> feature for the whole life of a block and carries fp32
//     partial sums of dshift/dscale in registers down its rows (the paper's D-tile idea of
//     "thread fixed to a feature, accumulate along the sequence", Sec. 3.3, done inside the dx
//     kernel so dy and x are not read a second time); every block writes one partial slot per
//     segment it touches and a second kernel adds the slots in a fixed order: no float atomics,
//     bitwise reproducible;
//   * blocks own contiguous, equally sized row ranges so that all CUs finish together, and
//     walk the segment table themselves, so fixed-length and packed varlen batches share the code.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#ifndef LNMOD_NT_LOAD
#define LNMOD_NT_LOAD 1
#endif
#ifndef LNMOD_MAX_WAVES_PER_EU
#define LNMOD_MAX_WAVES_PER_EU 3   // the launches keep 2 to 3 waves per SIMD resident, not more
#endif
#ifndef LNMOD_NT_STORE
#define LNMOD_NT_STORE 1
#endif

namespace lnmod {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;

// Waves per SIMD the compiler must leave room for (512 VGPRs per SIMD lane), as a function of
// what one lane keeps live: the fp32 values of its part of the row plus two address registers
// per 16-byte chunk.  Without it the scheduler spends registers on hoisted loads until a single
// wave fills the SIMD and nothing hides the HBM latency.
constexpr int row_waves_per_eu(int vpl, int elems_per_chunk, int rows_live = 1) {
    const int cost = vpl * (elems_per_chunk * rows_live + 2);
    const int w = cost <= 40 ? 8 : cost <= 50 ? 6 : cost <= 60 ? 5 : cost <= 100 ? 4 : cost <= 130 ? 3 : 2;
    return w > LNMOD_MAX_WAVES_PER_EU ? LNMOD_MAX_WAVES_PER_EU : w;
}
// Kernels that keep `streams` packed 16-byte registers per chunk and rebuild fp32 values per pass.
constexpr int tok_waves_per_eu(int vpl, int streams) {
    const int regs = vpl * (4 * streams + 1) + 40;
    const int w = 512 / regs;
    return w > LNMOD_MAX_WAVES_PER_EU ? LNMOD_MAX_WAVES_PER_EU : w < 1 ? 1 : w;
}
#define LNMOD_OCCUPANCY(W) __attribute__((amdgpu_waves_per_eu(W)))

struct bf16_io {};
struct f32_io {};

// ---- 16-byte chunk <-> fp32 lanes -------------------------------------------------------
template <typename Tag> struct IO;

template <> struct IO<bf16_io> {
    static constexpr int E = 8;            // elements per 16-byte chunk
    static constexpr int kBytes = 2;
    __device__ static inline void unpack(const u32x4& r, float (&v)[8]) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            v[2 * j] = __builtin_bit_cast(float, r[j] << 16);
            v[2 * j + 1] = __builtin_bit_cast(float, r[j] & 0xffff0000u);
        }
    }
    // round to nearest even, two values per v_cvt_pk_bf16_f32
    __device__ static inline u32x4 pack(const float (&v)[8]) {
        u32x4 r;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            f32x2 f = {v[2 * j], v[2 * j + 1]};
            r[j] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
        }
        return r;
    }
};

template <> struct IO<f32_io> {
    static constexpr int E = 4;
    static constexpr int kBytes = 4;
    // whole-vector bit casts only: a bit cast of a single vector element is miscompiled by
    // this toolchain (every element reads as element 0)
    __device__ static inline void unpack(const u32x4& r, float (&v)[4]) {
        const f32x4 f = __builtin_bit_cast(f32x4, r);
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = f[j];
    }
    __device__ static inline u32x4 pack(const float (&v)[4]) {
        const f32x4 f = {v[0], v[1], v[2], v[3]};
        return __builtin_bit_cast(u32x4, f);
    }
};

// Addresses are (wave-uniform base + uniform byte offset) + a 32-bit unsigned lane offset, so
// the backend can keep the base in SGPRs and spend one VGPR per chunk instead of a 64-bit pair.
// The readfirstlane pair is free for a value that already sits in SGPRs; it stops loop
// strength reduction from turning every chunk address into its own 64-bit per-lane induction
// variable.
__device__ inline int64_t uniform64(int64_t v) {
    const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(v));
    const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(static_cast<uint64_t>(v) >> 32));
    return static_cast<int64_t>((static_cast<uint64_t>(hi) << 32) | lo);
}

__device__ inline u32x4 load16(const void* base, int64_t uniform_off, uint32_t lane_off) {
    const u32x4* p = reinterpret_cast<const u32x4*>(static_cast<const char*>(base) + uniform_off + lane_off);
#if LNMOD_NT_LOAD
    return __builtin_nontemporal_load(p);
#else
    return *p;
#endif
}

__device__ inline u32x4 load16_cached(const void* base, int64_t uniform_off, uint32_t lane_off) {
    return *reinterpret_cast<const u32x4*>(static_cast<const char*>(base) + uniform_off + lane_off);
}

__device__ inline void store16(void* base, int64_t uniform_off, uint32_t lane_off, const u32x4& v) {
    u32x4* p = reinterpret_cast<u32x4*>(static_cast<char*>(base) + uniform_off + lane_off);
#if LNMOD_NT_STORE
    __builtin_nontemporal_store(v, p);
#else
    *p = v;
#endif
}

// Variants that pin the uniform part into SGPRs (see uniform64) for kernels whose many live
// accumulators leave no room for 64-bit per-lane address pairs.
__device__ inline u32x4 load16_u(const void* base, int64_t uniform_off, uint32_t lane_off) {
    return load16(base, uniform64(uniform_off), lane_off);
}
__device__ inline void store16_u(void* base, int64_t uniform_off, uint32_t lane_off, const u32x4& v) {
    store16(base, uniform64(uniform_off), lane_off, v);
}

// ---- wave-wide sum: DPP butterflies inside each row of 16 lanes, then the 4 rows ----------
template <int CTRL> __device__ inline float dpp_add(float v) {
    int t = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false);
    return v + __builtin_bit_cast(float, t);
}

// Every lane returns the same value: the partners of each step hold each other's operands,
// fp32 addition is commutative, and the last four adds run in one fixed order.
__device__ inline float wave_sum(float v) {
    v = dpp_add<0xB1>(v);    // quad_perm [1,0,3,2]
    v = dpp_add<0x4E>(v);    // quad_perm [2,3,0,1]
    v = dpp_add<0x141>(v);   // row_half_mirror
    v = dpp_add<0x140>(v);   // row_mirror
    const int b = __builtin_bit_cast(int, v);
    float s = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 0));
    s += __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 16));
    s += __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 32));
    s += __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 48));
    return s;
}

// ---- segment table: fixed-length samples (cu == nullptr) or packed offsets on the device ----
struct Segments {
    const int32_t* cu;   // [nseg+1] token offsets, or nullptr for nseg samples of S tokens
    int64_t S;
    int64_t nseg;
};

__device__ inline int64_t seg_begin(const Segments& s, int64_t m) {
    return s.cu ? static_cast<int64_t>(s.cu[m]) : m * s.S;
}

// Largest m in [0, nseg-1] whose first token is <= row (skips empty segments in front of row).
// Terminates and stays in range for any table contents.
__device__ inline int64_t find_segment(const Segments& s, int64_t row) {
    if (!s.cu) return row / s.S;
    int64_t lo = 0, hi = s.nseg - 1;
    while (lo < hi) {
        const int64_t mid = (lo + hi + 1) >> 1;
        if (static_cast<int64_t>(s.cu[mid]) <= row) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// =============================================================================================
// Forward, modulation row per sample / per segment.  One wave per token row; the block's WPB
// waves take the rows of the block's range round-robin.
// =============================================================================================
struct FwdArgs {
    const void* x;
    const void* shift;
    const void* scale;
    void* y;
    float* mean;
    float* rstd;
    Segments seg;
    int64_t T;               // total token rows
    int64_t rows_per_cluster; // rows of the contiguous region one cluster of blocks streams through
    int32_t nb;              // blocks per cluster (per-token kernels: unused)
    int32_t D;
    int32_t nchunks;         // D / E
    float eps;
    float inv_D;
};

template <typename Tag, int VPL, int WPB, bool EXACT, bool PF = true>
__global__ __launch_bounds__(WPB* kWave) LNMOD_OCCUPANCY(row_waves_per_eu(VPL, IO<Tag>::E + (PF ? 4 : 0)))
void fwd_seg_kernel(const FwdArgs a) {
    using io = IO<Tag>;
    constexpr int E = io::E;
    constexpr int Q = E / 4;            // float4 parts per chunk
    constexpr int CH = VPL * kWave;     // chunk slots per row
    extern __shared__ f32x4 lds[];      // [2][Q][CH]: (1+scale) parts, then shift parts

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t row_bytes = static_cast<int64_t>(a.D) * io::kBytes;

    // cluster of a.nb blocks <-> contiguous region of rows; inside the region the cluster's
    // waves take consecutive rows, so at any moment the cluster streams through one window
    const int64_t cluster = blockIdx.x / a.nb;
    const int64_t member = blockIdx.x - cluster * a.nb;
    int64_t r0 = cluster * a.rows_per_cluster;
    int64_t r1 = r0 + a.rows_per_cluster;
    if (r1 > a.T) r1 = a.T;

    while (r0 < r1) {
        const int64_t m = find_segment(a.seg, r0);
        int64_t stop = seg_begin(a.seg, m + 1);
        if (stop > r1) stop = r1;
        if (stop <= r0) stop = r0 + 1;          // malformed table: still make progress

        __syncthreads();                        // readers of the previous segment's rows are done
        for (int c = threadIdx.x; c < CH; c += WPB * kWave) {
            if (EXACT || c < a.nchunks) {
                const uint32_t lo = static_cast<uint32_t>(c) * 16u;
                float sc[E], sh[E];
                io::unpack(load16_cached(a.scale, m * row_bytes, lo), sc);
                io::unpack(load16_cached(a.shift, m * row_bytes, lo), sh);
#pragma unroll
                for (int q = 0; q < Q; ++q) {
                    f32x4 p = {1.0f + sc[4 * q], 1.0f + sc[4 * q + 1], 1.0f + sc[4 * q + 2], 1.0f + sc[4 * q + 3]};
                    f32x4 s = {sh[4 * q], sh[4 * q + 1], sh[4 * q + 2], sh[4 * q + 3]};
                    lds[(0 * Q + q) * CH + c] = p;
                    lds[(1 * Q + q) * CH + c] = s;
                }
            }
        }
        __syncthreads();

        // Software pipeline: the wave requests its next row before it works on the current one,
        // so a few waves per CU keep the memory system busy (few, deep streams reach a higher
        // HBM bandwidth than many shallow ones).
        auto fetch = [&](int64_t row, u32x4 (&q)[VPL]) {
#pragma unroll
            for (int i = 0; i < VPL; ++i) {
                const int c = i * kWave + lane;
                if (row < stop && (EXACT || c < a.nchunks))
                    q[i] = load16(a.x, row * row_bytes, static_cast<uint32_t>(c) * 16u);
                else
                    q[i] = u32x4{0u, 0u, 0u, 0u};
            }
        };
        const int64_t row_step = static_cast<int64_t>(a.nb) * WPB;
        u32x4 raw[VPL];
        if (PF) fetch(r0 + member * WPB + wave, raw);

        for (int64_t row = r0 + member * WPB + wave; row < stop; row += row_step) {
            const int64_t base = row * row_bytes;
            u32x4 nxt[VPL];
            if (PF) {
                fetch(row + row_step, nxt);
                __builtin_amdgcn_sched_barrier(0);           // keep the requests up here
            } else {
                fetch(row, raw);
            }
            float v[VPL][E];
            float s = 0.0f;
#pragma unroll
            for (int i = 0; i < VPL; ++i) {
                io::unpack(raw[i], v[i]);
#pragma unroll
                for (int e = 0; e < E; ++e) s += v[i][e];
            }
            const float mu = wave_sum(s) / static_cast<float>(a.D);   // exact for constant rows
            float q2 = 0.0f;
#pragma unroll
            for (int i = 0; i < VPL; ++i) {
                const bool ok = EXACT || (i * kWave + lane) < a.nchunks;
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    v[i][e] = ok ? v[i][e] - mu : 0.0f;
                    q2 += v[i][e] * v[i][e];
                }
            }
            const float var = wave_sum(q2) * a.inv_D;
            const float rs = 1.0f / sqrtf(var + a.eps);
            if (lane == 0) {
                a.mean[row] = mu;
                a.rstd[row] = rs;
            }
#pragma unroll
            for (int i = 0; i < VPL; ++i) {
                const int c = i * kWave + lane;
                if (EXACT || c < a.nchunks) {
                    float o[E];
#pragma unroll
                    for (int q = 0; q < Q; ++q) {
                        const f32x4 p = lds[(0 * Q + q) * CH + c];
                        const f32x4 sh = lds[(1 * Q + q) * CH + c];
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[4 * q + e] = (v[i][4 * q + e] * rs) * p[e] + sh[e];
                    }
                    store16(a.y, base, static_cast<uint32_t>(c) * 16u, io::pack(o));
                }
                // keep the LDS reads of later chunks from being hoisted above this one: in a
                // branch-free body the scheduler otherwise issues all of them first and spills
                __builtin_amdgcn_sched_barrier(0);
            }
            if (PF) {
#pragma unroll
                for (int i = 0; i < VPL; ++i) raw[i] = nxt[i];
            }
        }
        r0 = stop;
    }
}

// =============================================================================================
// Forward, modulation row per token: shift/scale [T, D] stream with x; no LDS, no segments.
// =============================================================================================
// Makes the packed registers opaque between passes, so that the fp32 copies of one pass are
// rebuilt (one shift or mask per value) instead of being carried in registers to the next.
template <int N> __device__ inline void forget(u32x4 (&r)[N]) {
#pragma unroll
    for (int i = 0; i < N; ++i) asm volatile("" : "+v"(r[i]));
}

template <typename Tag, int VPL, int WPB, bool EXACT>
__global__ __launch_bounds__(WPB* kWave) LNMOD_OCCUPANCY(tok_waves_per_eu(VPL, 3))
void fwd_tok_kernel(const FwdArgs a) {
    using io = IO<Tag>;
    constexpr int E = io::E;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t row_bytes = static_cast<int64_t>(a.D) * io::kBytes;

    // all waves of the grid take consecutive rows: the launch streams through one moving window
    const int64_t r0 = static_cast<int64_t>(blockIdx.x) * WPB;
    const int64_t r1 = a.T;
    const int64_t row_step = static_cast<int64_t>(gridDim.x) * WPB;

    for (int64_t row = r0 + wave; row < r1; row += row_step) {
        const int64_t base = row * row_bytes;
        u32x4 raw[VPL], rsc[VPL], rsh[VPL];
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            const int c = i * kWave + lane;
            if (EXACT || c < a.nchunks) {
                raw[i] = load16(a.x, base, static_cast<uint32_t>(c) * 16u);
                rsc[i] = load16(a.scale, base, static_cast<uint32_t>(c) * 16u);
                rsh[i] = load16(a.shift, base, static_cast<uint32_t>(c) * 16u);
            } else {
                raw[i] = rsc[i] = rsh[i] = u32x4{0u, 0u, 0u, 0u};
            }
        }
        float s = 0.0f;
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            float v[E];
            io::unpack(raw[i], v);
#pragma unroll
            for (int e = 0; e < E; ++e) s += v[e];
        }
        const float mu = wave_sum(s) / static_cast<float>(a.D);   // exact for constant rows
        forget(raw);
        float q2 = 0.0f;
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            if (EXACT || (i * kWave + lane) < a.nchunks) {
                float v[E];
                io::unpack(raw[i], v);
#pragma unroll
                for (int e = 0; e < E; ++e) q2 += (v[e] - mu) * (v[e] - mu);
            }
        }
        const float var = wave_sum(q2) * a.inv_D;
        const float rs = 1.0f / sqrtf(var + a.eps);
        if (lane == 0) {
            a.mean[row] = mu;
            a.rstd[row] = rs;
        }
        forget(raw);
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            const int c = i * kWave + lane;
            if (EXACT || c < a.nchunks) {
                float v[E], sc[E], sh[E], o[E];
                io::unpack(raw[i], v);
                io::unpack(rsc[i], sc);
                io::unpack(rsh[i], sh);
#pragma unroll
                for (int e = 0; e < E; ++e) o[e] = ((v[e] - mu) * rs) * (1.0f + sc[e]) + sh[e];
                store16(a.y, base, static_cast<uint32_t>(c) * 16u, io::pack(o));
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
}

// =============================================================================================
// Backward, modulation row per sample / per segment.
// K waves share a row: wave w, lane l owns chunks (i*K + w)*64 + l, i < VPL, for the whole
// life of the block, so (1+scale) and the dshift/dscale partial sums of those features live
// in registers.  R consecutive rows are processed per step; the two row sums cross waves
// through a double-buffered LDS array and one barrier per step.
// Partial slot of (block b, segment m) is b + m: along the staircase of (block, segment)
// incidences b + m strictly increases, so slots never collide, and there are at most
// nblocks + nseg - 1 of them.
// =============================================================================================
struct BwdArgs {
    const void* dy;
    const void* x;
    const void* scale;
    const float* mean;
    const float* rstd;
    void* dx;
    void* dshift;            // per-token mode only (I/O dtype)
    void* dscale;            // per-token mode only
    float* ws;               // [nslots][2][D] fp32 partial sums
    Segments seg;
    int64_t T;
    int64_t rows_per_cluster;
    int32_t nb;              // blocks per cluster
    int32_t D;
    int32_t nchunks;
    float inv_D;
};

constexpr int bwd_waves_per_eu(int vpl, int elems_per_chunk, int rows) {
    // live per lane and chunk: 1+scale and two accumulators (fp32), `rows` packed copies of dy
    // and x with their addresses; plus unpack temporaries and loop state
    const int regs = vpl * (3 * elems_per_chunk + 10 * rows) + 28;
    const int w = 512 / regs;
    return w > LNMOD_MAX_WAVES_PER_EU ? LNMOD_MAX_WAVES_PER_EU : w < 1 ? 1 : w;
}

template <typename Tag, int VPL, int K, int R, bool EXACT, bool PF = true>
__global__ __launch_bounds__(K* kWave) LNMOD_OCCUPANCY(bwd_waves_per_eu(VPL, IO<Tag>::E, PF ? 2 * R : R))
void bwd_seg_kernel(const BwdArgs a) {
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

    const int64_t cluster = blockIdx.x / a.nb;
    const int64_t member = blockIdx.x - cluster * a.nb;
    int64_t r0 = cluster * a.rows_per_cluster;
    int64_t r1 = r0 + a.rows_per_cluster;
    if (r1 > a.T) r1 = a.T;
    int buf = 0;

    while (r0 < r1) {
        const int64_t m = find_segment(a.seg, r0);
        int64_t stop = seg_begin(a.seg, m + 1);
        if (stop > r1) stop = r1;
        if (stop <= r0) stop = r0 + 1;

        float A[VPL][E], acc_s[VPL][E], acc_c[VPL][E];
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            u32x4 r = u32x4{0u, 0u, 0u, 0u};
            if (ok[i]) r = load16_cached(a.scale, m * row_bytes, static_cast<uint32_t>(chunk[i]) * 16u);
            io::unpack(r, A[i]);
#pragma unroll
            for (int e = 0; e < E; ++e) {
                A[i][e] += 1.0f;
                acc_s[i][e] = 0.0f;
                acc_c[i][e] = 0.0f;
            }
        }

        // Software pipeline: the packed dy/x of the block's next step are requested before the
        // current step is computed, so every block keeps loads in flight while it does
        // arithmetic, waits at its barrier and stores.
        auto fetch = [&](int64_t base, u32x4 (&qdy)[R][VPL], u32x4 (&qx)[R][VPL], float (&qmu)[R],
                         float (&qrs)[R]) {
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
                        qdy[j][i] = load16_u(a.dy, row * row_bytes, lo);
                        qx[j][i] = load16_u(a.x, row * row_bytes, lo);
                    } else {
                        qdy[j][i] = u32x4{0u, 0u, 0u, 0u};
                        qx[j][i] = u32x4{0u, 0u, 0u, 0u};
                    }
                }
            }
        };
        const int64_t step = static_cast<int64_t>(a.nb) * R;
        u32x4 rdy[R][VPL], rx[R][VPL];
        float mu[R], rs[R];
        if (PF) fetch(r0 + member * R, rdy, rx, mu, rs);     // rows at or beyond `stop` read as zeros

        for (int64_t base = r0 + member * R; base < stop; base += step) {
            u32x4 ndy[R][VPL], nx[R][VPL];
            float nmu[R], nrs[R];
            if (PF) {
                fetch(base + step, ndy, nx, nmu, nrs);
                __builtin_amdgcn_sched_barrier(0);           // keep the requests up here
            } else {
                fetch(base, rdy, rx, mu, rs);
            }
            // pass 1 over the registers: row sums for dx and the running dshift/dscale sums.
            // xhat and g are not kept: they are rebuilt from the packed registers in pass 2,
            // which costs a few ALU operations and saves the registers that occupancy needs.
            float c1[R], c2[R];
#pragma unroll
            for (int j = 0; j < R; ++j) {
                float p1 = 0.0f, p2 = 0.0f;
#pragma unroll
                for (int i = 0; i < VPL; ++i) {
                    float dyv[E], xv[E];
                    io::unpack(rdy[j][i], dyv);
                    io::unpack(rx[j][i], xv);
#pragma unroll
                    for (int e = 0; e < E; ++e) {
                        // xhat as (x - mean) * rstd, not x*rstd - mean*rstd: the latter loses every digit
                        // on (near-)constant rows, where rstd is as large as 1/sqrt(eps)
                        const float h = (xv[e] - mu[j]) * rs[j];
                        const float gg = dyv[e] * A[i][e];
                        p1 += gg;
                        p2 += gg * h;
                        acc_s[i][e] += dyv[e];
                        acc_c[i][e] += dyv[e] * h;
                    }
                    // Pin the running sums here.  They are only consumed at the end of the loop,
                    // so the optimiser would otherwise sink these adds below the barrier and keep
                    // every unpacked dy and xhat alive until then (twice the row in registers).
#pragma unroll
                    for (int e = 0; e < E; ++e) asm volatile("" : "+v"(acc_s[i][e]), "+v"(acc_c[i][e]));
                    // one chunk at a time: stops the scheduler from unpacking every chunk up front
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
            // pass 2: dx = rstd * (g - c1 - xhat*c2).  The empty asm makes the packed registers
            // opaque so that common-subexpression elimination cannot carry pass 1's fp32 values
            // across the barrier instead of rebuilding them.
#pragma unroll
            for (int j = 0; j < R; ++j) {
#pragma unroll
                for (int i = 0; i < VPL; ++i) asm volatile("" : "+v"(rdy[j][i]), "+v"(rx[j][i]));
            }
#pragma unroll
            for (int j = 0; j < R; ++j) {
                const int64_t row = base + j;
                if (row < stop) {
                    const float k1 = rs[j] * (c1[j] * a.inv_D), k2 = rs[j] * (c2[j] * a.inv_D);
#pragma unroll
                    for (int i = 0; i < VPL; ++i) {
                        if (ok[i]) {
                            float dyv[E], xv[E], o[E];
                            io::unpack(rdy[j][i], dyv);
                            io::unpack(rx[j][i], xv);
#pragma unroll
                            for (int e = 0; e < E; ++e) {
                                const float h = (xv[e] - mu[j]) * rs[j];
                                o[e] = (dyv[e] * A[i][e]) * rs[j] - k1 - h * k2;
                            }
                            store16_u(a.dx, row * row_bytes, static_cast<uint32_t>(chunk[i]) * 16u, io::pack(o));
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
            if (PF) {
#pragma unroll
                for (int j = 0; j < R; ++j) {
                    mu[j] = nmu[j];
                    rs[j] = nrs[j];
#pragma unroll
                    for (int i = 0; i < VPL; ++i) {
                        rdy[j][i] = ndy[j][i];
                        rx[j][i] = nx[j][i];
                    }
                }
            }
        }

        // this block's partial sums for segment m
        float* slot = a.ws + ((cluster + m) * a.nb + member) * 2 * a.D;
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            if (ok[i]) {
                f32x4* ps = reinterpret_cast<f32x4*>(slot + static_cast<int64_t>(chunk[i]) * E);
                f32x4* pc = reinterpret_cast<f32x4*>(slot + a.D + static_cast<int64_t>(chunk[i]) * E);
#pragma unroll
                for (int q = 0; q < E / 4; ++q) {
                    ps[q] = f32x4{acc_s[i][4 * q], acc_s[i][4 * q + 1], acc_s[i][4 * q + 2], acc_s[i][4 * q + 3]};
                    pc[q] = f32x4{acc_c[i][4 * q], acc_c[i][4 * q + 1], acc_c[i][4 * q + 2], acc_c[i][4 * q + 3]};
                }
            }
        }
        r0 = stop;
    }
}

// Second pass: dshift/dscale[m, d] = sum of the partial slots of segment m, slots in ascending
// block order split over 16 waves (wave w takes slots w, w+16, ...), the 16 wave sums then added
// in wave order.  The order depends only on the shapes, so results repeat bit for bit.
struct ReduceArgs {
    const float* ws;
    float* dshift;           // [nseg, D]
    float* dscale;
    Segments seg;
    int64_t T;
    int64_t rows_per_cluster;
    int32_t nb;              // blocks per cluster = partial slots per (cluster, segment)
    int32_t D;
    int32_t dblocks;         // ceil(D / 64)
};

constexpr int kReduceWaves = 16;

// (a template only so that the header can be included in several translation units)
// grid.x = nseg * 2 * dblocks, decoded as (segment, dshift|dscale, block of 64 features)
template <int kUnused = 0>
__global__ __launch_bounds__(kReduceWaves* kWave) void bwd_reduce_kernel(const ReduceArgs a) {
    __shared__ float red[kReduceWaves][kWave];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int64_t bid = blockIdx.x;
    const int d = static_cast<int>(bid % a.dblocks) * kWave + lane;
    const int which = static_cast<int>((bid / a.dblocks) & 1);      // 0: dshift, 1: dscale
    const int64_t m = bid / (2 * static_cast<int64_t>(a.dblocks));
    int64_t n0 = seg_begin(a.seg, m), n1 = seg_begin(a.seg, m + 1);
    if (n0 < 0) n0 = 0;                       // a malformed table must not lead outside ws
    if (n1 > a.T) n1 = a.T;
    float acc = 0.0f;
    if (n1 > n0 && d < a.D) {
        // clusters c_lo..c_hi touch this segment; (cluster c, segment m) owns slots (c+m)*nb ..
        const int64_t c_lo = n0 / a.rows_per_cluster, c_hi = (n1 - 1) / a.rows_per_cluster;
        const int64_t s_lo = (c_lo + m) * a.nb, s_hi = (c_hi + m + 1) * a.nb;
        for (int64_t sl = s_lo + wave; sl < s_hi; sl += kReduceWaves)
            acc += a.ws[(sl * 2 + which) * a.D + d];
    }
    red[wave][lane] = acc;
    __syncthreads();
    if (wave == 0 && d < a.D) {
        float t = 0.0f;
#pragma unroll
        for (int w = 0; w < kReduceWaves; ++w) t += red[w][lane];
        (which == 0 ? a.dshift : a.dscale)[m * a.D + d] = t;
    }
}

// =============================================================================================
// Backward, modulation row per token: one wave per row, dshift = dy and dscale = dy*xhat are
// written per token in the I/O dtype, nothing is summed over tokens.
// =============================================================================================
template <typename Tag, int VPL, int WPB, bool EXACT>
__global__ __launch_bounds__(WPB* kWave) LNMOD_OCCUPANCY(tok_waves_per_eu(VPL, 3))
void bwd_tok_kernel(const BwdArgs a) {
    using io = IO<Tag>;
    constexpr int E = io::E;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t row_bytes = static_cast<int64_t>(a.D) * io::kBytes;

    // all waves of the grid take consecutive rows: the launch streams through one moving window
    const int64_t r0 = static_cast<int64_t>(blockIdx.x) * WPB;
    const int64_t r1 = a.T;
    const int64_t row_step = static_cast<int64_t>(gridDim.x) * WPB;

    for (int64_t row = r0 + wave; row < r1; row += row_step) {
        const int64_t base = row * row_bytes;
        const float mu = a.mean[row], rs = a.rstd[row];
        u32x4 rdy[VPL], rx[VPL], rsc[VPL];
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            const int c = i * kWave + lane;
            if (EXACT || c < a.nchunks) {
                rdy[i] = load16(a.dy, base, static_cast<uint32_t>(c) * 16u);
                rx[i] = load16(a.x, base, static_cast<uint32_t>(c) * 16u);
                rsc[i] = load16(a.scale, base, static_cast<uint32_t>(c) * 16u);
            } else {
                rdy[i] = rx[i] = rsc[i] = u32x4{0u, 0u, 0u, 0u};
            }
        }
        float p1 = 0.0f, p2 = 0.0f;
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            float dyv[E], xv[E], sc[E];
            io::unpack(rdy[i], dyv);
            io::unpack(rx[i], xv);
            io::unpack(rsc[i], sc);
#pragma unroll
            for (int e = 0; e < E; ++e) {
                const float h = (xv[e] - mu) * rs;
                const float gg = dyv[e] * (1.0f + sc[e]);
                p1 += gg;
                p2 += gg * h;
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        const float k1 = rs * (wave_sum(p1) * a.inv_D);
        const float k2 = rs * (wave_sum(p2) * a.inv_D);
        forget(rdy);
        forget(rx);
        forget(rsc);
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            const int c = i * kWave + lane;
            if (EXACT || c < a.nchunks) {
                float dyv[E], xv[E], sc[E], o[E], ds[E];
                io::unpack(rdy[i], dyv);
                io::unpack(rx[i], xv);
                io::unpack(rsc[i], sc);
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    const float h = (xv[e] - mu) * rs;
                    o[e] = (dyv[e] * (1.0f + sc[e])) * rs - k1 - h * k2;
                    ds[e] = dyv[e] * h;
                }
                const uint32_t lo = static_cast<uint32_t>(c) * 16u;
                store16(a.dx, base, lo, io::pack(o));
                store16(a.dshift, base, lo, rdy[i]);
                store16(a.dscale, base, lo, io::pack(ds));
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
}

// =============================================================================================
// Measurement comparators (not part of the fused path): the unfused two-kernel chain
// LayerNorm -> xhat in HBM -> modulate, and a plain 16-byte copy as the bandwidth ceiling.
// =============================================================================================
template <typename Tag, int VPL, int WPB, bool EXACT>
__global__ __launch_bounds__(WPB* kWave) LNMOD_OCCUPANCY(row_waves_per_eu(VPL, IO<Tag>::E))
void unfused_ln_kernel(const FwdArgs a) {
    using io = IO<Tag>;
    constexpr int E = io::E;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t row_bytes = static_cast<int64_t>(a.D) * io::kBytes;
    // all waves of the grid take consecutive rows: the launch streams through one moving window
    const int64_t r0 = static_cast<int64_t>(blockIdx.x) * WPB;
    const int64_t r1 = a.T;
    const int64_t row_step = static_cast<int64_t>(gridDim.x) * WPB;
    for (int64_t row = r0 + wave; row < r1; row += row_step) {
        const int64_t base = row * row_bytes;
        u32x4 raw[VPL];
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            const int c = i * kWave + lane;
            if (EXACT || c < a.nchunks) raw[i] = load16(a.x, base, static_cast<uint32_t>(c) * 16u);
            else raw[i] = u32x4{0u, 0u, 0u, 0u};
        }
        float v[VPL][E];
        float s = 0.0f;
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            io::unpack(raw[i], v[i]);
#pragma unroll
            for (int e = 0; e < E; ++e) s += v[i][e];
        }
        const float mu = wave_sum(s) / static_cast<float>(a.D);   // exact for constant rows
        float q2 = 0.0f;
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            const bool ok = EXACT || (i * kWave + lane) < a.nchunks;
#pragma unroll
            for (int e = 0; e < E; ++e) {
                v[i][e] = ok ? v[i][e] - mu : 0.0f;
                q2 += v[i][e] * v[i][e];
            }
        }
        const float rs = 1.0f / sqrtf(wave_sum(q2) * a.inv_D + a.eps);
        if (lane == 0) {
            a.mean[row] = mu;
            a.rstd[row] = rs;
        }
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            const int c = i * kWave + lane;
            if (EXACT || c < a.nchunks) {
                float o[E];
#pragma unroll
                for (int e = 0; e < E; ++e) o[e] = v[i][e] * rs;
                store16(a.y, base, static_cast<uint32_t>(c) * 16u, io::pack(o));   // a.y: xhat buffer
            }
        }
    }
}

// y = xhat * (1 + scale[m]) + shift[m]; a.x is the xhat buffer.  One wave per row as above.
template <typename Tag, int VPL, int WPB, bool EXACT>
__global__ __launch_bounds__(WPB* kWave) void unfused_mod_kernel(const FwdArgs a) {
    using io = IO<Tag>;
    constexpr int E = io::E;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t row_bytes = static_cast<int64_t>(a.D) * io::kBytes;
    // all waves of the grid take consecutive rows: the launch streams through one moving window
    const int64_t r0 = static_cast<int64_t>(blockIdx.x) * WPB;
    const int64_t r1 = a.T;
    const int64_t row_step = static_cast<int64_t>(gridDim.x) * WPB;
    for (int64_t row = r0 + wave; row < r1; row += row_step) {
        const int64_t m = find_segment(a.seg, row);
        const int64_t base = row * row_bytes;
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            const int c = i * kWave + lane;
            if (EXACT || c < a.nchunks) {
                float v[E], sc[E], sh[E], o[E];
                io::unpack(load16(a.x, base, static_cast<uint32_t>(c) * 16u), v);
                io::unpack(load16_cached(a.scale, m * row_bytes, static_cast<uint32_t>(c) * 16u), sc);
                io::unpack(load16_cached(a.shift, m * row_bytes, static_cast<uint32_t>(c) * 16u), sh);
#pragma unroll
                for (int e = 0; e < E; ++e) o[e] = v[e] * (1.0f + sc[e]) + sh[e];
                store16(a.y, base, static_cast<uint32_t>(c) * 16u, io::pack(o));
            }
        }
    }
}

// Plain copy in the same access pattern as the row kernels: every wave moves 4 KB per step
// with 16-byte nontemporal accesses, the waves of the grid take consecutive 4 KB pieces, and
// the next piece is requested before the current one is stored.
constexpr int kCopyWaves = 4;
constexpr int kCopyVecs = 4;     // 16-byte vectors per lane and step

template <int kUnused = 0>
__global__ __launch_bounds__(kCopyWaves* kWave) void copy16_kernel(const u32x4* __restrict__ src,
                                                                   u32x4* __restrict__ dst, int64_t nvec) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    constexpr int64_t kPiece = static_cast<int64_t>(kCopyVecs) * kWave;
    const int64_t pieces = nvec / kPiece;
    const int64_t step = static_cast<int64_t>(gridDim.x) * kCopyWaves;
    auto fetch = [&](int64_t piece, u32x4 (&q)[kCopyVecs]) {
#pragma unroll
        for (int i = 0; i < kCopyVecs; ++i) {
            if (piece < pieces) q[i] = __builtin_nontemporal_load(src + piece * kPiece + i * kWave + lane);
            else q[i] = u32x4{0u, 0u, 0u, 0u};
        }
    };
    int64_t piece = static_cast<int64_t>(blockIdx.x) * kCopyWaves + wave;
    u32x4 cur[kCopyVecs];
    fetch(piece, cur);
    for (; piece < pieces; piece += step) {
        u32x4 nxt[kCopyVecs];
        fetch(piece + step, nxt);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < kCopyVecs; ++i) __builtin_nontemporal_store(cur[i], dst + piece * kPiece + i * kWave + lane);
#pragma unroll
        for (int i = 0; i < kCopyVecs; ++i) cur[i] = nxt[i];
    }
    if (blockIdx.x == 0) {                       // fewer than one piece left over
        for (int64_t i = pieces * kPiece + threadIdx.x; i < nvec; i += kCopyWaves * kWave) dst[i] = src[i];
    }
}

}  // namespace lnmod
