// lnmod_kernels.hpp -- gfx950 (MI355X, CDNA4) device code of the fused LayerNorm-Modulate operator.
//
// The operator (paper Sec. 3.3): per token row, mean and biased variance over the hidden
// dimension D in fp32, xhat = (x - mean) * rstd with rstd = 1/sqrt(var + eps), then
// y = xhat * (1 + scale) + shift; mean and rstd are saved for the backward.  The backward
// computes dx per row and the modulation gradients dshift = sum_n dy, dscale = sum_n dy*xhat
// along the token axis of each sample / packed segment (or per token, without a sum).
//
// Design for CDNA4 (64-wide wavefronts, no tensor-core work here: the path is bound by HBM):
//   * a token row is read once with 128-bit nontemporal loads and stays in registers (packed,
//     as loaded) for every use: partial mean, centred sum of squares, output; fp32 values are
//     rebuilt from the packed registers per pass (one shift or mask each), which keeps the
//     register count low enough for a second, prefetched copy of the next rows;
//   * K waves share a row: wave w, lane l owns the 16-byte chunks (i*K + w)*64 + l for the whole
//     life of its block, so everything that is per feature -- (1+scale), shift, and in the
//     backward the running dshift/dscale sums -- lives in that lane's registers;
//   * row reductions use DPP adds inside a wave (no LDS, no ds_bpermute) and v_readlane for the
//     four 16-lane rows; the K waves of a row exchange two floats each through LDS with one
//     barrier per step (double-buffered);
//   * the backward carries fp32 partial sums of dshift/dscale in registers down its rows (the
//     paper's D-tile idea of "thread fixed to a feature, accumulate along the sequence",
//     Sec. 3.3, done inside the dx kernel so dy and x are not read a second time); every block
//     writes one partial slot per segment it touches and a second kernel adds the slots in a
//     fixed order: no float atomics, bitwise reproducible;
//   * HBM on this part rewards few, deep, sequential streams: 4 to 6 waves per CU, each with its
//     next step's loads already in flight (software pipeline), and blocks grouped in clusters
//     that walk one contiguous region with consecutive rows, reach about 6 TB/s where one
//     private range per block and 16+ waves per CU reach 4.9 TB/s;
//   * blocks walk the segment table themselves, so fixed-length and packed varlen batches share
//     the code.
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

// Waves per SIMD the compiler must leave room for (512 VGPRs per SIMD lane).  Without a bound the
// scheduler spends registers on hoisted loads until a single wave fills the SIMD.
// Kernels in which K waves share a row and a lane keeps per-feature state in registers.
constexpr int bwd_waves_per_eu(int vpl, int elems_per_chunk, int rows) {
    // live per lane and chunk: 1+scale and two accumulators (fp32), `rows` packed copies of dy
    // and x with their addresses; plus unpack temporaries and loop state
    const int regs = vpl * (3 * elems_per_chunk + 10 * rows) + 28;
    const int w = 512 / regs;
    return w > LNMOD_MAX_WAVES_PER_EU ? LNMOD_MAX_WAVES_PER_EU : w < 1 ? 1 : w;
}
// The backward that recomputes the statistics keeps four more sums, a centre and the merge's
// temporaries live: with three chunks per lane it spills at three waves per SIMD, and its launch
// shapes of that width never put more than two there.
constexpr int bwd_seg_waves_per_eu(int vpl, int elems_per_chunk, int rows, bool recompute) {
    const int w = bwd_waves_per_eu(vpl, elems_per_chunk, rows);
    return recompute && vpl * elems_per_chunk >= 24 && w > 2 ? 2 : w;
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

// Sum over lanes 0..15 only (one DPP row), returned to every lane.
__device__ inline float row0_sum(float v) {
    v = dpp_add<0xB1>(v);
    v = dpp_add<0x4E>(v);
    v = dpp_add<0x141>(v);
    v = dpp_add<0x140>(v);
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 0));
}

// ---- segment table: fixed-length samples (cu == nullptr) or packed offsets on the device ----
struct Segments {
    const int32_t* cu;   // [nseg+1] token offsets, or nullptr for nseg samples of S tokens
    int64_t S;
    int64_t nseg;
};

// One entry of the segment table.  The table is an input that no kernel writes, so it is read
// through the constant address space: with a wave-uniform index that is a scalar load, which waits
// on the scalar counter alone, where a vector load would first wait for every store the wave still
// has in flight from the segment it has just finished (64 segments of 2048 rows at D = 1536:
// forward 157.5 -> 152.7 us, backward 225 -> 218.5).
typedef const int32_t __attribute__((address_space(4))) * const_i32_ptr;
__device__ inline int32_t table_at(const int32_t* cu, int64_t m) { return ((const_i32_ptr)cu)[m]; }

__device__ inline int64_t seg_begin(const Segments& s, int64_t m) {
    return s.cu ? static_cast<int64_t>(table_at(s.cu, m)) : m * s.S;
}

// Largest m in [0, nseg-1] whose first token is <= row (skips empty segments in front of row).
// Terminates and stays in range for any table contents.
__device__ inline int64_t find_segment(const Segments& s, int64_t row) {
    if (!s.cu) return row / s.S;
    int64_t lo = 0, hi = s.nseg - 1;
    while (lo < hi) {
        const int64_t mid = (lo + hi + 1) >> 1;
        if (static_cast<int64_t>(table_at(s.cu, mid)) <= row) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// =============================================================================================
// Forward arguments (all forward kernels)
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
    int32_t interleave;      // 1: cluster = block index modulo the cluster count (measurement only)
    int32_t D;
    int32_t nchunks;         // D / E
    float eps;
    float inv_D;
};

// Steps of R rows are handed to a cluster's blocks in turn across segment boundaries: a segment's
// first step goes to the block after the one that took the previous segment's last step.
// Starting every segment at block 0 would give the low-numbered blocks one step more in almost
// every segment (24 segments: up to 24 steps of about 300; the backward of 24 mixed segments at
// D = 5120 took 826 us that way and takes 805 with turns).  `turn` is the number of steps handed
// out in the region so far, modulo nb; the call returns the block's first row in [r0, stop) and
// adds the segment's steps.
template <int R>
__device__ __forceinline__ int64_t take_turn(uint32_t& turn, int64_t r0, int64_t stop, int64_t member, int32_t nb) {
    const uint32_t nbu = static_cast<uint32_t>(nb), mine = static_cast<uint32_t>(member);
    const int64_t first = r0 + static_cast<int64_t>(mine >= turn ? mine - turn : mine + nbu - turn) * R;
    turn = static_cast<uint32_t>((turn + static_cast<uint64_t>((stop - r0 + R - 1) / R) % nbu) % nbu);
    return first;
}

// =============================================================================================
// Forward.  K waves share a row: wave w, lane l owns chunks (i*K + w)*64 + l for the whole life
// of the block, so with one modulation row per sample / segment the (1+scale, shift) values of
// those features stay in registers and nothing of the modulation goes through LDS.  Each wave
// forms the mean and the centred sum of squares of its own part of the row (two passes over
// registers); the K partial results are merged with the exact pairwise-update formula
//   M2 = sum_k M2_k + sum_k n_k (mean_k - mean)^2,
// which keeps the two-pass accuracy, through a few LDS floats and one barrier per step.
//
// MODE selects what surrounds the normalisation:
//   kModSegment   y = xhat*(1+scale[m]) + shift[m], one modulation row per sample / segment
//   kModToken     y = xhat*(1+scale[n]) + shift[n], modulation rows streamed with x
//   kLnOnly       y = xhat                      (first kernel of the unfused comparator)
//   kModOnly      y = x*(1+scale[m]) + shift[m], no statistics (second kernel of the comparator)
//   kModFlat      kModSegment's result for batches of several segments, with one loop over the rows
//                 of the block's region instead of one loop per segment: a block's rows are
//                 member*R + k*nb*R whatever segment they fall in, and when a row lies beyond the
//                 segment whose modulation row the registers hold, the registers are reloaded on
//                 the spot.  The software pipeline never drains at a segment boundary (the next
//                 step's rows are already requested when the reload waits) and no step is left
//                 partly empty at a segment's end.
// =============================================================================================
constexpr int kModSegment = 0, kModToken = 1, kLnOnly = 2, kModOnly = 3, kModFlat = 4;

template <typename Tag, int VPL, int K, int R, bool EXACT, int MODE = kModSegment, bool PF = true>
__global__ __launch_bounds__(K* kWave)
LNMOD_OCCUPANCY(bwd_waves_per_eu(VPL, IO<Tag>::E, (MODE == kModToken ? 3 : 1) * (PF ? 2 * R : R)))
void fwd_split_kernel(const FwdArgs a) {
    using io = IO<Tag>;
    constexpr int E = io::E;
    constexpr bool kFlat = MODE == kModFlat;
    constexpr bool kSegMod = MODE == kModSegment || MODE == kModOnly || kFlat;   // A, B per segment in registers
    constexpr bool kTok = MODE == kModToken;
    constexpr bool kStats = MODE != kModOnly;
    constexpr int NS = kTok ? 3 : 1;                                     // streamed inputs per row
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
    // features each wave holds (all lanes compute the same K numbers)
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

    int64_t cluster = blockIdx.x / a.nb;
    int64_t member = blockIdx.x - cluster * a.nb;
    if (a.interleave) {
        const int64_t nclusters = gridDim.x / a.nb;
        member = blockIdx.x / nclusters;
        cluster = blockIdx.x - member * nclusters;
    }
    int64_t r0 = cluster * a.rows_per_cluster;
    int64_t r1 = r0 + a.rows_per_cluster;
    if (r1 > a.T) r1 = a.T;
    int buf = 0;
    uint32_t turn = 0;                       // see take_turn

    while (r0 < r1) {
        int64_t m = 0, stop = r1;
        if (kSegMod && !kFlat) {
            m = find_segment(a.seg, r0);
            stop = seg_begin(a.seg, m + 1);
            if (stop > r1) stop = r1;
            if (stop <= r0) stop = r0 + 1;      // malformed table: still make progress
        }
        // kFlat: the segment of the block's first row; seg_end is where the rows of m end
        int64_t seg_end = 0;
        if (kFlat) {
            int64_t first_row = r0 + member * R;
            if (first_row >= r1) first_row = r1 - 1;
            m = find_segment(a.seg, first_row);
            seg_end = m + 1 < a.seg.nseg ? seg_begin(a.seg, m + 1) : a.T;
        }

        float A[VPL][E], B[VPL][E];
        auto load_modulation = [&](int64_t mm) {
#pragma unroll
            for (int i = 0; i < VPL; ++i) {
                u32x4 rsc = u32x4{0u, 0u, 0u, 0u}, rsh = u32x4{0u, 0u, 0u, 0u};
                if (ok[i]) {
                    rsc = load16_cached(a.scale, uniform64(mm * row_bytes), static_cast<uint32_t>(chunk[i]) * 16u);
                    rsh = load16_cached(a.shift, uniform64(mm * row_bytes), static_cast<uint32_t>(chunk[i]) * 16u);
                }
                io::unpack(rsc, A[i]);
                io::unpack(rsh, B[i]);
#pragma unroll
                for (int e = 0; e < E; ++e) A[i][e] += 1.0f;
            }
        };
        if (kSegMod) load_modulation(m);

        // Software pipeline: the rows of the block's next step are requested before the current
        // step is computed, so a few waves per CU keep the memory system busy.
        // q[s][j][i]: s = 0 x, 1 scale, 2 shift (the last two only with per-token modulation)
        auto fetch = [&](int64_t base, u32x4 (&q)[NS][R][VPL]) {
#pragma unroll
            for (int j = 0; j < R; ++j) {
                const int64_t row = base + j;
#pragma unroll
                for (int i = 0; i < VPL; ++i) {
                    const uint32_t lo = static_cast<uint32_t>(chunk[i]) * 16u;
                    if (row < stop && ok[i]) {
                        q[0][j][i] = load16_u(a.x, row * row_bytes, lo);
                        if (kTok) {
                            q[NS - 2][j][i] = load16_u(a.scale, row * row_bytes, lo);
                            q[NS - 1][j][i] = load16_u(a.shift, row * row_bytes, lo);
                        }
                    } else {
#pragma unroll
                        for (int t = 0; t < NS; ++t) q[t][j][i] = u32x4{0u, 0u, 0u, 0u};
                    }
                }
            }
        };
        const int64_t step = static_cast<int64_t>(a.nb) * R;
        u32x4 raw[NS][R][VPL];
        const int64_t first = take_turn<R>(turn, r0, stop, member, a.nb);
        if (PF) fetch(first, raw);

        for (int64_t base = first; base < stop; base += step) {
            u32x4 nxt[NS][R][VPL];
            if (PF) {
                fetch(base + step, nxt);
                __builtin_amdgcn_sched_barrier(0);           // keep the requests up here
            } else {
                fetch(base, raw);
            }
            float mu[R], rs[R];
            if (kStats) {
                // this wave's part of each row: mean, then centred sum of squares
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
                // make the packed registers opaque, so that the fp32 values are rebuilt below
                // instead of being carried across the barrier in registers
#pragma unroll
                for (int j = 0; j < R; ++j) {
#pragma unroll
                    for (int i = 0; i < VPL; ++i) asm volatile("" : "+v"(raw[0][j][i]));
                }
            } else {
#pragma unroll
                for (int j = 0; j < R; ++j) {
                    mu[j] = 0.0f;
                    rs[j] = 1.0f;
                }
            }
#pragma unroll
            for (int j = 0; j < R; ++j) {
                const int64_t row = base + j;
                if (row < stop) {
                    if (kFlat && row >= seg_end) {
                        // the row belongs to a later segment (empty ones in between are skipped); the
                        // walk stays inside the table whatever the table holds
                        while (m + 1 < a.seg.nseg && seg_begin(a.seg, m + 1) <= row) ++m;
                        seg_end = m + 1 < a.seg.nseg ? seg_begin(a.seg, m + 1) : a.T;
                        if (seg_end <= row) seg_end = row + 1;      // malformed table: still make progress
                        load_modulation(m);
                    }
                    if (kStats && wave == 0 && lane == 0 && a.mean != nullptr) {
                        a.mean[row] = mu[j];
                        a.rstd[row] = rs[j];
                    }
#pragma unroll
                    for (int i = 0; i < VPL; ++i) {
                        if (ok[i]) {
                            float v[E], o[E];
                            io::unpack(raw[0][j][i], v);
                            if (kTok) {
                                float sc[E], sh[E];
                                io::unpack(raw[NS - 2][j][i], sc);
                                io::unpack(raw[NS - 1][j][i], sh);
#pragma unroll
                                for (int e = 0; e < E; ++e) o[e] = ((v[e] - mu[j]) * rs[j]) * (1.0f + sc[e]) + sh[e];
                            } else if (MODE == kLnOnly) {
#pragma unroll
                                for (int e = 0; e < E; ++e) o[e] = (v[e] - mu[j]) * rs[j];
                            } else if (MODE == kModOnly) {
#pragma unroll
                                for (int e = 0; e < E; ++e) o[e] = v[e] * A[i][e] + B[i][e];
                            } else {
#pragma unroll
                                for (int e = 0; e < E; ++e) o[e] = ((v[e] - mu[j]) * rs[j]) * A[i][e] + B[i][e];
                            }
                            store16_u(a.y, row * row_bytes, static_cast<uint32_t>(chunk[i]) * 16u, io::pack(o));
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
            if (PF) {
#pragma unroll
                for (int t = 0; t < NS; ++t) {
#pragma unroll
                    for (int j = 0; j < R; ++j) {
#pragma unroll
                        for (int i = 0; i < VPL; ++i) raw[t][j][i] = nxt[t][j][i];
                    }
                }
            }
        }
        r0 = stop;
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
    int32_t interleave;      // 1: cluster = block index modulo the cluster count (measurement only)
    int32_t D;
    int32_t nchunks;
    float inv_D;
    float eps;               // only read when the statistics are recomputed (RC)
};

// RC: mean and rstd are not read but formed again from x, for callers that keep only x between
// the passes (Sec. 3.3: only the operator's output has to be stored).  The variance is two-pass
// per wave, as in the forward: every wave first takes the mean c of its own part of the row, then
// sums x-c (the rounding residue of c), (x-c)^2, g and g*(x-c) in one pass over the registers.
// With one barrier the K waves' numbers are moved to one common centre c0 (wave 0's mean) and
// added (S1, S2, G1, G2; lane k of every wave takes wave k's), which gives
//   mean = c0 + S1/D,   sum (x-mean)^2 = S2 - S1^2/D,   sum g (x-mean) = G2 - (S1/D) G1.
// n_0 (c0 - mean)^2 <= D var, so the subtraction in the middle loses at most a factor K of fp32
// precision whatever the row holds (a centre taken from a few sampled elements has no such
// bound: outliers at the sampled positions would put it far from the mean).  The dshift/dscale
// sums are taken in the second pass, where xhat is rebuilt anyway.
template <typename Tag, int VPL, int K, int R, bool EXACT, bool TOK = false, bool PF = true, bool RC = false>
__global__ __launch_bounds__(K* kWave)
LNMOD_OCCUPANCY(bwd_seg_waves_per_eu(VPL, IO<Tag>::E, (TOK ? 3 : 2) * (PF ? 2 * R : R) / 2, RC))
void bwd_seg_kernel(const BwdArgs a) {
    using io = IO<Tag>;
    constexpr int E = io::E;
    constexpr int NS = TOK ? 3 : 2;            // streamed inputs per row: dy, x (, scale)
    __shared__ float part[2][R][K][2];
    __shared__ float stat[RC ? 2 : 1][R][K][RC ? 5 : 1];

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
    // RC: lane k < K merges wave k's sums and needs the number of features wave k holds; every
    // wave needs one over the number of features it holds itself
    float lane_cnt = 0.0f, inv_own = 0.0f;
    if (RC) {
        static_assert(K <= 16, "the merge runs on one DPP row");
        int n = 0, own = 0;
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            int left = a.nchunks - (i * K + lane) * kWave;
            left = left < 0 ? 0 : left > kWave ? kWave : left;
            n += left;
            int mine = a.nchunks - (i * K + wave) * kWave;
            mine = mine < 0 ? 0 : mine > kWave ? kWave : mine;
            own += mine;
        }
        lane_cnt = lane < K ? static_cast<float>(n * E) : 0.0f;
        inv_own = own > 0 ? 1.0f / static_cast<float>(own * E) : 0.0f;
    }

    int64_t cluster = blockIdx.x / a.nb;
    int64_t member = blockIdx.x - cluster * a.nb;
    if (a.interleave) {
        const int64_t nclusters = gridDim.x / a.nb;
        member = blockIdx.x / nclusters;
        cluster = blockIdx.x - member * nclusters;
    }
    int64_t r0 = cluster * a.rows_per_cluster;
    int64_t r1 = r0 + a.rows_per_cluster;
    if (r1 > a.T) r1 = a.T;
    int buf = 0;
    uint32_t turn = 0;                       // see take_turn

    while (r0 < r1) {
        int64_t m = 0, stop = r1;
        if (!TOK) {
            m = find_segment(a.seg, r0);
            stop = seg_begin(a.seg, m + 1);
            if (stop > r1) stop = r1;
            if (stop <= r0) stop = r0 + 1;      // malformed table: still make progress
        }

        // per segment: 1 + scale of this lane's features and the running dshift/dscale sums
        float A[VPL][E], acc_s[VPL][E], acc_c[VPL][E];
        if (!TOK) {
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
        }

        // Software pipeline: the packed rows of the block's next step are requested before the
        // current step is computed, so every block keeps loads in flight while it does
        // arithmetic, waits at its barrier and stores.  q[s][j][i]: s = 0 dy, 1 x, 2 scale.
        auto fetch = [&](int64_t base, u32x4 (&q)[NS][R][VPL], float (&qmu)[R], float (&qrs)[R]) {
#pragma unroll
            for (int j = 0; j < R; ++j) {
                const int64_t row = base + j;
                const bool live = row < stop;
                qmu[j] = !RC && live ? a.mean[row] : 0.0f;
                qrs[j] = !RC && live ? a.rstd[row] : 0.0f;
#pragma unroll
                for (int i = 0; i < VPL; ++i) {
                    if (live && ok[i]) {
                        const uint32_t lo = static_cast<uint32_t>(chunk[i]) * 16u;
                        q[0][j][i] = load16_u(a.dy, row * row_bytes, lo);
                        q[1][j][i] = load16_u(a.x, row * row_bytes, lo);
                        if (TOK) q[NS - 1][j][i] = load16_u(a.scale, row * row_bytes, lo);
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
        if (PF) fetch(first, raw, mu, rs);                   // rows at or beyond `stop` read as zeros

        for (int64_t base = first; base < stop; base += step) {
            u32x4 nxt[NS][R][VPL];
            float nmu[R], nrs[R];
            if (PF) {
                fetch(base + step, nxt, nmu, nrs);
                __builtin_amdgcn_sched_barrier(0);           // keep the requests up here
            } else {
                fetch(base, raw, mu, rs);
            }
            // pass 1 over the registers: row sums for dx and the running dshift/dscale sums.
            // xhat and g are not kept: they are rebuilt from the packed registers in pass 2,
            // which costs a few ALU operations and saves the registers the prefetch needs.
            float c1[R], c2[R];
            if constexpr (RC) {
                // this wave's part of each row: its mean (the centre), then the four centred sums
                float piv[R], s1[R], s2[R];
#pragma unroll
                for (int j = 0; j < R; ++j) {
                    {
                        float s = 0.0f;
#pragma unroll
                        for (int i = 0; i < VPL; ++i) {
                            float v[E];
                            io::unpack(raw[1][j][i], v);               // dead chunks hold zeros
#pragma unroll
                            for (int e = 0; e < E; ++e) s += v[e];
                        }
                        piv[j] = wave_sum(s) * inv_own;
                    }
                    float t1 = 0.0f, t2 = 0.0f, p1 = 0.0f, p2 = 0.0f;
#pragma unroll
                    for (int i = 0; i < VPL; ++i) {
                        float dyv[E], xv[E], scv[E];
                        io::unpack(raw[0][j][i], dyv);
                        io::unpack(raw[1][j][i], xv);
                        if (TOK) io::unpack(raw[NS - 1][j][i], scv);
#pragma unroll
                        for (int e = 0; e < E; ++e) {
                            const float xp = xv[e] - piv[j];
                            const float gg = dyv[e] * (TOK ? 1.0f + scv[e] : A[i][e]);
                            p1 += gg;
                            p2 += gg * xp;              // dead chunks: dy = 0, so gg = 0
                            if (ok[i]) {
                                t1 += xp;
                                t2 += xp * xp;
                            }
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    s1[j] = wave_sum(t1);
                    s2[j] = wave_sum(t2);
                    c1[j] = wave_sum(p1);
                    c2[j] = wave_sum(p2);
                }
                if (K > 1) {
                    if (lane == 0) {
#pragma unroll
                        for (int j = 0; j < R; ++j) {
                            stat[buf][j][wave][0] = piv[j];
                            stat[buf][j][wave][1] = s1[j];
                            stat[buf][j][wave][2] = s2[j];
                            stat[buf][j][wave][3] = c1[j];
                            stat[buf][j][wave][4] = c2[j];
                        }
                    }
                    __syncthreads();
                }
#pragma unroll
                for (int j = 0; j < R; ++j) {
                    // lane k < K moves wave k's sums to the first wave's centre c0 (e = c_k - c0);
                    // adding them over the lanes gives
                    //   S1 = sum (x-c0), S2 = sum (x-c0)^2, G1 = sum g, G2 = sum g (x-c0)
                    float c0 = piv[j], S1 = s1[j], S2 = s2[j], G1 = c1[j], G2 = c2[j];
                    if (K > 1) {
                        c0 = stat[buf][j][0][0];
                        float e = 0.0f, a1 = 0.0f, a2 = 0.0f, b1 = 0.0f, b2 = 0.0f;
                        if (lane < K) {
                            e = stat[buf][j][lane][0] - c0;
                            a1 = stat[buf][j][lane][1];
                            a2 = stat[buf][j][lane][2];
                            b1 = stat[buf][j][lane][3];
                            b2 = stat[buf][j][lane][4];
                        }
                        S1 = row0_sum(a1 + lane_cnt * e);
                        S2 = row0_sum(a2 + e * (2.0f * a1 + lane_cnt * e));
                        G1 = row0_sum(b1);
                        G2 = row0_sum(b2 + e * b1);
                    }
                    const float dm = S1 / static_cast<float>(a.D);       // mean - c0
                    float m2 = S2 - dm * S1;
                    m2 = m2 > 0.0f ? m2 : 0.0f;
                    mu[j] = c0 + dm;
                    rs[j] = 1.0f / sqrtf(m2 * a.inv_D + a.eps);
                    c1[j] = G1;
                    c2[j] = (G2 - dm * G1) * rs[j];
                }
                if (K > 1) buf ^= 1;
            } else {
    #pragma unroll
                for (int j = 0; j < R; ++j) {
                    float p1 = 0.0f, p2 = 0.0f;
    #pragma unroll
                    for (int i = 0; i < VPL; ++i) {
                        float dyv[E], xv[E], scv[E];
                        io::unpack(raw[0][j][i], dyv);
                        io::unpack(raw[1][j][i], xv);
                        if (TOK) io::unpack(raw[NS - 1][j][i], scv);
    #pragma unroll
                        for (int e = 0; e < E; ++e) {
                            // xhat as (x - mean) * rstd, not x*rstd - mean*rstd: the latter loses every digit
                            // on (near-)constant rows, where rstd is as large as 1/sqrt(eps)
                            const float h = (xv[e] - mu[j]) * rs[j];
                            const float gg = dyv[e] * (TOK ? 1.0f + scv[e] : A[i][e]);
                            p1 += gg;
                            p2 += gg * h;
                            if (!TOK) {
                                acc_s[i][e] += dyv[e];
                                acc_c[i][e] += dyv[e] * h;
                            }
                        }
                        if (!TOK) {
                            // Pin the running sums here.  They are only consumed at the end of the loop,
                            // so the optimiser would otherwise sink these adds below the barrier and keep
                            // every unpacked dy and xhat alive until then (twice the row in registers).
    #pragma unroll
                            for (int e = 0; e < E; ++e) asm volatile("" : "+v"(acc_s[i][e]), "+v"(acc_c[i][e]));
                        }
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
            }
            // pass 2: dx = rstd * (g - c1 - xhat*c2).  The empty asm makes the packed registers
            // opaque so that common-subexpression elimination cannot carry pass 1's fp32 values
            // across the barrier instead of rebuilding them.
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
                            float dyv[E], xv[E], scv[E], o[E], ds[E];
                            io::unpack(raw[0][j][i], dyv);
                            io::unpack(raw[1][j][i], xv);
                            if (TOK) io::unpack(raw[NS - 1][j][i], scv);
#pragma unroll
                            for (int e = 0; e < E; ++e) {
                                const float h = (xv[e] - mu[j]) * rs[j];
                                o[e] = (dyv[e] * (TOK ? 1.0f + scv[e] : A[i][e])) * rs[j] - k1 - h * k2;
                                if (TOK) ds[e] = dyv[e] * h;
                                if (RC && !TOK) {
                                    acc_s[i][e] += dyv[e];
                                    acc_c[i][e] += dyv[e] * h;
                                }
                            }
                            const uint32_t lo = static_cast<uint32_t>(chunk[i]) * 16u;
                            store16_u(a.dx, row * row_bytes, lo, io::pack(o));
                            if (TOK) {
                                // per token: dshift = dy (the packed registers as loaded), dscale = dy * xhat
                                store16_u(a.dshift, row * row_bytes, lo, raw[0][j][i]);
                                store16_u(a.dscale, row * row_bytes, lo, io::pack(ds));
                            }
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
                    for (int t = 0; t < NS; ++t) {
#pragma unroll
                        for (int i = 0; i < VPL; ++i) raw[t][j][i] = nxt[t][j][i];
                    }
                }
            }
        }

        if (!TOK) {
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
        }
        r0 = stop;
    }
}

// Second pass: out[k][m, d] = sum of the partial slots of segment m, k < nsum (dshift, dscale
// and, for the gated operator, dgate).  A block takes 64 * V consecutive features of one sum of
// one segment; its W = blockDim.x / 64 waves split the slots in ascending order (wave w takes
// slots w, w + W, ...), and the W wave sums are then added in wave order.  V and W are chosen
// from the shapes alone, so results repeat bit for bit.
struct ReduceArgs {
    const float* ws;         // [nslots][nsum][D]
    float* out[3];           // [nseg, D] each
    Segments seg;
    int64_t T;
    int64_t rows_per_cluster;
    int32_t nb;              // blocks per cluster = partial slots per (cluster, segment)
    int32_t D;
    int32_t dblocks;         // ceil(D / (64 * V))
    int32_t nsum;            // 2 or 3
    int64_t total;           // nseg * nsum * dblocks: (segment, sum, feature block) triples
};

constexpr int kReduceWaves = 16;     // most waves a reduce block may have
constexpr int kReduceFloats = 16;    // floats per lane a wave keeps in flight: 16 / V slot loads

template <int V> struct FVec { typedef float type __attribute__((ext_vector_type(V))); };
template <> struct FVec<1> { typedef float type; };

// Block b takes the triples b, b + gridDim.x, ... below a.total, each decoded as (segment, which
// sum, block of 64 * V features); the grid is min(total, a bound), so that any segment count the
// interface admits stays inside the launch limits.
template <int V, int G = 1>
__global__ __launch_bounds__(kReduceWaves* kWave) void bwd_reduce_kernel(const ReduceArgs a) {
    using vec = typename FVec<V>::type;
    constexpr int kReduceBatch = kReduceFloats / V;
    constexpr int FL = kWave / G;                 // lanes along the features; G groups of them take different slots
    __shared__ vec red[kReduceWaves][FL];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int W = blockDim.x >> 6;
    const int fl = lane % FL, grp = lane / FL;
    for (int64_t bid = blockIdx.x; bid < a.total; bid += gridDim.x) {
        const int d = (static_cast<int>(bid % a.dblocks) * FL + fl) * V;
        const int which = static_cast<int>((bid / a.dblocks) % a.nsum);
        const int64_t m = bid / (static_cast<int64_t>(a.nsum) * a.dblocks);
        int64_t n0 = seg_begin(a.seg, m), n1 = seg_begin(a.seg, m + 1);
        if (n0 < 0) n0 = 0;                       // a malformed table must not lead outside ws
        if (n1 > a.T) n1 = a.T;
        vec acc = vec(0.0f);
        if (n1 > n0 && d < a.D) {
            // clusters c_lo..c_hi touch this segment; (cluster c, segment m) owns slots (c+m)*nb ..
            const int64_t c_lo = n0 / a.rows_per_cluster, c_hi = (n1 - 1) / a.rows_per_cluster;
            const int64_t s_lo = (c_lo + m) * a.nb, s_hi = (c_hi + m + 1) * a.nb;
            const float* base = a.ws + static_cast<int64_t>(which) * a.D + d;
            const int64_t pitch = static_cast<int64_t>(a.nsum) * a.D;
            const int64_t stride = static_cast<int64_t>(W) * G;
            // kReduceBatch slots requested before the first is added (the chain of dependent round
            // trips, not the bytes, is what this kernel's time consists of); the additions keep slot order
            for (int64_t sl = s_lo + wave * G + grp; sl < s_hi; sl += kReduceBatch * stride) {
                vec v[kReduceBatch];
#pragma unroll
                for (int u = 0; u < kReduceBatch; ++u) {
                    const int64_t su = sl + static_cast<int64_t>(u) * stride;
                    v[u] = su < s_hi ? *reinterpret_cast<const vec*>(base + su * pitch) : vec(0.0f);
                }
#pragma unroll
                for (int u = 0; u < kReduceBatch; ++u) acc += v[u];
            }
        }
        if constexpr (G > 1) {
            // the G groups of the wave, in a fixed order
#pragma unroll
            for (int off = FL; off < kWave; off <<= 1) {
                if constexpr (V == 1) {
                    acc += __shfl_xor(acc, off);
                } else {
#pragma unroll
                    for (int e = 0; e < V; ++e) acc[e] += __shfl_xor(acc[e], off);
                }
            }
        }
        if (W > 1) {
            if (grp == 0) red[wave][fl] = acc;
            __syncthreads();
            if (wave == 0 && grp == 0) {
                acc = red[0][fl];
                for (int w = 1; w < W; ++w) acc += red[w][fl];
            }
            __syncthreads();                      // red is written again in the next round
        }
        if (wave == 0 && grp == 0 && d < a.D)
            *reinterpret_cast<vec*>(a.out[which] + m * a.D + d) = acc;
    }
}

// =============================================================================================
// Bandwidth reference (not part of the fused path)
// =============================================================================================
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

// The copy's pattern with NR read streams and NW write streams, to split the copy figure into what
// the memory system gives to reads, to writes and to the mixtures the row kernels produce.  Every
// output j is the 32-bit-lane sum of the inputs plus j (a position-dependent pattern without
// inputs); without outputs the sum is stored only if it equals a value it cannot take for the fill
// patterns used, which keeps the loads alive.  V vectors per lane and step; the block's waves take
// consecutive pieces.
struct ProbeArgs {
    const u32x4* in[4];
    u32x4* out[3];
    int64_t nvec;
};

template <int NR, int NW, int V>
__global__ __launch_bounds__(8 * kWave) void stream_probe_kernel(const ProbeArgs a) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int W = blockDim.x >> 6;
    constexpr int64_t kPiece = static_cast<int64_t>(V) * kWave;
    constexpr int NQ = NR > 0 ? NR : 1;
    const int64_t pieces = a.nvec / kPiece;               // a tail shorter than one piece is left out
    const int64_t step = static_cast<int64_t>(gridDim.x) * W;
    auto fetch = [&](int64_t piece, u32x4 (&q)[NQ][V]) {
#pragma unroll
        for (int r = 0; r < NQ; ++r) {
#pragma unroll
            for (int i = 0; i < V; ++i) {
                q[r][i] = u32x4{0u, 0u, 0u, 0u};
                if (r < NR && piece < pieces) q[r][i] = __builtin_nontemporal_load(a.in[r] + piece * kPiece + i * kWave + lane);
            }
        }
    };
    int64_t piece = static_cast<int64_t>(blockIdx.x) * W + wave;
    u32x4 cur[NQ][V], acc = u32x4{0u, 0u, 0u, 0u};
    fetch(piece, cur);
    for (; piece < pieces; piece += step) {
        u32x4 nxt[NQ][V];
        fetch(piece + step, nxt);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < V; ++i) {
            u32x4 v = NR > 0 ? cur[0][i] : u32x4{1u, 2u, static_cast<uint32_t>(i), static_cast<uint32_t>(piece)};
#pragma unroll
            for (int r = 1; r < NR; ++r) v += cur[r][i];
            if (NW == 0) acc += v;
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                const u32x4 o = v + u32x4{static_cast<uint32_t>(w), 0u, 0u, 0u};
                __builtin_nontemporal_store(o, a.out[w] + piece * kPiece + i * kWave + lane);
            }
        }
#pragma unroll
        for (int r = 0; r < NQ; ++r) {
#pragma unroll
            for (int i = 0; i < V; ++i) cur[r][i] = nxt[r][i];
        }
    }
    if (NW == 0 && acc.x == 0x9e3779b9u && acc.y == 0x7f4a7c15u) a.out[0][lane] = acc;
}

}  // namespace lnmod
