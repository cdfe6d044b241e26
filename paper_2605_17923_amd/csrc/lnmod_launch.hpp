// lnmod_launch.hpp -- host-side launch interface between the C ABI (lnmod_api.cpp) and the
// translation units that instantiate the gfx950 kernels.  Plain data in, hipError_t out.
#pragma once
#include <hip/hip_runtime_api.h>
#include <stddef.h>
#include <stdint.h>

namespace lnmod {

constexpr int kNumCU = 256;            // MI355X: 8 XCDs x 32 CUs
constexpr int64_t kMaxD = 8192;

// Launch shape of a row kernel: K waves per row, VPL 16-byte chunks per lane, R rows per block and
// step, per_cu resident blocks per compute unit that the grid is sized for.
struct Shape {
    int K;
    int VPL;
    int R;
    int per_cu;
    // Only ever set by a shaped call of the measurement library (the tables leave them 0):
    int clusters = 0;      // > 0: this many clusters of blocks instead of the plan's choice
    int interleave = 0;    // 1: cluster = block index modulo the cluster count (with 8 clusters every
                           // cluster then sits on one XCD, because consecutive blocks go to the XCDs in
                           // turn); 0: consecutive blocks form a cluster (every cluster on all XCDs)
    int flat = 0;          // per-sample forward: 1 one loop over all rows of a block's region (modulation
                           // registers reloaded where the segment changes), 2 one loop per segment,
                           // 0 the launcher's choice
};

struct Problem {
    int dtype;                 // LNMOD_BF16 / LNMOD_F32
    const int32_t* cu;         // device segment offsets or nullptr (fixed length)
    int64_t nseg;              // samples or segments
    int64_t S;                 // tokens per sample when cu == nullptr
    int64_t T;                 // total tokens
    int64_t D;
    float eps;
    // Launch shape to use instead of the measured table's entry, or nullptr.  The operator entry
    // points always pass nullptr; the measurement library's shaped calls pass the caller's shape,
    // per call, so that a sweep can time candidates without any process-wide state.
    const Shape* force = nullptr;
};

// How the token rows are spread over the grid.  `clusters` groups of `nb` blocks each own one
// contiguous region of `rows_per_cluster` rows; inside its region a cluster's blocks take
// consecutive rows, so the cluster streams through one moving window of memory (HBM rewards
// few concurrent sequential streams far more than one private stream per block).  nb shrinks
// when there are many segments, because every (cluster, segment) pair costs nb reloads of the
// modulation rows (forward) or nb partial-sum slots (backward).
struct RowPlan {
    int64_t blocks;            // clusters * nb
    int64_t clusters;
    int64_t rows_per_cluster;
    int32_t nb;
};

// Clusters a forward launch with one loop per segment should use when the batch has several
// segments.  Every block restarts its software pipeline once per segment of its cluster's region
// (about 2.2 us: the modulation rows, then the first rows, arrive with nothing else in flight), so
// more clusters mean fewer segments per block, but concurrent windows cost bandwidth.  The count
// that minimises
//     stream_us * penalty(C) + (nseg / C + 1) * 2.2 us,   penalty = 1, 1.01, 1.03, 1.06, 1.10
// over C = 2, 4, 8, 16, 32 is taken, a larger C only if it wins by 2 %.  A batch of several segments
// never gets a single cluster: all its blocks would reach every boundary at the same moment and
// the whole chip would drain (fp32, D = 5120, 8 equal segments: 566 us with one cluster, 541 with
// two, 535 with four).  Measured with 2 ... 32 clusters on 24 mixed, 8, 96 and 480 equal segments
// at D = 512 ... 2048 bf16 and D = 1536, 5120 fp32: the choice is within 3 % of the best count
// except on 96 segments at D = 2048 (231 us against 221 with eight clusters).
inline int64_t pick_clusters(double stream_us, int64_t nseg) {
    if (nseg <= 1) return 1;
    const int c[] = {2, 4, 8, 16, 32};
    const double penalty[] = {1.0, 1.01, 1.03, 1.06, 1.10};
    int64_t best = 2;
    double best_t = 0.0;
    for (int i = 0; i < 5 && (i == 0 || c[i] <= nseg); ++i) {
        const double t = stream_us * penalty[i] + (static_cast<double>(nseg) / c[i] + 1.0) * 2.2;
        if (i == 0 || t < best_t * 0.98) {
            best = c[i];
            best_t = t;
        }
    }
    return best;
}

// Blocks of a launch: one per rows_per_step rows, at most max_blocks (the resident blocks wanted).
inline int64_t grid_blocks(int64_t T, int64_t max_blocks, int rows_per_step) {
    int64_t g = (T + rows_per_step - 1) / rows_per_step;
    if (g > max_blocks) g = max_blocks;
    return g < 1 ? 1 : g;
}

// g blocks in clusters of nb.
inline RowPlan make_plan(int64_t T, int64_t g, int64_t nb) {
    RowPlan p{0, 0, 1, 1};
    if (T <= 0) return p;
    int64_t clusters = (g + nb - 1) / nb;
    const int64_t rpc = (T + clusters - 1) / clusters;
    clusters = (T + rpc - 1) / rpc;
    p.blocks = clusters * nb;
    p.clusters = clusters;
    p.rows_per_cluster = rpc;
    p.nb = static_cast<int32_t>(nb);
    return p;
}

// One cluster: all blocks move through the rows together (nothing changes per segment).
inline RowPlan plan_rows(int64_t T, int64_t max_blocks, int rows_per_step) {
    const int64_t g = grid_blocks(T, max_blocks, rows_per_step);
    return make_plan(T, g, g);
}

// Forward with per-segment modulation rows: `want` clusters (see pick_clusters).
inline RowPlan plan_rows_clusters(int64_t T, int64_t nseg, int64_t max_blocks, int rows_per_step,
                                  int64_t want, int64_t forced = 0) {
    const int64_t g = grid_blocks(T, max_blocks, rows_per_step);
    if (forced > 0) return make_plan(T, g, g / forced > 0 ? g / forced : 1);
    if (nseg <= 1 || want <= 1) return make_plan(T, g, g);
    // `want` clusters of equal size (a power of two of blocks per cluster is not needed: the forward
    // keeps no slots; with 768 blocks it gave 24 clusters where 16 were wanted, 154 against 142 us on
    // 64 segments of 2048 rows at D = 1536)
    const int64_t nb = (g + want - 1) / want;
    return make_plan(T, g, nb);
}

// Fraction of the streaming time a backward launch loses when its blocks form C clusters, i.e.
// move C windows through memory at once instead of one, interpolated in log2 C.  Two measured
// tables (equal segments of about 150 000 tokens in all, slots and restarts taken out): launches of
// one block per CU (D = 5120, 256 blocks): 1.2, 2.2, 4.8, 10.7, 12.4 % at C = 2, 4, 8, 16, 32; launches
// of several small blocks per CU (D = 1536, 768 blocks): 0, 0, 2, 5, 5.5 % and 12 % at C = 768;
// extrapolated in between and beyond.
inline double cluster_penalty(int64_t C, bool one_block_per_cu) {
    static const double wide[] = {0.0, 0.012, 0.022, 0.048, 0.107, 0.124, 0.16, 0.20, 0.24, 0.27, 0.30};
    static const double narrow[] = {0.0, 0.0, 0.0, 0.02, 0.05, 0.055, 0.07, 0.09, 0.10, 0.115, 0.13};
    const double* tab = one_block_per_cu ? wide : narrow;
    if (C <= 1) return 0.0;
    if (C >= 1024) return tab[10];
    int lo = 0;
    while ((int64_t{2} << lo) <= C) ++lo;                    // 2^lo <= C < 2^(lo+1), lo <= 9
    const double frac = static_cast<double>(C - (int64_t{1} << lo)) / static_cast<double>(int64_t{1} << lo);
    return tab[lo] + (tab[lo + 1] - tab[lo]) * frac;
}

// Row plan of a backward that keeps per-(block, segment) partial-sum slots.  With several
// segments the blocks per cluster nb (a power of two) minimise
//     stream_us * cluster_penalty(C)                              windows
//   + max(0, (C + nseg) * nb * slot_rows * stream_us / T - 58 us)  slots written and read back
//   + (nseg / C + 1) * 2 us (4 us with several blocks per CU)     pipeline restarts per block
//   + (nseg - 1) * 8 us if C = 1                                  all blocks restart at once
// where slot_rows is what one slot costs in units of one row's traffic and stream_us the time
// the rows take at the streaming rate.  The first 58 us of slot traffic are free: about 128 MB of
// slots are still in the last-level cache when the second pass reads them (480 segments of 312
// rows at D = 5120: 4088 slots of 41 KB cost 8 us together with the restarts, 15 584 slots 249 us).
// A lone cluster pays for every boundary with the whole chip: all its blocks drain their
// pipelines at the same moment (3 x 75 600 rows at D = 5120: 1233 us with one cluster, 1183 with two).
inline RowPlan plan_rows_slots(int64_t T, int64_t nseg, int64_t max_blocks, int rows_per_step,
                               double stream_us, double slot_rows, int64_t forced = 0) {
    if (T <= 0) return RowPlan{0, 0, 1, 1};
    const int64_t g = grid_blocks(T, max_blocks, rows_per_step);
    int64_t nb = g;
    if (forced > 0) {
        nb = g / forced > 0 ? g / forced : 1;
    } else if (nseg > 1) {
        double best = 0.0;
        bool have = false;
        for (int64_t cand = 1; cand < 2 * g; cand *= 2) {
            if (cand > g) cand = g;                          // the last candidate: one cluster
            int64_t C = (g + cand - 1) / cand;
            const int64_t rpc = (T + C - 1) / C;
            C = (T + rpc - 1) / rpc;
            double slots_us = static_cast<double>(C + nseg) * static_cast<double>(cand) * slot_rows * stream_us /
                                  static_cast<double>(T) - 58.0;
            if (slots_us < 0.0) slots_us = 0.0;
            const bool one_per_cu = max_blocks <= kNumCU;
            const double cost = stream_us * cluster_penalty(C, one_per_cu) + slots_us +
                                (static_cast<double>(nseg) / static_cast<double>(C) + 1.0) * (one_per_cu ? 2.0 : 4.0) +
                                (C == 1 ? static_cast<double>(nseg - 1) * 8.0 : 0.0);
            if (!have || cost < best) {
                have = true;
                best = cost;
                nb = cand;
            }
            if (cand == g) break;
        }
    }
    return make_plan(T, g, nb);
}

// How a row of `nchunks` 16-byte chunks is split: K waves per row, VPL chunks per lane.  A lane
// keeps about 16 features (up to 24 when one wave can take the whole row, which needs no
// barrier at all); longer rows are shared by more waves.
struct Split {
    int K;
    int VPL;
};

inline Split choose_split(int nchunks, int dtype) {
    const int per_feat16 = dtype == 0 ? 2 : 4;          // chunks holding 16 features
    const int solo_max = dtype == 0 ? 3 : 6;            // chunks per lane a single wave may take
    const int need = (nchunks + 63) / 64;
    if (need <= solo_max) {
        int vpl = need;
        if (dtype == 1 && vpl == 5) vpl = 6;            // instantiated: 1, 2, 3, 4, 6
        return {1, vpl};
    }
    int k = (nchunks + per_feat16 * 64 - 1) / (per_feat16 * 64);
    if (k == 7) k = 8;
    return {k, per_feat16};
}

// Launch shape of the per-sample / per-segment kernels: K waves per row, VPL chunks per lane, R
// rows per block and step, per_cu resident blocks per CU.  The shape comes from a table per element
// type, indexed by the row length in units of 512 features.  The tables were measured, not
// derived: every instantiated (K, VPL, R, per_cu) that covers the row with at most 60 % padding
// and 3 to 16 waves per CU was timed on one sample of about 770 MB per tensor at every multiple of
// 512 features from 512 to 8192 (the widths of the models of Sec. 4.1, D = 1536 and 5120, three
// times on different machines, the others twice), and the entry is the shape with the best worst
// run.  What the winners share: a wave count that is a multiple of the four SIMDs of a CU (or a
// single block of 5 or 6 waves), and 16 to 32 KB of row data in flight per CU.  Neighbouring
// widths do not share winners: an entry that is best at D = 4096 loses 28 % at D = 3584.

// Entry of a per-512-features table (index 1 ... 16; [0] is unused).  A row of at most 64 chunks
// on a single wave needs one chunk per lane whatever the first entry says.
inline Shape table_entry(const Shape (&tab)[17], int nchunks, int dtype) {
    const int per512 = dtype == 0 ? 64 : 128;
    const int cols = (nchunks + per512 - 1) / per512;
    Shape sh = tab[cols < 1 ? 1 : cols > 16 ? 16 : cols];
    if (sh.K == 1 && nchunks <= 64) sh.VPL = 1;
    return sh;
}

// T: the token count if known (0: not known); only the D = 1536 entry looks at it.
inline Shape fwd_shape(int nchunks, int dtype, int64_t T = 0) {
    if (dtype == 0) {
        static const Shape tab[17] = {
            {1, 1, 2, 8},                                                    // (unused)
            {1, 1, 2, 8}, {1, 2, 2, 4}, {1, 3, 1, 8}, {2, 2, 1, 4},          // D <=  512 ... 2048
            {2, 3, 1, 4}, {4, 2, 1, 3}, {4, 2, 1, 3}, {4, 2, 2, 1},          //      2560 ... 4096
            {4, 3, 1, 2}, {5, 2, 2, 1}, {4, 3, 1, 2}, {4, 3, 1, 2},          //      4608 ... 6144
            {6, 3, 1, 2}, {6, 3, 1, 2}, {6, 3, 1, 1}, {6, 3, 1, 1}};         //      6656 ... 8192
        // D = 1536: four blocks per CU are 4 % faster on the 32 760 rows of the Wan-1.3B workload,
        // the two tie on 65 520 rows, three are 3 % faster on 131 040 rows and 5 % on 252 000
        if (nchunks == 192) return {1, 3, 2, T >= 98304 ? 3 : 4};
        return table_entry(tab, nchunks, dtype);
    }
    // fp32: one row per step and two blocks per CU once several waves share a row (a wave's four
    // chunks carry twice the bytes of a bf16 wave's two: 266 against 287 us on 37800 x 5120)
    static const Shape tab32[17] = {
        {1, 2, 2, 8},
        {1, 2, 2, 8}, {1, 4, 1, 8}, {1, 6, 2, 4}, {2, 4, 2, 2},
        {4, 4, 1, 2}, {4, 4, 1, 2}, {4, 4, 1, 2}, {4, 4, 1, 2},
        {5, 4, 1, 2}, {5, 4, 1, 2}, {8, 4, 1, 2}, {6, 4, 1, 1},
        {8, 4, 1, 2}, {8, 4, 1, 2}, {8, 4, 1, 2}, {8, 4, 1, 2}};
    return table_entry(tab32, nchunks, dtype);
}

inline Shape bwd_shape(int nchunks, int dtype) {
    if (dtype == 0) {
        static const Shape tab[17] = {
            {1, 1, 2, 8},
            {1, 1, 2, 8}, {1, 2, 2, 3}, {3, 1, 1, 4}, {4, 1, 2, 2},
            {5, 1, 2, 1}, {6, 1, 2, 1}, {4, 2, 1, 3}, {4, 2, 2, 1},
            {5, 2, 2, 1}, {4, 3, 2, 1}, {6, 2, 1, 1}, {4, 3, 2, 1},
            {8, 2, 1, 1}, {6, 3, 2, 1}, {6, 3, 2, 1}, {6, 3, 2, 1}};
        if (nchunks == 192) return {3, 1, 1, 3};
        return table_entry(tab, nchunks, dtype);
    }
    // fp32, rows of 1 KB and more: mostly one row per step (a wave's four chunks of one row are as
    // many bytes as two bf16 rows) and, for the wide rows, more waves than the chunks need
    static const Shape tab32[17] = {
        {1, 2, 2, 3},
        {1, 2, 2, 3}, {1, 4, 1, 3}, {2, 4, 1, 2}, {2, 4, 1, 2},
        {3, 4, 2, 1}, {4, 4, 1, 1}, {5, 4, 2, 1}, {4, 4, 1, 2},
        {6, 4, 1, 1}, {6, 4, 1, 1}, {6, 4, 1, 1}, {6, 4, 1, 1},
        {8, 4, 1, 1}, {8, 4, 1, 1}, {8, 4, 1, 1}, {8, 4, 1, 1}};
    return table_entry(tab32, nchunks, dtype);
}

// Backward that forms the statistics again from x.  It has one more dependent chain per step
// (per-wave mean, four wave sums, the merge with a division and a square root), which fewer waves per
// row with more chunks each, or two blocks per CU, hide better than the shapes above; timed at
// D = 512 ... 8192 like the tables above; it then runs 2 to 20 % behind the backward that reads
// the saved statistics (D = 5120: 14 %).
inline Shape rc_bwd_shape(int nchunks, int dtype) {
    if (dtype == 0) {
        static const Shape tab[17] = {
            {1, 1, 2, 8},
            {1, 1, 2, 8}, {1, 2, 2, 4}, {1, 3, 2, 4}, {2, 2, 1, 4},
            {3, 2, 2, 3}, {3, 2, 2, 2}, {4, 2, 1, 3}, {4, 2, 2, 1},
            {4, 3, 1, 2}, {4, 3, 1, 2}, {4, 3, 1, 2}, {4, 3, 2, 1},
            {8, 2, 1, 2}, {8, 2, 2, 1}, {8, 2, 2, 1}, {8, 2, 2, 1}};
        return table_entry(tab, nchunks, dtype);
    }
    static const Shape tab32[17] = {
        {1, 2, 2, 3},
        {1, 2, 2, 3}, {1, 6, 1, 3}, {2, 4, 1, 3}, {3, 4, 1, 2},
        {3, 4, 2, 1}, {4, 4, 1, 1}, {5, 4, 2, 1}, {4, 4, 1, 2},
        {6, 4, 1, 1}, {6, 4, 1, 1}, {6, 4, 1, 1}, {8, 4, 1, 1},
        {8, 4, 1, 1}, {8, 4, 1, 1}, {8, 4, 1, 1}, {8, 4, 1, 1}};
    return table_entry(tab32, nchunks, dtype);
}

// The table's entry, or the shape the call carries (Problem::force).  A forced shape that does not
// cover the row makes the launch fail instead of computing on part of the row.
inline Shape pick_shape(const Shape* force, Shape table) { return force ? *force : table; }
inline bool covers(const Shape& s, int nchunks) { return s.K * s.VPL * 64 >= nchunks; }

// Per-token modulation (three input streams forward; three in, three out backward).  bf16: a table
// per 512 features like the ones above, from the same sweep over the (K, VPL) these kernels are
// compiled for (one wave alone, or two chunks per lane on 2 to 8 waves, or five chunks per lane on two waves).  Here too neighbours do
// not share winners: D = 2560 forward takes 526 us with {3,2,2,4} and 858 us with the {3,2,1,2}
// that is best at D = 3072.  fp32: tables of the same kind (four chunks per lane once a row is
// shared, up to six on a single wave).
inline Shape tok_fwd_shape(int nchunks, int dtype) {
    if (dtype == 0) {
        static const Shape tab[17] = {
            {1, 1, 2, 8},
            {1, 1, 2, 8}, {1, 2, 2, 4}, {1, 3, 2, 4}, {2, 2, 1, 4},
            {3, 2, 2, 4}, {3, 2, 1, 2}, {4, 2, 2, 3}, {4, 2, 1, 2},
            {5, 2, 1, 3}, {2, 5, 1, 2}, {8, 2, 1, 2}, {6, 2, 2, 2},
            {8, 2, 1, 2}, {8, 2, 1, 2}, {8, 2, 1, 2}, {8, 2, 1, 1}};
        // D = 4616 ... 5120: two waves with five chunks per lane (one wave per SIMD, 5 KB runs per wave and
        // stream, half as many waves at the barrier) take 452 us on 65 520 x 5120 where five waves with two
        // chunks take 476; the same split gained nothing in the per-token backward (750 against 730 us)
        return table_entry(tab, nchunks, dtype);
    }
    static const Shape tab32[17] = {
        {1, 2, 2, 4},
        {1, 2, 2, 4}, {1, 4, 1, 4}, {2, 4, 1, 4}, {2, 4, 2, 2},
        {3, 4, 1, 3}, {4, 4, 2, 4}, {4, 4, 1, 2}, {4, 4, 1, 1},
        {6, 4, 2, 2}, {5, 4, 1, 2}, {8, 4, 2, 2}, {6, 4, 1, 1},
        {8, 4, 1, 1}, {8, 4, 1, 1}, {8, 4, 1, 1}, {8, 4, 1, 2}};
    return table_entry(tab32, nchunks, dtype);
}

inline Shape tok_bwd_shape(int nchunks, int dtype) {
    if (dtype == 0) {
        static const Shape tab[17] = {
            {1, 1, 1, 6},
            {1, 1, 1, 6}, {1, 2, 2, 3}, {1, 3, 1, 3}, {2, 2, 1, 2},
            {3, 2, 1, 2}, {3, 2, 1, 2}, {4, 2, 1, 2}, {4, 2, 1, 1},
            {6, 2, 1, 2}, {5, 2, 1, 2}, {6, 2, 2, 1}, {8, 2, 2, 1},
            {8, 2, 2, 1}, {8, 2, 2, 1}, {8, 2, 1, 1}, {8, 2, 1, 1}};
        return table_entry(tab, nchunks, dtype);
    }
    static const Shape tab32[17] = {
        {1, 2, 2, 8},
        {1, 2, 2, 8}, {1, 4, 1, 8}, {2, 4, 1, 2}, {2, 4, 2, 2},
        {3, 4, 2, 1}, {3, 4, 1, 1}, {5, 4, 1, 1}, {5, 4, 1, 3},
        {5, 4, 1, 1}, {8, 4, 2, 2}, {6, 4, 1, 1}, {6, 4, 1, 1},
        {8, 4, 1, 1}, {8, 4, 1, 1}, {8, 4, 1, 1}, {8, 4, 1, 2}};
    return table_entry(tab32, nchunks, dtype);
}

// Which blocks form a cluster.  Consecutive blocks go to the eight XCDs in turn, so with
// cluster = block index modulo the cluster count (and a count that is a multiple of 8) all blocks
// of a cluster sit on one XCD and that XCD streams through one contiguous region; clusters of
// consecutive blocks are each spread over all XCDs.  Measured on packed batches (forward /
// backward us, same cluster count): 24 mixed segments at D = 5120 554 / 834 -> 550 / 828, 96 segments
// of 1560 rows 566 / 858 -> 559 / 844, 8 segments of 16 380 rows backward 687 -> 676, 64 segments of
// 2048 rows at D = 1536 forward 150 -> 146.  So every launch with more than one cluster interleaves;
// a shaped call says for itself.
inline int cluster_interleave(const Shape* force, const RowPlan& pl) {
    return force ? force->interleave : (pl.clusters > 1 ? 1 : 0);
}

// The backward's plan for this problem: the same function sizes the workspace, drives the main
// kernel's grid and tells the second pass which partial-sum slots belong to a segment.
RowPlan bwd_plan(int64_t T, int64_t nseg, int64_t D, int dtype, bool recompute, const Shape* force = nullptr);
// Slot of (cluster c, segment m, member j) is (c + m) * nb + j with c < clusters, m < nseg.
inline int64_t bwd_slots(const RowPlan& p, int64_t nseg) {
    return nseg < 1 ? 0 : (p.clusters + nseg - 1) * p.nb;
}

// Shape of the second pass: V features per lane, W waves per block, G groups of lanes per wave
// that take different slots (a block covers 64 / G * V features).  Wide blocks need enough
// (segment, sum, feature-block) triples to fill the chip; a wave should have about four slots
// to add, and a block never more than 16 waves.
struct ReduceShape {
    int V;
    int W;
    int G = 1;      // groups of lanes of a wave that take different slots (then V = 4)
};

inline ReduceShape reduce_shape(int64_t nseg, int nsum, int64_t D, int64_t clusters, int64_t nb) {
    ReduceShape sh{1, 1};
    const int64_t triples = nseg * nsum;
    if (triples * ((D + 255) / 256) >= 256) sh.V = 4;
    else if (triples * ((D + 127) / 128) >= 256) sh.V = 2;
    const int64_t slots = nb * (1 + (clusters - 1) / nseg);   // typical slots of one segment
    // Narrow blocks keep their width but read 16 bytes per lane: the lanes form 4 / V groups that take
    // different slots, so a wave covers several slots per load (second pass of 75 600 x 5120:
    // 6.1 -> 4.9 us, of 32 760 x 1536: 8.9 -> 6.4, of 2 x 32 760 x 5120: 9.9 -> 7.8; eight groups of
    // 32 features or sixteen of 16 were slower again)
    if (sh.V < 4 && D % 4 == 0) {
        sh.G = 4 / sh.V;
        sh.V = 4;
        while (sh.W < 16 && sh.W * 2 * sh.G <= slots) sh.W *= 2;
        return sh;
    }
    while (sh.W < 16 && sh.W * 2 * 4 <= slots) sh.W *= 2;
    return sh;
}

// The backward entry point that allocates nothing keeps its partial-sum slots in a static device
// array of this size (per GPU); static_workspace() returns that array's address on the current
// device.
constexpr size_t kStaticWorkspaceBytes = size_t(64) << 20;
hipError_t static_workspace(float** ptr);

// Text naming the kernel instantiations and grids that a call with these arguments launches.
int describe_fwd(const Problem& p, bool per_token, char* buf, size_t n);
int describe_bwd(const Problem& p, bool per_token, bool recompute, char* buf, size_t n);

struct ReduceArgs;
hipError_t launch_reduce(ReduceArgs r, int64_t clusters, hipStream_t st);

hipError_t launch_fwd_seg(const Problem& p, const void* x, const void* shift, const void* scale,
                          void* y, float* mean, float* rstd, hipStream_t st);
hipError_t launch_fwd_tok(const Problem& p, const void* x, const void* shift, const void* scale,
                          void* y, float* mean, float* rstd, hipStream_t st);
hipError_t launch_bwd_seg(const Problem& p, const void* dy, const void* x, const void* scale,
                          const float* mean, const float* rstd, void* dx, float* dshift,
                          float* dscale, float* ws, hipStream_t st);
hipError_t launch_bwd_tok(const Problem& p, const void* dy, const void* x, const void* scale,
                          const float* mean, const float* rstd, void* dx, void* dshift,
                          void* dscale, hipStream_t st);
hipError_t launch_unfused(const Problem& p, const void* x, const void* shift, const void* scale,
                          void* xhat, void* y, float* mean, float* rstd, hipStream_t st);
hipError_t launch_copy(const void* src, void* dst, size_t bytes, hipStream_t st);
bool probe_mixture_supported(int reads, int writes);
hipError_t launch_stream_probe(const void* const* in, int reads, void* const* out, int writes, size_t bytes,
                               int blocks, int waves, int vecs, hipStream_t st);

// Gated residual + LayerNorm-Modulate (per-sample / per-segment gate, shift, scale).
RowPlan gated_bwd_plan(int64_t T, int64_t nseg, int64_t D, int dtype);
Shape gated_fwd_table_shape(int nchunks, int dtype);             // the tables' entries, no override
Shape gated_bwd_table_shape(int nchunks, int dtype);
hipError_t launch_gated_fwd(const Problem& p, const void* x, const void* u, const void* gate,
                            const void* shift, const void* scale, void* h, void* y, float* mean,
                            float* rstd, hipStream_t st);
hipError_t launch_gate_residual(const Problem& p, const void* x, const void* u, const void* gate,
                                void* h, hipStream_t st);
hipError_t launch_gated_bwd(const Problem& p, const void* dy, const void* dh, const void* h,
                            const void* u, const void* gate, const void* scale, const float* mean,
                            const float* rstd, void* dx, void* du, float* dgate, float* dshift,
                            float* dscale, float* ws, hipStream_t st);
hipError_t launch_zero_f32(float* p, int64_t n, hipStream_t st);


// Fused Q-Norm + K-Norm (RMS normalisation with a learned weight of two tensors, one launch).
int32_t qknorm_bwd_blocks(int64_t N, int64_t D, int dtype);      // partial-sum slots per tensor
Shape qknorm_table_shape(int nchunks, int dtype, bool backward);  // rows wider than one head; no override
hipError_t launch_qknorm_fwd(int dtype, const void* q, const void* k, const void* wq, const void* wk,
                             int64_t N, int64_t D, float eps, void* q_out, void* k_out,
                             float* rstd_q, float* rstd_k, hipStream_t st);
hipError_t launch_qknorm_bwd(int dtype, const void* dq_out, const void* dk_out, const void* q,
                             const void* k, const void* wq, const void* wk, int64_t N, int64_t D,
                             const float* rstd_q, const float* rstd_k, void* dq, void* dk,
                             float* dwq, float* dwk, float* ws, hipStream_t st);

}  // namespace lnmod
