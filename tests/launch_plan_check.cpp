// Host-side invariants of the launch planning in csrc/lnmod_launch.hpp (compiled and run by
// test_launch_plan_cpu.py; no device code, no GPU).
#include <cstdint>
#include <cstdio>
#include <random>
#include "lnmod_launch.hpp"

using namespace lnmod;

static int bad = 0;
#define CHECK(cond, ...) do { if (!(cond)) { if (bad < 20) { std::printf("FAIL %s: ", #cond); std::printf(__VA_ARGS__); std::printf("\n"); } ++bad; } } while (0)

static void check_shape(const char* which, int dtype, int D, int nchunks, Shape s) {
    CHECK(s.K >= 1 && s.K <= 16, "%s dtype %d D %d: K %d", which, dtype, D, s.K);
    CHECK(s.VPL >= 1 && s.VPL <= 6, "%s dtype %d D %d: VPL %d", which, dtype, D, s.VPL);
    CHECK(s.R == 1 || s.R == 2, "%s dtype %d D %d: R %d", which, dtype, D, s.R);
    CHECK(s.per_cu >= 1 && s.per_cu * s.K <= 32, "%s dtype %d D %d: per_cu %d K %d", which, dtype, D, s.per_cu, s.K);
    // the K waves' VPL chunk columns must cover the row
    CHECK(s.K * s.VPL * 64 >= nchunks, "%s dtype %d D %d: %d x %d x 64 < %d chunks", which, dtype, D, s.K, s.VPL, nchunks);
}

static void check_plan(const char* which, RowPlan p, int64_t T, int64_t g) {
    CHECK(p.nb >= 1 && p.clusters >= 1, "%s T %lld: nb %d clusters %lld", which, (long long)T, p.nb, (long long)p.clusters);
    CHECK(p.blocks == p.clusters * p.nb, "%s T %lld: blocks", which, (long long)T);
    CHECK(p.clusters * p.rows_per_cluster >= T, "%s T %lld: regions do not cover the rows", which, (long long)T);
    CHECK((p.clusters - 1) * p.rows_per_cluster < T, "%s T %lld: an empty cluster", which, (long long)T);
    CHECK(p.blocks <= 2 * g + p.nb, "%s T %lld: %lld blocks for %lld wanted", which, (long long)T, (long long)p.blocks, (long long)g);
}

int main() {
    for (int dtype = 0; dtype < 2; ++dtype) {
        const int E = dtype == 0 ? 8 : 4;
        for (int D = E; D <= kMaxD; D += E) {
            const int n = D / E;
            check_shape("fwd", dtype, D, n, fwd_shape(n, dtype));
            check_shape("fwd, many rows", dtype, D, n, fwd_shape(n, dtype, 1000000));
            check_shape("bwd", dtype, D, n, bwd_shape(n, dtype));
            check_shape("rc_bwd", dtype, D, n, rc_bwd_shape(n, dtype));
            check_shape("tok_fwd", dtype, D, n, tok_fwd_shape(n, dtype));
            check_shape("tok_bwd", dtype, D, n, tok_bwd_shape(n, dtype));
        }
    }
    std::mt19937_64 rng(7);
    for (int it = 0; it < 20000; ++it) {
        const int64_t T = 1 + static_cast<int64_t>(rng() % (it % 3 == 0 ? 64 : 400000));
        const int64_t nseg = 1 + static_cast<int64_t>(rng() % (it % 5 == 0 ? 3000 : 40));
        const int64_t max_blocks = 256 * (1 + static_cast<int64_t>(rng() % 8));
        const int R = 1 + static_cast<int>(rng() % 2);
        const int64_t g = grid_blocks(T, max_blocks, R);
        CHECK(g >= 1 && g <= max_blocks, "grid_blocks %lld", (long long)g);
        check_plan("plan_rows", plan_rows(T, max_blocks, R), T, g);
        const double stream_us = static_cast<double>(T) * 30720.0 / 5.8e6;
        const int64_t want = pick_clusters(stream_us, nseg);
        CHECK(want >= 1 && want <= 32 && (want <= nseg || want <= 2) && (nseg == 1) == (want == 1), "pick_clusters %lld for %lld segments", (long long)want, (long long)nseg);
        check_plan("plan_rows_clusters", plan_rows_clusters(T, nseg, max_blocks, R, want), T, g);
        const RowPlan ps = plan_rows_slots(T, nseg, max_blocks, R, stream_us, 16.0 / 6.0);
        check_plan("plan_rows_slots", ps, T, g);
        // every (cluster, segment) incidence owns nb slots at (cluster + segment) * nb
        CHECK(bwd_slots(ps, nseg) >= (ps.clusters - 1 + nseg - 1 + 1) * ps.nb, "slots");
        if (nseg == 1) CHECK(ps.clusters == 1, "one segment wants one cluster, got %lld", (long long)ps.clusters);
        const ReduceShape rs = reduce_shape(nseg, 2 + it % 2, 8 * (1 + static_cast<int64_t>(rng() % 1024)), ps.clusters, ps.nb);
        CHECK((rs.V == 1 || rs.V == 2 || rs.V == 4) && rs.W >= 1 && rs.W <= 16 && (rs.W & (rs.W - 1)) == 0, "reduce shape V %d W %d", rs.V, rs.W);
        CHECK((rs.G == 1 || rs.G == 2 || rs.G == 4) && (rs.G == 1 || rs.V == 4), "reduce shape V %d G %d", rs.V, rs.G);
    }
    for (int wide = 0; wide < 2; ++wide) {
        for (int64_t C = 1; C < 2000; ++C) {
            const double p = cluster_penalty(C, wide != 0), q = cluster_penalty(C + 1, wide != 0);
            CHECK(p >= 0.0 && p <= 0.30 + 1e-12 && q + 1e-12 >= p, "cluster_penalty(%lld) = %g, next %g", (long long)C, p, q);
            CHECK(wide == 0 || p + 1e-12 >= cluster_penalty(C, false), "one block per CU pays less at %lld", (long long)C);
        }
    }
    // the plans the cost model was fitted to (D = 5120: 256 blocks, rows of 30 KB traffic)
    {
        const struct { int64_t T, nseg, clusters; } fit[] = {{152880, 24, 4}, {152880, 8, 2}, {149760, 96, 8},
                                                            {149760, 480, 32}, {226800, 3, 2}, {65520, 2, 2}};
        for (const auto& f : fit) {
            const RowPlan ps = plan_rows_slots(f.T, f.nseg, 256, 2, static_cast<double>(f.T) * 30720.0 / 5.8e6, 16.0 / 6.0);
            CHECK(ps.clusters == f.clusters, "T %lld nseg %lld: %lld clusters, fitted %lld", (long long)f.T,
                  (long long)f.nseg, (long long)ps.clusters, (long long)f.clusters);
        }
    }
    std::printf("checked, %d failures\n", bad);
    return bad == 0 ? 0 : 1;
}
