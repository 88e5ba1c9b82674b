// Host-only check of the launch planning in csrc/plan.hpp (no HIP): compiled and run by
// tests/test_plan_host.py.  Prints "ok" or the first violated invariant.
#include <cstdio>
#include <cstdlib>
#include <initializer_list>

#include "plan.hpp"

using namespace evospec;

#define REQUIRE(cond, ...) do { if (!(cond)) { std::printf("FAILED %s: ", #cond); std::printf(__VA_ARGS__); std::printf("\n"); return 1; } } while (0)

int main() {
    const int cus[] = {256, 304, 64};
    const int ds[] = {8, 64, 2048, 4096, 4104, 8192};
    const int ks[] = {1, 10, 16, 17, 64};
    const int rows_list[] = {1, 16, 17, 32, 33, 60, 64};
    for (int cu : cus)
        for (int d : ds)
            for (int k : ks)
                for (int rows : rows_list)
                    for (int V_act = 1; V_act <= 200000; V_act = V_act < 300 ? V_act + 1 : V_act + V_act / 7 + 13) {
                        if (k > V_act) continue;
                        for (int replicas : {1, 16}) {
                            const Plan p = make_plan(rows, V_act, d, k, cu, replicas);
                            REQUIRE(p.nw >= 4 && p.nw <= 12 && p.rgw == 1 && p.rc == 2, "shape nw=%d rgw=%d rc=%d", p.nw, p.rgw, p.rc);
                            REQUIRE(p.rt == 16 * p.nw * p.rgw, "rt=%d", p.rt);
                            REQUIRE(p.mb == mb_for_rows(rows) && 16 * p.mb >= rows, "mb=%d rows=%d", p.mb, rows);
                            REQUIRE((long)p.n_slabs * p.rt >= V_act && (long)(p.n_slabs - 1) * p.rt < V_act, "slabs=%d rt=%d V_act=%d", p.n_slabs, p.rt, V_act);
                            REQUIRE(p.lds_bytes <= (size_t)kLdsLimit, "lds=%zu", p.lds_bytes);
                            REQUIRE(p.gl >= 0 && p.gl <= 2, "gl=%d", p.gl);
                            // the workspace the ABI asks callers for covers the plan's own layout
                            REQUIRE(p.stats_off >= (size_t)p.n_slabs * kMTile * k * 8, "stats_off");
                            REQUIRE(p.total_bytes <= workspace_upper_bound(V_act, k), "total=%zu bound=%zu V_act=%d k=%d nw=%d", p.total_bytes,
                                    workspace_upper_bound(V_act, k), V_act, k, p.nw);
                        }
                    }
    // the shapes the benchmark configurations run with on 256 CUs (measured best of a sweep over nw)
    REQUIRE(make_plan(60, 36864, 4096, 10, 256).nw == 9, "36,864 rows");
    REQUIRE(make_plan(60, 32256, 4096, 10, 256).nw == 9, "32,256 rows: not the 1 MiB slabs of 8 wavefronts");
    REQUIRE(make_plan(8, 18432, 4096, 10, 256).nw == 5, "18,432 rows");
    REQUIRE(make_plan(60, 8448, 4096, 10, 256).nw == 4, "8,448 rows");
    REQUIRE(make_plan(60, 151936, 4096, 10, 256).nw == 10, "151,936 rows");
    // packed layout sizes
    REQUIRE(packed_d(4096) == 4096 && packed_d(8) == 256 && packed_d(264) == 512, "packed_d");
    REQUIRE(packed_rows(36864) == 36864 && packed_rows(1) == 16 && packed_rows(17) == 32, "packed_rows");
    REQUIRE(matrix_elems(33, 72, true) == 48u * 256u && matrix_elems(33, 72, false) == 33u * 72u, "matrix_elems");
    // large-M plan: lists and statistics do not overlap, one slab per 128 rows
    for (int M : {129, 960, 4096})
        for (int V_act : {1, 127, 128, 129, 32768, 151936}) {
            const GemmPlan g = make_gemm_plan(M, V_act, 10);
            REQUIRE(g.n_slabs == (V_act + 127) / 128 && g.list_len == 16, "gemm slabs");
            REQUIRE(g.stats_off >= (size_t)g.n_slabs * M * g.list_len * 8 && g.total_bytes >= g.stats_off + (size_t)g.n_slabs * M * 8, "gemm layout");
        }
    REQUIRE(gemm_list_len(16) == 16 && gemm_list_len(17) == 32 && gemm_list_len(64) == 64, "list_len");
    REQUIRE(use_gemm(129, 4096) && !use_gemm(128, 4096) && !use_gemm(960, 4104), "use_gemm");
    std::printf("ok\n");
    return 0;
}
