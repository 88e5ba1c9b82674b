// Host driver for the sanitizer build (-fsanitize=address,undefined) of the dynamic-buffer manager
// and the candidate formation: replays seeded request streams through the C ABI and checks, after
// every event, what the ABI promises (dense slots in range, bounded lists, bounded insertions, no core
// or repeated id written).  Prints "ok" when nothing failed; the sanitizers abort on their own findings.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <set>
#include <vector>

#include "evospec.h"
#include "evospec_arc.h"

#define REQUIRE(c, ...) do { if (!(c)) { std::printf("FAILED %s:%d: ", __FILE__, __LINE__); std::printf(__VA_ARGS__); std::printf("\n"); return 1; } } while (0)

static uint64_t g_state = 0x9e3779b97f4a7c15ull;
static uint32_t rnd() { g_state = g_state * 6364136223846793005ull + 1442695040888963407ull; return (uint32_t)(g_state >> 33); }
// ids with a heavy head, like token frequencies: small ids come back often
static int32_t skewed(int V) { const double u = (rnd() % 1000000) / 1e6; return (int32_t)(u * u * u * V); }

static int replay(evospec_arc_config cfg, int V, int n_core, int n_events) {
    std::vector<int32_t> core(n_core);
    for (int i = 0; i < n_core; ++i) core[i] = i * 3;
    std::set<int32_t> core_set(core.begin(), core.end());
    evospec_arc* arc = nullptr;
    REQUIRE(evospec_arc_create(&cfg, n_core ? core.data() : nullptr, n_core, &arc) == EVOSPEC_OK, "create");
    evospec_arc_config back;
    REQUIRE(evospec_arc_get_config(arc, &back) == EVOSPEC_OK && back.capacity == cfg.capacity && back.slot_base == cfg.slot_base, "config");
    std::vector<int32_t> slots(cfg.max_insert + 1), ids(cfg.max_insert + 1), cand, rs(cfg.capacity), ri(cfg.capacity), lst(cfg.capacity + cfg.ghost_capacity + 1);
    for (int e = 0; e < n_events; ++e) {
        cand.clear();
        const int n = (int)(rnd() % 200);
        for (int i = 0; i < n; ++i) cand.push_back(rnd() % 17 == 0 ? -1 - (int32_t)(rnd() % 5) : skewed(V));
        int n_out = -1;
        REQUIRE(evospec_arc_event(arc, cand.empty() ? nullptr : cand.data(), (int)cand.size(), slots.data(), ids.data(), &n_out) == EVOSPEC_OK, "event %d", e);
        REQUIRE(n_out >= 0 && n_out <= cfg.max_insert, "event %d wrote %d pairs", e, n_out);
        std::set<int32_t> written;
        for (int i = 0; i < n_out; ++i) {
            REQUIRE(slots[i] >= cfg.slot_base && slots[i] < cfg.slot_base + cfg.capacity, "slot %d", slots[i]);
            REQUIRE(ids[i] >= 0 && !core_set.count(ids[i]) && written.insert(ids[i]).second, "id %d", ids[i]);
        }
        int nr = 0;
        REQUIRE(evospec_arc_resident(arc, rs.data(), ri.data(), &nr) == EVOSPEC_OK && nr <= cfg.capacity, "resident");
        for (int i = 0; i < nr; ++i) REQUIRE(rs[i] == cfg.slot_base + i, "slots are not dense at %d", i);
        int64_t sz[7];
        REQUIRE(evospec_arc_sizes(arc, sz) == EVOSPEC_OK, "sizes");
        REQUIRE(sz[0] >= 0 && sz[0] <= cfg.capacity && sz[1] + sz[2] == nr && sz[3] <= cfg.ghost_capacity && sz[4] <= cfg.ghost_capacity, "list sizes");
        for (int which = 0; which < 4; ++which) {
            int nl = 0;
            REQUIRE(evospec_arc_list(arc, which, lst.data(), (int)lst.size(), &nl) == EVOSPEC_OK && nl == sz[1 + which], "list %d", which);
        }
        if (rnd() % 3 == 0 && nr > 0) {                 // hits on resident and on foreign tokens
            int32_t t[3] = {ri[rnd() % nr], skewed(V), -4};
            REQUIRE(evospec_arc_touch(arc, t, 3) == EVOSPEC_OK, "touch");
        }
        REQUIRE(evospec_arc_advance(arc, (int)(rnd() % 6)) == EVOSPEC_OK, "advance");
    }
    evospec_arc_destroy(arc);
    return 0;
}

static int candidates(int V) {
    // a CSR graph with ragged rows, some successors outside the vocabulary
    std::vector<int64_t> row_ptr(V + 1, 0);
    std::vector<int32_t> col;
    for (int v = 0; v < V; ++v) {
        const int deg = (int)(rnd() % 12);
        for (int j = 0; j < deg; ++j) col.push_back(rnd() % 23 == 0 ? V + (int32_t)(rnd() % 9) : (int32_t)(rnd() % V));
        row_ptr[v + 1] = (int64_t)col.size();
    }
    std::vector<int32_t> out(64);
    for (int t = 0; t < 3000; ++t) {
        int32_t a[12], b[12];
        const int na = (int)(rnd() % 12), nb = (int)(rnd() % 12);
        for (int i = 0; i < na; ++i) a[i] = (int32_t)(rnd() % (V + 3)) - 1;
        for (int i = 0; i < nb; ++i) b[i] = (int32_t)(rnd() % (V + 3)) - 1;
        const int ms = (int)(rnd() % 10), cap = (int)(rnd() % 65);
        const bool graph = ms > 0 || rnd() % 2;
        int n = -1;
        REQUIRE(evospec_form_candidates(a, na, b, nb, graph ? row_ptr.data() : nullptr, graph ? col.data() : nullptr, V, ms,
                                        out.data(), cap, &n) == EVOSPEC_OK, "form_candidates");
        REQUIRE(n >= 0 && n <= cap, "n=%d cap=%d", n, cap);
        std::set<int32_t> seen;
        for (int i = 0; i < n; ++i) REQUIRE(out[i] >= 0 && out[i] < V && seen.insert(out[i]).second, "candidate %d", out[i]);
    }
    return 0;
}

int main() {
    evospec_arc_config paper;
    evospec_arc_default_config(&paper);
    paper.slot_base = 32000;
    const evospec_arc_config small{16, 3, 5, 4, 2, 0, 7}, no_ghosts{8, 8, 0, 8, 0, 3, 0}, one{1, 0, 1, 1, 0, 0, 0}, slow{32, 0, 64, 1, 5, 10, 100};
    if (replay(paper, 151936, 2000, 3000)) return 1;
    if (replay(small, 500, 20, 3000)) return 1;
    if (replay(no_ghosts, 200, 0, 3000)) return 1;
    if (replay(one, 50, 5, 2000)) return 1;
    if (replay(slow, 4000, 300, 3000)) return 1;
    if (candidates(300)) return 1;
    std::printf("ok\n");
    return 0;
}
