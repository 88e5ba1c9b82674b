// Dynamic-buffer manager (host only): Adaptive Replacement Cache with the safeguards of the
// EvoSpec appendix ("ARC-based dynamic vocabulary maintenance", "Additional safeguards").
// The interface, the rules and the readings taken where the paper is silent are stated in
// include/evospec_arc.h.
//
// Each of T1, T2, B1, B2 is an intrusive doubly linked list over one node pool (head = least
// recently used); a hash map takes a token id to its node.  Every operation of an event is
// O(1) except the search for a victim that is old enough, which walks past the young tokens.
// Nothing in this file touches the GPU: it builds with the host compiler alone.
#include <cstdint>
#include <new>
#include <unordered_map>
#include <unordered_set>
#include <vector>

#include "evospec.h"
#include "evospec_arc.h"

namespace {

enum Where : int { kT1 = 0, kT2 = 1, kB1 = 2, kB2 = 3, kNone = 4 };

struct Node {
    int32_t id = -1;
    int where = kNone;
    int prev = -1, next = -1;      // indices into the pool
    int slot = -1;                 // resident tokens only
    int64_t born = 0;              // decoding step of insertion
};

struct List {
    int head = -1, tail = -1, size = 0;
};

}  // namespace

struct evospec_arc {
    evospec_arc_config cfg;
    int p = 0;
    int64_t step = 0, events = 0;
    std::vector<Node> pool;
    std::vector<int> free_nodes;
    List lists[4];
    std::unordered_map<int32_t, int> index;       // token id -> node (resident or ghost)
    std::unordered_set<int32_t> core;
    std::unordered_set<int32_t> seen;

    int alloc_node() {
        if (!free_nodes.empty()) { const int n = free_nodes.back(); free_nodes.pop_back(); return n; }
        pool.emplace_back();
        return (int)pool.size() - 1;
    }
    void unlink(int n) {
        Node& x = pool[n];
        List& l = lists[x.where];
        if (x.prev >= 0) pool[x.prev].next = x.next; else l.head = x.next;
        if (x.next >= 0) pool[x.next].prev = x.prev; else l.tail = x.prev;
        x.prev = x.next = -1;
        --l.size;
        x.where = kNone;
    }
    void push_mru(int n, int where) {
        Node& x = pool[n];
        List& l = lists[where];
        x.where = where;
        x.prev = l.tail;
        x.next = -1;
        if (l.tail >= 0) pool[l.tail].next = n; else l.head = n;
        l.tail = n;
        ++l.size;
    }
    void forget(int n) {                             // a ghost falls off its list
        index.erase(pool[n].id);
        unlink(n);
        free_nodes.push_back(n);
    }
    int resident() const { return lists[kT1].size + lists[kT2].size; }

    // least recently used token of T1 (if |T1| > p) or T2, else of the other list, that has been
    // resident for min_residency steps; -1 if there is none
    int victim() const {
        const int first = lists[kT1].size > p ? kT1 : kT2;
        const int order[2] = {first, first == kT1 ? kT2 : kT1};
        for (int w : order)
            for (int n = lists[w].head; n >= 0; n = pool[n].next)
                if (step - pool[n].born >= cfg.min_residency) return n;
        return -1;
    }
    void hit(int n) {                                // resident token requested again
        unlink(n);
        push_mru(n, kT2);
    }
};

extern "C" {

void evospec_arc_default_config(evospec_arc_config* cfg) {
    if (!cfg) return;
    cfg->capacity = 256;
    cfg->p0 = 128;
    cfg->ghost_capacity = 256;
    cfg->max_insert = 32;
    cfg->min_residency = 8;
    cfg->warmup_events = 50;
    cfg->slot_base = 0;
}

int evospec_arc_create(const evospec_arc_config* cfg, const int32_t* core_ids, int n_core, evospec_arc** out) {
    if (!cfg || !out) return EVOSPEC_NULL_POINTER;
    if (cfg->capacity < 1 || cfg->p0 < 0 || cfg->p0 > cfg->capacity || cfg->ghost_capacity < 0 ||
        cfg->max_insert < 0 || cfg->min_residency < 0 || cfg->warmup_events < 0 || n_core < 0)
        return EVOSPEC_BAD_SHAPE;
    if (n_core > 0 && !core_ids) return EVOSPEC_NULL_POINTER;
    evospec_arc* a = new (std::nothrow) evospec_arc();
    if (!a) return EVOSPEC_BAD_SHAPE;
    a->cfg = *cfg;
    a->p = cfg->p0;
    a->pool.reserve((size_t)cfg->capacity + 2 * (size_t)cfg->ghost_capacity + 8);
    a->core.reserve((size_t)n_core * 2 + 1);
    for (int i = 0; i < n_core; ++i) a->core.insert(core_ids[i]);
    *out = a;
    return EVOSPEC_OK;
}

void evospec_arc_destroy(evospec_arc* arc) { delete arc; }

int evospec_arc_get_config(const evospec_arc* arc, evospec_arc_config* out) {
    if (!arc || !out) return EVOSPEC_NULL_POINTER;
    *out = arc->cfg;
    return EVOSPEC_OK;
}

int evospec_arc_advance(evospec_arc* arc, int steps) {
    if (!arc) return EVOSPEC_NULL_POINTER;
    if (steps < 0) return EVOSPEC_BAD_SHAPE;
    arc->step += steps;
    return EVOSPEC_OK;
}

int evospec_arc_touch(evospec_arc* arc, const int32_t* ids, int n) {
    if (!arc || (n > 0 && !ids)) return EVOSPEC_NULL_POINTER;
    if (n < 0) return EVOSPEC_BAD_SHAPE;
    for (int i = 0; i < n; ++i) {
        auto it = arc->index.find(ids[i]);
        if (it == arc->index.end()) continue;
        const int w = arc->pool[it->second].where;
        if (w == kT1 || w == kT2) arc->hit(it->second);
    }
    return EVOSPEC_OK;
}

int evospec_arc_event(evospec_arc* arc, const int32_t* candidates, int n, int32_t* out_slots,
                      int32_t* out_ids, int* n_out) {
    if (!arc || !n_out || (n > 0 && !candidates)) return EVOSPEC_NULL_POINTER;
    if (n < 0) return EVOSPEC_BAD_SHAPE;
    if (arc->cfg.max_insert > 0 && (!out_slots || !out_ids)) return EVOSPEC_NULL_POINTER;
    evospec_arc& a = *arc;
    a.events += 1;
    const bool adapt = a.events > a.cfg.warmup_events;
    a.seen.clear();
    int written = 0;
    for (int i = 0; i < n; ++i) {
        const int32_t x = candidates[i];
        if (x < 0 || a.core.count(x) || !a.seen.insert(x).second) continue;
        auto it = a.index.find(x);
        int node = it == a.index.end() ? -1 : it->second;
        const int where = node < 0 ? (int)kNone : a.pool[node].where;
        if (where == kT1 || where == kT2) { a.hit(node); continue; }
        if (written >= a.cfg.max_insert) continue;
        const bool full = a.resident() >= a.cfg.capacity;
        if (full && a.victim() < 0) continue;
        // a ghost hit moves the target, then the token leaves its ghost list
        if (where == kB1) {
            if (adapt) {
                const int d = a.lists[kB2].size / a.lists[kB1].size;
                a.p += d > 1 ? d : 1;
                if (a.p > a.cfg.capacity) a.p = a.cfg.capacity;
            }
            a.unlink(node);
        } else if (where == kB2) {
            if (adapt) {
                const int d = a.lists[kB1].size / a.lists[kB2].size;
                a.p -= d > 1 ? d : 1;
                if (a.p < 0) a.p = 0;
            }
            a.unlink(node);
        }
        int slot;
        if (full) {
            const int v = a.victim();
            const int ghost = a.pool[v].where == kT1 ? kB1 : kB2;
            slot = a.pool[v].slot;
            a.unlink(v);
            a.pool[v].slot = -1;
            a.push_mru(v, ghost);
            if (a.lists[ghost].size > a.cfg.ghost_capacity) a.forget(a.lists[ghost].head);
        } else {
            slot = a.resident();
        }
        if (node < 0) {
            node = a.alloc_node();
            a.pool[node].id = x;
            a.index[x] = node;
        }
        a.pool[node].slot = slot;
        a.pool[node].born = a.step;
        a.push_mru(node, where == kB1 || where == kB2 ? kT2 : kT1);
        out_slots[written] = a.cfg.slot_base + slot;
        out_ids[written] = x;
        ++written;
    }
    *n_out = written;
    return EVOSPEC_OK;
}

int evospec_arc_sizes(const evospec_arc* arc, int64_t out[7]) {
    if (!arc || !out) return EVOSPEC_NULL_POINTER;
    out[0] = arc->p;
    for (int i = 0; i < 4; ++i) out[1 + i] = arc->lists[i].size;
    out[5] = arc->step;
    out[6] = arc->events;
    return EVOSPEC_OK;
}

int evospec_arc_list(const evospec_arc* arc, int which, int32_t* out, int cap, int* n_out) {
    if (!arc || !n_out) return EVOSPEC_NULL_POINTER;
    if (which < 0 || which > 3 || cap < 0) return EVOSPEC_BAD_SHAPE;
    const List& l = arc->lists[which];
    *n_out = l.size;
    if (l.size > cap) return EVOSPEC_BAD_SHAPE;
    if (l.size > 0 && !out) return EVOSPEC_NULL_POINTER;
    int i = 0;
    for (int n = l.head; n >= 0; n = arc->pool[n].next) out[i++] = arc->pool[n].id;
    return EVOSPEC_OK;
}

int evospec_arc_resident(const evospec_arc* arc, int32_t* out_slots, int32_t* out_ids, int* n_out) {
    if (!arc || !n_out) return EVOSPEC_NULL_POINTER;
    const int r = arc->resident();
    *n_out = r;
    if (r > 0 && (!out_slots || !out_ids)) return EVOSPEC_NULL_POINTER;
    for (int w = kT1; w <= kT2; ++w)
        for (int n = arc->lists[w].head; n >= 0; n = arc->pool[n].next) {
            const int s = arc->pool[n].slot;           // used slots are dense: 0 .. r-1
            out_slots[s] = arc->cfg.slot_base + s;
            out_ids[s] = arc->pool[n].id;
        }
    return EVOSPEC_OK;
}

int evospec_form_candidates(const int32_t* target_top, int n_target, const int32_t* mips_top, int n_mips,
                            const int64_t* row_ptr, const int32_t* col_idx, int V, int max_successors,
                            int32_t* out, int out_cap, int* n_out) {
    if (!n_out || (n_target > 0 && !target_top) || (n_mips > 0 && !mips_top)) return EVOSPEC_NULL_POINTER;
    if (n_target < 0 || n_mips < 0 || V <= 0 || max_successors < 0 || out_cap < 0) return EVOSPEC_BAD_SHAPE;
    if (out_cap > 0 && !out) return EVOSPEC_NULL_POINTER;
    if (max_successors > 0 && (!row_ptr || !col_idx)) return EVOSPEC_NULL_POINTER;
    std::unordered_set<int32_t> seen;
    int n = 0, n_seeds = 0;
    auto add = [&](int32_t x) {                      // ids outside the vocabulary never become candidates
        if (x >= 0 && x < V && n < out_cap && seen.insert(x).second) out[n++] = x;
    };
    for (int i = 0; i < n_target; ++i) add(target_top[i]);
    for (int i = 0; i < n_mips; ++i) add(mips_top[i]);
    n_seeds = n;
    // (no successors asked for: the graph may be absent; seeds that fill `out` leave no room for any)
    for (int s = 0; max_successors > 0 && s < n_seeds && n < out_cap; ++s) {
        const int64_t lo = row_ptr[out[s]], hi = row_ptr[out[s] + 1];
        for (int64_t j = lo; j < hi && j < lo + max_successors; ++j) add(col_idx[j]);
    }
    *n_out = n;
    return EVOSPEC_OK;
}

}  // extern "C"
