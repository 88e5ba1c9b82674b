#!/usr/bin/env python3
"""Benchmark of the active-vocabulary LM head on one MI355X.

A step is one pass of the whole hot path on one batch of synthetic input:
  1. the restricted head: projection + log-normaliser + top-k + id remap, and
  2. a dynamic-buffer update -- 32 new rows into ARC slots of the compact matrix (the paper caps
     insertions at 32 per failure event), applied behind the head and seen by the next step on that
     matrix (`evospec_active_lmhead_topk_then_update`; the two separate calls are timed as an extra).
All inputs are resident in HBM before the timed region.  Steps rotate over several copies of
W_act so that every step streams its weights from HBM rather than from the memory-side cache.

Prints ONE JSON line (see the keys below).  `--gpus N` with N > 1 is refused: this build is a
single-GPU kernel path.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E peak
METRIC = "active LM-head+top-k µs/step & HBM GB/s (d=4096, V_act=36864, M=60)"
UPDATE_ROWS = 32                # App. "Additional safeguards": at most 32 insertions per failure event


def algorithmic_bytes(V_act: int, d: int, M: int, k: int) -> int:
    """Bytes the method must move per step: each active weight row once, h, ids, outputs."""
    return V_act * d * 2 + M * d * 2 + V_act * 4 + M * (8 * k + 4)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="draft60", choices=["draft60", "tiny"])
    ap.add_argument("--copies", type=int, default=4, help="distinct W_act copies rotated over")
    ap.add_argument("--layout", default="packed", choices=["packed", "row_major"],
                    help="layout of the compact matrices W_act (the library's packed layout, or row-major)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true")
    ap.add_argument("--extras", default="all",
                    help="comma list of extra sections to run: core,depth,batched,host,sweep (default all); "
                         "a profiler run names the one it wants")
    ap.add_argument("--no-sweep", action="store_true",
                    help="skip extra.sweep (the head at the paper's own active-set sizes)")
    args = ap.parse_args()
    sections = {"core", "depth", "batched", "host", "sweep"} if args.extras == "all" else set(args.extras.split(","))
    if args.no_extras:
        sections = set()
    if args.no_sweep:
        sections.discard("sweep")
    if args.gpus != 1:
        print("bench.py: this build is a single-GPU kernel path; --gpus must be 1 "
              "(sharding over several GPUs is not part of it)", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import evospec_inputs as gi
    import paper_2605_27390_amd as ev

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    c = gi.CONFIGS[args.config]
    V, d, M, k = c["V"], c["d"], c["M"], c["k"]
    n_core, n_arc = c["n_core"], c["n_arc"]
    V_act = n_core + n_arc
    R = max(1, args.copies)
    K, Wm = args.steps, args.warmup

    def log(msg):
        print(f"[bench] {msg}", file=sys.stderr, flush=True)

    # ---------------------------------------------------------------- inputs (host -> HBM)
    t0 = time.time()
    W_lm_bits = gi.gen_W_lm(V, d)
    h_bits = gi.gen_h(M, d, gi.SEED_H + c["cfg"])
    ids0 = gi.active_ids(args.config)
    log(f"generated W_lm {W_lm_bits.shape}, h, ids in {time.time() - t0:.1f}s; "
        f"checksums W={gi.checksum(W_lm_bits):016x} h={gi.checksum(h_bits):016x} ids={gi.checksum(ids0):016x}")

    def dev_bf16(bits):
        return torch.from_numpy(bits.view(np.int16)).to(dev).view(torch.bfloat16)

    def new_matrix(rows, batch=None, layout=None):
        """An empty compact matrix (or `batch` of them) in the benchmark's layout."""
        if (layout or args.layout) == "packed":
            return ev.PackedMatrix(rows, d, device=dev, batch=batch)
        shape = (rows, d) if batch is None else (batch, rows, d)
        return torch.empty(shape, dtype=torch.bfloat16, device=dev)

    W_lm = dev_bf16(W_lm_bits)
    h = dev_bf16(h_bits)
    ids_dev = torch.from_numpy(ids0).to(dev)
    W_acts = [new_matrix(V_act) for _ in range(R)]
    act_ids = [torch.empty((V_act,), dtype=torch.int32, device=dev) for _ in range(R)]
    for r in range(R):
        ev.active_gather(W_lm, ids_dev, None, W_acts[r], act_ids[r])      # full rebuild = the same call
    # the sequence of dynamic-buffer updates every copy goes through (host bookkeeping only)
    n_updates = (K + Wm) // R + 2
    upd_slots, upd_ids = [], []
    state = ids0.copy()
    if n_arc >= UPDATE_ROWS:
        for u in range(n_updates):
            s_, n_ = gi.arc_update(V, state, n_core, UPDATE_ROWS, seed=7000 + u)
            state[s_] = n_
            upd_slots.append(torch.from_numpy(s_).to(dev))
            upd_ids.append(torch.from_numpy(n_).to(dev))
    ws = torch.empty(ev.workspace_bytes(M, V_act, d, k), dtype=torch.uint8, device=dev)
    out_v = torch.empty((M, k), dtype=torch.float32, device=dev)
    out_i = torch.empty((M, k), dtype=torch.int32, device=dev)
    out_l = torch.empty((M,), dtype=torch.float32, device=dev)
    torch.cuda.synchronize()

    def step(i):
        # the head on copy r as the previous update left it, and this step's update of the same
        # copy applied behind it (seen by the copy's next step): two launches
        r = i % R
        if upd_slots:
            u = i // R
            ev.active_lmhead_topk_then_update(h, W_acts[r], act_ids[r], k, W_lm, upd_ids[u], upd_slots[u],
                                              out_v, out_i, out_l, ws)
        else:
            ev.active_lmhead_topk(h, W_acts[r], act_ids[r], k, out_v, out_i, out_l, ws)

    def step_separate(i):
        r = i % R
        u = i // R
        ev.active_gather(W_lm, upd_ids[u % len(upd_ids)], upd_slots[u % len(upd_ids)], W_acts[r], act_ids[r])
        ev.active_lmhead_topk(h, W_acts[r], act_ids[r], k, out_v, out_i, out_l, ws)

    # ---------------------------------------------------------------- timed region
    for i in range(Wm):
        step(i)
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for i in range(Wm, Wm + K):
        step(i)
    e1.record()
    torch.cuda.synchronize()
    wall_s = time.perf_counter() - t0
    ev_ms = e0.elapsed_time(e1)
    ms_per_step = wall_s * 1e3 / K
    us_step = ms_per_step * 1e3
    alg_bytes = algorithmic_bytes(V_act, d, M, k)

    # ---------------------------------------------------------------- dominant kernel alone
    # (the slab kernel that streams W_act; HIP events on the launch stream, same rotation)
    def timed(fn, iters, warm=10):
        for i in range(warm):
            fn(i)
        torch.cuda.synchronize()
        a = torch.cuda.Event(enable_timing=True)
        b = torch.cuda.Event(enable_timing=True)
        a.record()
        for i in range(iters):
            fn(i)
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e3 / iters          # us

    n_ev = max(20, min(K, 200))
    part_us = timed(lambda i: ev.active_lmhead_partials(h, W_acts[i % R], act_ids[i % R], k, ws), n_ev)
    merge_us = timed(lambda i: ev.active_lmhead_merge(M, V_act, d, k, out_v, out_i, out_l, ws), n_ev)
    head_us = timed(lambda i: ev.active_lmhead_topk(h, W_acts[i % R], act_ids[i % R], k, out_v, out_i, out_l, ws), n_ev)
    roof = {
        "kernel": "lmhead_partials_kernel",
        "bound": "hbm",
        "achieved": round(alg_bytes / part_us / 1e3, 1),       # GB/s
        "peak": HBM_PEAK_GBPS,
        "unit": "GB/s",
        "frac": round(alg_bytes / part_us / 1e3 / HBM_PEAK_GBPS, 4),
        "traffic": None,
        "avg_kernel_us": round(part_us, 2),
        "algorithmic_bytes": alg_bytes,
    }
    # HBM bytes per launch from the rocprofv3 FETCH_SIZE / WRITE_SIZE passes recorded under profiles/ (a
    # counter pass cannot run inside this process); not measured in this run, so the line says where it is from
    tfile = os.path.join(ROOT, "profiles", f"hbm_traffic_{args.config}.json")
    if os.path.exists(tfile):
        try:
            tj = json.load(open(tfile))
            roof["traffic"] = tj.get("bytes_per_launch")
            roof["traffic_source"] = f"profiles/hbm_traffic_{args.config}.json: rocprofv3 --pmc passes of {tj.get('kernel')}, not this run"
        except Exception:
            pass

    extra = {"layout": args.layout, "partials_us": round(part_us, 2), "merge_us": round(merge_us, 2), "head_us": round(head_us, 2),
             "event_us_per_step": round(ev_ms * 1e3 / K, 2), "copies": R,
             "rows_per_s": round(M / (us_step * 1e-6), 1),
             "hbm_gbps_step": round(alg_bytes / us_step / 1e3, 1),
             "hbm_frac_step": round(alg_bytes / us_step / 1e3 / HBM_PEAK_GBPS, 4)}
    if "core" in sections and args.config == "draft60":
        # cache-warm figure (one copy), update kernels alone, and the unpruned head on the same GPU
        extra["head_us_cache_warm"] = round(timed(
            lambda i: ev.active_lmhead_topk(h, W_acts[0], act_ids[0], k, out_v, out_i, out_l, ws), n_ev), 2)
        # a decode loop re-reads ONE W_act every step: the same kernel without the rotation over copies
        # (part of the 302 MB then comes from the 256 MB memory-side cache, so this is not an HBM figure)
        one_us = timed(lambda i: ev.active_lmhead_partials(h, W_acts[0], act_ids[0], k, ws), n_ev)
        extra["single_copy"] = {"partials_us": round(one_us, 2),
                                "bytes_per_s_over_hbm_peak": round(alg_bytes / one_us / 1e3 / HBM_PEAK_GBPS, 4)}
        if upd_slots:
            extra["single_copy"]["step_us"] = round(timed(
                lambda i: ev.active_lmhead_topk_then_update(h, W_acts[0], act_ids[0], k, W_lm, upd_ids[0], upd_slots[0],
                                                            out_v, out_i, out_l, ws), n_ev), 2)
        if upd_slots:
            extra["step_us_separate_calls"] = round(timed(step_separate, n_ev), 2)
            extra["gather32_us"] = round(timed(
                lambda i: ev.active_gather(W_lm, upd_ids[0], upd_slots[0], W_acts[0], act_ids[0]), n_ev), 2)
        if upd_slots:
            # the same step replayed from a HIP graph (one graph = one step on each W_act copy)
            try:
                side = torch.cuda.Stream()
                side.wait_stream(torch.cuda.current_stream())
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.stream(side):
                    with torch.cuda.graph(graph, stream=side):
                        for r in range(R):
                            ev.active_lmhead_topk_then_update(h, W_acts[r], act_ids[r], k, W_lm, upd_ids[0], upd_slots[0],
                                                              out_v, out_i, out_l, ws)
                torch.cuda.current_stream().wait_stream(side)
                extra["step_us_graph_replay"] = round(timed(lambda i: graph.replay(), max(5, n_ev // R), warm=3) / R, 2)
                del graph
            except Exception as exc:                      # reported, never fatal for the benchmark line
                extra["step_us_graph_replay"] = f"failed: {type(exc).__name__}"
        extra["gather_full_us"] = round(timed(
            lambda i: ev.active_gather(W_lm, ids_dev, None, W_acts[i % R], act_ids[i % R]), 20, warm=3), 2)
        # the same head on a row-major copy of W_act (what a caller's own matrix would be)
        other = "row_major" if args.layout == "packed" else "packed"
        W_other = [new_matrix(V_act, layout=other) for _ in range(R)]
        ids_other = [torch.empty_like(act_ids[0]) for _ in range(R)]
        for r in range(R):
            ev.active_gather(W_lm, ids_dev, None, W_other[r], ids_other[r])
        extra[f"partials_us_{other}"] = round(timed(
            lambda i: ev.active_lmhead_partials(h, W_other[i % R], ids_other[i % R], k, ws), n_ev), 2)
        extra[f"gather_full_us_{other}"] = round(timed(
            lambda i: ev.active_gather(W_lm, ids_dev, None, W_other[i % R], ids_other[i % R]), 20, warm=3), 2)
        del W_other, ids_other
        ws_full = torch.empty(ev.workspace_bytes(M, V, d, k), dtype=torch.uint8, device=dev)
        full_us = timed(lambda i: ev.active_lmhead_topk(h, W_lm, None, k, out_v, out_i, out_l, ws_full), 30, warm=5)
        extra["fullvocab_head_us"] = round(full_us, 2)
        extra["speedup_vs_fullvocab"] = round(full_us / head_us, 3)
        extra["fullvocab_hbm_gbps"] = round(algorithmic_bytes(V, d, M, k) / full_us / 1e3, 1)
        # the unpruned head given the same advantage: all of W_lm copied into the packed layout
        W_full_p = ev.PackedMatrix(V, d, device=dev)
        ids_full = torch.empty((V,), dtype=torch.int32, device=dev)
        ev.active_gather(W_lm, torch.arange(V, dtype=torch.int32, device=dev), None, W_full_p, ids_full)
        full_p_us = timed(lambda i: ev.active_lmhead_topk(h, W_full_p, None, k, out_v, out_i, out_l, ws_full), 30, warm=5)
        extra["fullvocab_head_us_packed"] = round(full_p_us, 2)
        extra["speedup_vs_fullvocab_packed"] = round(full_p_us / head_us, 3)
        del ws_full, W_full_p, ids_full
    if "depth" in sections and args.config == "draft60":
        # per-depth tree expansion: 16,384 core + 2,048 ARC ids, M in {1, 4, 8}, and a 256-row update
        cd = gi.CONFIGS["depth"]
        ids_d = gi.active_ids("depth")
        Vd = ids_d.shape[0]
        ids_d_dev = torch.from_numpy(ids_d).to(dev)
        Wd = [new_matrix(Vd) for _ in range(8)]
        idd = [torch.empty((Vd,), dtype=torch.int32, device=dev) for _ in range(8)]
        for r in range(8):
            ev.active_gather(W_lm, ids_d_dev, None, Wd[r], idd[r])
        s_, n_ = gi.arc_update(V, ids_d, cd["n_core"], cd["update_rows"], seed=7100)
        s_dev, n_dev = torch.from_numpy(s_).to(dev), torch.from_numpy(n_).to(dev)
        depth = {"gather256_us": round(timed(lambda i: ev.active_gather(W_lm, n_dev, s_dev, Wd[i % 8], idd[i % 8]), n_ev), 2)}
        for Md in cd["Ms"]:
            hd = dev_bf16(gi.gen_h(Md, d, gi.SEED_H + 30 + Md))
            ov_, oi_, ol_ = (torch.empty((Md, k), dtype=torch.float32, device=dev),
                             torch.empty((Md, k), dtype=torch.int32, device=dev),
                             torch.empty((Md,), dtype=torch.float32, device=dev))
            us = timed(lambda i: ev.active_lmhead_topk(hd, Wd[i % 8], idd[i % 8], k, ov_, oi_, ol_, ws), n_ev)
            depth[f"head_us_M{Md}"] = round(us, 2)
            depth[f"hbm_gbps_M{Md}"] = round(algorithmic_bytes(Vd, d, Md, k) / us / 1e3, 1)
        extra["depth_V18432"] = depth
        del Wd, idd
    if "batched" in sections and args.config == "draft60":
        # batched serving: 16 sequences x 60 rows, shared 32,768-id core + 2,048 ARC ids per sequence
        cb = gi.CONFIGS["batched"]
        core_b, arcs_b = gi.batched_ids(V, cb["n_core"], cb["n_arc"], cb["S"])
        Mb, S_, Va = cb["M"], cb["S"], cb["n_arc"]
        W_core = new_matrix(cb["n_core"])
        ids_core = torch.empty((cb["n_core"],), dtype=torch.int32, device=dev)
        ev.active_gather(W_lm, torch.from_numpy(core_b).to(dev), None, W_core, ids_core)
        W_arc = new_matrix(Va, batch=S_)
        ids_arc = torch.empty((S_ * Va,), dtype=torch.int32, device=dev)
        for s_i in range(S_):
            ev.active_gather(W_lm, torch.from_numpy(arcs_b[s_i].copy()).to(dev), None,
                             W_arc.sub(s_i) if args.layout == "packed" else W_arc[s_i],
                             ids_arc[s_i * Va:(s_i + 1) * Va])
        hb = dev_bf16(gi.gen_h(Mb, d, gi.SEED_H + 5))
        row_off = [s * cb["rows_per_seq"] for s in range(S_ + 1)]
        ws_b = torch.empty(ev.workspace_bytes_segmented(Mb, cb["n_core"], Va, S_, d, k), dtype=torch.uint8, device=dev)
        seg_us = timed(lambda i: ev.active_lmhead_topk_segmented(hb, W_core, ids_core, W_arc,
                                                                 ids_arc.view(S_, Va), row_off, k, ws_b), 10, warm=2)
        flops = 2.0 * d * (Mb * cb["n_core"] + Mb * Va)
        extra["batched_M960"] = {"head_us": round(seg_us, 1), "tflops": round(flops / seg_us / 1e6, 1),
                                 "mfma_frac_bf16": round(flops / seg_us / 1e6 / 2500.0, 4),
                                 "rows_per_s": round(Mb / (seg_us * 1e-6), 1)}
        del W_core, W_arc, ws_b

    if "host" in sections and args.config == "draft60":
        # the step before the path: the C++ dynamic-buffer manager (paper defaults) on a stream of
        # failure events with Zipf-distributed candidates (20 seeds + up to 8 successors each, as
        # the appendix forms them), and the gather it drives with its own update sizes
        core_ids = ids0[:n_core]
        arc = ev.ArcManager(slot_base=n_core, core=core_ids)
        rng = np.random.default_rng(99)
        wz = gi.zipf_weights(V)
        wz = wz / wz.sum()
        perm = gi.zipf_ranking(V, gi.SEED_IDS + c["cfg"])
        n_events = 2000
        cand_lists = [perm[rng.choice(V, size=int(rng.integers(20, 181)), p=wz)].astype(np.int32) for _ in range(n_events)]
        sizes = []
        t0 = time.perf_counter()
        for cl in cand_lists:
            s_, i_ = arc.event_arrays(cl)
            sizes.append(int(s_.size))
            arc.advance(3)
        arc_s = time.perf_counter() - t0
        W_tmp = new_matrix(n_core + 256)
        I_tmp = torch.empty((n_core + 256,), dtype=torch.int32, device=dev)
        arc2 = ev.ArcManager(slot_base=n_core, core=core_ids)
        ups = []
        for cl in cand_lists[:200]:
            s_, i_ = arc2.event_arrays(cl)
            arc2.advance(3)
            if s_.size:
                ups.append((torch.from_numpy(s_.copy()).to(dev), torch.from_numpy(i_.copy()).to(dev)))
        g_us = timed(lambda i: ev.active_gather(W_lm, ups[i % len(ups)][1], ups[i % len(ups)][0], W_tmp, I_tmp), len(ups), warm=5)
        extra["arc_manager"] = {"events_per_s": round(n_events / arc_s, 1), "us_per_event": round(arc_s / n_events * 1e6, 2),
                                "mean_insertions_per_event": round(float(np.mean(sizes)), 2),
                                "max_insertions_per_event": int(max(sizes)), "gather_us_per_event": round(g_us, 2)}
        # a whole failure event of Path A: exact inner-product search over the full vocabulary
        # (M = 1, top 10), candidates from a synthetic co-occurrence graph, admission, gather
        row_ptr, col_idx = gi.bigram_graph(V, gi.SEED_IDS + 9)
        arc3 = ev.ArcManager(slot_base=n_core, core=core_ids)
        W_pa = new_matrix(n_core + 256)
        I_pa = torch.empty((n_core + 256,), dtype=torch.int32, device=dev)
        ws_pa = torch.empty(ev.path_a_workspace_bytes(V, d, 10, 32), dtype=torch.uint8, device=dev)
        h_t = [dev_bf16(gi.gen_h(1, d, gi.SEED_H + 100 + j)) for j in range(8)]
        tt = [rng.integers(0, V, 10).astype(np.int32) for _ in range(8)]
        n_pa = 60
        for j in range(5):
            ev.path_a_event(arc3, h_t[j % 8], W_lm, tt[j % 8], 10, row_ptr, col_idx, 8, W_pa, I_pa, ws_pa)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for j in range(n_pa):
            ev.path_a_event(arc3, h_t[j % 8], W_lm, tt[j % 8], 10, row_ptr, col_idx, 8, W_pa, I_pa, ws_pa)
            arc3.advance(3)
        torch.cuda.synchronize()
        extra["path_a_event_us"] = round((time.perf_counter() - t0) / n_pa * 1e6, 1)
        del W_pa, I_pa, ws_pa
        # Path B admission gate: 60 verification events, top-256 support over the full vocabulary
        E_kl = 60
        z_t = torch.randn((E_kl, V), dtype=torch.float32, device=dev) * 2.0
        h_kl = dev_bf16(gi.gen_h(E_kl, d, gi.SEED_H + 70))
        kl_out = ev.kl_gate(z_t, h_kl, W_lm, 256, 1.0)
        ws_kl = torch.empty(ev.kl_gate_workspace_bytes(E_kl, V), dtype=torch.uint8, device=dev)
        kl_us = timed(lambda i: ev.kl_gate(z_t, h_kl, W_lm, 256, 1.0, *kl_out, ws_kl), 30, warm=3)
        extra["kl_gate_60x256_us"] = round(kl_us, 1)
        del z_t
        if not args.no_cpu_baseline:
            import oracle
            ref = oracle.ArcOracle(slot_base=n_core, core=core_ids)
            t0 = time.perf_counter()
            for cl in cand_lists[:300]:
                ref.event(cl)
                ref.advance(3)
            extra["arc_manager"]["oracle_us_per_event"] = round((time.perf_counter() - t0) / 300 * 1e6, 2)
        del W_tmp, I_tmp

    if "sweep" in sections and args.config == "draft60":
        # the paper's own active-set sizes (Table 1 and the default setting), same rotation rule:
        # enough copies of W_act that the weights come from HBM
        sweep = []
        W_by_shape = {(V, d): W_lm}
        for name, d_s, V_s, nc, na, M_s, k_s in gi.SWEEP:
            if (V_s, d_s) not in W_by_shape:
                W_by_shape[(V_s, d_s)] = dev_bf16(gi.gen_W_lm(V_s, d_s, gi.SEED_W + 1))
            Wl = W_by_shape[(V_s, d_s)]
            core_s, arc_s = gi.core_arc_ids(V_s, nc, na, gi.SEED_IDS + 40)
            ids_s = torch.from_numpy(np.concatenate([core_s, arc_s])).to(dev)
            Va = nc + na
            Rs = max(2, int(-(-4 * 256e6 // (Va * d_s * 2))))
            Ws = [ev.PackedMatrix(Va, d_s, device=dev) if args.layout == "packed" else
                  torch.empty((Va, d_s), dtype=torch.bfloat16, device=dev) for _ in range(Rs)]
            Is = [torch.empty((Va,), dtype=torch.int32, device=dev) for _ in range(Rs)]
            for r in range(Rs):
                ev.active_gather(Wl, ids_s, None, Ws[r], Is[r])
            h_s = dev_bf16(gi.gen_h(M_s, d_s, gi.SEED_H + 60))
            ws_s = torch.empty(ev.workspace_bytes(M_s, Va, d_s, k_s), dtype=torch.uint8, device=dev)
            ov_s = torch.empty((M_s, k_s), dtype=torch.float32, device=dev)
            oi_s = torch.empty((M_s, k_s), dtype=torch.int32, device=dev)
            ol_s = torch.empty((M_s,), dtype=torch.float32, device=dev)
            us = timed(lambda i: ev.active_lmhead_topk(h_s, Ws[i % Rs], Is[i % Rs], k_s, ov_s, oi_s, ol_s, ws_s), 100)
            ws_f = torch.empty(ev.workspace_bytes(M_s, V_s, d_s, k_s), dtype=torch.uint8, device=dev)
            full = timed(lambda i: ev.active_lmhead_topk(h_s, Wl, None, k_s, ov_s, oi_s, ol_s, ws_f), 20, warm=3)
            sweep.append({"name": name, "d": d_s, "V": V_s, "V_act": Va, "M": M_s, "copies": Rs,
                          "head_us": round(us, 2),
                          "hbm_gbps": round(algorithmic_bytes(Va, d_s, M_s, k_s) / us / 1e3, 1),
                          "fullvocab_head_us": round(full, 2), "speedup_vs_fullvocab": round(full / us, 2)})
            del Ws, Is, ws_s, ws_f
        extra["sweep"] = sweep

    # ---------------------------------------------------------------- CPU oracle on the host cores
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        # the state of copy 0 after the timed steps is whatever it is: re-run one head on a fresh
        # copy of the initial active set so that GPU output and oracle see the same rows
        ev.active_gather(W_lm, ids_dev, None, W_acts[0], act_ids[0])
        ev.active_lmhead_topk(h, W_acts[0], act_ids[0], k, out_v, out_i, out_l, ws)
        torch.cuda.synchronize()
        gv, gi_, gl = out_v.cpu().numpy(), out_i.cpu().numpy(), out_l.cpu().numpy()
        W_act_host = W_lm_bits[ids0]
        t0 = time.perf_counter()
        ov, oi, ol = oracle.active_lmhead_topk(h_bits, W_act_host, ids0, k + 1)
        cpu_s = time.perf_counter() - t0
        cpu = {"value": round(cpu_s * 1e6, 1), "unit": "us/step", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": f"one full head step (all {V_act} active rows x {M} draft rows, fp64), no gather"}
        gap = np.abs(ov[:, k - 1] - ov[:, k]) / np.maximum(np.abs(ov[:, k - 1]), np.abs(ov[:, k]))
        clear = gap > 1e-3
        same = np.array([set(gi_[m]) == set(oi[m, :k]) for m in range(M)])
        extra["parity"] = {
            "logz_max_rel_err": float(np.max(np.abs(gl - ol) / np.abs(ol))),
            "top1_max_abs_err": float(np.max(np.abs(gv[:, 0] - ov[:, 0]))),
            "rows_with_clear_gap": int(clear.sum()),
            "id_sets_equal_on_clear_rows": bool(np.all(same[clear])),
            "near_tie_rows_exempt": int((~clear).sum()),
        }

    line = {
        "metric": METRIC if args.config == "draft60" else f"active LM-head+top-k us/step ({args.config})",
        "value": round(us_step, 2),
        "unit": "us/step",
        "n_gpus": 1,
        "steps": K,
        "warmup": Wm,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{args.config}: d={d}, V={V}, V_act={V_act} ({n_core} core + {n_arc} ARC), M={M}, k={k}, "
                               f"{UPDATE_ROWS if upd_slots else 0}-row ARC update per step, W_act {args.layout}"},
        "roofline": roof,
        "cpu_baseline": cpu,
        "extra": extra,
    }
    print(json.dumps(line), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
