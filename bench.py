#!/usr/bin/env python3
"""Benchmark of the search-space evaluator on one MI355X.

A step is one pass of the whole hot path over the resident, cell-sorted trace: per-cell
aggregation + rank selection, evaluation of every (cell, configuration) pair, per-cell
least-cost feasible configuration and per-window totals.  By default this is one call of
dyn_eval_select (selection reduced inside the evaluation kernel); --unfused times
dyn_eval_space followed by dyn_select_config instead.  Ingestion and profile upload are
timed separately.  Other entry points have modes of their own, each on the same workload and
with the same JSON line: --ticks T (load followed tick by tick inside a window), --mixed S
(pools that mix TP degrees), --path (selection with transition overheads between windows),
--hierarchy T [--overheads] [--spill] (the three controllers top down).
The headline mode also reports `pipelined`: the same steps with consecutive steps on alternating streams.

Prints one JSON line.  `value` = requests x configurations / step time.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X HBM3E, published peak
FP64_VECTOR_PEAK_TFLOPS = 78.6   # MI355X fp64 vector (FMA counted as two), published peak
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "space_kernel_traffic.json")


def kernel_source_hash():
    """Hash of the sources the space kernel is built from; the recorded HBM traffic is only
    reported while it still describes the kernel as it stands."""
    import hashlib
    h = hashlib.sha256()
    for name in ("k_space.hip", "dyn_internal.h"):
        with open(os.path.join(ROOT, "paper_2408_00741_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def recorded_traffic(workload_index):
    """HBM bytes per launch of the space kernel from the committed rocprofv3 counter runs, or None."""
    try:
        with open(TRAFFIC_FILE) as f:
            rec = json.load(f)
        if rec.get("source_hash") == kernel_source_hash() and rec.get("config") == workload_index:
            return rec.get("hbm_bytes_per_launch")
    except (OSError, ValueError):
        pass
    return None


def cpu_baseline(w, n_sample_windows, ticks=0, mixed=None, path=None, hier=None):
    """The CPU oracle, as it stands, on the first windows of the same workload (one thread)."""
    import numpy as np
    import oracle
    tr = w["trace"]
    hi = int(np.searchsorted(tr["t_s"], n_sample_windows * w["window_s"]))
    sub = {k: v[:hi] for k, v in tr.items()}
    k = w["configs"]["n_inst"].size
    if hier:
        T, epoch, tp_ref, f_ref, gpn, lay_n, lay_tp, trans, spill, k = hier
        st = oracle.ingest(sub, w["edges"], n_sample_windows, w["window_s"])
        fine = oracle.ingest(sub, w["edges"], n_sample_windows * T, w["window_s"] / T)
        t0 = time.perf_counter()
        oracle.hierarchy(w["profile"], st, fine, n_sample_windows, T, w["window_s"] / T, epoch, tp_ref, f_ref, gpn, lay_n, lay_tp,
                         w["slos"], w["pct"], transition=trans, spill=spill)
    elif mixed:
        n_share, n_max, budget, k = mixed
        st = oracle.ingest(sub, w["edges"], n_sample_windows, w["window_s"])
        t0 = time.perf_counter()
        oracle.mixed(w["profile"], st, n_sample_windows, w["window_s"], n_share, n_max, w["slos"], w["pct"], budget)
    elif ticks:
        st = oracle.ingest(sub, w["edges"], n_sample_windows * ticks, w["window_s"] / ticks)
        t0 = time.perf_counter()
        oracle.evaluate_ticks(w["profile"], st, n_sample_windows, ticks, w["window_s"] / ticks, w["configs"], w["slos"],
                              w["pct"], None, w["idle_cost_weight"])
    elif path:
        st = oracle.ingest(sub, w["edges"], n_sample_windows, w["window_s"])
        t0 = time.perf_counter()
        r = oracle.evaluate(w["profile"], st, n_sample_windows, w["window_s"], w["configs"], w["slos"], w["pct"], None,
                            w["idle_cost_weight"])
        oracle.select_path(r["cost"], (r["flags"] & 1).astype(np.uint8), n_sample_windows, w["n_class"], path[0], path[1])
    else:
        st = oracle.ingest(sub, w["edges"], n_sample_windows, w["window_s"])
        t0 = time.perf_counter()
        oracle.evaluate(w["profile"], st, n_sample_windows, w["window_s"], w["configs"], w["slos"], w["pct"], None,
                        w["idle_cost_weight"], want_space=False)
    dt = time.perf_counter() - t0
    return {"value": hi * k / dt, "unit": "evals/s", "cores": 1, "kind": "oracle",
            "sample": f"first {n_sample_windows} of {w['n_window']} windows ({hi} requests x {k} configurations, "
                      f"{dt:.1f} s, single thread)"}


def oracle_every_cell(w, gpu_sorted, gpu_sel):
    """The oracle over EVERY cell of the workload, its windows dealt to the host's cores (each task is one plain call of
    the single-threaded oracle), on the oracle's own ingestion of the raw trace; then the GPU's selections against it.
    Returns (all-core baseline entry, parity entry)."""
    import numpy as np
    import oracle
    NW, G, k = w["n_window"], w["n_class"], w["configs"]["n_inst"].size
    st = oracle.ingest(w["trace"], w["edges"], NW, w["window_s"])
    same_trace = all(np.array_equal(gpu_sorted[i], st[n]) for i, n in enumerate(("in_tok", "out_tok", "cell_off")))
    t0 = time.perf_counter()
    o = oracle.evaluate_parallel(w["profile"], st, NW, w["window_s"], w["configs"], w["slos"], w["pct"], None,
                                 w["idle_cost_weight"])
    dt = time.perf_counter() - t0
    R = w["trace"]["t_s"].size
    allcores = {"value": R * k / dt, "unit": "evals/s", "cores": o["threads"], "kind": "oracle",
                "sample": f"all {NW} windows ({R} requests x {k} configurations, {dt:.1f} s, windows dealt to "
                          f"{o['threads']} threads)"}
    bad = np.nonzero(gpu_sel["sel"] != o["sel"])[0]
    excused = 0
    if bad.size:       # ties within 1e-9 relative among oracle-feasible candidates are the stated tolerance
        ob = oracle.evaluate(w["profile"], st, NW, w["window_s"], w["configs"], w["slos"], w["pct"], None,
                             w["idle_cost_weight"], cell_ids=bad.astype(np.int64))
        for i, c in enumerate(bad):
            kg, ko = int(gpu_sel["sel"][c]), int(o["sel"][c])
            if kg >= 0 and ko >= 0 and (ob["flags"][i, kg] & 1) and \
                    abs(ob["cost"][i, kg] - ob["cost"][i, ko]) <= 1e-9 * abs(ob["cost"][i, ko]):
                excused += 1
    same = gpu_sel["sel"] == o["sel"]
    fin = same & (o["sel"] >= 0)
    rel = np.abs(gpu_sel["sel_energy_j"][fin] - o["sel_energy_j"][fin]) / np.abs(o["sel_energy_j"][fin])
    we, wi = oracle.window_totals(o["sel"], o["sel_energy_j"], NW, G)
    parity = {"cells": int(o["sel"].size), "sel_mismatch": int(bad.size), "excused": excused,
              "sel_energy_max_rel_err": float(rel.max()) if rel.size else 0.0,
              "sel_energy_bit_equal": bool(np.array_equal(gpu_sel["sel_energy_j"][same], o["sel_energy_j"][same])),
              "window_energy_bit_equal": bool(np.array_equal(gpu_sel["window_energy_j"], we)),
              "window_infeasible_equal": bool(np.array_equal(gpu_sel["window_infeasible"], wi)),
              "gpu_ingest_equals_oracle_ingest": bool(same_trace),
              "oracle": "every cell, on the oracle's own ingestion of the raw trace"}
    return allcores, parity


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=2, help="workload index (0..4); the headline is 2")
    ap.add_argument("--unfused", action="store_true", help="dyn_eval_space + dyn_select_config as two calls")
    ap.add_argument("--ticks", type=int, default=0,
                    help="tick-level variant: split every window into this many ticks (dyn_eval_select_ticks); "
                         "0 = the window-level headline path")
    ap.add_argument("--mixed", type=int, default=0,
                    help="mixed-pool search (dyn_eval_select_mixed) with this many load shares; per type up to "
                         "--mixed-gpus / TP instances, and a budget of --mixed-gpus GPUs per class")
    ap.add_argument("--mixed-gpus", type=int, default=32)
    ap.add_argument("--path", action="store_true",
                    help="dyn_eval_space + dyn_select_path: selection with transition overheads between consecutive "
                         "windows (layout = (TP, instances); overhead = 1 %% of the median selected energy per GPU "
                         "of difference between the layouts)")
    ap.add_argument("--hierarchy", type=int, default=0,
                    help="the three controllers top down (dyn_hierarchy) with this many ticks per window: epochs of "
                         "--epoch-windows windows, 8-GPU nodes, layouts = the (instances, TP) pairs of the workload's "
                         "configurations, reference = the largest TP at the highest frequency")
    ap.add_argument("--epoch-windows", type=int, default=6)
    ap.add_argument("--spill", action="store_true",
                    help="with --hierarchy: the scale-out controller applies the fragmentation rule; the profile's "
                         "capacities are scaled so that the busiest pool needs --peak-nodes nodes (the generated "
                         "profile leaves most pools below one node, where the rule has nothing to do)")
    ap.add_argument("--peak-nodes", type=float, default=6.5)
    ap.add_argument("--overheads", action="store_true",
                    help="with --hierarchy: the shard controller weighs re-sharding overheads (2 %% of the median window "
                         "energy per GPU of difference between two layouts)")
    ap.add_argument("--pipelined-streams", type=int, default=2,
                    help="headline mode only: after the timed region, the same number of steps once more with consecutive "
                         "steps alternating between this many streams and output sets (reported as `pipelined`, never as "
                         "`value`); 0 or 1 = skip")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--checksums", action="store_true",
                    help="add order-sensitive 64-bit checksums of every generated input array to the line (`inputs`)")
    ap.add_argument("--no-tune", action="store_true",
                    help="skip dyn_eval_tune in the set-up (the library's rule then picks the evaluation kernel's block shape)")
    ap.add_argument("--no-kernel-events", action="store_true",
                    help="do not bracket kernels with HIP events (roofline.achieved is then null)")
    ap.add_argument("--cpu-windows", type=int, default=0, help="windows in the CPU-baseline sample (0 = auto)")
    ap.add_argument("--copy-reference", action="store_true",
                    help="only run five plain 256 MiB device-to-device copies (a kernel of known traffic, used to "
                         "scale the FETCH_SIZE / WRITE_SIZE readings of a rocprofv3 --pmc run) and exit")
    args = ap.parse_args()
    if args.copy_reference:
        import torch
        n = 256 * 1024 * 1024
        x = torch.ones(n, dtype=torch.uint8, device="cuda")
        y = torch.empty_like(x)
        torch.cuda.synchronize()
        for _ in range(5):
            y.copy_(x)
        torch.cuda.synchronize()
        print(json.dumps({"copy_reference_bytes": n, "copies": 5}))
        return
    if args.gpus != 1:
        print("bench.py measures one GPU: there is no multi-GPU path (windows would shard independently "
              "across GPUs, with the profile and the candidate list replicated). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2408_00741_amd as dyn
    from workloads import SPECS, make

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    spec = SPECS[args.config]
    t0 = time.perf_counter()
    w = make(spec)
    gen_s = time.perf_counter() - t0
    tr = w["trace"]
    R, K, NW, G = spec.n_req, spec.n_config, spec.n_window, spec.n_class
    cells = NW * G
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()

    # ---- one-time set-up, timed separately: upload, ingestion, profile load
    t_s, x, y, mdl = dev(tr["t_s"]), dev(tr["in_tok"]), dev(tr["out_tok"]), dev(tr["model"])
    T = max(args.ticks, args.hierarchy, 1)  # the trace is sorted by tick when ticks are asked for
    NWF, len_s = NW * T, w["window_s"] / T
    ws_ing = torch.empty(dyn.dyn_trace_ingest_workspace(R, NWF, G), dtype=torch.uint8, device="cuda")
    dyn.dyn_trace_ingest(t_s, x, y, mdl, w["edges"], NWF, len_s, workspace=ws_ing)   # warm-up
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    singles = []
    for _ in range(5):                     # single calls on an idle GPU: the median of five
        e0.record()
        ins, outs, off, _ = dyn.dyn_trace_ingest(t_s, x, y, mdl, w["edges"], NWF, len_s, workspace=ws_ing)
        e1.record()
        torch.cuda.synchronize()
        singles.append(e0.elapsed_time(e1))
    ingest_ms = sorted(singles)[2]
    e0.record()
    for _ in range(10):                    # the same call back to back: without the launch latency of an idle GPU
        dyn.dyn_trace_ingest(t_s, x, y, mdl, w["edges"], NWF, len_s, workspace=ws_ing)
    e1.record()
    torch.cuda.synchronize()
    ingest_ms_b2b = e0.elapsed_time(e1) / 10
    assert dyn.dyn_workspace_status(ws_ing) == 0
    if args.hierarchy:                      # the controllers also need the window-level order
        coarse = dyn.dyn_trace_ingest(t_s, x, y, mdl, w["edges"], NW, w["window_s"])[:3]
        if args.spill:                      # size the synthetic node capacities to pools of several nodes
            tok = torch.cat([torch.zeros(1, dtype=torch.int64, device="cuda"), torch.cumsum(coarse[0].long() + coarse[1].long(), 0)])
            load = ((tok[coarse[2][1:]] - tok[coarse[2][:-1]]).double() / w["window_s"]).reshape(NW, G).cpu().numpy()
            P = dict(w["profile"])
            cap = P["max_load_tps"][:, -1, -1] * P["rho"][-1]
            P["max_load_tps"] = P["max_load_tps"] * float((load / cap).max() / args.peak_nodes)
            w["profile"] = P
    del t_s, x, y, mdl, ws_ing
    t0 = time.perf_counter()
    prof = dyn.dyn_profile_load(w["profile"])
    profile_load_ms = (time.perf_counter() - t0) * 1e3
    plan = dyn.Plan(w["configs"], w["slos"], w["pct"], None, w["idle_cost_weight"])

    space = {"energy_j": torch.empty((cells, K), dtype=torch.float64, device="cuda"),
             "p99_ttft_ms": torch.empty((cells, K), dtype=torch.float64, device="cuda"),
             "p99_tbt_ms": torch.empty((cells, K), dtype=torch.float64, device="cuda"),
             "flags": torch.empty((cells, K), dtype=torch.uint8, device="cuda")}
    sel = {"sel": torch.empty(cells, dtype=torch.int32, device="cuda"),
           "sel_energy_j": torch.empty(cells, dtype=torch.float64, device="cuda"),
           "sel_cost": torch.empty(cells, dtype=torch.float64, device="cuda"),
           "window_energy_j": torch.empty(NW, dtype=torch.float64, device="cuda"),
           "window_infeasible": torch.empty(NW, dtype=torch.int32, device="cuda")}
    ws = torch.empty(dyn.dyn_eval_ticks_workspace(R, NW, T, G, K) if args.ticks else dyn.dyn_eval_space_workspace(NW, G, K),
                     dtype=torch.uint8, device="cuda")

    headline_mode = not (args.hierarchy or args.path or args.mixed or args.ticks or args.unfused)
    if args.hierarchy:
        assert not args.ticks and not args.mixed and not args.path, "--hierarchy is a mode of its own"
        cfgs = w["configs"]
        uniq = np.unique(cfgs["tp_index"].astype(np.int64) * 100000 + cfgs["n_inst"])
        lay_n, lay_tp = (uniq % 100000).astype(np.int32), (uniq // 100000).astype(np.int32)
        n_f = int(w["profile"]["f_mhz"].size)
        hier_args = (T, args.epoch_windows, int(w["profile"]["tp"].size) - 1, n_f - 1, 8, lay_n, lay_tp)
        K = int(lay_n.size) + n_f           # candidates looked at per request: layouts per window + frequencies per tick
        ws = torch.empty(dyn.dyn_hierarchy_workspace(NW, T, G, lay_n.size), dtype=torch.uint8, device="cuda")
        hout, _ = dyn.dyn_hierarchy(prof, coarse, (ins, outs, off), NW, T, len_s, *hier_args[1:], w["slos"], w["pct"], workspace=ws)
        nodes_plain = int(hout["nodes"].sum().item())
        hout["window_energy_j"], hout["window_infeasible"] = sel["window_energy_j"], sel["window_infeasible"]
        hier_trans = None
        if args.overheads:
            e0 = hout["energy_j"][torch.isfinite(hout["energy_j"])]
            gpus = lay_n.astype(np.int64) * w["profile"]["tp"][lay_tp]
            hier_trans = 0.02 * float(e0.median()) * np.abs(gpus[:, None] - gpus[None, :]).astype(np.float64)
            hout["path_cost"] = torch.empty(G, dtype=torch.float64, device="cuda")

        def step():
            dyn.dyn_hierarchy(prof, coarse, (ins, outs, off), NW, T, len_s, *hier_args[1:], w["slos"], w["pct"], out=hout,
                              workspace=ws, transition_j=hier_trans, spill=args.spill)
    elif args.path:
        assert not args.ticks and not args.mixed, "--path, --mixed and --ticks are separate modes"
        cfgs = w["configs"]
        key = cfgs["tp_index"].astype(np.int64) * 100000 + cfgs["n_inst"]
        uniq, lay = np.unique(key, return_inverse=True)
        lay = lay.astype(np.int32)
        gpus = w["profile"]["tp"][uniq // 100000].astype(np.int64) * (uniq % 100000)
        dyn.dyn_eval_space(prof, ins, outs, off, NW, w["window_s"], plan, out=space, workspace=ws)
        e0 = dyn.dyn_select_config(prof, space, NW, w["window_s"], plan)["sel_energy_j"]
        e0 = e0[torch.isfinite(e0)]
        unit_j = float(e0.median()) * 0.01 if e0.numel() else 1.0
        trans = unit_j * np.abs(gpus[:, None] - gpus[None, :]).astype(np.float64)
        ws_path = torch.empty(dyn.dyn_select_path_workspace(NW, G, K, uniq.size), dtype=torch.uint8, device="cuda")
        psel = {"sel": sel["sel"], "sel_energy_j": sel["sel_energy_j"],
                "path_cost": torch.empty(G, dtype=torch.float64, device="cuda"),
                "window_energy_j": sel["window_energy_j"], "window_infeasible": sel["window_infeasible"]}

        def step():
            dyn.dyn_eval_space(prof, ins, outs, off, NW, w["window_s"], plan, out=space, workspace=ws)
            dyn.dyn_select_path(prof, space, NW, w["window_s"], plan, lay, trans, out=psel, workspace=ws_path)
    elif args.mixed:
        assert not args.ticks, "--mixed and --ticks are separate modes"
        tp = w["profile"]["tp"]
        n_max = [max(1, args.mixed_gpus // int(t)) for t in tp]
        mplan = dyn.MixedPlan(args.mixed, n_max, w["slos"], w["pct"], np.full(G, args.mixed_gpus, np.int32))
        ws = torch.empty(dyn.dyn_mixed_workspace(prof, NW, mplan), dtype=torch.uint8, device="cuda")
        msel = {"energy_j": torch.empty(cells, dtype=torch.float64, device="cuda"),
                "n_inst": torch.empty((cells, tp.size), dtype=torch.int32, device="cuda"),
                "f_index": torch.empty((cells, tp.size), dtype=torch.int32, device="cuda"),
                "share": torch.empty((cells, tp.size), dtype=torch.int32, device="cuda"),
                "window_energy_j": sel["window_energy_j"], "window_infeasible": sel["window_infeasible"]}
        n_entry = int(sum(n_max)) * args.mixed
        K = n_entry * int(w["profile"]["f_mhz"].size)     # (type, instances, shares, frequency) evaluated per cell

        def step():
            dyn.dyn_eval_select_mixed(prof, ins, outs, off, NW, w["window_s"], mplan, out=msel, workspace=ws)
    elif args.ticks:
        def step():
            dyn.dyn_eval_select_ticks(prof, ins, outs, off, NW, T, len_s, plan, out=space, sel=sel, workspace=ws)
    elif args.unfused:
        def step():
            dyn.dyn_eval_space(prof, ins, outs, off, NW, w["window_s"], plan, out=space, workspace=ws)
            dyn.dyn_select_config(prof, space, NW, w["window_s"], plan, out=sel)
    else:
        def step():
            dyn.dyn_eval_select(prof, ins, outs, off, NW, w["window_s"], plan, out=space, sel=sel, workspace=ws)

    tuned = None
    if (headline_mode or args.unfused) and not args.no_tune:
        # set-up, outside the timed region: the library times its evaluation kernel's block shapes on these buffers
        # and keeps the fastest (results do not depend on the shape)
        tuned = dyn.dyn_eval_tune(prof, ins, outs, off, NW, w["window_s"], plan, out=space, sel=sel, workspace=ws)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # ---- timed region: exactly `steps` steps between two device synchronisations
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall / args.steps * 1e3
    status = dyn.dyn_workspace_status(ws)
    assert status == 0, status

    # ---- the same step timed one by one with a pair of HIP events each, on the stream the kernels are launched on
    # (torch's current stream is the one the binding hands to the library): the median of at least 20 repetitions
    n_ev = max(args.steps, 20)
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_ev)]
    for e_a, e_b in pairs:
        e_a.record()
        step()
        e_b.record()
    torch.cuda.synchronize()
    per_step = sorted(e_a.elapsed_time(e_b) for e_a, e_b in pairs)
    ms_median = per_step[n_ev // 2]

    # ---- the same `steps` steps again with the library's per-kernel HIP events switched on (recorded
    # on the stream the kernels are launched on).  The event records themselves cost about 20 us per
    # step on this machine, which is why they are kept out of the throughput region above.
    ktime = {"cell": 0.0, "space": 0.0, "select": 0.0, "totals": 0.0, "tick_top": 0.0, "tick_space": 0.0, "tick_merge": 0.0,
             "mixed_types": 0.0, "mixed_combine": 0.0, "path": 0.0, "hierarchy": 0.0}
    ms_per_step_events = None
    if not args.no_kernel_events:
        dyn.dyn_timing_enable(True, args.steps)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        ms_per_step_events = (time.perf_counter() - t0) / args.steps * 1e3
        for name, kid in (("cell", dyn.DYN_K_CELL), ("space", dyn.DYN_K_SPACE), ("select", dyn.DYN_K_SELECT),
                          ("totals", dyn.DYN_K_TOTALS), ("tick_top", dyn.DYN_K_TICK_TOP),
                          ("tick_space", dyn.DYN_K_TICK_SPACE), ("tick_merge", dyn.DYN_K_TICK_MERGE),
                          ("mixed_types", dyn.DYN_K_MIXED_TYPES), ("mixed_combine", dyn.DYN_K_MIXED_COMBINE),
                          ("path", dyn.DYN_K_PATH), ("hierarchy", dyn.DYN_K_HIER)):
            ms, n = dyn.dyn_timing_read(kid)
            ktime[name] = ms / max(n, 1)
        dyn.dyn_timing_enable(False)

    # ---- the same steps with consecutive steps on alternating streams (own outputs and workspace each): one step's
    # aggregation and selection kernels then run beside another step's store-bound evaluation.  Reported next to the
    # single-stream figure; `value` stays the single-stream one.
    pipelined = None
    headline = not (args.hierarchy or args.path or args.mixed or args.ticks or args.unfused)
    if headline and args.pipelined_streams > 1:
        n_s = args.pipelined_streams
        sets = [(space, sel, ws)]
        for _ in range(n_s - 1):
            sets.append(({k: torch.empty_like(v) for k, v in space.items()}, {k: torch.empty_like(v) for k, v in sel.items()},
                         torch.empty_like(ws)))
        streams = [torch.cuda.Stream() for _ in range(n_s)]          # default priority

        def run(n):
            for i in range(n):
                sp, se, wk = sets[i % n_s]
                dyn.dyn_eval_select(prof, ins, outs, off, NW, w["window_s"], plan, out=sp, sel=se, workspace=wk,
                                    stream=streams[i % n_s])
        run(max(args.warmup, 2 * n_s))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run(args.steps)
        torch.cuda.synchronize()
        p_ms = (time.perf_counter() - t0) / args.steps * 1e3
        same = all(torch.equal(sets[0][1]["sel"], s_[1]["sel"]) and torch.equal(sets[0][0]["flags"], s_[0]["flags"]) for s_ in sets[1:])
        pipelined = {"streams": n_s, "ms_per_step": p_ms, "value": R * K / (p_ms * 1e-3), "unit": "evals/s",
                     "same_results_on_every_stream": bool(same)}
        del sets, streams

    # ---- what a plain fill of the same four output arrays reaches on this GPU (torch's fill kernel, 20 repetitions
    # after 3 warm-ups, HIP events): the practical ceiling for a kernel that only writes them
    fill_gbps = None
    if headline or args.unfused:
        def fill_all():
            for v_ in space.values():
                v_.fill_(0)
        keep_space = {k_: v_.clone() for k_, v_ in space.items()} if cells * K <= (1 << 26) else None
        for _ in range(3):
            fill_all()
        f0, f1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        f0.record()
        for _ in range(20):
            fill_all()
        f1.record()
        torch.cuda.synchronize()
        fill_gbps = 25.0 * cells * K * 20 / (f0.elapsed_time(f1) * 1e-3) / 1e9
        if keep_space is not None:
            for k_, v_ in keep_space.items():
                space[k_].copy_(v_)
            del keep_space
        else:
            step()                      # the outputs are read below
            torch.cuda.synchronize()

    # ---- roofline of the dominant kernel (space evaluation): 25 B written per (cell, configuration)
    space_bytes = 25.0 * cells * K
    space_ms = ktime["tick_space"] + ktime["tick_merge"] if args.ticks else ktime["space"]
    space_gbps = space_bytes / (space_ms * 1e-3) / 1e9 if space_ms > 0 else None
    # whole path, algorithmic bytes: read the request stream and offsets once, write the space,
    # re-read energy + flags for the selection, write the selection and the window totals
    path_bytes = (8.0 * R + 8.0 * (cells + 1) + 25.0 * cells * K + (9.0 * cells * K if (args.unfused or args.path) else 0.0)
                  + 20.0 * cells + 12.0 * NW + (8.0 * cells * (T - 1) if args.ticks else 0.0))
    path_gbps = path_bytes / (ms_per_step * 1e-3) / 1e9

    if args.hierarchy:
        # the two aggregations (by window and by tick) dominate: each reads the 8-byte request records once
        cell_ms = ktime["cell"]            # average over the two launches of a step
        gbps = 8.0 * R / (cell_ms * 1e-3) / 1e9 if cell_ms > 0 else None
        roofline = {"bound": "hbm", "kernel": "cell_aggregate_kernel (twice per step)", "achieved": gbps, "peak": HBM_PEAK_GBPS,
                    "unit": "GB/s", "frac": gbps / HBM_PEAK_GBPS if gbps else None, "traffic": None,
                    "algorithmic_bytes_per_launch": 8.0 * R, "avg_launch_ms": cell_ms}
        n_ep = -(-NW // args.epoch_windows)
        path_bytes = 2 * 8.0 * R + 8.0 * (cells + 1) * (T + 1) + 4.0 * cells * T + 16.0 * cells + 4.0 * n_ep * G + 12.0 * NW
        path_gbps = path_bytes / (ms_per_step * 1e-3) / 1e9
    elif args.mixed:
        # instruction-bound: the method's arithmetic is 18 fp64 operations per (cell, type, instances, shares,
        # frequency) look-up (share of the load, table look-up, energy, TTFT multiply)
        space_ms = ktime["mixed_types"]
        flops = 18.0 * cells * K
        tf = flops / (space_ms * 1e-3) / 1e12 if space_ms > 0 else None
        roofline = {"bound": "alu", "kernel": "mixed_type_kernel", "achieved": tf, "peak": FP64_VECTOR_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": tf / FP64_VECTOR_PEAK_TFLOPS if tf else None, "traffic": None,
                    "algorithmic_flops_per_launch": flops, "avg_launch_ms": space_ms}
        path_bytes = 8.0 * R + 8.0 * (cells + 1) + 2 * 9.0 * cells * n_entry + (8.0 + 12.0 * tp.size) * cells + 12.0 * NW
        path_gbps = path_bytes / (ms_per_step * 1e-3) / 1e9
    elif args.ticks:
        # instruction-bound: per (cell, configuration, tick) the method's arithmetic is 17 fp64 operations for the
        # table look-up and the energy term + 1 multiply for the tick's largest candidate
        flops = 18.0 * cells * K * T
        tf = flops / (space_ms * 1e-3) / 1e12 if space_ms > 0 else None
        roofline = {"bound": "alu", "kernel": "tick_tight_walk_kernel + tick_space_kernel + tick_general_kernel", "achieved": tf,
                    "peak": FP64_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": tf / FP64_VECTOR_PEAK_TFLOPS if tf else None, "traffic": None,
                    "algorithmic_flops_per_launch": flops, "avg_launch_ms": space_ms,
                    "hbm_gbps_of_the_same_launch": space_gbps}
    else:
        roofline = {"bound": "hbm", "kernel": "space_kernel", "achieved": space_gbps, "peak": HBM_PEAK_GBPS,
                    "unit": "GB/s", "frac": space_gbps / HBM_PEAK_GBPS if space_gbps else None,
                    "traffic": None if (args.unfused or args.path) else recorded_traffic(args.config),
                    "traffic_source": "profiles/space_kernel_traffic.json: FETCH_SIZE and WRITE_SIZE of two rocprofv3 --pmc runs of "
                                      "this command, scaled by a plain copy; null once the kernel's sources have changed since",
                    "algorithmic_bytes_per_launch": space_bytes, "avg_launch_ms": space_ms,
                    "plain_fill_of_the_same_arrays_gbps": fill_gbps,
                    "frac_of_plain_fill": (space_gbps / fill_gbps) if (space_gbps and fill_gbps) else None}

    if args.hierarchy:
        sel_h = hout["layout_sel"].cpu().numpy()
    elif args.mixed:
        en = msel["energy_j"].cpu().numpy()
        sel_h = np.where(np.isfinite(en), 0, -1)
    else:
        sel_h = sel["sel"].cpu().numpy()
    we = sel["window_energy_j"].cpu().numpy()
    out = {
        "metric": "(request x config) evals/sec at 1 MI355X; achieved HBM GB/s vs peak",
        "value": R * K / (ms_per_step * 1e-3),
        "unit": "evals/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f64",
        "data": "synthetic",
        "config": {"workload": f"configs[{args.config}] {spec.name}: {R} requests, {NW} windows x {G} classes = "
                               f"{cells} cells, {K} configurations", "requests": R, "cells": cells, "configs": K,
                   "ticks_per_window": args.ticks or args.hierarchy, "mixed_shares": args.mixed,
                   "entry_points": ("dyn_hierarchy" + ("+overheads" if args.overheads else "") + ("+spill" if args.spill else "")) if args.hierarchy else "dyn_eval_space+dyn_select_path" if args.path else "dyn_eval_select_mixed" if args.mixed else "dyn_eval_select_ticks" if args.ticks else
                                   "dyn_eval_space+dyn_select_config" if args.unfused else "dyn_eval_select"},
        "roofline": roofline,
        "ms_per_step_median": ms_median, "median_over_event_timed_steps": n_ev,
        "kernel_ms": ktime, "ms_per_step_with_kernel_events": ms_per_step_events, "pipelined": pipelined,
        "path": {"algorithmic_bytes": path_bytes, "gbps": path_gbps, "frac_of_hbm_peak": path_gbps / HBM_PEAK_GBPS},
        "setup": {"ingest_ms": ingest_ms, "ingest_ms_back_to_back": ingest_ms_b2b, "profile_load_ms": profile_load_ms, "generate_s": gen_s,
                  "ingest_requests_per_s": R / (ingest_ms * 1e-3), "tuned_windows_per_block": tuned},
        "result": {"workspace_status": status, "cells_without_feasible_config": int((sel_h < 0).sum()), "total_energy_wh": float(we.sum() / 3600.0)},
    }
    if args.hierarchy:
        out["result"]["nodes_over_all_epochs"] = int(hout["nodes"].sum().item())
        if args.spill:
            out["result"]["nodes_without_the_fragmentation_rule"] = nodes_plain
            out["config"]["peak_nodes"] = args.peak_nodes
    if args.checksums:
        from workloads import checksum
        out["inputs"] = {"seed": spec.seed,
                         **{f"trace.{k_}": f"{checksum(v_):016x}" for k_, v_ in tr.items()},
                         **{f"profile.{k_}": f"{checksum(v_):016x}" for k_, v_ in w["profile"].items()},
                         **{f"configs.{k_}": f"{checksum(v_):016x}" for k_, v_ in w["configs"].items()},
                         **{f"slos.{k_}": f"{checksum(v_):016x}" for k_, v_ in w["slos"].items()}}
        golden = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tests", "golden", "input_checksums.txt")
        rec = {tuple(l.split()[:2]): l.split()[2] for l in open(golden) if l.strip() and not l.startswith("#")}
        out["inputs"]["equal_to_the_recorded_checksums"] = all(
            rec.get((str(args.config), k_)) == v_ for k_, v_ in out["inputs"].items() if k_ != "seed")
    if not args.no_cpu_baseline:
        print("bench: GPU part done, timing the CPU oracle on a sample", file=sys.stderr, flush=True)
        nwin = args.cpu_windows or max(1, min(NW, int(NW * (5.0e9 if args.mixed else 1.5e9 if (args.path or args.ticks) else 1.0e10) / (R * K))))
        mixed = (args.mixed, n_max, np.full(G, args.mixed_gpus, np.int32), K) if args.mixed else None
        if args.hierarchy:
            nwin = args.cpu_windows or NW
        out["cpu_baseline"] = cpu_baseline(w, nwin, args.ticks, mixed, (lay, trans) if args.path else None,
                                           hier_args + (hier_trans, args.spill, K) if args.hierarchy else None)
        out["cpu_baseline"]["host_cores"] = os.cpu_count()
        if headline or args.unfused:   # the oracle over every cell on all cores; the selections of the timed steps against it
            gpu_sel = {k_: v.cpu().numpy() for k_, v in sel.items()}
            allc, par = oracle_every_cell(w, (ins.cpu().numpy(), outs.cpu().numpy(), off.cpu().numpy()), gpu_sel)
            out["cpu_baseline"]["allcores"] = allc
            out["parity"] = par
    prof.free()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
