"""Throughput of the fused `for` loop on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--configs C1,C2,...]

A step is one pass of the whole hot path: the fused loops of the five benchmark
configurations (merger, size-known vecbuilder, compacting vecbuilder, low- and
high-cardinality dictmerger, multi-builder loops) run back to back over
synthetic columns that are already resident in HBM.  Prints ONE JSON line:
value = total input bytes of a step / time of a step (GB/s), plus per-config
numbers, the operator-at-a-time GPU mode for comparison, the roofline of the
dominant kernel and the CPU oracle timed on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
CPU_SAMPLE_ROWS = {"C1": 1_000_000, "C2": 20_000_000, "C3": 100_000_000, "C4": 40_000_000, "C5": 40_000_000}


def median(xs):
    s = sorted(xs)
    return s[len(s) // 2]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--configs", default="C1,C2,C3,C4,C5")
    ap.add_argument("--scale", type=float, default=1.0, help="fraction of the full row counts (for quick checks)")
    ap.add_argument("--tune", default="", help='JSON of weld_tuning_t fields applied to every fused call, e.g. {"dict_strategy": 2}')
    ap.add_argument("--vecmerger-sweep", action="store_true",
                    help="also time the count-occurrences vecmerger program (1e8 32-bit keys) over vector sizes and strategies")
    ap.add_argument("--no-nested", action="store_true",
                    help="skip the nested-loop leg (one PageRank iteration over the synthetic power-law graph)")
    ap.add_argument("--no-unfused", action="store_true")
    ap.add_argument("--tune-launch", action="store_true",
                    help="before the warm-up, let weld_tune_launch pick each loop's persistent-grid size on its own data "
                         "(default: the library's own choice)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU; --gpus %d is not supported (the loop shards by "
                 "contiguous row ranges with one small exchange per builder, but no multi-GPU path is built)" % args.gpus)

    import torch
    from paper_1709_06416_amd import binding as wb
    from workloads import configs

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    names = [c for c in args.configs.split(",") if c]
    tune = json.loads(args.tune) if args.tune else None
    rows = {c: max(1, int(configs.FULL_ROWS[c] * args.scale)) for c in names}
    progs = {c: configs.PROGRAMS[c]() for c in names}
    cols = {c: configs.make_columns(c, rows[c], device="cuda") for c in names}
    torch.cuda.synchronize()
    in_bytes = {c: configs.IN_BYTES[c] * rows[c] for c in names}

    # --tune-launch: a loop that runs many times is tuned once on its own data (persistent-grid
    # size), outside the timed region, like its compilation.
    tunes, tuning_report = {}, {}
    for c in names:
        tunes[c] = tune
        if args.tune_launch:
            tunes[c], best_ms, default_ms = wb.tune_launch(progs[c], cols[c], tune=tune)
            tuning_report[c] = {"tune": tunes[c], "kernel_ms": round(best_ms, 4), "library_choice_ms": round(default_ms, 4)}
    loops = {c: wb.prepare(progs[c], tune=tunes[c]) for c in names}                  # marshalled once, like a host program would


    def drain(handles, collect=None):
        for c, r in handles:
            r.check()
            if collect is not None:
                collect[c]["call_ms"].append(r.elapsed_ms())
                collect[c]["kernel_ms"].append(r.kernel_ms())
                collect[c]["kernel"] = r.kernel_name()
                collect[c]["launches"] = r.kernel_count()
            r.free()

    # Steps are pipelined the way a host program that keeps evaluating would run them: the results of
    # a step are checked and freed while the GPU works on the next one, so the GPU does not idle
    # while the host wakes up from a wait and enqueues again (measured: 70 us per step).  Every
    # result of every step is checked and freed inside the timed region.
    def run(steps, collect=None):
        pending = None
        for _ in range(steps):
            cur = []
            for k, c in enumerate(names):
                cur.append((c, wb.fused_for(loops[c], cols[c])))                       # work is only enqueued
                if pending is not None and k == (len(names) - 1) // 2:
                    # the first half of this step is queued: look at the previous step now, so that the
                    # second half finds that step's blocks back in the pool (a dictionary's spill queues
                    # written to the addresses of the last step are still in the memory-side cache)
                    drain(pending, collect)
                    pending = None
            pending = cur
        if pending is not None:
            drain(pending, collect)

    run(args.warmup)
    stats = {c: {"call_ms": [], "kernel_ms": []} for c in names}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(args.steps, stats)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    total_in = sum(in_bytes.values())
    value = total_in / ms_per_step / 1e6

    per = {}
    for c in names:
        k = median(stats[c]["kernel_ms"])
        out_b = configs.OUT_BYTES[c] * rows[c]
        per[c] = {"rows": rows[c], "kernel": stats[c]["kernel"], "launches": stats[c]["launches"],
                  "call_ms": round(median(stats[c]["call_ms"]), 4), "kernel_ms": round(k, 4),
                  "kernel_ms_min": round(min(stats[c]["kernel_ms"]), 4),
                  "rows_per_s": rows[c] / k * 1e3, "input_GBps": round(in_bytes[c] / k / 1e6, 1),
                  "input_frac_of_hbm_peak": round(in_bytes[c] / k / 1e6 / HBM_PEAK_GBPS, 4),
                  "in_plus_out_GBps": round((in_bytes[c] + out_b) / k / 1e6, 1)}

    # ---- operator-at-a-time GPU mode, same columns (comparison arm)
    if not args.no_unfused:
        for c in names:
            ts, busy = [], []
            launches = 0
            for i in range(4):
                r = wb.fused_for(progs[c], cols[c], mode="unfused").check()
                if i:
                    ts.append(r.elapsed_ms())
                    busy.append(r.busy_ms())
                launches = r.kernel_count()
                r.free()
            # unfused_ms: first to last kernel, with the host waits an eager library has between operators (a
            # filter's length is read back before the next loop is sized); unfused_kernel_sum_ms: the GPU's own
            # time for the operator loops, without those waits - the ratio that fusion alone accounts for
            per[c]["unfused_ms"] = round(median(ts), 4)
            per[c]["unfused_kernel_sum_ms"] = round(median(busy), 4)
            per[c]["unfused_launches"] = launches
            per[c]["fused_speedup_over_unfused"] = round(median(ts) / per[c]["call_ms"], 2)
            per[c]["fused_speedup_over_unfused_kernel_sum"] = round(median(busy) / per[c]["call_ms"], 2)
        wb.lib.weld_pool_trim()

    # ---- a streaming-read kernel on this box (16-byte loads, the loops' own tile pattern, nothing else to
    # do): four launches per bracket so that the launch gap is not in the figure, best of six brackets.
    # It is a measured lower bound of what the memory system can deliver, not a ceiling: a loop whose
    # columns keep more bytes in flight can pass it, so `attainable_read_GBps` is the larger of the
    # probe and the fastest loop of this run.
    probe = torch.empty(1 << 30, dtype=torch.int32, device="cuda")
    probe.fill_(1)
    pts = []
    for _ in range(6):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _k in range(4):
            wb.probe_read(probe)
        e1.record()
        torch.cuda.synchronize()
        pts.append(e0.elapsed_time(e1) / 4)
    read_probe = probe.numel() * 4 / min(pts) / 1e6
    # plain copy of known size (1 GiB read + 1 GiB written): the kernel the HBM counters are scaled by
    dst = torch.empty_like(probe)
    cts = []
    for _ in range(4):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        wb.probe_copy(dst, probe)
        e1.record()
        torch.cuda.synchronize()
        cts.append(e0.elapsed_time(e1))
    copy_probe = 2 * probe.numel() * 4 / median(cts) / 1e6
    del probe, dst

    # ---- roofline of the dominant kernel: algorithmic bytes of its loop / its own duration
    dom = max(names, key=lambda c: per[c]["kernel_ms"])
    alg_bytes = (configs.IN_BYTES[dom] + configs.OUT_BYTES[dom]) * rows[dom]
    achieved = alg_bytes / per[dom]["kernel_ms"] / 1e6
    # HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (profiles/hbm_traffic.txt: config, kernel
    # name, bytes).  The kernel is named after its own text, so a row only counts for the kernel it was
    # measured on: after any change to a loop's code the figure is null until the counters are taken again.
    traffic_of = {}
    tfile = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if os.path.exists(tfile) and args.scale == 1.0:
        for ln in open(tfile):
            f = ln.split()
            if len(f) == 3 and f[0] in per and f[1] == per[f[0]]["kernel"]:
                traffic_of[f[0]] = int(f[2])
    attainable = max([read_probe] + [per[c]["input_GBps"] for c in names])
    for c in names:
        per[c]["hbm_traffic_bytes"] = traffic_of.get(c)
        per[c]["in_plus_out_frac_of_hbm_peak"] = round(per[c]["in_plus_out_GBps"] / HBM_PEAK_GBPS, 4)
        per[c]["in_plus_out_frac_of_attainable_read"] = round(per[c]["in_plus_out_GBps"] / attainable, 4)
    roofline = {"bound": "hbm", "kernel": per[dom]["kernel"], "workload": dom, "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                "traffic": traffic_of.get(dom), "read_probe_GBps": round(read_probe, 1),
                "attainable_read_GBps": round(attainable, 1), "copy_probe_GBps": round(copy_probe, 1)}

    # ---- the CPU oracle as it stands, on a bounded sample of the same workloads
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import interp
        try:
            import threadpoolctl
            limit = threadpoolctl.threadpool_limits(1)
        except Exception:
            limit = None
        tot_b, tot_s, desc = 0, 0.0, []
        for c in names:
            m = min(rows[c], CPU_SAMPLE_ROWS[c])
            host = [t[:m].cpu().numpy() for t in cols[c]]
            t1 = time.perf_counter()
            interp.run(progs[c], host)
            tot_s += time.perf_counter() - t1
            tot_b += configs.IN_BYTES[c] * m
            desc.append("%s:%d" % (c, m))
        del limit
        cpu = {"value": round(tot_b / tot_s / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
               "seconds": round(tot_s, 2),
               "sample": "first rows of each config (" + ", ".join(desc) + "), numpy operator-at-a-time oracle, 1 thread"}

    # ---- vecmerger strategies on the count-occurrences program (1e8 32-bit keys, uniform)
    # (Sec. 7.7 of the paper: local / shared / global copies over the size of the vector; here also LDS copies of
    # 8192-cell ranges, and merges queued by range of cells for a second kernel.  The default line carries four
    # sizes, --vecmerger-sweep all ten.)
    sweep = None
    if not args.no_nested or args.vecmerger_sweep:
        from workloads import rng
        from workloads.ir import Program
        nk = max(1, int(100_000_000 * args.scale))
        sweep = []
        sizes = (8, 64, 1024, 8192, 32768, 65536, 1 << 18, 1 << 19, 1 << 20, 1 << 24) if args.vecmerger_sweep else (8, 8192, 65536, 1 << 20)
        for m in sizes:
            keys = rng.uniform_int(6, 0, 0, nk, 0, m - 1, "cuda").to(torch.int32)
            for strat, label in ((1, "local"), (2, "shared"), (4, "shared by range"), (5, "queued by range"), (3, "global")):
                if (strat == 1 and m > 8) or (strat == 2 and m > 16384) or (strat == 4 and not 8192 < m <= 8192 * 64) or (strat == 5 and m <= 8192):
                    continue
                if strat == 3 and m < 8192 and not args.vecmerger_sweep:
                    continue            # 13-390 ms a run: same-address device atomics, in the long sweep only
                p = Program(["i32"])
                p.merge(p.vecmerger("i64", "add", m), [p.const("i64", 1)], keys=[p.un("cast", p.col(0), to="i64")])
                ts = []
                for i in range(5):
                    r = wb.fused_for(p, [keys], tune={"vecmerger_strategy": strat}).check()
                    if i >= 2:
                        ts.append(r.kernel_ms())
                    total = int(r.vec(0).sum().item()) if i == 0 else nk
                    kname = r.kernel_name()
                    r.free()
                    assert total == nk
                sweep.append({"length": m, "strategy": label, "kernel": kname, "kernel_ms": round(median(ts), 4),
                              "keys_per_s": nk / median(ts) * 1e3})
            del keys

    # ---- nested loops: one PageRank iteration (contributions map + nested for) and a CSR
    # matrix-vector product over the synthetic power-law graph; not part of `value`
    nested = None
    if not args.no_nested:
        try:
            from workloads import graphs
            for c in names:
                cols[c] = None                      # the step's columns are no longer needed
            torch.cuda.empty_cache()
            nv = max(1, int(graphs.PAGERANK_VERTICES * args.scale))
            rowptr, src, weight, outdeg = graphs.make_graph(nv, device="cuda")
            start, end = rowptr[:-1].contiguous(), rowptr[1:].contiguous()
            ne = src.numel()
            rank = torch.full((nv,), 1.0 / nv, dtype=torch.float64, device="cuda")
            pr, spmv, contrib_prog = graphs.program_pagerank(nv), graphs.program_spmv(), graphs.program_contrib()
            it_ms, inner_ms, total = [], [], None
            for i in range(args.warmup + max(5, args.steps // 2)):
                r1 = wb.fused_for(contrib_prog, [rank, outdeg])
                contrib = r1.check().vec(0)
                r2 = wb.nested_for(pr, [start, end], [src], [contrib]).check()
                if i >= args.warmup:
                    it_ms.append(r1.elapsed_ms() + r2.elapsed_ms())
                    inner_ms.append(r2.kernel_ms())
                total = float(r2.merger(1))
                kname = r2.kernel_name()
                r1.free()
                r2.free()
            sp_ms = []
            for i in range(args.warmup + 5):
                r = wb.nested_for(spmv, [start, end], [src, weight], [rank]).check()
                if i >= args.warmup:
                    sp_ms.append(r.elapsed_ms())
                sname = r.kernel_name()
                r.free()
            # algorithmic bytes of an iteration: every edge's source once, the contribution vector
            # once, both row offsets, ranks and out-degrees in, new ranks out
            alg = 4 * ne + 8 * nv + 2 * 8 * nv + 8 * nv + 8 * nv + 8 * nv
            nested = {"workload": "PageRank iteration, synthetic power-law graph", "vertices": nv, "edges": ne,
                      "iteration_ms": round(median(it_ms), 4), "inner_kernel_ms": round(median(inner_ms), 4),
                      "inner_kernel": kname, "edges_per_s": ne / median(it_ms) * 1e3,
                      "algorithmic_GBps": round(alg / median(it_ms) / 1e6, 1), "rank_sum_after_one_iteration": total,
                      "spmv_ms": round(median(sp_ms), 4), "spmv_edges_per_s": ne / median(sp_ms) * 1e3,
                      "spmv_inner_kernel": sname}
        except Exception as e:      # a leg beyond the step must not take the step's line with it
            nested = {"error": "%s: %s" % (type(e).__name__, str(e)[:300])}

    # ---- groupbuilder: the zip-code column grouped by its key (values = the codes themselves)
    groups = None
    if not args.no_nested and "C5" in names:
        try:
            gcols = configs.make_columns("C5", rows["C5"], device="cuda")
            gp = configs.program_group_by_zip()
            ts, npairs, ngroups = [], 0, 0
            for i in range(args.warmup + 5):
                r = wb.fused_for(gp, gcols).check()
                if i >= args.warmup:
                    ts.append(r.elapsed_ms())
                if i == 0:
                    gk, go, gv = r.groups(0)
                    npairs, ngroups = int(len(gv)), int(len(gk[0]))
                    assert int(go[-1]) == npairs
                gname = r.kernel_name()
                r.free()
            groups = {"workload": "groupbuilder over the zip-code column", "rows": rows["C5"], "pairs": npairs,
                      "groups": ngroups, "call_ms": round(median(ts), 4), "pairs_per_s": npairs / median(ts) * 1e3,
                      "loop_kernel": gname}
            del gcols
        except Exception as e:      # a leg beyond the step must not take the step's line with it
            groups = {"error": "%s: %s" % (type(e).__name__, str(e)[:300])}

    # ---- hash join shaped like TPC-H Q12: build a dictionary over `orders`, probe it from `lineitem`
    join = None
    if not args.no_nested:
        try:
            from workloads import joins
            no, nl = max(1, int(joins.ORDERS * args.scale)), max(1, int(joins.LINEITEMS * args.scale))
            orders, lines = joins.make_tables(no, nl, device="cuda")
            bp, pp = joins.program_build(no), joins.program_probe()
            bms, pms = [], []
            for i in range(args.warmup + 5):
                built = wb.fused_for(bp, orders)
                r = wb.fused_for(pp, lines, dicts=[(built, 0)]).check()
                if i >= args.warmup:
                    bms.append(built.elapsed_ms())
                    pms.append(r.elapsed_ms())
                if i == 0:
                    _, jv = r.dict(0)
                    matched = int(jv[0].sum() + jv[1].sum())
                bname, pname = built.kernel_name(), r.kernel_name()
                r.free()
                built.free()
            join = {"workload": "hash join shaped like TPC-H Q12", "orders": no, "lineitems": nl, "matched_lines": matched,
                    "build_ms": round(median(bms), 4), "probe_ms": round(median(pms), 4),
                    "build_rows_per_s": no / median(bms) * 1e3, "probe_rows_per_s": nl / median(pms) * 1e3,
                    "probe_input_GBps": round(17 * nl / median(pms) / 1e6, 1), "build_kernel": bname, "probe_kernel": pname}
            del orders, lines
        except Exception as e:
            join = {"error": "%s: %s" % (type(e).__name__, str(e)[:300])}

    line = {
        "metric": "fused-loop input GB/s (all five configs back to back)", "value": round(value, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": "C1..C5 fused loops, rows " + ", ".join("%s=%d" % (c, rows[c]) for c in names),
                   "input_bytes_per_step": total_in, "hbm_peak_GBps": HBM_PEAK_GBPS, "tune": tune,
                   "launch_tuning": tuning_report or None},
        "rows_per_s": sum(rows.values()) / ms_per_step * 1e3,
        "per_config": per, "roofline": roofline, "cpu_baseline": cpu,
    }
    if sweep is not None:
        line["vecmerger_sweep"] = sweep
    if nested is not None:
        line["nested_loop"] = nested
    if groups is not None:
        line["groupbuilder"] = groups
    if join is not None:
        line["hash_join"] = join
    print(json.dumps(line))


if __name__ == "__main__":
    main()
