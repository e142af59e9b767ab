#!/usr/bin/env python3
"""Benchmark: 64-set batched Forward Prune on the 50M-operator power-law DAG, one MI355X.

One "step" = one dgn_prune call = clear + seed + traversal + removal rule + ordered compaction over the
whole graph, with the graph's adjacency already resident in HBM.  The CSR build is timed separately (it is
amortised over the prunes of one recorded graph), for operator-major and for shuffled COO.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, vendor figure
COUNTERS = os.path.join("profiles", "prune_config3_hbm_counters.txt")


def measured_traffic(kernel):
    """HBM bytes per launch from the committed rocprofv3 counter summary, or None when the kernels have
    changed since the counters were taken (or the workload is not the one they were taken on)."""
    import hashlib
    try:
        vals = dict(line.split(": ", 1) for line in open(os.path.join(ROOT, COUNTERS)).read().splitlines()
                    if ": " in line and not line.startswith("#"))
        h = hashlib.sha256()
        for f in ("traverse.hip", "keep_compact.hip", "primitives.hip", "common.h"):
            h.update(open(os.path.join(ROOT, "paper_1707_08265_amd", "csrc", f), "rb").read())
        if h.hexdigest()[:16] != vals.get("source_hash", "").strip():
            return None
        return int(vals[kernel + "_traffic_bytes"])
    except (OSError, KeyError, ValueError):
        return None


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def timed_build(d, torch, np, desc, graph_mem, gb, scratch, sb, keep_last=True):
    """Median of the last two of three builds; returns (ms, handle of the last build or None)."""
    ms, handle = [], None
    for _ in range(3):
        if handle:
            d.dgn_graph_destroy(handle)
        torch.cuda.synchronize()
        tb = time.perf_counter()
        rc, handle = d.dgn_graph_build(desc, graph_mem, gb, scratch, sb)
        torch.cuda.synchronize()
        ms.append((time.perf_counter() - tb) * 1e3)
        assert rc == 0, d.dgn_strerror(rc)
    if not keep_last:
        d.dgn_graph_destroy(handle)
        handle = None
    return float(np.median(ms[1:])), handle


def shuffled_build_ms(d, torch, np, gg, g, in_op, in_t, out_op, out_t, gb, sb, scratch):
    """The same edges in a seeded random COO order (the keys of graphgen's permutation, sorted on the device: input
    preparation, untimed): every sort of the builder runs."""
    def perm(n, seed):
        keys = (gg.permutation_keys(n, seed) ^ np.uint64(1 << 63)).view(np.int64)      # order-preserving uint64 -> int64
        return torch.argsort(torch.from_numpy(keys).cuda(), stable=True)
    pi, po = perm(g.nnz_in, 12345), perm(g.nnz_out, 12346)
    s_in_op, s_in_t, s_out_op, s_out_t = in_op[pi], in_t[pi], out_op[po], out_t[po]
    del pi, po
    sdesc = d.make_coo_desc(g.num_ops, g.num_tensors, s_in_op, s_in_t, s_out_op, s_out_t, g.num_graphs,
                            g.graph_op_offsets, g.graph_tensor_offsets)
    smem = torch.empty(gb, dtype=torch.uint8, device=in_op.device)
    ms, _ = timed_build(d, torch, np, sdesc, smem, gb, scratch, sb, keep_last=False)
    return ms


def other_config(d, torch, np, gg, orc, k, steps, warmup, with_oracle):
    """One of the workloads the metric is not quoted on: build, K timed prunes, and the result against the oracle
    (whole workload for configs 0-2; the packed batch through the fixed-point certificate over all of M and K plus
    Algorithm 1 on three of its graphs)."""
    t0 = time.time()
    g, tg = gg.config(k, 1.0)
    E = g.nnz_in + g.nnz_out
    dev = torch.device("cuda:0")
    up = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(dev)
    in_op, in_t, out_op, out_t = up(g.in_op), up(g.in_tensor), up(g.out_op), up(g.out_tensor)
    desc = d.make_coo_desc(g.num_ops, g.num_tensors, in_op, in_t, out_op, out_t, g.num_graphs,
                           g.graph_op_offsets, g.graph_tensor_offsets)
    rc, gb, sb = d.dgn_graph_build_workspace(desc)
    assert rc == 0, d.dgn_strerror(rc)
    graph_mem = torch.empty(gb, dtype=torch.uint8, device=dev)
    scratch = torch.empty(sb, dtype=torch.uint8, device=dev)
    build_ms, handle = timed_build(d, torch, np, desc, graph_mem, gb, scratch, sb)
    del scratch, in_op, in_t, out_op, out_t
    rc, sizes = d.dgn_graph_get_sizes(handle)
    dg = d.DeviceGraph(handle, graph_mem, (), sizes)
    buf = d.PruneBuffers(dg, tg.num_sets)
    rowptr, idx = up(tg.tgt_rowptr), up(tg.tgt_idx)
    st = d.dgn_stats()
    for _ in range(warmup):
        rc = buf.prune(rowptr, idx, stats=st)
        assert rc == 0, d.dgn_strerror(rc)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(steps):
        rc = buf.prune(rowptr, idx, stats=st)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t1) / steps * 1e3
    assert rc == 0, d.dgn_strerror(rc)
    out = buf.to_host()
    res = {"workload": f"configs[{k}] {g.name}", "num_ops": g.num_ops, "num_sets": tg.num_sets, "num_graphs": g.num_graphs,
           "ms_per_step": round(ms, 4), "gteps": round(E / (ms * 1e-3) / 1e9, 3), "build_ms": round(build_ms, 3),
           "levels": int(st.levels), "operator_visits": int(st.tensor_visits), "launches": int(st.launches),
           "kept_ops": int(out["kept_count"][0]), "output_buffers": "recycled" if st.recycled else "cleared in full",
           "bit_exact_vs_oracle": None, "oracle": None}
    del buf, dg, graph_mem
    torch.cuda.empty_cache()
    if with_oracle:
        tb = time.time()
        if g.num_graphs == 1:
            adj = orc.build_adjacency(g.num_ops, g.num_tensors, g.in_op, g.in_tensor, g.out_op, g.out_tensor)
            t2 = time.perf_counter()
            ref = orc.forward_prune(adj, tg.num_sets, tg.tgt_rowptr, tg.tgt_idx, g.num_graphs, g.graph_op_offsets)
            res["oracle"] = {"seconds": round(time.perf_counter() - t2, 3), "sample": "whole workload, one core"}
            same = all(np.array_equal(out[n], getattr(ref, n)) for n in
                       ("tensor_mask", "op_mask", "op_flag", "kept_ops", "kept_masks", "kept_count", "per_query_count"))
        else:
            adj = orc.build_adjacency(g.num_ops, g.num_tensors, g.in_op, g.in_tensor, g.out_op, g.out_tensor)
            S = orc.seed_masks(g.num_tensors, tg.num_sets, tg.tgt_rowptr, tg.tgt_idx)
            same = orc.certificate(adj, S, out["tensor_mask"], out["op_mask"]) == 0
            same = same and np.array_equal(out["kept_ops"], np.nonzero(out["op_mask"])[0].astype(np.int32))
            del adj, S
            t2 = time.perf_counter()
            for gi in (0, g.num_graphs // 2, g.num_graphs - 1):
                one = gg.layered(20000, gg.BASE_SEED + 4000 + gi)
                t1g = gg.targets_tail(one, gg.BASE_SEED + 4000 + gi, tg.num_sets, 4, 4, 0.10)
                a1 = orc.build_adjacency(one.num_ops, one.num_tensors, one.in_op, one.in_tensor, one.out_op, one.out_tensor)
                r1 = orc.forward_prune(a1, t1g.num_sets, t1g.tgt_rowptr, t1g.tgt_idx)
                ta, tb_ = g.graph_tensor_offsets[gi], g.graph_tensor_offsets[gi + 1]
                oa, ob = g.graph_op_offsets[gi], g.graph_op_offsets[gi + 1]
                same = same and np.array_equal(out["tensor_mask"][ta:tb_], r1.tensor_mask)
                same = same and np.array_equal(out["op_mask"][oa:ob], r1.op_mask)
                same = same and np.array_equal(out["per_query_count"][gi * 64:(gi + 1) * 64], r1.per_query_count)
            res["oracle"] = {"seconds": round(time.perf_counter() - t2, 3),
                             "sample": "Algorithm 1 on 3 of the graphs, one core; all of M and K through the fixed-point certificate"}
        res["bit_exact_vs_oracle"] = bool(same)
        assert same, f"config {k}: GPU result differs from the oracle"
        log(f"config {k}: oracle check {time.time() - tb:.1f}s, bit-exact: {same}")
    log(f"config {k} ({g.name}): {ms:.3f} ms/step, {res['gteps']} GTEPS, build {build_ms:.2f} ms, levels={res['levels']} "
        f"visits={res['operator_visits']} kept={res['kept_ops']} ({time.time() - t0:.0f}s in all)")
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=3, help="workload family 0..4 (3 = the headline one)")
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the workload (testing only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--recompute-keep", action="store_true",
                    help="run the stand-alone removal-rule pass instead of reusing the traversal's K")
    ap.add_argument("--defer-percent", type=int, default=0, help="traversal schedule knob (0 = library default)")
    ap.add_argument("--defer-start-shift", type=int, default=0)
    ap.add_argument("--defer-floor-shift", type=int, default=0)
    ap.add_argument("--generic", action="store_true", help="force the one-launch-per-level traversal")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (known size, to scale profiler byte counters)")
    ap.add_argument("--no-shuffled-build", action="store_true",
                    help="skip the CSR build on the same edges in shuffled COO order (every sort runs)")
    ap.add_argument("--build-only", action="store_true", help="time the two CSR builds and stop (for profiling runs)")
    ap.add_argument("--no-other-configs", action="store_true", help="skip the four workloads the metric is not quoted on")
    ap.add_argument("--prune-only", action="store_true",
                    help="only the timed prunes: no other legs, configs, shuffled build or machine rates (for profiling runs)")
    ap.add_argument("--no-recycle", action="store_true",
                    help="clear all of M and K in every step instead of only what the previous step set")
    ap.add_argument("--trace-levels", action="store_true", help="print the per-level trace of the last step")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this path runs on ONE GPU only (no sharding or collectives are built); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import graphgen as gg
    import __graft_entry__
    __graft_entry__.ensure_built()          # a fresh checkout: build once; otherwise what is built is loaded
    import paper_1707_08265_amd as d

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")

    t0 = time.time()
    g, tg = gg.config(args.config, args.scale)
    E = g.nnz_in + g.nnz_out
    log(f"generated {g.name}: P={g.num_ops} T={g.num_tensors} E_in={g.nnz_in} E_out={g.nnz_out} "
        f"Q={tg.num_sets} targets={len(tg.tgt_idx)} in {time.time() - t0:.1f}s")

    # ---- CSR build (timed separately) ------------------------------------------------------
    up = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(dev)
    in_op, in_t, out_op, out_t = up(g.in_op), up(g.in_tensor), up(g.out_op), up(g.out_tensor)
    desc = d.make_coo_desc(g.num_ops, g.num_tensors, in_op, in_t, out_op, out_t, g.num_graphs,
                           g.graph_op_offsets, g.graph_tensor_offsets)
    rc, gb, sb = d.dgn_graph_build_workspace(desc)
    assert rc == 0, d.dgn_strerror(rc)
    graph_mem = torch.empty(gb, dtype=torch.uint8, device=dev)
    scratch = torch.empty(sb, dtype=torch.uint8, device=dev)
    build_ms, handle = timed_build(d, torch, np, desc, graph_mem, gb, scratch, sb)
    log(f"CSR build: {build_ms:.2f} ms ({E / build_ms / 1e6:.1f} GTEPS)")
    build_shuffled_ms = None
    if args.build_only or not (args.no_shuffled_build or args.prune_only):
        build_shuffled_ms = shuffled_build_ms(d, torch, np, gg, g, in_op, in_t, out_op, out_t, gb, sb, scratch)
        log(f"CSR build, shuffled COO: {build_shuffled_ms:.2f} ms ({E / build_shuffled_ms / 1e6:.1f} GTEPS)")
    del scratch
    if args.build_only:
        print(json.dumps({"build_ms": round(build_ms, 3), "build_shuffled_ms": round(build_shuffled_ms, 3),
                          "config": {"workload": f"configs[{args.config}] {g.name}"}}), flush=True)
        return
    rc, sizes = d.dgn_graph_get_sizes(handle)
    dg = d.DeviceGraph(handle, graph_mem, (), sizes)
    del in_op, in_t, out_op, out_t
    torch.cuda.empty_cache()

    # ---- prune --------------------------------------------------------------------------------
    buf = d.PruneBuffers(dg, tg.num_sets, recycle=not args.no_recycle)
    rowptr, idx = up(tg.tgt_rowptr), up(tg.tgt_idx)
    # timed steps: no HIP events inside the library (every event between two kernels idles the stream for a few
    # microseconds: two of them cost 8 us of a step).  The phases are timed in extra steps after the timed region:
    # as many again with events around the traversal only, then five with every phase bracketed
    opts = d.dgn_options(profile=0, recompute_keep=1 if args.recompute_keep else 0,
                         defer_percent=args.defer_percent, traversal=1 if args.generic else 0,
                         defer_start_shift=args.defer_start_shift, defer_floor_shift=args.defer_floor_shift)
    st = d.dgn_stats()
    trace = np.zeros((4096, 4), dtype=np.int32)
    if args.trace_levels:
        st.level_trace, st.level_trace_cap = trace.ctypes.data, trace.shape[0]
    for _ in range(args.warmup):
        rc = buf.prune(rowptr, idx, options=opts, stats=st)
        assert rc == 0, d.dgn_strerror(rc)
    phases = np.zeros((args.steps, 8))
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for i in range(args.steps):
        rc = buf.prune(rowptr, idx, options=opts, stats=st)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    assert rc == 0, d.dgn_strerror(rc)
    opts.profile = 2
    for i in range(args.steps):
        rc = buf.prune(rowptr, idx, options=opts, stats=st)
        assert rc == 0, d.dgn_strerror(rc)
        phases[i] = list(st.phase_ms)
    ms_per_step = elapsed / args.steps * 1e3
    gteps = E / (ms_per_step * 1e-3) / 1e9
    recycled = bool(st.recycled)
    level_launches = int(st.level_launches)
    atomics_per_step = int(st.atomic_updates)
    stats_visits = int(st.tensor_visits)
    levels_total, launches_total = int(st.levels), int(st.launches)
    opts.profile = 1
    phases_all = np.zeros((5, 8))
    # these extra steps also take the per-level trace (device clock at the start of every launch): the time from one
    # wide launch to the next is the level kernel's own duration, without the two single-workgroup launches that
    # the events around the traversal include
    traced = bool(args.trace_levels)
    st.level_trace, st.level_trace_cap = trace.ctypes.data, trace.shape[0]
    wide_us = []
    for i in range(5):
        rc = buf.prune(rowptr, idx, options=opts, stats=st)
        assert rc == 0, d.dgn_strerror(rc)
        phases_all[i] = list(st.phase_ms)
        nl = min(int(st.levels), trace.shape[0])
        if nl >= 2:
            wide = trace[:nl, 2] != -1
            dt = ((trace[1:nl, 3].astype(np.int64) - trace[:nl - 1, 3].astype(np.int64)) & 0xFFFFFFFF) / 100.0
            wide_us += dt[wide[1:] & wide[:-1]].tolist()
    narrow_levels = int((trace[:min(int(st.levels), trace.shape[0]), 2] == -1).sum())
    if not traced:
        st.level_trace, st.level_trace_cap = None, 0
    level_us_device_clock = float(np.mean(wide_us)) if wide_us else None
    opts.profile = 0
    ph = dict(zip(d.PHASES, phases_all.mean(0)[:7].tolist()))
    ph["traverse"] = float(phases.mean(0)[2])              # events around the traversal only
    log(f"prune: {ms_per_step:.3f} ms/step, {gteps:.1f} GTEPS; levels={st.levels} launches={st.launches} "
        f"visits={st.tensor_visits} max_frontier={st.max_frontier} recycled={int(recycled)}")
    log("phase ms (HIP events, extra steps after the timed ones; traverse: events around the traversal only, the others: "
        "5 steps with every phase bracketed): " + ", ".join(f"{k}={v:.3f}" for k, v in ph.items()))

    # the same steps with every word of M and K cleared each time (what a caller gets who writes to the output
    # buffers between calls, or prunes once)
    full_clear = None
    if recycled and not args.prune_only:
        buf2 = d.PruneBuffers(dg, tg.num_sets, recycle=False)
        for _ in range(2):
            rc = buf2.prune(rowptr, idx, options=opts, stats=st)
            assert rc == 0, d.dgn_strerror(rc)
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for i in range(args.steps):
            rc = buf2.prune(rowptr, idx, options=opts, stats=st)
        torch.cuda.synchronize()
        ms2 = (time.perf_counter() - t2) / args.steps * 1e3
        assert rc == 0 and not st.recycled
        full_clear = {"ms_per_step": round(ms2, 4), "gteps": round(E / (ms2 * 1e-3) / 1e9, 2)}
        log(f"prune with a full clear per step: {ms2:.3f} ms/step, {full_clear['gteps']:.1f} GTEPS")
        del buf2
    elif not recycled:
        full_clear = {"ms_per_step": round(ms_per_step, 4), "gteps": round(gteps, 2)}
    # recycled buffers with target sets that change from step to step (a second draw of the same recipe, taken in
    # turns with the workload's own): no step finds anything of its own result in place, only words to zero
    other_targets = None
    if recycled and not args.prune_only and g.num_graphs == 1 and args.config == 3:
        tg2 = gg.targets_tail(g, gg.BASE_SEED + 3000 + 1, tg.num_sets, 1, 16, 0.05)
        rowptr2, idx2 = up(tg2.tgt_rowptr), up(tg2.tgt_idx)
        pairs = [(rowptr, idx), (rowptr2, idx2)]
        for i in range(4):
            rc = buf.prune(*pairs[i & 1], options=opts, stats=st)
            assert rc == 0, d.dgn_strerror(rc)
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for i in range(args.steps):
            rc = buf.prune(*pairs[i & 1], options=opts, stats=st)
        torch.cuda.synchronize()
        ms3 = (time.perf_counter() - t2) / args.steps * 1e3
        assert rc == 0 and st.recycled
        other_targets = {"ms_per_step": round(ms3, 4), "gteps": round(E / (ms3 * 1e-3) / 1e9, 2),
                         "targets": "the workload's and a second draw of the same recipe, in turns"}
        log(f"prune, recycled buffers, two target draws in turns: {ms3:.3f} ms/step, {other_targets['gteps']:.1f} GTEPS")
        del rowptr2, idx2
    if recycled and not args.prune_only:
        rc = buf.prune(rowptr, idx, options=opts, stats=st)      # st and the buffers describe the timed workload again
        assert rc == 0
    # the same steps once more, each one timed on its own (a synchronisation after every step): median and minimum
    one_by_one = copy_gbs = rates = None
    if not args.prune_only:
        one = []
        for _ in range(max(args.steps, 20)):
            torch.cuda.synchronize()
            t2 = time.perf_counter()
            rc = buf.prune(rowptr, idx, options=opts, stats=st)
            torch.cuda.synchronize()
            one.append((time.perf_counter() - t2) * 1e3)
            assert rc == 0, d.dgn_strerror(rc)
        one_by_one = {"median": round(float(np.median(one)), 4), "min": round(float(np.min(one)), 4), "steps": len(one)}
        # what a plain device-to-device copy reaches on this GPU: the practical ceiling beside the published peak
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        dst.copy_(src)
        e0.record()
        for _ in range(5):
            dst.copy_(src)
        e1.record()
        torch.cuda.synchronize()
        copy_gbs = round(5 * 2 * (1 << 30) / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)
        del src, dst
        log(f"steps timed one by one: median {one_by_one['median']:.3f} ms, min {one_by_one['min']:.3f} ms; "
            f"1 GiB device copy: {copy_gbs} GB/s (read + write)")
        # the rates that bound the traversal, measured on this GPU over a buffer as large as the mask array (untimed leg)
        cal = torch.empty(max(8 * g.num_tensors, 1 << 24), dtype=torch.uint8, device=dev)
        rc, r = d.dgn_calibrate(cal, cal.numel())
        assert rc == 0, d.dgn_strerror(rc)
        rates = r.as_dict()
        del cal
        log("machine rates: " + ", ".join(f"{k}={v}" for k, v in rates.items()))
    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                       # one elementwise copy kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    if args.trace_levels:
        for lv in range(min(int(st.levels), trace.shape[0])):
            dt = ((int(trace[lv, 3]) - int(trace[lv - 1, 3])) & 0xFFFFFFFF) / 100.0 if lv else 0.0
            log(f"level {lv}: queue={trace[lv, 0]} processed={trace[lv, 1]} theta={trace[lv, 2]} us_since_prev={dt:.1f}")
    out = buf.to_host()
    P, T = g.num_ops, g.num_tensors

    inplace = readout = backward = incremental = transaction = None
    extras = {}
    if not args.prune_only:
        # ---- in-place pass on the pruned graph (Algorithm 3), timed on its own, not part of `value` ---
        ip = d.InplaceBuffers(dg)
        ip_ms = []
        for _ in range(1 + max(3, min(args.steps, 10))):
            torch.cuda.synchronize()
            tb = time.perf_counter()
            rc = ip.run(buf.op_mask, kept_ops=buf.kept_ops, kept_count=buf.kept_count)
            torch.cuda.synchronize()
            ip_ms.append((time.perf_counter() - tb) * 1e3)
            assert rc == 0, d.dgn_strerror(rc)
        ip_ms = float(np.median(ip_ms[1:]))
        ip_rename = ip.rename.cpu().numpy()
        inplace = {"ms": round(ip_ms, 4), "rounds": int(ip.rounds), "renamed_tensors": int(ip.renamed_count.item()),
                   "graph_tensors": int((ip_rename >= 0).sum()), "select": "all sets (union graph)",
                   "cpu_oracle_ms": None, "bit_exact_vs_oracle": None}
        log(f"in-place pass: {ip_ms:.3f} ms, {inplace['rounds']} rounds, {inplace['renamed_tensors']} of "
            f"{inplace['graph_tensors']} tensors renamed")
        del ip

        # ---- read-outs of the result (Sec. 3.2): ignore mask, per-set operator lists; timed on their own --
        ro = d.ReadoutBuffers(buf)
        ro_ms = {"ignore": [], "lists": []}
        for _ in range(1 + max(3, min(args.steps, 10))):
            torch.cuda.synchronize()
            tb = time.perf_counter()
            rc = ro.ignore()
            torch.cuda.synchronize()
            ro_ms["ignore"].append((time.perf_counter() - tb) * 1e3)
            assert rc == 0, d.dgn_strerror(rc)
            tb = time.perf_counter()
            rc = ro.per_set_lists()
            torch.cuda.synchronize()
            ro_ms["lists"].append((time.perf_counter() - tb) * 1e3)
            # (the lists have up to 64 entries per kept operator, counted in 32 bits: a packed batch of the size of
            # config 4 keeps too many operators for one call)
            lists_ok = rc == 0
            assert rc in (0, d.DGN_ERR_TOO_LARGE), d.dgn_strerror(rc)
        ro_ignore = ro.ignore_mask.cpu().numpy().view(np.uint64)
        ro_rowptr = ro.set_rowptr.cpu().numpy() if lists_ok else None
        ro_ops = ro.set_ops[: int(ro_rowptr[64])].cpu().numpy() if lists_ok else None
        readout = {"ignore_ms": round(float(np.median(ro_ms["ignore"][1:])), 4),
                   "ignored_tensors": int(ro.ignore_count.item()),
                   "per_set_lists_ms": round(float(np.median(ro_ms["lists"][1:])), 4) if lists_ok else None,
                   "list_entries": int(ro_rowptr[64]) if lists_ok else None, "bit_exact_vs_oracle": None}
        log(f"read-outs: ignore mask {readout['ignore_ms']:.3f} ms ({readout['ignored_tensors']} tensors), per-set lists "
            + (f"{readout['per_set_lists_ms']:.3f} ms ({readout['list_entries']} entries; includes two small read-backs)"
               if lists_ok else "skipped: more than 2^31 / 64 kept operators"))
        del ro

        # ---- transaction cache (Sec. 4.1): the same target sets asked for again -- a digest on the device and a
        # dictionary look-up instead of a prune; timed on its own
        tc = d.TransactionCache(dg, tg.num_sets, capacity=1)
        first = tc.prune(rowptr, idx)
        tx_ms = []
        for _ in range(1 + max(3, min(args.steps, 10))):
            torch.cuda.synchronize()
            tb = time.perf_counter()
            again = tc.prune(rowptr, idx)
            torch.cuda.synchronize()
            tx_ms.append((time.perf_counter() - tb) * 1e3)
            assert again is first
        tx_out = first.to_host()
        transaction = {"hit_ms": round(float(np.median(tx_ms[1:])), 4), "hits": tc.hits, "misses": tc.misses,
                       "digest_words": int(2 + len(tg.tgt_rowptr) + len(tg.tgt_idx)),
                       "equals_timed_result": bool(all(np.array_equal(tx_out[k], out[k]) for k in out))}
        log(f"transaction cache: a hit costs {transaction['hit_ms']:.3f} ms (digest of {transaction['digest_words']} "
            f"words + look-up); cached result equals the timed one: {transaction['equals_timed_result']}")
        assert transaction["equals_timed_result"]
        del tc, first, again

        # ---- incremental prune: the last target set added to a finished prune of the others --------------
        incremental = None
        if g.num_graphs == 1 and tg.num_sets > 1:
            last = tg.num_sets - 1
            rp_part = tg.tgt_rowptr.copy()
            rp_part[last + 1:] = rp_part[last]                 # the last set is empty in the first call
            rp_part_d = up(rp_part)
            inc_ms = []
            inc_st = d.dgn_stats()
            for _ in range(1 + max(3, min(args.steps, 10))):
                rc = buf.prune(rp_part_d, idx)
                assert rc == 0, d.dgn_strerror(rc)
                torch.cuda.synchronize()
                tb = time.perf_counter()
                rc = buf.prune(rowptr, idx, options=d.dgn_options(incremental=1), stats=inc_st)
                torch.cuda.synchronize()
                inc_ms.append((time.perf_counter() - tb) * 1e3)
                assert rc == 0, d.dgn_strerror(rc)
            inc_out = buf.to_host()
            same = all(np.array_equal(inc_out[k], out[k]) for k in out)
            incremental = {"ms": round(float(np.median(inc_ms[1:])), 4), "added_sets": 1,
                           "operator_visits": int(inc_st.tensor_visits), "levels": int(inc_st.levels),
                           "equals_one_shot_result": bool(same)}
            log(f"incremental prune (set {last} added to the other {last}): {incremental['ms']:.3f} ms, "
                f"{incremental['operator_visits']} visits in {incremental['levels']} levels; equals the one-shot result: {same}")
            assert same, "incremental prune differs from the one-shot prune"

        # ---- backward prune (Algorithm 2) on the same graph, 64 pairs, timed on its own ---------------
        backward = None
        if g.num_graphs == 1:
            n_src = 400 if args.config == 1 else 16
            obj_h, wrt_h = gg.backward_pairs(g, gg.BASE_SEED + 1000 * args.config, 64, n_src)
            bb = d.BackwardPruneBuffers(dg, 64)
            obj_d, wrt_d = up(obj_h), up(wrt_h)
            bst = d.dgn_stats()
            bw_ms = []
            for _ in range(1 + max(3, min(args.steps, 10))):
                torch.cuda.synchronize()
                tb = time.perf_counter()
                rc = bb.backward_prune(obj_d, wrt_d, stats=bst)
                torch.cuda.synchronize()
                bw_ms.append((time.perf_counter() - tb) * 1e3)
                assert rc == 0, d.dgn_strerror(rc)
            bw_ms = float(np.median(bw_ms[1:]))
            bw_out = bb.to_host()
            backward = {"ms": round(bw_ms, 4), "gteps": round(E / (bw_ms * 1e-3) / 1e9, 2), "pairs": 64,
                        "forward_passes": int(bst.reserved), "first_stage_levels": int(bst.levels),
                        "marked_tensors": int(np.count_nonzero(bw_out["tensor_mask"])),
                        "kept_ops": int(bw_out["kept_count"][0]),
                        "connected_pairs": int(np.count_nonzero(bw_out["per_query_count"])),
                        "cpu_oracle_ms_per_pair": None, "bit_exact_vs_oracle_sampled_pair": None}
            log(f"backward prune: {bw_ms:.3f} ms ({backward['gteps']} GTEPS), {backward['forward_passes']} forward passes, "
                f"{backward['marked_tensors']} tensors marked, {backward['kept_ops']} operators kept, "
                f"{backward['connected_pairs']} of 64 pairs connected")
            del bb
        extras = dict(ip_rename=ip_rename, ro_rowptr=ro_rowptr, ro_ignore=ro_ignore, ro_ops=ro_ops)
        if backward is not None:
            extras.update(bw_out=bw_out, obj_h=obj_h, wrt_h=wrt_h)

    P_k = int(out["kept_count"][0])
    T_c = int(np.count_nonzero(out["tensor_mask"]))
    fan_in = np.bincount(g.in_op, minlength=P)
    E_k = int(fan_in[out["kept_ops"]].sum())
    n_out = np.bincount(g.out_op, minlength=P)
    Eo_k = int(n_out[out["kept_ops"]].sum())
    # edges that one run of Algorithm 1 per target set would have gone through, summed over the sets
    sets_of = np.bitwise_count(out["kept_masks"][:P_k]).astype(np.int64)
    E_query = int(((fan_in[out["kept_ops"][:P_k]] + n_out[out["kept_ops"][:P_k]]) * sets_of).sum())

    # ---- algorithmic bytes per kernel launch (int32 ids, uint64 masks) ---------------------------
    wide = max(1, level_launches)
    traversal_bytes = 4 * T_c + 8 * P_k + 4 * E_k + 16 * E_k + 16 * P_k
    alg = {
        # all of M and K, or (recycled buffers) the log and the kept list read, their M, K and marker words zeroed
        # (a packed batch swept per graph stores K of every operator: only M is cleared)
        "k_clear": (12 * T_c + 13 * P_k) if recycled else (8 * T) if levels_total == 0 and g.num_graphs >= 64
                   else (8 * T + 8 * P),
        # the traversal's bytes per wide launch (the launches the events and the profiler time)
        "k_level": traversal_bytes / wide,
        # stand-alone: K from M; large single graphs: keep flags (P bytes) read, K of the kept operators, bitmap
        # written; else all of K read, flags written
        "k_keep_count": (4 * P + 12 * g.nnz_out + 8 * P + P) if args.recompute_keep
                        else (P + 8 * P_k + P // 8) if (g.num_graphs == 1 and P >= (1 << 22)) else (8 * P + P),
        "k_scatter": 12 * P_k,
    }
    dur_ms = {
        "k_clear": ph["clear"],
        "k_level": ph["traverse"] / wide,
        "k_keep_count": ph["count"],
        "k_scatter": ph["scatter"],
    }
    tot_ms = {"k_clear": ph["clear"], "k_level": ph["traverse"], "k_keep_count": ph["count"],
              "k_scatter": ph["scatter"]}
    dominant = max(tot_ms, key=tot_ms.get)
    achieved = alg[dominant] / (dur_ms[dominant] * 1e-3) / 1e9 if dur_ms[dominant] > 0 else 0.0
    b_alg_total = alg["k_clear"] + traversal_bytes + alg["k_keep_count"] + alg["k_scatter"]
    counters_apply = args.config == 3 and args.scale == 1.0 and not args.recompute_keep
    traffic = measured_traffic(dominant) if counters_apply else None
    roofline = {
        "bound": "hbm", "kernel": dominant, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
        "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
        "traffic": traffic,
        # the same kernel's measured HBM bytes per launch over its launch time: what the memory system is asked for,
        # as opposed to the algorithmic bytes behind `achieved` (random 8-byte accesses move whole 64-byte sectors)
        "traffic_GBs": None if not traffic or dur_ms[dominant] <= 0 else round(traffic / (dur_ms[dominant] * 1e-3) / 1e9, 1),
        "traffic_frac": None if not traffic or dur_ms[dominant] <= 0
                        else round(traffic / (dur_ms[dominant] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "traffic_source": (COUNTERS + " (committed rocprofv3 --pmc summary, not measured in this run; null when the kernel "
                           "sources have changed since)"),
        "launch_ms": round(dur_ms[dominant], 4), "launches_per_step": 1 if dominant != "k_level" else level_launches,
        "k_level_launch_ms_device_clock": None if level_us_device_clock is None else round(level_us_device_clock / 1e3, 4),
        "per_kernel_GBs": {k: round(alg[k] / (dur_ms[k] * 1e-3) / 1e9, 1) if dur_ms[k] > 0 else None for k in alg},
        "whole_path_algorithmic_GBs": round(b_alg_total / (ms_per_step * 1e-3) / 1e9, 1),
        "whole_path_frac": round(b_alg_total / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "measured_copy_GBs": copy_gbs,
        "whole_path_measured_GBs": None, "whole_path_measured_frac": None,
        "atomics": None, "latency_floor_ms": None, "machine_rates": rates,
    }
    # What does bound the traversal: the 64-bit atomics it issues, against the rate this GPU sustains for random
    # atomics over an array of the masks' size; and its chain of dependent accesses -- per wide level a launch and
    # five accesses that each need the one before (state, stamp bytes or queue entry, operator record, output
    # masks / input ids, atomic), per level of the single-workgroup kernel three loads and an atomic -- at the
    # unloaded latencies measured on this GPU
    if rates is not None and ph["traverse"] > 0:
        a_gps = atomics_per_step / (ph["traverse"] * 1e-3) / 1e9
        roofline["atomics"] = {"per_step": atomics_per_step, "achieved_Gps": round(a_gps, 2),
                               "ceiling_Gps": rates["random_atomic_gps"],
                               "frac": round(a_gps / rates["random_atomic_gps"], 4) if rates["random_atomic_gps"] else None,
                               "throughput_floor_ms": round(atomics_per_step / (rates["random_atomic_gps"] * 1e9) * 1e3, 4)
                                                     if rates["random_atomic_gps"] else None}
        # Random accesses as a whole: per operator visit its record, K, the outputs' masks and the input ids (one
        # memory sector each), per input edge the producer word beside the atomic.  A random load issued together with
        # an atomic costs what the pair rate says on top of the atomic (about a third of a load on its own).
        pair, ra = rates.get("random_load_and_atomic_gps"), rates["random_atomic_gps"]
        if pair and ra and stats_visits is not None:
            loads = 4 * stats_visits + max(atomics_per_step - stats_visits, 0)
            per_load_ns = max(1.0 / pair - 1.0 / ra, 0.0)
            floor_ms = (atomics_per_step / ra + loads * per_load_ns) / 1e9 * 1e3
            roofline["random_access"] = {"atomics_per_step": atomics_per_step, "loads_per_step_model": loads,
                                         "ns_per_atomic": round(1.0 / ra, 4), "ns_per_load_beside_an_atomic": round(per_load_ns, 4),
                                         "floor_ms": round(floor_ms, 4),
                                         "frac": round(floor_ms / ph["traverse"], 4)}
        chain_wide = rates["launch_back_to_back_us"] + (4 * rates["dependent_load_ns"] + rates["dependent_atomic_ns"]) / 1e3
        chain_narrow = (3 * rates["dependent_load_ns"] + rates["dependent_atomic_ns"]) / 1e3
        roofline["latency_floor_ms"] = round((level_launches * chain_wide + narrow_levels * chain_narrow) / 1e3, 4)
        roofline["latency_floor_levels"] = {"wide_launches": level_launches, "single_workgroup_levels": narrow_levels,
                                            "us_per_wide_level": round(chain_wide, 2),
                                            "us_per_single_workgroup_level": round(chain_narrow, 2)}

    # bytes that crossed the HBM interface in one prune according to the committed counter runs (every kernel of the
    # step: the level kernel once per launch), over the step time
    if traffic is not None and recycled and dominant == "k_level":
        others = [measured_traffic(k) for k in ("k_clear", "k_keep_count", "k_scatter")]
        if all(v is not None for v in others):
            moved = sum(others) + traffic * level_launches
            roofline["whole_path_measured_GBs"] = round(moved / (ms_per_step * 1e-3) / 1e9, 1)
            roofline["whole_path_measured_frac"] = round(moved / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)

    # ---- CPU baseline: the oracle as it stands, on this machine's host cores -------------------------
    cpu = None
    parity = None
    orc = None
    if not args.no_cpu_baseline:
        import oracle as orc
        tb = time.time()
        adj = orc.build_adjacency(P, T, g.in_op, g.in_tensor, g.out_op, g.out_tensor)
        adj_s = time.time() - tb
        times = []
        for _ in range(3):
            tb = time.perf_counter()
            ref = orc.forward_prune(adj, tg.num_sets, tg.tgt_rowptr, tg.tgt_idx, g.num_graphs, g.graph_op_offsets)
            times.append(time.perf_counter() - tb)
            if sum(times) > 30:
                break
        cpu_s = float(np.median(times))
        cpu = {"value": round(E / cpu_s / 1e9, 5), "unit": "GTEPS", "cores": 1, "kind": "oracle",
               "sample": f"whole workload ({g.name}, all {tg.num_sets} target sets), adjacency prebuilt "
                         f"({adj_s:.1f}s, untimed), median of {len(times)} runs = {cpu_s:.2f}s",
               "host_cores_available": os.cpu_count()}
        parity = all(np.array_equal(out[k], getattr(ref, k)) for k in
                     ("tensor_mask", "op_mask", "op_flag", "kept_ops", "kept_masks", "kept_count", "per_query_count"))
        log(f"oracle: {cpu_s:.2f}s -> {cpu['value']} GTEPS on 1 core; GPU output bit-exact vs oracle: {parity}")
        assert parity, "GPU result differs from the oracle"
    if cpu is not None and inplace is not None:
        ip_rename, ro_rowptr, ro_ignore, ro_ops = (extras[k] for k in ("ip_rename", "ro_rowptr", "ro_ignore", "ro_ops"))
        tb = time.perf_counter()
        ref_rd = orc.inplace(adj, ref.op_mask)
        inplace["cpu_oracle_ms"] = round((time.perf_counter() - tb) * 1e3, 1)
        inplace["bit_exact_vs_oracle"] = bool(np.array_equal(ip_rename, ref_rd))
        log(f"oracle in-place pass: {inplace['cpu_oracle_ms']:.0f} ms; GPU rename dictionary bit-exact: "
            f"{inplace['bit_exact_vs_oracle']}")
        assert inplace["bit_exact_vs_oracle"], "GPU rename dictionary differs from the oracle"
        ref_ig = orc.ignore_mask(adj, ref.op_mask, ref.tensor_mask)
        same_lists = True
        if ro_rowptr is not None:
            ref_rowptr, ref_ops = orc.per_set_lists(ref.op_mask)
            same_lists = np.array_equal(ro_rowptr, ref_rowptr) and np.array_equal(ro_ops, ref_ops)
        readout["bit_exact_vs_oracle"] = bool(np.array_equal(ro_ignore, ref_ig) and same_lists)
        assert readout["bit_exact_vs_oracle"], "GPU read-outs differ from the oracle"
        if backward is not None:                 # one pair (a graph-wide search each): the bounded sample
            bw_out, obj_h, wrt_h = extras["bw_out"], extras["obj_h"], extras["wrt_h"]
            i = int(np.flatnonzero(bw_out["per_query_count"])[0]) if backward["connected_pairs"] else 0
            tb = time.perf_counter()
            ref_m = orc.backward_mark(adj, obj_h[i:i + 1], wrt_h[i:i + 1])
            backward["cpu_oracle_ms_per_pair"] = round((time.perf_counter() - tb) * 1e3, 1)
            same = bool(np.array_equal((bw_out["tensor_mask"] >> np.uint64(i)) & np.uint64(1), ref_m))
            backward["bit_exact_vs_oracle_sampled_pair"] = same
            log(f"oracle backward prune, pair {i}: {backward['cpu_oracle_ms_per_pair']:.0f} ms; GPU marks bit-exact: {same}")
            assert same, "GPU backward-prune marks differ from the oracle"

    # ---- the workloads the metric is not quoted on, each built, pruned and checked on its own ------
    others_out = None
    if not (args.no_other_configs or args.prune_only) and args.scale == 1.0:
        del buf, dg, graph_mem, out, extras
        if cpu is not None:
            del adj, ref
        torch.cuda.empty_cache()
        others_out = {}
        for k in (0, 1, 2, 4):
            if k == args.config:
                continue
            others_out[f"config{k}"] = other_config(d, torch, np, gg, orc, k, args.steps, args.warmup, cpu is not None)

    line = {
        "metric": "pruned edges/sec (GTEPS), 64-query batched prune", "value": round(gteps, 2), "unit": "GTEPS",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u64", "data": "synthetic",
        # the same steps with every word of M and K cleared inside each step (a stateless call)
        "value_full_clear": None if full_clear is None else full_clear["gteps"],
        "ms_per_step_full_clear": None if full_clear is None else full_clear["ms_per_step"],
        "query_gteps": round(E_query / (ms_per_step * 1e-3) / 1e9, 2), "steps_timed_one_by_one_ms": one_by_one,
        "config": {"workload": f"configs[{args.config}] {g.name}" + ("" if args.scale == 1.0 else f" x{args.scale}"),
                   "num_ops": P, "num_tensors": T, "nnz_in": g.nnz_in, "nnz_out": g.nnz_out,
                   "num_sets": tg.num_sets, "num_graphs": g.num_graphs,
                   "keep_pass": "stand-alone" if args.recompute_keep else "fused into traversal",
                   "output_buffers": "recycled: each step zeroes what the previous step set" if recycled
                                     else "every word of M and K cleared each step"},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "phase_ms": {k: round(v, 4) for k, v in ph.items()},
        "build_ms": round(build_ms, 3),
        "build_shuffled_ms": None if build_shuffled_ms is None else round(build_shuffled_ms, 3),
        "inplace": inplace,
        "readout": readout,
        "backward_prune": backward,
        "incremental_prune": incremental,
        "full_clear_per_step": full_clear,
        "recycled_alternating_targets": other_targets,
        "transaction_cache": transaction,
        "other_configs": others_out,
        "build_plus_prune_gteps": round(E / ((build_ms + ms_per_step) * 1e-3) / 1e9, 2),
        "result": {"kept_ops": P_k, "coloured_tensors": T_c, "kept_in_edges": E_k, "kept_out_edges": Eo_k,
                   "levels": levels_total, "operator_visits": int(st.tensor_visits), "atomic_updates": atomics_per_step,
                   "max_queue": int(st.max_frontier), "launches": launches_total,
                   "bit_exact_vs_oracle": parity},
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
