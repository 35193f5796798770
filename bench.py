#!/usr/bin/env python3
"""Benchmark of the sampler's hot path on one MI355X.

A "step" is one gss_step (all hops: read snapshot, refresh, draw, dedupe/relabel, emit blocks) over one
batch of seeds; FCR full refreshes fall inside the timed region.  Inputs (CSR, seeds) are resident in HBM
before the clock starts.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg4_large_shared] [--only]

The line's headline is --workload (default: the largest configuration, cfg4_large_shared); the other four
configurations are measured in the same run and reported under "other_workloads" (--only skips them).
Per workload: the fill/drain-inclusive time of exactly K steps (ms_per_step, value), the steady-state time per step
with the pipeline full at both ends of the window (steady_ms_per_step), the time of one blocking gss_step alone
(blocking_step_ms), the roofline figures of the dominant kernel and the oracle on one host core.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth
VALU_PEAK_GINST = 256 * 4 * 2.4 / 4   # G wavefront-wide 32-bit vector instructions per second: CUs x SIMDs x GHz / 4 cycles each


def byte_model(w, indptr_bytes):
    """Algorithmic bytes per unit - what the method must move, sector granularity not counted:
      per frontier node and hop  4 (id) + 4k (cached row)
                                 + per-visit refresh (OTF, shared OTF): 2 indptr words + 8 n_new (n_new adjacency
                                   reads and n_new row writes), + 8 (stamp read / write) with the shared table
      per sampled edge           32 = 4 (pick write) + 4 (pick read) + 16 (dedupe insert: 8 read + 8 atomic) + 8 (COO)
      per new source node        8 = 4 (src_nodes write) + 4 (read as next frontier)
    FBL keeps no row: per node 4 + 2 indptr words, and 4 more per edge (the adjacency entry of the draw).
    OTF fetch: the row and 2 indptr words per node, 4 more for the fetched share of the edges.
    The implementation's own extra traffic (the mark phase probes the dedupe word again: 8 per edge) is returned
    separately and never enters `achieved`."""
    k = w.k
    otf = w.mode in (1, 2)
    n_new = int(w.refresh_fraction * k + 1e-9) if otf else 0
    per_node = 4 + 4 * k
    per_edge = 32
    if otf:
        per_node += 2 * indptr_bytes + 8 * n_new + (8 if w.mode == 2 else 0)
    if w.mode == 3:
        per_node = 4 + 2 * indptr_bytes
        per_edge += 4
    if w.mode == 5:
        per_node += 2 * indptr_bytes
        per_edge += 4 * w.refresh_fraction
    return dict(per_node=per_node, per_edge=per_edge, per_unique=8, impl_extra_per_edge=8)


def algorithmic_bytes(w, counts, indptr_bytes):
    nodes, edges, uniq = counts
    m = byte_model(w, indptr_bytes)
    return nodes * m["per_node"] + edges * m["per_edge"] + uniq * m["per_unique"]


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def fill_full_bytes(w, graph):
    """One refresh of every table of a set that was filled before: only the rows of nodes with more than k neighbors
    are recomputed (the others hold the whole adjacency): per such row the node id and two indptr words, and per table
    the adjacency entries the row must read + the row written."""
    total = 0
    ntab = 0 if w.mode == 3 else (1 if w.mode in (2, 4) else len(w.fanouts))   # (OTF_LAYER: counted like a fill)
    theta = max(w.k, getattr(w, "degree_threshold", -1))
    for r in graph.relations:
        deg = np.diff(r.indptr)
        heavy = deg[deg > theta]
        reads = np.where(heavy < 2 * w.k, heavy, w.k).sum() * 4
        total += (4 + 2 * r.indptr.itemsize) * len(heavy) + ntab * (int(reads) + 4 * w.k * len(heavy))
    return total


TUNING = {}       # --tuning field=value ...: layout choices (gss_tuning) for every sampler of the run; results do not depend on them


def make_sampler(w, dev_rels, graph):
    from paper_2406_17918_amd import gss
    return gss.Sampler(graph.num_nodes, dev_rels, k=w.k, mode=w.mode, num_layers=len(w.fanouts),
                       refresh_fraction=w.refresh_fraction, refresh_period=w.refresh_period, rng_seed=w.rng_seed,
                       degree_threshold=getattr(w, "degree_threshold", -1), tuning=dict(TUNING))


def run_gpu(w, graph, steps, warmup, profile_steps, steady_steps=0, blocking_steps=0):
    """Timed passes over consecutive step numbers of ONE sampler:
      1. `warmup` untimed steps, then exactly `steps` steps between two device synchronisations (the pipeline fills
         and drains inside the timed region);
      2. steady state: 2 * depth + `steady_steps` steps in one uninterrupted stream; the window runs from the
         completion of the step after which the pipeline has been full for `depth` steps to the completion of the
         step `steady_steps` later (host clock at the return of gss_step_wait);
      3. `profile_steps` steps with HIP-event brackets attached to every kernel dispatch (on the library's stream);
      4. `blocking_steps` blocking gss_step calls, nothing else in flight: the latency of one step alone."""
    import torch
    from paper_2406_17918_amd import gss
    dev_rels = gss.upload_graph(graph)
    s = make_sampler(w, dev_rels, graph)
    depth = s.pipeline_depth
    n_steady = (2 * depth + steady_steps) if steady_steps else 0
    n_total = warmup + steps + n_steady + profile_steps + blocking_steps
    seeds = [torch.from_numpy(w.seeds(graph, i)).cuda() for i in range(n_total)]
    cache_bytes = s.cache_bytes()

    def run_steps(first, last, on_done=None):
        # up to gss_pipeline_depth() steps are enqueued before the oldest is collected, so the GPU never waits for the host
        edges = 0
        inflight = 0
        for i in range(first, last):
            s.step_async(seeds[i], w.fanouts, i, w.seed_type)
            inflight += 1
            if inflight == depth:
                b = s.step_wait_raw()
                edges += b.total_edges
                inflight -= 1
                if on_done:
                    on_done(b)
        while inflight:
            b = s.step_wait_raw()
            edges += b.total_edges
            inflight -= 1
            if on_done:
                on_done(b)
        return edges

    pos = 0
    run_steps(pos, pos + warmup)            # untimed, same launch configuration as the timed region
    pos += warmup
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    edges = run_steps(pos, pos + steps)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    pos += steps
    res = dict(seconds=dt, edges=int(edges), prof={}, prof_counts=(0, 0, 0), prof_refreshes=0, prof_steps=0,
               cache_bytes=cache_bytes, depth=depth, steady=None, blocking=None)

    if n_steady:
        stamps, sedges = [], []

        def done(b):
            stamps.append(time.perf_counter())
            sedges.append(b.total_edges)
        run_steps(pos, pos + n_steady, done)
        torch.cuda.synchronize()
        pos += n_steady
        lo, hi = depth - 1, depth - 1 + steady_steps     # completions of steps lo and hi: full pipeline in between
        res["steady"] = dict(seconds=stamps[hi] - stamps[lo], steps=steady_steps, edges=int(sum(sedges[lo + 1:hi + 1])))

    if profile_steps:
        s.profile_enable(True)
        T, R = len(graph.num_nodes), len(graph.relations)
        nodes = pe = uniq = 0

        def account(b):
            nonlocal nodes, pe, uniq
            pe += b.total_edges
            for l in range(b.num_layers):
                for t in range(T):
                    nd = b.nodes[l * T + t]
                    uniq += nd.num_src - nd.num_dst
                for r in range(R):
                    nodes += b.nodes[l * T + graph.relations[r].dst_type].num_dst
        run_steps(pos, pos + profile_steps, account)
        refreshes = 0
        if w.mode in (0, 4, 6):
            refreshes = sum(1 for i in range(pos, pos + profile_steps) if i % w.refresh_period == 0 and i > 0)
        pos += profile_steps
        res.update(prof=s.profile_read(), prof_counts=(nodes, pe, uniq), prof_refreshes=refreshes, prof_steps=profile_steps)
        s.profile_enable(False)

    if blocking_steps:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(pos, pos + blocking_steps):
            s.step_raw(seeds[i], w.fanouts, i, w.seed_type)
        res["blocking"] = dict(seconds=time.perf_counter() - t0, steps=blocking_steps)
        pos += blocking_steps
    s.close()
    return res


def run_oracle(w, graph, first_step, max_steps, budget_s):
    """The oracle as it stands, one thread, on the steps first_step, first_step + 1, ... of the same workload (the
    steps before them are run untimed, so that its cache is in the state the GPU's timed region starts from), until
    `max_steps` steps or `budget_s` seconds.  It counts its own edges."""
    from oracle import gsso
    import ctypes as C
    rels = [gsso.Relation(r.src_type, r.dst_type, r.indptr, r.indices) for r in graph.relations]
    o = gsso.Sampler(graph.num_nodes, rels, k=w.k, mode=w.mode, num_layers=len(w.fanouts),
                     refresh_fraction=w.refresh_fraction, refresh_period=w.refresh_period, rng_seed=w.rng_seed,
                     degree_threshold=getattr(w, "degree_threshold", -1))
    lib = gsso.lib()
    fo = (C.c_int32 * len(w.fanouts))(*w.fanouts)
    p32 = C.POINTER(C.c_int32)
    L, R = len(w.fanouts), len(graph.relations)
    ne, pa, pb = C.c_int32(), p32(), p32()

    def one(i):
        sd = np.ascontiguousarray(w.seeds(graph, i))
        t0 = time.perf_counter()
        st = lib.gsso_step(o._h, sd.ctypes.data_as(p32), len(sd), w.seed_type, fo, L, i)
        dt = time.perf_counter() - t0
        assert st == 0
        e = 0
        for l in range(L):
            for r in range(R):
                lib.gsso_block_edges(o._h, l, r, C.byref(ne), C.byref(pa), C.byref(pb))
                e += ne.value
        return dt, e

    for i in range(first_step):
        one(i)
    seconds, edges, n = 0.0, 0, 0
    while n < max_steps and (seconds < budget_s or n < 2):
        dt, e = one(first_step + n)
        seconds += dt
        edges += e
        n += 1
    o.close()
    return dict(seconds=seconds, edges=edges, steps=n)


_TRAFFIC = None


def recorded_traffic(workload, kernel, lib_version, table="bytes_per_launch"):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE, each scaled by a plain copy of
    known size) - a RECORDED figure, kept in profiles/traffic.json together with the version string of the library
    it was measured on; None when the library has changed since.  table="valu_insts_per_launch" gives the
    SQ_INSTS_VALU count of the same kind of run instead."""
    global _TRAFFIC
    if _TRAFFIC is None:
        try:
            _TRAFFIC = json.load(open(os.path.join(ROOT, "profiles", "traffic.json")))
        except Exception:
            _TRAFFIC = {}
    if _TRAFFIC.get("library_version") != lib_version:
        return None
    return _TRAFFIC.get(table, {}).get(workload, {}).get(kernel)


def roofline_of(w, graph, res, lib_version):
    """step_tick is the kernel every phase of every step runs in (one launch carries one phase of each step in
    flight); fill_full is the FCR refresh.  Algorithmic bytes per launch = the bytes of the profiled steps divided by
    the launches that processed them."""
    prof, (nodes, edges, uniq) = res["prof"], res["prof_counts"]
    indptr_bytes = graph.relations[0].indptr.itemsize
    per_kernel = {}
    for name, (ms, launches) in prof.items():
        if launches == 0:
            continue
        if name == "fill_full":
            total_bytes = fill_full_bytes(w, graph) * res["prof_refreshes"]
        else:
            total_bytes = algorithmic_bytes(w, (nodes, edges, uniq), indptr_bytes)
        per_kernel[name] = dict(ms_total=ms, launches=int(launches), avg_us=1e3 * ms / launches,
                                alg_bytes_per_launch=total_bytes / launches,
                                gbs=(total_bytes / launches) / (1e-3 * ms / launches) / 1e9 if ms > 0 else 0.0)
    dom = max(per_kernel, key=lambda n: per_kernel[n]["ms_total"])
    d = per_kernel[dom]
    m = byte_model(w, indptr_bytes)
    roof = dict(bound="hbm", kernel=dom, achieved=round(d["gbs"], 3), peak=HBM_PEAK_GBS, unit="GB/s",
                frac=round(d["gbs"] / HBM_PEAK_GBS, 6),
                traffic=recorded_traffic(w.name, dom, lib_version),
                traffic_kind="recorded: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs summarised in profiles/ (null: none for this library version)",
                avg_launch_us=round(d["avg_us"], 3), alg_bytes_per_launch=round(d["alg_bytes_per_launch"], 1),
                launches_per_step=round(d["launches"] / max(res["prof_steps"], 1), 3),
                byte_model=m,
                impl_extra_bytes_per_launch=round(edges * m["impl_extra_per_edge"] / d["launches"], 1) if dom == "step_tick" else 0)
    kernels = {n: dict(avg_us=round(v["avg_us"], 3), launches=v["launches"], alg_gbs=round(v["gbs"], 3))
               for n, v in per_kernel.items()}
    # The sampling phases are bound by vector-instruction issue, not by HBM: the same launches against that roof.
    # achieved = VALU instructions issued per launch (SQ_INSTS_VALU, one count per wavefront instruction; recorded
    # like `traffic`) / the launch duration measured here.  peak = 256 CUs x 4 SIMDs x 2.4 GHz / 4 cycles per
    # wavefront instruction (a SIMD has 16 lanes: a 64-wide wavefront takes 4 cycles per 32-bit vector instruction;
    # the published 157.3 TFLOP/s of fp32 is this rate x 64 lanes x 2 flops x 2 for the packed forms).
    alu = None
    if "step_tick" in per_kernel:
        t = per_kernel["step_tick"]
        valu = recorded_traffic(w.name, "step_tick", lib_version, "valu_insts_per_launch")
        rate = valu / (1e-6 * t["avg_us"]) / 1e9 if valu else None
        alu = dict(bound="alu", kernel="step_tick", achieved=round(rate, 3) if rate else None, peak=VALU_PEAK_GINST,
                   unit="G wavefront VALU instructions/s", frac=round(rate / VALU_PEAK_GINST, 6) if rate else None,
                   valu_insts_per_launch=valu,
                   valu_insts_per_visited_node=round(valu * t["launches"] / max(nodes, 1), 1) if valu else None,
                   kind="recorded count (rocprofv3 --pmc SQ_INSTS_VALU, profiles/) over the live launch duration; null: none for this library version")
    return roof, kernels, alu


MODE_NAMES = ["FCR", "OTF", "SHARED_OTF", "FBL", "SHARED_FCR", "OTF_FETCH", "OTF_LAYER"]


def measure_workload(w, graph, steps, warmup, cpu_budget_s, lib_version):
    """Every figure of one workload (see run_gpu); the oracle leg is skipped when cpu_budget_s == 0."""
    steady_steps = max(steps, 200)
    res = run_gpu(w, graph, steps, warmup, profile_steps=max(steps, 100), steady_steps=steady_steps, blocking_steps=20)
    roof, kernels, alu = roofline_of(w, graph, res, lib_version)
    indptr_bytes = graph.relations[0].indptr.itemsize
    step_bytes = algorithmic_bytes(w, res["prof_counts"], indptr_bytes) / max(res["prof_steps"], 1)
    st = res["steady"]
    steady_ms = 1e3 * st["seconds"] / st["steps"]
    cpu = None
    if cpu_budget_s > 0:
        o = run_oracle(w, graph, warmup, 5000, cpu_budget_s)
        cpu = dict(value=round(o["edges"] / o["seconds"], 1), unit="sampled edges/s", cores=1, kind="oracle",
                   sample=f"steps {warmup} .. {warmup + o['steps'] - 1} of {w.name} (the step numbers the timed region starts at; as many as "
                          f"fit the time bound) after the same {warmup} warmup steps "
                          f"({o['seconds']:.2f} s of single-thread CPU work, {o['edges']} edges counted by the oracle itself; "
                          f"cache initialisation excluded)",
                   host_cpus=os.cpu_count(), host_cpu_model=cpu_model())
    return {
        "value": round(res["edges"] / res["seconds"], 1), "unit": "sampled edges/s",
        "ms_per_step": round(1e3 * res["seconds"] / steps, 5),
        "steady_ms_per_step": round(steady_ms, 5),
        "steady_value": round(st["edges"] / st["seconds"], 1),
        "steady_window_steps": st["steps"],
        "blocking_step_ms": round(1e3 * res["blocking"]["seconds"] / res["blocking"]["steps"], 5),
        "pipeline_depth": res["depth"],
        "config": {"workload": w.name, "graph": graph.meta, "nodes": graph.num_nodes,
                   "csr_entries": [int(len(r.indices)) for r in graph.relations], "batch": w.batch,
                   "fanouts": w.fanouts, "k": w.k, "mode": MODE_NAMES[w.mode],
                   "refresh_fraction": w.refresh_fraction, "refresh_period": w.refresh_period,
                   "stands_in_for": w.stands_in_for},
        "seeds_per_s": round(w.batch * steps / res["seconds"], 1),
        "steady_seeds_per_s": round(w.batch / (1e-3 * steady_ms), 1),
        "edges_per_step": round(res["edges"] / steps, 1),
        # algorithmic bytes over the kernel's own time, and over the wall time of a steady-state step (the gap is
        # launch latency and idle time between launches)
        "hbm_pct_of_peak": round(100.0 * roof["frac"], 4),
        "hbm_pct_of_peak_wall": round(100.0 * step_bytes / (1e-3 * steady_ms) / 1e9 / HBM_PEAK_GBS, 4),
        "alg_bytes_per_step": round(step_bytes, 1),
        "cache_bytes": res["cache_bytes"],
        "cache_bytes_logical": logical_cache_bytes(w, graph),
        "roofline": roof, "roofline_alu": alu, "kernels": kernels, "cpu_baseline": cpu,
    }


def logical_cache_bytes(w, graph):
    """The [tables, N, k] int32 cells of the cache as the paper counts it (one table set, no row padding)."""
    ntab = 0 if w.mode == 3 else (1 if w.mode in (2, 4) else len(w.fanouts))
    return int(sum(4 * w.k * ntab * (len(r.indptr) - 1) for r in graph.relations))


def paper_table(graph_name, steps, warmup):
    """The paper's method comparison (Table "Training Time Acceleration Across Methods": FBL, FCR, FCR-shared cache,
    OTF, OTF-shared cache at fanouts [20,20,20] / [10,10,10] / [5,5,5]) measured on this sampler: ms per minibatch
    step of 1,024 seeds (steady state, pipeline full) and the acceleration relative to FBL.  Per-layer cache rows are
    k = 2f wide; a shared table holds k = 3f slots, so that the three layers' bands partition the row."""
    import copy
    from paper_2406_17918_amd import synth
    base = synth.WORKLOADS[graph_name]
    graph = base.make_graph()
    rows = {}
    for f in (20, 10, 5):
        fan = [f, f, f]
        methods = [("FBL", synth.MODE_FBL, 2 * f, 0.0, 1),
                   ("FCR", synth.MODE_FCR, 2 * f, 0.0, 10),
                   ("FCR-shared cache", synth.MODE_SHARED_FCR, 3 * f, 0.0, 10),
                   ("OTF", synth.MODE_OTF, 2 * f, 0.2, 1),
                   ("OTF-shared cache", synth.MODE_SHARED_OTF, 3 * f, 0.1, 1),
                   ("OTF fetch, delta 0.5 (not in the paper's table)", synth.MODE_OTF_FETCH, 2 * f, 0.5, 1),
                   ("OTF, layer-wide refresh every 10 steps (not in the paper's table)", synth.MODE_OTF_LAYER,
                    2 * f, 0.2, 10)]
        for name, mode, k, frac, period in methods:
            w = copy.copy(base)
            w.fanouts, w.k, w.mode, w.refresh_fraction, w.refresh_period, w.batch = fan, k, mode, frac, period, 1024
            r = run_gpu(w, graph, steps, warmup, profile_steps=0, steady_steps=max(steps, 200))
            st = r["steady"]
            rows.setdefault(name, {})[str(fan)] = dict(ms_per_step=round(1e3 * st["seconds"] / st["steps"], 5),
                                                         edges_per_step=round(st["edges"] / st["steps"], 1), k=k)
    for name, d in rows.items():
        for key, v in d.items():
            ref = rows["FBL"][key]
            if name != "FBL":
                v["acceleration_pct_vs_fbl"] = round(100.0 * (1.0 - v["ms_per_step"] / ref["ms_per_step"]), 2)
    print(json.dumps({"metric": "ms per minibatch step by cache method (the paper's method table, measured on MI355X)",
                      "graph": graph_name, "nodes": graph.num_nodes, "batch": 1024, "steps": steps, "warmup": warmup,
                      "table": rows}))


def degree_split_table(graph_name, steps, warmup):
    """The dense/sparse split ("Graph Splitting and Sampling Strategies") measured on --workload: cache memory and
    ms per step without a split and with the degree threshold theta at k, 2k, 4k and 8k (nodes with deg <= theta
    keep no cache row and are sampled by the FBL draw)."""
    import copy
    from paper_2406_17918_amd import synth
    base = synth.WORKLOADS[graph_name]
    graph = base.make_graph()
    deg = [np.diff(r.indptr) for r in graph.relations]
    rows = []
    for theta in (-1, base.k, 2 * base.k, 4 * base.k, 8 * base.k):
        w = copy.copy(base)
        w.degree_threshold = theta
        r = run_gpu(w, graph, steps, warmup, profile_steps=0)
        dense = sum(int((d > theta).sum()) for d in deg) if theta >= 0 else sum(len(d) for d in deg)
        rows.append(dict(theta=theta, cached_rows=dense, cached_row_share=round(dense / sum(len(d) for d in deg), 5),
                         cache_bytes=r["cache_bytes"], ms_per_step=round(1e3 * r["seconds"] / steps, 5),
                         edges_per_s=round(r["edges"] / r["seconds"], 1)))
    print(json.dumps({"metric": "cache memory and ms per minibatch step by degree threshold (dense/sparse split)",
                      "workload": graph_name, "nodes": graph.num_nodes, "k": base.k, "steps": steps, "warmup": warmup,
                      "table": rows}))


def gather_bench(w, graph, steps, warmup, dim):
    """Feature gather for the input side of sampled minibatches: H[src_nodes] with H = [N, dim] float32.  The ids are the
    layer-0 src_nodes of `steps` real sampler steps; each gather is one launch, timed with HIP events on the stream it
    runs on.  Algorithmic bytes per gathered row: dim*4 read + dim*4 written + 4 (the id)."""
    import torch
    from paper_2406_17918_amd import gss
    dev_rels = gss.upload_graph(graph)
    s = gss.Sampler(graph.num_nodes, dev_rels, k=w.k, mode=w.mode, num_layers=len(w.fanouts),
                    refresh_fraction=w.refresh_fraction, refresh_period=w.refresh_period, rng_seed=w.rng_seed)
    t = w.seed_type
    ids = []
    for i in range(warmup + steps):
        b = s.step(torch.from_numpy(w.seeds(graph, i)).cuda(), w.fanouts, i, w.seed_type)
        ids.append(b[0].src_nodes[t].clone())
    s.close()
    feats = torch.empty((graph.num_nodes[t], dim), dtype=torch.float32, device="cuda").normal_()
    outs = [torch.empty((x.numel(), dim), dtype=torch.float32, device="cuda") for x in ids[:4]]
    for i in range(warmup):
        gss.gather_rows(feats, ids[i], outs[i % 4][:ids[i].numel()] if outs[i % 4].shape[0] >= ids[i].numel() else None)
    big = torch.empty((max(x.numel() for x in ids), dim), dtype=torch.float32, device="cuda")
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for j, i in enumerate(range(warmup, warmup + steps)):
        ev[j][0].record()
        gss.gather_rows(feats, ids[i], big[:ids[i].numel()])
        ev[j][1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    rows = sum(x.numel() for x in ids[warmup:])
    kernel_ms = sum(a.elapsed_time(b) for a, b in ev)
    per_row = 8 * dim + 4
    gbs = rows * per_row / (kernel_ms * 1e-3) / 1e9
    print(json.dumps({
        "metric": "feature gather for sampled minibatches: gathered rows/s + achieved HBM GB/s % of peak",
        "value": round(rows / dt, 1), "unit": "rows/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": round(1e3 * dt / steps, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name + " + feature gather", "feature_dim": dim, "rows_per_step": round(rows / steps, 1),
                   "table_rows": graph.num_nodes[t], "batch": w.batch},
        "roofline": {"bound": "hbm", "kernel": "gather_rows", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": None, "avg_launch_us": round(1e3 * kernel_ms / steps, 2),
                     "alg_bytes_per_launch": round(rows * per_row / steps, 1)},
        "cpu_baseline": None}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--workload", default="cfg4_large_shared",
                    help="the headline workload of the line (default: the largest single-GPU configuration)")
    ap.add_argument("--only", action="store_true", help="measure --workload alone (the default line also carries the other four)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0,
                    help="bound of the oracle's timed work on the headline workload (the others get a third of it each)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="first run a plain 256 MiB device copy (a kernel of known traffic, to scale rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--batch", type=int, default=0,
                    help="override the workload's batch size (throughput-regime sweeps; not one of the five configurations)")
    ap.add_argument("--paper-table", action="store_true",
                    help="instead of the benchmark line, print the paper's five-method comparison measured on --workload's graph")
    ap.add_argument("--degree-split-table", action="store_true",
                    help="instead of the benchmark line, print cache memory and ms per step of --workload by degree threshold")
    ap.add_argument("--gather", action="store_true",
                    help="instead of the sampler benchmark, time the feature gather H[src_nodes] on --workload's minibatches")
    ap.add_argument("--feature-dim", type=int, default=128)
    ap.add_argument("--tuning", nargs="*", default=[], metavar="FIELD=VALUE",
                    help="fields of gss_tuning (launch layout choices; A/B measurements), e.g. visit_once=2 pipeline_depth=8")
    a = ap.parse_args()
    for kv in a.tuning:
        key, val = kv.split("=")
        TUNING[key] = int(val)
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU (one replica of the sampler per GPU needs no communication); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    if a.copy_calibration:
        import torch
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if a.paper_table:
        paper_table(a.workload if a.workload != "cfg4_large_shared" else "cfg2_medium_fcr", a.steps, a.warmup)
        return

    if a.degree_split_table:
        degree_split_table(a.workload, a.steps, a.warmup)
        return

    from paper_2406_17918_amd import synth, gss
    lib_version = gss.load_library().gss_version().decode()
    w = synth.WORKLOADS[a.workload]
    if a.batch > 0:
        import copy
        w = copy.copy(w)
        w.batch = a.batch
    graphs = {}

    def graph_of(name):       # cfg3 and cfg4 run on the same graph: generated once
        key = "large" if name in ("cfg3_large_otf", "cfg4_large_shared") else name
        if key not in graphs:
            graphs[key] = synth.WORKLOADS[name].make_graph()
        return graphs[key]

    graph = graph_of(w.name)
    if a.gather:
        gather_bench(w, graph, min(a.steps, 100), min(a.warmup, 10), a.feature_dim)
        return
    cpu_s = 0.0 if a.no_cpu_baseline else a.cpu_seconds
    head = measure_workload(w, graph, a.steps, a.warmup, cpu_s, lib_version)
    out = {
        "metric": "sampled edges/sec per minibatch step (3-hop) + achieved HBM GB/s % of peak",
        "value": head.pop("value"), "unit": head.pop("unit"), "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": head.pop("ms_per_step"), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int32", "data": "synthetic", "library": lib_version,
    }
    if TUNING:
        out["tuning"] = dict(TUNING)
    out.update(head)
    if not a.only and a.batch == 0:
        key_of = lambda n: "large" if n in ("cfg3_large_otf", "cfg4_large_shared") else n
        names = [n for n in synth.WORKLOADS if n != w.name]
        others = {}
        for i, name in enumerate(names):
            for key in [k for k in graphs if k not in {key_of(n) for n in names[i:]}]:
                del graphs[key]       # host memory: keep only the graphs still to be measured
            others[name] = measure_workload(synth.WORKLOADS[name], graph_of(name), a.steps, a.warmup, cpu_s / 3.0, lib_version)
        out["other_workloads"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
