"""Helpers for the GPU-vs-oracle parity tests: run both samplers on the same seeded inputs and compare
every output bit for bit."""
import numpy as np

from oracle import gsso
from paper_2406_17918_amd import synth


# Layout choices (fields of gss_tuning) applied to every GPU sampler the helpers create: results never depend on them,
# which is what the tests that set them check.  Set through the `tuning` fixture of conftest.py.
_tuning = {}


def set_tuning(**fields):
    _tuning.clear()
    _tuning.update(fields)


def oracle_sampler(graph, w_or_kw):
    kw = w_or_kw if isinstance(w_or_kw, dict) else dict(
        k=w_or_kw.k, mode=w_or_kw.mode, num_layers=len(w_or_kw.fanouts), refresh_fraction=w_or_kw.refresh_fraction,
        refresh_period=w_or_kw.refresh_period, rng_seed=w_or_kw.rng_seed)
    rels = [gsso.Relation(r.src_type, r.dst_type, r.indptr, r.indices) for r in graph.relations]
    return gsso.Sampler(graph.num_nodes, rels, **kw)


def gpu_sampler(graph, w_or_kw, dev_rels=None):
    from paper_2406_17918_amd import gss
    kw = w_or_kw if isinstance(w_or_kw, dict) else dict(
        k=w_or_kw.k, mode=w_or_kw.mode, num_layers=len(w_or_kw.fanouts), refresh_fraction=w_or_kw.refresh_fraction,
        refresh_period=w_or_kw.refresh_period, rng_seed=w_or_kw.rng_seed)
    if dev_rels is None:
        dev_rels = gss.upload_graph(graph)
    return gss.Sampler(graph.num_nodes, dev_rels, tuning=dict(_tuning), **kw)


def assert_blocks_equal(gpu_blocks, ora_blocks, ctx=""):
    assert len(gpu_blocks) == len(ora_blocks)
    for l, (a, b) in enumerate(zip(gpu_blocks, ora_blocks)):
        assert a.num_dst == b.num_dst, (ctx, l, "num_dst", a.num_dst, b.num_dst)
        assert a.num_src == b.num_src, (ctx, l, "num_src", a.num_src, b.num_src)
        assert a.num_edges == b.num_edges, (ctx, l, "num_edges", a.num_edges, b.num_edges)
        for t in range(len(b.num_src)):
            assert np.array_equal(a.src_nodes[t].cpu().numpy(), b.src_nodes[t]), (ctx, l, "src_nodes", t)
        for r in range(len(b.num_edges)):
            assert np.array_equal(a.src_local[r].cpu().numpy(), b.src_local[r]), (ctx, l, "src_local", r)
            assert np.array_equal(a.dst_local[r].cpu().numpy(), b.dst_local[r]), (ctx, l, "dst_local", r)


def assert_caches_equal(gs, os_, num_relations, full=True, ctx=""):
    assert gs.num_tables == os_.num_tables
    for t in range(os_.num_tables):
        for r in range(num_relations):
            assert gs.checksum(t, r) == os_.checksum(t, r), (ctx, "checksum", t, r)
            if full:
                assert np.array_equal(gs.cache(t, r).cpu().numpy(), os_.cache(t, r)), (ctx, "cache", t, r)


def run_parity(graph, kw, fanouts, batch, steps, workload_seed=9, seed_type=0, full_cache_every=1, dev_rels=None,
               seeds_fn=None):
    import torch
    gs = gpu_sampler(graph, kw, dev_rels)
    os_ = oracle_sampler(graph, kw)
    R = len(graph.relations)
    assert_caches_equal(gs, os_, R, ctx="after create")
    total = 0
    for i, step in enumerate(steps):
        seeds = (seeds_fn(step) if seeds_fn else
                 synth.seeds_for_step(graph.num_nodes[seed_type], batch, workload_seed, step))
        gb = gs.step(torch.from_numpy(seeds).cuda(), fanouts, step, seed_type)
        ob = os_.step(seeds, fanouts, step, seed_type)
        assert_blocks_equal(gb, ob, ctx=f"step {step}")
        full = full_cache_every and (i % full_cache_every == 0 or i == len(steps) - 1)
        assert_caches_equal(gs, os_, R, full=bool(full), ctx=f"step {step}")
        total += sum(sum(b.num_edges) for b in ob)
    gs.close()
    os_.close()
    return total


def run_parity_pipelined(graph, kw, fanouts, batch, steps, workload_seed=9, seed_type=0, dev_rels=None):
    """As many steps in flight as the sampler holds (later steps enqueued before the oldest is collected): every step's blocks equal the oracle's,
    and the cache tables match after the last step."""
    import torch
    gs = gpu_sampler(graph, kw, dev_rels)
    os_ = oracle_sampler(graph, kw)
    steps = list(steps)
    seeds = [synth.seeds_for_step(graph.num_nodes[seed_type], batch, workload_seed, st) for st in steps]
    dev = [torch.from_numpy(x).cuda() for x in seeds]
    from paper_2406_17918_amd import gss
    total = 0
    done = 0
    for i in range(len(steps)):
        gs.step_async(dev[i], fanouts, steps[i], seed_type)
        if i + 1 - done == gs.pipeline_depth or i == len(steps) - 1:
            last = done + 1 if i < len(steps) - 1 else len(steps)
            while done < last:
                gb = gs.step_wait()
                ob = os_.step(seeds[done], fanouts, steps[done], seed_type)
                assert_blocks_equal(gb, ob, ctx=f"pipelined step {steps[done]}")
                total += sum(sum(b.num_edges) for b in ob)
                done += 1
    assert_caches_equal(gs, os_, len(graph.relations), full=True, ctx="after the pipelined run")
    gs.close()
    os_.close()
    return total
