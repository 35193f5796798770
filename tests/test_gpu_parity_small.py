"""GPU parity (bit-exact vs the oracle) on small graphs: every mode, ragged sizes, edge cases, typed graphs."""
import numpy as np
import pytest

from oracle import gsso
from paper_2406_17918_amd import synth
from parity_util import run_parity, run_parity_pipelined, gpu_sampler, oracle_sampler, assert_blocks_equal

pytestmark = pytest.mark.gpu

FCR, OTF, SHARED = gsso.MODE_FCR, gsso.MODE_OTF, gsso.MODE_SHARED_OTF
FBL, SHARED_FCR, OTF_FETCH, OTF_LAYER = gsso.MODE_FBL, gsso.MODE_SHARED_FCR, gsso.MODE_OTF_FETCH, gsso.MODE_OTF_LAYER


def graph_small(indptr64=False, n=3000, m=30000, seed=21):
    return synth.chunglu_graph(n, m, 2.2, seed, indptr64=indptr64)


CASES = [
    # k, mode, fraction, period, fanouts, batch
    (10, OTF, 0.25, 1, [5, 5], 128),
    (20, FCR, 0.0, 3, [15, 10, 5], 200),
    (20, OTF, 0.20, 1, [15, 10, 5], 257),
    (30, SHARED, 0.10, 1, [15, 10, 5], 300),
    (25, OTF, 0.20, 2, [25, 20], 64),
    (32, OTF, 0.5, 1, [32, 7], 33),
    (16, OTF, 1.0, 1, [4, 16, 3], 90),
    (1, OTF, 1.0, 1, [1, 1], 77),
    (17, SHARED, 0.3, 1, [8, 5, 4], 150),
    (8, FCR, 0.0, 1, [3, 8, 2, 5], 40),
    (12, SHARED, 0.25, 2, [3, 3], 500),
    (20, FBL, 0.0, 1, [15, 10, 5], 257),
    (32, FBL, 0.0, 1, [32, 20], 100),
    (5, FBL, 0.0, 1, [1, 5, 2], 333),
    (30, SHARED_FCR, 0.0, 2, [15, 10, 5], 300),
    (9, SHARED_FCR, 0.0, 1, [4, 5], 150),
    (20, OTF_FETCH, 0.4, 1, [15, 10, 5], 257),
    (10, OTF_FETCH, 1.0, 1, [5, 5], 128),
    (32, OTF_FETCH, 0.5, 1, [32, 7], 60),
    (16, OTF_FETCH, 0.0, 1, [4, 16, 3], 90),
    (8, OTF_FETCH, 0.3, 1, [8, 8], 200),
    (20, OTF_LAYER, 0.25, 3, [15, 10, 5], 200),
    (12, OTF_LAYER, 0.5, 1, [4, 4], 150),
    (32, OTF_LAYER, 1.0, 2, [32, 7], 50),
]


@pytest.mark.parametrize("k,mode,frac,period,fanouts,batch", CASES)
@pytest.mark.parametrize("indptr64", [False, True])
def test_parity_small_graph(k, mode, frac, period, fanouts, batch, indptr64):
    g = graph_small(indptr64)
    kw = dict(k=k, mode=mode, num_layers=len(fanouts), refresh_fraction=frac, refresh_period=period, rng_seed=1234567890123)
    total = run_parity(g, kw, fanouts, batch, steps=[0, 1, 2, 3, 5, 6, 9])
    assert total > 0


def test_parity_fewer_layers_than_tables_and_varying_batches():
    import torch
    g = graph_small()
    kw = dict(k=12, mode=OTF, num_layers=3, refresh_fraction=0.25, refresh_period=1, rng_seed=5)
    gs, os_ = gpu_sampler(g, kw), oracle_sampler(g, kw)
    plan = [(0, 10, [4, 4, 4]), (1, 0, [4, 4]), (2, 1, [12]), (3, 3000, [2, 3]), (7, 999, [5, 1, 5]), (7, 5, [3])]
    for step, batch, fan in plan:
        seeds = synth.seeds_for_step(g.num_nodes[0], batch, 3, step)
        gb = gs.step(torch.from_numpy(seeds).cuda(), fan, step)
        ob = os_.step(seeds, fan, step)
        assert_blocks_equal(gb, ob, ctx=f"step {step}")
        for t in range(3):
            assert np.array_equal(gs.cache(t).cpu().numpy(), os_.cache(t))


def test_parity_hub_and_isolated_nodes():
    # a star (one node of degree n-1), a clique of 40 (k < deg < 2k for k = 24) and isolated nodes
    n = 600
    rows, cols = [], []
    for v in range(1, 500):
        rows += [0, v]; cols += [v, 0]
    for a in range(500, 540):
        for b in range(500, 540):
            if a != b:
                rows.append(a); cols.append(b)
    order = np.lexsort((cols, rows))
    rows, cols = np.array(rows)[order], np.array(cols)[order]
    indptr = np.zeros(n + 1, np.int32)
    np.add.at(indptr, rows + 1, 1)
    g = synth.Graph([n], [synth.Relation(0, 0, np.cumsum(indptr).astype(np.int32), cols.astype(np.int32))])
    for mode, frac in [(OTF, 0.25), (SHARED, 0.25), (FCR, 0.0), (FBL, 0.0), (SHARED_FCR, 0.0), (OTF_FETCH, 0.5), (OTF_LAYER, 0.25)]:
        kw = dict(k=24, mode=mode, num_layers=2, refresh_fraction=frac, refresh_period=2, rng_seed=77)
        run_parity(g, kw, [10, 12], 64, steps=range(6),
                   seeds_fn=lambda step: np.concatenate([[0, 599, 510], synth.seeds_for_step(n - 100, 61, 1, step) + 1]).astype(np.int32))


def test_parity_typed_graph():
    g = synth.hetero_graph([1200, 2000, 60, 300], [(1, 2, 2600), (1, 0, 9000), (0, 0, 5000), (0, 3, 8000)], 2.2, seed=8)
    for mode, frac, k, fan in [(OTF, 0.2, 25, [25, 20]), (FCR, 0.0, 10, [4, 6]), (SHARED, 0.2, 12, [6, 5]),
                               (FBL, 0.0, 25, [25, 20]), (SHARED_FCR, 0.0, 12, [6, 5]), (OTF_FETCH, 0.3, 25, [25, 20])]:
        kw = dict(k=k, mode=mode, num_layers=2, refresh_fraction=frac, refresh_period=2, rng_seed=3)
        run_parity(g, kw, fan, 100, steps=range(5))
    # seeds of another type
    kw = dict(k=8, mode=OTF, num_layers=3, refresh_fraction=0.5, refresh_period=1, rng_seed=3)
    run_parity(g, kw, [3, 4, 5], 40, steps=range(3), seed_type=3)


def test_device_detected_errors():
    import torch
    from paper_2406_17918_amd import gss
    g = graph_small()
    kw = dict(k=8, mode=OTF, num_layers=2, refresh_fraction=0.25, refresh_period=1, rng_seed=1)
    rels = gss.upload_graph(g)
    for bad in ([5, 6, 5], [5, g.num_nodes[0]], [-1, 2]):
        s = gpu_sampler(g, kw, rels)
        with pytest.raises(gss.GssError) as e:
            s.step(torch.tensor(bad, dtype=torch.int32, device="cuda"), [3, 3], 0)
        assert e.value.status == gss.GSS_ERR_INVALID_SEED
        with pytest.raises(gss.GssError) as e:      # the handle is only good for destroy now
            s.step(torch.tensor([1], dtype=torch.int32, device="cuda"), [3, 3], 1)
        assert e.value.status == gss.GSS_ERR_DEVICE
        s.close()
    s = gpu_sampler(g, kw, rels)
    ok = torch.tensor([1, 2, 3], dtype=torch.int32, device="cuda")
    for fan, status in [([9, 3], gss.GSS_ERR_INVALID_ARG), ([3, 3, 3], gss.GSS_ERR_INVALID_ARG), ([0, 3], gss.GSS_ERR_INVALID_ARG)]:
        with pytest.raises(gss.GssError) as e:
            s.step(ok, fan, 0)
        assert e.value.status == status
    s.step(ok, [3, 3], 5)
    with pytest.raises(gss.GssError) as e:
        s.step(ok, [3, 3], 4)
    assert e.value.status == gss.GSS_ERR_STEP_ORDER
    s.step(ok, [3, 3], 5)      # host-detected errors leave the sampler usable
    s.close()
    # invalid graphs are rejected by gss_create
    bad_idx = g.relations[0].indices.copy(); bad_idx[7] = g.num_nodes[0]
    bad_ptr = g.relations[0].indptr.copy(); bad_ptr[10] = bad_ptr[11] + 1
    for rel in (synth.Relation(0, 0, g.relations[0].indptr, bad_idx), synth.Relation(0, 0, bad_ptr, g.relations[0].indices)):
        with pytest.raises(gss.GssError) as e:
            gpu_sampler(synth.Graph(g.num_nodes, [rel]), kw)
        assert e.value.status == gss.GSS_ERR_INVALID_GRAPH


@pytest.mark.parametrize("layout", ["hash", "direct"])
def test_parity_both_dedupe_table_layouts(layout, tuning):
    # the library picks the direct (one word per node) layout by itself; gss_tuning.dedupe_layout forces either one
    tuning(dedupe_layout={"direct": 1, "hash": 2}[layout])
    g = graph_small()
    for k, mode, frac, fanouts, batch in [(20, OTF, 0.2, [15, 10, 5], 257), (30, SHARED, 0.1, [15, 10, 5], 300), (20, FCR, 0.0, [7, 7], 64)]:
        kw = dict(k=k, mode=mode, num_layers=len(fanouts), refresh_fraction=frac, refresh_period=2, rng_seed=99)
        assert run_parity(g, kw, fanouts, batch, steps=range(5)) > 0
    gt = synth.hetero_graph([1200, 2000, 60, 300], [(1, 2, 2600), (1, 0, 9000), (0, 0, 5000), (0, 3, 8000)], 2.2, seed=8)
    kw = dict(k=25, mode=OTF, num_layers=2, refresh_fraction=0.2, refresh_period=1, rng_seed=3)
    run_parity(gt, kw, [25, 20], 100, steps=range(4))


def test_async_pipeline_matches_blocking_steps():
    # two steps in flight: enqueue step i+1 before collecting step i; results equal the oracle's
    import torch
    from paper_2406_17918_amd import gss
    g = graph_small()
    kw = dict(k=20, mode=OTF, num_layers=3, refresh_fraction=0.2, refresh_period=1, rng_seed=4)
    gs, os_ = gpu_sampler(g, kw), oracle_sampler(g, kw)
    fan = [15, 10, 5]
    n_steps = 9
    batches = [40 + 37 * i for i in range(n_steps)]        # varying sizes: buffers grow while a step is in flight
    seeds = [synth.seeds_for_step(g.num_nodes[0], batches[i], 6, i) for i in range(n_steps)]
    dev = [torch.from_numpy(x).cuda() for x in seeds]
    ref = [os_.step(seeds[i], fan, i) for i in range(n_steps)]
    gs.step_async(dev[0], fan, 0)
    for i in range(1, n_steps):
        gs.step_async(dev[i], fan, i)
        assert_blocks_equal(gs.step_wait(), ref[i - 1], ctx=f"step {i - 1}")
    assert_blocks_equal(gs.step_wait(), ref[n_steps - 1], ctx="last")
    with pytest.raises(gss.GssError) as e:                 # nothing in flight
        gs.step_wait()
    assert e.value.status == gss.GSS_ERR_INVALID_ARG
    F = gs.pipeline_depth
    assert 2 <= F <= gss.GSS_MAX_IN_FLIGHT
    for j in range(F):
        gs.step_async(dev[j % n_steps], fan, n_steps + j)
    with pytest.raises(gss.GssError) as e:                 # one more step in flight is refused
        gs.step_async(dev[0], fan, n_steps + F)
    assert e.value.status == gss.GSS_ERR_INVALID_ARG
    with pytest.raises(gss.GssError):                      # the blocking call refuses to jump the queue
        gs.step(dev[0], fan, n_steps + F)
    for j in range(F):
        assert_blocks_equal(gs.step_wait(), os_.step(seeds[j % n_steps], fan, n_steps + j), ctx=f"{F} in flight, {j}")
    for t in range(3):
        assert np.array_equal(gs.cache(t).cpu().numpy(), os_.cache(t))
    gs.close()


def test_parity_with_separate_scan_launch(tuning):
    # hops with more than 4096 tiles hand the tile scan to a one-workgroup kernel; force that path on a small graph
    tuning(scan_phase=1)
    g = graph_small()
    kw = dict(k=20, mode=OTF, num_layers=3, refresh_fraction=0.2, refresh_period=1, rng_seed=5)
    assert run_parity(g, kw, [15, 10, 5], 257, steps=range(4)) > 0
    gt = synth.hetero_graph([1200, 2000, 60, 300], [(1, 2, 2600), (1, 0, 9000), (0, 0, 5000), (0, 3, 8000)], 2.2, seed=8)
    kw = dict(k=25, mode=OTF, num_layers=2, refresh_fraction=0.2, refresh_period=1, rng_seed=3)
    run_parity(gt, kw, [25, 20], 100, steps=range(3))


@pytest.mark.parametrize("insert", ["", "split"])
@pytest.mark.parametrize("k,mode,frac,period,fanouts,batch", [c for c in CASES if c[0] in (10, 20, 30, 12, 8, 9, 5, 32)])
def test_pipelined_steps_small_graph(k, mode, frac, period, fanouts, batch, insert, tuning):
    # a full pipeline of steps in flight: every launch carries one phase of each of them ("split": every hop's dedupe
    # table inserts run as a phase of their own, which by default only large hops do)
    tuning(insert_phase=1 if insert == "split" else 0)
    g = graph_small()
    kw = dict(k=k, mode=mode, num_layers=len(fanouts), refresh_fraction=frac, refresh_period=period, rng_seed=31337)
    assert run_parity_pipelined(g, kw, fanouts, batch, steps=range(40)) > 0


@pytest.mark.parametrize("scan,insert", [("emit", "fused"), ("kernel", "split"), ("emit", "split")])
@pytest.mark.parametrize("mode,frac", [(OTF, 0.25), (FCR, 0.0), (FBL, 0.0), (SHARED, 0.2), (SHARED_FCR, 0.0), (OTF_FETCH, 0.5)])
def test_pipelined_steps_with_varying_layer_counts_and_irregular_waits(mode, frac, scan, insert, tuning):
    # steps in flight use 1, 2 or 3 of the 3 layers, skip step numbers (FCR epochs change at irregular points), and
    # the caller collects at irregular points: every step's blocks equal the oracle's, and so do the tables
    import torch
    # "kernel": hops get a separate scan phase; "split": and a separate insert phase (up to 5 phases per hop)
    tuning(scan_phase=1 if scan == "kernel" else 0, insert_phase={"split": 1, "fused": 2}[insert])
    g = graph_small()
    kw = dict(k=12, mode=mode, num_layers=3, refresh_fraction=frac, refresh_period=3, rng_seed=8)
    gs, os_ = gpu_sampler(g, kw), oracle_sampler(g, kw)
    fans = [[4, 4, 4], [4, 4], [3, 3, 3], [12], [2, 2, 2], [2, 2, 2], [4, 3], [4, 3], [4, 4, 4], [1, 1, 1], [5], [4, 4, 3]]
    steps = [0, 1, 2, 4, 5, 6, 7, 11, 12, 13, 20, 21]
    waits_after = [0, 0, 2, 0, 0, 0, 3, 0, 1, 0, 0, 0]     # collect this many after enqueueing step i
    seeds = [synth.seeds_for_step(g.num_nodes[0], 50 + 31 * i, 5, st) for i, st in enumerate(steps)]
    dev = [torch.from_numpy(x).cuda() for x in seeds]
    done = 0
    def collect():
        nonlocal done
        gb = gs.step_wait()
        ob = os_.step(seeds[done], fans[done], steps[done])
        assert_blocks_equal(gb, ob, ctx=f"step {steps[done]}")
        done += 1
    for i in range(len(steps)):
        while i - done >= gs.pipeline_depth:
            collect()
        gs.step_async(dev[i], fans[i], steps[i])
        for _ in range(waits_after[i]):
            collect()
    while done < len(steps):
        collect()
    if mode != FBL:
        for t in range(os_.num_tables):
            assert np.array_equal(gs.cache(t).cpu().numpy(), os_.cache(t))
    gs.close(); os_.close()


def test_cache_read_with_steps_in_flight_finishes_their_hops_first():
    import torch
    g = graph_small()
    kw = dict(k=12, mode=OTF, num_layers=3, refresh_fraction=0.5, refresh_period=1, rng_seed=2)
    gs, os_ = gpu_sampler(g, kw), oracle_sampler(g, kw)
    seeds = [synth.seeds_for_step(g.num_nodes[0], 200, 5, st) for st in range(4)]
    dev = [torch.from_numpy(x).cuda() for x in seeds]
    for i in range(4):
        gs.step_async(dev[i], [4, 4, 4], i)
    ref = [os_.step(seeds[i], [4, 4, 4], i) for i in range(4)]
    for t in range(3):                                     # the read-out covers every enqueued step
        assert np.array_equal(gs.cache(t).cpu().numpy(), os_.cache(t))
    for i in range(4):
        assert_blocks_equal(gs.step_wait(), ref[i], ctx=f"step {i}")
    gs.close(); os_.close()


# Dense/sparse degree split: nodes with deg <= theta keep no cache row and are sampled by the FBL draw.
SPLIT_CASES = [
    # k, mode, fraction, period, fanouts, batch, theta
    (10, OTF, 0.25, 1, [5, 5], 128, 10),          # theta = k: every cached row is a full row
    (20, FCR, 0.0, 3, [15, 10, 5], 200, 20),
    (20, OTF, 0.20, 1, [15, 10, 5], 257, 7),      # theta < k: short cached rows exist
    (30, SHARED, 0.10, 1, [15, 10, 5], 300, 30),
    (17, SHARED, 0.3, 1, [8, 5, 4], 150, 40),     # theta > 2k
    (9, SHARED_FCR, 0.0, 2, [4, 5], 150, 3),
    (12, OTF, 0.5, 1, [12, 12], 300, 0),          # theta = 0: only isolated nodes lose their (empty) row
    (8, FCR, 0.0, 1, [3, 8, 2, 5], 40, 10**9),    # nothing is cached: every node takes the FBL draw
    (20, FBL, 0.0, 1, [15, 10], 100, 5),          # FBL ignores the threshold
    (16, OTF_FETCH, 0.5, 1, [8, 6], 200, 16),
    (16, OTF_LAYER, 0.5, 2, [8, 6], 200, 20),
]


@pytest.mark.parametrize("k,mode,frac,period,fanouts,batch,theta", SPLIT_CASES)
@pytest.mark.parametrize("indptr64", [False, True])
def test_parity_degree_split(k, mode, frac, period, fanouts, batch, theta, indptr64):
    g = graph_small(indptr64)
    kw = dict(k=k, mode=mode, num_layers=len(fanouts), refresh_fraction=frac, refresh_period=period, rng_seed=99,
              degree_threshold=theta)
    total = run_parity(g, kw, fanouts, batch, steps=[0, 1, 2, 3, 5, 6])
    assert total > 0
    if not indptr64:
        total2 = run_parity_pipelined(g, kw, fanouts, batch, steps=range(8))
        assert total2 > 0


def test_degree_split_shrinks_the_tables():
    g = graph_small()
    deg = np.diff(g.relations[0].indptr)
    n = len(deg)
    for theta, mode, tables in [(-1, OTF, 2), (16, OTF, 2), (16, SHARED, 1), (10**6, FCR, 2)]:
        kw = dict(k=16, mode=mode, num_layers=2, refresh_fraction=0.25, refresh_period=1, rng_seed=1, degree_threshold=theta)
        gs = gpu_sampler(g, kw)
        rows = n if theta < 0 else int((deg > theta).sum())
        want = tables * rows * 16 * 4 + (0 if theta < 0 else 4 * n) + (8 * rows if mode == SHARED else 0)
        assert gs.cache_bytes() == want, (theta, mode)
        gs.close()


def test_parity_degree_split_typed_graph_and_hubs():
    # typed graph: the row maps and the compacted tables are per relation
    g = synth.hetero_graph([1200, 2000, 60, 300], [(1, 2, 2600), (1, 0, 9000), (0, 0, 5000), (0, 3, 8000)], 2.2, seed=8)
    for mode, frac, k, fan, theta in [(OTF, 0.2, 25, [25, 20], 25), (FCR, 0.0, 10, [4, 6], 4), (SHARED, 0.2, 12, [6, 5], 12),
                                      (SHARED_FCR, 0.0, 12, [6, 5], 30)]:
        kw = dict(k=k, mode=mode, num_layers=2, refresh_fraction=frac, refresh_period=2, rng_seed=3, degree_threshold=theta)
        run_parity(g, kw, fan, 100, steps=range(5))
    # a star, a clique of 40 and isolated nodes: theta between the clique degree and the hub degree
    n = 600
    rows, cols = [], []
    for v in range(1, 500):
        rows += [0, v]; cols += [v, 0]
    for a in range(500, 540):
        for b in range(500, 540):
            if a != b:
                rows.append(a); cols.append(b)
    order = np.lexsort((cols, rows))
    rows, cols = np.array(rows)[order], np.array(cols)[order]
    indptr = np.zeros(n + 1, np.int32)
    np.add.at(indptr, rows + 1, 1)
    g = synth.Graph([n], [synth.Relation(0, 0, np.cumsum(indptr).astype(np.int32), cols.astype(np.int32))])
    for theta in (1, 39, 100):
        for mode, frac in [(OTF, 0.25), (SHARED, 0.25), (FCR, 0.0), (SHARED_FCR, 0.0)]:
            kw = dict(k=24, mode=mode, num_layers=2, refresh_fraction=frac, refresh_period=2, rng_seed=77, degree_threshold=theta)
            total = run_parity(g, kw, [12, 12], 300, steps=range(5))
            assert total > 0


@pytest.mark.parametrize("per_tick", ["1", "2"])
@pytest.mark.parametrize("sets", ["1", "2", "3", "5"])
@pytest.mark.parametrize("mode,period", [(FCR, 1), (FCR, 2), (FCR, 5), (SHARED_FCR, 3), (FCR, 11), (OTF_LAYER, 1), (OTF_LAYER, 4)])
def test_fcr_refresh_with_steps_in_flight(mode, period, sets, per_tick, tuning):
    # FCR keeps 1-3 sets of tables: the next epoch's rows are computed ahead of time into a set no step in flight
    # reads (one set: in place, after the steps in flight have issued all their phases).  Step numbers jump over
    # epochs now and then, so the rows computed ahead are sometimes for the wrong epoch.
    import torch
    tuning(table_sets=int(sets), steps_per_tick=int(per_tick))   # 2 per tick: a launch starts two steps (up to 24 slices, the compact form)
    g = graph_small()
    kw = dict(k=12, mode=mode, num_layers=3, refresh_fraction=0.25 if mode == OTF_LAYER else 0.0, refresh_period=period, rng_seed=17)
    steps = [t for t in range(60) if t not in (7, 8, 9, 10, 11, 12, 13, 29, 41, 42)]
    assert run_parity_pipelined(g, kw, [4, 4, 4], 150, steps=steps) > 0


def test_parity_many_relations_and_node_types():
    # 5 node types and 10 relations: the widest argument layout (per-relation constants in device memory, four
    # slices per launch, so a tick of a 3-hop step takes three launches)
    g = synth.hetero_graph([900, 700, 500, 300, 200], [(0, 1, 4000), (1, 2, 3000), (2, 3, 2500), (3, 4, 1500), (4, 0, 2000)],
                           2.2, seed=12)
    assert len(g.relations) == 10
    for mode, frac, k, fan in [(OTF, 0.25, 12, [4, 5, 3]), (FCR, 0.0, 8, [3, 3, 3]), (SHARED, 0.2, 12, [4, 4, 4]), (FBL, 0.0, 6, [6, 2])]:
        kw = dict(k=k, mode=mode, num_layers=len(fan), refresh_fraction=frac, refresh_period=3, rng_seed=5)
        assert run_parity(g, kw, fan, 80, steps=range(4)) > 0
        assert run_parity_pipelined(g, kw, fan, 80, steps=range(20)) > 0


@pytest.mark.parametrize("mode,frac,period", [(FBL, 0.0, 1), (OTF_FETCH, 0.5, 1), (FCR, 0.0, 4), (SHARED_FCR, 0.0, 7),
                                                (OTF_LAYER, 0.25, 3), (OTF, 0.25, 1), (SHARED, 0.2, 2)])
def test_long_randomized_pipeline_with_growing_batches(mode, frac, period):
    # 150 steps with batch sizes that keep growing now and then (the slots' buffers - and the device table of their
    # pointers that the compact launches read - are replaced while other steps are in flight), 1 to 3 layers per
    # step, skipped step numbers and irregular waits: every step's blocks equal the oracle's, and so do the tables
    import torch
    rng = np.random.default_rng(2024 + int(mode))
    g = graph_small()
    kw = dict(k=12, mode=mode, num_layers=3, refresh_fraction=frac, refresh_period=period, rng_seed=77)
    gs, os_ = gpu_sampler(g, kw), oracle_sampler(g, kw)
    n_steps = 150
    step_no, steps, fans, batches = 0, [], [], []
    cap = 20
    for i in range(n_steps):
        step_no += 1 if rng.random() < 0.9 else int(rng.integers(2, 6))
        steps.append(step_no)
        L = int(rng.integers(1, 4))
        fans.append([int(rng.integers(1, 5)) for _ in range(L)] if mode in (SHARED, SHARED_FCR) else
                    [int(rng.integers(1, 13)) for _ in range(L)])
        if rng.random() < 0.08:
            cap = int(cap * 1.8) + 5                      # from here on, larger batches: buffers grow
        batches.append(int(rng.integers(1, cap + 1)))
    seeds = [synth.seeds_for_step(g.num_nodes[0], min(b, g.num_nodes[0]), 5, st) for b, st in zip(batches, steps)]
    dev = [torch.from_numpy(x).cuda() for x in seeds]
    done = 0
    def collect():
        nonlocal done
        gb = gs.step_wait()
        ob = os_.step(seeds[done], fans[done], steps[done])
        assert_blocks_equal(gb, ob, ctx=f"step {steps[done]} (#{done})")
        done += 1
    for i in range(n_steps):
        while i - done >= gs.pipeline_depth:
            collect()
        gs.step_async(dev[i], fans[i], steps[i])
        for _ in range(int(rng.integers(0, 3)) if rng.random() < 0.3 else 0):
            if done <= i:
                collect()
    while done < n_steps:
        collect()
    if mode != FBL:
        for t in range(os_.num_tables):
            assert np.array_equal(gs.cache(t).cpu().numpy(), os_.cache(t))
    gs.close(); os_.close()


@pytest.mark.parametrize("mode", [FCR, FBL, OTF])
def test_blocks_of_a_collected_step_stay_valid_while_later_steps_grow_the_buffers(mode):
    # The blocks of a step stay valid until pipeline_depth - 1 further steps have been enqueued - also when those steps
    # are larger and make the sampler allocate larger buffers: the memory behind the first step's blocks is neither
    # released nor written again.
    import torch
    g = graph_small()
    fan = [6, 4]
    kw = dict(k=12, mode=mode, num_layers=2, refresh_fraction=0.25, refresh_period=2, rng_seed=3)
    gs, os_ = gpu_sampler(g, kw), oracle_sampler(g, kw)
    seeds0 = synth.seeds_for_step(g.num_nodes[0], 16, 5, 0)
    dev0 = torch.from_numpy(seeds0).cuda()
    gs.step_async(dev0, fan, 0)
    raw = gs.step_wait_raw()
    ptrs = []
    for l in range(raw.num_layers):
        ptrs += [raw.nodes[l].src_nodes, raw.edges[l].src_local, raw.edges[l].dst_local]
    ptrs = [int(p) for p in ptrs if p]
    assert ptrs
    first = gs._wrap(raw)
    expect = os_.step(seeds0, fan, 0)
    keep, inflight = [], 0
    for j in range(1, gs.pipeline_depth):
        seeds = synth.seeds_for_step(g.num_nodes[0], 16 + 60 * j, 5, j)
        keep.append(torch.from_numpy(seeds).cuda())
        gs.step_async(keep[-1], fan, j)
        assert all(p in gs._allocator.live for p in ptrs), f"buffers of step 0 released when step {j} was enqueued"
        inflight += 1
        if j % 3 == 0:                      # collect now and then; the rest stays in flight
            while inflight:
                gs.step_wait()
                inflight -= 1
    while inflight:
        gs.step_wait()
        inflight -= 1
    assert_blocks_equal(first, expect, ctx="step 0, read after the later steps")
    gs.close(); os_.close()


@pytest.mark.parametrize("build", ["dense", "plain"])
@pytest.mark.parametrize("k,mode,frac,period,fanouts,batch", [c for c in CASES if c[0] in (20, 30, 32, 9, 8)])
def test_both_register_budgets_of_the_step_kernel(k, mode, frac, period, fanouts, batch, build, tuning):
    # the step kernel is built twice (seven or eight workgroups per CU); launches choose by their size, which these
    # small cases never reach: force either build for every launch
    tuning(tick_build={"dense": 1, "plain": 2}[build])
    g = graph_small()
    kw = dict(k=k, mode=mode, num_layers=len(fanouts), refresh_fraction=frac, refresh_period=period, rng_seed=99)
    assert run_parity(g, kw, fanouts, batch, steps=[0, 1, 2, 5]) > 0
    assert run_parity_pipelined(g, kw, fanouts, batch, steps=range(30)) > 0


@pytest.mark.parametrize("build", ["dense", "plain"])
def test_both_register_budgets_typed_graph(build, tuning):
    tuning(tick_build={"dense": 1, "plain": 2}[build])
    gt = synth.hetero_graph([1200, 2000, 60, 300], [(1, 2, 2600), (1, 0, 9000), (0, 0, 5000), (0, 3, 8000)], 2.2, seed=8)
    kw = dict(k=25, mode=OTF, num_layers=2, refresh_fraction=0.2, refresh_period=1, rng_seed=3)
    assert run_parity_pipelined(gt, kw, [25, 20], 100, steps=range(12)) > 0


SHARED_CASES = [
    # k, fraction, period, fanouts, batch, theta
    (30, 0.10, 1, [15, 10, 5], 300, -1),
    (17, 0.3, 1, [8, 5, 4], 150, -1),
    (12, 0.25, 2, [3, 3], 500, -1),
    (32, 1.0, 1, [8, 8, 8, 8], 40, -1),          # four hops, every slot redrawn at each visit
    (24, 0.25, 1, [12, 12], 300, 30),           # degree split: nodes without a row draw from the adjacency per hop
    (9, 0.5, 1, [9], 700, -1),                  # one hop
    (20, 0.2, 1, [2, 3, 4, 5, 6], 30, -1),      # five hops: more than a visit-once step holds, runs hop by hop
]


@pytest.mark.parametrize("visit_once", [1, 2])
@pytest.mark.parametrize("k,frac,period,fanouts,batch,theta", SHARED_CASES)
def test_shared_table_steps_both_ways(k, frac, period, fanouts, batch, theta, visit_once, tuning):
    # the shared table with a refresh per visit runs its steps as visit-once steps (each node visited by the first hop
    # that reaches it, which draws all its remaining hops' picks) or hop by hop: the same blocks and tables either way
    tuning(visit_once=visit_once)
    g = graph_small()
    kw = dict(k=k, mode=SHARED, num_layers=len(fanouts), refresh_fraction=frac, refresh_period=period, rng_seed=4242,
              degree_threshold=theta)
    assert run_parity(g, kw, fanouts, batch, steps=[0, 1, 2, 3, 5, 8]) > 0
    assert run_parity_pipelined(g, kw, fanouts, batch, steps=range(25)) > 0


@pytest.mark.parametrize("k,frac,period,fanouts,batch,theta", SHARED_CASES)
def test_visit_once_steps_with_insert_phases(k, frac, period, fanouts, batch, theta, tuning):
    # the place phases only put the picks into frontier order; insert phases of their own enter them into the dedupe
    # table (gss_tuning.insert_phase = 1; the library never chooses it by itself for these steps)
    tuning(visit_once=1, insert_phase=1)
    g = graph_small()
    kw = dict(k=k, mode=SHARED, num_layers=len(fanouts), refresh_fraction=frac, refresh_period=period, rng_seed=4243,
              degree_threshold=theta)
    assert run_parity(g, kw, fanouts, batch, steps=[0, 1, 2, 3, 5, 8]) > 0
    assert run_parity_pipelined(g, kw, fanouts, batch, steps=range(25)) > 0


def test_visit_once_steps_mixed_with_hop_by_hop_steps(tuning):
    # steps of up to four hops run visit-once, a five-hop step between them hop by hop; batches of very different
    # sizes (the holding area grows), an empty batch, repeated and out-of-range seeds
    import torch
    from paper_2406_17918_amd import gss
    g = graph_small()
    kw = dict(k=20, mode=SHARED, num_layers=5, refresh_fraction=0.2, refresh_period=1, rng_seed=9)
    gs, os_ = gpu_sampler(g, kw), oracle_sampler(g, kw)
    plan = [(0, 60, [5, 5, 5]), (1, 0, [5, 5]), (2, 7, [2, 3, 4, 5, 6]), (3, 900, [4, 4, 4, 4]), (4, 3, [20]),
            (6, 2500, [6, 7]), (7, 33, [1, 2, 3, 4, 5]), (8, 64, [5, 5, 5])]
    seeds = [synth.seeds_for_step(g.num_nodes[0], b, 3, st) for st, b, _ in plan]
    dev = [torch.from_numpy(x).cuda() for x in seeds]
    for i, (st, b, fan) in enumerate(plan[:4]):
        assert_blocks_equal(gs.step(dev[i], fan, st), os_.step(seeds[i], fan, st), ctx=f"step {st}")
    for i, (st, b, fan) in enumerate(plan[4:], 4):
        gs.step_async(dev[i], fan, st)
    for i, (st, b, fan) in enumerate(plan[4:], 4):
        assert_blocks_equal(gs.step_wait(), os_.step(seeds[i], fan, st), ctx=f"pipelined step {st}")
    assert np.array_equal(gs.cache(0).cpu().numpy(), os_.cache(0))
    gs.close(); os_.close()
    for bad in ([5, 6, 5], [5, g.num_nodes[0]], [-1, 2]):
        s = gpu_sampler(g, kw)
        with pytest.raises(gss.GssError) as e:
            s.step(torch.tensor(bad, dtype=torch.int32, device="cuda"), [3, 3, 3], 0)
        assert e.value.status == gss.GSS_ERR_INVALID_SEED
        s.close()


WIDE_CASES = [
    # k, mode, fraction, period, fanouts, batch: rows of 33 .. 64 slots take a whole wavefront per node
    (33, OTF, 0.25, 1, [33, 7], 60),
    (48, FCR, 0.0, 3, [20, 20, 20], 100),
    (60, SHARED, 0.1, 1, [20, 20, 20], 120),
    (64, OTF, 0.2, 1, [64, 1], 40),
    (64, OTF, 1.0, 1, [30, 40], 77),
    (40, SHARED, 0.3, 2, [20, 15], 150),
    (64, FBL, 0.0, 1, [64, 33], 50),
    (40, FBL, 0.0, 1, [20, 20, 20], 90),
    (60, SHARED_FCR, 0.0, 2, [20, 20, 20], 100),
    (48, OTF_FETCH, 0.4, 1, [40, 10], 80),
    (64, OTF_FETCH, 1.0, 1, [33, 64], 30),
    (36, OTF_LAYER, 0.25, 2, [36, 5], 60),
    (64, OTF_LAYER, 0.5, 1, [10, 20], 90),
]


@pytest.mark.parametrize("k,mode,frac,period,fanouts,batch", WIDE_CASES)
@pytest.mark.parametrize("indptr64", [False, True])
def test_parity_rows_wider_than_half_a_wavefront(k, mode, frac, period, fanouts, batch, indptr64):
    # a denser graph, so that all three degree regimes (deg <= k, k < deg < 2k, deg >= 2k) occur at these widths
    g = synth.chunglu_graph(2500, 90000, 2.1, 5, indptr64=indptr64)
    kw = dict(k=k, mode=mode, num_layers=len(fanouts), refresh_fraction=frac, refresh_period=period, rng_seed=987654321)
    assert run_parity(g, kw, fanouts, batch, steps=[0, 1, 2, 3, 5, 6]) > 0
    assert run_parity_pipelined(g, kw, fanouts, batch, steps=range(16)) > 0


def test_wide_rows_degree_split_and_typed_graph():
    g = synth.chunglu_graph(2500, 90000, 2.1, 5)
    for mode, frac in [(OTF, 0.25), (SHARED, 0.25), (FCR, 0.0)]:
        kw = dict(k=40, mode=mode, num_layers=2, refresh_fraction=frac, refresh_period=2, rng_seed=77, degree_threshold=50)
        assert run_parity(g, kw, [20, 20], 200, steps=range(4)) > 0
    gt = synth.hetero_graph([1200, 2000, 60, 300], [(1, 2, 26000), (1, 0, 90000), (0, 0, 50000), (0, 3, 80000)], 2.2, seed=8)
    for mode, frac, k, fan in [(OTF, 0.2, 50, [50, 20]), (SHARED, 0.2, 64, [30, 30]), (FBL, 0.0, 40, [40, 20])]:
        kw = dict(k=k, mode=mode, num_layers=2, refresh_fraction=frac, refresh_period=1, rng_seed=3)
        assert run_parity(gt, kw, fan, 100, steps=range(4)) > 0
        assert run_parity_pipelined(gt, kw, fan, 100, steps=range(10)) > 0


@pytest.mark.parametrize("k,mode,frac,period,fanouts,batch", [c for c in CASES if c[0] in (20, 30, 32, 9, 12)])
def test_parity_with_the_lds_stage_of_the_dedupe(k, mode, frac, period, fanouts, batch, tuning):
    # every hop gets an insert phase, and the insert phases (and the place phases of visit-once steps) first dedupe
    # their tile of 1024 picks in LDS: only the tile's first pick of an id goes on to the global table
    tuning(lds_dedupe=1, insert_phase=1, visit_once=1)
    g = graph_small()
    kw = dict(k=k, mode=mode, num_layers=len(fanouts), refresh_fraction=frac, refresh_period=period, rng_seed=2718)
    assert run_parity(g, kw, fanouts, batch, steps=[0, 1, 2, 5]) > 0
    assert run_parity_pipelined(g, kw, fanouts, batch, steps=range(20)) > 0
    gt = synth.hetero_graph([1200, 2000, 60, 300], [(1, 2, 2600), (1, 0, 9000), (0, 0, 5000), (0, 3, 8000)], 2.2, seed=8)
    if mode in (OTF, FCR) and len(fanouts) == 2:
        assert run_parity_pipelined(gt, kw, fanouts, 100, steps=range(8)) > 0


NARROW_CASES = [c for c in CASES if c[0] <= 20 and c[1] in (FCR, OTF, OTF_LAYER, SHARED_FCR)] + [
    # k, mode, fraction, period, fanouts, batch: rows of 17 .. 20 slots take 21 lanes, up to 16 slots 16 lanes
    (20, OTF, 1.0, 1, [20, 20], 333), (19, OTF, 0.3, 2, [7, 19, 2], 190), (18, FCR, 0.0, 2, [18, 9], 400),
    (17, OTF_LAYER, 0.4, 2, [5, 17], 260), (16, FCR, 0.0, 1, [16, 16], 130), (13, OTF, 0.25, 1, [13, 2, 6], 210),
    (9, OTF, 0.5, 1, [9, 9, 9], 64), (3, OTF, 0.4, 1, [3, 2], 900), (2, SHARED_FCR, 0.0, 3, [1, 1], 500),
    (20, SHARED_FCR, 0.0, 2, [10, 6, 4], 150),
]


@pytest.mark.parametrize("k,mode,frac,period,fanouts,batch", NARROW_CASES)
def test_parity_with_three_or_four_nodes_per_wavefront(k, mode, frac, period, fanouts, batch, tuning):
    # the sample phase with 21 or 16 lanes per frontier node in every launch (the library's own choice only for
    # launches with 16,384 nodes and more): blocking and pipelined, with and without the degree split
    tuning(group_width=1)
    g = graph_small()
    kw = dict(k=k, mode=mode, num_layers=len(fanouts), refresh_fraction=frac, refresh_period=period, rng_seed=60221023)
    assert run_parity(g, kw, fanouts, batch, steps=[0, 1, 2, 3, 5, 6, 9]) > 0
    assert run_parity_pipelined(g, kw, fanouts, batch, steps=range(22)) > 0
    if mode in (OTF, FCR):
        kw["degree_threshold"] = k
        assert run_parity_pipelined(g, kw, fanouts, batch, steps=range(12)) > 0


def test_narrow_groups_on_a_graph_with_hubs_and_at_a_large_batch(tuning):
    # a star, a clique (k < deg < 2k) and isolated nodes with narrow groups; then a batch large enough for the library
    # to choose them by itself (its launches mix both widths while the pipeline fills)
    n = 600
    rows, cols = [], []
    for v in range(1, n - 100):
        rows += [0, v]; cols += [v, 0]
    for a in range(400, 430):
        for b in range(a + 1, 430):
            rows += [a, b]; cols += [b, a]
    order = np.lexsort((cols, rows))
    r_, c_ = np.asarray(rows)[order], np.asarray(cols)[order]
    keep = np.ones(len(r_), bool); keep[1:] = (r_[1:] != r_[:-1]) | (c_[1:] != c_[:-1])
    r_, c_ = r_[keep], c_[keep]
    indptr = np.zeros(n + 1, np.int32); np.add.at(indptr, r_ + 1, 1); indptr = np.cumsum(indptr).astype(np.int32)
    g = synth.Graph([n], [synth.Relation(0, 0, indptr, c_.astype(np.int32))])
    tuning(group_width=1)
    for k, frac in ((20, 0.25), (16, 0.5)):
        kw = dict(k=k, mode=OTF, num_layers=2, refresh_fraction=frac, refresh_period=1, rng_seed=99)
        assert run_parity(g, kw, [k, 5], 300, steps=range(6)) > 0
    tuning()
    big = graph_small(n=60000, m=900000, seed=5)
    kw = dict(k=20, mode=OTF, num_layers=2, refresh_fraction=0.2, refresh_period=1, rng_seed=7)
    assert run_parity_pipelined(big, kw, [10, 5], 20000, steps=range(10)) > 0
