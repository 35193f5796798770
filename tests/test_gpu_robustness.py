"""GPU tests of the host driver's failure handling and rarely taken paths: an allocator that runs out of memory
(at gss_create and while a step's buffers grow), buffers of a few bytes that grow by a few bytes, the wrap-around of
the dedupe-table version counter, and the hashed dedupe layout at the size of the large workload.  Every kernel exits
normally in all of them."""
import numpy as np
import pytest

from oracle import gsso
from paper_2406_17918_amd import synth
from parity_util import run_parity, run_parity_pipelined, oracle_sampler, assert_blocks_equal

pytestmark = pytest.mark.gpu


def failing_allocator(fail_at=None):
    from paper_2406_17918_amd import gss

    class Failing(gss._TorchAllocator):
        """PyTorch's caching allocator, except that call number `fail_at` (1-based) returns NULL."""

        def __init__(self):
            super().__init__("cuda:0")
            self.calls = 0
            self.fail_at = fail_at

        def _alloc(self, ctx, nbytes):
            self.calls += 1
            if self.fail_at is not None and self.calls == self.fail_at:
                return None
            return super()._alloc(ctx, nbytes)

    return Failing()


@pytest.mark.parametrize("mode,frac,theta", [(gsso.MODE_FCR, 0.0, -1), (gsso.MODE_SHARED_OTF, 0.25, 3), (gsso.MODE_OTF, 0.25, -1)])
def test_allocator_returning_null_at_create(mode, frac, theta):
    # every allocation of gss_create fails once: GSS_ERR_OOM, no handle, and everything handed out before is returned
    from paper_2406_17918_amd import gss
    g = synth.chunglu_graph(2000, 15000, 2.2, 5)
    rels = gss.upload_graph(g)
    kw = dict(k=8, mode=mode, num_layers=2, refresh_fraction=frac, refresh_period=2, rng_seed=1, degree_threshold=theta)
    probe = failing_allocator()
    gss.Sampler(g.num_nodes, rels, allocator=probe, **kw).close()
    assert probe.calls >= 5 and not probe.live
    for n in range(1, probe.calls + 1):
        a = failing_allocator(n)
        with pytest.raises(gss.GssError) as e:
            gss.Sampler(g.num_nodes, rels, allocator=a, **kw)
        assert e.value.status == gss.GSS_ERR_OOM, n
        assert not a.live, (n, len(a.live))


@pytest.mark.parametrize("layout", [1, 2])
def test_allocator_returning_null_while_a_step_grows_its_buffers(layout):
    # the n-th allocation of the first step (and of a later, larger one) fails: GSS_ERR_OOM, the sampler is unchanged -
    # the same step then succeeds and equals the oracle's - and destroy returns everything
    import torch
    from paper_2406_17918_amd import gss
    g = synth.chunglu_graph(2000, 15000, 2.2, 5)
    rels = gss.upload_graph(g)
    kw = dict(k=8, mode=gsso.MODE_OTF, num_layers=2, refresh_fraction=0.25, refresh_period=1, rng_seed=1)
    fan = [4, 5]
    probe = failing_allocator()
    s = gss.Sampler(g.num_nodes, rels, allocator=probe, tuning=dict(dedupe_layout=layout, pipeline_depth=3), **kw)
    created = probe.calls
    s.step(torch.from_numpy(synth.seeds_for_step(2000, 50, 1, 0)).cuda(), fan, 0)
    first_step = probe.calls - created
    s.close()
    assert first_step >= 8 and not probe.live
    for n in list(range(1, first_step + 1, 3)) + [first_step]:
        a = failing_allocator()
        s = gss.Sampler(g.num_nodes, rels, allocator=a, tuning=dict(dedupe_layout=layout, pipeline_depth=3), **kw)
        o = oracle_sampler(g, kw)
        seeds = synth.seeds_for_step(2000, 50, 1, 0)
        a.fail_at = a.calls + n
        with pytest.raises(gss.GssError) as e:
            s.step(torch.from_numpy(seeds).cuda(), fan, 0)
        assert e.value.status == gss.GSS_ERR_OOM, n
        a.fail_at = None
        assert_blocks_equal(s.step(torch.from_numpy(seeds).cuda(), fan, 0), o.step(seeds, fan, 0), ctx=f"retry after failure {n}")
        # a larger batch grows the buffers again; fail the first of those allocations
        big = synth.seeds_for_step(2000, 400, 1, 1)
        a.fail_at = a.calls + 1
        with pytest.raises(gss.GssError) as e:
            s.step(torch.from_numpy(big).cuda(), fan, 1)
        assert e.value.status == gss.GSS_ERR_OOM
        a.fail_at = None
        assert_blocks_equal(s.step(torch.from_numpy(big).cuda(), fan, 1), o.step(big, fan, 1), ctx="larger batch")
        for t in range(2):
            assert np.array_equal(s.cache(t).cpu().numpy(), o.cache(t))
        s.close()
        o.close()
        assert not a.live, (n, len(a.live))


@pytest.mark.parametrize("layout", [1, 2])
def test_dedupe_version_counter_wraps(layout, tuning):
    # every hop of every step takes a fresh version of its slot's dedupe table, so that the table is never cleared
    # between hops; started a few versions before the end of the version space, the counter wraps within a few
    # steps: the table is cleared once and the versions start over
    tuning(dedupe_layout=layout, pipeline_depth=2, first_dedupe_version=0xFFFFFFF0 - 7)
    g = synth.chunglu_graph(3000, 30000, 2.2, 21)
    for mode, frac in [(gsso.MODE_OTF, 0.2), (gsso.MODE_FCR, 0.0)]:
        kw = dict(k=20, mode=mode, num_layers=3, refresh_fraction=frac, refresh_period=2, rng_seed=99)
        assert run_parity(g, kw, [15, 10, 5], 200, steps=range(12)) > 0
        assert run_parity_pipelined(g, kw, [15, 10, 5], 200, steps=range(14)) > 0


def test_hashed_dedupe_layout_on_the_large_graph(tuning):
    # the open-addressing layout (the library's choice above 8 GiB of direct words) at the size of the large
    # workload: 2.45 M nodes, frontiers of 20k nodes, 313k picks per step
    tuning(dedupe_layout=2)
    w = synth.WORKLOADS["cfg3_large_otf"]
    g = w.make_graph()
    steps = list(range(8))
    total = run_parity(g, w, w.fanouts, w.batch, steps, workload_seed=w.workload_seed, full_cache_every=10**9)
    total2 = run_parity_pipelined(g, w, w.fanouts, w.batch, steps, workload_seed=w.workload_seed)
    assert total2 == total > 0


@pytest.mark.parametrize("mode,frac", [(gsso.MODE_SHARED_OTF, 0.25), (gsso.MODE_OTF, 0.25), (gsso.MODE_FBL, 0.0)])
def test_buffers_of_a_few_bytes_grow_by_a_few_bytes(mode, frac, tuning):
    # one seed with fanout 2 makes output buffers of 8 bytes; the next steps on the same slot need 12, 16, 20 ... bytes
    # (a buffer was once booked as 16 bytes where 8 had been asked of the allocator).  The binding refuses a block
    # whose arrays do not fit the allocations they live in.
    import torch
    from paper_2406_17918_amd import gss
    tuning(pipeline_depth=1)
    g = synth.chunglu_graph(2000, 15000, 2.2, 5)
    kw = dict(k=8, mode=mode, num_layers=3, refresh_fraction=frac, refresh_period=1, rng_seed=5)
    gs, os_ = gss.Sampler(g.num_nodes, gss.upload_graph(g), tuning=dict(pipeline_depth=1), **kw), oracle_sampler(g, kw)
    step = 0
    for fan in ([2], [1, 1, 2], [2, 2], [2, 1, 1]):
        for batch in (1, 2, 3, 4, 5, 7):
            seeds = synth.seeds_for_step(2000, batch, 9, step)
            assert_blocks_equal(gs.step(torch.from_numpy(seeds).cuda(), fan, step), os_.step(seeds, fan, step), ctx=f"{fan} x {batch}")
            step += 1
    gs.close(); os_.close()


def guarded_allocator(guard=4096):
    from paper_2406_17918_amd import gss

    class Guarded(gss._TorchAllocator):
        """Every allocation sits between two guard zones filled with a pattern; check() verifies them."""

        def __init__(self):
            super().__init__("cuda:0")
            self.whole = {}

        def _alloc(self, ctx, nbytes):
            n = int(nbytes)
            t = self.torch.full((n + 2 * guard,), 0xA5, dtype=self.torch.uint8, device=self.device)
            p = t.data_ptr() + guard
            self.whole[p] = t
            self.live[p] = t[guard:guard + n]
            return p

        def _free(self, ctx, ptr):
            self.check(int(ptr))
            self.whole.pop(int(ptr), None)
            super()._free(ctx, ptr)

        def check(self, only=None):
            for p, t in self.whole.items():
                if only is not None and p != only:
                    continue
                n = t.numel() - 2 * guard
                assert bool((t[:guard] == 0xA5).all()) and bool((t[guard + n:] == 0xA5).all()), f"write outside an allocation of {n} bytes"

    return Guarded()


@pytest.mark.parametrize("mode,frac,k,fan,theta", [
    (gsso.MODE_SHARED_OTF, 0.2, 12, [3, 4, 2], -1), (gsso.MODE_SHARED_OTF, 0.3, 9, [4, 4], 12), (gsso.MODE_OTF, 0.25, 10, [5, 3, 2], -1),
    (gsso.MODE_FCR, 0.0, 10, [4, 4, 4], -1), (gsso.MODE_FBL, 0.0, 8, [3, 3], -1), (gsso.MODE_OTF, 0.2, 40, [20, 10], -1)])
def test_no_write_lands_outside_an_allocation(mode, frac, k, fan, theta, tuning):
    # every buffer the library asks for sits between guard zones; batches of 1 to 600 seeds in random order (buffers of
    # a few bytes up to many tiles, growing while steps are in flight); the zones are intact after every collected
    # step and when a buffer is returned, and the blocks equal the oracle's
    import torch
    from paper_2406_17918_amd import gss
    g = synth.chunglu_graph(3000, 30000, 2.2, 21)
    kw = dict(k=k, mode=mode, num_layers=len(fan), refresh_fraction=frac, refresh_period=2, rng_seed=31, degree_threshold=theta)
    a = guarded_allocator()
    gs, os_ = gss.Sampler(g.num_nodes, gss.upload_graph(g), allocator=a, **kw), oracle_sampler(g, kw)
    rs = np.random.default_rng(7)
    batches = [int(b) for b in rs.choice([1, 2, 3, 5, 9, 30, 64, 129, 300, 600], size=40)]
    seeds = [synth.seeds_for_step(3000, b, 4, i) for i, b in enumerate(batches)]
    dev = [torch.from_numpy(x).cuda() for x in seeds]
    done = 0
    for i in range(len(batches)):
        while i - done >= gs.pipeline_depth:
            assert_blocks_equal(gs.step_wait(), os_.step(seeds[done], fan, done), ctx=f"step {done}")
            a.check()
            done += 1
        gs.step_async(dev[i], fan, i)
    while done < len(batches):
        assert_blocks_equal(gs.step_wait(), os_.step(seeds[done], fan, done), ctx=f"step {done}")
        done += 1
    torch.cuda.synchronize()
    a.check()
    gs.close(); os_.close()
    assert not a.whole


@pytest.mark.parametrize("mode,frac,k,fan,tune", [
    (gsso.MODE_OTF, 0.2, 25, [25, 20], {}), (gsso.MODE_SHARED_OTF, 0.2, 64, [30, 30], {}), (gsso.MODE_FCR, 0.0, 12, [6, 6], {}),
    (gsso.MODE_OTF_FETCH, 0.5, 16, [8, 8], {}), (gsso.MODE_OTF_LAYER, 0.25, 16, [8, 4], {}), (gsso.MODE_SHARED_FCR, 0.0, 20, [10, 10], {}),
    (gsso.MODE_OTF, 0.2, 12, [6, 6], dict(lds_dedupe=1, insert_phase=1)), (gsso.MODE_OTF, 0.2, 12, [6, 6], dict(dedupe_layout=2))])
def test_no_write_lands_outside_an_allocation_on_a_typed_graph(mode, frac, k, fan, tune, tuning):
    # the same on a graph with four node types and seven relations (per-type frontiers, per-relation outputs), in the
    # remaining modes, with the LDS stage of the dedupe and with the hashed table
    import torch
    from paper_2406_17918_amd import gss
    g = synth.hetero_graph([1200, 2000, 60, 300], [(1, 2, 2600), (1, 0, 9000), (0, 0, 5000), (0, 3, 8000)], 2.2, seed=8)
    kw = dict(k=k, mode=mode, num_layers=len(fan), refresh_fraction=frac, refresh_period=3, rng_seed=13)
    a = guarded_allocator()
    gs, os_ = gss.Sampler(g.num_nodes, gss.upload_graph(g), allocator=a, tuning=tune, **kw), oracle_sampler(g, kw)
    rs = np.random.default_rng(11)
    batches = [int(b) for b in rs.choice([1, 2, 3, 7, 40, 150, 400], size=24)]
    seeds = [synth.seeds_for_step(g.num_nodes[0], b, 6, i) for i, b in enumerate(batches)]
    dev = [torch.from_numpy(x).cuda() for x in seeds]
    done = 0
    for i in range(len(batches)):
        while i - done >= gs.pipeline_depth:
            assert_blocks_equal(gs.step_wait(), os_.step(seeds[done], fan, done), ctx=f"step {done}")
            a.check()
            done += 1
        gs.step_async(dev[i], fan, i)
    while done < len(batches):
        assert_blocks_equal(gs.step_wait(), os_.step(seeds[done], fan, done), ctx=f"step {done}")
        done += 1
    torch.cuda.synchronize()
    a.check()
    gs.close(); os_.close()
    assert not a.whole
