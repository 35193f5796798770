"""gss_cache_checksum_static - the entry point that allocates nothing (partial sums in a static device array) - gives
the checksum of gss_cache_checksum: two calls in a row, the second on a smaller table, plus the size limit."""
import pytest

from oracle import gsso
from paper_2406_17918_amd import synth

pytestmark = pytest.mark.gpu


def test_static_checksum_equals_the_allocating_one_on_two_calls_in_a_row():
    import torch
    from paper_2406_17918_amd import gss
    out = torch.zeros(1, dtype=torch.int64, device="cuda")
    big = synth.chunglu_graph(6000, 60000, 2.2, 3)         # 6000 x 20 cells: eight chunks of partial sums
    small = synth.chunglu_graph(300, 2000, 2.2, 4)         # 300 x 20 cells: one chunk, the scratch keeps the older sums
    results = []
    for g in (big, small):
        rels = gss.upload_graph(g)
        s = gss.Sampler(g.num_nodes, rels, k=20, mode=gsso.MODE_OTF, num_layers=2, refresh_fraction=0.25, rng_seed=7)
        o = gsso.Sampler(g.num_nodes, [gsso.Relation(0, 0, g.relations[0].indptr, g.relations[0].indices)], k=20,
                         mode=gsso.MODE_OTF, num_layers=2, refresh_fraction=0.25, rng_seed=7)
        seeds = synth.seeds_for_step(g.num_nodes[0], 100, 1, 0)
        s.step(torch.from_numpy(seeds).cuda(), [5, 5], 0)
        o.step(seeds, [5, 5], 0)
        for layer in (0, 1):
            want = s.checksum(layer, 0)
            s.checksum_static(out, layer, 0)
            got = int(out.item()) & 0xFFFFFFFFFFFFFFFF
            assert got == want == o.checksum(layer, 0), (g.num_nodes, layer)
            results.append(got)
        s.close()
        o.close()
    assert len(set(results)) == 4


def test_static_checksum_rejects_what_it_cannot_hold():
    import torch
    from paper_2406_17918_amd import gss
    g = synth.chunglu_graph(300, 2000, 2.2, 4)
    s = gss.Sampler(g.num_nodes, gss.upload_graph(g), k=8, mode=gsso.MODE_FCR, num_layers=1, rng_seed=7)
    out = torch.zeros(3, dtype=torch.int64, device="cuda")
    lib = gss.load_library()
    assert lib.gss_cache_checksum_static(s._h, 0, 0, None, None) == gss.GSS_ERR_INVALID_ARG
    assert lib.gss_cache_checksum_static(s._h, 1, 0, out.data_ptr(), None) == gss.GSS_ERR_INVALID_ARG
    assert lib.gss_cache_checksum_static(s._h, 0, 0, out.data_ptr() + 4, None) == gss.GSS_ERR_INVALID_ARG
    s.step_async(torch.tensor([1, 2], dtype=torch.int32, device="cuda"), [3], 0)
    assert lib.gss_cache_checksum_static(s._h, 0, 0, out.data_ptr(), None) == gss.GSS_ERR_INVALID_ARG   # a step is in flight
    s.step_wait()
    assert lib.gss_cache_checksum_static(s._h, 0, 0, out.data_ptr(), None) == gss.GSS_OK
    torch.cuda.synchronize()
    assert (int(out[0].item()) & 0xFFFFFFFFFFFFFFFF) == s.checksum(0, 0)
    s.close()


def test_static_checksum_size_limit():
    # 8.5 M nodes x 32 slots = 272 M cells: more than the static array's partial sums cover (2^28 cells)
    import numpy as np
    import torch
    from paper_2406_17918_amd import gss
    n = 8_500_000
    g = synth.Graph([n], [synth.Relation(0, 0, np.zeros(n + 1, dtype=np.int32), np.zeros(0, dtype=np.int32))])
    s = gss.Sampler(g.num_nodes, gss.upload_graph(g), k=32, mode=gsso.MODE_OTF, num_layers=1, refresh_fraction=0.5, rng_seed=7)
    out = torch.zeros(1, dtype=torch.int64, device="cuda")
    with pytest.raises(gss.GssError) as e:
        s.checksum_static(out)
    assert e.value.status == gss.GSS_ERR_INVALID_ARG and "exceed the static scratch" in str(e.value)
    assert s.checksum(0, 0) != 0          # the allocating entry point has no such limit
    s.close()
