"""Pin of the reading that the two per-slot draws of a visited node - EVICT (which slots are redrawn) and PICK
(which slots are drawn for the fanout) - come from ONE Philox block per slot: EVICT from output words (0,1), PICK from
words (2,3).  With the real Philox source (not an injected one): over many keyed (node, step) draws the evicted set
and the picked set of a row are independent and each uniform, and the refresh followed by the draw keeps drawing
every neighbor equally often."""
from itertools import combinations
from math import comb

import numpy as np

from oracle import gsso

K, N_NEW, F = 8, 2, 3
SEED = 0x1234ABCD5678


def sets_for(node, step, layer=1, relation=0):
    ev = [gsso.priority(gsso.philox_draw(SEED, gsso.EVICT, layer, relation, node, j, 0, step), j) for j in range(K)]
    pk = [gsso.priority(gsso.philox_draw(SEED, gsso.PICK, layer, relation, node, j, 0, step), j) for j in range(K)]
    return tuple(sorted(np.argsort(ev)[:N_NEW].tolist())), tuple(sorted(np.argsort(pk)[:F].tolist()))


def test_evicted_and_picked_sets_of_one_block_are_independent_and_uniform():
    e_index = {c: i for i, c in enumerate(combinations(range(K), N_NEW))}
    p_index = {c: i for i, c in enumerate(combinations(range(K), F))}
    joint = np.zeros((len(e_index), len(p_index)), dtype=np.int64)
    overlap = np.zeros(N_NEW + 1, dtype=np.int64)
    n = 0
    for node in range(400):
        for step in range(300):
            e, p = sets_for(node, step)
            joint[e_index[e], p_index[p]] += 1
            overlap[len(set(e) & set(p))] += 1
            n += 1
    assert n == 120_000
    # each set uniform over its C(8,2) / C(8,3) values
    for marg in (joint.sum(1), joint.sum(0)):
        exp = n / len(marg)
        z = (((marg - exp) ** 2 / exp).sum() - (len(marg) - 1)) / np.sqrt(2 * (len(marg) - 1))
        assert abs(z) < 4.0, z
    # independent: the joint table is flat (28 x 56 cells, about 77 draws each) ...
    exp = n / joint.size
    z = (((joint - exp) ** 2 / exp).sum() - (joint.size - 1)) / np.sqrt(2 * (joint.size - 1))
    assert abs(z) < 4.0, z
    # ... and the overlap of the two sets is hypergeometric
    hyper = np.array([comb(F, m) * comb(K - F, N_NEW - m) / comb(K, N_NEW) for m in range(N_NEW + 1)])
    chi = float(((overlap - n * hyper) ** 2 / (n * hyper)).sum())
    assert chi < 18.4, (chi, overlap)          # chi2(2): p = 1e-4
    # a planted dependence is seen: PICK reading the EVICT words gives identical orders
    same = sum(set(np.argsort([gsso.philox_draw(SEED, gsso.EVICT, 1, 0, v, j, 0, 5) for j in range(K)])[:N_NEW].tolist())
               <= set(np.argsort([gsso.philox_draw(SEED, gsso.EVICT, 1, 0, v, j, 0, 5) for j in range(K)])[:F].tolist())
               for v in range(50))
    assert same == 50 and overlap[N_NEW] < 0.2 * n


def test_refresh_then_pick_with_the_real_source_draws_every_neighbor_equally_often():
    # one node with 12 neighbors, a row of 8, 2 slots redrawn per step, 3 picked: over many steps every neighbor is picked
    # equally often, and so is every pair of neighbors (the picks of a step are a uniform 3-subset)
    deg = 12
    adj = np.arange(100, 100 + deg, dtype=np.int32)
    rng = gsso.Rng(SEED)
    row = gsso.fill_full_row(rng, adj, K, layer=1, relation=0, node=7, stepword=0)
    steps, thin = 36_000, 6                 # samples a few steps apart: a row keeps 6 of its 8 entries per step
    single = np.zeros(deg, dtype=np.int64)
    pairs = np.zeros((deg, deg), dtype=np.int64)
    taken = 0
    for t in range(1, steps + 1):
        row = gsso.refresh_part_row(rng, adj, row, N_NEW, layer=1, relation=0, node=7, step=t)
        assert len(set(row.tolist())) == K and set(row.tolist()) <= set(adj.tolist())
        if t % thin:
            continue
        picks = gsso.pick_row(rng, row, F, layer=1, relation=0, node=7, step=t) - 100
        assert len(picks) == F
        single[picks] += 1
        for a, b in combinations(sorted(picks.tolist()), 2):
            pairs[a, b] += 1
        taken += 1
    e1 = taken * F / deg
    x1 = float(((single - e1) ** 2 / e1).sum()) * (deg - 1) / (deg - F)        # without-replacement correction
    assert (x1 - (deg - 1)) / np.sqrt(2 * (deg - 1)) < 4.0, single
    up = pairs[np.triu_indices(deg, 1)]
    e2 = taken * comb(F, 2) / comb(deg, 2)
    x2 = float(((up - e2) ** 2 / e2).sum())
    assert (x2 - (len(up) - 1)) / np.sqrt(2 * (len(up) - 1)) < 4.5, x2
