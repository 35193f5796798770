"""Pins for the oracle's row operations: FILL_FULL, REFRESH_PART (Alg. 2 RefreshCache), PICK (SampleFromCache).

Validity invariants on random inputs, and exact uniformity by brute force: the random source is replaced by an
enumerator that walks every possible outcome of the draws, so each result must occur exactly equally often.
"""
import itertools
from collections import Counter
from math import comb, factorial

import numpy as np
import pytest

from oracle import gsso


def philox(seed=0):
    return gsso.Rng(seed)


def prio_rng(table):
    """Random source whose draw for (purpose, index) is table[purpose][index] in the 48 high bits (the low 16 bits
    of a priority are taken by the index)."""
    return gsso.Rng(fn=lambda purpose, layer, rel, node, index, attempt, step: table[purpose][index] << 16)


class SeqRng:
    """Random source for `below(deg)` draws: returns the given positions in call order; once exhausted it
    cycles 0,1,2,... (which always terminates a rejection loop) and flags the run as exhausted."""

    def __init__(self, deg, seq, prio_table=None):
        self.deg, self.seq, self.i, self.exhausted = deg, seq, 0, False
        self.prio_table = prio_table or {}
        self.rng = gsso.Rng(fn=self._draw)

    def _draw(self, purpose, layer, rel, node, index, attempt, step):
        if purpose in self.prio_table:
            return self.prio_table[purpose][index] << 16
        if self.i < len(self.seq):
            pos = self.seq[self.i]
        else:
            self.exhausted = True
            pos = (self.i - len(self.seq)) % self.deg
        self.i += 1
        return (pos * 2**64 + self.deg - 1) // self.deg   # smallest x64 with floor(x64*deg / 2^64) == pos


# ----------------------------------------------------------------- validity
@pytest.mark.parametrize("k", [1, 4, 10, 20, 30, 33, 40, 64])
def test_fill_full_validity(k):
    rs = np.random.default_rng(k)
    for trial in range(60):
        deg = int(rs.choice([0, 1, k - 1, k, k + 1, 2 * k - 1, 2 * k, 2 * k + 1, 5 * k + 3, 1000]))
        deg = max(deg, 0)
        adj = np.sort(rs.choice(100000, size=deg, replace=False)).astype(np.int32)
        row = gsso.fill_full_row(philox(trial), adj, k, layer=1, relation=0, node=trial, stepword=3)
        n = min(deg, k)
        assert (row[:n] >= 0).all() and (row[n:] == -1).all()
        assert len(set(row[:n].tolist())) == n
        assert set(row[:n].tolist()) <= set(adj.tolist())
        if deg <= k:
            assert np.array_equal(row[:n], adj)              # whole adjacency, CSR order
        elif deg < 2 * k:
            assert (np.diff(row) > 0).all()                  # ascending position order (adj is sorted)


def test_fill_full_depends_on_key_fields():
    adj = np.arange(100, dtype=np.int32)
    base = gsso.fill_full_row(philox(1), adj, 8, layer=0, relation=0, node=5, stepword=0)
    assert not np.array_equal(base, gsso.fill_full_row(philox(2), adj, 8, node=5))
    assert not np.array_equal(base, gsso.fill_full_row(philox(1), adj, 8, node=6))
    assert not np.array_equal(base, gsso.fill_full_row(philox(1), adj, 8, node=5, stepword=10))
    assert not np.array_equal(base, gsso.fill_full_row(philox(1), adj, 8, node=5, layer=1))
    assert not np.array_equal(base, gsso.fill_full_row(philox(1), adj, 8, node=5, relation=1))
    assert np.array_equal(base, gsso.fill_full_row(philox(1), adj, 8, node=5))


@pytest.mark.parametrize("k,n_new", [(10, 2), (20, 4), (30, 3), (25, 5), (4, 4), (6, 1), (33, 3), (40, 8), (64, 6), (64, 64)])
def test_refresh_part_validity(k, n_new):
    rs = np.random.default_rng(100 + k)
    for trial in range(80):
        deg = int(rs.choice([k - 1, k, k + 1, k + 2, 2 * k - 1, 2 * k, 2 * k + 1, 7 * k, 3000]))
        adj = np.sort(rs.choice(100000, size=deg, replace=False)).astype(np.int32)
        row0 = gsso.fill_full_row(philox(trial), adj, k, node=trial)
        row1 = gsso.refresh_part_row(philox(trial), adj, row0, n_new, node=trial, step=trial + 1)
        if deg <= k:
            assert np.array_equal(row0, row1)                # the row is the whole adjacency: never changes
            continue
        assert len(set(row1.tolist())) == k and set(row1.tolist()) <= set(adj.tolist())
        changed = np.flatnonzero(row0 != row1)
        assert len(changed) <= n_new                         # at least k - n_new slots stay in place
        # which slots were evicted is a function of the EVICT priorities only
        e = [gsso.priority(gsso.philox_draw(trial, gsso.EVICT, 0, 0, trial, j, 0, trial + 1), j) for j in range(k)]
        evicted = sorted(sorted(range(k), key=lambda j: e[j])[:n_new])
        assert set(changed.tolist()) <= set(evicted)
        retained = set(np.delete(row0, evicted).tolist())
        assert all(int(row1[j]) not in retained for j in evicted)
        if deg < 2 * k:
            # redrawn ids sit in the evicted slots in ascending adjacency position
            assert (np.diff(row1[evicted]) > 0).all()


def test_refresh_part_zero_new_is_noop():
    adj = np.arange(50, dtype=np.int32)
    row0 = gsso.fill_full_row(philox(3), adj, 10)
    assert np.array_equal(row0, gsso.refresh_part_row(philox(3), adj, row0, 0, step=9))


def test_pick_validity_and_order():
    rs = np.random.default_rng(5)
    for trial in range(200):
        k = int(rs.integers(1, 31))
        length = int(rs.integers(0, k + 1))
        f = int(rs.integers(1, k + 1))
        row = np.full(k, -1, np.int32)
        row[:length] = rs.choice(10**6, size=length, replace=False)
        out = gsso.pick_row(philox(trial), row, f, node=trial, step=trial)
        if length <= f:
            assert np.array_equal(out, row[:length])
        else:
            assert len(out) == f and len(set(out.tolist())) == f
            pos = [int(np.flatnonzero(row == x)[0]) for x in out]
            assert pos == sorted(pos)                        # ascending slot order


def test_pick_shared_bands_partition_the_row():
    # One ranking per (step, node); layer l takes ranks [off_l, off_l + f_l). With len == k == sum(f) the
    # bands are pairwise disjoint and cover the row.
    k, fan = 30, [15, 10, 5]
    row = (np.arange(k, dtype=np.int32) * 7 + 3)
    for node in range(20):
        bands, off = [], 0
        for l, f in enumerate(fan):
            bands.append(gsso.pick_row(philox(9), row, f, shared=True, band_offset=off,
                                       layer=gsso.SHARED_LAYER, node=node, step=4))
            off += f
        allids = np.concatenate(bands)
        assert len(set(allids.tolist())) == k and set(allids.tolist()) == set(row.tolist())
        # band membership follows the priority ranking
        p = [gsso.priority(gsso.philox_draw(9, gsso.PICK, gsso.SHARED_LAYER, 0, node, j, 0, 4), j) for j in range(k)]
        order = sorted(range(k), key=lambda j: p[j])
        assert set(bands[0].tolist()) == set(row[order[:15]].tolist())
        assert set(bands[1].tolist()) == set(row[order[15:25]].tolist())
        assert set(bands[2].tolist()) == set(row[order[25:]].tolist())


def test_pick_shared_short_rows_clamp_the_band():
    # len < off + f: the band slides down to start = len - f; len <= f: the whole row.
    row = np.full(30, -1, np.int32)
    row[:12] = np.arange(12) + 100
    p = [gsso.priority(gsso.philox_draw(0, gsso.PICK, gsso.SHARED_LAYER, 0, 7, j, 0, 2), j) for j in range(12)]
    order = sorted(range(12), key=lambda j: p[j])
    out = gsso.pick_row(philox(0), row, 5, shared=True, band_offset=25, layer=gsso.SHARED_LAYER, node=7, step=2)
    assert set(out.tolist()) == set(row[order[7:12]].tolist())
    out = gsso.pick_row(philox(0), row, 10, shared=True, band_offset=15, layer=gsso.SHARED_LAYER, node=7, step=2)
    assert set(out.tolist()) == set(row[order[2:12]].tolist())
    out = gsso.pick_row(philox(0), row, 15, shared=True, band_offset=0, layer=gsso.SHARED_LAYER, node=7, step=2)
    assert np.array_equal(out, row[:12])


# ----------------------------------------------------------------- exact uniformity (brute force)
@pytest.mark.parametrize("m,f", [(3, 1), (4, 2), (5, 2), (5, 3), (6, 4), (7, 3)])
def test_pick_exactly_uniform_over_all_priority_orders(m, f):
    row = np.arange(m, dtype=np.int32) + 10
    counts = Counter()
    for perm in itertools.permutations(range(m)):
        out = gsso.pick_row(prio_rng({gsso.PICK: perm}), row, f)
        counts[tuple(out.tolist())] += 1
    assert len(counts) == comb(m, f)
    assert set(counts.values()) == {factorial(m) // comb(m, f)}


def test_priority_ties_go_to_the_smaller_index():
    row = np.arange(6, dtype=np.int32) + 10
    out = gsso.pick_row(prio_rng({gsso.PICK: [5, 5, 5, 5, 5, 5]}), row, 2)
    assert out.tolist() == [10, 11]
    out = gsso.pick_row(prio_rng({gsso.PICK: [9, 1, 9, 1, 1, 9]}), row, 2)
    assert out.tolist() == [11, 13]


@pytest.mark.parametrize("d,k", [(3, 2), (5, 3), (5, 4), (7, 4)])
def test_fill_full_priority_regime_exactly_uniform(d, k):
    # k < d < 2k: the k positions of smallest priority
    adj = np.arange(d, dtype=np.int32) + 20
    counts = Counter()
    for perm in itertools.permutations(range(d)):
        row = gsso.fill_full_row(prio_rng({gsso.FILL_FULL: perm}), adj, k)
        counts[tuple(row.tolist())] += 1
    assert len(counts) == comb(d, k)
    assert set(counts.values()) == {factorial(d) // comb(d, k)}


@pytest.mark.parametrize("d,k,depth", [(4, 2, 6), (5, 2, 5), (6, 3, 5), (8, 2, 4), (8, 4, 4)])
def test_fill_full_rejection_regime_exactly_uniform(d, k, depth):
    # d >= 2k: all candidate sequences of `depth` draws; among the runs that finish within them every ordered
    # k-tuple of distinct positions occurs equally often.
    adj = np.arange(d, dtype=np.int32) + 30
    counts = Counter()
    finished = 0
    for seq in itertools.product(range(d), repeat=depth):
        src = SeqRng(d, seq)
        row = gsso.fill_full_row(src.rng, adj, k)
        assert len(set(row.tolist())) == k
        if not src.exhausted:
            counts[tuple(row.tolist())] += 1
            finished += 1
    assert finished > 0
    n_ordered = factorial(d) // factorial(d - k)
    assert len(counts) == n_ordered
    assert len(set(counts.values())) == 1


def test_rejection_round_major_order():
    # slots 0,1,2 draw in round 0; a slot that collides retries in round 1 (after every slot had its round-0 turn)
    adj = np.arange(10, dtype=np.int32) + 50
    calls = []

    def fn(purpose, layer, rel, node, index, attempt, step):
        calls.append((index, attempt))
        pos = {(0, 0): 4, (1, 0): 4, (2, 0): 7, (1, 1): 7, (1, 2): 2}[(index, attempt)]
        return (pos * 2**64 + 9) // 10

    row = gsso.fill_full_row(gsso.Rng(fn=fn), adj, 3)
    assert calls == [(0, 0), (1, 0), (2, 0), (1, 1), (1, 2)]
    assert row.tolist() == [54, 52, 57]


def test_fcr_period_one_is_plain_uniform_sampling_exactly():
    # FILL_FULL then PICK with fresh randomness each step (FCR, R = 1): deg 5, k 4, f 2 -> all 5! x 4! outcomes;
    # every one of the 10 neighbor pairs must come up equally often (a uniform f-subset of a uniform k-subset).
    adj = np.arange(5, dtype=np.int32) + 40
    counts = Counter()
    for pf in itertools.permutations(range(5)):
        row = gsso.fill_full_row(prio_rng({gsso.FILL_FULL: pf}), adj, 4)
        for pp in itertools.permutations(range(4)):
            out = gsso.pick_row(prio_rng({gsso.PICK: pp}), row, 2)
            counts[frozenset(out.tolist())] += 1
    assert len(counts) == 10 and set(counts.values()) == {factorial(5) * factorial(4) // 10}


def test_refresh_part_priority_regime_keeps_rows_uniform():
    # deg 5, k 3, n_new 1 (k < deg < 2k): uniform row in -> uniform row out, over all EVICT and FILL_PART orders.
    adj = np.arange(5, dtype=np.int32) + 60
    counts = Counter()
    for init in itertools.combinations(range(5), 3):                 # uniform initial row
        row0 = adj[list(init)]
        for pe in itertools.permutations(range(3)):
            for pq in itertools.permutations(range(5)):
                row1 = gsso.refresh_part_row(prio_rng({gsso.EVICT: pe, gsso.FILL_PART: pq}), adj, row0, 1)
                assert len(set(row1.tolist())) == 3
                counts[frozenset(row1.tolist())] += 1
    assert len(counts) == 10 and len(set(counts.values())) == 1


@pytest.mark.parametrize("d,k,n_new,depth", [(4, 2, 1, 4), (6, 3, 2, 3), (7, 3, 1, 3)])
def test_refresh_part_rejection_regime_keeps_rows_uniform(d, k, n_new, depth):
    # deg >= 2k: every initial row, all EVICT orders and all candidate sequences of `depth` draws; among the
    # finished runs each k-subset is equally likely.
    adj = np.arange(d, dtype=np.int32) + 70
    counts = Counter()
    for init in itertools.combinations(range(d), k):
        row0 = adj[list(init)]
        for pe in itertools.permutations(range(k)):
            for seq in itertools.product(range(d), repeat=depth):
                src = SeqRng(d, seq, {gsso.EVICT: pe})
                row1 = gsso.refresh_part_row(src.rng, adj, row0, n_new)
                assert len(set(row1.tolist())) == k
                if not src.exhausted:
                    counts[frozenset(row1.tolist())] += 1
    assert len(counts) == comb(d, k) and len(set(counts.values())) == 1


def test_refresh_then_pick_stays_uniform():
    # REFRESH_PART o PICK: deg 5, k 3, n_new 1, f 2 from a uniform initial row: each neighbor pair equally often.
    adj = np.arange(5, dtype=np.int32) + 80
    counts = Counter()
    for init in itertools.combinations(range(5), 3):
        row0 = adj[list(init)]
        for pe in itertools.permutations(range(3)):
            for pq in itertools.permutations(range(5)):
                row1 = gsso.refresh_part_row(prio_rng({gsso.EVICT: pe, gsso.FILL_PART: pq}), adj, row0, 1)
                for pp in itertools.permutations(range(3)):
                    out = gsso.pick_row(prio_rng({gsso.PICK: pp}), row1, 2)
                    counts[frozenset(out.tolist())] += 1
    assert len(counts) == 10 and len(set(counts.values())) == 1


@pytest.mark.parametrize("k,f,deg", [(40, 20, 90), (64, 20, 100), (64, 20, 70), (60, 20, 400)])
def test_wide_rows_fill_then_pick_is_uniform_chi_square(k, f, deg):
    # rows of 33-64 slots follow the same row functions; with the real generator, a full fill followed by the draw
    # picks every neighbor equally often (both fill regimes: deg < 2k and deg >= 2k)
    adj = np.arange(1000, 1000 + deg, dtype=np.int32)
    count = Counter()
    trials = 3000
    for t in range(trials):
        row = gsso.fill_full_row(philox(77), adj, k, node=5, stepword=t)
        picks = gsso.pick_row(philox(77), row, f, node=5, step=t)
        assert len(picks) == f and len(set(picks.tolist())) == f
        count.update(picks.tolist())
    exp = trials * f / deg
    chi2 = sum((count.get(int(a), 0) - exp) ** 2 / exp for a in adj)
    # chi-square with deg - 1 degrees of freedom: mean deg - 1, sd sqrt(2 (deg - 1)); 5 sd
    assert chi2 < (deg - 1) + 5 * (2 * (deg - 1)) ** 0.5, chi2
