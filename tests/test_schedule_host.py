"""Host logic of the step pipeline (no GPU): which phases of the steps in flight share a launch.

The planner is compiled on its own (g++) and driven through simulated sequences of enqueues and waits.  Stream
order between launches is the library's only synchronisation, so what must hold is: a phase only ever depends on
phases issued in EARLIER launches, and every launch makes progress."""
import ctypes as C
import os
import subprocess

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SAMPLE, MARK, SCAN, EMIT, INSERT, PLACE, CHAIN = 0, 1, 2, 3, 4, 5, 6


@pytest.fixture(scope="module")
def shim(tmp_path_factory):
    so = str(tmp_path_factory.mktemp("sched") / "schedule_shim.so")
    subprocess.run(["g++", "-O1", "-std=c++17", "-Wall", "-Wextra", "-shared", "-fPIC", "-I",
                    os.path.join(ROOT, "paper_2406_17918_amd", "csrc"), os.path.join(HERE, "native", "schedule_shim.cpp"),
                    "-o", so], check=True)
    lib = C.CDLL(so)
    lib.sched_items.argtypes = [C.c_int, C.c_uint, C.c_uint, C.c_int, C.POINTER(C.c_int8), C.POINTER(C.c_int8)]
    pi = C.POINTER(C.c_int)
    lib.sched_plan.argtypes = [pi, C.POINTER(C.c_uint), C.POINTER(C.c_uint), pi, pi, pi, C.c_int, C.c_int, C.c_int, pi, pi]
    return lib


def items_of(layers, scan_hops, insert_hops=0, chain=False):
    out = []
    for h in range(layers):
        # (a visit-once step has a place phase where the others have the sample phase; either does the dedupe table
        # inserts itself unless the hop has an insert phase)
        out += [(h, PLACE if chain else SAMPLE)] + ([(h, INSERT)] if (insert_hops >> h) & 1 else []) + [(h, MARK)]
        out += ([(h, SCAN)] if (scan_hops >> h) & 1 else []) + [(h, EMIT)]
    return out


def test_phase_list_of_a_step(shim):
    for layers in range(1, 9):
        for scan_hops in (0, 1, 0b101, (1 << layers) - 1):
            for insert_hops in (0, 1 << (layers - 1), (1 << layers) - 1):
                for chain in (0, 1):
                    hop = (C.c_int8 * 48)(); phase = (C.c_int8 * 48)()
                    n = shim.sched_items(layers, scan_hops, insert_hops, chain, hop, phase)
                    assert [(hop[i], phase[i]) for i in range(n)] == items_of(layers, scan_hops & ((1 << layers) - 1), insert_hops, chain)


class Sim:
    """Steps are enqueued in order; `flight` holds the indices of those not yet collected, oldest first."""

    def __init__(self, shim, otf, shared):
        self.shim, self.otf, self.shared = shim, otf, shared
        self.steps = []          # per step: dict(L, scan, next, cnext, at={item index: tick}, cat={chain phase: tick})
        self.flight = []
        self.ticks = 0

    def enqueue(self, layers, scan_hops=0, insert_hops=0, chain=False):
        # the driver lets the steps in flight finish issuing before a step of another depth joins (OTF, per-layer tables)
        if self.otf and not self.shared and self.flight and self.steps[self.flight[-1]]["L"] != layers:
            self.drain()
        self.steps.append(dict(L=layers, scan=scan_hops, ins=insert_hops, next=0, at={}, chain=chain, cnext=0, cat={},
                               nchain=layers if chain else 0, items=items_of(layers, scan_hops, insert_hops, chain)))
        self.flight.append(len(self.steps) - 1)
        self.tick()

    def tick(self):
        n = len(self.flight)
        arr = lambda key, ty=C.c_int: (ty * max(n, 1))(*[int(self.steps[i][key]) for i in self.flight])
        ts, ti = (C.c_int * (2 * n + 1))(), (C.c_int * (2 * n + 1))()
        m = self.shim.sched_plan(arr("L"), arr("scan", C.c_uint), arr("ins", C.c_uint), arr("chain"), arr("next"),
                                 arr("cnext"), n, int(self.otf), int(self.shared), ts, ti)
        assert 0 <= m <= 2 * n
        chosen = [(self.flight[ts[j]], ti[j]) for j in range(m)]
        assert len(set(chosen)) == m and [c[0] for c in chosen] == sorted(c[0] for c in chosen)
        for i in {c[0] for c in chosen}:                                      # at most one list phase and one chain phase per step
            mine = [it for st_, it in chosen if st_ == i]
            assert sum(it >= 0 for it in mine) <= 1 and sum(it < 0 for it in mine) <= 1
        for i, it in chosen:
            st = self.steps[i]
            if it >= 0:
                assert it == st["next"] < len(st["items"])
                st["at"][it] = self.ticks
                st["next"] += 1
            else:
                assert -1 - it == st["cnext"] < st["nchain"]
                st["cat"][st["cnext"]] = self.ticks
                st["cnext"] += 1
        self.ticks += 1
        return m

    def is_open(self, i):
        st = self.steps[i]
        return st["next"] < len(st["items"]) or st["cnext"] < st["nchain"]

    def open(self):
        return [i for i in self.flight if self.is_open(i)]

    def drain(self):
        while self.open():
            assert self.tick() >= 1

    def wait_oldest(self):
        i = self.flight[0]
        stalled = 0
        while self.is_open(i):
            before = self.steps[i]["next"] + self.steps[i]["cnext"]
            assert self.tick() >= 1
            # the oldest step makes progress - at once, except that a place phase may wait a few ticks for a younger
            # step's chain to come round to its light hop
            stalled = 0 if self.steps[i]["next"] + self.steps[i]["cnext"] > before else stalled + 1
            assert stalled <= 8 and (stalled == 0 or self.steps[i]["chain"])
        self.flight.pop(0)

    def sample_tick(self, i, h):
        st = self.steps[i]
        return st["at"].get(st["items"].index((h, SAMPLE)))


@pytest.mark.parametrize("otf,shared", [(False, False), (True, False), (True, True)])
@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_every_phase_depends_only_on_earlier_ticks(shim, otf, shared, seed):
    rs = np.random.default_rng(seed)
    sim = Sim(shim, otf, shared)
    for step in range(120):
        while len(sim.flight) >= 12 or (sim.flight and rs.random() < 0.25):
            sim.wait_oldest()
        layers = int(rs.choice([1, 2, 3, 3, 3, 5, 8])) if seed else 3
        scan = int(rs.integers(0, 1 << layers)) if rs.random() < 0.3 else 0
        ins = int(rs.integers(0, 1 << layers)) if rs.random() < 0.5 else 0
        sim.enqueue(layers, scan, ins)
    while sim.flight:
        sim.wait_oldest()
    for i, st in enumerate(sim.steps):
        ticks = [st["at"][j] for j in range(len(st["items"]))]
        assert ticks == sorted(set(ticks))                                    # a step's own phases: strictly later ticks
        if not otf or i == 0:
            continue
        prev = sim.steps[i - 1]
        for h in range(st["L"]):
            mine = sim.sample_tick(i, h)
            if shared:                                                        # one table: after every sample phase before
                assert all(sim.sample_tick(i - 1, g) < mine for g in range(prev["L"]))
            elif prev["L"] == st["L"]:                                        # per-layer tables: same hop of the step before
                assert sim.sample_tick(i - 1, h) < mine
            else:                                                             # another depth: the steps never overlap
                assert max(prev["at"].values()) < min(st["at"].values())


def test_independent_steps_advance_together_and_a_full_pipeline_costs_one_tick_per_step(shim):
    sim = Sim(shim, otf=False, shared=False)
    for step in range(40):
        if len(sim.flight) == 12:
            sim.wait_oldest()
        sim.enqueue(3)
    # steady state: every enqueue issued exactly one tick, and each tick carried a phase of every open step
    assert sim.ticks == 40
    for i, st in enumerate(sim.steps[:30]):
        assert [st["at"][j] for j in range(9)] == list(range(i, i + 9))
    sim2 = Sim(shim, otf=True, shared=False)
    for step in range(40):
        if len(sim2.flight) == 12:
            sim2.wait_oldest()
        sim2.enqueue(3)
    assert sim2.ticks == 40                                                   # OTF's ordering is met by the skew alone
    sim3 = Sim(shim, otf=True, shared=True)
    for step in range(20):
        if len(sim3.flight) == 12:
            sim3.wait_oldest()
        sim3.enqueue(3)
    while sim3.flight:
        sim3.wait_oldest()
    assert sim3.ticks == 20 * 7 + 2                                           # shared table: 7 ticks per step, 9 for the last


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_visit_once_steps(shim, seed):
    # one table for all hops, refreshed per visit: chain phases (the only ones that touch the table) of consecutive
    # steps never overlap and keep their order; a hop's place phase comes after its chain phase; old-style steps
    # (sample phases touch the table) may be mixed in
    rs = np.random.default_rng(seed)
    sim = Sim(shim, otf=True, shared=True)
    for step in range(80):
        while len(sim.flight) >= 10 or (sim.flight and rs.random() < 0.2):
            sim.wait_oldest()
        layers = int(rs.choice([1, 2, 3, 3, 4]))
        sim.enqueue(layers, scan_hops=int(rs.integers(0, 1 << layers)) if rs.random() < 0.3 else 0,
                    insert_hops=int(rs.integers(0, 1 << layers)) if rs.random() < 0.4 else 0,
                    chain=bool(seed == 0 or rs.random() < 0.7))
    while sim.flight:
        sim.wait_oldest()

    def table_ticks(st):
        return sorted(st["cat"].values()) if st["chain"] else [st["at"][st["items"].index((h, SAMPLE))] for h in range(st["L"])]
    for i, st in enumerate(sim.steps):
        ticks = [st["at"][j] for j in range(len(st["items"]))]
        assert ticks == sorted(set(ticks))
        if st["chain"]:
            assert [st["cat"][c] for c in range(st["L"])] == sorted(set(st["cat"].values()))
            for h in range(st["L"]):
                assert st["cat"][h] < st["at"][st["items"].index((h, PLACE))]
        if i:
            assert max(table_ticks(sim.steps[i - 1])) < min(table_ticks(st))
    # the place phases of the outer hops share a tick only with the chain phase of a hop 0, or with none
    chain_hop_at = {}
    for st in sim.steps:
        for c, t in st["cat"].items():
            assert t not in chain_hop_at                                       # one chain phase per tick
            chain_hop_at[t] = c
    for st in sim.steps:
        if st["chain"]:
            for h in range(1, st["L"]):
                assert chain_hop_at.get(st["at"][st["items"].index((h, PLACE))], 0) == 0
    if seed == 0:
        # steady state of 3-hop steps: three ticks per step (the chain), the nine list phases trail behind
        sim = Sim(shim, otf=True, shared=True)
        for step in range(30):
            if len(sim.flight) == 8:
                sim.wait_oldest()
            sim.enqueue(3, chain=True)
        while sim.flight:
            sim.wait_oldest()
        st = sim.steps[10]
        assert [st["cat"][c] for c in range(3)] == [30, 31, 32]
        assert [st["at"][j] for j in range(9)] == [31, 32, 33, 36, 37, 38, 39, 40, 41]
        assert sim.ticks == 30 * 3 + 7                                        # (the last step drains without waiting)
        # the same with an insert phase on the outermost hop: its place phase still joins a hop-0 tick, the insert
        # phase the tick after (the chain phase of hop 1), and the step ends one tick later
        sim = Sim(shim, otf=True, shared=True)
        for step in range(30):
            if len(sim.flight) == 8:
                sim.wait_oldest()
            sim.enqueue(3, insert_hops=0b100, chain=True)
        while sim.flight:
            sim.wait_oldest()
        st = sim.steps[10]
        assert st["items"][6:8] == [(2, PLACE), (2, INSERT)]
        assert [st["cat"][c] for c in range(3)] == [30, 31, 32]
        assert [st["at"][j] for j in range(10)] == [31, 32, 33, 36, 37, 38, 39, 40, 41, 42]
        assert sim.ticks == 30 * 3 + 8
