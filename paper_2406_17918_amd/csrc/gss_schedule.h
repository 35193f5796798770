// Which phases of the steps in flight share a launch: plain host logic, no device code, so that it can
// be compiled and checked on its own.
#pragma once
#include <stdint.h>

namespace gss {

// A step is a chain of phases: per hop sample -> [insert ->] mark -> [scan ->] emit.
// A "visit-once" step (one table for all hops, refreshed per visit) splits the work differently: its CHAIN phases, one
// per hop, do everything that touches the cache table - they find the nodes a hop visits for the first time in this
// step and draw the picks of all their remaining hops at once, into a holding area -, and a list of per-hop phases
// place -> mark -> [scan ->] emit puts the picks into frontier order, dedupes and emits.  Only the chain phases of
// consecutive steps depend on each other; the list trails behind and shares launches with the chains of later steps.
enum Phase : int32_t { PH_SAMPLE = 0, PH_MARK = 1, PH_SCAN = 2, PH_EMIT = 3, PH_INSERT = 4, PH_PLACE = 5, PH_CHAIN = 6 };

constexpr int SCHED_MAX_LAYERS = 8;
constexpr int SCHED_MAX_ITEMS = SCHED_MAX_LAYERS * 5;      // per hop at most: sample | place, insert, mark, scan, emit

// The phases of one step in order, and how many of them have been put into a launch.
struct StepItems {
  int L = 0;
  int num_items = 0, next_item = 0;
  int num_chain = 0, next_chain = 0;     // visit-once steps: chain phase c belongs to hop c; one per launch
  int8_t item_hop[SCHED_MAX_ITEMS] = {};
  int8_t item_phase[SCHED_MAX_ITEMS] = {};

  // hop h gets a separate scan phase iff bit h of `scan_hops` is set (hops with very many tiles), and a
  // separate insert phase iff bit h of `insert_hops` is set (large hops: the dedupe table inserts leave
  // the sample phase - or the place phase of a visit-once step -, which shortens the longest phase of a launch).
  // `chain`: a visit-once step.
  void build(int layers, uint32_t scan_hops, uint32_t insert_hops, bool chain = false) {
    L = layers; num_items = 0; next_item = 0;
    num_chain = chain ? layers : 0; next_chain = 0;
    auto push = [&](int h, Phase ph) { item_hop[num_items] = (int8_t)h; item_phase[num_items++] = (int8_t)ph; };
    for (int h = 0; h < layers; ++h) {
      push(h, chain ? PH_PLACE : PH_SAMPLE);
      if ((insert_hops >> h) & 1u) push(h, PH_INSERT);
      push(h, PH_MARK);
      if ((scan_hops >> h) & 1u) push(h, PH_SCAN);
      push(h, PH_EMIT);
    }
  }
  bool open() const { return next_item < num_items || next_chain < num_chain; }
  int samples_issued() const {           // hops whose sample phase has been issued
    int n = 0;
    for (int i = 0; i < next_item; ++i) n += item_phase[i] == PH_SAMPLE;
    return n;
  }
  // every phase of the step that reads or writes a cache table has been issued
  bool table_work_issued() const { return num_chain ? next_chain == num_chain : samples_issued() == L; }
};

// A phase chosen for a launch: item >= 0 is an index into the step's list, item < 0 stands for chain phase -1 - item.
struct TickPick { int step, item; };

// One tick: of the steps in flight (oldest first) pick the phases that may run now; they go to `take` (at most two
// per step: a chain phase and a list phase), their number is returned.  Stream order between ticks is the only
// synchronisation, so a phase may only depend on phases issued in EARLIER ticks.  Within a step that holds by
// construction: one list phase and one chain phase per tick, and the place phase of hop h waits until chain phase h
// has been issued in an earlier tick.  Across steps only the phases that touch the cache tables matter (sample
// phases; chain phases):
//   otf && !shared  hop h of every step updates the same per-layer table: the sample phase of (t, h)
//                   needs that of (t-1, h) issued earlier (steps of different depth never overlap);
//   otf && shared   one table serves all hops: every such phase of step t-1 must have been issued;
//   otherwise       the tables are read-only between refreshes (or absent): no dependency.
// The oldest step with phases left is always ready - its chain phase, if it has any left, else (no other chain phase
// can be in the way then, unless a younger step's, which ends within a few ticks) its list phase -, so ticks always
// make progress.
inline int plan_tick(const StepItems* const* steps, int n, bool otf, bool shared, TickPick* take) {
  // first pass: the chain phase of this tick, if any (at most one: chains of consecutive steps never overlap)
  int chain_step = -1, chain_hop = -1;
  {
    const StepItems* prev = nullptr;
    for (int i = 0; i < n && chain_step < 0; ++i) {
      const StepItems& st = *steps[i];
      if (st.next_chain < st.num_chain && (!(otf && prev && prev->open()) || prev->table_work_issued())) {
        chain_step = i; chain_hop = st.next_chain;
      }
      prev = &st;
    }
  }
  int m = 0;
  const StepItems* prev = nullptr;       // the step before (its progress as of the end of the last tick)
  for (int i = 0; i < n; ++i) {
    const StepItems& st = *steps[i];
    const bool prev_busy = otf && prev && prev->open();
    if (i == chain_step) take[m++] = TickPick{i, -1 - st.next_chain};
    if (st.next_item < st.num_items) {
      const int ph = st.item_phase[st.next_item], hop = st.item_hop[st.next_item];
      bool ready = true;
      if (ph == PH_PLACE) {
        // its own chain phase must have been issued; and the place phases of the outer hops - the heaviest of the
        // list: they enter every pick into the dedupe table - wait for a launch whose chain phase is the light one of
        // hop 0 (or that has none), so that the launches of a full pipeline come out even
        ready = st.next_chain > hop && (hop == 0 || chain_hop <= 0);
      } else if (ph == PH_SAMPLE && prev_busy) {
        ready = shared ? prev->table_work_issued() : (prev->L == st.L && prev->samples_issued() > hop);
      }
      if (ready) take[m++] = TickPick{i, st.next_item};
    }
    prev = &st;
  }
  return m;
}

}  // namespace gss
