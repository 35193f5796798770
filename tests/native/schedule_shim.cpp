// Test shim: exposes the tick planner (host-only logic of the step pipeline) to ctypes.
#include "gss_schedule.h"

extern "C" {

// Phases of a step with `layers` hops; returns their number.
int sched_items(int layers, unsigned scan_hops, unsigned insert_hops, int chain, signed char* hop, signed char* phase) {
  gss::StepItems it;
  it.build(layers, scan_hops, insert_hops, chain != 0);
  for (int i = 0; i < it.num_items; ++i) { hop[i] = it.item_hop[i]; phase[i] = it.item_phase[i]; }
  return it.num_items;
}

// One tick over n steps in flight (oldest first), step i having `layers[i]` hops, `next_item[i]` list phases and
// `next_chain[i]` chain phases issued.  take_step / take_item receive the chosen phases (item < 0: chain phase -1 - item).
int sched_plan(const int* layers, const unsigned* scan_hops, const unsigned* insert_hops, const int* chain,
               const int* next_item, const int* next_chain, int n, int otf, int shared, int* take_step, int* take_item) {
  gss::StepItems items[64];
  const gss::StepItems* ptr[64];
  gss::TickPick picks[128];
  if (n > 64) return -1;
  for (int i = 0; i < n; ++i) {
    items[i].build(layers[i], scan_hops[i], insert_hops[i], chain[i] != 0);
    items[i].next_item = next_item[i];
    items[i].next_chain = next_chain[i];
    ptr[i] = &items[i];
  }
  const int m = gss::plan_tick(ptr, n, otf != 0, shared != 0, picks);
  for (int j = 0; j < m; ++j) { take_step[j] = picks[j].step; take_item[j] = picks[j].item; }
  return m;
}

}  // extern "C"
