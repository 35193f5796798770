// C ABI and host step driver of the sampler (see include/gss.h for the contract).
//
// The driver never waits for the device inside a step: frontier sizes live in device memory
// (`state`), launches are sized by host-known upper bounds with early exit, and the counts plus the
// error flag arrive in pinned host memory, written by the step's last kernel.
//
// A step is a chain of phases - per hop: sample, (insert,) mark, (scan,) emit - each a latency-bound pass
// that leaves most of the chip idle.  So the steps in flight (up to gss_pipeline_depth(), each in its own
// "slot": device state, scratch, dedupe table, output buffers) are software-pipelined through ONE launch
// per enqueued step, a "tick": the tick carries the next phase of every step in flight that
// may run now, one slice of the grid each.  Stream order between ticks gives every dependency:
//   - a step's own phases follow each other, one per tick;
//   - OTF: hop h of every step touches the same per-layer table, so the sample phase of (t, h) goes
//     into a tick only after the sample phase of (t-1, h) went into an EARLIER one;
//   - SHARED_OTF: one table serves all hops, so a step's first sample phase waits until every sample
//     phase of the step before has been issued;
//   - the other modes: steps do not depend on each other.  A refresh of FCR / OTF_LAYER fills a set of
//     tables that is not in use (there are up to five), so steps of the old epoch still in flight go on
//     reading theirs.
// A step with P phases is complete P ticks after it was enqueued; gss_step_wait issues the
// missing ticks itself when fewer steps follow.  Host cost per step: one launch, which also completes the
// finished step's event.
#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "gss_device.h"

using namespace gss;

namespace {
constexpr uint32_t VERSION_FIRST = 1u, VERSION_LAST = 0xFFFFFFF0u;
constexpr int MAX_TABLE_SETS = 5;
constexpr int TICK_EVENTS = 2 * GSS_MAX_IN_FLIGHT;   // more than the steps that can be finished and not yet collected
constexpr int64_t SAMPLE_WIDE_GROUPS = 4096;      // expected frontier nodes of a hop from which a sample group takes two nodes (several relations)
constexpr int64_t INSERT_SPLIT_SLOTS = 48 * 1024;   // expected pick slots of a hop from which its inserts get their own phase
constexpr int64_t TWO_STEP_PICKS = 400 * 1024;    // expected picks of a step up to which two steps share a tick
constexpr int64_t NARROW_MIN_NODES = 16 * 1024;     // expected frontier nodes of a launch's sample slices from which they take narrow groups
constexpr int64_t INSERT_SMALL_SLOTS = 16 * 1024;   // ... and up to which they do, too (narrow hops)
constexpr int DENSE_TICK_WGS = 5000;                // workgroups of a launch from which the kernel's eight-per-CU build is used
static_assert(GSS_MAX_LAYERS <= SCHED_MAX_LAYERS, "the phase list of a step holds GSS_MAX_LAYERS hops");

struct Buf {
  void* p = nullptr;
  size_t bytes = 0;
};

// Start / stop events attached to kernel launches; events are pooled and reused after each read.
struct EventTimer : LaunchTimer {
  struct Bracket { int kid; hipEvent_t a, b; };
  std::vector<Bracket> open_;
  std::vector<hipEvent_t> pool_;
  double ms[KID_COUNT] = {};
  int64_t launches[KID_COUNT] = {};
  hipEvent_t get() {
    if (!pool_.empty()) { hipEvent_t e = pool_.back(); pool_.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
  }
  bool bracket(int kid, hipEvent_t* start, hipEvent_t* stop) override {
    hipEvent_t a = get(), b = get();
    if (!a || !b) { if (a) pool_.push_back(a); if (b) pool_.push_back(b); return false; }
    open_.push_back({kid, a, b});
    *start = a; *stop = b;
    return true;
  }
  void collect() {   // the streams must be idle
    for (const Bracket& br : open_) {
      float t = 0.f;
      if (hipEventElapsedTime(&t, br.a, br.b) == hipSuccess) { ms[br.kid] += (double)t; ++launches[br.kid]; }
      else (void)hipGetLastError();
      pool_.push_back(br.a); pool_.push_back(br.b);
    }
    open_.clear();
  }
  void reset() { collect(); for (int i = 0; i < KID_COUNT; ++i) { ms[i] = 0; launches[i] = 0; } }
  ~EventTimer() override { collect(); for (hipEvent_t e : pool_) (void)hipEventDestroy(e); }
};

// Everything one step in flight owns.
struct Slot {
  int32_t* state_d = nullptr;
  int32_t* state_h = nullptr;            // pinned copy of the device state, written by the last emit phase
  int32_t* state_h_dev = nullptr;        // the same memory as the device sees it
  Buf hash, direct, picks, order, ranks, partial_first, partial_edge, first_off, edge_off;
  Buf visit, held, list, counts;         // visit-once steps: visit table (8 bytes per node), holding area, node lists and their counters
  int chain_parity = 0;                  // which of the two counter sets the slot's next visit-once step uses
  uint32_t ver = VERSION_FIRST;          // next unused dedupe table version
  Buf src_nodes[GSS_MAX_LAYERS][GSS_MAX_NODE_TYPES];
  Buf src_local[GSS_MAX_LAYERS][GSS_MAX_RELATIONS], dst_local[GSS_MAX_LAYERS][GSS_MAX_RELATIONS];
  hipEvent_t done = nullptr;             // completes when the step's last phase has run (the event of that tick, borrowed)
  bool pending = false;                  // enqueued and not yet collected
  bool used = false;                     // has held a step: its output buffers may still be read by the caller
  int L = 0, num_seeds = 0, seed_type = 0;
  // plan of the step the slot holds (host-known upper bounds of every hop)
  const int32_t* seeds = nullptr;
  int64_t step = 0;
  int32_t fanouts[GSS_MAX_LAYERS] = {};
  int64_t fub[GSS_MAX_LAYERS + 1][GSS_MAX_NODE_TYPES] = {};
  int64_t slots_ub[GSS_MAX_LAYERS][GSS_MAX_RELATIONS] = {};
  int64_t slot_base[GSS_MAX_LAYERS][GSS_MAX_RELATIONS] = {};
  int64_t total_slots[GSS_MAX_LAYERS] = {};
  uint64_t hash_cap = 0;
  bool refresh_now = false;
  uint32_t ver0 = 0;                     // dedupe table version of hop 0 (hop h uses ver0 + h)
  int table_set = 0;                     // FCR: the set of tables the step reads
  StepItems items;                       // the step's phases in order, and how many of them have been put into a tick
  uint32_t insert_hops = 0;              // hops whose dedupe table inserts run as a phase of their own
  bool chain = false;                    // a visit-once step (chain phases + place / mark / emit)
  ChainArgs chain_args;                  // ... and what its chain phases share
  std::vector<gss_block_nodes> out_nodes;
  std::vector<gss_block_edges> out_edges;
};
}  // namespace

struct gss_sampler {
  int T = 0, R = 0, L = 0, k = 0, S = 0, n_new = 0, period = 1, num_tables = 0;
  gss_mode mode = GSS_MODE_FCR;
  double fetch_fraction = 0.0;           // OTF_FETCH: delta
  uint64_t seed = 0;
  hipStream_t stream = nullptr;          // the caller's stream
  hipEvent_t user_ready = nullptr;       // recorded on the caller's stream when it has work pending at enqueue
  hipStream_t work = nullptr;            // internal, non-blocking: every tick runs here
  gss_alloc_fn alloc = nullptr;
  gss_free_fn free_fn = nullptr;
  void* alloc_ctx = nullptr;
  int64_t num_nodes[GSS_MAX_NODE_TYPES] = {};
  int64_t total_nodes = 0;
  uint32_t key_off[GSS_MAX_NODE_TYPES] = {};
  gss_relation rel[GSS_MAX_RELATIONS] = {};
  // FCR keeps up to MAX_TABLE_SETS sets of tables (the other modes one).  A refresh fills the set after the
  // current one, so the steps of the old epoch that are still in flight go on reading theirs and nothing
  // has to drain.  The rows of the next epoch are a pure function of (seed, epoch): they are computed
  // ahead of time, on a stream of their own, as soon as no step in flight reads that set any more - with
  // three sets or more that is right at the start of an epoch (the stragglers of the previous epochs read the
  // other sets), with two sets only once those have issued all their phases.
  int32_t* table[MAX_TABLE_SETS][GSS_MAX_LAYERS][GSS_MAX_RELATIONS] = {};
  int nsets = 1;
  int cur_set = 0;                       // the set that holds the current epoch
  hipStream_t fill_stream = nullptr;
  hipEvent_t fill_go = nullptr, fill_done = nullptr;
  int64_t prefetched_epoch = -1;         // epoch whose rows are (being) written into the idle set; -1: none
  long long* stamp[GSS_MAX_RELATIONS] = {};
  int32_t theta = -1;                    // degree split: nodes with deg <= theta keep no cache row (< 0: no split)
  int32_t* row_of[GSS_MAX_RELATIONS] = {};   // degree split: node -> table row or -1
  int64_t table_rows[GSS_MAX_RELATIONS] = {};  // rows of every table of the relation
  // Epoch-refreshed modes: the nodes with a row and more than k neighbors, per relation.  The other rows hold the
  // whole adjacency and never change: once a set of tables has been filled, a refresh recomputes the listed rows only.
  int32_t* heavy_list[GSS_MAX_RELATIONS] = {};
  int64_t num_heavy[GSS_MAX_RELATIONS] = {};
  bool heavy_ready = false;
  bool set_filled[MAX_TABLE_SETS] = {};
  int64_t cache_bytes = 0;               // tables + row maps + stamps
  int32_t* state_d = nullptr;            // create-time state (graph validation, initial fill)
  int32_t* state_h = nullptr;
  int32_t* fill_state_d = nullptr;       // error flag of the refreshes computed ahead of time on the fill stream, and its
  int32_t* fill_state_h = nullptr;       // pinned host copy (copied after every such refresh, checked when its epoch starts)
  int state_words = 0;
  Buf checksum;
  bool use_direct = true;
  bool shared = false;                   // one table serves all layers (SHARED_OTF, SHARED_FCR)
  bool fcr = false;                      // every table is rewritten when floor(step/R) changes (FCR, SHARED_FCR, OTF_LAYER)
  bool layer_partial = false;            // ... by a partial refresh of every row instead of a fill (OTF_LAYER)
  bool otf = false;                      // partial refresh per visit (OTF, SHARED_OTF)
  bool force_scan_kernel = false;        // gss_tuning.scan_phase: always use the separate scan phase
  int insert_policy = 0;                 // gss_tuning.insert_phase - 0: large and narrow hops get an insert phase; 1: all hops, 2: none
  int dense_policy = 0;                  // gss_tuning.tick_build - 0: launches of DENSE_TICK_WGS workgroups and more use the dense build; 1: all, 2: none
  uint32_t first_version = VERSION_FIRST;   // where a slot's dedupe-table version counter starts
  int tick_cap = 1;                      // slices one launch can carry
  int group_w = 32;                      // lanes per frontier node in the sample phase: 64 or 32 ...
  int narrow_w = 0;                      // ... or, in launches whose sample slices expect many nodes, 21 or 16 (0: never)
  bool narrow_always = false;            // gss_tuning.group_width = 1: in every launch
  bool lds_stage = false;                // gss_tuning.lds_dedupe: the per-tile LDS stage of the dedupe
  int chain_wg_cap = 4096;               // most workgroups of a chain slice, which stride over the rest (the 4,096-seed workload: 2,048 +5 %, 8,192 +5 %)
  bool visit_once_forced = false;        // gss_tuning.visit_once == 1: also the steps of blocking calls
  bool blocking_call = false;            // inside gss_step
  bool visit_once = false;               // steps run as visit-once steps where their size allows (SHARED_OTF on one relation)
  RelConst relc_h[GSS_MAX_RELATIONS] = {};   // per relation constants: host copy and device copy
  RelConst* relc_d = nullptr;
  SlotConst slotc_h[GSS_MAX_IN_FLIGHT] = {};   // per slot: the scratch pointers all phases of its step share; host copy and
  SlotConst* slotc_d = nullptr;               // device table (read by the compact launches of one-relation graphs)
  // Frontier sizes are only known on the device, and the host-known upper bounds are loose (every pick
  // a new node): hop h of recent steps filled this share of its bound.  Grids are sized by it; the
  // kernels stride over whatever the frontier turns out to be, so a wrong guess only costs time.
  float fill_ratio[GSS_MAX_LAYERS];
  Slot slot[GSS_MAX_IN_FLIGHT];
  HopParams tick_all[2 * GSS_MAX_IN_FLIGHT], tick_launch[TICK_MAX_SLICES];   // scratch of tick(): slices of a tick, and of one launch
  hipEvent_t tick_ev[TICK_EVENTS] = {};  // completion events of the ticks in which steps finish, used round-robin
  int tick_ev_next = 0;
  int steps_per_tick = 1, unlaunched = 0; // steps enqueued since the last tick
  int ring = GSS_MAX_IN_FLIGHT;          // slots in use, round-robin: the most steps that may be in flight
  int enq = 0;                           // slot the next enqueue uses
  int64_t epoch = 0, last_step = -1;
  bool poisoned = false;
  EventTimer* timer = nullptr;           // non-null while profiling is enabled
  char err[256] = {0};
};

namespace {

// Why the last gss_create of this thread failed (gss_last_error(NULL) returns it): there is no handle to ask then.
thread_local char g_create_err[256] = {0};

gss_status fail(gss_sampler* s, gss_status st, const char* fmt, ...) {
  if (s) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(s->err, sizeof s->err, fmt, ap);
    va_end(ap);
  }
  return st;
}

void* dev_alloc(gss_sampler* s, size_t bytes) {
  if (bytes == 0) bytes = 16;
  if (s->alloc) return s->alloc(s->alloc_ctx, bytes);
  void* p = nullptr;
  if (hipMalloc(&p, bytes) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
  return p;
}
void dev_free(gss_sampler* s, void* p) {
  if (!p) return;
  if (s->alloc) s->free_fn(s->alloc_ctx, p); else (void)hipFree(p);
}
// grow-only buffer; contents are not preserved.  Only called for a slot whose previous step has
// been collected, so nothing in flight reads the buffer that is released.
// When the allocation fails the buffer stays as it was.
bool ensure(gss_sampler* s, Buf& b, size_t bytes) {
  if (b.bytes >= bytes && b.p) return true;
  bytes = std::max<size_t>(bytes, 16);
  void* p = dev_alloc(s, bytes);
  if (!p) return false;
  dev_free(s, b.p);
  b.p = p;
  b.bytes = bytes;                       // (what was asked of the allocator, never more)
  return true;
}
void release(gss_sampler* s, Buf& b) { dev_free(s, b.p); b.p = nullptr; b.bytes = 0; }

#define HIP_TRY(s, call)                                                                      \
  do {                                                                                        \
    hipError_t e_ = (call);                                                                   \
    if (e_ != hipSuccess) return fail(s, GSS_ERR_DEVICE, "%s: %s", #call, hipGetErrorString(e_)); \
  } while (0)

int row_stride(int k) { return k <= 16 ? 16 : k <= 32 ? 32 : 64; }

int32_t n_new_of(double fraction, int k) {
  double x = fraction * (double)k + 1e-9;
  if (x < 0.0) return 0;
  int64_t n = (int64_t)x;
  return (int32_t)std::min<int64_t>(n, k);
}

// Fills the tables of `set`: FILL_FULL of every row (src_set < 0), or - OTF_LAYER - the rows of `src_set` with
// n_new slots redrawn (the two sets may be the same one).
gss_status fill_all_tables(gss_sampler* s, uint32_t stepword, int32_t* state_d, hipStream_t st, int set = 0, int src_set = -1) {
  if (s->num_tables == 0) return GSS_OK;   // FBL keeps no cache
  for (int r = 0; r < s->R; ++r) {
    FillParams P{};
    P.indptr = s->rel[r].indptr;
    P.indices = s->rel[r].indices;
    P.ntab = s->num_tables;
    for (int t = 0; t < s->num_tables; ++t) {
      P.table[t] = s->table[set][t][r];
      P.src_table[t] = (src_set >= 0 && s->layer_partial) ? s->table[src_set][t][r] : nullptr;
      P.layer_word[t] = s->shared ? 0xFFu : (uint32_t)t;
    }
    P.state = state_d;
    P.row_of = s->row_of[r];
    P.n_dst = s->num_nodes[s->rel[r].dst_type];
    P.is64 = s->rel[r].indptr_is_64;
    P.k = s->k;
    P.S = s->S;
    P.n_new = s->n_new;
    P.relation = (uint32_t)r;
    P.stepword = stepword;
    P.seed_lo = (uint32_t)(s->seed & 0xffffffffu);
    P.seed_hi = (uint32_t)(s->seed >> 32);
    if (P.n_dst <= 0) continue;
    if (s->heavy_ready && s->set_filled[set]) HIP_TRY(s, launch_fill_heavy(P, s->heavy_list[r], s->num_heavy[r], st, s->timer));
    else HIP_TRY(s, launch_fill_full(P, st, s->timer));
  }
  s->set_filled[set] = true;
  return GSS_OK;
}

gss_status read_create_state(gss_sampler* s) {
  HIP_TRY(s, hipMemcpyAsync(s->state_h, s->state_d, sizeof(int32_t) * (size_t)s->state_words, hipMemcpyDeviceToHost, s->stream));
  HIP_TRY(s, hipStreamSynchronize(s->stream));
  return GSS_OK;
}

gss_status sync_all(gss_sampler* s) {
  if (s->fill_stream) HIP_TRY(s, hipStreamSynchronize(s->fill_stream));
  if (s->work) HIP_TRY(s, hipStreamSynchronize(s->work));
  HIP_TRY(s, hipStreamSynchronize(s->stream));
  return GSS_OK;
}

// The oldest step in flight: slots are used round-robin, so it is the first pending one from `enq` on.
Slot* oldest_pending(gss_sampler* s) {
  for (int n = 0; n < s->ring; ++n) {
    Slot& sl = s->slot[(s->enq + n) % s->ring];
    if (sl.pending) return &sl;
  }
  return nullptr;
}

bool scans_in_emit(const gss_sampler* s, const Slot& sl, int h) {
  return sl.total_slots[h] / TILE <= EMIT_SCAN_MAX_TILES && !s->force_scan_kernel;
}

// The scratch pointers that all phases of the step held by `sl` share.
SlotConst slot_const(const gss_sampler* s, const Slot& sl) {
  SlotConst c;
  memset(static_cast<void*>(&c), 0, sizeof c);
  c.ht.direct = s->use_direct ? (uint64_t*)sl.direct.p : nullptr;
  c.ht.entries = (HashEntry*)sl.hash.p;
  c.ht.mask = sl.hash_cap ? sl.hash_cap - 1 : 0;
  c.state = sl.state_d;
  c.state_host = sl.state_h_dev;
  c.picks = (int32_t*)sl.picks.p; c.order = (uint32_t*)sl.order.p; c.ranks = (uint32_t*)sl.ranks.p;
  c.partial_first = (int32_t*)sl.partial_first.p; c.partial_edge = (int32_t*)sl.partial_edge.p;
  c.first_off = (int32_t*)sl.first_off.p; c.edge_off = (int32_t*)sl.edge_off.p;
  return c;
}

// Kernel arguments of item `it` (one phase of one hop) of the step held by `sl`.
void fill_slice(gss_sampler* s, Slot& sl, int it, HopParams& P, int width) {
  const int T = s->T, R = s->R, L = sl.L, h = sl.items.item_hop[it], l = L - 1 - h;
  memset(static_cast<void*>(&P), 0, sizeof P);
  P.phase = sl.items.item_phase[it];
  P.R = R; P.T = T; P.hop = h; P.f = sl.fanouts[l]; P.k = s->k; P.S = s->S;
  P.n_new = (s->mode == GSS_MODE_OTF_FETCH) ? n_new_of(s->fetch_fraction, P.f) : s->n_new;   // OTF_FETCH: per draw
  P.mode = (int)s->mode; P.refresh_now = sl.refresh_now ? 1 : 0;
  P.band_offset = 0;
  for (int q = 0; q < l; ++q) P.band_offset += sl.fanouts[q];
  P.num_tiles_ub = (int32_t)(sl.total_slots[h] / TILE);
  P.scan_in_emit = scans_in_emit(s, sl, h) ? 1 : 0;
  // bit 0: the hop has an insert phase; bit 1: insert and place phases dedupe their tile in LDS first
  P.insert_split = (int32_t)((sl.insert_hops >> h) & 1u) | (s->lds_stage ? 2 : 0);
  P.edge_count_off = (GSS_MAX_LAYERS + 1) * T;
  P.ver = sl.ver0 + (uint32_t)h;
  P.step = (uint32_t)sl.step;
  P.layer_word = s->shared ? 0xFFu : (uint32_t)l;
  P.shared = s->shared ? 1 : 0;
  P.layer = l;
  P.seed_lo = (uint32_t)(s->seed & 0xffffffffu);
  P.seed_hi = (uint32_t)(s->seed >> 32);
  const SlotConst sc = slot_const(s, sl);
  P.ht = sc.ht;
  P.state = sc.state;
  P.state_host = (h == L - 1) ? sc.state_host : nullptr;
  P.state_words = s->state_words;
  P.picks = sc.picks; P.order = sc.order; P.ranks = sc.ranks;
  P.partial_first = sc.partial_first; P.partial_edge = sc.partial_edge;
  P.first_off = sc.first_off; P.edge_off = sc.edge_off;
  P.slot = (int32_t)(&sl - s->slot);
  if (sl.chain) {               // visit-once step: the place phase reads the hop's picks from the holding area
    if (P.phase == PH_PLACE) {
      P.visit = (const uint64_t*)sl.visit.p;
      P.held = (const int32_t*)sl.held.p + sl.chain_args.off[h];
    }
  }
  int64_t max_f = 1;
  for (int t = 0; t < T; ++t) {
    TypeParam& tp = P.type[t];
    tp.frontier = (h == 0) ? (t == sl.seed_type ? sl.seeds : nullptr) : (const int32_t*)sl.src_nodes[l + 1][t].p;
    tp.src_nodes = (int32_t*)sl.src_nodes[l][t].p;
    tp.key_off = s->key_off[t];
    tp.n_nodes = (int32_t)s->num_nodes[t];
    tp.count_override = (h == 0) ? (t == sl.seed_type ? sl.num_seeds : 0) : -1;
    tp.frontier_cap = (int32_t)((h == 0) ? (t == sl.seed_type ? sl.num_seeds : 0) : sl.fub[h][t]);
    max_f = std::max(max_f, sl.fub[h][t]);
  }
  for (int r = 0; r < R; ++r) {
    RelParam& rp = P.rel[r];
    rp.table = s->num_tables ? s->table[sl.table_set][s->shared ? 0 : l][r] : nullptr;
    rp.src_local = (int32_t*)sl.src_local[l][r].p; rp.dst_local = (int32_t*)sl.dst_local[l][r].p;
    rp.src_type = (int16_t)s->rel[r].src_type; rp.dst_type = (int16_t)s->rel[r].dst_type;
    rp.slot_base = (int32_t)sl.slot_base[h][r];
  }
  // grid of the slice: sample - one 32-lane group per frontier node, 8 groups per workgroup, y = relation
  // or node type; mark / emit - one workgroup per 1024-slot tile; scan - one workgroup
  // Sized by the expected frontier (workgroups that find no work still occupy a slot for a microsecond,
  // and the slots are what the long-running sample workgroups of the same launch leave free).
  const double expect = std::min(1.0, 1.1 * (double)s->fill_ratio[h]);   // (10 % of slack: 25 % cost the typed workload 1 %)
  if (P.phase == PH_SAMPLE) {
    const int64_t groups = (int64_t)(expect * (double)max_f) + 8;
    // (on graphs with several relations a wide slice gives every group two nodes: most (node, relation) pairs of a
    // typed graph are empty rows, a workgroup spends about a microsecond before its first node, and half as many
    // workgroups ask for a slot - the seven-relation workload -7 %; with one relation every node is real work and one
    // node per group is the shorter chain: the 2.45M-node workloads -2 % - unless a tick starts two steps (FBL, OTF
    // fetch): its launches are as crowded as a typed graph's, and two nodes per group are 6-8 % faster there)
    const int64_t want = std::min(groups, max_f);
    const int64_t per = ((R > 1 || s->steps_per_tick == 2) && want > SAMPLE_WIDE_GROUPS) ? 2 : 1;
    // (at most 2,048 workgroups, which then stride over the frontier: more of them crowd out the other slices of a
    // full tick - 16,384-seed steps +9 % with 8,192.  The shared-table refresh mode runs its sample phases nearly
    // alone, one step after the other: there 8,192 are 1.5 % faster)
    const int64_t cap = (s->otf && s->shared) ? 8192 : 2048;
    const int64_t gpw = 4 * (64 / width);        // groups of a workgroup (four wavefronts): 64 / 32 / 21 / 16 lanes per node
    P.gx = (int32_t)std::min<int64_t>(std::max<int64_t>((want + gpw * per - 1) / (gpw * per), 1), cap);
    P.gy = R;                                    // per relation: a group per frontier node
    P.gxd = (int32_t)((P.gx * gpw + 255) / 256); P.gyd = T;   // per node type: a thread per frontier node
  } else if (P.phase == PH_SCAN) {
    P.gx = 1; P.gy = 1;
  } else {                                     // insert, place, mark, emit: tiles
    const int64_t tiles = (int64_t)(expect * (double)P.num_tiles_ub) + R;
    // (one workgroup per expected live tile, also on very large hops: with a cap of 1,024 workgroups, each walking
    // over several tiles, steps of 65,536 seeds were 7 % slower, of 262,144 seeds 11 %.  On graphs with several
    // relations, whose ticks are crowded with the rows of the sample slices, the cap stays: the seven-relation
    // workload is 2 % faster with it)
    const int64_t tile_cap = R > 1 ? 1024 : 16384;
    int64_t gx = std::min<int64_t>(std::max<int64_t>(std::min<int64_t>(tiles, P.num_tiles_ub), 1), tile_cap);
    // an emit workgroup that scans in LDS keeps the edge offsets of its own tiles there
    if (P.scan_in_emit) gx = std::max<int64_t>(gx, (P.num_tiles_ub + EMIT_OWN_TILES - 1) / EMIT_OWN_TILES);
    P.gx = (int32_t)gx;
    P.gy = 1;
    if (P.phase == PH_PLACE) {                 // ... and a row of workgroups with a thread per dst node
      const int64_t nodes = std::min<int64_t>((int64_t)(expect * (double)max_f) + 8, max_f);
      P.gxd = (int32_t)std::max<int64_t>((nodes + 255) / 256, 1);
      P.gyd = 1;
    }
  }
}

// Kernel arguments of chain phase c of the visit-once step held by `sl`.
void fill_chain_slice(gss_sampler* s, Slot& sl, int c, HopParams& P) {
  memset(static_cast<void*>(&P), 0, sizeof P);
  const ChainArgs& C = sl.chain_args;
  P.phase = PH_CHAIN;
  P.R = 1; P.T = 1; P.hop = c; P.f = C.f(c); P.k = s->k; P.S = s->S;
  P.n_new = s->n_new; P.mode = (int)s->mode; P.refresh_now = sl.refresh_now ? 1 : 0;
  P.step = (uint32_t)sl.step;
  P.layer_word = 0xFFu; P.shared = 1; P.layer = sl.L - 1 - c;
  P.seed_lo = (uint32_t)(s->seed & 0xffffffffu);
  P.seed_hi = (uint32_t)(s->seed >> 32);
  P.state = sl.state_d;
  P.state_words = s->state_words;
  P.slot = (int32_t)(&sl - s->slot);
  P.ver = sl.ver0 + (uint32_t)c;
  P.type[0].frontier = sl.seeds;
  P.type[0].key_off = s->key_off[0];
  P.type[0].n_nodes = (int32_t)s->num_nodes[0];
  P.type[0].count_override = sl.num_seeds;
  P.type[0].frontier_cap = sl.num_seeds;
  P.rel[0].table = s->table[sl.table_set][0][0];
  // one 32-lane group per node of hop c's frontier (sized by what recent steps filled of the host-known bound), eight
  // groups per workgroup, which stride over the rest
  int64_t groups = sl.num_seeds;
  if (c > 0) groups = std::min<int64_t>((int64_t)(std::min(1.0, 1.1 * (double)s->fill_ratio[c]) * (double)sl.fub[c][0]) + 8, sl.fub[c][0]);
  P.gx = (int32_t)std::min<int64_t>(std::max<int64_t>((groups + 7) / 8, 1), s->chain_wg_cap);
  P.gy = 1;
}

// One tick: the next phase of every step in flight that may run now (oldest first), in as few launches
// as the slice capacity allows.  Only sample phases depend on other steps:
//   OTF         (t, h) after the sample phase of (t-1, h), issued in an EARLIER tick;
//   SHARED_OTF  after every sample phase of step t-1.
// Sets *issued to the number of phases put into the tick.
gss_status tick(gss_sampler* s, int* issued) {
  Slot* flight[GSS_MAX_IN_FLIGHT];
  const StepItems* items[GSS_MAX_IN_FLIGHT];
  int nf = 0;
  for (int q = 0; q < s->ring; ++q) {       // the steps in flight, oldest first
    Slot& sl = s->slot[(s->enq + q) % s->ring];
    if (sl.pending) { flight[nf] = &sl; items[nf++] = &sl.items; }
  }
  TickPick pick[2 * GSS_MAX_IN_FLIGHT];
  const int n = plan_tick(items, nf, s->otf, s->shared, pick);
  Slot* take[2 * GSS_MAX_IN_FLIGHT];
  for (int i = 0; i < n; ++i) take[i] = flight[pick[i].step];
  if (issued) *issued = n;
  // Workgroups start in grid order, and the chip holds about as many as a full tick has.  The slices with few
  // workgroups (mark / emit of the inner hops, the inner sample phases) are the long dependent chains that decide when
  // the launch ends; the widest sample slice is thousands of short-lived workgroups.  So the narrow slices go to the
  // front of the grid and start at once, and the wide ones fill in behind them (measured against widest-first:
  // a full tick of the 1,024-seed FCR workload 16.5 instead of 23.5 us, of the OTF ones 3-5 % less).
  HopParams* all = s->tick_all;          // (tens of KB: kept in the handle, not on the caller's stack)
  HopParams* P = s->tick_launch;
  int order[2 * GSS_MAX_IN_FLIGHT];
  const ChainArgs* chain = nullptr;      // of the tick's chain phase (chain phases of different steps never share a tick)
  // Lanes per frontier node, for all sample slices of the tick: the narrow groups (three or four nodes per wavefront)
  // where the launch has enough nodes for the vector instructions to be what bounds it; few nodes are bound by their
  // dependent chains, and fewer, longer-lived wavefronts only lengthen those (the 128-seed workload +4 %, the
  // 1,024-seed ones -2 .. 0 %, steps of 16,384 seeds and more -8 .. -10 %).
  int width = s->group_w;
  if (s->narrow_w) {
    double nodes = 0.0;
    for (int i = 0; i < n; ++i)
      if (pick[i].item >= 0 && take[i]->items.item_phase[pick[i].item] == PH_SAMPLE) {
        const int h = take[i]->items.item_hop[pick[i].item];
        double mf = 1.0;
        for (int t = 0; t < s->T; ++t) mf = std::max(mf, (double)take[i]->fub[h][t]);
        nodes += std::min(1.0, 1.1 * (double)s->fill_ratio[h]) * mf;
      }
    if (s->narrow_always || nodes >= (double)NARROW_MIN_NODES) width = s->narrow_w;
  }
  for (int i = 0; i < n; ++i) {
    if (pick[i].item >= 0) fill_slice(s, *take[i], pick[i].item, all[i], width);
    else { fill_chain_slice(s, *take[i], -1 - pick[i].item, all[i]); chain = &take[i]->chain_args; }
    order[i] = i;
  }
  auto weight = [&](int i) { return all[i].gx * all[i].gy + all[i].gxd * all[i].gyd; };
  // (a chain slice - the phase the next step waits for - leads the grid whatever its width: the 4,096-seed workload
  // with the shared table -8 % per step)
  auto rank_of = [&](int i) { return all[i].phase == PH_CHAIN ? -1 : weight(i); };
  std::sort(order, order + n, [&](int a, int b) { return rank_of(a) < rank_of(b); });
  // A step whose last phase (an emit phase, which writes its counts + error flag into pinned host memory) is in
  // this tick is done when the tick's last launch is: that launch completes the step's `done` event itself.
  // (Several steps may end with one tick: they share its event.)
  hipEvent_t done = nullptr;
  for (int i = 0; i < n; ++i)
    if (pick[i].item >= 0 && pick[i].item + 1 == take[i]->items.num_items) {
      if (!done) { done = s->tick_ev[s->tick_ev_next]; s->tick_ev_next = (s->tick_ev_next + 1) % TICK_EVENTS; }
      take[i]->done = done;
    }
  s->unlaunched = 0;
  for (int first = 0; first < n; first += s->tick_cap) {
    const int m = std::min(n - first, s->tick_cap);
    int wgs = 0;
    for (int i = 0; i < m; ++i) { P[i] = all[order[first + i]]; wgs += weight(order[first + i]); }
    const bool last = first + m == n;
    // (where the sample phase only reads rows and ranks them - the epoch-refreshed per-layer tables without a degree
    // split - the code whose scalar registers the dense build parks in vector lanes never runs: these take it at every
    // size, 1-4 % per step on the 1,024-seed workload; FBL and OTF fetch, which draw from the adjacency, lose 2-7 %)
    const bool rows_only = s->fcr && !s->shared && s->theta < 0;
    const bool dense = s->dense_policy == 1 || (s->dense_policy == 0 && (rows_only || wgs >= DENSE_TICK_WGS));
    hipError_t e = launch_tick(P, m, s->relc_h, s->relc_d, s->slotc_d, s->visit_once, chain, s->work, s->timer, last ? done : nullptr, dense, width);
    if (e != hipSuccess) { s->poisoned = true; return fail(s, GSS_ERR_DEVICE, "launch: %s", hipGetErrorString(e)); }
  }
  for (int i = 0; i < n; ++i) {
    if (pick[i].item >= 0) ++take[i]->items.next_item; else ++take[i]->items.next_chain;
  }
  return GSS_OK;
}

// Issue ticks until every step in flight has all its phases enqueued.
gss_status drain(gss_sampler* s) {
  for (;;) {
    bool open = false;
    for (const Slot& sl : s->slot) open |= sl.pending && sl.items.open();
    if (!open) return GSS_OK;
    int issued = 0;
    gss_status st = tick(s, &issued);
    if (st != GSS_OK) return st;
    // (the oldest step with phases left is always ready: the step before it has issued all of its own)
    if (issued == 0) { s->poisoned = true; return fail(s, GSS_ERR_DEVICE, "pipeline: no step is ready"); }
  }
}

// Rewrite the tables of `set` for the epoch that starts at step `stepword` on the fill stream: after everything
// the work stream has been given so far; the work stream waits for `fill_done` before it gets a step that reads
// the set.
gss_status fill_on_fill_stream(gss_sampler* s, uint32_t stepword, int set) {
  HIP_TRY(s, hipEventRecord(s->fill_go, s->work));
  HIP_TRY(s, hipStreamWaitEvent(s->fill_stream, s->fill_go, 0));
  gss_status rs = fill_all_tables(s, stepword, s->fill_state_d, s->fill_stream, set, s->cur_set);
  if (rs != GSS_OK) { s->poisoned = true; return rs; }
  HIP_TRY(s, hipMemcpyAsync(s->fill_state_h, s->fill_state_d, sizeof(int32_t), hipMemcpyDeviceToHost, s->fill_stream));
  HIP_TRY(s, hipEventRecord(s->fill_done, s->fill_stream));
  return GSS_OK;
}

// FCR: start computing the next epoch's rows into the idle set of tables once every step in flight
// that reads that set has all its phases enqueued (the event orders the fill after them).
gss_status maybe_prefetch_epoch(gss_sampler* s) {
  if (!s->fcr || s->nsets < 2 || s->prefetched_epoch >= 0 || (s->epoch + 1) * s->period >= (int64_t(1) << 32))
    return GSS_OK;
  const int idle = (s->cur_set + 1) % s->nsets;
  for (const Slot& o : s->slot)
    if (o.pending && o.table_set == idle && o.items.open()) return GSS_OK;
  gss_status rs = fill_on_fill_stream(s, (uint32_t)((s->epoch + 1) * s->period), idle);
  if (rs != GSS_OK) return rs;
  s->prefetched_epoch = s->epoch + 1;
  return GSS_OK;
}

void destroy_impl(gss_sampler* s) {
  if (!s) return;
  (void)sync_all(s);
  for (int t = 0; t < GSS_MAX_LAYERS; ++t)
    for (int r = 0; r < GSS_MAX_RELATIONS; ++r)
      for (int q = 0; q < MAX_TABLE_SETS; ++q) dev_free(s, s->table[q][t][r]);
  for (Slot& sl : s->slot) {
    for (int t = 0; t < GSS_MAX_LAYERS; ++t) {
      for (int r = 0; r < GSS_MAX_RELATIONS; ++r) { release(s, sl.src_local[t][r]); release(s, sl.dst_local[t][r]); }
      for (int q = 0; q < GSS_MAX_NODE_TYPES; ++q) release(s, sl.src_nodes[t][q]);
    }
    Buf* bufs[] = {&sl.hash, &sl.direct, &sl.picks, &sl.order, &sl.ranks, &sl.partial_first, &sl.partial_edge,
                   &sl.first_off, &sl.edge_off, &sl.visit, &sl.held, &sl.list, &sl.counts};
    for (Buf* b : bufs) release(s, *b);
    dev_free(s, sl.state_d);
    if (sl.state_h) (void)hipHostFree(sl.state_h);
  }
  dev_free(s, s->relc_d);
  dev_free(s, s->slotc_d);
  if (s->work) (void)hipStreamDestroy(s->work);
  if (s->fill_stream) (void)hipStreamDestroy(s->fill_stream);
  if (s->fill_go) (void)hipEventDestroy(s->fill_go);
  if (s->fill_done) (void)hipEventDestroy(s->fill_done);
  for (hipEvent_t ev : s->tick_ev) if (ev) (void)hipEventDestroy(ev);
  for (int r = 0; r < GSS_MAX_RELATIONS; ++r) { dev_free(s, s->stamp[r]); dev_free(s, s->row_of[r]); dev_free(s, s->heavy_list[r]); }
  dev_free(s, s->state_d);
  if (s->state_h) (void)hipHostFree(s->state_h);
  dev_free(s, s->fill_state_d);
  if (s->fill_state_h) (void)hipHostFree(s->fill_state_h);
  if (s->user_ready) (void)hipEventDestroy(s->user_ready);
  release(s, s->checksum);
  delete s->timer;
  delete s;
}

}  // namespace

extern "C" {

const char* gss_version(void) { return "gss 0.3 (gfx950)"; }

const char* gss_last_error(const gss_sampler* s) { return s ? s->err : g_create_err; }

gss_status gss_create(const gss_graph* g, const gss_config* c, gss_sampler** out) {
  return gss_create_tuned(g, c, nullptr, out);
}

gss_status gss_create_tuned(const gss_graph* g, const gss_config* c, const gss_tuning* tune, gss_sampler** out) {
  auto early = [](gss_status st, const char* what) { snprintf(g_create_err, sizeof g_create_err, "create: %s", what); return st; };
  if (!out) return early(GSS_ERR_INVALID_ARG, "invalid argument (out is NULL)");
  *out = nullptr;
  if (!g || !c || !g->num_nodes || !g->relations) return early(GSS_ERR_INVALID_ARG, "invalid argument");
  if (g->num_node_types < 1 || g->num_node_types > GSS_MAX_NODE_TYPES || g->num_relations < 1 ||
      g->num_relations > GSS_MAX_RELATIONS)
    return early(GSS_ERR_INVALID_ARG, "invalid argument");
  if (c->k < 1 || c->k > GSS_MAX_K || c->num_layers < 1 || c->num_layers > GSS_MAX_LAYERS) return early(GSS_ERR_INVALID_ARG, "invalid argument");
  if ((int)c->mode < (int)GSS_MODE_FCR || (int)c->mode > (int)GSS_MODE_OTF_LAYER) return early(GSS_ERR_INVALID_ARG, "invalid argument");
  const bool m_fcr = c->mode == GSS_MODE_FCR || c->mode == GSS_MODE_SHARED_FCR || c->mode == GSS_MODE_OTF_LAYER;
  const bool m_otf = c->mode == GSS_MODE_OTF || c->mode == GSS_MODE_SHARED_OTF;
  const bool m_shared = c->mode == GSS_MODE_SHARED_OTF || c->mode == GSS_MODE_SHARED_FCR;
  if (m_fcr && c->refresh_period < 1) return early(GSS_ERR_INVALID_ARG, "invalid argument");
  if ((m_otf || c->mode == GSS_MODE_OTF_FETCH || c->mode == GSS_MODE_OTF_LAYER) &&
      !(c->refresh_fraction >= 0.0 && c->refresh_fraction <= 1.0))
    return early(GSS_ERR_INVALID_ARG, "invalid argument");
  if ((c->alloc == nullptr) != (c->free == nullptr)) return early(GSS_ERR_INVALID_ARG, "invalid argument");
  gss_tuning tn;
  memset(&tn, 0, sizeof tn);
  if (tune) tn = *tune;
  if (tn.dedupe_layout < 0 || tn.dedupe_layout > 2 || tn.table_sets < 0 || tn.table_sets > MAX_TABLE_SETS ||
      tn.pipeline_depth < 0 || tn.pipeline_depth > GSS_MAX_IN_FLIGHT || tn.steps_per_tick < 0 || tn.steps_per_tick > 2 ||
      tn.insert_phase < 0 || tn.insert_phase > 2 || tn.scan_phase < 0 || tn.scan_phase > 1 || tn.tick_build < 0 ||
      tn.tick_build > 2 || tn.visit_once < 0 || tn.visit_once > 2 || tn.chain_workgroups < 0 || tn.chain_workgroups > 65536 || tn.lds_dedupe < 0 || tn.lds_dedupe > 1 || (tn.group_width != 0 && tn.group_width != 1 && tn.group_width != 32) || tn.first_dedupe_version >= VERSION_LAST)
    return early(GSS_ERR_INVALID_ARG, "invalid argument (tuning field out of range)");
  for (int32_t v : tn.reserved)
    if (v != 0) return early(GSS_ERR_INVALID_ARG, "invalid argument (tuning: reserved fields must be 0)");
  int64_t total_nodes = 0;
  for (int t = 0; t < g->num_node_types; ++t) {
    if (g->num_nodes[t] < 0 || g->num_nodes[t] >= (int64_t(1) << 31)) return early(GSS_ERR_INVALID_GRAPH, "invalid graph");
    total_nodes += g->num_nodes[t];
  }
  if (total_nodes >= (int64_t(1) << 32)) return early(GSS_ERR_INVALID_GRAPH, "invalid graph");   // (type, id) must fit a 32-bit key
  for (int r = 0; r < g->num_relations; ++r) {
    const gss_relation& q = g->relations[r];
    if (q.src_type < 0 || q.src_type >= g->num_node_types || q.dst_type < 0 || q.dst_type >= g->num_node_types ||
        !q.indptr || q.nnz < 0 || (q.nnz > 0 && !q.indices))
      return early(GSS_ERR_INVALID_GRAPH, "invalid graph");
    if (!q.indptr_is_64 && q.nnz >= (int64_t(1) << 31)) return early(GSS_ERR_INVALID_GRAPH, "invalid graph");
  }

  gss_sampler* s = new (std::nothrow) gss_sampler();
  if (!s) return early(GSS_ERR_OOM, "out of host memory");
  s->T = g->num_node_types; s->R = g->num_relations; s->L = c->num_layers; s->k = c->k; s->S = row_stride(c->k);
  s->mode = c->mode;
  s->fcr = m_fcr; s->otf = m_otf; s->shared = m_shared;
  s->layer_partial = c->mode == GSS_MODE_OTF_LAYER;
  s->n_new = (m_otf || s->layer_partial) ? n_new_of(c->refresh_fraction, c->k) : 0;
  s->fetch_fraction = (c->mode == GSS_MODE_OTF_FETCH) ? c->refresh_fraction : 0.0;
  s->period = c->refresh_period >= 1 ? c->refresh_period : 1;
  s->num_tables = (c->mode == GSS_MODE_FBL) ? 0 : (m_shared ? 1 : c->num_layers);
  s->seed = c->rng_seed;
  s->theta = (c->mode == GSS_MODE_FBL) ? -1 : c->degree_threshold;
  s->stream = (hipStream_t)c->hip_stream;
  s->alloc = c->alloc; s->free_fn = c->free; s->alloc_ctx = c->alloc_ctx;
  s->total_nodes = total_nodes;
  uint32_t off = 0;
  for (int t = 0; t < s->T; ++t) { s->num_nodes[t] = g->num_nodes[t]; s->key_off[t] = off; off += (uint32_t)g->num_nodes[t]; }
  for (int r = 0; r < s->R; ++r) s->rel[r] = g->relations[r];

  g_create_err[0] = 0;
  // (the message of the failing call, if it left one on the handle, else the status name)
  auto bail = [&](gss_status st) {
    static const char* const names[] = {"ok", "invalid argument", "invalid graph", "invalid seed", "allocation failed",
                                        "device error", "step order"};
    snprintf(g_create_err, sizeof g_create_err, "create: %s", s->err[0] ? s->err : names[(int)st]);
    destroy_impl(s);
    return st;
  };
  auto hipfail = [&](hipError_t err) {
    if (!s->err[0]) snprintf(s->err, sizeof s->err, "%s", hipGetErrorString(err));
    return bail(GSS_ERR_DEVICE);
  };

  s->force_scan_kernel = tn.scan_phase == 1;
  s->insert_policy = tn.insert_phase;
  s->dense_policy = tn.tick_build;
  s->first_version = tn.first_dedupe_version ? tn.first_dedupe_version : VERSION_FIRST;
  s->tick_cap = tick_capacity(s->R, s->T);
  // One table for all hops and a refresh per visit: the steps run as visit-once steps (chain phases) where the graph
  // has one relation; all its launches use the build of the step kernel that holds the chain's code and arguments.
  s->visit_once = c->mode == GSS_MODE_SHARED_OTF && s->R == 1 && s->T == 1 && s->k <= 32 && tn.visit_once != 2;
  if (s->visit_once) s->tick_cap = CHAIN_TICK_SLICES;
  if (tn.chain_workgroups) s->chain_wg_cap = tn.chain_workgroups;
  // (the stage lives in builds of the step kernel of their own: one-relation graphs with rows of up to 32 slots, one
  // step per launch; elsewhere the field is ignored)
  s->lds_stage = tn.lds_dedupe == 1 && s->R == 1 && s->T == 1 && s->k <= 32;
  if (s->lds_stage && !s->visit_once) s->tick_cap = 12;
  s->visit_once_forced = tn.visit_once == 1;
  for (float& r : s->fill_ratio) r = 1.0f;
  // Dedupe table layout: one 8-byte word per node (no probing, one atomic per insert) unless that
  // would be large; gss_tuning.dedupe_layout overrides the choice.
  s->use_direct = (uint64_t)total_nodes * 8ull <= (8ull << 30);
  if (tn.dedupe_layout) s->use_direct = tn.dedupe_layout == 1;

  s->state_words = ST_COUNTS + (GSS_MAX_LAYERS + 1) * s->T + GSS_MAX_LAYERS * s->R;
  const size_t state_bytes = sizeof(int32_t) * (size_t)s->state_words;
  s->state_d = (int32_t*)dev_alloc(s, state_bytes);
  if (!s->state_d) return bail(GSS_ERR_OOM);
  hipError_t e = hipHostMalloc((void**)&s->state_h, state_bytes, hipHostMallocDefault);
  if (e != hipSuccess) { s->state_h = nullptr; return hipfail(e); }
  if ((e = hipMemsetAsync(s->state_d, 0, state_bytes, s->stream)) != hipSuccess) return hipfail(e);
  if ((e = hipEventCreateWithFlags(&s->user_ready, hipEventDisableTiming)) != hipSuccess) { s->user_ready = nullptr; return hipfail(e); }
  // Modes whose sample phases write no table have no dependency between steps: a tick can start two of them,
  // which halves the launches and the idle time between them per step, where a launch has the slices for it
  // (one-relation graphs: the compact form carries 24).  Measured on the 1,024-seed workload: FBL and OTF fetch
  // -15 % per step; the epoch-refreshed modes gain nothing (their refresh kernel shares the chip with launches
  // twice as large) and keep one step per tick.
  s->steps_per_tick = (!s->otf && !s->fcr && s->R == 1 && s->T == 1 && s->k <= 32) ? 2 : 1;
  if (tn.steps_per_tick) s->steps_per_tick = (!s->otf && s->k <= 32 && tn.steps_per_tick == 2) ? 2 : 1;
  if (s->lds_stage) s->steps_per_tick = 1;
  // Lanes per frontier node in the sample phase.  A row of k slots keeps k lanes busy, and a wavefront's vector
  // instructions cost the same however many of its lanes take part: rows of up to 20 slots can get 21 lanes (three
  // nodes per wavefront), of up to 16 slots 16 lanes (four), instead of 32 (two) - chosen per launch, see tick().
  // One-relation graphs, the modes with cached rows and one step per launch (these builds exist for the plain launch
  // of up to 12 slices only).
  s->group_w = s->k > 32 ? 64 : 32;
  const bool rows_mode = c->mode == GSS_MODE_FCR || c->mode == GSS_MODE_OTF || c->mode == GSS_MODE_OTF_LAYER || c->mode == GSS_MODE_SHARED_FCR;
  if (s->k <= 20 && s->R == 1 && s->T == 1 && rows_mode && s->steps_per_tick == 1 && !s->lds_stage && !s->visit_once && tn.group_width != 32) {
    s->narrow_w = s->k <= 16 ? 16 : 21;
    s->narrow_always = tn.group_width == 1;
    s->tick_cap = std::min(s->tick_cap, 12);
  }
  // A step of L hops has up to 4 L phases, one per launch: with two more steps than that in flight the step a
  // caller waits for has left the queue before.  (Deeper rings only widen the memory the launches touch: every slot
  // has scratch and a dedupe table of its own - 4 L + 4 was 1 % slower on the 1,024-seed workloads, 4 L too shallow.)
  s->ring = std::min(GSS_MAX_IN_FLIGHT, s->steps_per_tick * (4 * s->L + 2));
  // (a visit-once step's list phases trail its chain by a little more than three steps' worth of launches - the place
  // phase of every hop past the first waits for the next step's first chain phase -: five steps in flight cover that
  // for up to three hops; six were 0.6 % slower on the 4,096-seed shared-table workload, four 8 %)
  if (s->visit_once) s->ring = std::min(GSS_MAX_IN_FLIGHT, std::max(5, s->L + 2));
  if (tn.pipeline_depth) s->ring = tn.pipeline_depth;
  if ((e = hipStreamCreateWithFlags(&s->work, hipStreamNonBlocking)) != hipSuccess) { s->work = nullptr; return hipfail(e); }
  for (hipEvent_t& ev : s->tick_ev)
    if ((e = hipEventCreateWithFlags(&ev, hipEventDisableTiming)) != hipSuccess) { ev = nullptr; return hipfail(e); }
  if (m_fcr) {
    if ((e = hipStreamCreateWithFlags(&s->fill_stream, hipStreamNonBlocking)) != hipSuccess) { s->fill_stream = nullptr; return hipfail(e); }
    if ((e = hipEventCreateWithFlags(&s->fill_go, hipEventDisableTiming)) != hipSuccess) { s->fill_go = nullptr; return hipfail(e); }
    if ((e = hipEventCreateWithFlags(&s->fill_done, hipEventDisableTiming)) != hipSuccess) { s->fill_done = nullptr; return hipfail(e); }
    s->fill_state_d = (int32_t*)dev_alloc(s, state_bytes);
    if (!s->fill_state_d) return bail(GSS_ERR_OOM);
    if ((e = hipMemsetAsync(s->fill_state_d, 0, state_bytes, s->stream)) != hipSuccess) return hipfail(e);
    if ((e = hipHostMalloc((void**)&s->fill_state_h, state_bytes, hipHostMallocDefault)) != hipSuccess) { s->fill_state_h = nullptr; return hipfail(e); }
    memset(s->fill_state_h, 0, state_bytes);
  }

  // The fill kernels index the adjacency through indptr: validate the graph before touching it.
  for (int r = 0; r < s->R; ++r) {
    const gss_relation& q = s->rel[r];
    e = launch_validate_graph(q.indptr, q.indptr_is_64, s->num_nodes[q.dst_type], q.indices, q.nnz,
                              s->num_nodes[q.src_type], s->state_d, s->stream);
    if (e != hipSuccess) return hipfail(e);
  }
  if (read_create_state(s) != GSS_OK) return bail(GSS_ERR_DEVICE);
  if (s->state_h[ST_ERROR] & ERR_GRAPH) return bail(GSS_ERR_INVALID_GRAPH);

  // Degree split: number the nodes that keep a row (deg > theta), per relation; the tables then hold
  // only those rows.  The row counts come back in the state words after the error flag.
  for (int r = 0; r < s->R; ++r) s->table_rows[r] = s->num_nodes[s->rel[r].dst_type];
  if (s->theta >= 0) {
    int64_t max_n = 0;
    for (int r = 0; r < s->R; ++r) max_n = std::max(max_n, s->num_nodes[s->rel[r].dst_type]);
    int32_t* chunk_counts = (int32_t*)dev_alloc(s, sizeof(int32_t) * (size_t)(max_n / 1024 + 2));
    if (!chunk_counts) return bail(GSS_ERR_OOM);
    for (int r = 0; r < s->R && e == hipSuccess; ++r) {
      const gss_relation& q = s->rel[r];
      const int64_t n = s->num_nodes[q.dst_type];
      s->row_of[r] = (int32_t*)dev_alloc(s, sizeof(int32_t) * (size_t)n);
      if (!s->row_of[r]) { dev_free(s, chunk_counts); return bail(GSS_ERR_OOM); }
      s->cache_bytes += (int64_t)sizeof(int32_t) * n;
      e = launch_build_row_map(q.indptr, q.indptr_is_64, n, s->theta, chunk_counts, s->row_of[r],
                               s->state_d + ST_COUNTS + r, s->stream);
    }
    const gss_status rs = (e == hipSuccess) ? read_create_state(s) : GSS_ERR_DEVICE;
    dev_free(s, chunk_counts);     // the stream is idle after the readback
    if (rs != GSS_OK) return bail(GSS_ERR_DEVICE);
    for (int r = 0; r < s->R; ++r) s->table_rows[r] = s->state_h[ST_COUNTS + r];
  }
  // FCR: as many sets of tables as the epochs the steps in flight can span, plus the one being computed ahead
  // (a step reads its epoch's set until its last sample phase has run: with `ring` steps in flight and a refresh
  // every `period` steps that is 2 + ring / period sets, three at least, MAX_TABLE_SETS at most) - when they are
  // small next to the free device memory (at most 1/8 of it all together), else two, else - when not even a
  // second one fits into half of it - one, refreshed in place after the steps in flight have drained.
  // gss_tuning.table_sets overrides.
  size_t set_bytes = 0;
  for (int r = 0; r < s->R; ++r) set_bytes += sizeof(int32_t) * (size_t)s->table_rows[r] * (size_t)s->S * (size_t)s->num_tables;
  if (s->fcr) {
    size_t free_b = 0, total_b = 0;
    if (hipMemGetInfo(&free_b, &total_b) != hipSuccess) { (void)hipGetLastError(); free_b = 0; }
    const int want = std::min(MAX_TABLE_SETS, std::max(3, 2 + s->ring / std::max(1, s->period)));
    s->nsets = ((size_t)want * set_bytes <= free_b / 8) ? want : (3 * set_bytes <= free_b / 8) ? 3
               : (2 * set_bytes <= free_b / 2) ? 2 : 1;
    if (tn.table_sets) s->nsets = tn.table_sets;
  }
  for (int q = 0; q < s->nsets; ++q)
    for (int t = 0; t < s->num_tables; ++t)
      for (int r = 0; r < s->R; ++r) {
        const size_t bytes = sizeof(int32_t) * (size_t)s->table_rows[r] * (size_t)s->S;
        s->table[q][t][r] = (int32_t*)dev_alloc(s, bytes);
        if (!s->table[q][t][r]) return bail(GSS_ERR_OOM);
        s->cache_bytes += (int64_t)bytes;
      }
  if (s->mode == GSS_MODE_SHARED_OTF)
    for (int r = 0; r < s->R; ++r) {
      const int64_t n = s->table_rows[r];
      s->stamp[r] = (long long*)dev_alloc(s, sizeof(long long) * (size_t)n);
      if (!s->stamp[r]) return bail(GSS_ERR_OOM);
      s->cache_bytes += (int64_t)sizeof(long long) * n;
      if (n > 0 && (e = launch_fill_i64(s->stamp[r], n, -1, s->stream)) != hipSuccess) return hipfail(e);
    }
  for (int r = 0; r < s->R; ++r) {
    RelConst& rc = s->relc_h[r];
    rc.indptr = s->rel[r].indptr; rc.indices = s->rel[r].indices;
    rc.stamp = s->stamp[r]; rc.row_of = s->row_of[r];
    rc.is64 = s->rel[r].indptr_is_64;
    rc.n_dst = (int32_t)s->num_nodes[s->rel[r].dst_type];
  }
  s->relc_d = (RelConst*)dev_alloc(s, sizeof(RelConst) * GSS_MAX_RELATIONS);
  if (!s->relc_d) return bail(GSS_ERR_OOM);
  if ((e = hipMemcpyAsync(s->relc_d, s->relc_h, sizeof(RelConst) * GSS_MAX_RELATIONS, hipMemcpyHostToDevice, s->stream)) != hipSuccess)
    return hipfail(e);
  s->slotc_d = (SlotConst*)dev_alloc(s, sizeof(SlotConst) * GSS_MAX_IN_FLIGHT);
  if (!s->slotc_d) return bail(GSS_ERR_OOM);
  if ((e = hipMemsetAsync(s->slotc_d, 0, sizeof(SlotConst) * GSS_MAX_IN_FLIGHT, s->stream)) != hipSuccess) return hipfail(e);
  if (!ensure(s, s->checksum, 8)) return bail(GSS_ERR_OOM);
  for (int i = 0; i < s->ring; ++i) {      // (the slots beyond the ring are never used)
    Slot& sl = s->slot[i];
    sl.state_d = (int32_t*)dev_alloc(s, state_bytes);
    if (!sl.state_d) return bail(GSS_ERR_OOM);
    if ((e = hipMemsetAsync(sl.state_d, 0, state_bytes, s->stream)) != hipSuccess) return hipfail(e);
    e = hipHostMalloc((void**)&sl.state_h, state_bytes, hipHostMallocDefault);
    if (e != hipSuccess) { sl.state_h = nullptr; return hipfail(e); }
    if ((e = hipHostGetDevicePointer((void**)&sl.state_h_dev, sl.state_h, 0)) != hipSuccess) return hipfail(e);
    sl.out_nodes.resize((size_t)GSS_MAX_LAYERS * s->T);
    sl.out_edges.resize((size_t)GSS_MAX_LAYERS * s->R);
  }
  if (s->fcr) {   // the list of rows a refresh has to recompute (nodes with a row and more than k neighbors)
    int64_t max_n = 0;
    for (int r = 0; r < s->R; ++r) max_n = std::max(max_n, s->num_nodes[s->rel[r].dst_type]);
    int32_t* chunk_counts = (int32_t*)dev_alloc(s, sizeof(int32_t) * (size_t)(max_n / 1024 + 2));
    int32_t* map = (int32_t*)dev_alloc(s, sizeof(int32_t) * (size_t)std::max<int64_t>(max_n, 1));
    gss_status hs = (chunk_counts && map) ? GSS_OK : GSS_ERR_OOM;
    for (int r = 0; r < s->R && hs == GSS_OK; ++r) {
      const gss_relation& q = s->rel[r];
      const int64_t n = s->num_nodes[q.dst_type];
      if (n <= 0) continue;
      e = launch_build_row_map(q.indptr, q.indptr_is_64, n, std::max(s->k, s->theta), chunk_counts, map,
                               s->state_d + ST_COUNTS, s->stream);
      if (e != hipSuccess || read_create_state(s) != GSS_OK) { hs = GSS_ERR_DEVICE; break; }
      s->num_heavy[r] = s->state_h[ST_COUNTS];
      if (s->num_heavy[r] > 0) {
        s->heavy_list[r] = (int32_t*)dev_alloc(s, sizeof(int32_t) * (size_t)s->num_heavy[r]);
        if (!s->heavy_list[r]) { hs = GSS_ERR_OOM; break; }
        s->cache_bytes += (int64_t)sizeof(int32_t) * s->num_heavy[r];
        if (launch_list_from_map(map, n, s->heavy_list[r], s->stream) != hipSuccess ||
            hipStreamSynchronize(s->stream) != hipSuccess) { hs = GSS_ERR_DEVICE; break; }
      }
    }
    dev_free(s, chunk_counts);
    dev_free(s, map);
    if (hs != GSS_OK) return bail(hs);
    s->heavy_ready = true;
  }
  if (fill_all_tables(s, 0, s->state_d, s->stream) != GSS_OK) return bail(GSS_ERR_DEVICE);
  if (read_create_state(s) != GSS_OK) return bail(GSS_ERR_DEVICE);
  if (s->state_h[ST_ERROR] != 0) return bail(GSS_ERR_INVALID_GRAPH);   // e.g. repeated neighbor ids in a row
  *out = s;
  return GSS_OK;
}

gss_status gss_destroy(gss_sampler* s) {
  destroy_impl(s);
  return GSS_OK;
}

// Makes the buffers of slot `sl` large enough for a step planned like `plan` (L hops, max_slots pick slots, max_keys
// dedupe keys), clears a new dedupe table on `st`, and brings the slot's entry of the device table up to date.
static gss_status grow_slot(gss_sampler* s, Slot& sl, const Slot& plan, int L, int64_t max_slots, int64_t max_keys,
                            hipStream_t st, bool* grew) {
  const int T = s->T, R = s->R;
  bool any = false;
  auto need = [&](Buf& b, size_t bytes) { if (b.bytes >= bytes && b.p) return true; any = true; return ensure(s, b, bytes); };
  if (s->use_direct && !sl.direct.p) {
    if (!need(sl.direct, sizeof(uint64_t) * (size_t)std::max<int64_t>(s->total_nodes, 1)))
      return fail(s, GSS_ERR_OOM, "step: dedupe table allocation failed");
    HIP_TRY(s, hipMemsetAsync(sl.direct.p, 0xFF, sl.direct.bytes, st));
    sl.ver = s->first_version;
  }
  if (!s->use_direct) {
    uint64_t cap = 1024;
    while (cap < 2 * (uint64_t)max_keys) cap <<= 1;
    if (sl.hash.bytes < cap * sizeof(HashEntry)) {
      if (!need(sl.hash, cap * sizeof(HashEntry))) return fail(s, GSS_ERR_OOM, "step: dedupe table allocation failed");
      HIP_TRY(s, hipMemsetAsync(sl.hash.p, 0xFF, sl.hash.bytes, st));
      sl.ver = s->first_version;
    }
  }
  sl.hash_cap = s->use_direct ? 0 : sl.hash.bytes / sizeof(HashEntry);   // power of two by construction
  const size_t slot_bytes = sizeof(int32_t) * (size_t)std::max<int64_t>(max_slots, 1);
  const size_t tile_bytes = sizeof(int32_t) * (size_t)std::max<int64_t>(max_slots / TILE, 1);
  if (!need(sl.picks, slot_bytes) || !need(sl.order, slot_bytes) || !need(sl.ranks, slot_bytes) ||
      !need(sl.partial_first, tile_bytes) || !need(sl.partial_edge, tile_bytes) ||
      !need(sl.first_off, tile_bytes) || !need(sl.edge_off, tile_bytes))
    return fail(s, GSS_ERR_OOM, "step: scratch allocation failed");
  for (int h = 0; h < L; ++h) {
    const int l = L - 1 - h;
    for (int t = 0; t < T; ++t)
      if (!need(sl.src_nodes[l][t], sizeof(int32_t) * (size_t)std::max<int64_t>(plan.fub[h + 1][t], 1)))
        return fail(s, GSS_ERR_OOM, "step: output allocation failed");
    for (int r = 0; r < R; ++r)
      if (!need(sl.src_local[l][r], sizeof(int32_t) * (size_t)std::max<int64_t>(plan.slots_ub[h][r], 1)) ||
          !need(sl.dst_local[l][r], sizeof(int32_t) * (size_t)std::max<int64_t>(plan.slots_ub[h][r], 1)))
        return fail(s, GSS_ERR_OOM, "step: output allocation failed");
  }
  if (plan.chain) {
    const ChainArgs& C = plan.chain_args;
    if (!sl.visit.p) {
      if (!need(sl.visit, sizeof(uint64_t) * (size_t)std::max<int64_t>(s->total_nodes, 1)))
        return fail(s, GSS_ERR_OOM, "step: visit table allocation failed");
      HIP_TRY(s, hipMemsetAsync(sl.visit.p, 0xFF, sl.visit.bytes, st));
    }
    const size_t held = (size_t)C.off[L - 1] + (size_t)C.V[L - 1] * C.f(L - 1);
    if (!need(sl.held, sizeof(int32_t) * std::max<size_t>(held, 1))) return fail(s, GSS_ERR_OOM, "step: holding area allocation failed");
    size_t entries = 0;
    for (int h = 1; h < L; ++h) entries = (size_t)C.loff[h] + (size_t)CHAIN_SEGS * C.lcap[h];
    if (!need(sl.list, sizeof(uint64_t) * std::max<size_t>(entries, 1))) return fail(s, GSS_ERR_OOM, "step: node list allocation failed");
    if (!sl.counts.p) {
      if (!need(sl.counts, sizeof(uint32_t) * 2 * CHAIN_MAX_HOPS * CHAIN_SEGS * CHAIN_COUNT_STRIDE)) return fail(s, GSS_ERR_OOM, "step: node list allocation failed");
      HIP_TRY(s, hipMemsetAsync(sl.counts.p, 0, sl.counts.bytes, st));
    }
  }
  // the slot's entry of the device table follows its buffers (they only change while they grow)
  const int idx = (int)(&sl - s->slot);
  const SlotConst sc = slot_const(s, sl);
  if (memcmp(&sc, &s->slotc_h[idx], sizeof sc) != 0) {
    s->slotc_h[idx] = sc;
    HIP_TRY(s, hipMemcpyAsync(s->slotc_d + idx, &s->slotc_h[idx], sizeof sc, hipMemcpyHostToDevice, st));
  }
  if (grew) *grew = any;
  return GSS_OK;
}

gss_status gss_step_async(gss_sampler* s, const int32_t* seeds, int32_t num_seeds, int32_t seed_type,
                          const int32_t* fanouts, int32_t num_layers, int64_t step) {
  if (!s) return GSS_ERR_INVALID_ARG;
  s->err[0] = 0;
  if (s->poisoned) return fail(s, GSS_ERR_DEVICE, "a previous step failed on the device; destroy the sampler");
  if (!fanouts || num_seeds < 0 || (num_seeds > 0 && !seeds) || seed_type < 0 || seed_type >= s->T ||
      num_layers < 1 || num_layers > s->L || step < 0 || step >= (int64_t(1) << 32))
    return fail(s, GSS_ERR_INVALID_ARG, "step: invalid argument");
  int64_t fsum = 0;
  for (int l = 0; l < num_layers; ++l) {
    if (fanouts[l] < 1 || fanouts[l] > s->k) return fail(s, GSS_ERR_INVALID_ARG, "step: fanout[%d]=%d not in [1,k]", l, fanouts[l]);
    fsum += fanouts[l];
  }
  if (s->shared && fsum > s->k) return fail(s, GSS_ERR_INVALID_ARG, "step: shared mode needs sum(fanouts) <= k");
  if (step < s->last_step) return fail(s, GSS_ERR_STEP_ORDER, "step: %lld after %lld", (long long)step, (long long)s->last_step);
  if ((int64_t)num_seeds > s->num_nodes[seed_type]) return fail(s, GSS_ERR_INVALID_SEED, "step: more seeds than nodes");
  Slot& sl = s->slot[s->enq];
  Slot& prev = s->slot[(s->enq + s->ring - 1) % s->ring];   // the step enqueued just before this one
  if (sl.pending) return fail(s, GSS_ERR_INVALID_ARG, "step: %d steps are already in flight; call gss_step_wait first", s->ring);

  // ---- plan: host-known upper bounds of every hop ----
  const int T = s->T, R = s->R, L = num_layers;
  int64_t max_slots = 0, max_keys = 0;
  memset(sl.fub, 0, sizeof sl.fub);
  sl.fub[0][seed_type] = num_seeds;
  for (int h = 0; h < L; ++h) {
    const int f = fanouts[L - 1 - h];
    int64_t base = 0;
    for (int t = 0; t < T; ++t) sl.fub[h + 1][t] = sl.fub[h][t];
    for (int r = 0; r < R; ++r) {
      sl.slots_ub[h][r] = sl.fub[h][s->rel[r].dst_type] * f;
      sl.slot_base[h][r] = base;
      base += (sl.slots_ub[h][r] + TILE - 1) / TILE * TILE;
      sl.fub[h + 1][s->rel[r].src_type] += sl.slots_ub[h][r];
    }
    int64_t keys = 0;
    for (int t = 0; t < T; ++t) { sl.fub[h + 1][t] = std::min(sl.fub[h + 1][t], s->num_nodes[t]); keys += sl.fub[h + 1][t]; }
    sl.total_slots[h] = base;
    max_slots = std::max(max_slots, base);
    max_keys = std::max(max_keys, keys);
  }
  if (max_slots >= (int64_t(1) << 31)) return fail(s, GSS_ERR_INVALID_ARG, "step: batch too large (pick slots >= 2^31)");
  // ---- visit-once step?  Its holding index space is laid out by bounds that are not capped by the number of nodes:
  //      V[h+1] = V[h] * (1 + f[h]).  Steps whose holding area would pass 2^28 picks (1 GiB) run the per-hop way. ----
  ChainArgs chain_args;
  memset(static_cast<void*>(&chain_args), 0, sizeof chain_args);
  // (a blocking gss_step has the launches to itself: hop by hop it needs one fewer, and none of them carries two phases)
  bool chain = s->visit_once && L <= CHAIN_MAX_HOPS && !(s->blocking_call && !s->visit_once_forced);
  if (chain) {
    int64_t V = num_seeds, off = 0, band = 0;
    int64_t band_of[GSS_MAX_LAYERS] = {};
    for (int l = 0; l < L; ++l) { band_of[l] = band; band += fanouts[l]; }   // layer l's band starts at the sum of the lower layers' fanouts
    for (int h = 0; h < L && chain; ++h) {
      const int f = fanouts[L - 1 - h];
      chain_args.V[h] = (int32_t)V; chain_args.off[h] = (uint32_t)off;
      chain_args.fbl[h] = (uint32_t)f | ((uint32_t)band_of[L - 1 - h] << 8) | ((uint32_t)(L - 1 - h) << 16);
      // list h + 1: CHAIN_SEGS segments, each for the picks of every CHAIN_SEGS-th pair of hop h's frontier nodes
      if (h + 1 < L) {
        const int64_t cap = ((V + 1) / 2 + CHAIN_SEGS - 1) / CHAIN_SEGS * 2 * f;
        chain_args.loff[h + 1] = chain_args.loff[h] + (h ? (uint32_t)CHAIN_SEGS * chain_args.lcap[h] : 0u);
        chain_args.lcap[h + 1] = (uint32_t)cap;
        if (cap * CHAIN_SEGS >= (int64_t(1) << 28)) chain = false;
      }
      off += V * f;
      V += V * f;
      if (off >= (int64_t(1) << 28)) chain = false;
    }
    chain_args.L = L;
  }

  hipStream_t st = s->work;
  // ---- OTF: hops of steps with different layer counts would meet on the same per-layer table in one
  //      tick: let the steps in flight finish issuing first ----
  if (s->otf && !s->shared && prev.pending && prev.L != L) {
    gss_status ds = drain(s);
    if (ds != GSS_OK) return ds;
  }
  // ---- FCR refresh: the set of tables about to be overwritten was read by the steps of the epoch
  //      before the current one; with a short refresh period some may still have phases to issue ----
  const int64_t epoch = s->fcr ? step / s->period : 0;
  const int fill_set = (s->cur_set + 1) % s->nsets;   // (one set: the refresh overwrites the tables in place)
  const bool prefetched = s->fcr && epoch != s->epoch && s->prefetched_epoch == epoch;
  if (s->fcr && epoch != s->epoch && !prefetched) {
    bool open = false;
    for (const Slot& o : s->slot) open |= o.pending && o.table_set == fill_set && o.items.open();
    if (open) {
      gss_status ds = drain(s);
      if (ds != GSS_OK) return ds;
    }
  }

  // ---- order the work stream after the caller's stream (seeds are ready; memory the allocator
  //      hands out may still be in use by earlier work of the caller's stream) ----
  if (hipStreamQuery(s->stream) != hipSuccess) {   // (an idle caller stream needs no event)
    (void)hipGetLastError();
    HIP_TRY(s, hipEventRecord(s->user_ready, s->stream));
    HIP_TRY(s, hipStreamWaitEvent(st, s->user_ready, 0));
  }

  // ---- buffers (grow-only) of this slot - and, with the same sizes, of every slot of the ring that has not held a
  //      step yet: the allocations of a run then all happen at its first step, not once per slot as the ring is first
  //      walked.  (A slot that has held a step keeps its buffers until it is used again: the caller may still be
  //      reading that step's blocks.) ----
  sl.chain = chain;
  sl.chain_args = chain_args;
  {
    bool grew = false;
    gss_status gs = grow_slot(s, sl, sl, L, max_slots, max_keys, st, &grew);
    if (gs != GSS_OK) return gs;
    if (grew)
      for (int q = 0; q < s->ring; ++q) {
        Slot& o = s->slot[q];
        if (&o == &sl || o.pending || o.used) continue;
        if ((gs = grow_slot(s, o, sl, L, max_slots, max_keys, st, nullptr)) != GSS_OK) return gs;
      }
  }
  if (chain) {
    sl.chain_args.held = (int32_t*)sl.held.p;
    sl.chain_args.visit = (uint64_t*)sl.visit.p;
    sl.chain_args.list = (uint64_t*)sl.list.p;
    sl.chain_args.counts = (uint32_t*)sl.counts.p + sl.chain_parity * CHAIN_MAX_HOPS * CHAIN_SEGS * CHAIN_COUNT_STRIDE;
    sl.chain_args.counts_next = (uint32_t*)sl.counts.p + (1 - sl.chain_parity) * CHAIN_MAX_HOPS * CHAIN_SEGS * CHAIN_COUNT_STRIDE;
    sl.chain_parity ^= 1;
  }
  if (sl.ver + (uint32_t)L >= VERSION_LAST) {        // version space exhausted: start over with a clean table
    if (s->use_direct) HIP_TRY(s, hipMemsetAsync(sl.direct.p, 0xFF, sl.direct.bytes, st));
    else HIP_TRY(s, hipMemsetAsync(sl.hash.p, 0xFF, sl.hash.bytes, st));
    if (sl.visit.p) HIP_TRY(s, hipMemsetAsync(sl.visit.p, 0xFF, sl.visit.bytes, st));
    sl.ver = VERSION_FIRST;
  }
  s->last_step = step;
  sl.L = L; sl.num_seeds = num_seeds; sl.seed_type = seed_type; sl.seeds = seeds; sl.step = step;
  for (int l = 0; l < L; ++l) sl.fanouts[l] = fanouts[l];
  sl.refresh_now = s->otf && s->n_new > 0 && (step % s->period == 0);
  sl.ver0 = sl.ver;
  sl.ver += (uint32_t)L;
  uint32_t scan_hops = 0;                // hops whose emit phase does not scan the tile totals itself
  for (int h = 0; h < L; ++h) scan_hops |= scans_in_emit(s, sl, h) ? 0u : (1u << h);
  // The dedupe table inserts of a hop run as a phase of their own
  //   - on wide hops (INSERT_SPLIT_SLOTS expected picks and more) of the modes without a refresh in the sample phase:
  //     there the inserts are most of the phase; with a refresh they are a small part of it and the extra pass over
  //     the picks costs more than it saves (measured);
  //   - on narrow hops (up to INSERT_SMALL_SLOTS): their sample workgroups are the longest dependent chains of a
  //     launch, and the load + atomic of the insert are two more links (the 128-seed workload: -10 % per step);
  //     not with one table for all hops and a refresh, where a step's phases run one after the other and a phase
  //     more is a launch more;
  //   as long as a tick still fits one launch.
  sl.insert_hops = 0;
  int phases = 3 * L;
  for (int h = 0; h < L; ++h) phases += scans_in_emit(s, sl, h) ? 0 : 1;
  for (int h = L - 1; h >= 0; --h) {                     // the outermost hop is the widest
    const double expect = std::min(1.0, 1.25 * (double)s->fill_ratio[h]) * (double)sl.total_slots[h];
    // (visit-once steps: only on request.  Taking the inserts out of the place phase of the outermost hop - which shares
    // a launch with the chain phase of hop 0 and is the longest slice of that launch - was measured on the 4,096-seed
    // shared-table workload: 0.1197 instead of 0.1177 ms per step.  The launches of a full pipeline are bound by the
    // work they hold, not by their longest slice.)
    const bool wide = !chain && !s->otf && expect >= (double)INSERT_SPLIT_SLOTS;
    const bool narrow = !chain && !(s->otf && s->shared) && expect <= (double)INSERT_SMALL_SLOTS;
    // (a tick of visit-once steps holds a chain phase and one list phase of each step in flight, whatever the number
    // of a step's phases)
    const bool fits = chain || phases < s->tick_cap;
    const bool split = s->insert_policy == 1 || (s->insert_policy == 0 && fits && (wide || narrow));
    if (split) { sl.insert_hops |= 1u << h; ++phases; }
  }
  sl.items.build(L, scan_hops, sl.insert_hops, chain);

  // ---- Alg. 3: full refresh when the refresh epoch changes, into the set of tables that is not in use
  //      (stream order puts it after the steps that last read that set: their phases are all issued) ----
  if (s->fcr && epoch != s->epoch) {
    if (s->prefetched_epoch >= 0) {      // the idle set is being (or has been) written on the fill stream
      HIP_TRY(s, hipStreamWaitEvent(st, s->fill_done, 0));
      // the refresh started an epoch ago and is normally long done: its error flag is checked here, before any
      // step reads its rows
      HIP_TRY(s, hipEventSynchronize(s->fill_done));
      if (s->fill_state_h[ST_ERROR] != 0) {
        s->poisoned = true;
        return fail(s, GSS_ERR_DEVICE, "refresh: device error flag 0x%x", s->fill_state_h[ST_ERROR]);
      }
    }
    if (!prefetched) {                   // (a step number jumped over the epoch computed ahead, or none was)
      gss_status rs = fill_all_tables(s, (uint32_t)(epoch * s->period), sl.state_d, st, fill_set, s->cur_set);
      if (rs != GSS_OK) { s->poisoned = true; return rs; }
    }
    s->prefetched_epoch = -1;
    s->cur_set = fill_set;
    s->epoch = epoch;
  }
  sl.table_set = s->cur_set;
  sl.pending = true;
  sl.used = true;
  s->enq = (s->enq + 1) % s->ring;
  // (two steps share a tick only while their launches are small: from about 400k expected picks per step on, a
  // launch of two is slower than two launches - measured with fanouts 20 / 20 / 20)
  double expect_picks = 0.0;
  for (int h = 0; h < L; ++h) expect_picks += std::min(1.0, 1.25 * (double)s->fill_ratio[h]) * (double)sl.total_slots[h];
  const int per_tick = (s->steps_per_tick == 2 && expect_picks <= (double)TWO_STEP_PICKS) ? 2 : 1;
  if (++s->unlaunched >= per_tick) {
    gss_status ts = tick(s, nullptr);   // one launch: the first phase of the new step(s) and the next phase of every older one
    if (ts != GSS_OK) return ts;
  }
  // With one table for all hops and a refresh per visit, a step's launches that touch the table - L chain phases of a
  // visit-once step, or its sample phases with the mark and emit phases between them - must all run before the next
  // step's first: they are issued now, so that this chain never waits for the host (issued one per call, the others
  // came from gss_step_wait just in time, and the queue ran dry whenever the caller collected a step: 11 us of idle
  // time per step on the 4,096-seed shared-table workload).  The other phases of the older steps ride along as they
  // become ready.
  while (s->otf && s->shared && s->unlaunched == 0 && !sl.items.table_work_issued()) {
    int issued = 0;
    gss_status ts = tick(s, &issued);
    if (ts != GSS_OK) return ts;
    if (issued == 0) break;             // (cannot happen: the oldest step with phases left is always ready)
  }
  return maybe_prefetch_epoch(s);
}

gss_status gss_step_wait(gss_sampler* s, gss_blocks* out) {
  if (!s || !out) return GSS_ERR_INVALID_ARG;
  Slot* oldest = oldest_pending(s);
  if (!oldest) return fail(s, GSS_ERR_INVALID_ARG, "step_wait: no step in flight");
  Slot& sl = *oldest;
  while (sl.items.open()) {  // fewer steps followed this one than it has phases
    int issued = 0;                      // (the oldest step in flight is always ready)
    gss_status ms = tick(s, &issued);
    if (ms != GSS_OK) return ms;
    if (issued == 0) { s->poisoned = true; return fail(s, GSS_ERR_DEVICE, "pipeline: the oldest step is not ready"); }
  }
  sl.pending = false;
  hipError_t e = hipEventSynchronize(sl.done);
  if (e != hipSuccess) { s->poisoned = true; return fail(s, GSS_ERR_DEVICE, "step_wait: %s", hipGetErrorString(e)); }
  const int32_t flag = sl.state_h[ST_ERROR];
  if (flag != 0) {
    s->poisoned = true;
    if (flag & (ERR_SEED_RANGE | ERR_SEED_DUP))
      return fail(s, GSS_ERR_INVALID_SEED, "step: seed %s", (flag & ERR_SEED_RANGE) ? "out of range" : "repeated");
    return fail(s, GSS_ERR_DEVICE, "step: device error flag 0x%x", flag);
  }
  const int T = s->T, R = s->R, L = sl.L;
  int64_t total_edges = 0;
  for (int h = 0; h < L; ++h) {
    const int l = L - 1 - h;
    float ratio = 0.f;
    for (int t = 0; t < T; ++t) {
      gss_block_nodes& bn = sl.out_nodes[(size_t)l * T + t];
      bn.num_dst = (h == 0) ? (t == sl.seed_type ? sl.num_seeds : 0) : sl.state_h[ST_COUNTS + h * T + t];
      if (sl.fub[h][t] > 0) ratio = std::max(ratio, (float)bn.num_dst / (float)sl.fub[h][t]);
      bn.num_src = sl.state_h[ST_COUNTS + (h + 1) * T + t];
      bn.src_nodes = (const int32_t*)sl.src_nodes[l][t].p;
    }
    s->fill_ratio[h] = std::max(ratio, 0.9f * s->fill_ratio[h]);   // up at once, down slowly
    for (int r = 0; r < R; ++r) {
      gss_block_edges& be = sl.out_edges[(size_t)l * R + r];
      be.num_edges = sl.state_h[ST_COUNTS + (GSS_MAX_LAYERS + 1) * T + h * R + r];
      be.src_local = (const int32_t*)sl.src_local[l][r].p;
      be.dst_local = (const int32_t*)sl.dst_local[l][r].p;
      total_edges += be.num_edges;
    }
  }
  out->num_layers = L; out->num_node_types = T; out->num_relations = R;
  out->nodes = sl.out_nodes.data();
  out->edges = sl.out_edges.data();
  out->total_edges = total_edges;
  return GSS_OK;
}

gss_status gss_step(gss_sampler* s, const int32_t* seeds, int32_t num_seeds, int32_t seed_type,
                    const int32_t* fanouts, int32_t num_layers, int64_t step, gss_blocks* out) {
  if (!s || !out) return GSS_ERR_INVALID_ARG;
  if (oldest_pending(s))
    return fail(s, GSS_ERR_INVALID_ARG, "step: collect the steps in flight with gss_step_wait first");
  s->blocking_call = true;
  gss_status st = gss_step_async(s, seeds, num_seeds, seed_type, fanouts, num_layers, step);
  s->blocking_call = false;
  if (st != GSS_OK) return st;
  return gss_step_wait(s, out);
}

gss_status gss_profile_enable(gss_sampler* s, int32_t on) {
  if (!s) return GSS_ERR_INVALID_ARG;
  gss_status st = sync_all(s);
  if (st != GSS_OK) return st;
  if (on) {
    if (!s->timer) s->timer = new (std::nothrow) EventTimer();
    if (!s->timer) return fail(s, GSS_ERR_OOM, "profile: out of host memory");
    s->timer->reset();
  } else {
    delete s->timer;
    s->timer = nullptr;
  }
  return GSS_OK;
}

gss_status gss_profile_read(gss_sampler* s, double* ms, int64_t* launches) {
  if (!s || !ms || !launches) return GSS_ERR_INVALID_ARG;
  if (!s->timer) return fail(s, GSS_ERR_INVALID_ARG, "profile: not enabled");
  gss_status st = sync_all(s);
  if (st != GSS_OK) return st;
  s->timer->collect();
  for (int i = 0; i < KID_COUNT; ++i) { ms[i] = s->timer->ms[i]; launches[i] = s->timer->launches[i]; }
  return GSS_OK;
}

gss_status gss_gather_rows(const void* table, int64_t num_rows, int64_t row_bytes, const int32_t* ids, int64_t num_ids,
                           void* out, void* hip_stream) {
  if (num_rows < 0 || row_bytes < 1 || row_bytes > (int64_t(1) << 20) || num_ids < 0) return GSS_ERR_INVALID_ARG;
  if (num_ids == 0) return GSS_OK;
  if (!ids || !out || (num_rows > 0 && !table)) return GSS_ERR_INVALID_ARG;
  const hipError_t e = launch_gather_rows(table, num_rows, row_bytes, ids, num_ids, out, (hipStream_t)hip_stream);
  return e == hipSuccess ? GSS_OK : GSS_ERR_DEVICE;
}

int32_t gss_pipeline_depth(const gss_sampler* s) { return s ? s->ring : 0; }

gss_status gss_cache_bytes(const gss_sampler* s, int64_t* out) {
  if (!s || !out) return GSS_ERR_INVALID_ARG;
  *out = s->cache_bytes;
  return GSS_OK;
}

gss_status gss_cache_read(gss_sampler* s, int32_t layer, int32_t relation, int32_t* out_rows) {
  if (!s || !out_rows || layer < 0 || layer >= s->num_tables || relation < 0 || relation >= s->R)
    return fail(s, GSS_ERR_INVALID_ARG, "cache_read: invalid argument");
  gss_status st = drain(s);              // every enqueued step has finished touching the tables
  if (st == GSS_OK) st = sync_all(s);
  if (st != GSS_OK) return st;
  const int64_t n = s->num_nodes[s->rel[relation].dst_type];
  if (n > 0) HIP_TRY(s, launch_cache_read(s->table[s->cur_set][layer][relation], s->row_of[relation], n, s->k, s->S, out_rows, s->stream));
  HIP_TRY(s, hipStreamSynchronize(s->stream));
  return GSS_OK;
}

gss_status gss_cache_checksum(gss_sampler* s, int32_t layer, int32_t relation, uint64_t* out) {
  if (!s || !out || layer < 0 || layer >= s->num_tables || relation < 0 || relation >= s->R)
    return fail(s, GSS_ERR_INVALID_ARG, "cache_checksum: invalid argument");
  gss_status st = drain(s);              // every enqueued step has finished touching the tables
  if (st == GSS_OK) st = sync_all(s);
  if (st != GSS_OK) return st;
  const int64_t n = s->num_nodes[s->rel[relation].dst_type];
  HIP_TRY(s, hipMemsetAsync(s->checksum.p, 0, 8, s->stream));
  if (n > 0) HIP_TRY(s, launch_cache_checksum(s->table[s->cur_set][layer][relation], s->row_of[relation], n, s->k, s->S, (unsigned long long*)s->checksum.p, s->stream));
  HIP_TRY(s, hipMemcpyAsync(out, s->checksum.p, 8, hipMemcpyDeviceToHost, s->stream));
  HIP_TRY(s, hipStreamSynchronize(s->stream));
  return GSS_OK;
}

gss_status gss_cache_checksum_static(gss_sampler* s, int32_t layer, int32_t relation, uint64_t* out_device, void* hip_stream) {
  if (!s || !out_device || layer < 0 || layer >= s->num_tables || relation < 0 || relation >= s->R)
    return fail(s, GSS_ERR_INVALID_ARG, "cache_checksum_static: invalid argument");
  if (((uintptr_t)out_device & 7u) != 0) return fail(s, GSS_ERR_INVALID_ARG, "cache_checksum_static: out_device is not 8-byte aligned");
  if (oldest_pending(s)) return fail(s, GSS_ERR_INVALID_ARG, "cache_checksum_static: collect the steps in flight first");
  const int64_t n = s->num_nodes[s->rel[relation].dst_type];
  if (n * (int64_t)s->k > (int64_t)GSS_CHECKSUM_STATIC_MAX_CELLS)
    return fail(s, GSS_ERR_INVALID_ARG, "cache_checksum_static: %lld cells exceed the static scratch (at most %lld)",
                (long long)(n * s->k), (long long)GSS_CHECKSUM_STATIC_MAX_CELLS);
  HIP_TRY(s, launch_cache_checksum_static(s->table[s->cur_set][layer][relation], s->row_of[relation], n, s->k, s->S,
                                          (unsigned long long*)out_device, (hipStream_t)hip_stream));
  return GSS_OK;
}

}  // extern "C"
