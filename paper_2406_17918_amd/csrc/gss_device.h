// Shared declarations between the kernels (gss_kernels.hip) and the host step driver (gss_api.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gss.h"
#include "gss_schedule.h"

namespace gss {

constexpr uint32_t EDGE_BIT = 0x80000000u;   // order words: < EDGE_BIT frontier index, >= EDGE_BIT pick slot
constexpr int TILE = 1024;                    // pick slots per tile (mark and emit phases)
constexpr int TILE_THREADS = 256;
constexpr int EMIT_SCAN_MAX_TILES = 4096;       // up to this many tiles per hop, the emit phase scans the tile totals itself

enum Purpose : uint32_t { P_FILL_FULL = 0, P_FILL_PART = 1, P_EVICT = 2, P_PICK = 3, P_FBL = 4, P_FETCH = 5 };

// device state words (int32)
enum : int { ST_ERROR = 0, ST_TICKET = 1, ST_COUNTS = 4 };
enum : int {
  ERR_SEED_RANGE = 1, ERR_SEED_DUP = 2, ERR_TABLE_FULL = 4, ERR_TABLE_MISS = 8, ERR_GRAPH = 16,
  ERR_REJECT_OVERFLOW = 32
};

struct __attribute__((aligned(16))) HashEntry {
  uint64_t keyver;   // (version << 32) | key
  uint64_t val;      // (~version << 32) | order word
};
struct DedupeTable {
  uint64_t* direct;    // non-null: one word per node, indexed by key (direct layout)
  HashEntry* entries;  // hashed layout
  uint64_t mask;       // hashed layout: capacity - 1 (capacity is a power of two)
};

// Per relation, fixed for the life of the sampler (only the sample phase reads it).  Small graphs carry it
// in the kernel arguments; larger ones read it from device memory, which keeps their slices small enough
// for six (up to 8 relations) or four of them to fit into one launch.
struct RelConst {
  const void* indptr;
  const int32_t* indices;
  long long* stamp;       // shared mode: last refresh step per row (-1 = never)
  const int32_t* row_of;  // degree split: node -> table row, -1 for nodes without a row; null: row = node
  int32_t is64;
  int32_t n_dst;
};
// Per relation and hop.
struct RelParam {
  int32_t* table;         // cache table used by this hop: [rows, S]
  int32_t* src_local;     // this hop's COO outputs
  int32_t* dst_local;
  int32_t slot_base;      // first pick slot of the relation in this hop (multiple of TILE)
  int16_t src_type, dst_type;
};

struct TypeParam {
  const int32_t* frontier;  // this hop's dst nodes of the type
  int32_t* src_nodes;       // this hop's output
  uint32_t key_off;         // offset that makes (type, id) a single 32-bit table key
  int32_t n_nodes;
  int32_t count_override;   // hop 0: frontier size known on the host; later hops: -1 (read from state)
  int32_t frontier_cap;     // allocated length of `frontier` (an upper bound of the frontier size)
};

// A step is a chain of phases: per hop sample -> mark -> [scan ->] emit.  The kernels of one phase
// are latency-bound and leave most of the chip idle, so ONE launch ("tick") carries a phase of every
// step in flight that is ready for it: one "slice" each, with its own arguments and its own range of workgroups.
// Stream order between ticks provides every dependency; the host only picks which phases share a tick.
// (enum Phase: gss_schedule.h)

// Arguments of one slice: one phase of one hop of one step.
struct HopCommon {
  DedupeTable ht;
  int32_t* state;
  int32_t* state_host;      // pinned host copy of `state`, written by the last hop's emit phase (or null)
  int32_t* picks;           // [slots] sampled global id or -1
  uint32_t* order;          // [slots] order word of the pick's id
  uint32_t* ranks;          // [slots] rank among firsts (lo 16) / among edges (hi 16) within the tile
  int32_t* partial_first;   // [tiles]
  int32_t* partial_edge;
  union {
    struct {                // scan and emit phases
      int32_t* first_off;
      int32_t* edge_off;
    };
    struct {                // place phase of a visit-once step: the hop's part of the holding area, the step's visit
      const int32_t* held;  // table (node -> holding index, see ChainArgs)
      const uint64_t* visit;
    };
  };
  int32_t phase;            // Phase
  int32_t gx, gy, gxd, gyd; // the slice's workgroups: gy rows of gx, then gyd rows of gxd
  int32_t R, T;
  int32_t hop, f, k, S;
  int32_t n_new, mode, refresh_now, band_offset;
  int32_t num_tiles_ub, edge_count_off;
  int32_t scan_in_emit, state_words;
  int32_t shared, layer;        // shared: one table for all layers, per-layer rank bands; layer: l of this hop
  int32_t insert_split, slot;   // the hop has an insert phase: the sample phase leaves the picks' table inserts to it; slot: the step's slot
  uint32_t ver, step, layer_word, seed_lo, seed_hi;
  // (visit-once steps: the version of the step's visit table entries is that of its hop 0 dedupe entries)
  __host__ __device__ uint32_t visit_ver() const { return ver - (uint32_t)hop; }
};
// Visit-once steps (one table for all hops, refreshed per visit, one relation).  The chain phase of hop c visits the nodes
// that hop c reaches for the first time in this step and draws, from the node's one (refreshed) row, the picks of ALL its
// remaining hops c .. L-1.  A visited node gets a "holding index" Q: seeds Q = seed index; a node first reached through
// pick j of hop c-1 of the node with index Qp: Q = V[c-1] + Qp * f[c-1] + j, with V[0] = number of seeds and
// V[h+1] = V[h] * (1 + f[h]) - an index space with holes, laid out by host-known bounds.  The picks of hop h of node
// Q are held at held[off[h] + Q * f[h] + 0 .. f[h]) (picks first, then -1).
//   visit[v]       = (~ver << 32) | Q, claimed with a compare-and-swap: whichever pick comes first visits the node
//   list h >= 1    the nodes first reached by hop h, as (Q << 32) | v, appended by the chain phase of hop h-1 while it
//                  looks up its own hop's picks.  CHAIN_SEGS segments with a counter each (appends to one counter would
//                  serialise); the pair of nodes a wavefront works on appends to segment (item index / 2) % CHAIN_SEGS,
//                  so a segment of list h+1 holds at most ceil(V[h] / (2 CHAIN_SEGS)) * 2 * f[h] entries.
// The counters come in two sets: a step's first chain phase clears the set that the slot's next step will use.
// Nothing here decides an output order: the place / mark / emit phases do that from the frontier, exactly as for
// other steps.  Which of several picks of a node claims it only decides the node's Q and list position, which no
// output shows.
constexpr int CHAIN_MAX_HOPS = 4;
constexpr int CHAIN_SEGS = 32;
constexpr int CHAIN_COUNT_STRIDE = 32;       // words between two counters: one 128-byte line each (atomics on one line serialise)
constexpr int CHAIN_TICK_SLICES = 8;        // most slices of a launch of the build that runs visit-once steps
struct ChainArgs {
  int32_t* held;
  uint64_t* visit;
  uint64_t* list;
  uint32_t* counts;                   // [CHAIN_MAX_HOPS][CHAIN_SEGS] of this step, CHAIN_COUNT_STRIDE words apart
  uint32_t* counts_next;              // the other set
  uint32_t off[CHAIN_MAX_HOPS];       // start of hop h's picks in `held`
  int32_t V[CHAIN_MAX_HOPS];          // size of hop h's holding index space
  uint32_t loff[CHAIN_MAX_HOPS];      // start of list h in `list`
  uint32_t lcap[CHAIN_MAX_HOPS];      // entries a segment of list h can hold
  uint32_t fbl[CHAIN_MAX_HOPS];       // per hop: fanout | first rank of its band << 8 | layer << 16 (whole words: the
  int32_t L;                          // kernel reads its arguments with scalar loads, which have no byte form)
  __host__ __device__ int f(int h) const { return (int)(fbl[h] & 0xFFu); }
  __host__ __device__ int band(int h) const { return (int)((fbl[h] >> 8) & 0xFFu); }
  __host__ __device__ uint32_t layer(int h) const { return (fbl[h] >> 16) & 0xFFu; }
};
// Kernel arguments are limited to 4 KB, so the relation / node type arrays come in three sizes.
template <int MAXR, int MAXT>
struct HopParamsT : HopCommon {
  static constexpr int MAX_R = MAXR, MAX_T = MAXT;
  RelParam rel[MAXR];
  TypeParam type[MAXT];
  const RelConst* relc;     // device memory, [R]
  __host__ __device__ const RelConst& rc(int r) const { return relc[r]; }
  void set_consts(const RelConst*, const RelConst* device) { relc = device; }
};
struct HopParamsMono : HopCommon {      // one relation, one node type: twelve slices fit into a launch
  static constexpr int MAX_R = 1, MAX_T = 1;
  RelParam rel[1];
  TypeParam type[1];
  RelConst relc[1];
  __host__ __device__ const RelConst& rc(int) const { return relc[0]; }
  void set_consts(const RelConst* host, const RelConst*) { relc[0] = host[0]; }
};
struct HopParamsSmall : HopCommon {
  static constexpr int MAX_R = 2, MAX_T = 2;
  RelParam rel[2];
  TypeParam type[2];
  RelConst relc[2];         // in the kernel arguments: no dependent load before the first row read
  __host__ __device__ const RelConst& rc(int r) const { return relc[r]; }
  void set_consts(const RelConst* host, const RelConst*) { relc[0] = host[0]; relc[1] = host[1]; }
};
using HopParams = HopParamsT<GSS_MAX_RELATIONS, GSS_MAX_NODE_TYPES>;
using HopParamsMid = HopParamsT<8, 4>;
// (Samplers that run visit-once steps use a build of the step kernel of their own, whose launches carry the arguments
// of a chain slice - at most one each, as chain phases of different steps never share a launch.  The other builds
// hold none of that code: it costs them registers.)
struct HopParamsStaged : HopParamsMono {};    // the same slice in the build whose insert phases hold the LDS stage of the dedupe
struct HopParamsChain : HopParamsStaged {};   // ... and in launches that also carry a chain's arguments
template <class HP> struct ChainOf { static constexpr bool HAS_CHAIN = false; };
template <> struct ChainOf<HopParamsChain> { static constexpr bool HAS_CHAIN = true; ChainArgs chain; };
template <class HP, int D>
struct TickT : ChainOf<HP> {
  using Slice = HP;
  static constexpr int SLICES = D;
  HP s[D];
  int32_t end[D];           // running total of the slices' workgroups: slice i owns [end[i-1], end[i])
};
// One relation, one node type, more than twelve slices: the compact form.  What every slice of the sampler
// shares travels once per launch (MonoShared), what all phases of a step share - the scratch of its slot - is
// read from a device table (SlotConst, written when a slot's buffers change), and a slice (MonoSlice) carries
// only what belongs to its hop and phase: 24 slices fit into a launch, so a tick can carry two steps' phases.
struct SlotConst {
  DedupeTable ht;
  int32_t* state;
  int32_t* state_host;
  int32_t* picks;
  uint32_t* order;
  uint32_t* ranks;
  int32_t* partial_first;
  int32_t* partial_edge;
  int32_t* first_off;
  int32_t* edge_off;
};
struct MonoShared {
  RelConst relc;
  const SlotConst* slots;   // device memory, [slots of the sampler]
  uint32_t key_off;
  int32_t n_nodes;
  int32_t k, S, mode, shared, state_words, edge_count_off;
  uint32_t seed_lo, seed_hi;
};
struct MonoSlice {
  int32_t* table;
  int32_t* src_local;
  int32_t* dst_local;
  const int32_t* frontier;
  int32_t* src_nodes;
  int32_t count_override, frontier_cap;
  int32_t num_tiles_ub, gx, gxd, band_offset;
  uint32_t ver, step, layer_word;
  uint8_t slot, phase, hop, layer, f, n_new, refresh_now, scan_in_emit, insert_split, publish, gy, gyd;
};
template <int D>
struct TickMono {
  static constexpr int SLICES = D;
  MonoShared h;
  MonoSlice s[D];
  int32_t end[D];
};
constexpr int TICK_MONO_SLICES = 24;
constexpr int TICK_MAX_SLICES = 24;           // most slices of a launch in any layout
constexpr int EMIT_OWN_TILES = 16;            // tiles one emit workgroup owns at most when it scans the tile totals in LDS
// Largest number of slices one launch can carry for a graph with R relations and T node types.
int tick_capacity(int R, int T);

struct FillParams {
  const void* indptr;
  const int32_t* indices;
  int32_t* table[GSS_MAX_LAYERS];
  const int32_t* src_table[GSS_MAX_LAYERS];   // non-null: partial refresh (n_new slots per row) of these rows instead of a fill
  uint32_t layer_word[GSS_MAX_LAYERS];
  int32_t* state;
  const int32_t* row_of;  // degree split: node -> table row or -1 (no row); null: row = node
  int64_t n_dst;
  int32_t ntab, is64, k, S;
  int32_t n_new, pad_;
  uint32_t relation, stepword, seed_lo, seed_hi;
};

// Optional per-launch timing (measurement aid): the launch attaches the two events to the dispatch
// itself, so their difference is the kernel's own start-to-end time.
enum KernelId : int { KID_FILL_FULL = 0, KID_STEP_TICK = 1, KID_COUNT = 2 };
struct LaunchTimer {
  virtual ~LaunchTimer() = default;
  virtual bool bracket(int kernel_id, hipEvent_t* start, hipEvent_t* stop) = 0;   // false: launch untimed
};

hipError_t launch_fill_full(const FillParams& P, hipStream_t st, LaunchTimer* timer);
// The rows of the listed nodes only (those with more than k neighbors), for a table set filled before.
hipError_t launch_fill_heavy(const FillParams& P, const int32_t* heavy, int64_t nheavy, hipStream_t st, LaunchTimer* timer);
hipError_t launch_list_from_map(const int32_t* map, int64_t n, int32_t* list, hipStream_t st);
// One tick: a single launch over n <= tick_capacity slices.  `relc_host` / `relc_dev`: the R RelConst records
// (host copy, device copy).  `done`, if non-null, completes when the launch has.  `dense`: use the build of the kernel
// that fits eight workgroups on a CU instead of seven (for launches of several times the chip's capacity; the compact
// launch of one-relation graphs has no such build).  `chain_build`: the sampler runs visit-once steps (one relation; at
// most CHAIN_TICK_SLICES slices per launch); `chain`: the arguments of the launch's chain slice, if it has one.
// `width`: lanes per frontier node in the sample phase - 64 for rows of more than 32 slots, 32, or (one-relation graphs,
// at most 12 slices, no chain, no LDS stage) 21 / 16 for rows of up to 20 / 16 slots; the grids of the sample slices must
// have been sized for it (256 / 64 * (64 / width) nodes per workgroup).
hipError_t launch_tick(const HopParams* slices, int n, const RelConst* relc_host, const RelConst* relc_dev,
                       const SlotConst* slots_dev, bool chain_build, const ChainArgs* chain, hipStream_t st, LaunchTimer* timer,
                       hipEvent_t done, bool dense, int width);
hipError_t launch_validate_graph(const void* indptr, int is64, int64_t n_dst, const int32_t* indices, int64_t nnz,
                                 int64_t n_src, int32_t* state, hipStream_t st);
hipError_t launch_cache_read(const int32_t* table, const int32_t* row_of, int64_t n, int k, int S, int32_t* out,
                             hipStream_t st);
hipError_t launch_cache_checksum(const int32_t* table, const int32_t* row_of, int64_t n, int k, int S,
                                 unsigned long long* out, hipStream_t st);
// The checksum into a device word, with partial sums in the library's static scratch array: allocates nothing.
// n * k must not exceed GSS_CHECKSUM_STATIC_MAX_CELLS.
hipError_t launch_cache_checksum_static(const int32_t* table, const int32_t* row_of, int64_t n, int k, int S,
                                        unsigned long long* out, hipStream_t st);
// Degree split: row_of[v] = rank of v among the nodes with deg > theta, or -1; *num_rows = their number.
// `chunk_counts` is scratch of ceil(n / 1024) + 1 words.
hipError_t launch_build_row_map(const void* indptr, int is64, int64_t n, int32_t theta, int32_t* chunk_counts,
                                int32_t* row_of, int32_t* num_rows, hipStream_t st);
hipError_t launch_fill_i64(long long* p, int64_t n, long long value, hipStream_t st);
hipError_t launch_gather_rows(const void* table, int64_t num_rows, int64_t row_bytes, const int32_t* ids, int64_t num_ids,
                              void* out, hipStream_t st);

}  // namespace gss
