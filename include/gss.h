/*
 * gss.h — C ABI of the MI355X cache-backed multi-hop neighbor sampler
 * (GraphSnapShot's GraphSDSampler).
 *
 * The library keeps, per node, a cached snapshot of k neighbors over a CSR
 * graph resident in device memory, refreshes it according to one of the
 * paper's cache strategies and, per minibatch, draws the per-layer fanout
 * from the cached rows, dedupes/relabels the frontier and emits per-layer
 * bipartite blocks.  All steps run in HIP kernels on one GPU (gfx950).
 *
 * Conventions
 *   - fanouts are in LAYER order: index 0 is the input side (outermost hop);
 *     hop h (counted from the seeds) uses layer l = L-1-h  (SampleBlocks,
 *     "for l = L to 1", Alg. 2 / Alg. 3).
 *   - CSR row v of a relation lists the nodes v aggregates FROM; an emitted
 *     edge is (src = neighbor, dst = v).
 *   - "device" pointers are HIP device memory on the current device;
 *     "host" pointers are ordinary host memory.
 *   - Every random choice is a pure function of
 *     (rng_seed, step, layer, relation, node, slot, attempt) through
 *     Philox4x32-10, so results do not depend on scheduling.
 *
 * Threading: calls on one handle must not overlap.  gss_create and the cache
 * read-out run on config.hip_stream; the kernels of a step run on an internal
 * stream that is ordered after everything enqueued on config.hip_stream at the
 * time of the call (so seeds produced on that stream are ready), and gss_step /
 * gss_step_wait return only after the step is done.  The steps in flight are
 * software-pipelined: the phases of a step (per hop: sample, mark, emit) are
 * spread over consecutive launches, and each launch carries one phase of every
 * step in flight that the cache allows to run; results are those of running
 * the steps one after another.
 */
#ifndef GSS_H
#define GSS_H
#include <stddef.h>
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  GSS_OK = 0,
  GSS_ERR_INVALID_ARG = 1,    /* null pointer, size or parameter out of its documented range      */
  GSS_ERR_INVALID_GRAPH = 2,  /* indptr not monotone / ends wrong, neighbor id out of range        */
  GSS_ERR_INVALID_SEED = 3,   /* a seed id out of range or repeated (detected on the device)       */
  GSS_ERR_OOM = 4,            /* the allocator returned NULL                                        */
  GSS_ERR_DEVICE = 5,         /* a HIP call failed, or an internal capacity was exceeded           */
  GSS_ERR_STEP_ORDER = 6      /* step smaller than the previous step on this handle                */
} gss_status;

/* Cache strategies of the paper:
 *   FCR        "Fully Cache Refresh" (Alg. 3): every table is re-sampled when floor(step/R) changes.
 *   OTF        "On-The-Fly" refresh (Alg. 2 RefreshCache, OTF-Partial): each visited node's row has
 *              n_new = floor(gamma*k) slots redrawn before the draw, every T-th step.
 *   SHARED_OTF "Shared Cache Design" / OTF-Shared: one table serves all layers; layer l draws the
 *              priority ranks [off_l, off_l+f_l) of one per-(step,node) ranking (disjoint bands when
 *              the row is full), and a row is refreshed at most once per step.
 *   FBL        "Full Batch Load", the paper's baseline: no cache; every step draws a uniform
 *              min(deg,f)-subset straight from the adjacency (k only bounds the fanouts).
 *   SHARED_FCR "FCR with Shared Cache" (FCR-SC): the shared table with per-layer rank bands,
 *              re-sampled in full every R steps.
 *   OTF_FETCH  "OTF Fetch" (the static + dynamic mix of Alg. 1): the tables stay the static snapshot of
 *              gss_create; a node with more than k neighbors takes floor(delta*f) of its f neighbors
 *              fresh from the adjacency (excluding its cached picks) and the rest from its row;
 *              delta = refresh_fraction.
 *   OTF_LAYER  Alg. 2 read literally (RefreshCache redraws a gamma share of the whole layer cache every T
 *              steps): when floor(step/T) changes, every row of every per-layer table of a node with more than
 *              k neighbors has n_new = floor(gamma*k) slots redrawn, keyed by the first step of the new epoch;
 *              visits do not refresh.  T = refresh_period >= 1, gamma = refresh_fraction. */
typedef enum { GSS_MODE_FCR = 0, GSS_MODE_OTF = 1, GSS_MODE_SHARED_OTF = 2, GSS_MODE_FBL = 3,
               GSS_MODE_SHARED_FCR = 4, GSS_MODE_OTF_FETCH = 5, GSS_MODE_OTF_LAYER = 6 } gss_mode;

#define GSS_MAX_K 64           /* one cache row fits a wavefront (rows of up to 32 slots: half of one) */
#define GSS_MAX_LAYERS 8
#define GSS_MAX_NODE_TYPES 8
#define GSS_MAX_RELATIONS 16
#define GSS_MAX_IN_FLIGHT 32    /* upper bound of gss_pipeline_depth(): steps enqueued and not yet collected */

/* One relation (edge type) as CSR over its destination node type.  Arrays are BORROWED: the caller
 * keeps them alive and unmodified until gss_destroy.  Rows must hold no repeated neighbor id. */
typedef struct {
  int32_t src_type, dst_type;   /* row v (a dst_type node) lists its src_type neighbors           */
  int64_t nnz;                  /* number of CSR entries                                          */
  const void* indptr;           /* device, [num_nodes[dst_type] + 1], int32 or int64              */
  int32_t indptr_is_64;         /* 0: int32 indptr, 1: int64 indptr                               */
  const int32_t* indices;       /* device, [nnz], ids within src_type                             */
} gss_relation;

typedef struct {
  int32_t num_node_types;       /* 1 for a homogeneous graph                                      */
  const int64_t* num_nodes;     /* host, [num_node_types], each < 2^31                            */
  int32_t num_relations;
  const gss_relation* relations;/* host array of descriptors (the CSR arrays themselves: device)  */
} gss_graph;

/* Optional device allocator (e.g. a framework's caching allocator).  NULL => hipMalloc/hipFree. */
typedef void* (*gss_alloc_fn)(void* ctx, size_t bytes);
typedef void (*gss_free_fn)(void* ctx, void* ptr);

typedef struct {
  int32_t k;                    /* cache row width, 1..GSS_MAX_K (the paper's amplified fanout)   */
  gss_mode mode;
  int32_t num_layers;           /* L: number of per-layer tables (shared modes keep one, FBL none)  */
  double refresh_fraction;      /* gamma (OTF) / rho (shared): share of a row redrawn, in [0,1];
                                   n_new = floor(refresh_fraction*k + 1e-9).  OTF_FETCH: delta, the
                                   share of a draw fetched fresh, floor(delta*f + 1e-9) per node.  */
  int32_t refresh_period;       /* FCR modes: R >= 1.  OTF modes: T, refresh only when step % T == 0
                                   (values < 1 mean 1).                                           */
  uint64_t rng_seed;
  void* hip_stream;             /* hipStream_t; NULL = the default stream                         */
  gss_alloc_fn alloc;           /* may be NULL (then free must be NULL too)                       */
  gss_free_fn free;
  void* alloc_ctx;
  int32_t degree_threshold;     /* theta of the dense/sparse split ("Graph Splitting and Sampling
                                   Strategies"); < 0: no split, every node has a cache row.
                                   theta >= 0: per relation only nodes with deg(v) > theta keep a row
                                   (tables shrink to the dense nodes); the others are sampled like
                                   FBL, keyed by the step and the layer.  Ignored by GSS_MODE_FBL.  */
} gss_config;

/* Per layer and node type: the block's node sets. */
typedef struct {
  int32_t num_dst;              /* frontier size of this hop                                      */
  int32_t num_src;              /* num_dst + number of new distinct sampled ids                   */
  const int32_t* src_nodes;     /* device, [num_src] global ids within the type; the first num_dst
                                   entries are the dst nodes in frontier order, the rest are new
                                   ids in first-occurrence order                                  */
} gss_block_nodes;

/* Per layer and relation: the block's edges in (dst-major, slot-minor) order. */
typedef struct {
  int32_t num_edges;
  const int32_t* src_local;     /* device, [num_edges] index into src_nodes of the relation's src_type */
  const int32_t* dst_local;     /* device, [num_edges] index into the dst_type frontier (non-decreasing) */
} gss_block_edges;

/* Result of one step.  Host arrays are owned by the handle; device pointers and host arrays stay
 * valid until the next gss_step / gss_destroy on the handle.  Layer 0 is the input side. */
typedef struct {
  int32_t num_layers, num_node_types, num_relations;
  const gss_block_nodes* nodes; /* host, [num_layers * num_node_types], index l*num_node_types + t */
  const gss_block_edges* edges; /* host, [num_layers * num_relations],  index l*num_relations + r  */
  int64_t total_edges;          /* sum of num_edges over layers and relations                      */
} gss_blocks;

typedef struct gss_sampler gss_sampler;

/* StaticSample / Initialize (Alg. 1, Alg. 2): validates the graph, allocates the cache tables
 * ([num_nodes[dst_type], k] int32 per layer and relation, -1 padded) and fills every row with a
 * uniform min(deg,k)-subset of the node's adjacency (step word 0).  Blocks until the fill is done.
 * On error *out is NULL, nothing is leaked and gss_last_error(NULL) says why.  The library reads no environment
 * variable. */
gss_status gss_create(const gss_graph* graph, const gss_config* config, gss_sampler** out);

/* How the work is laid out - never what is computed: every field changes launch shapes, buffer layouts or memory use
 * only, and results stay bit-identical.  0 in a field = the library's own choice.  For memory budgeting (table_sets,
 * pipeline_depth), measurements and tests. */
typedef struct {
  int32_t dedupe_layout;        /* 1: direct (one 8-byte word per node and step in flight), 2: hashed (open addressing,
                                   16-byte entries, sized by the batch).  Default: direct up to 8 GiB of words.       */
  int32_t table_sets;           /* epoch-refreshed modes (FCR, SHARED_FCR, OTF_LAYER): 1..5 sets of tables.  A refresh
                                   writes a set that no step in flight reads; with one set it waits for them.  Default:
                                   2 + depth / period sets (3 at least, 5 at most) when they fit 1/8 of the free device
                                   memory at gss_create, else 3, else 2 (if they fit half of it), else 1.            */
  int32_t pipeline_depth;       /* 1..GSS_MAX_IN_FLIGHT: value of gss_pipeline_depth().  Default 4 L + 2 (twice that
                                   where a launch starts two steps; max(5, L + 2) with visit-once steps).  Every step in flight owns scratch, outputs and
                                   (direct layout) a dedupe table.                                                    */
  int32_t steps_per_tick;       /* 1 | 2: steps a launch starts (2 only in modes that never write a table)           */
  int32_t insert_phase;         /* 1: every hop gets a separate insert phase (visit-once steps: after the place phase,
                                   which they otherwise never get), 2: none does                                      */
  int32_t scan_phase;           /* 1: every hop gets a separate scan phase                                           */
  int32_t tick_build;           /* 1: every launch uses the step kernel's 8-workgroups-per-CU build, 2: none does     */
  uint32_t first_dedupe_version;/* start of each slot's dedupe-table version counter (tests of the wrap-around)       */
  int32_t visit_once;           /* SHARED_OTF on a graph with one relation.  Default: the steps of gss_step_async run as
                                   visit-once steps where their size allows (each node is visited by the first hop that
                                   reaches it and draws the picks of all its remaining hops there: one dependent launch
                                   per hop, the rest of the work trails behind in the launches of later steps), those of
                                   the blocking gss_step hop by hop (sample, mark, emit per hop).  1: visit-once also
                                   in gss_step, 2: always hop by hop                                                   */
  int32_t chain_workgroups;     /* visit-once steps: most workgroups of a chain phase, which stride over the hop's nodes
                                   (1..65536; default 4096)                                                           */
  int32_t lds_dedupe;           /* 1: the insert and place phases first dedupe each tile of 1024 picks in an LDS hash
                                   table and send only the tile's first pick of an id to the global dedupe table.
                                   Default off: measured slower (profiles/lds_dedupe_stage_ab.txt)                     */
  int32_t group_width;          /* lanes per frontier node in the sample phase.  Default: 32 (64 for rows of more than
                                   32 slots), and on one-relation graphs in FCR / OTF / OTF_LAYER / SHARED_FCR, in
                                   launches whose sample phases expect 16,384 nodes or more, 21 for rows of 17 to 20
                                   slots (three nodes per wavefront) and 16 for rows of up to 16 slots (four).
                                   32: never the narrow groups; 1: the narrow groups in every launch                  */
  int32_t reserved[4];          /* must be 0                                                                          */
} gss_tuning;

/* gss_create with the layout choices of `tuning` (NULL: all defaults, which is what gss_create passes). */
gss_status gss_create_tuned(const gss_graph* graph, const gss_config* config, const gss_tuning* tuning, gss_sampler** out);

/* SampleBlocks (Alg. 2 / Alg. 3): one minibatch.
 *   seeds      device, [num_seeds] distinct ids of node type seed_type (borrowed for the call)
 *   fanouts    host, [num_layers], layer order, 1 <= f <= k; shared modes: sum(f) <= k
 *   num_layers 1..config.num_layers
 *   step       0 <= step < 2^32, non-decreasing over the handle's life
 * Order per hop: (FCR: full refresh if the epoch changed) -> per frontier node read the cached row,
 * refresh it (OTF/SHARED), draw the fanout -> dedupe + relabel -> emit the block.  Returns after one
 * end-of-step readback of the counts and the error flag.  Host-detected errors leave the sampler
 * unchanged; GSS_ERR_INVALID_SEED / GSS_ERR_DEVICE are detected after the kernels ran and leave it
 * usable only for gss_destroy. */
gss_status gss_step(gss_sampler* s, const int32_t* seeds, int32_t num_seeds, int32_t seed_type,
                    const int32_t* fanouts, int32_t num_layers, int64_t step, gss_blocks* out);

/* The same step split in two so that the host never idles the GPU between minibatches:
 * gss_step_async validates, plans the step, issues ONE launch (the step's first phase together with the
 * next phase of every older step in flight) and returns at once - in the modes without any refresh (FBL, OTF_FETCH)
 * on graphs with one relation only every second call launches, for the two newest steps together; in SHARED_OTF,
 * whose steps are one dependent chain of launches (a step's sample or chain phases must all run before the next
 * step's first), as many launches as that chain has, so that it never waits for the host;
 * gss_step_wait issues the launches the OLDEST step in flight still needs, blocks until it has finished and
 * fills *out exactly like gss_step.  A step with P phases (3 to 4 per hop) completes after P launches, so a caller
 * that keeps gss_pipeline_depth(s) steps in flight pays one launch (or half a launch) per step.  At most gss_pipeline_depth(s) steps may be in flight (one more gss_step_async returns
 * GSS_ERR_INVALID_ARG); `seeds` must stay valid until the step has been waited for; the blocks of a step
 * stay valid until gss_pipeline_depth(s) - 1 further steps have been enqueued.  Device-detected errors surface in
 * the wait.  gss_step(...) == gss_step_async(...) followed by gss_step_wait(...). */
gss_status gss_step_async(gss_sampler* s, const int32_t* seeds, int32_t num_seeds, int32_t seed_type,
                          const int32_t* fanouts, int32_t num_layers, int64_t step);
gss_status gss_step_wait(gss_sampler* s, gss_blocks* out);

/* The number of steps the handle can hold in flight (<= GSS_MAX_IN_FLIGHT), which is also the depth a caller
 * should keep for one launch per step: a few more than the phases of a num_layers-hop step.
 * Fixed at gss_create.  0 for a NULL handle. */
int32_t gss_pipeline_depth(const gss_sampler* s);

/* Frees every device and host buffer of the handle (after synchronising its stream). NULL is allowed. */
gss_status gss_destroy(gss_sampler* s);

/* Test / checkpoint surface: copy cache table (layer, relation) as a dense [num_nodes[dst_type], k]
 * int32 array (-1 padded; rows of nodes without a cache row are all -1) into device memory `out_rows`.  Shared modes have one table per relation:
 * layer must be 0; FBL has none (GSS_ERR_INVALID_ARG).  Blocks until the copy is done. */
gss_status gss_cache_read(gss_sampler* s, int32_t layer, int32_t relation, int32_t* out_rows);

/* 64-bit order-independent checksum of the same dense table: the wrapping sum over cells c (row-major
 * index) of mix(c * 0x9E3779B97F4A7C15 + (uint32)value), mix = the splitmix64 finaliser.  *out: host. */
gss_status gss_cache_checksum(gss_sampler* s, int32_t layer, int32_t relation, uint64_t* out);

/* gss_cache_checksum for callers that cannot allocate device memory or wait for the device: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  The same checksum of table (layer, relation), written
 * to *out_device (device memory, 8 bytes, 8-byte aligned) by two kernels enqueued on hip_stream (hipStream_t; NULL = the
 * default stream); the call does not wait for them, allocates nothing and calls no allocating routine.  The per-chunk
 * partial sums live in a static device array of the library (128 KB on every GPU it runs on, held until the process
 * ends), which bounds the table: num_nodes[dst_type] * k <= GSS_CHECKSUM_STATIC_MAX_CELLS, else GSS_ERR_INVALID_ARG.
 * All calls on one GPU share that array: calls that overlap on one GPU (different streams or threads) race.
 * No step may be in flight on the handle (GSS_ERR_INVALID_ARG otherwise), and hip_stream must be ordered after the
 * handle's earlier work by the caller (gss_step / gss_step_wait return only after a step's kernels are done). */
#define GSS_CHECKSUM_STATIC_MAX_CELLS (1ll << 28)
gss_status gss_cache_checksum_static(gss_sampler* s, int32_t layer, int32_t relation, uint64_t* out_device, void* hip_stream);

/* Device memory held by the cache itself, in bytes: tables (the epoch-refreshed modes keep up to five sets of
 * them, so that a refresh never waits for steps in flight: as many as the epochs the steps in flight can span plus
 * one, three at least, when that takes at most 1/8 of the free device memory at gss_create, else two, else one),
 * plus (with a degree threshold) the node -> row maps, plus the shared-mode refresh stamps, plus (epoch-refreshed
 * modes) the list of the nodes whose rows a refresh recomputes.  *out: host. */
gss_status gss_cache_bytes(const gss_sampler* s, int64_t* out);

/* Feature gather for a block's src_nodes (the value side of the K-V cache of "System Components": keys are node
 * ids, values the embeddings H_v): out[i] = table[ids[i]] for i < num_ids.
 *   table    device, [num_rows] rows of row_bytes bytes each (any element type; 1 <= row_bytes <= 2^20)
 *   ids      device, [num_ids] int32; an id outside [0, num_rows) yields a row of zero bytes
 *   out      device, [num_ids] rows of row_bytes bytes, written in full
 * Enqueued on hip_stream (hipStream_t; NULL = the default stream) and not waited for; nothing is allocated.
 * Rows are moved with 16-byte accesses when table, out and row_bytes are multiples of 16 (else 8, 4 or 1). */
gss_status gss_gather_rows(const void* table, int64_t num_rows, int64_t row_bytes, const int32_t* ids, int64_t num_ids,
                           void* out, void* hip_stream);

/* Human-readable description of the last error on the handle ("" if none). Never NULL.
 * With s == NULL: why the calling thread's last gss_create failed ("" if it did not). */
const char* gss_last_error(const gss_sampler* s);

/* Kernel timing (measurement aid; off by default).  While enabled, every kernel launch of the handle is
 * launched with a start and a stop event attached to the dispatch (its own begin-to-end time).  gss_profile_read waits for the stream, adds the
 * elapsed time of every bracket recorded since the previous read to per-kernel totals and returns them:
 * kernel ids: 0 fill_full (FCR refresh), 1 step_tick (one phase of every ready step in flight).  `ms` and
 * `launches` are host arrays of GSS_NUM_KERNELS entries (totals since enabling). Enabling resets the totals. */
#define GSS_NUM_KERNELS 2
gss_status gss_profile_enable(gss_sampler* s, int32_t on);
gss_status gss_profile_read(gss_sampler* s, double* ms, int64_t* launches);

/* Library version string. */
const char* gss_version(void);

#ifdef __cplusplus
}
#endif
#endif
