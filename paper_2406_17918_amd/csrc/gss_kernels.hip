// HIP kernels of the cache-backed multi-hop neighbor sampler, written for gfx950 (CDNA4, wave64).
//
// Kernel map:
//   fill_full_kernel   StaticSample / Initialize (Alg. 1, Alg. 2) and FCR CacheRefresh (Alg. 3):
//                      one half-wavefront per cache row, all per-layer tables of a relation in one pass.
//   step_tick_kernel   one launch carries one phase of every step in flight that is ready for it
//                      (the slices own consecutive ranges of a one-dimensional grid).  The phases of a hop:
//     sample  per frontier node (one half-wavefront): read the cached row, partial refresh (Alg. 2
//             RefreshCache / OTF-Partial / shared rho-refresh), draw the fanout (SampleFromCache),
//             write the picks and insert them into the dedupe table;
//     mark    per pick: look up the table, flag first occurrences, per-tile ranks and tile totals;
//     scan    (only hops with more than EMIT_SCAN_MAX_TILES tiles) tile totals -> offsets, one workgroup;
//     emit    per pick: local ids, COO in (dst-major, slot-minor) order, new src_nodes, counts.
//
// Nothing here is a dense contraction, so no MFMA: the work is row reads, keyed integer hashing
// (Philox4x32-10), group-level ranking through LDS broadcasts and ballots, and atomics on the dedupe table.
#include <hip/hip_ext.h>

#include <cstring>
#include <type_traits>

#include "gss_device.h"

namespace gss {

// ------------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11).  One block = four 32-bit words.
//   draw   x64 = (w1 << 32) | w0
//   the two per-slot draws of a visited node share one block (purpose word 2):
//   EVICT reads words (0,1), PICK reads words (2,3).
//   priority(index) = x64 with its low 16 bits replaced by the index (no ties).
// ------------------------------------------------------------------------------------------
struct Block4 { uint32_t w0, w1, w2, w3; };

// a ^ b ^ c in one instruction (the three-input bitwise op of gfx950; 0x96 is the truth table of the three-way xor):
// written out, the compiler emits two xors per word and round, a quarter of a block's vector instructions
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) {
  return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

__device__ __forceinline__ Block4 philox4x32_10(uint32_t k0, uint32_t k1, uint32_t c0, uint32_t c1,
                                                uint32_t c2, uint32_t c3) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;   // one 32x32->64 multiply gives hi and lo
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    c0 = xor3((uint32_t)(p1 >> 32), c1, k0);
    c1 = (uint32_t)p1;
    c2 = xor3((uint32_t)(p0 >> 32), c3, k1);
    c3 = (uint32_t)p0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return Block4{c0, c1, c2, c3};
}

struct DrawKey {
  uint32_t k0, k1;     // rng_seed lo / hi
  uint32_t node;       // counter word 0
  uint32_t step;       // counter word 2
  uint32_t tag;        // layer << 8 | relation << 16 (the purpose is OR-ed in per draw)
};
__device__ __forceinline__ Block4 draw_block(const DrawKey& K, uint32_t purpose, uint32_t index, uint32_t attempt) {
  return philox4x32_10(K.k0, K.k1, K.node, index | (attempt << 16), K.step, K.tag | purpose);
}
__device__ __forceinline__ uint64_t lo64(const Block4& b) { return ((uint64_t)b.w1 << 32) | b.w0; }
__device__ __forceinline__ uint64_t hi64(const Block4& b) { return ((uint64_t)b.w3 << 32) | b.w2; }
__device__ __forceinline__ uint64_t priority(uint64_t x64, uint32_t index) { return (x64 & ~0xFFFFull) | index; }
// floor(x64 * m / 2^64) for m < 2^32
__device__ __forceinline__ uint32_t below(uint64_t x64, uint32_t m) {
  const uint64_t t = (uint64_t)(uint32_t)x64 * m;
  const uint64_t u = (x64 >> 32) * m + (t >> 32);
  return (uint32_t)(u >> 32);
}
constexpr int ITEMS_PER_THREAD = TILE / TILE_THREADS;   // consecutive pick slots a thread of a tile phase owns
constexpr uint64_t PRIO_NONE = ~0ull;   // larger than every real priority (their low 16 bits are < 64)

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & 63u); }
struct Wg { int x, y; };   // position of the workgroup within its slice's grid

__device__ __forceinline__ int64_t load_indptr(const void* indptr, int is64, int64_t v) {
  return is64 ? ((const int64_t*)indptr)[v] : (int64_t)((const int32_t*)indptr)[v];
}

// ------------------------------------------------------------------------------------------
// Groups of W lanes.  A cache row of k <= 32 slots occupies half a wavefront (W = 32), and a
// wavefront works on two nodes at once (every Philox block and every compare is shared by both);
// rows of 33 .. 64 slots take the whole wavefront (W = 64).
// Lanes of a group talk through a small LDS scratch: a lane writes its item, every lane then reads
// item i at the same address (an LDS broadcast), which replaces per-iteration cross-lane moves.
// LDS operations of one wavefront execute in order, so no barrier is needed inside a group; the
// accesses are volatile to keep the compiler from reordering them.
// ------------------------------------------------------------------------------------------
template <int W>
struct GroupLdsT {
  uint64_t prio[2 * W];  // priorities by slot, or by adjacency position in the k < deg < 2k regime
  uint64_t ab[2 * W];    // lo: value fixed in the slot (or -1); hi: this round's candidate (or -2)
  int32_t out[2 * W];    // values compacted in position order
};
template <int W> using MaskT = typename std::conditional<W == 64, uint64_t, uint32_t>::type;   // one bit per lane of a group
__device__ __forceinline__ int mask_popc(uint32_t m) { return __popc(m); }
__device__ __forceinline__ int mask_popc(uint64_t m) { return __popcll((unsigned long long)m); }
__device__ __forceinline__ int mask_ffs(uint32_t m) { return __ffs((int)m); }
__device__ __forceinline__ int mask_ffs(uint64_t m) { return __ffsll((unsigned long long)m); }
template <int W>
struct GrpT {
  static constexpr int WIDTH = W;
  static constexpr int PER_WAVE = 64 / W;               // groups of a wavefront (W = 21: three, and lane 63 has no group)
  static constexpr int PER_WG = (TILE_THREADS / 64) * PER_WAVE;   // groups of a workgroup
  static constexpr bool POW2 = (W & (W - 1)) == 0;
  static constexpr int LOG2_WIDTH = W == 64 ? 6 : (W == 32 ? 5 : (W == 16 ? 4 : (W == 8 ? 3 : 0)));
  using Mask = MaskT<W>;
  // LDS address space made explicit: volatile accesses through a generic pointer would be emitted as
  // flat memory instructions instead of ds_read / ds_write.
  typedef __attribute__((address_space(3))) volatile GroupLdsT<W>* LdsPtr;
  int sub;                 // lane within the group
  int half;                // group within the wavefront
  bool idle;               // a lane beyond the wavefront's last group (only when W does not divide 64): it takes no part
  LdsPtr L;
  __device__ __forceinline__ void init(GroupLdsT<W>* lds) {        // `lds`: one scratch per group of the workgroup
    if constexpr (W == 32 || W == 64) {
      sub = (int)(threadIdx.x & (unsigned)(W - 1));
      half = W == 32 ? (int)((threadIdx.x >> 5) & 1u) : 0;
      idle = false;
      L = (LdsPtr)&lds[threadIdx.x / (unsigned)W];
    } else {
      const int lane = (int)(threadIdx.x & 63u);
      half = lane / W;
      idle = half >= PER_WAVE;
      if (idle) half = PER_WAVE - 1;
      sub = lane - half * W;
      L = (LdsPtr)&lds[(int)(threadIdx.x >> 6) * PER_WAVE + half];
    }
  }
  __device__ __forceinline__ int index_in_workgroup() const { return (int)(threadIdx.x >> 6) * PER_WAVE + half; }
  __device__ __forceinline__ Mask below() const { return ((Mask)1 << sub) - (Mask)1; }          // the lanes before this one
  __device__ __forceinline__ bool in(Mask m) const { return ((m >> sub) & (Mask)1) != 0; }       // is this lane's bit set
  __device__ __forceinline__ static Mask all() { return (W == 64 || W == 32) ? ~(Mask)0 : (Mask)(((Mask)1 << (W & 31)) - (Mask)1); }
  __device__ __forceinline__ static Mask first(int n) { return n >= W ? all() : (((Mask)1 << n) - (Mask)1); }
};
using GroupLds = GroupLdsT<32>;
using Grp = GrpT<32>;
using GroupLdsPtr = Grp::LdsPtr;
template <int W>
__device__ __forceinline__ MaskT<W> grp_ballot(const GrpT<W>& G, bool pred) {
  const uint64_t b = __ballot(pred);
  if constexpr (W == 64) return b;
  else if constexpr (W == 32) return G.half ? (uint32_t)(b >> 32) : (uint32_t)b;
  else return (uint32_t)(b >> (G.half * W)) & GrpT<W>::all();
}
__device__ __forceinline__ uint32_t below_mask(int sub) { return (1u << sub) - 1u; }

// number of the n priorities in LDS smaller than p (all priorities are distinct)
template <int W>
__device__ __forceinline__ int grp_rank(const GrpT<W>& G, int n, uint64_t p) {
  int r = 0;
#pragma unroll 4
  for (int i = 0; i < n; ++i) r += (G.L->prio[i] < p) ? 1 : 0;
  return r;
}
// The same over the first n entries with n the same in every lane of the wavefront (a slot count of the launch, not of
// the node): the loop counter stays in scalar registers and four entries are compared per round.  Entries from n up to the
// next multiple of four must hold PRIO_NONE (every lane of a group stores its slot's priority, PRIO_NONE beyond the row).
template <int W>
__device__ __forceinline__ int grp_rank_uniform(const GrpT<W>& G, int n, uint64_t p) {
  const int n4 = (__builtin_amdgcn_readfirstlane(n) + 3) & ~3;
  int r = 0;
  for (int i = 0; i < n4; i += 4) {
    const uint64_t q0 = G.L->prio[i], q1 = G.L->prio[i + 1], q2 = G.L->prio[i + 2], q3 = G.L->prio[i + 3];
    r += (q0 < p) ? 1 : 0;          // (one compare and one add-with-carry each)
    r += (q1 < p) ? 1 : 0;
    r += (q2 < p) ? 1 : 0;
    r += (q3 < p) ? 1 : 0;
  }
  return r;
}
template <int W>
__device__ __forceinline__ void grp_rank2(const GrpT<W>& G, int n, uint64_t p0, uint64_t p1, int& r0, int& r1) {
  r0 = 0; r1 = 0;
#pragma unroll 4
  for (int i = 0; i < n; ++i) {
    const uint64_t q = G.L->prio[i];
    r0 += (q < p0) ? 1 : 0;
    r1 += (q < p1) ? 1 : 0;
  }
}

// Round-major rejection fill.  Slots of `pend` need an id, slots of `fixed` hold one in `val`.
// In round a every pending slot j draws pos = below(deg; index=j, attempt=a) and proposes
// adj[pos]; it is accepted unless the id is already in the row or proposed by a lower pending slot
// in the same round (which is what slot-ascending sequential processing of a round yields).
// FEW: few slots are pending (a partial refresh): instead of every lane scanning all k slots, the
// group walks over the pending slots, and every lane compares its own id with that slot's proposal.
// From eight pending slots down, several rounds are drawn at once (below).
template <bool FEW, int W>
__device__ __forceinline__ int grp_rejection_fill(const GrpT<W>& G, MaskT<W> pend, MaskT<W> fixed, int val, int k,
                                                  const int32_t* __restrict__ adj, uint32_t deg,
                                                  const DrawKey& K, uint32_t purpose, int32_t* state) {
  using Mask = MaskT<W>;
  constexpr int GRP = W;
  for (uint32_t a = 0; pend != 0; ++a) {
    if (a >= 65536u) {   // acceptance probability is > 1/2 per draw: unreachable for a simple graph
      if (G.sub == 0) atomicOr(&state[ST_ERROR], ERR_REJECT_OVERFLOW);
      break;
    }
    const int np = mask_popc(pend);
    if (GrpT<W>::POW2 && !FEW && np <= 8 && a + (uint32_t)GRP <= 65536u) {   // (the lane -> (slot, round) split below wants a power of two)
      // Few slots pending: a round would run the whole Philox block and a trip to the adjacency for a handful of
      // lanes.  Instead the 32 lanes compute the proposals of A = 16 / 8 / 4 consecutive rounds at once (lane ->
      // (pending slot q, round t); a proposal is a pure function of slot and round), and the rounds are then
      // resolved in order from LDS: same outcome, one block and one trip for all of them.
      const int lg = np <= 2 ? 1 : (np <= 4 ? 2 : 3);
      const int A = GRP >> lg;
      const int q = G.sub >> (GrpT<W>::LOG2_WIDTH - lg), t = G.sub & (A - 1);
      Mask m = pend;
      for (int i = 0; i < q; ++i) m &= m - (Mask)1;                  // drop the q lowest pending slots
      const int jq = (q < np) ? mask_ffs(m) - 1 : -1;                // slot of pending index q
      int c = -3;
      if (jq >= 0) c = adj[below(lo64(draw_block(K, purpose, (uint32_t)jq, a + (uint32_t)t)), deg)];
      G.L->out[G.sub] = c;                                           // proposal of (q, t) at q * A + t
      const bool mine0 = G.in(pend);
      const int my_q = mask_popc(pend & G.below());                  // pending index of the lane's own slot
      uint32_t pm = (1u << np) - 1u;                                 // pending, by pending index
      for (int tt = 0; tt < A && pm != 0u; ++tt) {
        const bool have = G.in(fixed);
        uint32_t acc = 0u;
        for (uint32_t w = pm; w != 0u; w &= w - 1u) {               // (w is the same in all lanes of the group)
          const int qq = __ffs((int)w) - 1;
          const int cj = G.L->out[qq * A + tt];
          // lane l < np stands for the pending slot of index l: a lower pending slot with the same proposal
          const bool lower = G.sub < qq && ((pm >> G.sub) & 1u) && G.L->out[G.sub * A + tt] == cj;
          if (grp_ballot(G, (have && val == cj) || lower) == (Mask)0) acc |= 1u << qq;
        }
        const bool got = mine0 && ((acc >> my_q) & 1u);
        if (got) val = G.L->out[my_q * A + tt];
        fixed |= grp_ballot(G, got);
        pm &= ~acc;
      }
      pend = grp_ballot(G, mine0 && ((pm >> my_q) & 1u));
      a += (uint32_t)A - 1u;
      continue;
    }
    const bool mine = G.in(pend);
    int cand = -3;
    if (mine) cand = adj[below(lo64(draw_block(K, purpose, (uint32_t)G.sub, a)), deg)];
    bool reject = false;
    if (FEW) {
      const bool have = G.in(fixed);
      if (mine) G.L->out[G.sub] = cand;
      for (Mask m = pend; m != 0; m &= m - (Mask)1) {      // m is the same in all lanes of the group
        const int j = mask_ffs(m) - 1;
        const int cj = G.L->out[j];
        const bool hit = (have && val == cj) || (mine && G.sub < j && cand == cj);
        const bool taken = grp_ballot(G, hit) != (Mask)0;
        if (G.sub == j) reject = taken;
      }
    } else {
      if (G.sub < k) {
        const int fx = G.in(fixed) ? val : -1;
        G.L->ab[G.sub] = (uint64_t)(uint32_t)fx | ((uint64_t)(uint32_t)(mine ? cand : -2) << 32);
      }
#pragma unroll 4
      for (int i = 0; i < k; ++i) {
        const uint64_t e = G.L->ab[i];
        reject |= ((int)(uint32_t)e == cand) | (((int)(uint32_t)(e >> 32) == cand) & (i < G.sub));
      }
    }
    const bool acc = mine && !reject;
    if (acc) val = cand;
    const Mask accm = grp_ballot(G, acc);
    pend &= ~accm;
    fixed |= accm;
  }
  return val;
}

// k < deg < 2k <= 2 W: the group owns adjacency positions sub and sub + W.  The `want` eligible
// positions of smallest priority are written to L->out[0..want) in ascending position order.
template <int W>
__device__ __forceinline__ void grp_select_positions(const GrpT<W>& G, int d, int want, bool elig0, bool elig1,
                                                     int a0, int a1, const DrawKey& K, uint32_t purpose) {
  const int p0 = G.sub, p1 = G.sub + W;
  uint64_t q0 = PRIO_NONE, q1 = PRIO_NONE;
  if (elig0) q0 = priority(lo64(draw_block(K, purpose, (uint32_t)p0, 0)), (uint32_t)p0);
  if (elig1) q1 = priority(lo64(draw_block(K, purpose, (uint32_t)p1, 0)), (uint32_t)p1);
  G.L->prio[p0] = q0;
  G.L->prio[p1] = q1;
  int r0, r1;
  grp_rank2(G, d, q0, q1, r0, r1);
  const bool s0 = elig0 && r0 < want, s1 = elig1 && r1 < want;
  const MaskT<W> m0 = grp_ballot(G, s0), m1 = grp_ballot(G, s1);
  if (s0) G.L->out[mask_popc(m0 & G.below())] = a0;
  if (s1) G.L->out[mask_popc(m0) + mask_popc(m1 & G.below())] = a1;
}

// FILL_FULL for one row: returns the value of slot `sub` (-1 beyond the row).
template <int W>
__device__ __forceinline__ int grp_fill_full_row(const GrpT<W>& G, const int32_t* __restrict__ adj, uint32_t deg, int k,
                                                 const DrawKey& K, uint32_t purpose, int32_t* state) {
  constexpr int GRP = W;
  if (deg <= (uint32_t)k) return ((uint32_t)G.sub < deg) ? adj[G.sub] : -1;
  if (deg < 2u * (uint32_t)k) {
    const int d = (int)deg;
    const bool e0 = G.sub < d, e1 = G.sub + GRP < d;
    const int a0 = e0 ? adj[G.sub] : -1, a1 = e1 ? adj[G.sub + GRP] : -1;
    grp_select_positions(G, d, k, e0, e1, a0, a1, K, purpose);
    return (G.sub < k) ? G.L->out[G.sub] : -1;
  }
  const int v = grp_rejection_fill<false>(G, GrpT<W>::first(k), (MaskT<W>)0, -1, k, adj, deg, K, purpose, state);
  return (G.sub < k) ? v : -1;
}

// REFRESH_PART for one full row of a node with deg > k (Alg. 2 RefreshCache): the n_new slots of smallest
// EVICT priority (`sb`: the slot's EVICT/PICK block) are redrawn from adj(v) \ retained.  `val` is the slot's
// current id; returns its new one and the mask of redrawn slots.
template <int W>
__device__ __forceinline__ int grp_refresh_part(const GrpT<W>& G, int val, int k, int n_new, const Block4& sb,
                                                const int32_t* __restrict__ adj, uint32_t deg, const DrawKey& K,
                                                int32_t* state, MaskT<W>& evict) {
  constexpr int GRP = W;
  const int sub = G.sub;
  const MaskT<W> slots = GrpT<W>::first(k);
  const uint64_t e = (sub < k) ? priority(lo64(sb), (uint32_t)sub) : PRIO_NONE;
  G.L->prio[sub] = e;
  // The n_new slots of smallest priority.  Priorities are uniform 64-bit numbers, so the slots below the
  // (n_new + 5) / k quantile nearly always include them: then a slot only has to be compared with those few (a slot
  // above the mark has at least n_new slots below it and is not ranked at all).  The wavefront walks over the slots
  // that are below the mark in either of its groups - a scalar loop; a slot above the mark in one's own group adds
  // nothing to a rank below it.  If a group has fewer than n_new slots below the mark, every slot is ranked among all.
  uint64_t mark = PRIO_NONE;
  if (n_new + 5 < k) mark = (uint64_t)(uint32_t)(4294967040.0f * (float)(n_new + 5) / (float)k) << 32;
  const bool low = e < mark;
  const uint64_t wave_low = __ballot(low), wave_here = __ballot(sub == 0);
  uint64_t scan = wave_low;
  bool enough = __popcll((unsigned long long)wave_low) >= n_new;
  if constexpr (W == 32) {
    const uint32_t lo = (uint32_t)wave_low, hi = (uint32_t)(wave_low >> 32);
    enough = (__popc(lo) >= n_new || !(wave_here & 1ull)) && (__popc(hi) >= n_new || !((wave_here >> 32) & 1ull));
    scan = lo | hi;
  } else if constexpr (W < 32) {
    enough = true;
    scan = 0ull;
#pragma unroll
    for (int q = 0; q < GrpT<W>::PER_WAVE; ++q) {
      const uint32_t m = (uint32_t)(wave_low >> (q * W)) & GrpT<W>::all();
      enough = enough && (__popc(m) >= n_new || !((wave_here >> (q * W)) & 1ull));
      scan |= m;
    }
  }
  int er;
  if (enough) {
    er = low ? 0 : k;
    for (uint64_t m = scan; m != 0; m &= m - 1) er += (G.L->prio[__builtin_ctzll(m)] < e) ? 1 : 0;
  } else {
    er = grp_rank_uniform(G, k, e);
  }
  evict = grp_ballot(G, sub < k && er < n_new);
  const MaskT<W> retained = slots & ~evict;
  if (deg < 2u * (uint32_t)k) {
    // priority regime: a position is eligible unless its id sits in a retained slot
    const int d = (int)deg;
    bool e0 = sub < d, e1 = sub + GRP < d;
    const int a0 = e0 ? adj[sub] : -1, a1 = e1 ? adj[sub + GRP] : -1;
    if (sub < k) G.L->ab[sub] = (uint64_t)(uint32_t)(G.in(retained) ? val : -1);
#pragma unroll 4
    for (int j = 0; j < k; ++j) {
      const int rv = (int)(uint32_t)G.L->ab[j];
      e0 &= (rv != a0);
      e1 &= (rv != a1);
    }
    grp_select_positions(G, d, n_new, e0, e1, a0, a1, K, P_FILL_PART);
    if (G.in(evict)) val = G.L->out[mask_popc(evict & G.below())];
  } else {
    val = grp_rejection_fill<true>(G, evict, retained, val, k, adj, deg, K, P_FILL_PART, state);
  }
  return val;
}

// ------------------------------------------------------------------------------------------
// fill_full_kernel: a workgroup takes chunks of FILL_CHUNK rows.
//   A  one thread per row reads indptr (base, degree) into LDS and flags rows with deg > k;
//   B  rows with deg <= k (83-89 % of all rows in the power-law workloads) are plain copies of the
//      adjacency: one thread per table cell, coalesced, every load independent of the others;
//   C  the flagged rows are compacted into a list, and (row, table) pairs are dealt to the eight
//      32-lane groups, so both halves of every wavefront run the Philox / rejection code together.
// ------------------------------------------------------------------------------------------
constexpr int FILL_CHUNK = 64;    // rows per chunk: small enough that a few thousand workgroups share the rejection work
template <int W>
__global__ __launch_bounds__(256) void fill_full_kernel(FillParams P) {
  __shared__ GroupLdsT<W> lds[256 / W];
  __shared__ long long row_base[FILL_CHUNK];
  __shared__ int row_deg[FILL_CHUNK];
  __shared__ int row_at[FILL_CHUNK];          // table row of the node, -1: the node keeps no row (degree split)
  __shared__ int heavy_rows[FILL_CHUNK];
  __shared__ int wave_heavy[4];
  GrpT<W> G;
  G.init(lds);
  const int tid = (int)threadIdx.x, lane = lane_id(), wave = tid >> 6;
  const int sshift = (P.S == 64) ? 6 : (P.S == 32) ? 5 : 4;
  const int64_t nchunks = (P.n_dst + FILL_CHUNK - 1) / FILL_CHUNK;
  for (int64_t chunk = blockIdx.x; chunk < nchunks; chunk += gridDim.x) {
    const int64_t v0 = chunk * FILL_CHUNK;
    const int rows = (int)((P.n_dst - v0 < FILL_CHUNK) ? (P.n_dst - v0) : FILL_CHUNK);
    // ---- A: degrees ----
    bool heavy = false;
    if (tid < rows) {
      const int64_t b = load_indptr(P.indptr, P.is64, v0 + tid);
      const int64_t d = load_indptr(P.indptr, P.is64, v0 + tid + 1) - b;
      row_base[tid] = b;
      row_deg[tid] = (int)d;                       // degrees are < 2^31 (checked when the graph is validated)
      const int at = P.row_of ? P.row_of[v0 + tid] : (int)(v0 + tid);
      row_at[tid] = at;
      heavy = d > P.k && at >= 0;
    }
    const uint64_t hm = __ballot(heavy);
    if (lane == 0) wave_heavy[wave] = __popcll(hm);
    __syncthreads();
    int before = 0, nheavy = 0;
    for (int q = 0; q < 4; ++q) { const int c = wave_heavy[q]; if (q < wave) before += c; nheavy += c; }
    if (heavy) heavy_rows[before + __popcll(hm & ((1ull << lane) - 1ull))] = tid;
    // ---- B: light rows, one thread per cell ----
    const int cells = rows << sshift;
    for (int c = tid; c < cells; c += 256) {
      const int row = c >> sshift, slot = c & (P.S - 1);
      const int d = row_deg[row];
      if (d > P.k || row_at[row] < 0) continue;
      const int val = (slot < d) ? P.indices[row_base[row] + slot] : -1;
      const int64_t at = ((int64_t)row_at[row] << sshift) + slot;
      for (int t = 0; t < P.ntab; ++t) P.table[t][at] = val;
    }
    __syncthreads();
    // ---- C: heavy rows, one W-lane group per (row, table) ----
    const int items = nheavy * P.ntab;
    for (int it = tid / W; it < items; it += 256 / W) {
      const int row = heavy_rows[it / P.ntab], t = it % P.ntab;
      const int64_t v = v0 + row;
      DrawKey K{P.seed_lo, P.seed_hi, (uint32_t)v, P.stepword, (P.layer_word[t] << 8) | (P.relation << 16)};
      int val;
      if (P.src_table[t]) {
        // layer-wide partial refresh: the row of the previous epoch (possibly the same memory) with n_new slots redrawn
        val = (G.sub < P.k) ? P.src_table[t][((int64_t)row_at[row] << sshift) + G.sub] : -1;
        Block4 sb{0u, 0u, 0u, 0u};
        if (G.sub < P.k) sb = draw_block(K, P_EVICT, (uint32_t)G.sub, 0);
        MaskT<W> evict;
        val = grp_refresh_part(G, val, P.k, P.n_new, sb, P.indices + row_base[row], (uint32_t)row_deg[row], K, P.state, evict);
      } else {
        val = grp_fill_full_row(G, P.indices + row_base[row], (uint32_t)row_deg[row], P.k, K, P_FILL_FULL, P.state);
      }
      if (G.sub < P.S) P.table[t][((int64_t)row_at[row] << sshift) + G.sub] = val;
    }
    __syncthreads();
  }
}

// fill_heavy_kernel: the same rows for a table set that has been filled before.  Rows of nodes with at most k
// neighbors hold the whole adjacency and never change, so a later refresh only recomputes the rows of the nodes
// with more (a list made once at set-up): one 32-lane group per (row, table), no chunk staging, no barriers.
template <int W>
__global__ __launch_bounds__(256) void fill_heavy_kernel(FillParams P, const int32_t* __restrict__ heavy, int64_t nheavy) {
  __shared__ GroupLdsT<W> lds[256 / W];
  GrpT<W> G;
  G.init(lds);
  constexpr int GROUPS = 256 / W;
  const int sshift = (P.S == 64) ? 6 : (P.S == 32) ? 5 : 4;
  const int64_t items = nheavy * P.ntab;
  for (int64_t it = (int64_t)blockIdx.x * GROUPS + (int64_t)(threadIdx.x / W); it < items; it += (int64_t)gridDim.x * GROUPS) {
    const int64_t v = heavy[it / P.ntab];
    const int t = (int)(it % P.ntab);
    const int64_t b = load_indptr(P.indptr, P.is64, v);
    const uint32_t deg = (uint32_t)(load_indptr(P.indptr, P.is64, v + 1) - b);
    const int64_t at = (P.row_of ? (int64_t)P.row_of[v] : v) << sshift;
    DrawKey K{P.seed_lo, P.seed_hi, (uint32_t)v, P.stepword, (P.layer_word[t] << 8) | (P.relation << 16)};
    int val;
    if (P.src_table[t]) {
      val = (G.sub < P.k) ? P.src_table[t][at + G.sub] : -1;
      Block4 sb{0u, 0u, 0u, 0u};
      if (G.sub < P.k) sb = draw_block(K, P_EVICT, (uint32_t)G.sub, 0);
      MaskT<W> evict;
      val = grp_refresh_part(G, val, P.k, P.n_new, sb, P.indices + b, deg, K, P.state, evict);
    } else {
      val = grp_fill_full_row(G, P.indices + b, deg, P.k, K, P_FILL_FULL, P.state);
    }
    if (G.sub < P.S) P.table[t][at + G.sub] = val;
  }
}

// ------------------------------------------------------------------------------------------
// Dedupe table: per key (node type offset + id) the smallest "order word" inserted in this hop.
//   direct layout  one 64-bit word per node: (~version << 32) | order, reduced with atomicMin.
//   hashed layout  open addressing, linear probing, 16-byte entries:
//                    keyver = (version << 32) | key     claimed with a 64-bit CAS
//                    val    = (~version << 32) | order  reduced with a 64-bit atomicMin
// Words of an older version count as empty (their high half is larger), so nothing is cleared
// between hops.  Device-scope atomics are the scarce resource here (about 26 per ns on the whole
// chip, against 50-200 random loads per ns), so every insert first LOADS the word and skips the
// atomic when the stored order is already smaller.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t hash_key(uint32_t key) {
  uint32_t h = key * 0x9E3779B1u;
  return h ^ (h >> 15);
}

__device__ __forceinline__ uint64_t load_relaxed(const uint64_t* p) {
  return __hip_atomic_load((const unsigned long long*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Reduces word *w with (version, order).  Returns the previous order of this version, or 0xFFFFFFFF.
__device__ __forceinline__ uint32_t word_min(uint64_t* w, uint32_t ver, uint32_t order) {
  const uint64_t myval = ((uint64_t)(~ver) << 32) | order;
  uint64_t cur = load_relaxed(w);
  if (cur > myval) cur = atomicMin((unsigned long long*)w, (unsigned long long)myval);
  return ((uint32_t)(cur >> 32) == ~ver) ? (uint32_t)cur : 0xFFFFFFFFu;
}

// Inserts (key, order).  Returns the previous order for the key in this version, or 0xFFFFFFFF.
__device__ __forceinline__ uint32_t table_insert_min(const DedupeTable& H, uint32_t ver, uint32_t key,
                                                     uint32_t order, int32_t* state) {
  if (H.direct) return word_min(&H.direct[key], ver, order);
  const uint64_t mine = ((uint64_t)ver << 32) | key;
  uint64_t h = hash_key(key) & H.mask;
  for (uint64_t probes = 0; probes <= H.mask; ++probes) {
    unsigned long long* kv = (unsigned long long*)&H.entries[h].keyver;
    uint64_t cur = __hip_atomic_load(kv, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if ((uint32_t)(cur >> 32) != ver) {           // empty or stale: try to claim it
      const uint64_t old = atomicCAS(kv, (unsigned long long)cur, (unsigned long long)mine);
      cur = (old == cur) ? mine : old;
    }
    if (cur == mine) return word_min(&H.entries[h].val, ver, order);
    h = (h + 1) & H.mask;
  }
  atomicOr(&state[ST_ERROR], ERR_TABLE_FULL);
  return 0xFFFFFFFFu;
}

__device__ __forceinline__ uint32_t table_lookup(const DedupeTable& H, uint32_t ver, uint32_t key, int32_t* state) {
  if (H.direct) return (uint32_t)H.direct[key];
  const uint64_t mine = ((uint64_t)ver << 32) | key;
  uint64_t h = hash_key(key) & H.mask;
  for (uint64_t probes = 0; probes <= H.mask; ++probes) {
    const HashEntry e = H.entries[h];
    if (e.keyver == mine) return (uint32_t)e.val;
    if ((uint32_t)(e.keyver >> 32) != ver) break;   // hit an empty slot: the key was never inserted
    h = (h + 1) & H.mask;
  }
  atomicOr(&state[ST_ERROR], ERR_TABLE_MISS);
  return 0u;
}

// Relation / node type r of a slice.  The compact launch builds a slice's arguments in registers, where nothing
// can be indexed at run time: its layout (one relation, one node type) has nothing to index anyway.
struct HopParamsMonoRegs : HopParamsMono { static constexpr bool IN_REGISTERS = true; };
template <class HP, class = void> struct in_registers { static constexpr bool value = false; };
template <class HP> struct in_registers<HP, decltype((void)HP::IN_REGISTERS)> { static constexpr bool value = true; };
template <class HP>
__device__ __forceinline__ const RelParam& rel_of(const HP& P, int r) {
  if constexpr (in_registers<HP>::value) return P.rel[0]; else return P.rel[r];
}
template <class HP>
__device__ __forceinline__ const TypeParam& type_of(const HP& P, int t) {
  if constexpr (in_registers<HP>::value) return P.type[0]; else return P.type[t];
}
template <class HP>
__device__ __forceinline__ int frontier_count(const HP& P, int t) {
  const int o = type_of(P, t).count_override;
  return o >= 0 ? o : P.state[ST_COUNTS + P.hop * P.T + t];
}

// Live tiles of a hop.  Pick slots are laid out by host-known upper bounds (relation r owns the tiles from
// slot_base[r] / TILE on), but only the first ceil(F * f / TILE) tiles of a relation hold picks, F being the
// frontier size of its dst type, known on the device.  The insert, mark and emit phases walk the concatenation
// of the live ranges: live index j -> (relation, tile).  first[r] = live index of relation r's first tile,
// first[R] = number of live tiles, nslots[r] = F * f.
struct LiveLds {
  int first[GSS_MAX_RELATIONS + 1];
  uint32_t nslots[GSS_MAX_RELATIONS];
};
template <class HP>
__device__ __forceinline__ void live_tiles_setup(const HP& P, LiveLds* L) {
  if ((int)threadIdx.x < P.R) {
    // (P is indexed with uniform indices only: a per-lane index would move the arguments to scratch memory)
    int dst_type = 0;
    for (int q = 0; q < P.R; ++q) if ((int)threadIdx.x == q) dst_type = rel_of(P, q).dst_type;
    int count = -1;
    for (int t = 0; t < P.T; ++t) if (dst_type == t) count = type_of(P, t).count_override;
    if (count < 0) count = P.state[ST_COUNTS + P.hop * P.T + dst_type];
    L->nslots[threadIdx.x] = (uint32_t)count * (uint32_t)P.f;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int run = 0;
    for (int q = 0; q < P.R; ++q) { L->first[q] = run; run += (int)((L->nslots[q] + TILE - 1) / TILE); }
    L->first[P.R] = run;
  }
  __syncthreads();
}
struct LiveTile { int r; uint32_t tile, local0, nslots; };
template <class HP>
__device__ __forceinline__ LiveTile live_tile(const HP& P, const LiveLds* L, int j) {
  int r = 0;
  while (r + 1 < P.R && j >= L->first[r + 1]) ++r;
  LiveTile t;
  t.r = r;
  const uint32_t tl = (uint32_t)(j - L->first[r]);
  t.tile = (uint32_t)(rel_of(P, r).slot_base / TILE) + tl;
  t.local0 = tl * TILE;
  t.nslots = L->nslots[r];
  return t;
}

// ------------------------------------------------------------------------------------------
// sample phase: rows wg.y < R of the slice's grid: relation y, one 32-lane group per frontier node.
//               rows wg.y >= R: node type y-R, one thread per frontier node (insert the dst
//               nodes into the dedupe table with order = frontier index, copy them to src_nodes).
// ------------------------------------------------------------------------------------------
// Node type t of a hop, one thread per frontier node: the dst nodes enter the dedupe table (order = frontier index)
// and head the hop's src_nodes.  Workgroup x of the P.gxd that share the work.
template <class HP>
__device__ __forceinline__ void dst_node_rows(const HP& P, int t, int x) {
  const TypeParam& TP = type_of(P, t);
  const int F = frontier_count(P, t);
  for (int i = x * (int)blockDim.x + (int)threadIdx.x; i < F; i += P.gxd * (int)blockDim.x) {
    const int v = TP.frontier[i];
    if ((uint32_t)v >= (uint32_t)TP.n_nodes) { atomicOr(&P.state[ST_ERROR], ERR_SEED_RANGE); continue; }
    TP.src_nodes[i] = v;
    if (P.hop > 0 && P.ht.direct) {
      // Beyond the seeds the dst nodes are distinct (the previous hop's dedupe made them so), and a frontier index is
      // smaller than every pick's order word: whatever the picks of the same launch do to the node's word with their
      // atomic minimum, before or after, a plain store of the frontier index leaves the minimum there.  (Random
      // device-scope atomics run at 27 per ns on the whole chip, whatever the table size; plain stores at 50-180.)
      __hip_atomic_store((unsigned long long*)&P.ht.direct[TP.key_off + (uint32_t)v], ((unsigned long long)(~P.ver) << 32) | (uint32_t)i,
                         __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      continue;
    }
    const uint32_t old = table_insert_min(P.ht, P.ver, TP.key_off + (uint32_t)v, (uint32_t)i, P.state);
    if (old < EDGE_BIT && old != (uint32_t)i) atomicOr(&P.state[ST_ERROR], ERR_SEED_DUP);
  }
}

template <class HP, int W>
__device__ __forceinline__ void sample_phase(const HP& P, const Wg wg, GroupLdsT<W>* lds) {
  if (wg.y >= P.R) {
    dst_node_rows(P, wg.y - P.R, wg.x);
    return;
  }
  using Mask = MaskT<W>;
  constexpr int GRP = W;
  GrpT<W> G;
  G.init(lds);
  if (G.idle) return;                 // (no barrier below: the phase is a per-group loop)
  const int r = wg.y;
  const RelParam& RP = rel_of(P, r);
  const RelConst& RC = P.rc(r);
  const int grp = wg.x * GrpT<W>::PER_WG + G.index_in_workgroup();
  // the first node id is loaded before the frontier size is known (both loads travel together);
  // `frontier_cap` is the allocated length of the frontier array
  const int v_first = (grp < type_of(P, RP.dst_type).frontier_cap) ? type_of(P, RP.dst_type).frontier[grp] : 0;
  const int F = frontier_count(P, RP.dst_type);
  const int ngrp = P.gx * GrpT<W>::PER_WG;
  const int k = P.k, f = P.f, sub = G.sub;
  const int32_t* __restrict__ frontier = type_of(P, RP.dst_type).frontier;
  const uint32_t src_key_off = type_of(P, RP.src_type).key_off;

  int v_ahead = v_first;
  for (int i = grp; i < F; i += ngrp) {
    const int v = v_ahead;
    if (i + ngrp < F) v_ahead = frontier[i + ngrp];   // the id of the group's next node travels while this one is worked on
    const uint32_t g0 = (uint32_t)RP.slot_base + (uint32_t)i * (uint32_t)f;
    if ((uint32_t)v >= (uint32_t)RC.n_dst) {        // reported by the node-type pass; emit nothing
      if (sub < f) P.picks[g0 + sub] = -1;
      continue;
    }
    DrawKey K{P.seed_lo, P.seed_hi, (uint32_t)v, P.step, (P.layer_word << 8) | ((uint32_t)r << 16)};
    int val;
    bool sel;
    // Degree split: the node's table row comes from the row map; nodes without a row are sampled
    // like Full Batch Load.  The adjacency bounds are requested together with the map entry.
    int at = v;
    bool uncached = P.mode == GSS_MODE_FBL;
    int64_t b = 0, d64 = 0;
    if (RC.row_of) {
      at = RC.row_of[v];
      b = load_indptr(RC.indptr, RC.is64, v);
      d64 = load_indptr(RC.indptr, RC.is64, (int64_t)v + 1) - b;
      uncached |= at < 0;
    } else if (uncached) {
      b = load_indptr(RC.indptr, RC.is64, v);
      d64 = load_indptr(RC.indptr, RC.is64, (int64_t)v + 1) - b;
    }
    if (uncached) {
      // Full Batch Load: no cache, a uniform min(deg,f)-subset straight from the adjacency,
      // keyed by the step and the hop's own layer (also when the cached nodes share one table)
      K.tag = ((uint32_t)P.layer << 8) | ((uint32_t)r << 16);
      val = grp_fill_full_row(G, RC.indices + b, (uint32_t)d64, f, K, P_FBL, P.state);
      sel = (int64_t)sub < (d64 < f ? d64 : (int64_t)f);
    } else {
    int32_t* row = RP.table + (int64_t)at * P.S;
    val = (sub < k) ? row[sub] : -1;
    // On a refresh step the adjacency bounds (and the shared-mode stamp) are loaded together with
    // the row rather than after it: one round trip less on the critical path of every visited node.
    long long stamp = -1;
    const bool fetch_mode = P.mode == GSS_MODE_OTF_FETCH && P.n_new > 0;
    if (P.refresh_now || fetch_mode) {
      if (!RC.row_of) {
        b = load_indptr(RC.indptr, RC.is64, v);
        d64 = load_indptr(RC.indptr, RC.is64, (int64_t)v + 1) - b;
      }
      if (P.mode == GSS_MODE_SHARED_OTF) stamp = RC.stamp[at];
    }
    const int len = mask_popc(grp_ballot(G, val >= 0));

    // ---- does this visit refresh the row? (only full rows can belong to a node with deg > k) ----
    bool refresh = false;
    const uint32_t deg = (uint32_t)d64;
    if (P.refresh_now && len == k) {
      bool due = true;
      if (P.mode == GSS_MODE_SHARED_OTF) {
        due = stamp != (long long)P.step;
        if (due && sub == 0) RC.stamp[at] = (long long)P.step;
      }
      refresh = due && d64 > k;
    }
    // OTF Fetch: a node with more than k neighbors takes n_new of its f neighbors fresh from the adjacency
    // and only f - n_new from the (full) row
    const bool fetch = fetch_mode && d64 > k;
    const int fdraw = fetch ? f - P.n_new : f;
    // one Philox block per slot serves both per-slot draws: EVICT (words 0,1) and PICK (words 2,3)
    Block4 sb{0u, 0u, 0u, 0u};
    if ((refresh || len > fdraw) && sub < k) sb = draw_block(K, P_EVICT, (uint32_t)sub, 0);

    if (refresh) {
      Mask evict;
      val = grp_refresh_part(G, val, k, P.n_new, sb, RC.indices + b, deg, K, P.state, evict);
      if (G.in(evict)) row[sub] = val;
    }

    // ---- draw the fanout from the row ----
    if (len <= fdraw) {
      sel = sub < len;
    } else {
      const uint64_t pp = (sub < len) ? priority(hi64(sb), (uint32_t)sub) : PRIO_NONE;
      G.L->prio[sub] = pp;
      const int rank = grp_rank_uniform(G, k, pp);       // (slots from len on hold PRIO_NONE)
      int start = 0;
      if (P.shared) start = min(P.band_offset, len - fdraw);
      sel = sub < len && rank >= start && rank < start + fdraw;
    }
    if (fetch) {
      // the cached picks move to lanes 0 .. fdraw-1 (ascending slot order); lanes fdraw .. f-1 draw fresh
      // neighbors from adj(v) \ {cached picks} by the redraw procedure of the partial refresh, on this
      // f-wide list instead of the row
      const Mask selm0 = grp_ballot(G, sel);
      if (sel) G.L->out[mask_popc(selm0 & G.below())] = val;
      int cv = (sub < fdraw) ? G.L->out[sub] : -1;
      const Mask kept = GrpT<W>::first(fdraw);                        // fdraw < f <= W
      const Mask redraw = GrpT<W>::first(f) & ~kept;
      const int32_t* adj = RC.indices + b;
      const uint32_t deg = (uint32_t)d64;
      if (deg < 2u * (uint32_t)f) {
        const int d = (int)deg;
        bool e0 = sub < d, e1 = sub + GRP < d;
        const int a0 = e0 ? adj[sub] : -1, a1 = e1 ? adj[sub + GRP] : -1;
        if (sub < f) G.L->ab[sub] = (uint64_t)(uint32_t)(G.in(kept) ? cv : -1);
#pragma unroll 4
        for (int j = 0; j < f; ++j) {
          const int rv = (int)(uint32_t)G.L->ab[j];
          e0 &= (rv != a0);
          e1 &= (rv != a1);
        }
        grp_select_positions(G, d, P.n_new, e0, e1, a0, a1, K, P_FETCH);
        if (G.in(redraw)) cv = G.L->out[mask_popc(redraw & G.below())];
      } else {
        cv = grp_rejection_fill<true>(G, redraw, kept, cv, f, adj, deg, K, P_FETCH, P.state);
      }
      val = cv;
      sel = sub < f;
    }
    }
    const Mask selm = grp_ballot(G, sel);
    const int cnt = mask_popc(selm);
    if (sel) {
      const uint32_t g = g0 + (uint32_t)mask_popc(selm & G.below());
      P.picks[g] = val;
      bool inserts = !P.insert_split;                  // (bit 1, the LDS stage, is only ever set in the staged builds)
      if constexpr (std::is_base_of<HopParamsStaged, HP>::value) inserts = !(P.insert_split & 1);
      if (inserts) table_insert_min(P.ht, P.ver, src_key_off + (uint32_t)val, EDGE_BIT | g, P.state);
    }
    if (sub >= cnt && sub < f) P.picks[g0 + sub] = -1;
  }
}

// Optional first stage of the dedupe, per tile, in LDS ("LDS-staged unique, spilling to the global table"): the tile's
// picks enter an open-addressing table of 2 * TILE 64-bit words, (key << 32) | slot within the tile, reduced with
// a 64-bit LDS minimum; only the pick that holds the smallest slot of its id within the tile goes on to the global
// table - the others could not win there anyway.  Returns, per thread, which of its ITEMS_PER_THREAD picks go on.
// All threads of the workgroup call it (barriers inside); `key[q]` is only read where `valid` has bit q set.
constexpr int TILE_HASH = 2 * TILE;
struct DedupeLds { unsigned long long word[TILE_HASH]; };
__device__ __forceinline__ uint32_t tile_firsts(DedupeLds* D, const uint32_t* key, uint32_t valid, uint32_t slot0) {
  unsigned long long* tab = D->word;
  for (int i = (int)threadIdx.x; i < TILE_HASH; i += (int)blockDim.x) tab[i] = ~0ull;
  __syncthreads();
  uint32_t home[ITEMS_PER_THREAD];
#pragma unroll
  for (int q = 0; q < ITEMS_PER_THREAD; ++q) {
    home[q] = 0u;
    if (!((valid >> q) & 1u)) continue;
    const unsigned long long mine = ((unsigned long long)key[q] << 32) | (slot0 + (uint32_t)q);
    uint32_t h = (key[q] * 0x9E3779B1u) >> 21;                    // 11 bits: TILE_HASH entries
    for (;;) {                                                    // (at most TILE of the 2 TILE entries are ever taken)
      unsigned long long cur = __hip_atomic_load(&tab[h], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      if (cur == ~0ull &&                                         // empty: try to take it (on failure `cur` = who did)
          __hip_atomic_compare_exchange_strong(&tab[h], &cur, mine, __ATOMIC_RELAXED, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP))
        break;                                                    // taken: this pick is the smallest so far
      if ((uint32_t)(cur >> 32) == key[q]) {
        __hip_atomic_fetch_min(&tab[h], mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        break;
      }
      h = (h + 1u) & (uint32_t)(TILE_HASH - 1);
    }
    home[q] = h;
  }
  __syncthreads();
  uint32_t first = 0u;
#pragma unroll
  for (int q = 0; q < ITEMS_PER_THREAD; ++q)
    if (((valid >> q) & 1u) && (uint32_t)__hip_atomic_load(&tab[home[q]], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) == slot0 + (uint32_t)q)
      first |= 1u << q;
  __syncthreads();                                                // (the table is cleared again for the next tile)
  return first;
}

// ------------------------------------------------------------------------------------------
// Visit-once steps (see ChainArgs): chain phase and place phase.
// ------------------------------------------------------------------------------------------
// Marks node v as visited in this step with holding index Q (`mine` = (~version << 32) | Q).  True for exactly one
// of the picks that name the same node in one step.
__device__ __forceinline__ bool claim_visit(uint64_t* visit, uint32_t v, uint64_t mine) {
  unsigned long long* w = (unsigned long long*)&visit[v];
  const uint64_t cur = __hip_atomic_load(w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if ((uint32_t)(cur >> 32) == (uint32_t)(mine >> 32)) return false;      // visited already
  // (a word of another version can only turn into one of this step's version)
  return atomicCAS(w, (unsigned long long)cur, (unsigned long long)mine) == cur;
}
// The same for a seed (holding index Q < num_seeds).  A seed must be visited as a seed even if a pick of another seed
// names it and claims it before its own group gets to it: words of later versions and smaller indices are smaller, so an
// atomic minimum lets the seed take the entry over (the pick's entry in list 1 then points at an index the visit table
// no longer holds, and is skipped).
__device__ __forceinline__ void claim_seed(uint64_t* visit, uint32_t v, uint64_t mine) {
  __hip_atomic_fetch_min((unsigned long long*)&visit[v], (unsigned long long)mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// The one visit of node v in this step, by the hop c that reaches it first: read the row, refresh it when the step
// refreshes (Alg. 2 RefreshCache on the shared table: once per node and step), rank the slots once by PICK priority,
// and take for every hop h = c .. L-1 the ranks [band[h], band[h] + f[h]) ("Shared Cache Design": per-layer bands of
// one per-(step, node) ranking) - what the per-hop sample phase computes when it meets the node again in hop h.
// Nodes without a cache row (degree split) draw every hop straight from the adjacency, keyed by the hop's layer.
// Returns hop c's pick number `sub` (-1 beyond the node's picks).
template <class HP>
__device__ __forceinline__ int visit_node(const HP& P, const ChainArgs& C, const Grp& G, int c, int v, uint32_t Q) {
  const RelParam& RP = rel_of(P, 0);
  const RelConst& RC = P.rc(0);
  const int k = P.k, sub = G.sub;
  DrawKey K{P.seed_lo, P.seed_hi, (uint32_t)v, P.step, P.layer_word << 8};
  int at = v;
  int64_t b = 0, d64 = 0;
  if (RC.row_of) at = RC.row_of[v];
  if (RC.row_of || P.refresh_now) {
    b = load_indptr(RC.indptr, RC.is64, v);
    d64 = load_indptr(RC.indptr, RC.is64, (int64_t)v + 1) - b;
  }
  int mine = -1;
  if (at < 0) {
    for (int h = c; h < C.L; ++h) {
      const int f = C.f(h);
      K.tag = C.layer(h) << 8;
      int val = grp_fill_full_row(G, RC.indices + b, (uint32_t)d64, f, K, P_FBL, P.state);
      const int cnt = (int)(d64 < f ? d64 : (int64_t)f);
      if (sub >= cnt) val = -1;
      if (sub < f) C.held[C.off[h] + Q * (uint32_t)f + (uint32_t)sub] = val;
      if (h == c) mine = val;
    }
    return mine;
  }
  int32_t* row = RP.table + (int64_t)at * P.S;
  int val = (sub < k) ? row[sub] : -1;
  const int len = __popc(grp_ballot(G, val >= 0));
  const bool refresh = P.refresh_now && len == k && d64 > k;
  bool ranked = false;
  for (int h = c; h < C.L; ++h) ranked |= len > C.f(h);
  Block4 sb{0u, 0u, 0u, 0u};
  if ((refresh || ranked) && sub < k) sb = draw_block(K, P_EVICT, (uint32_t)sub, 0);
  if (refresh) {
    uint32_t evict;
    val = grp_refresh_part(G, val, k, P.n_new, sb, RC.indices + b, (uint32_t)d64, K, P.state, evict);
    if ((evict >> sub) & 1u) row[sub] = val;
  }
  int rank = 0;
  if (ranked) {
    const uint64_t pp = (sub < len) ? priority(hi64(sb), (uint32_t)sub) : PRIO_NONE;
    G.L->prio[sub] = pp;
    rank = grp_rank_uniform(G, k, pp);                  // (slots from len on hold PRIO_NONE)
  }
  for (int h = c; h < C.L; ++h) {
    const int f = C.f(h);
    bool sel = sub < len;
    if (len > f) {
      const int start = min(C.band(h), len - f);
      sel = sub < len && rank >= start && rank < start + f;
    }
    const uint32_t selm = grp_ballot(G, sel);
    const int cnt = __popc(selm);
    if (sel) G.L->out[__popc(selm & below_mask(sub))] = val;       // picks in slot order, through LDS
    const int pick = (sub < cnt) ? G.L->out[sub] : -1;
    if (sub < f) C.held[C.off[h] + Q * (uint32_t)f + (uint32_t)sub] = pick;
    if (h == c) mine = pick;
  }
  return mine;
}

// chain phase of hop c: one 32-lane group per node of the frontier of hop c, eight groups per workgroup, striding.
// The nodes that hop c reaches first - the seeds for c = 0, else list c - are visited.  Unless c is the last hop, hop
// c's picks of every frontier node - of the ones just visited, and of the nodes of earlier hops, whose picks are held -
// then claim their nodes: a pick that comes first appends its node to list c + 1.
struct ChainLds { uint32_t start[CHAIN_MAX_HOPS * CHAIN_SEGS + 2]; };
template <bool AHEAD, class HP>
__device__ __forceinline__ void chain_phase(const HP& P, const ChainArgs& C, const Wg wg, GroupLds* lds, ChainLds* CL) {
  Grp G;
  G.init(lds);
  const int c = P.hop, sub = G.sub, L = C.L;
  const int grp = wg.x * (int)(blockDim.x >> 5) + (int)(threadIdx.x >> 5);
  const int ngrp = P.gx * (int)(blockDim.x >> 5);
  const RelConst& RC = P.rc(0);
  const uint64_t vtag = (uint64_t)(~P.visit_ver()) << 32;
  const uint32_t F0 = (uint32_t)C.V[0];
  const bool claims = c + 1 < L;
  // ---- the items: seeds (unless only list c has work to do), then the segments of lists 1 .. c ----
  const int first_list = claims ? 0 : c;                 // the last hop only visits
  const uint32_t nseeds = first_list == 0 ? F0 : 0u;
  const int h0 = first_list > 1 ? first_list : 1;        // first list kept in segments
  const int nsegs = c >= h0 ? (c - h0 + 1) * CHAIN_SEGS : 0;
  if (c == 0 && wg.x == 0 && threadIdx.x < CHAIN_MAX_HOPS * CHAIN_SEGS) C.counts_next[threadIdx.x * CHAIN_COUNT_STRIDE] = 0u;
  if (nsegs > 0) {
    if ((int)threadIdx.x < nsegs) {
      const uint32_t n = C.counts[(h0 * CHAIN_SEGS + (int)threadIdx.x) * CHAIN_COUNT_STRIDE];
      const uint32_t cap = C.lcap[h0 + (int)threadIdx.x / CHAIN_SEGS];
      if (n > cap) atomicOr(&P.state[ST_ERROR], ERR_TABLE_FULL);
      CL->start[threadIdx.x + 1] = n < cap ? n : cap;
    }
    __syncthreads();
    if (threadIdx.x < 64) {
      // exclusive prefix of the segment sizes (size of segment q at start[q + 1] -> its first item at start[q]) by the
      // first wavefront, two segments per lane: a lane's stores depend, through the shuffles, on the loads of every
      // lane below it, which are the only other readers of the words it overwrites
      const int l = (int)threadIdx.x;
      static_assert(CHAIN_MAX_HOPS * CHAIN_SEGS <= 128, "two segments per lane");
      const uint32_t a = 2 * l < nsegs ? CL->start[2 * l + 1] : 0u, b = 2 * l + 1 < nsegs ? CL->start[2 * l + 2] : 0u;
      uint32_t inc = a + b;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const uint32_t t = (uint32_t)__shfl_up((int)inc, o);
        if (l >= o) inc += t;
      }
      const uint32_t ex = nseeds + inc - (a + b);
      if (2 * l < nsegs) CL->start[2 * l] = ex;
      if (2 * l + 1 < nsegs) CL->start[2 * l + 1] = ex + a;
      if (l == 63) CL->start[nsegs] = nseeds + inc;
    }
    __syncthreads();
  }
  const uint32_t total = nsegs > 0 ? CL->start[nsegs] : nseeds;
  const int32_t* __restrict__ seeds = type_of(P, 0).frontier;
  const int fc = C.f(c);
  // item g -> the node: its id (seeds) or its list entry (Q << 32 | v), and the list it is in
  auto item = [&](uint32_t g, int& h) -> uint64_t {
    if (g < nseeds) { h = 0; return ((uint64_t)g << 32) | (uint32_t)seeds[g]; }
    int q = 0;                                           // the segment that holds item g (start[] is ascending)
    for (int step = 64; step > 0; step >>= 1)
      if (q + step < nsegs && CL->start[q + step] <= g) q += step;
    h = h0 + q / CHAIN_SEGS;
    return C.list[C.loff[h] + (uint32_t)(q % CHAIN_SEGS) * C.lcap[h] + (g - CL->start[q])];
  };
  int h_ahead = 0;
  uint64_t e_ahead = (AHEAD && (uint32_t)grp < total) ? item((uint32_t)grp, h_ahead) : 0ull;
  for (uint32_t g = (uint32_t)grp; g < total; g += (uint32_t)ngrp) {
    // ---- which node (the group's next item travels while this one is worked on - not in the build held to 64
    //      vector registers, where the item in flight meant two registers spilled to scratch memory, and a kernel that
    //      uses scratch memory is followed by 4.5 us of idle time before the next launch starts) ----
    uint64_t e;
    int h;
    if constexpr (AHEAD) {
      e = e_ahead;
      h = h_ahead;
      if (g + (uint32_t)ngrp < total) e_ahead = item(g + (uint32_t)ngrp, h_ahead);
    } else {
      e = item(g, h);
    }
    const int v = (int)(uint32_t)e;
    const uint32_t Q = (uint32_t)(e >> 32);
    const bool fresh = h == c;                           // first reached by this hop: to be visited
    // (list 1 may name a seed that a pick claimed before the seed's own visit took the entry over)
    if (h == 1 && C.visit[v] != (vtag | Q)) continue;
    // ---- hop c's picks of the node: drawn now, or held since its visit ----
    int id = -1;
    if (c == 0) {
      if ((uint32_t)v < (uint32_t)RC.n_dst) {
        // the seed's entry of the visit table: nobody waits for the result.  (A repeated seed is visited twice; the
        // place phase reports it, and the step's results are discarded.)
        if (sub == 0) claim_seed(C.visit, (uint32_t)v, vtag | Q);
        id = visit_node(P, C, G, 0, v, Q);
      } else {
        // an id out of range (the place phase reports it): it holds no picks
        for (int h = 0; h < L; ++h)
          if (sub < C.f(h)) C.held[C.off[h] + Q * (uint32_t)C.f(h) + (uint32_t)sub] = -1;
      }
    } else if (fresh) {
      id = visit_node(P, C, G, c, v, Q);
    } else if (sub < fc) {
      id = C.held[C.off[c] + Q * (uint32_t)fc + (uint32_t)sub];
    }
    if (!claims) continue;
    // ---- every pick claims its node; the winners join list c + 1 ----
    const uint32_t Qc = (uint32_t)C.V[c] + Q * (uint32_t)fc + (uint32_t)sub;
    bool won = false;
    if (id >= 0) won = claim_visit(C.visit, (uint32_t)id, vtag | Qc);
    const uint64_t wm = __ballot(won);                   // both nodes of the wavefront: they share a segment
    if (wm != 0ull) {
      const uint32_t seg = (g >> 1) % CHAIN_SEGS;
      const int leader = __ffsll((unsigned long long)wm) - 1;
      uint32_t base = 0u;
      if (lane_id() == leader) base = atomicAdd(&C.counts[((c + 1) * CHAIN_SEGS + seg) * CHAIN_COUNT_STRIDE], (uint32_t)__popcll(wm));
      base = (uint32_t)__shfl((int)base, leader);
      if (won) {
        const uint32_t at = base + (uint32_t)__popcll(wm & ((1ull << lane_id()) - 1ull));
        if (at < C.lcap[c + 1]) C.list[C.loff[c + 1] + seg * C.lcap[c + 1] + at] = ((uint64_t)Qc << 32) | (uint32_t)id;
        // (beyond the capacity: cannot happen; the next chain phase reports the counter)
      }
    }
  }
}

// place phase of hop h: tiles of pick slots in frontier order.  Slot i * f + j takes pick j of frontier node i from
// the holding area (through the node's holding index in the visit table) and enters it into the dedupe table; rows
// wg.y >= 1 of the slice handle the dst nodes.  From here on the hop looks like any other: mark, emit.
template <class HP>
__device__ __forceinline__ void place_phase(const HP& P, const Wg wg, LiveLds* live, DedupeLds* D) {
  if (wg.y >= 1) {
    dst_node_rows(P, 0, wg.x);
    return;
  }
  live_tiles_setup(P, live);
  const TypeParam& TP = type_of(P, 0);
  const uint32_t f = (uint32_t)P.f;
  const bool staged = (P.insert_split & 2) != 0;
  for (int j = wg.x; j < live->first[1]; j += P.gx) {
    const LiveTile lt = live_tile(P, live, j);
    const uint32_t nslots = lt.nslots;
    const uint32_t g = lt.local0 + ITEMS_PER_THREAD * threadIdx.x;       // one relation: its slots start at 0
    uint32_t i = g / f, jj = g - i * f;
    int id[ITEMS_PER_THREAD];
    uint32_t Q = 0;
    bool have = false;
#pragma unroll
    for (int q = 0; q < ITEMS_PER_THREAD; ++q) {
      id[q] = -1;
      if (g + q < nslots) {
        if (!have || jj == 0u) {            // the first slot of the thread, or a new frontier node
          have = true;
          const int v = TP.frontier[i];
          Q = 0xFFFFFFFFu;
          if ((uint32_t)v < (uint32_t)TP.n_nodes) {
            const uint64_t w = P.visit[v];
            if ((uint32_t)(w >> 32) == ~P.visit_ver()) Q = (uint32_t)w;
            else atomicOr(&P.state[ST_ERROR], ERR_TABLE_MISS);   // (cannot happen: every frontier node was visited)
          }
        }
        if (Q != 0xFFFFFFFFu) id[q] = P.held[Q * f + jj];
      }
      if (++jj == f) { jj = 0u; ++i; }
    }
    if (g < nslots) *reinterpret_cast<int4*>(P.picks + g) = make_int4(id[0], id[1], id[2], id[3]);
    if (P.insert_split & 1) continue;     // (uniform: the hop has an insert phase, which enters the picks into the table)
    uint32_t key[ITEMS_PER_THREAD], go = 0u;
#pragma unroll
    for (int q = 0; q < ITEMS_PER_THREAD; ++q) {
      key[q] = TP.key_off + (uint32_t)id[q];
      if (id[q] >= 0) go |= 1u << q;
    }
    if (staged) go = tile_firsts(D, key, go, ITEMS_PER_THREAD * threadIdx.x);
#pragma unroll
    for (int q = 0; q < ITEMS_PER_THREAD; ++q)
      if ((go >> q) & 1u) table_insert_min(P.ht, P.ver, key[q], EDGE_BIT | (g + q), P.state);
  }
}

// ------------------------------------------------------------------------------------------
// insert phase (large hops only; smaller ones insert in the sample phase): per pick, reduce the dedupe
// table word of its id with the pick's slot.  Four consecutive slots per thread, four independent
// table accesses in flight - in the sample phase the insert is the tail of a long dependent chain.
// ------------------------------------------------------------------------------------------
template <bool STAGED, class HP>
__device__ __forceinline__ void insert_phase(const HP& P, const Wg wg, LiveLds* live, DedupeLds* D) {
  // The workgroup's first tile is requested before the live counts are known (if it lies in relation 0 its
  // address does not depend on them, and the buffer covers every tile of the grid): the picks travel while the
  // counts are fetched.
  int4 pv_first = make_int4(-1, -1, -1, -1);
  if (wg.x < P.num_tiles_ub)
    pv_first = *reinterpret_cast<const int4*>(P.picks + (uint32_t)rel_of(P, 0).slot_base + (uint32_t)wg.x * TILE + 4u * threadIdx.x);
  live_tiles_setup(P, live);
  if (!STAGED || (P.insert_split & 2) == 0) {
    for (int j = wg.x; j < live->first[P.R]; j += P.gx) {
      const LiveTile lt = live_tile(P, live, j);
      const RelParam& RP = rel_of(P, lt.r);
      const uint32_t nslots = lt.nslots;
      const uint32_t loc = lt.local0 + 4u * threadIdx.x;
      const uint32_t g = (uint32_t)RP.slot_base + loc;
      if (loc >= nslots) continue;
      const int4 pv = (j == wg.x && lt.r == 0) ? pv_first : *reinterpret_cast<const int4*>(P.picks + g);
      const uint32_t key_off = type_of(P, RP.src_type).key_off;
      const int id[4] = {pv.x, pv.y, pv.z, pv.w};
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if (loc + q < nslots && id[q] >= 0) table_insert_min(P.ht, P.ver, key_off + (uint32_t)id[q], EDGE_BIT | (g + q), P.state);
    }
    return;
  }
  // with the LDS stage: every thread of the workgroup takes part in every tile (barriers)
  if constexpr (STAGED)
  for (int j = wg.x; j < live->first[P.R]; j += P.gx) {
    const LiveTile lt = live_tile(P, live, j);
    const RelParam& RP = rel_of(P, lt.r);
    const uint32_t nslots = lt.nslots;
    const uint32_t loc = lt.local0 + 4u * threadIdx.x;
    const uint32_t g = (uint32_t)RP.slot_base + loc;
    int4 pv = make_int4(-1, -1, -1, -1);
    if (loc < nslots) pv = (j == wg.x && lt.r == 0) ? pv_first : *reinterpret_cast<const int4*>(P.picks + g);
    const uint32_t key_off = type_of(P, RP.src_type).key_off;
    const int id[4] = {pv.x, pv.y, pv.z, pv.w};
    uint32_t key[4], go = 0u;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      key[q] = key_off + (uint32_t)id[q];
      if (loc + q < nslots && id[q] >= 0) go |= 1u << q;
    }
    go = tile_firsts(D, key, go, 4u * threadIdx.x);
#pragma unroll
    for (int q = 0; q < 4; ++q)
      if ((go >> q) & 1u) table_insert_min(P.ht, P.ver, key[q], EDGE_BIT | (g + q), P.state);
  }
}

// ------------------------------------------------------------------------------------------
// mark phase: tiles of TILE pick slots.  For every valid pick: order word of its id in the
// dedupe table, first-occurrence flag, ranks within the tile.  Tile totals go to `partial_*`.
// (A "last workgroup done" hand-off inside this kernel was measured and rejected: a device-scope
// fence per workgroup costs 1-15 us under load, a separate one-workgroup launch costs 2.4 us.)
// ------------------------------------------------------------------------------------------

// exclusive scan of two small counters over a 256-thread workgroup; returns totals in tot0/tot1
__device__ __forceinline__ void block_scan2(int v0, int v1, int& ex0, int& ex1, int& tot0, int& tot1, int* lds) {
  const int lane = lane_id(), w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  int i0 = v0, i1 = v1;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int a = __shfl_up(i0, o), b = __shfl_up(i1, o);
    if (lane >= o) { i0 += a; i1 += b; }
  }
  __syncthreads();
  if (lane == 63) { lds[w] = i0; lds[16 + w] = i1; }
  __syncthreads();
  int b0 = 0, b1 = 0, t0 = 0, t1 = 0;
  for (int q = 0; q < nw; ++q) {
    const int a = lds[q], b = lds[16 + q];
    if (q < w) { b0 += a; b1 += b; }
    t0 += a; t1 += b;
  }
  ex0 = b0 + i0 - v0; ex1 = b1 + i1 - v1; tot0 = t0; tot1 = t1;
}

constexpr int ITEMS = TILE / TILE_THREADS;   // 4 consecutive pick slots per thread: one 16-byte load / store each
static_assert(ITEMS == 4, "the mark and emit phases move int4 vectors");

template <class HP>
__device__ __forceinline__ void mark_phase(const HP& P, const Wg wg, int* lds, LiveLds* live) {
  // (the first tile's picks are requested ahead of the live counts, as in the insert phase)
  int4 pv_first = make_int4(-1, -1, -1, -1);
  if (wg.x < P.num_tiles_ub)
    pv_first = *reinterpret_cast<const int4*>(P.picks + (uint32_t)rel_of(P, 0).slot_base + (uint32_t)wg.x * TILE + ITEMS * threadIdx.x);
  live_tiles_setup(P, live);
  for (int j = wg.x; j < live->first[P.R]; j += P.gx) {
    const LiveTile lt = live_tile(P, live, j);
    const RelParam& RP = rel_of(P, lt.r);
    const uint32_t tile = lt.tile, nslots = lt.nslots;
    const uint32_t loc = lt.local0 + ITEMS * threadIdx.x;
    const uint32_t g = (uint32_t)RP.slot_base + loc;
    const int4 pv = (j == wg.x && lt.r == 0) ? pv_first : *reinterpret_cast<const int4*>(P.picks + g);   // (the buffer covers whole tiles)
    const uint32_t key_off = type_of(P, RP.src_type).key_off;
    int id[ITEMS] = {pv.x, pv.y, pv.z, pv.w};
    uint32_t w[ITEMS];
    int first[ITEMS], valid[ITEMS];
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
      if (loc + j >= nslots) id[j] = -1;
      valid[j] = id[j] >= 0 ? 1 : 0;
      w[j] = 0;
    }
#pragma unroll
    for (int j = 0; j < ITEMS; ++j)               // four independent table reads in flight
      if (valid[j]) w[j] = table_lookup(P.ht, P.ver, key_off + (uint32_t)id[j], P.state);
    int nf = 0, ne = 0;
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
      first[j] = (valid[j] && w[j] == (EDGE_BIT | (g + j))) ? 1 : 0;
      nf += first[j]; ne += valid[j];
    }
    int exf, exe, tf, te;
    block_scan2(nf, ne, exf, exe, tf, te, lds);
    uint32_t rk[ITEMS];
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
      rk[j] = (uint32_t)exf | ((uint32_t)exe << 16);
      exf += first[j]; exe += valid[j];
    }
    if (loc < nslots) {
      *reinterpret_cast<uint4*>(P.order + g) = make_uint4(w[0], w[1], w[2], w[3]);
      *reinterpret_cast<uint4*>(P.ranks + g) = make_uint4(rk[0], rk[1], rk[2], rk[3]);
    }
    if (threadIdx.x == 0) { P.partial_first[tile] = tf; P.partial_edge[tile] = te; }
  }
}

// Tile totals -> exclusive offsets and the hop's counts.  First occurrences run over the relations
// of one source node type in ascending order; edges restart per relation.  store(relation, tile within the
// relation, tile, first_off, edge_off) receives the offsets; when `write_counts`, num_src per node type (= next frontier size)
// and num_edges per relation go to the device state.
template <class HP, class Store>
__device__ __forceinline__ void scan_tiles(const HP& P, const LiveLds* live, Store store, bool write_counts, int* lds) {
  const int nthreads = (int)blockDim.x;
  for (int s = 0; s < P.T; ++s) {
    int run_first = 0;
    for (int r = 0; r < P.R; ++r) {
      const RelParam& RP = rel_of(P, r);
      if (RP.src_type != s) continue;
      const int ntiles = live->first[r + 1] - live->first[r];
      const int tbase = RP.slot_base / TILE;
      int run_edge = 0;
      for (int c = 0; c < ntiles; c += nthreads) {
        const int t = c + (int)threadIdx.x;
        int pf = 0, pe = 0;
        if (t < ntiles) { pf = P.partial_first[tbase + t]; pe = P.partial_edge[tbase + t]; }
        int exf, exe, tf, te;
        block_scan2(pf, pe, exf, exe, tf, te, lds);
        if (t < ntiles) store(r, t, tbase + t, run_first + exf, run_edge + exe);
        run_first += tf; run_edge += te;
      }
      if (write_counts && threadIdx.x == 0) P.state[ST_COUNTS + P.edge_count_off + P.hop * P.R + r] = run_edge;
    }
    if (write_counts && threadIdx.x == 0) P.state[ST_COUNTS + (P.hop + 1) * P.T + s] = frontier_count(P, s) + run_first;
  }
}

// scan phase (one workgroup): only hops with more than EMIT_SCAN_MAX_TILES tiles; otherwise every
// workgroup of the emit phase scans the tile totals itself, which saves a phase.
template <class HP>
__device__ __forceinline__ void scan_phase(const HP& P, int* lds, LiveLds* live) {
  live_tiles_setup(P, live);
  scan_tiles(P, live, [&](int, int, int tile, int fo, int eo) { P.first_off[tile] = fo; P.edge_off[tile] = eo; }, true, lds);
}

// ------------------------------------------------------------------------------------------
// emit phase: local ids and COO.  A pick whose id is a dst node has order < EDGE_BIT (the
// frontier index); otherwise order points at the id's first occurrence g0, whose local id is
// num_dst + (offset of g0's tile) + (rank of g0 within its tile).
// ------------------------------------------------------------------------------------------
// picks / order words / rank words of the four slots a thread owns in a tile
struct TileRegs { int4 pv; uint4 wv, rv; };
template <class HP>
__device__ __forceinline__ TileRegs load_tile_regs(const HP& P, uint32_t tile) {
  const uint32_t g = tile * TILE + ITEMS * threadIdx.x;   // relation slot bases are multiples of TILE
  TileRegs t;
  t.pv = *reinterpret_cast<const int4*>(P.picks + g);
  t.wv = *reinterpret_cast<const uint4*>(P.order + g);
  t.rv = *reinterpret_cast<const uint4*>(P.ranks + g);
  return t;
}

// (Loading a tile's vectors before the offsets are known, to overlap them with the tile-total scan,
// was measured and rejected: launches are sized by upper bounds, and the surplus workgroups' loads
// cost more than the overlap saves.)
template <class HP, class IntPtr, class EdgeOff>
__device__ __forceinline__ void emit_tiles(const HP& P, const Wg wg, const LiveLds* live, IntPtr first_off, EdgeOff edge_off_of) {
  for (int j = wg.x; j < live->first[P.R]; j += P.gx) {
    const LiveTile lt = live_tile(P, live, j);
    const RelParam& RP = rel_of(P, lt.r);
    const uint32_t tile = lt.tile, nslots = lt.nslots;
    const uint32_t loc = lt.local0 + ITEMS * threadIdx.x;
    if (loc >= nslots) continue;
    const uint32_t g = (uint32_t)RP.slot_base + loc;
    // three 16-byte loads in flight, then (for picks whose first occurrence is elsewhere) up to four
    // independent reads of that occurrence's rank word
    const TileRegs regs = load_tile_regs(P, tile);
    const int4 pv = regs.pv;
    const uint4 wv = regs.wv;
    const uint4 rv = regs.rv;
    const int num_dst_src = frontier_count(P, RP.src_type);
    const int eoff = edge_off_of(tile, j);
    int32_t* __restrict__ src_nodes = type_of(P, RP.src_type).src_nodes;
    const int id[ITEMS] = {pv.x, pv.y, pv.z, pv.w};
    const uint32_t w[ITEMS] = {wv.x, wv.y, wv.z, wv.w};
    const uint32_t rk[ITEMS] = {rv.x, rv.y, rv.z, rv.w};
    bool valid[ITEMS];
    uint32_t rk1[ITEMS];
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
      valid[j] = loc + j < nslots && id[j] >= 0;
      rk1[j] = rk[j];
      if (valid[j] && w[j] >= EDGE_BIT) {
        const uint32_t g1 = w[j] & ~EDGE_BIT;
        if (g1 != g + j) rk1[j] = P.ranks[g1];
      }
    }
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
      if (!valid[j]) continue;
      int lid;
      if (w[j] < EDGE_BIT) {
        lid = (int)w[j];                           // a dst node: its frontier index
      } else {
        const uint32_t g1 = w[j] & ~EDGE_BIT;
        lid = num_dst_src + first_off[g1 / TILE] + (int)(rk1[j] & 0xFFFFu);
        if (g1 == g + j) src_nodes[lid] = id[j];   // the first occurrence publishes the new source node
      }
      const int e = eoff + (int)(rk[j] >> 16);
      RP.src_local[e] = lid;
      RP.dst_local[e] = (int)((loc + j) / (uint32_t)P.f);
    }
  }
}

// The last hop's workgroup 0 also copies the device state (counts of every hop, error flag) into
// pinned host memory: the step needs no copy command after its kernels.
template <class HP>
__device__ __forceinline__ void publish_state(const HP& P, const Wg wg) {
  if (P.state_host == nullptr || wg.x != 0) return;
  __syncthreads();   // this workgroup's own count stores are visible to all its threads
  for (int i = (int)threadIdx.x; i < P.state_words; i += (int)blockDim.x) P.state_host[i] = P.state[i];
}

// Up to EMIT_SCAN_MAX_TILES tiles, every workgroup turns the tile totals into offsets in its own LDS
// (a few KB read from L2): first-occurrence offsets of all tiles (any tile may hold the first
// occurrence of one of this workgroup's picks), edge offsets of its own tiles only.  Workgroup 0 also
// publishes the hop's counts.
struct EmitLds {
  int scan[32];
  int first_off[EMIT_SCAN_MAX_TILES];
  int edge_own[EMIT_OWN_TILES];
};
template <class HP>
__device__ __forceinline__ void emit_phase(const HP& P, const Wg wg, EmitLds* L, LiveLds* live) {
  live_tiles_setup(P, live);
  // (the grid is sized by an estimate: a workgroup beyond the live tiles has nothing to emit; workgroup 0 stays
  // for the hop's counts)
  if (wg.x >= live->first[P.R] && wg.x != 0) return;
  if (!P.scan_in_emit) {            // offsets were produced by the scan phase
    const int32_t* eo = P.edge_off;
    emit_tiles(P, wg, live, (const int32_t*)P.first_off, [=](uint32_t tile, int) { return eo[tile]; });
    publish_state(P, wg);
    return;
  }
  // the workgroup's own tiles are the live tiles me, me + gx, ...: at most EMIT_OWN_TILES of them
  const int gx = P.gx, me = wg.x;
  scan_tiles(P, live, [&](int r, int t, int tile, int fo, int eo) {
    L->first_off[tile] = fo;
    const int j = live->first[r] + t;
    if (j % gx == me) L->edge_own[j / gx] = eo;
  }, wg.x == 0, L->scan);
  __syncthreads();
  emit_tiles(P, wg, live, (const int*)L->first_off, [=](uint32_t, int j) { return L->edge_own[j / gx]; });
  publish_state(P, wg);
}

// ------------------------------------------------------------------------------------------
// step_tick_kernel: a one-dimensional grid holds the workgroups of all slices back to back (slice i
// owns [end[i-1], end[i]), x-major within its gx * gy rectangle), so no workgroup is launched in vain.
// ------------------------------------------------------------------------------------------
template <int W>
union TickLds {
  GroupLdsT<W> group[GrpT<W>::PER_WG];
  int scan[32];
  EmitLds emit;
};
static_assert(sizeof(DedupeLds) <= sizeof(EmitLds), "the LDS stage of the dedupe borrows the emit phase's scratch");
// Scalar registers, not vector registers or LDS, decide how many workgroups a CU holds: with the 106 the
// compiler takes by itself 6 were resident per CU (measured: 191 per XCD at the peak of a full tick), capped at
// 96 it is 7 (223 per XCD); the spills go to lanes of a vector register.  Capping further for 8 costs more in
// spill code than the slots bring.
// The workgroup `block` of the slice with arguments P.
template <int W, bool DENSE, class HP>
__device__ __forceinline__ void run_slice(const HP& P, int block, const ChainArgs* C = nullptr) {
  // rows 0 .. gy-1 of the slice are gx workgroups wide, the gyd rows after them gxd (sample phase: the
  // rows of the node types need one thread per frontier node, not one 32-lane group)
  Wg wg;
  wg.x = block;
  wg.y = 0;
  while (wg.y < P.gy && wg.x >= P.gx) { wg.x -= P.gx; ++wg.y; }
  if (wg.y == P.gy && P.gxd > 0)
    while (wg.x >= P.gxd) { wg.x -= P.gxd; ++wg.y; }
  __shared__ TickLds<W> lds;
  __shared__ LiveLds live;
  __shared__ typename std::conditional<std::is_same<HP, HopParamsChain>::value && W == 32, ChainLds, int>::type chain_lds;
  (void)chain_lds;
  switch (P.phase) {
    case PH_SAMPLE: sample_phase(P, wg, lds.group); break;
    case PH_MARK:   mark_phase(P, wg, lds.scan, &live); break;
    case PH_SCAN:   scan_phase(P, lds.scan, &live); break;
    case PH_INSERT: insert_phase<std::is_base_of<HopParamsStaged, HP>::value>(P, wg, &live, reinterpret_cast<DedupeLds*>(&lds.emit)); break;
    case PH_EMIT:   emit_phase(P, wg, &lds.emit, &live); break;
    default:
      if constexpr (std::is_same<HP, HopParamsChain>::value && W == 32) {     // (only this build holds the visit-once code)
        if (P.phase == PH_PLACE) place_phase(P, wg, &live, reinterpret_cast<DedupeLds*>(&lds.emit));
        else if (P.phase == PH_CHAIN) chain_phase<!DENSE>(P, *C, wg, lds.group, &chain_lds);
      }
      break;
  }
}
template <class TP, int W, bool DENSE = false>
__device__ __forceinline__ void tick_body(const TP& M_by_value) {
  // The builds that carry a chain's arguments read their arguments where the launch put them, in the kernel argument
  // segment (constant memory: scalar loads with run-time offsets), not through the by-value parameter: indexing that with
  // the slice number made the compiler copy the whole structure to scratch memory there (from 8 slices on).  The other
  // builds keep the parameter: with the pointer the 1,024-seed FCR workload ran 4 % slower.
  typedef const __attribute__((address_space(4))) TP* KernargPtr;
  const TP& M = TP::HAS_CHAIN ? *(const TP*)(KernargPtr)__builtin_amdgcn_kernarg_segment_ptr() : M_by_value;
  int z = 0;
#pragma unroll
  for (int i = 0; i < TP::SLICES - 1; ++i) z += ((int)blockIdx.x >= M.end[i]) ? 1 : 0;
  const ChainArgs* chain = nullptr;
  if constexpr (TP::HAS_CHAIN) chain = &M.chain;
  run_slice<W, DENSE>(M.s[z], (int)blockIdx.x - (z ? M.end[z - 1] : 0), chain);
}
// Two builds of the same kernel.  With its scalar registers capped at 96 the kernel takes 67-72 vector registers:
// seven workgroups per CU.  The dense build is held to 64 (eight workgroups per CU) and pays for it with more scalar
// registers parked in vector lanes.  Launches of several times the chip's capacity gain from the eighth workgroup
// (65,536-seed steps -4 %, the seven-relation workload -1.5 %); ordinary ticks, whose time is set by the dependent
// chains of a few narrow slices, lose 3-6 % on the workloads with a refresh in the sample phase.
template <class TP, int W>
__global__ __launch_bounds__(256) __attribute__((amdgpu_num_sgpr(96))) void step_tick_kernel(TP M) { tick_body<TP, W>(M); }
template <class TP, int W = 32>
__global__ __launch_bounds__(256) __attribute__((amdgpu_num_sgpr(96), amdgpu_waves_per_eu(8, 8))) void step_tick_dense_kernel(TP M) {
  tick_body<TP, W, true>(M);
}
// The compact form for one-relation graphs: the slice's full arguments are put together from the launch's shared
// part, the slice's own part and the slot's entry of the device table (one more scalar load at the start).
template <int D>
__global__ __launch_bounds__(256) __attribute__((amdgpu_num_sgpr(96))) void step_tick_mono_kernel(TickMono<D> M) {
  int z = 0;
#pragma unroll
  for (int i = 0; i < D - 1; ++i) z += ((int)blockIdx.x >= M.end[i]) ? 1 : 0;
  const MonoSlice& c = M.s[z];
  const SlotConst& sc = M.h.slots[c.slot];
  HopParamsMonoRegs H;
  H.ht = sc.ht;
  H.state = sc.state;
  H.state_host = c.publish ? sc.state_host : nullptr;
  H.picks = sc.picks; H.order = sc.order; H.ranks = sc.ranks;
  H.partial_first = sc.partial_first; H.partial_edge = sc.partial_edge;
  H.first_off = sc.first_off; H.edge_off = sc.edge_off;
  H.phase = c.phase;
  H.gx = c.gx; H.gy = c.gy; H.gxd = c.gxd; H.gyd = c.gyd;
  H.R = 1; H.T = 1;
  H.hop = c.hop; H.f = c.f; H.k = M.h.k; H.S = M.h.S;
  H.n_new = c.n_new; H.mode = M.h.mode; H.refresh_now = c.refresh_now; H.band_offset = c.band_offset;
  H.num_tiles_ub = c.num_tiles_ub; H.edge_count_off = M.h.edge_count_off;
  H.scan_in_emit = c.scan_in_emit; H.state_words = M.h.state_words;
  H.shared = M.h.shared; H.layer = c.layer;
  H.insert_split = c.insert_split; H.slot = c.slot;
  H.ver = c.ver; H.step = c.step; H.layer_word = c.layer_word; H.seed_lo = M.h.seed_lo; H.seed_hi = M.h.seed_hi;
  H.rel[0].table = c.table; H.rel[0].src_local = c.src_local; H.rel[0].dst_local = c.dst_local;
  H.rel[0].slot_base = 0; H.rel[0].src_type = 0; H.rel[0].dst_type = 0;
  H.type[0].frontier = c.frontier; H.type[0].src_nodes = c.src_nodes;
  H.type[0].key_off = M.h.key_off; H.type[0].n_nodes = M.h.n_nodes;
  H.type[0].count_override = c.count_override; H.type[0].frontier_cap = c.frontier_cap;
  H.relc[0] = M.h.relc;
  run_slice<32, false>(H, (int)blockIdx.x - (z ? M.end[z - 1] : 0));
}

// ------------------------------------------------------------------------------------------
// Graph validation, cache read-out, checksum
// ------------------------------------------------------------------------------------------
__global__ void validate_graph_kernel(const void* indptr, int is64, int64_t n_dst, const int32_t* indices,
                                      int64_t nnz, int64_t n_src, int32_t* state) {
  const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t nth = (int64_t)gridDim.x * blockDim.x;
  bool bad = false;
  if (tid == 0) bad |= load_indptr(indptr, is64, 0) != 0 || load_indptr(indptr, is64, n_dst) != nnz;
  for (int64_t v = tid; v < n_dst; v += nth) {
    const int64_t d = load_indptr(indptr, is64, v + 1) - load_indptr(indptr, is64, v);
    bad |= d < 0 || d >= (int64_t(1) << 31);
  }
  for (int64_t e = tid; e < nnz; e += nth) bad |= (uint64_t)(int64_t)indices[e] >= (uint64_t)n_src;
  if (bad) atomicOr(&state[ST_ERROR], ERR_GRAPH);
}

__global__ void cache_read_kernel(const int32_t* table, const int32_t* row_of, int64_t n, int k, int S, int32_t* out) {
  const int64_t total = n * k;
  for (int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; c < total; c += (int64_t)gridDim.x * blockDim.x) {
    const int64_t v = c / k;
    const int j = (int)(c - v * k);
    const int64_t at = row_of ? (int64_t)row_of[v] : v;
    out[c] = at >= 0 ? table[at * S + j] : -1;
  }
}

__device__ __forceinline__ uint64_t mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

__global__ void cache_checksum_kernel(const int32_t* table, const int32_t* row_of, int64_t n, int k, int S,
                                      unsigned long long* out) {
  const int64_t total = n * k;
  uint64_t sum = 0;
  for (int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; c < total; c += (int64_t)gridDim.x * blockDim.x) {
    const int64_t v = c / k;
    const int j = (int)(c - v * k);
    const int64_t at = row_of ? (int64_t)row_of[v] : v;
    const int val = at >= 0 ? table[at * S + j] : -1;
    sum += mix64((uint64_t)c * 0x9E3779B97F4A7C15ull + (uint64_t)(uint32_t)val);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const uint32_t lo = __shfl_down((uint32_t)sum, o), hi = __shfl_down((uint32_t)(sum >> 32), o);
    sum += ((uint64_t)hi << 32) | lo;
  }
  if (lane_id() == 0) atomicAdd(out, (unsigned long long)sum);
}

// The same checksum without any allocation: every workgroup reduces one chunk of CK_CHUNK cells into its own word of a
// static scratch array (no atomics, nothing to clear), and a second one-workgroup kernel adds the words up into the
// caller's device word.  The array's name is only a host-side stand-in: kernels get the address that
// hipGetSymbolAddress returns for the current device (each GPU holds its own copy).
constexpr int CK_CHUNK = 16384;
constexpr int CK_MAX_PARTIALS = (int)(GSS_CHECKSUM_STATIC_MAX_CELLS / CK_CHUNK);
static __device__ __align__(256) unsigned long long scratch[CK_MAX_PARTIALS];   // 128 KB on every GPU the library runs on

__device__ __forceinline__ uint64_t block_sum_u64(uint64_t sum, unsigned long long* lds) {   // 256 threads; valid in thread 0
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const uint32_t lo = __shfl_down((uint32_t)sum, o), hi = __shfl_down((uint32_t)(sum >> 32), o);
    sum += ((uint64_t)hi << 32) | lo;
  }
  if (lane_id() == 0) lds[threadIdx.x >> 6] = sum;
  __syncthreads();
  return lds[0] + lds[1] + lds[2] + lds[3];
}

__global__ __launch_bounds__(256) void checksum_partials_kernel(const int32_t* table, const int32_t* row_of, int64_t n, int k,
                                                                int S, unsigned long long* partials) {
  __shared__ unsigned long long lds[4];
  const int64_t total = n * k, c0 = (int64_t)blockIdx.x * CK_CHUNK;
  uint64_t sum = 0;
  for (int i = (int)threadIdx.x; i < CK_CHUNK; i += 256) {
    const int64_t c = c0 + i;
    if (c >= total) break;
    const int64_t v = c / k;
    const int j = (int)(c - v * k);
    const int64_t at = row_of ? (int64_t)row_of[v] : v;
    const int val = at >= 0 ? table[at * S + j] : -1;
    sum += mix64((uint64_t)c * 0x9E3779B97F4A7C15ull + (uint64_t)(uint32_t)val);
  }
  const uint64_t t = block_sum_u64(sum, lds);
  if (threadIdx.x == 0) partials[blockIdx.x] = t;
}

__global__ __launch_bounds__(256) void checksum_finish_kernel(const unsigned long long* partials, int count, unsigned long long* out) {
  __shared__ unsigned long long lds[4];
  uint64_t sum = 0;
  for (int i = (int)threadIdx.x; i < count; i += 256) sum += partials[i];
  const uint64_t t = block_sum_u64(sum, lds);
  if (threadIdx.x == 0) *out = t;
}

// Row map of the degree split (built once, when the sampler is created).  Nodes are taken in chunks
// of 1024: count the nodes with deg > theta per chunk, scan the chunk counts (one workgroup), then
// number the nodes of every chunk.
constexpr int MAP_CHUNK = 1024;
__device__ __forceinline__ bool has_row(const void* indptr, int is64, int64_t v, int64_t n, int32_t theta) {
  return v < n && load_indptr(indptr, is64, v + 1) - load_indptr(indptr, is64, v) > (int64_t)theta;
}
__global__ __launch_bounds__(MAP_CHUNK) void row_map_count_kernel(const void* indptr, int is64, int64_t n, int32_t theta,
                                                                  int32_t* chunk_counts) {
  __shared__ int lds[32];
  const int64_t nchunks = (n + MAP_CHUNK - 1) / MAP_CHUNK;
  for (int64_t c = blockIdx.x; c < nchunks; c += gridDim.x) {
    const int flag = has_row(indptr, is64, c * MAP_CHUNK + threadIdx.x, n, theta) ? 1 : 0;
    int e0, e1, t0, t1;
    block_scan2(flag, 0, e0, e1, t0, t1, lds);
    if (threadIdx.x == 0) chunk_counts[c] = t0;
    __syncthreads();
  }
}
__global__ __launch_bounds__(MAP_CHUNK) void row_map_scan_kernel(int64_t nchunks, int32_t* chunk_counts, int32_t* num_rows) {
  __shared__ int lds[32];
  int run = 0;
  for (int64_t c0 = 0; c0 < nchunks; c0 += MAP_CHUNK) {
    const int64_t c = c0 + threadIdx.x;
    const int cnt = c < nchunks ? chunk_counts[c] : 0;
    int e0, e1, t0, t1;
    block_scan2(cnt, 0, e0, e1, t0, t1, lds);
    if (c < nchunks) chunk_counts[c] = run + e0;
    run += t0;
    __syncthreads();
  }
  if (threadIdx.x == 0) *num_rows = run;
}
__global__ __launch_bounds__(MAP_CHUNK) void row_map_assign_kernel(const void* indptr, int is64, int64_t n, int32_t theta,
                                                                   const int32_t* chunk_counts, int32_t* row_of) {
  __shared__ int lds[32];
  const int64_t nchunks = (n + MAP_CHUNK - 1) / MAP_CHUNK;
  for (int64_t c = blockIdx.x; c < nchunks; c += gridDim.x) {
    const int64_t v = c * MAP_CHUNK + threadIdx.x;
    const int flag = has_row(indptr, is64, v, n, theta) ? 1 : 0;
    int e0, e1, t0, t1;
    block_scan2(flag, 0, e0, e1, t0, t1, lds);
    if (v < n) row_of[v] = flag ? chunk_counts[c] + e0 : -1;
    __syncthreads();
  }
}

// list[row_of[v]] = v for the nodes that have a row in the map
__global__ void list_from_map_kernel(const int32_t* __restrict__ map, int64_t n, int32_t* __restrict__ list) {
  for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v < n; v += (int64_t)gridDim.x * blockDim.x) {
    const int r = map[v];
    if (r >= 0) list[r] = (int32_t)v;
  }
}

// ------------------------------------------------------------------------------------------
// Feature gather (the value side of the K-V cache: out[i] = H[ids[i]]).  LANES lanes (a power of two)
// share a row and walk over its 16 / 8 / 4 / 1-byte chunks, so a wavefront reads whole rows with
// consecutive vector loads; this is the one HBM-bound kernel of the library.
// ------------------------------------------------------------------------------------------
template <class VEC>
__global__ __launch_bounds__(256) void gather_rows_kernel(const VEC* __restrict__ table, int64_t num_rows, int chunks,
                                                          const int32_t* __restrict__ ids, int64_t num_ids,
                                                          VEC* __restrict__ out, int lanes_log2) {
  const int lanes = 1 << lanes_log2;
  const int rows_per_block = 256 >> lanes_log2;
  const int c0 = (int)threadIdx.x & (lanes - 1);
  for (int64_t i = (int64_t)blockIdx.x * rows_per_block + ((int)threadIdx.x >> lanes_log2); i < num_ids;
       i += (int64_t)gridDim.x * rows_per_block) {
    const int64_t v = ids[i];
    const bool ok = v >= 0 && v < num_rows;
    const VEC* __restrict__ src = table + v * chunks;
    VEC* __restrict__ dst = out + i * chunks;
    for (int c = c0; c < chunks; c += lanes) dst[c] = ok ? src[c] : VEC{};
  }
}

__global__ void fill_i64_kernel(long long* p, int64_t n, long long value) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = value;
}

// ------------------------------------------------------------------------------------------
// Launch wrappers (host)
// ------------------------------------------------------------------------------------------
static inline unsigned clamp_grid(int64_t want, int64_t cap) {
  if (want < 1) want = 1;
  return (unsigned)(want < cap ? want : cap);
}

hipError_t launch_fill_full(const FillParams& P, hipStream_t st, LaunchTimer* timer) {
  const unsigned grid = clamp_grid((P.n_dst + FILL_CHUNK - 1) / FILL_CHUNK, 8192);
  hipEvent_t start = nullptr, stop = nullptr;
  void (*const kernel)(FillParams) = P.k > 32 ? fill_full_kernel<64> : fill_full_kernel<32>;   // rows wider than half a wavefront
  if (timer && timer->bracket(KID_FILL_FULL, &start, &stop))      // the events get the dispatch's own start / end times
    hipExtLaunchKernelGGL(kernel, dim3(grid), dim3(256), 0, st, start, stop, 0, P);
  else
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(256), 0, st, P);
  return hipGetLastError();
}

hipError_t launch_fill_heavy(const FillParams& P, const int32_t* heavy, int64_t nheavy, hipStream_t st, LaunchTimer* timer) {
  if (nheavy <= 0) return hipSuccess;
  const int groups = P.k > 32 ? 4 : 8;
  const unsigned grid = clamp_grid((nheavy * P.ntab + groups - 1) / groups, 16384);
  hipEvent_t start = nullptr, stop = nullptr;
  void (*const kernel)(FillParams, const int32_t*, int64_t) = P.k > 32 ? fill_heavy_kernel<64> : fill_heavy_kernel<32>;
  if (timer && timer->bracket(KID_FILL_FULL, &start, &stop))
    hipExtLaunchKernelGGL(kernel, dim3(grid), dim3(256), 0, st, start, stop, 0, P, heavy, nheavy);
  else
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(256), 0, st, P, heavy, nheavy);
  return hipGetLastError();
}

hipError_t launch_list_from_map(const int32_t* map, int64_t n, int32_t* list, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(list_from_map_kernel, dim3(clamp_grid((n + 255) / 256, 8192)), dim3(256), 0, st, map, n, list);
  return hipGetLastError();
}

int tick_capacity(int R, int T) {
  if (R == 1 && T == 1) return TICK_MONO_SLICES;
  if (R <= HopParamsSmall::MAX_R && T <= HopParamsSmall::MAX_T) return 9;
  if (R <= HopParamsMid::MAX_R && T <= HopParamsMid::MAX_T) return 6;
  return 4;
}

template <class HP, int D>
static hipError_t launch_tick_t(const HopParams* P, int n, const RelConst* relc_host, const RelConst* relc_dev,
                                const ChainArgs* chain, hipStream_t st, LaunchTimer* timer, hipEvent_t done, bool dense,
                                int width = 0) {
  using TP = TickT<HP, D>;
  static_assert(sizeof(TP) <= 4000, "kernel arguments are limited to 4 KB");
  TP M;
  if constexpr (TP::HAS_CHAIN) {
    if (chain) M.chain = *chain; else memset(static_cast<void*>(&M.chain), 0, sizeof M.chain);
  } else if (chain) {
    return hipErrorInvalidValue;
  }
  int total = 0;
  for (int i = 0; i < D; ++i) {
    const HopParams& src = P[i < n ? i : 0];        // unused slices repeat the first and own no workgroup
    static_cast<HopCommon&>(M.s[i]) = static_cast<const HopCommon&>(src);
    for (int r = 0; r < HP::MAX_R; ++r) M.s[i].rel[r] = src.rel[r];
    for (int t = 0; t < HP::MAX_T; ++t) M.s[i].type[t] = src.type[t];
    M.s[i].set_consts(relc_host, relc_dev);
    if (i < n) total += src.gx * src.gy + src.gxd * src.gyd;
    M.end[i] = total;
  }
  hipEvent_t start = nullptr, stop = nullptr;
  // rows of more than 32 slots: the build with one node per wavefront (it has no dense variant, and no chain code);
  // rows of up to 20 / 16 slots on one-relation graphs: the builds with three / four nodes per wavefront
  const bool wide = P[0].k > 32;
  void (*kernel)(TP) = dense ? step_tick_dense_kernel<TP> : step_tick_kernel<TP, 32>;
  if constexpr (TP::HAS_CHAIN) {
    if (wide || (width != 0 && width != 32)) return hipErrorInvalidValue;
  } else if (wide) {
    if (width != 0 && width != 64) return hipErrorInvalidValue;
    kernel = step_tick_kernel<TP, 64>;
  } else if (width == 21 || width == 16) {
    if constexpr (std::is_same<HP, HopParamsMono>::value) {
      if (width == 21) kernel = dense ? step_tick_dense_kernel<TP, 21> : step_tick_kernel<TP, 21>;
      else kernel = dense ? step_tick_dense_kernel<TP, 16> : step_tick_kernel<TP, 16>;
    } else {
      return hipErrorInvalidValue;
    }
  } else if (width != 0 && width != 32) {
    return hipErrorInvalidValue;
  }
  if (timer && timer->bracket(KID_STEP_TICK, &start, &stop))
    hipExtLaunchKernelGGL(kernel, dim3((unsigned)total), dim3(256), 0, st, start, stop, 0, M);
  else if (done)   // the dispatch itself completes the event: no separate marker between this launch and the next
    hipExtLaunchKernelGGL(kernel, dim3((unsigned)total), dim3(256), 0, st, nullptr, done, 0, M);
  else
    hipLaunchKernelGGL(kernel, dim3((unsigned)total), dim3(256), 0, st, M);
  if (timer && done) {
    const hipError_t e = hipEventRecord(done, st);
    if (e != hipSuccess) return e;
  }
  return hipGetLastError();
}

// The compact launch: slices of one-relation graphs, up to TICK_MONO_SLICES of them.
static hipError_t launch_tick_mono(const HopParams* P, int n, const RelConst* relc_host, const SlotConst* slots_dev,
                                   hipStream_t st, LaunchTimer* timer, hipEvent_t done) {
  using TM = TickMono<TICK_MONO_SLICES>;
  static_assert(sizeof(TM) <= 4000, "kernel arguments are limited to 4 KB");
  TM M;
  memset(static_cast<void*>(&M), 0, sizeof M);
  const HopParams& A = P[0];
  M.h.relc = relc_host[0];
  M.h.slots = slots_dev;
  M.h.key_off = A.type[0].key_off; M.h.n_nodes = A.type[0].n_nodes;
  M.h.k = A.k; M.h.S = A.S; M.h.mode = A.mode; M.h.shared = A.shared;
  M.h.state_words = A.state_words; M.h.edge_count_off = A.edge_count_off;
  M.h.seed_lo = A.seed_lo; M.h.seed_hi = A.seed_hi;
  int total = 0;
  for (int i = 0; i < TICK_MONO_SLICES; ++i) {
    const HopParams& src = P[i < n ? i : 0];        // unused slices repeat the first and own no workgroup
    MonoSlice& c = M.s[i];
    c.table = src.rel[0].table; c.src_local = src.rel[0].src_local; c.dst_local = src.rel[0].dst_local;
    c.frontier = src.type[0].frontier; c.src_nodes = src.type[0].src_nodes;
    c.count_override = src.type[0].count_override; c.frontier_cap = src.type[0].frontier_cap;
    c.num_tiles_ub = src.num_tiles_ub; c.gx = src.gx; c.gxd = src.gxd; c.band_offset = src.band_offset;
    c.ver = src.ver; c.step = src.step; c.layer_word = src.layer_word;
    c.slot = (uint8_t)src.slot; c.phase = (uint8_t)src.phase; c.hop = (uint8_t)src.hop; c.layer = (uint8_t)src.layer;
    c.f = (uint8_t)src.f; c.n_new = (uint8_t)src.n_new; c.refresh_now = (uint8_t)src.refresh_now;
    c.scan_in_emit = (uint8_t)src.scan_in_emit; c.insert_split = (uint8_t)src.insert_split;
    c.publish = src.state_host ? 1 : 0; c.gy = (uint8_t)src.gy; c.gyd = (uint8_t)src.gyd;
    if (src.rel[0].slot_base != 0 || src.f > 255 || src.n_new > 255 || src.gy > 255 || src.gyd > 255)
      return hipErrorInvalidValue;
    if (i < n) total += src.gx * src.gy + src.gxd * src.gyd;
    M.end[i] = total;
  }
  hipEvent_t start = nullptr, stop = nullptr;
  if (timer && timer->bracket(KID_STEP_TICK, &start, &stop))
    hipExtLaunchKernelGGL(step_tick_mono_kernel<TICK_MONO_SLICES>, dim3((unsigned)total), dim3(256), 0, st, start, stop, 0, M);
  else if (done)
    hipExtLaunchKernelGGL(step_tick_mono_kernel<TICK_MONO_SLICES>, dim3((unsigned)total), dim3(256), 0, st, nullptr, done, 0, M);
  else
    hipLaunchKernelGGL(step_tick_mono_kernel<TICK_MONO_SLICES>, dim3((unsigned)total), dim3(256), 0, st, M);
  if (timer && done) {
    const hipError_t e = hipEventRecord(done, st);
    if (e != hipSuccess) return e;
  }
  return hipGetLastError();
}

hipError_t launch_tick(const HopParams* P, int n, const RelConst* relc_host, const RelConst* relc_dev,
                       const SlotConst* slots_dev, bool chain_build, const ChainArgs* chain, hipStream_t st, LaunchTimer* timer,
                       hipEvent_t done, bool dense, int width) {
  if (n < 1 || n > tick_capacity(P[0].R, P[0].T)) return hipErrorInvalidValue;
  const int R = P[0].R, T = P[0].T;
  if (chain_build) {
    if (R != 1 || T != 1 || n > CHAIN_TICK_SLICES) return hipErrorInvalidValue;
    if (n == 1) return launch_tick_t<HopParamsChain, 1>(P, n, relc_host, relc_dev, chain, st, timer, done, dense);
    if (n <= 4) return launch_tick_t<HopParamsChain, 4>(P, n, relc_host, relc_dev, chain, st, timer, done, dense);
    return launch_tick_t<HopParamsChain, CHAIN_TICK_SLICES>(P, n, relc_host, relc_dev, chain, st, timer, done, dense);
  }
  if (chain) return hipErrorInvalidValue;
  if (P[0].insert_split & 2) {      // the sampler uses the LDS stage of the dedupe: a build of its own (one relation, rows of up to 32 slots)
    if (R != 1 || T != 1 || n > 12 || P[0].k > 32) return hipErrorInvalidValue;
    return launch_tick_t<HopParamsStaged, 12>(P, n, relc_host, relc_dev, nullptr, st, timer, done, dense);
  }
  const bool narrow = width == 21 || width == 16;
  if (narrow && (chain_build || (P[0].insert_split & 2) || R != 1 || T != 1 || n > 12)) return hipErrorInvalidValue;
  if (R == 1 && T == 1 && n > 12) {
    if (!slots_dev || P[0].k > 32) return hipErrorInvalidValue;   // (the compact form has no build for wide rows)
    return launch_tick_mono(P, n, relc_host, slots_dev, st, timer, done);
  }
  if (R == 1 && T == 1) {
    // (the one-slice builds with narrow groups would spill vector registers when held to 64 of them)
    if (n == 1) return launch_tick_t<HopParamsMono, 1>(P, n, relc_host, relc_dev, chain, st, timer, done, dense && !narrow, width);
    if (n <= 4) return launch_tick_t<HopParamsMono, 4>(P, n, relc_host, relc_dev, chain, st, timer, done, dense, width);
    if (n <= 8) return launch_tick_t<HopParamsMono, 8>(P, n, relc_host, relc_dev, chain, st, timer, done, dense, width);
    return launch_tick_t<HopParamsMono, 12>(P, n, relc_host, relc_dev, chain, st, timer, done, dense, width);
  }
  if (R <= HopParamsSmall::MAX_R && T <= HopParamsSmall::MAX_T) {
    if (n == 1) return launch_tick_t<HopParamsSmall, 1>(P, n, relc_host, relc_dev, chain, st, timer, done, dense);
    if (n <= 3) return launch_tick_t<HopParamsSmall, 3>(P, n, relc_host, relc_dev, chain, st, timer, done, dense);
    if (n <= 6) return launch_tick_t<HopParamsSmall, 6>(P, n, relc_host, relc_dev, chain, st, timer, done, dense);
    return launch_tick_t<HopParamsSmall, 9>(P, n, relc_host, relc_dev, chain, st, timer, done, dense);
  }
  if (R <= HopParamsMid::MAX_R && T <= HopParamsMid::MAX_T) {
    if (n == 1) return launch_tick_t<HopParamsMid, 1>(P, n, relc_host, relc_dev, chain, st, timer, done, dense);
    if (n <= 3) return launch_tick_t<HopParamsMid, 3>(P, n, relc_host, relc_dev, chain, st, timer, done, dense);
    return launch_tick_t<HopParamsMid, 6>(P, n, relc_host, relc_dev, chain, st, timer, done, dense);
  }
  if (n == 1) return launch_tick_t<HopParams, 1>(P, n, relc_host, relc_dev, chain, st, timer, done, dense);
  if (n == 2) return launch_tick_t<HopParams, 2>(P, n, relc_host, relc_dev, chain, st, timer, done, dense);
  return launch_tick_t<HopParams, 4>(P, n, relc_host, relc_dev, chain, st, timer, done, dense);
}

hipError_t launch_validate_graph(const void* indptr, int is64, int64_t n_dst, const int32_t* indices, int64_t nnz,
                                 int64_t n_src, int32_t* state, hipStream_t st) {
  const int64_t work = nnz > n_dst ? nnz : n_dst;
  const unsigned grid = clamp_grid((work + 255) / 256, 8192);
  hipLaunchKernelGGL(validate_graph_kernel, dim3(grid), dim3(256), 0, st, indptr, is64, n_dst, indices, nnz, n_src, state);
  return hipGetLastError();
}

hipError_t launch_cache_read(const int32_t* table, const int32_t* row_of, int64_t n, int k, int S, int32_t* out,
                             hipStream_t st) {
  const unsigned grid = clamp_grid((n * k + 255) / 256, 8192);
  hipLaunchKernelGGL(cache_read_kernel, dim3(grid), dim3(256), 0, st, table, row_of, n, k, S, out);
  return hipGetLastError();
}

hipError_t launch_cache_checksum(const int32_t* table, const int32_t* row_of, int64_t n, int k, int S,
                                 unsigned long long* out, hipStream_t st) {
  const unsigned grid = clamp_grid((n * k + 255) / 256, 4096);
  hipLaunchKernelGGL(cache_checksum_kernel, dim3(grid), dim3(256), 0, st, table, row_of, n, k, S, out);
  return hipGetLastError();
}

hipError_t launch_cache_checksum_static(const int32_t* table, const int32_t* row_of, int64_t n, int k, int S,
                                        unsigned long long* out, hipStream_t st) {
  constexpr int MAX_DEVICES = 64;
  static unsigned long long* scratch_of[MAX_DEVICES];     // device address of `scratch`, per device (set once; racing
  int dev = -1;                                            // first calls store the same value)
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  if (!scratch_of[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    scratch_of[dev] = (unsigned long long*)p;
  }
  const int64_t total = n * k;
  if (total > (int64_t)GSS_CHECKSUM_STATIC_MAX_CELLS) return hipErrorInvalidValue;
  const int chunks = (int)((total + CK_CHUNK - 1) / CK_CHUNK);
  unsigned long long* partials = scratch_of[dev];
  if (chunks > 0)
    hipLaunchKernelGGL(checksum_partials_kernel, dim3((unsigned)chunks), dim3(256), 0, st, table, row_of, n, k, S, partials);
  hipLaunchKernelGGL(checksum_finish_kernel, dim3(1), dim3(256), 0, st, (const unsigned long long*)partials, chunks, out);
  return hipGetLastError();
}

hipError_t launch_build_row_map(const void* indptr, int is64, int64_t n, int32_t theta, int32_t* chunk_counts,
                                int32_t* row_of, int32_t* num_rows, hipStream_t st) {
  const int64_t nchunks = (n + MAP_CHUNK - 1) / MAP_CHUNK;
  const unsigned grid = clamp_grid(nchunks, 4096);
  if (nchunks > 0) hipLaunchKernelGGL(row_map_count_kernel, dim3(grid), dim3(MAP_CHUNK), 0, st, indptr, is64, n, theta, chunk_counts);
  hipLaunchKernelGGL(row_map_scan_kernel, dim3(1), dim3(MAP_CHUNK), 0, st, nchunks, chunk_counts, num_rows);
  if (nchunks > 0) hipLaunchKernelGGL(row_map_assign_kernel, dim3(grid), dim3(MAP_CHUNK), 0, st, indptr, is64, n, theta, chunk_counts, row_of);
  return hipGetLastError();
}

template <class VEC>
static hipError_t launch_gather_t(const void* table, int64_t num_rows, int64_t row_bytes, const int32_t* ids,
                                  int64_t num_ids, void* out, hipStream_t st) {
  const int chunks = (int)(row_bytes / (int64_t)sizeof(VEC));
  int lanes_log2 = 0;
  while ((1 << lanes_log2) < chunks && lanes_log2 < 6) ++lanes_log2;
  const int rows_per_block = 256 >> lanes_log2;
  const unsigned grid = clamp_grid((num_ids + rows_per_block - 1) / rows_per_block, 1 << 20);
  hipLaunchKernelGGL(gather_rows_kernel<VEC>, dim3(grid), dim3(256), 0, st, (const VEC*)table, num_rows, chunks, ids,
                     num_ids, (VEC*)out, lanes_log2);
  return hipGetLastError();
}

hipError_t launch_gather_rows(const void* table, int64_t num_rows, int64_t row_bytes, const int32_t* ids, int64_t num_ids,
                              void* out, hipStream_t st) {
  const uintptr_t align = (uintptr_t)table | (uintptr_t)out | (uintptr_t)row_bytes;   // widest vector all three allow
  if (align % 16 == 0) return launch_gather_t<uint4>(table, num_rows, row_bytes, ids, num_ids, out, st);
  if (align % 8 == 0) return launch_gather_t<uint2>(table, num_rows, row_bytes, ids, num_ids, out, st);
  if (align % 4 == 0) return launch_gather_t<uint32_t>(table, num_rows, row_bytes, ids, num_ids, out, st);
  return launch_gather_t<uint8_t>(table, num_rows, row_bytes, ids, num_ids, out, st);
}

hipError_t launch_fill_i64(long long* p, int64_t n, long long value, hipStream_t st) {
  const unsigned grid = clamp_grid((n + 255) / 256, 8192);
  hipLaunchKernelGGL(fill_i64_kernel, dim3(grid), dim3(256), 0, st, p, n, value);
  return hipGetLastError();
}

}  // namespace gss
