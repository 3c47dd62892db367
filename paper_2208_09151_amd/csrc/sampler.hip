// Superbatch neighbour sampling on gfx950 (Ginex Section 3.1 "Superbatch Sample";
// sampling rule of Section 2.1 "Neighborhood Sampling").
//
// All S batches of the superbatch advance hop by hop in the same launches, so a hop is a
// handful of grid-wide kernels over (batch, frontier slot) instead of S small ones:
//
//   plan    every batch gets a hash table sized for what the hop can add at most
//           (list + frontier * fanout, two slots per possible entry), packed back to back;
//           the used region is cleared and the batch's current list re-inserted.  Tables
//           sized to the need instead of the worst case keep many entries per cache line
//           and the working set of the batches in flight inside L2 / Infinity Cache.
//   pick    a group of G lanes (G = 16/32/64 >= fanout) serves one frontier node: the
//           lanes draw their Philox words in parallel, resolve Floyd's subset rule with
//           group ballots, rank the picks, read the neighbours and insert them into the
//           batch's open-addressing hash table, keeping the smaller candidate rank per id.
//           The rank (frontier slot * fanout + pick slot) is exactly the order in which a
//           sequential scan would meet the candidate, so after the kernel every new id
//           holds the rank of its first occurrence.  A lane knows at once whether its
//           candidate lost (the id is in the list already, or in the table with a smaller
//           rank); a candidate that holds its slot may still be displaced by a smaller rank
//           arriving later, and the displacing lane records that.  The group's ballot of
//           holders is the first-occurrence mask.
//   count   per 256 frontier slots: number of picks and of first occurrences (mask minus
//           displaced), from sequential arrays: no table access.
//   scan    one block per batch scans its tile counts; one block turns the per-batch
//           totals into output offsets.
//   emit    appends the first occurrences to the batch's list at their scanned positions,
//           writes the hop's rowptr and the adj_col entries of the first occurrences.
//   col     the remaining picks get their position for adj_col: an id of an earlier stage
//           saw it in the table when it lost, an id seen earlier in this hop looks it up
//           through its slot.
//
// The seeds go through the same count/scan/emit path as a stage with one candidate per
// slot, which also removes repeated seeds.
//
// Where the hash set of a batch's seeds and first hop fits LDS (the usual case), those two
// stages run in one workgroup per batch with the table in LDS instead (k_front_lds, further
// down); the later hops, whose sets are far too large for that, run as described above.
#include <cstdlib>
#include <cstring>
#include <vector>

#include "common.hpp"

namespace ginex {
namespace {

constexpr int TB = 256;                  // threads per block everywhere in this file
constexpr uint32_t PEND = 0x40000000u;   // value = PEND + rank while an id is new in this stage

// Philox4x32-10 (Salmon et al., SC'11), counter (node, batch, hop, draw), key = seed.
// Returns words 0 (low) and 1 (high) of the block as one 64-bit draw.
__device__ __forceinline__ uint64_t philox_draw(uint64_t seed, uint32_t node, uint32_t batch,
                                                uint32_t hop, uint32_t draw) {
  uint32_t c0 = node, c1 = batch, c2 = hop, c3 = draw;
  uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    c0 = hi1 ^ c1 ^ k0;
    c1 = lo1;
    c2 = hi0 ^ c3 ^ k1;
    c3 = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return ((uint64_t)c1 << 32) | c0;
}

struct Tables {
  uint64_t* tab;         // packed per-batch tables, one 64-bit (key, value) word per slot
  int64_t* tab_off;      // [S] first slot of batch b's table
  uint32_t* tab_slots;   // [S] its number of slots
  uint64_t* first;       // [S][fr_slots] bit s set: pick s of the slot holds its id's table slot
  uint64_t* displaced;   // [S][fr_slots] bit s set: ... but a smaller rank took it over later
  int32_t* cand;         // [S][cand_slots] candidate node ids of the running stage
  uint32_t* ref;         // [S][cand_slots] where a pick finds its list position: OLD_ID |
                         // position (an id of an earlier stage), else its table slot
  uint8_t* cnt;          // [S][fr_slots] picks per frontier slot
  int64_t cand_slots, fr_slots;
  int32_t* wlist;        // [S][stride_ids] the growing list of every batch
  int64_t stride_ids;
};

// A slot is one 64-bit word: key in the high half, value in the low half, all ones = free.
// The value of an id of an earlier stage is its list position, that of an id new in this
// stage PEND + the smallest candidate rank it was seen with.
constexpr uint64_t FREE_SLOT = ~0ull;
constexpr uint32_t OLD_ID = 0x80000000u;

__device__ __forceinline__ uint32_t hash_slot(uint32_t id, uint32_t slots) {
  return __umulhi(id * 2654435761u, slots);
}

// Puts the list a batch has so far back into its freshly sized table.
__device__ __forceinline__ void table_put(uint64_t* t, uint32_t slots, uint32_t id, uint32_t value) {
  const unsigned long long mine = ((unsigned long long)id << 32) | value;
  unsigned long long* tab = reinterpret_cast<unsigned long long*>(t);
  uint32_t h = hash_slot(id, slots);
  while (atomicCAS(&tab[h], FREE_SLOT, mine) != FREE_SLOT) h = h + 1 == slots ? 0 : h + 1;
}

// Inserts candidate (id, rank) of the running stage, keeping the smaller rank per id, and
// leaves the pick's reference for k_col.  One 64-bit compare-and-swap when the id is new
// (the usual case); an id that is present needs a second atomic only if this rank is smaller
// than the stored one, and the rank it replaces is recorded as displaced.  Returns whether
// the candidate holds its id's slot now (a smaller rank may still take it over later).
__device__ __forceinline__ bool place_candidate(const Tables& T, int b, int k, uint32_t id,
                                                uint32_t rank) {
  const uint32_t slots = T.tab_slots[b];
  unsigned long long* tab = reinterpret_cast<unsigned long long*>(T.tab + T.tab_off[b]);
  const unsigned long long mine = ((unsigned long long)id << 32) | (PEND + rank);
  uint32_t* ref = T.ref + (int64_t)b * T.cand_slots + rank;
  uint32_t h = hash_slot(id, slots);
  while (true) {
    const unsigned long long old = atomicCAS(&tab[h], FREE_SLOT, mine);
    if (old == FREE_SLOT) {
      *ref = h;
      return true;
    }
    if ((uint32_t)(old >> 32) == id) {
      const uint32_t there = (uint32_t)old;
      if (there < PEND) {             // in the list since an earlier stage: `there` is its position
        *ref = OLD_ID | there;
        return false;
      }
      *ref = h;
      if (there < (uint32_t)mine) return false;
      const uint32_t before = (uint32_t)atomicMin(&tab[h], mine);
      if (before < (uint32_t)mine) return false;   // an even smaller rank got in between
      const uint32_t gone = before - PEND;
      atomicOr((unsigned long long*)&T.displaced[(int64_t)b * T.fr_slots + gone / k],
               1ull << (gone % k));
      return true;
    }
    h = h + 1 == slots ? 0 : h + 1;
  }
}

// Which (batch, tile) a block works on.  Grids are one-dimensional and the hardware deals
// consecutive workgroups round-robin to the 8 XCDs, each with its own L2; block n therefore
// takes a tile of a batch whose index is congruent to n modulo 8, so that all tiles of a
// batch, and with them the batch's lists, candidates and hash table, stay in one XCD's L2
// instead of being fetched by all eight.  (Only locality depends on the dealing order, not
// correctness.  The table's inserts gain nothing from it: a device-scope atomic is carried
// out on the memory side of the fabric whatever the L2 holds; the plain reads do.)
constexpr int XCDS = 8;

struct Where {
  int b;          // batch, or -1 if the block has none
  int64_t tile;   // tile of the batch's frontier slots
};

__device__ __forceinline__ Where where_am_i(int S, int64_t tiles_per_batch) {
  const int64_t n = blockIdx.x;
  const int64_t m = n / XCDS;
  Where w;
  w.tile = m % tiles_per_batch;
  const int64_t b = (m / tiles_per_batch) * XCDS + n % XCDS;
  w.b = b < S ? (int)b : -1;
  return w;
}

inline unsigned grid_blocks(int S, int64_t tiles_per_batch) {
  return (unsigned)(XCDS * ceil_div(S, XCDS) * tiles_per_batch);
}

// Launches are sized on the host for the worst case a hop allows (every node so far with a
// full fanout of new neighbours), which is several times what a frontier really holds, and
// a block that finds nothing to do still costs its dispatch.  So a grid holds at most this
// many tiles per batch and a block strides over the tiles its batch really has.
constexpr int64_t SLOT_TILES = 128;   // tiles of TB frontier slots
constexpr int64_t PICK_TILES = 512;   // tiles of TB/G frontier nodes

// GINEX_SAMPLER_TILES=n in the environment replaces both caps (any n >= 1 gives the same
// result: only the assignment of tiles to blocks, and with it the order in which candidates
// reach the hash tables, changes; the determinism tests use it).
inline int64_t tile_cap(int64_t standard) {
  const char* env = getenv("GINEX_SAMPLER_TILES");
  const long n = env ? atol(env) : 0;
  return n >= 1 ? n : standard;
}

inline int64_t capped(int64_t tiles, int64_t most) { return tiles < most ? tiles : most; }

// Single block: table sizes and offsets for the stage that is about to run.
__global__ __launch_bounds__(TB) void k_table_plan(Tables T, int S, int64_t num_nodes, int k,
                                                   const int32_t* __restrict__ nfront,
                                                   const int32_t* __restrict__ nlist,
                                                   int64_t* __restrict__ total_slots) {
  __shared__ int64_t smem[TB / WAVE + 1];
  int64_t run = 0;
  for (int base = 0; base < S; base += TB) {
    const int b = base + threadIdx.x;
    int64_t slots = 0;
    if (b < S) {
      int64_t bound = (int64_t)nlist[b] + (int64_t)nfront[b] * k;
      if (bound > num_nodes) bound = num_nodes;
      slots = 2 * bound < 32 ? 32 : 2 * bound;
    }
    int64_t total;
    const int64_t ex = block_exclusive_scan<int64_t, TB>(slots, smem, total);
    if (b < S) {
      T.tab_off[b] = run + ex;
      T.tab_slots[b] = (uint32_t)slots;
    }
    run += total;
  }
  if (threadIdx.x == 0) *total_slots = run;
}

__global__ __launch_bounds__(TB) void k_table_clear(Tables T, const int64_t* __restrict__ total_slots,
                                                    const int32_t* __restrict__ nfront, int S,
                                                    int64_t front) {
  const int64_t n = *total_slots;
  const int64_t span = (int64_t)gridDim.x * TB;
  const int64_t me = (int64_t)blockIdx.x * TB + threadIdx.x;
  for (int64_t i = me; i < n; i += span) T.tab[i] = FREE_SLOT;
  // and the displacements of the stage before: displaced[b][0 .. nfront[b]) <- 0
  for (int64_t i = me; i < (int64_t)S * front; i += span) {
    const int64_t b = i / front, j = i - b * front;
    if (j < nfront[b]) T.displaced[b * T.fr_slots + j] = 0;
  }
}

// Put the list a batch has so far back into its freshly sized table.
__global__ __launch_bounds__(TB) void k_reinsert(Tables T, const int32_t* __restrict__ nlist,
                                                 int S, int64_t tpb) {
  const Where at = where_am_i(S, tpb);
  if (at.b < 0) return;
  const int b = at.b;
  uint64_t* t = T.tab + T.tab_off[b];
  const uint32_t slots = T.tab_slots[b];
  for (int64_t j = at.tile * TB + threadIdx.x; j < nlist[b]; j += tpb * TB)
    table_put(t, slots, (uint32_t)T.wlist[b * T.stride_ids + j], (uint32_t)j);
}

// Stage "seeds": slot j of batch b holds seed j.
__global__ __launch_bounds__(TB) void k_seed_stage(Tables T, const int32_t* __restrict__ seeds,
                                                   const int64_t* __restrict__ seed_off,
                                                   const int32_t* __restrict__ nfront, int S,
                                                   int64_t tpb) {
  const Where at = where_am_i(S, tpb);
  if (at.b < 0) return;
  const int b = at.b;
  for (int64_t j = at.tile * TB + threadIdx.x; j < nfront[b]; j += tpb * TB) {
    const uint32_t id = (uint32_t)seeds[seed_off[b] + j];
    T.cand[b * T.cand_slots + j] = (int32_t)id;
    T.first[b * T.fr_slots + j] = place_candidate(T, b, 1, id, (uint32_t)j) ? 1ull : 0ull;
    T.cnt[b * T.fr_slots + j] = 1;
  }
}

// Where the neighbour list of node v starts and how long it is.  NC: neighbour lists are
// looked up in the neighbour cache first (Section 3.2: address table, then the count in front
// of the record, then the neighbours); a miss falls back to the CSR, which then may sit in
// host memory.  `cached` tells which array `lo` indexes.
template <typename OffT, bool NC>
__device__ __forceinline__ void row_of(uint32_t v, const OffT* __restrict__ offsets,
                                       const int64_t* __restrict__ nc_address_table,
                                       const int32_t* __restrict__ nc_cache_array, int64_t& lo,
                                       int64_t& deg, bool& cached) {
  int64_t at = -1;
  if (NC) at = nc_address_table[v];
  cached = at >= 0;
  if (cached) {
    deg = nc_cache_array[at];
    lo = at + 1;
  } else {
    lo = (int64_t)offsets[v];
    deg = (int64_t)offsets[v + 1] - lo;
  }
}

// What one lane of a G-lane group contributes to the picks of frontier node v, whose list has
// `deg` entries: c = number of picks of the node (min(deg, k)), and, for a lane with sub < c,
// `slot` = its place among the node's picks (ascending row position) and `pick` = the row
// position it takes.  Every lane of the wave calls it (the group shuffles and ballots inside
// need them all).
template <int G>
__device__ __forceinline__ void group_choose(uint32_t v, int64_t deg, int k, int hop, uint64_t seed,
                                             uint32_t batch, int& c, int& slot, int64_t& pick) {
  const int lane = lane_id();
  const int sub = threadIdx.x & (G - 1);
  c = deg < k ? (int)deg : k;
  pick = sub;
  slot = sub;
  if (__any(deg > k)) {
    // Floyd's subset rule, every lane of the wave takes part so that the group
    // shuffles and ballots stay convergent; groups with deg <= k discard the result.
    const int64_t d = deg > k ? deg : (int64_t)k + 1;
    const int64_t j = d - k + sub;
    const uint64_t r = philox_draw(seed, v, batch, (uint32_t)hop, (uint32_t)sub);
    const int64_t t = (int64_t)__umul64hi(r, (uint64_t)(j + 1));
    int64_t mine = t;
    const int group_shift = lane & ~(G - 1);
    const uint64_t group_mask = G == 64 ? ~0ull : ((1ull << (G & 63)) - 1);
    for (int i = 1; i < k; ++i) {
      const int64_t ti = __shfl(t, i, G);
      const uint64_t hit = (__ballot(sub < i && mine == ti) >> group_shift) & group_mask;
      if (sub == i && hit) mine = j;
    }
    int rank = 0;
    for (int m = 0; m < k; ++m) rank += __shfl(mine, m, G) < mine;
    if (deg > k) {
      pick = mine;
      slot = rank;
    }
  }
}

template <int G, typename OffT, bool NC>
__global__ __launch_bounds__(TB) void k_pick(Tables T, const OffT* __restrict__ offsets,
                                             const int32_t* __restrict__ indices,
                                             const int64_t* __restrict__ nc_address_table,
                                             const int32_t* __restrict__ nc_cache_array,
                                             const int32_t* __restrict__ nfront, int k, int hop,
                                             uint64_t seed, uint32_t first_batch, int S,
                                             int64_t tpb) {
  const Where here = where_am_i(S, tpb);
  if (here.b < 0) return;
  const int b = here.b;
  const int lane = lane_id();
  const int sub = threadIdx.x & (G - 1);
  const int64_t tiles_needed = ((int64_t)nfront[b] + TB / G - 1) / (TB / G);
  for (int64_t tile = here.tile; tile < tiles_needed; tile += tpb) {
    const int64_t idx = tile * (TB / G) + threadIdx.x / G;
    const bool active = idx < nfront[b];
    const uint32_t v = active ? (uint32_t)T.wlist[b * T.stride_ids + idx] : 0u;
    int64_t lo = 0, deg = 0, pick;
    bool cached = false;
    if (active) row_of<OffT, NC>(v, offsets, nc_address_table, nc_cache_array, lo, deg, cached);
    int c, slot;
    group_choose<G>(v, deg, k, hop, seed, first_batch + (uint32_t)b, c, slot, pick);
    bool holds = false;
    if (active && sub < c) {
      const uint32_t u = (uint32_t)(cached ? nc_cache_array : indices)[lo + pick];
      const uint32_t rank = (uint32_t)(idx * k + slot);
      T.cand[b * T.cand_slots + rank] = (int32_t)u;
      holds = place_candidate(T, b, k, u, rank);
    }
    // The group's first-occurrence mask, bit = pick slot.  The slots of a group's active lanes
    // are distinct (a permutation of 0..c-1), so every holder contributes the bit of its slot.
    uint64_t mask = 0;
    {
      const int group_shift = lane & ~(G - 1);
      const uint64_t group_mask = G == 64 ? ~0ull : ((1ull << (G & 63)) - 1);
      for (int m = 0; m < k; ++m)
        if ((__ballot(holds && slot == m) >> group_shift) & group_mask) mask |= 1ull << m;
    }
    if (active && sub == 0) {
      T.cnt[b * T.fr_slots + idx] = (uint8_t)c;
      T.first[b * T.fr_slots + idx] = mask;
    }
  }
}

// tile_sums[b][tile] = (picks << 32 | first occurrences) of 256 frontier slots; the final
// first-occurrence mask of a slot is what its lanes held minus what was displaced later
__global__ __launch_bounds__(TB) void k_count(Tables T, const int32_t* __restrict__ nfront,
                                              uint64_t* __restrict__ tile_sums, int64_t tiles,
                                              int S, int64_t tpb) {
  __shared__ uint64_t red[TB / WAVE];
  const Where here = where_am_i(S, tpb);
  if (here.b < 0) return;
  const int b = here.b;
  const int nf = nfront[b];
  for (int64_t tile = here.tile; tile * TB < nf; tile += tpb) {
    const int64_t idx = tile * TB + threadIdx.x;
    uint64_t first = 0;
    int c = 0;
    if (idx < nf) {
      c = T.cnt[b * T.fr_slots + idx];
      first = T.first[b * T.fr_slots + idx] & ~T.displaced[b * T.fr_slots + idx];
      T.first[b * T.fr_slots + idx] = first;
    }
    uint64_t packed = ((uint64_t)c << 32) | (uint64_t)__popcll(first);
    packed = wave_reduce_sum(packed);
    __syncthreads();   // red may still be read from the tile before
    if (lane_id() == 0) red[threadIdx.x / WAVE] = packed;
    __syncthreads();
    if (threadIdx.x == 0) {
      uint64_t s = 0;
      for (int w = 0; w < TB / WAVE; ++w) s += red[w];
      tile_sums[b * tiles + tile] = s;
    }
  }
}

// One block per batch: exclusive scan of the batch's tile sums, in place; totals out.
__global__ __launch_bounds__(TB) void k_scan_batch(uint64_t* __restrict__ tile_sums, int64_t tiles,
                                                   const int32_t* __restrict__ nfront,
                                                   uint64_t* __restrict__ batch_total) {
  __shared__ uint64_t smem[TB / WAVE + 1];
  const int b = blockIdx.x;
  const int64_t used = ((int64_t)nfront[b] + TB - 1) / TB;
  uint64_t carry = 0;
  for (int64_t base = 0; base < used; base += TB) {
    const int64_t i = base + threadIdx.x;
    const uint64_t v = i < used ? tile_sums[b * tiles + i] : 0;
    uint64_t total;
    const uint64_t ex = block_exclusive_scan<uint64_t, TB>(v, smem, total);
    if (i < used) tile_sums[b * tiles + i] = carry + ex;
    carry += total;
  }
  if (threadIdx.x == 0) batch_total[b] = carry;
}

struct Meta {            // device mirror of the small host outputs
  int64_t* ids_offsets;  // [S+1]
  int64_t* hop_sizes;    // [S*(H+1)]
  int64_t* row_off;      // [S*H+1]
  int64_t* col_off;      // [S*H+1]
  int64_t* totals;       // [0] ids, [1] rowptr entries, [2] col entries
};

// Single block: per-batch output bases of the stage, new list lengths, running totals.
// stage < 0 is the seed stage.
__global__ __launch_bounds__(TB) void k_stage_offsets(
    Meta M, int S, int H, int stage, const uint64_t* __restrict__ batch_total,
    const int32_t* __restrict__ nfront, const int32_t* __restrict__ nlist,
    int32_t* __restrict__ nlist_next, int64_t* __restrict__ row_base,
    int64_t* __restrict__ col_base) {
  __shared__ int64_t smem[TB / WAVE + 1];
  int64_t row_run = stage < 0 ? 0 : M.totals[1];
  int64_t col_run = stage < 0 ? 0 : M.totals[2];
  for (int base = 0; base < S; base += TB) {
    const int b = base + threadIdx.x;
    const bool ok = b < S;
    const uint64_t tot = ok ? batch_total[b] : 0;
    const int64_t rows = ok ? (int64_t)nfront[b] + 1 : 0;
    const int64_t cols = (int64_t)(tot >> 32);
    int64_t rt, ct;
    const int64_t rex = block_exclusive_scan<int64_t, TB>(rows, smem, rt);
    const int64_t cex = block_exclusive_scan<int64_t, TB>(cols, smem, ct);
    if (ok) {
      const int32_t grown = nlist[b] + (int32_t)(tot & 0xFFFFFFFFu);
      nlist_next[b] = grown;
      M.hop_sizes[(int64_t)b * (H + 1) + stage + 1] = grown;
      if (stage >= 0) {
        row_base[b] = row_run + rex;
        col_base[b] = col_run + cex;
        M.row_off[(int64_t)stage * S + b] = row_run + rex;
        M.col_off[(int64_t)stage * S + b] = col_run + cex;
      }
    }
    row_run += rt;
    col_run += ct;
  }
  if (threadIdx.x == 0) {
    if (stage < 0) {
      M.totals[1] = 0;
      M.totals[2] = 0;
    } else {
      M.totals[1] = row_run;
      M.totals[2] = col_run;
      if (stage == H - 1) {
        M.row_off[(int64_t)S * H] = row_run;
        M.col_off[(int64_t)S * H] = col_run;
      }
    }
  }
}

// Appends first occurrences to the lists, writes rowptr and the adj_col entries of the first
// occurrences.  Two phases per tile of TB frontier slots: one thread per slot scans the
// counts (picks and first occurrences in front of each slot) into LDS, then one thread per
// CANDIDATE does the writes, so that `cand`, the list and adj_col are accessed with
// consecutive lanes on consecutive addresses (a thread per slot walking its fanout picks
// touches a different cache line in every lane).
__global__ __launch_bounds__(TB) void k_emit(Tables T, const int32_t* __restrict__ nfront,
                                             const int32_t* __restrict__ nlist, int k,
                                             const uint64_t* __restrict__ tile_sums, int64_t tiles,
                                             int64_t* __restrict__ rowptr, int64_t rowptr_capacity,
                                             const int64_t* __restrict__ row_base,
                                             int32_t* __restrict__ col, int64_t col_capacity,
                                             const int64_t* __restrict__ col_base, int S,
                                             int64_t tpb) {
  __shared__ uint64_t smem[TB / WAVE + 1];
  __shared__ uint64_t s_first[TB];
  __shared__ uint32_t s_edges[TB], s_firsts[TB];
  __shared__ uint8_t s_cnt[TB];
  const Where here = where_am_i(S, tpb);
  if (here.b < 0) return;
  const int b = here.b;
  const int nf = nfront[b];
  const uint32_t list_len = (uint32_t)nlist[b];
  // tile 0 always runs: an empty frontier still has a rowptr entry
  for (int64_t tile = here.tile; tile * TB < nf || tile == 0; tile += tpb) {
    const int64_t idx = tile * TB + threadIdx.x;
    const bool active = idx < nf;
    const uint64_t first = active ? T.first[b * T.fr_slots + idx] : 0;
    const int c = active ? T.cnt[b * T.fr_slots + idx] : 0;
    const uint64_t packed = ((uint64_t)c << 32) | (uint64_t)__popcll(first);
    uint64_t total;
    const uint64_t ex = block_exclusive_scan<uint64_t, TB>(packed, smem, total) +
                        (nf > 0 ? tile_sums[b * tiles + tile] : 0);
    const int64_t edges_before = (int64_t)(ex >> 32);
    if (rowptr) {
      const int64_t rb = row_base[b];
      if (active && rb + idx < rowptr_capacity) rowptr[rb + idx] = edges_before;
      if ((active && idx == nf - 1) || (nf == 0 && idx == 0)) {
        const int64_t last = nf == 0 ? 0 : idx + 1;
        if (rb + last < rowptr_capacity) rowptr[rb + last] = edges_before + c;
      }
    }
    s_first[threadIdx.x] = first;
    s_cnt[threadIdx.x] = (uint8_t)c;
    s_edges[threadIdx.x] = (uint32_t)edges_before;
    s_firsts[threadIdx.x] = (uint32_t)(ex & 0xFFFFFFFFu);
    __syncthreads();
    if ((uint32_t)(total & 0xFFFFFFFFu)) {      // the tile has first occurrences (uniform)
      // A first occurrence's slot in `cand` is overwritten with its list position: the table
      // keeps PEND + its rank, so later duplicates find the position through the rank without
      // a scattered write into the table here (the next stage rebuilds the tables anyway).
      const int64_t slots_here = nf - tile * TB < TB ? nf - tile * TB : TB;
      const uint32_t ncand = (uint32_t)(slots_here * k);
      int32_t* cand = T.cand + b * T.cand_slots + tile * TB * k;
      int32_t* list = T.wlist + b * T.stride_ids;
      const int64_t cb = col ? col_base[b] : 0;
      for (uint32_t r = threadIdx.x; r < ncand; r += TB) {
        const uint32_t sl = r / (uint32_t)k, pick = r - sl * (uint32_t)k;
        const uint64_t f = s_first[sl];
        if (pick < s_cnt[sl] && (f >> pick & 1)) {
          const uint32_t pos = list_len + s_firsts[sl] + (uint32_t)__popcll(f & ((1ull << pick) - 1));
          list[pos] = cand[r];
          cand[r] = (int32_t)pos;
          const int64_t d = cb + s_edges[sl] + pick;
          if (col && d < col_capacity) col[d] = (int32_t)pos;
        }
      }
    }
    __syncthreads();   // the LDS arrays are rewritten for the next tile
  }
}

// adj_col of the picks that are not first occurrences, one thread per candidate (see k_emit).
// An id of an earlier stage carries its list position in its reference; an id that is new in
// this stage is looked up through its slot, whose final value is PEND + the rank of the id's
// first occurrence, whose entry in `cand` now holds the position.
__global__ __launch_bounds__(TB) void k_col(Tables T, const int32_t* __restrict__ nfront, int k,
                                            const int64_t* __restrict__ rowptr,
                                            int64_t rowptr_capacity,
                                            const int64_t* __restrict__ row_base,
                                            int32_t* __restrict__ col, int64_t col_capacity,
                                            const int64_t* __restrict__ col_base, int S,
                                            int64_t tpb) {
  __shared__ uint64_t s_first[TB];
  __shared__ int64_t s_dst[TB];
  __shared__ uint8_t s_cnt[TB];
  __shared__ uint32_t s_any;
  const Where here = where_am_i(S, tpb);
  if (here.b < 0) return;
  const int b = here.b;
  const int nf = nfront[b];
  const uint64_t* t = T.tab + T.tab_off[b];
  const int32_t* cand_b = T.cand + b * T.cand_slots;
  for (int64_t tile = here.tile; tile * TB < nf; tile += tpb) {
    const int64_t idx = tile * TB + threadIdx.x;
    if (threadIdx.x == 0) s_any = 0;
    __syncthreads();
    uint64_t first = 0;
    int c = 0;
    int64_t dst = 0;
    if (idx < nf && row_base[b] + idx < rowptr_capacity) {
      c = T.cnt[b * T.fr_slots + idx];
      first = T.first[b * T.fr_slots + idx];
      dst = col_base[b] + rowptr[row_base[b] + idx];
    }
    s_first[threadIdx.x] = first;
    s_cnt[threadIdx.x] = (uint8_t)c;
    s_dst[threadIdx.x] = dst;
    if (__popcll(first) != c) s_any = 1;
    __syncthreads();
    if (s_any) {                                  // uniform over the block
      const int64_t slots_here = nf - tile * TB < TB ? nf - tile * TB : TB;
      const uint32_t ncand = (uint32_t)(slots_here * k);
      const uint32_t* ref = T.ref + b * T.cand_slots + tile * TB * k;
      for (uint32_t r = threadIdx.x; r < ncand; r += TB) {
        const uint32_t sl = r / (uint32_t)k, pick = r - sl * (uint32_t)k;
        if (pick < s_cnt[sl] && !(s_first[sl] >> pick & 1)) {
          const int64_t d = s_dst[sl] + pick;
          if (d < col_capacity) {
            const uint32_t where = ref[r];
            col[d] = where & OLD_ID ? (int32_t)(where & ~OLD_ID)
                                    : cand_b[(uint32_t)t[where] - PEND];
          }
        }
      }
    }
    __syncthreads();
  }
}

__global__ __launch_bounds__(TB) void k_ids_offsets(Meta M, int S, const int32_t* __restrict__ nlist) {
  __shared__ int64_t smem[TB / WAVE + 1];
  int64_t run = 0;
  for (int base = 0; base < S; base += TB) {
    const int b = base + threadIdx.x;
    const int64_t n = b < S ? nlist[b] : 0;
    int64_t total;
    const int64_t ex = block_exclusive_scan<int64_t, TB>(n, smem, total);
    if (b < S) M.ids_offsets[b] = run + ex;
    run += total;
  }
  if (threadIdx.x == 0) {
    M.ids_offsets[S] = run;
    M.totals[0] = run;
  }
}

__global__ __launch_bounds__(TB) void k_copy_ids(Tables T, Meta M, const int32_t* __restrict__ nlist,
                                                 int32_t* __restrict__ ids, int64_t ids_capacity) {
  const int b = blockIdx.y;
  const int64_t n = nlist[b];
  const int64_t dst = M.ids_offsets[b];
  for (int64_t j = (int64_t)blockIdx.x * TB + threadIdx.x; j < n; j += (int64_t)gridDim.x * TB)
    if (dst + j < ids_capacity) ids[dst + j] = T.wlist[b * T.stride_ids + j];
}

// Precondition check (only when asked for): every seed inside [0, num_nodes).
__global__ __launch_bounds__(TB) void k_validate_seeds(const int32_t* __restrict__ seeds, int64_t n,
                                                       int64_t num_nodes,
                                                       unsigned long long* __restrict__ bad) {
  const int64_t j = (int64_t)blockIdx.x * TB + threadIdx.x;
  if (j < n && (uint32_t)seeds[j] >= (uint64_t)num_nodes) atomicAdd(bad, 1ull);
}

// Precondition check (only when asked for): offsets start at 0, never decrease and end at
// num_edges; every entry of indices inside [0, num_nodes).
template <typename OffT>
__global__ __launch_bounds__(TB) void k_validate_csr(const OffT* __restrict__ offsets,
                                                     const int32_t* __restrict__ indices,
                                                     int64_t num_nodes, int64_t num_edges,
                                                     unsigned long long* __restrict__ bad) {
  const int64_t span = (int64_t)gridDim.x * TB;
  unsigned long long mine = 0;
  for (int64_t j = (int64_t)blockIdx.x * TB + threadIdx.x; j < num_nodes || j < num_edges;
       j += span) {
    if (j < num_nodes) {
      mine += (int64_t)offsets[j] > (int64_t)offsets[j + 1];
      if (j == 0) mine += offsets[0] != 0 || (int64_t)offsets[num_nodes] != num_edges;
    }
    if (j < num_edges) mine += (uint32_t)indices[j] >= (uint64_t)num_nodes;
  }
  if (mine) atomicAdd(bad, mine);
}

__global__ void k_seed_counts(const int64_t* __restrict__ seed_off, int S, int32_t* nfront,
                              int32_t* nlist) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b < S) {
    nfront[b] = (int32_t)(seed_off[b + 1] - seed_off[b]);
    nlist[b] = 0;
  }
}

struct Plan {
  int64_t stride_front[GINEX_MAX_HOPS];  // bound on the frontier at hop h, per batch
  int64_t stride_ids;                    // bound on the final list, per batch
  int64_t cand_slots, fr_slots, tiles;
  int64_t table_slots;                   // per batch, worst case (2 per list entry)
  bool ok;
};

Plan make_plan(int64_t num_nodes, int64_t max_batch, const int32_t* fanout, int32_t H) {
  Plan p{};
  p.ok = true;
  // the seed stage has one slot per given seed (repeats included); after it a list never
  // holds more than num_nodes entries
  p.cand_slots = p.fr_slots = max_batch > 1 ? max_batch : 1;
  int64_t front = max_batch < num_nodes ? max_batch : num_nodes;
  if (front < 1) front = 1;
  for (int h = 0; h < H; ++h) {
    p.stride_front[h] = front;
    if (front * fanout[h] > p.cand_slots) p.cand_slots = front * fanout[h];
    if (front > p.fr_slots) p.fr_slots = front;
    int64_t next = front * (1 + (int64_t)fanout[h]);
    front = next < num_nodes ? next : num_nodes;
  }
  p.stride_ids = front;
  if (p.cand_slots >= (int64_t)PEND || p.stride_ids >= (int64_t)PEND) p.ok = false;
  p.tiles = ceil_div(p.fr_slots, TB);
  // a stage's table holds at most min(num_nodes, list + frontier * fanout) <= stride_ids ids
  p.table_slots = 2 * p.stride_ids + 32;
  return p;
}

struct Workspace {
  uint64_t* tab;
  int32_t* wlist;
  int32_t* cand;
  uint32_t* ref;
  uint8_t* cnt;
  uint64_t* tile_sums;
  uint64_t* batch_total;
  uint64_t* first;
  uint64_t* displaced;
  int64_t* tab_off;
  uint32_t* tab_slots;
  int64_t* tab_total;
  int32_t *nfront, *nlist_a, *nlist_b;
  int64_t *row_base, *col_base, *seed_off;
  int64_t* meta;
  size_t bytes;
};

int64_t meta_elems(int32_t S, int32_t H) {
  return (int64_t)(S + 1) + (int64_t)S * (H + 1) + 2 * ((int64_t)S * H + 1) + 4;
}

Workspace carve(void* base, const Plan& p, int32_t S, int32_t H) {
  Arena a(base);
  Workspace w;
  w.tab = a.take<uint64_t>((size_t)S * p.table_slots);
  w.wlist = a.take<int32_t>((size_t)S * p.stride_ids);
  w.cand = a.take<int32_t>((size_t)S * p.cand_slots);
  w.ref = a.take<uint32_t>((size_t)S * p.cand_slots);
  w.cnt = a.take<uint8_t>((size_t)S * p.fr_slots);
  w.tile_sums = a.take<uint64_t>((size_t)S * p.tiles);
  w.batch_total = a.take<uint64_t>(S);
  w.first = a.take<uint64_t>((size_t)S * p.fr_slots);
  w.displaced = a.take<uint64_t>((size_t)S * p.fr_slots);
  w.tab_off = a.take<int64_t>(S);
  w.tab_slots = a.take<uint32_t>(S);
  w.tab_total = a.take<int64_t>(1);
  w.nfront = a.take<int32_t>(S);
  w.nlist_a = a.take<int32_t>(S);
  w.nlist_b = a.take<int32_t>(S);
  w.row_base = a.take<int64_t>(S);
  w.col_base = a.take<int64_t>(S);
  w.seed_off = a.take<int64_t>(S + 1);
  w.meta = a.take<int64_t>(meta_elems(S, H));
  w.bytes = (a.used + 255) & ~size_t(255);
  return w;
}

int32_t check_shape(int64_t num_nodes, int32_t S, int64_t max_batch, const int32_t* fanout,
                    int32_t H, const char* who) {
  if (num_nodes <= 0 || num_nodes > INT32_MAX)
    return fail(GINEX_ERR_ARG, "%s: num_nodes=%lld out of range", who, (long long)num_nodes);
  if (S < 1 || S > 65535) return fail(GINEX_ERR_ARG, "%s: S=%d outside [1, 65535]", who, S);
  if (max_batch < 0) return fail(GINEX_ERR_ARG, "%s: negative batch size", who);
  if (H < 1 || H > GINEX_MAX_HOPS || !fanout)
    return fail(GINEX_ERR_ARG, "%s: H=%d outside [1, %d] or fanout null", who, H, GINEX_MAX_HOPS);
  for (int h = 0; h < H; ++h)
    if (fanout[h] < 1 || fanout[h] > GINEX_MAX_FANOUT)
      return fail(GINEX_ERR_ARG, "%s: fanout[%d]=%d outside [1, %d]", who, h, fanout[h],
                  GINEX_MAX_FANOUT);
  return GINEX_OK;
}

inline int64_t pick_tiles(int64_t front, int group) {
  return capped(ceil_div(front, TB / group), tile_cap(PICK_TILES));
}

// ---- seeds and hop 0 in LDS ------------------------------------------------------------------
//
// A batch's seeds and the candidates of its first hop are few enough (at most LDS_MAX_IDS)
// for their hash set to live in LDS: one workgroup per batch clears a table of LDS_SLOTS
// 64-bit slots in its own LDS, deduplicates the seeds, draws the picks of hop 0, inserts them
// (same slot word and the same rule as the tables in HBM: the smallest candidate rank per id
// wins), appends the first occurrences to the batch's list and resolves every pick's list
// position, all without a table access outside the CU.  What crosses batches (where a
// batch's adj segment starts) is left to k_stage_offsets; the picks' positions and the rows'
// edge counts wait in the batch's scratch arrays until k_adj_copy moves them there.
// The later hops do not fit (a batch's set reaches 10^5 ids) and keep the tables in HBM.
constexpr int LDS_SLOTS = 16384;       // 128 KB
constexpr int LDS_BLOCK = 1024;        // threads, and the most seeds a batch may have here
constexpr int LDS_MAX_IDS = 12288;     // seeds + candidates of hop 0: load factor 0.75 at most

__device__ __forceinline__ uint32_t lds_place(unsigned long long* tab, uint32_t id, uint32_t value,
                                              uint32_t& old_value) {
  // Inserts (id, value) unless the id is there; returns the slot; old_value = what the slot
  // held for this id before (all ones if the id was new).  A present id keeps the smaller value.
  const unsigned long long mine = ((unsigned long long)id << 32) | value;
  uint32_t h = hash_slot(id, LDS_SLOTS);
  while (true) {
    const unsigned long long old = atomicCAS(&tab[h], FREE_SLOT, mine);
    if (old == FREE_SLOT) {
      old_value = 0xFFFFFFFFu;
      return h;
    }
    if ((uint32_t)(old >> 32) == id) {
      old_value = (uint32_t)old;
      if (old_value >= PEND && old_value > value) atomicMin(&tab[h], mine);
      return h;
    }
    h = h + 1 == LDS_SLOTS ? 0 : h + 1;
  }
}

template <int G, typename OffT, bool NC>
__global__ __launch_bounds__(LDS_BLOCK) void k_front_lds(
    Tables T, const OffT* __restrict__ offsets, const int32_t* __restrict__ indices,
    const int64_t* __restrict__ nc_address_table, const int32_t* __restrict__ nc_cache_array,
    const int32_t* __restrict__ seeds, const int64_t* __restrict__ seed_off, int k, uint64_t seed,
    uint32_t first_batch, int H, Meta M, int32_t* __restrict__ nlist_seeds,
    uint64_t* __restrict__ batch_total) {
  __shared__ unsigned long long tab[LDS_SLOTS];
  __shared__ uint64_t s_first[LDS_BLOCK];
  __shared__ uint32_t s_edges[LDS_BLOCK], s_firsts[LDS_BLOCK];
  __shared__ uint8_t s_cnt[LDS_BLOCK];
  __shared__ int64_t s_lo[LDS_BLOCK];     // start of a frontier node's neighbour list; ~start if it is a cached one
  __shared__ int32_t s_deg[LDS_BLOCK];
  __shared__ uint64_t smem[LDS_BLOCK / WAVE + 1];
  const int b = blockIdx.x;
  const int tid = threadIdx.x;
  const int ns = (int)(seed_off[b + 1] - seed_off[b]);
  int32_t* list = T.wlist + (int64_t)b * T.stride_ids;
  int32_t* cand = T.cand + (int64_t)b * T.cand_slots;
  uint32_t* ref = T.ref + (int64_t)b * T.cand_slots;
  for (int i = tid; i < LDS_SLOTS; i += LDS_BLOCK) tab[i] = FREE_SLOT;
  if (b == 0 && tid == 0) {
    M.totals[1] = 0;
    M.totals[2] = 0;
  }
  __syncthreads();
  // the seeds: a seed repeated inside the batch is kept once, at its first position
  uint32_t id = 0, slot_of_mine = 0, before;
  if (tid < ns) {
    id = (uint32_t)seeds[seed_off[b] + tid];
    slot_of_mine = lds_place(tab, id, PEND + (uint32_t)tid, before);
  }
  __syncthreads();
  const bool kept = tid < ns && (uint32_t)tab[slot_of_mine] == PEND + (uint32_t)tid;
  uint64_t total64;
  const uint32_t at = (uint32_t)block_exclusive_scan<uint64_t, LDS_BLOCK>(kept ? 1ull : 0ull, smem, total64);
  const int n0 = (int)total64;
  if (kept) {
    list[at] = (int32_t)id;
    tab[slot_of_mine] = ((unsigned long long)id << 32) | at;   // from now on: an id of the list, with its position
  }
  if (tid == 0) {
    M.hop_sizes[(int64_t)b * (H + 1)] = n0;
    nlist_seeds[b] = n0;
  }
  __syncthreads();
  // hop 0: the frontier is the list.  First every node's neighbour list is located, one
  // thread per node, so that the rounds below wait for memory once and not once each.
  if (tid < n0) {
    int64_t lo, deg;
    bool cached;
    row_of<OffT, NC>((uint32_t)list[tid], offsets, nc_address_table, nc_cache_array, lo, deg,
                     cached);
    s_lo[tid] = cached ? ~lo : lo;
    s_deg[tid] = (int32_t)(deg < 0x7FFFFFFF ? deg : 0x7FFFFFFF);
  }
  __syncthreads();
  // One G-lane group per node and round; the reads of the picked neighbours of ROUNDS rounds
  // are issued before any is inserted, so that they are in flight together.
  constexpr int ROUNDS = 8;
  const int sub = tid & (G - 1);
  const int per_round = LDS_BLOCK / G;
  for (int base = 0; base < n0; base += per_round * ROUNDS) {
    uint32_t u[ROUNDS], rank[ROUNDS];
#pragma unroll
    for (int q = 0; q < ROUNDS; ++q) {
      const int idx = base + q * per_round + tid / G;
      const bool active = idx < n0;
      const uint32_t v = active ? (uint32_t)list[idx] : 0u;
      int64_t deg = active ? (int64_t)s_deg[idx] : 0;
      if (deg == 0x7FFFFFFF) {   // saturated in LDS (a list of 2^31 entries or more): look again
        int64_t lo;
        bool cached;
        row_of<OffT, NC>(v, offsets, nc_address_table, nc_cache_array, lo, deg, cached);
      }
      int c, slot;
      int64_t pick;
      group_choose<G>(v, deg, k, 0, seed, first_batch + (uint32_t)b, c, slot, pick);
      rank[q] = 0xFFFFFFFFu;
      u[q] = 0;
      if (active && sub < c) {
        const int64_t lo = s_lo[idx];
        u[q] = (uint32_t)(lo < 0 ? nc_cache_array[~lo + pick] : indices[lo + pick]);
        rank[q] = (uint32_t)(idx * k + slot);
      }
      if (active && sub == 0) s_cnt[idx] = (uint8_t)c;
    }
#pragma unroll
    for (int q = 0; q < ROUNDS; ++q)
      if (rank[q] != 0xFFFFFFFFu) {
        cand[rank[q]] = (int32_t)u[q];
        const uint32_t h = lds_place(tab, u[q], PEND + rank[q], before);
        ref[rank[q]] = before < PEND ? OLD_ID | before : h;
      }
  }
  __syncthreads();
  // per node: which of its picks are first occurrences (they hold their id's slot), and the
  // picks / first occurrences in front of the node
  uint64_t first = 0;
  int c = 0;
  if (tid < n0) {
    c = s_cnt[tid];
    for (int s = 0; s < c; ++s) {
      const uint32_t rank = (uint32_t)(tid * k + s);
      const uint32_t r = ref[rank];
      if (!(r & OLD_ID) && (uint32_t)tab[r] == PEND + rank) first |= 1ull << s;
    }
  }
  const uint64_t ex = block_exclusive_scan<uint64_t, LDS_BLOCK>(((uint64_t)c << 32) | (uint64_t)__popcll(first),
                                                                smem, total64);
  s_first[tid] = first;
  s_edges[tid] = (uint32_t)(ex >> 32);
  s_firsts[tid] = (uint32_t)(ex & 0xFFFFFFFFu);
  __syncthreads();
  // one thread per candidate: first occurrences go to the list, their slot gets the position
  const uint32_t ncand = (uint32_t)n0 * (uint32_t)k;
  for (uint32_t r = tid; r < ncand; r += LDS_BLOCK) {
    const uint32_t node = r / (uint32_t)k, pick = r - node * (uint32_t)k;
    const uint64_t f = s_first[node];
    if (pick < s_cnt[node] && (f >> pick & 1)) {
      const uint32_t pos = (uint32_t)n0 + s_firsts[node] + (uint32_t)__popcll(f & ((1ull << pick) - 1));
      const uint32_t u = (uint32_t)cand[r];
      list[pos] = (int32_t)u;
      tab[ref[r]] = ((unsigned long long)u << 32) | pos;
    }
  }
  __syncthreads();
  // every pick's position in the list (adj_col), parked in `cand` (same thread per entry as above)
  for (uint32_t r = tid; r < ncand; r += LDS_BLOCK) {
    const uint32_t node = r / (uint32_t)k, pick = r - node * (uint32_t)k;
    if (pick < s_cnt[node]) {
      const uint32_t where = ref[r];
      cand[r] = (int32_t)(where & OLD_ID ? where & ~OLD_ID : (uint32_t)tab[where]);
    }
  }
  __syncthreads();   // `ref` is free now: it parks the rows' edge offsets
  if (tid < n0) {
    ref[tid] = s_edges[tid];
    T.cnt[(int64_t)b * T.fr_slots + tid] = s_cnt[tid];
  }
  if (tid == 0) batch_total[b] = total64;
}

// adj of hop 0 from the scratch arrays k_front_lds left: rowptr of every frontier node, and
// the list position of every pick at its place in the batch's segment.
__global__ __launch_bounds__(TB) void k_adj_copy(Tables T, const int32_t* __restrict__ nfront, int k,
                                                 const uint64_t* __restrict__ batch_total,
                                                 int64_t* __restrict__ rowptr, int64_t rowptr_capacity,
                                                 const int64_t* __restrict__ row_base,
                                                 int32_t* __restrict__ col, int64_t col_capacity,
                                                 const int64_t* __restrict__ col_base) {
  const int b = blockIdx.y;
  const int n0 = nfront[b];
  const int32_t* cand = T.cand + (int64_t)b * T.cand_slots;
  const uint32_t* edges = T.ref + (int64_t)b * T.cand_slots;
  const int64_t rb = row_base[b], cb = col_base[b];
  const int64_t span = (int64_t)gridDim.x * TB;
  for (int64_t r = (int64_t)blockIdx.x * TB + threadIdx.x; r <= n0; r += span)
    if (rb + r < rowptr_capacity)
      rowptr[rb + r] = r < n0 ? (int64_t)edges[r] : (int64_t)(batch_total[b] >> 32);
  const int64_t ncand = (int64_t)n0 * k;
  for (int64_t r = (int64_t)blockIdx.x * TB + threadIdx.x; r < ncand; r += span) {
    const int64_t node = r / k, pick = r - node * k;
    if (pick < T.cnt[(int64_t)b * T.fr_slots + node]) {
      const int64_t d = cb + edges[node] + pick;
      if (d < col_capacity) col[d] = cand[r];
    }
  }
}

template <typename OffT, bool NC>
void launch_pick(const Tables& T, const Plan& p, const ginex_csr_t* g, const int32_t* nfront, int k,
                 int hop, int32_t S, uint64_t seed, uint32_t first_batch, hipStream_t st) {
  const OffT* off = static_cast<const OffT*>(g->offsets);
  const int64_t front = p.stride_front[hop];
  if (k <= 16) {
    const int64_t tpb = pick_tiles(front, 16);
    hipLaunchKernelGGL((k_pick<16, OffT, NC>), dim3(grid_blocks(S, tpb)), dim3(TB), 0, st, T, off,
                       g->indices, g->nc_address_table, g->nc_cache_array, nfront, k, hop, seed,
                       first_batch, S, tpb);
  } else if (k <= 32) {
    const int64_t tpb = pick_tiles(front, 32);
    hipLaunchKernelGGL((k_pick<32, OffT, NC>), dim3(grid_blocks(S, tpb)), dim3(TB), 0, st, T, off,
                       g->indices, g->nc_address_table, g->nc_cache_array, nfront, k, hop, seed,
                       first_batch, S, tpb);
  } else {
    const int64_t tpb = pick_tiles(front, 64);
    hipLaunchKernelGGL((k_pick<64, OffT, NC>), dim3(grid_blocks(S, tpb)), dim3(TB), 0, st, T, off,
                       g->indices, g->nc_address_table, g->nc_cache_array, nfront, k, hop, seed,
                       first_batch, S, tpb);
  }
}

template <typename OffT, bool NC>
void launch_front(const Tables& T, const ginex_csr_t* g, const int32_t* seeds,
                  const int64_t* seed_off, int k, int32_t S, int32_t H, uint64_t seed,
                  uint32_t first_batch, const Meta& M, int32_t* nlist_seeds, uint64_t* batch_total,
                  hipStream_t st) {
  const OffT* off = static_cast<const OffT*>(g->offsets);
#define GINEX_FRONT(G)                                                                          \
  hipLaunchKernelGGL((k_front_lds<G, OffT, NC>), dim3((unsigned)S), dim3(LDS_BLOCK), 0, st, T, off, \
                     g->indices, g->nc_address_table, g->nc_cache_array, seeds, seed_off, k, seed, \
                     first_batch, H, M, nlist_seeds, batch_total)
  if (k <= 16) GINEX_FRONT(16);
  else if (k <= 32) GINEX_FRONT(32);
  else GINEX_FRONT(64);
#undef GINEX_FRONT
}

}  // namespace
}  // namespace ginex

using namespace ginex;

extern "C" size_t ginex_sample_workspace_bytes(int64_t num_nodes, int32_t S, int64_t max_batch,
                                               const int32_t* fanout, int32_t H) {
  if (check_shape(num_nodes, S, max_batch, fanout, H, "ginex_sample_workspace_bytes")) return 0;
  const Plan p = make_plan(num_nodes, max_batch, fanout, H);
  if (!p.ok) {
    set_error("ginex_sample_workspace_bytes: a batch could exceed 2^30 list entries");
    return 0;
  }
  return carve(nullptr, p, S, H).bytes;
}

extern "C" int32_t ginex_sample_superbatch(
    const ginex_csr_t* g, const int32_t* seeds, const int64_t* seed_offsets, int32_t S,
    const int32_t* fanout, int32_t H, uint64_t rng_seed, uint32_t first_batch_index,
    int32_t* ids, int64_t ids_capacity, int64_t* ids_offsets, int64_t* hop_sizes,
    int64_t* adj_rowptr, int64_t rowptr_capacity, int32_t* adj_col, int64_t col_capacity,
    int64_t* adj_row_offsets, int64_t* adj_col_offsets, int64_t* totals, void* ws,
    size_t ws_bytes, void* stream) {
  const char* who = "ginex_sample_superbatch";
  if (!g || !g->offsets || (g->num_edges > 0 && !g->indices))
    return fail(GINEX_ERR_ARG, "%s: graph descriptor or its arrays are null", who);
  if ((g->nc_address_table == nullptr) != (g->nc_cache_array == nullptr))
    return fail(GINEX_ERR_ARG, "%s: neighbour cache needs both its address table and its array",
                who);
  if (!seed_offsets || !ids_offsets || !hop_sizes || !adj_row_offsets || !adj_col_offsets ||
      !totals || !ws)
    return fail(GINEX_ERR_ARG, "%s: a required pointer is null", who);
  if ((adj_rowptr == nullptr) != (adj_col == nullptr))
    return fail(GINEX_ERR_ARG, "%s: adj_rowptr and adj_col must both be given or both be null", who);
  if (ids_capacity < 0 || rowptr_capacity < 0 || col_capacity < 0 || (ids_capacity > 0 && !ids))
    return fail(GINEX_ERR_ARG, "%s: bad output capacity", who);
  int64_t max_batch = 0;
  if (S >= 1) {
    if (seed_offsets[0] != 0) return fail(GINEX_ERR_INPUT, "%s: seed_offsets[0] must be 0", who);
    for (int b = 0; b < S; ++b) {
      const int64_t n = seed_offsets[b + 1] - seed_offsets[b];
      if (n < 0) return fail(GINEX_ERR_INPUT, "%s: seed_offsets not monotone at %d", who, b);
      if (n > max_batch) max_batch = n;
    }
  }
  if (int32_t rc = check_shape(g->num_nodes, S, max_batch, fanout, H, who)) return rc;
  if (seed_offsets[S] > 0 && !seeds) return fail(GINEX_ERR_ARG, "%s: seeds is null", who);
  const Plan p = make_plan(g->num_nodes, max_batch, fanout, H);
  if (!p.ok) return fail(GINEX_ERR_ARG, "%s: a batch could exceed 2^30 list entries", who);
  const Workspace w = carve(ws, p, S, H);
  if (ws_bytes < w.bytes)
    return fail(GINEX_ERR_WORKSPACE, "%s: workspace of %zu bytes given, %zu needed", who, ws_bytes,
                w.bytes);
  if ((uintptr_t)ws & 255) return fail(GINEX_ERR_ARG, "%s: workspace must be 256-byte aligned", who);

  hipStream_t st = (hipStream_t)stream;
  Tables T;
  T.tab = w.tab; T.tab_off = w.tab_off; T.tab_slots = w.tab_slots; T.first = w.first;
  T.displaced = w.displaced; T.cand = w.cand; T.ref = w.ref; T.cnt = w.cnt;
  T.cand_slots = p.cand_slots; T.fr_slots = p.fr_slots; T.wlist = w.wlist;
  T.stride_ids = p.stride_ids;
  Meta M;
  M.ids_offsets = w.meta;
  M.hop_sizes = M.ids_offsets + (S + 1);
  M.row_off = M.hop_sizes + (int64_t)S * (H + 1);
  M.col_off = M.row_off + ((int64_t)S * H + 1);
  M.totals = M.col_off + ((int64_t)S * H + 1);

  GINEX_HIP(hipMemcpyAsync(w.seed_off, seed_offsets, sizeof(int64_t) * (S + 1),
                           hipMemcpyHostToDevice, st));
  const char* validate_env = getenv("GINEX_VALIDATE");
  if (validate_env && validate_env[0] == '1' && seed_offsets[S] > 0) {
    // the first slot of the (not yet used) batch_total array serves as the counter
    unsigned long long bad = 0;
    unsigned long long* d_bad = reinterpret_cast<unsigned long long*>(w.batch_total);
    GINEX_HIP(fill_async<unsigned long long>(d_bad, 1, 0ull, st));
    hipLaunchKernelGGL(k_validate_seeds, dim3((unsigned)ceil_div(seed_offsets[S], TB)), dim3(TB), 0,
                       st, seeds, seed_offsets[S], g->num_nodes, d_bad);
    GINEX_LAUNCH_CHECK();
    GINEX_HIP(hipMemcpyAsync(&bad, d_bad, sizeof(bad), hipMemcpyDeviceToHost, st));
    GINEX_HIP(hipStreamSynchronize(st));
    if (bad)
      return fail(GINEX_ERR_INPUT, "%s: %llu seeds outside [0, %lld)", who, bad,
                  (long long)g->num_nodes);
    GINEX_HIP(fill_async<unsigned long long>(d_bad, 1, 0ull, st));
    if (g->offsets_64)
      hipLaunchKernelGGL(k_validate_csr<int64_t>, dim3(4096), dim3(TB), 0, st,
                         (const int64_t*)g->offsets, g->indices, g->num_nodes, g->num_edges, d_bad);
    else
      hipLaunchKernelGGL(k_validate_csr<int32_t>, dim3(4096), dim3(TB), 0, st,
                         (const int32_t*)g->offsets, g->indices, g->num_nodes, g->num_edges, d_bad);
    GINEX_LAUNCH_CHECK();
    GINEX_HIP(hipMemcpyAsync(&bad, d_bad, sizeof(bad), hipMemcpyDeviceToHost, st));
    GINEX_HIP(hipStreamSynchronize(st));
    if (bad)
      return fail(GINEX_ERR_INPUT, "%s: the CSR breaks %llu of its invariants (offsets from 0 to "
                  "num_edges without a decrease, indices inside [0, %lld))", who, bad,
                  (long long)g->num_nodes);
  }
  int32_t* nlist = w.nlist_a;
  int32_t* nlist_next = w.nlist_b;
  int first_stage = -1;
  // Seeds and hop 0 of a batch in the LDS of one workgroup, when their hash set fits there
  // (GINEX_SAMPLER_LDS=0 keeps them on the tables in HBM; same result).
  const char* lds_env = getenv("GINEX_SAMPLER_LDS");
  const bool front_lds = max_batch <= LDS_BLOCK &&
                         max_batch * (1 + (int64_t)fanout[0]) <= LDS_MAX_IDS &&
                         !(lds_env && lds_env[0] == '0');
  if (front_lds) {
    const int k0 = fanout[0];
    if (g->nc_address_table) {
      if (g->offsets_64)
        launch_front<int64_t, true>(T, g, seeds, w.seed_off, k0, S, H, rng_seed, first_batch_index, M,
                                    w.nlist_b, w.batch_total, st);
      else
        launch_front<int32_t, true>(T, g, seeds, w.seed_off, k0, S, H, rng_seed, first_batch_index, M,
                                    w.nlist_b, w.batch_total, st);
    } else if (g->offsets_64) {
      launch_front<int64_t, false>(T, g, seeds, w.seed_off, k0, S, H, rng_seed, first_batch_index, M,
                                   w.nlist_b, w.batch_total, st);
    } else {
      launch_front<int32_t, false>(T, g, seeds, w.seed_off, k0, S, H, rng_seed, first_batch_index, M,
                                   w.nlist_b, w.batch_total, st);
    }
    GINEX_LAUNCH_CHECK();
    // the list after the seeds (nlist_b) is the frontier of hop 0; nlist_a receives the list after hop 0
    hipLaunchKernelGGL(k_stage_offsets, dim3(1), dim3(TB), 0, st, M, S, H, 0, w.batch_total,
                       w.nlist_b, w.nlist_b, w.nlist_a, w.row_base, w.col_base);
    GINEX_LAUNCH_CHECK();
    if (adj_rowptr) {
      const int64_t per_batch = ceil_div(max_batch * (int64_t)k0 + 1, TB);
      hipLaunchKernelGGL(k_adj_copy, dim3((unsigned)(per_batch < 16 ? per_batch : 16), (unsigned)S),
                         dim3(TB), 0, st, T, w.nlist_b, k0, w.batch_total, adj_rowptr,
                         rowptr_capacity, w.row_base, adj_col, col_capacity, w.col_base);
      GINEX_LAUNCH_CHECK();
    }
    first_stage = 1;
  } else {
    hipLaunchKernelGGL(k_seed_counts, dim3((unsigned)ceil_div(S, TB)), dim3(TB), 0, st, w.seed_off,
                       S, w.nfront, w.nlist_a);
    GINEX_LAUNCH_CHECK();
  }
  for (int stage = first_stage; stage < H; ++stage) {
    const int k = stage < 0 ? 1 : fanout[stage];
    const int64_t front = stage < 0 ? (max_batch > 0 ? max_batch : 1) : p.stride_front[stage];
    // in a hop the frontier is the whole list as it stands when the hop starts
    const int32_t* nfront = stage < 0 ? w.nfront : nlist;
    const int64_t tpb = capped(ceil_div(front, TB), tile_cap(SLOT_TILES));
    const dim3 grid_slots(grid_blocks(S, tpb));
    hipLaunchKernelGGL(k_table_plan, dim3(1), dim3(TB), 0, st, T, S, g->num_nodes, k, nfront,
                       nlist, w.tab_total);
    hipLaunchKernelGGL(k_table_clear, dim3(4096), dim3(TB), 0, st, T, w.tab_total, nfront, S, front);
    GINEX_LAUNCH_CHECK();
    if (stage >= 0) {
      hipLaunchKernelGGL(k_reinsert, grid_slots, dim3(TB), 0, st, T, nlist, S, tpb);
      GINEX_LAUNCH_CHECK();
    }
    if (stage < 0) {
      hipLaunchKernelGGL(k_seed_stage, grid_slots, dim3(TB), 0, st, T, seeds, w.seed_off, nfront, S,
                         tpb);
    } else if (g->nc_address_table) {
      if (g->offsets_64)
        launch_pick<int64_t, true>(T, p, g, nfront, k, stage, S, rng_seed, first_batch_index, st);
      else
        launch_pick<int32_t, true>(T, p, g, nfront, k, stage, S, rng_seed, first_batch_index, st);
    } else if (g->offsets_64) {
      launch_pick<int64_t, false>(T, p, g, nfront, k, stage, S, rng_seed, first_batch_index, st);
    } else {
      launch_pick<int32_t, false>(T, p, g, nfront, k, stage, S, rng_seed, first_batch_index, st);
    }
    GINEX_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_count, grid_slots, dim3(TB), 0, st, T, nfront, w.tile_sums, p.tiles, S,
                       tpb);
    GINEX_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_scan_batch, dim3(S), dim3(TB), 0, st, w.tile_sums, p.tiles, nfront,
                       w.batch_total);
    GINEX_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_stage_offsets, dim3(1), dim3(TB), 0, st, M, S, H, stage, w.batch_total,
                       nfront, nlist, nlist_next, w.row_base, w.col_base);
    GINEX_LAUNCH_CHECK();
    const bool adj = stage >= 0 && adj_rowptr != nullptr;
    hipLaunchKernelGGL(k_emit, grid_slots, dim3(TB), 0, st, T, nfront, nlist, k, w.tile_sums,
                       p.tiles, adj ? adj_rowptr : (int64_t*)nullptr, rowptr_capacity, w.row_base,
                       adj ? adj_col : (int32_t*)nullptr, col_capacity, w.col_base, S, tpb);
    GINEX_LAUNCH_CHECK();
    if (adj) {
      hipLaunchKernelGGL(k_col, grid_slots, dim3(TB), 0, st, T, nfront, k, adj_rowptr,
                         rowptr_capacity, w.row_base, adj_col, col_capacity, w.col_base, S, tpb);
      GINEX_LAUNCH_CHECK();
    }
    int32_t* t = nlist; nlist = nlist_next; nlist_next = t;
  }
  hipLaunchKernelGGL(k_ids_offsets, dim3(1), dim3(TB), 0, st, M, S, nlist);
  GINEX_LAUNCH_CHECK();
  if (ids_capacity > 0) {
    hipLaunchKernelGGL(k_copy_ids, dim3((unsigned)ceil_div(p.stride_ids, TB * 4), S), dim3(TB), 0,
                       st, T, M, nlist, ids, ids_capacity);
    GINEX_LAUNCH_CHECK();
  }
  // the small host outputs sit back to back in the workspace: one copy brings them all over
  {
    std::vector<int64_t> host(meta_elems(S, H));
    GINEX_HIP(hipMemcpyAsync(host.data(), w.meta, sizeof(int64_t) * host.size(),
                             hipMemcpyDeviceToHost, st));
    GINEX_HIP(hipStreamSynchronize(st));
    const int64_t* at = host.data();
    memcpy(ids_offsets, at, sizeof(int64_t) * (S + 1));
    at += S + 1;
    memcpy(hop_sizes, at, sizeof(int64_t) * S * (H + 1));
    at += (int64_t)S * (H + 1);
    memcpy(adj_row_offsets, at, sizeof(int64_t) * ((int64_t)S * H + 1));
    at += (int64_t)S * H + 1;
    memcpy(adj_col_offsets, at, sizeof(int64_t) * ((int64_t)S * H + 1));
    at += (int64_t)S * H + 1;
    memcpy(totals, at, sizeof(int64_t) * 3);
  }
  if (totals[0] > ids_capacity)
    return fail(GINEX_ERR_CAPACITY, "%s: ids needs %lld entries, capacity %lld", who,
                (long long)totals[0], (long long)ids_capacity);
  if (adj_rowptr && (totals[1] > rowptr_capacity || totals[2] > col_capacity))
    return fail(GINEX_ERR_CAPACITY, "%s: adj needs %lld rowptr / %lld col entries", who,
                (long long)totals[1], (long long)totals[2]);
  return GINEX_OK;
}
