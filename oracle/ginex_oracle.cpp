// CPU oracle for the inspector-executor hot path of Ginex (arXiv 2208.09151).
//
// THIS IS TEST INFRASTRUCTURE.  Only tests, the smoke check and the benchmark's
// cpu_baseline leg may link or call it.  It is single-threaded, slow and plain
// on purpose, shares no code with the HIP library, and never calls it.
//
// Every function below states the passage of the paper it follows.  Where the
// paper leaves a choice open, the choice taken is written beside the code.
//
// Pin status (what each function is checked against, other than itself):
//   philox4x32_10          published known-answer vectors + an independent big-int version
//   floyd_picks            distinctness/range/count, chi-square uniformity, whole-row case
//   sample_batch           structural invariants against the CSR, independence of S
//   next_use               naive forward scan, the worked five-node example of the paper
//   changeset (heap)       the sort-based definition, exhaustive search of all eviction
//                          choices on tiny traces, LRU and static-cache upper bounds
//   changeset_resume       equals the standard changeset when started from the standard
//                          prefetch, the sort-based definition, exhaustive search from the
//                          given start state, a line-by-line replay of its final state
//   changeset_lru          a textbook LRU list on single-access traces, the closed form of a
//                          cyclic trace, the sort-based definition, the stand-alone LRU
//                          miss counter, Belady's miss count as a lower bound
//   neighbour cache        the layout values the paper states for its figure, an exact
//                          rational ranking in Python, lookup == CSR row for every cached
//                          node, sampling through the cache == sampling without it
//   static_select          star / ladder / all-equal graphs whose ranking is known in closed
//                          form, "no unselected node has a larger out-degree" against a
//                          library histogram, the order inside ties
//   static_misses          a hand-counted trace, total - sum of the members' access counts
//                          against a library histogram, the empty and the complete cache
//   gather / cache replay  the worked ten-node example of the paper, out[p] == slow[ids[p]]
//   resolve_lines          the same example, the address table of the cache replay before
//                          every iteration, hit counts
//
// Build: g++ -O2 -std=c++17 -shared -fPIC ginex_oracle.cpp -o libginex_oracle.so

#include <algorithm>
#include <cstdint>
#include <cstring>
#include <queue>
#include <vector>

namespace {

constexpr int32_t NEVER = 0x7fffffff;  // "not accessed again in this superbatch"

// ---------------------------------------------------------------------------
// Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy
// as 1, 2, 3", SC'11).  Ten rounds; each round multiplies two counter words by
// fixed odd constants, swaps high/low halves across lanes and xors in the key;
// the key is advanced by the Weyl constants between rounds.
// ---------------------------------------------------------------------------
void philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
  const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    uint64_t p0 = M0 * c0;
    uint64_t p1 = M1 * c2;
    uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    uint32_t n1 = (uint32_t)p1;
    uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += W0; k1 += W1;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

uint64_t mulhi64(uint64_t a, uint64_t b) {
  return (uint64_t)(((unsigned __int128)a * (unsigned __int128)b) >> 64);
}

// One 64-bit draw for (seed, node, batch, hop, draw index).  The counter carries
// the four coordinates, the key carries the seed; words 0 and 1 of the output
// block form the draw (word 1 is the high half).
uint64_t draw64(uint64_t seed, uint32_t node, uint32_t batch, uint32_t hop, uint32_t i) {
  uint32_t ctr[4] = {node, batch, hop, i};
  uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  uint32_t x[4];
  philox4x32_10(ctr, key, x);
  return ((uint64_t)x[1] << 32) | x[0];
}

// GraphSAGE-style neighbourhood sampling takes at most k of a node's
// neighbours (Section 2.1, "Neighborhood Sampling").  The draw is uniform
// without replacement over the POSITIONS 0..deg-1 of the node's adjacency row:
// the whole row when deg <= k, otherwise Robert Floyd's subset algorithm
// (Bentley & Floyd, CACM 1987): for j = deg-k .. deg-1 draw t uniform in
// [0, j]; take t unless it was taken already, in which case take j.
// The result is returned in ascending position order.
int floyd_picks(uint64_t seed, uint32_t node, uint32_t batch, uint32_t hop,
                int64_t deg, int k, int64_t* picks) {
  if (deg <= k) {
    for (int64_t p = 0; p < deg; ++p) picks[p] = p;
    return (int)deg;
  }
  for (int i = 0; i < k; ++i) {
    int64_t j = deg - k + i;
    uint64_t r = draw64(seed, node, batch, hop, (uint32_t)i);
    int64_t t = (int64_t)mulhi64(r, (uint64_t)(j + 1));
    bool taken = false;
    for (int m = 0; m < i; ++m) taken = taken || (picks[m] == t);
    picks[i] = taken ? j : t;
  }
  std::sort(picks, picks + k);
  return k;
}

inline int64_t off_at(const void* offsets, int offsets_64, int64_t v) {
  return offsets_64 ? ((const int64_t*)offsets)[v] : (int64_t)((const int32_t*)offsets)[v];
}

}  // namespace

extern "C" {

int64_t oracle_neighbor_lookup(const int64_t* address_table, const int32_t* cache_array,
                               int32_t v, int64_t* degree);
int32_t oracle_sample_superbatch_cached(
    int64_t num_nodes, const void* offsets, int32_t offsets_64, const int32_t* indices,
    const int64_t* address_table, const int32_t* cache_array,
    const int32_t* seeds, const int64_t* seed_offsets, int32_t S,
    const int32_t* fanout, int32_t H, uint64_t rng_seed, uint32_t first_batch_index,
    int32_t* ids, int64_t ids_capacity, int64_t* ids_offsets, int64_t* hop_sizes,
    int64_t* adj_rowptr, int64_t rowptr_capacity, int32_t* adj_col, int64_t col_capacity,
    int64_t* adj_row_offsets, int64_t* adj_col_offsets, int64_t* need, int64_t* lookups);

int32_t oracle_never(void) { return NEVER; }

// ---------------------------------------------------------------------------
// Neighbour cache (Section 3.2).
//
// Structure ("Neighbor Cache Structure", Figure 6a): address_table has one entry per
// node, the index into cache_array where the node's record starts, or -1; a record is the
// number of neighbours followed by the neighbour ids.
//
// Policy ("Neighbor Cache Policy"): nodes are ranked by the ratio of their number of
// out-neighbours (how often the list is likely to be asked for) to their number of
// in-neighbours (what the list costs to keep), larger first.  The CSR rows are the
// in-neighbour lists, so in-degree = row length and out-degree = the number of times the
// node occurs in `indices`.
// Choices the paper leaves open: the ratio is compared as the integer
// floor(out * 2^32 / in) so that no floating point decides the order; ties go to the
// smaller id; nodes without in-neighbours are never cached (nothing to serve); records are
// laid out in rank order from index 0; filling stops at the first node whose record does
// not fit into the `budget` entries of cache_array.
// ---------------------------------------------------------------------------
int32_t oracle_neighbor_cache_build(int64_t num_nodes, const void* offsets, int32_t offsets_64,
                                    const int32_t* indices, int64_t budget,
                                    int64_t* address_table, int32_t* cache_array,
                                    int64_t* cached_nodes, int64_t* used_entries) {
  const int64_t num_edges = off_at(offsets, offsets_64, num_nodes);
  std::vector<int64_t> out_degree(num_nodes, 0);
  for (int64_t e = 0; e < num_edges; ++e) ++out_degree[indices[e]];
  struct Ranked { uint64_t ratio; int32_t id; };
  std::vector<Ranked> order;
  for (int64_t v = 0; v < num_nodes; ++v) {
    address_table[v] = -1;
    const int64_t in_degree = off_at(offsets, offsets_64, v + 1) - off_at(offsets, offsets_64, v);
    if (in_degree > 0)
      order.push_back({((uint64_t)out_degree[v] << 32) / (uint64_t)in_degree, (int32_t)v});
  }
  std::sort(order.begin(), order.end(), [](const Ranked& a, const Ranked& b) {
    if (a.ratio != b.ratio) return a.ratio > b.ratio;
    return a.id < b.id;
  });
  int64_t used = 0, count = 0;
  for (const Ranked& r : order) {
    const int64_t lo = off_at(offsets, offsets_64, r.id);
    const int64_t in_degree = off_at(offsets, offsets_64, r.id + 1) - lo;
    if (used + 1 + in_degree > budget) break;
    address_table[r.id] = used;
    cache_array[used] = (int32_t)in_degree;
    for (int64_t j = 0; j < in_degree; ++j) cache_array[used + 1 + j] = indices[lo + j];
    used += 1 + in_degree;
    ++count;
  }
  *cached_nodes = count;
  *used_entries = used;
  return 0;
}

// Lookup (Figure 6b): three reads.  Returns the index of the first neighbour inside
// cache_array and the neighbour count, or -1 (miss).
int64_t oracle_neighbor_lookup(const int64_t* address_table, const int32_t* cache_array,
                               int32_t v, int64_t* degree) {
  const int64_t at = address_table[v];   // read 1
  if (at < 0) return -1;
  *degree = cache_array[at];             // read 2
  return at + 1;                         // read 3 is the caller's, from here on
}

void oracle_philox4x32_10(const uint32_t* ctr, const uint32_t* key, uint32_t* out) {
  philox4x32_10(ctr, key, out);
}

uint64_t oracle_draw64(uint64_t seed, uint32_t node, uint32_t batch, uint32_t hop, uint32_t i) {
  return draw64(seed, node, batch, hop, i);
}

int32_t oracle_floyd_picks(uint64_t seed, uint32_t node, uint32_t batch, uint32_t hop,
                           int64_t deg, int32_t k, int64_t* picks) {
  return floyd_picks(seed, node, batch, hop, deg, k, picks);
}

// ---------------------------------------------------------------------------
// Superbatch sample (Section 3.1, "Superbatch Sample"): every batch of the
// superbatch is sampled ahead of time and yields `ids`, the 1-D list of all
// sampled node ids, and `adj`, the connectivity among them.
//
// One batch: the list starts as the seeds.  At hop h every node that is in the
// list when the hop starts (seeds included again) draws up to fanout[h]
// neighbours; each drawn neighbour not yet in the list is appended, in the
// order frontier node by frontier node, pick by pick.  adj for the hop is a
// CSR over the frontier: row r lists, for frontier node ids[r], the list
// positions of its picks.
//
// Row v of the input CSR holds the nodes that may be sampled for v.
//
// Outputs, batch-major: ids_offsets[S+1]; hop_sizes[b*(H+1)+h] = list length
// after the seeds (h=0) and after hop h-1; segment g = b*H+h of adj has
// rowptr at adj_row_offsets[g] (frontier+1 entries, starting at 0) and col at
// adj_col_offsets[g].  Returns 0, or -1 if a capacity is too small (then the
// *_need outputs hold the required element counts).
// ---------------------------------------------------------------------------
int32_t oracle_sample_superbatch(
    int64_t num_nodes, const void* offsets, int32_t offsets_64, const int32_t* indices,
    const int32_t* seeds, const int64_t* seed_offsets, int32_t S,
    const int32_t* fanout, int32_t H, uint64_t rng_seed, uint32_t first_batch_index,
    int32_t* ids, int64_t ids_capacity, int64_t* ids_offsets, int64_t* hop_sizes,
    int64_t* adj_rowptr, int64_t rowptr_capacity, int32_t* adj_col, int64_t col_capacity,
    int64_t* adj_row_offsets, int64_t* adj_col_offsets, int64_t* need /*[3]*/) {
  return oracle_sample_superbatch_cached(
      num_nodes, offsets, offsets_64, indices, nullptr, nullptr, seeds, seed_offsets, S, fanout, H,
      rng_seed, first_batch_index, ids, ids_capacity, ids_offsets, hop_sizes, adj_rowptr,
      rowptr_capacity, adj_col, col_capacity, adj_row_offsets, adj_col_offsets, need, nullptr);
}

// The same sampling with the neighbour lists fetched through the neighbour cache
// (Section 3.2): a node whose list is cached is served from cache_array, any other from
// the CSR.  address_table == nullptr means no cache.  lookups (optional, [2]) receives the
// number of hits and misses.
int32_t oracle_sample_superbatch_cached(
    int64_t num_nodes, const void* offsets, int32_t offsets_64, const int32_t* indices,
    const int64_t* address_table, const int32_t* cache_array,
    const int32_t* seeds, const int64_t* seed_offsets, int32_t S,
    const int32_t* fanout, int32_t H, uint64_t rng_seed, uint32_t first_batch_index,
    int32_t* ids, int64_t ids_capacity, int64_t* ids_offsets, int64_t* hop_sizes,
    int64_t* adj_rowptr, int64_t rowptr_capacity, int32_t* adj_col, int64_t col_capacity,
    int64_t* adj_row_offsets, int64_t* adj_col_offsets, int64_t* need /*[3]*/,
    int64_t* lookups /*[2] or null*/) {
  int64_t hits = 0, misses = 0;
  std::vector<int32_t> local(num_nodes, -1);
  std::vector<int32_t> list;
  std::vector<int64_t> picks(64);
  int64_t n_ids = 0, n_row = 0, n_col = 0;
  bool fits = true;
  ids_offsets[0] = 0;
  adj_row_offsets[0] = 0;
  adj_col_offsets[0] = 0;
  for (int32_t b = 0; b < S; ++b) {
    list.clear();
    for (int64_t s = seed_offsets[b]; s < seed_offsets[b + 1]; ++s) {
      int32_t v = seeds[s];
      if (local[v] < 0) {  // a repeated seed keeps its first position
        local[v] = (int32_t)list.size();
        list.push_back(v);
      }
    }
    hop_sizes[(int64_t)b * (H + 1)] = (int64_t)list.size();
    for (int32_t h = 0; h < H; ++h) {
      const int k = fanout[h];
      if ((int64_t)picks.size() < k) picks.resize(k);
      const int64_t frontier = (int64_t)list.size();
      const int64_t col_base = n_col;
      for (int64_t r = 0; r < frontier; ++r) {
        if (n_row < rowptr_capacity) adj_rowptr[n_row] = n_col - col_base; else fits = false;
        ++n_row;
        const int32_t v = list[r];
        int64_t deg;
        const int32_t* row;
        const int64_t at = address_table ? oracle_neighbor_lookup(address_table, cache_array, v, &deg)
                                         : -1;
        if (at >= 0) {
          row = cache_array + at;
          ++hits;
        } else {
          const int64_t lo = off_at(offsets, offsets_64, v);
          deg = off_at(offsets, offsets_64, v + 1) - lo;
          row = indices + lo;
          ++misses;
        }
        const int cnt = floyd_picks(rng_seed, (uint32_t)v, first_batch_index + (uint32_t)b,
                                    (uint32_t)h, deg, k, picks.data());
        for (int t = 0; t < cnt; ++t) {
          const int32_t u = row[picks[t]];
          if (local[u] < 0) {
            local[u] = (int32_t)list.size();
            list.push_back(u);
          }
          if (n_col < col_capacity) adj_col[n_col] = local[u]; else fits = false;
          ++n_col;
        }
      }
      if (n_row < rowptr_capacity) adj_rowptr[n_row] = n_col - col_base; else fits = false;
      ++n_row;
      adj_row_offsets[(int64_t)b * H + h + 1] = n_row;
      adj_col_offsets[(int64_t)b * H + h + 1] = n_col;
      hop_sizes[(int64_t)b * (H + 1) + h + 1] = (int64_t)list.size();
    }
    for (size_t j = 0; j < list.size(); ++j) {
      if (n_ids < ids_capacity) ids[n_ids] = list[j]; else fits = false;
      ++n_ids;
      local[list[j]] = -1;
    }
    ids_offsets[b + 1] = n_ids;
  }
  need[0] = n_ids; need[1] = n_row; need[2] = n_col;
  if (lookups) { lookups[0] = hits; lookups[1] = misses; }
  return fits ? 0 : -1;
}

// ---------------------------------------------------------------------------
// Next accessed iteration (Section 3.4): for the access of node v at iteration
// i, the smallest j > i with v in ids_j, or NEVER.  Computed by one backward
// pass that remembers where each node was seen last.  first_iter[v] (optional)
// receives the first iteration that accesses v, or NEVER.
// ---------------------------------------------------------------------------
void oracle_next_use(int64_t num_nodes, const int32_t* ids, const int64_t* ids_offsets,
                     int32_t S, int32_t* next_iter, int32_t* first_iter) {
  std::vector<int32_t> seen(num_nodes, NEVER);
  for (int32_t i = S - 1; i >= 0; --i)
    for (int64_t p = ids_offsets[i]; p < ids_offsets[i + 1]; ++p) {
      next_iter[p] = seen[ids[p]];
      seen[ids[p]] = i;
    }
  if (first_iter) std::memcpy(first_iter, seen.data(), sizeof(int32_t) * num_nodes);
}

}  // extern "C"

namespace {

// Order in which candidates are kept (Section 3.4: f_Belady keeps, of
// union(C_i, ids_i), as many elements as the cache has entries, those accessed
// earliest first).  The paper does not order candidates whose next accessed
// iteration is equal; the reading taken here: a resident row comes before an
// incoming one, then the smaller node id comes first.
struct Key {
  int32_t next; int32_t incoming; int32_t id;
  bool operator<(const Key& o) const {
    if (next != o.next) return next < o.next;
    if (incoming != o.incoming) return incoming < o.incoming;
    return id < o.id;
  }
};

// C_0 (Section 3.3: the cache is prefetched with the rows that appear in the
// first iterations until it is full): the `cap` smallest of (first_iter, id);
// the row of rank r gets cache line r.
std::vector<int32_t> initial_state(int64_t num_nodes, const std::vector<int32_t>& first_iter,
                                   int64_t cap) {
  std::vector<std::pair<int32_t, int32_t>> order;
  for (int64_t v = 0; v < num_nodes; ++v)
    if (first_iter[v] != NEVER) order.push_back({first_iter[v], (int32_t)v});
  std::sort(order.begin(), order.end());
  if ((int64_t)order.size() > cap) order.resize(cap);
  std::vector<int32_t> init(order.size());
  for (size_t r = 0; r < order.size(); ++r) init[r] = order[r].second;
  return init;
}

struct ChangesetOut {
  int32_t* init_ids; int64_t* init_count;
  int32_t* in_ids; int32_t* out_ids; int32_t* in_positions; int64_t cs_capacity;
  int64_t* cs_offsets; int64_t* miss_count;
  int64_t written = 0; bool fits = true;
  void emit(int32_t in_id, int32_t out_id, int32_t pos) {
    if (written < cs_capacity) {
      in_ids[written] = in_id; out_ids[written] = out_id; in_positions[written] = pos;
    } else {
      fits = false;
    }
    ++written;
  }
};

// Replacement policies.  Both keep, out of union(C_i, ids_i), the `cap` elements with
// the smallest key; they differ only in the key an access leaves on a row.
//   Belady (Section 3.4): the iteration of the row's next access (NEVER if none).
//   LRU (Section 2.3, the policy Belady's is measured against): S-1-i for an access in
//   iteration i, so that a row used longer ago has a larger key; a prefetched row that
//   has not been used yet has key S, larger than any used row's.
enum Policy { BELADY = 0, LRU = 1 };

// Cache state carried from one superbatch into the next (an extension: the paper starts every
// superbatch from a fresh prefetch, Section 3.1).  start_ids[r] is the row held by cache
// line r when the superbatch begins (start_count <= cap lines are occupied, from line 0);
// it replaces the prefetched C_0.  final_ids[line] receives the row each line holds after
// the last iteration (-1 = empty).
struct Carry {
  const int32_t* start_ids;
  int64_t start_count;
  int32_t* final_ids;
};

inline int32_t key_after_access(Policy policy, int32_t S, int32_t i, int32_t next) {
  return policy == BELADY ? next : S - 1 - i;
}
inline int32_t key_of_prefetched(Policy policy, int32_t S, int32_t first) {
  return policy == BELADY ? first : S;
}

int32_t changeset_with_heap(Policy policy, int64_t num_nodes, const int32_t* ids,
                            const int64_t* ids_offsets, int32_t S, int64_t cap,
                            int32_t* init_ids, int64_t* init_count, int32_t* in_ids,
                            int32_t* out_ids, int32_t* in_positions, int64_t cs_capacity,
                            int64_t* cs_offsets, int64_t* miss_count, const Carry* carry = nullptr);
int32_t changeset_from_definition(Policy policy, int64_t num_nodes, const int32_t* ids,
                                  const int64_t* ids_offsets, int32_t S, int64_t cap,
                                  int32_t* init_ids, int64_t* init_count, int32_t* in_ids,
                                  int32_t* out_ids, int32_t* in_positions, int64_t cs_capacity,
                                  int64_t* cs_offsets, int64_t* miss_count,
                                  const Carry* carry = nullptr);

}  // namespace

extern "C" {

// ---------------------------------------------------------------------------
// Changeset precomputation (Sections 3.3 "Feature Cache Update" and 3.4).
// Simulates C_{i+1} = f_Belady(union(C_i, ids_i)) and records, per iteration,
// in_ids = C_{i+1} \ C_i, out_ids = C_i \ C_{i+1} and in_positions = where each
// in-id sits inside ids_i.  A row that misses and is not kept is served from
// the slow tier and bypasses the cache.
// List order (paper silent): in_ids by ascending position in ids_i; out_ids by
// ascending cache line; in_ids[j] takes the line of out_ids[j].
// S records are written; ids within one iteration must be distinct.
//
// This variant keeps residents in a max-heap on (next, id) with lazy
// invalidation and drops, per iteration, exactly as many candidates as missed.
// Returns 0, or -1 when cs_capacity is too small (cs_offsets[S] = needed).
// ---------------------------------------------------------------------------
int32_t oracle_changeset(int64_t num_nodes, const int32_t* ids, const int64_t* ids_offsets,
                         int32_t S, int64_t cap,
                         int32_t* init_ids, int64_t* init_count,
                         int32_t* in_ids, int32_t* out_ids, int32_t* in_positions,
                         int64_t cs_capacity, int64_t* cs_offsets, int64_t* miss_count) {
  return changeset_with_heap(BELADY, num_nodes, ids, ids_offsets, S, cap, init_ids, init_count,
                             in_ids, out_ids, in_positions, cs_capacity, cs_offsets, miss_count);
}

// The same lists for the LRU policy (Section 2.3), same C_0, same list order.
int32_t oracle_changeset_lru(int64_t num_nodes, const int32_t* ids, const int64_t* ids_offsets,
                             int32_t S, int64_t cap,
                             int32_t* init_ids, int64_t* init_count,
                             int32_t* in_ids, int32_t* out_ids, int32_t* in_positions,
                             int64_t cs_capacity, int64_t* cs_offsets, int64_t* miss_count) {
  return changeset_with_heap(LRU, num_nodes, ids, ids_offsets, S, cap, init_ids, init_count,
                             in_ids, out_ids, in_positions, cs_capacity, cs_offsets, miss_count);
}

}  // extern "C"

namespace {

int32_t changeset_with_heap(Policy policy, int64_t num_nodes, const int32_t* ids,
                            const int64_t* ids_offsets, int32_t S, int64_t cap,
                            int32_t* init_ids, int64_t* init_count, int32_t* in_ids,
                            int32_t* out_ids, int32_t* in_positions, int64_t cs_capacity,
                            int64_t* cs_offsets, int64_t* miss_count, const Carry* carry) {
  const int64_t total = ids_offsets[S];
  std::vector<int32_t> next_iter(total > 0 ? total : 1), first_iter(num_nodes);
  oracle_next_use(num_nodes, ids, ids_offsets, S, next_iter.data(), first_iter.data());

  ChangesetOut o{init_ids, init_count, in_ids, out_ids, in_positions, cs_capacity,
                 cs_offsets, miss_count};
  std::vector<int32_t> init = carry ? std::vector<int32_t>(carry->start_ids,
                                                           carry->start_ids + carry->start_count)
                                    : initial_state(num_nodes, first_iter, cap);
  *init_count = (int64_t)init.size();
  std::vector<int32_t> line_of(num_nodes, -1), key_of(num_nodes, NEVER);
  typedef std::pair<int32_t, int32_t> Entry;  // (next, id); the largest is on top
  std::priority_queue<Entry> heap;
  for (size_t r = 0; r < init.size(); ++r) {
    init_ids[r] = init[r];
    line_of[init[r]] = (int32_t)r;
    key_of[init[r]] = key_of_prefetched(policy, S, first_iter[init[r]]);
    heap.push({key_of[init[r]], init[r]});
  }
  int64_t occupancy = (int64_t)init.size();

  struct Incoming { Key key; int32_t pos; };
  std::vector<Incoming> incoming;
  std::vector<std::pair<int32_t, int32_t>> evicted;  // (line, id)
  cs_offsets[0] = 0;
  for (int32_t i = 0; i < S; ++i) {
    incoming.clear();
    evicted.clear();
    for (int64_t p = ids_offsets[i]; p < ids_offsets[i + 1]; ++p) {
      const int32_t v = ids[p];
      const int32_t key = key_after_access(policy, S, i, next_iter[p]);
      if (line_of[v] >= 0) {
        key_of[v] = key;
        heap.push({key, v});
      } else {
        incoming.push_back({Key{key, 1, v}, (int32_t)(p - ids_offsets[i])});
      }
    }
    miss_count[i] = (int64_t)incoming.size();
    std::sort(incoming.begin(), incoming.end(),
              [](const Incoming& a, const Incoming& b) { return a.key < b.key; });
    // Free lines exist only when every accessed row fitted into C_0; then
    // nothing ever misses.  Otherwise the cache is full and each miss forces
    // one candidate out.
    int64_t to_drop = occupancy + (int64_t)incoming.size() - cap;
    if (to_drop < 0) to_drop = 0;
    int64_t kept_in = (int64_t)incoming.size();
    while (to_drop > 0) {
      while (!heap.empty()) {
        const Entry& e = heap.top();
        if (line_of[e.second] >= 0 && key_of[e.second] == e.first) break;
        heap.pop();
      }
      bool drop_incoming;
      if (kept_in == 0) drop_incoming = false;
      else if (heap.empty()) drop_incoming = true;
      else {
        Key res{heap.top().first, 0, heap.top().second};
        drop_incoming = res < incoming[kept_in - 1].key;
      }
      if (drop_incoming) {
        --kept_in;
      } else {
        const int32_t v = heap.top().second;
        heap.pop();
        evicted.push_back({line_of[v], v});
        line_of[v] = -1;
        --occupancy;
      }
      --to_drop;
    }
    incoming.resize(kept_in);
    std::sort(incoming.begin(), incoming.end(),
              [](const Incoming& a, const Incoming& b) { return a.pos < b.pos; });
    std::sort(evicted.begin(), evicted.end());
    // incoming rows first reuse the evicted lines, pairwise; any beyond that
    // (possible only while the cache is not full) would take fresh lines.
    for (size_t j = 0; j < incoming.size(); ++j) {
      const int32_t v = incoming[j].key.id;
      int32_t line, out_id;
      if (j < evicted.size()) { line = evicted[j].first; out_id = evicted[j].second; }
      else { line = (int32_t)occupancy; out_id = -1; }
      line_of[v] = line;
      key_of[v] = incoming[j].key.next;
      heap.push({key_of[v], v});
      ++occupancy;
      o.emit(v, out_id, incoming[j].pos);
    }
    cs_offsets[i + 1] = o.written;
  }
  if (carry && carry->final_ids) {
    for (int64_t l = 0; l < cap; ++l) carry->final_ids[l] = -1;
    for (int64_t v = 0; v < num_nodes; ++v)
      if (line_of[v] >= 0) carry->final_ids[line_of[v]] = (int32_t)v;
  }
  return o.fits ? 0 : -1;
}

// The same result computed straight from the definition: every iteration the
// whole candidate set is sorted by the keeping order and cut at `cap`.
// O(S * cap log cap); for small inputs and for checking the heap variant.
int32_t changeset_from_definition(Policy policy, int64_t num_nodes, const int32_t* ids,
                                  const int64_t* ids_offsets, int32_t S, int64_t cap,
                                  int32_t* init_ids, int64_t* init_count, int32_t* in_ids,
                                  int32_t* out_ids, int32_t* in_positions, int64_t cs_capacity,
                                  int64_t* cs_offsets, int64_t* miss_count, const Carry* carry) {
  const int64_t total = ids_offsets[S];
  std::vector<int32_t> next_iter(total > 0 ? total : 1), first_iter(num_nodes);
  oracle_next_use(num_nodes, ids, ids_offsets, S, next_iter.data(), first_iter.data());
  ChangesetOut o{init_ids, init_count, in_ids, out_ids, in_positions, cs_capacity,
                 cs_offsets, miss_count};
  std::vector<int32_t> init = carry ? std::vector<int32_t>(carry->start_ids,
                                                           carry->start_ids + carry->start_count)
                                    : initial_state(num_nodes, first_iter, cap);
  *init_count = (int64_t)init.size();
  // cache lines: node id and its next accessed iteration, -1 = empty line
  std::vector<int32_t> line_id(cap, -1), line_next(cap, NEVER), line_of(num_nodes, -1);
  for (size_t r = 0; r < init.size(); ++r) {
    init_ids[r] = init[r];
    line_id[r] = init[r];
    line_next[r] = key_of_prefetched(policy, S, first_iter[init[r]]);
    line_of[init[r]] = (int32_t)r;
  }
  struct Cand { Key key; int32_t pos; int32_t line; };
  std::vector<Cand> cand;
  cs_offsets[0] = 0;
  for (int32_t i = 0; i < S; ++i) {
    const int64_t lo = ids_offsets[i], hi = ids_offsets[i + 1];
    for (int64_t p = lo; p < hi; ++p)
      if (line_of[ids[p]] >= 0)
        line_next[line_of[ids[p]]] = key_after_access(policy, S, i, next_iter[p]);
    cand.clear();
    for (int64_t l = 0; l < cap; ++l)
      if (line_id[l] >= 0) cand.push_back({Key{line_next[l], 0, line_id[l]}, -1, (int32_t)l});
    int64_t misses = 0;
    for (int64_t p = lo; p < hi; ++p)
      if (line_of[ids[p]] < 0) {
        cand.push_back({Key{key_after_access(policy, S, i, next_iter[p]), 1, ids[p]},
                        (int32_t)(p - lo), -1});
        ++misses;
      }
    miss_count[i] = misses;
    std::sort(cand.begin(), cand.end(),
              [](const Cand& a, const Cand& b) { return a.key < b.key; });
    std::vector<Cand> ins, outs;
    for (size_t r = 0; r < cand.size(); ++r) {
      const bool kept = (int64_t)r < cap;
      if (kept && cand[r].key.incoming) ins.push_back(cand[r]);
      if (!kept && !cand[r].key.incoming) outs.push_back(cand[r]);
    }
    std::sort(ins.begin(), ins.end(), [](const Cand& a, const Cand& b) { return a.pos < b.pos; });
    std::sort(outs.begin(), outs.end(), [](const Cand& a, const Cand& b) { return a.line < b.line; });
    for (size_t j = 0; j < outs.size(); ++j) {
      line_of[outs[j].key.id] = -1;
      line_id[outs[j].line] = -1;
    }
    int64_t free_line = 0;
    for (size_t j = 0; j < ins.size(); ++j) {
      int32_t line, out_id = -1;
      if (j < outs.size()) { line = outs[j].line; out_id = outs[j].key.id; }
      else {
        while (line_id[free_line] >= 0) ++free_line;
        line = (int32_t)free_line;
      }
      line_id[line] = ins[j].key.id;
      line_next[line] = ins[j].key.next;
      line_of[ins[j].key.id] = line;
      o.emit(ins[j].key.id, out_id, ins[j].pos);
    }
    cs_offsets[i + 1] = o.written;
  }
  if (carry && carry->final_ids)
    for (int64_t l = 0; l < cap; ++l) carry->final_ids[l] = line_id[l];
  return o.fits ? 0 : -1;
}

}  // namespace

extern "C" {

int32_t oracle_changeset_by_sorting(int64_t num_nodes, const int32_t* ids,
                                    const int64_t* ids_offsets, int32_t S, int64_t cap,
                                    int32_t* init_ids, int64_t* init_count,
                                    int32_t* in_ids, int32_t* out_ids, int32_t* in_positions,
                                    int64_t cs_capacity, int64_t* cs_offsets,
                                    int64_t* miss_count) {
  return changeset_from_definition(BELADY, num_nodes, ids, ids_offsets, S, cap, init_ids,
                                   init_count, in_ids, out_ids, in_positions, cs_capacity,
                                   cs_offsets, miss_count);
}

int32_t oracle_changeset_lru_by_sorting(int64_t num_nodes, const int32_t* ids,
                                        const int64_t* ids_offsets, int32_t S, int64_t cap,
                                        int32_t* init_ids, int64_t* init_count,
                                        int32_t* in_ids, int32_t* out_ids, int32_t* in_positions,
                                        int64_t cs_capacity, int64_t* cs_offsets,
                                        int64_t* miss_count) {
  return changeset_from_definition(LRU, num_nodes, ids, ids_offsets, S, cap, init_ids,
                                   init_count, in_ids, out_ids, in_positions, cs_capacity,
                                   cs_offsets, miss_count);
}

// Belady changesets of a superbatch that starts from a given cache state instead of a
// fresh prefetch (see Carry); init_ids/init_count echo the start state.
int32_t oracle_changeset_resume(int64_t num_nodes, const int32_t* ids, const int64_t* ids_offsets,
                                int32_t S, int64_t cap, const int32_t* start_ids,
                                int64_t start_count, int32_t* final_ids, int32_t* init_ids,
                                int64_t* init_count, int32_t* in_ids, int32_t* out_ids,
                                int32_t* in_positions, int64_t cs_capacity, int64_t* cs_offsets,
                                int64_t* miss_count) {
  const Carry carry{start_ids, start_count, final_ids};
  return changeset_with_heap(BELADY, num_nodes, ids, ids_offsets, S, cap, init_ids, init_count,
                             in_ids, out_ids, in_positions, cs_capacity, cs_offsets, miss_count,
                             &carry);
}

int32_t oracle_changeset_resume_by_sorting(int64_t num_nodes, const int32_t* ids,
                                           const int64_t* ids_offsets, int32_t S, int64_t cap,
                                           const int32_t* start_ids, int64_t start_count,
                                           int32_t* final_ids, int32_t* init_ids,
                                           int64_t* init_count, int32_t* in_ids, int32_t* out_ids,
                                           int32_t* in_positions, int64_t cs_capacity,
                                           int64_t* cs_offsets, int64_t* miss_count) {
  const Carry carry{start_ids, start_count, final_ids};
  return changeset_from_definition(BELADY, num_nodes, ids, ids_offsets, S, cap, init_ids,
                                   init_count, in_ids, out_ids, in_positions, cs_capacity,
                                   cs_offsets, miss_count, &carry);
}

// Miss count of a least-recently-used cache started from the same C_0 under
// the same rules (a miss is served from the slow tier; after iteration i the
// cache keeps the `cap` most recently used rows of union(C_i, ids_i), ties by
// node id).  Used only as an upper bound on Belady's miss count.
int64_t oracle_lru_misses(int64_t num_nodes, const int32_t* ids, const int64_t* ids_offsets,
                          int32_t S, int64_t cap, const int32_t* init_ids, int64_t init_count) {
  std::vector<int32_t> last_use(num_nodes, -1);
  std::vector<char> resident(num_nodes, 0);
  std::vector<int32_t> members(init_ids, init_ids + init_count);
  for (int32_t v : members) resident[v] = 1;
  int64_t misses = 0;
  for (int32_t i = 0; i < S; ++i) {
    for (int64_t p = ids_offsets[i]; p < ids_offsets[i + 1]; ++p) {
      const int32_t v = ids[p];
      if (!resident[v]) { ++misses; members.push_back(v); resident[v] = 1; }
      last_use[v] = i;
    }
    if ((int64_t)members.size() > cap) {
      std::sort(members.begin(), members.end(), [&](int32_t a, int32_t b) {
        if (last_use[a] != last_use[b]) return last_use[a] > last_use[b];
        return a < b;
      });
      for (size_t r = cap; r < members.size(); ++r) resident[members[r]] = 0;
      members.resize(cap);
    }
  }
  return misses;
}

// Content of a static cache (Section 2.3 "Challenge 1": the policy of the
// systems the paper compares with keeps the nodes of highest out-degree in
// memory for the whole run).  Rows of the CSR are in-neighbour lists, so a
// node's out-degree is the number of times it occurs in `indices`.  The cache
// takes the `cap` nodes of highest out-degree; among equal out-degrees the
// smaller id comes first (the paper does not say).  out_ids[r] = node of rank r.
// Returns how many were written: min(cap, num_nodes).
int64_t oracle_static_select(int64_t num_nodes, const int32_t* indices, int64_t num_edges,
                             int64_t cap, int32_t* out_ids) {
  std::vector<int64_t> out_degree(num_nodes, 0);
  for (int64_t e = 0; e < num_edges; ++e) ++out_degree[indices[e]];
  std::vector<int32_t> order(num_nodes);
  for (int64_t v = 0; v < num_nodes; ++v) order[v] = (int32_t)v;
  std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
    return out_degree[a] > out_degree[b];   // stable: equal degrees stay in id order
  });
  const int64_t count = cap < num_nodes ? cap : num_nodes;
  for (int64_t r = 0; r < count; ++r) out_ids[r] = order[r];
  return count < 0 ? 0 : count;
}

// Miss count of a cache whose content never changes (the static policies the
// paper compares with, Section 2.3 "Challenge 1").
int64_t oracle_static_misses(int64_t num_nodes, const int32_t* ids, int64_t total,
                             const int32_t* members, int64_t count) {
  std::vector<char> resident(num_nodes, 0);
  for (int64_t r = 0; r < count; ++r) resident[members[r]] = 1;
  int64_t misses = 0;
  for (int64_t p = 0; p < total; ++p) misses += !resident[ids[p]];
  return misses;
}

// ---------------------------------------------------------------------------
// Gather and cache update (Section 3.3, the worked example of "Feature Cache
// Update"): the batch input holds, in the order of ids, the feature row of
// every id.  By definition out[p] = slow[ids[p]].
// ---------------------------------------------------------------------------
void oracle_gather(const uint8_t* slow, int64_t row_bytes, const int32_t* ids, int64_t n,
                   uint8_t* out) {
  for (int64_t p = 0; p < n; ++p)
    std::memcpy(out + p * row_bytes, slow + (int64_t)ids[p] * row_bytes, row_bytes);
}

// The executor's view: gather through the cache, then apply the update.
// address_table[v] is the cache line of v or -1.  For each id the row comes
// from the cache on a hit, else from the slow tier; afterwards row
// in_positions[j] of the batch input replaces the line held by out_ids[j] and
// the address table is patched.  Returns the number of hits.
int64_t oracle_gather_update(uint8_t* cache, int32_t* address_table, const uint8_t* slow,
                             int64_t row_bytes, const int32_t* ids, int64_t n, uint8_t* out,
                             const int32_t* in_ids, const int32_t* out_ids,
                             const int32_t* in_positions, int64_t n_change) {
  int64_t hits = 0;
  for (int64_t p = 0; p < n; ++p) {
    const int32_t line = address_table[ids[p]];
    const uint8_t* src = line >= 0 ? cache + (int64_t)line * row_bytes
                                   : slow + (int64_t)ids[p] * row_bytes;
    hits += line >= 0;
    std::memcpy(out + p * row_bytes, src, row_bytes);
  }
  for (int64_t j = 0; j < n_change; ++j) {
    const int32_t line = address_table[out_ids[j]];
    std::memcpy(cache + (int64_t)line * row_bytes, out + (int64_t)in_positions[j] * row_bytes,
                row_bytes);
    address_table[out_ids[j]] = -1;
    address_table[in_ids[j]] = line;
  }
  return hits;
}

// Feature cache initialization (Section 3.1): load the rows named in `init`
// and build the address table.
// What the address table returns for every access of a superbatch (Section 3.3 "Feature
// Cache Structure": the entry of a node is its cache line, or -1): the table is set up
// from `init` (line r holds init_ids[r]) and, after the lookups of iteration i, patched
// with update_i exactly as the cache update does (in_ids[j] inherits the line of
// out_ids[j]).  No rows are moved; lines[p] is the lookup result for access p.
void oracle_resolve_lines(int64_t num_nodes, const int32_t* ids, const int64_t* ids_offsets,
                          int32_t S, const int32_t* init_ids, int64_t init_count,
                          const int32_t* in_ids, const int32_t* out_ids,
                          const int64_t* cs_offsets, int32_t* lines) {
  std::vector<int32_t> address_table(num_nodes, -1);
  for (int64_t r = 0; r < init_count; ++r) address_table[init_ids[r]] = (int32_t)r;
  for (int32_t i = 0; i < S; ++i) {
    for (int64_t p = ids_offsets[i]; p < ids_offsets[i + 1]; ++p)
      lines[p] = address_table[ids[p]];
    for (int64_t j = cs_offsets[i]; j < cs_offsets[i + 1]; ++j) {
      const int32_t line = address_table[out_ids[j]];
      address_table[out_ids[j]] = -1;
      address_table[in_ids[j]] = line;
    }
  }
}

void oracle_cache_init(uint8_t* cache, int32_t* address_table, int64_t num_nodes,
                       const uint8_t* slow, int64_t row_bytes, const int32_t* init_ids,
                       int64_t init_count) {
  for (int64_t v = 0; v < num_nodes; ++v) address_table[v] = -1;
  for (int64_t r = 0; r < init_count; ++r) {
    std::memcpy(cache + r * row_bytes, slow + (int64_t)init_ids[r] * row_bytes, row_bytes);
    address_table[init_ids[r]] = (int32_t)r;
  }
}

}  // extern "C"
