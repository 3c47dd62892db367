// Changeset precomputation on gfx950 (Ginex Section 3.4, lists of Section 3.3).
//
// Part 1, next accessed iteration of every access, fully parallel:
//   (node, flat position) pairs are radix-sorted by node (stable, so each node's accesses
//   stay in iteration order); an access's successor in the sorted array tells its next
//   accessed iteration, the head of each node's run tells the node's first access.
// Part 2, C_0: run heads (first iteration, node) sorted by first iteration; the first
//   `cap` of them fill cache lines 0..cap-1.
// Part 3, the recurrence C_{i+1} = f_Belady(union(C_i, ids_i)), serial over iterations and
//   parallel inside one.  The cache is full from C_0 on (otherwise everything fitted and
//   nothing ever changes), so iteration i must drop exactly as many candidates as it had
//   misses.  Keys are (next iteration, incoming?, node id); next iterations take only
//   S-i distinct values, so a histogram per next iteration (kept incrementally for the
//   residents, rebuilt for the incoming rows) finds the threshold bucket j*; only inside
//   j* does the id order matter, and there the k-th smallest id is found by setting the
//   members' bits in a bitmap over node ids and locating the k-th set bit through per-part
//   counts.  Evicted lines and inserted positions are then compacted in line / position
//   order and paired.
//   The same loop serves the LRU policy (other keys) and a superbatch that resumes from the
//   cache state of the previous one (C_0 given instead of computed).
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <mutex>

#include "common.hpp"
#include "primitives.hpp"

namespace ginex {
namespace {

constexpr int TB = 256;
constexpr int BIG = 1024;          // threads of the single-block kernels
constexpr int TOUCH_ITEMS = 8;     // accesses per thread in the touch kernel
constexpr int PART_SHIFT = 16;     // a part of a bitmap covers 2^16 node ids ...
constexpr int PART_WORDS = 1 << (PART_SHIFT - 5);   // ... in 2048 words

enum { MODE_NONE = 0, MODE_ALL = 1, MODE_SELECT = 2 };

struct Ctrl {        // decisions of the running iteration (device memory)
  int32_t jstar;     // threshold bucket (S+1: nothing is dropped)
  int32_t mode_in;   // incoming rows of bucket j*: none / all / ids <= T are inserted
  int32_t mode_res;  // resident rows of bucket j*: all / ids <= T are kept
  int32_t keep;      // how many members of the selected class stay
  int32_t T;         // id threshold of the select
  int32_t n_change;  // evictions (= insertions) of the iteration
  int32_t use_dead;  // the select runs on the standing bitmap of dead residents
  int32_t marked;    // bit 0: residents of bucket j* have their bits in the scratch bitmap,
                     // bit 1: incoming rows of bucket j* in theirs (both are cleared in k_flags)
};
enum { MARKED_RES = 1, MARKED_IN = 2 };
// State::fault (device, one word): set when a launch sequence that leaves the live select out
// meets an iteration that needs it (cannot happen when every row of the superbatch fits the
// cache beside the rows it already holds; checked by the host after the loop).

struct State {
  int32_t* res_id;      // [cap] node held by each cache line
  int32_t* res_next;    // [cap] its next accessed iteration (S = never)
  int32_t* addr;        // [N] line of a node or -1
  uint32_t* rhist;      // [S+1] residents per next iteration
  uint32_t* ihist;      // [S+1] incoming rows of the running iteration per next iteration
  uint32_t* bitmap;     // [words] select scratch (residents of bucket j*), all zero between iterations
  uint32_t* sel_part;   // [parts] its set bits per part, all zero between iterations
  uint32_t* bitmap_in;  // [words] the same for the incoming rows of bucket j*
  uint32_t* sel_part_in;
  uint32_t* dead_bits;  // [words] residents that are never accessed again, kept up to date
  uint32_t* dead_part;  // [parts] its set bits per part, kept up to date
  Ctrl* ctrl;
  int32_t* fault;
  uint64_t* evict_words;  // bit l%64 of word l/64: line l is evicted in this iteration
  uint32_t* evict_tiles;  // evictions per tile of EVICT_TILE lines
  uint32_t* in_tiles;     // insertions per tile of positions in ids_i
  int32_t* acc_line;      // [longest iteration] line of each access of the running iteration, -1 = miss
  uint64_t* pair;         // [max_change] meeting point of the t-th eviction and the t-th insertion
  int64_t cap, num_nodes;
  int64_t words, parts;   // of the two bitmaps
  int32_t S;
  int64_t max_change;     // entries of pair
  int32_t lru;            // 0: Belady keys (next accessed iteration), 1: LRU keys
  int32_t dead_scatter;   // evictions among the dead residents are found from the id bitmap
                          // (large caches) instead of by a pass over all cache lines
  int32_t dead_only;      // every eviction falls among the dead residents: no live select
};

// Iteration that holds flat position p: the largest i with off[i] <= p.  `off` is the
// block's LDS copy of ids_offsets (total ids < 2^31, so 32 bits do).
__device__ __forceinline__ int32_t iter_of(const int32_t* off, int32_t S, int32_t p) {
  int32_t lo = 0, hi = S;
  while (hi - lo > 1) {
    const int32_t mid = (lo + hi) >> 1;
    if (off[mid] <= p) lo = mid; else hi = mid;
  }
  return lo;
}

__device__ __forceinline__ void load_offsets(int32_t* lds_off, const int64_t* __restrict__ off,
                                             int32_t S) {
  for (int j = threadIdx.x; j <= S; j += blockDim.x) lds_off[j] = (int32_t)off[j];
  __syncthreads();
}

// ---- part 1 -----------------------------------------------------------------------

constexpr int LOOK_ITEMS = 8;
constexpr int LOOK_TILE = TB * LOOK_ITEMS;

__device__ __forceinline__ bool run_head(const uint64_t* __restrict__ sorted, int64_t j) {
  return j == 0 || (uint32_t)(sorted[j - 1] >> 32) != (uint32_t)(sorted[j] >> 32);
}

// number of run heads (= distinct nodes) per tile of the sorted pairs
__global__ __launch_bounds__(TB) void k_count_heads(const uint64_t* __restrict__ sorted, int64_t n,
                                                    uint32_t* __restrict__ head_tiles) {
  __shared__ uint32_t red[TB / WAVE];
  uint32_t heads = 0;
  const int64_t base = (int64_t)blockIdx.x * LOOK_TILE;
#pragma unroll
  for (int i = 0; i < LOOK_ITEMS; ++i) {
    const int64_t j = base + i * TB + threadIdx.x;
    if (j < n) heads += run_head(sorted, j);
  }
  heads = wave_reduce_sum(heads);
  if (lane_id() == 0) red[threadIdx.x / WAVE] = heads;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t s = 0;
    for (int w = 0; w < TB / WAVE; ++w) s += red[w];
    head_tiles[blockIdx.x] = s;
  }
}

// Precondition check (only when asked for): ids inside [0, num_nodes) and no id twice in
// one iteration.  In the node-sorted pairs a repeated id shows up as two neighbours of the
// same node whose positions fall into the same iteration.  counts[0] = out of range,
// counts[1] = repeats.
__global__ __launch_bounds__(TB) void k_validate(const uint64_t* __restrict__ sorted, int64_t n,
                                                 const int64_t* __restrict__ off, int32_t S,
                                                 int64_t num_nodes,
                                                 unsigned long long* __restrict__ counts) {
  extern __shared__ int32_t lds_off[];
  load_offsets(lds_off, off, S);
  const int64_t j = (int64_t)blockIdx.x * TB + threadIdx.x;
  if (j >= n) return;
  const uint64_t cur = sorted[j];
  const uint32_t v = (uint32_t)(cur >> 32);
  if ((int64_t)v >= num_nodes) atomicAdd(&counts[0], 1ull);
  if (j + 1 < n) {
    const uint64_t r = sorted[j + 1];
    if ((uint32_t)(r >> 32) == v &&
        iter_of(lds_off, S, (int32_t)(r & 0xFFFFFFFFu)) ==
            iter_of(lds_off, S, (int32_t)(cur & 0xFFFFFFFFu)))
      atomicAdd(&counts[1], 1ull);
  }
}

// next_iter of every access: the iteration of its right neighbour in the sorted order if
// that is the same node, else S ("never")
__global__ __launch_bounds__(TB) void k_look_right(const uint64_t* __restrict__ sorted, int64_t n,
                                                   const int64_t* __restrict__ off, int32_t S,
                                                   int32_t* __restrict__ next_iter) {
  extern __shared__ int32_t lds_off[];
  load_offsets(lds_off, off, S);
  const int64_t base = (int64_t)blockIdx.x * LOOK_TILE;
#pragma unroll
  for (int i = 0; i < LOOK_ITEMS; ++i) {
    const int64_t j = base + i * TB + threadIdx.x;
    if (j < n) {
      const uint64_t cur = sorted[j];
      int32_t nxt = S;
      if (j + 1 < n) {
        const uint64_t r = sorted[j + 1];
        if ((uint32_t)(r >> 32) == (uint32_t)(cur >> 32))
          nxt = iter_of(lds_off, S, (int32_t)(r & 0xFFFFFFFFu));
      }
      next_iter[cur & 0xFFFFFFFFu] = nxt;
    }
  }
}

// heads[r] = (first iteration << 32 | node) for the r-th distinct node (ascending id)
__global__ __launch_bounds__(TB) void k_heads_write(const uint64_t* __restrict__ sorted, int64_t n,
                                                    const int64_t* __restrict__ off, int32_t S,
                                                    const uint32_t* __restrict__ head_bases,
                                                    uint64_t* __restrict__ heads) {
  extern __shared__ int32_t lds_off[];
  __shared__ uint32_t smem[TB / WAVE + 1];
  load_offsets(lds_off, off, S);
  const int64_t base = (int64_t)blockIdx.x * LOOK_TILE + (int64_t)threadIdx.x * LOOK_ITEMS;
  uint32_t flags = 0, cnt = 0;
#pragma unroll
  for (int i = 0; i < LOOK_ITEMS; ++i) {
    const int64_t j = base + i;
    if (j < n && run_head(sorted, j)) {
      flags |= 1u << i;
      ++cnt;
    }
  }
  uint32_t total;
  uint32_t at = head_bases[blockIdx.x] + block_exclusive_scan<uint32_t, TB>(cnt, smem, total);
#pragma unroll
  for (int i = 0; i < LOOK_ITEMS; ++i)
    if (flags >> i & 1) {
      const uint64_t cur = sorted[base + i];
      const uint32_t first = (uint32_t)iter_of(lds_off, S, (int32_t)(cur & 0xFFFFFFFFu));
      heads[at++] = ((uint64_t)first << 32) | (cur >> 32);
    }
}

// ---- part 2 -----------------------------------------------------------------------

__global__ __launch_bounds__(TB) void k_init_state(const uint64_t* __restrict__ heads,
                                                   int64_t count, int32_t* __restrict__ init_ids,
                                                   State st) {
  extern __shared__ uint32_t lds_hist[];  // S+1 bins
  for (int j = threadIdx.x; j <= st.S; j += TB) lds_hist[j] = 0;
  __syncthreads();
  const int64_t span = (int64_t)gridDim.x * TB;
  for (int64_t s = (int64_t)blockIdx.x * TB + threadIdx.x; s < count; s += span) {
    const uint64_t h = heads[s];
    const int32_t v = (int32_t)(h & 0xFFFFFFFFu);
    // Belady: the key of a prefetched row is its first access; LRU: it has not been used
    // yet, which is the oldest possible key
    const int32_t first = st.lru ? st.S : (int32_t)(h >> 32);
    init_ids[s] = v;
    st.res_id[s] = v;
    st.res_next[s] = first;
    st.addr[v] = (int32_t)s;
    atomicAdd(&lds_hist[first], 1u);
  }
  __syncthreads();
  for (int j = threadIdx.x; j <= st.S; j += TB)
    if (lds_hist[j]) atomicAdd(&st.rhist[j], lds_hist[j]);
}

// first_of[node] = first iteration that accesses the node (the array is preset to S, "never")
__global__ __launch_bounds__(TB) void k_scatter_first(const uint64_t* __restrict__ heads,
                                                      int64_t count,
                                                      int32_t* __restrict__ first_of) {
  const int64_t r = (int64_t)blockIdx.x * TB + threadIdx.x;
  if (r < count) first_of[heads[r] & 0xFFFFFFFFu] = (int32_t)(heads[r] >> 32);
}

// The state a superbatch starts from when the cache is carried over: line s holds
// start_ids[s], keyed by the row's first access in this superbatch.  A row that is never
// accessed is a dead resident from the start.  bad[0] counts ids outside [0, num_nodes) and
// ids that occur twice (both are skipped).
__global__ __launch_bounds__(TB) void k_init_state_resume(const int32_t* __restrict__ start_ids,
                                                          const int32_t* __restrict__ first_of,
                                                          State st,
                                                          unsigned long long* __restrict__ bad) {
  extern __shared__ uint32_t lds_hist[];  // S+1 bins
  for (int j = threadIdx.x; j <= st.S; j += TB) lds_hist[j] = 0;
  __syncthreads();
  const int64_t span = (int64_t)gridDim.x * TB;
  for (int64_t s = (int64_t)blockIdx.x * TB + threadIdx.x; s < st.cap; s += span) {
    const int32_t v = start_ids[s];
    if (v < 0 || v >= st.num_nodes || atomicCAS(&st.addr[v], -1, (int32_t)s) != -1) {
      atomicAdd(bad, 1ull);
      continue;
    }
    const int32_t first = first_of[v];
    st.res_id[s] = v;
    st.res_next[s] = first;
    atomicAdd(&lds_hist[first], 1u);
    if (first == st.S) atomicOr(&st.dead_bits[(uint32_t)v >> 5], 1u << ((uint32_t)v & 31));
  }
  __syncthreads();
  for (int j = threadIdx.x; j <= st.S; j += TB)
    if (lds_hist[j]) atomicAdd(&st.rhist[j], lds_hist[j]);
}

// addr[node of rank r] = r for the first `count` heads (C_0 when everything fits)
__global__ __launch_bounds__(TB) void k_scatter_rank(const uint64_t* __restrict__ heads,
                                                     int64_t count, int32_t* __restrict__ addr) {
  const int64_t r = (int64_t)blockIdx.x * TB + threadIdx.x;
  if (r < count) addr[heads[r] & 0xFFFFFFFFu] = (int32_t)r;
}

// src_line[p] = addr[ids[p]]: every accessed row is resident, nothing ever changes
__global__ __launch_bounds__(TB) void k_lookup_lines(const int32_t* __restrict__ ids, int64_t n,
                                                     const int32_t* __restrict__ addr,
                                                     int32_t* __restrict__ src_line) {
  constexpr int ITEMS = 4;
  const int64_t base = (int64_t)blockIdx.x * (TB * ITEMS) + threadIdx.x;
  int32_t v[ITEMS];
#pragma unroll
  for (int t = 0; t < ITEMS; ++t) {
    const int64_t p = base + t * TB;
    v[t] = ids[p < n ? p : 0];
  }
#pragma unroll
  for (int t = 0; t < ITEMS; ++t) v[t] = addr[v[t]];
#pragma unroll
  for (int t = 0; t < ITEMS; ++t) {
    const int64_t p = base + t * TB;
    if (p < n) src_line[p] = v[t];
  }
}

// miss_count[i] = |ids_i| (a cache without lines: every access misses)
__global__ __launch_bounds__(TB) void k_iteration_lengths(const int64_t* __restrict__ off, int32_t S,
                                                          int64_t* __restrict__ miss_count) {
  const int32_t i = blockIdx.x * TB + threadIdx.x;
  if (i < S) miss_count[i] = off[i + 1] - off[i];
}

__global__ __launch_bounds__(TB) void k_copy_init(const uint64_t* __restrict__ heads, int64_t count,
                                                  int32_t* __restrict__ init_ids) {
  const int64_t s = (int64_t)blockIdx.x * TB + threadIdx.x;
  if (s < count) init_ids[s] = (int32_t)(heads[s] & 0xFFFFFFFFu);
}

// ---- part 3 -----------------------------------------------------------------------
//
// One iteration of the recurrence is six dependent launches:
//   k_touch      hits get their new key, hits and misses are histogrammed by key, the line of
//                every access (or -1) is kept for the later phases and for the executor
//   k_threshold  one block: walks the histograms down from "never", fixes the threshold
//                bucket j*, what happens inside it and the size of the changeset; when the
//                evictions fall among the dead residents (the usual case of a large cache)
//                it also finds the id threshold T, from part counts of the standing dead-row
//                bitmap that are kept up to date wherever a bit changes
//   k_mark       otherwise: the members of the selected class of bucket j* set their bit in a
//                scratch bitmap over node ids and count themselves per part
//   k_find       one block: T = the keep-th set bit, from the part counts
//   k_flags      eviction flags per cache line (dead residents of a large cache: the bits above
//                T of their bitmap are turned into line flags through the address table
//                instead) and insertion counts per tile of accesses; the scratch bitmap is
//                cleared by the members that set it
//   k_emit_pair  both lists in their order (every block sums the tile counts in front of it:
//                no scan launch), and the cache state of C_{i+1}: the t-th insertion takes
//                the line of the t-th eviction, the two sides meeting in one 64-bit word per
//                t that the second to arrive completes
// A carried cache that has room for every row of the superbatch never needs k_mark and k_find
// (all evictions fall among the dead rows): its iterations are four launches.
// No phase makes a pass over a whole bitmap or scans all tiles in one block: the cost of an
// iteration follows its accesses and, unless the dead-row path applies, the cache lines.
// Measured and dropped earlier: a single cooperative kernel with grid.sync() between the
// phases (about 0.1 ms per barrier on 1024 blocks), and running the single-block phases in
// the last block to finish of the launch before them with a device-wide fence per block
// (writes back and invalidates L2 on this multi-XCD part: three to four times slower).

// ready[i] = number of prefetched rows whose first access lies in iterations 0..i: the
// prefix of C_0 (it is ordered by first access) that iteration i can touch.
__global__ __launch_bounds__(TB) void k_init_ready(const uint64_t* __restrict__ heads,
                                                   int64_t n_init, int32_t S,
                                                   int64_t* __restrict__ ready) {
  const int32_t i = blockIdx.x * TB + threadIdx.x;
  if (i >= S) return;
  int64_t lo = 0, hi = n_init;   // first rank whose first access is later than i
  while (lo < hi) {
    const int64_t mid = (lo + hi) >> 1;
    if ((int32_t)(heads[mid] >> 32) <= i) lo = mid + 1; else hi = mid;
  }
  ready[i] = lo;
}

struct Iter {           // what a phase needs to know about the running iteration
  const int32_t* ids;   // ids_i
  const int32_t* next;  // next accessed iteration of each access of ids_i (Belady keys)
  int64_t n;            // |ids_i|
  int32_t i;
  int32_t key;          // >= 0: every access of the iteration takes this key (LRU: S-1-i,
                        // smaller = used more recently); < 0: the key is next[p]
  int32_t lo_bin;       // smallest bucket a candidate of this iteration can fall into
  int32_t* src_line;    // out (may be null): cache line of each access in C_i, -1 for a miss
};

__device__ __forceinline__ int32_t key_of(const Iter& it, int64_t p) {
  return it.key >= 0 ? it.key : it.next[p];
}

struct Outputs {
  int32_t* in_ids;
  int32_t* out_ids;
  int32_t* in_positions;
  int64_t cs_capacity;
  int64_t* cs_offsets;
  int64_t* miss_count;
};

__device__ __forceinline__ uint32_t block_sum_u32(uint32_t v, uint32_t* red) {
  v = wave_reduce_sum(v);
  __syncthreads();  // red may still be read from an earlier call
  if (lane_id() == 0) red[threadIdx.x / WAVE] = v;
  __syncthreads();
  uint32_t s = 0;
  for (int w = 0; w < (int)blockDim.x / WAVE; ++w) s += red[w];
  return s;
}

__device__ __forceinline__ void dead_bit_set(const State& st, uint32_t v) {
  atomicOr(&st.dead_bits[v >> 5], 1u << (v & 31));
  atomicAdd(&st.dead_part[v >> PART_SHIFT], 1u);
}

// Refresh the keys of the hits, histogram hits and misses by key, keep every access's line.
// lds: 2*(S+1) counters.  One block covers TB*TOUCH_ITEMS accesses.
__global__ __launch_bounds__(TB) void k_touch(State st, Iter it, unsigned long long* miss_out) {
  extern __shared__ uint32_t lds[];
  __shared__ uint32_t red[TB / WAVE];
  uint32_t* hr = lds;
  uint32_t* hi = lds + st.S + 1;
  for (int j = threadIdx.x; j < 2 * (st.S + 1); j += TB) lds[j] = 0;
  __syncthreads();
  uint32_t misses = 0;
  const int64_t base = (int64_t)blockIdx.x * (TB * TOUCH_ITEMS);
  // id, then address-table entry, then the line's state: the reads of one level are issued
  // for all items before any is used, so that they are in flight together.  An item beyond
  // the end repeats the block's first item (in range) and is skipped when it is processed.
  int32_t v[TOUCH_ITEMS], line[TOUCH_ITEMS], nx[TOUCH_ITEMS];
#pragma unroll
  for (int t = 0; t < TOUCH_ITEMS; ++t) {
    int64_t p = base + t * TB + threadIdx.x;
    p = p < it.n ? p : base;
    v[t] = it.ids[p];
    nx[t] = key_of(it, p);
  }
#pragma unroll
  for (int t = 0; t < TOUCH_ITEMS; ++t) line[t] = st.addr[v[t]];
#pragma unroll
  for (int t = 0; t < TOUCH_ITEMS; ++t) {
    const int64_t p = base + t * TB + threadIdx.x;
    if (p < it.n) {
      st.acc_line[p] = line[t];
      if (it.src_line) it.src_line[p] = line[t];   // the state is C_i here
    }
  }
  int32_t old_key[TOUCH_ITEMS];
  if (st.lru) {
#pragma unroll
    for (int t = 0; t < TOUCH_ITEMS; ++t) old_key[t] = line[t] >= 0 ? st.res_next[line[t]] : 0;
  }
#pragma unroll
  for (int t = 0; t < TOUCH_ITEMS; ++t) {
    if (base + t * TB + threadIdx.x >= it.n) continue;
    if (line[t] >= 0) {
      // An LRU hit leaves a bucket that is still walked (an older one): take it out of
      // the count there; counters wrap, the flush below adds them modulo 2^32.  A Belady
      // hit leaves bucket i, which no later iteration looks at.
      if (st.lru) atomicSub(&hr[old_key[t]], 1u);
      st.res_next[line[t]] = nx[t];
      atomicAdd(&hr[nx[t]], 1u);
      // the row's last access: a dead resident from now on
      if (nx[t] == st.S && !st.lru) dead_bit_set(st, (uint32_t)v[t]);
    } else {
      atomicAdd(&hi[nx[t]], 1u);
      ++misses;
    }
  }
  const uint32_t total = block_sum_u32(misses, red);
  for (int j = it.lo_bin + threadIdx.x; j <= st.S; j += TB) {
    if (hr[j]) atomicAdd(&st.rhist[j], hr[j]);
    if (hi[j]) atomicAdd(&st.ihist[j], hi[j]);
  }
  if (threadIdx.x == 0 && total) atomicAdd(miss_out, (unsigned long long)total);
}

// One block of NT threads.  Walks the buckets from "never" downwards until as many
// candidates as there were misses are dropped; fixes the threshold bucket, what happens
// inside it, the size of the changeset, and rolls the resident histogram forward to C_{i+1}.
template <int NT>
__device__ void p_threshold(const State& st, int32_t i, int32_t lo_bin, const int64_t* miss_count,
                            int64_t* cs_offsets) {
  __shared__ int64_t smem[NT / WAVE + 1];
  __shared__ int32_t s_jstar;
  __shared__ uint32_t s_kept;
  const int32_t S = st.S;
  const int64_t n_drop = miss_count[i];
  const int32_t bins = S - lo_bin + 1;            // buckets lo_bin .. S, walked as r = S - j
  const int32_t per = (bins + NT - 1) / NT;
  const int32_t r0 = threadIdx.x * per;
  int64_t mine = 0;
  for (int32_t r = r0; r < r0 + per && r < bins; ++r)
    mine += (int64_t)st.rhist[S - r] + st.ihist[S - r];
  int64_t total;
  int64_t before = block_exclusive_scan<int64_t, NT>(mine, smem, total);
  if (threadIdx.x == 0) {
    // default: nothing is dropped (no misses); overwritten below by the thread that
    // finds the threshold bucket
    s_jstar = S + 1;
    s_kept = 0;
    Ctrl c{};
    c.jstar = S + 1;
    c.mode_in = MODE_ALL;
    c.mode_res = MODE_ALL;
    c.T = -1;
    *st.ctrl = c;
    cs_offsets[i + 1] = cs_offsets[i];
  }
  __syncthreads();
  if (n_drop > 0) {
    for (int32_t r = r0; r < r0 + per && r < bins; ++r) {
      const int32_t j = S - r;
      const int64_t R = st.rhist[j], I = st.ihist[j];
      if (before <= n_drop && before + R + I > n_drop) {
        const int64_t rem = n_drop - before;  // still to drop, all from bucket j
        Ctrl c{};
        c.jstar = j;
        int64_t from_res = 0;
        if (rem == 0) {
          c.mode_in = MODE_ALL; c.mode_res = MODE_ALL;
        } else if (rem < I) {
          c.mode_in = MODE_SELECT; c.mode_res = MODE_ALL; c.keep = (int32_t)(I - rem);
        } else if (rem == I) {
          c.mode_in = MODE_NONE; c.mode_res = MODE_ALL;
        } else {
          c.mode_in = MODE_NONE; c.mode_res = MODE_SELECT;
          from_res = rem - I;
          c.keep = (int32_t)(R - from_res);
          // in the "never" bucket the members are exactly the dead residents, whose
          // bitmap is maintained incrementally: no marking pass is needed
          c.use_dead = j == S && !st.lru;
        }
        c.T = -1;
        // evictions inside j*; those of the buckets above j* are added after the barrier
        s_jstar = j;
        s_kept = (uint32_t)(R + I - rem);
        c.n_change = (int32_t)from_res;
        *st.ctrl = c;
      }
      before += R + I;
    }
  }
  __syncthreads();
  const int32_t jstar = s_jstar;
  // residents evicted from the buckets above j*, and the histogram of C_{i+1}
  int64_t above = 0;
  for (int32_t r = r0; r < r0 + per && r < bins; ++r) {
    const int32_t j = S - r;
    if (j > jstar) {
      above += st.rhist[j];
      st.rhist[j] = 0;
    } else if (j == jstar) {
      st.rhist[j] = s_kept;
    } else {
      st.rhist[j] += st.ihist[j];
    }
    st.ihist[j] = 0;
  }
  int64_t above_total;
  block_exclusive_scan<int64_t, NT>(above, smem, above_total);
  if (threadIdx.x == 0 && n_drop > 0) {
    st.ctrl->n_change += (int32_t)above_total;
    cs_offsets[i + 1] = cs_offsets[i] + st.ctrl->n_change;
  }
  __syncthreads();
}

// One block of NT threads: the position of the keep-th set bit (1-based, from the bottom) of
// `bits`, found through `part` (set bits per PART_WORDS words); -1 if there are fewer set bits.
// Every thread gets the result.  With `trim`, the part counts are rewritten to what remains
// once every bit above that position is cleared.
template <int NT>
__device__ int32_t p_kth_set_bit(const uint32_t* __restrict__ bits, uint32_t* __restrict__ part,
                                 int64_t parts, int64_t words, int64_t keep, bool trim) {
  __shared__ int64_t smem[NT / WAVE + 1];
  __shared__ int64_t s_part, s_before;
  __shared__ int32_t s_found;
  // 1. the part that holds the keep-th set bit
  const int64_t per = (parts + NT - 1) / NT;
  const int64_t q0 = threadIdx.x * per;
  int64_t mine = 0;
  for (int64_t q = q0; q < q0 + per && q < parts; ++q) mine += part[q];
  int64_t total;
  int64_t before = block_exclusive_scan<int64_t, NT>(mine, smem, total);
  if (threadIdx.x == 0) {
    s_part = -1;
    s_found = -1;
  }
  __syncthreads();
  for (int64_t q = q0; q < q0 + per && q < parts; ++q) {
    const int64_t cnt = part[q];
    if (before < keep && before + cnt >= keep) {
      s_part = q;
      s_before = before;
    }
    before += cnt;
  }
  __syncthreads();
  if (s_part < 0) return -1;  // fewer set bits than asked for (uniform over the block)
  if (trim) {
    for (int64_t q = q0; q < q0 + per && q < parts; ++q)
      if (q > s_part) part[q] = 0;
      else if (q == s_part) part[q] = (uint32_t)(keep - s_before);
  }
  // 2. the word inside that part, then the bit inside the word
  constexpr int WPT = PART_WORDS / NT;
  const int64_t w0 = s_part * PART_WORDS + (int64_t)threadIdx.x * WPT;
  int64_t cntw = 0;
  for (int t = 0; t < WPT; ++t)
    if (w0 + t < words) cntw += __popc(bits[w0 + t]);
  int64_t tot2;
  int64_t bw = s_before + block_exclusive_scan<int64_t, NT>(cntw, smem, tot2);
  for (int t = 0; t < WPT; ++t)
    if (w0 + t < words) {
      uint32_t word = bits[w0 + t];
      const int pc = __popc(word);
      if (bw < keep && bw + pc >= keep) {
        int need = (int)(keep - bw);  // the need-th set bit of this word, 1-based
        int bit = 0;
        while (true) {
          bit = __ffs(word) - 1;
          if (--need == 0) break;
          word &= word - 1;
        }
        s_found = (int32_t)((w0 + t) * 32 + bit);
      }
      bw += pc;
    }
  __syncthreads();
  return s_found;
}

// T of the running iteration = the id whose bit is the keep-th set bit of `bits`.
template <int NT>
__device__ void p_bits_find(const State& st, const uint32_t* __restrict__ bits,
                            uint32_t* __restrict__ part, bool trim) {
  Ctrl* c = st.ctrl;
  const int32_t T = p_kth_set_bit<NT>(bits, part, st.parts, st.words, c->keep, trim);
  if (threadIdx.x == 0 && T >= 0) c->T = T;   // fewer set bits than asked for cannot happen: T stays -1
  __syncthreads();
}

__global__ __launch_bounds__(BIG) void k_threshold(State st, int32_t i, int32_t lo_bin, Outputs o,
                                                   int64_t evict_tiles) {
  p_threshold<BIG>(st, i, lo_bin, o.miss_count, o.cs_offsets);
  Ctrl c = *st.ctrl;   // written by this block, in front of the barrier that ends p_threshold
  // k_mark will set the bits of the selected class only
  c.marked = (c.mode_res == MODE_SELECT && !c.use_dead ? MARKED_RES : 0) |
             (c.mode_in == MODE_SELECT ? MARKED_IN : 0);
  if (threadIdx.x == 0) st.ctrl->marked = c.marked;
  if (st.dead_only && !c.use_dead && threadIdx.x == 0 &&
      (c.mode_res == MODE_SELECT || c.mode_in == MODE_SELECT))
    *st.fault = 1;
  if (c.use_dead) {
    p_bits_find<BIG>(st, st.dead_bits, st.dead_part, true);
    if (st.dead_scatter)     // the scatter counts evictions per tile with atomics
      for (int64_t q = threadIdx.x; q < evict_tiles; q += BIG) st.evict_tiles[q] = 0;
  }
}

__global__ __launch_bounds__(BIG) void k_find(State st) {
  const Ctrl c = *st.ctrl;
  if (c.use_dead || (c.mode_res != MODE_SELECT && c.mode_in != MODE_SELECT)) return;
  if (c.mode_res == MODE_SELECT) p_bits_find<BIG>(st, st.bitmap, st.sel_part, false);
  else p_bits_find<BIG>(st, st.bitmap_in, st.sel_part_in, false);
}

constexpr int MARK_ITEMS = 8;   // lines / accesses per thread in the mark phases

// ---- Belady: what an iteration decides without looking at the cache ---------------------------
//
// The candidates of iteration i per next-use bucket are the residents that the iteration does
// not access (a histogram R_i that rolls forward by the rule of p_threshold) plus the
// iteration's accesses by their new key (a histogram H_i of next_iter alone), and the number
// to drop is the iteration's length minus R_i[i], the residents keyed to it.  So the threshold
// bucket j* of every iteration, the number of rows to drop from it, and R_{i+1} follow from S
// histograms in front of the loop.  What depends on the cache is which accesses are hits: the
// split of bucket j* into residents and incoming rows (it decides the class the id select runs
// on) and the size of the changeset.  The touch phase counts those and marks the members of
// bucket j* of both classes on the way, so that the loop needs neither the threshold launch
// over histograms of the state nor a marking launch.
constexpr int STATIC_S_MAX = 2048;      // iterations up to which the S x (S + 1) histograms are kept
constexpr int64_t TOUCH_FEW = 400000;   // accesses of an iteration below which a thread of k_touch_static takes four

struct StaticIter {      // per iteration, written by k_static_roll
  int32_t jstar;         // threshold bucket, S + 1: nothing is dropped
  int32_t rem;           // rows to drop from bucket j*
  int32_t res_idle;      // residents of bucket j* that the iteration does not access
  int32_t acc_jstar;     // accesses of the iteration whose new key is j*
  int32_t res_above;     // residents above j* that the iteration does not access
  int32_t pad;
};

// H[i][k] = accesses of iteration i whose next accessed iteration is k.  blockIdx.y = iteration.
__global__ __launch_bounds__(TB) void k_key_hists(const int32_t* __restrict__ next_iter,
                                                  const int64_t* __restrict__ off, int32_t S,
                                                  uint32_t* __restrict__ hists) {
  extern __shared__ uint32_t lds_h[];   // S + 1 bins
  const int32_t i = blockIdx.y;
  const int64_t lo = off[i], n = off[i + 1] - lo;
  const int64_t base = (int64_t)blockIdx.x * (TB * TOUCH_ITEMS);
  if (base >= n) return;                // uniform
  for (int j = threadIdx.x; j <= S; j += TB) lds_h[j] = 0;
  __syncthreads();
#pragma unroll
  for (int t = 0; t < TOUCH_ITEMS; ++t) {
    const int64_t p = base + t * TB + threadIdx.x;
    if (p < n) atomicAdd(&lds_h[next_iter[lo + p]], 1u);
  }
  __syncthreads();
  for (int j = i + 1 + threadIdx.x; j <= S; j += TB)
    if (lds_h[j]) atomicAdd(&hists[(int64_t)i * (S + 1) + j], lds_h[j]);
}

// One block: the thresholds of all iterations, one after the other.  rhist holds R_0 (the
// residents of the start state by key).  Bins are walked as r = S - j, `per` consecutive r to a
// thread; a bin's word packs (idle residents << 32 | candidates).
__global__ __launch_bounds__(BIG) void k_static_roll(State st, const uint32_t* __restrict__ hists,
                                                     const int64_t* __restrict__ off,
                                                     StaticIter* __restrict__ plan,
                                                     int64_t* __restrict__ miss_count) {
  __shared__ uint32_t s_res[STATIC_S_MAX + 1];
  __shared__ uint64_t slots[BIG / WAVE];
  __shared__ int32_t s_jstar, s_rem;
  const int32_t S = st.S;
  const int per = (S + 1 + BIG - 1) / BIG;            // at most 3
  const int r0 = threadIdx.x * per;
  for (int j = threadIdx.x; j <= S; j += BIG) s_res[j] = st.rhist[j];
  // the histogram values and the length of an iteration are requested an iteration ahead
  uint32_t ahead[3] = {0, 0, 0};
  for (int t = 0; t < per; ++t) {
    const int j = S - (r0 + t);
    if (j > 0) ahead[t] = hists[j];
  }
  int64_t n_ahead = off[1] - off[0];
  __syncthreads();
  for (int32_t i = 0; i < S; ++i) {
    const int64_t n = n_ahead;
    const int64_t drop = n - (int64_t)s_res[i];       // the misses: the cache is full
    uint64_t word[3];
    uint64_t mine = 0;
    for (int t = 0; t < per; ++t) {
      const int j = S - (r0 + t);
      word[t] = 0;
      if (j > i) {                                     // (no candidate has a key up to i)
        const uint64_t idle = s_res[j];
        word[t] = (idle << 32) | (idle + ahead[t]);
      }
      mine += word[t];
    }
    if (i + 1 < S) {
      for (int t = 0; t < per; ++t) {
        const int j = S - (r0 + t);
        ahead[t] = j > i + 1 ? hists[(int64_t)(i + 1) * (S + 1) + j] : 0u;
      }
      n_ahead = off[i + 2] - off[i + 1];
    }
    if (threadIdx.x == 0) {
      s_jstar = S + 1;
      s_rem = 0;
      miss_count[i] = drop;
    }
    // exclusive prefix over the threads with one barrier (see block_prefix_one_barrier)
    const uint64_t inc = wave_inclusive_scan(mine);
    if (lane_id() == WAVE - 1) slots[threadIdx.x / WAVE] = inc;
    __syncthreads();
    uint64_t before = inc - mine;
    for (int q = 0; q < (int)(threadIdx.x / WAVE); ++q) before += slots[q];
    StaticIter me{};
    bool found = false;
    if (drop > 0)
      for (int t = 0; t < per; ++t) {
        const int j = S - (r0 + t);
        const int64_t cum = (int64_t)(before & 0xFFFFFFFFull), c = (int64_t)(word[t] & 0xFFFFFFFFull);
        if (j > i && cum <= drop && cum + c > drop) {
          me.jstar = j;
          me.rem = (int32_t)(drop - cum);
          me.res_idle = (int32_t)(word[t] >> 32);
          me.acc_jstar = (int32_t)(c - (int64_t)(word[t] >> 32));
          me.res_above = (int32_t)(before >> 32);
          found = true;
        }
        before += word[t];
      }
    if (found) {
      plan[i] = me;
      s_jstar = me.jstar;
      s_rem = me.rem;
    }
    __syncthreads();
    const int32_t jstar = s_jstar, rem = s_rem;
    if (threadIdx.x == 0 && jstar > S) {
      StaticIter none{};
      none.jstar = S + 1;
      plan[i] = none;
    }
    // R_{i+1}: everything below j* stays, bucket j* loses rem, everything above goes
    for (int t = 0; t < per; ++t) {
      const int j = S - (r0 + t);
      if (j < 0) continue;
      const uint32_t c = (uint32_t)(word[t] & 0xFFFFFFFFull);
      s_res[j] = j <= i ? 0u : j < jstar ? c : j == jstar ? c - (uint32_t)rem : 0u;
    }
    __syncthreads();
  }
}

// k_touch with the threshold bucket known (ITEMS accesses per thread: four while an iteration is
// bound by the latency of its chain, eight once it is bound by its scattered accesses): no histograms; hits keyed to or above j* are
// counted (ctr[0], ctr[1]), and the members of bucket j* mark themselves, refreshed residents
// in the residents' scratch bitmap, misses in the incoming rows'.  The blocks from
// touch_blocks on walk the cache lines and mark the residents of bucket j* that the iteration
// does not access (a line that a touch block refreshes to j* meanwhile may be marked by both:
// the part count goes to whoever sets the bit).
__device__ __forceinline__ void mark_once(uint32_t* bits, uint32_t* part, uint32_t v) {
  const uint32_t bit = 1u << (v & 31);
  if (!(atomicOr(&bits[v >> 5], bit) & bit)) atomicAdd(&part[v >> PART_SHIFT], 1u);
}

template <int ITEMS>
__global__ __launch_bounds__(TB) void k_touch_static(State st, Iter it,
                                                     const StaticIter* __restrict__ plan,
                                                     uint32_t* __restrict__ ctr,
                                                     int64_t touch_blocks) {
  __shared__ uint32_t red[TB / WAVE];
  const StaticIter si = plan[it.i];
  const int32_t jstar = si.jstar;
  const bool mark_res = jstar < st.S;     // (bucket "never": the standing dead-row bitmap serves)
  if ((int64_t)blockIdx.x >= touch_blocks) {
    if (!mark_res || si.res_idle == 0) return;
    const int64_t base = ((int64_t)blockIdx.x - touch_blocks) * (TB * MARK_ITEMS);
#pragma unroll
    for (int t = 0; t < MARK_ITEMS; ++t) {
      const int64_t l = base + t * TB + threadIdx.x;
      if (l < st.cap && st.res_next[l] == jstar)
        mark_once(st.bitmap, st.sel_part, (uint32_t)st.res_id[l]);
    }
    return;
  }
  const int64_t base = (int64_t)blockIdx.x * (TB * ITEMS);
  int32_t v[ITEMS], line[ITEMS], nx[ITEMS];
#pragma unroll
  for (int t = 0; t < ITEMS; ++t) {
    int64_t p = base + t * TB + threadIdx.x;
    p = p < it.n ? p : base;
    v[t] = it.ids[p];
    nx[t] = it.next[p];
  }
#pragma unroll
  for (int t = 0; t < ITEMS; ++t) line[t] = st.addr[v[t]];
  uint32_t at_jstar = 0, above = 0;
#pragma unroll
  for (int t = 0; t < ITEMS; ++t) {
    const int64_t p = base + t * TB + threadIdx.x;
    if (p >= it.n) continue;
    st.acc_line[p] = line[t];
    if (it.src_line) it.src_line[p] = line[t];   // the state is C_i here
    if (line[t] >= 0) {
      st.res_next[line[t]] = nx[t];
      if (nx[t] == st.S) dead_bit_set(st, (uint32_t)v[t]);   // the row's last access
      if (nx[t] == jstar) {
        ++at_jstar;
        if (mark_res) mark_once(st.bitmap, st.sel_part, (uint32_t)v[t]);
      } else if (nx[t] > jstar) {
        ++above;
      }
    } else if (nx[t] == jstar) {
      mark_once(st.bitmap_in, st.sel_part_in, (uint32_t)v[t]);
    }
  }
  // (a block has at most TB * ITEMS accesses: the two counts share a word)
  const uint32_t both = block_sum_u32((at_jstar << 16) | above, red);
  if (threadIdx.x == 0) {
    if (both >> 16) atomicAdd(&ctr[0], both >> 16);
    if (both & 0xFFFFu) atomicAdd(&ctr[1], both & 0xFFFFu);
  }
}

// One block: the rest of the iteration's decision (what p_threshold decides inside bucket j*),
// the size of the changeset, and the id select.
__global__ __launch_bounds__(BIG) void k_decide(State st, int32_t i,
                                                const StaticIter* __restrict__ plan,
                                                uint32_t* __restrict__ ctr, Outputs o,
                                                int64_t evict_tiles) {
  const StaticIter si = plan[i];
  const int64_t hits_at = ctr[0], hits_above = ctr[1];
  __syncthreads();                       // every thread has read the counters
  if (threadIdx.x == 0) {
    ctr[0] = 0;
    ctr[1] = 0;
    Ctrl c{};
    c.jstar = si.jstar;
    c.mode_in = MODE_ALL;
    c.mode_res = MODE_ALL;
    c.T = -1;
    int64_t from_res = 0;
    if (si.jstar <= st.S) {
      const int64_t R = (int64_t)si.res_idle + hits_at, I = (int64_t)si.acc_jstar - hits_at;
      const int64_t rem = si.rem;
      if (rem == 0) {
      } else if (rem < I) {
        c.mode_in = MODE_SELECT; c.keep = (int32_t)(I - rem);
      } else if (rem == I) {
        c.mode_in = MODE_NONE;
      } else {
        c.mode_in = MODE_NONE; c.mode_res = MODE_SELECT;
        from_res = rem - I;
        c.keep = (int32_t)(R - from_res);
        c.use_dead = si.jstar == st.S;
      }
      c.n_change = (int32_t)((int64_t)si.res_above + hits_above + from_res);
      c.marked = (si.jstar < st.S && R > 0 ? MARKED_RES : 0) | (I > 0 ? MARKED_IN : 0);
    }
    *st.ctrl = c;
    o.cs_offsets[i + 1] = o.cs_offsets[i] + c.n_change;
  }
  __syncthreads();
  const Ctrl c = *st.ctrl;
  if (c.mode_res == MODE_SELECT) {
    if (c.use_dead) {
      p_bits_find<BIG>(st, st.dead_bits, st.dead_part, true);
      if (st.dead_scatter)
        for (int64_t q = threadIdx.x; q < evict_tiles; q += BIG) st.evict_tiles[q] = 0;
    } else {
      p_bits_find<BIG>(st, st.bitmap, st.sel_part, false);
    }
  } else if (c.mode_in == MODE_SELECT) {
    p_bits_find<BIG>(st, st.bitmap_in, st.sel_part_in, false);
  }
}

constexpr int EVICT_TILE = WAVE * WAVE;   // cache lines per tile: 64 flag words of 64 lines

// The members of a class are distinct ids and the bitmap is all zero before the marking, so
// every call sets a new bit: neither atomic needs its result.
__device__ __forceinline__ void select_bit_set(const State& st, uint32_t v) {
  atomicOr(&st.bitmap[v >> 5], 1u << (v & 31));
  atomicAdd(&st.sel_part[v >> PART_SHIFT], 1u);
}
__device__ __forceinline__ void select_bit_set_in(const State& st, uint32_t v) {
  atomicOr(&st.bitmap_in[v >> 5], 1u << (v & 31));
  atomicAdd(&st.sel_part_in[v >> PART_SHIFT], 1u);
}

// Set the bit of every member of the selected class in bucket j*.
__device__ void p_mark_residents(const State& st, const Ctrl& c, int64_t vb) {
  const int64_t base = vb * (TB * MARK_ITEMS);
#pragma unroll
  for (int t = 0; t < MARK_ITEMS; ++t) {
    const int64_t s = base + t * TB + threadIdx.x;
    if (s < st.cap && st.res_next[s] == c.jstar) select_bit_set(st, (uint32_t)st.res_id[s]);
  }
}

__device__ void p_mark_incoming(const State& st, const Ctrl& c, const Iter& it, int64_t vb) {
  const int64_t base = vb * (TB * MARK_ITEMS);
#pragma unroll
  for (int t = 0; t < MARK_ITEMS; ++t) {
    const int64_t p = base + t * TB + threadIdx.x;
    if (p < it.n && st.acc_line[p] < 0 && key_of(it, p) == c.jstar)
      select_bit_set_in(st, (uint32_t)it.ids[p]);
  }
}

// Large caches, evictions among the dead residents only (the usual case once a cache is
// full): the evicted rows are the set bits above T of the standing dead-row bitmap, a short
// stretch at its upper end, so they are found from there and their lines flagged through
// the address table, instead of reading the key and id of every cache line.  The flag
// words are all zero when the phase starts (the emit phase clears what it consumes), the
// tile counts were zeroed by k_threshold; the bits above T leave the bitmap here.
__device__ void p_dead_scatter(const State& st, const Ctrl& c, int64_t vb, int64_t vblocks) {
  // the stretch above T is short as a rule, so a small grid strides over it from T's word on
  const int64_t t_word = c.T < 0 ? 0 : c.T >> 5;   // T = -1: every dead row goes
  for (int64_t w = t_word + vb * TB + threadIdx.x; w < st.words; w += vblocks * TB) {
    const uint32_t all = st.dead_bits[w];
    uint32_t bits = all;
    if (c.T >= 0 && w == t_word) bits &= (c.T & 31) == 31 ? 0u : ~((2u << (c.T & 31)) - 1u);
    if (!bits) continue;
    st.dead_bits[w] = all & ~bits;
    while (bits) {
      const int32_t v = (int32_t)(w * 32 + (__ffs(bits) - 1));
      bits &= bits - 1;
      const int32_t line = st.addr[v];   // a dead row is resident, so this is its line
      if (line >= 0) {
        atomicOr((unsigned long long*)&st.evict_words[line >> 6], 1ull << (line & 63));
        atomicAdd(&st.evict_tiles[line / EVICT_TILE], 1u);
      }
    }
  }
}

// blocks [0, res_blocks): residents, the next in_blocks blocks: incoming rows; only one
// class is selected, and none when the select runs on the dead rows.
__global__ __launch_bounds__(TB) void k_mark(State st, Iter it, int64_t res_blocks) {
  const Ctrl c = *st.ctrl;
  if (c.use_dead) return;
  if ((int64_t)blockIdx.x < res_blocks) {
    if (c.mode_res == MODE_SELECT) p_mark_residents(st, c, blockIdx.x);
  } else if (c.mode_in == MODE_SELECT) {
    p_mark_incoming(st, c, it, blockIdx.x - res_blocks);
  }
}

__device__ __forceinline__ bool evicts(const Ctrl& c, int32_t next, int32_t id) {
  return next > c.jstar || (next == c.jstar && c.mode_res == MODE_SELECT && id > c.T);
}

__device__ __forceinline__ bool inserts(const Ctrl& c, int32_t next, int32_t id) {
  return next < c.jstar ||
         (next == c.jstar && (c.mode_in == MODE_ALL || (c.mode_in == MODE_SELECT && id <= c.T)));
}

// Eviction flags of one tile of cache lines.  A wave reads 64 consecutive lines at a time
// (coalesced) and its ballot is a 64-bit flag word; the four waves of the block share the
// tile's 64 words.  The tile's total goes to evict_tiles.  Residents that marked themselves
// for the select take their word of the scratch bitmap back to zero.
__device__ void p_evict_flags(const State& st, const Ctrl& c, int64_t vb) {
  __shared__ uint32_t red[TB / WAVE];
  constexpr int PER_WAVE = WAVE / (TB / WAVE);
  const int64_t first_word = vb * WAVE + (threadIdx.x / WAVE) * PER_WAVE;
  const bool unmark = c.marked & MARKED_RES;
  // all keys of the wave's 16 x 64 lines first, so that the loads are in flight together;
  // a line beyond the end repeats line 0 and is masked out below
  int32_t next[PER_WAVE];
#pragma unroll
  for (int g = 0; g < PER_WAVE; ++g) {
    const int64_t line = (first_word + g) * WAVE + lane_id();
    next[g] = st.res_next[line < st.cap ? line : 0];
  }
  uint32_t cnt = 0;
#pragma unroll
  for (int g = 0; g < PER_WAVE; ++g) {
    const int64_t line = (first_word + g) * WAVE + lane_id();
    bool out = false;
    if (line < st.cap && next[g] >= c.jstar) {   // the common case needs no look at the node id
      const int32_t id = st.res_id[line];
      out = evicts(c, next[g], id);
      if (unmark && next[g] == c.jstar) st.bitmap[(uint32_t)id >> 5] = 0;
    }
    const uint64_t word = __ballot(out);
    if ((first_word + g) * WAVE < st.cap && lane_id() == 0) {
      st.evict_words[first_word + g] = word;
      cnt += __popcll(word);
    }
  }
  const uint32_t total = block_sum_u32(cnt, red);
  if (threadIdx.x == 0) st.evict_tiles[vb] = total;
}

constexpr int IN_ITEMS = 8;        // accesses per thread in the insertion phases ...
constexpr int IN_ITEMS_MANY = 4;   // ... of an iteration with TOUCH_FEW accesses or more (smaller tiles
                                   // rank and place faster once the phases are bound by their accesses)

// Insertions per tile of TB*IN_ITEMS accesses; incoming rows that marked themselves for the
// select take their word of the scratch bitmap back to zero.
template <int IN_ITEMS>
__device__ void p_in_count(const State& st, const Ctrl& c, const Iter& it, int64_t vb) {
  __shared__ uint32_t red[TB / WAVE];
  const int64_t base = (vb * TB + threadIdx.x) * IN_ITEMS;
  const bool unmark = c.marked & MARKED_IN;
  // line, key and id of all items first (an item beyond the end repeats item 0 of the
  // iteration and is not counted)
  int32_t line[IN_ITEMS], key[IN_ITEMS], v[IN_ITEMS];
#pragma unroll
  for (int t = 0; t < IN_ITEMS; ++t) {
    const int64_t p = base + t < it.n ? base + t : 0;
    line[t] = st.acc_line[p];
    key[t] = key_of(it, p);
    v[t] = it.ids[p];
  }
  uint32_t cnt = 0;
#pragma unroll
  for (int t = 0; t < IN_ITEMS; ++t)
    if (base + t < it.n && line[t] < 0 && key[t] <= c.jstar) {
      cnt += inserts(c, key[t], v[t]);
      if (unmark && key[t] == c.jstar) st.bitmap_in[(uint32_t)v[t] >> 5] = 0;
    }
  const uint32_t total = block_sum_u32(cnt, red);
  if (threadIdx.x == 0) st.in_tiles[vb] = total;
}

// blocks [0, evict_tiles): eviction flags and counts per tile, by a pass over the tile's lines
// or, dead rows of a large cache, by the scatter from the bitmap (the blocks then stride over
// the stretch above T); the next in_tiles blocks: insertions per tile; one more block takes
// the part counts of the scratch bitmap back to zero.
template <int IN_ITEMS>
__global__ __launch_bounds__(TB) void k_flags(State st, Iter it, int64_t evict_tiles,
                                              int64_t in_tiles) {
  const Ctrl c = *st.ctrl;
  const int64_t vb = blockIdx.x;
  if (vb < evict_tiles) {
    if (st.dead_scatter && c.use_dead) {
      if (c.n_change > 0) p_dead_scatter(st, c, vb, evict_tiles);
    } else if (c.n_change > 0 || (c.marked & MARKED_RES)) {
      p_evict_flags(st, c, vb);
    }
  } else if (vb < evict_tiles + in_tiles) {
    if (c.n_change > 0 || (c.marked & MARKED_IN)) p_in_count<IN_ITEMS>(st, c, it, vb - evict_tiles);
  } else {
    if (c.marked & MARKED_RES)
      for (int64_t q = threadIdx.x; q < st.parts; q += TB) st.sel_part[q] = 0;
    if (c.marked & MARKED_IN)
      for (int64_t q = threadIdx.x; q < st.parts; q += TB) st.sel_part_in[q] = 0;
  }
}

// ---- the last phase: lists and the state of C_{i+1} ----------------------------------------
//
// The t-th insertion takes the line of the t-th eviction.  The two sides compute their ranks
// independently; they meet in pair[t], one 64-bit word (iteration tag, side, line or
// position) that each side swaps in atomically: the side that finds the other's word there
// knows line and position and writes the line's new state.  Everything that crosses from one
// block to another travels inside that word, so no fence is needed; the state arrays are
// read by the next launch.
constexpr uint64_t PAIR_EVICT = 1ull << 39;

__device__ __forceinline__ uint64_t pair_tag(int32_t i) { return (uint64_t)(i + 1) << 40; }

__device__ __forceinline__ void finish_line(const State& st, int32_t line, int32_t v, int32_t key) {
  st.res_id[line] = v;
  st.res_next[line] = key;
  st.addr[v] = line;
}

// Sum of counts[0 .. n) by the whole block.
__device__ __forceinline__ uint32_t block_prefix_of(const uint32_t* __restrict__ counts, int64_t n,
                                                    uint32_t* red) {
  uint32_t s = 0;
  for (int64_t q = threadIdx.x; q < n; q += TB) s += counts[q];
  return block_sum_u32(s, red);
}

__device__ __forceinline__ uint64_t shfl_u64(uint64_t v, int src) {
  const uint32_t lo = __shfl((uint32_t)v, src, WAVE);
  const uint32_t hi = __shfl((uint32_t)(v >> 32), src, WAVE);
  return ((uint64_t)hi << 32) | lo;
}

// One wave per tile of 64 flag words: the evicted lines in line order.  The tile's set bits
// are dealt to the lanes round-robin by rank (lane l takes the l-th, (l+64)-th ... set bit,
// located through the wave's running popcounts), so that the chain of dependent memory
// operations behind every eviction is as long for a clustered tile as for an even one.
__device__ void p_evict_emit(const State& st, const Ctrl& c, const Iter& it, const Outputs& o,
                             int64_t vb, int64_t tiles) {
  __shared__ uint32_t red[TB / WAVE];
  constexpr int TPB = TB / WAVE;                 // tiles per block
  const int64_t first_tile = vb * TPB;
  const int w = threadIdx.x / WAVE;
  const int64_t tile = first_tile + w;
  // the block's own tiles first: most blocks of a large cache have nothing to emit
  uint32_t own[TPB];
  uint32_t any = 0;
#pragma unroll
  for (int k = 0; k < TPB; ++k) {
    own[k] = first_tile + k < tiles ? st.evict_tiles[first_tile + k] : 0;
    any |= own[k];
  }
  if (!any) return;                              // uniform over the block
  const int64_t word_at = tile * WAVE + lane_id();
  const uint64_t word = tile < tiles && word_at * WAVE < st.cap ? st.evict_words[word_at] : 0;
  uint32_t tile_base = block_prefix_of(st.evict_tiles, first_tile, red);
#pragma unroll
  for (int k = 0; k < TPB; ++k)
    if (k < w) tile_base += own[k];
  if (tile >= tiles) return;                     // uniform over the wave
  const bool scattered = st.dead_scatter && c.use_dead;
  if (st.dead_scatter && word) st.evict_words[word_at] = 0;   // consumed: zero for the next scatter
  const uint32_t mine = (uint32_t)__popcll(word);
  const uint32_t incl = wave_inclusive_scan(mine);
  const uint32_t total = __shfl(incl, WAVE - 1, WAVE);
  const int64_t dst = o.cs_offsets[it.i];
  const uint64_t tag = pair_tag(it.i);
  for (uint32_t k0 = 0; k0 < total; k0 += WAVE) {        // uniform trip count: shuffles inside
    const uint32_t k = k0 + lane_id();
    int lo = 0, hi = WAVE - 1;                   // the first word whose running count exceeds k
#pragma unroll
    for (int step = 0; step < 6; ++step) {
      const int mid = (lo + hi) >> 1;
      if (__shfl(incl, mid, WAVE) > k) hi = mid; else lo = mid + 1;
    }
    const int j = lo < WAVE ? lo : WAVE - 1;
    uint64_t bits = shfl_u64(word, j);
    const uint32_t before = __shfl(incl, j, WAVE) - __shfl(mine, j, WAVE);
    if (k >= total) continue;
    for (uint32_t r = k - before; r > 0; --r) bits &= bits - 1;
    const int32_t line = (int32_t)((tile * WAVE + j) * WAVE + (__ffsll((unsigned long long)bits) - 1));
    const uint32_t at = tile_base + k;
    const int32_t gone = st.res_id[line];
    const int32_t key = st.res_next[line];
    if (dst + at < o.cs_capacity) o.out_ids[dst + at] = gone;
    st.addr[gone] = -1;
    if (key == st.S && !st.lru && !scattered) {   // a dead resident leaves the standing bitmap
      atomicAnd(&st.dead_bits[(uint32_t)gone >> 5], ~(1u << ((uint32_t)gone & 31)));
      // (its part count was rewritten by k_threshold when the dead rows were selected from)
      if (!c.use_dead) atomicSub(&st.dead_part[(uint32_t)gone >> PART_SHIFT], 1u);
    }
    if (at < st.max_change) {
      // the reads of this line's old state are complete (their values were used above)
      // before the word is swapped in: from then on the other side may rewrite the line
      __asm__ volatile("" ::: "memory");
      const uint64_t other = atomicExch((unsigned long long*)&st.pair[at],
                                        tag | PAIR_EVICT | (uint32_t)line);
      if ((other & ~((1ull << 40) - 1)) == tag) {
        const int64_t p = (int64_t)(other & 0xFFFFFFFFull);
        finish_line(st, line, it.ids[p], key_of(it, p));
      }
    }
  }
}

// The inserted positions of one tile of accesses in position order; the block's insertions
// are first gathered in LDS by rank and then dealt one to a thread, for the same reason as
// above.
template <int IN_ITEMS>
__device__ void p_in_emit(const State& st, const Ctrl& c, const Iter& it, const Outputs& o,
                          int64_t vb) {
  __shared__ uint32_t smem[TB / WAVE + 1];
  __shared__ uint32_t red[TB / WAVE];
  __shared__ int32_t s_pos[TB * IN_ITEMS];
  if (st.in_tiles[vb] == 0) return;              // uniform over the block
  const int64_t base = (vb * TB + threadIdx.x) * IN_ITEMS;
  uint32_t flags = 0, cnt = 0;
  int32_t v[IN_ITEMS], key[IN_ITEMS], line[IN_ITEMS];
#pragma unroll
  for (int t = 0; t < IN_ITEMS; ++t) {
    const int64_t p = base + t < it.n ? base + t : 0;
    line[t] = st.acc_line[p];
    key[t] = key_of(it, p);
    v[t] = it.ids[p];
  }
#pragma unroll
  for (int t = 0; t < IN_ITEMS; ++t)
    if (base + t < it.n && line[t] < 0 && inserts(c, key[t], v[t])) {
      flags |= 1u << t;
      ++cnt;
    }
  uint32_t total;
  uint32_t rank = block_exclusive_scan<uint32_t, TB>(cnt, smem, total);
  const uint32_t tile_base = block_prefix_of(st.in_tiles, vb, red);
#pragma unroll
  for (int t = 0; t < IN_ITEMS; ++t)
    if (flags >> t & 1) s_pos[rank++] = threadIdx.x * IN_ITEMS + t;   // position inside the tile
  __syncthreads();
  const int64_t dst = o.cs_offsets[it.i];
  const uint64_t tag = pair_tag(it.i);
  const int64_t tile_first = vb * (int64_t)(TB * IN_ITEMS);
  for (uint32_t k = threadIdx.x; k < total; k += TB) {
    const int64_t p = tile_first + s_pos[k];
    const uint32_t at = tile_base + k;
    const int32_t id = it.ids[p];
    const int32_t nk = key_of(it, p);
    if (dst + at < o.cs_capacity) {
      o.in_ids[dst + at] = id;
      o.in_positions[dst + at] = (int32_t)p;
    }
    if (at < st.max_change) {
      const uint64_t other = atomicExch((unsigned long long*)&st.pair[at], tag | (uint32_t)p);
      if ((other & ~((1ull << 40) - 1)) == tag)
        finish_line(st, (int32_t)(other & 0xFFFFFFFFull), id, nk);
    }
  }
}

template <int IN_ITEMS>
__global__ __launch_bounds__(TB) void k_emit_pair(State st, Iter it, Outputs o, int64_t evict_tiles) {
  const Ctrl c = *st.ctrl;
  if (c.n_change <= 0) return;
  const int64_t evict_blocks = (evict_tiles + TB / WAVE - 1) / (TB / WAVE);
  if ((int64_t)blockIdx.x < evict_blocks) p_evict_emit(st, c, it, o, blockIdx.x, evict_tiles);
  else p_in_emit<IN_ITEMS>(st, c, it, o, blockIdx.x - evict_blocks);
}

// popcount of one part of a bitmap (the part counts of the dead-row bitmap after a resumed
// superbatch's start state has been marked)
__global__ __launch_bounds__(TB) void k_part_count(const uint32_t* __restrict__ bits, int64_t words,
                                                   uint32_t* __restrict__ part) {
  __shared__ uint32_t red[TB / WAVE];
  const int64_t base = (int64_t)blockIdx.x * PART_WORDS;
  uint32_t cnt = 0;
  for (int t = threadIdx.x; t < PART_WORDS; t += TB)
    if (base + t < words) cnt += __popc(bits[base + t]);
  const uint32_t total = block_sum_u32(cnt, red);
  if (threadIdx.x == 0) part[blockIdx.x] = total;
}

// ---- part 3 without a loop over the state: a carried cache that holds the whole superbatch ----
//
// When the carried cache has a line for every distinct row of the superbatch, an iteration
// never evicts a row that is still needed (the live candidates alone never exceed the
// capacity), so:
//   * hits and misses are known up front: an access misses iff it is the first access of a row
//     the start state does not hold; it is inserted iff the row is accessed again later
//     (otherwise it ranks behind every resident and bypasses the cache);
//   * a row keeps one line for the whole superbatch, the start line or the one it is given;
//   * iteration i evicts the n_i dead residents with the largest ids, n_i = its insertions,
//     where a resident is dead once its last access has passed (or from the start).
// The insertion lists are therefore a compaction over all accesses, and only the choice of
// the evicted rows is sequential.  All of them lie at the upper end of the id space: with M
// evictions in total, none has an id below lo_id, the M-th largest id among the rows that are
// dead from the start (they alone would supply M victims, and later arrivals only raise the
// thresholds).  The rows from lo_id up that are ever dead residents (the M rows dead from the
// start, and the rows that die during the superbatch: a few thousand, however wide that id
// range has become) are the candidates; they are numbered in id order, and one workgroup
// replays the S iterations on a bitmap over these numbers in LDS: it sets the bits of the
// rows that die in the iteration, takes the top n_i set bits out, orders these rows by cache
// line and pairs them with the insertions.  A candidate that is itself inserted during this
// call gets its line written into the candidates' line array by the thread that pairs it and
// read back, iterations later and a workgroup barrier apart, by the thread that evicts it.
// What the path cannot take (more than PLAN_CAND_MAX candidates, an iteration with more than
// PLAN_SORT_MAX insertions, S above PLAN_S_MAX, fewer rows dead from the start than
// insertions) goes through the loop above.
constexpr int PLAN_CAND_WORDS = 16384;              // LDS bitmap of the replay ...
constexpr int PLAN_CAND_MAX = PLAN_CAND_WORDS * 32; // ... over at most 524 288 candidates
constexpr int PLAN_SORT_MAX = 4096;      // evictions of one iteration the replay can order
constexpr int PLAN_RANK_DIRECT = 256;    // up to here every eviction is compared with every other
// (the replay's LDS: 64 KB of bitmap, 32 KB for the ordering, 16 KB of offsets; a workgroup
// of this GPU may use up to 160 KB)
constexpr int PLAN_S_MAX = 2048;         // iterations (LDS histograms of k_plan_heads)
enum { PLAN_M = 0, PLAN_MAX_N = 1, PLAN_LO_ID = 2, PLAN_DEAD = 3, PLAN_TAIL = 4, PLAN_FAILED = 5,
       PLAN_WHERE = 6, PLAN_CANDS = 7, PLAN_SCALARS = 8 };

struct Plan {
  uint32_t* ins_bits;    // [ceil(total / 32)] bit p: access p (flat position) is an insertion
  uint32_t* ins_tiles;   // insertions per tile of TB words, then their exclusive scan
  uint32_t* ins_base;    // [ceil(total / 32)] insertions in front of each word (tiles that have any)
  int32_t* ins_cand;     // [distinct rows] candidate number of each inserted row, -1 = not one
  int64_t* scalars;      // [PLAN_SCALARS]
  uint32_t* cand_tiles;  // candidates per tile of TB words of the id bitmap, then their scan
  uint32_t* cand_base;   // [words] candidates in front of each word of the id bitmap (from lo_id's word on)
  int32_t* cand_id;      // [PLAN_CAND_MAX] candidates in id order
  int32_t* cand_line;    // [PLAN_CAND_MAX] their cache line, -1 while not resident
  uint32_t* cand_dead;   // [PLAN_CAND_WORDS] bit c: candidate c is dead from the start
  uint32_t* arr_off;     // [S + 2] candidates that die in iteration d: count at d + 1, then offsets
  uint32_t* arr_cur;     // [S + 1] fill cursors
  int32_t* arr_cand;     // [PLAN_CAND_MAX] their numbers, grouped by iteration
  int64_t ins_words, ins_tile_count, cand_tile_count;
};

// Pass over the node-sorted accesses: the head of a run is the row's first access.  If the
// start state does not hold the row, that access misses, and it is an insertion if the run
// goes on.  Misses per iteration go to miss_count, insertions per iteration to
// cs_offsets[i + 1] (scanned afterwards) and to the bitmap over positions.
__global__ __launch_bounds__(TB) void k_plan_heads(const uint64_t* __restrict__ sorted, int64_t n,
                                                   const int64_t* __restrict__ off, int32_t S,
                                                   const int32_t* __restrict__ addr,
                                                   uint32_t* __restrict__ ins_bits,
                                                   unsigned long long* __restrict__ miss_count,
                                                   unsigned long long* __restrict__ cs_offsets) {
  extern __shared__ int32_t lds_plan[];   // offsets [S+1], misses [S], insertions [S]
  int32_t* lds_off = lds_plan;
  uint32_t* h_miss = reinterpret_cast<uint32_t*>(lds_plan + S + 1);
  uint32_t* h_ins = h_miss + S;
  for (int j = threadIdx.x; j < 2 * S; j += TB) h_miss[j] = 0;
  load_offsets(lds_off, off, S);
  const int64_t tiles = (n + LOOK_TILE - 1) / LOOK_TILE;
  for (int64_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
    const int64_t base = tile * LOOK_TILE;
#pragma unroll
    for (int i = 0; i < LOOK_ITEMS; ++i) {
      const int64_t j = base + i * TB + threadIdx.x;
      if (j >= n || !run_head(sorted, j)) continue;
      const uint64_t cur = sorted[j];
      const uint32_t v = (uint32_t)(cur >> 32);
      if (addr[v] >= 0) continue;
      const int32_t p = (int32_t)(cur & 0xFFFFFFFFu);
      const int32_t it = iter_of(lds_off, S, p);
      atomicAdd(&h_miss[it], 1u);
      if (j + 1 < n && (uint32_t)(sorted[j + 1] >> 32) == v) {
        atomicAdd(&h_ins[it], 1u);
        atomicOr(&ins_bits[p >> 5], 1u << (p & 31));
      }
    }
  }
  __syncthreads();
  for (int j = threadIdx.x; j < S; j += TB) {
    if (h_miss[j]) atomicAdd(&miss_count[j], (unsigned long long)h_miss[j]);
    if (h_ins[j]) atomicAdd(&cs_offsets[j + 1], (unsigned long long)h_ins[j]);
  }
}

// One block: cs_offsets from the insertion counts, their total M and maximum, the number of
// rows that are dead from the start, lo_id (num_nodes when nothing is evicted, -1 when the
// rows dead from the start are fewer than M) and the first sorted access of a row >= lo_id.
__global__ __launch_bounds__(BIG) void k_plan_scan(State st, const uint64_t* __restrict__ sorted,
                                                   int64_t n, int64_t* __restrict__ cs_offsets,
                                                   int64_t* __restrict__ scalars) {
  __shared__ int64_t smem[BIG / WAVE + 1];
  const int32_t S = st.S;
  const int32_t per = (S + BIG - 1) / BIG;
  const int32_t j0 = threadIdx.x * per;
  int64_t mine = 0, largest = 0;
  for (int32_t j = j0; j < j0 + per && j < S; ++j) {
    const int64_t c = cs_offsets[j + 1];
    mine += c;
    largest = c > largest ? c : largest;
  }
  int64_t M;
  int64_t run = block_exclusive_scan<int64_t, BIG>(mine, smem, M);
  for (int32_t j = j0; j < j0 + per && j < S; ++j) {
    run += cs_offsets[j + 1];
    cs_offsets[j + 1] = run;
  }
  // the largest count: waves first, then thread 0 over the waves
#pragma unroll
  for (int d = WAVE / 2; d > 0; d >>= 1) {
    const int64_t o = __shfl_xor(largest, d, WAVE);
    largest = o > largest ? o : largest;
  }
  if (lane_id() == 0) smem[threadIdx.x / WAVE] = largest;
  __syncthreads();
  if (threadIdx.x == 0) {
    int64_t m = 0;
    for (int w = 0; w < BIG / WAVE; ++w) m = smem[w] > m ? smem[w] : m;
    scalars[PLAN_MAX_N] = m;
    scalars[PLAN_M] = M;
    scalars[PLAN_FAILED] = 0;
    scalars[PLAN_WHERE] = 0;
  }
  __syncthreads();
  const int64_t pper = (st.parts + BIG - 1) / BIG;
  int64_t dead_mine = 0;
  for (int64_t q = threadIdx.x * pper; q < (threadIdx.x + 1) * pper && q < st.parts; ++q)
    dead_mine += st.dead_part[q];
  int64_t dead;
  block_exclusive_scan<int64_t, BIG>(dead_mine, smem, dead);
  int32_t lo_id = (int32_t)st.num_nodes;
  if (M >= 1)   // uniform
    lo_id = dead >= M ? p_kth_set_bit<BIG>(st.dead_bits, st.dead_part, st.parts, st.words,
                                            dead - M + 1, false)
                      : -1;
  if (threadIdx.x == 0) {
    int64_t lo = 0, hi = n;
    while (lo < hi) {
      const int64_t mid = (lo + hi) >> 1;
      if ((int64_t)(sorted[mid] >> 32) < (int64_t)lo_id) lo = mid + 1; else hi = mid;
    }
    scalars[PLAN_TAIL] = lo;
    scalars[PLAN_LO_ID] = lo_id;
    scalars[PLAN_DEAD] = dead;
  }
}

// set bits per tile of TB words
__global__ __launch_bounds__(TB) void k_bit_tiles(const uint32_t* __restrict__ bits, int64_t words,
                                                  uint32_t* __restrict__ tiles) {
  __shared__ uint32_t red[TB / WAVE];
  const int64_t w = (int64_t)blockIdx.x * TB + threadIdx.x;
  const uint32_t total = block_sum_u32(w < words ? (uint32_t)__popc(bits[w]) : 0u, red);
  if (threadIdx.x == 0) tiles[blockIdx.x] = total;
}

// in_ids / in_positions of the whole superbatch: the set bits of ins_bits in position order
// (iterations are consecutive stretches of positions, so this is iteration by iteration and
// inside an iteration by position, as the lists are defined).
__global__ __launch_bounds__(TB) void k_ins_emit(const uint32_t* __restrict__ bits, int64_t words,
                                                 const uint32_t* __restrict__ tile_base,
                                                 const int32_t* __restrict__ ids,
                                                 const int64_t* __restrict__ off, int32_t S,
                                                 int32_t* __restrict__ in_ids,
                                                 int32_t* __restrict__ in_positions,
                                                 uint32_t* __restrict__ ins_base,
                                                 int32_t* __restrict__ ins_cand) {
  extern __shared__ int32_t lds_off[];
  __shared__ uint32_t smem[TB / WAVE + 1];
  const uint32_t first = tile_base[blockIdx.x];
  if (tile_base[blockIdx.x + 1] == first) return;   // nothing in this tile (uniform)
  load_offsets(lds_off, off, S);
  const int64_t w = (int64_t)blockIdx.x * TB + threadIdx.x;
  uint32_t word = w < words ? bits[w] : 0u;
  uint32_t total;
  uint32_t rank = first + block_exclusive_scan<uint32_t, TB>((uint32_t)__popc(word), smem, total);
  if (w < words) ins_base[w] = rank;
  while (word) {
    const int32_t p = (int32_t)(w * 32 + (__ffs(word) - 1));
    word &= word - 1;
    in_ids[rank] = ids[p];
    in_positions[rank] = p - lds_off[iter_of(lds_off, S, p)];
    ins_cand[rank] = -1;
    ++rank;
  }
}

// src_line of the insertions: their row arrives with this access
__global__ __launch_bounds__(TB) void k_ins_lines(const uint32_t* __restrict__ bits, int64_t words,
                                                  int32_t* __restrict__ src_line) {
  const int64_t w = (int64_t)blockIdx.x * TB + threadIdx.x;
  uint32_t word = w < words ? bits[w] : 0u;
  while (word) {
    src_line[w * 32 + (__ffs(word) - 1)] = -1;
    word &= word - 1;
  }
}

// The id bitmap of the candidates, from lo_id's word on: first the rows dead from the start ...
// (lo_id comes from the device-side scalars: this and the next two kernels run before the host
// has read them, so that the host learns the exact number of candidates with the same copy)
__global__ __launch_bounds__(TB) void k_cand_start(const uint32_t* __restrict__ dead_bits,
                                                   int64_t words, int64_t num_nodes,
                                                   const int64_t* __restrict__ scalars,
                                                   uint32_t* __restrict__ cand_bits) {
  const int64_t lo_id = scalars[PLAN_LO_ID];
  if (lo_id < 0 || lo_id >= num_nodes) return;      // nothing is evicted, or this path is not taken
  const int64_t span = (int64_t)gridDim.x * TB;
  for (int64_t w = (lo_id >> 5) + (int64_t)blockIdx.x * TB + threadIdx.x; w < words; w += span) {
    uint32_t word = dead_bits[w];
    if (w == (lo_id >> 5)) word &= ~((1u << (lo_id & 31)) - 1u);
    cand_bits[w] = word;
  }
}

// Is sorted[j] the last access of a row that is resident when it dies?  (A row the start state
// does not hold is resident only if it was inserted, that is, if it has an earlier access.)
__device__ __forceinline__ bool plan_arrival(const uint64_t* __restrict__ sorted, int64_t n,
                                             int64_t j, const int32_t* __restrict__ addr,
                                             const int32_t* off, int32_t S,
                                             int32_t& v, int32_t& d, bool& inserted) {
  const uint64_t cur = sorted[j];
  v = (int32_t)(cur >> 32);
  if (j + 1 < n && (int32_t)(sorted[j + 1] >> 32) == v) return false;
  const bool earlier = j > 0 && (int32_t)(sorted[j - 1] >> 32) == v;
  inserted = addr[v] < 0;
  if (!earlier && inserted) return false;
  d = iter_of(off, S, (int32_t)(cur & 0xFFFFFFFFu));
  return true;
}

// ... then (PLACE = false) the rows >= lo_id that die during the superbatch, counted per
// iteration at arr_off[d + 1].  PLACE = true, after the candidates are numbered: their numbers
// go to arr_cand at the cursors, and a row that is inserted during this call leaves its number
// with its insertion record (with arr_ids, the rows themselves go there instead, and nothing
// else is written).  A block works on one stretch of the sorted pairs and counts
// per iteration in LDS first, so that the counters and cursors in global memory, a few
// addresses that every arrival would otherwise meet at, see one atomic per block and iteration.
// lds: S + 1 offsets, S counters.
template <bool PLACE>
__global__ __launch_bounds__(TB) void k_plan_arrivals(const uint64_t* __restrict__ sorted, int64_t n,
                                                      const int64_t* __restrict__ scalars,
                                                      const int32_t* __restrict__ addr,
                                                      const int64_t* __restrict__ off, int32_t S,
                                                      uint32_t* __restrict__ cand_bits,
                                                      const uint32_t* __restrict__ cand_base,
                                                      int64_t num_nodes, Plan pl,
                                                      int32_t* __restrict__ arr_ids) {
  extern __shared__ int32_t lds_off[];
  uint32_t* s_cnt = reinterpret_cast<uint32_t*>(lds_off + S + 1);
  const int64_t lo_id = scalars[PLAN_LO_ID];
  if (lo_id < 0 || lo_id >= num_nodes) return;
  for (int d = threadIdx.x; d < S; d += TB) s_cnt[d] = 0;
  load_offsets(lds_off, off, S);
  const int64_t lo_word = lo_id >> 5;
  const int64_t tail = scalars[PLAN_TAIL];
  const int64_t per = (((n - tail + gridDim.x - 1) / gridDim.x + TB - 1) / TB) * TB;
  const int64_t first = tail + (int64_t)blockIdx.x * per;
  const int64_t last = first + per < n ? first + per : n;
  for (int64_t j = first + threadIdx.x; j < last; j += TB) {
    int32_t v, d;
    bool inserted;
    if (!plan_arrival(sorted, n, j, addr, lds_off, S, v, d, inserted)) continue;
    if (!PLACE) atomicOr(&cand_bits[(uint32_t)v >> 5], 1u << (v & 31));
    atomicAdd(&s_cnt[d], 1u);
  }
  __syncthreads();
  for (int d = threadIdx.x; d < S; d += TB) {
    const uint32_t c = s_cnt[d];
    if (!PLACE) {
      if (c) atomicAdd(&pl.arr_off[d + 1], c);
    } else {
      s_cnt[d] = c ? atomicAdd(&pl.arr_cur[d], c) : 0u;   // the block's places in the iteration's list
    }
  }
  if (!PLACE) return;
  __syncthreads();
  for (int64_t j = first + threadIdx.x; j < last; j += TB) {
    int32_t v, d;
    bool inserted;
    if (!plan_arrival(sorted, n, j, addr, lds_off, S, v, d, inserted)) continue;
    if (arr_ids) {                                   // the stepped path wants the rows themselves
      arr_ids[atomicAdd(&s_cnt[d], 1u)] = v;
      continue;
    }
    const uint32_t below = (1u << (v & 31)) - 1u;
    const uint32_t c = cand_base[((uint32_t)v >> 5) - lo_word] + __popc(cand_bits[(uint32_t)v >> 5] & below);
    // (the host takes this path only with at most PLAN_CAND_MAX candidates: c is below that)
    pl.arr_cand[atomicAdd(&s_cnt[d], 1u)] = (int32_t)c;
    if (inserted && c < (uint32_t)PLAN_CAND_MAX) {
      int64_t h = j;                                 // the row's first access is its insertion
      while (h > 0 && (int32_t)(sorted[h - 1] >> 32) == v) --h;
      const uint32_t p = (uint32_t)(sorted[h] & 0xFFFFFFFFu);
      pl.ins_cand[pl.ins_base[p >> 5] + __popc(pl.ins_bits[p >> 5] & ((1u << (p & 31)) - 1u))] = (int32_t)c;
    }
  }
}

// Numbers the candidates in id order: cand_base per bitmap word, id, start line (-1 for a row
// that is inserted during this call) and the dead-from-the-start flag per candidate.
__global__ __launch_bounds__(TB) void k_cand_emit(const uint32_t* __restrict__ cand_bits,
                                                  const uint32_t* __restrict__ dead_bits,
                                                  int64_t lo_word, int64_t nwords,
                                                  const uint32_t* __restrict__ tile_base,
                                                  const int32_t* __restrict__ addr, Plan pl) {
  __shared__ uint32_t smem[TB / WAVE + 1];
  const int64_t w = (int64_t)blockIdx.x * TB + threadIdx.x;
  uint32_t word = w < nwords ? cand_bits[lo_word + w] : 0u;
  const uint32_t dead = w < nwords ? dead_bits[lo_word + w] : 0u;
  uint32_t total;
  uint32_t c = tile_base[blockIdx.x] + block_exclusive_scan<uint32_t, TB>((uint32_t)__popc(word), smem, total);
  if (w < nwords) pl.cand_base[w] = c;
  while (word) {
    const int b = __ffs(word) - 1;
    word &= word - 1;
    if (c < (uint32_t)PLAN_CAND_MAX) {
      const int32_t v = (int32_t)((lo_word + w) * 32 + b);
      pl.cand_id[c] = v;
      pl.cand_line[c] = addr[v];
      if (dead >> b & 1) atomicOr(&pl.cand_dead[c >> 5], 1u << (c & 31));
    }
    ++c;
  }
}

// One block: arr_off <- offsets (arr_off[i] .. arr_off[i + 1] are the candidates that die in
// iteration i), arr_cur <- the same, as cursors.
__global__ __launch_bounds__(BIG) void k_plan_arrival_offsets(uint32_t* __restrict__ arr_off,
                                                              uint32_t* __restrict__ arr_cur,
                                                              int32_t S,
                                                              int64_t* __restrict__ scalars) {
  __shared__ uint32_t smem[BIG / WAVE + 1];
  const int32_t per = (S + BIG - 1) / BIG;
  const int32_t j0 = threadIdx.x * per;
  uint32_t mine = 0;
  for (int32_t j = j0; j < j0 + per && j < S; ++j) mine += arr_off[j + 1];
  uint32_t total;
  uint32_t run = block_exclusive_scan<uint32_t, BIG>(mine, smem, total);
  for (int32_t j = j0; j < j0 + per && j < S; ++j) {
    arr_cur[j] = run;
    run += arr_off[j + 1];
    arr_off[j + 1] = run;
  }
  // the candidates: the M rows dead from the start and the rows that die during the superbatch
  if (threadIdx.x == 0) scalars[PLAN_CANDS] = scalars[PLAN_M] + (int64_t)total;
}

// Exclusive prefix of v over the BIG threads of the block, and the block total, with a single
// barrier: every thread adds up the totals of the waves in front of its own.  `slots` (one
// per wave) must not be rewritten before a later barrier.
__device__ __forceinline__ uint32_t block_prefix_one_barrier(uint32_t v, uint32_t* slots,
                                                             uint32_t& total) {
  const uint32_t inc = wave_inclusive_scan(v);
  const int w = threadIdx.x / WAVE;
  if (lane_id() == WAVE - 1) slots[w] = inc;
  __syncthreads();
  uint32_t before = 0, all = 0;
#pragma unroll
  for (int q = 0; q < BIG / WAVE; ++q) {
    const uint32_t t = slots[q];
    all += t;
    if (q < w) before += t;
  }
  total = all;
  return before + inc - v;
}

// The replay (see the head of this part).  One block.  scalars[PLAN_FAILED] is set, before the
// state is touched, when there are more candidates than the bitmap holds, and later if an
// invariant does not hold; the host then runs the loop instead.
// The iteration's offsets sit in LDS, and what an iteration reads from global memory at
// addresses that do not depend on the selection (the candidates that die in it, its
// insertions) is requested an iteration ahead, so that the chain of dependent memory accesses
// per iteration is: selection in LDS -> id and line of the selected candidates -> stores.
__global__ __launch_bounds__(BIG) void k_plan_replay(State st, Plan pl, int64_t n_cand_tiles,
                                                     const int64_t* __restrict__ cs_offsets,
                                                     const int32_t* __restrict__ in_ids,
                                                     int32_t* __restrict__ out_ids) {
  __shared__ uint32_t bits[PLAN_CAND_WORDS + BIG];   // room for one more word per thread, see WPT
  __shared__ int32_t s_a[PLAN_SORT_MAX];
  __shared__ int32_t s_b[PLAN_SORT_MAX];
  __shared__ uint32_t s_arr[PLAN_S_MAX + 1];       // arr_off
  __shared__ int32_t s_cs[PLAN_S_MAX + 1];         // cs_offsets (below 2^31: they index int32 lists)
  __shared__ uint32_t slots_select[BIG / WAVE], slots_rank[BIG / WAVE];
  __shared__ int32_t slots_lo[BIG / WAVE], slots_hi[BIG / WAVE];
  __shared__ int32_t s_failed;
  static_assert(PLAN_CAND_WORDS + BIG <= (1 << 26), "a noted word packs its index and a count up to 32");
  static_assert(BIG + PLAN_SORT_MAX / 2 <= PLAN_SORT_MAX && 2 * BIG <= PLAN_SORT_MAX,
                "the fine buckets of the ranking and the coarse buckets' records fit the two arrays");
  constexpr int EPT = PLAN_SORT_MAX / BIG;         // evictions of a thread
  const int32_t S = st.S;
  const uint32_t n_cand = pl.cand_tiles[n_cand_tiles];
  if (n_cand > (uint32_t)PLAN_CAND_MAX) {          // uniform
    if (threadIdx.x == 0) pl.scalars[PLAN_FAILED] = 4;
    return;
  }
  // consecutive bitmap words of a thread: as many as the candidates there are need, and an
  // odd number, so that the threads of a wave that read their t-th word hit different banks
  int WPT = (int)(((n_cand + 31) / 32 + BIG - 1) / BIG);
  if (WPT > 1) WPT |= 1;
  for (int w = threadIdx.x; w < WPT * BIG; w += BIG) bits[w] = w < PLAN_CAND_WORDS ? pl.cand_dead[w] : 0u;
  for (int j = threadIdx.x; j <= S; j += BIG) {
    s_arr[j] = pl.arr_off[j];
    s_cs[j] = (int32_t)cs_offsets[j];
  }
  if (threadIdx.x == 0) s_failed = 0;
  __syncthreads();
  // requested ahead for iteration 0
  int32_t next_arr[EPT], next_in[EPT], next_ic[EPT];
#pragma unroll
  for (int e = 0; e < EPT; ++e) {
    const int32_t k = threadIdx.x + e * BIG;
    next_arr[e] = (uint32_t)k < s_arr[1] ? pl.arr_cand[k] : -1;
    const bool have = k < s_cs[1];
    next_in[e] = have ? in_ids[k] : -1;
    next_ic[e] = have ? pl.ins_cand[k] : -1;
  }
  for (int32_t i = 0; i < S; ++i) {
    const uint32_t a0 = s_arr[i], a1 = s_arr[i + 1];
    const int32_t c0 = s_cs[i];
    const int32_t n = s_cs[i + 1] - c0;
    // the rows whose last access is in this iteration are dead from here on
#pragma unroll
    for (int e = 0; e < EPT; ++e)
      if (next_arr[e] >= 0) atomicOr(&bits[(uint32_t)next_arr[e] >> 5], 1u << (next_arr[e] & 31));
    for (uint32_t a = a0 + EPT * BIG + threadIdx.x; a < a1; a += BIG) {
      const uint32_t c = (uint32_t)pl.arr_cand[a];
      atomicOr(&bits[c >> 5], 1u << (c & 31));
    }
    int32_t my_in[EPT], my_ic[EPT];
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      my_in[e] = next_in[e];
      my_ic[e] = next_ic[e];
    }
    if (i + 1 < S) {        // the requests for the next iteration
      const int32_t c1 = s_cs[i + 1], n1 = s_cs[i + 2] - c1;
#pragma unroll
      for (int e = 0; e < EPT; ++e) {
        const int32_t k = threadIdx.x + e * BIG;
        next_arr[e] = a1 + (uint32_t)k < s_arr[i + 2] ? pl.arr_cand[a1 + k] : -1;
        next_in[e] = k < n1 ? in_ids[c1 + k] : -1;
        next_ic[e] = k < n1 ? pl.ins_cand[c1 + k] : -1;
      }
    }
    if (n == 0) continue;   // uniform; the next barrier orders the bits set above
    if (WPT > 1)            // (s_b is free: the barrier that ended the iteration before)
      for (int32_t q = threadIdx.x; q < n; q += BIG) s_b[q] = -1;
    __syncthreads();
    // the top n set bits: set bits of the chunks above a thread's own, from a block scan
    uint32_t cnt = 0;
    for (int t = 0; t < WPT; ++t) cnt += __popc(bits[threadIdx.x * WPT + t]);
    uint32_t total;
    const uint32_t below = block_prefix_one_barrier(cnt, slots_select, total);
    const uint32_t above = total - below - cnt;
    if (total < (uint32_t)n) {                      // cannot happen (see the head of this part)
      s_failed = 1;
      pl.scalars[PLAN_WHERE] = i;
    } else if (above < (uint32_t)n) {
      uint32_t take = cnt < (uint32_t)n - above ? cnt : (uint32_t)n - above;
      uint32_t k = above;
      if (WPT == 1) {
        uint32_t word = bits[threadIdx.x];
        while (take) {
          const int b = 31 - __clz(word);
          word &= ~(1u << b);
          s_a[k++] = (int32_t)(threadIdx.x * 32 + b);
          --take;
        }
        bits[threadIdx.x] = word;
      } else {
        // Several words per thread: the selection falls on the few threads at the upper end,
        // hundreds of bits each.  They only note their words (word and bits to take from its
        // top, in s_b at the word's first place in s_a; the other entries of s_b are -1), and
        // the whole block then takes the words apart, one a thread.
        for (int t = WPT - 1; t >= 0 && take; --t) {
          const uint32_t wi = threadIdx.x * WPT + t;
          const uint32_t pc = (uint32_t)__popc(bits[wi]);
          if (!pc) continue;
          const uint32_t tw = pc < take ? pc : take;
          s_b[k] = (int32_t)((wi << 5) | (tw - 1));
          k += tw;
          take -= tw;
        }
      }
    }
    __syncthreads();
    if (s_failed) break;                            // uniform
    if (WPT > 1) {
      for (uint32_t q = threadIdx.x; q < (uint32_t)n; q += BIG) {
        const int32_t d = s_b[q];
        if (d < 0) continue;
        const uint32_t wi = (uint32_t)d >> 5, tw = ((uint32_t)d & 31u) + 1u;
        uint32_t word = bits[wi];
        for (uint32_t r = 0; r < tw; ++r) {
          const int b = 31 - __clz(word);
          word &= ~(1u << b);
          s_a[q + r] = (int32_t)(wi * 32 + b);
        }
        bits[wi] = word;
      }
      __syncthreads();
    }
    // the evicted rows and their lines
    int32_t my_v[EPT], my_line[EPT];
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      const int32_t k = threadIdx.x + e * BIG;
      my_v[e] = my_line[e] = -1;
      if (k >= n) continue;
      const int32_t c = s_a[k];
      my_v[e] = pl.cand_id[c];
      my_line[e] = pl.cand_line[c];
      s_b[k] = my_line[e];
      if (my_line[e] < 0) {                         // a dead resident has a line: cannot happen
        s_failed = 2;
        pl.scalars[PLAN_WHERE] = i;
      }
    }
    if (n > PLAN_RANK_DIRECT) {                     // uniform: the range of the evicted lines
      int32_t lo = INT32_MAX, hi = 0;
#pragma unroll
      for (int e = 0; e < EPT; ++e)
        if (my_v[e] >= 0) {
          lo = my_line[e] < lo ? my_line[e] : lo;
          hi = my_line[e] > hi ? my_line[e] : hi;
        }
#pragma unroll
      for (int d = WAVE / 2; d > 0; d >>= 1) {
        const int32_t olo = __shfl_xor(lo, d, WAVE), ohi = __shfl_xor(hi, d, WAVE);
        lo = olo < lo ? olo : lo;
        hi = ohi > hi ? ohi : hi;
      }
      if (lane_id() == 0) {
        slots_lo[threadIdx.x / WAVE] = lo;
        slots_hi[threadIdx.x / WAVE] = hi;
      }
    }
    __syncthreads();
    if (s_failed) break;                            // uniform; no line may be used as an index then
    // out_ids in line order: the rank of a line is the number of smaller ones
    int32_t my_rank[EPT];
    if (n <= PLAN_RANK_DIRECT) {                    // uniform: every thread counts over all lines
#pragma unroll
      for (int e = 0; e < EPT; ++e) {
        my_rank[e] = 0;
        if (my_v[e] < 0) continue;
        int32_t r = 0;
        for (int32_t q = 0; q < n; ++q) r += s_b[q] < my_line[e];
        my_rank[e] = r;
      }
    } else {
      // Many evictions: the lines are dealt to buckets that grow with the line, a scan of the
      // bucket sizes gives the number of lines in the buckets below, and a line is compared
      // with the members of its own bucket only.  The evicted lines crowd where rows come and
      // go, so buckets of equal width over their range would leave most of them in a few:
      // BIG coarse buckets of equal width are counted first, and a coarse bucket with m
      // members is cut into about m/4 fine ones (a power of two, at most one per line), fewer
      // than BIG + n/2 in all.
      // s_a is free (every thread has read its candidates): the fine counters; s_b holds the
      // coarse counts, then first fine bucket and cut of every coarse bucket, then the lines
      // by fine bucket.
      int32_t range_lo = INT32_MAX, range_hi = 0;
#pragma unroll
      for (int q = 0; q < BIG / WAVE; ++q) {
        range_lo = slots_lo[q] < range_lo ? slots_lo[q] : range_lo;
        range_hi = slots_hi[q] > range_hi ? slots_hi[q] : range_hi;
      }
      int coarse_shift = 0;                         // (line - range_lo) >> coarse_shift < BIG
      while (((range_hi - range_lo) >> coarse_shift) >= BIG) ++coarse_shift;
      s_b[threadIdx.x] = 0;
#pragma unroll
      for (int e = 0; e < EPT; ++e) s_a[threadIdx.x + e * BIG] = 0;
      __syncthreads();
      int32_t coarse[EPT], bucket[EPT], slot[EPT];
#pragma unroll
      for (int e = 0; e < EPT; ++e) {
        coarse[e] = bucket[e] = slot[e] = 0;
        if (my_v[e] < 0) continue;
        coarse[e] = (my_line[e] - range_lo) >> coarse_shift;
        atomicAdd(&s_b[coarse[e]], 1);
      }
      __syncthreads();
      {
        const uint32_t members = (uint32_t)s_b[threadIdx.x];
        int cut = 0;                                // the coarse bucket becomes 1 << cut fine ones
        while ((4u << cut) < members && cut < coarse_shift) ++cut;
        uint32_t fine_total;
        const uint32_t fine_first = block_prefix_one_barrier(1u << cut, slots_rank, fine_total);
        s_b[threadIdx.x] = (int32_t)fine_first;     // (only this thread read the entry)
        s_b[BIG + threadIdx.x] = cut;
      }
      __syncthreads();
#pragma unroll
      for (int e = 0; e < EPT; ++e) {
        if (my_v[e] < 0) continue;
        const int cut = s_b[BIG + coarse[e]];
        const int32_t within = (my_line[e] - range_lo) & ((1 << coarse_shift) - 1);
        bucket[e] = s_b[coarse[e]] + (within >> (coarse_shift - cut));
        slot[e] = atomicAdd(&s_a[bucket[e]], 1);
      }
      __syncthreads();
      {
        uint32_t cnt_b[EPT], sum = 0;
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
          cnt_b[e] = (uint32_t)s_a[threadIdx.x * EPT + e];
          sum += cnt_b[e];
        }
        uint32_t all;
        uint32_t run = block_prefix_one_barrier(sum, slots_select, all);
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
          s_a[threadIdx.x * EPT + e] = (int32_t)run;
          run += cnt_b[e];
        }
      }
      __syncthreads();
#pragma unroll
      for (int e = 0; e < EPT; ++e)
        if (my_v[e] >= 0) s_b[s_a[bucket[e]] + slot[e]] = my_line[e];
      __syncthreads();
#pragma unroll
      for (int e = 0; e < EPT; ++e) {
        my_rank[e] = 0;
        if (my_v[e] < 0) continue;
        const int32_t first = s_a[bucket[e]];
        const int32_t end = bucket[e] + 1 < PLAN_SORT_MAX ? s_a[bucket[e] + 1] : n;
        int32_t r = first;
        for (int32_t q = first; q < end; ++q) r += s_b[q] < my_line[e];
        my_rank[e] = r;
      }
    }
#pragma unroll
    for (int e = 0; e < EPT; ++e)
      if (my_v[e] >= 0) out_ids[c0 + my_rank[e]] = my_v[e];
    __syncthreads();   // both arrays are free now: they carry the insertions to the threads that hold their lines
#pragma unroll
    for (int e = 0; e < EPT; ++e)
      if (my_v[e] >= 0) {
        s_a[threadIdx.x + e * BIG] = my_in[e];
        s_b[threadIdx.x + e * BIG] = my_ic[e];
      }
    __syncthreads();
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      if (my_v[e] < 0) continue;
      const int32_t w = s_a[my_rank[e]];
      const int32_t wc = s_b[my_rank[e]];
      const int32_t line = my_line[e];
      st.addr[w] = line;
      st.res_id[line] = w;
      if (wc >= 0) pl.cand_line[wc] = line;        // read when the row is evicted again
    }
    __syncthreads();   // also makes these writes visible to the block's later reads
  }
  if (threadIdx.x == 0 && s_failed) pl.scalars[PLAN_FAILED] = s_failed;
}

// ---- the same regime with more candidates or evictions than the replay holds ------------------
//
// Hits, misses and insertions are known up front as above; the choice of the evicted rows runs
// on the standing bitmap of dead rows in global memory instead, three launches per iteration
// that evicts: k_step_find (one block: the id T above which the iteration's n dead rows lie),
// k_step_scatter (their bits leave the bitmap, their lines are flagged), k_step_emit (the
// flagged lines in line order take the iteration's insertions; other blocks set the bits of the
// rows that die in the next iteration).  No pass touches the accesses.

// The rows of arr_ids[a0, a1) are dead residents from now on.
// (The list of an iteration comes in ascending stretches, so neighbouring lanes mostly fall
// into the same part of the bitmap: the first lane of each run adds the run's length to the
// part's count, instead of one atomic per row on a few hundred addresses.)
__device__ __forceinline__ void step_arrivals(const State& st, const int32_t* __restrict__ arr_ids,
                                              uint32_t a0, uint32_t a1, int64_t vb, int64_t vblocks) {
  const int lane = lane_id();
  for (int64_t first = a0 + vb * TB + (threadIdx.x - lane); first < a1; first += vblocks * TB) {
    const int64_t a = first + lane;                // whole waves stay in the loop together
    const bool valid = a < a1;
    const uint32_t v = valid ? (uint32_t)arr_ids[a] : 0u;
    const uint32_t part = valid ? v >> PART_SHIFT : 0xFFFFFFFFu;
    if (valid) atomicOr(&st.dead_bits[v >> 5], 1u << (v & 31));
    const uint32_t prev = __shfl_up(part, 1, WAVE);
    const bool leader = valid && (lane == 0 || prev != part);
    const uint64_t leaders = __ballot(leader);
    const int valid_lanes = __popcll(__ballot(valid));   // the valid lanes are the lowest ones
    if (leader) {
      const uint64_t higher = lane == WAVE - 1 ? 0ull : leaders & ~((2ull << lane) - 1ull);
      const int next = higher ? __ffsll((unsigned long long)higher) - 1 : valid_lanes;
      atomicAdd(&st.dead_part[part], (uint32_t)(next - lane));
    }
  }
}

__global__ __launch_bounds__(TB) void k_step_arrive(State st, const int32_t* __restrict__ arr_ids,
                                                    uint32_t a0, uint32_t a1) {
  step_arrivals(st, arr_ids, a0, a1, blockIdx.x, gridDim.x);
}

// One block.  n rows are evicted: the n dead rows with the largest ids.
__global__ __launch_bounds__(BIG) void k_step_find(State st, int64_t n, int64_t evict_tiles) {
  __shared__ int64_t smem[BIG / WAVE + 1];
  int64_t mine = 0;
  for (int64_t q = threadIdx.x; q < st.parts; q += BIG) mine += st.dead_part[q];
  int64_t total;
  block_exclusive_scan<int64_t, BIG>(mine, smem, total);
  const int64_t keep = total - n;
  int32_t T = -1;
  if (keep > 0) {
    T = p_kth_set_bit<BIG>(st.dead_bits, st.dead_part, st.parts, st.words, keep, true);
  } else {
    for (int64_t q = threadIdx.x; q < st.parts; q += BIG) st.dead_part[q] = 0;
  }
  if (threadIdx.x == 0) {
    if (keep < 0) *st.fault = 1;   // fewer dead rows than insertions: cannot happen in this regime
    Ctrl c{};
    c.jstar = st.S;
    c.mode_in = MODE_ALL;
    c.mode_res = MODE_SELECT;
    c.keep = (int32_t)keep;
    c.T = T;
    c.n_change = (int32_t)n;
    c.use_dead = 1;
    *st.ctrl = c;
  }
  for (int64_t q = threadIdx.x; q < evict_tiles; q += BIG) st.evict_tiles[q] = 0;
}

__global__ void k_step_verdict(const int32_t* __restrict__ fault, int64_t* __restrict__ scalars) {
  if (*fault) {
    scalars[PLAN_FAILED] = 8;
    scalars[PLAN_WHERE] = -1;
  }
}

__global__ __launch_bounds__(TB) void k_step_scatter(State st) {
  const Ctrl c = *st.ctrl;
  p_dead_scatter(st, c, blockIdx.x, gridDim.x);
}

// blocks [0, evict_blocks): a block per TB flag words (TB / WAVE tiles), the evicted lines in
// line order; the t-th of them takes the t-th insertion of the iteration, whose list starts
// at in_ids[dst].  The evicted lines crowd in few tiles (where rows come and go), so the
// block's evictions are dealt to all its threads by rank: a thread finds the flag word of its
// rank in the block's running popcounts (LDS), then the bit inside the word.
// The other blocks: the rows that die in the next iteration.
__global__ __launch_bounds__(TB) void k_step_emit(State st, int64_t evict_tiles, int64_t evict_blocks,
                                                  int64_t dst, const int32_t* __restrict__ in_ids,
                                                  int32_t* __restrict__ out_ids,
                                                  const int32_t* __restrict__ arr_ids, uint32_t a0,
                                                  uint32_t a1) {
  __shared__ uint32_t red[TB / WAVE];
  __shared__ uint32_t smem[TB / WAVE + 1];
  __shared__ uint64_t s_word[TB];
  __shared__ uint32_t s_incl[TB];
  if ((int64_t)blockIdx.x >= evict_blocks) {
    step_arrivals(st, arr_ids, a0, a1, blockIdx.x - evict_blocks, gridDim.x - evict_blocks);
    return;
  }
  constexpr int TPB = TB / WAVE;
  const int64_t first_tile = (int64_t)blockIdx.x * TPB;
  uint32_t any = 0;
#pragma unroll
  for (int k = 0; k < TPB; ++k)
    any |= first_tile + k < evict_tiles ? st.evict_tiles[first_tile + k] : 0;
  if (!any) return;                                // uniform over the block
  const int64_t word_at = first_tile * WAVE + threadIdx.x;
  const uint64_t word = word_at < evict_tiles * WAVE && word_at * WAVE < st.cap
                            ? st.evict_words[word_at] : 0;
  if (word) st.evict_words[word_at] = 0;           // consumed: zero for the next scatter
  const uint32_t mine = (uint32_t)__popcll(word);
  uint32_t total;
  const uint32_t before_me = block_exclusive_scan<uint32_t, TB>(mine, smem, total);
  s_word[threadIdx.x] = word;
  s_incl[threadIdx.x] = before_me + mine;
  const int64_t base = dst + block_prefix_of(st.evict_tiles, first_tile, red);   // (barriers inside)
  for (uint32_t r = threadIdx.x; r < total; r += TB) {
    int lo = 0, hi = TB - 1;                       // the first word whose running count exceeds r
#pragma unroll
    for (int step = 0; step < 8; ++step) {
      const int mid = (lo + hi) >> 1;
      if (s_incl[mid] > r) hi = mid; else lo = mid + 1;
    }
    uint64_t bits = s_word[lo];
    for (uint32_t skip = r - (s_incl[lo] - (uint32_t)__popcll(bits)); skip > 0; --skip) bits &= bits - 1;
    const int32_t line = (int32_t)((first_tile * WAVE + lo) * WAVE + (__ffsll((unsigned long long)bits) - 1));
    const int64_t at = base + r;
    const int32_t gone = st.res_id[line];
    const int32_t comes = in_ids[at];
    out_ids[at] = gone;
    // (the evicted row keeps its entry of the address table: it is never accessed again, and the
    // lookup after the last iteration finds the line it had)
    st.addr[comes] = line;
    st.res_id[line] = comes;
  }
}

struct Workspace {
  uint64_t *pairs_a, *pairs_b, *heads_a, *heads_b;
  uint32_t* key_hists;      // [S x (S + 1)] accesses per iteration and next accessed iteration (S <= STATIC_S_MAX)
  StaticIter* static_plan;  // [S]
  uint32_t* touch_ctr;      // [2] hits keyed to / above the threshold bucket, of the running iteration
  uint32_t* hist;
  uint32_t* head_tiles;
  int32_t* next_iter;
  int32_t* first_of;
  int64_t* d_offsets;
  int64_t* d_ready;
  int64_t* d_cs_offsets;
  unsigned long long* d_counts;
  State st;
  Plan plan;
  int64_t look_tiles, evict_tiles, in_tiles, max_heads, max_change;
  size_t bytes;
};

int bits_for(int64_t values) {  // bits needed to hold 0 .. values-1
  int b = 1;
  while (b < 63 && (int64_t(1) << b) < values) ++b;
  return b;
}

Workspace carve(void* base, int64_t num_nodes, int64_t total, int32_t S, int64_t cap,
                int64_t max_n) {
  Arena a(base);
  Workspace w{};
  const int64_t t = total > 0 ? total : 1;
  w.max_heads = t < num_nodes ? t : num_nodes;
  w.pairs_a = a.take<uint64_t>(t);
  w.pairs_b = a.take<uint64_t>(t);
  w.heads_a = a.take<uint64_t>(w.max_heads);
  w.heads_b = a.take<uint64_t>(w.max_heads);
  w.hist = a.take<uint32_t>(radix_plan(t).hist_elems);
  w.look_tiles = ceil_div(t, LOOK_TILE);
  w.head_tiles = a.take<uint32_t>(w.look_tiles + 1 + scan_scratch_elems(w.look_tiles + 1));
  w.next_iter = a.take<int32_t>(t);
  w.key_hists = a.take<uint32_t>(S <= STATIC_S_MAX ? (size_t)S * (S + 1) : 0);
  w.static_plan = a.take<StaticIter>(S);
  w.touch_ctr = a.take<uint32_t>(2);
  w.first_of = a.take<int32_t>(num_nodes);   // resumed superbatches only
  w.d_offsets = a.take<int64_t>(S + 1);
  w.d_ready = a.take<int64_t>(S);
  w.d_cs_offsets = a.take<int64_t>(S + 1);
  w.d_counts = a.take<unsigned long long>(2);
  State& st = w.st;
  const int64_t c = cap > 0 ? cap : 1;
  st.cap = cap;
  st.num_nodes = num_nodes;
  st.S = S;
  st.res_id = a.take<int32_t>(c);
  st.res_next = a.take<int32_t>(c);
  st.addr = a.take<int32_t>(num_nodes);
  st.rhist = a.take<uint32_t>(S + 2);
  st.ihist = a.take<uint32_t>(S + 2);
  st.words = ceil_div(num_nodes, 32);
  st.parts = ceil_div(st.words, PART_WORDS);
  st.bitmap = a.take<uint32_t>(st.words);
  st.dead_bits = a.take<uint32_t>(st.words);
  st.sel_part = a.take<uint32_t>(st.parts);
  st.bitmap_in = a.take<uint32_t>(st.words);
  st.sel_part_in = a.take<uint32_t>(st.parts);
  st.dead_part = a.take<uint32_t>(st.parts);
  st.ctrl = a.take<Ctrl>(1);
  st.fault = a.take<int32_t>(1);
  w.evict_tiles = ceil_div(c, (int64_t)EVICT_TILE);
  st.evict_words = a.take<uint64_t>(w.evict_tiles * WAVE);
  w.in_tiles = ceil_div(max_n > 0 ? max_n : 1, (int64_t)TB * IN_ITEMS_MANY);
  st.evict_tiles = a.take<uint32_t>(w.evict_tiles);
  st.in_tiles = a.take<uint32_t>(w.in_tiles);
  w.max_change = max_n < c ? max_n : c;
  if (w.max_change < 1) w.max_change = 1;
  st.acc_line = a.take<int32_t>(max_n > 0 ? max_n : 1);
  st.pair = a.take<uint64_t>(w.max_change);
  st.max_change = w.max_change;
  Plan& pl = w.plan;
  pl.ins_words = ceil_div(t, 32);
  pl.ins_tile_count = ceil_div(pl.ins_words, TB);
  pl.cand_tile_count = ceil_div(st.words, TB);
  pl.ins_bits = a.take<uint32_t>(pl.ins_words);
  pl.ins_tiles = a.take<uint32_t>(pl.ins_tile_count + 1 + scan_scratch_elems(pl.ins_tile_count + 1));
  pl.ins_base = a.take<uint32_t>(pl.ins_words);
  pl.ins_cand = a.take<int32_t>(w.max_heads);
  pl.scalars = a.take<int64_t>(PLAN_SCALARS);
  pl.cand_tiles = a.take<uint32_t>(pl.cand_tile_count + 1 + scan_scratch_elems(pl.cand_tile_count + 1));
  pl.cand_base = a.take<uint32_t>(st.words);
  pl.cand_id = a.take<int32_t>(PLAN_CAND_MAX);
  pl.cand_line = a.take<int32_t>(PLAN_CAND_MAX);
  pl.cand_dead = a.take<uint32_t>(PLAN_CAND_WORDS);
  pl.arr_off = a.take<uint32_t>(S + 2);
  pl.arr_cur = a.take<uint32_t>(S + 1);
  pl.arr_cand = a.take<int32_t>(PLAN_CAND_MAX);
  w.bytes = (a.used + 255) & ~size_t(255);
  return w;
}

int32_t check_shape(int64_t num_nodes, int64_t total, int32_t S, int64_t cap, const char* who) {
  if (num_nodes <= 0 || num_nodes > INT32_MAX)
    return fail(GINEX_ERR_ARG, "%s: num_nodes=%lld out of range", who, (long long)num_nodes);
  if (S < 1 || S > 8191) return fail(GINEX_ERR_ARG, "%s: S=%d outside [1, 8191]", who, S);
  if (total < 0 || total > INT32_MAX)
    return fail(GINEX_ERR_ARG, "%s: total ids=%lld outside [0, 2^31)", who, (long long)total);
  if (cap < 0 || cap > INT32_MAX)
    return fail(GINEX_ERR_ARG, "%s: cap=%lld out of range", who, (long long)cap);
  return GINEX_OK;
}

}  // namespace
}  // namespace ginex

using namespace ginex;

extern "C" size_t ginex_changeset_workspace_bytes(int64_t num_nodes, int64_t total_ids, int32_t S,
                                                  int64_t cap) {
  if (check_shape(num_nodes, total_ids, S, cap, "ginex_changeset_workspace_bytes")) return 0;
  // the longest iteration is not known here: bound it by the total (and by num_nodes,
  // since the ids of one iteration are distinct)
  const int64_t max_n = total_ids < num_nodes ? total_ids : num_nodes;
  return carve(nullptr, num_nodes, total_ids, S, cap, max_n).bytes;
}

namespace ginex {
namespace {

// Both replacement policies share every kernel: a policy only decides the key an access
// leaves behind (Belady: its next accessed iteration; LRU: S-1-i, so that the least
// recently used rows hold the largest keys) and the key of the prefetched rows.
int32_t changeset_run(const char* who, bool lru, int64_t num_nodes, const int32_t* ids,
                      const int64_t* ids_offsets, int32_t S, int64_t cap, int32_t* init_ids,
                      int64_t* init_count, int32_t* in_ids, int32_t* out_ids,
                      int32_t* in_positions, int64_t cs_capacity, int64_t* cs_offsets,
                      int64_t* miss_count, int32_t* src_line, int64_t* total_changes,
                      int64_t* init_ready, const int32_t* start_ids, int32_t* final_ids, void* ws,
                      size_t ws_bytes, void* stream, bool allow_planned = true) {
  if (!ids_offsets || !init_count || !cs_offsets || !miss_count || !total_changes || !ws)
    return fail(GINEX_ERR_ARG, "%s: a required pointer is null", who);
  if (S >= 1 && ids_offsets[0] != 0)
    return fail(GINEX_ERR_INPUT, "%s: ids_offsets[0] must be 0", who);
  int64_t max_n = 0;
  for (int32_t i = 0; S >= 1 && i < S; ++i) {
    const int64_t n = ids_offsets[i + 1] - ids_offsets[i];
    if (n < 0) return fail(GINEX_ERR_INPUT, "%s: ids_offsets not monotone at %d", who, i);
    if (n > num_nodes)
      return fail(GINEX_ERR_INPUT, "%s: iteration %d has more ids than nodes", who, i);
    if (n > max_n) max_n = n;
  }
  const int64_t total = S >= 1 ? ids_offsets[S] : 0;
  if (int32_t rc = check_shape(num_nodes, total, S, cap, who)) return rc;
  if (total > 0 && !ids) return fail(GINEX_ERR_ARG, "%s: ids is null", who);
  if (cap > 0 && !init_ids && !start_ids)
    return fail(GINEX_ERR_ARG, "%s: init_ids is null", who);
  if (start_ids && cap < 1)
    return fail(GINEX_ERR_ARG, "%s: a carried cache needs cap >= 1", who);
  if (cs_capacity < 0 || (cs_capacity > 0 && (!in_ids || !out_ids || !in_positions)))
    return fail(GINEX_ERR_ARG, "%s: bad changeset output arrays", who);
  const int64_t bound = total < num_nodes ? total : num_nodes;
  Workspace w = carve(ws, num_nodes, total, S, cap, bound);
  if (ws_bytes < w.bytes)
    return fail(GINEX_ERR_WORKSPACE, "%s: workspace of %zu bytes given, %zu needed", who, ws_bytes,
                w.bytes);
  if ((uintptr_t)ws & 255) return fail(GINEX_ERR_ARG, "%s: workspace must be 256-byte aligned", who);
  hipStream_t st = (hipStream_t)stream;
  State& state = w.st;
  state.lru = lru ? 1 : 0;
  // Worth a tenth launch per iteration only where a pass over the cache lines is long;
  // GINEX_DEAD_SCATTER=0/1 overrides the choice (both ways give the same lists).
  const char* scatter_env = getenv("GINEX_DEAD_SCATTER");
  state.dead_scatter = !lru && (scatter_env ? scatter_env[0] == '1' : cap >= (int64_t(1) << 20));
  state.dead_only = 0;

  GINEX_HIP(hipMemcpyAsync(w.d_offsets, ids_offsets, sizeof(int64_t) * (S + 1),
                           hipMemcpyHostToDevice, st));
  GINEX_HIP(fill_async<int64_t>(miss_count, S, 0, st));
  GINEX_HIP(fill_async<int64_t>(cs_offsets, S + 1, 0, st));
  *init_count = start_ids ? cap : 0;
  *total_changes = 0;
  if (init_ready)
    for (int32_t i = 0; i < S; ++i) init_ready[i] = start_ids ? cap : 0;
  if (total == 0) {
    if (start_ids && final_ids)
      GINEX_HIP(hipMemcpyAsync(final_ids, start_ids, sizeof(int32_t) * cap,
                               hipMemcpyDeviceToDevice, st));
    GINEX_HIP(hipStreamSynchronize(st));
    return GINEX_OK;
  }

  // part 1: sort (node, position) by node, then look right
  // (the first pass reads the ids themselves and forms the pairs on the way)
  uint64_t* sorted = nullptr;
  const char* validate_env = getenv("GINEX_VALIDATE");
  const bool validate = validate_env && validate_env[0] == '1';
  // when validating, sort on all 32 id bits so that ids beyond num_nodes are ordered too
  GINEX_HIP(radix_sort_values_with_positions(ids, w.pairs_a, w.pairs_b, total,
                                             validate ? 64 : 32 + bits_for(num_nodes), w.hist, st,
                                             &sorted));
  if (validate) {
    unsigned long long bad[2] = {0, 0};
    GINEX_HIP(fill_async<unsigned long long>(w.d_counts, 2, 0ull, st));
    hipLaunchKernelGGL(k_validate, dim3((unsigned)ceil_div(total, TB)), dim3(TB),
                       sizeof(int32_t) * (S + 1), st, sorted, total, w.d_offsets, S, num_nodes,
                       w.d_counts);
    GINEX_LAUNCH_CHECK();
    GINEX_HIP(hipMemcpyAsync(bad, w.d_counts, sizeof(bad), hipMemcpyDeviceToHost, st));
    GINEX_HIP(hipStreamSynchronize(st));
    if (bad[0] || bad[1])
      return fail(GINEX_ERR_INPUT, "%s: %llu ids outside [0, %lld), %llu ids repeated inside an "
                  "iteration", who, bad[0], (long long)num_nodes, bad[1]);
  }
  hipLaunchKernelGGL(k_count_heads, dim3((unsigned)w.look_tiles), dim3(TB), 0, st, sorted, total,
                     w.head_tiles);
  GINEX_LAUNCH_CHECK();
  GINEX_HIP(fill_async<uint32_t>(w.head_tiles + w.look_tiles, 1, 0u, st));
  GINEX_HIP(exclusive_scan_inplace<uint32_t>(w.head_tiles, w.look_tiles + 1,
                                             w.head_tiles + w.look_tiles + 1, st));
  uint32_t distinct32 = 0;
  GINEX_HIP(hipMemcpyAsync(&distinct32, w.head_tiles + w.look_tiles, sizeof(uint32_t),
                           hipMemcpyDeviceToHost, st));
  GINEX_HIP(hipStreamSynchronize(st));
  const int64_t distinct = distinct32;
  if (distinct > w.max_heads)
    return fail(GINEX_ERR_INPUT, "%s: %lld distinct ids among %lld nodes: ids out of range?", who,
                (long long)distinct, (long long)num_nodes);

  // part 2: C_0
  const size_t off_lds = sizeof(int32_t) * (S + 1);
  hipLaunchKernelGGL(k_heads_write, dim3((unsigned)w.look_tiles), dim3(TB), off_lds, st, sorted,
                     total, w.d_offsets, S, w.head_tiles, w.heads_a);
  GINEX_LAUNCH_CHECK();
  uint64_t* heads = w.heads_a;
  if (!start_ids)   // C_0: the heads in order of first access
    GINEX_HIP(radix_sort_u64(w.heads_a, w.heads_b, distinct, 32, 32 + bits_for(S), w.hist, st,
                             &heads));
  const int64_t n_init = start_ids ? cap : (distinct < cap ? distinct : cap);
  *init_count = n_init;
  if (init_ready && n_init > 0 && !start_ids) {   // every path below waits for the stream before it returns
    hipLaunchKernelGGL(k_init_ready, dim3((unsigned)ceil_div(S, TB)), dim3(TB), 0, st, heads, n_init,
                       S, w.d_ready);
    GINEX_LAUNCH_CHECK();
    GINEX_HIP(hipMemcpyAsync(init_ready, w.d_ready, sizeof(int64_t) * S, hipMemcpyDeviceToHost,
                             st));
  }
  if (!start_ids && (distinct <= cap || cap == 0)) {
    // everything fits (no row ever misses), or there is no cache (every row misses and
    // nothing is inserted): all changesets are empty
    if (n_init > 0) {
      hipLaunchKernelGGL(k_copy_init, dim3((unsigned)ceil_div(n_init, TB)), dim3(TB), 0, st, heads,
                         n_init, init_ids);
      GINEX_LAUNCH_CHECK();
    }
    if (cap == 0) {
      hipLaunchKernelGGL(k_iteration_lengths, dim3((unsigned)ceil_div(S, TB)), dim3(TB), 0, st,
                         w.d_offsets, S, miss_count);
      GINEX_LAUNCH_CHECK();
      if (src_line) GINEX_HIP(fill_async<int32_t>(src_line, total, -1, st));
    } else if (src_line) {
      // every accessed row sits in the line of its rank for the whole superbatch
      hipLaunchKernelGGL(k_scatter_rank, dim3((unsigned)ceil_div(n_init, TB)), dim3(TB), 0, st,
                         heads, n_init, state.addr);
      hipLaunchKernelGGL(k_lookup_lines, dim3((unsigned)ceil_div(total, TB * 4)), dim3(TB), 0, st,
                         ids, total, state.addr, src_line);
      GINEX_LAUNCH_CHECK();
    }
    GINEX_HIP(hipStreamSynchronize(st));
    return GINEX_OK;
  }
  // A carried cache with room for every row of the superbatch never evicts a row that is
  // still needed: each iteration keeps all live candidates, so the threshold bucket is
  // "never" and the select runs on the dead rows.  The changesets then follow without a loop
  // over the state (the planned path; GINEX_PLANNED=0 switches it off); where that path does
  // not apply, the loop runs without the two launches of the live select.
  // GINEX_LIVE_SELECT=1 keeps them in, and the planned path out.  All ways give the same lists.
  const char* live_env = getenv("GINEX_LIVE_SELECT");
  const char* plan_env = getenv("GINEX_PLANNED");
  state.dead_only = start_ids && distinct <= cap && !(live_env && live_env[0] == '1');
  const bool planned = state.dead_only && allow_planned && S <= PLAN_S_MAX &&
                       !(plan_env && plan_env[0] == '0');
  // the cache cannot hold every row: Belady needs the next accessed iteration of every access
  // (the planned path reads what it needs from the sorted pairs)
  if (!lru && !planned) {
    hipLaunchKernelGGL(k_look_right, dim3((unsigned)w.look_tiles), dim3(TB), off_lds, st, sorted,
                       total, w.d_offsets, S, w.next_iter);
    GINEX_LAUNCH_CHECK();
  }
  GINEX_HIP(fill_async<int32_t>(state.fault, 1, 0, st));
  GINEX_HIP(fill_async<int32_t>(state.addr, num_nodes, -1, st));
  GINEX_HIP(fill_async<uint32_t>(state.rhist, S + 2, 0u, st));
  GINEX_HIP(fill_async<uint32_t>(state.ihist, S + 2, 0u, st));
  GINEX_HIP(fill_async<uint32_t>(state.bitmap, state.words, 0u, st));
  GINEX_HIP(fill_async<uint32_t>(state.dead_bits, state.words, 0u, st));
  GINEX_HIP(fill_async<uint32_t>(state.sel_part, state.parts, 0u, st));
  GINEX_HIP(fill_async<uint32_t>(state.bitmap_in, state.words, 0u, st));
  GINEX_HIP(fill_async<uint32_t>(state.sel_part_in, state.parts, 0u, st));
  GINEX_HIP(fill_async<uint32_t>(state.dead_part, state.parts, 0u, st));
  GINEX_HIP(fill_async<uint64_t>(state.pair, w.max_change, 0ull, st));
  if (state.dead_scatter)
    GINEX_HIP(fill_async<uint64_t>(state.evict_words, w.evict_tiles * WAVE, 0ull, st));
  {
    int64_t blocks = ceil_div(cap, TB * 8);
    if (blocks > 4096) blocks = 4096;
    if (start_ids) {
      unsigned long long bad = 0;
      GINEX_HIP(fill_async<int32_t>(w.first_of, num_nodes, S, st));
      GINEX_HIP(fill_async<unsigned long long>(w.d_counts, 1, 0ull, st));
      hipLaunchKernelGGL(k_scatter_first, dim3((unsigned)ceil_div(distinct, TB)), dim3(TB), 0, st,
                         heads, distinct, w.first_of);
      hipLaunchKernelGGL(k_init_state_resume, dim3((unsigned)blocks), dim3(TB),
                         sizeof(uint32_t) * (S + 1), st, start_ids, w.first_of, state, w.d_counts);
      GINEX_LAUNCH_CHECK();
      // the part counts of the dead rows the start state brought along
      hipLaunchKernelGGL(k_part_count, dim3((unsigned)state.parts), dim3(TB), 0, st,
                         state.dead_bits, state.words, state.dead_part);
      GINEX_LAUNCH_CHECK();
      GINEX_HIP(hipMemcpyAsync(&bad, w.d_counts, sizeof(bad), hipMemcpyDeviceToHost, st));
      GINEX_HIP(hipStreamSynchronize(st));
      if (bad)
        return fail(GINEX_ERR_INPUT, "%s: %llu entries of start_ids are out of range or repeated",
                    who, bad);
    } else {
      hipLaunchKernelGGL(k_init_state, dim3((unsigned)blocks), dim3(TB),
                         sizeof(uint32_t) * (S + 1), st, heads, cap, init_ids, state);
      GINEX_LAUNCH_CHECK();
    }
  }

  if (planned) {
    const Plan& pl = w.plan;
    GINEX_HIP(fill_async<uint32_t>(pl.ins_bits, pl.ins_words, 0u, st));
    GINEX_HIP(fill_async<uint32_t>(pl.arr_off, S + 2, 0u, st));
    GINEX_HIP(fill_async<uint32_t>(pl.cand_dead, PLAN_CAND_WORDS, 0u, st));
    {
      int64_t blocks = w.look_tiles < 512 ? w.look_tiles : 512;
      hipLaunchKernelGGL(k_plan_heads, dim3((unsigned)blocks), dim3(TB),
                         sizeof(int32_t) * (3 * (size_t)S + 1), st, sorted, total, w.d_offsets, S,
                         state.addr, pl.ins_bits, (unsigned long long*)miss_count,
                         (unsigned long long*)cs_offsets);
      hipLaunchKernelGGL(k_plan_scan, dim3(1), dim3(BIG), 0, st, state, sorted, total, cs_offsets,
                         pl.scalars);
      // the id bitmap of the candidates (in the select's scratch bitmap, which is all zero
      // here) and their number, still without the host
      int64_t tail_blocks = ceil_div(total, (int64_t)TB * 16);
      tail_blocks = tail_blocks < 1 ? 1 : (tail_blocks > 1024 ? 1024 : tail_blocks);
      hipLaunchKernelGGL(k_cand_start, dim3((unsigned)tail_blocks), dim3(TB), 0, st,
                         state.dead_bits, state.words, num_nodes, pl.scalars, state.bitmap);
      hipLaunchKernelGGL(k_plan_arrivals<false>, dim3((unsigned)tail_blocks), dim3(TB), 2 * off_lds, st,
                         sorted, total, pl.scalars, state.addr, w.d_offsets, S, state.bitmap,
                         pl.cand_base, num_nodes, pl, (int32_t*)nullptr);
      hipLaunchKernelGGL(k_plan_arrival_offsets, dim3(1), dim3(BIG), 0, st, pl.arr_off,
                         pl.arr_cur, S, pl.scalars);
      GINEX_LAUNCH_CHECK();
    }
    int64_t sc[PLAN_SCALARS] = {};
    GINEX_HIP(hipMemcpyAsync(sc, pl.scalars, sizeof(sc), hipMemcpyDeviceToHost, st));
    GINEX_HIP(hipStreamSynchronize(st));
    const int64_t M = sc[PLAN_M], lo_id = sc[PLAN_LO_ID];
    // the replay in LDS where its arrays hold the call, else (or with GINEX_PLANNED=2) the
    // steps on the bitmap in global memory; neither with fewer dead rows than insertions
    const bool stepped = M > 0 && lo_id >= 0 &&
                         ((plan_env && plan_env[0] == '2') || sc[PLAN_MAX_N] > PLAN_SORT_MAX ||
                          sc[PLAN_CANDS] > PLAN_CAND_MAX);
    const bool fits = M == 0 || lo_id >= 0;
    // GINEX_TRACE=1: one line on stderr that says which way the call went
    const char* trace_env = getenv("GINEX_TRACE");
    const bool trace = trace_env && trace_env[0] == '1';
    if (trace)
      fprintf(stderr, "[ginex] %s: %lld insertions, at most %lld per iteration, %lld rows dead from "
              "the start, lowest possible victim %lld of %lld ids, %lld candidates: %s\n", who,
              (long long)M, (long long)sc[PLAN_MAX_N], (long long)sc[PLAN_DEAD], (long long)lo_id,
              (long long)num_nodes, (long long)sc[PLAN_CANDS],
              !fits ? "loop" : stepped ? "stepped path" : "planned path");
    if (fits) {
      *total_changes = M;
      if (M > cs_capacity)
        return fail(GINEX_ERR_CAPACITY, "%s: %lld changeset records, capacity %lld", who,
                    (long long)M, (long long)cs_capacity);
      if (M > 0) {
        // the insertion lists
        hipLaunchKernelGGL(k_bit_tiles, dim3((unsigned)pl.ins_tile_count), dim3(TB), 0, st,
                           pl.ins_bits, pl.ins_words, pl.ins_tiles);
        GINEX_LAUNCH_CHECK();
        GINEX_HIP(fill_async<uint32_t>(pl.ins_tiles + pl.ins_tile_count, 1, 0u, st));
        GINEX_HIP(exclusive_scan_inplace<uint32_t>(pl.ins_tiles, pl.ins_tile_count + 1,
                                                   pl.ins_tiles + pl.ins_tile_count + 1, st));
        hipLaunchKernelGGL(k_ins_emit, dim3((unsigned)pl.ins_tile_count), dim3(TB), off_lds, st,
                           pl.ins_bits, pl.ins_words, pl.ins_tiles, ids, w.d_offsets, S, in_ids,
                           in_positions, pl.ins_base, pl.ins_cand);
        GINEX_LAUNCH_CHECK();
        int64_t tail_blocks = ceil_div(total - sc[PLAN_TAIL], TB);
        tail_blocks = tail_blocks < 1 ? 1 : (tail_blocks > 1024 ? 1024 : tail_blocks);
        if (stepped) {
          // the rows that die, as ids grouped by iteration (in the array that holds the
          // candidate numbers of the insertions for the replay, which does not run)
          int32_t* const arr_ids = pl.ins_cand;
          hipLaunchKernelGGL(k_plan_arrivals<true>, dim3((unsigned)tail_blocks), dim3(TB),
                             2 * off_lds, st, sorted, total, pl.scalars, state.addr, w.d_offsets, S,
                             state.bitmap, pl.cand_base, num_nodes, pl, arr_ids);
          GINEX_LAUNCH_CHECK();
          std::vector<int64_t> cs(S + 1);
          std::vector<uint32_t> arr(S + 2);
          GINEX_HIP(hipMemcpyAsync(cs.data(), cs_offsets, sizeof(int64_t) * (S + 1),
                                   hipMemcpyDeviceToHost, st));
          GINEX_HIP(hipMemcpyAsync(arr.data(), pl.arr_off, sizeof(uint32_t) * (S + 1),
                                   hipMemcpyDeviceToHost, st));
          GINEX_HIP(hipStreamSynchronize(st));
          arr[S + 1] = arr[S];
          if (!state.dead_scatter)
            GINEX_HIP(fill_async<uint64_t>(state.evict_words, w.evict_tiles * WAVE, 0ull, st));
          const int64_t evict_blocks = ceil_div(w.evict_tiles, TB / WAVE);
          int64_t scatter_blocks = ceil_div(state.words, TB);
          scatter_blocks = scatter_blocks > 256 ? 256 : scatter_blocks;
          auto arrive_blocks = [](uint32_t count) {
            const int64_t b = ceil_div((int64_t)count, TB);
            return (unsigned)(b < 1 ? 1 : (b > 64 ? 64 : b));
          };
          if (arr[1] > arr[0])
            hipLaunchKernelGGL(k_step_arrive, dim3(arrive_blocks(arr[1] - arr[0])), dim3(TB), 0, st,
                               state, arr_ids, arr[0], arr[1]);
          for (int32_t i = 0; i < S; ++i) {
            const int64_t n = cs[i + 1] - cs[i];
            const uint32_t a0 = arr[i + 1], a1 = i + 1 < S ? arr[i + 2] : arr[i + 1];
            if (n > 0) {
              hipLaunchKernelGGL(k_step_find, dim3(1), dim3(BIG), 0, st, state, n, w.evict_tiles);
              hipLaunchKernelGGL(k_step_scatter, dim3((unsigned)scatter_blocks), dim3(TB), 0, st,
                                 state);
              hipLaunchKernelGGL(k_step_emit,
                                 dim3((unsigned)evict_blocks + (a1 > a0 ? arrive_blocks(a1 - a0) : 0u)),
                                 dim3(TB), 0, st, state, w.evict_tiles, evict_blocks, cs[i], in_ids,
                                 out_ids, arr_ids, a0, a1);
            } else if (a1 > a0) {
              hipLaunchKernelGGL(k_step_arrive, dim3(arrive_blocks(a1 - a0)), dim3(TB), 0, st, state,
                                 arr_ids, a0, a1);
            }
          }
          GINEX_LAUNCH_CHECK();
          // (a step that met fewer dead rows than insertions leaves its mark in the word the
          // copy below brings over beside the replay's)
          hipLaunchKernelGGL(k_step_verdict, dim3(1), dim3(1), 0, st, state.fault, pl.scalars);
          GINEX_LAUNCH_CHECK();
        } else {
        // the candidates numbered in id order
        const int64_t lo_word = lo_id >> 5;
        const int64_t nwords = state.words - lo_word;
        const int64_t ctiles = ceil_div(nwords, TB);
        hipLaunchKernelGGL(k_bit_tiles, dim3((unsigned)ctiles), dim3(TB), 0, st,
                           state.bitmap + lo_word, nwords, pl.cand_tiles);
        GINEX_LAUNCH_CHECK();
        GINEX_HIP(fill_async<uint32_t>(pl.cand_tiles + ctiles, 1, 0u, st));
        GINEX_HIP(exclusive_scan_inplace<uint32_t>(pl.cand_tiles, ctiles + 1,
                                                   pl.cand_tiles + ctiles + 1, st));
        hipLaunchKernelGGL(k_cand_emit, dim3((unsigned)ctiles), dim3(TB), 0, st, state.bitmap,
                           state.dead_bits, lo_word, nwords, pl.cand_tiles, state.addr, pl);
        hipLaunchKernelGGL(k_plan_arrivals<true>, dim3((unsigned)tail_blocks), dim3(TB), 2 * off_lds, st,
                           sorted, total, pl.scalars, state.addr, w.d_offsets, S, state.bitmap,
                           pl.cand_base, num_nodes, pl, (int32_t*)nullptr);
        hipLaunchKernelGGL(k_plan_replay, dim3(1), dim3(BIG), 0, st, state, pl, ctiles, cs_offsets,
                           in_ids, out_ids);
        GINEX_LAUNCH_CHECK();
        }
      }
      if (src_line) {
        // every row has one line for the whole superbatch: the start state's or the one it was given
        hipLaunchKernelGGL(k_lookup_lines, dim3((unsigned)ceil_div(total, TB * 4)), dim3(TB), 0, st,
                           ids, total, state.addr, src_line);
        if (M > 0)
          hipLaunchKernelGGL(k_ins_lines, dim3((unsigned)pl.ins_tile_count), dim3(TB), 0, st,
                             pl.ins_bits, pl.ins_words, src_line);
        GINEX_LAUNCH_CHECK();
      }
      if (final_ids)
        GINEX_HIP(hipMemcpyAsync(final_ids, state.res_id, sizeof(int32_t) * cap,
                                 hipMemcpyDeviceToDevice, st));
      int64_t failed[2] = {0, 0};
      GINEX_HIP(hipMemcpyAsync(failed, pl.scalars + PLAN_FAILED, sizeof(failed),
                               hipMemcpyDeviceToHost, st));
      GINEX_HIP(hipStreamSynchronize(st));
      if (!failed[0]) return GINEX_OK;
      if (trace)
        fprintf(stderr, "[ginex] %s: the replay gave up (reason %lld, iteration %lld), loop\n", who,
                (long long)failed[0], (long long)failed[1]);
      // the replay gave up, possibly after it had changed the state: start over, through the loop
      return changeset_run(who, lru, num_nodes, ids, ids_offsets, S, cap, init_ids, init_count,
                           in_ids, out_ids, in_positions, cs_capacity, cs_offsets, miss_count,
                           src_line, total_changes, init_ready, start_ids, final_ids, ws, ws_bytes,
                           stream, false);
    }
    // not for this path: the loop, from the untouched start state
    GINEX_HIP(fill_async<uint32_t>(state.bitmap, state.words, 0u, st));
    GINEX_HIP(fill_async<int64_t>(miss_count, S, 0, st));
    GINEX_HIP(fill_async<int64_t>(cs_offsets, S + 1, 0, st));
    hipLaunchKernelGGL(k_look_right, dim3((unsigned)w.look_tiles), dim3(TB), off_lds, st, sorted,
                       total, w.d_offsets, S, w.next_iter);
    GINEX_LAUNCH_CHECK();
  }

  // part 3: the recurrence, with no host round trip between iterations
  const size_t touch_lds = sizeof(uint32_t) * 2 * (S + 1);
  Outputs outs{in_ids, out_ids, in_positions, cs_capacity, cs_offsets, miss_count};
  // Belady with a cache that does not hold the superbatch: the threshold bucket of every
  // iteration from histograms of next_iter alone, in front of the loop (GINEX_STATIC_THRESHOLDS=0:
  // from histograms of the state, iteration by iteration, as LRU needs it)
  const char* static_env = getenv("GINEX_STATIC_THRESHOLDS");
  const bool static_thresholds = !lru && !state.dead_only && S <= STATIC_S_MAX &&
                                 !(static_env && static_env[0] == '0');
  if (static_thresholds) {
    int64_t longest = 0;
    for (int32_t i = 0; i < S; ++i)
      longest = std::max<int64_t>(longest, ids_offsets[i + 1] - ids_offsets[i]);
    GINEX_HIP(fill_async<uint32_t>(w.key_hists, (int64_t)S * (S + 1), 0u, st));
    GINEX_HIP(fill_async<uint32_t>(w.touch_ctr, 2, 0u, st));
    if (longest > 0)
      hipLaunchKernelGGL(k_key_hists, dim3((unsigned)ceil_div(longest, TB * TOUCH_ITEMS), (unsigned)S),
                         dim3(TB), sizeof(uint32_t) * (S + 1), st, w.next_iter, w.d_offsets, S,
                         w.key_hists);
    hipLaunchKernelGGL(k_static_roll, dim3(1), dim3(BIG), 0, st, state, w.key_hists, w.d_offsets,
                       w.static_plan, miss_count);
    GINEX_LAUNCH_CHECK();
  }
  {
    const int64_t res_blocks = ceil_div(cap, TB * MARK_ITEMS);
    const int64_t evict_blocks = ceil_div(w.evict_tiles, TB / WAVE);
    for (int32_t i = 0; i < S; ++i) {
      Iter it;
      const int64_t lo = ids_offsets[i];
      it.ids = ids + lo;
      it.next = w.next_iter + lo;
      it.n = ids_offsets[i + 1] - lo;
      it.i = i;
      it.key = lru ? S - 1 - i : -1;
      it.lo_bin = lru ? S - 1 - i : i + 1;
      it.src_line = src_line ? src_line + lo : nullptr;
      if (static_thresholds) {
        if (it.n > 0) {
          if (it.n < TOUCH_FEW) {
            const int64_t touch_blocks = ceil_div(it.n, TB * 4);
            hipLaunchKernelGGL(k_touch_static<4>, dim3((unsigned)(touch_blocks + res_blocks)), dim3(TB),
                               0, st, state, it, w.static_plan, w.touch_ctr, touch_blocks);
          } else {
            const int64_t touch_blocks = ceil_div(it.n, TB * 8);
            hipLaunchKernelGGL(k_touch_static<8>, dim3((unsigned)(touch_blocks + res_blocks)), dim3(TB),
                               0, st, state, it, w.static_plan, w.touch_ctr, touch_blocks);
          }
        }
        hipLaunchKernelGGL(k_decide, dim3(1), dim3(BIG), 0, st, state, i, w.static_plan, w.touch_ctr,
                           outs, w.evict_tiles);
        GINEX_LAUNCH_CHECK();
        if (it.n == 0) continue;
        if (it.n < TOUCH_FEW) {
          const int64_t in_tiles = ceil_div(it.n, (int64_t)TB * IN_ITEMS);
          hipLaunchKernelGGL(k_flags<IN_ITEMS>, dim3((unsigned)(w.evict_tiles + in_tiles + 1)), dim3(TB),
                             0, st, state, it, w.evict_tiles, in_tiles);
          hipLaunchKernelGGL(k_emit_pair<IN_ITEMS>, dim3((unsigned)(evict_blocks + in_tiles)), dim3(TB),
                             0, st, state, it, outs, w.evict_tiles);
        } else {
          const int64_t in_tiles = ceil_div(it.n, (int64_t)TB * IN_ITEMS_MANY);
          hipLaunchKernelGGL(k_flags<IN_ITEMS_MANY>, dim3((unsigned)(w.evict_tiles + in_tiles + 1)),
                             dim3(TB), 0, st, state, it, w.evict_tiles, in_tiles);
          hipLaunchKernelGGL(k_emit_pair<IN_ITEMS_MANY>, dim3((unsigned)(evict_blocks + in_tiles)),
                             dim3(TB), 0, st, state, it, outs, w.evict_tiles);
        }
        GINEX_LAUNCH_CHECK();
        continue;
      }
      if (it.n > 0) {
        hipLaunchKernelGGL(k_touch, dim3((unsigned)ceil_div(it.n, TB * TOUCH_ITEMS)), dim3(TB),
                           touch_lds, st, state, it, (unsigned long long*)(miss_count + i));
        GINEX_LAUNCH_CHECK();
      }
      hipLaunchKernelGGL(k_threshold, dim3(1), dim3(BIG), 0, st, state, i, it.lo_bin, outs,
                         w.evict_tiles);
      GINEX_LAUNCH_CHECK();
      if (it.n == 0) continue;  // nothing missed, nothing changes
      const int64_t in_tiles = ceil_div(it.n, (int64_t)TB * IN_ITEMS);
      if (!state.dead_only) {
        hipLaunchKernelGGL(k_mark, dim3((unsigned)(res_blocks + ceil_div(it.n, TB * MARK_ITEMS))),
                           dim3(TB), 0, st, state, it, res_blocks);
        hipLaunchKernelGGL(k_find, dim3(1), dim3(BIG), 0, st, state);
        GINEX_LAUNCH_CHECK();
      }
      hipLaunchKernelGGL(k_flags<IN_ITEMS>, dim3((unsigned)(w.evict_tiles + in_tiles + 1)), dim3(TB), 0,
                         st, state, it, w.evict_tiles, in_tiles);
      hipLaunchKernelGGL(k_emit_pair<IN_ITEMS>, dim3((unsigned)(evict_blocks + in_tiles)), dim3(TB), 0, st,
                         state, it, outs, w.evict_tiles);
      GINEX_LAUNCH_CHECK();
    }
  }
  if (start_ids && final_ids)
    GINEX_HIP(hipMemcpyAsync(final_ids, state.res_id, sizeof(int32_t) * cap,
                             hipMemcpyDeviceToDevice, st));
  GINEX_HIP(hipMemcpyAsync(total_changes, cs_offsets + S, sizeof(int64_t), hipMemcpyDeviceToHost,
                           st));
  int32_t fault = 0;
  GINEX_HIP(hipMemcpyAsync(&fault, state.fault, sizeof(fault), hipMemcpyDeviceToHost, st));
  GINEX_HIP(hipStreamSynchronize(st));
  if (fault)
    return fail(GINEX_ERR_INPUT, "%s: an iteration needed a select among live rows although all "
                "%lld rows of the superbatch fit the cache of %lld lines: ids repeated inside an "
                "iteration?", who, (long long)distinct, (long long)cap);
  if (*total_changes > cs_capacity)
    return fail(GINEX_ERR_CAPACITY, "%s: %lld changeset records, capacity %lld", who,
                (long long)*total_changes, (long long)cs_capacity);
  return GINEX_OK;
}

}  // namespace
}  // namespace ginex

extern "C" int32_t ginex_changeset(int64_t num_nodes, const int32_t* ids,
                                   const int64_t* ids_offsets, int32_t S, int64_t cap,
                                   int32_t* init_ids, int64_t* init_count, int32_t* in_ids,
                                   int32_t* out_ids, int32_t* in_positions, int64_t cs_capacity,
                                   int64_t* cs_offsets, int64_t* miss_count, int32_t* src_line,
                                   int64_t* total_changes, int64_t* init_ready, void* ws,
                                   size_t ws_bytes, void* stream) {
  return changeset_run("ginex_changeset", false, num_nodes, ids, ids_offsets, S, cap, init_ids,
                       init_count, in_ids, out_ids, in_positions, cs_capacity, cs_offsets,
                       miss_count, src_line, total_changes, init_ready, nullptr, nullptr, ws,
                       ws_bytes, stream);
}

extern "C" int32_t ginex_changeset_resume(int64_t num_nodes, const int32_t* ids,
                                          const int64_t* ids_offsets, int32_t S, int64_t cap,
                                          const int32_t* start_ids, int32_t* final_ids,
                                          int32_t* in_ids, int32_t* out_ids,
                                          int32_t* in_positions, int64_t cs_capacity,
                                          int64_t* cs_offsets, int64_t* miss_count,
                                          int32_t* src_line, int64_t* total_changes, void* ws,
                                          size_t ws_bytes, void* stream) {
  if (!start_ids)
    return fail(GINEX_ERR_ARG, "ginex_changeset_resume: start_ids is null");
  int64_t init_count = 0;
  return changeset_run("ginex_changeset_resume", false, num_nodes, ids, ids_offsets, S, cap,
                       nullptr, &init_count, in_ids, out_ids, in_positions, cs_capacity,
                       cs_offsets, miss_count, src_line, total_changes, nullptr, start_ids,
                       final_ids, ws, ws_bytes, stream);
}

extern "C" int32_t ginex_changeset_lru(int64_t num_nodes, const int32_t* ids,
                                       const int64_t* ids_offsets, int32_t S, int64_t cap,
                                       int32_t* init_ids, int64_t* init_count, int32_t* in_ids,
                                       int32_t* out_ids, int32_t* in_positions,
                                       int64_t cs_capacity, int64_t* cs_offsets,
                                       int64_t* miss_count, int32_t* src_line,
                                       int64_t* total_changes, int64_t* init_ready, void* ws,
                                       size_t ws_bytes, void* stream) {
  return changeset_run("ginex_changeset_lru", true, num_nodes, ids, ids_offsets, S, cap, init_ids,
                       init_count, in_ids, out_ids, in_positions, cs_capacity, cs_offsets,
                       miss_count, src_line, total_changes, init_ready, nullptr, nullptr, ws,
                       ws_bytes, stream);
}

// ---- the variant that allocates nothing ------------------------------------------------
//
// The workspace of ginex_changeset_noalloc is a static device array.  Every GPU the library
// runs on holds its own copy at its own address until the process ends; in host code the
// array's name is only a stand-in for the symbol, so the device address is looked up once per
// device (with that device current) and that pointer is what the kernels are given.
static __device__ __align__(256) unsigned char scratch[GINEX_NOALLOC_SCRATCH_BYTES];

namespace ginex {
namespace {

constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[MAX_DEVICES] = {};

int32_t scratch_for_current_device(const char* who, void** out) {
  int device = -1;
  GINEX_HIP(hipGetDevice(&device));
  if (device < 0 || device >= MAX_DEVICES)
    return fail(GINEX_ERR_HIP, "%s: device index %d outside [0, %d)", who, device, MAX_DEVICES);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    void* ptr = nullptr;
    GINEX_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return fail(GINEX_ERR_HIP, "%s: the scratch array has no device address", who);
    g_scratch_ptr[device] = ptr;
  }
  *out = g_scratch_ptr[device];
  return GINEX_OK;
}

}  // namespace
}  // namespace ginex

extern "C" int32_t ginex_changeset_noalloc(int64_t num_nodes, const int32_t* ids,
                                           const int64_t* ids_offsets, int32_t S, int64_t cap,
                                           int32_t* init_ids, int64_t* init_count,
                                           int32_t* in_ids, int32_t* out_ids,
                                           int32_t* in_positions, int64_t cs_capacity,
                                           int64_t* cs_offsets, int64_t* miss_count,
                                           int32_t* src_line, int64_t* total_changes,
                                           int64_t* init_ready, void* stream) {
  const char* who = "ginex_changeset_noalloc";
  if (!ids_offsets) return fail(GINEX_ERR_ARG, "%s: ids_offsets is null", who);
  const int64_t total = S >= 1 ? ids_offsets[S] : 0;
  if (int32_t rc = check_shape(num_nodes, total, S, cap, who)) return rc;
  const int64_t bound = total < num_nodes ? total : num_nodes;
  const size_t need = carve(nullptr, num_nodes, total, S, cap, bound).bytes;
  if (need > (size_t)GINEX_NOALLOC_SCRATCH_BYTES)
    return fail(GINEX_ERR_WORKSPACE,
                "%s: this shape (num_nodes=%lld, %lld ids, S=%d, cap=%lld) needs %zu bytes of "
                "scratch, the built-in array holds %zu: use ginex_changeset with a workspace", who,
                (long long)num_nodes, (long long)total, S, (long long)cap, need,
                (size_t)GINEX_NOALLOC_SCRATCH_BYTES);
  void* ws = nullptr;
  if (int32_t rc = scratch_for_current_device(who, &ws)) return rc;
  return changeset_run(who, false, num_nodes, ids, ids_offsets, S, cap, init_ids, init_count,
                       in_ids, out_ids, in_positions, cs_capacity, cs_offsets, miss_count,
                       src_line, total_changes, init_ready, nullptr, nullptr, ws,
                       (size_t)GINEX_NOALLOC_SCRATCH_BYTES, stream);
}
