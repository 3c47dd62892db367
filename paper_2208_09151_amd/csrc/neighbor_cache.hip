// Neighbour cache construction (Section 3.2): rank the nodes by out-degree / in-degree and
// lay the rows of the best ones out as (count, neighbours) records behind a direct-address
// table.  A one-off set-up step, bound by one pass over `indices` (which may come over the
// host link) and two 32-bit radix sorts of one word per node.
#include "common.hpp"
#include "primitives.hpp"

namespace ginex {
namespace {

constexpr int TB = 256;

__device__ __forceinline__ int64_t off_at(const void* offsets, int off64, int64_t v) {
  return off64 ? static_cast<const int64_t*>(offsets)[v]
               : (int64_t) static_cast<const int32_t*>(offsets)[v];
}

// floor(out * 2^32 / in), complemented so that an ascending sort puts the largest ratio
// first.  A node without in-neighbours sorts last.
__device__ __forceinline__ uint64_t sort_key(uint32_t out_degree, int64_t in_degree) {
  const uint64_t ratio = in_degree > 0 ? ((uint64_t)out_degree << 32) / (uint64_t)in_degree : 0;
  return ~ratio;
}

// items[v] = (low half of the key << 32) | v: sorted first on the low half ...
__global__ __launch_bounds__(TB) void k_items_low(const void* __restrict__ offsets, int off64,
                                                  const uint32_t* __restrict__ out_degree,
                                                  int64_t num_nodes, uint64_t* __restrict__ items) {
  const int64_t v = (int64_t)blockIdx.x * TB + threadIdx.x;
  if (v >= num_nodes) return;
  const uint64_t key = sort_key(out_degree[v], off_at(offsets, off64, v + 1) - off_at(offsets, off64, v));
  items[v] = (key << 32) | (uint64_t)v;
}

// ... then, the sort being stable, on the high half.
__global__ __launch_bounds__(TB) void k_items_high(const void* __restrict__ offsets, int off64,
                                                   const uint32_t* __restrict__ out_degree,
                                                   int64_t num_nodes, uint64_t* __restrict__ items) {
  const int64_t j = (int64_t)blockIdx.x * TB + threadIdx.x;
  if (j >= num_nodes) return;
  const uint64_t v = items[j] & 0xFFFFFFFFull;
  const uint64_t key = sort_key(out_degree[v], off_at(offsets, off64, v + 1) - off_at(offsets, off64, v));
  items[j] = (key & 0xFFFFFFFF00000000ull) | v;
}

// Entries the record of the node at rank j would take: 1 + in-degree; 0 = not cacheable.
__global__ __launch_bounds__(TB) void k_costs(const uint64_t* __restrict__ ranked,
                                              const void* __restrict__ offsets, int off64,
                                              int64_t num_nodes, int64_t* __restrict__ cost) {
  const int64_t j = (int64_t)blockIdx.x * TB + threadIdx.x;
  if (j >= num_nodes) return;
  const int64_t v = (int64_t)(ranked[j] & 0xFFFFFFFFull);
  const int64_t in_degree = off_at(offsets, off64, v + 1) - off_at(offsets, off64, v);
  cost[j] = in_degree > 0 ? 1 + in_degree : 0;
}

// `start` = exclusive prefix sum of the costs in rank order.  The records that end inside
// the budget form a prefix of the ranking, since a record that does not fit pushes the
// start of every later one beyond the budget.
__global__ __launch_bounds__(TB) void k_place(const uint64_t* __restrict__ ranked,
                                              const int64_t* __restrict__ start,
                                              const void* __restrict__ offsets, int off64,
                                              int64_t num_nodes, int64_t budget,
                                              int64_t* __restrict__ address_table,
                                              int32_t* __restrict__ cache_array,
                                              unsigned long long* __restrict__ counters) {
  __shared__ unsigned long long red[2][TB / WAVE];
  const int64_t j = (int64_t)blockIdx.x * TB + threadIdx.x;
  unsigned long long nodes = 0, entries = 0;
  bool placed = false;
  if (j < num_nodes) {
    const int64_t v = (int64_t)(ranked[j] & 0xFFFFFFFFull);
    const int64_t in_degree = off_at(offsets, off64, v + 1) - off_at(offsets, off64, v);
    const int64_t at = start[j];
    if (in_degree > 0 && at + 1 + in_degree <= budget) {
      address_table[v] = at;
      cache_array[at] = (int32_t)in_degree;
      nodes = 1;
      entries = 1 + (unsigned long long)in_degree;
      placed = true;
    } else {
      address_table[v] = -1;
    }
  }
  nodes = wave_reduce_sum(nodes);
  entries = wave_reduce_sum(entries);
  if (lane_id() == 0) {
    red[0][threadIdx.x / WAVE] = nodes;
    red[1][threadIdx.x / WAVE] = entries;
  }
  __syncthreads();
  if (threadIdx.x < 2) {
    unsigned long long s = 0;
    for (int w = 0; w < TB / WAVE; ++w) s += red[threadIdx.x][w];
    if (s) atomicAdd(&counters[threadIdx.x], s);
  }
  // counters[2]: one past the last rank that was placed (ranks rise with the lane, so the
  // highest placed lane of a wave speaks for it)
  const uint64_t placed_lanes = __ballot(placed);
  if (placed_lanes && lane_id() == 63 - __clzll(placed_lanes))
    atomicMax(&counters[2], (unsigned long long)(j + 1));
}

// One wave per rank below `ranks` (one past the last cached rank): copy the node's row
// behind its count.
__global__ __launch_bounds__(TB) void k_copy_rows(const uint64_t* __restrict__ ranked,
                                                  int64_t ranks, const void* __restrict__ offsets,
                                                  int off64, const int32_t* __restrict__ indices,
                                                  const int64_t* __restrict__ address_table,
                                                  int32_t* __restrict__ cache_array) {
  const int64_t j = (int64_t)blockIdx.x * (TB / WAVE) + threadIdx.x / WAVE;
  if (j >= ranks) return;
  const int64_t v = (int64_t)(ranked[j] & 0xFFFFFFFFull);
  const int64_t at = address_table[v];
  if (at < 0) return;   // a node without neighbours among the cached ranks
  const int64_t lo = off_at(offsets, off64, v);
  const int64_t in_degree = off_at(offsets, off64, v + 1) - lo;
  for (int64_t t = lane_id(); t < in_degree; t += WAVE) cache_array[at + 1 + t] = indices[lo + t];
}

struct Workspace {
  uint32_t* out_degree;
  uint64_t* items_a;
  uint64_t* items_b;
  int64_t* cost;
  int64_t* scan_scratch;
  uint32_t* hist;
  unsigned long long* counters;
  size_t bytes;
};

Workspace carve(void* base, int64_t num_nodes) {
  Arena a(base);
  Workspace w;
  w.out_degree = a.take<uint32_t>(num_nodes);
  w.items_a = a.take<uint64_t>(num_nodes);
  w.items_b = a.take<uint64_t>(num_nodes);
  w.cost = a.take<int64_t>(num_nodes);
  w.scan_scratch = a.take<int64_t>(scan_scratch_elems(num_nodes));
  w.hist = a.take<uint32_t>(radix_plan(num_nodes).hist_elems);
  w.counters = a.take<unsigned long long>(4);
  w.bytes = (a.used + 255) & ~size_t(255);
  return w;
}

}  // namespace
}  // namespace ginex

using namespace ginex;

extern "C" size_t ginex_neighbor_cache_workspace_bytes(int64_t num_nodes) {
  if (num_nodes <= 0 || num_nodes > INT32_MAX) {
    set_error("ginex_neighbor_cache_workspace_bytes: num_nodes=%lld out of range",
              (long long)num_nodes);
    return 0;
  }
  return carve(nullptr, num_nodes).bytes;
}

extern "C" int32_t ginex_neighbor_cache_build(const ginex_csr_t* g, int64_t budget,
                                              int64_t* address_table, int32_t* cache_array,
                                              int64_t* cached_nodes, int64_t* used_entries,
                                              void* ws, size_t ws_bytes, void* stream) {
  const char* who = "ginex_neighbor_cache_build";
  if (!g || !g->offsets || (g->num_edges > 0 && !g->indices))
    return fail(GINEX_ERR_ARG, "%s: graph descriptor or its arrays are null", who);
  if (!address_table || !cached_nodes || !used_entries || !ws)
    return fail(GINEX_ERR_ARG, "%s: a required pointer is null", who);
  if (g->num_nodes <= 0 || g->num_nodes > INT32_MAX)
    return fail(GINEX_ERR_ARG, "%s: num_nodes=%lld out of range", who, (long long)g->num_nodes);
  if (g->num_edges < 0) return fail(GINEX_ERR_ARG, "%s: negative num_edges", who);
  if (budget < 0 || (budget > 0 && !cache_array))
    return fail(GINEX_ERR_ARG, "%s: bad budget or cache_array null", who);
  const int64_t n = g->num_nodes;
  const Workspace w = carve(ws, n);
  if (ws_bytes < w.bytes)
    return fail(GINEX_ERR_WORKSPACE, "%s: workspace of %zu bytes given, %zu needed", who, ws_bytes,
                w.bytes);
  if ((uintptr_t)ws & 255) return fail(GINEX_ERR_ARG, "%s: workspace must be 256-byte aligned", who);
  hipStream_t st = (hipStream_t)stream;
  const int off64 = g->offsets_64 ? 1 : 0;
  const unsigned node_blocks = (unsigned)ceil_div(n, TB);

  GINEX_HIP(fill_async<uint32_t>(w.out_degree, n, 0u, st));
  GINEX_HIP(fill_async<unsigned long long>(w.counters, 4, 0ull, st));
  GINEX_HIP(occurrences_async(g->indices, g->num_edges, n, w.out_degree, w.counters + 3, st));
  hipLaunchKernelGGL(k_items_low, dim3(node_blocks), dim3(TB), 0, st, g->offsets, off64,
                     w.out_degree, n, w.items_a);
  GINEX_LAUNCH_CHECK();
  uint64_t* half = nullptr;
  GINEX_HIP(radix_sort_u64(w.items_a, w.items_b, n, 32, 64, w.hist, st, &half));
  hipLaunchKernelGGL(k_items_high, dim3(node_blocks), dim3(TB), 0, st, g->offsets, off64,
                     w.out_degree, n, half);
  GINEX_LAUNCH_CHECK();
  uint64_t* ranked = nullptr;
  GINEX_HIP(radix_sort_u64(half, half == w.items_a ? w.items_b : w.items_a, n, 32, 64, w.hist, st,
                           &ranked));
  hipLaunchKernelGGL(k_costs, dim3(node_blocks), dim3(TB), 0, st, ranked, g->offsets, off64, n,
                     w.cost);
  GINEX_LAUNCH_CHECK();
  GINEX_HIP(exclusive_scan_inplace<int64_t>(w.cost, n, w.scan_scratch, st));
  hipLaunchKernelGGL(k_place, dim3(node_blocks), dim3(TB), 0, st, ranked, w.cost, g->offsets, off64,
                     n, budget, address_table, cache_array, w.counters);
  GINEX_LAUNCH_CHECK();
  unsigned long long counts[4] = {0, 0, 0, 0};
  GINEX_HIP(hipMemcpyAsync(counts, w.counters, sizeof(counts), hipMemcpyDeviceToHost, st));
  GINEX_HIP(hipStreamSynchronize(st));
  if (counts[3])
    return fail(GINEX_ERR_INPUT, "%s: %llu entries of indices outside [0, %lld)", who, counts[3],
                (long long)n);
  *cached_nodes = (int64_t)counts[0];
  *used_entries = (int64_t)counts[1];
  if (counts[0] > 0) {
    const int64_t ranks = (int64_t)counts[2];
    hipLaunchKernelGGL(k_copy_rows, dim3((unsigned)ceil_div(ranks, TB / WAVE)), dim3(TB), 0, st,
                       ranked, ranks, g->offsets, off64, g->indices, address_table, cache_array);
    GINEX_LAUNCH_CHECK();
    GINEX_HIP(hipStreamSynchronize(st));
  }
  return GINEX_OK;
}
