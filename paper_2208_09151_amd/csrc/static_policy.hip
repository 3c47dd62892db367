// Static feature cache (Ginex Section 2.3 "Challenge 1": the policy of the systems the paper
// compares with): the rows of the highest out-degree nodes are loaded once and never
// replaced.  Selecting them is a histogram of `indices` (rows are in-neighbour lists, so a
// node's out-degree is how often it occurs there) and one stable radix sort of a word per
// node on the degree bits; a static run then goes through the ordinary executor
// (ginex_cache_init with the selection, ginex_gather with empty changesets), and its misses
// are counted from the address table.
#include "common.hpp"
#include "primitives.hpp"

namespace ginex {
namespace {

constexpr int TB = 256;

__global__ __launch_bounds__(TB) void k_max_u32(const uint32_t* __restrict__ v, int64_t n,
                                                uint32_t* __restrict__ result) {
  uint32_t m = 0;
  const int64_t span = (int64_t)gridDim.x * TB;
  for (int64_t i = (int64_t)blockIdx.x * TB + threadIdx.x; i < n; i += span) m = max(m, v[i]);
#pragma unroll
  for (int d = WAVE / 2; d > 0; d >>= 1) m = max(m, __shfl_xor(m, d, WAVE));
  if (lane_id() == 0 && m) atomicMax(result, m);
}

// items[v] = ((max_degree - degree[v]) << 32) | v: ascending keys = descending degrees, and
// a stable sort on the key bits keeps equal degrees in id order.
__global__ __launch_bounds__(TB) void k_degree_items(const uint32_t* __restrict__ degree,
                                                     int64_t num_nodes, uint32_t max_degree,
                                                     uint64_t* __restrict__ items) {
  const int64_t v = (int64_t)blockIdx.x * TB + threadIdx.x;
  if (v < num_nodes) items[v] = ((uint64_t)(max_degree - degree[v]) << 32) | (uint64_t)v;
}

__global__ __launch_bounds__(TB) void k_take_ids(const uint64_t* __restrict__ ranked, int64_t count,
                                                 int32_t* __restrict__ out) {
  const int64_t r = (int64_t)blockIdx.x * TB + threadIdx.x;
  if (r < count) out[r] = (int32_t)(ranked[r] & 0xFFFFFFFFull);
}

// *misses += number of ids whose address-table entry is -1
__global__ __launch_bounds__(TB) void k_count_misses(const int32_t* __restrict__ addr,
                                                     const int32_t* __restrict__ ids, int64_t n,
                                                     unsigned long long* __restrict__ misses) {
  __shared__ uint32_t red[TB / WAVE];
  uint32_t mine = 0;
  const int64_t span = (int64_t)gridDim.x * TB;
  for (int64_t p = (int64_t)blockIdx.x * TB + threadIdx.x; p < n; p += span)
    mine += addr[ids[p]] < 0;
  mine = wave_reduce_sum(mine);
  if (lane_id() == 0) red[threadIdx.x / WAVE] = mine;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t s = 0;
    for (int w = 0; w < TB / WAVE; ++w) s += red[w];
    if (s) atomicAdd(misses, (unsigned long long)s);
  }
}

struct Workspace {
  uint32_t* degree;
  uint64_t* items_a;
  uint64_t* items_b;
  uint32_t* hist;
  unsigned long long* counters;   // [0] entries of indices out of range, [1] (low half) max degree
  size_t bytes;
};

Workspace carve(void* base, int64_t num_nodes) {
  Arena a(base);
  Workspace w;
  w.degree = a.take<uint32_t>(num_nodes);
  w.items_a = a.take<uint64_t>(num_nodes);
  w.items_b = a.take<uint64_t>(num_nodes);
  w.hist = a.take<uint32_t>(radix_plan(num_nodes).hist_elems);
  w.counters = a.take<unsigned long long>(2);
  w.bytes = (a.used + 255) & ~size_t(255);
  return w;
}

int bits_for_u32(uint32_t values_minus_one) {   // bits needed to hold 0 .. values_minus_one
  int b = 1;
  while (b < 32 && (values_minus_one >> b) != 0) ++b;
  return b;
}

}  // namespace
}  // namespace ginex

using namespace ginex;

extern "C" size_t ginex_static_select_workspace_bytes(int64_t num_nodes) {
  if (num_nodes <= 0 || num_nodes > INT32_MAX) {
    set_error("ginex_static_select_workspace_bytes: num_nodes=%lld out of range",
              (long long)num_nodes);
    return 0;
  }
  return carve(nullptr, num_nodes).bytes;
}

extern "C" int32_t ginex_static_select(const ginex_csr_t* g, int64_t cap, int32_t* static_ids,
                                       int64_t* count, void* ws, size_t ws_bytes, void* stream) {
  const char* who = "ginex_static_select";
  if (!g || (g->num_edges > 0 && !g->indices))
    return fail(GINEX_ERR_ARG, "%s: graph descriptor or its indices are null", who);
  if (!count || !ws) return fail(GINEX_ERR_ARG, "%s: a required pointer is null", who);
  if (g->num_nodes <= 0 || g->num_nodes > INT32_MAX)
    return fail(GINEX_ERR_ARG, "%s: num_nodes=%lld out of range", who, (long long)g->num_nodes);
  if (g->num_edges < 0) return fail(GINEX_ERR_ARG, "%s: negative num_edges", who);
  if (cap < 0 || (cap > 0 && !static_ids))
    return fail(GINEX_ERR_ARG, "%s: bad cap or static_ids null", who);
  const int64_t n = g->num_nodes;
  const Workspace w = carve(ws, n);
  if (ws_bytes < w.bytes)
    return fail(GINEX_ERR_WORKSPACE, "%s: workspace of %zu bytes given, %zu needed", who, ws_bytes,
                w.bytes);
  if ((uintptr_t)ws & 255) return fail(GINEX_ERR_ARG, "%s: workspace must be 256-byte aligned", who);
  hipStream_t st = (hipStream_t)stream;
  const int64_t take = cap < n ? cap : n;
  *count = take;

  GINEX_HIP(fill_async<uint32_t>(w.degree, n, 0u, st));
  GINEX_HIP(fill_async<unsigned long long>(w.counters, 2, 0ull, st));
  GINEX_HIP(occurrences_async(g->indices, g->num_edges, n, w.degree, w.counters, st));
  {
    int64_t blocks = ceil_div(n, (int64_t)TB * 8);
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(k_max_u32, dim3((unsigned)blocks), dim3(TB), 0, st, w.degree, n,
                       reinterpret_cast<uint32_t*>(w.counters + 1));
    GINEX_LAUNCH_CHECK();
  }
  unsigned long long counters[2] = {0, 0};
  GINEX_HIP(hipMemcpyAsync(counters, w.counters, sizeof(counters), hipMemcpyDeviceToHost, st));
  GINEX_HIP(hipStreamSynchronize(st));
  if (counters[0])
    return fail(GINEX_ERR_INPUT, "%s: %llu entries of indices outside [0, %lld)", who, counters[0],
                (long long)n);
  const uint32_t max_degree = (uint32_t)counters[1];
  hipLaunchKernelGGL(k_degree_items, dim3((unsigned)ceil_div(n, TB)), dim3(TB), 0, st, w.degree, n,
                     max_degree, w.items_a);
  GINEX_LAUNCH_CHECK();
  uint64_t* ranked = w.items_a;
  if (max_degree > 0)
    GINEX_HIP(radix_sort_u64(w.items_a, w.items_b, n, 32, 32 + bits_for_u32(max_degree), w.hist, st,
                             &ranked));
  if (take > 0) {
    hipLaunchKernelGGL(k_take_ids, dim3((unsigned)ceil_div(take, TB)), dim3(TB), 0, st, ranked, take,
                       static_ids);
    GINEX_LAUNCH_CHECK();
  }
  GINEX_HIP(hipStreamSynchronize(st));
  return GINEX_OK;
}

extern "C" int32_t ginex_cache_count_misses(const ginex_cache_t* c, const int32_t* ids, int64_t n,
                                            int64_t* misses, void* stream) {
  const char* who = "ginex_cache_count_misses";
  if (!c || !c->addr) return fail(GINEX_ERR_ARG, "%s: cache descriptor or its address table is null", who);
  if (n < 0 || (n > 0 && !ids) || !misses)
    return fail(GINEX_ERR_ARG, "%s: ids/misses null or n negative", who);
  if (n == 0) return GINEX_OK;
  int64_t blocks = ceil_div(n, (int64_t)TB * 8);
  if (blocks > 8192) blocks = 8192;
  hipLaunchKernelGGL(k_count_misses, dim3((unsigned)blocks), dim3(TB), 0, (hipStream_t)stream,
                     c->addr, ids, n, reinterpret_cast<unsigned long long*>(misses));
  GINEX_LAUNCH_CHECK();
  return GINEX_OK;
}
