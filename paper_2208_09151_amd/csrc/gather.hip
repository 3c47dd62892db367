// Executor kernels: feature cache initialization, gather, cache update
// (Ginex Section 3.1 "Feature Cache Initialization" / "Main Loop", Section 3.3).
//
// All three are row copies.  A row of R bytes is moved as R/16 16-byte chunks; one thread
// moves one chunk, so 16..64 consecutive lanes cover a row and consecutive rows of the
// output are written back to back (fully coalesced stores).  A thread handles UNROLL
// chunks that lie far apart to keep several independent loads in flight; the source of a
// chunk is either a cache line in HBM or a row of the slow tier.
#include "common.hpp"

namespace ginex {
namespace {

typedef unsigned int chunk_t __attribute__((ext_vector_type(4)));  // 16 bytes
constexpr int THREADS = 256;
constexpr int UNROLL = 4;
// chunks per thread in k_gather_lines: with one dependent load less per chunk than k_gather and
// no id load in all-resident waves, two chunks per thread (twice the waves) beat four
// (30.3 against 31.8 us per launch on configuration 4; 1: 32.1, 3: 31.3, 6: 32.3, 8: 32.7);
// a launch that is bound by the host link keeps four, like the cache fill
constexpr int LINES_UNROLL = 2;
// The gather runs in blocks of one wave: finer to schedule at the end of a launch (37.7 us
// per 177 k rows of 512 B against 38.3 with 256 threads and 39.9 with 1024); four chunks per
// thread (1, 2, 6, 8 are 1-5 % slower).
constexpr int GATHER_THREADS = 64;

// out[p,:] = addr[ids[p]] >= 0 ? rows[addr[ids[p]],:] : slow[ids[p],:]
// SHIFT >= 0: a row has 2^SHIFT chunks (the usual case), so chunk -> (row, column) is a
// shift and a mask; SHIFT < 0: any row size, by a 64-bit division, which costs 5 % of the
// kernel's time on 512-byte rows.  (Non-temporal loads of the rows change nothing;
// non-temporal stores of the output are worth 8-10 %.)
template <int SHIFT>
__global__ __launch_bounds__(GATHER_THREADS) void k_gather(
    const chunk_t* __restrict__ rows, const int32_t* __restrict__ addr,
    const chunk_t* __restrict__ slow, const int32_t* __restrict__ ids, int64_t n,
    int32_t cpr /*chunks per row*/, chunk_t* __restrict__ out) {
  const int64_t total = n * cpr;
  const int64_t span = (int64_t)gridDim.x * GATHER_THREADS;
  int64_t c0 = (int64_t)blockIdx.x * GATHER_THREADS + threadIdx.x;
  for (; c0 < total; c0 += span * UNROLL) {
    // The three dependent reads (id, address-table entry, row chunk) of the UNROLL chunks
    // are issued level by level, so that each level's loads are in flight together.  A
    // chunk beyond the end repeats chunk c0 (in range) and is dropped at the store: no
    // branch separates the loads, which would make each wait for all earlier ones.
    int32_t id[UNROLL], col[UNROLL];
    const chunk_t* src[UNROLL];
    chunk_t v[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      int64_t c = c0 + u * span;
      c = c < total ? c : c0;
      const int64_t p = SHIFT >= 0 ? c >> (SHIFT & 31) : c / cpr;
      col[u] = SHIFT >= 0 ? (int32_t)(c & ((1 << (SHIFT & 31)) - 1)) : (int32_t)(c - p * cpr);
      id[u] = ids[p];
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int32_t line = addr[id[u]];
      src[u] = line >= 0 ? rows + (int64_t)line * cpr : slow + (int64_t)id[u] * cpr;
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) v[u] = src[u][col[u]];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int64_t c = c0 + u * span;
      if (c < total) __builtin_nontemporal_store(v[u], out + c);
    }
  }
}

// The same copy with the source of every row resolved ahead of time: lines[p] is the cache
// line of ids[p] or -1 (slow tier).  Both arrays are read in output order, so the random
// 4-byte probe of the address table (a 128-byte line fetched per row) and one level of the
// dependent load chain are gone: what is left per row is R bytes in, R bytes out and 8 bytes
// of sequential index data.
template <int SHIFT, int U>
__global__ __launch_bounds__(GATHER_THREADS) void k_gather_lines(
    const chunk_t* __restrict__ rows, const chunk_t* __restrict__ slow,
    const int32_t* __restrict__ ids, const int32_t* __restrict__ lines, int64_t n,
    int32_t cpr /*chunks per row*/, chunk_t* __restrict__ out) {
  const int64_t total = n * cpr;
  const int64_t span = (int64_t)gridDim.x * GATHER_THREADS;
  int64_t c0 = (int64_t)blockIdx.x * GATHER_THREADS + threadIdx.x;
  for (; c0 < total; c0 += span * U) {
    int64_t p[U];
    int32_t line[U], col[U];
    chunk_t v[U];
    bool slow_row = false;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      int64_t c = c0 + u * span;
      c = c < total ? c : c0;
      p[u] = SHIFT >= 0 ? c >> (SHIFT & 31) : c / cpr;
      col[u] = SHIFT >= 0 ? (int32_t)(c & ((1 << (SHIFT & 31)) - 1)) : (int32_t)(c - p[u] * cpr);
      line[u] = lines[p[u]];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) slow_row |= line[u] < 0;
    // The node id of a row is needed only where the row comes from the slow tier: a wave
    // whose rows are all resident (every wave of an iteration without misses) never loads
    // one.  The test is per wave, so both ways stay straight-line code with the loads of a
    // level in flight together.
    if (!__any(slow_row)) {
#pragma unroll
      for (int u = 0; u < U; ++u) v[u] = rows[(int64_t)line[u] * cpr + col[u]];
    } else {
      int32_t id[U];
#pragma unroll
      for (int u = 0; u < U; ++u) id[u] = ids[p[u]];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const chunk_t* src = line[u] >= 0 ? rows + (int64_t)line[u] * cpr : slow + (int64_t)id[u] * cpr;
        v[u] = src[col[u]];
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t c = c0 + u * span;
      if (c < total) __builtin_nontemporal_store(v[u], out + c);
    }
  }
}

// Cache update (Section 3.3 "Feature Cache Update"), one wave per changeset record j:
// line = addr[out_ids[j]]; rows[line,:] = out[in_positions[j],:]; addr[out_ids[j]] = -1;
// addr[in_ids[j]] = line.  Every lane of the wave reads the evicted row's entry before lane 0
// overwrites it (one wave, program order), and no other record touches these two entries
// (in_ids and out_ids of an iteration are disjoint sets of distinct ids), so rows and address
// table change in one launch.
__global__ __launch_bounds__(THREADS) void k_update(
    chunk_t* __restrict__ rows, int32_t* __restrict__ addr, const chunk_t* __restrict__ out,
    const int32_t* __restrict__ in_ids, const int32_t* __restrict__ out_ids,
    const int32_t* __restrict__ in_positions, int64_t n_change, int32_t cpr) {
  const int64_t waves = (int64_t)gridDim.x * (THREADS / WAVE);
  for (int64_t j = ((int64_t)blockIdx.x * THREADS + threadIdx.x) / WAVE; j < n_change; j += waves) {
    const int32_t gone = out_ids[j];
    const int32_t line = addr[gone];
    const int64_t src = (int64_t)in_positions[j] * cpr, dst = (int64_t)line * cpr;
    for (int32_t col = lane_id(); col < cpr; col += WAVE) rows[dst + col] = out[src + col];
    if (lane_id() == 0) {
      addr[gone] = -1;
      addr[in_ids[j]] = line;
    }
  }
}

// rows[r,:] = slow[init_ids[r],:]; addr[init_ids[r]] = r, for lines r in [begin, end).
// Unlike k_gather this kernel keeps the three dependent reads of a chunk behind one another
// (one chunk in flight per thread at a time): the host link is saturated either way, and
// with four times as many link reads in flight per wave a gather running beside the fill
// took twice as long again and slowed the fill down by 5-30 %.
__global__ __launch_bounds__(THREADS) void k_cache_fill(
    chunk_t* __restrict__ rows, int32_t* __restrict__ addr, const chunk_t* __restrict__ slow,
    const int32_t* __restrict__ init_ids, int64_t begin, int64_t end, int32_t cpr) {
  const int64_t total = end * cpr;
  const int64_t span = (int64_t)gridDim.x * THREADS;
  int64_t c0 = begin * cpr + (int64_t)blockIdx.x * THREADS + threadIdx.x;
  for (; c0 < total; c0 += span * UNROLL) {
    chunk_t v[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int64_t c = c0 + u * span;
      if (c < total) {
        const int64_t r = c / cpr;
        const int32_t col = (int32_t)(c - r * cpr);
        const int32_t id = init_ids[r];
        v[u] = slow[(int64_t)id * cpr + col];
        if (col == 0) addr[id] = (int32_t)r;
      }
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int64_t c = c0 + u * span;
      if (c < total) rows[c] = v[u];
    }
  }
}

// The same fill with a second source in front of the slow tier: a row that another cache
// (the previous superbatch's) still holds is copied from there, HBM to HBM.
__global__ __launch_bounds__(THREADS) void k_cache_fill_warm(
    chunk_t* __restrict__ rows, int32_t* __restrict__ addr, const chunk_t* __restrict__ slow,
    const chunk_t* __restrict__ prev_rows, const int32_t* __restrict__ prev_addr,
    const int32_t* __restrict__ init_ids, int64_t begin, int64_t end, int32_t cpr) {
  const int64_t total = end * cpr;
  const int64_t span = (int64_t)gridDim.x * THREADS;
  int64_t c0 = begin * cpr + (int64_t)blockIdx.x * THREADS + threadIdx.x;
  for (; c0 < total; c0 += span * UNROLL) {
    chunk_t v[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int64_t c = c0 + u * span;
      if (c < total) {
        const int64_t r = c / cpr;
        const int32_t col = (int32_t)(c - r * cpr);
        const int32_t id = init_ids[r];
        const int32_t line = prev_addr[id];
        const chunk_t* src = line >= 0 ? prev_rows + (int64_t)line * cpr : slow + (int64_t)id * cpr;
        v[u] = src[col];
        if (col == 0) addr[id] = (int32_t)r;
      }
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int64_t c = c0 + u * span;
      if (c < total) rows[c] = v[u];
    }
  }
}

inline unsigned grid_for(int64_t items, int per_thread) {
  int64_t blocks = ceil_div(items, (int64_t)THREADS * per_thread);
  if (blocks < 1) blocks = 1;
  if (blocks > (1 << 20)) blocks = 1 << 20;
  return (unsigned)blocks;
}

int32_t check_cache(const ginex_cache_t* c, const char* who) {
  if (!c) return fail(GINEX_ERR_ARG, "%s: cache descriptor is null", who);
  if (c->cap < 0 || c->num_nodes <= 0 || c->num_nodes > INT32_MAX || c->cap > INT32_MAX)
    return fail(GINEX_ERR_ARG, "%s: cap=%lld num_nodes=%lld out of range", who,
                (long long)c->cap, (long long)c->num_nodes);
  if (c->row_bytes <= 0 || c->row_bytes % 16 != 0 || c->row_bytes / 16 > INT32_MAX)
    return fail(GINEX_ERR_ARG, "%s: row_bytes=%lld must be a positive multiple of 16", who,
                (long long)c->row_bytes);
  if (!c->addr || !c->slow || (c->cap > 0 && !c->rows))
    return fail(GINEX_ERR_ARG, "%s: null rows/addr/slow pointer", who);
  if (((uintptr_t)c->rows | (uintptr_t)c->slow) & 15)
    return fail(GINEX_ERR_ARG, "%s: rows and slow must be 16-byte aligned", who);
  return GINEX_OK;
}

}  // namespace
}  // namespace ginex

using namespace ginex;

namespace ginex {
namespace {

// Grid of the warm fill: its link reads are diluted by HBM-to-HBM copies, so it takes more
// blocks than the cold fill to keep the same number of link reads in flight.
constexpr unsigned WARM_BLOCKS = 128;

int32_t launch_fill(const ginex_cache_t* c, const int32_t* init_ids, int64_t begin, int64_t end,
                    hipStream_t st) {
  if (end <= begin) return GINEX_OK;
  const int32_t cpr = (int32_t)(c->row_bytes / 16);
  // The fill is bound by the host link, which 64 blocks (1 MB of reads in flight; a link
  // read takes about 7 us) keep busier than a full grid does (57 against 54.6 GB/s); 32
  // blocks reach 53 GB/s, 16 blocks 34.  Link reads in flight slow every other kernel's
  // HBM traffic down: a gather that runs beside the fill takes 1.2x (32 blocks), 2x (64) or
  // 6x (128) its time alone, and behind a full grid kernels on other streams make no
  // progress at all until the fill ends.
  unsigned blocks = grid_for((end - begin) * cpr, UNROLL);
  if (blocks > 64) blocks = 64;
  hipLaunchKernelGGL(k_cache_fill, dim3(blocks), dim3(THREADS), 0, st, (chunk_t*)c->rows, c->addr,
                     (const chunk_t*)c->slow, init_ids, begin, end, cpr);
  GINEX_LAUNCH_CHECK();
  return GINEX_OK;
}

}  // namespace
}  // namespace ginex

extern "C" int32_t ginex_cache_init(const ginex_cache_t* c, const int32_t* init_ids,
                                    int64_t init_count, void* stream) {
  if (int32_t rc = check_cache(c, "ginex_cache_init")) return rc;
  if (init_count < 0 || init_count > c->cap)
    return fail(GINEX_ERR_ARG, "ginex_cache_init: init_count=%lld outside [0, cap=%lld]",
                (long long)init_count, (long long)c->cap);
  if (init_count > 0 && !init_ids) return fail(GINEX_ERR_ARG, "ginex_cache_init: init_ids is null");
  hipStream_t st = (hipStream_t)stream;
  GINEX_HIP(fill_async<int32_t>(c->addr, c->num_nodes, -1, st));
  return launch_fill(c, init_ids, 0, init_count, st);
}

extern "C" int32_t ginex_cache_init_warm(const ginex_cache_t* c, const ginex_cache_t* prev,
                                         const int32_t* init_ids, int64_t begin, int64_t end,
                                         void* stream) {
  const char* who = "ginex_cache_init_warm";
  if (int32_t rc = check_cache(c, who)) return rc;
  if (int32_t rc = check_cache(prev, who)) return rc;
  if (prev->row_bytes != c->row_bytes || prev->num_nodes != c->num_nodes || prev->slow != c->slow)
    return fail(GINEX_ERR_ARG, "%s: the two caches must front the same slow tier", who);
  if (prev->rows == c->rows || prev->addr == c->addr)
    return fail(GINEX_ERR_ARG, "%s: the two caches must not share their arrays", who);
  if (begin < 0 || end < begin || end > c->cap)
    return fail(GINEX_ERR_ARG, "%s: [%lld, %lld) outside [0, cap=%lld]", who, (long long)begin,
                (long long)end, (long long)c->cap);
  if (end > begin && !init_ids) return fail(GINEX_ERR_ARG, "%s: init_ids is null", who);
  hipStream_t st = (hipStream_t)stream;
  if (begin == 0) GINEX_HIP(fill_async<int32_t>(c->addr, c->num_nodes, -1, st));
  if (end > begin) {
    const int32_t cpr = (int32_t)(c->row_bytes / 16);
    unsigned blocks = grid_for((end - begin) * cpr, UNROLL);
    if (blocks > WARM_BLOCKS) blocks = WARM_BLOCKS;
    hipLaunchKernelGGL(k_cache_fill_warm, dim3(blocks), dim3(THREADS), 0, st, (chunk_t*)c->rows,
                       c->addr, (const chunk_t*)c->slow, (const chunk_t*)prev->rows, prev->addr,
                       init_ids, begin, end, cpr);
    GINEX_LAUNCH_CHECK();
  }
  return GINEX_OK;
}

extern "C" int32_t ginex_cache_init_part(const ginex_cache_t* c, const int32_t* init_ids,
                                         int64_t begin, int64_t end, void* stream) {
  if (int32_t rc = check_cache(c, "ginex_cache_init_part")) return rc;
  if (begin < 0 || end < begin || end > c->cap)
    return fail(GINEX_ERR_ARG, "ginex_cache_init_part: [%lld, %lld) outside [0, cap=%lld]",
                (long long)begin, (long long)end, (long long)c->cap);
  if (end > begin && !init_ids)
    return fail(GINEX_ERR_ARG, "ginex_cache_init_part: init_ids is null");
  hipStream_t st = (hipStream_t)stream;
  if (begin == 0) GINEX_HIP(fill_async<int32_t>(c->addr, c->num_nodes, -1, st));
  return launch_fill(c, init_ids, begin, end, st);
}

namespace ginex {
namespace {

int32_t check_update(const ginex_cache_t* c, const void* out, const int32_t* in_ids,
                     const int32_t* out_ids, const int32_t* in_positions, int64_t n_change,
                     const char* who) {
  if (n_change < 0 || n_change > c->cap)
    return fail(GINEX_ERR_ARG, "%s: n_change=%lld outside [0, cap=%lld]", who,
                (long long)n_change, (long long)c->cap);
  if (n_change > 0 && (!in_ids || !out_ids || !in_positions || !out))
    return fail(GINEX_ERR_ARG, "%s: a changeset list or the batch input is null", who);
  if (((uintptr_t)out) & 15) return fail(GINEX_ERR_ARG, "%s: out must be 16-byte aligned", who);
  return GINEX_OK;
}

int32_t launch_update(const ginex_cache_t* c, const void* out, const int32_t* in_ids,
                      const int32_t* out_ids, const int32_t* in_positions, int64_t n_change,
                      hipStream_t st) {
  if (n_change == 0) return GINEX_OK;
  const int32_t cpr = (int32_t)(c->row_bytes / 16);
  hipLaunchKernelGGL(k_update, dim3(grid_for(n_change * WAVE, 1)), dim3(THREADS), 0, st,
                     (chunk_t*)c->rows, c->addr, (const chunk_t*)out, in_ids, out_ids, in_positions,
                     n_change, cpr);
  GINEX_LAUNCH_CHECK();
  return GINEX_OK;
}

}  // namespace
}  // namespace ginex

extern "C" int32_t ginex_cache_update(const ginex_cache_t* c, const void* out,
                                      const int32_t* in_ids, const int32_t* out_ids,
                                      const int32_t* in_positions, int64_t n_change,
                                      void* stream) {
  if (int32_t rc = check_cache(c, "ginex_cache_update")) return rc;
  if (int32_t rc = check_update(c, out, in_ids, out_ids, in_positions, n_change,
                                "ginex_cache_update"))
    return rc;
  return launch_update(c, out, in_ids, out_ids, in_positions, n_change, (hipStream_t)stream);
}

namespace ginex {
namespace {

// Chunks a gather keeps in flight over the host link when many of its rows come from the slow
// tier: what the cache fill found best (64 blocks of 256 threads with UNROLL chunks each;
// more requests in flight lower the link's throughput, see launch_fill).
constexpr int64_t LINK_CHUNKS_IN_FLIGHT = 64 * THREADS * UNROLL;

// lines == nullptr: the gather probes the address table itself.  n_slow: rows known to come
// from the slow tier, or -1.
int32_t gather_run(const char* who, const ginex_cache_t* c, const int32_t* ids,
                   const int32_t* lines, int64_t n, int64_t n_slow, void* out,
                   const int32_t* in_ids, const int32_t* out_ids, const int32_t* in_positions,
                   int64_t n_change, void* stream) {
  if (int32_t rc = check_cache(c, who)) return rc;
  if (n < 0 || n_change > n)
    return fail(GINEX_ERR_ARG, "%s: n=%lld n_change=%lld inconsistent", who, (long long)n,
                (long long)n_change);
  if (n > 0 && (!ids || !out)) return fail(GINEX_ERR_ARG, "%s: ids/out is null", who);
  if (int32_t rc = check_update(c, out, in_ids, out_ids, in_positions, n_change, who)) return rc;
  hipStream_t st = (hipStream_t)stream;
  if (n > 0) {
    const int32_t cpr = (int32_t)(c->row_bytes / 16);
    // one pass of the kernel's loop up to 2^24 blocks (8 TB of rows), more passes beyond
    const bool link_bound = n_slow > 0 && n_slow * 4 >= n * 3;
    const int per_thread = lines && !link_bound ? LINES_UNROLL : UNROLL;
    int64_t blocks = ceil_div(n * cpr, (int64_t)GATHER_THREADS * per_thread);
    if (blocks > (1 << 24)) blocks = 1 << 24;
    // A launch that reads at least three quarters of its rows from the slow tier runs on a
    // smaller grid whose blocks stride over the rows, so that about as many link reads are in
    // flight as the cache fill keeps (51.8 -> 56.2 GB/s with nothing resident).  With fewer
    // slow rows the smaller grid starves the resident ones of HBM parallelism (at 42 % slow
    // rows the launch took 3 % longer), so those keep the full grid.
    if (link_bound) {
      const int64_t want = ceil_div(LINK_CHUNKS_IN_FLIGHT * n, n_slow * (int64_t)GATHER_THREADS * UNROLL);
      if (want < blocks) blocks = want;
    }
    const dim3 grid((unsigned)blocks);
#define GINEX_GATHER(S)                                                                       \
  do {                                                                                        \
    if (lines && link_bound)                                                                  \
      hipLaunchKernelGGL((k_gather_lines<S, UNROLL>), grid, dim3(GATHER_THREADS), 0, st,       \
                         (const chunk_t*)c->rows, (const chunk_t*)c->slow, ids, lines, n, cpr, \
                         (chunk_t*)out);                                                      \
    else if (lines)                                                                           \
      hipLaunchKernelGGL((k_gather_lines<S, LINES_UNROLL>), grid, dim3(GATHER_THREADS), 0, st, \
                         (const chunk_t*)c->rows, (const chunk_t*)c->slow, ids, lines, n, cpr, \
                         (chunk_t*)out);                                                      \
    else                                                                                      \
      hipLaunchKernelGGL((k_gather<S>), grid, dim3(GATHER_THREADS), 0, st,                     \
                         (const chunk_t*)c->rows, c->addr, (const chunk_t*)c->slow, ids, n,    \
                         cpr, (chunk_t*)out);                                                 \
  } while (0)
    switch (cpr) {      // rows of 16 B .. 4 KB with a power-of-two size
      case 1: GINEX_GATHER(0); break;
      case 2: GINEX_GATHER(1); break;
      case 4: GINEX_GATHER(2); break;
      case 8: GINEX_GATHER(3); break;
      case 16: GINEX_GATHER(4); break;
      case 32: GINEX_GATHER(5); break;
      case 64: GINEX_GATHER(6); break;
      case 128: GINEX_GATHER(7); break;
      case 256: GINEX_GATHER(8); break;
      default: GINEX_GATHER(-1);
    }
#undef GINEX_GATHER
    GINEX_LAUNCH_CHECK();
  }
  return launch_update(c, out, in_ids, out_ids, in_positions, n_change, st);
}

}  // namespace
}  // namespace ginex

extern "C" int32_t ginex_gather(const ginex_cache_t* c, const int32_t* ids, int64_t n, void* out,
                                const int32_t* in_ids, const int32_t* out_ids,
                                const int32_t* in_positions, int64_t n_change, void* stream) {
  return gather_run("ginex_gather", c, ids, nullptr, n, -1, out, in_ids, out_ids, in_positions,
                    n_change, stream);
}

extern "C" int32_t ginex_gather_lines(const ginex_cache_t* c, const int32_t* ids,
                                      const int32_t* src_line, int64_t n, int64_t n_slow,
                                      void* out, const int32_t* in_ids, const int32_t* out_ids,
                                      const int32_t* in_positions, int64_t n_change,
                                      void* stream) {
  if (n > 0 && !src_line) return fail(GINEX_ERR_ARG, "ginex_gather_lines: src_line is null");
  if (n_slow > n) return fail(GINEX_ERR_ARG, "ginex_gather_lines: n_slow=%lld exceeds n=%lld",
                              (long long)n_slow, (long long)n);
  return gather_run("ginex_gather_lines", c, ids, src_line, n, n_slow, out, in_ids, out_ids,
                    in_positions, n_change, stream);
}
