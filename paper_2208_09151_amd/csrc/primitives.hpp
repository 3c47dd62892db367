// Device-wide building blocks written for wave64: exclusive scan and a stable LSD radix
// sort of 64-bit words on a chosen bit range.  Internal header; every function enqueues
// on the given stream and never synchronises or allocates.
#pragma once

#include "common.hpp"

namespace ginex {

// ---------------------------------------------------------------------------------
// Exclusive scan of uint32 counters (three kernels, recursive on the tile sums).
// ---------------------------------------------------------------------------------
constexpr int SCAN_THREADS = 256;
constexpr int SCAN_ITEMS = 16;
constexpr int SCAN_TILE = SCAN_THREADS * SCAN_ITEMS;

template <typename T>
__global__ __launch_bounds__(SCAN_THREADS) void k_scan_tiles(T* __restrict__ data, int64_t n,
                                                             T* __restrict__ tile_sums) {
  __shared__ T smem[SCAN_THREADS / WAVE + 1];
  const int64_t base = (int64_t)blockIdx.x * SCAN_TILE + (int64_t)threadIdx.x * SCAN_ITEMS;
  T v[SCAN_ITEMS];
  T sum = 0;
#pragma unroll
  for (int i = 0; i < SCAN_ITEMS; ++i) {
    v[i] = (base + i < n) ? data[base + i] : T(0);
    sum += v[i];
  }
  T total;
  T run = block_exclusive_scan<T, SCAN_THREADS>(sum, smem, total);
#pragma unroll
  for (int i = 0; i < SCAN_ITEMS; ++i) {
    if (base + i < n) data[base + i] = run;
    run += v[i];
  }
  if (threadIdx.x == 0 && tile_sums) tile_sums[blockIdx.x] = total;
}

template <typename T>
__global__ __launch_bounds__(SCAN_THREADS) void k_scan_add(T* __restrict__ data, int64_t n,
                                                           const T* __restrict__ tile_bases) {
  const T add = tile_bases[blockIdx.x];
  const int64_t base = (int64_t)blockIdx.x * SCAN_TILE + (int64_t)threadIdx.x * SCAN_ITEMS;
#pragma unroll
  for (int i = 0; i < SCAN_ITEMS; ++i)
    if (base + i < n) data[base + i] += add;
}

// Scratch elements needed by exclusive_scan_inplace for n elements.
inline int64_t scan_scratch_elems(int64_t n) {
  int64_t total = 0;
  while (n > SCAN_TILE) {
    n = ceil_div(n, SCAN_TILE);
    total += n;
  }
  return total + 1;
}

// data[i] <- sum of data[0..i).  `scratch` holds scan_scratch_elems(n) elements.
template <typename T>
inline hipError_t exclusive_scan_inplace(T* data, int64_t n, T* scratch, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  const int64_t tiles = ceil_div(n, SCAN_TILE);
  if (tiles == 1) {
    hipLaunchKernelGGL(k_scan_tiles<T>, dim3(1), dim3(SCAN_THREADS), 0, st, data, n, (T*)nullptr);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(k_scan_tiles<T>, dim3((unsigned)tiles), dim3(SCAN_THREADS), 0, st, data, n,
                     scratch);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  e = exclusive_scan_inplace<T>(scratch, tiles, scratch + tiles, st);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_scan_add<T>, dim3((unsigned)tiles), dim3(SCAN_THREADS), 0, st, data, n,
                     scratch);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// Occurrence histogram: count[v] += number of times v occurs in values[0..n).  With the CSR
// rows holding in-neighbours this is the out-degree of every node.  Entries outside
// [0, bins) are counted in *bad and skipped.  `values` may live in host-pinned memory.
// ---------------------------------------------------------------------------------
static __global__ __launch_bounds__(256) void k_occurrences(const int32_t* __restrict__ values,
                                                            int64_t n, int64_t bins,
                                                            uint32_t* __restrict__ count,
                                                            unsigned long long* __restrict__ bad) {
  const int64_t span = (int64_t)gridDim.x * 256;
  for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < n; e += span) {
    const int32_t v = values[e];
    if ((uint32_t)v < (uint64_t)bins) atomicAdd(&count[v], 1u);
    else atomicAdd(bad, 1ull);
  }
}

inline hipError_t occurrences_async(const int32_t* values, int64_t n, int64_t bins, uint32_t* count,
                                    unsigned long long* bad, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  int64_t blocks = ceil_div(n, (int64_t)256 * 16);
  if (blocks > 16384) blocks = 16384;
  hipLaunchKernelGGL(k_occurrences, dim3((unsigned)blocks), dim3(256), 0, st, values, n, bins, count,
                     bad);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// Stable LSD radix sort of uint64 words on bits [bit_lo, bit_hi), 8 bits per pass.
// Each pass: (1) per-tile digit histogram, (2) exclusive scan of the digit-major
// histogram, (3) scatter.  In the scatter a wave owns a contiguous run of its tile and
// ranks its 64 keys per step with ballot-built peer masks, so equal digits keep their
// input order; keys are then staged in LDS in digit order and written out in runs.
// ---------------------------------------------------------------------------------
constexpr int RS_THREADS = 256;
constexpr int RS_WAVES = RS_THREADS / WAVE;
constexpr int RS_ITEMS = 16;                    // keys per thread
constexpr int RS_TILE = RS_THREADS * RS_ITEMS;  // 4096 keys, 32 KB of LDS staging
constexpr int RS_BINS = 256;

// Where a pass reads its words: an array of words, or (the first pass of a sort of
// (value, position) pairs) an array of 32-bit values, word j = value j << 32 | j, so that the
// pairs need not be written out and read back first.
struct RadixWords {
  const uint64_t* in;
  __device__ __forceinline__ uint64_t operator()(int64_t j) const { return in[j]; }
};
struct RadixValuesWithPositions {
  const int32_t* values;
  __device__ __forceinline__ uint64_t operator()(int64_t j) const {
    return ((uint64_t)(uint32_t)values[j] << 32) | (uint64_t)j;
  }
};

template <typename Source>
static __global__ __launch_bounds__(RS_THREADS) void k_radix_hist(Source in, int64_t n, int shift,
                                                                  int64_t tiles,
                                                                  uint32_t* __restrict__ hist) {
  __shared__ uint32_t bins[RS_BINS];
  bins[threadIdx.x] = 0;
  __syncthreads();
  const int64_t base = (int64_t)blockIdx.x * RS_TILE;
#pragma unroll
  for (int i = 0; i < RS_ITEMS; ++i) {
    const int64_t j = base + i * RS_THREADS + threadIdx.x;
    if (j < n) atomicAdd(&bins[(in(j) >> shift) & (RS_BINS - 1)], 1u);
  }
  __syncthreads();
  hist[(int64_t)threadIdx.x * tiles + blockIdx.x] = bins[threadIdx.x];
}

template <typename Source>
static __global__ __launch_bounds__(RS_THREADS) void k_radix_scatter(
    Source in, uint64_t* __restrict__ out, int64_t n, int shift, int64_t tiles,
    const uint32_t* __restrict__ hist_scanned) {
  __shared__ uint64_t staged[RS_TILE];
  __shared__ uint32_t wave_count[RS_WAVES][RS_BINS];
  __shared__ uint32_t digit_start[RS_BINS];   // start of each digit inside the tile
  __shared__ int64_t digit_dst[RS_BINS];      // global destination of the digit's run
  __shared__ uint32_t scan_smem[RS_THREADS / WAVE + 1];

  const int w = threadIdx.x / WAVE;
  const int lane = lane_id();
  for (int i = threadIdx.x; i < RS_WAVES * RS_BINS; i += RS_THREADS) (&wave_count[0][0])[i] = 0;
  __syncthreads();

  const int64_t tile_base = (int64_t)blockIdx.x * RS_TILE;
  const int64_t wave_base = tile_base + (int64_t)w * (WAVE * RS_ITEMS);
  uint64_t key[RS_ITEMS];
  uint32_t rank[RS_ITEMS];  // rank among the wave's keys with the same digit
#pragma unroll
  for (int i = 0; i < RS_ITEMS; ++i) {
    const int64_t j = wave_base + i * WAVE + lane;
    const bool valid = j < n;
    key[i] = valid ? in(j) : 0;
    const uint32_t d = (uint32_t)(key[i] >> shift) & (RS_BINS - 1);
    uint64_t peers = __ballot(valid);
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      const uint64_t m = __ballot((d >> b) & 1);
      peers &= ((d >> b) & 1) ? m : ~m;
    }
    const uint32_t before = __popcll(peers & ((1ull << lane) - 1));
    const int leader = __ffsll((unsigned long long)peers) - 1;
    uint32_t prev = 0;
    if (valid && lane == leader) {
      prev = wave_count[w][d];
      wave_count[w][d] = prev + __popcll(peers);
    }
    __builtin_amdgcn_wave_barrier();  // keep the LDS update ahead of the next step's read
    prev = __shfl(prev, leader < 0 ? 0 : leader, WAVE);
    rank[i] = prev + before;
  }
  __syncthreads();

  // thread t owns digit t: turn per-wave counts into per-wave starts, get tile totals
  {
    const int d = threadIdx.x;
    uint32_t run = 0;
#pragma unroll
    for (int ww = 0; ww < RS_WAVES; ++ww) {
      const uint32_t c = wave_count[ww][d];
      wave_count[ww][d] = run;
      run += c;
    }
    uint32_t total;
    const uint32_t start = block_exclusive_scan<uint32_t, RS_THREADS>(run, scan_smem, total);
    digit_start[d] = start;
    digit_dst[d] = (int64_t)hist_scanned[(int64_t)d * tiles + blockIdx.x] - (int64_t)start;
  }
  __syncthreads();

#pragma unroll
  for (int i = 0; i < RS_ITEMS; ++i) {
    const int64_t j = wave_base + i * WAVE + lane;
    if (j < n) {
      const uint32_t d = (uint32_t)(key[i] >> shift) & (RS_BINS - 1);
      staged[digit_start[d] + wave_count[w][d] + rank[i]] = key[i];
    }
  }
  __syncthreads();

  const int64_t remaining = n - tile_base;
  const int count = remaining < RS_TILE ? (int)remaining : RS_TILE;
  for (int i = threadIdx.x; i < count; i += RS_THREADS) {
    const uint64_t k = staged[i];
    const uint32_t d = (uint32_t)(k >> shift) & (RS_BINS - 1);
    out[digit_dst[d] + i] = k;
  }
}

struct RadixPlan {
  int64_t tiles;
  int64_t hist_elems;   // uint32 counters (+ scan scratch) the sort needs
};

inline RadixPlan radix_plan(int64_t n) {
  RadixPlan p;
  p.tiles = n > 0 ? ceil_div(n, RS_TILE) : 1;
  const int64_t h = p.tiles * RS_BINS;
  p.hist_elems = h + scan_scratch_elems(h);
  return p;
}

// Sorts `n` words by bits [bit_lo, bit_hi).  `a` holds the input, `b` is a buffer of the
// same size; returns (through *sorted) which of the two holds the result.  The total
// number of keys must stay below 2^32 (uint32 histogram).
template <typename Source>
inline hipError_t radix_pass(Source in, uint64_t* out, int64_t n, int shift, const RadixPlan& p,
                             uint32_t* hist, hipStream_t st) {
  const int64_t h = p.tiles * RS_BINS;
  hipLaunchKernelGGL(k_radix_hist<Source>, dim3((unsigned)p.tiles), dim3(RS_THREADS), 0, st, in, n,
                     shift, p.tiles, hist);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  e = exclusive_scan_inplace<uint32_t>(hist, h, hist + h, st);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_radix_scatter<Source>, dim3((unsigned)p.tiles), dim3(RS_THREADS), 0, st, in,
                     out, n, shift, p.tiles, hist);
  return hipGetLastError();
}

inline hipError_t radix_sort_u64(uint64_t* a, uint64_t* b, int64_t n, int bit_lo, int bit_hi,
                                 uint32_t* hist, hipStream_t st, uint64_t** sorted) {
  *sorted = a;
  if (n <= 1) return hipSuccess;
  const RadixPlan p = radix_plan(n);
  for (int shift = bit_lo; shift < bit_hi; shift += 8) {
    const hipError_t e = radix_pass(RadixWords{a}, b, n, shift, p, hist, st);
    if (e != hipSuccess) return e;
    uint64_t* t = a; a = b; b = t;
  }
  *sorted = a;
  return hipSuccess;
}

// The words (values[j] << 32 | j), j in [0, n), sorted by bits [32, bit_hi) of the word, that
// is by the low bits of the value; equal values keep the order of their positions.  `a` and
// `b` are two buffers of n words; *sorted tells which of them holds the result.
inline hipError_t radix_sort_values_with_positions(const int32_t* values, uint64_t* a, uint64_t* b,
                                                   int64_t n, int bit_hi, uint32_t* hist,
                                                   hipStream_t st, uint64_t** sorted) {
  *sorted = a;
  if (n <= 0) return hipSuccess;
  const RadixPlan p = radix_plan(n);
  hipError_t e = radix_pass(RadixValuesWithPositions{values}, a, n, 32, p, hist, st);
  if (e != hipSuccess) return e;
  for (int shift = 40; shift < bit_hi; shift += 8) {
    e = radix_pass(RadixWords{a}, b, n, shift, p, hist, st);
    if (e != hipSuccess) return e;
    uint64_t* t = a; a = b; b = t;
  }
  *sorted = a;
  return hipSuccess;
}

}  // namespace ginex
