// Shared host/device helpers of the gfx950 library: error reporting, a bump allocator
// for the caller's workspace, wave64/block scans, fill kernels.  Internal; the public
// interface is include/ginex.h.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>

#include "ginex.h"

namespace ginex {

constexpr int WAVE = 64;

void set_error(const char* fmt, ...);
int32_t fail(int32_t code, const char* fmt, ...);

#define GINEX_HIP(call)                                                              \
  do {                                                                               \
    hipError_t e_ = (call);                                                          \
    if (e_ != hipSuccess)                                                            \
      return ::ginex::fail(GINEX_ERR_HIP, "%s failed: %s (%s:%d)", #call,            \
                           hipGetErrorString(e_), __FILE__, __LINE__);               \
  } while (0)

#define GINEX_LAUNCH_CHECK() GINEX_HIP(hipGetLastError())

// Bump allocator over the caller's workspace.  Run once with base == nullptr to measure
// and once with the real pointer to carve; both runs take the same path, so the size
// query and the call can never disagree.
struct Arena {
  char* base;
  size_t used = 0;
  explicit Arena(void* b) : base(static_cast<char*>(b)) {}
  template <typename T>
  T* take(size_t count) {
    used = (used + 255) & ~size_t(255);
    T* p = base ? reinterpret_cast<T*>(base + used) : nullptr;
    used += count * sizeof(T);
    return p;
  }
};

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// ---- device helpers -------------------------------------------------------------

__device__ __forceinline__ int lane_id() { return threadIdx.x & (WAVE - 1); }

// Inclusive scan across the 64 lanes of a wave.
template <typename T>
__device__ __forceinline__ T wave_inclusive_scan(T v) {
#pragma unroll
  for (int d = 1; d < WAVE; d <<= 1) {
    T o = __shfl_up(v, d, WAVE);
    if (lane_id() >= d) v += o;
  }
  return v;
}

template <typename T>
__device__ __forceinline__ T wave_reduce_sum(T v) {
#pragma unroll
  for (int d = WAVE / 2; d > 0; d >>= 1) v += __shfl_xor(v, d, WAVE);
  return v;
}

// Exclusive scan over a block of THREADS threads (a multiple of 64, at most 1024).
// `total` receives the block sum in every thread.  `smem` needs THREADS/64 + 1 slots.
template <typename T, int THREADS>
__device__ __forceinline__ T block_exclusive_scan(T v, T* smem, T& total) {
  constexpr int NW = THREADS / WAVE;
  const int w = threadIdx.x / WAVE;
  T inc = wave_inclusive_scan(v);
  if (lane_id() == WAVE - 1) smem[w] = inc;
  __syncthreads();
  if (threadIdx.x < WAVE) {
    T s = threadIdx.x < NW ? smem[threadIdx.x] : T(0);
    T si = wave_inclusive_scan(s);
    if (threadIdx.x < NW) smem[threadIdx.x] = si - s;
    if (threadIdx.x == NW - 1) smem[NW] = si;
  }
  __syncthreads();
  T base = smem[w];
  total = smem[NW];
  __syncthreads();
  return base + inc - v;
}

template <typename T>
__global__ void k_fill(T* p, int64_t n, T value) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) p[i] = value;
}

template <typename T>
inline hipError_t fill_async(T* p, int64_t n, T value, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  int64_t blocks = ceil_div(n, 256 * 8);
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(k_fill<T>, dim3((unsigned)blocks), dim3(256), 0, st, p, n, value);
  return hipGetLastError();
}

}  // namespace ginex
