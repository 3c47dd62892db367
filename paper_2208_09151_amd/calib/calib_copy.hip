// Calibration for the HBM traffic counters: a plain copy kernel of known size.
// `rocprofv3 --pmc FETCH_SIZE -- calib_copy` (then WRITE_SIZE) reads what the counters
// report for copying exactly `bytes` bytes; the ratio known/reported scales the counter
// readings of the library's kernels.  Standalone program, not part of libginex.so.
//
//   calib_copy [MiB (default 1024)] [repetitions (default 5)]
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>

typedef unsigned int chunk_t __attribute__((ext_vector_type(4)));

// One 16-byte chunk per thread and as many blocks as that takes: the fastest plain copy
// found on this GPU (grid-stride loops and several chunks per thread are 20-30 % slower at
// 1 GiB), so its rate also serves as the practical streaming ceiling.
__global__ __launch_bounds__(256) void k_plain_copy(const chunk_t* __restrict__ src,
                                                    chunk_t* __restrict__ dst, int64_t chunks) {
  const int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (c < chunks) dst[c] = src[c];
}

#define CHECK(x)                                                                   \
  do {                                                                             \
    hipError_t e = (x);                                                            \
    if (e != hipSuccess) {                                                         \
      fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e));                       \
      return 1;                                                                    \
    }                                                                              \
  } while (0)

int main(int argc, char** argv) {
  const int64_t mib = argc > 1 ? atoll(argv[1]) : 1024;
  const int reps = argc > 2 ? atoi(argv[2]) : 5;
  const int64_t bytes = mib << 20, chunks = bytes / 16;
  chunk_t *src, *dst;
  CHECK(hipMalloc(&src, bytes));
  CHECK(hipMalloc(&dst, bytes));
  CHECK(hipMemset(src, 1, bytes));
  CHECK(hipMemset(dst, 0, bytes));
  hipEvent_t a, b;
  CHECK(hipEventCreate(&a));
  CHECK(hipEventCreate(&b));
  for (int r = 0; r < reps; ++r) {
    CHECK(hipEventRecord(a, 0));
    hipLaunchKernelGGL(k_plain_copy, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, 0, src, dst,
                       chunks);
    CHECK(hipEventRecord(b, 0));
    CHECK(hipEventSynchronize(b));
    float ms = 0;
    CHECK(hipEventElapsedTime(&ms, a, b));
    printf("k_plain_copy: %lld bytes read + %lld written in %.3f ms = %.1f GB/s\n",
           (long long)bytes, (long long)bytes, ms, 2.0 * bytes / ms / 1e6);
  }
  CHECK(hipFree(src));
  CHECK(hipFree(dst));
  return 0;
}
