// hbm_probe.hip -- plain copy and read kernels of known size.
//
// Used for two things: to see what fraction of the 8 TB/s HBM peak a trivial
// streaming kernel reaches on the box, and to calibrate rocprofv3's FETCH_SIZE /
// WRITE_SIZE counters (the factor between what they report for this copy and
// the bytes it is known to move scales the counters read for cos_verify).
//
//   hbm_probe [MiB per buffer = 4096] [iterations = 10]
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

#define CHECK(x)                                                                 \
  do {                                                                           \
    hipError_t e_ = (x);                                                         \
    if (e_ != hipSuccess) {                                                      \
      std::fprintf(stderr, "%s failed: %s\n", #x, hipGetErrorString(e_));        \
      return 1;                                                                  \
    }                                                                            \
  } while (0)

constexpr int kThreads = 256;
constexpr int kPerThread = 8;  // 16-byte vectors per thread

// dst[i] = src[i]: count vectors read, count vectors written.
__global__ void __launch_bounds__(kThreads) hbm_probe_copy(const uint4* __restrict__ src,
                                                           uint4* __restrict__ dst, size_t count) {
  const size_t base = (size_t)blockIdx.x * kThreads * kPerThread + threadIdx.x;
  uint4 v[kPerThread];
#pragma unroll
  for (int u = 0; u < kPerThread; ++u) {
    const size_t i = base + (size_t)u * kThreads;
    if (i < count) v[u] = src[i];
  }
#pragma unroll
  for (int u = 0; u < kPerThread; ++u) {
    const size_t i = base + (size_t)u * kThreads;
    if (i < count) dst[i] = v[u];
  }
}

// Read count vectors, write one word per workgroup.
__global__ void __launch_bounds__(kThreads) hbm_probe_read(const uint4* __restrict__ src,
                                                           unsigned* __restrict__ out, size_t count) {
  const size_t base = (size_t)blockIdx.x * kThreads * kPerThread + threadIdx.x;
  unsigned acc = 0;
  uint4 v[kPerThread];
#pragma unroll
  for (int u = 0; u < kPerThread; ++u) {
    const size_t i = base + (size_t)u * kThreads;
    v[u] = (i < count) ? src[i] : make_uint4(0, 0, 0, 0);
  }
#pragma unroll
  for (int u = 0; u < kPerThread; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  // xor over the workgroup's lanes is not needed for the measurement: one lane per wave writes
  if ((threadIdx.x & 63) == 0) out[blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6)] = acc;
}

int main(int argc, char** argv) {
  const size_t mib = argc > 1 ? std::strtoull(argv[1], nullptr, 10) : 4096;
  const int iters = argc > 2 ? std::atoi(argv[2]) : 10;
  const size_t bytes = mib << 20;
  const size_t count = bytes / sizeof(uint4);
  const size_t blocks = (count + (size_t)kThreads * kPerThread - 1) / ((size_t)kThreads * kPerThread);
  if (blocks == 0 || blocks > 0x7fffffffull) {
    std::fprintf(stderr, "size out of range\n");
    return 1;
  }
  uint4 *src = nullptr, *dst = nullptr;
  unsigned* out = nullptr;
  CHECK(hipMalloc(&src, bytes));
  CHECK(hipMalloc(&dst, bytes));
  CHECK(hipMalloc(&out, blocks * (kThreads / 64) * sizeof(unsigned)));
  CHECK(hipMemset(src, 1, bytes));
  CHECK(hipMemset(dst, 0, bytes));
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0));
  CHECK(hipEventCreate(&e1));
  for (int which = 0; which < 2; ++which) {
    float best = 1e30f, total = 0.0f;
    for (int it = 0; it < iters + 2; ++it) {
      CHECK(hipEventRecord(e0, nullptr));
      if (which == 0)
        hipLaunchKernelGGL(hbm_probe_copy, dim3((unsigned)blocks), dim3(kThreads), 0, nullptr, src, dst, count);
      else
        hipLaunchKernelGGL(hbm_probe_read, dim3((unsigned)blocks), dim3(kThreads), 0, nullptr, src, out, count);
      CHECK(hipGetLastError());
      CHECK(hipEventRecord(e1, nullptr));
      CHECK(hipEventSynchronize(e1));
      float ms = 0.0f;
      CHECK(hipEventElapsedTime(&ms, e0, e1));
      if (it >= 2) {
        total += ms;
        if (ms < best) best = ms;
      }
    }
    const double moved = which == 0 ? 2.0 * bytes : 1.0 * bytes;
    std::printf("%s: buffer %zu MiB, bytes moved per launch %.0f, avg %.4f ms (%.1f GB/s), best %.4f ms (%.1f GB/s)\n",
                which == 0 ? "hbm_probe_copy" : "hbm_probe_read", mib, moved, total / iters,
                moved / (total / iters) * 1e-6, best, moved / best * 1e-6);
  }
  CHECK(hipFree(src));
  CHECK(hipFree(dst));
  CHECK(hipFree(out));
  return 0;
}
