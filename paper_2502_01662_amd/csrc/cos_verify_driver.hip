// cos_verify_driver.hip -- a plain C++ caller of the C ABI: no Python, no PyTorch.
//
// Fills device buffers of a given shape with counter-based pseudo-random inputs,
// calls cos_verify a number of times and reports the time per call.  It exists
// for two reasons: as the program rocprofv3 counter runs are pointed at (nothing
// else launches kernels in the process), and as a check that the library is
// usable through its header alone.  The inputs have the workloads' shapes but
// not their recipes; parity with the float64 reference is tested elsewhere.
//
//   cos_verify_driver [n=4] [B=512] [gamma=6] [V=256000] [dtype=bf16|f32|f16]
//                     [mode=ensemble|contrastive|mix] [calls=10]
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "cos_verify.h"

#define CHECK(x)                                                          \
  do {                                                                    \
    hipError_t e_ = (x);                                                  \
    if (e_ != hipSuccess) {                                               \
      std::fprintf(stderr, "%s failed: %s\n", #x, hipGetErrorString(e_)); \
      return 1;                                                           \
    }                                                                     \
  } while (0)

namespace {

// SplitMix64 finaliser: one independent 64-bit value per counter.
__host__ __device__ inline unsigned long long mix64(unsigned long long z) {
  z += 0x9e3779b97f4a7c15ull;
  z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
  z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
  return z ^ (z >> 31);
}

// Sum of four uniforms, centred and scaled: a bell-shaped spread of about +-7.
__device__ inline float bell(unsigned long long h) {
  const float a = (float)(h & 0xffff), b = (float)((h >> 16) & 0xffff);
  const float c = (float)((h >> 32) & 0xffff), d = (float)(h >> 48);
  return (a + b + c + d - 131070.0f) * (7.0f / 131070.0f);
}

template <typename T>
__device__ inline T narrow(float v);
template <>
__device__ inline float narrow<float>(float v) {
  return v;
}
template <>
__device__ inline unsigned short narrow<unsigned short>(float v) {  // bfloat16, round to nearest even
  unsigned int u = __float_as_uint(v);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (unsigned short)(u >> 16);
}
template <>
__device__ inline _Float16 narrow<_Float16>(float v) {
  return (_Float16)v;
}

template <typename T>
__global__ void fill_logits(T* dst, size_t count, unsigned long long seed) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (size_t)gridDim.x * blockDim.x)
    dst[i] = narrow<T>(bell(mix64(seed + i)));
}

__global__ void fill_side(int* drafts, int* proposer, double* u_accept, double* u_resample, int n, int B,
                          int gamma, int V, unsigned long long seed) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < B * gamma) {
    drafts[i] = (int)(mix64(seed + 3 * (unsigned long long)i) % (unsigned long long)V);
    // half of the drafts are accepted outright (u = 0), the rest take their chance
    const unsigned long long h = mix64(seed + 3 * (unsigned long long)i + 1);
    u_accept[i] = (h & 1) ? 0.0 : (double)(h >> 11) * (1.0 / 9007199254740992.0);
  }
  if (i < B) {
    proposer[i] = (int)(mix64(seed + 0x1000000ull + i) % (unsigned long long)n);
    u_resample[i] = (double)(mix64(seed + 0x2000000ull + i) >> 11) * (1.0 / 9007199254740992.0);
  }
}

}  // namespace

int main(int argc, char** argv) {
  const int n = argc > 1 ? std::atoi(argv[1]) : 4;
  const int B = argc > 2 ? std::atoi(argv[2]) : 512;
  const int gamma = argc > 3 ? std::atoi(argv[3]) : 6;
  const int V = argc > 4 ? std::atoi(argv[4]) : 256000;
  const char* dts = argc > 5 ? argv[5] : "bf16";
  const char* ms = argc > 6 ? argv[6] : "ensemble";
  const int calls = argc > 7 ? std::atoi(argv[7]) : 10;
  cos_dtype_t dt;
  if (!std::strcmp(dts, "bf16")) dt = COS_DTYPE_BF16;
  else if (!std::strcmp(dts, "f32")) dt = COS_DTYPE_F32;
  else if (!std::strcmp(dts, "f16")) dt = COS_DTYPE_F16;
  else { std::fprintf(stderr, "dtype must be bf16, f32 or f16\n"); return 2; }
  cos_combine_t mode;
  std::vector<double> weights;
  if (!std::strcmp(ms, "ensemble")) {
    mode = COS_COMBINE_ENSEMBLE;
    weights.assign(n > 0 ? n : 1, n > 0 ? 1.0 / n : 1.0);
  } else if (!std::strcmp(ms, "contrastive")) {
    mode = COS_COMBINE_CONTRASTIVE;
    weights = {0.5, 0.1};
  } else if (!std::strcmp(ms, "mix")) {
    mode = COS_COMBINE_LOGIT_MIX;
    weights.assign(n > 0 ? n : 1, n > 0 ? 1.0 / n : 1.0);
  } else { std::fprintf(stderr, "mode must be ensemble, contrastive or mix\n"); return 2; }
  const size_t ws_bytes = cos_verify_workspace_bytes(n, B, gamma, V, dt, mode);
  if (ws_bytes == 0 || B < 1 || calls < 1) {
    std::fprintf(stderr, "unsupported shape\n");
    return 2;
  }
  const size_t esize = dt == COS_DTYPE_F32 ? 4 : 2;
  const size_t count = (size_t)n * B * (gamma + 1) * V;
  void *logits = nullptr, *ws = nullptr;
  int *drafts = nullptr, *proposer = nullptr, *alen = nullptr, *toks = nullptr;
  double *ua = nullptr, *ur = nullptr;
  CHECK(hipMalloc(&logits, count * esize));
  CHECK(hipMalloc(&ws, ws_bytes));
  CHECK(hipMalloc(&drafts, sizeof(int) * B * gamma));
  CHECK(hipMalloc(&proposer, sizeof(int) * B));
  CHECK(hipMalloc(&alen, sizeof(int) * B));
  CHECK(hipMalloc(&toks, sizeof(int) * B * (gamma + 1)));
  CHECK(hipMalloc(&ua, sizeof(double) * B * gamma));
  CHECK(hipMalloc(&ur, sizeof(double) * B));
  const unsigned long long seed = 20250201ull;
  if (dt == COS_DTYPE_F32)
    hipLaunchKernelGGL(fill_logits<float>, dim3(4096), dim3(256), 0, nullptr, (float*)logits, count, seed);
  else if (dt == COS_DTYPE_BF16)
    hipLaunchKernelGGL(fill_logits<unsigned short>, dim3(4096), dim3(256), 0, nullptr, (unsigned short*)logits, count, seed);
  else
    hipLaunchKernelGGL(fill_logits<_Float16>, dim3(4096), dim3(256), 0, nullptr, (_Float16*)logits, count, seed);
  hipLaunchKernelGGL(fill_side, dim3((B * gamma + 255) / 256 + 1), dim3(256), 0, nullptr, drafts, proposer, ua, ur,
                     n, B, gamma, V, seed ^ 0xabcdefull);
  CHECK(hipGetLastError());
  CHECK(hipDeviceSynchronize());

  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0));
  CHECK(hipEventCreate(&e1));
  auto call = [&]() {
    return cos_verify(logits, dt, n, B, gamma, V, drafts, proposer, mode, weights.data(), ua, ur, alen, toks, ws,
                      ws_bytes, nullptr, nullptr);
  };
  for (int i = 0; i < 2; ++i) {  // warm-up
    const cos_status_t st = call();
    if (st != COS_OK) {
      std::fprintf(stderr, "cos_verify: %s\n", cos_status_string(st));
      return 1;
    }
  }
  CHECK(hipDeviceSynchronize());
  CHECK(hipEventRecord(e0, nullptr));
  for (int i = 0; i < calls; ++i)
    if (call() != COS_OK) return 1;
  CHECK(hipEventRecord(e1, nullptr));
  CHECK(hipEventSynchronize(e1));
  float total_ms = 0.0f;
  CHECK(hipEventElapsedTime(&total_ms, e0, e1));
  std::vector<int> h_alen(B);
  CHECK(hipMemcpy(h_alen.data(), alen, sizeof(int) * B, hipMemcpyDeviceToHost));
  std::vector<long> hist(gamma + 1, 0);
  for (int b = 0; b < B; ++b)
    if (h_alen[b] >= 0 && h_alen[b] <= gamma) ++hist[h_alen[b]];
  const double per_call = total_ms / calls;
  const double bytes = (double)count * esize;
  std::printf("cos_verify n=%d B=%d gamma=%d V=%d %s %s: %.4f ms per call over %d calls, %.0f GB/s of logits, "
              "%.0f positions/s; accepted_len histogram",
              n, B, gamma, V, dts, ms, per_call, calls, bytes / per_call * 1e-6, (double)B * gamma / per_call * 1e3);
  for (int j = 0; j <= gamma; ++j) std::printf(" %ld", hist[j]);
  std::printf("\n");
  return 0;
}
