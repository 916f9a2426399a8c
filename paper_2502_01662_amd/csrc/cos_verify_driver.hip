// cos_verify_driver.hip -- a plain C++ caller of the C ABI: no Python, no PyTorch.
//
// Fills device buffers of a given shape with counter-based pseudo-random inputs,
// calls cos_verify a number of times and reports the time per call.  It exists
// for two reasons: as the program rocprofv3 counter runs are pointed at (nothing
// else launches kernels in the process), and as a check that the library is
// usable through its header alone.  The inputs have the workloads' shapes and
// the spread of their logits (independent N(0, 3^2) values), not their recipes;
// parity with the float64 reference is tested elsewhere.
//
//   cos_verify_driver [n=4] [B=512] [gamma=6] [V=256000] [dtype=bf16|f32|f16]
//                     [mode=ensemble|contrastive|mix] [calls=10] [alpha] [nomask]
//     alpha   also ask for the acceptance rates of every draft position
//     nomask  contrastive mode with alpha_cd = 0
//   cos_verify_driver calibrate [MiB per buffer = 1024] [iterations = 3]
//     plain copy and read kernels of known size: what fraction of the HBM peak a
//     trivial streaming kernel reaches, and the factors between what rocprofv3's
//     FETCH_SIZE / WRITE_SIZE counters report and the bytes really moved, which
//     scale the counters read for cos_verify's kernels.
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

// A normal variate of standard deviation 3 from one 64-bit hash (Box-Muller on its two halves): the
// spread of the workloads' logits, with their unbounded tails (a handful of tokens near the top).
__device__ inline float bell(unsigned long long h) {
  const float u1 = ((float)(h >> 40) + 0.5f) * (1.0f / 16777216.0f);            // (0, 1)
  const float u2 = ((float)((h >> 16) & 0xffffff) + 0.5f) * (1.0f / 16777216.0f);
  return 3.0f * sqrtf(-2.0f * logf(u1)) * cosf(6.28318530717958648f * u2);
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

// ---- calibration kernels: 8 16-byte vectors per thread ----
constexpr int kProbeThreads = 256;
constexpr int kProbePerThread = 8;

// dst[i] = src[i]: count vectors read, count vectors written.
__global__ void __launch_bounds__(kProbeThreads) hbm_probe_copy(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                                                size_t count) {
  const size_t base = (size_t)blockIdx.x * kProbeThreads * kProbePerThread + threadIdx.x;
  uint4 v[kProbePerThread];
#pragma unroll
  for (int u = 0; u < kProbePerThread; ++u) {
    const size_t i = base + (size_t)u * kProbeThreads;
    if (i < count) v[u] = src[i];
  }
#pragma unroll
  for (int u = 0; u < kProbePerThread; ++u) {
    const size_t i = base + (size_t)u * kProbeThreads;
    if (i < count) dst[i] = v[u];
  }
}

// Read count vectors (plain loads, or with the non-temporal hint cos_verify's streams carry), write one
// word per wavefront.
template <bool NT>
__global__ void __launch_bounds__(kProbeThreads) hbm_probe_read(const uint4* __restrict__ src, unsigned* __restrict__ out,
                                                                size_t count) {
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
  const size_t base = (size_t)blockIdx.x * kProbeThreads * kProbePerThread + threadIdx.x;
  unsigned acc = 0;
  u32x4 v[kProbePerThread];
#pragma unroll
  for (int u = 0; u < kProbePerThread; ++u) {
    const size_t i = base + (size_t)u * kProbeThreads;
    const u32x4* at = reinterpret_cast<const u32x4*>(src + (i < count ? i : 0));
    v[u] = NT ? __builtin_nontemporal_load(at) : *at;
  }
#pragma unroll
  for (int u = 0; u < kProbePerThread; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  // every lane's loads must matter (a store from one lane alone lets the compiler load for that lane alone)
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) acc ^= __shfl_xor(acc, d, 64);
  if ((threadIdx.x & 63) == 0) out[blockIdx.x * (kProbeThreads / 64) + (threadIdx.x >> 6)] = acc;
}

int calibrate(size_t mib, int iters) {
  const size_t bytes = mib << 20;
  const size_t count = bytes / sizeof(uint4);
  const size_t blocks = (count + (size_t)kProbeThreads * kProbePerThread - 1) / ((size_t)kProbeThreads * kProbePerThread);
  if (blocks == 0 || blocks > 0x7fffffffull || iters < 1) {
    std::fprintf(stderr, "size out of range\n");
    return 2;
  }
  uint4 *src = nullptr, *dst = nullptr;
  unsigned* out = nullptr;
  CHECK(hipMalloc(&src, bytes));
  CHECK(hipMalloc(&dst, bytes));
  CHECK(hipMalloc(&out, blocks * (kProbeThreads / 64) * sizeof(unsigned)));
  CHECK(hipMemset(src, 1, bytes));
  CHECK(hipMemset(dst, 0, bytes));
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0));
  CHECK(hipEventCreate(&e1));
  const char* names[3] = {"hbm_probe_copy", "hbm_probe_read<plain>", "hbm_probe_read<non-temporal>"};
  for (int which = 0; which < 3; ++which) {
    float best = 1e30f, total = 0.0f;
    for (int it = 0; it < iters + 2; ++it) {
      CHECK(hipEventRecord(e0, nullptr));
      const dim3 grid((unsigned)blocks), block(kProbeThreads);
      if (which == 0)
        hipLaunchKernelGGL(hbm_probe_copy, grid, block, 0, nullptr, src, dst, count);
      else if (which == 1)
        hipLaunchKernelGGL(hbm_probe_read<false>, grid, block, 0, nullptr, src, out, count);
      else
        hipLaunchKernelGGL(hbm_probe_read<true>, grid, block, 0, nullptr, src, out, count);
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
                names[which], mib, moved, total / iters, moved / (total / iters) * 1e-6, best, moved / best * 1e-6);
  }
  CHECK(hipFree(src));
  CHECK(hipFree(dst));
  CHECK(hipFree(out));
  return 0;
}

}  // namespace

int main(int argc, char** argv) {
  if (argc > 1 && !std::strcmp(argv[1], "calibrate"))
    return calibrate(argc > 2 ? std::strtoull(argv[2], nullptr, 10) : 1024, argc > 3 ? std::atoi(argv[3]) : 3);
  bool want_alpha = false, nomask = false;
  for (int i = 8; i < argc; ++i) {
    if (!std::strcmp(argv[i], "alpha")) want_alpha = true;
    else if (!std::strcmp(argv[i], "nomask")) nomask = true;
    else { std::fprintf(stderr, "unknown flag %s\n", argv[i]); return 2; }
  }
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
    weights = {0.5, nomask ? 0.0 : 0.1};
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
  double *ua = nullptr, *ur = nullptr, *alpha = nullptr;
  if (want_alpha) CHECK(hipMalloc(&alpha, sizeof(double) * B * gamma));
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
  cos_options_t opt = {};
  opt.struct_bytes = sizeof(opt);
  opt.alpha = alpha;
  auto call = [&]() {
    return cos_verify_ex(logits, dt, n, B, gamma, V, drafts, proposer, mode, weights.data(), ua, ur, alen, toks, ws,
                         ws_bytes, nullptr, &opt, nullptr);
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
  std::printf("cos_verify n=%d B=%d gamma=%d V=%d %s %s%s%s: %.4f ms per call over %d calls, %.0f GB/s of logits, "
              "%.0f positions/s; accepted_len histogram",
              n, B, gamma, V, dts, ms, nomask ? " (no mask)" : "", want_alpha ? " + acceptance rates" : "", per_call, calls,
              bytes / per_call * 1e-6, (double)B * gamma / per_call * 1e3);
  for (int j = 0; j <= gamma; ++j) std::printf(" %ld", hist[j]);
  std::printf("\n");
  return 0;
}
