// Stand-alone driver of the C ABI (no Python, no torch): allocates one pipeline stage's
// matrices with hipMalloc, fills them with hash-generated low-rank-free noise, and runs
// optimizer steps.  It exists for hardware-counter runs (a profiler attaches to a plain
// executable) and as a C usage example of include/br.h.
//
//   br_native_bench [--layers N] [--steps K] [--freq F] [--math 0|1|2] [--copy-calibration] [--mfma-peak]
//
// --mfma-peak runs br_mfma_peak instead of the optimizer: a register-only loop of
// v_mfma_f32_32x32x2_f32 on every SIMD, once as a ~25 ms burst and once sustained for ~0.5 s,
// which gives the FP32 matrix-core rate this machine actually holds (clocks drop under
// sustained load), the practical ceiling for the contraction kernel.
//
// --copy-calibration additionally launches br_plain_copy on 1 GiB (reads 1 GiB, writes 1 GiB),
// the known-traffic kernel against which HBM byte counters are scaled.
#include <hip/hip_runtime.h>

#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../include/br.h"

#define CHECK_HIP(x)                                                                  \
  do {                                                                                \
    hipError_t e_ = (x);                                                              \
    if (e_ != hipSuccess) {                                                           \
      std::fprintf(stderr, "%s failed: %s\n", #x, hipGetErrorString(e_));             \
      return 1;                                                                       \
    }                                                                                 \
  } while (0)

__global__ void br_fill_noise(float* dst, size_t n, unsigned seed, float scale) {
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
    unsigned x = (unsigned)i * 2654435761u ^ seed;
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    dst[i] = scale * ((float)(x >> 8) * (1.0f / 8388608.0f) - 1.0f);  // uniform in [-scale, scale)
  }
}

__global__ void br_plain_copy(const float4* __restrict__ src, float4* __restrict__ dst, size_t n4) {
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) dst[i] = src[i];
}

typedef float br_floatx16 __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(256) void br_mfma_peak(float* out, int iters) {
  br_floatx16 c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
  unsigned x = (threadIdx.x + 1 + blockIdx.x * 977) * 2654435761u;
  x ^= x >> 15; x *= 0x2c1b3c6du; x ^= x >> 12;
  float a0 = (float)(x & 0xffff) / 65536.f - 0.5f, a1 = (float)(x >> 16) / 65536.f - 0.5f;
  x *= 0x297a2d39u; x ^= x >> 15;
  float b0 = (float)(x & 0xffff) / 65536.f - 0.5f, b1 = (float)(x >> 16) / 65536.f - 0.5f;
  for (int i = 0; i < iters; i += 4) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      c0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, c0, 0, 0, 0);
      c1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, c1, 0, 0, 0);
      c2 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, c2, 0, 0, 0);
      c3 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, c3, 0, 0, 0);
    }
  }
  float s = 0.f;
  for (int v = 0; v < 16; ++v) s += c0[v] + c1[v] + c2[v] + c3[v];
  if (s == 12345.f) out[threadIdx.x] = s;  // keeps the loop alive
}

static int mfma_peak() {
  float* d = nullptr;
  CHECK_HIP(hipMalloc(&d, 4096));
  hipEvent_t e0, e1;
  CHECK_HIP(hipEventCreate(&e0));
  CHECK_HIP(hipEventCreate(&e1));
  const int grid = 256 * 4;  // four workgroups of four waves per compute unit
  const int iters_list[2] = {50000, 1000000};
  for (int k = 0; k < 2; ++k) {
    hipLaunchKernelGGL(br_mfma_peak, dim3(grid), dim3(256), 0, 0, d, 1000);
    CHECK_HIP(hipDeviceSynchronize());
    CHECK_HIP(hipEventRecord(e0, 0));
    hipLaunchKernelGGL(br_mfma_peak, dim3(grid), dim3(256), 0, 0, d, iters_list[k]);
    CHECK_HIP(hipEventRecord(e1, 0));
    CHECK_HIP(hipEventSynchronize(e1));
    float ms = 0.f;
    CHECK_HIP(hipEventElapsedTime(&ms, e0, e1));
    double flops = (double)grid * 4 * iters_list[k] * 4.0 * 4096.0;
    std::printf("br_mfma_peak %s: %.1f ms, %.1f TFLOP/s FP32 MFMA\n", k ? "sustained" : "burst", ms, flops / (ms * 1e-3) / 1e12);
  }
  CHECK_HIP(hipFree(d));
  return 0;
}

int main(int argc, char** argv) {
  int layers = 8, steps = 2, freq = 10, calib = 0, math = BR_MATH_F32;
  for (int i = 1; i < argc; ++i) {
    if (!std::strcmp(argv[i], "--layers") && i + 1 < argc) layers = std::atoi(argv[++i]);
    else if (!std::strcmp(argv[i], "--steps") && i + 1 < argc) steps = std::atoi(argv[++i]);
    else if (!std::strcmp(argv[i], "--freq") && i + 1 < argc) freq = std::atoi(argv[++i]);
    else if (!std::strcmp(argv[i], "--copy-calibration")) calib = 1;
    else if (!std::strcmp(argv[i], "--math") && i + 1 < argc) math = std::atoi(argv[++i]);
    else if (!std::strcmp(argv[i], "--mfma-peak")) return mfma_peak();
    else { std::fprintf(stderr, "unknown argument %s\n", argv[i]); return 2; }
  }
  const int64_t layer_shapes[7][2] = {{2560, 2560}, {2560, 2560}, {2560, 2560}, {2560, 2560},
                                      {2560, 6912}, {2560, 6912}, {6912, 2560}};
  std::vector<br_matrix_desc> descs;
  for (int l = 0; l < layers; ++l)
    for (int k = 0; k < 7; ++k) descs.push_back(br_matrix_desc{layer_shapes[k][0], layer_shapes[k][1], BR_F32, BR_F32, 1, 0});
  br_hparams hp;
  std::memset(&hp, 0, sizeof(hp));
  hp.beta1 = 0.9f; hp.beta2 = 0.95f; hp.eps = 1e-8f; hp.stat_beta = -1.f;
  hp.geometry = BR_BILATERAL; hp.source = BR_SRC_SECOND; hp.power_iters = 1; hp.math = math;
  hp.cache_rotated_moment = 1;
  size_t state = 0, scratch = 0;
  if (br_workspace_bytes(descs.data(), (int32_t)descs.size(), &hp, &state, &scratch) != BR_OK) {
    std::fprintf(stderr, "br_workspace_bytes: %s\n", br_last_error(nullptr));
    return 1;
  }
  void* ws = nullptr;
  CHECK_HIP(hipMalloc(&ws, state + scratch));
  std::vector<void*> params(descs.size());
  std::vector<const void*> grads(descs.size());
  for (size_t i = 0; i < descs.size(); ++i) {
    size_t n = (size_t)descs[i].m * descs[i].n;
    float *w, *g;
    CHECK_HIP(hipMalloc(&w, n * 4));
    CHECK_HIP(hipMalloc(&g, n * 4));
    hipLaunchKernelGGL(br_fill_noise, dim3(2048), dim3(256), 0, 0, w, n, 17u + (unsigned)i, 0.02f);
    hipLaunchKernelGGL(br_fill_noise, dim3(2048), dim3(256), 0, 0, g, n, 9001u + (unsigned)i, 0.01f);
    params[i] = w;
    grads[i] = g;
  }
  CHECK_HIP(hipDeviceSynchronize());
  if (calib) {
    const size_t n4 = (size_t)1 << 26;  // 1 GiB of float4
    float4 *a, *b;
    CHECK_HIP(hipMalloc(&a, n4 * 16));
    CHECK_HIP(hipMalloc(&b, n4 * 16));
    CHECK_HIP(hipMemset(a, 0, n4 * 16));
    for (int r = 0; r < 3; ++r) hipLaunchKernelGGL(br_plain_copy, dim3(4096), dim3(256), 0, 0, a, b, n4);
    CHECK_HIP(hipDeviceSynchronize());
    CHECK_HIP(hipFree(a));
    CHECK_HIP(hipFree(b));
  }
  br_ctx* ctx = nullptr;
  if (br_init(&ctx, descs.data(), (int32_t)descs.size(), &hp, ws, state + scratch, nullptr) != BR_OK) {
    std::fprintf(stderr, "br_init: %s\n", br_last_error(nullptr));
    return 1;
  }
  CHECK_HIP(hipDeviceSynchronize());
  auto t0 = std::chrono::steady_clock::now();
  for (int t = 1; t <= steps; ++t) {
    br_status st = br_accumulate_stats(ctx, grads.data(), (int32_t)grads.size());
    if (st == BR_OK && freq > 0 && t % freq == 0) st = br_refresh_basis(ctx);
    if (st == BR_OK) st = br_step(ctx, params.data(), grads.data(), (int32_t)grads.size(), 1e-3f);
    if (st != BR_OK) {
      std::fprintf(stderr, "step %d failed: %s\n", t, br_last_error(ctx));
      return 1;
    }
  }
  CHECK_HIP(hipDeviceSynchronize());
  double ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
  std::printf("%s: %zu matrices, %d steps (refresh every %d), %.2f ms/step, state %.2f GB, scratch %.2f GB\n",
              br_version(), descs.size(), steps, freq, ms / steps, state / 1e9, scratch / 1e9);
  br_destroy(ctx);
  return 0;
}
