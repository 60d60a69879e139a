// Stand-alone driver of the C ABI (no Python, no torch): allocates one pipeline stage's
// matrices with hipMalloc, fills them with hash-generated noise, and runs optimizer steps through
// the calls of include/br.h and nothing else.  It exists for hardware-counter runs (a profiler
// attaches to a plain executable) and as a C usage example of the library.
//
//   br_native_bench [--layers N] [--steps K] [--freq F] [--math 0|1|2] [--refresh-math 0|1|2] [--small] [--copy-calibration]
//   br_native_bench --host-only
//
// --small uses one layer of small ragged matrices instead of the 3B-class shapes (a quick run of every
// call, e.g. under host-side sanitizers).  --host-only needs no GPU: it walks the library's host logic
// alone (workspace planning for many configurations, every argument check of br_workspace_bytes,
// br_init and br_clip_gradients_static) and is what a sanitizer build runs on a machine without one.
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

// Host logic only: no kernel is launched, no device memory exists.  Returns the number of surprises.
static int host_only() {
  int bad = 0;
  auto expect = [&](br_status got, br_status want, const char* what) {
    if (got != want) { std::fprintf(stderr, "host-only: %s returned %d, expected %d (%s)\n", what, (int)got, (int)want, br_last_error(nullptr)); ++bad; }
  };
  const int64_t shapes[][2] = {{1, 1}, {37, 53}, {256, 256}, {2560, 6912}, {6912, 2560}, {32000, 2560}, {13000, 40}, {1 << 20, 3}};
  size_t planned = 0;
  for (int math = 0; math < 3; ++math)
    for (int geometry = 0; geometry < 2; ++geometry)
      for (int source = 0; source < 2; ++source)
        for (int iters = 1; iters <= 2; ++iters)
          for (int cache = 0; cache < 2; ++cache)
            for (int dt = 0; dt < 2; ++dt) {
              std::vector<br_matrix_desc> d;
              for (auto& sh : shapes) d.push_back(br_matrix_desc{sh[0], sh[1], dt, dt, 1, 0});
              for (int r = 0; r < 70; ++r) d.push_back(br_matrix_desc{96, 130, dt, BR_F32, r % 7 != 0, 0});  // more than one launch batch
              br_hparams hp;
              std::memset(&hp, 0, sizeof(hp));
              hp.beta1 = 0.9f; hp.beta2 = 0.95f; hp.eps = 1e-8f; hp.stat_beta = -1.f;
              hp.geometry = geometry; hp.source = source; hp.power_iters = iters; hp.math = math; hp.cache_rotated_moment = cache;
              hp.stats_on_refresh_only = cache;
              hp.refresh_math = (geometry + source + iters) % 3;
              size_t st = 0, sc = 0;
              expect(br_workspace_bytes(d.data(), (int32_t)d.size(), &hp, &st, &sc), BR_OK, "br_workspace_bytes");
              if (st == 0 || sc == 0) { std::fprintf(stderr, "host-only: empty plan\n"); ++bad; }
              ++planned;
              // br_init's own checks, all ahead of any HIP call
              br_ctx* ctx = nullptr;
              expect(br_init(&ctx, d.data(), (int32_t)d.size(), &hp, nullptr, st + sc, nullptr), BR_ERR_INVALID_ARG, "br_init(null workspace)");
              expect(br_init(&ctx, d.data(), (int32_t)d.size(), &hp, reinterpret_cast<void*>(0x1010), st + sc, nullptr), BR_ERR_WORKSPACE, "br_init(misaligned)");
              expect(br_init(&ctx, d.data(), (int32_t)d.size(), &hp, reinterpret_cast<void*>(0x10000), st + sc - 1, nullptr), BR_ERR_WORKSPACE, "br_init(too small)");
              if (ctx) { std::fprintf(stderr, "host-only: a failed br_init left a context\n"); ++bad; }
            }
  br_hparams hp;
  std::memset(&hp, 0, sizeof(hp));
  hp.beta1 = 0.9f; hp.beta2 = 0.95f; hp.eps = 1e-8f; hp.stat_beta = -1.f; hp.power_iters = 1;
  br_matrix_desc one{8, 8, BR_F32, BR_F32, 1, 0};
  size_t st = 0, sc = 0;
  expect(br_workspace_bytes(nullptr, 1, &hp, &st, &sc), BR_ERR_INVALID_ARG, "null descriptors");
  expect(br_workspace_bytes(&one, 0, &hp, &st, &sc), BR_ERR_INVALID_ARG, "n_mats = 0");
  expect(br_workspace_bytes(&one, 1, &hp, nullptr, &sc), BR_ERR_INVALID_ARG, "null output");
  br_matrix_desc neg{-4, 8, BR_F32, BR_F32, 1, 0}, dty{8, 8, 7, BR_F32, 1, 0}, res{8, 8, BR_F32, BR_F32, 1, 5};
  expect(br_workspace_bytes(&neg, 1, &hp, &st, &sc), BR_ERR_SHAPE, "negative dimension");
  expect(br_workspace_bytes(&dty, 1, &hp, &st, &sc), BR_ERR_DTYPE, "unknown dtype");
  expect(br_workspace_bytes(&res, 1, &hp, &st, &sc), BR_ERR_INVALID_ARG, "reserved field");
  br_hparams h2 = hp; h2.power_iters = 0;
  expect(br_workspace_bytes(&one, 1, &h2, &st, &sc), BR_ERR_INVALID_ARG, "power_iters = 0");
  h2 = hp; h2.math = 9;
  expect(br_workspace_bytes(&one, 1, &h2, &st, &sc), BR_ERR_INVALID_ARG, "unknown math mode");
  h2 = hp; h2.stats_on_refresh_only = 2;
  expect(br_workspace_bytes(&one, 1, &h2, &st, &sc), BR_ERR_INVALID_ARG, "stats_on_refresh_only = 2");
  // the entry point without a context: argument checks come before anything touches a device
  void* g = reinterpret_cast<void*>(0x10000);
  float result_stub[2];
  expect(br_clip_gradients_static(nullptr, &g, 1, 1.f, result_stub, nullptr), BR_ERR_INVALID_ARG, "static clip: null descriptors");
  expect(br_clip_gradients_static(&one, &g, BR_STATIC_CLIP_MAX_MATS + 1, 1.f, result_stub, nullptr), BR_ERR_WORKSPACE, "static clip: too many");
  expect(br_clip_gradients_static(&one, &g, 1, 0.f, result_stub, nullptr), BR_ERR_INVALID_ARG, "static clip: max_norm = 0");
  expect(br_clip_gradients_static(&neg, &g, 1, 1.f, result_stub, nullptr), BR_ERR_SHAPE, "static clip: negative dimension");
  void* odd = reinterpret_cast<void*>(0x10004);
  expect(br_clip_gradients_static(&one, &odd, 1, 1.f, result_stub, nullptr), BR_ERR_INVALID_ARG, "static clip: misaligned gradient");
  std::printf("host-only: %zu configurations planned, %d surprises\n", planned, bad);
  return bad;
}

int main(int argc, char** argv) {
  if (argc == 2 && !std::strcmp(argv[1], "--host-only")) return host_only() ? 1 : 0;
  int layers = 8, steps = 2, freq = 10, calib = 0, math = BR_MATH_F32, small = 0, refresh_math = BR_REFRESH_AUTO;
  for (int i = 1; i < argc; ++i) {
    if (!std::strcmp(argv[i], "--layers") && i + 1 < argc) layers = std::atoi(argv[++i]);
    else if (!std::strcmp(argv[i], "--steps") && i + 1 < argc) steps = std::atoi(argv[++i]);
    else if (!std::strcmp(argv[i], "--freq") && i + 1 < argc) freq = std::atoi(argv[++i]);
    else if (!std::strcmp(argv[i], "--copy-calibration")) calib = 1;
    else if (!std::strcmp(argv[i], "--math") && i + 1 < argc) math = std::atoi(argv[++i]);
    else if (!std::strcmp(argv[i], "--small")) small = 1;
    else if (!std::strcmp(argv[i], "--refresh-math") && i + 1 < argc) refresh_math = std::atoi(argv[++i]);
    else { std::fprintf(stderr, "unknown argument %s\n", argv[i]); return 2; }
  }
  const int64_t big_shapes[7][2] = {{2560, 2560}, {2560, 2560}, {2560, 2560}, {2560, 2560},
                                    {2560, 6912}, {2560, 6912}, {6912, 2560}};
  const int64_t small_shapes[7][2] = {{264, 136}, {264, 136}, {200, 200}, {37, 53}, {1700, 40}, {136, 264}, {600, 72}};
  const int64_t (*layer_shapes)[2] = small ? small_shapes : big_shapes;
  std::vector<br_matrix_desc> descs;
  for (int l = 0; l < layers; ++l)
    for (int k = 0; k < 7; ++k) descs.push_back(br_matrix_desc{layer_shapes[k][0], layer_shapes[k][1], BR_F32, BR_F32, 1, 0});
  br_hparams hp;
  std::memset(&hp, 0, sizeof(hp));
  hp.beta1 = 0.9f; hp.beta2 = 0.95f; hp.eps = 1e-8f; hp.stat_beta = -1.f;
  hp.geometry = BR_BILATERAL; hp.source = BR_SRC_SECOND; hp.power_iters = 1; hp.math = math;
  hp.cache_rotated_moment = 1;
  hp.refresh_math = refresh_math;
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
