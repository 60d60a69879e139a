// Stand-alone measurement probes (NOT part of the library and not a user of its C ABI): machine peaks
// and single-kernel timings that call the library's internal launchers directly.  They are the source of
// the machine-peak figures the kernels are judged against.
//
//   br_probes --mfma-peak
//   br_probes --stream-peak
//   br_probes --tile-store
//   br_probes --lowp-gemm M N K BATCH NPROD MIRROR
//   br_probes --f32-gemm M N K BATCH TA TB QR LDC BETA
//
// --f32-gemm times the FP32 matrix-core contraction alone at one shape (10 launches), e.g. the
// trailing updates of the QR: QR = 1 selects the variant the factorisation uses, LDC > N updates
// a block inside a wider matrix, BETA != 0 makes the kernel read C as well.
//
// --lowp-gemm checks and times the BF16 matrix-core contraction alone: BATCH products
// C = A B^T (A: M x K, B: N x K, FP32 noise split into BF16 planes by the library's own split
// kernel; MIRROR = 1 computes A A^T on the lower tiles only), compared on a strided sample of
// the output with a plain one-thread-per-element kernel that forms the same BF16 products in
// FP64, then timed over 10 launches.
//
// --mfma-peak: a register-only loop of v_mfma_f32_32x32x2_f32 on every SIMD, once as a ~25 ms burst
// and once sustained for ~0.5 s, which gives the FP32 matrix-core rate this machine actually holds
// (clocks drop under sustained load), the practical ceiling for the contraction kernel; then the
// same for v_mfma_f32_32x32x16_bf16.
//
// --stream-peak measures what the memory system sustains for the access mixes of the elementwise
// kernels on 1 GiB arrays of noise: reads only, writes only, a copy, and the 2-read 1-write mix of
// the first-moment update, each workgroup walking one contiguous range (as the library's kernels
// do) and, for comparison, the last one with a grid-stride loop.
#include <hip/hip_runtime.h>

#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../include/br.h"
#include "br_internal.h"

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

typedef float br_f4 __attribute__((ext_vector_type(4)));

// mode 0: read, 1: write, 2: copy a -> b, 3: b = 0.9 b + 0.1 a; contiguous range per workgroup, or grid-stride
__global__ __launch_bounds__(256) void br_stream(const br_f4* __restrict__ a, br_f4* __restrict__ b, size_t n4, int mode, int strided) {
  size_t lo, hi, step;
  if (strided) {
    lo = (size_t)blockIdx.x * 256; hi = n4; step = (size_t)gridDim.x * 256;
  } else {
    const size_t per = (n4 + gridDim.x - 1) / gridDim.x;
    lo = (size_t)blockIdx.x * per; hi = (lo + per < n4) ? lo + per : n4; step = 256;
  }
  br_f4 acc = {0.f, 0.f, 0.f, 0.f};
  for (size_t i = lo + threadIdx.x; i < hi; i += step) {
    if (mode == 0) acc += __builtin_nontemporal_load(a + i);
    else if (mode == 1) __builtin_nontemporal_store(br_f4{1.f, 2.f, 3.f, 4.f}, b + i);
    else if (mode == 2) __builtin_nontemporal_store(__builtin_nontemporal_load(a + i), b + i);
    else __builtin_nontemporal_store(0.9f * __builtin_nontemporal_load(b + i) + 0.1f * __builtin_nontemporal_load(a + i), b + i);
  }
  if (mode == 0 && acc.x == 1.2345f) b[0] = acc;
}

// ---- --tile-store ----------------------------------------------------------------------------
// What one 512-thread workgroup per compute unit can write: each workgroup stores 256 x 256 FP32 tiles of a
// large row-major matrix, one after the other, waiting for its stores at the end of every tile (as a contraction
// kernel's epilogue does).  mode 0: 4-byte stores in the arrangement of a 32 x 32 matrix-instruction accumulator
// (a lane = one column, four consecutive rows per group); mode 1: the same values in 16-byte stores (a lane = four
// consecutive columns of one row); mode 2: 16-byte stores, a wave writing one whole 1 KB tile row per instruction.
__global__ __launch_bounds__(512) void br_tile_store(float* __restrict__ C, int ldc, int tiles_n, int total_tiles, int mode) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 2, wn = wave & 3, li = lane & 31, lk = lane >> 5;
  for (int v = blockIdx.x; v < total_tiles; v += gridDim.x) {
    const int tm = v / tiles_n, tn = v - tm * tiles_n;
    float* __restrict__ T = C + (size_t)tm * 256 * ldc + (size_t)tn * 256;
    const float x = (float)v;
    if (mode == 0) {
#pragma unroll
      for (int a = 0; a < 8; ++a) {
        const int mi = a >> 1, ni = a & 1;
        const int col = (wn * 2 + ni) * 32 + li;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int row = (wm * 4 + mi) * 32 + 8 * (e >> 2) + 4 * lk + (e & 3);
          T[(size_t)row * ldc + col] = x + e;
        }
      }
    } else if (mode == 1) {
#pragma unroll
      for (int a = 0; a < 8; ++a) {
        const int mi = a >> 1, ni = a & 1;
        const int colq = (wn * 2 + ni) * 32 + (li & ~3);
#pragma unroll
        for (int vg = 0; vg < 4; ++vg) {
          const int row = (wm * 4 + mi) * 32 + 8 * vg + 4 * lk + (lane & 3);
          *reinterpret_cast<br_f4*>(T + (size_t)row * ldc + colq) = br_f4{x, x + 1.f, x + 2.f, x + 3.f};
        }
      }
    } else {
#pragma unroll
      for (int r = 0; r < 32; ++r) {
        const int row = wave * 32 + r;
        *reinterpret_cast<br_f4*>(T + (size_t)row * ldc + lane * 4) = br_f4{x, x + 1.f, x + 2.f, x + 3.f};
      }
    }
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
  }
}

static int tile_store() {
  const int n = 16384, tiles_n = n / 256, total = tiles_n * tiles_n;
  float* c;
  CHECK_HIP(hipMalloc(&c, (size_t)n * n * 4));
  CHECK_HIP(hipMemset(c, 0, (size_t)n * n * 4));
  hipEvent_t e0, e1;
  CHECK_HIP(hipEventCreate(&e0));
  CHECK_HIP(hipEventCreate(&e1));
  for (int grid : {256, 64})
    for (int mode = 0; mode < 3; ++mode) {
      hipLaunchKernelGGL(br_tile_store, dim3(grid), dim3(512), 0, 0, c, n, tiles_n, total, mode);
      CHECK_HIP(hipDeviceSynchronize());
      CHECK_HIP(hipEventRecord(e0, 0));
      for (int r = 0; r < 5; ++r) hipLaunchKernelGGL(br_tile_store, dim3(grid), dim3(512), 0, 0, c, n, tiles_n, total, mode);
      CHECK_HIP(hipEventRecord(e1, 0));
      CHECK_HIP(hipEventSynchronize(e1));
      float ms = 0.f;
      CHECK_HIP(hipEventElapsedTime(&ms, e0, e1));
      const double per_tile_us = ms / 5 * 1e3 / ((double)total / grid);
      std::printf("br_tile_store grid %3d mode %d: %.3f ms per GiB, %.2f us per 256 KB tile and workgroup, %.0f GB/s\n", grid, mode, ms / 5,
                  per_tile_us, (double)n * n * 4 / (ms / 5 * 1e-3) / 1e9);
    }
  CHECK_HIP(hipFree(c));
  return 0;
}

static int stream_peak() {
  const size_t n4 = (size_t)1 << 26;  // 1 GiB per array
  br_f4 *a, *b;
  CHECK_HIP(hipMalloc(&a, n4 * 16));
  CHECK_HIP(hipMalloc(&b, n4 * 16));
  hipLaunchKernelGGL(br_fill_noise, dim3(4096), dim3(256), 0, 0, (float*)a, n4 * 4, 1u, 1.0f);
  hipLaunchKernelGGL(br_fill_noise, dim3(4096), dim3(256), 0, 0, (float*)b, n4 * 4, 2u, 1.0f);
  hipEvent_t e0, e1;
  CHECK_HIP(hipEventCreate(&e0));
  CHECK_HIP(hipEventCreate(&e1));
  const char* names[5] = {"read", "write", "copy (1 read, 1 write)", "2 reads, 1 write", "2 reads, 1 write, grid-stride loop"};
  const double arrays[5] = {1, 1, 2, 3, 3};
  for (int k = 0; k < 5; ++k) {
    const int mode = k < 4 ? k : 3, strided = k == 4;
    hipLaunchKernelGGL(br_stream, dim3(2048), dim3(256), 0, 0, a, b, n4, mode, strided);
    CHECK_HIP(hipDeviceSynchronize());
    CHECK_HIP(hipEventRecord(e0, 0));
    for (int r = 0; r < 5; ++r) hipLaunchKernelGGL(br_stream, dim3(2048), dim3(256), 0, 0, a, b, n4, mode, strided);
    CHECK_HIP(hipEventRecord(e1, 0));
    CHECK_HIP(hipEventSynchronize(e1));
    float ms = 0.f;
    CHECK_HIP(hipEventElapsedTime(&ms, e0, e1));
    std::printf("br_stream %-36s %7.3f ms  %6.0f GB/s\n", names[k], ms / 5, arrays[k] * n4 * 16 / (ms / 5 * 1e-3) / 1e9);
  }
  return 0;
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

typedef __bf16 br_bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned br_uintx4 __attribute__((ext_vector_type(4)));

// Same register-only loop on v_mfma_f32_32x32x16_bf16 with pseudo-random BF16 operands.
__global__ __launch_bounds__(256) void br_mfma_peak_bf16(float* out, int iters) {
  br_floatx16 c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
  unsigned x = (threadIdx.x + 1 + blockIdx.x * 977) * 2654435761u;
  br_uintx4 ua, ub, uc, ud;
  for (int e = 0; e < 4; ++e) {
    x ^= x >> 15; x *= 0x2c1b3c6du; x ^= x >> 12;
    ua[e] = (x & 0x807f807fu) | 0x3f003f00u;  // two BF16 values of magnitude 0.5 .. 1, random signs
    x *= 0x297a2d39u; x ^= x >> 15;
    ub[e] = (x & 0x807f807fu) | 0x3f003f00u;
    uc[e] = ua[e] ^ 0x80000000u;
    ud[e] = ub[e] ^ 0x00008000u;
  }
  const br_bf16x8 a0 = __builtin_bit_cast(br_bf16x8, ua), a1 = __builtin_bit_cast(br_bf16x8, uc);
  const br_bf16x8 b0 = __builtin_bit_cast(br_bf16x8, ub), b1 = __builtin_bit_cast(br_bf16x8, ud);
  for (int i = 0; i < iters; i += 4) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b0, c0, 0, 0, 0);
      c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b1, c1, 0, 0, 0);
      c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b0, c2, 0, 0, 0);
      c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b1, c3, 0, 0, 0);
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
  for (int waves = 1; waves <= 2; ++waves) {  // waves per SIMD
    for (int k = 0; k < 2; ++k) {
      const int g2 = 256 * waves;
      hipLaunchKernelGGL(br_mfma_peak_bf16, dim3(g2), dim3(256), 0, 0, d, 1000);
      CHECK_HIP(hipDeviceSynchronize());
      CHECK_HIP(hipEventRecord(e0, 0));
      hipLaunchKernelGGL(br_mfma_peak_bf16, dim3(g2), dim3(256), 0, 0, d, iters_list[k] / waves);
      CHECK_HIP(hipEventRecord(e1, 0));
      CHECK_HIP(hipEventSynchronize(e1));
      float ms = 0.f;
      CHECK_HIP(hipEventElapsedTime(&ms, e0, e1));
      double flops = (double)g2 * 4 * (iters_list[k] / waves) * 4.0 * 32768.0;
      std::printf("br_mfma_peak_bf16 %s, %d wave(s) per SIMD: %.1f ms, %.1f TFLOP/s BF16 MFMA\n", k ? "sustained" : "burst", waves, ms,
                  flops / (ms * 1e-3) / 1e12);
    }
  }
  CHECK_HIP(hipFree(d));
  return 0;
}

// ---- --lowp-gemm ---------------------------------------------------------------------------
__device__ inline float nb_bf16_round(float f) {
  unsigned u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return __uint_as_float(u & 0xffff0000u);
}

// ref[s] for sample s = (i, j) on a strided grid; err[0] = max |C - ref|, err[1] = max |ref| (as uint bits of floats)
__global__ void br_lowp_reference(const float* A, const float* B, const float* C, int M, int N, int K, int nprod, int si, int sj,
                                  int mirror, float alpha, unsigned* err) {
  const int ni = (M + si - 1) / si, nj = (N + sj - 1) / sj;
  const int s = blockIdx.x * blockDim.x + threadIdx.x;
  if (s >= ni * nj) return;
  const int i = (s / nj) * si, j = (s % nj) * sj;
  double acc = 0.0;
  for (int k = 0; k < K; ++k) {
    const float a = A[(size_t)i * K + k], b = B[(size_t)j * K + k];
    const float ah = nb_bf16_round(a), bh = nb_bf16_round(b);
    const float al = nb_bf16_round(a - ah), bl = nb_bf16_round(b - bh);
    double p = (double)ah * bh;
    if (nprod >= 3) p += (double)ah * bl + (double)al * bh;
    if (nprod == 4 && (!mirror || i / 256 == j / 256)) p += (double)al * bl;  // mirrored: diagonal tiles only
    acc += p;
  }
  const float ref = (float)(alpha * acc);
  const float d = fabsf(C[(size_t)i * N + j] - ref);
  atomicMax(&err[0], __float_as_uint(d));
  atomicMax(&err[1], __float_as_uint(fabsf(ref)));
}

static int lowp_gemm_bench(int M, int N, int K, int batch, int nprod, int mirror) {
  if (M <= 0 || N <= 0 || K <= 0 || batch < 1 || batch > BR_MAXB || (nprod != 1 && nprod != 3 && nprod != 4) || (mirror && M != N)) {
    std::fprintf(stderr, "bad --lowp-gemm arguments\n");
    return 2;
  }
  const BrPlaneLayout pa = br_plane_layout(M, K), pb = br_plane_layout(N, K);
  std::vector<float*> A(batch), B(batch), C(batch);
  std::vector<uint16_t*> Ap(batch), Bp(batch);
  for (int i = 0; i < batch; ++i) {
    CHECK_HIP(hipMalloc(&A[i], (size_t)M * K * 4));
    CHECK_HIP(hipMalloc(&C[i], (size_t)M * N * 4));
    CHECK_HIP(hipMalloc(&Ap[i], pa.elems * 4));
    hipLaunchKernelGGL(br_fill_noise, dim3(2048), dim3(256), 0, 0, A[i], (size_t)M * K, 101u + i, 1.0f);
    if (mirror) {
      B[i] = A[i];
      Bp[i] = Ap[i];
    } else {
      CHECK_HIP(hipMalloc(&B[i], (size_t)N * K * 4));
      CHECK_HIP(hipMalloc(&Bp[i], pb.elems * 4));
      hipLaunchKernelGGL(br_fill_noise, dim3(2048), dim3(256), 0, 0, B[i], (size_t)N * K, 7001u + i, 1.0f);
    }
    CHECK_HIP(hipMemset(C[i], 0xff, (size_t)M * N * 4));  // NaN pattern: unwritten outputs are caught
  }
  const int want_lo = nprod > 1;
  CHECK_HIP(br_launch_split_planes(0, A.data(), Ap.data(), batch, M, K, K, 0, want_lo));
  if (!mirror) CHECK_HIP(br_launch_split_planes(0, B.data(), Bp.data(), batch, N, K, K, 0, want_lo));
  BrLowpBatch lb;
  std::memset(&lb, 0, sizeof(lb));
  for (int i = 0; i < batch; ++i) { lb.A[i] = Ap[i]; lb.B[i] = Bp[i]; lb.C[i] = C[i]; }
  const float alpha = 0.5f;
  BrLowpArgs la{M, N, K, N, alpha, 0.f, batch, mirror, nprod};
  const char* name = nullptr;
  CHECK_HIP(br_launch_gemm_lowp(0, la, lb, &name));
  CHECK_HIP(hipDeviceSynchronize());
  unsigned* err;
  CHECK_HIP(hipMalloc(&err, 8));
  const int si = M <= 512 ? 1 : 7, sj = N <= 512 ? 1 : 5;
  const int samples = ((M + si - 1) / si) * ((N + sj - 1) / sj);
  double worst = 0.0;
  for (int i = 0; i < batch; i += (batch > 2 ? batch - 1 : 1)) {
    CHECK_HIP(hipMemset(err, 0, 8));
    hipLaunchKernelGGL(br_lowp_reference, dim3((samples + 255) / 256), dim3(256), 0, 0, A[i], B[i], C[i], M, N, K, nprod, si, sj,
                       mirror, alpha, err);
    unsigned h[2];
    CHECK_HIP(hipMemcpy(h, err, 8, hipMemcpyDeviceToHost));
    float d, r;
    std::memcpy(&d, &h[0], 4);
    std::memcpy(&r, &h[1], 4);
    std::printf("matrix %d: max |C - ref| = %.3e, max |ref| = %.3e, ratio %.3e\n", i, d, r, d / r);
    if (!(d / r < 1e-4)) worst = 1.0;
    if (d / r > worst) worst = d / r;
  }
  hipEvent_t e0, e1;
  CHECK_HIP(hipEventCreate(&e0));
  CHECK_HIP(hipEventCreate(&e1));
  const int reps = 20;
  // the first launches after an idle period run slower (the clocks ramp up): time the steady state
  for (int r = 0; r < reps; ++r) CHECK_HIP(br_launch_gemm_lowp(0, la, lb, nullptr));
  CHECK_HIP(hipEventRecord(e0, 0));
  for (int r = 0; r < reps; ++r) CHECK_HIP(br_launch_gemm_lowp(0, la, lb, nullptr));
  CHECK_HIP(hipEventRecord(e1, 0));
  CHECK_HIP(hipEventSynchronize(e1));
  float ms = 0.f;
  CHECK_HIP(hipEventElapsedTime(&ms, e0, e1));
  double flops = 2.0 * M * N * (double)K * batch * (mirror ? 0.5 : 1.0);
  std::printf("%s M=%d N=%d K=%d batch=%d mirror=%d: %.3f ms/launch, %.1f TFLOP/s (algorithmic), check %s\n", name, M, N, K, batch,
              mirror, ms / reps, flops / (ms / reps * 1e-3) / 1e12, worst < 1e-4 ? "OK" : "FAILED");
  return worst < 1e-4 ? 0 : 1;
}

// ---- --f32-gemm ----------------------------------------------------------------------------
// Times one batched FP32 contraction at a given shape: C (M x N, row stride LDC) <- beta C +
// alpha op(A) op(B), the operands stored with their natural row strides.  QR = 1 runs the
// variant used inside the QR factorisation.  Timing only (the parity tests cover the values).
static int f32_gemm_bench(int M, int N, int K, int batch, int ta, int tb, int qr, int ldc, float beta) {
  if (M <= 0 || N <= 0 || K <= 0 || batch < 1 || batch > BR_MAXB || ldc < N) {
    std::fprintf(stderr, "bad --f32-gemm arguments\n");
    return 2;
  }
  const size_t ea = (size_t)M * K, eb = (size_t)N * K, ec = (size_t)M * ldc;
  BrGemmBatch gb;
  std::memset(&gb, 0, sizeof(gb));
  for (int i = 0; i < batch; ++i) {
    float *a, *b, *c;
    CHECK_HIP(hipMalloc(&a, ea * 4));
    CHECK_HIP(hipMalloc(&b, eb * 4));
    CHECK_HIP(hipMalloc(&c, ec * 4));
    hipLaunchKernelGGL(br_fill_noise, dim3(2048), dim3(256), 0, 0, a, ea, 11u + i, 1.0f);
    hipLaunchKernelGGL(br_fill_noise, dim3(2048), dim3(256), 0, 0, b, eb, 911u + i, 1.0f);
    CHECK_HIP(hipMemset(c, 0, ec * 4));
    gb.A[i] = a; gb.B[i] = b; gb.C[i] = c;
  }
  BrGemmArgs a{M, N, K, ta ? M : K, tb ? K : N, ldc, ta, tb, 1e-3f, beta, batch, 0};
  a.qr_role = qr;
  float* partial = nullptr;
  if (qr) {
    a.partial_floats = (size_t)16 << 20;
    CHECK_HIP(hipMalloc(&partial, a.partial_floats * 4));
    a.partial = partial;
  }
  const char* name = nullptr;
  CHECK_HIP(br_launch_gemm(0, a, gb, &name));
  CHECK_HIP(hipDeviceSynchronize());
  hipEvent_t e0, e1;
  CHECK_HIP(hipEventCreate(&e0));
  CHECK_HIP(hipEventCreate(&e1));
  const int reps = 10;
  CHECK_HIP(hipEventRecord(e0, 0));
  for (int r = 0; r < reps; ++r) CHECK_HIP(br_launch_gemm(0, a, gb, nullptr));
  CHECK_HIP(hipEventRecord(e1, 0));
  CHECK_HIP(hipEventSynchronize(e1));
  float ms = 0.f;
  CHECK_HIP(hipEventElapsedTime(&ms, e0, e1));
  const double flops = 2.0 * M * N * (double)K * batch;
  std::printf("%s M=%d N=%d K=%d batch=%d ldc=%d beta=%g: %.3f ms/launch, %.1f TFLOP/s\n", name, M, N, K, batch, ldc, beta, ms / reps,
              flops / (ms / reps * 1e-3) / 1e12);
  return 0;
}

int main(int argc, char** argv) {
  if (argc == 11 && !std::strcmp(argv[1], "--f32-gemm"))
    return f32_gemm_bench(std::atoi(argv[2]), std::atoi(argv[3]), std::atoi(argv[4]), std::atoi(argv[5]), std::atoi(argv[6]),
                          std::atoi(argv[7]), std::atoi(argv[8]), std::atoi(argv[9]), (float)std::atof(argv[10]));
  if (argc == 8 && !std::strcmp(argv[1], "--lowp-gemm"))
    return lowp_gemm_bench(std::atoi(argv[2]), std::atoi(argv[3]), std::atoi(argv[4]), std::atoi(argv[5]), std::atoi(argv[6]),
                           std::atoi(argv[7]));
  if (argc == 2 && !std::strcmp(argv[1], "--mfma-peak")) return mfma_peak();
  if (argc == 2 && !std::strcmp(argv[1], "--stream-peak")) return stream_peak();
  if (argc == 2 && !std::strcmp(argv[1], "--tile-store")) return tile_store();
  std::fprintf(stderr, "usage: br_probes --mfma-peak | --stream-peak | --tile-store | --lowp-gemm M N K BATCH NPROD MIRROR | "
                       "--f32-gemm M N K BATCH TA TB QR LDC BETA\n");
  return 2;
}
