// Elementwise kernels of the basis-rotation step: HBM-bound, coalesced 16-byte non-temporal accesses,
// batched over matrices through blockIdx.y.  Every workgroup takes ONE CONTIGUOUS range of its matrix,
// and the launches use as many workgroups as it takes to give each thread a single 16-byte item (see
// grid_for): a 2-read 1-write stream then runs at 6.4 TB/s, against 5.2 TB/s with long per-workgroup
// ranges and 4.6 TB/s with a grid-stride loop.
//
//   br_ema_first_moment   M <- beta1 M + (1-beta1) G                  (Algorithm 1, first-moment update)
//   br_adam_rotated       S~ <- beta2 S~ + (1-beta2) G~.G~ ; X = M~/sqrt(S~+eps)
//                                                                     (Algorithm 1, second moment and update)
//   br_adam_plain         the same update for tensors that are not rotated, fused with
//                         the weight update (embeddings, LM head: experimental details)
//   br_norm_finalize      deterministic second stage of the per-matrix norm reductions
#include "br_internal.h"

namespace br {

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

// Round to nearest even; NaN stays NaN (quiet).  Branch-free: both results are computed, one is selected.
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  const uint32_t u = __float_as_uint(f);
  const uint32_t rounded = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
  const uint32_t quiet = (u >> 16) | 0x0040u;
  return (uint16_t)(((u & 0x7fffffffu) > 0x7f800000u) ? quiet : rounded);
}

typedef float f4v __attribute__((ext_vector_type(4)));
typedef unsigned u2v __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float4 nt_load4(const float* base, int64_t i4) {
  const f4v v = __builtin_nontemporal_load(reinterpret_cast<const f4v*>(base) + i4);
  return make_float4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ void nt_store4(float* base, int64_t i4, float4 a) {
  const f4v v = {a.x, a.y, a.z, a.w};
  __builtin_nontemporal_store(v, reinterpret_cast<f4v*>(base) + i4);
}

__device__ __forceinline__ float4 nt_load_grad4(const void* g, int64_t i4, bool bf16) {
  if (bf16) {
    const u2v raw = __builtin_nontemporal_load(reinterpret_cast<const u2v*>(g) + i4);
    return make_float4(__uint_as_float(raw.x << 16), __uint_as_float(raw.x & 0xffff0000u),
                       __uint_as_float(raw.y << 16), __uint_as_float(raw.y & 0xffff0000u));
  }
  return nt_load4(reinterpret_cast<const float*>(g), i4);
}

// This workgroup's contiguous share [lo, hi) of n4 16-byte items.
__device__ __forceinline__ void block_range(int64_t n4, int64_t* lo, int64_t* hi) {
  const int64_t per = (n4 + gridDim.x - 1) / gridDim.x;
  *lo = (int64_t)blockIdx.x * per;
  *hi = (*lo + per < n4) ? *lo + per : n4;
}

__device__ __forceinline__ float4 load_grad4(const void* g, int64_t i4, bool bf16) {
  if (bf16) {
    uint2 raw = reinterpret_cast<const uint2*>(g)[i4];
    return make_float4(__uint_as_float(raw.x << 16), __uint_as_float(raw.x & 0xffff0000u),
                       __uint_as_float(raw.y << 16), __uint_as_float(raw.y & 0xffff0000u));
  }
  return reinterpret_cast<const float4*>(g)[i4];
}

__device__ __forceinline__ float load_grad1(const void* g, int64_t i, bool bf16) {
  return bf16 ? bf16_bits_to_f32(reinterpret_cast<const uint16_t*>(g)[i]) : reinterpret_cast<const float*>(g)[i];
}

__global__ __launch_bounds__(256) void br_ema_first_moment(BrPtrBatch p, int64_t count, int grad_bf16, float beta1) {
  const int b = blockIdx.y;
  const void* __restrict__ G = p.in0[b];
  float* __restrict__ M = reinterpret_cast<float*>(p.out0[b]);
  float* __restrict__ G32 = reinterpret_cast<float*>(p.out1[b]);
  const float w = 1.0f - beta1;
  const int64_t n4 = count >> 2;
  int64_t lo, hi;
  block_range(n4, &lo, &hi);
  // two independent 16-byte pairs in flight per lane
  for (int64_t i = lo + threadIdx.x; i < hi; i += 2 * 256) {
    const int64_t j = i + 256;
    const bool two = j < hi;
    float4 g0 = nt_load_grad4(G, i, grad_bf16);
    float4 m0 = nt_load4(M, i);
    float4 g1 = g0, m1 = m0;
    if (two) {
      g1 = nt_load_grad4(G, j, grad_bf16);
      m1 = nt_load4(M, j);
    }
    m0.x = beta1 * m0.x + w * g0.x;
    m0.y = beta1 * m0.y + w * g0.y;
    m0.z = beta1 * m0.z + w * g0.z;
    m0.w = beta1 * m0.w + w * g0.w;
    nt_store4(M, i, m0);
    if (G32) nt_store4(G32, i, g0);
    if (two) {
      m1.x = beta1 * m1.x + w * g1.x;
      m1.y = beta1 * m1.y + w * g1.y;
      m1.z = beta1 * m1.z + w * g1.z;
      m1.w = beta1 * m1.w + w * g1.w;
      nt_store4(M, j, m1);
      if (G32) nt_store4(G32, j, g1);
    }
  }
  if (blockIdx.x == 0) {
    for (int64_t i = (n4 << 2) + threadIdx.x; i < count; i += blockDim.x) {
      float g = load_grad1(G, i, grad_bf16);
      M[i] = beta1 * M[i] + w * g;
      if (G32) G32[i] = g;
    }
  }
}

template <class Args>
__device__ __forceinline__ float adam_x(float m, float s, const Args& a) {
  float num = m * a.c1;
  float den = s * a.c2;
  return a.eps_outside ? num / (sqrtf(den) + a.eps) : num / sqrtf(den + a.eps);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// partials layout: [batch][2][gridDim.x]
__global__ __launch_bounds__(256) void br_adam_rotated(BrAdamBatch p, int64_t count, BrAdamArgs a, float* partials) {
  __shared__ float red[2][4];
  const int b = blockIdx.y;
  float* __restrict__ GX = p.GX[b];
  float* __restrict__ S = p.S[b];
  float* __restrict__ Mr = p.Mrot[b];
  const float w2 = 1.0f - a.beta2;
  const float w1 = 1.0f - a.beta1;
  const bool upd = a.update_mrot != 0;
  const int64_t n4 = count >> 2;
  int64_t lo, hi;
  block_range(n4, &lo, &hi);
  float sg = 0.f, sx = 0.f;
  auto body = [&](float4 g, float4 s, float4 m, int64_t i) {
    if (upd) {
      m.x = a.beta1 * m.x + w1 * g.x;
      m.y = a.beta1 * m.y + w1 * g.y;
      m.z = a.beta1 * m.z + w1 * g.z;
      m.w = a.beta1 * m.w + w1 * g.w;
      nt_store4(Mr, i, m);
    }
    s.x = a.beta2 * s.x + w2 * (g.x * g.x);
    s.y = a.beta2 * s.y + w2 * (g.y * g.y);
    s.z = a.beta2 * s.z + w2 * (g.z * g.z);
    s.w = a.beta2 * s.w + w2 * (g.w * g.w);
    float4 x = make_float4(adam_x(m.x, s.x, a), adam_x(m.y, s.y, a), adam_x(m.z, s.z, a), adam_x(m.w, s.w, a));
    nt_store4(S, i, s);
    nt_store4(GX, i, x);
    if (a.compute_norms) {
      sg += g.x * g.x + g.y * g.y + g.z * g.z + g.w * g.w;
      sx += x.x * x.x + x.y * x.y + x.z * x.z + x.w * x.w;
    }
  };
  // two independent 16-byte triples in flight per lane
  for (int64_t i = lo + threadIdx.x; i < hi; i += 2 * 256) {
    const int64_t j = i + 256;
    const bool two = j < hi;
    float4 g0 = nt_load4(GX, i);
    float4 s0 = nt_load4(S, i);
    float4 m0 = nt_load4(Mr, i);
    float4 g1 = g0, s1 = s0, m1 = m0;
    if (two) {
      g1 = nt_load4(GX, j);
      s1 = nt_load4(S, j);
      m1 = nt_load4(Mr, j);
    }
    body(g0, s0, m0, i);
    if (two) body(g1, s1, m1, j);
  }
  if (blockIdx.x == 0) {
    for (int64_t i = (n4 << 2) + threadIdx.x; i < count; i += blockDim.x) {
      float g = GX[i];
      float m = Mr[i];
      if (upd) {
        m = a.beta1 * m + w1 * g;
        Mr[i] = m;
      }
      float s = a.beta2 * S[i] + w2 * (g * g);
      float x = adam_x(m, s, a);
      S[i] = s;
      GX[i] = x;
      if (a.compute_norms) {
        sg += g * g;
        sx += x * x;
      }
    }
  }
  if (a.compute_norms) {
    sg = wave_sum(sg);
    sx = wave_sum(sx);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) {
      red[0][wave] = sg;
      red[1][wave] = sx;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      float* dst = partials + (size_t)b * 2 * gridDim.x;
      dst[blockIdx.x] = (red[0][0] + red[0][1]) + (red[0][2] + red[0][3]);
      dst[gridDim.x + blockIdx.x] = (red[1][0] + red[1][1]) + (red[1][2] + red[1][3]);
    }
  }
}

__global__ __launch_bounds__(64) void br_norm_finalize(const float* partials, int nblocks, BrAdamBatch out) {
  const int b = blockIdx.x;
  const float* src = partials + (size_t)b * 2 * nblocks;
  float s0 = 0.f, s1 = 0.f;
  for (int i = threadIdx.x; i < nblocks; i += 64) {
    s0 += src[i];
    s1 += src[nblocks + i];
  }
  s0 = wave_sum(s0);
  s1 = wave_sum(s1);
  if (threadIdx.x == 0 && out.norms[b]) {
    out.norms[b][0] = s0;
    out.norms[b][1] = s1;
  }
}

struct ShadowPtrs {
  uint16_t* p[BR_MAXB];
};

__global__ __launch_bounds__(256) void br_adam_plain(BrPtrBatch p, ShadowPtrs sh, int64_t count, BrPlainArgs a) {
  const int b = blockIdx.y;
  const void* __restrict__ G = p.in0[b];
  const float* __restrict__ M = reinterpret_cast<const float*>(p.in1[b]);
  float* __restrict__ S = reinterpret_cast<float*>(p.out0[b]);
  float* __restrict__ W = reinterpret_cast<float*>(p.out1[b]);
  uint16_t* __restrict__ shadow = sh.p[b];
  const float w = 1.0f - a.beta2;
  bool bad = false;
  auto one = [&](float g, float m, float s, float wo, float& so, float& wn) {
    so = a.beta2 * s + w * (g * g);
    wn = a.decay * wo - a.lr * adam_x(m, so, a);
    bad |= (__float_as_uint(wn) & 0x7f800000u) == 0x7f800000u;
  };
  // every workgroup walks one contiguous range, 16 bytes per lane and array, non-temporal
  const int64_t n4 = count >> 2;
  int64_t lo, hi;
  block_range(n4, &lo, &hi);
  for (int64_t i = lo + threadIdx.x; i < hi; i += 256) {
    const float4 g = nt_load_grad4(G, i, a.grad_bf16);
    const float4 m = nt_load4(M, i), s = nt_load4(S, i), wo = nt_load4(W, i);
    float4 so, wn;
    one(g.x, m.x, s.x, wo.x, so.x, wn.x);
    one(g.y, m.y, s.y, wo.y, so.y, wn.y);
    one(g.z, m.z, s.z, wo.z, so.z, wn.z);
    one(g.w, m.w, s.w, wo.w, so.w, wn.w);
    nt_store4(S, i, so);
    nt_store4(W, i, wn);
    if (shadow) {
      const u2v o = {(uint32_t)f32_to_bf16_rne(wn.x) | ((uint32_t)f32_to_bf16_rne(wn.y) << 16),
                     (uint32_t)f32_to_bf16_rne(wn.z) | ((uint32_t)f32_to_bf16_rne(wn.w) << 16)};
      __builtin_nontemporal_store(o, reinterpret_cast<u2v*>(shadow) + i);
    }
  }
  if (blockIdx.x == 0) {
    for (int64_t i = (n4 << 2) + threadIdx.x; i < count; i += blockDim.x) {
      float so, wn;
      one(load_grad1(G, i, a.grad_bf16), M[i], S[i], W[i], so, wn);
      S[i] = so;
      W[i] = wn;
      if (shadow) shadow[i] = f32_to_bf16_rne(wn);
    }
  }
  if (a.health && __any(bad) && (threadIdx.x & 63) == 0) atomicAdd(a.health + BR_HEALTH_NONFINITE_WEIGHT, 1);
}

// in0 = gradient (f32 or bf16); one partial per workgroup at partials[slot0 + blockIdx.y * gridDim.x + blockIdx.x]
__global__ __launch_bounds__(256) void br_grad_sumsq(BrPtrBatch p, int64_t count, int grad_bf16, float* partials, int slot0) {
  __shared__ float red[4];
  const void* __restrict__ G = p.in0[blockIdx.y];
  const int64_t n4 = count >> 2;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  // four independent 16-byte loads in flight per thread, each with a running sum of its own
  auto sq = [](const float4& g) { return (g.x * g.x + g.y * g.y) + (g.z * g.z + g.w * g.w); };
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (; i + 3 * stride < n4; i += 4 * stride) {
    const float4 g0 = nt_load_grad4(G, i, grad_bf16);
    const float4 g1 = nt_load_grad4(G, i + stride, grad_bf16);
    const float4 g2 = nt_load_grad4(G, i + 2 * stride, grad_bf16);
    const float4 g3 = nt_load_grad4(G, i + 3 * stride, grad_bf16);
    s0 += sq(g0);
    s1 += sq(g1);
    s2 += sq(g2);
    s3 += sq(g3);
  }
  for (; i < n4; i += stride) s0 += sq(nt_load_grad4(G, i, grad_bf16));
  float s = (s0 + s1) + (s2 + s3);
  if (blockIdx.x == 0) {
    for (int64_t j = (n4 << 2) + threadIdx.x; j < count; j += blockDim.x) {
      float g = load_grad1(G, j, grad_bf16);
      s += g * g;
    }
  }
  s = wave_sum(s);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) partials[slot0 + blockIdx.y * gridDim.x + blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}

__global__ __launch_bounds__(256) void br_clip_finalize(const float* __restrict__ partials, int n, float max_norm,
                                                        float* __restrict__ result) {
  __shared__ float red[4];
  float s = 0.f;
  for (int i = threadIdx.x; i < n; i += 256) s += partials[i];
  s = wave_sum(s);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    const float norm = sqrtf((red[0] + red[1]) + (red[2] + red[3]));
    const float f = max_norm / (norm + 1e-6f);
    result[0] = norm;
    result[1] = f < 1.0f ? f : 1.0f;
  }
}

__global__ __launch_bounds__(256) void br_scale_inplace(BrPtrBatch p, int64_t count, int grad_bf16,
                                                        const float* __restrict__ result) {
  const float f = result[1];
  if (f >= 1.0f) return;  // nothing to clip: leave the gradients untouched
  void* G = p.out0[blockIdx.y];
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  if (grad_bf16) {
    uint16_t* g = reinterpret_cast<uint16_t*>(G);
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += stride)
      g[i] = f32_to_bf16_rne(f * bf16_bits_to_f32(g[i]));
  } else {
    float* g = reinterpret_cast<float*>(G);
    const int64_t n4 = count >> 2;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
      float4 v = reinterpret_cast<float4*>(g)[i];
      v.x *= f; v.y *= f; v.z *= f; v.w *= f;
      reinterpret_cast<float4*>(g)[i] = v;
    }
    if (blockIdx.x == 0)
      for (int64_t i = (n4 << 2) + threadIdx.x; i < count; i += blockDim.x) g[i] *= f;
  }
}

// Delay Compensation: G <- G + lambda G.G.(Wn - Ws).  Four entries per lane; every workgroup walks
// one contiguous range of its matrix.
__global__ __launch_bounds__(256) void br_delay_compensate(BrPtrBatch p, int64_t count, int grad_bf16, int param_bf16,
                                                           float lambda) {
  const void* __restrict__ Wn = p.in0[blockIdx.y];
  const void* __restrict__ Ws = p.in1[blockIdx.y];
  void* __restrict__ G = p.out0[blockIdx.y];
  const int64_t n4 = count >> 2;
  int64_t lo, hi;
  block_range(n4, &lo, &hi);
  for (int64_t i = lo + threadIdx.x; i < hi; i += 256) {
    float4 g = nt_load_grad4(G, i, grad_bf16);
    const float4 a = nt_load_grad4(Wn, i, param_bf16), b = nt_load_grad4(Ws, i, param_bf16);
    g.x += lambda * g.x * g.x * (a.x - b.x);
    g.y += lambda * g.y * g.y * (a.y - b.y);
    g.z += lambda * g.z * g.z * (a.z - b.z);
    g.w += lambda * g.w * g.w * (a.w - b.w);
    if (grad_bf16) {
      const u2v o = {(uint32_t)f32_to_bf16_rne(g.x) | ((uint32_t)f32_to_bf16_rne(g.y) << 16),
                     (uint32_t)f32_to_bf16_rne(g.z) | ((uint32_t)f32_to_bf16_rne(g.w) << 16)};
      __builtin_nontemporal_store(o, reinterpret_cast<u2v*>(G) + i);
    } else {
      nt_store4(reinterpret_cast<float*>(G), i, g);
    }
  }
  if (blockIdx.x == 0) {
    for (int64_t i = (n4 << 2) + threadIdx.x; i < count; i += blockDim.x) {
      float g = load_grad1(G, i, grad_bf16);
      g += lambda * g * g * (load_grad1(Wn, i, param_bf16) - load_grad1(Ws, i, param_bf16));
      if (grad_bf16) reinterpret_cast<uint16_t*>(G)[i] = f32_to_bf16_rne(g);
      else reinterpret_cast<float*>(G)[i] = g;
    }
  }
}

struct MatPtrs {
  float* p[BR_MAXB];
};

__global__ __launch_bounds__(256) void br_set_identity(MatPtrs m, int n) {
  float* __restrict__ Q = m.p[blockIdx.y];
  const int64_t total = (int64_t)n * n;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
    int64_t r = i / n;
    Q[i] = (i - r * n == r) ? 1.0f : 0.0f;
  }
}

__global__ __launch_bounds__(256) void br_bf16_to_f32(const uint16_t* __restrict__ src, float* __restrict__ dst,
                                                      int64_t count) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += stride)
    dst[i] = bf16_bits_to_f32(src[i]);
}

// One 16-byte item per thread and as many workgroups as that takes: on this memory system a 2-read 1-write stream
// over 634 M entries runs at 6.45 TB/s that way, against 5.15 TB/s with 16 workgroups per compute unit that each
// loop over a long contiguous range (measured with caps of 4 K, 16 K, 64 K, 256 K and 1 M workgroups per launch:
// 5.15, 5.35, 5.67, 6.10, 6.44 TB/s; no further gain beyond 1 M).  `cap` bounds the grid where a kernel indexes
// per-workgroup partial sums by it.
static inline int grid_for(int64_t work_items, int batch, int64_t cap = 0x7fffffffLL) {
  (void)batch;
  int64_t blocks = (work_items + 255) / 256;
  if (blocks > cap) blocks = cap;
  if (blocks < 1) blocks = 1;
  return (int)blocks;
}

}  // namespace br

hipError_t br_launch_ema(hipStream_t s, const BrPtrBatch& p, int batch, int64_t count, int grad_bf16, float beta1) {
  if (batch <= 0 || count <= 0) return hipSuccess;
  dim3 grid(br::grid_for(count / 4 + 1, batch), batch);
  hipLaunchKernelGGL(br::br_ema_first_moment, grid, dim3(256), 0, s, p, count, grad_bf16, beta1);
  return hipGetLastError();
}

hipError_t br_launch_adam_rotated(hipStream_t s, const BrAdamBatch& p, int batch, int64_t count, const BrAdamArgs& a,
                                  float* norm_partials) {
  if (batch <= 0 || count <= 0) return hipSuccess;
  const int gx = br::grid_for(count / 4 + 1, batch, a.compute_norms ? BR_NORM_BLOCKS : 0x7fffffffLL);
  dim3 grid(gx, batch);
  hipLaunchKernelGGL(br::br_adam_rotated, grid, dim3(256), 0, s, p, count, a, norm_partials);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || !a.compute_norms) return e;
  hipLaunchKernelGGL(br::br_norm_finalize, dim3(batch), dim3(64), 0, s, norm_partials, gx, p);
  return hipGetLastError();
}

hipError_t br_launch_adam_plain(hipStream_t s, const BrPtrBatch& p, uint16_t* const* shadow, int batch, int64_t count,
                                const BrPlainArgs& a) {
  if (batch <= 0 || count <= 0) return hipSuccess;
  br::ShadowPtrs sh;
  for (int i = 0; i < BR_MAXB; ++i) sh.p[i] = (i < batch) ? shadow[i] : nullptr;
  dim3 grid(br::grid_for(count / 4 + 1, batch), batch);
  hipLaunchKernelGGL(br::br_adam_plain, grid, dim3(256), 0, s, p, sh, count, a);
  return hipGetLastError();
}

hipError_t br_launch_sumsq(hipStream_t s, const BrPtrBatch& p, int batch, int64_t count, int grad_bf16, float* partials,
                           int slot0) {
  if (batch <= 0 || count <= 0) return hipSuccess;
  hipLaunchKernelGGL(br::br_grad_sumsq, dim3(BR_CLIP_BLOCKS, batch), dim3(256), 0, s, p, count, grad_bf16, partials, slot0);
  return hipGetLastError();
}

hipError_t br_launch_clip_finalize(hipStream_t s, const float* partials, int n_partials, float max_norm, float* result) {
  hipLaunchKernelGGL(br::br_clip_finalize, dim3(1), dim3(256), 0, s, partials, n_partials, max_norm, result);
  return hipGetLastError();
}

hipError_t br_launch_scale_inplace(hipStream_t s, const BrPtrBatch& p, int batch, int64_t count, int grad_bf16,
                                   const float* result) {
  if (batch <= 0 || count <= 0) return hipSuccess;
  dim3 grid(br::grid_for(grad_bf16 ? count : count / 4 + 1, batch), batch);
  hipLaunchKernelGGL(br::br_scale_inplace, grid, dim3(256), 0, s, p, count, grad_bf16, result);
  return hipGetLastError();
}

hipError_t br_launch_delay_compensate(hipStream_t s, const BrPtrBatch& p, int batch, int64_t count, int grad_bf16,
                                      int param_bf16, float lambda) {
  if (batch <= 0 || count <= 0) return hipSuccess;
  dim3 grid(br::grid_for(count / 4 + 1, batch), batch);
  hipLaunchKernelGGL(br::br_delay_compensate, grid, dim3(256), 0, s, p, count, grad_bf16, param_bf16, lambda);
  return hipGetLastError();
}

hipError_t br_launch_set_identity(hipStream_t s, float* const* mats, int batch, int n) {
  if (batch <= 0 || n <= 0) return hipSuccess;
  br::MatPtrs m;
  for (int i = 0; i < BR_MAXB; ++i) m.p[i] = (i < batch) ? mats[i] : nullptr;
  dim3 grid(br::grid_for((int64_t)n * n, batch), batch);
  hipLaunchKernelGGL(br::br_set_identity, grid, dim3(256), 0, s, m, n);
  return hipGetLastError();
}

hipError_t br_launch_bf16_to_f32(hipStream_t s, const uint16_t* src, float* dst, int64_t count) {
  if (count <= 0) return hipSuccess;
  hipLaunchKernelGGL(br::br_bf16_to_f32, dim3(br::grid_for(count, 1)), dim3(256), 0, s, src, dst, count);
  return hipGetLastError();
}
