// BF16 matrix-core contractions for the optimizer step (math modes BR_MATH_BF16 and
// BR_MATH_BF16X3): the statistics G G^T, G^T G (Algorithm 2 lines 2, 5), the rotations
// Q_L^T G Q_R (Algorithm 1 lines 8-9) and the rotate-back Q_L X Q_R^T (line 11).
//
// Operands are first rewritten as BF16 "planes" by br_split_planes:
//     hi = bf16(x),  lo = bf16(x - hi)            (round to nearest even)
// stored K-BLOCKED: element (row, k) of an R-row plane sits at ((k / 32) * R + row) * 32 + k % 32,
// so the 128 rows x 32 k that one workgroup needs per iteration are one contiguous 8 KB run of
// whole cache lines (a row-major plane would touch half of 128 different lines instead).
// optionally transposed, so that EVERY contraction has the form C[i][j] = sum_k A[i][k] B[j][k]
// with k contiguous in memory for both operands: the MFMA operand of a lane (8 consecutive k of
// one row) is then a single 16-byte load from LDS and no transposition happens in the kernel.
//   NPROD = 1: C = A_hi B_hi^T                                  (plain BF16 inputs)
//   NPROD = 3: C = A_hi B_hi^T + A_hi B_lo^T + A_lo B_hi^T      (16-bit mantissa inputs, FP32
//              accumulation: a product term is off by about 2^-16, the dropped lo*lo term)
//   NPROD = 4: adds A_lo B_lo^T.  Used for the statistics G G^T, G^T G, whose diagonal would
//              otherwise carry the systematic bias sum_k lo_k^2, and whose error the refresh
//              amplifies by the condition number of the statistics.
//
// Kernel: 128 x 128 output tile per 256-thread workgroup, four wave64s in 2 x 2, each 64 x 64 =
// four v_mfma_f32_32x32x16_bf16 accumulators; K advances 32 per iteration through double-buffered
// LDS; LDS rows are 64 data bytes + 16 pad, which makes the 16-byte operand reads conflict-free.
#include "br_internal.h"

namespace {

constexpr int LBM = 128, LBN = 128, LBK = 32;
constexpr int ROW_CHUNKS = 5;  // uint4 per LDS row: 4 data (32 bf16) + 1 pad
constexpr int NUM_XCD = 8;
constexpr int GROUP_M = 8;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

struct LowpKernArgs {
  int M, N, Kp;          // Kp: padded K (multiple of 32)
  int ldc;
  size_t a_plane, b_plane;  // distance from the hi plane to the lo plane, in elements
  float alpha, beta;
  int tiles_m, tiles_n, total_tiles, mirror;
};

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

__device__ __forceinline__ uint4 load_chunk(const uint16_t* __restrict__ p, bool ok) {
  uint4 v = make_uint4(0u, 0u, 0u, 0u);
  if (ok) v = *reinterpret_cast<const uint4*>(p);
  return v;
}

// Registers that carry the next K tile from global memory to LDS.
template <int NPLANES>
struct Stage {
  uint4 a[NPLANES][2], b[NPLANES][2];
  __device__ __forceinline__ void fetch(const uint16_t* __restrict__ Ah, const uint16_t* __restrict__ Bh,
                                        const LowpKernArgs& g, int m0, int n0, int k0, int lrow, int lchunk) {
    const int k = k0 + lchunk * 8;
#pragma unroll
    for (int p = 0; p < NPLANES; ++p) {
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int ra = m0 + lrow + 64 * i, rb = n0 + lrow + 64 * i;
        // K-blocked plane: element (row, k) at ((k / 32) * rows + row) * 32 + k % 32
        a[p][i] = load_chunk(Ah + p * g.a_plane + ((size_t)(k0 >> 5) * g.M + ra) * 32 + lchunk * 8, ra < g.M && k < g.Kp);
        b[p][i] = load_chunk(Bh + p * g.b_plane + ((size_t)(k0 >> 5) * g.N + rb) * 32 + lchunk * 8, rb < g.N && k < g.Kp);
      }
    }
  }
  __device__ __forceinline__ void stash(uint4 (*st)[128][ROW_CHUNKS], int lrow, int lchunk) const {
#pragma unroll
    for (int p = 0; p < NPLANES; ++p) {
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        st[p][lrow + 64 * i][lchunk] = a[p][i];
        st[2 + p][lrow + 64 * i][lchunk] = b[p][i];
      }
    }
  }
};

}  // namespace

namespace br {

template <int NPROD>
__global__ __launch_bounds__(256, 2) void br_gemm_bf16_mfma(LowpKernArgs g, BrLowpBatch batch) {
  // [stage][plane: A_hi, A_lo, B_hi, B_lo][row][chunk]
  __shared__ uint4 lds[2][4][128][ROW_CHUNKS];

  int bid = blockIdx.x;
  const int per = gridDim.x / NUM_XCD;
  if (bid < per * NUM_XCD) bid = (bid % NUM_XCD) * per + bid / NUM_XCD;
  const int mat = bid / g.total_tiles;
  const int t = bid - mat * g.total_tiles;
  int tm, tn;
  if (g.mirror) {
    int r = (int)((sqrtf(8.0f * (float)t + 1.0f) - 1.0f) * 0.5f);
    while ((r + 1) * (r + 2) / 2 <= t) ++r;
    while (r * (r + 1) / 2 > t) --r;
    tm = r;
    tn = t - r * (r + 1) / 2;
  } else {
    const int group = GROUP_M * g.tiles_n;
    const int grp = t / group;
    const int first_m = grp * GROUP_M;
    const int gm = min(GROUP_M, g.tiles_m - first_m);
    const int r = t - grp * group;
    tn = r / gm;
    tm = first_m + (r - tn * gm);
  }
  const uint16_t* __restrict__ Ah = batch.A[mat];
  const uint16_t* __restrict__ Bh = batch.B[mat];
  float* __restrict__ C = batch.C[mat];
  uint16_t* __restrict__ shadow = batch.shadow[mat];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = tm * LBM, n0 = tn * LBN;
  constexpr int NPLANES = (NPROD == 1) ? 1 : 2;

  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // per-thread load slots: rows (tid >> 2) and (tid >> 2) + 64, 16-byte chunk (tid & 3) of the K tile
  const int lrow = tid >> 2, lchunk = tid & 3;
  Stage<NPLANES> stg;
  const int lk = lane >> 5, li = lane & 31;
  auto mfma_tile = [&](int st) {
#pragma unroll
    for (int s = 0; s < LBK / 16; ++s) {
      bf16x8 a_hi[2], b_hi[2], a_lo[2], b_lo[2];
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        a_hi[q] = __builtin_bit_cast(bf16x8, lds[st][0][wm * 64 + q * 32 + li][s * 2 + lk]);
        b_hi[q] = __builtin_bit_cast(bf16x8, lds[st][2][wn * 64 + q * 32 + li][s * 2 + lk]);
        if (NPROD >= 3) {
          a_lo[q] = __builtin_bit_cast(bf16x8, lds[st][1][wm * 64 + q * 32 + li][s * 2 + lk]);
          b_lo[q] = __builtin_bit_cast(bf16x8, lds[st][3][wn * 64 + q * 32 + li][s * 2 + lk]);
        }
      }
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
          if (NPROD == 4)
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_lo[mi], b_lo[ni], acc[mi][ni], 0, 0, 0);
          if (NPROD >= 3) {
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_lo[mi], b_hi[ni], acc[mi][ni], 0, 0, 0);
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_hi[mi], b_lo[ni], acc[mi][ni], 0, 0, 0);
          }
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_hi[mi], b_hi[ni], acc[mi][ni], 0, 0, 0);
        }
    }
  };

  // Two K tiles are in flight from global memory (one register stage each) while a third is being
  // multiplied out of LDS: at BF16 matrix-core speed one tile of lookahead does not cover the
  // memory latency.
  const int nkt = (g.Kp + LBK - 1) / LBK;
  Stage<NPLANES> stg2;
  stg.fetch(Ah, Bh, g, m0, n0, 0, lrow, lchunk);
  if (nkt > 1) stg2.fetch(Ah, Bh, g, m0, n0, LBK, lrow, lchunk);
  stg.stash(lds[0], lrow, lchunk);
  __syncthreads();
  for (int kt = 0; kt < nkt; kt += 2) {
    // even tile kt: LDS stage 0; tile kt+1 waits in stg2; fetch kt+2 into stg
    if (kt + 2 < nkt) stg.fetch(Ah, Bh, g, m0, n0, (kt + 2) * LBK, lrow, lchunk);
    mfma_tile(0);
    if (kt + 1 < nkt) stg2.stash(lds[1], lrow, lchunk);
    __syncthreads();
    if (kt + 1 >= nkt) break;
    // odd tile kt+1: LDS stage 1; tile kt+2 waits in stg; fetch kt+3 into stg2
    if (kt + 3 < nkt) stg2.fetch(Ah, Bh, g, m0, n0, (kt + 3) * LBK, lrow, lchunk);
    mfma_tile(1);
    if (kt + 2 < nkt) stg.stash(lds[0], lrow, lchunk);
    __syncthreads();
  }

  const bool use_beta = (g.beta != 0.0f);
  const bool off_diag = g.mirror && (tm != tn);
#pragma unroll
  for (int mi = 0; mi < 2; ++mi) {
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) {
      const int col = n0 + wn * 64 + ni * 32 + li;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = m0 + wm * 64 + mi * 32 + 8 * (v >> 2) + 4 * lk + (v & 3);
        if (row < g.M && col < g.N) {
          size_t off = (size_t)row * (size_t)g.ldc + col;
          float val = g.alpha * acc[mi][ni][v];
          if (use_beta) val += g.beta * C[off];
          C[off] = val;
          if (shadow) shadow[off] = f32_to_bf16_rne(val);
          if (off_diag) C[(size_t)col * (size_t)g.ldc + row] = val;
        }
      }
    }
  }
}

// ---- operand preparation -----------------------------------------------------------------
struct SplitArgs {
  const float* src[BR_MAXB];
  uint16_t* dst[BR_MAXB];  // hi plane; the lo plane follows at +plane elements
};

// Same orientation: plane rows = source rows, k = source column, padded with zeros to ldp (multiple of 32).
__global__ __launch_bounds__(256) void br_split_planes(SplitArgs a, int R, int Ccols, int lds_, int ldp, size_t plane,
                                                       int want_lo) {
  const float* __restrict__ X = a.src[blockIdx.y];
  uint16_t* __restrict__ H = a.dst[blockIdx.y];
  const int chunks_per_row = ldp >> 3;
  const int64_t total = (int64_t)R * chunks_per_row;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
    const int r = (int)(i / chunks_per_row);
    const int c0 = (int)(i - (int64_t)r * chunks_per_row) * 8;
    float x[8];
    const float* row = X + (size_t)r * lds_;
    if (c0 + 7 < Ccols && ((lds_ & 3) == 0)) {
      float4 u = *reinterpret_cast<const float4*>(row + c0);
      float4 w = *reinterpret_cast<const float4*>(row + c0 + 4);
      x[0] = u.x; x[1] = u.y; x[2] = u.z; x[3] = u.w; x[4] = w.x; x[5] = w.y; x[6] = w.z; x[7] = w.w;
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) x[e] = (c0 + e < Ccols) ? row[c0 + e] : 0.f;
    }
    uint32_t hi[4], lo[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint16_t h0 = f32_to_bf16_rne(x[2 * e]), h1 = f32_to_bf16_rne(x[2 * e + 1]);
      hi[e] = (uint32_t)h0 | ((uint32_t)h1 << 16);
      const uint16_t l0 = f32_to_bf16_rne(x[2 * e] - bf16_to_f32(h0));
      const uint16_t l1 = f32_to_bf16_rne(x[2 * e + 1] - bf16_to_f32(h1));
      lo[e] = (uint32_t)l0 | ((uint32_t)l1 << 16);
    }
    const size_t o = ((size_t)(c0 >> 5) * R + r) * 32 + (c0 & 31);
    *reinterpret_cast<uint4*>(H + o) = make_uint4(hi[0], hi[1], hi[2], hi[3]);
    if (want_lo) *reinterpret_cast<uint4*>(H + plane + o) = make_uint4(lo[0], lo[1], lo[2], lo[3]);
  }
}

// Transposed: plane rows = source columns, k = source row, padded with zeros to ldp (multiple of 32).
// 64 x 64 tiles through LDS; blockIdx.x enumerates tiles.
__global__ __launch_bounds__(256) void br_split_planes_t(SplitArgs a, int R, int Ccols, int lds_, int ldp, size_t plane,
                                                         int want_lo) {
  __shared__ float tile[64][65];
  const float* __restrict__ X = a.src[blockIdx.y];
  uint16_t* __restrict__ H = a.dst[blockIdx.y];
  const int tiles_c = (Ccols + 63) >> 6;
  const int tr = blockIdx.x / tiles_c, tc = blockIdx.x - tr * tiles_c;
  const int r0 = tr * 64, c0 = tc * 64;
  const int tid = threadIdx.x;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int rr = i * 4 + (tid >> 6), cc = tid & 63;
    const int r = r0 + rr, c = c0 + cc;
    tile[rr][cc] = (r < R && c < Ccols) ? X[(size_t)r * lds_ + c] : 0.f;
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int cc = (tid >> 3) + 32 * i, rch = tid & 7;
    const int c = c0 + cc, rbase = r0 + rch * 8;
    if (c < Ccols && rbase < ldp) {
      uint32_t hi[4], lo[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float x0 = tile[rch * 8 + 2 * e][cc], x1 = tile[rch * 8 + 2 * e + 1][cc];
        const uint16_t h0 = f32_to_bf16_rne(x0), h1 = f32_to_bf16_rne(x1);
        hi[e] = (uint32_t)h0 | ((uint32_t)h1 << 16);
        const uint16_t l0 = f32_to_bf16_rne(x0 - bf16_to_f32(h0)), l1 = f32_to_bf16_rne(x1 - bf16_to_f32(h1));
        lo[e] = (uint32_t)l0 | ((uint32_t)l1 << 16);
      }
      const size_t o = ((size_t)(rbase >> 5) * Ccols + c) * 32 + (rbase & 31);
      *reinterpret_cast<uint4*>(H + o) = make_uint4(hi[0], hi[1], hi[2], hi[3]);
      if (want_lo) *reinterpret_cast<uint4*>(H + plane + o) = make_uint4(lo[0], lo[1], lo[2], lo[3]);
    }
  }
}

}  // namespace br

hipError_t br_launch_split_planes(hipStream_t s, const float* const* src, uint16_t* const* dst, int batch, int R, int Ccols,
                                  int ld_src, int transpose, int ldp, size_t plane, int want_lo) {
  if (batch <= 0 || R <= 0 || Ccols <= 0) return hipSuccess;
  if (batch > BR_MAXB || (ldp & 31) || ldp < (transpose ? R : Ccols)) return hipErrorInvalidValue;
  br::SplitArgs a;
  for (int i = 0; i < BR_MAXB; ++i) {
    a.src[i] = (i < batch) ? src[i] : nullptr;
    a.dst[i] = (i < batch) ? dst[i] : nullptr;
  }
  if (!transpose) {
    int64_t blocks = ((int64_t)R * (ldp >> 3) + 255) / 256;
    int64_t cap = (4096 + batch - 1) / batch;
    if (blocks > cap) blocks = cap;
    hipLaunchKernelGGL(br::br_split_planes, dim3((int)blocks, batch), dim3(256), 0, s, a, R, Ccols, ld_src, ldp, plane, want_lo);
  } else {
    // the padded tail r in [R, ldp) is covered because tiles extend to multiples of 64 >= ldp
    int64_t tiles = (int64_t)((R + 63) / 64) * ((Ccols + 63) / 64);
    if (tiles > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(br::br_split_planes_t, dim3((int)tiles, batch), dim3(256), 0, s, a, R, Ccols, ld_src, ldp, plane, want_lo);
  }
  return hipGetLastError();
}

hipError_t br_launch_gemm_lowp(hipStream_t s, const BrLowpArgs& a, const BrLowpBatch& b, const char** kernel_name) {
  if (kernel_name)
    *kernel_name = (a.nprod == 4) ? "br_gemm_bf16_mfma<4>" : (a.nprod == 3) ? "br_gemm_bf16_mfma<3>" : "br_gemm_bf16_mfma<1>";
  if (a.batch <= 0 || a.M <= 0 || a.N <= 0) return hipSuccess;
  if (a.batch > BR_MAXB || (a.Kp & 31)) return hipErrorInvalidValue;
  if (a.mirror && a.M != a.N) return hipErrorInvalidValue;
  LowpKernArgs k;
  k.M = a.M; k.N = a.N; k.Kp = a.Kp;
  k.ldc = a.ldc;
  k.a_plane = a.a_plane; k.b_plane = a.b_plane;
  k.alpha = a.alpha; k.beta = a.beta;
  k.tiles_m = (a.M + LBM - 1) / LBM;
  k.tiles_n = (a.N + LBN - 1) / LBN;
  k.mirror = a.mirror ? 1 : 0;
  k.total_tiles = k.mirror ? k.tiles_m * (k.tiles_m + 1) / 2 : k.tiles_m * k.tiles_n;
  long long grid = (long long)k.total_tiles * a.batch;
  if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
  if (a.nprod == 4)
    hipLaunchKernelGGL((br::br_gemm_bf16_mfma<4>), dim3((int)grid), dim3(256), 0, s, k, b);
  else if (a.nprod == 3)
    hipLaunchKernelGGL((br::br_gemm_bf16_mfma<3>), dim3((int)grid), dim3(256), 0, s, k, b);
  else
    hipLaunchKernelGGL((br::br_gemm_bf16_mfma<1>), dim3((int)grid), dim3(256), 0, s, k, b);
  return hipGetLastError();
}
