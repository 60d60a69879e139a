// Batched FP32 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x2_f32).
//
// Serves every dense contraction of the path: the statistics G G^T and G^T G
// (Algorithm 2, the updates of L and R), the power-iteration product L Q and the block-reflector
// updates of the QR (Section 3.2), the rotations Q_L^T G Q_R (Algorithm 1, the rotation step)
// and the rotate-back-and-apply W <- W - lr Q_L X Q_R^T (Algorithm 1, the parameter update).
//
// Design: a 128 x 128 output tile per 256-thread workgroup (four wave64s in a 2 x 2
// grid, each owning 64 x 64 = four 32 x 32 MFMA accumulators), K advanced 16 at a
// time through double-buffered LDS.  Both operands sit in LDS k-major ([k][m] and
// [k][n]) so that one MFMA operand fetch is one conflict-free ds_read_b32 per lane;
// operands whose storage is k-minor are transposed on their way into LDS.
// Workgroup ids are remapped so that each XCD (own L2) works on a contiguous run of
// tiles.
#include "br_internal.h"

#include <algorithm>

namespace {

constexpr int BM = 128;
constexpr int BN = 128;
constexpr int BK = 16;
constexpr int LDS_LD = 132;  // 128 + 4: keeps float4 rows 16-byte aligned, shifts banks by 4 per k
constexpr int NUM_XCD = 8;
constexpr int GROUP_M = 8;
constexpr int SYM_GROUP_M = 8;  // band height of the symmetric launches' triangular tile order (5 to 16 measure the same)

typedef float floatx16 __attribute__((ext_vector_type(16)));

struct GemmKernArgs {
  int M, N, K;
  int lda, ldb, ldc;
  float alpha, beta;
  int tiles_m, tiles_n;
  int total_tiles;
  int mirror;
  int splitk;        // SPLIT kernels only: number of K ranges per output tile
  int kt_per_split;  // K tiles (of BK) per range
  float* partial;    // SPLIT kernels with splitk > 1: [batch][splitk][M][N] partial products
  const int* skip;   // optional, one int per matrix: non-zero = this matrix's C is left untouched
  int* health;       // optional health words: a stored value that is not finite bumps BR_HEALTH_NONFINITE_WEIGHT
  BrAdamArgs adam;   // ADAM kernels only
};

__device__ __forceinline__ bool not_finite(float v) { return (__float_as_uint(v) & 0x7f800000u) == 0x7f800000u; }

__device__ __forceinline__ float adam_quotient(float m, float s, const BrAdamArgs& a) {
  const float num = m * a.c1, den = s * a.c2;
  return a.eps_outside ? num / (sqrtf(den) + a.eps) : num / sqrtf(den + a.eps);
}

// Round to nearest even; NaN stays NaN (quiet).  Branch-free: both results are computed, one is selected.
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  const uint32_t u = __float_as_uint(f);
  const uint32_t rounded = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
  const uint32_t quiet = (u >> 16) | 0x0040u;
  return (uint16_t)(((u & 0x7fffffffu) > 0x7f800000u) ? quiet : rounded);
}

// Load four consecutive elements of a stored row; out-of-range elements read as zero.
template <bool VEC>
__device__ __forceinline__ float4 load4(const float* __restrict__ base, int row, int col, int ld,
                                        int rows, int cols) {
  float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
  if (row < rows && col < cols) {
    const float* p = base + (size_t)row * (size_t)ld + col;
    if (VEC && col + 3 < cols) {
      v = *reinterpret_cast<const float4*>(p);
    } else {
      v.x = p[0];
      if (col + 1 < cols) v.y = p[1];
      if (col + 2 < cols) v.z = p[2];
      if (col + 3 < cols) v.w = p[3];
    }
  }
  return v;
}

// One operand tile (BK x 128 in LDS, [k][d]).  KMAJOR: the operand is stored with k as
// its row index (rows = K extent, cols = tile extent).  Otherwise it is stored with the
// tile dimension as its row index and is transposed while being written to LDS.
template <bool KMAJOR, bool VEC>
struct TileLoader {
  static constexpr int PASSES = BK / 8;       // 16-byte loads per thread for one BK x 128 tile
  static constexpr int TPR = BK / 4;          // threads per stored row of a k-minor operand
  static constexpr int RPP = 256 / TPR;       // rows per pass of a k-minor operand
  float4 r[PASSES];
  const float* fp[PASSES];  // per-thread source pointers of the unguarded path
  size_t fstep;             // their advance per K tile
  // Unguarded path for tiles that lie wholly inside the operands (and K a multiple of BK):
  // plain 16-byte loads through pointers that advance by a constant, no bounds logic.
  __device__ __forceinline__ void init_fast(const float* __restrict__ base, int ld, int d0, int k0, int tid) {
#pragma unroll
    for (int i = 0; i < PASSES; ++i) {
      if (KMAJOR) {
        int k = (tid >> 5) + 8 * i;
        int d = (tid & 31) * 4;
        fp[i] = base + (size_t)(k0 + k) * (size_t)ld + d0 + d;
      } else {
        int d = tid / TPR + RPP * i;
        int k = (tid % TPR) * 4;
        fp[i] = base + (size_t)(d0 + d) * (size_t)ld + k0 + k;
      }
    }
    fstep = KMAJOR ? (size_t)BK * (size_t)ld : (size_t)BK;
  }
  __device__ __forceinline__ void fetch_fast() {
#pragma unroll
    for (int i = 0; i < PASSES; ++i) {
      r[i] = *reinterpret_cast<const float4*>(fp[i]);
      fp[i] += fstep;
    }
  }
  __device__ __forceinline__ void fetch(const float* __restrict__ base, int ld, int d0, int k0,
                                        int D, int K, int tid) {
    if (KMAJOR) {
#pragma unroll
      for (int i = 0; i < PASSES; ++i) {
        int k = (tid >> 5) + 8 * i;
        int d = (tid & 31) * 4;
        r[i] = load4<VEC>(base, k0 + k, d0 + d, ld, K, D);
      }
    } else {
#pragma unroll
      for (int i = 0; i < PASSES; ++i) {
        int d = tid / TPR + RPP * i;
        int k = (tid % TPR) * 4;
        r[i] = load4<VEC>(base, d0 + d, k0 + k, ld, D, K);
      }
    }
  }
  __device__ __forceinline__ void stash(float (*lds)[LDS_LD], int tid) const {
    if (KMAJOR) {
#pragma unroll
      for (int i = 0; i < PASSES; ++i) {
        int k = (tid >> 5) + 8 * i;
        int d = (tid & 31) * 4;
        *reinterpret_cast<float4*>(&lds[k][d]) = r[i];
      }
    } else {
#pragma unroll
      for (int i = 0; i < PASSES; ++i) {
        int d = tid / TPR + RPP * i;
        int k = (tid % TPR) * 4;
        lds[k + 0][d] = r[i].x;
        lds[k + 1][d] = r[i].y;
        lds[k + 2][d] = r[i].z;
        lds[k + 3][d] = r[i].w;
      }
    }
  }
};

}  // namespace

namespace br {

// SPLIT = false: the contraction kernel of the optimizer step.  SPLIT = true: the variant used
// inside the QR factorisation, whose skinny products (32 or 128 output rows, K = thousands)
// would otherwise run on a handful of workgroups: blockIdx additionally selects one of
// `splitk` K ranges and the partial product goes to `partial`, summed in a fixed order by
// br_splitk_reduce (deterministic, no atomics).
// ADAM = true (step kernels with op(B) stored K x N only): the product is a rotated gradient G~ and the
// epilogue is Algorithm 1 from the second moment to the quotient: S~ <- b2 S~ + (1-b2) G~.G~ in place,
// M~ <- b1 M~ + (1-b1) G~ in place when adam.update_mrot, and X = M~ / sqrt(S~ + eps) stored to C; G~ itself
// never reaches memory.
template <bool TA, bool TB, bool VEC, bool SPLIT, bool ADAM>
__global__ __launch_bounds__(256, 4) void br_gemm_f32_mfma(GemmKernArgs g, BrGemmBatch batch) {
  __shared__ __attribute__((aligned(16))) float As[2][BK][LDS_LD];
  __shared__ __attribute__((aligned(16))) float Bs[2][BK][LDS_LD];

  // XCD-aware remap: hardware deals consecutive workgroup ids round-robin to the 8 XCDs;
  // give each XCD a contiguous run of logical tiles so neighbours share operands in its L2.
  int bid = blockIdx.x;
  const int nblk = gridDim.x;
  const int per = nblk / NUM_XCD;
  if (bid < per * NUM_XCD) bid = (bid % NUM_XCD) * per + bid / NUM_XCD;

  int mat, tm, tn, split = 0;
  {
    int per_mat = g.total_tiles;
    if (SPLIT) {
      split = bid % g.splitk;
      bid /= g.splitk;
    }
    mat = bid / per_mat;
    int t = bid - mat * per_mat;
    if (g.mirror) {
      // Tiles with tm >= tn, in bands of SYM_GROUP_M tile rows, column by column inside a band (as the unmirrored
      // order below: the tiles in flight on one XCD then share a band's few row panels instead of each row
      // bringing its own).  A band starts where the plain row-by-row count t = tm (tm + 1) / 2 + tn puts its
      // first row, so the row of t in that count names the band.
      int r = (int)((sqrtf(8.0f * (float)t + 1.0f) - 1.0f) * 0.5f);
      while ((r + 1) * (r + 2) / 2 <= t) ++r;
      while (r * (r + 1) / 2 > t) --r;
      const int first = r / SYM_GROUP_M * SYM_GROUP_M;
      const int gm = min(SYM_GROUP_M, g.tiles_m - first);
      int local = t - first * (first + 1) / 2;
      const int rect = first * gm;  // the band's full columns, left of its diagonal block
      if (local < rect) {
        tn = local / gm;
        tm = first + (local - tn * gm);
      } else {
        local -= rect;
        int j = 0;
        while (local >= gm - j) { local -= gm - j; ++j; }  // column first + j holds rows first + j .. first + gm - 1
        tn = first + j;
        tm = first + j + local;
      }
    } else {
      // Grouped order: GROUP_M tile rows at a time, column by column inside the group, so that the
      // ~128 tiles in flight on one XCD form an 8 x 16 patch (24 operand panels) instead of
      // two and a half tile rows (50+ panels): fewer distinct panels stream through its L2.
      const int group = GROUP_M * g.tiles_n;
      const int grp = t / group;
      const int first_m = grp * GROUP_M;
      const int gm = min(GROUP_M, g.tiles_m - first_m);
      const int r = t - grp * group;
      tn = r / gm;
      tm = first_m + (r - tn * gm);
    }
  }
  if (g.skip && g.skip[mat]) return;  // uniform over the workgroup, ahead of every barrier
  const float* __restrict__ A = batch.A[mat];
  const float* __restrict__ B = batch.B[mat];
  float* __restrict__ C = batch.C[mat];
  uint16_t* __restrict__ shadow = batch.shadow[mat];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = tm * BM, n0 = tn * BN;

  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  TileLoader<TA, VEC> la;    // op(A) = A^T  <=> A stored K x M  <=> k-major
  TileLoader<!TB, VEC> lb;   // op(B) = B    <=> B stored K x N  <=> k-major

  int kt0 = 0;
  int nkt = (g.K + BK - 1) / BK;
  if (SPLIT) {
    kt0 = split * g.kt_per_split;
    nkt = min(nkt, kt0 + g.kt_per_split);
  }
  const int lk = lane >> 5;  // which of the two k of an MFMA this lane feeds
  const int li = lane & 31;  // row of A / column of B inside the 32-wide MFMA tile
  auto mfma_tile = [&](int cur) {
#pragma unroll
    for (int kk = 0; kk < BK; kk += 2) {
      float a0 = As[cur][kk + lk][wm * 64 + li];
      float a1 = As[cur][kk + lk][wm * 64 + 32 + li];
      float b0 = Bs[cur][kk + lk][wn * 64 + li];
      float b1 = Bs[cur][kk + lk][wn * 64 + 32 + li];
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
    }
  };
  const bool interior = VEC && (m0 + BM <= g.M) && (n0 + BN <= g.N) && (g.K % BK == 0);
  if (interior) {
    la.init_fast(A, g.lda, m0, kt0 * BK, tid);
    lb.init_fast(B, g.ldb, n0, kt0 * BK, tid);
    la.fetch_fast();
    lb.fetch_fast();
    la.stash(As[0], tid);
    lb.stash(Bs[0], tid);
    __syncthreads();
    for (int kt = kt0; kt < nkt - 1; ++kt) {
      const int cur = (kt - kt0) & 1;
      la.fetch_fast();
      lb.fetch_fast();
      // keep the next tile's global loads HERE, a whole tile of matrix instructions ahead of the
      // stores into LDS that wait for them (the scheduler otherwise sinks them next to those stores)
      __builtin_amdgcn_sched_barrier(0);
      mfma_tile(cur);
      la.stash(As[cur ^ 1], tid);
      lb.stash(Bs[cur ^ 1], tid);
      __syncthreads();
    }
    if (nkt > kt0) mfma_tile((nkt - 1 - kt0) & 1);
  } else {
    la.fetch(A, g.lda, m0, kt0 * BK, g.M, g.K, tid);
    lb.fetch(B, g.ldb, n0, kt0 * BK, g.N, g.K, tid);
    la.stash(As[0], tid);
    lb.stash(Bs[0], tid);
    __syncthreads();
    for (int kt = kt0; kt < nkt; ++kt) {
      const int cur = (kt - kt0) & 1;
      if (kt + 1 < nkt) {
        la.fetch(A, g.lda, m0, (kt + 1) * BK, g.M, g.K, tid);
        lb.fetch(B, g.ldb, n0, (kt + 1) * BK, g.N, g.K, tid);
      }
      mfma_tile(cur);
      if (kt + 1 < nkt) {
        la.stash(As[cur ^ 1], tid);
        lb.stash(Bs[cur ^ 1], tid);
      }
      __syncthreads();
    }
  }

  if (SPLIT && g.splitk > 1) {
    float* __restrict__ P = g.partial + ((size_t)mat * g.splitk + split) * (size_t)g.M * g.N;
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
      for (int ni = 0; ni < 2; ++ni) {
        const int col = n0 + wn * 64 + ni * 32 + li;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = m0 + wm * 64 + mi * 32 + 8 * (v >> 2) + 4 * lk + (v & 3);
          if (row < g.M && col < g.N) P[(size_t)row * g.N + col] = g.alpha * acc[mi][ni][v];
        }
      }
    return;
  }
  if (ADAM) {
    float* __restrict__ S = batch.S[mat];
    float* __restrict__ Mr = batch.Mrot[mat];
    const BrAdamArgs ad = g.adam;
    const float w1 = 1.0f - ad.beta1, w2 = 1.0f - ad.beta2;
    if (m0 + BM <= g.M && n0 + BN <= g.N) {
      // Tile wholly inside the matrix: no bounds tests; one lane offset walks the lane's 32 rows in the order the
      // accumulators hold them (steps of one row and of five rows, the same for every lane; the two 32-wide column
      // blocks of a row are 128 bytes apart), the moments of eight rows are fetched before the first store to them.
      const size_t ld = (size_t)g.ldc;
      size_t o = (size_t)(m0 + wm * 64 + 4 * lk) * ld + (n0 + wn * 64 + li);
#pragma unroll
      for (int u = 0; u < 4; ++u) {  // units of eight rows
        const int mi = u >> 1, h = u & 1;
        float so[8][2], mo[8][2];
        size_t ol = o;
#pragma unroll
        for (int r = 0; r < 8; ++r) {
#pragma unroll
          for (int ni = 0; ni < 2; ++ni) {
            so[r][ni] = S[ol + ni * 32];
            mo[r][ni] = Mr[ol + ni * 32];
          }
          ol += ((r & 3) == 3) ? 5 * ld : ld;
          asm volatile("" : "+v"(ol));
        }
#pragma unroll
        for (int r = 0; r < 8; ++r) {
#pragma unroll
          for (int ni = 0; ni < 2; ++ni) {
            const float gt = g.alpha * acc[mi][ni][h * 8 + r];
            float mt = mo[r][ni];
            if (ad.update_mrot) {
              mt = ad.beta1 * mt + w1 * gt;
              Mr[o + ni * 32] = mt;
            }
            const float st = ad.beta2 * so[r][ni] + w2 * (gt * gt);
            S[o + ni * 32] = st;
            C[o + ni * 32] = adam_quotient(mt, st, ad);
          }
          o += ((r & 3) == 3) ? 5 * ld : ld;
          asm volatile("" : "+v"(o));
        }
      }
      return;
    }
#pragma unroll
    for (int mi = 0; mi < 2; ++mi) {
#pragma unroll
      for (int ni = 0; ni < 2; ++ni) {
        const int col = n0 + wn * 64 + ni * 32 + li;
        // both moments of this accumulator's sixteen entries are fetched before the first store
        float sold[16], mold[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = m0 + wm * 64 + mi * 32 + 8 * (v >> 2) + 4 * lk + (v & 3);
          const bool in = row < g.M && col < g.N;
          const size_t off = (size_t)row * (size_t)g.ldc + col;
          sold[v] = in ? S[off] : 0.f;
          mold[v] = in ? Mr[off] : 0.f;
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = m0 + wm * 64 + mi * 32 + 8 * (v >> 2) + 4 * lk + (v & 3);
          if (row < g.M && col < g.N) {
            const size_t off = (size_t)row * (size_t)g.ldc + col;
            const float gt = g.alpha * acc[mi][ni][v];
            float mt = mold[v];
            if (ad.update_mrot) {
              mt = ad.beta1 * mt + w1 * gt;
              Mr[off] = mt;
            }
            const float st = ad.beta2 * sold[v] + w2 * (gt * gt);
            S[off] = st;
            C[off] = adam_quotient(mt, st, ad);
          }
        }
      }
    }
    return;
  }
  const bool use_beta = (g.beta != 0.0f);
  const bool off_diag = g.mirror && (tm != tn);
  bool bad = false;
#pragma unroll
  for (int mi = 0; mi < 2; ++mi) {
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) {
      const int col = n0 + wn * 64 + ni * 32 + li;
      // The old values of this accumulator's sixteen outputs are fetched together, before any of
      // them is stored: a load issued after a store to the same matrix would wait for that store.
      float old[16];
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = m0 + wm * 64 + mi * 32 + 8 * (v >> 2) + 4 * lk + (v & 3);
        old[v] = (use_beta && row < g.M && col < g.N) ? C[(size_t)row * (size_t)g.ldc + col] : 0.f;
      }
#pragma unroll
      for (int vg = 0; vg < 4; ++vg) {
        const int row0 = m0 + wm * 64 + mi * 32 + 8 * vg + 4 * lk;
        float val[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int row = row0 + e;
          val[e] = g.alpha * acc[mi][ni][vg * 4 + e];
          if (use_beta) val[e] += g.beta * old[vg * 4 + e];
          if (row < g.M && col < g.N) {
            size_t off = (size_t)row * (size_t)g.ldc + col;
            C[off] = val[e];
            if (shadow) shadow[off] = f32_to_bf16_rne(val[e]);
            bad |= not_finite(val[e]);
          }
        }
        if (off_diag && col < g.N) {
          // transposed copy of a symmetric result: this lane's four rows are four consecutive columns there
          float* dst = C + (size_t)col * (size_t)g.ldc + row0;
          if (VEC && row0 + 3 < g.M && ((g.ldc & 3) == 0)) {
            *reinterpret_cast<float4*>(dst) = make_float4(val[0], val[1], val[2], val[3]);
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (row0 + e < g.M) dst[e] = val[e];
          }
        }
      }
    }
  }
  // one count per wave that stored something not finite (integer atomic: the results stay deterministic)
  if (g.health && __any(bad) && lane == 0) atomicAdd(g.health + BR_HEALTH_NONFINITE_WEIGHT, 1);
}

struct ReduceArgs {
  float* C[BR_MAXB];
};

// C_b = beta C_b + sum_s partial[b][s]   (fixed summation order)
__global__ __launch_bounds__(256) void br_splitk_reduce(ReduceArgs r, const float* __restrict__ partial, int M, int N,
                                                        int ldc, int splitk, float beta, const int* __restrict__ skip) {
  if (skip && skip[blockIdx.y]) return;
  float* __restrict__ C = r.C[blockIdx.y];
  const size_t mn = (size_t)M * N;
  const float* __restrict__ P = partial + (size_t)blockIdx.y * splitk * mn;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < mn; i += stride) {
    float s = 0.f;
    for (int k = 0; k < splitk; ++k) s += P[(size_t)k * mn + i];
    const size_t row = i / N, col = i - row * N;
    float* dst = C + row * (size_t)ldc + col;
    *dst = (beta != 0.0f) ? beta * *dst + s : s;
  }
}

}  // namespace br

namespace {

template <bool TA, bool TB, bool SPLIT, bool ADAM>
hipError_t launch_variant(hipStream_t s, const GemmKernArgs& k, const BrGemmBatch& b, int grid, bool vec) {
  if (vec)
    hipLaunchKernelGGL((br::br_gemm_f32_mfma<TA, TB, true, SPLIT, ADAM>), dim3(grid), dim3(256), 0, s, k, b);
  else
    hipLaunchKernelGGL((br::br_gemm_f32_mfma<TA, TB, false, SPLIT, ADAM>), dim3(grid), dim3(256), 0, s, k, b);
  return hipGetLastError();
}

template <bool SPLIT>
hipError_t launch_any(hipStream_t s, const BrGemmArgs& a, const GemmKernArgs& k, const BrGemmBatch& b, int grid, bool vec) {
  if (!a.transA && !a.transB) return launch_variant<false, false, SPLIT, false>(s, k, b, grid, vec);
  if (!a.transA && a.transB) return launch_variant<false, true, SPLIT, false>(s, k, b, grid, vec);
  if (a.transA && !a.transB) return launch_variant<true, false, SPLIT, false>(s, k, b, grid, vec);
  return launch_variant<true, true, SPLIT, false>(s, k, b, grid, vec);
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

hipError_t br_launch_gemm(hipStream_t s, const BrGemmArgs& a, const BrGemmBatch& b, const char** kernel_name) {
  static const char* names[8] = {"br_gemm_f32_mfma<nn>", "br_gemm_f32_mfma<nt>", "br_gemm_f32_mfma<tn>",
                                 "br_gemm_f32_mfma<tt>", "br_gemm_f32_mfma<nn,split>", "br_gemm_f32_mfma<nt,split>",
                                 "br_gemm_f32_mfma<tn,split>", "br_gemm_f32_mfma<tt,split>"};
  if (kernel_name) {
    *kernel_name = names[(a.qr_role ? 4 : 0) + (a.transA ? 2 : 0) + (a.transB ? 1 : 0)];
    if (a.adam_epilogue) *kernel_name = a.transA ? "br_gemm_f32_mfma<tn,adam>" : "br_gemm_f32_mfma<nn,adam>";
    // symmetric products (the statistics) run the same kernels on the lower triangle of tiles, each stored twice
    if (a.mirror && !a.qr_role) *kernel_name = a.transA ? "br_gemm_f32_mfma<tn,sym>" : "br_gemm_f32_mfma<nt,sym>";
  }
  if (a.batch <= 0 || a.M <= 0 || a.N <= 0) return hipSuccess;
  if (a.batch > BR_MAXB || a.K < 0) return hipErrorInvalidValue;
  if (a.mirror && (a.M != a.N)) return hipErrorInvalidValue;
  if (a.adam_epilogue && (a.transB || a.mirror || a.qr_role)) return hipErrorInvalidValue;
  if (a.adam_epilogue)
    for (int i = 0; i < a.batch; ++i)
      if (!b.S[i] || !b.Mrot[i]) return hipErrorInvalidValue;
  GemmKernArgs k;
  k.M = a.M; k.N = a.N; k.K = a.K;
  k.lda = a.lda; k.ldb = a.ldb; k.ldc = a.ldc;
  k.alpha = a.alpha; k.beta = a.beta;
  k.tiles_m = (a.M + BM - 1) / BM;
  k.tiles_n = (a.N + BN - 1) / BN;
  k.mirror = a.mirror ? 1 : 0;
  k.total_tiles = k.mirror ? k.tiles_m * (k.tiles_m + 1) / 2 : k.tiles_m * k.tiles_n;
  k.splitk = 1;
  k.kt_per_split = (a.K + BK - 1) / BK;
  k.partial = nullptr;
  k.skip = a.skip;
  k.health = a.health;
  k.adam = a.adam;
  long long grid = (long long)k.total_tiles * a.batch;
  if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
  bool vec = (a.lda % 4 == 0) && (a.ldb % 4 == 0);
  for (int i = 0; i < a.batch && vec; ++i) vec = aligned16(b.A[i]) && aligned16(b.B[i]) && (!a.mirror || aligned16(b.C[i]));
  if (a.adam_epilogue)
    return a.transA ? launch_variant<true, false, false, true>(s, k, b, (int)grid, vec)
                    : launch_variant<false, false, false, true>(s, k, b, (int)grid, vec);
  if (!a.qr_role) return launch_any<false>(s, a, k, b, (int)grid, vec);
  // Split K when the launch would leave most of the 256 compute units idle.  (Splitting launches
  // of a few tiles per compute unit as well, to shorten their tails, was measured and gained nothing.)
  const int nkt = (a.K + BK - 1) / BK;
  if (a.partial && !a.mirror && grid < 384 && nkt >= 32) {
    long long want = (768 + grid - 1) / grid;
    long long by_k = nkt / 8;  // at least 8 K tiles (128 columns of K) per range
    long long by_mem = (long long)(a.partial_floats / ((size_t)a.M * a.N * a.batch));
    long long sk = std::min(std::min(want, by_k), std::min<long long>(by_mem, 64));
    if (sk > 1) {
      k.kt_per_split = (int)((nkt + sk - 1) / sk);
      k.splitk = (nkt + k.kt_per_split - 1) / k.kt_per_split;
      k.partial = a.partial;
    }
  }
  hipError_t e = launch_any<true>(s, a, k, b, (int)(grid * k.splitk), vec);
  if (e != hipSuccess || k.splitk == 1) return e;
  br::ReduceArgs r;
  for (int i = 0; i < BR_MAXB; ++i) r.C[i] = (i < a.batch) ? b.C[i] : nullptr;
  long long blocks = ((long long)a.M * a.N + 255) / 256;
  if (blocks > 64) blocks = 64;
  hipLaunchKernelGGL(br::br_splitk_reduce, dim3((int)blocks, a.batch), dim3(256), 0, s, r, k.partial, a.M, a.N, a.ldc,
                     k.splitk, a.beta, a.skip);
  return hipGetLastError();
}
