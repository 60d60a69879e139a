// Householder QR building blocks for the basis refresh (Section 3.2: "power iteration
// followed by QR decomposition"; Algorithm 2 lines 3 and 6).
//
// The factorisation is blocked (panel width BR_QR_NB = 32) in compact-WY form:
//   H_1 H_2 ... H_nb = I - V T V^T,  V unit lower trapezoidal, T upper triangular.
// This file holds the panel kernel (one 1024-thread workgroup per matrix of the batch);
// the trailing-matrix and Q-forming updates are GEMMs issued by the host logic.
//
// Panel kernel, one pass per column.  A panel row is 32 floats = one 128-byte line; it
// is owned by 8 adjacent lanes (4 columns each), so every wave64 access touches 8 whole
// lines.  Pass j applies reflector H_j to the rest of the panel and, in the same sweep
// over the rows, accumulates (a) the dot products of the NEXT column with all later
// columns (its norm and the w-vector of H_{j+1}) and (b) V[:, 0:j]^T v_j for column j of
// T.  Each pass therefore reads and writes the active part of the panel exactly once.
#include "br_internal.h"

namespace br {

constexpr int QR_THREADS = 1024;
constexpr int QR_ROWS_PER_SWEEP = QR_THREADS / 8;  // 128
constexpr int QR_WAVES = QR_THREADS / 64;          // 16

__device__ __forceinline__ void panel_load(const float* __restrict__ row, int c0, int nb, bool vec, float a[4]) {
  if (vec && c0 + 3 < nb) {
    float4 t = *reinterpret_cast<const float4*>(row + c0);
    a[0] = t.x; a[1] = t.y; a[2] = t.z; a[3] = t.w;
  } else {
#pragma unroll
    for (int q = 0; q < 4; ++q) a[q] = (c0 + q < nb) ? row[c0 + q] : 0.f;
  }
}

__device__ __forceinline__ void panel_store(float* __restrict__ row, int c0, int nb, bool vec, const float a[4]) {
  if (vec && c0 + 3 < nb) {
    *reinterpret_cast<float4*>(row + c0) = make_float4(a[0], a[1], a[2], a[3]);
  } else {
#pragma unroll
    for (int q = 0; q < 4; ++q)
      if (c0 + q < nb) row[c0 + q] = a[q];
  }
}

__device__ __forceinline__ float pick4(const float a[4], int q) {
  float r = a[0];
  r = (q == 1) ? a[1] : r;
  r = (q == 2) ? a[2] : r;
  r = (q == 3) ? a[3] : r;
  return r;
}

// Sum acc[] over all threads that own the same columns; result for column c in comb[c].
__device__ __forceinline__ void panel_reduce(float acc[4], float (*red)[32], float* comb, int tid) {
  const int lane = tid & 63, wave = tid >> 6, sub = tid & 7;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    float v = acc[q];
    v += __shfl_xor(v, 8, 64);
    v += __shfl_xor(v, 16, 64);
    v += __shfl_xor(v, 32, 64);
    acc[q] = v;
  }
  if (lane < 8) {
#pragma unroll
    for (int q = 0; q < 4; ++q) red[wave][sub * 4 + q] = acc[q];
  }
  __syncthreads();
  if (tid < 32) {
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < QR_WAVES; ++w) s += red[w][tid];
    comb[tid] = s;
  }
  __syncthreads();
}

__global__ __launch_bounds__(QR_THREADS) void br_qr_panel(BrQrPanelBatch p, int rows, int nb, int lda, int vec_ok,
                                                          int ldv, int pre_rows) {
  __shared__ float red[QR_WAVES][32];
  __shared__ float comb[32];
  __shared__ float dvec[32];
  __shared__ float zl[32];
  __shared__ float pivrow[2][32];
  __shared__ float Tl[32][33];

  float* __restrict__ A = p.A[blockIdx.x];
  float* __restrict__ Vc = p.Vc[blockIdx.x];
  float* __restrict__ Tg = p.T[blockIdx.x];
  float* __restrict__ diag = p.diag[blockIdx.x];
  const bool vec = vec_ok != 0;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int sub = tid & 7;
  const int rg = tid >> 3;
  const int c0 = sub * 4;
  const int group_base = lane & ~7;
  const int nsweeps = (rows + QR_ROWS_PER_SWEEP - 1) / QR_ROWS_PER_SWEEP;

  for (int i = tid; i < 32 * 33; i += QR_THREADS) (&Tl[0][0])[i] = 0.f;
  if (tid < 32) {
    pivrow[0][tid] = 0.f;
    pivrow[1][tid] = 0.f;
  }
  __syncthreads();

  float acc[4];
  // Pre-pass: dot products of column 0 with every column; stash row 0.
  acc[0] = acc[1] = acc[2] = acc[3] = 0.f;
  for (int it = 0; it < nsweeps; ++it) {
    const int r = rg + QR_ROWS_PER_SWEEP * it;
    const bool active = r < rows;
    float a[4] = {0.f, 0.f, 0.f, 0.f};
    if (active) panel_load(A + (size_t)r * lda, c0, nb, vec, a);
    const float x0 = __shfl(a[0], group_base, 64);
    if (active) {
#pragma unroll
      for (int q = 0; q < 4; ++q) acc[q] += x0 * a[q];
      if (r == 0) {
#pragma unroll
        for (int q = 0; q < 4; ++q) pivrow[0][c0 + q] = a[q];
      }
    }
  }
  panel_reduce(acc, red, comb, tid);
  if (tid < 32) dvec[tid] = comb[tid];
  __syncthreads();

  for (int j = 0; j < nb; ++j) {
    const int cur = j & 1;
    const float alpha = pivrow[cur][j];
    const float normsq = dvec[j];
    float beta = 0.f, tau = 0.f, scale = 0.f;
    if (normsq > 0.f) {
      const float nrm = sqrtf(normsq);
      beta = (alpha >= 0.f) ? -nrm : nrm;
      tau = (beta - alpha) / beta;
      scale = 1.0f / (alpha - beta);
    }
    float w[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int c = c0 + q;
      const float pr = pivrow[cur][c];
      w[q] = (c > j && c < nb) ? tau * (pr + scale * (dvec[c] - alpha * pr)) : 0.f;
    }
    const int jn = (j + 1 < 32) ? j + 1 : 31;  // owner of the next column (unused when j + 1 == nb)
    acc[0] = acc[1] = acc[2] = acc[3] = 0.f;
    for (int it = j / QR_ROWS_PER_SWEEP; it < nsweeps; ++it) {
      const int r = rg + QR_ROWS_PER_SWEEP * it;
      const bool active = (r >= j) && (r < rows);
      float a[4] = {0.f, 0.f, 0.f, 0.f};
      float* rowp = A + (size_t)r * lda;
      if (active) panel_load(rowp, c0, nb, vec, a);
      const float aj = __shfl(pick4(a, j & 3), group_base | (j >> 2), 64);
      const float v = (r == j) ? 1.0f : aj * scale;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int c = c0 + q;
        if (c > j) a[q] -= v * w[q];
        else if (c == j) a[q] = (r == j) ? beta : v;
      }
      const float xn = __shfl(pick4(a, jn & 3), group_base | (jn >> 2), 64);
      if (active) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int c = c0 + q;
          if (c < j) acc[q] += a[q] * v;
          else if (c > j && r > j) acc[q] += xn * a[q];
        }
        panel_store(rowp, c0, nb, vec, a);
        if (r == j + 1) {
#pragma unroll
          for (int q = 0; q < 4; ++q) pivrow[cur ^ 1][c0 + q] = a[q];
        }
      }
    }
    panel_reduce(acc, red, comb, tid);
    if (tid < 32) {
      if (tid > j) dvec[tid] = comb[tid];
      else if (tid < j) zl[tid] = comb[tid];
    }
    __syncthreads();
    if (tid < j) {
      float s = 0.f;
      for (int l = tid; l < j; ++l) s += Tl[tid][l] * zl[l];
      Tl[tid][j] = -tau * s;
    } else if (tid == j) {
      Tl[j][j] = tau;
      diag[j] = beta;
    }
    __syncthreads();
  }

  // Block-reflector factor, zero padded to BR_QR_NB x BR_QR_NB.
  for (int i = tid; i < BR_QR_NB * BR_QR_NB; i += QR_THREADS) {
    const int r = i / BR_QR_NB, c = i - r * BR_QR_NB;
    Tg[i] = (r < nb && c < nb) ? Tl[r][c] : 0.f;
  }
  // Clean copy of the reflectors: unit diagonal, zeros above it and right of column nb.  The
  // copy is a 32-column slice of a wider reflector block (row stride ldv); the pre_rows rows of
  // that block above this panel's first row are zero in these columns.
  for (int i = tid; i < pre_rows * BR_QR_NB; i += QR_THREADS) {
    const int r = i / BR_QR_NB, c = i - r * BR_QR_NB;
    Vc[-(ptrdiff_t)(r + 1) * ldv + c] = 0.f;
  }
  for (int it = 0; it < nsweeps; ++it) {
    const int r = rg + QR_ROWS_PER_SWEEP * it;
    if (r < rows) {
      float a[4];
      panel_load(A + (size_t)r * lda, c0, nb, vec, a);
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int c = c0 + q;
        a[q] = (c >= nb || c > r) ? 0.f : ((c == r) ? 1.0f : a[q]);
      }
      *reinterpret_cast<float4*>(Vc + (size_t)r * ldv + c0) = make_float4(a[0], a[1], a[2], a[3]);
    }
  }
}

// Vc (rows x width, row stride width) <- reflectors stored below the diagonal of an already
// factorised block of nb <= width columns: unit diagonal, zeros above, zero padding right of nb.
__global__ __launch_bounds__(256) void br_qr_extract_v(BrQrPanelBatch p, int rows, int nb, int lda, int width) {
  const float* __restrict__ A = p.A[blockIdx.y];
  float* __restrict__ Vc = p.Vc[blockIdx.y];
  const int64_t total = (int64_t)rows * width;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
    const int r = (int)(i / width), c = (int)(i - (int64_t)r * width);
    float v = 0.f;
    if (c < nb) v = (c > r) ? 0.f : ((c == r) ? 1.0f : A[(size_t)r * lda + c]);
    Vc[i] = v;
  }
}

// Merge the 32-wide block-reflector factors of one outer block into its BR_QR_NBO-wide factor:
//   T = [ T_a  -T_a (V_a^T V_b) T_b ]
//       [ 0     T_b             ]      applied panel by panel,
// with the cross products V_a^T V_b read from the Gram matrix G = V^T V of the outer block.
// One 256-thread workgroup per matrix; everything lives in LDS.
struct BuildTArgs {
  const float* G[BR_MAXB];   // BR_QR_NBO x BR_QR_NBO
  const float* Tp[BR_MAXB];  // npanels consecutive BR_QR_NB x BR_QR_NB factors
  float* T[BR_MAXB];         // BR_QR_NBO x BR_QR_NBO output
};

__global__ __launch_bounds__(256) void br_qr_build_t(BuildTArgs a, int npanels) {
  __shared__ float T[BR_QR_NBO][BR_QR_NBO + 1];
  __shared__ float Z[BR_QR_NBO][BR_QR_NB + 1];
  const float* __restrict__ G = a.G[blockIdx.x];
  const float* __restrict__ Tp = a.Tp[blockIdx.x];
  float* __restrict__ Tout = a.T[blockIdx.x];
  const int tid = threadIdx.x;
  for (int i = tid; i < BR_QR_NBO * BR_QR_NBO; i += 256) T[i / BR_QR_NBO][i % BR_QR_NBO] = 0.f;
  __syncthreads();
  for (int pnl = 0; pnl < npanels; ++pnl) {
    const int o = pnl * BR_QR_NB;
    for (int i = tid; i < BR_QR_NB * BR_QR_NB; i += 256)
      T[o + i / BR_QR_NB][o + i % BR_QR_NB] = Tp[(size_t)pnl * BR_QR_NB * BR_QR_NB + i];
    __syncthreads();
    if (pnl == 0) continue;
    // Z = T[0:o, 0:o] * G[0:o, o:o+32]
    for (int i = tid; i < o * BR_QR_NB; i += 256) {
      const int r = i / BR_QR_NB, c = i - r * BR_QR_NB;
      float s = 0.f;
      for (int l = r; l < o; ++l) s += T[r][l] * G[(size_t)l * BR_QR_NBO + o + c];
      Z[r][c] = s;
    }
    __syncthreads();
    // T[0:o, o:o+32] = -Z * T_b
    for (int i = tid; i < o * BR_QR_NB; i += 256) {
      const int r = i / BR_QR_NB, c = i - r * BR_QR_NB;
      float s = 0.f;
      for (int l = 0; l <= c; ++l) s += Z[r][l] * T[o + l][o + c];
      T[r][o + c] = -s;
    }
    __syncthreads();
  }
  for (int i = tid; i < BR_QR_NBO * BR_QR_NBO; i += 256) Tout[i] = T[i / BR_QR_NBO][i % BR_QR_NBO];
}

struct SignArgs {
  float* Q[BR_MAXB];
  const float* diag[BR_MAXB];
};

__global__ __launch_bounds__(256) void br_qr_fix_signs(SignArgs a, int n) {
  float* __restrict__ Q = a.Q[blockIdx.y];
  const float* __restrict__ d = a.diag[blockIdx.y];
  const int64_t total = (int64_t)n * n;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
    const int c = (int)(i % n);
    if (d[c] < 0.f) Q[i] = -Q[i];
  }
}

}  // namespace br

hipError_t br_launch_qr_panel(hipStream_t s, const BrQrPanelBatch& p, int batch, int rows, int nb, int lda, int ldv,
                              int pre_rows) {
  if (batch <= 0) return hipSuccess;
  if (batch > BR_MAXB || rows < nb || nb < 1 || nb > BR_QR_NB || lda < nb || ldv < BR_QR_NB || (ldv & 3) || pre_rows < 0)
    return hipErrorInvalidValue;
  int vec = (lda % 4 == 0);
  for (int i = 0; i < batch && vec; ++i) vec = ((reinterpret_cast<uintptr_t>(p.A[i]) & 15u) == 0);
  hipLaunchKernelGGL(br::br_qr_panel, dim3(batch), dim3(br::QR_THREADS), 0, s, p, rows, nb, lda, vec, ldv, pre_rows);
  return hipGetLastError();
}

hipError_t br_launch_qr_extract_v(hipStream_t s, const BrQrPanelBatch& p, int batch, int rows, int nb, int lda,
                                  int width) {
  if (batch <= 0) return hipSuccess;
  if (batch > BR_MAXB || rows < nb || nb < 1 || nb > width) return hipErrorInvalidValue;
  int64_t blocks = ((int64_t)rows * width + 255) / 256;
  int64_t cap = (4096 + batch - 1) / batch;
  if (blocks > cap) blocks = cap;
  hipLaunchKernelGGL(br::br_qr_extract_v, dim3((int)blocks, batch), dim3(256), 0, s, p, rows, nb, lda, width);
  return hipGetLastError();
}

hipError_t br_launch_qr_build_t(hipStream_t s, const float* const* G, const float* const* Tp, float* const* T, int batch,
                                int npanels) {
  if (batch <= 0) return hipSuccess;
  if (batch > BR_MAXB || npanels < 1 || npanels * BR_QR_NB > BR_QR_NBO) return hipErrorInvalidValue;
  br::BuildTArgs a;
  for (int i = 0; i < BR_MAXB; ++i) {
    a.G[i] = (i < batch) ? G[i] : nullptr;
    a.Tp[i] = (i < batch) ? Tp[i] : nullptr;
    a.T[i] = (i < batch) ? T[i] : nullptr;
  }
  hipLaunchKernelGGL(br::br_qr_build_t, dim3(batch), dim3(256), 0, s, a, npanels);
  return hipGetLastError();
}

hipError_t br_launch_qr_fix_signs(hipStream_t s, float* const* Q, const float* const* diag, int batch, int n) {
  if (batch <= 0) return hipSuccess;
  if (batch > BR_MAXB) return hipErrorInvalidValue;
  br::SignArgs a;
  for (int i = 0; i < BR_MAXB; ++i) {
    a.Q[i] = (i < batch) ? Q[i] : nullptr;
    a.diag[i] = (i < batch) ? diag[i] : nullptr;
  }
  int64_t blocks = ((int64_t)n * n + 255) / 256;
  int64_t cap = (2048 + batch - 1) / batch;
  if (blocks > cap) blocks = cap;
  hipLaunchKernelGGL(br::br_qr_fix_signs, dim3((int)blocks, batch), dim3(256), 0, s, a, n);
  return hipGetLastError();
}
