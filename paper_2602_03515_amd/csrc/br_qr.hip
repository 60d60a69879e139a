// Householder QR building blocks for the basis refresh (Section 3.2: one power-iteration
// product, then a QR factorisation; the Power calls of Algorithm 2).
//
// The factorisation is blocked recursively (panels of BR_QR_NB = 32 columns, middle blocks of
// BR_QR_NBM = 128 merged in LDS, then merged pairwise up to top blocks of 256 or BR_QR_NBT = 512) in
// compact-WY form:
//   H_1 H_2 ... H_nb = I - V T V^T,  V unit lower trapezoidal, T upper triangular.
// This file holds the panel kernel; the trailing-matrix and Q-forming updates are GEMMs issued
// by the host logic.  A panel is held ENTIRELY IN REGISTERS from its first load to its final
// store: a 1024-thread workgroup keeps up to 1536 rows, and a taller panel is shared by a cluster
// of workgroups (gridDim.y, one slab of rows each) that combine their partial dot products
// through global memory once per column.
//
// Panel kernel (br_qr_panel), one pass per column.  A panel row is 32 floats = one 128-byte line; it
// is owned by 8 adjacent lanes (4 columns each), so every wave64 access touches 8 whole
// lines.  Pass j applies reflector H_j to the rest of the panel and, in the same sweep
// over the rows, accumulates (a) the dot products of the NEXT column with all later
// columns (its norm and the w-vector of H_{j+1}) and (b) V[:, 0:j]^T v_j for column j of
// T.  Each pass therefore reads and writes the active part of the panel exactly once.
#include "br_internal.h"

#include <algorithm>

namespace br {

constexpr int QR_THREADS = 1024;
constexpr int QR_ROWS_PER_SWEEP = QR_THREADS / 8;  // 128
constexpr int QR_WAVES = QR_THREADS / 64;          // 16
constexpr int QR_RESIDENT_SWEEPS = 12;             // a workgroup keeps up to 12 x 128 = 1536 rows in registers
constexpr int QR_MAX_SLAB = QR_RESIDENT_SWEEPS * QR_ROWS_PER_SWEEP;
constexpr int QR_XCH_SLOTS = 64;                   // per (step, workgroup): 32 partial sums + the next pivot row

// One lane's four columns of a panel row travel as a float4 VALUE (never through a pointer), so
// that groups of rows stay in registers.
__device__ __forceinline__ float4 panel_load(const float* __restrict__ row, int c0, int nb, bool vec) {
  float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
  if (vec && c0 + 3 < nb) {
    t = *reinterpret_cast<const float4*>(row + c0);
  } else {
    if (c0 < nb) t.x = row[c0];
    if (c0 + 1 < nb) t.y = row[c0 + 1];
    if (c0 + 2 < nb) t.z = row[c0 + 2];
    if (c0 + 3 < nb) t.w = row[c0 + 3];
  }
  return t;
}

__device__ __forceinline__ void panel_store(float* __restrict__ row, int c0, int nb, bool vec, float4 a) {
  if (vec && c0 + 3 < nb) {
    *reinterpret_cast<float4*>(row + c0) = a;
  } else {
    if (c0 < nb) row[c0] = a.x;
    if (c0 + 1 < nb) row[c0 + 1] = a.y;
    if (c0 + 2 < nb) row[c0 + 2] = a.z;
    if (c0 + 3 < nb) row[c0 + 3] = a.w;
  }
}

__device__ __forceinline__ float pick4(float4 a, int q) {
  float r = a.x;
  r = (q == 1) ? a.y : r;
  r = (q == 2) ? a.z : r;
  r = (q == 3) ? a.w : r;
  return r;
}

// Sum of v over the eight row groups of a wave (the lanes that own the same columns).
__device__ __forceinline__ float group_sum(float v) {
  v += __shfl_xor(v, 8, 64);
  v += __shfl_xor(v, 16, 64);
  v += __shfl_xor(v, 32, 64);
  return v;
}

// Sum of acc over all threads of the workgroup that own the same columns; the sum for column tid
// is returned to threads tid < 32 (other threads get zero).  One barrier.
__device__ __forceinline__ float panel_reduce(float4 acc, float (*red)[32], int tid) {
  const int lane = tid & 63, wave = tid >> 6, sub = tid & 7;
  acc.x = group_sum(acc.x);
  acc.y = group_sum(acc.y);
  acc.z = group_sum(acc.z);
  acc.w = group_sum(acc.w);
  if (lane < 8) {
    red[wave][sub * 4 + 0] = acc.x;
    red[wave][sub * 4 + 1] = acc.y;
    red[wave][sub * 4 + 2] = acc.z;
    red[wave][sub * 4 + 3] = acc.w;
  }
  __syncthreads();
  float s = 0.f;
  if (tid < 32) {
#pragma unroll
    for (int w = 0; w < QR_WAVES; ++w) s += red[w][tid];
  }
  return s;
}

// Cluster part of the reduction (gridDim.y > 1): every workgroup publishes its 32 partial sums
// (workgroup 0 also the pivot row of the next pass) and reads the others'.  A published value is
// one 8-byte word, the float and a tag that names the panel and the step, written and read with
// single 8-byte atomic accesses: a reader polls the word itself until the tag is the one it
// waits for, so the exchange is one store and one load deep, without a separate arrival counter.
// The buffer is zeroed before a factorisation and tags are unique within it (never zero).
// Each workgroup sums the partials in workgroup order, so that all of them hold bit-identical
// values.  The wait is bounded (the workgroups of a launch must all be resident; a launch that
// shares the GPU with other work could starve one): a workgroup whose wait runs out sets its
// matrix's `failed` flag, bumps the context's health word and carries on with a NaN, so that every
// kernel still ends.  The host logic leaves the previous basis of a flagged matrix in place.
struct Cluster {
  unsigned long long* xch;  // [step][workgroup][QR_XCH_SLOTS] of this matrix
  int* failed;              // this matrix's flag
  int* health;              // the context's health words (may be null)
  unsigned tag0;            // this panel's tags are tag0 + step + 1
  unsigned spin_limit;
  int w, nw;
};

__device__ __forceinline__ unsigned long long xch_pack(float v, unsigned tag) {
  return ((unsigned long long)tag << 32) | (unsigned long long)__float_as_uint(v);
}

__device__ __forceinline__ float xch_wait(const unsigned long long* slot, unsigned tag, unsigned limit, bool& gave_up) {
  for (unsigned spins = 0; spins < limit; ++spins) {
    const unsigned long long v = __hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if ((unsigned)(v >> 32) == tag) return __uint_as_float((unsigned)v);
    __builtin_amdgcn_s_sleep(1);
  }
  gave_up = true;
  return __builtin_nanf("");
}

// Threads 0..31 pass their column's partial sum and get the cluster's sum back.  The partners' words are
// polled side by side, not one after the other: group g of 32 threads (g = tid / 32) waits for workgroup g's
// 32 sums and parks them in LDS, so the exchange stays one store and one load deep whatever the size of the
// cluster, and threads 0..31 then add the partials in workgroup order.  The last group of 32 threads carries
// the next pivot row (read from pivnext in workgroup 0, written to it in the others).  One barrier inside.
// Clusters of more workgroups than there are groups to spare fall back to polling in turn.
constexpr int QR_POLL_GROUPS = QR_THREADS / 32 - 1;  // groups of 32 threads besides the one for the pivot row
constexpr int QR_WIDE_CLUSTER = 8;                   // widest cluster chosen for speed alone (taller panels take what their rows need)
__device__ __forceinline__ float cluster_combine(const Cluster& cl, int step, float part, float* pivnext, float (*xs)[32], int tid) {
  const unsigned tag = cl.tag0 + (unsigned)step + 1u;
  unsigned long long* base = cl.xch + (size_t)step * cl.nw * QR_XCH_SLOTS;
  float s = 0.f;
  bool gave_up = false;
  const int grp = tid >> 5, col = tid & 31;
  if (tid < 32)
    __hip_atomic_store(base + (size_t)cl.w * QR_XCH_SLOTS + tid, xch_pack(part, tag), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (grp == QR_POLL_GROUPS) {  // another wave than the first sums': the waits overlap
    if (cl.w == 0)
      __hip_atomic_store(base + 32 + col, xch_pack(pivnext[col], tag), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else
      pivnext[col] = xch_wait(base + 32 + col, tag, cl.spin_limit, gave_up);
  }
  if (cl.nw <= QR_POLL_GROUPS) {
    if (grp < cl.nw && grp != cl.w) xs[grp][col] = xch_wait(base + (size_t)grp * QR_XCH_SLOTS + col, tag, cl.spin_limit, gave_up);
    __syncthreads();
    if (tid < 32)
      for (int ww = 0; ww < cl.nw; ++ww) s += (ww == cl.w) ? part : xs[ww][tid];
  } else if (tid < 32) {
    for (int ww = 0; ww < cl.nw; ++ww)
      s += (ww == cl.w) ? part : xch_wait(base + (size_t)ww * QR_XCH_SLOTS + tid, tag, cl.spin_limit, gave_up);
  }
  if (gave_up) {  // rare: flag the matrix (plain store; every writer stores the same 1) and count it
    *cl.failed = 1;
    if (cl.health) atomicAdd(cl.health + BR_HEALTH_QR_GAVE_UP, 1);
  }
  return s;
}

// State shared by all rows during pass j.
struct PassParams {
  int j, jn;          // current column, owner column of the next one
  float scale, beta;  // v = x * scale below the diagonal; R_jj
  float4 w;           // tau * (v^T A[:, c]) for this lane's four columns (0 for c <= j)
  float wn;           // the same for column j + 1 (0 when there is none)
};

__device__ __forceinline__ float4 fma4(float s, float4 a, float4 acc) {
  return make_float4(acc.x + s * a.x, acc.y + s * a.y, acc.z + s * a.z, acc.w + s * a.w);
}

// Apply reflector j to one row (columns c0..c0+3 of row r, in `a`) and accumulate this row's
// contribution to the dot products needed by pass j + 1 and by column j of V^T V.
// Written for instruction count (the kernel is bound by vector-ALU issue): the update is one FMA per
// entry because w is zero for the columns up to j; column j itself is patched by one select on a
// per-lane mask that is fixed for the whole pass; both kinds of sums (entries times v for the columns
// before j, entries times the new column j + 1 for those after) are accumulated for every column and
// told apart once per pass, not per row.  Columns j and j + 1 are read BEFORE the update, so that the
// two cross-lane reads do not depend on it: the updated entry of column j + 1 is a_old - v * w_next.
struct PassMasks {
  bool eq[4];  // this lane's entry k is column j
};

template <bool FIRST_SWEEP>
__device__ __forceinline__ void pass_row(float4& a, int r, bool active, const PassParams& pp, const PassMasks& pm,
                                         int c0, int group_base, float4& accv, float4& accx, float* pivnext) {
  const int j = pp.j;
  const float aj = __shfl(pick4(a, j & 3), group_base | (j >> 2), 64);
  const float an_old = __shfl(pick4(a, pp.jn & 3), group_base | (pp.jn >> 2), 64);
  const bool piv = (r == j);
  const float v = piv ? 1.0f : aj * pp.scale;
  const float own = piv ? pp.beta : v;  // what column j keeps: R_jj in the pivot row, the reflector below it
  a.x = pm.eq[0] ? own : fmaf(-v, pp.w.x, a.x);
  a.y = pm.eq[1] ? own : fmaf(-v, pp.w.y, a.y);
  a.z = pm.eq[2] ? own : fmaf(-v, pp.w.z, a.z);
  a.w = pm.eq[3] ? own : fmaf(-v, pp.w.w, a.w);
  const float xn = fmaf(-v, pp.wn, an_old);
  const float va = active ? v : 0.f;
  const float xa = (active && r > j) ? xn : 0.f;
  accv = fma4(va, a, accv);
  accx = fma4(xa, a, accx);
  // the next pivot row (panel row j + 1 <= 32) can only sit in the first sweep: the others stay free of branches
  if (FIRST_SWEEP && r == j + 1) *reinterpret_cast<float4*>(pivnext + c0) = a;
}

__device__ __forceinline__ float4 clean_v(float4 a, int c0, int r, int nb) {
  float4 o;
  o.x = (c0 + 0 >= nb || c0 + 0 > r) ? 0.f : ((c0 + 0 == r) ? 1.0f : a.x);
  o.y = (c0 + 1 >= nb || c0 + 1 > r) ? 0.f : ((c0 + 1 == r) ? 1.0f : a.y);
  o.z = (c0 + 2 >= nb || c0 + 2 > r) ? 0.f : ((c0 + 2 == r) ? 1.0f : a.z);
  o.w = (c0 + 3 >= nb || c0 + 3 > r) ? 0.f : ((c0 + 3 == r) ? 1.0f : a.w);
  return o;
}

// U sweeps of 128 rows per workgroup (U * 128 >= slab), all in registers; the passes touch no
// memory at all.
// Workgroup (x, y) holds rows [y * slab, min(rows, (y + 1) * slab)) of panel x.
template <int U>
__global__ __launch_bounds__(QR_THREADS) void br_qr_panel(BrQrPanelBatch p, int rows, int nb, int lda, int vec_ok,
                                                          int ldv, int pre_rows, int slab, BrQrClusterBatch cb) {
  __shared__ float red[QR_WAVES][32];
  __shared__ __attribute__((aligned(16))) float dvec[32];
  __shared__ __attribute__((aligned(16))) float pivrow[2][32];
  __shared__ float Sl[32][33];  // Sl[l][j] = v_l^T v_j for l < j: the strict upper triangle of V^T V
  __shared__ float Xl[32][33];  // columns of T while they are being solved for
  __shared__ float taus[32];
  __shared__ float xs[QR_POLL_GROUPS][32];  // the partner workgroups' partial sums of one exchange

  float* __restrict__ A = p.A[blockIdx.x];
  float* __restrict__ Vc = p.Vc[blockIdx.x];
  float* __restrict__ Tg = p.T[blockIdx.x];
  float* __restrict__ diag = p.diag[blockIdx.x];
  const bool vec = vec_ok != 0;
  Cluster cl;
  cl.xch = cb.xch[blockIdx.x];
  cl.failed = cb.failed[blockIdx.x];
  cl.health = cb.health;
  cl.spin_limit = cb.spin_limit;
  cl.tag0 = cb.tag0;
  cl.w = blockIdx.y;
  cl.nw = gridDim.y;
  const bool first = (cl.w == 0);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int sub = tid & 7;
  const int c0 = sub * 4;
  const int group_base = lane & ~7;
  const int row0 = cl.w * slab;                  // first row of this workgroup's slab
  const int rend = min(rows, row0 + slab);       // one past its last row
  const int rg = row0 + (tid >> 3);              // this thread's row in sweep 0

  for (int i = tid; i < 32 * 33; i += QR_THREADS) {
    (&Sl[0][0])[i] = 0.f;
    (&Xl[0][0])[i] = 0.f;
  }
  if (tid < 32) {
    taus[tid] = 0.f;
    pivrow[0][tid] = 0.f;
    pivrow[1][tid] = 0.f;
  }
  __syncthreads();

  float4 ra[U];
  const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int r = rg + QR_ROWS_PER_SWEEP * u;
    ra[u] = zero4;
    if (r < rend) ra[u] = panel_load(A + (size_t)r * lda, c0, nb, vec);
  }

  // Pre-pass: dot products of column 0 with every column; stash row 0.
  float4 acc = zero4;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int r = rg + QR_ROWS_PER_SWEEP * u;
    const float x0 = __shfl(ra[u].x, group_base, 64);
    if (r < rend) {
      acc = fma4(x0, ra[u], acc);
      if (r == 0) *reinterpret_cast<float4*>(&pivrow[0][c0]) = ra[u];
    }
  }
  {
    float sum = panel_reduce(acc, red, tid);
    if (cl.nw > 1) sum = cluster_combine(cl, 0, sum, pivrow[0], xs, tid);
    if (tid < 32) dvec[tid] = sum;
    __syncthreads();
  }

  for (int j = 0; j < nb; ++j) {
    const int cur = j & 1;
    const float alpha = pivrow[cur][j];
    const float normsq = dvec[j];
    float tau = 0.f;
    PassParams pp;
    pp.j = j;
    pp.jn = (j + 1 < 32) ? j + 1 : 31;  // unused when j + 1 == nb
    pp.beta = 0.f;
    pp.scale = 0.f;
    if (normsq > 0.f) {
      const float nrm = sqrtf(normsq);
      pp.beta = (alpha >= 0.f) ? -nrm : nrm;
      tau = (pp.beta - alpha) / pp.beta;
      pp.scale = 1.0f / (alpha - pp.beta);
    }
    {
      const float4 pr = *reinterpret_cast<const float4*>(&pivrow[cur][c0]);
      const float4 dv = *reinterpret_cast<const float4*>(&dvec[c0]);
      pp.w.x = (c0 + 0 > j && c0 + 0 < nb) ? tau * (pr.x + pp.scale * (dv.x - alpha * pr.x)) : 0.f;
      pp.w.y = (c0 + 1 > j && c0 + 1 < nb) ? tau * (pr.y + pp.scale * (dv.y - alpha * pr.y)) : 0.f;
      pp.w.z = (c0 + 2 > j && c0 + 2 < nb) ? tau * (pr.z + pp.scale * (dv.z - alpha * pr.z)) : 0.f;
      pp.w.w = (c0 + 3 > j && c0 + 3 < nb) ? tau * (pr.w + pp.scale * (dv.w - alpha * pr.w)) : 0.f;
    }
    {
      const int jn = pp.jn;
      const float prn = pivrow[cur][jn], dvn = dvec[jn];
      pp.wn = (j + 1 < nb) ? tau * (prn + pp.scale * (dvn - alpha * prn)) : 0.f;
    }
    PassMasks pm;
#pragma unroll
    for (int e = 0; e < 4; ++e) pm.eq[e] = (c0 + e == j);
    // Every sweep, unconditionally: the loop body is free of branches, so the cross-lane reads of
    // different sweeps overlap.  Rows past the slab hold zeros and stay zero; rows above row j are
    // finished and whatever the pass does to them is masked out of the sums and of the reflectors.
    float4 accv = zero4, accx = zero4;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int r = rg + QR_ROWS_PER_SWEEP * u;
      if (u == 0) pass_row<true>(ra[u], r, (r >= j) && (r < rend), pp, pm, c0, group_base, accv, accx, pivrow[cur ^ 1]);
      else pass_row<false>(ra[u], r, (r >= j) && (r < rend), pp, pm, c0, group_base, accv, accx, pivrow[cur ^ 1]);
      if (u % 6 == 5) __builtin_amdgcn_sched_barrier(0);  // at most six sweeps' cross-lane values in registers at once
    }
    acc.x = (c0 + 0 < j) ? accv.x : ((c0 + 0 > j) ? accx.x : 0.f);
    acc.y = (c0 + 1 < j) ? accv.y : ((c0 + 1 > j) ? accx.y : 0.f);
    acc.z = (c0 + 2 < j) ? accv.z : ((c0 + 2 > j) ? accx.z : 0.f);
    acc.w = (c0 + 3 < j) ? accv.w : ((c0 + 3 > j) ? accx.w : 0.f);
    {
      // Column sums of this pass: for c > j the dot products of the next pass, for c < j the entries
      // v_c^T v_j of the Gram matrix of the reflectors.
      float sum = panel_reduce(acc, red, tid);
      if (cl.nw > 1) sum = cluster_combine(cl, j + 1, sum, pivrow[cur ^ 1], xs, tid);
      if (tid < 32) {
        if (tid > j) dvec[tid] = sum;
        else if (tid < j) Sl[tid][j] = sum;
        else {
          taus[j] = tau;
          if (first) diag[j] = pp.beta;
        }
      }
      __syncthreads();
    }
  }

  // Block-reflector factor.  H_1 ... H_nb = I - V T V^T with T^-1 = diag(1 / tau) + strict upper
  // triangle of V^T V: thread t solves for column t of T by back substitution.  A reflector with
  // tau = 0 is the identity; its row and column of T are zero.
  if (first && tid < 32) {
    const int t = tid;
    const float tt = (t < nb) ? taus[t] : 0.f;
    Xl[t][t] = tt;
    for (int r = t - 1; r >= 0; --r) {
      float sacc = 0.f;
      for (int l = r + 1; l <= t; ++l) sacc += Sl[r][l] * Xl[l][t];
      Xl[r][t] = (tt != 0.f) ? -taus[r] * sacc : 0.f;
    }
  }
  __syncthreads();

  if (first) {
    // Block-reflector factor, zero padded to BR_QR_NB x BR_QR_NB.
    for (int i = tid; i < BR_QR_NB * BR_QR_NB; i += QR_THREADS) {
      const int r = i / BR_QR_NB, c = i - r * BR_QR_NB;
      Tg[i] = (r < nb && c < nb && r <= c) ? Xl[r][c] : 0.f;
    }
    // The clean copy of the reflectors (below) is a 32-column slice of a wider reflector block
    // (row stride ldv); the pre_rows rows of that block above this panel's first row are zero
    // in these columns.
    for (int i = tid; i < pre_rows * BR_QR_NB; i += QR_THREADS) {
      const int r = i / BR_QR_NB, c = i - r * BR_QR_NB;
      Vc[-(ptrdiff_t)(r + 1) * ldv + c] = 0.f;
    }
  }
  // Factorised panel back to the matrix, and the clean copy: unit diagonal, zeros above it and
  // right of column nb.
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int r = rg + QR_ROWS_PER_SWEEP * u;
    if (r < rend) {
      panel_store(A + (size_t)r * lda, c0, nb, vec, ra[u]);
      *reinterpret_cast<float4*>(Vc + (size_t)r * ldv + c0) = clean_v(ra[u], c0, r, nb);
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

// Merge the 32-wide block-reflector factors of one middle block into its BR_QR_NBM-wide factor:
//   T = [ T_a  -T_a (V_a^T V_b) T_b ]
//       [ 0     T_b             ]      applied panel by panel,
// with the cross products V_a^T V_b read from the Gram matrix G = V^T V of the middle block.
// One 1024-thread workgroup per matrix; T, the panel's slice of G and the intermediate product
// live in LDS.
struct BuildTArgs {
  const float* G[BR_MAXB];   // BR_QR_NBM x BR_QR_NBM
  const float* Tp[BR_MAXB];  // npanels consecutive BR_QR_NB x BR_QR_NB factors
  float* T[BR_MAXB];         // BR_QR_NBM x BR_QR_NBM output
};

constexpr int BUILD_T_THREADS = 1024;

__global__ __launch_bounds__(BUILD_T_THREADS) void br_qr_build_t(BuildTArgs a, int npanels) {
  __shared__ float T[BR_QR_NBM][BR_QR_NBM + 1];
  __shared__ float Z[BR_QR_NBM][BR_QR_NB + 1];
  __shared__ float Gs[BR_QR_NBM][BR_QR_NB + 1];
  const float* __restrict__ G = a.G[blockIdx.x];
  const float* __restrict__ Tp = a.Tp[blockIdx.x];
  float* __restrict__ Tout = a.T[blockIdx.x];
  const int tid = threadIdx.x;
  for (int i = tid; i < BR_QR_NBM * BR_QR_NBM; i += BUILD_T_THREADS) T[i / BR_QR_NBM][i % BR_QR_NBM] = 0.f;
  __syncthreads();
  for (int pnl = 0; pnl < npanels; ++pnl) {
    const int o = pnl * BR_QR_NB;
    for (int i = tid; i < BR_QR_NB * BR_QR_NB; i += BUILD_T_THREADS)
      T[o + i / BR_QR_NB][o + i % BR_QR_NB] = Tp[(size_t)pnl * BR_QR_NB * BR_QR_NB + i];
    for (int i = tid; i < o * BR_QR_NB; i += BUILD_T_THREADS) {
      const int r = i / BR_QR_NB, c = i - r * BR_QR_NB;
      Gs[r][c] = G[(size_t)r * BR_QR_NBM + o + c];
    }
    __syncthreads();
    if (pnl == 0) continue;
    // Z = T[0:o, 0:o] * G[0:o, o:o+32]
    for (int i = tid; i < o * BR_QR_NB; i += BUILD_T_THREADS) {
      const int r = i / BR_QR_NB, c = i - r * BR_QR_NB;
      float s = 0.f;
      for (int l = r; l < o; ++l) s += T[r][l] * Gs[l][c];
      Z[r][c] = s;
    }
    __syncthreads();
    // T[0:o, o:o+32] = -Z * T_b
    for (int i = tid; i < o * BR_QR_NB; i += BUILD_T_THREADS) {
      const int r = i / BR_QR_NB, c = i - r * BR_QR_NB;
      float s = 0.f;
      for (int l = 0; l <= c; ++l) s += Z[r][l] * T[o + l][o + c];
      T[r][o + c] = -s;
    }
    __syncthreads();
  }
  for (int i = tid; i < BR_QR_NBM * BR_QR_NBM; i += BUILD_T_THREADS) Tout[i] = T[i / BR_QR_NBM][i % BR_QR_NBM];
}

// Merged factor T (2w x 2w) of two child blocks of width w: the children's factors are copied onto
// the diagonal here, the rest is zeroed; the coupling block -T_0 (V_0^T V_1) T_1 is then written
// over the upper right corner by small contractions.
struct AssembleTArgs {
  const float* Tc[BR_MAXB];  // nchild consecutive w x w factors
  float* T[BR_MAXB];         // 2w x 2w output
};

__global__ __launch_bounds__(256) void br_qr_assemble_t(AssembleTArgs a, int nchild, int w) {
  const float* __restrict__ Tc = a.Tc[blockIdx.y];
  float* __restrict__ T = a.T[blockIdx.y];
  const int w2 = 2 * w;
  for (int i = blockIdx.x * 256 + threadIdx.x; i < w2 * w2; i += gridDim.x * 256) {
    const int r = i / w2, c = i - r * w2;
    const int cb = r / w;
    float v = 0.f;
    if (c / w == cb && cb < nchild) v = Tc[(size_t)cb * w * w + (size_t)(r - cb * w) * w + (c - cb * w)];
    T[i] = v;
  }
}

struct ZeroArgs {
  int* ptr[BR_MAXB];
};

__global__ __launch_bounds__(256) void br_zero_ints(ZeroArgs a, int n) {
  int* __restrict__ p = a.ptr[blockIdx.y];
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) p[i] = 0;
}

struct SignArgs {
  float* Q[BR_MAXB];
  const float* diag[BR_MAXB];
};

// Q <- diag(sign(d)): the matrix the reflectors are applied to when the orthogonal factor is
// formed.  (H_1 ... H_k) diag(s) equals (H_1 ... H_k I) with its columns' signs flipped, entry by
// entry and bit for bit, so starting from the signed identity makes diag(R) >= 0 without a pass
// over Q afterwards.
__global__ __launch_bounds__(256) void br_qr_signed_identity(SignArgs a, int n, const int* __restrict__ skip) {
  if (skip && skip[blockIdx.y]) return;  // this matrix's factorisation was abandoned: its previous basis stays
  float* __restrict__ Q = a.Q[blockIdx.y];
  const float* __restrict__ d = a.diag[blockIdx.y];
  const int64_t total = (int64_t)n * n;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
    const int r = (int)(i / n), c = (int)(i - (int64_t)r * n);
    Q[i] = (r == c) ? ((d[c] < 0.f) ? -1.0f : 1.0f) : 0.0f;
  }
}


// ---- a panel's block reflector applied to the rest of its middle block -------------------
// C <- (I - V T^T V^T) C for the rows x ncols block C right of a factorised panel (ncols <= 96,
// V: rows x 32 clean reflectors, T: 32 x 32).  As three general contractions this is all latency
// (M = 32, N <= 96, K = thousands: a split-K launch, its reduction, two more launches); here it is
// two launches of small workgroups:
//   br_qr_panel_vtc    partial[slab] = V_slab^T C_slab   (32 x ncols per PA_VSLAB rows; FP32 MFMA, a wave
//                      per quarter of the rows and 32 columns, the quarters summed in LDS in a fixed order)
//   br_qr_panel_apply  W = sum of the partials in slab order (deterministic), X = T^T W in LDS,
//                      C_slab <- C_slab - V_slab X   (PA_SLAB rows per workgroup).
typedef float qr_floatx16 __attribute__((ext_vector_type(16)));
constexpr int PA_SLAB = 256;    // rows per workgroup of br_qr_panel_apply
constexpr int PA_VSLAB = 1024;  // rows per workgroup of br_qr_panel_vtc (four quarters of 256, one wave each per 32 columns)
constexpr int PA_MAXC = 96;

struct PanelApplyArgs {
  const float* V[BR_MAXB];
  const float* T[BR_MAXB];
  float* C[BR_MAXB];
};

__global__ __launch_bounds__(768) void br_qr_panel_vtc(PanelApplyArgs a, int rows, int ncols, int ldv, int ldc,
                                                       float* __restrict__ partial) {
  __shared__ float red[4][32][PA_MAXC + 1];
  const int mat = blockIdx.y, slab = blockIdx.x, nslab = gridDim.x;
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63, lk = lane >> 5, li = lane & 31;
  const int cb = wave % 3, rq = wave / 3;  // 32-column block of C, quarter of the slab's rows
  const float* __restrict__ V = a.V[mat];
  const float* __restrict__ C = a.C[mat];
  const int col = cb * 32 + li;
  const bool col_ok = col < ncols;
  if (cb * 32 < ncols) {  // wave-uniform
    const int r_begin = slab * PA_VSLAB + rq * (PA_VSLAB / 4);
    const int r_end = min(rows, r_begin + PA_VSLAB / 4);
    qr_floatx16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    // W[j][c] += V[r][j] C[r][c]: the matrix instruction takes A[i = j][k = r] and B[k = r][j = c], two rows per issue
    for (int r = r_begin; r < r_end; r += 16) {
      float av[8], bv[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int rr = r + 2 * u + lk;
        const bool ok = rr < r_end;
        av[u] = ok ? V[(size_t)rr * ldv + li] : 0.f;
        bv[u] = (ok && col_ok) ? C[(size_t)rr * ldc + col] : 0.f;
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av[u], bv[u], acc, 0, 0, 0);
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) red[rq][8 * (v >> 2) + 4 * lk + (v & 3)][col] = acc[v];
  }
  __syncthreads();
  float* __restrict__ P = partial + ((size_t)mat * nslab + slab) * (32 * PA_MAXC);
  for (int e = tid; e < 32 * PA_MAXC; e += 768) {
    const int j = e / PA_MAXC, c = e - j * PA_MAXC;
    if (c < ncols) P[e] = ((red[0][j][c] + red[1][j][c]) + red[2][j][c]) + red[3][j][c];  // fixed order
  }
}

__global__ __launch_bounds__(512) void br_qr_panel_apply(PanelApplyArgs a, int rows, int ncols, int ldv, int ldc,
                                                         const float* __restrict__ partial, int nvslab) {
  __shared__ float Wl[32][PA_MAXC + 1];
  __shared__ float Xl[32][PA_MAXC + 1];
  __shared__ float Tl[32][33];
  const int mat = blockIdx.y, slab = blockIdx.x;
  const int tid = threadIdx.x;
  const float* __restrict__ V = a.V[mat];
  const float* __restrict__ T = a.T[mat];
  float* __restrict__ C = a.C[mat];
  for (int i = tid; i < 32 * 32; i += 512) Tl[i >> 5][i & 31] = T[i];
  const float* __restrict__ P = partial + (size_t)mat * nvslab * (32 * PA_MAXC);
  {
    float sum[6];  // 32 * 96 / 512 entries per thread, summed over the partials in slab order (deterministic)
#pragma unroll
    for (int q = 0; q < 6; ++q) sum[q] = 0.f;
    for (int sl = 0; sl < nvslab; ++sl) {
#pragma unroll
      for (int q = 0; q < 6; ++q) {
        const int e = tid + 512 * q;
        const int c = e % PA_MAXC;
        if (c < ncols) sum[q] += P[(size_t)sl * (32 * PA_MAXC) + e];
      }
    }
#pragma unroll
    for (int q = 0; q < 6; ++q) {
      const int e = tid + 512 * q;
      Wl[e / PA_MAXC][e % PA_MAXC] = sum[q];
    }
  }
  __syncthreads();
  for (int e = tid; e < 32 * PA_MAXC; e += 512) {  // X = T^T W, T upper triangular
    const int j = e / PA_MAXC, c = e - j * PA_MAXC;
    float s = 0.f;
    for (int l = 0; l <= j; ++l) s += Tl[l][j] * Wl[l][c];
    Xl[j][c] = s;
  }
  __syncthreads();
  const int wave = tid >> 6, lane = tid & 63, lk = lane >> 5, li = lane & 31;
  const int nblk = (ncols + 31) / 32;
  const int r0 = slab * PA_SLAB + wave * 32;  // eight waves, 32 rows each
  if (r0 >= rows) return;
  // C[r][c] -= sum_k V[r][k] X[k][c]: A[i = row][k] = V, B[k][j = c] = X
  float av[16];
  {
    const int rr = r0 + li;
    const float* vrow = V + (size_t)rr * ldv + lk;
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) av[kk] = (rr < rows) ? vrow[2 * kk] : 0.f;
  }
  for (int cb = 0; cb < nblk; ++cb) {
    qr_floatx16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
    for (int kk = 0; kk < 16; ++kk)
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av[kk], Xl[2 * kk + lk][cb * 32 + li], acc, 0, 0, 0);
    const int col = cb * 32 + li;
    float old[16];  // all loads before the first store (a load behind a store to the same matrix waits for it)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int rr = r0 + 8 * (v >> 2) + 4 * lk + (v & 3);
      old[v] = (rr < rows && col < ncols) ? C[(size_t)rr * ldc + col] : 0.f;
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int rr = r0 + 8 * (v >> 2) + 4 * lk + (v & 3);
      if (rr < rows && col < ncols) C[(size_t)rr * ldc + col] = old[v] - acc[v];
    }
  }
}

}  // namespace br

int br_qr_panel_cluster(int rows) { return (rows + br::QR_MAX_SLAB - 1) / br::QR_MAX_SLAB; }

// Room for the widest cluster a launch may choose: the workgroups the rows need, or QR_WIDE_CLUSTER
// when a small batch leaves compute units free.
size_t br_qr_panel_xch_floats(int rows) {
  const int nw = std::max(br_qr_panel_cluster(rows), br::QR_WIDE_CLUSTER);
  return (size_t)(BR_QR_NB + 1) * nw * br::QR_XCH_SLOTS * 2;  // 8-byte slots
}

hipError_t br_launch_qr_panel(hipStream_t s, const BrQrPanelBatch& p, const BrQrClusterBatch& cb, int batch, int rows, int nb,
                              int lda, int ldv, int pre_rows) {
  if (batch <= 0) return hipSuccess;
  if (batch > BR_MAXB || rows < nb || nb < 1 || nb > BR_QR_NB || lda < nb || ldv < BR_QR_NB || (ldv & 3) || pre_rows < 0)
    return hipErrorInvalidValue;
  int vec = (lda % 4 == 0);
  for (int i = 0; i < batch && vec; ++i) vec = ((reinterpret_cast<uintptr_t>(p.A[i]) & 15u) == 0);
  // A cluster waits for all of its workgroups: every workgroup of a launch must be resident at
  // the same time (one 1024-thread workgroup per compute unit), so large batches go in pieces.
  // How many fit is asked of the device once (three quarters of its compute units, at most
  // BR_QR_MAX_RESIDENT): on a partition with fewer units the pieces shrink, and a panel whose
  // cluster alone does not fit is refused instead of being left to its bounded wait.
  static int cap_of_device[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  if (cap_of_device[dev] == 0) {
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return hipErrorInvalidDevice;
    const int cap = cus * 3 / 4;
    cap_of_device[dev] = cap < 1 ? 1 : (cap > BR_QR_MAX_RESIDENT ? BR_QR_MAX_RESIDENT : cap);
  }
  const int resident_cap = cap_of_device[dev];
  // Workgroups per panel: what the rows need at least; more (up to QR_WIDE_CLUSTER) when the whole batch then
  // still fits in one launch.  A panel costs about 40 us + 10 us per sweep of 128 rows in a workgroup of its own
  // and 25 to 40 us more in a cluster (an exchange per column, nearly the same for two workgroups as for eight,
  // the partners' words being polled side by side): shorter slabs on more compute units pay for tall panels of
  // a small batch (measured on the 3B-class stage: 50.4 -> 44.0 ms of panel time per refresh; no further gain
  // beyond eight).  At least four sweeps of rows per workgroup: panels of up to 1023 rows stay in one workgroup,
  // where an exchange would cost what the shorter sweeps save.
  int nw = br_qr_panel_cluster(rows);
  {
    const int fits = resident_cap / batch;
    const int by_rows = rows / (4 * br::QR_ROWS_PER_SWEEP);
    const int wide = std::min(std::min(fits, br::QR_WIDE_CLUSTER), std::min(by_rows, br::QR_POLL_GROUPS));
    if (wide > nw) nw = wide;
  }
  // balanced slabs, whole sweeps, no workgroup without rows
  int slab = (rows + nw - 1) / nw;
  slab = (slab + br::QR_ROWS_PER_SWEEP - 1) / br::QR_ROWS_PER_SWEEP * br::QR_ROWS_PER_SWEEP;
  nw = (rows + slab - 1) / slab;
  if (nw > 1)
    for (int i = 0; i < batch; ++i)
      if (!cb.xch[i] || !cb.failed[i]) return hipErrorInvalidValue;
  const int per_launch = resident_cap / nw;
  if (per_launch < 1) return hipErrorInvalidValue;
  for (int off = 0; off < batch; off += per_launch) {
    const int b = (batch - off < per_launch) ? batch - off : per_launch;
    BrQrPanelBatch pp;
    BrQrClusterBatch cc;
    cc.tag0 = cb.tag0;
    cc.spin_limit = cb.spin_limit;
    cc.health = cb.health;
    for (int i = 0; i < BR_MAXB; ++i) {
      const bool live = i < b;
      cc.failed[i] = live ? cb.failed[off + i] : nullptr;
      pp.A[i] = live ? p.A[off + i] : nullptr;
      pp.Vc[i] = live ? p.Vc[off + i] : nullptr;
      pp.T[i] = live ? p.T[off + i] : nullptr;
      pp.diag[i] = live ? p.diag[off + i] : nullptr;
      cc.xch[i] = live ? cb.xch[off + i] : nullptr;
    }
    const int sweeps = slab / br::QR_ROWS_PER_SWEEP;
    if (sweeps <= 3)
      hipLaunchKernelGGL((br::br_qr_panel<3>), dim3(b, nw), dim3(br::QR_THREADS), 0, s, pp, rows, nb, lda, vec, ldv, pre_rows,
                         slab, cc);
    else if (sweeps <= 5)
      hipLaunchKernelGGL((br::br_qr_panel<5>), dim3(b, nw), dim3(br::QR_THREADS), 0, s, pp, rows, nb, lda, vec, ldv, pre_rows,
                         slab, cc);
    else if (sweeps <= 7)
      hipLaunchKernelGGL((br::br_qr_panel<7>), dim3(b, nw), dim3(br::QR_THREADS), 0, s, pp, rows, nb, lda, vec, ldv, pre_rows,
                         slab, cc);
    else if (sweeps <= 10)
      hipLaunchKernelGGL((br::br_qr_panel<10>), dim3(b, nw), dim3(br::QR_THREADS), 0, s, pp, rows, nb, lda, vec, ldv, pre_rows,
                         slab, cc);
    else
      hipLaunchKernelGGL((br::br_qr_panel<br::QR_RESIDENT_SWEEPS>), dim3(b, nw), dim3(br::QR_THREADS), 0, s, pp, rows, nb, lda,
                         vec, ldv, pre_rows, slab, cc);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

size_t br_qr_panel_apply_floats(int batch, int rows) {
  return (size_t)batch * ((rows + br::PA_VSLAB - 1) / br::PA_VSLAB) * 32 * br::PA_MAXC;
}

hipError_t br_launch_qr_panel_apply(hipStream_t s, const float* const* V, const float* const* T, float* const* C, int batch,
                                    int rows, int ncols, int ldv, int ldc, float* partial, size_t partial_floats) {
  if (batch <= 0 || ncols <= 0) return hipSuccess;
  if (batch > BR_MAXB || rows < 1 || ncols > br::PA_MAXC || ldv < BR_QR_NB || ldc < ncols || !partial ||
      partial_floats < br_qr_panel_apply_floats(batch, rows))
    return hipErrorInvalidValue;
  br::PanelApplyArgs a;
  for (int i = 0; i < BR_MAXB; ++i) {
    a.V[i] = (i < batch) ? V[i] : nullptr;
    a.T[i] = (i < batch) ? T[i] : nullptr;
    a.C[i] = (i < batch) ? C[i] : nullptr;
  }
  const int nvslab = (rows + br::PA_VSLAB - 1) / br::PA_VSLAB;
  const int nslab = (rows + br::PA_SLAB - 1) / br::PA_SLAB;
  hipLaunchKernelGGL(br::br_qr_panel_vtc, dim3(nvslab, batch), dim3(768), 0, s, a, rows, ncols, ldv, ldc, partial);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(br::br_qr_panel_apply, dim3(nslab, batch), dim3(512), 0, s, a, rows, ncols, ldv, ldc, partial, nvslab);
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
  if (batch > BR_MAXB || npanels < 1 || npanels * BR_QR_NB > BR_QR_NBM) return hipErrorInvalidValue;
  br::BuildTArgs a;
  for (int i = 0; i < BR_MAXB; ++i) {
    a.G[i] = (i < batch) ? G[i] : nullptr;
    a.Tp[i] = (i < batch) ? Tp[i] : nullptr;
    a.T[i] = (i < batch) ? T[i] : nullptr;
  }
  hipLaunchKernelGGL(br::br_qr_build_t, dim3(batch), dim3(br::BUILD_T_THREADS), 0, s, a, npanels);
  return hipGetLastError();
}

hipError_t br_launch_qr_assemble_t(hipStream_t s, const float* const* Tc, float* const* T, int batch, int nchild, int w) {
  if (batch <= 0) return hipSuccess;
  if (batch > BR_MAXB || nchild < 1 || nchild > 2 || w < BR_QR_NB || 2 * w > BR_QR_NBT) return hipErrorInvalidValue;
  br::AssembleTArgs a;
  for (int i = 0; i < BR_MAXB; ++i) {
    a.Tc[i] = (i < batch) ? Tc[i] : nullptr;
    a.T[i] = (i < batch) ? T[i] : nullptr;
  }
  hipLaunchKernelGGL(br::br_qr_assemble_t, dim3(32, batch), dim3(256), 0, s, a, nchild, w);
  return hipGetLastError();
}

hipError_t br_launch_zero_ints(hipStream_t s, int* const* ptrs, int batch, int n) {
  if (batch <= 0 || n <= 0) return hipSuccess;
  if (batch > BR_MAXB) return hipErrorInvalidValue;
  br::ZeroArgs a;
  for (int i = 0; i < BR_MAXB; ++i) a.ptr[i] = (i < batch) ? ptrs[i] : nullptr;
  hipLaunchKernelGGL(br::br_zero_ints, dim3((n + 255) / 256, batch), dim3(256), 0, s, a, n);
  return hipGetLastError();
}

hipError_t br_launch_qr_signed_identity(hipStream_t s, float* const* Q, const float* const* diag, int batch, int n,
                                        const int* skip) {
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
  hipLaunchKernelGGL(br::br_qr_signed_identity, dim3((int)blocks, batch), dim3(256), 0, s, a, n, skip);
  return hipGetLastError();
}
