// BF16 matrix-core contractions for the optimizer step (math modes BR_MATH_BF16 and
// BR_MATH_BF16X3): the statistics G G^T, G^T G (Algorithm 2, the updates of L and R), the rotations
// Q_L^T G Q_R (Algorithm 1, the rotation step) and the rotate-back Q_L X Q_R^T (its parameter update).
//
// Operands are first rewritten as BF16 "planes" by br_split_planes:
//     hi = bf16(x),  lo = bf16(x - hi)            (round to nearest even)
// optionally transposed, so that EVERY contraction has the form C[i][j] = sum_k A[i][k] B[j][k]
// with k contiguous for both operands.  A plane is stored as the IMAGE OF THE LDS TILES the
// contraction kernel works on (BrPlaneLayout in br_internal.h): rows padded to a multiple of
// 256, k padded to a multiple of 64 (zeros), k-blocked by 16, and the two 16-byte halves of each
// 32-byte (row, k-block) run swapped on every other group of 8 rows.  The 256 rows x 16 k that
// one workgroup needs from one operand per k-block are therefore one contiguous 8 KB run of
// memory whose byte order is exactly the order wanted in LDS: the kernel moves it with
// global_load_lds_dwordx4 (memory -> LDS without passing through registers, each wave 1 KB per
// instruction), and the matrix-core operand of a lane (8 consecutive k of one row) is a single
// conflict-free ds_read_b128.
//   NPROD = 1: C = A_hi B_hi^T                                  (plain BF16 inputs)
//   NPROD = 3: C = A_hi B_hi^T + A_hi B_lo^T + A_lo B_hi^T      (16-bit mantissa inputs, FP32
//              accumulation: a product term is off by about 2^-16, the dropped lo*lo term)
//   NPROD = 4: adds A_lo B_lo^T (in a mirrored product: on the diagonal tiles only).  Used for the statistics G G^T, G^T G, whose diagonal would
//              otherwise carry the systematic bias sum_k lo_k^2, and whose error the refresh
//              amplifies by the condition number of the statistics.
//
// Kernel: one 512-thread workgroup (eight wave64s, 2 x 4, each 128 x 64 = eight
// v_mfma_f32_32x32x16_bf16 accumulators) per compute unit and 256 x 256 output tile.  Operands
// stream through a ring of five 32 KB LDS stages (all 160 KB): a stage is 32 k of A and B
// (NPROD = 1) or 16 k of A_hi, A_lo, B_hi, B_lo (NPROD >= 3).  Four stages are always in flight
// from memory.  The grid is one workgroup per compute unit; each walks its share of the tiles and
// requests the first stages of its next tile before the epilogue of the current one.
// There is ONE workgroup barrier per stage and it sits between two groups of the stage's matrix
// instructions: operands are fetched from LDS one group ahead of their use, so the matrix pipe
// keeps running across the barrier.
// What bounds it (NPROD = 1, measured with the pieces of the loop switched off one at a time): per
// stage the matrix pipes need about 0.49 us, the LDS reads alone (96 KB at a little over 100 bytes
// per clock) 0.42 us, the memory -> LDS loads alone 0.29 us when every line hits L2 and 0.5 to
// 0.6 us with the real tile mix, and the three do not overlap freely: with all of them running
// the clock falls from 2.2 to 1.8 GHz (power), and a stage takes 0.85 to 0.95 us.  The tile is as
// large as the register file allows (128 flop per operand byte for NPROD = 1, three and four
// times that for the split products).  A 4-wave variant with 128 x 128 wave tiles (a third less
// LDS traffic, accumulators in AGPRs) was measured slower: one wave per SIMD leaves the matrix
// pipe idle across each stage's barrier (1470 against 1860 TFLOP/s with nothing but matrix
// instructions in the loop).
#include "br_internal.h"

namespace {

constexpr int TILE = BR_PLANE_ROW_PAD;  // 256 x 256 output tile; planes pad their rows to it
constexpr int NUM_XCD = 8;
constexpr int GROUP_M = 8;
constexpr int SUB_U4 = TILE * 2;        // uint4 per sub-tile: 256 rows x 16 k of one plane (8 KB)
constexpr int STAGE_U4 = 4 * SUB_U4;    // four sub-tiles per stage (32 KB)
constexpr int STAGES = 5;
constexpr int LOADS = 4;                // 1 KB loads per wave and stage (one per sub-tile)
constexpr int FM = 4, FN = 2;           // 32 x 32 accumulators per wave (wave tile 128 x 64)

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

struct LowpKernArgs {
  int M, N;              // logical output extent
  int Mp, Np, Kp;        // padded operand extents (rows to 256, k to 64)
  int ldc;
  size_t a_plane, b_plane;  // distance from the hi plane to the lo plane, in elements
  float alpha, beta;
  int tiles_m, tiles_n, total_tiles, mirror;
  int all_tiles;         // total_tiles x matrices of the launch: the length of the tile sequence the grid walks
  // plane-emitting epilogues: the result's transpose as operand planes (rows = N index, k = M index)
  int out_kp;            // padded k extent of the emitted planes (M to a multiple of 64)
  size_t out_plane;      // elements from their hi plane to their lo plane
  int out_lo;            // also emit the lo plane
  BrAdamArgs adam;       // EPI_ADAM
  int adam_t;            // EPI_ADAM: the tile is G~^T (row = column of G~): the moments are indexed [col][row]
  int b_stride;          // padded row count that addresses the B planes (Np, or a larger set's when B is a view into it)
  int out_stride;        // the same for the emitted planes
  int emit_t;            // EPI_F32: the transpose of the stored result also leaves as planes (pointer in the batch's S slot)
  float out_scale;       // emitted planes hold out_scale times the value (FP16 planes: a power of two that centres the range)
  const int* skip;       // EPI_F32, optional: one int per matrix, non-zero = nothing is stored for that matrix
  int* health;           // EPI_F32, optional: a stored value that is not finite bumps BR_HEALTH_NONFINITE_WEIGHT
};

__device__ __forceinline__ bool not_finite(float v) { return (__float_as_uint(v) & 0x7f800000u) == 0x7f800000u; }

enum { EPI_F32 = 0, EPI_PLANES = 1, EPI_ADAM = 2 };

// Round to nearest even; NaN stays NaN (quiet).  Both results are computed and one is selected: a branch here
// would be taken apart per lane, a hundred times over in the plane-emitting epilogues.
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  const uint32_t u = __float_as_uint(f);
  const uint32_t rounded = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
  const uint32_t quiet = (u >> 16) | 0x0040u;
  return (uint16_t)(((u & 0x7fffffffu) > 0x7f800000u) ? quiet : rounded);
}

__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

// FP16 planes (the refresh's split products): hi = fp16(x), lo = fp16(x - hi), both round to nearest even, subnormal
// results kept (the f16 matrix instruction honours them): 22 mantissa bits for |x| >= 2^-3, an absolute 2^-25 below.
// Values beyond the FP16 range are clamped to it (the callers' scales keep operands far inside).
__device__ __forceinline__ uint16_t f32_to_f16_rne(float f) {
  f = fminf(fmaxf(f, -65504.0f), 65504.0f);
  return __builtin_bit_cast(uint16_t, (_Float16)f);
}
__device__ __forceinline__ float f16_to_f32(uint16_t h) { return (float)__builtin_bit_cast(_Float16, h); }

template <bool F16>
__device__ __forceinline__ uint16_t to_plane(float f) { return F16 ? f32_to_f16_rne(f) : f32_to_bf16_rne(f); }
template <bool F16>
__device__ __forceinline__ float from_plane(uint16_t h) { return F16 ? f16_to_f32(h) : bf16_to_f32(h); }

// The 16-byte half h (8 k) of row r inside a k-block sits at position h ^ swz(r).  The operand
// reads of a wave touch 32 consecutive rows at one logical half: with the swap, any 8 or 16
// consecutive rows spread over all LDS banks.
__device__ __forceinline__ int swz(int row) { return (row >> 3) & 1; }

// s_waitcnt immediate (gfx9 encoding) that waits on vmcnt only.
constexpr int waitcnt_vm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }
// ... and one that waits for lgkmcnt(0) only (LDS reads returned).
constexpr int waitcnt_lgkm0() { return 15 | (3 << 14) | (7 << 4) | (0 << 8); }

// Emission of a result's transpose as operand planes.  An accumulator lane holds, for one plane row
// (col), four groups of four consecutive k: k = kbase + 8 g + 4 lk + (0..3), g = 0..3, lk = lane / 32;
// w[g] are those four values as two packed BF16 pairs.  Lanes l and l ^ 32 hold the two halves of every
// aligned 8-k chunk (16 bytes of a plane row): the pair swaps halves, so that each lane stores whole
// 16-byte chunks (lk = 0 those of g = 0 and 2, lk = 1 those of g = 1 and 3) instead of 8-byte halves.
__device__ __forceinline__ void emit_chunks(uint16_t* __restrict__ P, const uint32_t (&w)[4][2], int kbase, int col, int stride,
                                            int lk) {
#pragma unroll
  for (int pr = 0; pr < 2; ++pr) {
    // my half of the chunk my partner stores goes over; its half of the chunk I store comes back
    const uint32_t s0 = lk ? w[2 * pr][0] : w[2 * pr + 1][0];
    const uint32_t s1 = lk ? w[2 * pr][1] : w[2 * pr + 1][1];
    const uint32_t r0 = (uint32_t)__shfl_xor((int)s0, 32, 64);
    const uint32_t r1 = (uint32_t)__shfl_xor((int)s1, 32, 64);
    const uint32_t m0 = lk ? w[2 * pr + 1][0] : w[2 * pr][0];
    const uint32_t m1 = lk ? w[2 * pr + 1][1] : w[2 * pr][1];
    const int kc = kbase + 8 * (2 * pr + lk);
    const size_t o = (((size_t)(kc >> 4) * stride + col) * 2 + (((kc >> 3) & 1) ^ swz(col))) * 8;
    *reinterpret_cast<uint4*>(P + o) = lk ? make_uint4(r0, r1, m0, m1) : make_uint4(m0, m1, r0, r1);
  }
}

// Two values to a packed pair of BF16 (round to nearest even): the hardware's packed conversion, one instruction
// where the integer formulation takes seven per value.
typedef __bf16 br_bf16x2 __attribute__((ext_vector_type(2)));
typedef float br_f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t bf16_pair(float a, float b) {
  const br_f32x2 v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, br_bf16x2));
}

template <bool F16>
__device__ __forceinline__ void pack_hi_lo(const float (&val)[4], uint32_t (&hi)[2], uint32_t (&lo)[2], bool want_lo, float scale) {
  if (!F16) {
    hi[0] = bf16_pair(val[0], val[1]);
    hi[1] = bf16_pair(val[2], val[3]);
    lo[0] = lo[1] = 0u;
    if (want_lo) {
      lo[0] = bf16_pair(val[0] - __uint_as_float(hi[0] << 16), val[1] - __uint_as_float(hi[0] & 0xffff0000u));
      lo[1] = bf16_pair(val[2] - __uint_as_float(hi[1] << 16), val[3] - __uint_as_float(hi[1] & 0xffff0000u));
    }
    return;
  }
  uint16_t h[4], l[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float x = F16 ? val[e] * scale : val[e];
    h[e] = to_plane<F16>(x);
    l[e] = want_lo ? to_plane<F16>(x - from_plane<F16>(h[e])) : (uint16_t)0;
  }
  hi[0] = (uint32_t)h[0] | ((uint32_t)h[1] << 16);
  hi[1] = (uint32_t)h[2] | ((uint32_t)h[3] << 16);
  lo[0] = (uint32_t)l[0] | ((uint32_t)l[1] << 16);
  lo[1] = (uint32_t)l[2] | ((uint32_t)l[3] << 16);
}

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

}  // namespace

namespace br {

// EPI selects what happens to the 256 x 256 tile of alpha A B^T:
//   EPI_F32     C = tile + beta C in FP32 (optionally mirrored, optional BF16 image; with emit_t the
//               transpose of what was stored also leaves as operand planes, as under EPI_PLANES);
//   EPI_PLANES  nothing is stored in FP32: the TRANSPOSE of the result is written as BF16 operand
//               planes (hi, and lo when out_lo) ready to be the A or B operand of the next
//               contraction.  An accumulator lane holds 4 consecutive M indices of one N index,
//               i.e. 4 consecutive k of one plane row: half of a 16-byte chunk, whose other half sits in
//               lane + 32; the two swap halves and each stores whole chunks (emit_chunks);
//   EPI_ADAM    the tile is a rotated gradient G~: Adam's moments are advanced in place
//               (S~ <- b2 S~ + (1-b2) G~ G~, and M~ <- b1 M~ + (1-b1) G~ when adam.update_mrot;
//               Algorithm 1, from the rotated moment to the update) and X = M~ / sqrt(S~ + eps) leaves as planes like above.
//               With adam_t the tile is G~^T instead (right factor only: G~^T = Q_R^T G^T), the
//               moments are indexed [col][row], and what leaves are the planes of X itself.
// F16: the planes hold FP16 values and the products are v_mfma_f32_32x32x16_f16 (same shape, same lane layout and
// rate as the BF16 instruction).
template <int NPROD, int EPI, bool F16 = false>
__global__ __launch_bounds__(512, 1) void br_gemm_bf16_mfma(LowpKernArgs g, BrLowpBatch batch) {
  constexpr bool SPLIT = NPROD > 1;
  constexpr int KS = SPLIT ? 1 : 2;   // k-steps (16 k) per stage
  constexpr int G = SPLIT ? 4 : 2;    // groups of matrix instructions per k-step
  constexpr int MPG = FM / G;         // accumulator rows per group
  constexpr int U = KS * G;           // groups per stage
  constexpr int S = STAGES, LPT = LOADS;
  static_assert(U % 2 == 0, "operand double buffering assumes an even number of groups per stage");
  __shared__ uint4 lds[S * STAGE_U4];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 2, wn = wave & 3;
  const int lk = lane >> 5, li = lane & 31;

  // Position v of the launch's tile sequence -> (matrix, tile row, tile column).  Positions that
  // are congruent modulo the number of XCDs (the workgroups of one XCD, and all the positions a
  // workgroup visits: the grid is a multiple of that number whenever it visits more than one) cover
  // one contiguous run of tiles, so an XCD's L2 sees neighbouring tiles at the same time.
  const int per = g.all_tiles / NUM_XCD;
  auto decode = [&](int v, int& mat, int& tm, int& tn) {
    if (v < per * NUM_XCD) v = (v % NUM_XCD) * per + v / NUM_XCD;
    mat = v / g.total_tiles;
    const int t = v - mat * g.total_tiles;
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
  };

  floatx16 acc[FM][FN];

  // uint4 strides: one k-block (16 k) of a plane = rows * 2, one plane = elements / 8.  Wave w
  // moves the w-th KB of each sub-tile: source and destination are both linear, 64 lanes x 16 bytes.
  const size_t a_kb = (size_t)g.Mp * 2, b_kb = (size_t)g.b_stride * 2;
  const size_t a_pl = g.a_plane >> 3, b_pl = g.b_plane >> 3;
  const uint4* a_src = nullptr;
  const uint4* b_src = nullptr;
  auto aim = [&](int mat, int tm, int tn) {  // the operand loads of the tile at (mat, tm, tn) start here
    a_src = reinterpret_cast<const uint4*>(batch.A[mat]) + (size_t)tm * (TILE * 2) + wave * 64 + lane;
    b_src = reinterpret_cast<const uint4*>(batch.B[mat]) + (size_t)tn * (TILE * 2) + wave * 64 + lane;
  };
  auto load1k = [&](const uint4* src, int dst_u4) {
    __builtin_amdgcn_global_load_lds((gptr_t)src, (lptr_t)&lds[dst_u4], 16, 0, 0);
  };
  // Sub-tiles of a stage.  NPROD = 1: A(k-step 0), B(0), A(1), B(1).  Split: A_hi, A_lo, B_hi, B_lo.
  auto issue = [&](int st, int kt) {
    const int base = st * STAGE_U4 + wave * 64;
    if (!SPLIT) {
      const uint4* a = a_src + (size_t)(2 * kt) * a_kb;
      const uint4* b = b_src + (size_t)(2 * kt) * b_kb;
      load1k(a, base);
      load1k(b, base + SUB_U4);
      load1k(a + a_kb, base + 2 * SUB_U4);
      load1k(b + b_kb, base + 3 * SUB_U4);
    } else {
      const uint4* a = a_src + (size_t)kt * a_kb;
      const uint4* b = b_src + (size_t)kt * b_kb;
      load1k(a, base);
      load1k(a + a_pl, base + SUB_U4);
      load1k(b, base + 2 * SUB_U4);
      load1k(b + b_pl, base + 3 * SUB_U4);
    }
  };

  struct AFrag { bf16x8 hi[MPG], lo[MPG]; };  // FP16 planes travel in the same registers and are re-typed at the instruction
  struct BFrag { bf16x8 hi[FN], lo[FN]; };
  const int half = lk ^ swz(li);  // wave tile rows start at multiples of 32: swz(row) == swz(li)
  const int a_row = (wm * FM * 32 + li) * 2 + half, b_row = (wn * FN * 32 + li) * 2 + half;
  auto fetch_a = [&](AFrag& f, int st, int ks, int grp) {
    const int base = st * STAGE_U4 + (SPLIT ? 0 : 2 * ks * SUB_U4) + a_row + grp * MPG * 64;
#pragma unroll
    for (int q = 0; q < MPG; ++q) {
      f.hi[q] = __builtin_bit_cast(bf16x8, lds[base + q * 64]);
      if (SPLIT) f.lo[q] = __builtin_bit_cast(bf16x8, lds[base + SUB_U4 + q * 64]);
    }
  };
  auto fetch_b = [&](BFrag& f, int st, int ks) {
    const int base = st * STAGE_U4 + (SPLIT ? 2 * SUB_U4 : (2 * ks + 1) * SUB_U4) + b_row;
#pragma unroll
    for (int q = 0; q < FN; ++q) {
      f.hi[q] = __builtin_bit_cast(bf16x8, lds[base + q * 64]);
      if (SPLIT) f.lo[q] = __builtin_bit_cast(bf16x8, lds[base + SUB_U4 + q * 64]);
    }
  };
#define BR_MMA(x, y, c)                                                                                                        \
  do {                                                                                                                         \
    if constexpr (F16)                                                                                                         \
      c = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8, x), __builtin_bit_cast(half8, y), c, 0, 0, 0);      \
    else                                                                                                                       \
      c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, y, c, 0, 0, 0);                                                           \
  } while (0)
  // NPROD = 4 exists for the symmetric statistics, whose DIAGONAL would otherwise carry the bias
  // sum_k lo_k^2 (every term positive).  Off the diagonal the lo*lo terms have random signs and sum
  // to about 2^-18 / sqrt(K) of the matrix's scale, below FP32 resolution: only the tiles on the
  // diagonal of a mirrored product issue the fourth instruction.
  bool lolo = true;
  auto multiply = [&](const AFrag& a, const BFrag& b, int grp) {
#pragma unroll
    for (int q = 0; q < MPG; ++q) {
      const int mi = grp * MPG + q;
#pragma unroll
      for (int ni = 0; ni < FN; ++ni) {
        if (NPROD == 4 && lolo) BR_MMA(a.lo[q], b.lo[ni], acc[mi][ni]);
        if (NPROD >= 3) {
          BR_MMA(a.lo[q], b.hi[ni], acc[mi][ni]);
          BR_MMA(a.hi[q], b.lo[ni], acc[mi][ni]);
        }
        BR_MMA(a.hi[q], b.hi[ni], acc[mi][ni]);
      }
    }
  };

  // The ring always holds S stages: past the end of k the LAST one is loaded again into the
  // stage that has just been freed (nobody reads it), which keeps the loop free of branches and
  // the number of loads in flight constant.
  const int nkt = g.Kp / (16 * KS);
  auto prologue = [&]() {
#pragma unroll
    for (int p = 0; p < S; ++p) issue(p, min(p, nkt - 1));
  };
  // A workgroup walks the tile sequence with the grid as its stride.  The first S stages of a
  // tile are requested before the epilogue of the tile before it, so their latency hides there.
  int mat, tm, tn;
  decode(blockIdx.x, mat, tm, tn);
  aim(mat, tm, tn);
  prologue();
  for (int v = blockIdx.x; v < g.all_tiles; v += gridDim.x) {
  float* __restrict__ C = batch.C[mat];
  uint16_t* __restrict__ shadow = batch.shadow[mat];
  const int m0 = tm * TILE, n0 = tn * TILE;
  lolo = !g.mirror || tm == tn;
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
  // This wave's share of stage 0 has landed.  After the first tile the count also holds the
  // epilogue's stores, which may complete out of order with the loads: wait for everything.
  if (v == (int)blockIdx.x) __builtin_amdgcn_s_waitcnt(waitcnt_vm((S - 1) * LPT));
  else __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
  // Bare barriers: __syncthreads() would add a fence that waits for ALL outstanding loads, the
  // ones of the later stages included, and serialise the pipeline.
  __builtin_amdgcn_s_barrier();
  AFrag af[2];
  BFrag bf[2];
  fetch_b(bf[0], 0, 0);
  fetch_a(af[0], 0, 0, 0);
  int st = 0;
  // One stage = U groups of matrix instructions; group u's operands are fetched during group u - 1.
  auto stage = [&](int kt, bool last) {
    const int nst = (st + 1 == S) ? 0 : st + 1;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int ks = u / G, grp = u % G;
      if (u + 1 < U) {
        const int nks = (u + 1) / G, ngrp = (u + 1) % G;
        if (ngrp == 0) fetch_b(bf[nks & 1], st, nks);
        fetch_a(af[(u + 1) & 1], st, nks, ngrp);
      } else if (!last) {
        __builtin_amdgcn_s_waitcnt(waitcnt_lgkm0());            // this wave is done reading stage st
        __builtin_amdgcn_s_waitcnt(waitcnt_vm((S - 2) * LPT));  // its share of stage kt + 1 has landed
        __builtin_amdgcn_s_barrier();                           // ... everybody's; and stage st is free
        issue(st, min(kt + S, nkt - 1));
        fetch_b(bf[KS & 1], nst, 0);
        fetch_a(af[0], nst, 0, 0);
      }
      multiply(af[u & 1], bf[ks & 1], grp);
    }
    if (KS & 1) bf[0] = bf[1];  // odd k-steps per stage: the next stage's B operands were fetched into bf[1]
    st = nst;
  };
  for (int kt = 0; kt + 1 < nkt; ++kt) stage(kt, false);
  stage(nkt - 1, true);
  __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));  // the surplus loads of the last iterations
  int mat_n = mat, tm_n = tm, tn_n = tn;
  if (v + (int)gridDim.x < g.all_tiles) {
    __builtin_amdgcn_s_waitcnt(waitcnt_lgkm0());
    __builtin_amdgcn_s_barrier();  // every wave has read its last operands and its surplus loads have landed: the ring is free
    decode(v + (int)gridDim.x, mat_n, tm_n, tn_n);
    aim(mat_n, tm_n, tn_n);
    prologue();
  }

  if (EPI == EPI_F32) {
    const bool use_beta = (g.beta != 0.0f);
    const bool off_diag = g.mirror && (tm != tn);
    const int Mlim = (g.skip && g.skip[mat]) ? 0 : g.M;  // a skipped matrix stores nothing
    bool bad = false;
    // Tiles that lie wholly inside the matrix and need nothing but C = alpha acc (+ beta C): no bounds tests, one
    // lane pointer, row offsets that are the same for every lane.
    // Tiles that lie wholly inside the matrix take paths without bounds tests, on lane pointers that WALK the
    // lane's 64 rows in the order the accumulators hold them (steps of one row and of five rows, the same for
    // every lane; the two 32-wide column blocks of a row are 128 bytes apart).  The general path below spends
    // several times the instructions per value on tests and 64-bit address arithmetic, and with one workgroup per
    // compute unit nothing hides an epilogue's instruction stream: +9 to 10 % on whole launches at K = 2560.
    // (The empty asm statements keep each walk a walk: otherwise the compiler forms all 128 addresses up front.)
    const bool inside = (m0 + TILE <= Mlim) && (n0 + TILE <= g.N);
    if (inside && !shadow && !g.emit_t && !g.mirror) {
      const size_t ld = (size_t)g.ldc;
      float* __restrict__ ps = C + (size_t)(m0 + wm * FM * 32 + 4 * lk) * ld + (n0 + wn * FN * 32 + li);
      if (!use_beta) {
#pragma unroll
        for (int mi = 0; mi < FM; ++mi) {
#pragma unroll
          for (int e = 0; e < 16; ++e) {
#pragma unroll
            for (int ni = 0; ni < FN; ++ni) {
              const float val = g.alpha * acc[mi][ni][e];
              ps[ni * 32] = val;
              if (g.health) bad |= not_finite(val);
            }
            ps += ((e & 3) == 3) ? 5 * ld : ld;
            asm volatile("" : "+v"(ps));
          }
        }
      } else {
        // read-modify-write: the old values of eight rows (both column blocks) are fetched one such unit ahead
        const float* __restrict__ pl = ps;
        float oldf[2][8 * FN];
        auto fetch_unit = [&](int u, float* dst) {
          const int h = u & 1;
#pragma unroll
          for (int r = 0; r < 8; ++r) {
#pragma unroll
            for (int ni = 0; ni < FN; ++ni) dst[r * FN + ni] = pl[ni * 32];
            pl += (((h * 8 + r) & 3) == 3) ? 5 * ld : ld;
            asm volatile("" : "+v"(pl));
          }
        };
        fetch_unit(0, oldf[0]);
#pragma unroll
        for (int u = 0; u < 2 * FM; ++u) {
          const int mi = u >> 1, h = u & 1;
          if (u + 1 < 2 * FM) fetch_unit(u + 1, oldf[(u + 1) & 1]);
#pragma unroll
          for (int r = 0; r < 8; ++r) {
            const int e = h * 8 + r;
#pragma unroll
            for (int ni = 0; ni < FN; ++ni) {
              // beta times the old value goes into the fused multiply-add unrounded: one rounding at the size of C
              const float val = __builtin_fmaf(g.beta, oldf[u & 1][r * FN + ni], g.alpha * acc[mi][ni][e]);
              ps[ni * 32] = val;
              if (g.health) bad |= not_finite(val);
            }
            ps += ((e & 3) == 3) ? 5 * ld : ld;
            asm volatile("" : "+v"(ps));
          }
        }
      }
      if (g.health && __any(bad) && lane == 0) atomicAdd(g.health + BR_HEALTH_NONFINITE_WEIGHT, 1);
    } else {
    // Old values of an accumulator's sixteen outputs are fetched together, one accumulator ahead
    // of the stores: a load issued after a store to the same matrix would wait for it.
    float oldv[2][16];
    auto fetch_old = [&](int a, float* dst) {
      const int mi = a / FN, ni = a % FN;
      const int col = n0 + (wn * FN + ni) * 32 + li;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = m0 + (wm * FM + mi) * 32 + 8 * (v >> 2) + 4 * lk + (v & 3);
        dst[v] = (use_beta && row < Mlim && col < g.N) ? C[(size_t)row * (size_t)g.ldc + col] : 0.f;
      }
    };
    fetch_old(0, oldv[0]);
#pragma unroll
    for (int mi = 0; mi < FM; ++mi) {
#pragma unroll
      for (int ni = 0; ni < FN; ++ni) {
        const int col = n0 + (wn * FN + ni) * 32 + li;
        const int a = mi * FN + ni;
        if (a + 1 < FM * FN) fetch_old(a + 1, oldv[(a + 1) & 1]);
        const float* old = oldv[a & 1];
        uint32_t wh[4][2], wl[4][2];  // emit_t: the stored values as packed BF16 pairs (hi, lo), one entry per group of four rows
#pragma unroll
        for (int vg = 0; vg < 4; ++vg) {
          const int row0 = m0 + (wm * FM + mi) * 32 + 8 * vg + 4 * lk;
          float val[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int row = row0 + e;
            val[e] = g.alpha * acc[mi][ni][vg * 4 + e];
            if (use_beta) val[e] += g.beta * old[vg * 4 + e];
            if (row < Mlim && col < g.N) {
              const size_t off = (size_t)row * (size_t)g.ldc + col;
              C[off] = val[e];
              if (shadow) shadow[off] = f32_to_bf16_rne(val[e]);
              bad |= not_finite(val[e]);
            }
          }
          if (g.emit_t) pack_hi_lo<F16>(val, wh[vg], wl[vg], g.out_lo != 0, g.out_scale);
          if (off_diag && col < g.N && Mlim > 0) {
            // transposed copy of a symmetric result: this lane's four rows are four consecutive columns there
            float* dst = C + (size_t)col * (size_t)g.ldc + row0;
            if (row0 + 3 < g.M && ((g.ldc & 3) == 0)) {
              *reinterpret_cast<float4*>(dst) = make_float4(val[0], val[1], val[2], val[3]);
            } else {
#pragma unroll
              for (int e = 0; e < 4; ++e)
                if (row0 + e < g.M) dst[e] = val[e];
            }
          }
        }
        {
          // the stored values once more, transposed, as operand planes (hi + lo when out_lo): what the next
          // contraction of a chain of updates reads; exactly zero in the padding (the operands are zero there)
          const int kbase = m0 + (wm * FM + mi) * 32;
          if (g.emit_t && kbase < g.out_kp && Mlim > 0) {  // out_kp is a multiple of 64: all four groups or none
            uint16_t* __restrict__ Pt = reinterpret_cast<uint16_t*>(batch.S[mat]);
            emit_chunks(Pt, wh, kbase, col, g.out_stride, lk);
            if (g.out_lo) emit_chunks(Pt + g.out_plane, wl, kbase, col, g.out_stride, lk);
          }
        }
      }
    }
    if (g.health && __any(bad) && lane == 0) atomicAdd(g.health + BR_HEALTH_NONFINITE_WEIGHT, 1);
    }
  } else {
    uint16_t* __restrict__ Pout = shadow;  // the emitted planes travel in the batch's 16-bit output slot
    float* __restrict__ S = batch.S[mat];
    float* __restrict__ Mr = batch.Mrot[mat];
    const BrAdamArgs ad = g.adam;
    const float w1 = 1.0f - ad.beta1, w2 = 1.0f - ad.beta2;
    if (EPI == EPI_ADAM && !g.adam_t && m0 + TILE <= g.M && n0 + TILE <= g.N) {
      // Tiles wholly inside the matrix: no bounds tests, and two lane pointers each for the moments (one that
      // stores, one that loads a unit of eight rows ahead) that walk the lane's rows as in the FP32 epilogue.
      const size_t ld = (size_t)g.ldc;
      const size_t o0 = (size_t)(m0 + wm * FM * 32 + 4 * lk) * ld + (n0 + wn * FN * 32 + li);
      float* __restrict__ sS = S + o0;
      float* __restrict__ sM = Mr + o0;
      const float* __restrict__ lS = sS;
      const float* __restrict__ lM = sM;
      float mo[2][8 * FN], so[2][8 * FN];
      auto fetch_unit = [&](int u, float* md, float* sd) {
        const int h = u & 1;
#pragma unroll
        for (int r = 0; r < 8; ++r) {
#pragma unroll
          for (int ni = 0; ni < FN; ++ni) {
            md[r * FN + ni] = lM[ni * 32];
            sd[r * FN + ni] = lS[ni * 32];
          }
          const size_t step = (((h * 8 + r) & 3) == 3) ? 5 * ld : ld;
          lM += step;
          lS += step;
          asm volatile("" : "+v"(lM), "+v"(lS));
        }
      };
      fetch_unit(0, mo[0], so[0]);
#pragma unroll
      for (int mi = 0; mi < FM; ++mi) {
        uint32_t wh[FN][4][2], wl[FN][4][2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int u = mi * 2 + h;
          if (u + 1 < 2 * FM) fetch_unit(u + 1, mo[(u + 1) & 1], so[(u + 1) & 1]);
#pragma unroll
          for (int vgl = 0; vgl < 2; ++vgl) {
            const int vg = h * 2 + vgl;
            float val[FN][4];
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
              const int r = vgl * 4 + e4;
#pragma unroll
              for (int ni = 0; ni < FN; ++ni) {
                const float gt = g.alpha * acc[mi][ni][vg * 4 + e4];
                float mt = mo[u & 1][r * FN + ni];
                if (ad.update_mrot) {
                  mt = ad.beta1 * mt + w1 * gt;
                  sM[ni * 32] = mt;
                }
                const float st2 = ad.beta2 * so[u & 1][r * FN + ni] + w2 * (gt * gt);
                sS[ni * 32] = st2;
                const float num = mt * ad.c1, den = st2 * ad.c2;
                val[ni][e4] = ad.eps_outside ? num * __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(den) + ad.eps)
                                             : num * __builtin_amdgcn_rsqf(den + ad.eps);
              }
              const size_t step = (e4 == 3) ? 5 * ld : ld;
              sM += step;
              sS += step;
              asm volatile("" : "+v"(sM), "+v"(sS));
            }
#pragma unroll
            for (int ni = 0; ni < FN; ++ni) pack_hi_lo<F16>(val[ni], wh[ni][vg], wl[ni][vg], g.out_lo != 0, g.out_scale);
          }
        }
        const int kbase = m0 + (wm * FM + mi) * 32;
        if (kbase < g.out_kp) {
#pragma unroll
          for (int ni = 0; ni < FN; ++ni) {
            const int col = n0 + (wn * FN + ni) * 32 + li;
            emit_chunks(Pout, wh[ni], kbase, col, g.out_stride, lk);
            if (g.out_lo) emit_chunks(Pout + g.out_plane, wl[ni], kbase, col, g.out_stride, lk);
          }
        }
      }
    } else {
    // EPI_ADAM: the moments of an accumulator's sixteen entries are fetched together, one accumulator
    // ahead of the stores (a load issued after a store to the same array would wait for it).
    float moldv[2][16], soldv[2][16];
    auto fetch_moments = [&](int a, float* md, float* sd) {
      const int mi = a / FN, ni = a % FN;
      const int col = n0 + (wn * FN + ni) * 32 + li;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = m0 + (wm * FM + mi) * 32 + 8 * (v >> 2) + 4 * lk + (v & 3);
        const bool in = row < g.M && col < g.N;
        const size_t off = g.adam_t ? (size_t)col * (size_t)g.ldc + row : (size_t)row * (size_t)g.ldc + col;
        md[v] = in ? Mr[off] : 0.f;
        sd[v] = in ? S[off] : 0.f;
      }
    };
    if (EPI == EPI_ADAM) fetch_moments(0, moldv[0], soldv[0]);
#pragma unroll
    for (int mi = 0; mi < FM; ++mi) {
#pragma unroll
      for (int ni = 0; ni < FN; ++ni) {
        const int col = n0 + (wn * FN + ni) * 32 + li;  // plane row; below Np by construction
        const int a = mi * FN + ni;
        if (EPI == EPI_ADAM && a + 1 < FM * FN) fetch_moments(a + 1, moldv[(a + 1) & 1], soldv[(a + 1) & 1]);
        const float* mold = moldv[a & 1];
        const float* sold = soldv[a & 1];
        uint32_t wh[4][2], wl[4][2];
#pragma unroll
        for (int vg = 0; vg < 4; ++vg) {
          const int row0 = m0 + (wm * FM + mi) * 32 + 8 * vg + 4 * lk;  // plane k of val[0]
          float val[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            val[e] = g.alpha * acc[mi][ni][vg * 4 + e];  // exactly zero in the padding: the operands are zero there
            if (EPI == EPI_ADAM) {
              const int row = row0 + e;
              float x = 0.f;
              if (row < g.M && col < g.N) {
                const size_t off = g.adam_t ? (size_t)col * (size_t)g.ldc + row : (size_t)row * (size_t)g.ldc + col;
                const float gt = val[e];
                float mt = mold[vg * 4 + e];
                if (ad.update_mrot) {
                  mt = ad.beta1 * mt + w1 * gt;
                  Mr[off] = mt;
                }
                const float st2 = ad.beta2 * sold[vg * 4 + e] + w2 * (gt * gt);
                S[off] = st2;
                const float num = mt * ad.c1, den = st2 * ad.c2;
                // one-ulp hardware reciprocal square root / reciprocal (the arguments are normal numbers:
                // den + eps >= eps); the quotient leaves as BF16 planes anyway
                x = ad.eps_outside ? num * __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(den) + ad.eps)
                                   : num * __builtin_amdgcn_rsqf(den + ad.eps);
              }
              val[e] = x;
            }
          }
          pack_hi_lo<F16>(val, wh[vg], wl[vg], g.out_lo != 0, g.out_scale);
        }
        {
          const int kbase = m0 + (wm * FM + mi) * 32;
          if (kbase < g.out_kp) {  // out_kp is a multiple of 64: all four groups or none
            emit_chunks(Pout, wh, kbase, col, g.out_stride, lk);
            if (g.out_lo) emit_chunks(Pout + g.out_plane, wl, kbase, col, g.out_stride, lk);
          }
        }
      }
    }
    }
  }
  mat = mat_n;
  tm = tm_n;
  tn = tn_n;
  }  // tiles of this workgroup
}

// ---- operand preparation -----------------------------------------------------------------
struct SplitArgs {
  const float* src[BR_MAXB];
  uint16_t* dst[BR_MAXB];  // hi plane; the lo plane follows at +plane elements
};

// What a split kernel writes: BF16 planes of x, or FP16 planes of scale * x.
struct PlaneFormat {
  int f16;
  float scale;
};

// scale = base * 2^(target - e) with max = f * 2^e, f in [0.5, 1): the largest entry lands in [2^(target-1), 2^target).
__device__ __forceinline__ float normalising_scale(float base, const unsigned* maxbits, int target_exp) {
  if (!maxbits) return base;
  const float mx = __uint_as_float(maxbits[blockIdx.y]);
  if (!(mx > 0.f) || (__float_as_uint(mx) & 0x7f800000u) == 0x7f800000u) return base;
  int e;
  (void)frexpf(mx, &e);
  return ldexpf(base, target_exp - e);
}

template <bool F16>
__device__ __forceinline__ void split8_as(const float* x, uint4* hi4, uint4* lo4, float scale) {
  uint32_t hi[4], lo[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float x0 = F16 ? x[2 * e] * scale : x[2 * e], x1 = F16 ? x[2 * e + 1] * scale : x[2 * e + 1];
    const uint16_t h0 = to_plane<F16>(x0), h1 = to_plane<F16>(x1);
    hi[e] = (uint32_t)h0 | ((uint32_t)h1 << 16);
    const uint16_t l0 = to_plane<F16>(x0 - from_plane<F16>(h0));
    const uint16_t l1 = to_plane<F16>(x1 - from_plane<F16>(h1));
    lo[e] = (uint32_t)l0 | ((uint32_t)l1 << 16);
  }
  *hi4 = make_uint4(hi[0], hi[1], hi[2], hi[3]);
  *lo4 = make_uint4(lo[0], lo[1], lo[2], lo[3]);
}

__device__ __forceinline__ void split8(const float* x, uint4* hi4, uint4* lo4, PlaneFormat f = PlaneFormat{0, 1.f}) {
  if (f.f16) split8_as<true>(x, hi4, lo4, f.scale);
  else split8_as<false>(x, hi4, lo4, 1.f);
}

// Largest magnitude of each matrix of a batch, as the bit pattern of a non-negative float (which orders like the
// integer it is: an integer atomic maximum, the same result in any order).  maxbits must be zero beforehand.
__global__ __launch_bounds__(256) void br_absmax(SplitArgs a, int R, int Ccols, int ld_src, unsigned* __restrict__ maxbits) {
  __shared__ unsigned red[4];
  const float* __restrict__ X = a.src[blockIdx.y];
  const int64_t total = (int64_t)R * Ccols;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  float m = 0.f;
  if (ld_src == Ccols && (total & 3) == 0 && (reinterpret_cast<uintptr_t>(X) & 15u) == 0) {
    // contiguous matrix: 16-byte loads, four in flight per thread
    const float4* __restrict__ X4 = reinterpret_cast<const float4*>(X);
    const int64_t n4 = total >> 2;
    auto mx = [](const float4& v) { return fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))); };
    float m1 = 0.f, m2 = 0.f, m3 = 0.f;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (; i + 3 * stride < n4; i += 4 * stride) {
      const float4 v0 = X4[i], v1 = X4[i + stride], v2 = X4[i + 2 * stride], v3 = X4[i + 3 * stride];
      m = fmaxf(m, mx(v0));
      m1 = fmaxf(m1, mx(v1));
      m2 = fmaxf(m2, mx(v2));
      m3 = fmaxf(m3, mx(v3));
    }
    for (; i < n4; i += stride) m = fmaxf(m, mx(X4[i]));
    m = fmaxf(fmaxf(m, m1), fmaxf(m2, m3));
  } else {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
      const int64_t r = i / Ccols;
      m = fmaxf(m, fabsf(X[r * ld_src + (i - r * Ccols)]));
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = __float_as_uint(m);
  __syncthreads();
  if (threadIdx.x == 0) atomicMax(maxbits + blockIdx.y, max(max(red[0], red[1]), max(red[2], red[3])));
}

// Same orientation: plane rows = source rows, k = source column.  One thread per 16-byte chunk
// of the padded plane, chunk index within 32 k fastest, then row, then 32-k group: a wave reads
// 16 whole 128-byte lines of the source and writes two contiguous 512-byte runs of plane.
__global__ __launch_bounds__(256) void br_split_planes(SplitArgs a, int R, int Ccols, int ld_src, int Rp, int Kp, size_t plane,
                                                       int want_lo, PlaneFormat fmt, const unsigned* maxbits, int target_exp) {
  fmt.scale = normalising_scale(fmt.scale, maxbits, target_exp);
  const float* __restrict__ X = a.src[blockIdx.y];
  uint16_t* __restrict__ H = a.dst[blockIdx.y];
  const int64_t total = (int64_t)Rp * (Kp >> 3);
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  const bool vec = ((ld_src & 3) == 0) && ((reinterpret_cast<uintptr_t>(X) & 15u) == 0);
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
    const int c = (int)(i & 3);
    const int64_t rr = i >> 2;
    const int kb32 = (int)(rr / Rp);
    const int r = (int)(rr - (int64_t)kb32 * Rp);
    const int c0 = kb32 * 32 + c * 8;
    float x[8];
    if (r < R && c0 + 7 < Ccols && vec) {
      const float* row = X + (size_t)r * ld_src;
      float4 u = *reinterpret_cast<const float4*>(row + c0);
      float4 w = *reinterpret_cast<const float4*>(row + c0 + 4);
      x[0] = u.x; x[1] = u.y; x[2] = u.z; x[3] = u.w; x[4] = w.x; x[5] = w.y; x[6] = w.z; x[7] = w.w;
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) x[e] = (r < R && c0 + e < Ccols) ? X[(size_t)r * ld_src + c0 + e] : 0.f;
    }
    uint4 hi4, lo4;
    split8(x, &hi4, &lo4, fmt);
    const size_t o = (((size_t)(c0 >> 4) * Rp + r) * 2 + (((c0 >> 3) & 1) ^ swz(r))) * 8;
    *reinterpret_cast<uint4*>(H + o) = hi4;
    if (want_lo) *reinterpret_cast<uint4*>(H + plane + o) = lo4;
  }
}

// Transposed: plane rows = source columns, k = source row.  64 x 64 tiles through LDS;
// blockIdx.x enumerates tiles over the PADDED plane (Kp / 64 along k, Rp / 64 along rows), so
// the zero padding is written by the same pass.
__global__ __launch_bounds__(256) void br_split_planes_t(SplitArgs a, int R, int Ccols, int ld_src, int Rp, int Kp, size_t plane,
                                                         int want_lo, PlaneFormat fmt, const unsigned* maxbits, int target_exp) {
  __shared__ float tile[64][65];
  fmt.scale = normalising_scale(fmt.scale, maxbits, target_exp);
  const float* __restrict__ X = a.src[blockIdx.y];
  uint16_t* __restrict__ H = a.dst[blockIdx.y];
  const int tiles_c = Rp >> 6;
  const int tr = blockIdx.x / tiles_c, tc = blockIdx.x - tr * tiles_c;
  const int r0 = tr * 64, c0 = tc * 64;  // source row (= k) and source column (= plane row) origin
  const int tid = threadIdx.x;
  const bool vec = ((ld_src & 3) == 0) && ((reinterpret_cast<uintptr_t>(X) & 15u) == 0);
  if (vec && r0 + 64 <= R && c0 + 64 <= Ccols) {
    // whole tile inside the source: four 16-byte loads per thread, all in flight together
    float4 v[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int rr = i * 16 + (tid >> 4), c4 = (tid & 15) * 4;
      v[i] = *reinterpret_cast<const float4*>(X + (size_t)(r0 + rr) * ld_src + c0 + c4);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int rr = i * 16 + (tid >> 4), c4 = (tid & 15) * 4;
      tile[rr][c4 + 0] = v[i].x;
      tile[rr][c4 + 1] = v[i].y;
      tile[rr][c4 + 2] = v[i].z;
      tile[rr][c4 + 3] = v[i].w;
    }
  } else {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int rr = i * 4 + (tid >> 6), cc = tid & 63;
      const int r = r0 + rr, c = c0 + cc;
      tile[rr][cc] = (r < R && c < Ccols) ? X[(size_t)r * ld_src + c] : 0.f;
    }
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int cc = (tid >> 3) + 32 * i, rch = tid & 7;
    const int prow = c0 + cc, k0 = r0 + rch * 8;
    float x[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = tile[rch * 8 + e][cc];
    uint4 hi4, lo4;
    split8(x, &hi4, &lo4, fmt);
    const size_t o = (((size_t)(k0 >> 4) * Rp + prow) * 2 + (((k0 >> 3) & 1) ^ swz(prow))) * 8;
    *reinterpret_cast<uint4*>(H + o) = hi4;
    if (want_lo) *reinterpret_cast<uint4*>(H + plane + o) = lo4;
  }
}


// First moment and both plane sets of a gradient in one pass (Algorithm 1's first-moment update, and the operands
// of Algorithm 2's statistics and of Algorithm 1's gradient rotation): M <- beta1 M + (1 - beta1) G, planes of G and
// planes of G^T, the gradient read once.  One 64 x 64 tile per workgroup, transposed through LDS;
// tiles past the matrix write the planes' zero padding.
struct IngestArgs {
  const float* G[BR_MAXB];
  float* M[BR_MAXB];
  uint16_t* P[BR_MAXB];   // planes of G    (rows x cols)
  uint16_t* PT[BR_MAXB];  // planes of G^T  (cols x rows)
};

__global__ __launch_bounds__(256) void br_ingest_planes(IngestArgs a, int R, int Cc, float beta1, int RpP, int KpP, size_t planeP,
                                                        int RpT, int KpT, size_t planeT, int tiles_c, int want_lo) {
  __shared__ float tile[64][65];
  const float* __restrict__ G = a.G[blockIdx.y];
  float* __restrict__ M = a.M[blockIdx.y];
  uint16_t* __restrict__ P = a.P[blockIdx.y];
  uint16_t* __restrict__ PT = a.PT[blockIdx.y];
  const int tr = blockIdx.x / tiles_c, tc = blockIdx.x - tr * tiles_c;
  const int r0 = tr * 64, c0 = tc * 64;
  const int tid = threadIdx.x;
  const float w = 1.0f - beta1;
  const bool vec = ((Cc & 3) == 0) && (((reinterpret_cast<uintptr_t>(G) | reinterpret_cast<uintptr_t>(M)) & 15u) == 0);
  if (vec && r0 + 64 <= R && c0 + 64 <= Cc) {
    float4 g[4], m[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int rr = i * 16 + (tid >> 4), c4 = (tid & 15) * 4;
      const size_t o = (size_t)(r0 + rr) * Cc + c0 + c4;
      typedef float nt_f4 __attribute__((ext_vector_type(4)));
      const nt_f4 gv = __builtin_nontemporal_load(reinterpret_cast<const nt_f4*>(G + o));
      const nt_f4 mv = __builtin_nontemporal_load(reinterpret_cast<const nt_f4*>(M + o));
      g[i] = make_float4(gv.x, gv.y, gv.z, gv.w);
      m[i] = make_float4(mv.x, mv.y, mv.z, mv.w);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int rr = i * 16 + (tid >> 4), c4 = (tid & 15) * 4;
      const size_t o = (size_t)(r0 + rr) * Cc + c0 + c4;
      m[i].x = beta1 * m[i].x + w * g[i].x;
      m[i].y = beta1 * m[i].y + w * g[i].y;
      m[i].z = beta1 * m[i].z + w * g[i].z;
      m[i].w = beta1 * m[i].w + w * g[i].w;
      {
        typedef float nt_f4 __attribute__((ext_vector_type(4)));
        const nt_f4 mo = {m[i].x, m[i].y, m[i].z, m[i].w};
        __builtin_nontemporal_store(mo, reinterpret_cast<nt_f4*>(M + o));
      }
      tile[rr][c4 + 0] = g[i].x;
      tile[rr][c4 + 1] = g[i].y;
      tile[rr][c4 + 2] = g[i].z;
      tile[rr][c4 + 3] = g[i].w;
    }
  } else {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int rr = i * 4 + (tid >> 6), cc = tid & 63;
      const int r = r0 + rr, c = c0 + cc;
      float gv = 0.f;
      if (r < R && c < Cc) {
        const size_t o = (size_t)r * Cc + c;
        gv = G[o];
        M[o] = beta1 * M[o] + w * gv;
      }
      tile[rr][cc] = gv;
    }
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    // planes of G: plane row = source row, 8 consecutive source columns per chunk
    {
      const int rr = (tid >> 3) + 32 * i, ch = tid & 7;
      const int prow = r0 + rr, k0 = c0 + ch * 8;
      if (k0 < KpP) {
        float x[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = tile[rr][ch * 8 + e];
        uint4 hi4, lo4;
        split8(x, &hi4, &lo4);
        const size_t o = (((size_t)(k0 >> 4) * RpP + prow) * 2 + (((k0 >> 3) & 1) ^ swz(prow))) * 8;
        *reinterpret_cast<uint4*>(P + o) = hi4;
        if (want_lo) *reinterpret_cast<uint4*>(P + planeP + o) = lo4;
      }
    }
    // planes of G^T: plane row = source column, 8 consecutive source rows per chunk
    {
      const int cc = (tid >> 3) + 32 * i, rch = tid & 7;
      const int prow = c0 + cc, k0 = r0 + rch * 8;
      if (k0 < KpT) {
        float x[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = tile[rch * 8 + e][cc];
        uint4 hi4, lo4;
        split8(x, &hi4, &lo4);
        const size_t o = (((size_t)(k0 >> 4) * RpT + prow) * 2 + (((k0 >> 3) & 1) ^ swz(prow))) * 8;
        *reinterpret_cast<uint4*>(PT + o) = hi4;
        if (want_lo) *reinterpret_cast<uint4*>(PT + planeT + o) = lo4;
      }
    }
  }
}

}  // namespace br

hipError_t br_launch_absmax(hipStream_t s, const float* const* src, int batch, int R, int Ccols, int ld_src, unsigned* maxbits) {
  if (batch <= 0 || R <= 0 || Ccols <= 0) return hipSuccess;
  if (batch > BR_MAXB || ld_src < Ccols || !maxbits) return hipErrorInvalidValue;
  br::SplitArgs a;
  for (int i = 0; i < BR_MAXB; ++i) {
    a.src[i] = (i < batch) ? src[i] : nullptr;
    a.dst[i] = nullptr;
  }
  int64_t blocks = ((int64_t)R * Ccols + 256 * 16 - 1) / (256 * 16);
  int64_t cap = (4096 + batch - 1) / batch;
  if (blocks > cap) blocks = cap;
  hipLaunchKernelGGL(br::br_absmax, dim3((int)blocks, batch), dim3(256), 0, s, a, R, Ccols, ld_src, maxbits);
  return hipGetLastError();
}

hipError_t br_launch_split_planes(hipStream_t s, const float* const* src, uint16_t* const* dst, int batch, int R, int Ccols,
                                  int ld_src, int transpose, int want_lo, int f16, float scale, const unsigned* maxbits,
                                  int target_exp) {
  if (batch <= 0 || R <= 0 || Ccols <= 0) return hipSuccess;
  if (batch > BR_MAXB || ld_src < Ccols) return hipErrorInvalidValue;
  br::SplitArgs a;
  for (int i = 0; i < BR_MAXB; ++i) {
    a.src[i] = (i < batch) ? src[i] : nullptr;
    a.dst[i] = (i < batch) ? dst[i] : nullptr;
  }
  const BrPlaneLayout pl = transpose ? br_plane_layout(Ccols, R) : br_plane_layout(R, Ccols);
  if (pl.rows_p > 0x7fffffffLL || pl.k_p > 0x7fffffffLL) return hipErrorInvalidValue;
  if (maxbits && !f16) return hipErrorInvalidValue;
  const br::PlaneFormat fmt{f16 ? 1 : 0, f16 ? scale : 1.f};
  if (!transpose) {
    int64_t blocks = (pl.rows_p * (pl.k_p >> 3) + 255) / 256;
    int64_t cap = (8192 + batch - 1) / batch;
    if (blocks > cap) blocks = cap;
    hipLaunchKernelGGL(br::br_split_planes, dim3((int)blocks, batch), dim3(256), 0, s, a, R, Ccols, ld_src, (int)pl.rows_p,
                       (int)pl.k_p, pl.elems, want_lo, fmt, maxbits, target_exp);
  } else {
    int64_t tiles = (pl.k_p >> 6) * (pl.rows_p >> 6);
    if (tiles > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(br::br_split_planes_t, dim3((int)tiles, batch), dim3(256), 0, s, a, R, Ccols, ld_src, (int)pl.rows_p,
                       (int)pl.k_p, pl.elems, want_lo, fmt, maxbits, target_exp);
  }
  return hipGetLastError();
}

hipError_t br_launch_ingest_planes(hipStream_t s, const float* const* G, float* const* M, uint16_t* const* P, uint16_t* const* PT,
                                   int batch, int R, int Ccols, float beta1, int want_lo) {
  if (batch <= 0 || R <= 0 || Ccols <= 0) return hipSuccess;
  if (batch > BR_MAXB) return hipErrorInvalidValue;
  br::IngestArgs a;
  for (int i = 0; i < BR_MAXB; ++i) {
    a.G[i] = (i < batch) ? G[i] : nullptr;
    a.M[i] = (i < batch) ? M[i] : nullptr;
    a.P[i] = (i < batch) ? P[i] : nullptr;
    a.PT[i] = (i < batch) ? PT[i] : nullptr;
  }
  const BrPlaneLayout lp = br_plane_layout(R, Ccols), lt = br_plane_layout(Ccols, R);
  if (lp.rows_p > 0x7fffffffLL || lt.rows_p > 0x7fffffffLL) return hipErrorInvalidValue;
  const int64_t tiles_r = lp.rows_p >> 6, tiles_c = lt.rows_p >> 6;
  if (tiles_r * tiles_c > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(br::br_ingest_planes, dim3((int)(tiles_r * tiles_c), batch), dim3(256), 0, s, a, R, Ccols, beta1,
                     (int)lp.rows_p, (int)lp.k_p, lp.elems, (int)lt.rows_p, (int)lt.k_p, lt.elems, (int)tiles_c, want_lo);
  return hipGetLastError();
}

namespace {
// Compute units of the current device, rounded down to a multiple of the XCD count (cached per device).
int lowp_resident_workgroups() {
  static int cached[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
  if (cached[dev] == 0) {
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < NUM_XCD) return 0;
    cached[dev] = cus / NUM_XCD * NUM_XCD;
  }
  return cached[dev];
}

template <int EPI>
void launch_lowp(hipStream_t s, int nprod, int grid, const LowpKernArgs& k, const BrLowpBatch& b, bool f16) {
  if (f16)  // FP16 planes: the three-product split only (callers check)
    hipLaunchKernelGGL((br::br_gemm_bf16_mfma<3, EPI, true>), dim3(grid), dim3(512), 0, s, k, b);
  else if (nprod == 4)
    hipLaunchKernelGGL((br::br_gemm_bf16_mfma<4, EPI>), dim3(grid), dim3(512), 0, s, k, b);
  else if (nprod == 3)
    hipLaunchKernelGGL((br::br_gemm_bf16_mfma<3, EPI>), dim3(grid), dim3(512), 0, s, k, b);
  else
    hipLaunchKernelGGL((br::br_gemm_bf16_mfma<1, EPI>), dim3(grid), dim3(512), 0, s, k, b);
}
}  // namespace

hipError_t br_launch_gemm_lowp(hipStream_t s, const BrLowpArgs& a, const BrLowpBatch& b, const char** kernel_name) {
  if (kernel_name)
    *kernel_name = a.f16 ? "br_gemm_f16_mfma<3>"
                         : (a.nprod == 4) ? "br_gemm_bf16_mfma<4>" : (a.nprod == 3) ? "br_gemm_bf16_mfma<3>" : "br_gemm_bf16_mfma<1>";
  if (a.f16 && (a.nprod != 3 || a.epilogue == BR_EPI_ADAM || a.mirror)) return hipErrorInvalidValue;
  if (a.batch <= 0 || a.M <= 0 || a.N <= 0 || a.K <= 0) return hipSuccess;
  if (a.batch > BR_MAXB) return hipErrorInvalidValue;
  if (a.mirror && a.M != a.N) return hipErrorInvalidValue;
  if (a.epilogue != BR_EPI_F32 && (a.mirror || a.beta != 0.f)) return hipErrorInvalidValue;
  if (a.epilogue != BR_EPI_F32 && a.epilogue != BR_EPI_PLANES && a.epilogue != BR_EPI_ADAM) return hipErrorInvalidValue;
  const BrPlaneLayout pa = br_plane_layout(a.M, a.K), pb = br_plane_layout(a.N, a.K);
  if (pa.rows_p > 0x7fffffffLL || pb.rows_p > 0x7fffffffLL || pa.k_p > 0x7fffffffLL) return hipErrorInvalidValue;
  for (int i = 0; i < a.batch; ++i) {
    if ((reinterpret_cast<uintptr_t>(b.A[i]) & 15u) || (reinterpret_cast<uintptr_t>(b.B[i]) & 15u)) return hipErrorInvalidValue;
    if (a.epilogue != BR_EPI_F32 && (!b.shadow[i] || (reinterpret_cast<uintptr_t>(b.shadow[i]) & 15u))) return hipErrorInvalidValue;
    if (a.epilogue == BR_EPI_ADAM && (!b.S[i] || !b.Mrot[i])) return hipErrorInvalidValue;
  }
  LowpKernArgs k;
  k.M = a.M; k.N = a.N;
  k.Mp = (int)pa.rows_p; k.Np = (int)pb.rows_p; k.Kp = (int)pa.k_p;
  k.ldc = a.ldc;
  k.a_plane = pa.elems; k.b_plane = pb.elems;
  k.alpha = a.alpha; k.beta = a.beta;
  k.tiles_m = k.Mp / TILE;
  k.tiles_n = k.Np / TILE;
  k.mirror = a.mirror ? 1 : 0;
  k.total_tiles = k.mirror ? k.tiles_m * (k.tiles_m + 1) / 2 : k.tiles_m * k.tiles_n;
  const BrPlaneLayout po = br_plane_layout(a.N, a.M);  // planes of the transposed result
  k.out_kp = (int)po.k_p;
  k.out_plane = po.elems;
  k.out_lo = a.out_lo ? 1 : 0;
  k.adam = a.adam;
  k.adam_t = a.adam_transposed ? 1 : 0;
  // operand B, or the emitted planes, as a view into a larger plane set: same tiles, the set's strides
  k.b_stride = k.Np;
  if (a.b_stride_rows) {
    if (a.b_stride_rows < k.Np || (a.b_stride_rows % TILE) || a.b_plane_elems == 0) return hipErrorInvalidValue;
    k.b_stride = a.b_stride_rows;
    k.b_plane = a.b_plane_elems;
  }
  k.out_stride = k.Np;
  if (a.out_stride_rows) {
    if (a.out_stride_rows < k.Np || (a.out_stride_rows % TILE) || a.out_plane_elems == 0) return hipErrorInvalidValue;
    k.out_stride = a.out_stride_rows;
    k.out_plane = a.out_plane_elems;
  }
  k.skip = a.skip;
  k.health = a.health;
  k.out_scale = a.f16 ? a.out_scale : 1.f;
  k.emit_t = a.emit_transposed ? 1 : 0;
  if (k.emit_t) {
    if (a.epilogue != BR_EPI_F32 || a.mirror) return hipErrorInvalidValue;
    for (int i = 0; i < a.batch; ++i)
      if (!b.S[i] || (reinterpret_cast<uintptr_t>(b.S[i]) & 15u)) return hipErrorInvalidValue;
  }
  long long grid = (long long)k.total_tiles * a.batch;
  if (grid > 0x7fffffffLL - 65536) return hipErrorInvalidValue;  // the kernel adds its grid size to a tile position
  k.all_tiles = (int)grid;
  // one workgroup per compute unit (rounded down to whole XCDs) walks the tiles when there are more tiles than that
  const int resident = lowp_resident_workgroups();
  if (resident <= 0) return hipErrorInvalidDevice;
  if (grid > resident) grid = resident;
  if (a.epilogue == BR_EPI_ADAM) launch_lowp<EPI_ADAM>(s, a.nprod, (int)grid, k, b, false);
  else if (a.epilogue == BR_EPI_PLANES) launch_lowp<EPI_PLANES>(s, a.nprod, (int)grid, k, b, a.f16 != 0);
  else launch_lowp<EPI_F32>(s, a.nprod, (int)grid, k, b, a.f16 != 0);
  return hipGetLastError();
}
