// Internal launch interface between the host logic (br_api.hip) and the kernels.
// Everything here is device-pointer + size based; no torch types anywhere.
#ifndef BR_INTERNAL_H_
#define BR_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#define BR_MAXB 64  // matrices handled by one batched launch (pointers travel as kernel arguments)

// ---- batched GEMM on FP32 matrix cores -------------------------------------------------
// C_b = alpha * op(A_b) * op(B_b) + beta * C_b,  b = 0..batch-1, all row-major.
// op(A) is M x K: stored M x K (lda >= K) when transA == 0, K x M (lda >= M) when transA == 1.
// op(B) is K x N: stored K x N (ldb >= N) when transB == 0, N x K (ldb >= K) when transB == 1.
// shadow_b (optional): bfloat16 image of the final C_b (same ld as C), written with RNE.
// mirror: C is square and symmetric (A-op and B-op are transposes of each other): only tiles
//         on or below the diagonal are computed, each is also stored transposed.
struct BrGemmBatch {
  const float* A[BR_MAXB];
  const float* B[BR_MAXB];
  float* C[BR_MAXB];
  uint16_t* shadow[BR_MAXB];
  float* S[BR_MAXB];     // adam_epilogue: second moment in the rotated basis (row stride ldc), updated in place
  float* Mrot[BR_MAXB];  // adam_epilogue: rotated first moment (row stride ldc); rewritten when adam.update_mrot
};

struct BrAdamArgs {
  float beta1, beta2, eps;
  float c1, c2;     // bias-correction multipliers for the first/second moment (1 when disabled)
  int eps_outside;
  int compute_norms;
  int update_mrot;  // 1: M~ <- beta1 M~ + (1-beta1) G~ before it is used (cached rotated moment)
};

// Health words of a context (device memory, int32): counters that kernels bump when something went wrong.
enum { BR_HEALTH_QR_GAVE_UP = 0, BR_HEALTH_NONFINITE_WEIGHT = 1, BR_HEALTH_WORDS = 4 };

struct BrGemmArgs {
  int M, N, K;
  int lda, ldb, ldc;
  int transA, transB;
  float alpha, beta;
  int batch;
  int mirror;
  int qr_role = 0;             // 1: launch the split-K capable variant used inside the QR
  float* partial = nullptr;    // qr_role: scratch for split-K partial products (optional)
  size_t partial_floats = 0;   // its capacity in floats
  // adam_epilogue: the product alpha op(A) op(B) is a rotated gradient G~.  Instead of storing it, the
  // kernel advances Adam's moments in place (batch.S, batch.Mrot) and stores X = M~ / sqrt(S~ + eps) to C.
  // Needs transB == 0, no mirror, not qr_role; beta is ignored.
  int adam_epilogue = 0;
  BrAdamArgs adam = {};
  const int* skip = nullptr;   // device array, one int per matrix of the batch: non-zero = leave that matrix's C untouched
  int* health = nullptr;       // device health words: BR_HEALTH_NONFINITE_WEIGHT is bumped when a stored value is not finite
};

hipError_t br_launch_gemm(hipStream_t s, const BrGemmArgs& a, const BrGemmBatch& b, const char** kernel_name);

// ---- BF16 matrix-core contractions on pre-split operand planes ----------------------------
// A plane holds an R x K operand as BF16 in the order the contraction kernel wants its LDS tiles:
// rows padded to a multiple of BR_PLANE_ROW_PAD, k to a multiple of BR_PLANE_K_PAD (zeros),
// k-blocked by 16, and the two 16-byte halves of each 32-byte (row, k-block) run swapped on every
// other group of 8 rows:
//   element (row, k) at ((k / 16) * rows_p + row) * 16 + ((((k % 16) / 8) ^ ((row / 8) % 2)) * 8) + k % 8.
// The lo plane (when there is one) follows the hi plane at +elems elements.
#define BR_PLANE_ROW_PAD 256
#define BR_PLANE_K_PAD 64
struct BrPlaneLayout {
  int64_t rows_p, k_p;
  size_t elems;  // elements of one plane
};
inline BrPlaneLayout br_plane_layout(int64_t rows, int64_t k) {
  BrPlaneLayout l;
  l.rows_p = (rows + BR_PLANE_ROW_PAD - 1) / BR_PLANE_ROW_PAD * BR_PLANE_ROW_PAD;
  l.k_p = (k + BR_PLANE_K_PAD - 1) / BR_PLANE_K_PAD * BR_PLANE_K_PAD;
  l.elems = (size_t)l.rows_p * (size_t)l.k_p;
  return l;
}
// C_b = alpha * A_b B_b^T + beta * C_b with A_b the planes of an M x K operand and B_b those of an
// N x K operand (16-byte aligned).  nprod = 1 uses the hi planes only, nprod = 3 adds the two
// hi*lo cross terms, nprod = 4 also lo*lo.
// Epilogues.  BR_EPI_F32: C as above (shadow = optional BF16 image of C).  BR_EPI_PLANES: no FP32
// store; the TRANSPOSE of alpha A B^T is written to shadow as operand planes of
// br_plane_layout(N, M) (hi, plus lo when out_lo), padding included.  BR_EPI_ADAM: the product is a
// rotated gradient; S and Mrot (m x n FP32, row stride ldc) are advanced in place as
// br_adam_rotated does and X leaves as planes like BR_EPI_PLANES.  The last two need beta = 0
// and no mirroring.
enum { BR_EPI_F32 = 0, BR_EPI_PLANES = 1, BR_EPI_ADAM = 2 };
struct BrLowpBatch {
  const uint16_t* A[BR_MAXB];
  const uint16_t* B[BR_MAXB];
  float* C[BR_MAXB];
  uint16_t* shadow[BR_MAXB];
  float* S[BR_MAXB];
  float* Mrot[BR_MAXB];
};
struct BrLowpArgs {
  int M, N, K;
  int ldc;
  float alpha, beta;
  int batch, mirror, nprod;
  int epilogue = BR_EPI_F32;
  int out_lo = 0;
  BrAdamArgs adam = {};
  int adam_transposed = 0;  // BR_EPI_ADAM: the product is G~^T; moments (row stride ldc) are indexed [col][row]
  // Views into a larger plane set (sub-blocks that start at multiples of 256 rows and 64 k): the B
  // operand, and the emitted planes, then take that set's padded row count and hi-to-lo distance.
  int b_stride_rows = 0;
  size_t b_plane_elems = 0;
  int out_stride_rows = 0;
  size_t out_plane_elems = 0;
  // BR_EPI_F32 only: the transpose of the stored result also leaves as operand planes (hi, and lo when
  // out_lo) through the pointer carried in the batch's S slot.
  int emit_transposed = 0;
  const int* skip = nullptr;   // BR_EPI_F32: device array, one int per matrix: non-zero = store nothing for that matrix
  int* health = nullptr;       // BR_EPI_F32: BR_HEALTH_NONFINITE_WEIGHT is bumped when a stored value is not finite
  // FP16 planes (nprod = 3, BR_EPI_F32 or BR_EPI_PLANES): both operands are hi + lo FP16 planes of scaled values and
  // the products are f16 matrix instructions; alpha carries the inverse of the operands' scales; emitted planes
  // hold out_scale times the value.
  int f16 = 0;
  float out_scale = 1.f;
};
hipError_t br_launch_gemm_lowp(hipStream_t s, const BrLowpArgs& a, const BrLowpBatch& b, const char** kernel_name);
// hi = bf16(x), lo = bf16(x - hi) of an R x C FP32 matrix (row stride ld_src) into planes of
// br_plane_layout(R, C); transpose != 0 writes the planes of the transposed matrix,
// br_plane_layout(C, R).  The padding is written too (zeros).
// f16 != 0: FP16 planes of scale * x instead (hi = fp16, lo = fp16 of the remainder; values beyond the FP16 range are
// clamped).  With maxbits (one word per matrix, written by br_launch_absmax) the scale of matrix i is further
// multiplied by the power of two that brings its largest magnitude into [2^(target_exp-1), 2^target_exp).
hipError_t br_launch_split_planes(hipStream_t s, const float* const* src, uint16_t* const* dst, int batch, int R, int Ccols,
                                  int ld_src, int transpose, int want_lo, int f16 = 0, float scale = 1.f,
                                  const unsigned* maxbits = nullptr, int target_exp = 0);
// maxbits[i] = bit pattern of max |src[i]| (R x Ccols, row stride ld_src).  maxbits must be ZERO beforehand.
hipError_t br_launch_absmax(hipStream_t s, const float* const* src, int batch, int R, int Ccols, int ld_src, unsigned* maxbits);
// The first moment and both plane sets of the R x C gradients G[i] (contiguous) in one pass:
// M <- beta1 M + (1 - beta1) G, planes of G into P (br_plane_layout(R, C)), planes of G^T into PT.
hipError_t br_launch_ingest_planes(hipStream_t s, const float* const* G, float* const* M, uint16_t* const* P, uint16_t* const* PT,
                                   int batch, int R, int Ccols, float beta1, int want_lo);

// ---- elementwise ----------------------------------------------------------------------
struct BrPtrBatch {
  const void* in0[BR_MAXB];
  const void* in1[BR_MAXB];
  void* out0[BR_MAXB];
  void* out1[BR_MAXB];
};

// M <- beta1 M + (1-beta1) G.  in0 = G (f32 or bf16), out0 = M (f32), out1 = optional f32 copy of G.
hipError_t br_launch_ema(hipStream_t s, const BrPtrBatch& p, int batch, int64_t count, int grad_bf16,
                         float beta1);

struct BrAdamBatch {
  float* GX[BR_MAXB];     // G~ on entry, X = M~ / sqrt(S~ + eps) on exit
  float* S[BR_MAXB];      // second moment in the rotated basis, updated in place
  float* Mrot[BR_MAXB];   // rotated first moment; rewritten when update_mrot
  float* norms[BR_MAXB];  // per matrix [||G~||^2, ||X||^2] when compute_norms
};
// norm_partials: [batch][2][BR_NORM_BLOCKS] per-workgroup sums, reduced by a second kernel.
#define BR_NORM_BLOCKS 256
hipError_t br_launch_adam_rotated(hipStream_t s, const BrAdamBatch& p, int batch, int64_t count,
                                  const BrAdamArgs& a, float* norm_partials);

// Plain Adam for unrotated tensors, fully fused: in0 = G (f32/bf16), in1 = M (already updated),
// out0 = S, out1 = W master (f32); shadow = optional bf16 parameter image.
struct BrPlainArgs {
  float beta2, eps, c1, c2, lr, decay;  // decay = 1 - lr*wd
  int eps_outside, grad_bf16;
  int* health = nullptr;  // BR_HEALTH_NONFINITE_WEIGHT is bumped when a stored weight is not finite
};
hipError_t br_launch_adam_plain(hipStream_t s, const BrPtrBatch& p, uint16_t* const* shadow, int batch,
                                int64_t count, const BrPlainArgs& a);

// Global-norm clipping.  sumsq: per-(matrix, block) partial sums of squares into partials[slot0 + b*blocks + x];
// finalize: fixed-order sum of n_partials values -> result[0] = norm, result[1] = min(1, max_norm/(norm+1e-6));
// scale: G <- result[1] * G in place (no-op pass when the factor is 1).
#define BR_CLIP_BLOCKS 64
hipError_t br_launch_sumsq(hipStream_t s, const BrPtrBatch& p, int batch, int64_t count, int grad_bf16, float* partials,
                           int slot0);
hipError_t br_launch_clip_finalize(hipStream_t s, const float* partials, int n_partials, float max_norm, float* result);
hipError_t br_launch_scale_inplace(hipStream_t s, const BrPtrBatch& p, int batch, int64_t count, int grad_bf16,
                                   const float* result);
// G <- G + lambda G.G.(Wn - Ws): in0 = Wn, in1 = Ws (f32 or bf16 by param_bf16), out0 = G (f32 or bf16 by grad_bf16).
hipError_t br_launch_delay_compensate(hipStream_t s, const BrPtrBatch& p, int batch, int64_t count, int grad_bf16,
                                      int param_bf16, float lambda);
hipError_t br_launch_set_identity(hipStream_t s, float* const* mats, int batch, int n);
hipError_t br_launch_bf16_to_f32(hipStream_t s, const uint16_t* src, float* dst, int64_t count);

// ---- QR ---------------------------------------------------------------------------------
#define BR_QR_NB 32    // inner panel width of the blocked Householder factorisation
#define BR_QR_NBM 128  // middle block: four panels, merged into one block reflector inside LDS
#define BR_QR_NBT 512  // widest top block: middle blocks merged pairwise (128 -> 256 -> 512); one trailing-matrix update per top block

struct BrQrPanelBatch {
  float* A[BR_MAXB];     // top-left corner of the panel inside the matrix being factorised
  float* Vc[BR_MAXB];    // clean copy of the reflectors (unit diagonal, zeros above), row stride ldv
  float* T[BR_MAXB];     // BR_QR_NB x BR_QR_NB upper-triangular block-reflector factor
  float* diag[BR_MAXB];  // nb diagonal entries of R for this panel
};
// Panels taller than one workgroup's register capacity are factorised by a cluster of at least
// br_qr_panel_cluster(rows) workgroups per matrix (more, for speed, when a small batch of tall panels leaves
// compute units free), which exchange partial sums through xch (br_qr_panel_xch_floats(rows) floats per matrix,
// 8-byte aligned: room for the widest cluster the launcher may choose).  Every exchanged word carries the
// tag tag0 + step + 1 (step <= 32): xch must be ZERO before the first panel of a factorisation,
// and tag0 must differ by at least 64 between the panels that share it afterwards.
#define BR_QR_MAX_RESIDENT 192  // most workgroups of one panel launch (all of them must be on the chip at once)
// spin_limit: polls of one exchanged value before a workgroup gives up waiting for its cluster; 0 = give up
// without polling (every exchange fails: the host-forced test of the failure path).  A workgroup that gives
// up sets failed[matrix] (one int per matrix of the batch, device memory) and bumps
// health[BR_HEALTH_QR_GAVE_UP]; its results are garbage from then on and must not be used.
#define BR_QR_SPIN_LIMIT_DEFAULT (1u << 22)
struct BrQrClusterBatch {
  unsigned long long* xch[BR_MAXB];
  int* failed[BR_MAXB];
  int* health;
  unsigned tag0;
  unsigned spin_limit;
};
int br_qr_panel_cluster(int rows);
size_t br_qr_panel_xch_floats(int rows);
// Householder-factorise the rows x nb panel in place (reflectors below the diagonal, R on and
// above).
// Vc points at this panel's first row and first column inside a reflector block of row stride
// ldv; the pre_rows rows of that block above it are zero-filled in the panel's columns.
hipError_t br_launch_qr_panel(hipStream_t s, const BrQrPanelBatch& p, const BrQrClusterBatch& cb, int batch, int rows, int nb,
                              int lda, int ldv, int pre_rows);
hipError_t br_launch_zero_ints(hipStream_t s, int* const* ptrs, int batch, int n);
// C <- (I - V T^T V^T) C: a factorised panel's block reflector (V: rows x 32 clean reflectors, row
// stride ldv; T: 32 x 32) applied to the rows x ncols block C (ncols <= 96, row stride ldc) to its
// right.  partial: scratch of at least br_qr_panel_apply_floats(batch, rows) floats.
size_t br_qr_panel_apply_floats(int batch, int rows);
hipError_t br_launch_qr_panel_apply(hipStream_t s, const float* const* V, const float* const* T, float* const* C, int batch,
                                    int rows, int ncols, int ldv, int ldc, float* partial, size_t partial_floats);
// Copy the reflectors of an already factorised block of nb columns out into Vc (rows x width).
hipError_t br_launch_qr_extract_v(hipStream_t s, const BrQrPanelBatch& p, int batch, int rows, int nb, int lda,
                                  int width);
// Assemble the BR_QR_NBM-wide block-reflector factor from npanels inner factors and the Gram
// matrix of the block's reflectors.
hipError_t br_launch_qr_build_t(hipStream_t s, const float* const* G, const float* const* Tp, float* const* T, int batch,
                                int npanels);
// Diagonal blocks of a merged factor T (2w x 2w) from its nchild (1 or 2) child factors (consecutive
// w x w matrices); everything else zero.
hipError_t br_launch_qr_assemble_t(hipStream_t s, const float* const* Tc, float* const* T, int batch, int nchild, int w);
// Q = diag(sign(diag[j])) (zero counts as +).  skip (optional): device array, non-zero = leave that Q untouched.
hipError_t br_launch_qr_signed_identity(hipStream_t s, float* const* Q, const float* const* diag, int batch, int n,
                                        const int* skip);

#endif  // BR_INTERNAL_H_
