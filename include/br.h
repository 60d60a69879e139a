/*
 * br.h -- C ABI of the basis-rotation optimizer step for AMD MI355X (gfx950).
 *
 * The library applies "Adam with basis rotation" (Algorithm 1 of the paper) with
 * the second-moment "Eigenbasis-Estimation" of Algorithm 2 to a list of weight
 * matrices, one pipeline stage's share, on one GPU.  Every step of the path runs in
 * hand-written HIP kernels; there is no CPU fallback.
 *
 * Per optimizer step t = 1, 2, ... the caller issues, in Algorithm 1's order:
 *
 *     br_accumulate_stats(ctx, grads, n)          first moment + Kronecker statistics
 *     if (t % freq == 0) br_refresh_basis(ctx)    Eigenbasis-Estimation (Power + QR)
 *     br_step(ctx, params, grads, n, lr_t)        rotate, Adam in the rotated basis, rotate back
 *
 * The refresh schedule, the learning-rate schedule and the ring of delayed
 * gradients (Appendix B: the gradient consumed at step t was evaluated at
 * W_{max(t-1-tau,0)}) are host policy outside the library: the library only ever
 * sees the pointer of the gradient to consume.
 *
 * Conventions
 *   layout     every matrix is row-major and contiguous: element (i, j) of an
 *              m x n matrix is at base[i*n + j]; m = rows.
 *   memory     all pointers named dev_* / params / grads entries are DEVICE pointers,
 *              16-byte aligned; arrays of pointers and descriptor arrays are HOST
 *              memory, read during the call only.
 *   ownership  the caller owns parameters, gradients and the single workspace
 *              buffer.  The library never allocates or frees device memory; it keeps
 *              pointers into the workspace until br_destroy.
 *   streams    all work is enqueued on the HIP stream given to br_init (a
 *              hipStream_t passed as void*, NULL = the null stream).  No call
 *              synchronises with the host except br_profile_end and br_check_health.
 *   graphs     br_accumulate_stats, br_refresh_basis, br_step, br_clip_gradients and
 *              br_delay_compensate only launch kernels (no allocation, no memset, no
 *              synchronisation), so they may be issued while the stream is being
 *              captured into a HIP graph.  A captured call freezes what the host
 *              folds into kernel arguments: the pointer arrays, lr, and with
 *              bias_correction the factors of the step number it was captured at; the
 *              host-side state (step counter, "statistics fresh", "basis changed")
 *              advances at capture time, not at replay.  Profiling must be off.
 *              Two consequences.  (1) With cache_rotated_moment, a step captured while the
 *              cached M~ is current contains "advance M~", one captured right after a refresh or
 *              br_notify_state_written contains "rebuild M~ from M": capture a plain-step
 *              graph after an eager (or captured) post-refresh step, and replay it only between
 *              refreshes.  (2) The first br_step of BF16 parameters initialises their FP32 master
 *              copies; br_step returns BR_ERR_STATE when asked to capture that step: run one
 *              step eagerly first.
 *   errors     every call returns a br_status; nothing throws or aborts.  Argument
 *              errors are detected on the host before anything is launched.  After
 *              BR_ERR_HIP the context is unusable (sticky).  br_last_error gives text.
 *   threads    one context, one calling thread at a time.
 *   determinism identical inputs give bit-identical outputs (no floating-point
 *              atomics anywhere).
 */
#ifndef BR_H_
#define BR_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct br_ctx br_ctx; /* opaque, host memory, owned by the library */

typedef enum {
  BR_OK = 0,
  BR_ERR_INVALID_ARG = 1, /* null pointer, bad enum, bad count                       */
  BR_ERR_SHAPE = 2,       /* non-positive or too large dimension, n_mats mismatch    */
  BR_ERR_DTYPE = 3,       /* unknown element type                                    */
  BR_ERR_STATE = 4,       /* calls out of order (e.g. br_step without its statistics) */
  BR_ERR_WORKSPACE = 5,   /* workspace too small or misaligned                       */
  BR_ERR_HIP = 6,         /* a HIP runtime call failed; sticky                       */
  BR_ERR_UNSUPPORTED = 7  /* a documented option that this build does not implement  */
} br_status;

typedef enum { BR_F32 = 0, BR_BF16 = 1 } br_dtype;

/* Rotation geometry G of Algorithm 2.  Unilateral rotates only the side of size
 * min(m, n) (Section 3.2; memory-overhead appendix); a square matrix keeps the
 * left factor, as Algorithm 2's unilateral branch does. */
typedef enum { BR_BILATERAL = 0, BR_UNILATERAL = 1 } br_geometry;

/* Approximation source S of Algorithm 2.  SECOND keeps L, R (its first branch); FIRST uses
 * M M^T and M^T M at refresh time and keeps no statistics buffers (its second branch). */
typedef enum { BR_SRC_SECOND = 0, BR_SRC_FIRST = 1 } br_source;

/* Input precision of the step's matrix-core contractions (statistics, rotations, rotate-back).
 * F32 issues FP32 MFMA.  BF16 rounds both operands to BF16 (parity bar 2e-2).  BF16X3 splits
 * each FP32 operand into hi + lo BF16 parts and adds the products hi*hi + hi*lo + lo*hi in FP32:
 * 16-bit mantissa inputs, same 1e-4 bar as F32, about a third of the matrix-core time.  What the
 * refresh's large products run in is chosen separately (br_refresh_math). */
typedef enum { BR_MATH_F32 = 0, BR_MATH_BF16 = 1, BR_MATH_BF16X3 = 2 } br_math;

/* Arithmetic of the refresh's large products (A^k Q of the Power calls and the products of the QR's block reflectors
 * of 256 and more columns: V T, V^T C and the update of C) for factors above order 512; panels, merges and everything on smaller factors are FP32 always.
 * F32: FP32 MFMA.  F16X3: each FP32 operand is scaled by a power of two and split into hi + lo FP16 parts
 * (22 mantissa bits; for entries below 2^-3 of the operand's scale an absolute 2^-25 of it), the products
 * hi*hi + hi*lo + lo*hi are accumulated in FP32 on the f16 matrix cores: bases agree with the float64 oracle to
 * 1e-6 like the FP32 refresh's, at three to four times its rate.  AUTO: F32 under BR_MATH_F32, F16X3 under the
 * BF16 math modes. */
typedef enum { BR_REFRESH_AUTO = 0, BR_REFRESH_F32 = 1, BR_REFRESH_F16X3 = 2 } br_refresh_math;

/* Which buffer br_get_state returns. */
typedef enum {
  BR_STATE_M = 0,      /* first moment, original space, m x n  (Algorithm 1)             */
  BR_STATE_S = 1,      /* second moment in the rotated basis, m x n  (Algorithm 1)       */
  BR_STATE_L = 2,      /* EMA of G G^T, m x m  (Algorithm 2)                             */
  BR_STATE_R = 3,      /* EMA of G^T G, n x n  (Algorithm 2)                             */
  BR_STATE_QL = 4,     /* left rotation U, m x m                                         */
  BR_STATE_QR = 5,     /* right rotation V, n x n                                        */
  BR_STATE_MASTER = 6, /* FP32 master weights of a BF16 parameter, m x n                 */
  BR_STATE_NORMS = 7,  /* 1 x 2: ||G~||_F^2 and ||X||_F^2 of the latest step             */
  BR_STATE_MROT = 8    /* cached rotated first moment M~, m x n (cache_rotated_moment)   */
} br_state_kind;

typedef struct {
  int64_t m, n;        /* rows, columns                                                  */
  int32_t param_dtype; /* br_dtype of the parameter buffer                               */
  int32_t grad_dtype;  /* br_dtype of the gradient buffer                                */
  int32_t rotate;      /* 0: plain Adam for this tensor (embeddings etc., App. D)        */
  int32_t reserved;    /* must be 0                                                      */
} br_matrix_desc;

typedef struct {
  float beta1, beta2;  /* Adam moment decay rates (Algorithm 1)                           */
  float eps;           /* inside the square root, as Algorithm 1's update has it          */
  float weight_decay;  /* decoupled: W <- W - lr*wd*W on the pre-step W; 0 = Algorithm 1 */
  float stat_beta;     /* decay of L, R; negative: use beta2 (Algorithm 2)               */
  int32_t geometry;    /* br_geometry                                                    */
  int32_t source;      /* br_source                                                      */
  int32_t power_iters; /* multiplications by L (R) before the single QR; paper: 1        */
  int32_t bias_correction;  /* 1: divide moments by (1 - beta^t); 0 = Algorithm 1        */
  int32_t eps_outside_sqrt; /* 1: m / (sqrt(s) + eps);            0 = Algorithm 1        */
  int32_t math;        /* br_math                                                        */
  int32_t compute_norms;    /* 1: keep ||G~||_F^2, ||X||_F^2 per matrix (BR_STATE_NORMS) */
  int32_t stats_on_refresh_only; /* 0: L, R are accumulated at every step (br_accumulate_stats).
                          1: Algorithm 2 as it is called from Algorithm 1: L and R are updated inside
                          Eigenbasis-Estimation, i.e. only from the gradient of a step whose
                          br_refresh_basis runs; br_accumulate_stats then only keeps the gradient
                          pointers (they must stay valid until br_step, as they must anyway) and
                          br_refresh_basis folds that gradient into L, R before its Power calls.  A
                          br_refresh_basis that is not preceded by this step's br_accumulate_stats
                          uses the statistics as they stand.                                    */
  int32_t refresh_math; /* br_refresh_math                                                  */
  int32_t cache_rotated_moment; /* 1: also keep M~ = Q_L^T M Q_R in the state and, while the
                          basis is unchanged, advance it by M~ <- beta1 M~ + (1-beta1) G~
                          (equal to rotating M, by linearity) instead of rotating M every
                          step; M~ is recomputed from M after every refresh.  Costs m*n
                          floats per rotated matrix, saves a quarter of the step's
                          contractions.  0: rotate M every step (Algorithm 1 as printed). */
} br_hparams;

/* One line per kernel symbol of a profiled region (see br_profile_begin). */
typedef struct {
  char kernel[64];   /* short name of the kernel family/instance                        */
  int64_t launches;  /* launches recorded                                               */
  double ms;         /* sum of HIP-event durations of those launches, milliseconds      */
  double flops;      /* algorithmic floating-point operations of those launches         */
  double bytes;      /* algorithmic HBM bytes of those launches                         */
} br_profile_entry;

/*
 * Size of the workspace br_init needs for these matrices: `state_bytes` holds the
 * optimizer state (M, S~, L, R, Q_L, Q_R, master weights: the FP32 buffers of the
 * memory-overhead appendix), `scratch_bytes` the temporaries of one step or one
 * refresh.  The workspace must be at least state_bytes + scratch_bytes long and
 * 256-byte aligned.  Host-only; launches nothing.
 */
br_status br_workspace_bytes(const br_matrix_desc* descs, int32_t n_mats, const br_hparams* hp,
                             size_t* state_bytes, size_t* scratch_bytes);

/*
 * Create a context over `n_mats` matrices.  Zero-fills the state, sets
 * Q_L = Q_R = I (so the steps before the first refresh are plain Adam) and t = 0.
 * `dev_workspace` is device memory of `workspace_bytes` bytes owned by the caller,
 * which must outlive the context.  `hip_stream` is a hipStream_t.
 */
br_status br_init(br_ctx** out, const br_matrix_desc* descs, int32_t n_mats, const br_hparams* hp,
                  void* dev_workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Consume this step's (delayed) gradients: M <- beta1 M + (1-beta1) G for every
 * matrix (Algorithm 1, first-moment update) and, for the second-order source,
 * L <- b L + (1-b) G G^T, R <- b R + (1-b) G^T G on the rotated sides
 * (Algorithm 2, updates of L and R), accumulated every step.
 * `grads`: host array of n_mats device pointers, matrix i being m_i x n_i of
 * grad_dtype.  Must be called exactly once before each br_step.
 */
br_status br_accumulate_stats(br_ctx* ctx, const void* const* grads, int32_t n_mats);

/*
 * Global-norm gradient clipping over all matrices of the context (the training recipe of the
 * experimental-details appendix clips at 1.0): norm = sqrt(sum of squares of every gradient
 * entry); every gradient is multiplied IN PLACE by min(1, max_norm / (norm + 1e-6)).  Call it
 * before br_accumulate_stats.  Nothing is copied to the host: the norm and the factor stay in
 * device memory (br_get_clip_result).  BF16 gradients are rescaled with round-to-nearest-even.
 * `grads`: host array of n_mats device pointers (writable).
 */
br_status br_clip_gradients(br_ctx* ctx, void* const* grads, int32_t n_mats, float max_norm);

/*
 * Delay Compensation of stale gradients (appendix "Experiments for Other Baselines", first-order
 * Taylor formula): for every matrix, IN PLACE,
 *     G <- G + lambda * G . G . (W_now - W_stale)
 * with W_stale the weights the gradient was taken at and W_now the current ones, both in the
 * matrix's param_dtype, G in its grad_dtype (BF16 results rounded to nearest even).  Call it
 * before br_clip_gradients / br_accumulate_stats.  All three arrays: n_mats device pointers.
 * lambda must lie in [0, 1].
 */
br_status br_delay_compensate(br_ctx* ctx, void* const* grads, const void* const* params_now,
                              const void* const* params_stale, int32_t n_mats, float lambda);

/* Device pointer to two floats: the global norm and the factor of the latest br_clip_gradients. */
br_status br_get_clip_result(br_ctx* ctx, void** dev_ptr);

/*
 * br_clip_gradients for callers that cannot allocate device memory and hold no context or
 * workspace: code that runs under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same kernels and arithmetic; the per-workgroup partial sums live in a device array
 * inside the library (1 MiB per GPU, held until the process ends), the result goes to the caller.
 * Calls no hipMalloc/hipFree or other allocating routine, and no memset; only launches kernels on
 * `hip_stream` (a hipStream_t; NULL = the null stream), whose device must be the current one.
 *   descs      host array of n_mats descriptors; m, n and grad_dtype are used
 *   grads      host array of n_mats device pointers (16-byte aligned), scaled IN PLACE by
 *              min(1, max_norm / (norm + 1e-6)), BF16 with round-to-nearest-even
 *   dev_result device pointer to two floats (8-byte aligned) owned by the caller: receives the
 *              global norm and the applied factor
 * At most BR_STATIC_CLIP_MAX_MATS matrices per call: more returns BR_ERR_WORKSPACE and launches
 * nothing.  Other argument errors as br_clip_gradients; the text is behind br_last_error(NULL).
 * All calls on one GPU share that GPU's array: calls that overlap on one GPU (two streams, two
 * threads) race; calls ordered on one stream, or separated by synchronisation, are safe.
 */
#define BR_STATIC_CLIP_MAX_MATS 4096
br_status br_clip_gradients_static(const br_matrix_desc* descs, void* const* grads, int32_t n_mats,
                                   float max_norm, void* dev_result, void* hip_stream);

/*
 * Eigenbasis-Estimation for every rotated side (Algorithm 2's Power calls and
 * Section 3.2): P <- A^power_iters Q with A = L or R (first-order source: M M^T,
 * M^T M), then Q <- the orthogonal factor of the Householder QR of P with
 * diag(R) >= 0.  Needs no gradients; uses the statistics as they stand.
 */
br_status br_refresh_basis(br_ctx* ctx);

/*
 * Algorithm 1 from the rotation to the parameter update, for every matrix: G~ = Q_L^T G Q_R, M~ = Q_L^T M Q_R,
 * S~ <- beta2 S~ + (1-beta2) G~.G~, X = M~ / sqrt(S~ + eps),
 * W <- W - lr * Q_L X Q_R^T - lr * weight_decay * W.  Increments t.
 * `params`: host array of device pointers to the weights (param_dtype), updated in
 * place; a BF16 parameter is the round-to-nearest-even image of its FP32 master
 * copy kept in the state (initialised from the parameter at the first step).
 * `grads`: the same gradients that were given to br_accumulate_stats.
 * Returns BR_ERR_STATE if br_accumulate_stats has not run since the last step.
 */
br_status br_step(br_ctx* ctx, void* const* params, const void* const* grads, int32_t n_mats,
                  float lr);

/*
 * Borrow a pointer to one state buffer of matrix `mat` (valid until br_destroy).
 * The caller may read or overwrite it between calls (tests inject a fixed basis;
 * a checkpoint is a copy of the state part of the workspace plus t); after writing
 * Q_L, Q_R or M call br_notify_state_written.
 * A buffer that does not exist for this matrix (e.g. L of an unrotated side)
 * returns BR_ERR_INVALID_ARG.
 */
br_status br_get_state(br_ctx* ctx, int32_t mat, int32_t which, void** dev_ptr, int64_t* rows,
                       int64_t* cols);

/*
 * Tell the library that the caller has overwritten Q_L, Q_R or M through pointers from
 * br_get_state: quantities derived from them (the cached M~) are rebuilt at the next step.
 * Not needed after restoring a whole-state checkpoint taken between steps.
 */
br_status br_notify_state_written(br_ctx* ctx);

/*
 * Health words: BR_HEALTH_WORDS (4) int32 counters in the state part of the workspace, zero from
 * br_init on, that kernels bump when something went wrong:
 *   [0]  a workgroup cluster of the QR panel kernel gave up its bounded wait for its partners (all
 *        workgroups of a panel launch must be resident at once; the launches are sized for a GPU that
 *        the library has to itself, and work on other streams can starve a cluster).  The bases of the
 *        affected matrices are left as they were BEFORE that refresh: nothing non-finite reaches
 *        the weights, the refresh is simply lost for them;
 *   [1]  a weight that is not finite was stored by br_step (counted per wavefront that saw one).
 * br_get_health returns the device pointer (no synchronisation; readable from a caller's own kernel
 * or copy).  br_check_health copies the words to the host, which SYNCHRONISES the stream (not
 * allowed while capturing), writes them to `counts` (4 values, may be NULL) and returns
 * BR_ERR_STATE with a text for br_last_error when any is non-zero, BR_OK otherwise.  The counters
 * are never reset by the library (they are part of a checkpoint); a caller may zero them.
 */
br_status br_get_health(br_ctx* ctx, void** dev_ptr);
br_status br_check_health(br_ctx* ctx, int32_t* counts);

/*
 * Bound of the QR panel clusters' wait, in polls of one exchanged value (default 2^22, about a
 * second; negative restores it).  0 makes every exchange give up at once without polling: the
 * failure path, forced from the host so that every kernel still ends normally (used by the tests).
 */
br_status br_set_qr_wait_limit(br_ctx* ctx, int64_t polls);

/* Number of completed steps t, and a way to set it when restoring a checkpoint. */
br_status br_get_step_count(const br_ctx* ctx, int64_t* t);
br_status br_set_step_count(br_ctx* ctx, int64_t t);

/*
 * Timing for the benchmark.  Between br_profile_begin and br_profile_end every kernel
 * launch is bracketed by HIP events on the context's stream.  br_profile_end
 * synchronises the stream, stops recording and writes one entry per kernel symbol (at
 * most `cap`) with launch counts, summed durations and algorithmic work.
 */
br_status br_profile_begin(br_ctx* ctx);
br_status br_profile_end(br_ctx* ctx, br_profile_entry* out, int32_t cap, int32_t* n_out);

/* Text of the latest error of this context ("" if none).  Never NULL. */
const char* br_last_error(const br_ctx* ctx);

/* Library version string, e.g. "br-hip 0.1 gfx950". */
const char* br_version(void);

/* Free the host-side context.  Device memory stays the caller's. */
void br_destroy(br_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* BR_H_ */
