// Host logic of the C ABI declared in include/br.h: argument validation, workspace
// layout, grouping of same-shape matrices into batched launches, and the sequencing of
// Algorithm 1 / Algorithm 2 as kernel launches on the caller's stream.
#include "../../include/br.h"
#include "br_internal.h"

#include <algorithm>
#include <functional>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <map>
#include <new>
#include <string>
#include <vector>

namespace {

constexpr int kStepChunk = 32;     // matrices per batched step launch ([G|M] doubles it to BR_MAXB)
constexpr int kRefreshChunk = 64;   // factor matrices per batched refresh launch
constexpr int kLowpChunk = 16;      // matrices per batched step launch in the BF16 math modes: what sizes their scratch
constexpr int64_t kMaxDim = 1 << 24;
constexpr size_t kNormPartialBytes = (size_t)BR_MAXB * 2 * BR_NORM_BLOCKS * sizeof(float);
constexpr size_t kSplitKBytes = (size_t)64 << 20;  // partial products of the QR's split-K contractions
// Per refresh unit, behind its factors' scratch: one int per factor "its factorisation was abandoned" (first 256 bytes),
// then two words per factor for the largest magnitudes of A and of the current power-iteration operand (256 bytes each).
constexpr size_t kFailFlagBytes = 768;
static_assert(BR_MAXB * sizeof(int) <= 256, "one flag per matrix of a batched launch");

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct MatState {
  br_matrix_desc d;
  bool rot_l = false, rot_r = false;
  float *M = nullptr, *S = nullptr, *L = nullptr, *R = nullptr, *QL = nullptr, *QR = nullptr;
  float *master = nullptr, *norms = nullptr, *Mrot = nullptr;
  // BF16 math modes: operand planes of the bases in both orientations (state region, rebuilt when
  // the bases change) and of this step's gradient (scratch, valid from br_accumulate_stats to br_step)
  uint16_t *qlp = nullptr, *qlt = nullptr, *qrp = nullptr, *qrt = nullptr, *gp = nullptr, *gtp = nullptr;
  bool master_ready = false;
};

struct Group {  // matrices that can share a batched launch
  int64_t m, n;
  int pdt, gdt;
  bool rot_l, rot_r;
  std::vector<int> idx;
  size_t lowp_chunk = 0;  // matrices per batched step launch in the BF16 math modes
};

struct RefreshJob {
  int mat;
  bool left;
};

struct ProfRec {
  const char* name;
  size_t ev;  // index of the start event; the stop event follows it
  double flops, bytes;
};

// Factor matrices of one order that are refreshed by the same batched launches, one unit after
// the other on the caller's stream.  (Running units concurrently on several streams was tried and
// is slower: the 1024-thread panel workgroups are not placed while any contraction is running.)
struct RefreshUnit {
  int64_t k;
  std::vector<RefreshJob> jobs;
};

struct Layout {
  size_t state_bytes = 0, scratch_bytes = 0;
  size_t gplane_bytes = 0;  // gradient planes of all rotated matrices, ahead of the per-phase scratch
  std::vector<Group> groups;
  std::map<int64_t, std::vector<RefreshJob>> refresh;  // factor order -> jobs
  std::vector<RefreshUnit> units;
};

}  // namespace

struct br_ctx {
  std::vector<MatState> mats;
  br_hparams hp;
  Layout lay;
  hipStream_t stream = nullptr;
  char* scratch = nullptr;
  char* phase = nullptr;  // scratch shared by the phases of a step (after the norm partials and the gradient planes)
  bool qplanes_valid = false;  // BF16 math modes: the bases' operand planes match the bases
  float* clip_result = nullptr;  // 2 floats at the end of the state region
  int* health = nullptr;         // BR_HEALTH_WORDS counters behind them
  unsigned qr_spin_limit = BR_QR_SPIN_LIMIT_DEFAULT;
  int64_t t = 0;
  bool stats_fresh = false;
  int g32_group = -1;            // group whose FP32 images of BF16 gradients, written by br_accumulate_stats, are still in the
                                 // scratch at br_step: only when it is the context's ONLY rotated group and a single chunk
                                 // (groups and chunks take turns on the same scratch, in both calls); -1: none
  bool stats_pending = false;    // stats_on_refresh_only: this step's gradients have not been folded into L, R
  std::vector<const void*> pending_grads;
  bool mrot_valid = true;  // cached M~ equals Q_L^T M Q_R (true at t = 0: both are zero)
  bool dead = false;
  std::string err;
  bool prof_on = false;
  std::vector<hipEvent_t> events;
  size_t events_used = 0;
  std::vector<ProfRec> recs;
};

namespace {

thread_local std::string g_static_err;

br_status fail(br_ctx* c, br_status st, const std::string& msg) {
  if (c) c->err = msg;
  return st;
}

void sides(const br_matrix_desc& d, const br_hparams& hp, bool* l, bool* r) {
  *l = *r = false;
  if (!d.rotate) return;
  if (hp.geometry == BR_BILATERAL) {
    *l = *r = true;
  } else if (d.m <= d.n) {
    *l = true;  // smaller side; a square matrix keeps the left factor (Algorithm 2, unilateral branch)
  } else {
    *r = true;
  }
}

br_status validate(const br_matrix_desc* descs, int32_t n_mats, const br_hparams* hp, std::string* why) {
  if (!descs || !hp) { *why = "null descriptor or hyper-parameter pointer"; return BR_ERR_INVALID_ARG; }
  if (n_mats <= 0) { *why = "n_mats must be positive"; return BR_ERR_INVALID_ARG; }
  if (hp->geometry != BR_BILATERAL && hp->geometry != BR_UNILATERAL) { *why = "unknown geometry"; return BR_ERR_INVALID_ARG; }
  if (hp->source != BR_SRC_SECOND && hp->source != BR_SRC_FIRST) { *why = "unknown source"; return BR_ERR_INVALID_ARG; }
  if (hp->math != BR_MATH_F32 && hp->math != BR_MATH_BF16 && hp->math != BR_MATH_BF16X3) { *why = "unknown math mode"; return BR_ERR_INVALID_ARG; }
  if (hp->power_iters < 1 || hp->power_iters > 8) { *why = "power_iters must be in 1..8"; return BR_ERR_INVALID_ARG; }
  if (!(hp->beta1 >= 0.f && hp->beta1 < 1.f) || !(hp->beta2 >= 0.f && hp->beta2 < 1.f)) { *why = "beta1/beta2 must be in [0,1)"; return BR_ERR_INVALID_ARG; }
  if (!(hp->stat_beta < 1.f)) { *why = "stat_beta must be below 1 (negative selects beta2)"; return BR_ERR_INVALID_ARG; }
  if (!(hp->eps >= 0.f) || !(hp->weight_decay >= 0.f)) { *why = "eps and weight_decay must be non-negative"; return BR_ERR_INVALID_ARG; }
  if (hp->cache_rotated_moment != 0 && hp->cache_rotated_moment != 1) { *why = "cache_rotated_moment must be 0 or 1"; return BR_ERR_INVALID_ARG; }
  if (hp->refresh_math != BR_REFRESH_AUTO && hp->refresh_math != BR_REFRESH_F32 && hp->refresh_math != BR_REFRESH_F16X3) { *why = "unknown refresh_math"; return BR_ERR_INVALID_ARG; }
  if (hp->stats_on_refresh_only != 0 && hp->stats_on_refresh_only != 1) { *why = "stats_on_refresh_only must be 0 or 1"; return BR_ERR_INVALID_ARG; }
  for (int i = 0; i < n_mats; ++i) {
    const br_matrix_desc& d = descs[i];
    if (d.m <= 0 || d.n <= 0 || d.m > kMaxDim || d.n > kMaxDim) { *why = "matrix " + std::to_string(i) + ": dimensions must be in 1..2^24"; return BR_ERR_SHAPE; }
    if ((d.param_dtype != BR_F32 && d.param_dtype != BR_BF16) || (d.grad_dtype != BR_F32 && d.grad_dtype != BR_BF16)) { *why = "matrix " + std::to_string(i) + ": unknown dtype"; return BR_ERR_DTYPE; }
    if (d.reserved != 0) { *why = "br_matrix_desc.reserved must be 0"; return BR_ERR_INVALID_ARG; }
  }
  return BR_OK;
}

// Number of m x n FP32 scratch buffers one matrix of a group needs during a step.
// Bilateral: T1 = Q_L^T G (later Q_L X), G~ (later X), T2 = Q_L^T M, and M~ unless it is cached
// in the state.  Unilateral: G~ (later X), and M~ unless cached.  Plus an FP32 image of a BF16
// gradient (last slot).
int step_buffers(const Group& g, const br_hparams& hp) {
  int nb = 0;
  if (g.rot_l && g.rot_r) nb = hp.cache_rotated_moment ? 3 : 4;
  else if (g.rot_l || g.rot_r) nb = hp.cache_rotated_moment ? 1 : 2;
  if (g.gdt == BR_BF16 && (g.rot_l || g.rot_r)) nb += 1;
  return nb;
}

// Scratch of one matrix during a step in the BF16 math modes.  Slots, each large enough for an
// m x n FP32 matrix or for a pair of BF16 planes of it (either orientation, padded as
// br_plane_layout says).
enum { LS_T1 = 0, LS_T1P, LS_GX, LS_XP, LS_YP, LS_MP, LS_T2, LS_T2P, LS_MROT, LS_G32, LS_COUNT };
struct LowpLayout {
  size_t slot, per_mat;
};
LowpLayout lowp_layout(const Group& g) {
  LowpLayout l;
  const size_t a = br_plane_layout(g.m, g.n).elems, b = br_plane_layout(g.n, g.m).elems;
  l.slot = align256(4 * std::max(a, b));  // two BF16 planes, or (rows and k only grow by padding) an FP32 m x n matrix
  l.per_mat = LS_COUNT * l.slot;
  return l;
}
// bytes of the operand planes (hi, or hi + lo) of a rows x k matrix
inline size_t plane_bytes(int64_t rows, int64_t k, const br_hparams& hp) {
  return align256((hp.math == BR_MATH_BF16X3 ? 4 : 2) * br_plane_layout(rows, k).elems);
}

struct RefreshScratch {
  size_t P0, P1, gram, V, Y, W, T, Tp, Tl, G, X, Z, diag, xch, planesA, planesB, qrp, total;
};

// Doubling levels of the QR's block-reflector merges above the LDS-merged middle block: level l
// joins two factors of width BR_QR_NBM << l.  One level (top blocks of 256 columns) is what the
// FP32 refresh uses: a second one (512) makes its K = 512 trailing updates 15 % faster and was
// measured to give all of it back in the wider blocks' own merges and applies.  The split FP16
// refresh takes two: its top-block updates are short products (K = the block's width) whose
// epilogues move 12 bytes per entry of C, and 512-column blocks halve the number of passes over C.
constexpr int kQrMaxLevels = 2;
static_assert((BR_QR_NBM << kQrMaxLevels) == BR_QR_NBT, "widest top block = middle block doubled kQrMaxLevels times");
// Factors above this order run their large products (A Q, and the top blocks' updates of the QR) as split FP16
// products on the 16-bit matrix cores when the refresh math says so (BR_REFRESH_F16X3; by default in the BF16 math
// modes); smaller ones, and everything under BR_REFRESH_F32 (the default of BR_MATH_F32), stay on the FP32 matrix cores.
constexpr int64_t kSplitRefreshMinOrder = 512;
inline bool split_refresh(const br_hparams& hp, int64_t k) {
  const bool wanted = hp.refresh_math == BR_REFRESH_F16X3 || (hp.refresh_math == BR_REFRESH_AUTO && hp.math != BR_MATH_F32);
  return wanted && k > kSplitRefreshMinOrder;
}
inline int qr_levels(const br_hparams& hp, int64_t k) { return split_refresh(hp, k) ? 2 : 1; }
// Powers of two that centre the operands of the split FP16 products in the FP16 range (see qr_batch).
constexpr float kScaleV = 64.f, kScaleY = 64.f, kScaleC = 128.f, kScaleW = 64.f, kScaleT = 64.f;
// floats before level l's pair of child factors in the Tl scratch
inline size_t qr_level_offset(int l) {
  size_t off = 0;
  for (int i = 0; i < l; ++i) off += 2 * (size_t)(BR_QR_NBM << i) * (BR_QR_NBM << i);
  return off;
}

// bytes of the hi + lo planes of a k x BR_QR_NBT matrix in either orientation
inline size_t qr_plane_chunk(int64_t k) {
  return align256(4 * std::max(br_plane_layout(BR_QR_NBT, k).elems, br_plane_layout(k, BR_QR_NBT).elems));
}

// bytes of the hi + lo planes of a top block's triangular factor
inline size_t qr_factor_plane_bytes() { return align256(4 * br_plane_layout(BR_QR_NBT, BR_QR_NBT).elems); }

RefreshScratch refresh_scratch(int64_t k, const br_hparams& hp) {
  RefreshScratch r;
  size_t kk = align256((size_t)k * k * 4);
  size_t blocks = (size_t)((k + BR_QR_NBT - 1) / BR_QR_NBT);
  size_t off = 0;
  r.P0 = off; off += kk;
  r.P1 = off; if (hp.power_iters > 1) off += kk;
  r.gram = off; if (hp.source == BR_SRC_FIRST) off += kk;
  r.V = off; off += align256((size_t)k * BR_QR_NBT * 4);       // reflectors of one top block
  r.Y = off; off += align256((size_t)k * BR_QR_NBT * 4);       // V T or V T^T
  r.W = off; off += align256((size_t)k * BR_QR_NBT * 4);       // V^T C
  r.T = off; off += align256(blocks * BR_QR_NBT * BR_QR_NBT * 4);  // one factor per top block
  r.Tp = off; off += align256((size_t)(BR_QR_NBM / BR_QR_NB) * BR_QR_NB * BR_QR_NB * 4);  // panel factors of a middle block
  r.Tl = off; off += align256(qr_level_offset(kQrMaxLevels) * 4);  // child factors of every doubling level
  r.G = off; off += align256((size_t)BR_QR_NBM * BR_QR_NBM * 4);  // Gram matrix of a middle block's reflectors
  r.X = off; off += align256((size_t)(BR_QR_NBT / 2) * (BR_QR_NBT / 2) * 4);  // V_0^T V_1
  r.Z = off; off += align256((size_t)(BR_QR_NBT / 2) * (BR_QR_NBT / 2) * 4);  // T_0 (V_0^T V_1)
  r.diag = off; off += align256((size_t)k * 4);
  r.xch = off; off += align256(br_qr_panel_xch_floats((int)k) * 4);            // cluster exchange of one panel launch
  // split products: hi + lo planes of the statistics and of the transposed basis for the power iteration
  const size_t pl = split_refresh(hp, k) ? align256(4 * br_plane_layout(k, k).elems) : 0;
  r.planesA = off; off += pl;
  r.planesB = off; off += pl;
  // ... and of V^T, V T, (V^T C)^T, V and T for the top blocks' updates of the QR
  r.qrp = off; if (split_refresh(hp, k)) off += 4 * qr_plane_chunk(k) + qr_factor_plane_bytes();
  r.total = off;
  return r;
}

void plan(const br_matrix_desc* descs, int32_t n_mats, const br_hparams& hp, Layout* lay) {
  lay->groups.clear();
  lay->refresh.clear();
  lay->gplane_bytes = 0;
  size_t state = 0, scratch = 0;
  for (int i = 0; i < n_mats; ++i) {
    const br_matrix_desc& d = descs[i];
    bool l, r;
    sides(d, hp, &l, &r);
    size_t mn = align256((size_t)d.m * d.n * 4);
    state += 2 * mn;  // M, S
    if (hp.source == BR_SRC_SECOND) {
      if (l) state += align256((size_t)d.m * d.m * 4);
      if (r) state += align256((size_t)d.n * d.n * 4);
    }
    if (l) state += align256((size_t)d.m * d.m * 4);
    if (r) state += align256((size_t)d.n * d.n * 4);
    if (d.param_dtype == BR_BF16) state += mn;
    if ((l || r) && hp.cache_rotated_moment) state += mn;
    if (hp.math != BR_MATH_F32) {
      if (l) state += 2 * plane_bytes(d.m, d.m, hp);
      if (r) state += 2 * plane_bytes(d.n, d.n, hp);
      if (l || r) lay->gplane_bytes += plane_bytes(d.m, d.n, hp) + plane_bytes(d.n, d.m, hp);
    }
    state += 256;  // norms
    Group* g = nullptr;
    for (auto& c : lay->groups)
      if (c.m == d.m && c.n == d.n && c.pdt == d.param_dtype && c.gdt == d.grad_dtype && c.rot_l == l && c.rot_r == r) g = &c;
    if (!g) {
      lay->groups.push_back(Group{d.m, d.n, d.param_dtype, d.grad_dtype, l, r, {}});
      g = &lay->groups.back();
    }
    g->idx.push_back(i);
    if (l) lay->refresh[d.m].push_back(RefreshJob{i, true});
    if (r) lay->refresh[d.n].push_back(RefreshJob{i, false});
  }
  size_t lowp_need = 0;
  for (auto& g : lay->groups) {
    size_t chunk = std::min<size_t>(g.idx.size(), kStepChunk);
    size_t need = chunk * step_buffers(g, hp) * align256((size_t)g.m * g.n * 4);
    if (hp.math != BR_MATH_F32 && (g.rot_l || g.rot_r)) {
      need = std::min<size_t>(g.idx.size(), kLowpChunk) * lowp_layout(g).per_mat;
      lowp_need = std::max(lowp_need, need);
    }
    scratch = std::max(scratch, need);
  }
  // Groups of small matrices take more of them per launch, within the scratch the largest group needs
  // anyway: a launch of 1600 tiles is 6.25 rounds on 256 compute units and pays for 7, one of 3200
  // for 13 instead of 12.5 (8 % measured).
  for (auto& g : lay->groups) {
    if (hp.math == BR_MATH_F32 || !(g.rot_l || g.rot_r)) continue;
    const size_t fit = lowp_need / lowp_layout(g).per_mat;
    g.lowp_chunk = std::min<size_t>(std::min<size_t>(g.idx.size(), kStepChunk), std::max<size_t>(fit, 1));
  }
  // Refresh units: every order's jobs in chunks of at most kRefreshChunk, evenly sized.
  lay->units.clear();
  size_t refresh_bytes = 0;
  for (auto& kv : lay->refresh) {
    const size_t n = kv.second.size();
    const size_t chunks = (n + kRefreshChunk - 1) / kRefreshChunk;
    for (size_t ci = 0; ci < chunks; ++ci) {
      const size_t lo = n * ci / chunks, hi = n * (ci + 1) / chunks;
      RefreshUnit u;
      u.k = kv.first;
      u.jobs.assign(kv.second.begin() + lo, kv.second.begin() + hi);
      refresh_bytes = std::max(refresh_bytes, align256(u.jobs.size() * refresh_scratch(u.k, hp).total + kFailFlagBytes + kSplitKBytes));
      lay->units.push_back(u);
    }
  }
  scratch = std::max(scratch, refresh_bytes);
  state += 256;  // global gradient norm and clipping factor
  state += 256;  // health words
  lay->state_bytes = state;
  lay->scratch_bytes = scratch + kNormPartialBytes + lay->gplane_bytes;
}

// ---- launch bookkeeping ------------------------------------------------------------------
bool hip_ok(br_ctx* c, hipError_t e, const char* what) {
  if (e == hipSuccess) return true;
  c->dead = true;
  c->err = std::string(what) + ": " + hipGetErrorString(e);
  return false;
}

struct Timed {  // brackets one launch (or a region) with events while profiling is on
  br_ctx* c;
  bool live = false;
  Timed(br_ctx* ctx, const char* name, double flops, double bytes) : c(ctx) {
    if (!c->prof_on) return;
    if (c->events_used + 2 > c->events.size()) {
      size_t want = c->events.size() + 512;
      while (c->events.size() < want) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) return;
        c->events.push_back(e);
      }
    }
    c->recs.push_back(ProfRec{name, c->events_used, flops, bytes});
    live = (hipEventRecord(c->events[c->events_used], c->stream) == hipSuccess);
    if (!live) c->recs.pop_back();
  }
  ~Timed() {
    if (!live) return;
    if (hipEventRecord(c->events[c->events_used + 1], c->stream) != hipSuccess) c->recs.pop_back();
    else c->events_used += 2;
  }
};

// step = true: one of the optimizer step's contractions (timed individually while profiling).
// step = false: a contraction inside the QR (split-K capable variant, timed as part of the region).
bool gemm(br_ctx* c, BrGemmArgs a, const BrGemmBatch& b, bool step = true, float* partial = nullptr,
          hipStream_t qr_stream = nullptr) {
  if (!step) {
    a.qr_role = 1;
    a.partial = partial;
    a.partial_floats = partial ? kSplitKBytes / sizeof(float) : 0;
    return hip_ok(c, br_launch_gemm(qr_stream ? qr_stream : c->stream, a, b, nullptr), "gemm launch");
  }
  if (c->prof_on) {
    const char* name = nullptr;
    double flops = 2.0 * a.M * a.N * (double)a.K * a.batch;
    if (a.mirror) flops *= 0.5 * (1.0 + 1.0 / std::max(1, (a.M + 127) / 128));
    BrGemmArgs probe{0, 0, 0, 0, 0, 0, a.transA, a.transB, 0, 0, 0, 0};
    probe.adam_epilogue = a.adam_epilogue;
    probe.mirror = a.mirror;
    (void)br_launch_gemm(nullptr, probe, b, &name);
    Timed tm(c, name, flops, 0.0);
    return hip_ok(c, br_launch_gemm(c->stream, a, b, nullptr), "gemm launch");
  }
  return hip_ok(c, br_launch_gemm(c->stream, a, b, nullptr), "gemm launch");
}

inline float* scratch_buf(br_ctx* c, size_t per_mat_bufs, size_t bytes_each, int mat_in_chunk, int which) {
  return reinterpret_cast<float*>(c->phase + ((size_t)mat_in_chunk * per_mat_bufs + which) * bytes_each);
}


// ---- BF16 math modes: operand planes and contractions -------------------------------------------
struct LowpCtx {
  br_ctx* c;
  const Group* g;
  LowpLayout lay;
  int B;
  int nprod;
  char* base;  // scratch of this chunk
  bool quiet = false;  // no per-launch profile records (launches inside a region that is timed as a whole)
  uint16_t* slot16(int i, int s) const { return reinterpret_cast<uint16_t*>(base + (size_t)i * lay.per_mat + (size_t)s * lay.slot); }
  float* slot32(int i, int s) const { return reinterpret_cast<float*>(base + (size_t)i * lay.per_mat + (size_t)s * lay.slot); }
};

// planes of the R x C matrices src[i] (row stride ld, C when 0), optionally transposed
bool lowp_split(const LowpCtx& x, const float* const* src, int R, int Ccols, bool transpose, uint16_t* const* dst, int ld = 0) {
  if (ld == 0) ld = Ccols;
  if (x.quiet)
    return hip_ok(x.c, br_launch_split_planes(x.c->stream, src, dst, x.B, R, Ccols, ld, transpose ? 1 : 0, x.nprod == 3 ? 1 : 0),
                  "plane split launch");
  Timed tm(x.c, "br_split_planes", 0.0, (double)R * Ccols * x.B * (4.0 + (x.nprod == 3 ? 4.0 : 2.0)));
  return hip_ok(x.c, br_launch_split_planes(x.c->stream, src, dst, x.B, R, Ccols, ld, transpose ? 1 : 0,
                                            x.nprod == 3 ? 1 : 0), "plane split launch");
}

// hi + lo FP16 planes of scale * src[i] (the refresh's split products).  With maxbits the scale of matrix i is
// multiplied by the power of two that brings its largest magnitude into [2^(target_exp-1), 2^target_exp).
bool f16_split(const LowpCtx& x, const float* const* src, int R, int Ccols, bool transpose, uint16_t* const* dst, int ld,
               float scale, const unsigned* maxbits = nullptr, int target_exp = 0) {
  if (ld == 0) ld = Ccols;
  return hip_ok(x.c, br_launch_split_planes(x.c->stream, src, dst, x.B, R, Ccols, ld, transpose ? 1 : 0, 1, 1, scale, maxbits,
                                            target_exp), "plane split launch");
}

// C_i = alpha A_i B_i^T + beta C_i with A_i: M x K planes, B_i: N x K planes.  With an epilogue other
// than BR_EPI_F32 the transposed result leaves as planes in out16 (see BrLowpArgs).
bool lowp_gemm(const LowpCtx& x, uint16_t* const* A, int M, uint16_t* const* Bp, int N, int K, float* const* C, int ldc,
               float alpha, float beta, uint16_t* const* out16, bool mirror, int nprod = 0, int epilogue = BR_EPI_F32,
               const BrAdamArgs* adam = nullptr, float* const* S = nullptr, float* const* Mrot = nullptr,
               bool adam_transposed = false, int* health = nullptr) {
  if (nprod == 0) nprod = x.nprod;
  BrLowpBatch b;
  std::memset(&b, 0, sizeof(b));
  for (int i = 0; i < x.B; ++i) {
    b.A[i] = A[i];
    b.B[i] = Bp[i];
    b.C[i] = C ? C[i] : nullptr;
    b.shadow[i] = out16 ? out16[i] : nullptr;
    b.S[i] = S ? S[i] : nullptr;
    b.Mrot[i] = Mrot ? Mrot[i] : nullptr;
  }
  BrLowpArgs a{M, N, K, ldc, alpha, beta, x.B, mirror ? 1 : 0, nprod};
  a.epilogue = epilogue;
  a.out_lo = (x.nprod == 3) ? 1 : 0;
  if (adam) a.adam = *adam;
  a.adam_transposed = adam_transposed ? 1 : 0;
  a.health = health;
  double flops = 2.0 * M * N * (double)K * x.B;
  if (mirror) flops *= 0.5 * (1.0 + 1.0 / std::max(1, (M + 255) / 256));
  if (x.quiet) return hip_ok(x.c, br_launch_gemm_lowp(x.c->stream, a, b, nullptr), "bf16 gemm launch");
  const char* name = nullptr;
  (void)br_launch_gemm_lowp(nullptr, BrLowpArgs{0, 0, 0, 0, 0.f, 0.f, 0, 0, nprod}, b, &name);
  Timed tm(x.c, name, flops, 0.0);
  return hip_ok(x.c, br_launch_gemm_lowp(x.c->stream, a, b, nullptr), "bf16 gemm launch");
}

// Operand planes of this step's gradients in both orientations (kept until br_step), and a2 in the
// BF16 modes for one chunk: L <- b L + (1-b) G G^T, R <- b R + (1-b) G^T G.
bool lowp_stats(const LowpCtx& x, const float* const* G32, size_t off, bool with_stats, bool planes_ready = false) {
  const Group& g = *x.g;
  const br_hparams& hp = x.c->hp;
  const int m = (int)g.m, n = (int)g.n;
  uint16_t *gp[BR_MAXB], *gtp[BR_MAXB];
  float* out[BR_MAXB];
  for (int i = 0; i < x.B; ++i) {
    gp[i] = x.c->mats[g.idx[off + i]].gp;
    gtp[i] = x.c->mats[g.idx[off + i]].gtp;
  }
  if (!planes_ready && (!lowp_split(x, G32, m, n, false, gp) || !lowp_split(x, G32, m, n, true, gtp))) return false;
  if (!with_stats) return true;
  if (g.rot_l) {
    for (int i = 0; i < x.B; ++i) out[i] = x.c->mats[g.idx[off + i]].L;
    if (!lowp_gemm(x, gp, m, gp, m, n, out, m, 1.0f - hp.stat_beta, hp.stat_beta, nullptr, true, x.nprod == 3 ? 4 : 1)) return false;
  }
  if (g.rot_r) {
    for (int i = 0; i < x.B; ++i) out[i] = x.c->mats[g.idx[off + i]].R;
    if (!lowp_gemm(x, gtp, n, gtp, n, m, out, n, 1.0f - hp.stat_beta, hp.stat_beta, nullptr, true, x.nprod == 3 ? 4 : 1)) return false;
  }
  return true;
}

// a4-a6 in the BF16 modes for one chunk.  Every contraction is A B^T on planes with k contiguous.
// Fused form (no norms requested): no intermediate exists in FP32.
// Each contraction hands its result to the next one as operand planes straight from its
// accumulators, which emit the TRANSPOSE of what they hold; so the chain alternates between a
// product and its transpose:
//   (Q_L^T G)^T = G^T Q_L          -> planes of T = Q_L^T G
//   G~ = T Q_R, Adam in the epilogue (moments advanced in place)  -> planes of X^T
//   (Q_L X)^T = X^T Q_L^T          -> planes of Y = Q_L X
//   W <- decay W - lr Y Q_R^T      (FP32 epilogue)
// Left factor only: X^T from Q_L^T G directly, then W <- decay W - lr Q_L X.  Right factor only: the
// first contraction is taken transposed, G~^T = Q_R^T G^T, so that X itself leaves as planes for
// W <- decay W - lr X Q_R^T.
// Otherwise every product is stored in FP32 and split again (rotate_in / rotate back below).
bool lowp_step(const LowpCtx& x, size_t off, const float* const* G32, float* const* Wp, uint16_t* const* shadow,
               float* const* Mt, bool advance, const BrAdamArgs& aa, float lr, float decay, float* partials) {
  br_ctx* c = x.c;
  const Group& g = *x.g;
  const int m = (int)g.m, n = (int)g.n, B = x.B;
  const int64_t count = g.m * g.n;
  uint16_t *QLp[BR_MAXB], *QLt[BR_MAXB], *QRp[BR_MAXB], *QRt[BR_MAXB], *GP[BR_MAXB], *GTP[BR_MAXB];
  uint16_t *P0[BR_MAXB], *P1[BR_MAXB];
  const float* src[BR_MAXB];
  float* dst[BR_MAXB];
  float* GX[BR_MAXB];
  float* Sp[BR_MAXB];
  for (int i = 0; i < B; ++i) {
    const MatState& ms = c->mats[g.idx[off + i]];
    QLp[i] = ms.qlp; QLt[i] = ms.qlt; QRp[i] = ms.qrp; QRt[i] = ms.qrt;
    GP[i] = ms.gp; GTP[i] = ms.gtp;
    GX[i] = x.slot32(i, LS_GX);
    Sp[i] = ms.S;
  }
  if (!c->qplanes_valid) {  // the bases changed (or this is the first step): rebuild their operand planes
    if (g.rot_l) {
      for (int i = 0; i < B; ++i) src[i] = c->mats[g.idx[off + i]].QL;
      if (!lowp_split(x, src, m, m, false, QLp) || !lowp_split(x, src, m, m, true, QLt)) return false;
    }
    if (g.rot_r) {
      for (int i = 0; i < B; ++i) src[i] = c->mats[g.idx[off + i]].QR;
      if (!lowp_split(x, src, n, n, false, QRp) || !lowp_split(x, src, n, n, true, QRt)) return false;
    }
  }
  const bool bilateral = g.rot_l && g.rot_r;
  if (!aa.compute_norms && g.rot_l) {
    uint16_t *T1P[BR_MAXB], *XTP[BR_MAXB], *YP[BR_MAXB];
    for (int i = 0; i < B; ++i) { T1P[i] = x.slot16(i, LS_T1P); XTP[i] = x.slot16(i, LS_XP); YP[i] = x.slot16(i, LS_YP); }
    if (!advance) {  // M~ = Q_L^T M Q_R from the first moment itself
      for (int i = 0; i < B; ++i) { src[i] = c->mats[g.idx[off + i]].M; P0[i] = x.slot16(i, LS_MP); P1[i] = x.slot16(i, LS_T2P); }
      if (!lowp_split(x, src, m, n, true, P0)) return false;  // planes of M^T
      if (bilateral) {
        if (!lowp_gemm(x, P0, n, QLt, m, m, nullptr, 0, 1.f, 0.f, P1, false, 0, BR_EPI_PLANES)) return false;  // planes of Q_L^T M
        if (!lowp_gemm(x, P1, m, QRt, n, n, Mt, n, 1.f, 0.f, nullptr, false)) return false;                   // M~
      } else {
        if (!lowp_gemm(x, QLt, m, P0, n, m, Mt, n, 1.f, 0.f, nullptr, false)) return false;                   // M~ = Q_L^T M
      }
    }
    if (bilateral) {
      if (!lowp_gemm(x, GTP, n, QLt, m, m, nullptr, 0, 1.f, 0.f, T1P, false, 0, BR_EPI_PLANES)) return false;            // T
      if (!lowp_gemm(x, T1P, m, QRt, n, n, nullptr, n, 1.f, 0.f, XTP, false, 0, BR_EPI_ADAM, &aa, Sp, Mt)) return false;  // X^T
      if (!lowp_gemm(x, XTP, n, QLp, m, m, nullptr, 0, 1.f, 0.f, YP, false, 0, BR_EPI_PLANES)) return false;             // Y
      return lowp_gemm(x, YP, m, QRp, n, n, Wp, n, -lr, decay, shadow, false, 0, BR_EPI_F32, nullptr, nullptr, nullptr, false, c->health);                                          // W
    }
    if (!lowp_gemm(x, QLt, m, GTP, n, m, nullptr, n, 1.f, 0.f, XTP, false, 0, BR_EPI_ADAM, &aa, Sp, Mt)) return false;    // X^T
    return lowp_gemm(x, QLp, m, XTP, n, m, Wp, n, -lr, decay, shadow, false, 0, BR_EPI_F32, nullptr, nullptr, nullptr, false, c->health);                                            // W -= lr Q_L X
  }
  if (!aa.compute_norms && g.rot_r) {  // right factor only, fused: G~^T = Q_R^T G^T carries Adam, X leaves as planes
    uint16_t* XP[BR_MAXB];
    for (int i = 0; i < B; ++i) XP[i] = x.slot16(i, LS_XP);
    if (!advance) {  // M~ = M Q_R from the first moment itself
      for (int i = 0; i < B; ++i) { src[i] = c->mats[g.idx[off + i]].M; P0[i] = x.slot16(i, LS_MP); }
      if (!lowp_split(x, src, m, n, false, P0)) return false;
      if (!lowp_gemm(x, P0, m, QRt, n, n, Mt, n, 1.f, 0.f, nullptr, false)) return false;
    }
    if (!lowp_gemm(x, QRt, n, GP, m, n, nullptr, n, 1.f, 0.f, XP, false, 0, BR_EPI_ADAM, &aa, Sp, Mt, true)) return false;  // X
    return lowp_gemm(x, XP, m, QRp, n, n, Wp, n, -lr, decay, shadow, false, 0, BR_EPI_F32, nullptr, nullptr, nullptr, false, c->health);                                              // W -= lr X Q_R^T
  }
  // rotate one m x n matrix into `out`; its planes are given (gradient) or made here from `in` (first moment)
  auto rotate_in = [&](const float* const* in, uint16_t* const* in_p, uint16_t* const* in_tp, float* const* out, int s_t,
                       int s_tp, int s_plane) -> bool {
    uint16_t* made[BR_MAXB];
    for (int i = 0; i < B; ++i) made[i] = x.slot16(i, s_plane);
    if (g.rot_l) {  // needs the planes of in^T ([n][m])
      if (!in_tp) {
        if (!lowp_split(x, in, m, n, true, made)) return false;
        in_tp = made;
      }
      if (!bilateral) return lowp_gemm(x, QLt, m, in_tp, n, m, out, n, 1.f, 0.f, nullptr, false);  // out = Q_L^T in
      for (int i = 0; i < B; ++i) dst[i] = x.slot32(i, s_t);
      if (!lowp_gemm(x, QLt, m, in_tp, n, m, dst, n, 1.f, 0.f, nullptr, false)) return false;       // T = Q_L^T in
      for (int i = 0; i < B; ++i) { P1[i] = x.slot16(i, s_tp); src[i] = x.slot32(i, s_t); }
      if (!lowp_split(x, src, m, n, false, P1)) return false;                                       // T planes [m][n]
      return lowp_gemm(x, P1, m, QRt, n, n, out, n, 1.f, 0.f, nullptr, false);                      // out = T Q_R
    }
    if (!in_p) {
      if (!lowp_split(x, in, m, n, false, made)) return false;
      in_p = made;
    }
    return lowp_gemm(x, in_p, m, QRt, n, n, out, n, 1.f, 0.f, nullptr, false);                      // out = in Q_R
  };
  if (!rotate_in(G32, GP, GTP, GX, LS_T1, LS_T1P, LS_MP)) return false;
  if (!advance) {
    const float* msrc[BR_MAXB];
    for (int i = 0; i < B; ++i) msrc[i] = c->mats[g.idx[off + i]].M;
    if (!rotate_in(msrc, nullptr, nullptr, Mt, LS_T2, LS_T2P, LS_MP)) return false;
  }
  {
    BrAdamBatch ab;
    std::memset(&ab, 0, sizeof(ab));
    for (int i = 0; i < B; ++i) {
      const MatState& ms = c->mats[g.idx[off + i]];
      ab.GX[i] = GX[i];
      ab.S[i] = ms.S;
      ab.Mrot[i] = Mt[i];
      ab.norms[i] = ms.norms;
    }
    Timed tm(c, "br_adam_rotated", 8.0 * count * B, (advance ? 24.0 : 20.0) * count * B);
    if (!hip_ok(c, br_launch_adam_rotated(c->stream, ab, B, count, aa, partials), "rotated adam launch")) return false;
  }
  // rotate back and apply: W <- decay W - lr Q_L X Q_R^T
  for (int i = 0; i < B; ++i) { src[i] = GX[i]; P0[i] = x.slot16(i, LS_XP); }
  if (bilateral) {
    if (!lowp_split(x, src, m, n, true, P0)) return false;                                    // X^T planes [n][m]
    for (int i = 0; i < B; ++i) dst[i] = x.slot32(i, LS_T1);
    if (!lowp_gemm(x, QLp, m, P0, n, m, dst, n, 1.f, 0.f, nullptr, false)) return false;       // Y = Q_L X
    for (int i = 0; i < B; ++i) { src[i] = x.slot32(i, LS_T1); P1[i] = x.slot16(i, LS_T1P); }
    if (!lowp_split(x, src, m, n, false, P1)) return false;
    return lowp_gemm(x, P1, m, QRp, n, n, Wp, n, -lr, decay, shadow, false, 0, BR_EPI_F32, nullptr, nullptr, nullptr, false, c->health);                  // W -= lr Y Q_R^T
  }
  if (g.rot_l) {
    if (!lowp_split(x, src, m, n, true, P0)) return false;
    return lowp_gemm(x, QLp, m, P0, n, m, Wp, n, -lr, decay, shadow, false, 0, BR_EPI_F32, nullptr, nullptr, nullptr, false, c->health);                  // W -= lr Q_L X
  }
  if (!lowp_split(x, src, m, n, false, P0)) return false;
  return lowp_gemm(x, P0, m, QRp, n, n, Wp, n, -lr, decay, shadow, false, 0, BR_EPI_F32, nullptr, nullptr, nullptr, false, c->health);                    // W -= lr X Q_R^T
}

}  // namespace

void br_set_static_error(const std::string& msg) { g_static_err = msg; }

// =========================================================================================
extern "C" {

const char* br_version(void) { return "br-hip 0.1 gfx950"; }

const char* br_last_error(const br_ctx* ctx) { return ctx ? ctx->err.c_str() : g_static_err.c_str(); }

br_status br_workspace_bytes(const br_matrix_desc* descs, int32_t n_mats, const br_hparams* hp, size_t* state_bytes,
                             size_t* scratch_bytes) {
  std::string why;
  br_status st = validate(descs, n_mats, hp, &why);
  if (st != BR_OK) { g_static_err = why; return st; }
  if (!state_bytes || !scratch_bytes) { g_static_err = "null output pointer"; return BR_ERR_INVALID_ARG; }
  Layout lay;
  plan(descs, n_mats, *hp, &lay);
  *state_bytes = lay.state_bytes;
  *scratch_bytes = lay.scratch_bytes;
  return BR_OK;
}

br_status br_init(br_ctx** out, const br_matrix_desc* descs, int32_t n_mats, const br_hparams* hp, void* dev_workspace,
                  size_t workspace_bytes, void* hip_stream) {
  if (!out) { g_static_err = "null context output pointer"; return BR_ERR_INVALID_ARG; }
  *out = nullptr;
  std::string why;
  br_status st = validate(descs, n_mats, hp, &why);
  if (st != BR_OK) { g_static_err = why; return st; }
  if (!dev_workspace) { g_static_err = "null workspace"; return BR_ERR_INVALID_ARG; }
  if (reinterpret_cast<uintptr_t>(dev_workspace) & 255u) { g_static_err = "workspace must be 256-byte aligned"; return BR_ERR_WORKSPACE; }
  br_ctx* c = new (std::nothrow) br_ctx();
  if (!c) { g_static_err = "out of host memory"; return BR_ERR_INVALID_ARG; }
  c->hp = *hp;
  if (c->hp.stat_beta < 0.f) c->hp.stat_beta = c->hp.beta2;
  plan(descs, n_mats, c->hp, &c->lay);
  if (workspace_bytes < c->lay.state_bytes + c->lay.scratch_bytes) {
    g_static_err = "workspace too small: need " + std::to_string(c->lay.state_bytes + c->lay.scratch_bytes) + " bytes";
    br_destroy(c);
    return BR_ERR_WORKSPACE;
  }
  c->stream = reinterpret_cast<hipStream_t>(hip_stream);
  char* p = reinterpret_cast<char*>(dev_workspace);
  c->mats.resize(n_mats);
  for (int i = 0; i < n_mats; ++i) {
    MatState& m = c->mats[i];
    m.d = descs[i];
    sides(m.d, c->hp, &m.rot_l, &m.rot_r);
    size_t mn = align256((size_t)m.d.m * m.d.n * 4);
    auto take = [&](size_t bytes) { float* q = reinterpret_cast<float*>(p); p += bytes; return q; };
    m.M = take(mn);
    m.S = take(mn);
    if (c->hp.source == BR_SRC_SECOND) {
      if (m.rot_l) m.L = take(align256((size_t)m.d.m * m.d.m * 4));
      if (m.rot_r) m.R = take(align256((size_t)m.d.n * m.d.n * 4));
    }
    if (m.rot_l) m.QL = take(align256((size_t)m.d.m * m.d.m * 4));
    if (m.rot_r) m.QR = take(align256((size_t)m.d.n * m.d.n * 4));
    if (m.d.param_dtype == BR_BF16) m.master = take(mn);
    if ((m.rot_l || m.rot_r) && c->hp.cache_rotated_moment) m.Mrot = take(mn);
    if (c->hp.math != BR_MATH_F32) {
      auto take16 = [&](size_t bytes) { return reinterpret_cast<uint16_t*>(take(bytes)); };
      if (m.rot_l) { m.qlp = take16(plane_bytes(m.d.m, m.d.m, c->hp)); m.qlt = take16(plane_bytes(m.d.m, m.d.m, c->hp)); }
      if (m.rot_r) { m.qrp = take16(plane_bytes(m.d.n, m.d.n, c->hp)); m.qrt = take16(plane_bytes(m.d.n, m.d.n, c->hp)); }
    }
    m.norms = take(256);
  }
  {
    char* gp = reinterpret_cast<char*>(dev_workspace) + c->lay.state_bytes + kNormPartialBytes;
    for (int i = 0; i < n_mats && c->hp.math != BR_MATH_F32; ++i) {
      MatState& m = c->mats[i];
      if (!m.rot_l && !m.rot_r) continue;
      m.gp = reinterpret_cast<uint16_t*>(gp); gp += plane_bytes(m.d.m, m.d.n, c->hp);
      m.gtp = reinterpret_cast<uint16_t*>(gp); gp += plane_bytes(m.d.n, m.d.m, c->hp);
    }
  }
  c->clip_result = reinterpret_cast<float*>(p);
  c->health = reinterpret_cast<int*>(p + 256);
  c->scratch = reinterpret_cast<char*>(dev_workspace) + c->lay.state_bytes;
  c->phase = c->scratch + kNormPartialBytes + c->lay.gplane_bytes;
  // zero state, identity bases
  if (!hip_ok(c, hipMemsetAsync(dev_workspace, 0, c->lay.state_bytes, c->stream), "state clear")) {
    g_static_err = c->err; br_destroy(c); return BR_ERR_HIP;
  }
  for (auto& kv : c->lay.refresh) {
    const auto& jobs = kv.second;
    for (size_t off = 0; off < jobs.size(); off += BR_MAXB) {
      float* ptrs[BR_MAXB];
      int b = (int)std::min<size_t>(BR_MAXB, jobs.size() - off);
      for (int i = 0; i < b; ++i) {
        const MatState& m = c->mats[jobs[off + i].mat];
        ptrs[i] = jobs[off + i].left ? m.QL : m.QR;
      }
      if (!hip_ok(c, br_launch_set_identity(c->stream, ptrs, b, (int)kv.first), "identity init")) {
        g_static_err = c->err; br_destroy(c); return BR_ERR_HIP;
      }
    }
  }
  *out = c;
  return BR_OK;
}

void br_destroy(br_ctx* ctx) {
  if (!ctx) return;
  for (hipEvent_t e : ctx->events) (void)hipEventDestroy(e);
  delete ctx;
}

br_status br_get_step_count(const br_ctx* ctx, int64_t* t) {
  if (!ctx || !t) return BR_ERR_INVALID_ARG;
  *t = ctx->t;
  return BR_OK;
}

br_status br_set_step_count(br_ctx* ctx, int64_t t) {
  if (!ctx) return BR_ERR_INVALID_ARG;
  if (t < 0) return fail(ctx, BR_ERR_INVALID_ARG, "step count must be non-negative");
  ctx->t = t;
  for (auto& m : ctx->mats) m.master_ready = (t > 0) && m.master;
  return BR_OK;
}

br_status br_notify_state_written(br_ctx* ctx) {
  if (!ctx) return BR_ERR_INVALID_ARG;
  ctx->mrot_valid = false;
  ctx->qplanes_valid = false;
  return BR_OK;
}

br_status br_get_state(br_ctx* ctx, int32_t mat, int32_t which, void** dev_ptr, int64_t* rows, int64_t* cols) {
  if (!ctx) return BR_ERR_INVALID_ARG;
  if (!dev_ptr || !rows || !cols) return fail(ctx, BR_ERR_INVALID_ARG, "null output pointer");
  if (mat < 0 || mat >= (int32_t)ctx->mats.size()) return fail(ctx, BR_ERR_INVALID_ARG, "matrix index out of range");
  MatState& m = ctx->mats[mat];
  float* p = nullptr;
  int64_t r = 0, cdim = 0;
  switch (which) {
    case BR_STATE_M: p = m.M; r = m.d.m; cdim = m.d.n; break;
    case BR_STATE_S: p = m.S; r = m.d.m; cdim = m.d.n; break;
    case BR_STATE_L: p = m.L; r = cdim = m.d.m; break;
    case BR_STATE_R: p = m.R; r = cdim = m.d.n; break;
    case BR_STATE_QL: p = m.QL; r = cdim = m.d.m; break;
    case BR_STATE_QR: p = m.QR; r = cdim = m.d.n; break;
    case BR_STATE_MASTER: p = m.master; r = m.d.m; cdim = m.d.n; break;
    case BR_STATE_NORMS: p = m.norms; r = 1; cdim = 2; break;
    case BR_STATE_MROT: p = m.Mrot; r = m.d.m; cdim = m.d.n; break;
    default: return fail(ctx, BR_ERR_INVALID_ARG, "unknown state kind");
  }
  if (!p) return fail(ctx, BR_ERR_INVALID_ARG, "this matrix has no such buffer");
  *dev_ptr = p;
  *rows = r;
  *cols = cdim;
  return BR_OK;
}

static br_status check_call(br_ctx* ctx, const void* const* a, const void* const* b, bool need_b, int32_t n_mats) {
  if (!ctx) return BR_ERR_INVALID_ARG;
  if (ctx->dead) return BR_ERR_HIP;
  if (!a || (need_b && !b)) return fail(ctx, BR_ERR_INVALID_ARG, "null pointer array");
  if (n_mats != (int32_t)ctx->mats.size()) return fail(ctx, BR_ERR_SHAPE, "n_mats differs from br_init");
  for (int i = 0; i < n_mats; ++i) {
    if (!a[i] || (need_b && !b[i])) return fail(ctx, BR_ERR_INVALID_ARG, "null device pointer for matrix " + std::to_string(i));
    if ((reinterpret_cast<uintptr_t>(a[i]) & 15u) || (need_b && (reinterpret_cast<uintptr_t>(b[i]) & 15u)))
      return fail(ctx, BR_ERR_INVALID_ARG, "device pointers must be 16-byte aligned (matrix " + std::to_string(i) + ")");
  }
  return BR_OK;
}

br_status br_get_health(br_ctx* ctx, void** dev_ptr) {
  if (!ctx || !dev_ptr) return BR_ERR_INVALID_ARG;
  *dev_ptr = ctx->health;
  return BR_OK;
}

br_status br_check_health(br_ctx* ctx, int32_t* counts) {
  if (!ctx) return BR_ERR_INVALID_ARG;
  if (ctx->dead) return BR_ERR_HIP;
  hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(ctx->stream, &cap) == hipSuccess && cap != hipStreamCaptureStatusNone)
    return fail(ctx, BR_ERR_STATE, "br_check_health synchronises and cannot run while the stream is being captured");
  int32_t h[BR_HEALTH_WORDS] = {0, 0, 0, 0};
  if (!hip_ok(ctx, hipMemcpyAsync(h, ctx->health, sizeof(h), hipMemcpyDeviceToHost, ctx->stream), "health copy")) return BR_ERR_HIP;
  if (!hip_ok(ctx, hipStreamSynchronize(ctx->stream), "health sync")) return BR_ERR_HIP;
  if (counts) std::memcpy(counts, h, sizeof(h));
  if (h[BR_HEALTH_QR_GAVE_UP] == 0 && h[BR_HEALTH_NONFINITE_WEIGHT] == 0) return BR_OK;
  std::string msg;
  if (h[BR_HEALTH_QR_GAVE_UP])
    msg += "a QR panel cluster gave up waiting for its partner workgroups " + std::to_string(h[BR_HEALTH_QR_GAVE_UP]) +
           " time(s): the affected bases were left as they were before that refresh (was the GPU shared with other work?)";
  if (h[BR_HEALTH_NONFINITE_WEIGHT]) {
    if (!msg.empty()) msg += "; ";
    msg += "non-finite weights were stored (" + std::to_string(h[BR_HEALTH_NONFINITE_WEIGHT]) + " wavefront(s) saw one)";
  }
  return fail(ctx, BR_ERR_STATE, msg);
}

br_status br_set_qr_wait_limit(br_ctx* ctx, int64_t polls) {
  if (!ctx) return BR_ERR_INVALID_ARG;
  if (polls > 0xffffffffLL) return fail(ctx, BR_ERR_INVALID_ARG, "wait limit must fit 32 bits");
  ctx->qr_spin_limit = polls < 0 ? BR_QR_SPIN_LIMIT_DEFAULT : (unsigned)polls;
  return BR_OK;
}

br_status br_get_clip_result(br_ctx* ctx, void** dev_ptr) {
  if (!ctx || !dev_ptr) return BR_ERR_INVALID_ARG;
  *dev_ptr = ctx->clip_result;
  return BR_OK;
}

br_status br_delay_compensate(br_ctx* ctx, void* const* grads, const void* const* params_now,
                              const void* const* params_stale, int32_t n_mats, float lambda) {
  br_status st = check_call(ctx, reinterpret_cast<const void* const*>(grads), params_now, true, n_mats);
  if (st == BR_OK) st = check_call(ctx, params_stale, nullptr, false, n_mats);
  if (st != BR_OK) return st;
  br_ctx* c = ctx;
  if (!(lambda >= 0.f && lambda <= 1.f)) return fail(c, BR_ERR_INVALID_ARG, "lambda must lie in [0, 1]");
  if (c->stats_fresh) return fail(c, BR_ERR_STATE, "compensate the gradients before br_accumulate_stats");
  for (const Group& g : c->lay.groups) {
    const int64_t count = g.m * g.n;
    for (size_t off = 0; off < g.idx.size(); off += BR_MAXB) {
      const int B = (int)std::min<size_t>(BR_MAXB, g.idx.size() - off);
      BrPtrBatch pb;
      std::memset(&pb, 0, sizeof(pb));
      for (int i = 0; i < B; ++i) {
        pb.in0[i] = params_now[g.idx[off + i]];
        pb.in1[i] = params_stale[g.idx[off + i]];
        pb.out0[i] = grads[g.idx[off + i]];
      }
      const double gb = (g.gdt == BR_BF16 ? 2.0 : 4.0), wb = (g.pdt == BR_BF16 ? 2.0 : 4.0);
      Timed tm(c, "br_delay_compensate", 5.0 * count * B, (double)count * B * (2.0 * gb + 2.0 * wb));
      if (!hip_ok(c, br_launch_delay_compensate(c->stream, pb, B, count, g.gdt == BR_BF16, g.pdt == BR_BF16, lambda),
                  "delay compensation launch"))
        return BR_ERR_HIP;
    }
  }
  return BR_OK;
}

br_status br_clip_gradients(br_ctx* ctx, void* const* grads, int32_t n_mats, float max_norm) {
  br_status st = check_call(ctx, reinterpret_cast<const void* const*>(grads), nullptr, false, n_mats);
  if (st != BR_OK) return st;
  br_ctx* c = ctx;
  if (!(max_norm > 0.f)) return fail(c, BR_ERR_INVALID_ARG, "max_norm must be positive");
  if (c->stats_fresh) return fail(c, BR_ERR_STATE, "clip the gradients before br_accumulate_stats");
  if ((size_t)n_mats * BR_CLIP_BLOCKS * sizeof(float) > kNormPartialBytes)
    return fail(c, BR_ERR_UNSUPPORTED, "too many matrices for the clipping reduction");
  float* partials = reinterpret_cast<float*>(c->scratch);
  for (int pass = 0; pass < 2; ++pass) {
    int slot = 0;
    for (const Group& g : c->lay.groups) {
      const int64_t count = g.m * g.n;
      for (size_t off = 0; off < g.idx.size(); off += BR_MAXB) {
        const int B = (int)std::min<size_t>(BR_MAXB, g.idx.size() - off);
        BrPtrBatch pb;
        std::memset(&pb, 0, sizeof(pb));
        for (int i = 0; i < B; ++i) {
          pb.in0[i] = grads[g.idx[off + i]];
          pb.out0[i] = grads[g.idx[off + i]];
        }
        const double gbytes = (double)count * B * (g.gdt == BR_BF16 ? 2.0 : 4.0);
        if (pass == 0) {
          Timed tm(c, "br_grad_sumsq", 2.0 * count * B, gbytes);
          if (!hip_ok(c, br_launch_sumsq(c->stream, pb, B, count, g.gdt == BR_BF16, partials, slot), "sumsq launch")) return BR_ERR_HIP;
        } else {
          Timed tm(c, "br_scale_inplace", 1.0 * count * B, 2.0 * gbytes);
          if (!hip_ok(c, br_launch_scale_inplace(c->stream, pb, B, count, g.gdt == BR_BF16, c->clip_result), "scale launch")) return BR_ERR_HIP;
        }
        slot += B * BR_CLIP_BLOCKS;
      }
    }
    if (pass == 0 && !hip_ok(c, br_launch_clip_finalize(c->stream, partials, slot, max_norm, c->clip_result), "clip finalize launch")) return BR_ERR_HIP;
  }
  return BR_OK;
}

// a2 in BR_MATH_F32 for one chunk of a group: L <- b L + (1-b) G G^T, R <- b R + (1-b) G^T G (Algorithm 2,
// updates of L and R) from the FP32 gradients g32.
static bool stats_chunk_f32(br_ctx* c, const Group& g, size_t off, int B, const float* const* g32) {
  const br_hparams& hp = c->hp;
  BrGemmBatch gb;
  std::memset(&gb, 0, sizeof(gb));
  if (g.rot_l) {  // L <- b L + (1-b) G G^T
    for (int i = 0; i < B; ++i) { gb.A[i] = g32[i]; gb.B[i] = g32[i]; gb.C[i] = c->mats[g.idx[off + i]].L; }
    BrGemmArgs a{(int)g.m, (int)g.m, (int)g.n, (int)g.n, (int)g.n, (int)g.m, 0, 1, 1.0f - hp.stat_beta, hp.stat_beta, B, 1};
    if (!gemm(c, a, gb)) return false;
  }
  if (g.rot_r) {  // R <- b R + (1-b) G^T G
    for (int i = 0; i < B; ++i) { gb.A[i] = g32[i]; gb.B[i] = g32[i]; gb.C[i] = c->mats[g.idx[off + i]].R; }
    BrGemmArgs a{(int)g.n, (int)g.n, (int)g.m, (int)g.n, (int)g.n, (int)g.n, 1, 0, 1.0f - hp.stat_beta, hp.stat_beta, B, 1};
    if (!gemm(c, a, gb)) return false;
  }
  return true;
}

// stats_on_refresh_only: the statistics update that br_accumulate_stats left out, from the gradient
// pointers it kept (Algorithm 2 updates L and R inside Eigenbasis-Estimation, which Algorithm 1 calls
// on refresh steps only).  Runs at the start of br_refresh_basis, before the refresh takes the scratch.
static bool fold_pending_statistics(br_ctx* c) {
  const br_hparams& hp = c->hp;
  for (const Group& g : c->lay.groups) {
    if (!(g.rot_l || g.rot_r) || hp.source != BR_SRC_SECOND) continue;
    const int64_t count = g.m * g.n;
    const size_t mn = align256((size_t)count * 4);
    const int nbuf = step_buffers(g, hp);
    const bool lowp = hp.math != BR_MATH_F32;
    const size_t chunk = lowp ? g.lowp_chunk : kStepChunk;
    for (size_t off = 0; off < g.idx.size(); off += chunk) {
      const int B = (int)std::min<size_t>(chunk, g.idx.size() - off);
      if (lowp) {  // the gradients' operand planes were made by br_accumulate_stats and live until br_step
        LowpCtx lx{c, &g, lowp_layout(g), B, hp.math == BR_MATH_BF16X3 ? 3 : 1, c->phase};
        if (!lowp_stats(lx, nullptr, off, true, true)) return false;
        continue;
      }
      const float* g32[kStepChunk];
      for (int i = 0; i < B; ++i) {
        const void* gp = c->pending_grads[g.idx[off + i]];
        if (g.gdt == BR_BF16) {
          float* dst = scratch_buf(c, nbuf, mn, i, nbuf - 1);
          if (!hip_ok(c, br_launch_bf16_to_f32(c->stream, reinterpret_cast<const uint16_t*>(gp), dst, count), "gradient widen")) return false;
          g32[i] = dst;
        } else {
          g32[i] = reinterpret_cast<const float*>(gp);
        }
      }
      if (!stats_chunk_f32(c, g, off, B, g32)) return false;
    }
  }
  return true;
}

br_status br_accumulate_stats(br_ctx* ctx, const void* const* grads, int32_t n_mats) {
  br_status st = check_call(ctx, grads, nullptr, false, n_mats);
  if (st != BR_OK) return st;
  br_ctx* c = ctx;
  if (c->stats_fresh) return fail(c, BR_ERR_STATE, "br_accumulate_stats called twice without br_step");
  const br_hparams& hp = c->hp;
  // Statistics now (every step), or left to this step's br_refresh_basis, if there is one (Algorithm 2 as printed)
  const bool stats_now = hp.source == BR_SRC_SECOND && !hp.stats_on_refresh_only;
  for (const Group& g : c->lay.groups) {
    const int64_t count = g.m * g.n;
    const size_t mn = align256((size_t)count * 4);
    const int nbuf = step_buffers(g, hp);
    const bool rotated = g.rot_l || g.rot_r;
    const bool need_g32 = rotated && g.gdt == BR_BF16;
    const bool lowp = rotated && hp.math != BR_MATH_F32;
    const size_t chunk = lowp ? g.lowp_chunk : kStepChunk;
    for (size_t off = 0; off < g.idx.size(); off += chunk) {
      const int B = (int)std::min<size_t>(chunk, g.idx.size() - off);
      LowpCtx lx{c, &g, lowp ? lowp_layout(g) : LowpLayout{}, B, hp.math == BR_MATH_BF16X3 ? 3 : 1, c->phase};
      BrPtrBatch pb;
      std::memset(&pb, 0, sizeof(pb));
      const float* g32[kStepChunk];
      for (int i = 0; i < B; ++i) {
        const MatState& m = c->mats[g.idx[off + i]];
        pb.in0[i] = grads[g.idx[off + i]];
        pb.out0[i] = m.M;
        pb.out1[i] = !need_g32 ? nullptr : (lowp ? lx.slot32(i, LS_G32) : scratch_buf(c, nbuf, mn, i, nbuf - 1));
        g32[i] = need_g32 ? reinterpret_cast<const float*>(pb.out1[i]) : reinterpret_cast<const float*>(grads[g.idx[off + i]]);
      }
      if (lowp && g.gdt == BR_F32) {
        // BF16 math modes, FP32 gradients: the first moment and both plane sets of G from one read of G
        float* Mp[BR_MAXB];
        uint16_t *gp[BR_MAXB], *gtp[BR_MAXB];
        for (int i = 0; i < B; ++i) {
          const MatState& m = c->mats[g.idx[off + i]];
          Mp[i] = m.M; gp[i] = m.gp; gtp[i] = m.gtp;
        }
        const int lo = hp.math == BR_MATH_BF16X3 ? 1 : 0;
        {
          Timed tm(c, "br_ingest_planes", 2.0 * count * B, (double)count * B * (12.0 + (lo ? 8.0 : 4.0)));
          if (!hip_ok(c, br_launch_ingest_planes(c->stream, g32, Mp, gp, gtp, B, (int)g.m, (int)g.n, hp.beta1, lo),
                      "ingest launch")) return BR_ERR_HIP;
        }
        if (!lowp_stats(lx, g32, off, stats_now, true)) return BR_ERR_HIP;
        continue;
      }
      {
        double bytes = (double)count * B * (8.0 + (g.gdt == BR_BF16 ? 2.0 : 4.0) + (need_g32 ? 4.0 : 0.0));
        Timed tm(c, "br_ema_first_moment", 2.0 * count * B, bytes);
        if (!hip_ok(c, br_launch_ema(c->stream, pb, B, count, g.gdt == BR_BF16, hp.beta1), "first-moment launch")) return BR_ERR_HIP;
      }
      if (lowp) {
        if (!lowp_stats(lx, g32, off, stats_now)) return BR_ERR_HIP;
        continue;
      }
      if (!stats_now || !rotated) continue;
      if (!stats_chunk_f32(c, g, off, B, g32)) return BR_ERR_HIP;
    }
  }
  c->stats_fresh = true;
  c->g32_group = -1;
  {
    int rotated_groups = 0, only = -1;
    for (size_t gi = 0; gi < c->lay.groups.size(); ++gi)
      if (c->lay.groups[gi].rot_l || c->lay.groups[gi].rot_r) { ++rotated_groups; only = (int)gi; }
    if (rotated_groups == 1) {
      const Group& g = c->lay.groups[only];
      const size_t chunk = hp.math != BR_MATH_F32 ? g.lowp_chunk : (size_t)kStepChunk;
      if (g.gdt == BR_BF16 && g.idx.size() <= chunk) c->g32_group = only;
    }
  }
  if (hp.stats_on_refresh_only && hp.source == BR_SRC_SECOND) {
    c->pending_grads.assign(grads, grads + n_mats);
    c->stats_pending = true;
  }
  return BR_OK;
}

// Blocked Householder QR of the k x k matrices P (in place) for a batch of jobs, orthogonal
// factor written to Q with the sign convention diag(R) >= 0, everything on stream s.
// Recursive blocking.  Panels of BR_QR_NB columns are factorised by the panel kernel and applied
// inside their middle block of BR_QR_NBM columns, whose reflectors are merged into one compact-WY
// factor in LDS.  From there blocks are merged pairwise up to a top block of BR_QR_NBT columns:
// the first child is factorised and applied to the second child's columns, the second child is
// factorised, and
//   T = [ T_0  -T_0 (V_0^T V_1) T_1 ]
//       [ 0     T_1                 ]
// The top block is applied to the trailing matrix, and later to Q, with K = BR_QR_NBT
// contractions (the longer K is, the closer those run to the rate of a step contraction).
// failed: B ints of scratch; a matrix whose panel clusters gave up their bounded wait gets its flag set
// by the panel kernel, and every launch that writes Q then leaves that matrix's previous basis alone.
static bool qr_batch(br_ctx* c, hipStream_t s, int B, int k, float* const* P, float* const* Q, const RefreshScratch& rs,
                     char* base, size_t stride, float* partial, int* failed) {
  const int NB = BR_QR_NB, NBM = BR_QR_NBM;
  const int levels = qr_levels(c->hp, k);
  const int NBT = NBM << levels;  // width of a top block
  const int ntop = (k + NBT - 1) / NBT;
  auto F = [&](int i, size_t off) { return reinterpret_cast<float*>(base + i * stride + off); };
  auto V = [&](int i) { return F(i, rs.V); };  // reflectors of the current top block, row stride NBT
  auto Y = [&](int i) { return F(i, rs.Y); };
  auto W = [&](int i) { return F(i, rs.W); };
  auto Ttop = [&](int i, int tb) { return F(i, rs.T) + (size_t)tb * NBT * NBT; };
  auto Tp = [&](int i, int pnl) { return F(i, rs.Tp) + (size_t)pnl * NB * NB; };
  auto Tl = [&](int i, int l, int slot) {
    const size_t w = (size_t)(NBM << l);
    return F(i, rs.Tl) + qr_level_offset(l) + (size_t)slot * w * w;
  };
  auto D = [&](int i) { return F(i, rs.diag); };
  auto mm = [&](const BrGemmArgs& a, const BrGemmBatch& gb) { return gemm(c, a, gb, false, partial, s); };
  BrQrPanelBatch pb;
  BrQrClusterBatch cb;
  BrGemmBatch gb;
  std::memset(&gb, 0, sizeof(gb));
  {  // the clusters' exchange words carry tags that are unique from here on: start from zero
    int* xp[BR_MAXB];
    for (int i = 0; i < B; ++i) xp[i] = reinterpret_cast<int*>(F(i, rs.xch));
    if (!hip_ok(c, br_launch_zero_ints(s, xp, B, (int)br_qr_panel_xch_floats(k)), "exchange clear launch")) return false;
    int* fp[1] = {failed};
    if (!hip_ok(c, br_launch_zero_ints(s, fp, 1, BR_MAXB), "failure flag clear launch")) return false;
  }
  const int* skip_q = nullptr;  // set for the phase that writes Q
  // The update both phases share: C <- C - Yb (V^T C) for the rows x ncols blocks C (row stride k), with
  // Yb = V T^T or V T.  Above kSplitRefreshMinOrder the three contractions (Yb itself included) run on the 16-bit
  // matrix cores as split FP16 products: every operand is hi + lo FP16 (22 mantissa bits, or an absolute
  // 2^-25 of the operand's scale for small entries; subnormal lo parts are kept and the matrix instruction
  // honours them), three partial products hi*hi + hi*lo + lo*hi accumulated in FP32, C itself stays FP32.
  // These two products are three quarters of the refresh, and they run at three to four times the rate of
  // the FP32 matrix cores.  FP16's range is narrow, so each operand kind carries a fixed power-of-two scale
  // (undone through alpha): reflectors are at most 1 in magnitude (x 64), T and V T likewise moderate (x 64); the
  // matrix being factorised arrives normalised (largest entry of A below 2^-7, so |A Q| <= 1 up to order
  // 16384 and its column norms, which bound every later entry of C, stay below 2^9; x 128), Q's entries are at
  // most 1 (x 128), and |V^T C| <= sqrt(2) |c_j| (x 64).  Values beyond the range would be clamped, not
  // turned into infinities.  The operand
  // planes of C^T are not made again for every block: the whole matrix is split once per phase
  // (planes of P^T, planes of Q^T), a block's C^T is a view into that set (blocks start at multiples
  // of 256), and the update's epilogue rewrites the view from the values it stores.  The product
  // V^T C leaves its kernel transposed and already split, as the operand of the second one.
  const bool x3 = split_refresh(c->hp, k);
  LowpCtx lx{c, nullptr, LowpLayout{}, B, 3, nullptr};
  lx.quiet = true;
  const size_t qchunk = qr_plane_chunk(k);
  const BrPlaneLayout Lk = br_plane_layout(k, k);
  // hi plane of the view that starts at plane row row0 and at k0 inside the k x k plane set at `set`
  auto view = [&](size_t set, int i, int row0, int k0) {
    return reinterpret_cast<uint16_t*>(base + i * stride + set) + (((size_t)(k0 >> 4) * Lk.rows_p + row0) * 2) * 8;
  };
  auto split_whole = [&](float* const* Mx, size_t set) -> bool {  // planes of the transposed k x k matrices
    const float* src[BR_MAXB];
    uint16_t* dst[BR_MAXB];
    for (int i = 0; i < B; ++i) { src[i] = Mx[i]; dst[i] = reinterpret_cast<uint16_t*>(base + i * stride + set); }
    return f16_split(lx, src, k, k, true, dst, 0, kScaleC);
  };
  // Vb: the block's reflectors (rows x width, row stride NBT); Tb (row stride ldt): the block's factor, Yb = Vb Tb^T, or
  // Vb Tb with t_plain; Cp: the blocks C (FP32); set/row0/k0: where their transposes live as planes; emit: keep
  // those planes current.  The FP32 path forms Yb in Y first; the split path forms it as planes directly.
  auto apply_block = [&](float* const* Vb, int width, float* const* Tb, int ldt, bool t_plain, float* const* Cp, int rows,
                         int ncols, size_t set, int row0, int k0, bool emit) -> bool {
    if (!x3 || width < 256) {
      for (int i = 0; i < B; ++i) { gb.A[i] = Vb[i]; gb.B[i] = Tb[i]; gb.C[i] = Y(i); }
      if (!mm(BrGemmArgs{rows, width, width, NBT, ldt, width, 0, t_plain ? 0 : 1, 1.f, 0.f, B, 0}, gb)) return false;
      for (int i = 0; i < B; ++i) { gb.A[i] = Vb[i]; gb.B[i] = Cp[i]; gb.C[i] = W(i); }
      if (!mm(BrGemmArgs{width, ncols, rows, NBT, k, ncols, 1, 0, 1.f, 0.f, B, 0}, gb)) return false;
      for (int i = 0; i < B; ++i) { gb.A[i] = Y(i); gb.B[i] = W(i); gb.C[i] = Cp[i]; }
      BrGemmArgs ua{rows, ncols, width, width, ncols, k, 0, 0, -1.f, 1.f, B, 0};
      ua.skip = skip_q;
      return mm(ua, gb);
    }
    const float* src[BR_MAXB];
    uint16_t *pv[BR_MAXB], *py[BR_MAXB], *pw[BR_MAXB], *pk[BR_MAXB], *pt[BR_MAXB];
    for (int i = 0; i < B; ++i) {
      char* q = base + i * stride + rs.qrp;
      pv[i] = reinterpret_cast<uint16_t*>(q);
      py[i] = reinterpret_cast<uint16_t*>(q + qchunk);
      pw[i] = reinterpret_cast<uint16_t*>(q + 2 * qchunk);
      pk[i] = reinterpret_cast<uint16_t*>(q + 3 * qchunk);
      pt[i] = reinterpret_cast<uint16_t*>(q + 4 * qchunk);
    }
    for (int i = 0; i < B; ++i) src[i] = Vb[i];
    if (!f16_split(lx, src, rows, width, true, pv, NBT, kScaleV)) return false;   // planes of V^T   [width][rows]
    if (!f16_split(lx, src, rows, width, false, pk, NBT, kScaleV)) return false;  // planes of V     [rows][width]
    for (int i = 0; i < B; ++i) src[i] = Tb[i];
    if (!f16_split(lx, src, width, width, t_plain, pt, ldt, kScaleT)) return false;  // planes of Tb (or Tb^T)  [width][width]
    BrLowpBatch lb;
    std::memset(&lb, 0, sizeof(lb));
    // Yb^T = Tb V^T (or Tb^T V^T), leaving its kernel transposed and split: planes of Yb [rows][width]
    for (int i = 0; i < B; ++i) { lb.A[i] = pt[i]; lb.B[i] = pk[i]; lb.shadow[i] = py[i]; }
    BrLowpArgs ya{width, rows, width, 0, 1.f / (kScaleT * kScaleV), 0.f, B, 0, 3};
    ya.epilogue = BR_EPI_PLANES;
    ya.out_lo = 1;
    ya.f16 = 1;
    ya.out_scale = kScaleY;
    if (!hip_ok(c, br_launch_gemm_lowp(s, ya, lb, nullptr), "qr factor product launch")) return false;
    std::memset(&lb, 0, sizeof(lb));
    for (int i = 0; i < B; ++i) { lb.A[i] = pv[i]; lb.B[i] = view(set, i, row0, k0); lb.shadow[i] = pw[i]; }
    BrLowpArgs wa{width, ncols, rows, 0, 1.f / (kScaleV * kScaleC), 0.f, B, 0, 3};  // (V^T C)^T as planes [ncols][width]
    wa.epilogue = BR_EPI_PLANES;
    wa.out_lo = 1;
    wa.f16 = 1;
    wa.out_scale = kScaleW;
    wa.b_stride_rows = (int)Lk.rows_p;
    wa.b_plane_elems = Lk.elems;
    if (!hip_ok(c, br_launch_gemm_lowp(s, wa, lb, nullptr), "qr bf16 product launch")) return false;
    std::memset(&lb, 0, sizeof(lb));
    for (int i = 0; i < B; ++i) {
      lb.A[i] = py[i]; lb.B[i] = pw[i]; lb.C[i] = Cp[i];
      if (emit) lb.S[i] = reinterpret_cast<float*>(view(set, i, row0, k0));  // the updated C^T, for the next block
    }
    BrLowpArgs ua{rows, ncols, width, k, -1.f / (kScaleY * kScaleW), 1.f, B, 0, 3};
    ua.skip = skip_q;
    ua.f16 = 1;
    ua.out_scale = kScaleC;
    if (emit) {
      ua.out_lo = 1;
      ua.emit_transposed = 1;
      ua.out_stride_rows = (int)Lk.rows_p;
      ua.out_plane_elems = Lk.elems;
    }
    return hip_ok(c, br_launch_gemm_lowp(s, ua, lb, nullptr), "qr bf16 update launch");
  };
  if (x3 && k > 256 && !split_whole(P, rs.planesA)) return false;
  // Factorises columns [c0, c0 + ncols) of every P (ncols <= NBM << level) inside the top block that
  // starts at S0; the block's factor goes to slot `slot` of the level's scratch, or to the top block's
  // own place at the top level.
  std::function<bool(int, int, int, int, int, int)> factor = [&](int level, int c0, int ncols, int S0, int slot, int tb) -> bool {
    const int w = NBM << level;
    const int vo = c0 - S0;  // first row and first column of this block inside the reflector block
    const int r0 = k - c0;   // rows of this block
    auto Tdst = [&](int i) { return level == levels ? Ttop(i, tb) : Tl(i, level, slot); };
    auto V0 = [&](int i) { return V(i) + (size_t)vo * NBT + vo; };
    if (level == 0) {
      const int npanels = (ncols + NB - 1) / NB;
      for (int pnl = 0; pnl < npanels; ++pnl) {
        const int j0 = c0 + pnl * NB;
        const int nb = std::min(NB, c0 + ncols - j0);
        const int prow = k - j0;
        const int voff = j0 - S0;
        std::memset(&pb, 0, sizeof(pb));
        std::memset(&cb, 0, sizeof(cb));
        for (int i = 0; i < B; ++i) {
          pb.A[i] = P[i] + (size_t)j0 * k + j0;
          pb.Vc[i] = V(i) + (size_t)voff * NBT + voff;
          pb.T[i] = Tp(i, pnl);
          pb.diag[i] = D(i) + j0;
          cb.xch[i] = reinterpret_cast<unsigned long long*>(F(i, rs.xch));
          cb.failed[i] = failed + i;
        }
        cb.health = c->health;
        cb.spin_limit = c->qr_spin_limit;
        cb.tag0 = (unsigned)(j0 / NB) * 64u;
        if (!hip_ok(c, br_launch_qr_panel(s, pb, cb, B, prow, nb, k, NBT, voff), "qr panel launch")) return false;
        const int nin = c0 + ncols - (j0 + nb);  // columns of the middle block still to the right
        if (nin <= 0) continue;
        // C <- (I - Vp Tp^T Vp^T) C on the middle block's remaining columns, in the panel's rows
        const size_t pfl = partial ? kSplitKBytes / sizeof(float) : 0;
        if (nin <= 96 && pfl >= br_qr_panel_apply_floats(B, prow)) {
          const float* vv[BR_MAXB];
          const float* tt[BR_MAXB];
          float* cc[BR_MAXB];
          for (int i = 0; i < B; ++i) { vv[i] = pb.Vc[i]; tt[i] = Tp(i, pnl); cc[i] = P[i] + (size_t)j0 * k + j0 + nb; }
          if (!hip_ok(c, br_launch_qr_panel_apply(s, vv, tt, cc, B, prow, nin, NBT, k, partial, pfl), "qr panel apply launch"))
            return false;
          continue;
        }
        // (orders too large for the scratch: the same as three general contractions)
        // Yt = Vp Tp^T  (prow x NB), Vp = this panel's slice of V
        for (int i = 0; i < B; ++i) { gb.A[i] = pb.Vc[i]; gb.B[i] = Tp(i, pnl); gb.C[i] = Y(i); }
        if (!mm(BrGemmArgs{prow, NB, NB, NBT, NB, NB, 0, 1, 1.f, 0.f, B, 0}, gb)) return false;
        // W = Vp^T C
        for (int i = 0; i < B; ++i) { gb.A[i] = pb.Vc[i]; gb.B[i] = P[i] + (size_t)j0 * k + j0 + nb; gb.C[i] = W(i); }
        if (!mm(BrGemmArgs{NB, nin, prow, NBT, k, NBM, 1, 0, 1.f, 0.f, B, 0}, gb)) return false;
        // C <- C - Yt W
        for (int i = 0; i < B; ++i) { gb.A[i] = Y(i); gb.B[i] = W(i); gb.C[i] = P[i] + (size_t)j0 * k + j0 + nb; }
        if (!mm(BrGemmArgs{prow, nin, NB, NB, NBM, k, 0, 0, -1.f, 1.f, B, 0}, gb)) return false;
      }
      // Merge the panels' factors: G = V_mid^T V_mid, then T_mid from the panel factors and G.
      const float* gp[BR_MAXB];
      const float* tpp[BR_MAXB];
      float* tb_[BR_MAXB];
      if (npanels > 1) {
        for (int i = 0; i < B; ++i) { gb.A[i] = V0(i); gb.B[i] = V0(i); gb.C[i] = F(i, rs.G); }
        if (!mm(BrGemmArgs{NBM, NBM, r0, NBT, NBT, NBM, 1, 0, 1.f, 0.f, B, 0}, gb)) return false;
      }
      for (int i = 0; i < B; ++i) { gp[i] = F(i, rs.G); tpp[i] = Tp(i, 0); tb_[i] = Tdst(i); }
      return hip_ok(c, br_launch_qr_build_t(s, gp, tpp, tb_, B, npanels), "qr factor merge launch");
    }
    const int wc = w / 2;
    const int n0 = std::min(wc, ncols), n1 = ncols - n0;
    if (!factor(level - 1, c0, n0, S0, 0, tb)) return false;
    if (n1 > 0) {
      // apply the first child to the second child's columns: Yt = V_0 T_0^T ; C <- C - Yt (V_0^T C)
      float *vb[BR_MAXB], *cp[BR_MAXB], *t0[BR_MAXB];
      for (int i = 0; i < B; ++i) { vb[i] = V0(i); t0[i] = Tl(i, level - 1, 0); cp[i] = P[i] + (size_t)c0 * k + c0 + wc; }
      // (these columns are factorised next; their planes are read again only if that factorisation has split
      // applies of its own, i.e. children of 256 columns or more)
      if (!apply_block(vb, wc, t0, wc, false, cp, r0, n1, rs.planesA, c0 + wc, c0, wc >= 512)) return false;
      if (!factor(level - 1, c0 + wc, n1, S0, 1, tb)) return false;
    }
    {  // merged factor: diagonal blocks, then the coupling block -T_0 (V_0^T V_1) T_1
      const float* tc[BR_MAXB];
      float* td[BR_MAXB];
      for (int i = 0; i < B; ++i) { tc[i] = Tl(i, level - 1, 0); td[i] = Tdst(i); }
      if (!hip_ok(c, br_launch_qr_assemble_t(s, tc, td, B, n1 > 0 ? 2 : 1, wc), "qr factor assemble launch")) return false;
    }
    if (n1 > 0) {
      for (int i = 0; i < B; ++i) { gb.A[i] = V0(i); gb.B[i] = V0(i) + wc; gb.C[i] = F(i, rs.X); }
      if (!mm(BrGemmArgs{wc, wc, r0, NBT, NBT, wc, 1, 0, 1.f, 0.f, B, 0}, gb)) return false;
      for (int i = 0; i < B; ++i) { gb.A[i] = Tl(i, level - 1, 0); gb.B[i] = F(i, rs.X); gb.C[i] = F(i, rs.Z); }
      if (!mm(BrGemmArgs{wc, wc, wc, wc, wc, wc, 0, 0, 1.f, 0.f, B, 0}, gb)) return false;
      for (int i = 0; i < B; ++i) { gb.A[i] = F(i, rs.Z); gb.B[i] = Tl(i, level - 1, 1); gb.C[i] = Tdst(i) + wc; }
      if (!mm(BrGemmArgs{wc, wc, wc, wc, wc, w, 0, 0, -1.f, 0.f, B, 0}, gb)) return false;
    }
    return true;
  };
  float *cblk[BR_MAXB], *vblk[BR_MAXB], *tblk[BR_MAXB];
  for (int tb = 0; tb < ntop; ++tb) {
    const int S0 = tb * NBT;
    const int ns = std::min(NBT, k - S0);  // columns of this top block
    const int rows = k - S0;
    if (ns < NBT) {  // the reflector block of a narrow last top block: unused columns must read as zero
      int* vp[BR_MAXB];
      for (int i = 0; i < B; ++i) vp[i] = reinterpret_cast<int*>(V(i));
      if (!hip_ok(c, br_launch_zero_ints(s, vp, B, rows * NBT), "reflector clear launch")) return false;
    }
    if (!factor(levels, S0, ns, S0, 0, tb)) return false;
    const int nt = k - S0 - ns;
    if (nt <= 0) continue;
    // Yt = V T^T ; C <- C - Yt (V^T C)   on the trailing columns
    for (int i = 0; i < B; ++i) { cblk[i] = P[i] + (size_t)S0 * k + S0 + ns; vblk[i] = V(i); tblk[i] = Ttop(i, tb); }
    if (!apply_block(vblk, NBT, tblk, NBT, false, cblk, rows, nt, rs.planesA, S0 + ns, S0, true)) return false;
  }
  // Q = H_1 ... H_k applied to the identity, last block reflector first.  Before top block tb is
  // applied, Q differs from the identity only in Q[S1:, S1:] with S1 the next block's offset,
  // so only the columns from S0 on change.
  // The identity carries the signs that make diag(R) >= 0 (a column of Q flips with its sign).
  const float* dg[BR_MAXB];
  for (int i = 0; i < B; ++i) dg[i] = D(i);
  skip_q = failed;  // from here on Q is written: an abandoned factorisation keeps its previous basis
  if (!hip_ok(c, br_launch_qr_signed_identity(s, Q, dg, B, k, skip_q), "signed identity launch")) return false;
  if (x3 && !split_whole(Q, rs.planesB)) return false;
  for (int tb = ntop - 1; tb >= 0; --tb) {
    const int S0 = tb * NBT;
    const int ns = std::min(NBT, k - S0);
    const int rows = k - S0;
    std::memset(&pb, 0, sizeof(pb));
    for (int i = 0; i < B; ++i) {
      pb.A[i] = P[i] + (size_t)S0 * k + S0;
      pb.Vc[i] = V(i);
    }
    if (!hip_ok(c, br_launch_qr_extract_v(s, pb, B, rows, ns, k, NBT), "qr extract launch")) return false;
    // Y = V T ; Qsub <- Qsub - Y (V^T Qsub),  Qsub = Q[S0:, S0:]
    for (int i = 0; i < B; ++i) { cblk[i] = Q[i] + (size_t)S0 * k + S0; vblk[i] = V(i); tblk[i] = Ttop(i, tb); }
    if (!apply_block(vblk, NBT, tblk, NBT, true, cblk, rows, rows, rs.planesB, S0, S0, true)) return false;
  }
  return true;
}

br_status br_refresh_basis(br_ctx* ctx) {
  if (!ctx) return BR_ERR_INVALID_ARG;
  if (ctx->dead) return BR_ERR_HIP;
  br_ctx* c = ctx;
  const br_hparams& hp = c->hp;
  char* base = c->phase;
  if (c->stats_pending) {
    if (!fold_pending_statistics(c)) return BR_ERR_HIP;
    c->stats_pending = false;
  }
  c->g32_group = -1;      // the refresh takes the scratch that held the FP32 images of BF16 gradients
  c->mrot_valid = false;  // the bases change: M~ must be rebuilt from M at the next step
  c->qplanes_valid = false;
  for (const RefreshUnit& u : c->lay.units) {
    const int k = (int)u.k;
    const int B = (int)u.jobs.size();
    const RefreshScratch rs = refresh_scratch(k, hp);
    float* Q[BR_MAXB];
    float* P0[BR_MAXB];
    float* P1[BR_MAXB];
    const float* A[BR_MAXB];
    BrGemmBatch gb;
    std::memset(&gb, 0, sizeof(gb));
    for (int i = 0; i < B; ++i) {
      const RefreshJob& j = u.jobs[i];
      const MatState& m = c->mats[j.mat];
      Q[i] = j.left ? m.QL : m.QR;
      P0[i] = reinterpret_cast<float*>(base + i * rs.total + rs.P0);
      P1[i] = reinterpret_cast<float*>(base + i * rs.total + rs.P1);
      if (hp.source == BR_SRC_SECOND) {
        A[i] = j.left ? m.L : m.R;
      } else {  // first-order source: Gram matrix of the first moment (Algorithm 2, first-order branch)
        float* gram = reinterpret_cast<float*>(base + i * rs.total + rs.gram);
        A[i] = gram;
        BrGemmBatch one;
        std::memset(&one, 0, sizeof(one));
        one.A[0] = m.M; one.B[0] = m.M; one.C[0] = gram;
        BrGemmArgs a = j.left ? BrGemmArgs{k, k, (int)m.d.n, (int)m.d.n, (int)m.d.n, k, 0, 1, 1.f, 0.f, 1, 1}
                              : BrGemmArgs{k, k, (int)m.d.m, (int)m.d.n, (int)m.d.n, k, 1, 0, 1.f, 0.f, 1, 1};
        if (!gemm(c, a, one)) return BR_ERR_HIP;
      }
    }
    // P <- A^iters Q.  Above kSplitRefreshMinOrder the product runs on the 16-bit matrix cores as a split FP16
    // product (hi + lo FP16 operands, three partial products, FP32 accumulation: see qr_batch), in every math mode.
    // The orthogonal factor does not depend on the scale of P, so both operands are normalised by powers of two
    // taken from their largest magnitudes (A's into [2^8, 2^9), the multiplied matrix's into [2^5, 2^6)) and alpha is
    // the constant 2^-22: P comes out as (A / a) (X / x) with a, x the largest entries rounded up to powers of two and
    // divided by 2^-7 resp. 1, i.e. |P| <= sqrt(k) 2^-7, which is what the split products of the QR expect.
    float** src = Q;
    float** dst = P0;
    const bool lowp = split_refresh(hp, k);
    LowpCtx lx{c, nullptr, LowpLayout{}, B, 3, nullptr};
    uint16_t *plA[BR_MAXB], *plB[BR_MAXB];
    for (int i = 0; i < B && lowp; ++i) {
      plA[i] = reinterpret_cast<uint16_t*>(base + i * rs.total + rs.planesA);
      plB[i] = reinterpret_cast<uint16_t*>(base + i * rs.total + rs.planesB);
    }
    unsigned* maxA = reinterpret_cast<unsigned*>(base + (size_t)B * rs.total + 256);
    unsigned* maxX = reinterpret_cast<unsigned*>(base + (size_t)B * rs.total + 512);
    if (lowp) {
      int* zp[1] = {reinterpret_cast<int*>(maxA)};
      if (!hip_ok(c, br_launch_zero_ints(c->stream, zp, 1, BR_MAXB), "magnitude clear launch")) return BR_ERR_HIP;
      if (!hip_ok(c, br_launch_absmax(c->stream, A, B, k, k, k, maxA), "magnitude launch")) return BR_ERR_HIP;
      if (!f16_split(lx, A, k, k, false, plA, 0, 1.f, maxA, 9)) return BR_ERR_HIP;
    }
    for (int it = 0; it < hp.power_iters; ++it) {
      if (lowp) {
        const float* s32[BR_MAXB];
        for (int i = 0; i < B; ++i) s32[i] = src[i];
        int* zp[1] = {reinterpret_cast<int*>(maxX)};
        if (!hip_ok(c, br_launch_zero_ints(c->stream, zp, 1, BR_MAXB), "magnitude clear launch")) return BR_ERR_HIP;
        if (!hip_ok(c, br_launch_absmax(c->stream, s32, B, k, k, k, maxX), "magnitude launch")) return BR_ERR_HIP;
        if (!f16_split(lx, s32, k, k, true, plB, 0, 1.f, maxX, 6)) return BR_ERR_HIP;  // planes of src^T: B[j][l] = src[l][j]
        BrLowpBatch lb;
        std::memset(&lb, 0, sizeof(lb));
        for (int i = 0; i < B; ++i) { lb.A[i] = plA[i]; lb.B[i] = plB[i]; lb.C[i] = dst[i]; }
        BrLowpArgs la{k, k, k, k, std::ldexp(1.0f, -22), 0.f, B, 0, 3};
        la.f16 = 1;
        Timed tm(c, "br_gemm_f16_mfma<3>", 2.0 * k * (double)k * k * B, 0.0);
        if (!hip_ok(c, br_launch_gemm_lowp(c->stream, la, lb, nullptr), "split product launch")) return BR_ERR_HIP;
      } else {
        for (int i = 0; i < B; ++i) { gb.A[i] = A[i]; gb.B[i] = src[i]; gb.C[i] = dst[i]; }
        if (!gemm(c, BrGemmArgs{k, k, k, k, k, k, 0, 0, 1.f, 0.f, B, 0}, gb)) return BR_ERR_HIP;
      }
      src = dst;
      dst = (dst == P0) ? P1 : P0;
    }
    {
      Timed tm(c, "qr_householder(region)", (8.0 / 3.0) * (double)k * k * k * B, 0.0);
      int* failed = reinterpret_cast<int*>(base + (size_t)B * rs.total);
      float* part = reinterpret_cast<float*>(base + (size_t)B * rs.total + kFailFlagBytes);
      if (!qr_batch(c, c->stream, B, k, src, Q, rs, base, rs.total, part, failed)) return BR_ERR_HIP;
    }
  }
  return BR_OK;
}

br_status br_step(br_ctx* ctx, void* const* params, const void* const* grads, int32_t n_mats, float lr) {
  br_status st = check_call(ctx, reinterpret_cast<const void* const*>(params), grads, true, n_mats);
  if (st != BR_OK) return st;
  br_ctx* c = ctx;
  if (!c->stats_fresh) return fail(c, BR_ERR_STATE, "br_step needs br_accumulate_stats for this step first");
  if (!(lr == lr)) return fail(c, BR_ERR_INVALID_ARG, "learning rate is NaN");
  const br_hparams& hp = c->hp;
  {
    // The first step of a BF16 parameter copies it into its FP32 master.  Captured into a graph, that copy would
    // run again at every replay and throw away what the master has accumulated below one BF16 ulp.
    bool master_missing = false;
    for (const MatState& ms : c->mats) master_missing |= (ms.master != nullptr && !ms.master_ready);
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (master_missing && hipStreamIsCapturing(c->stream, &cap) == hipSuccess && cap != hipStreamCaptureStatusNone)
      return fail(c, BR_ERR_STATE, "the first br_step of BF16 parameters initialises their FP32 master copies and must not be "
                                   "captured into a graph: run one step eagerly first");
  }
  const int64_t t = c->t + 1;
  BrAdamArgs aa;
  aa.beta1 = hp.beta1;
  aa.beta2 = hp.beta2;
  aa.eps = hp.eps;
  aa.c1 = hp.bias_correction ? (float)(1.0 / (1.0 - std::pow((double)hp.beta1, (double)t))) : 1.0f;
  aa.c2 = hp.bias_correction ? (float)(1.0 / (1.0 - std::pow((double)hp.beta2, (double)t))) : 1.0f;
  aa.eps_outside = hp.eps_outside_sqrt;
  aa.compute_norms = hp.compute_norms;
  // With the cache on and the basis unchanged since the last step, M~ advances by its own EMA;
  // otherwise it is obtained by rotating M (and stored in the cache when there is one).
  const bool cached = hp.cache_rotated_moment != 0;
  const bool advance = cached && c->mrot_valid;
  aa.update_mrot = advance ? 1 : 0;
  const float decay = 1.0f - lr * hp.weight_decay;
  float* partials = reinterpret_cast<float*>(c->scratch);

  for (const Group& g : c->lay.groups) {
    const int64_t count = g.m * g.n;
    const size_t mn = align256((size_t)count * 4);
    const int nbuf = step_buffers(g, hp);
    const bool rotated = g.rot_l || g.rot_r;
    const bool bilateral = g.rot_l && g.rot_r;
    const int m = (int)g.m, n = (int)g.n;
    // scratch slots
    const int sT1 = 0, sGt = bilateral ? 1 : 0, sT2 = 2, sMt = bilateral ? 3 : 1;
    const bool lowp = rotated && hp.math != BR_MATH_F32;
    const size_t chunk = lowp ? g.lowp_chunk : kStepChunk;
    for (size_t off = 0; off < g.idx.size(); off += chunk) {
      const int B = (int)std::min<size_t>(chunk, g.idx.size() - off);
      LowpCtx lx{c, &g, lowp ? lowp_layout(g) : LowpLayout{}, B, hp.math == BR_MATH_BF16X3 ? 3 : 1, c->phase};
      float* Wp[kStepChunk];         // FP32 weights that receive the update
      uint16_t* shadow[kStepChunk];  // BF16 parameter image, or null
      const float* G32[kStepChunk];
      for (int i = 0; i < B; ++i) {
        MatState& ms = c->mats[g.idx[off + i]];
        void* prm = params[g.idx[off + i]];
        if (g.pdt == BR_BF16) {
          if (!ms.master_ready) {
            if (!hip_ok(c, br_launch_bf16_to_f32(c->stream, reinterpret_cast<const uint16_t*>(prm), ms.master, count), "master init")) return BR_ERR_HIP;
            ms.master_ready = true;
          }
          Wp[i] = ms.master;
          shadow[i] = reinterpret_cast<uint16_t*>(prm);
        } else {
          Wp[i] = reinterpret_cast<float*>(prm);
          shadow[i] = nullptr;
        }
      }
      if (!rotated) {
        BrPtrBatch pb;
        std::memset(&pb, 0, sizeof(pb));
        for (int i = 0; i < B; ++i) {
          const MatState& ms = c->mats[g.idx[off + i]];
          pb.in0[i] = grads[g.idx[off + i]];
          pb.in1[i] = ms.M;
          pb.out0[i] = ms.S;
          pb.out1[i] = Wp[i];
        }
        BrPlainArgs pa{hp.beta2, hp.eps, aa.c1, aa.c2, lr, decay, hp.eps_outside_sqrt, g.gdt == BR_BF16, c->health};
        double bytes = (double)count * B * (4.0 + 8.0 + 8.0 + (g.gdt == BR_BF16 ? 2.0 : 4.0) + (g.pdt == BR_BF16 ? 2.0 : 0.0));
        Timed tm(c, "br_adam_plain", 10.0 * count * B, bytes);
        if (!hip_ok(c, br_launch_adam_plain(c->stream, pb, shadow, B, count, pa), "plain adam launch")) return BR_ERR_HIP;
        continue;
      }
      // FP32 image of BF16 gradients.  The fused chain of the BF16 modes reads the gradients' operand planes
      // only and needs none.  Otherwise br_accumulate_stats wrote the same images into the same slots; they are
      // still there when nothing else has used the scratch since (a single rotated group, no refresh).
      const bool image_unused = lowp && !aa.compute_norms;
      const bool image_kept = image_unused || (c->g32_group >= 0 && &g == &c->lay.groups[c->g32_group]);
      for (int i = 0; i < B; ++i) {
        const void* gp = grads[g.idx[off + i]];
        if (g.gdt == BR_BF16) {
          float* dst = lowp ? lx.slot32(i, LS_G32) : scratch_buf(c, nbuf, mn, i, nbuf - 1);
          if (!image_kept &&
              !hip_ok(c, br_launch_bf16_to_f32(c->stream, reinterpret_cast<const uint16_t*>(gp), dst, count), "gradient widen")) return BR_ERR_HIP;
          G32[i] = dst;
        } else {
          G32[i] = reinterpret_cast<const float*>(gp);
        }
      }
      if (lowp) {
        float* Mtl[kStepChunk];
        for (int i = 0; i < B; ++i) Mtl[i] = cached ? c->mats[g.idx[off + i]].Mrot : lx.slot32(i, LS_MROT);
        if (!lowp_step(lx, off, G32, Wp, shadow, Mtl, advance, aa, lr, decay, partials)) return BR_ERR_HIP;
        continue;
      }
      BrGemmBatch gb;
      std::memset(&gb, 0, sizeof(gb));
      float* Gt[kStepChunk];
      float* Mt[kStepChunk];
      for (int i = 0; i < B; ++i) {
        const MatState& ms = c->mats[g.idx[off + i]];
        Gt[i] = scratch_buf(c, nbuf, mn, i, sGt);
        Mt[i] = cached ? ms.Mrot : scratch_buf(c, nbuf, mn, i, sMt);
      }
      // Adam's moments are advanced in the epilogue of the contraction that produces G~, so that G~ never reaches
      // memory (the appendix on related optimizers notes that the rotated update can be fused this way).  That
      // epilogue needs M~ as an input when it is not advanced from G~ itself: on such steps M is rotated first, by
      // launches of its own.  With norms requested the products are stored and br_adam_rotated does the rest.
      const bool fused = !aa.compute_norms;
      const int nrot = advance ? B : 2 * B;  // unfused: rotate G only, or G and M, in one launch
      auto adam_args = [&](BrGemmArgs a) {
        a.adam_epilogue = 1;
        a.adam = aa;
        return a;
      };
      auto with_moments = [&]() {
        for (int i = 0; i < B; ++i) { gb.S[i] = c->mats[g.idx[off + i]].S; gb.Mrot[i] = Mt[i]; }
      };
      if (bilateral) {
        // T = Q_L^T [G | M], then [G~ | M~] = T Q_R
        if (fused && !advance) {  // M~ = Q_L^T M Q_R ahead of the fused launch
          for (int i = 0; i < B; ++i) {
            const MatState& ms = c->mats[g.idx[off + i]];
            gb.A[i] = ms.QL; gb.B[i] = ms.M; gb.C[i] = scratch_buf(c, nbuf, mn, i, sT2);
          }
          if (!gemm(c, BrGemmArgs{m, n, m, m, n, n, 1, 0, 1.f, 0.f, B, 0}, gb)) return BR_ERR_HIP;
          for (int i = 0; i < B; ++i) {
            const MatState& ms = c->mats[g.idx[off + i]];
            gb.A[i] = scratch_buf(c, nbuf, mn, i, sT2); gb.B[i] = ms.QR; gb.C[i] = Mt[i];
          }
          if (!gemm(c, BrGemmArgs{m, n, n, n, n, n, 0, 0, 1.f, 0.f, B, 0}, gb)) return BR_ERR_HIP;
        }
        for (int i = 0; i < B; ++i) {
          const MatState& ms = c->mats[g.idx[off + i]];
          gb.A[i] = ms.QL; gb.B[i] = G32[i]; gb.C[i] = scratch_buf(c, nbuf, mn, i, sT1);
          gb.A[B + i] = ms.QL; gb.B[B + i] = ms.M; gb.C[B + i] = scratch_buf(c, nbuf, mn, i, sT2);
        }
        if (!gemm(c, BrGemmArgs{m, n, m, m, n, n, 1, 0, 1.f, 0.f, fused ? B : nrot, 0}, gb)) return BR_ERR_HIP;
        for (int i = 0; i < B; ++i) {
          const MatState& ms = c->mats[g.idx[off + i]];
          gb.A[i] = scratch_buf(c, nbuf, mn, i, sT1); gb.B[i] = ms.QR; gb.C[i] = Gt[i];
          gb.A[B + i] = scratch_buf(c, nbuf, mn, i, sT2); gb.B[B + i] = ms.QR; gb.C[B + i] = Mt[i];
        }
        if (fused) {
          with_moments();
          if (!gemm(c, adam_args(BrGemmArgs{m, n, n, n, n, n, 0, 0, 1.f, 0.f, B, 0}), gb)) return BR_ERR_HIP;
        } else if (!gemm(c, BrGemmArgs{m, n, n, n, n, n, 0, 0, 1.f, 0.f, nrot, 0}, gb)) {
          return BR_ERR_HIP;
        }
      } else {
        const BrGemmArgs a = g.rot_l ? BrGemmArgs{m, n, m, m, n, n, 1, 0, 1.f, 0.f, nrot, 0}
                                     : BrGemmArgs{m, n, n, n, n, n, 0, 0, 1.f, 0.f, nrot, 0};
        auto one_side = [&](bool moment_too) {
          for (int i = 0; i < B; ++i) {
            const MatState& ms = c->mats[g.idx[off + i]];
            const int j = moment_too ? B + i : i;
            if (g.rot_l) {
              gb.A[i] = ms.QL; gb.B[i] = G32[i]; gb.C[i] = Gt[i];
              gb.A[j] = ms.QL; gb.B[j] = moment_too ? ms.M : G32[i]; gb.C[j] = moment_too ? Mt[i] : Gt[i];
            } else {
              gb.A[i] = G32[i]; gb.B[i] = ms.QR; gb.C[i] = Gt[i];
              gb.A[j] = moment_too ? ms.M : G32[i]; gb.B[j] = ms.QR; gb.C[j] = moment_too ? Mt[i] : Gt[i];
            }
          }
        };
        if (fused) {
          if (!advance) {  // M~ = Q_L^T M (or M Q_R) ahead of the fused launch
            for (int i = 0; i < B; ++i) {
              const MatState& ms = c->mats[g.idx[off + i]];
              if (g.rot_l) { gb.A[i] = ms.QL; gb.B[i] = ms.M; } else { gb.A[i] = ms.M; gb.B[i] = ms.QR; }
              gb.C[i] = Mt[i];
            }
            BrGemmArgs am = a;
            am.batch = B;
            if (!gemm(c, am, gb)) return BR_ERR_HIP;
          }
          one_side(false);
          with_moments();
          BrGemmArgs ag = adam_args(a);
          ag.batch = B;
          if (!gemm(c, ag, gb)) return BR_ERR_HIP;
        } else {
          one_side(true);
          if (!gemm(c, a, gb)) return BR_ERR_HIP;
        }
      }
      if (!fused) {  // Adam in the rotated basis; X overwrites G~
        BrAdamBatch ab;
        std::memset(&ab, 0, sizeof(ab));
        for (int i = 0; i < B; ++i) {
          const MatState& ms = c->mats[g.idx[off + i]];
          ab.GX[i] = Gt[i];
          ab.S[i] = ms.S;
          ab.Mrot[i] = Mt[i];
          ab.norms[i] = ms.norms;
        }
        Timed tm(c, "br_adam_rotated", 8.0 * count * B, (advance ? 24.0 : 20.0) * count * B);
        if (!hip_ok(c, br_launch_adam_rotated(c->stream, ab, B, count, aa, partials), "rotated adam launch")) return BR_ERR_HIP;
      }
      // rotate back and apply: W <- decay W - lr Q_L X Q_R^T   (X sits in the G~ buffer)
      std::memset(&gb, 0, sizeof(gb));
      auto weight_update = [&](BrGemmArgs a) {  // the launch that stores the weights also watches them for non-finite values
        a.health = c->health;
        return a;
      };
      if (bilateral) {
        for (int i = 0; i < B; ++i) {
          const MatState& ms = c->mats[g.idx[off + i]];
          gb.A[i] = ms.QL; gb.B[i] = Gt[i]; gb.C[i] = scratch_buf(c, nbuf, mn, i, sT1);
        }
        if (!gemm(c, BrGemmArgs{m, n, m, m, n, n, 0, 0, 1.f, 0.f, B, 0}, gb)) return BR_ERR_HIP;
        for (int i = 0; i < B; ++i) {
          const MatState& ms = c->mats[g.idx[off + i]];
          gb.A[i] = scratch_buf(c, nbuf, mn, i, sT1); gb.B[i] = ms.QR; gb.C[i] = Wp[i]; gb.shadow[i] = shadow[i];
        }
        if (!gemm(c, weight_update(BrGemmArgs{m, n, n, n, n, n, 0, 1, -lr, decay, B, 0}), gb)) return BR_ERR_HIP;
      } else if (g.rot_l) {
        for (int i = 0; i < B; ++i) {
          const MatState& ms = c->mats[g.idx[off + i]];
          gb.A[i] = ms.QL; gb.B[i] = Gt[i]; gb.C[i] = Wp[i]; gb.shadow[i] = shadow[i];
        }
        if (!gemm(c, weight_update(BrGemmArgs{m, n, m, m, n, n, 0, 0, -lr, decay, B, 0}), gb)) return BR_ERR_HIP;
      } else {
        for (int i = 0; i < B; ++i) {
          const MatState& ms = c->mats[g.idx[off + i]];
          gb.A[i] = Gt[i]; gb.B[i] = ms.QR; gb.C[i] = Wp[i]; gb.shadow[i] = shadow[i];
        }
        if (!gemm(c, weight_update(BrGemmArgs{m, n, n, n, n, n, 0, 1, -lr, decay, B, 0}), gb)) return BR_ERR_HIP;
      }
    }
  }
  c->mrot_valid = true;
  c->qplanes_valid = true;
  c->t = t;
  c->stats_fresh = false;
  c->g32_group = -1;
  c->stats_pending = false;  // a step without a refresh: Algorithm 2's statistics do not see this gradient
  return BR_OK;
}

br_status br_profile_begin(br_ctx* ctx) {
  if (!ctx) return BR_ERR_INVALID_ARG;
  if (ctx->dead) return BR_ERR_HIP;
  ctx->recs.clear();
  ctx->events_used = 0;
  ctx->prof_on = true;
  return BR_OK;
}

br_status br_profile_end(br_ctx* ctx, br_profile_entry* out, int32_t cap, int32_t* n_out) {
  if (!ctx) return BR_ERR_INVALID_ARG;
  if (!out || !n_out || cap <= 0) return fail(ctx, BR_ERR_INVALID_ARG, "null or empty profile output");
  ctx->prof_on = false;
  if (!hip_ok(ctx, hipStreamSynchronize(ctx->stream), "profile sync")) return BR_ERR_HIP;
  std::vector<br_profile_entry> acc;
  for (const ProfRec& r : ctx->recs) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, ctx->events[r.ev], ctx->events[r.ev + 1]) != hipSuccess) continue;
    br_profile_entry* e = nullptr;
    for (auto& x : acc)
      if (std::strncmp(x.kernel, r.name, sizeof(x.kernel) - 1) == 0) e = &x;
    if (!e) {
      br_profile_entry ne;
      std::memset(&ne, 0, sizeof(ne));
      std::strncpy(ne.kernel, r.name, sizeof(ne.kernel) - 1);
      acc.push_back(ne);
      e = &acc.back();
    }
    e->launches += 1;
    e->ms += ms;
    e->flops += r.flops;
    e->bytes += r.bytes;
  }
  int32_t n = (int32_t)std::min<size_t>(acc.size(), (size_t)cap);
  for (int32_t i = 0; i < n; ++i) out[i] = acc[i];
  *n_out = n;
  ctx->recs.clear();
  ctx->events_used = 0;
  return BR_OK;
}

}  // extern "C"
