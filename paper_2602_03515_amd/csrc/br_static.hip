// Global-norm gradient clipping for callers that cannot allocate device memory and hold no
// workspace (code under HIP graph capture, tight serving loops): the same kernels as
// br_clip_gradients, with the per-workgroup partial sums in a file-scope device array instead of
// the context's workspace.  Nothing here calls hipMalloc/hipFree or any allocating routine.
#include "../../include/br.h"
#include "br_internal.h"

#include <cstring>
#include <mutex>
#include <string>

// One partial sum per (matrix, workgroup) of the sum-of-squares pass.  Every GPU the library runs
// on holds its own copy of this array (1 MiB) until the process ends.
static __device__ __align__(256) float scratch[(size_t)BR_STATIC_CLIP_MAX_MATS * BR_CLIP_BLOCKS];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_mu;
float* g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each device, once resolved

// The array's name is only a host-side handle: the address a kernel can use comes from the runtime,
// per device, with that device current.
hipError_t scratch_on_current_device(float** out, int* device) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = reinterpret_cast<float*>(p);
  }
  *out = g_scratch_ptr[dev];
  *device = dev;
  return hipSuccess;
}

}  // namespace

void br_set_static_error(const std::string& msg);  // br_api.hip: text behind br_last_error(NULL)

extern "C" br_status br_clip_gradients_static(const br_matrix_desc* descs, void* const* grads, int32_t n_mats, float max_norm,
                                              void* dev_result, void* hip_stream) {
  if (!descs || !grads || !dev_result) { br_set_static_error("null descriptor, gradient array or result pointer"); return BR_ERR_INVALID_ARG; }
  if (n_mats <= 0) { br_set_static_error("n_mats must be positive"); return BR_ERR_INVALID_ARG; }
  if (n_mats > BR_STATIC_CLIP_MAX_MATS) {
    br_set_static_error("br_clip_gradients_static handles at most " + std::to_string(BR_STATIC_CLIP_MAX_MATS) + " matrices per call");
    return BR_ERR_WORKSPACE;
  }
  if (!(max_norm > 0.f)) { br_set_static_error("max_norm must be positive"); return BR_ERR_INVALID_ARG; }
  if (reinterpret_cast<uintptr_t>(dev_result) & 7u) { br_set_static_error("result pointer must be 8-byte aligned"); return BR_ERR_INVALID_ARG; }
  for (int i = 0; i < n_mats; ++i) {
    const br_matrix_desc& d = descs[i];
    if (d.m <= 0 || d.n <= 0 || d.m > (1 << 24) || d.n > (1 << 24)) { br_set_static_error("matrix " + std::to_string(i) + ": dimensions must be in 1..2^24"); return BR_ERR_SHAPE; }
    if (d.grad_dtype != BR_F32 && d.grad_dtype != BR_BF16) { br_set_static_error("matrix " + std::to_string(i) + ": unknown gradient dtype"); return BR_ERR_DTYPE; }
    if (!grads[i] || (reinterpret_cast<uintptr_t>(grads[i]) & 15u)) { br_set_static_error("gradient " + std::to_string(i) + " is null or not 16-byte aligned"); return BR_ERR_INVALID_ARG; }
  }
  float* partials = nullptr;
  int dev = 0;
  hipError_t e = scratch_on_current_device(&partials, &dev);
  if (e != hipSuccess) { br_set_static_error(std::string("static scratch address: ") + hipGetErrorString(e)); return BR_ERR_HIP; }
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  float* result = reinterpret_cast<float*>(dev_result);
  // Runs of consecutive matrices with one element count and gradient type share a launch.  Every
  // slot that the final sum reads is written by this call's first pass: nothing needs clearing.
  for (int pass = 0; pass < 2; ++pass) {
    int slot = 0;
    for (int i0 = 0; i0 < n_mats;) {
      const int64_t count = descs[i0].m * descs[i0].n;
      const int gdt = descs[i0].grad_dtype;
      int B = 1;
      while (i0 + B < n_mats && B < BR_MAXB && descs[i0 + B].m * descs[i0 + B].n == count && descs[i0 + B].grad_dtype == gdt) ++B;
      BrPtrBatch pb;
      std::memset(&pb, 0, sizeof(pb));
      for (int i = 0; i < B; ++i) { pb.in0[i] = grads[i0 + i]; pb.out0[i] = grads[i0 + i]; }
      e = (pass == 0) ? br_launch_sumsq(s, pb, B, count, gdt == BR_BF16, partials, slot)
                      : br_launch_scale_inplace(s, pb, B, count, gdt == BR_BF16, result);
      if (e != hipSuccess) { br_set_static_error(std::string("clip launch: ") + hipGetErrorString(e)); return BR_ERR_HIP; }
      slot += B * BR_CLIP_BLOCKS;
      i0 += B;
    }
    if (pass == 0) {
      e = br_launch_clip_finalize(s, partials, slot, max_norm, result);
      if (e != hipSuccess) { br_set_static_error(std::string("clip finalize launch: ") + hipGetErrorString(e)); return BR_ERR_HIP; }
    }
  }
  return BR_OK;
}
