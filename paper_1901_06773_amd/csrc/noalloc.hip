// Entry point for callers that cannot allocate device memory (code under HIP graph capture,
// tight serving loops, harnesses that forbid hipMalloc): batch-norm forward with the
// reduction workspace in a file-scope device array instead of a caller-supplied buffer.
//
// The array lives once per GPU for as long as the process does.  Its name is only a
// host-side stand-in: the device address is looked up once per device with
// hipGetSymbolAddress (that device current) and only that address is ever handed to
// kernels.  Calls that overlap on one GPU share the array and race; calls on one stream,
// or ordered by events, do not.  Nothing in the array has to start at zero: the reduction
// writes every partial sum the finishing pass reads, and the finishing pass writes every
// coefficient the apply pass reads.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <initializer_list>
#include <mutex>

#include "../../include/accudnn.h"
#include "dtype.h"
#include "kernels.h"

using namespace acc;

namespace {

constexpr int kMaxChannels = ACC_NOALLOC_BN_MAX_C;
// layout of bn_workspace_bytes(): double part[2][kBnMaxSlabs][c] | float coef[4][c]
constexpr size_t kScratchBytes =
    (size_t)2 * kBnMaxSlabs * kMaxChannels * sizeof(double) + (size_t)4 * kMaxChannels * sizeof(float);

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_lock;
void* g_scratch_ptr[kMaxDevices] = {};

// device address of this GPU's copy of the array, looked up on first use
hipError_t scratch_address(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> hold(g_lock);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

}  // namespace

extern "C" int acc_op_bn_fwd_noalloc(const void* x, const float* gamma, const float* beta, const void* res, void* y,
                                     float* mean, float* istd, int rows, int c, int relu, float eps, int dtype,
                                     void* stream) {
  if (dtype != ACC_F32 && dtype != ACC_BF16) {
    set_thread_error("acc_op_bn_fwd_noalloc: dtype must be ACC_F32 or ACC_BF16");
    return ACC_EINVAL;
  }
  if (c <= 0 || c > kMaxChannels) {
    set_thread_error("acc_op_bn_fwd_noalloc: the built-in workspace holds at most ACC_NOALLOC_BN_MAX_C channels");
    return ACC_EINVAL;
  }
  if (bn_workspace_bytes(c) > kScratchBytes) {   // (cannot happen while the layout above is the launcher's)
    set_thread_error("acc_op_bn_fwd_noalloc: workspace layout outgrew the built-in array");
    return ACC_EINVAL;
  }
  for (const void* p : {x, (const void*)gamma, (const void*)beta, res, (const void*)y, (const void*)mean, (const void*)istd})
    if (reinterpret_cast<uintptr_t>(p) & 15) {
      set_thread_error("acc_op_bn_fwd_noalloc: pointers must be 16-byte aligned");
      return ACC_EINVAL;
    }
  void* ws = nullptr;
  hipError_t e = scratch_address(&ws);
  if (e != hipSuccess) {
    set_thread_error("acc_op_bn_fwd_noalloc: hipGetSymbolAddress failed");
    return ACC_EHIP;
  }
  e = bn_forward(x, gamma, beta, res, y, mean, istd, rows, c, relu, eps, ws, dtype, (hipStream_t)stream);
  if (e == hipSuccess) return ACC_OK;
  set_thread_error(e == hipErrorInvalidValue ? "acc_op_bn_fwd_noalloc: null pointer, rows <= 0 or c not a multiple of 4"
                                             : hipGetErrorString(e));
  return e == hipErrorInvalidValue ? ACC_EINVAL : ACC_EHIP;
}
