// Single-operation entry points of the C ABI: thin argument checks around the kernel
// launchers, for per-layer parity tests and roofline measurements.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <initializer_list>

#include "../../include/accudnn.h"
#include "kernels.h"
#include "dtype.h"

using namespace acc;

namespace {
inline size_t al256(size_t b) { return (b + 255) & ~(size_t)255; }
inline int out_dim(int in, int r, int stride, int pad) { return (in + 2 * pad - r) / stride + 1; }
inline bool conv_ok(int n, int h, int w, int cin, int cout, int r, int s, int stride, int pad) {
  return n > 0 && h > 0 && w > 0 && cin > 0 && cout > 0 && r > 0 && s == r && stride > 0 && pad >= 0 && pad < r &&
         h + 2 * pad >= r && w + 2 * pad >= s;
}
inline bool dtype_ok(int dt) { return dt == ACC_F32 || dt == ACC_BF16; }
// the kernels move 16 bytes at a time: null is let through here (checked where it matters)
inline bool al16(std::initializer_list<const void*> ps) {
  for (const void* p : ps) if (reinterpret_cast<uintptr_t>(p) & 15) return false;
  return true;
}
inline int status(hipError_t e) { return e == hipSuccess ? ACC_OK : (e == hipErrorInvalidValue ? ACC_EINVAL : ACC_EHIP); }
}  // namespace

extern "C" size_t acc_op_conv_workspace(int n, int h, int w, int cin, int cout, int r, int s, int stride, int pad) {
  if (!conv_ok(n, h, w, cin, cout, r, s, stride, pad)) return 0;
  const int ho = out_dim(h, r, stride, pad), wo = out_dim(w, s, stride, pad);
  // the sub-filters of a strided data gradient are aligned one by one
  return al256(wgrad_workspace_bytes(n, ho, wo, cin, cout, r, s, -1)) + al256((size_t)cout * cin * r * s * sizeof(float)) +
         (stride > 1 ? kMaxDgradParts * 256 : 0);
}

extern "C" int acc_op_conv_fwd(const void* x, const void* w, void* y, int n, int h, int wd, int cin, int cout,
                               int r, int s, int stride, int pad, int dtype, void* stream) {
  if (!x || !w || !y || !dtype_ok(dtype) || !conv_ok(n, h, wd, cin, cout, r, s, stride, pad)) return ACC_EINVAL;
  if (!al16({x, w, y})) return ACC_EINVAL;
  ConvGeom g{};
  g.in = x; g.w = w; g.out = y; g.dtype = dtype;
  g.n_img = n; g.h = h; g.wd = wd; g.c = cin;
  g.p = out_dim(h, r, stride, pad); g.q = out_dim(wd, s, stride, pad); g.n_out = cout;
  g.r = r; g.s = s; g.stride = stride; g.pad = pad;
  g.out_h = g.p; g.out_w = g.q; g.out_stride = 1;
  return status(conv_igemm(g, (hipStream_t)stream));
}

extern "C" int acc_op_conv_dgrad(const void* dy, const void* w, void* dx, int n, int h, int wd, int cin, int cout,
                                 int r, int s, int stride, int pad, int accumulate, void* workspace,
                                 size_t workspace_bytes, int dtype, void* stream) {
  if (!dy || !w || !dx || !dtype_ok(dtype) || !conv_ok(n, h, wd, cin, cout, r, s, stride, pad)) return ACC_EINVAL;
  if (!al16({dy, w, dx, workspace})) return ACC_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  const int ho = out_dim(h, r, stride, pad), wo = out_dim(wd, s, stride, pad);
  hipError_t e;
  if (stride > 1 && (r > 1 || pad > 0)) {
    // one stride-1 convolution per residue class of the dx position
    DgradPart parts[kMaxDgradParts];
    bool covers_all = false;
    size_t wt_bytes = 0;
    const int np = dgrad_split(h, wd, cin, cout, r, s, stride, pad, (int)dt_size(dtype), parts, &covers_all, &wt_bytes);
    if (np < 0 || !workspace || workspace_bytes < wt_bytes) return ACC_EINVAL;
    if (!covers_all && !accumulate) {
      const size_t bytes = (size_t)n * h * wd * cin * dt_size(dtype);
      if (bytes % 4) return ACC_EINVAL;
      if ((e = fill_zero((float*)dx, bytes / 4, st)) != hipSuccess) return status(e);
    }
    for (int i = 0; i < np; ++i) {
      const DgradPart& pt = parts[i];
      if ((e = filter_gather_transpose(w, workspace, cout, cin, r, s, stride, pt, dtype, st)) != hipSuccess) return status(e);
      ConvGeom g{};
      g.in = dy; g.w = (const char*)workspace + pt.wt_offset; g.out = dx; g.dtype = dtype;
      g.n_img = n; g.h = ho; g.wd = wo; g.c = cout; g.n_out = cin;
      g.p = pt.p; g.q = pt.q; g.r = pt.nr; g.s = pt.ns; g.stride = 1; g.pad = pt.pad_y; g.pad_dx = pt.pad_x - pt.pad_y;
      g.out_h = h; g.out_w = wd; g.out_stride = stride; g.out_y0 = pt.y0; g.out_x0 = pt.x0;
      g.accumulate = accumulate;
      if ((e = conv_igemm(g, st)) != hipSuccess) return status(e);
    }
    return ACC_OK;
  }
  const size_t filt = al256((size_t)cout * cin * r * s * sizeof(float));
  if (!workspace || workspace_bytes < filt) return ACC_EINVAL;
  void* wt = workspace;
  e = filter_flip_transpose(w, wt, cout, cin, r, s, dtype, st);
  if (e != hipSuccess) return status(e);
  ConvGeom g{};
  g.in = dy; g.w = wt; g.out = dx; g.dtype = dtype;
  g.n_img = n; g.h = ho; g.wd = wo; g.c = cout; g.n_out = cin;
  g.r = r; g.s = s; g.stride = 1; g.accumulate = accumulate;
  g.out_h = h; g.out_w = wd;
  if (stride == 1) {
    g.p = h; g.q = wd; g.pad = r - 1 - pad; g.out_stride = 1;
  } else {
    g.p = ho; g.q = wo; g.pad = 0; g.out_stride = stride;
    if (!accumulate) {
      const size_t bytes = (size_t)n * h * wd * cin * dt_size(dtype);
      if (bytes % 4) return ACC_EINVAL;
      e = fill_zero((float*)dx, bytes / 4, st);
      if (e != hipSuccess) return status(e);
    }
  }
  return status(conv_igemm(g, st));
}

extern "C" int acc_op_conv_wgrad(const void* x, const void* dy, float* dw, int n, int h, int wd, int cin, int cout,
                                 int r, int s, int stride, int pad, void* workspace, size_t workspace_bytes,
                                 int dtype, void* stream) {
  if (!x || !dy || !dw || !dtype_ok(dtype) || !conv_ok(n, h, wd, cin, cout, r, s, stride, pad)) return ACC_EINVAL;
  if (!al16({x, dy, dw, workspace})) return ACC_EINVAL;
  const int ho = out_dim(h, r, stride, pad), wo = out_dim(wd, s, stride, pad);
  const size_t need = wgrad_workspace_bytes(n, ho, wo, cin, cout, r, s, dtype);
  if (need && (!workspace || workspace_bytes < need)) return ACC_EINVAL;
  WgradGeom g{};
  g.x = x; g.dy = dy; g.dw = dw; g.dtype = dtype;
  g.n_img = n; g.h = h; g.wd = wd; g.cin = cin; g.p = ho; g.q = wo; g.cout = cout;
  g.r = r; g.s = s; g.stride = stride; g.pad = pad; g.workspace = (float*)workspace;
  return status(conv_wgrad(g, (hipStream_t)stream));
}

extern "C" size_t acc_op_bn_workspace(int c) { return c > 0 ? al256(bn_workspace_bytes(c)) : 0; }

extern "C" int acc_op_bn_fwd(const void* x, const float* gamma, const float* beta, const void* res, void* y,
                             float* mean, float* istd, int rows, int c, int relu, float eps, void* workspace,
                             int dtype, void* stream) {
  if (!dtype_ok(dtype) || !al16({x, gamma, beta, res, y, mean, istd, workspace})) return ACC_EINVAL;
  return status(bn_forward(x, gamma, beta, res, y, mean, istd, rows, c, relu, eps, workspace, dtype,
                           (hipStream_t)stream));
}

extern "C" int acc_op_bn_bwd(const void* x, const void* dy, const void* y, const float* gamma, const float* mean,
                             const float* istd, void* dx, float* dgamma, float* dbeta, void* g_out, int rows, int c,
                             void* workspace, int dtype, void* stream) {
  if (!dtype_ok(dtype) || !al16({x, dy, y, gamma, mean, istd, dx, dgamma, dbeta, g_out, workspace})) return ACC_EINVAL;
  return status(bn_backward(x, dy, y, gamma, mean, istd, dx, dgamma, dbeta, g_out, rows, c, workspace, dtype,
                            (hipStream_t)stream));
}

extern "C" int acc_op_maxpool_fwd(const void* x, void* y, int n, int h, int wd, int c, int r, int stride, int pad,
                                  int dtype, void* stream) {
  if (!x || !y || !dtype_ok(dtype) || !al16({x, y})) return ACC_EINVAL;
  return status(maxpool_forward(x, y, n, h, wd, c, r, r, stride, pad, dtype, (hipStream_t)stream));
}

extern "C" int acc_op_maxpool_bwd(const void* x, const void* dy, void* dx, int n, int h, int wd, int c, int r,
                                  int stride, int pad, int accumulate, int dtype, void* stream) {
  if (!x || !dy || !dx || !dtype_ok(dtype) || !al16({x, dy, dx})) return ACC_EINVAL;
  return status(maxpool_backward(x, dy, dx, n, h, wd, c, r, r, stride, pad, accumulate, dtype, (hipStream_t)stream));
}

extern "C" int acc_op_gap_fwd(const void* x, void* y, int n, int hw, int c, int dtype, void* stream) {
  if (!x || !y || !dtype_ok(dtype)) return ACC_EINVAL;
  return status(gap_forward(x, y, n, hw, c, dtype, (hipStream_t)stream));
}

extern "C" int acc_op_gap_bwd(const void* dy, void* dx, int n, int hw, int c, int accumulate, int dtype, void* stream) {
  if (!dy || !dx || !dtype_ok(dtype)) return ACC_EINVAL;
  return status(gap_backward(dy, dx, n, hw, c, accumulate, dtype, (hipStream_t)stream));
}

extern "C" int acc_op_softmax_ce(const void* z, const int32_t* labels, float* loss_rows, float* loss, void* dz, int n,
                                 int classes, int dtype, void* stream) {
  if (!z || !labels || !dtype_ok(dtype) || n <= 0 || classes <= 0 || (!loss_rows && !dz) || (loss_rows && !loss))
    return ACC_EINVAL;
  hipError_t e = hipSuccess;
  if (loss_rows) e = softmax_ce_forward(z, labels, loss_rows, loss, n, classes, dtype, (hipStream_t)stream);
  if (e == hipSuccess && dz) e = softmax_ce_backward(z, labels, dz, n, classes, dtype, (hipStream_t)stream);
  return status(e);
}
