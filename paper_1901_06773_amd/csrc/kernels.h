// Launchers of the gfx950 kernels.  Every launcher checks that its operand shapes
// fit what the kernel and its grid assume and returns hipErrorInvalidValue otherwise;
// nothing here allocates.  All activations NHWC fp32, filters O-H-W-I (K-contiguous rows).
#pragma once
#include <hip/hip_runtime.h>
#include <cstddef>
#include <cstdint>

namespace acc {

// Implicit-GEMM view of a convolution-like gather:
//   out[m][n] (+)= sum_{r,t,c} in[img, p*stride+r-pad, q*stride+t-pad, c] * w[n][(r,t,c)]
// with row m = (img, p, q) over a P x Q grid.  The result row is written to pixel
// (p*out_stride, q*out_stride) of an out_h x out_w image with `n_out` channels.
// A weight-gradient reduction that has not been launched yet: dw[i] = part[0][i] + part[1][i]
// + ... (count elements, `splits` parts, in that order).  count == 0: nothing to do.
struct ReduceJob {
  const float* part;
  float* dw;
  size_t count;
  int splits;
};

struct ConvGeom {
  const float* in;
  const float* w;
  float* out;
  int n_img, h, wd, c;      // input image size and channels
  int p, q;                 // rows enumerate n_img x p x q positions
  int n_out;                // GEMM N (output channels)
  int r, s, stride, pad;
  int out_h, out_w, out_stride;
  int accumulate;           // out += result
  // Optional side job: extra workgroups appended to the launch add up the parts of a weight
  // gradient (independent data; saves a launch of its own).
  ReduceJob side;
};

// Optional probe of one launch: which template instance ran (index into conv_variant_name())
// and, when the two events are set, timestamps recorded directly around the main kernel.
struct LaunchProbe {
  int variant = -1;
  hipEvent_t before = nullptr, after = nullptr;
};
hipError_t conv_igemm(const ConvGeom& g, hipStream_t st, LaunchProbe* probe = nullptr);
enum { V_IGEMM_FAST = 0, V_IGEMM_GENERIC, V_WGRAD_FAST, V_WGRAD_GENERIC, V_COUNT };
const char* conv_variant_name(int v);

// dw[co][(r,t,ci)] = sum_{img,p,q} dy[img,p,q,co] * x[img, p*stride+r-pad, q*stride+t-pad, ci]
struct WgradGeom {
  const float* x;
  const float* dy;
  float* dw;
  int n_img, h, wd, cin;
  int p, q, cout;
  int r, s, stride, pad;
  float* workspace;         // split-K partials, wgrad_workspace_bytes() bytes (may be null if 0)
  // Optional side job: extra workgroups appended to the launch write the flipped and
  // transposed filter wt[ci][r'][t'][co] = w[co][R-1-r'][S-1-t'][ci] of this layer (the data
  // gradient that follows needs it).  Both null: no side job.
  const float* flip_w;
  float* flip_wt;
};
size_t wgrad_workspace_bytes(int n_img, int p, int q, int cin, int cout, int r, int s);
// If `deferred` is given and the gradient is split over the minibatch, the reduction of the
// parts is not launched but described there (the caller appends it to a later launch or
// runs reduce_parts); otherwise dw is complete when the stream reaches the end of this call.
hipError_t conv_wgrad(const WgradGeom& g, hipStream_t st, LaunchProbe* probe = nullptr,
                      ReduceJob* deferred = nullptr);
hipError_t reduce_parts(const ReduceJob& job, hipStream_t st);

// wt[ci][r'][t'][co] = w[co][R-1-r'][S-1-t'][ci]  (filter of the transposed convolution)
hipError_t filter_flip_transpose(const float* w, float* wt, int cout, int cin, int r, int s,
                                 hipStream_t st);

// Batch norm over rows x c (NHWC flattened).  workspace: bn_workspace_bytes(c).
size_t bn_workspace_bytes(int c);
hipError_t bn_forward(const float* x, const float* gamma, const float* beta, const float* res,
                      float* y, float* mean, float* istd, long rows, int c, int relu, float eps,
                      void* workspace, hipStream_t st);
hipError_t bn_backward(const float* x, const float* dy, const float* y, const float* gamma,
                       const float* mean, const float* istd, float* dx, float* dgamma, float* dbeta,
                       float* g_out, long rows, int c, void* workspace, hipStream_t st);

hipError_t maxpool_forward(const float* x, float* y, int n, int h, int wd, int c, int r, int s,
                           int stride, int pad, hipStream_t st);
hipError_t maxpool_backward(const float* x, const float* dy, float* dx, int n, int h, int wd, int c,
                            int r, int s, int stride, int pad, int accumulate, hipStream_t st);
hipError_t gap_forward(const float* x, float* y, int n, int hw, int c, hipStream_t st);
hipError_t gap_backward(const float* dy, float* dx, int n, int hw, int c, int accumulate,
                        hipStream_t st);
hipError_t bias_add(float* y, const float* b, long rows, int c, hipStream_t st);
hipError_t column_sum(const float* dy, float* db, long rows, int c, hipStream_t st);
// loss_rows: n floats of scratch; loss: one float
hipError_t softmax_ce_forward(const float* z, const int32_t* labels, float* loss_rows, float* loss,
                              int n, int classes, hipStream_t st);
hipError_t softmax_ce_backward(const float* z, const int32_t* labels, float* dz, int n, int classes,
                               hipStream_t st);
hipError_t sgd_update(float* w, const float* g, float lr, size_t count, hipStream_t st);
hipError_t fill_zero(float* p, size_t count, hipStream_t st);
// y[n][hw][c] = x[n][c][hw]
hipError_t nchw_to_nhwc(const float* x, float* y, int n, int c, int hw, hipStream_t st);

}  // namespace acc
