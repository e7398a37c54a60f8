// Launchers of the gfx950 kernels.  Every launcher checks that its operand shapes
// fit what the kernel and its grid assume and returns hipErrorInvalidValue otherwise;
// nothing here allocates.  Activations NHWC, filters O-H-W-I (K-contiguous rows); `dtype`
// (DT_F32 / DT_BF16 of dtype.h, the values of ACC_F32 / ACC_BF16) is the storage type of
// activations, activation gradients and of the filter copy the kernels read; arithmetic is
// fp32 (bf16 products on the matrix cores accumulate in fp32), weight gradients, batch-norm
// parameters and statistics, biases and the loss are always fp32.
#pragma once
#include <hip/hip_runtime.h>
#include <cstddef>
#include <cstdint>

#include "dgrad_split.h"

namespace acc {

// A weight-gradient reduction that has not been launched yet: dw[i] = part[0][i] + part[1][i]
// + ... (count elements, `splits` parts, in that order).  count == 0: nothing to do.
struct ReduceJob {
  const float* part;
  float* dw;
  size_t count;
  int splits;
};

// A filter to flip and transpose on the side of another launch (storage type of that launch):
// wt[ci][r'][t'][co] = w[co][R-1-r'][S-1-t'][ci].  wt == nullptr: nothing to do.
struct FlipJob {
  const void* w;
  void* wt;
  int cout, cin, r, s;
};

// Optional work of a data-gradient launch for the batch norm (with ReLU) whose output was the
// convolution's input: the result is the gradient of that output, so the launch masks it with
// [y > 0] before storing it and leaves, per block of 32 rows and per channel, the sums of the
// masked gradient g and of g * xhat (xhat = (x - mean) * istd) in sums[2][stride][n_out]
// (floats; stride >= conv_stat_slabs(rows)).  x, y: the batch norm's input and output, laid
// out like the launch's dense output.  sums == nullptr: off.
struct BnBackwardSums {
  const void* x;
  const void* y;
  const float* mean;
  const float* istd;
  float* sums;
  int stride;
};

// Implicit-GEMM view of a convolution-like gather:
//   out[m][n] (+)= sum_{r,t,c} in[img, p*stride+r-pad, q*stride+t-pad, c] * w[n][(r,t,c)]
// with row m = (img, p, q) over a P x Q grid (columns use pad + pad_dx).  The result row is
// written to pixel (out_y0 + p*out_stride, out_x0 + q*out_stride) of an out_h x out_w image
// with `n_out` channels.
struct ConvGeom {
  const void* in;           // dtype
  const void* w;            // dtype
  void* out;                // dtype
  int dtype;
  int n_img, h, wd, c;      // input image size and channels
  int p, q;                 // rows enumerate n_img x p x q positions
  int n_out;                // GEMM N (output channels)
  int r, s, stride, pad;
  int pad_dx;               // column padding is pad + pad_dx (>= 0)
  int out_h, out_w, out_stride;
  int out_y0, out_x0;       // first output pixel
  int accumulate;           // out += result
  const float* bias;        // optional: + bias[n] (fp32), then
  int relu;                 // ... max(., 0) if set; both only without accumulate
  // Optional side jobs: extra workgroups appended to the launch add up the parts of a weight
  // gradient, and / or write the flipped, transposed filter that a later data gradient needs
  // (independent data; saves launches of their own).
  ReduceJob side;
  FlipJob flip;
  // Optional (fp32 storage, plain dense output): per-channel sums of the result and of its
  // square over every block of 32 rows, as the batch norm that follows wants them:
  // stats[0][b][n] = sum, stats[1][b][n] = sum of squares, b < conv_stat_slabs(rows), layout
  // float[2][stats_stride][n_out] with stats_stride >= conv_stat_slabs(rows).
  float* stats;
  int stats_stride;
  BnBackwardSums bnb;   // fp32 storage, plain dense output, no accumulation
};
// Largest number of row slabs a batch-norm statistics pass adds up.
constexpr int kBnMaxSlabs = 1024;
// Number of 32-row blocks conv_igemm writes sums for (2 per 64-row tile).
inline long conv_stat_slabs(long rows) { return ((rows + 63) / 64) * 2; }
// Partial sums a convolution launch has left for a batch norm: float part[2][stride][c], `slabs` of
// them valid (each the fp32 sum over one block of 32 rows).
struct BnSums {
  const float* part;
  int slabs, stride;
};

// Optional probe of one launch: which template instance ran (index into conv_variant_name())
// and, when the two events are set, timestamps recorded directly around the main kernel.
struct LaunchProbe {
  int variant = -1;
  hipEvent_t before = nullptr, after = nullptr;
};
hipError_t conv_igemm(const ConvGeom& g, hipStream_t st, LaunchProbe* probe = nullptr);
// The 128 x 128 kernel for bf16 storage (conv_igemm_bf16.hip): whether it takes this launch (a
// function of the shape and the alignment only), and the launch itself; conv_igemm() routes to it.
bool conv_igemm_bf16_takes(const ConvGeom& g, long M, long K);
hipError_t conv_igemm_bf16(const ConvGeom& g, int M, int K, hipStream_t st, const LaunchProbe* probe);
enum { V_IGEMM_FAST = 0, V_IGEMM_GENERIC, V_WGRAD_FAST, V_WGRAD_GENERIC, V_IGEMM_DIRECT, V_WGRAD_DIRECT, V_WGRAD_BF16,
       V_IGEMM_BF16, V_IGEMM_DIRECT_2G, V_COUNT };
const char* conv_variant_name(int v);

// dw[co][(r,t,ci)] = sum_{img,p,q} dy[img,p,q,co] * x[img, p*stride+r-pad, q*stride+t-pad, ci]
struct WgradGeom {
  const void* x;            // dtype
  const void* dy;           // dtype
  float* dw;                // fp32
  int dtype;
  int n_img, h, wd, cin;
  int p, q, cout;
  int r, s, stride, pad;
  float* workspace;         // split-K partials, wgrad_workspace_bytes() bytes (may be null if 0)
  // Optional side job: extra workgroups appended to the launch write the flipped and
  // transposed filter wt[ci][r'][t'][co] = w[co][R-1-r'][S-1-t'][ci] of this layer (the data
  // gradient that follows needs it).  Both null: no side job.
  const void* flip_w;       // dtype
  void* flip_wt;            // dtype
  // Optional side job: extra workgroups add up the parts of an earlier weight gradient.
  ReduceJob side;
};
// dtype: DT_F32 / DT_BF16 (the two storage types cut the minibatch range differently), or -1 = the
// larger of the two
size_t wgrad_workspace_bytes(int n_img, int p, int q, int cin, int cout, int r, int s, int dtype);
// If `deferred` is given and the gradient is split over the minibatch, the reduction of the
// parts is not launched but described there (the caller appends it to a later launch or
// runs reduce_parts); otherwise dw is complete when the stream reaches the end of this call.
hipError_t conv_wgrad(const WgradGeom& g, hipStream_t st, LaunchProbe* probe = nullptr,
                      ReduceJob* deferred = nullptr);
hipError_t reduce_parts(const ReduceJob& job, hipStream_t st);

// wt[ci][r'][t'][co] = w[co][R-1-r'][S-1-t'][ci]  (filter of the transposed convolution)
hipError_t filter_flip_transpose(const void* w, void* wt, int cout, int cin, int r, int s, int dtype,
                                 hipStream_t st);

// Sub-filter of one residue class of a strided data gradient (see dgrad_split.h), written at
// wt + part.wt_offset.
hipError_t filter_gather_transpose(const void* w, void* wt, int cout, int cin, int r, int s, int stride,
                                   const DgradPart& part, int dtype, hipStream_t st);

// Batch norm over rows x c (NHWC flattened).  workspace: bn_workspace_bytes(c).
// x, res, y, dy, dx, g_out: dtype; gamma, beta, mean, istd, dgamma, dbeta: fp32.
size_t bn_workspace_bytes(int c);
// ready_sums (may be null): the partial sums of x and x*x are already there (conv_igemm wrote
// them, ConvGeom::stats) and are not computed again.
hipError_t bn_forward(const void* x, const float* gamma, const float* beta, const void* res,
                      void* y, float* mean, float* istd, long rows, int c, int relu, float eps,
                      void* workspace, int dtype, hipStream_t st, const BnSums* ready_sums = nullptr);
// ready_sums (may be null): the sums of g and g * xhat are already there (a data-gradient launch
// wrote them, ConvGeom::bnb, and masked dy); they are not computed again, and y must be null.
hipError_t bn_backward(const void* x, const void* dy, const void* y, const float* gamma,
                       const float* mean, const float* istd, void* dx, float* dgamma, float* dbeta,
                       void* g_out, long rows, int c, void* workspace, int dtype, hipStream_t st,
                       const BnSums* ready_sums = nullptr);

hipError_t maxpool_forward(const void* x, void* y, int n, int h, int wd, int c, int r, int s,
                           int stride, int pad, int dtype, hipStream_t st);
hipError_t maxpool_backward(const void* x, const void* dy, void* dx, int n, int h, int wd, int c,
                            int r, int s, int stride, int pad, int accumulate, int dtype, hipStream_t st);
hipError_t gap_forward(const void* x, void* y, int n, int hw, int c, int dtype, hipStream_t st);
hipError_t gap_backward(const void* dy, void* dx, int n, int hw, int c, int accumulate, int dtype,
                        hipStream_t st);
// y[row][ch] += b[ch], then max(., 0) if relu
hipError_t bias_add(void* y, const float* b, long rows, int c, int dtype, hipStream_t st, int relu = 0);
// Backward of y = relu(x + b) over rows x c (c % 4 == 0): g = dy * [y > 0] is written over dy (y may
// be null: no mask, dy untouched) and db[ch] = sum over the rows of g (fixed order).
// workspace: relu_bias_workspace_bytes(c) bytes.
size_t relu_bias_workspace_bytes(int c);
// dy[i] = y[i] > 0 ? dy[i] : 0, in place
hipError_t relu_mask(void* dy, const void* y, size_t count, int dtype, hipStream_t st);
hipError_t relu_bias_backward(void* dy, const void* y, float* db, long rows, int c, void* workspace, int dtype,
                              hipStream_t st);
hipError_t column_sum(const void* dy, float* db, long rows, int c, int dtype, hipStream_t st);
// loss_rows: n floats of scratch; loss: one float
hipError_t softmax_ce_forward(const void* z, const int32_t* labels, float* loss_rows, float* loss,
                              int n, int classes, int dtype, hipStream_t st);
hipError_t softmax_ce_backward(const void* z, const int32_t* labels, void* dz, int n, int classes,
                               int dtype, hipStream_t st);
// w <- w - lr * g (fp32); w_bf16 (may be null): rounded copy of the updated weights
hipError_t sgd_update(float* w, const float* g, float lr, size_t count, void* w_bf16, hipStream_t st);
hipError_t fill_zero(float* p, size_t count, hipStream_t st);
// y[n][hw][c] (dtype) = x[n][c][hw] (fp32)
hipError_t nchw_to_nhwc(const float* x, void* y, int n, int c, int hw, int dtype, hipStream_t st);

// Text that acc_last_error(NULL) returns on this thread (calls that have no context).
void set_thread_error(const char* text);

}  // namespace acc
