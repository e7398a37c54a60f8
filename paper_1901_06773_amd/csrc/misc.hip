// The small kernels that close the training step: filter flip/transposition for the data
// gradient, max-pooling, global average pooling, bias, softmax cross-entropy, SGD.
// None of them is on the roofline-critical path; all are coalesced along the channel
// axis of NHWC and use fixed-order reductions.
#include "kernels.h"
#include "dtype.h"
#include "dgrad_split.h"

namespace acc {
namespace {

constexpr int THREADS = 256;

inline unsigned grid_for(size_t work, size_t cap = 256 * 32) {
  size_t b = (work + THREADS - 1) / THREADS;
  if (b < 1) b = 1;
  return (unsigned)(b < cap ? b : cap);
}

// wt[ci][r'][t'][co] = w[co][R-1-r'][S-1-t'][ci]; a 32x32 LDS tile transposes (co, ci)
// so that both the read (ci fastest) and the write (co fastest) are coalesced.
template <class T>
__global__ __launch_bounds__(256) void flip_transpose_kernel(const T* __restrict__ w,
                                                             T* __restrict__ wt, int cout, int cin,
                                                             int r, int s) {
  __shared__ T tile[32][33];
  const int tap = blockIdx.z;                       // r'*s + t' of the output
  const int kr = r - 1 - tap / s, kt = s - 1 - tap % s;
  const int src_tap = kr * s + kt;
  const int co0 = blockIdx.y * 32, ci0 = blockIdx.x * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
  for (int i = ty; i < 32; i += 8) {
    const int co = co0 + i, ci = ci0 + tx;
    tile[i][tx] = (co < cout && ci < cin) ? w[((size_t)co * r * s + src_tap) * cin + ci] : T(0);
  }
  __syncthreads();
  for (int i = ty; i < 32; i += 8) {
    const int ci = ci0 + i, co = co0 + tx;
    if (ci < cin && co < cout) wt[((size_t)ci * r * s + tap) * cout + co] = tile[tx][i];
  }
}

// wt[ci][r'][t'][co] = w[co][r0 + (nr-1-r')*step][t0 + (ns-1-t')*step][ci]: the sub-filter of one
// residue class of a strided data gradient; same tiling as above.
template <class T>
__global__ __launch_bounds__(256) void gather_transpose_kernel(const T* __restrict__ w,
                                                               T* __restrict__ wt, int cout, int cin,
                                                               int r, int s, int nr, int ns, int r0,
                                                               int t0, int step) {
  __shared__ T tile[32][33];
  const int tap = blockIdx.z;                       // r'*ns + t' of the output
  const int kr = r0 + (nr - 1 - tap / ns) * step, kt = t0 + (ns - 1 - tap % ns) * step;
  const int src_tap = kr * s + kt;
  const int co0 = blockIdx.y * 32, ci0 = blockIdx.x * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
  for (int i = ty; i < 32; i += 8) {
    const int co = co0 + i, ci = ci0 + tx;
    tile[i][tx] = (co < cout && ci < cin) ? w[((size_t)co * r * s + src_tap) * cin + ci] : T(0);
  }
  __syncthreads();
  for (int i = ty; i < 32; i += 8) {
    const int ci = ci0 + i, co = co0 + tx;
    if (ci < cin && co < cout) wt[((size_t)ci * nr * ns + tap) * cout + co] = tile[tx][i];
  }
}

// one thread per (n, p, q, 4 channels); the first maximum in (r, t) scan order wins
template <class T>
__global__ __launch_bounds__(THREADS) void maxpool_fwd_kernel(const T* __restrict__ x,
                                                              T* __restrict__ y, int n, int h, int wd,
                                                              int c, int r, int s, int stride, int pad,
                                                              int ho, int wo) {
  const int cg = c >> 2;
  const size_t total = (size_t)n * ho * wo * cg;
  for (size_t i = (size_t)blockIdx.x * THREADS + threadIdx.x; i < total; i += (size_t)gridDim.x * THREADS) {
    const int g = (int)(i % cg);
    size_t rest = i / cg;
    const int q = (int)(rest % wo); rest /= wo;
    const int p = (int)(rest % ho);
    const int img = (int)(rest / ho);
    float best[4] = {0.f, 0.f, 0.f, 0.f};
    bool have = false;
    for (int kr = 0; kr < r; ++kr) {
      const int iy = p * stride + kr - pad;
      if ((unsigned)iy >= (unsigned)h) continue;
      for (int kt = 0; kt < s; ++kt) {
        const int ix = q * stride + kt - pad;
        if ((unsigned)ix >= (unsigned)wd) continue;
        float v[4];
        Elem<T>::load4(x + ((size_t)(img * h + iy) * wd + ix) * c + g * 4, v);
#pragma unroll
        for (int j = 0; j < 4; ++j) best[j] = (!have || v[j] > best[j]) ? v[j] : best[j];
        have = true;
      }
    }
    Elem<T>::store4(y + i * 4, best);
  }
}

// Gather form of the max-pool gradient: one thread per input position and group of V
// channels (V = 4 as float4 when c % 4 == 0, else 1); for every window that covers the
// position, find the window's first maximum again and take the window's dy where this
// position is the winner.  Windows are visited in (p, q) order, so the sum has a fixed order.
template <class T, int V>
__global__ __launch_bounds__(THREADS) void maxpool_bwd_kernel(const T* __restrict__ x,
                                                              const T* __restrict__ dy, T* dx,
                                                              int n, int h, int wd, int c, int r, int s,
                                                              int stride, int pad, int ho, int wo,
                                                              int accumulate) {
  struct Vec { float v[V]; };
  auto ld = [](const T* p) { Vec r; if constexpr (V == 4) Elem<T>::load4(p, r.v); else r.v[0] = Elem<T>::load(p); return r; };
  auto st = [](T* p, const Vec& r) { if constexpr (V == 4) Elem<T>::store4(p, r.v); else Elem<T>::store(p, r.v[0]); };
  const int cg = c / V;
  const size_t total = (size_t)n * h * wd * cg;
  for (size_t i = (size_t)blockIdx.x * THREADS + threadIdx.x; i < total; i += (size_t)gridDim.x * THREADS) {
    const int g = (int)(i % cg);
    size_t rest = i / cg;
    const int ix = (int)(rest % wd); rest /= wd;
    const int iy = (int)(rest % h);
    const int img = (int)(rest / h);
    const int me = iy * wd + ix;
    // windows p with p*stride - pad <= iy <= p*stride - pad + r - 1
    int p_lo = (iy + pad - r + 1 + stride - 1);
    p_lo = p_lo > 0 ? p_lo / stride : 0;
    int p_hi = (iy + pad) / stride; if (p_hi > ho - 1) p_hi = ho - 1;
    int q_lo = (ix + pad - s + 1 + stride - 1);
    q_lo = q_lo > 0 ? q_lo / stride : 0;
    int q_hi = (ix + pad) / stride; if (q_hi > wo - 1) q_hi = wo - 1;
    Vec acc;
#pragma unroll
    for (int j = 0; j < V; ++j) acc.v[j] = 0.f;
    for (int p = p_lo; p <= p_hi; ++p)
      for (int q = q_lo; q <= q_hi; ++q) {
        Vec best;
        int at[V];
#pragma unroll
        for (int j = 0; j < V; ++j) { best.v[j] = 0.f; at[j] = -1; }
        for (int kr = 0; kr < r; ++kr) {
          const int yy = p * stride + kr - pad;
          if ((unsigned)yy >= (unsigned)h) continue;
          for (int kt = 0; kt < s; ++kt) {
            const int xx = q * stride + kt - pad;
            if ((unsigned)xx >= (unsigned)wd) continue;
            const Vec v = ld(x + ((size_t)(img * h + yy) * wd + xx) * c + g * V);
#pragma unroll
            for (int j = 0; j < V; ++j)
              if (at[j] < 0 || v.v[j] > best.v[j]) { best.v[j] = v.v[j]; at[j] = yy * wd + xx; }
          }
        }
        const Vec d = ld(dy + ((size_t)(img * ho + p) * wo + q) * c + g * V);
#pragma unroll
        for (int j = 0; j < V; ++j)
          if (at[j] == me) acc.v[j] += d.v[j];
      }
    T* out = dx + i * V;
    if (accumulate) {
      const Vec o = ld(out);
#pragma unroll
      for (int j = 0; j < V; ++j) acc.v[j] = o.v[j] + acc.v[j];
    }
    st(out, acc);
  }
}

// The same for 3x3 windows at stride 2 with padding 1 (the stem pool of the ResNets): one thread
// per 2x2 block of input positions and four channels.  The block (rows 2a, 2a+1, columns 2b,
// 2b+1) is covered by the windows p in {a, a+1}, q in {b, b+1} and by no other, so each
// window's maximum is looked up once for the four positions instead of once per position
// (36 loads for four results instead of 81).  Windows are visited in the same (p, q) order
// and the same first maximum wins, so every sum has the same terms in the same order as in
// the kernel above.
template <class T>
__global__ __launch_bounds__(THREADS) void maxpool3s2_bwd_kernel(const T* __restrict__ x,
                                                                 const T* __restrict__ dy, T* dx, int n,
                                                                 int h, int wd, int c, int ho, int wo,
                                                                 int accumulate) {
  const int cg = c >> 2, hb = (h + 1) >> 1, wb = (wd + 1) >> 1;
  const size_t total = (size_t)n * hb * wb * cg;
  for (size_t i = (size_t)blockIdx.x * THREADS + threadIdx.x; i < total; i += (size_t)gridDim.x * THREADS) {
    const int g = (int)(i % cg);
    size_t rest = i / cg;
    const int b = (int)(rest % wb); rest /= wb;
    const int a = (int)(rest % hb);
    const int img = (int)(rest / hb);
    float acc[2][2][4] = {};
    for (int p = a; p <= a + 1 && p < ho; ++p)
      for (int q = b; q <= b + 1 && q < wo; ++q) {
        float best[4] = {0.f, 0.f, 0.f, 0.f};
        int at[4] = {-1, -1, -1, -1};
#pragma unroll
        for (int kr = 0; kr < 3; ++kr) {
          const int yy = 2 * p + kr - 1;
          if ((unsigned)yy >= (unsigned)h) continue;
#pragma unroll
          for (int kt = 0; kt < 3; ++kt) {
            const int xx = 2 * q + kt - 1;
            if ((unsigned)xx >= (unsigned)wd) continue;
            float v[4];
            Elem<T>::load4(x + ((size_t)(img * h + yy) * wd + xx) * c + g * 4, v);
#pragma unroll
            for (int j = 0; j < 4; ++j)
              if (at[j] < 0 || v[j] > best[j]) { best[j] = v[j]; at[j] = yy * wd + xx; }
          }
        }
        float d[4];
        Elem<T>::load4(dy + ((size_t)(img * ho + p) * wo + q) * c + g * 4, d);
#pragma unroll
        for (int ry = 0; ry < 2; ++ry)
#pragma unroll
          for (int rx = 0; rx < 2; ++rx) {
            const int me = (2 * a + ry) * wd + 2 * b + rx;
#pragma unroll
            for (int j = 0; j < 4; ++j)
              if (at[j] == me) acc[ry][rx][j] += d[j];
          }
      }
#pragma unroll
    for (int ry = 0; ry < 2; ++ry)
#pragma unroll
      for (int rx = 0; rx < 2; ++rx) {
        const int iy = 2 * a + ry, ix = 2 * b + rx;
        if (iy >= h || ix >= wd) continue;
        T* out = dx + ((size_t)(img * h + iy) * wd + ix) * c + g * 4;
        float o[4] = {acc[ry][rx][0], acc[ry][rx][1], acc[ry][rx][2], acc[ry][rx][3]};
        if (accumulate) {
          float old[4];
          Elem<T>::load4(out, old);
#pragma unroll
          for (int j = 0; j < 4; ++j) o[j] = old[j] + o[j];
        }
        Elem<T>::store4(out, o);
      }
  }
}

// y[n][c] = mean over hw of x[n][hw][c]
template <class T>
__global__ __launch_bounds__(THREADS) void gap_fwd_kernel(const T* __restrict__ x, T* __restrict__ y,
                                                          int n, int hw, int c) {
  const size_t total = (size_t)n * c;
  for (size_t i = (size_t)blockIdx.x * THREADS + threadIdx.x; i < total; i += (size_t)gridDim.x * THREADS) {
    const int ch = (int)(i % c);
    const int img = (int)(i / c);
    float sum = 0.f;
    for (int k = 0; k < hw; ++k) sum += Elem<T>::load(x + ((size_t)img * hw + k) * c + ch);
    Elem<T>::store(y + i, sum / (float)hw);
  }
}

template <class T>
__global__ __launch_bounds__(THREADS) void gap_bwd_kernel(const T* __restrict__ dy, T* dx, int n,
                                                          int hw, int c, int accumulate) {
  const size_t total = (size_t)n * hw * c;
  const float inv = 1.f / (float)hw;
  for (size_t i = (size_t)blockIdx.x * THREADS + threadIdx.x; i < total; i += (size_t)gridDim.x * THREADS) {
    const int ch = (int)(i % c);
    const int img = (int)(i / ((size_t)hw * c));
    const float v = Elem<T>::load(dy + (size_t)img * c + ch) * inv;
    Elem<T>::store(dx + i, accumulate ? Elem<T>::load(dx + i) + v : v);
  }
}

template <class T>
__global__ __launch_bounds__(THREADS) void bias_add_kernel(T* y, const float* __restrict__ b, size_t total,
                                                           int c, int relu) {
  for (size_t i = (size_t)blockIdx.x * THREADS + threadIdx.x; i < total; i += (size_t)gridDim.x * THREADS) {
    float v = Elem<T>::load(y + i) + b[i % c];
    if (relu) v = fmaxf(v, 0.f);
    Elem<T>::store(y + i, v);
  }
}

// Backward of y = relu(x + b): a workgroup takes one slab of rows and up to 256 channels (four
// per thread), writes g = dy * [y > 0] over dy and the per-channel sums of g over its slab to
// part[slab][c]; rows of a slab are spread over the threads that share a channel group and
// added in a fixed order.  The second kernel adds the slabs in order.
constexpr int RB_MAX_SLABS = 512;
template <class T>
__global__ __launch_bounds__(THREADS) void relu_bias_bwd_kernel(T* dy, const T* __restrict__ y,
                                                                double* __restrict__ part, long rows, int c,
                                                                int tpr, int rpi, long rows_per_slab) {
  __shared__ double red[THREADS][4];
  const int tid = threadIdx.x;
  const int lane_r = tid / tpr, lane_c = tid - lane_r * tpr;
  const int cg = blockIdx.y * tpr + lane_c;
  const bool active = lane_r < rpi && cg * 4 < c;
  const long r_lo = (long)blockIdx.x * rows_per_slab;
  const long r_hi = r_lo + rows_per_slab < rows ? r_lo + rows_per_slab : rows;
  double s[4] = {0, 0, 0, 0};
  if (active)
    for (long r = r_lo + lane_r; r < r_hi; r += rpi) {
      const size_t off = (size_t)r * c + (size_t)cg * 4;
      float gv[4];
      Elem<T>::load4(dy + off, gv);
      if (y) {
        float yv[4];
        Elem<T>::load4(y + off, yv);
#pragma unroll
        for (int j = 0; j < 4; ++j) gv[j] = yv[j] > 0.f ? gv[j] : 0.f;
        Elem<T>::store4(dy + off, gv);
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) s[j] += (double)gv[j];
    }
#pragma unroll
  for (int j = 0; j < 4; ++j) red[tid][j] = s[j];
  __syncthreads();
  if (lane_r == 0 && cg * 4 < c) {
    for (int rr = 1; rr < rpi; ++rr)
#pragma unroll
      for (int j = 0; j < 4; ++j) s[j] += red[rr * tpr + lane_c][j];
#pragma unroll
    for (int j = 0; j < 4; ++j) part[(size_t)blockIdx.x * c + (size_t)cg * 4 + j] = s[j];
  }
}

template <class T>
__global__ __launch_bounds__(THREADS) void relu_mask_kernel(T* dy, const T* __restrict__ y, size_t count) {
  for (size_t i = (size_t)blockIdx.x * THREADS + threadIdx.x; i < count; i += (size_t)gridDim.x * THREADS)
    if (!(Elem<T>::load(y + i) > 0.f)) Elem<T>::store(dy + i, 0.f);
}

__global__ __launch_bounds__(THREADS) void slab_sum_kernel(const double* __restrict__ part, float* __restrict__ db,
                                                           int slabs, int c) {
  const int ch = blockIdx.x * THREADS + threadIdx.x;
  if (ch >= c) return;
  double sum = 0.0;
  for (int k = 0; k < slabs; ++k) sum += part[(size_t)k * c + ch];
  db[ch] = (float)sum;
}

// db[ch] = sum over rows, one thread per channel, rows in order
template <class T>
__global__ __launch_bounds__(THREADS) void column_sum_kernel(const T* __restrict__ dy,
                                                             float* __restrict__ db, long rows, int c) {
  const int ch = blockIdx.x * THREADS + threadIdx.x;
  if (ch >= c) return;
  float sum = 0.f;
  for (long r = 0; r < rows; ++r) sum += Elem<T>::load(dy + (size_t)r * c + ch);
  db[ch] = sum;
}

// Fixed-order block reductions (tree over a power-of-two block, same order every run).
__device__ __forceinline__ float block_max(float v, float* sh) {
  sh[threadIdx.x] = v;
  __syncthreads();
  for (int s = THREADS / 2; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) sh[threadIdx.x] = fmaxf(sh[threadIdx.x], sh[threadIdx.x + s]);
    __syncthreads();
  }
  const float r = sh[0];
  __syncthreads();
  return r;
}
__device__ __forceinline__ float block_sum(float v, float* sh) {
  sh[threadIdx.x] = v;
  __syncthreads();
  for (int s = THREADS / 2; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) sh[threadIdx.x] += sh[threadIdx.x + s];
    __syncthreads();
  }
  const float r = sh[0];
  __syncthreads();
  return r;
}

// one workgroup per sample: loss_rows[i] = logsumexp(z_i) - z_i[label]; optionally
// dz = (softmax - onehot) / n
template <class T>
__global__ __launch_bounds__(THREADS) void softmax_ce_kernel(const T* __restrict__ z,
                                                             const int32_t* __restrict__ labels,
                                                             float* __restrict__ loss_rows,
                                                             T* __restrict__ dz, int n, int classes) {
  __shared__ float sh[THREADS];
  const int i = blockIdx.x;
  const T* zi = z + (size_t)i * classes;
  float mx = -INFINITY;
  for (int j = threadIdx.x; j < classes; j += THREADS) mx = fmaxf(mx, Elem<T>::load(zi + j));
  mx = block_max(mx, sh);
  float se = 0.f;
  for (int j = threadIdx.x; j < classes; j += THREADS) se += expf(Elem<T>::load(zi + j) - mx);
  se = block_sum(se, sh);
  // everything relative to the row maximum: z - mx is exact for the logits near the maximum (the only ones
  // that matter), so neither the loss nor a probability close to one loses digits to the size of the logits
  const float lg = logf(se);
  const int lab = labels[i];
  // a label outside [0, classes) reads nothing: the row's loss is NaN and its gradient has no one-hot term
  const bool lab_ok = (unsigned)lab < (unsigned)classes;
  if (loss_rows && threadIdx.x == 0) loss_rows[i] = lab_ok ? lg - (Elem<T>::load(zi + lab) - mx) : NAN;
  if (dz) {
    const float inv_n = 1.f / (float)n;
    for (int j = threadIdx.x; j < classes; j += THREADS)
      Elem<T>::store(dz + (size_t)i * classes + j, (expf((Elem<T>::load(zi + j) - mx) - lg) - (j == lab ? 1.f : 0.f)) * inv_n);
  }
}

// loss = (1/n) * sum of rows, added in index order by one wave-sized loop
__global__ void loss_mean_kernel(const float* __restrict__ loss_rows, float* __restrict__ loss, int n) {
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    double s = 0.0;
    for (int i = 0; i < n; ++i) s += (double)loss_rows[i];
    *loss = (float)(s / n);
  }
}

// w <- w - lr * g on the fp32 master weights; in bf16 mode the rounded copy the kernels read is
// refreshed in the same pass
__global__ __launch_bounds__(THREADS) void sgd_kernel(float* __restrict__ w, const float* __restrict__ g,
                                                      float lr, size_t count, bf16_t* __restrict__ w16) {
  for (size_t i = (size_t)blockIdx.x * THREADS + threadIdx.x; i < count; i += (size_t)gridDim.x * THREADS) {
    const float v = fmaf(-lr, g[i], w[i]);
    w[i] = v;
    if (w16) w16[i] = float_to_bf16(v);
  }
}

__global__ __launch_bounds__(THREADS) void fill_zero_kernel(float* __restrict__ p, size_t count) {
  for (size_t i = (size_t)blockIdx.x * THREADS + threadIdx.x; i < count; i += (size_t)gridDim.x * THREADS)
    p[i] = 0.f;
}

// y[n][hw][c] = x[n][c][hw]: reads coalesced along hw for each channel, one pixel per thread
template <class T>
__global__ __launch_bounds__(THREADS) void nchw_to_nhwc_kernel(const float* __restrict__ x, T* __restrict__ y,
                                                               int n, int c, int hw) {
  const size_t total = (size_t)n * hw;
  for (size_t i = (size_t)blockIdx.x * THREADS + threadIdx.x; i < total; i += (size_t)gridDim.x * THREADS) {
    const size_t img = i / hw, pos = i - img * hw;
    const float* src = x + img * (size_t)c * hw + pos;
    T* dst = y + i * c;
    for (int ch = 0; ch < c; ++ch) Elem<T>::store(dst + ch, src[(size_t)ch * hw]);
  }
}

}  // namespace

// runs `call` with T = float or bf16_t according to dtype
#define ACC_DISPATCH(dtype, call)                                   \
  do {                                                              \
    if ((dtype) == DT_F32) { using T = float; call; }               \
    else if ((dtype) == DT_BF16) { using T = bf16_t; call; }        \
    else return hipErrorInvalidValue;                               \
  } while (0)

hipError_t nchw_to_nhwc(const float* x, void* y, int n, int c, int hw, int dtype, hipStream_t st) {
  if (!x || !y || n <= 0 || c <= 0 || hw <= 0) return hipErrorInvalidValue;
  ACC_DISPATCH(dtype, hipLaunchKernelGGL(nchw_to_nhwc_kernel<T>, dim3(grid_for((size_t)n * hw)), dim3(THREADS), 0, st,
                                         x, (T*)y, n, c, hw));
  return hipGetLastError();
}

hipError_t filter_flip_transpose(const void* w, void* wt, int cout, int cin, int r, int s, int dtype,
                                 hipStream_t st) {
  if (!w || !wt || cout <= 0 || cin <= 0 || r <= 0 || s <= 0 || r * s > 65535) return hipErrorInvalidValue;
  const dim3 grid((cin + 31) / 32, (cout + 31) / 32, r * s);
  if (grid.y > 65535) return hipErrorInvalidValue;
  ACC_DISPATCH(dtype, hipLaunchKernelGGL(flip_transpose_kernel<T>, grid, dim3(256), 0, st, (const T*)w, (T*)wt, cout,
                                         cin, r, s));
  return hipGetLastError();
}

hipError_t filter_gather_transpose(const void* w, void* wt, int cout, int cin, int r, int s, int stride,
                                   const DgradPart& pt, int dtype, hipStream_t st) {
  if (!w || !wt || cout <= 0 || cin <= 0 || r <= 0 || s <= 0 || stride <= 0 || pt.nr <= 0 || pt.ns <= 0 ||
      pt.r0 < 0 || pt.t0 < 0 || pt.r0 + (pt.nr - 1) * stride >= r || pt.t0 + (pt.ns - 1) * stride >= s ||
      pt.nr * pt.ns > 65535)
    return hipErrorInvalidValue;
  const dim3 grid((cin + 31) / 32, (cout + 31) / 32, pt.nr * pt.ns);
  if (grid.y > 65535) return hipErrorInvalidValue;
  ACC_DISPATCH(dtype, hipLaunchKernelGGL(gather_transpose_kernel<T>, grid, dim3(256), 0, st, (const T*)w,
                                         (T*)((char*)wt + pt.wt_offset), cout, cin, r, s, pt.nr, pt.ns, pt.r0,
                                         pt.t0, stride));
  return hipGetLastError();
}

hipError_t maxpool_forward(const void* x, void* y, int n, int h, int wd, int c, int r, int s,
                           int stride, int pad, int dtype, hipStream_t st) {
  if (!x || !y || n <= 0 || h <= 0 || wd <= 0 || c <= 0 || (c & 3) || r <= 0 || s <= 0 || stride <= 0 ||
      pad < 0 || pad >= r || pad >= s)
    return hipErrorInvalidValue;
  const int ho = (h + 2 * pad - r) / stride + 1, wo = (wd + 2 * pad - s) / stride + 1;
  if (ho <= 0 || wo <= 0) return hipErrorInvalidValue;
  const size_t total = (size_t)n * ho * wo * (c / 4);
  ACC_DISPATCH(dtype, hipLaunchKernelGGL(maxpool_fwd_kernel<T>, dim3(grid_for(total)), dim3(THREADS), 0, st,
                                         (const T*)x, (T*)y, n, h, wd, c, r, s, stride, pad, ho, wo));
  return hipGetLastError();
}

hipError_t maxpool_backward(const void* x, const void* dy, void* dx, int n, int h, int wd, int c,
                            int r, int s, int stride, int pad, int accumulate, int dtype, hipStream_t st) {
  if (!x || !dy || !dx || n <= 0 || h <= 0 || wd <= 0 || c <= 0 || r <= 0 || s <= 0 || stride <= 0 ||
      pad < 0 || pad >= r || pad >= s)
    return hipErrorInvalidValue;
  const int ho = (h + 2 * pad - r) / stride + 1, wo = (wd + 2 * pad - s) / stride + 1;
  if (ho <= 0 || wo <= 0) return hipErrorInvalidValue;
  if (c % 4 == 0 && r == 3 && s == 3 && stride == 2 && pad == 1) {
    const size_t total = (size_t)n * ((h + 1) / 2) * ((wd + 1) / 2) * (c / 4);
    ACC_DISPATCH(dtype, hipLaunchKernelGGL(maxpool3s2_bwd_kernel<T>, dim3(grid_for(total, 256 * 64)), dim3(THREADS), 0, st,
                                           (const T*)x, (const T*)dy, (T*)dx, n, h, wd, c, ho, wo, accumulate));
  } else if (c % 4 == 0) {
    const size_t total = (size_t)n * h * wd * (c / 4);
    ACC_DISPATCH(dtype, hipLaunchKernelGGL((maxpool_bwd_kernel<T, 4>), dim3(grid_for(total, 256 * 64)), dim3(THREADS), 0,
                                           st, (const T*)x, (const T*)dy, (T*)dx, n, h, wd, c, r, s, stride, pad, ho,
                                           wo, accumulate));
  } else {
    const size_t total = (size_t)n * h * wd * c;
    ACC_DISPATCH(dtype, hipLaunchKernelGGL((maxpool_bwd_kernel<T, 1>), dim3(grid_for(total, 256 * 64)), dim3(THREADS), 0,
                                           st, (const T*)x, (const T*)dy, (T*)dx, n, h, wd, c, r, s, stride, pad, ho,
                                           wo, accumulate));
  }
  return hipGetLastError();
}

hipError_t gap_forward(const void* x, void* y, int n, int hw, int c, int dtype, hipStream_t st) {
  if (!x || !y || n <= 0 || hw <= 0 || c <= 0) return hipErrorInvalidValue;
  ACC_DISPATCH(dtype, hipLaunchKernelGGL(gap_fwd_kernel<T>, dim3(grid_for((size_t)n * c)), dim3(THREADS), 0, st,
                                         (const T*)x, (T*)y, n, hw, c));
  return hipGetLastError();
}

hipError_t gap_backward(const void* dy, void* dx, int n, int hw, int c, int accumulate, int dtype, hipStream_t st) {
  if (!dy || !dx || n <= 0 || hw <= 0 || c <= 0) return hipErrorInvalidValue;
  ACC_DISPATCH(dtype, hipLaunchKernelGGL(gap_bwd_kernel<T>, dim3(grid_for((size_t)n * hw * c)), dim3(THREADS), 0, st,
                                         (const T*)dy, (T*)dx, n, hw, c, accumulate));
  return hipGetLastError();
}

hipError_t bias_add(void* y, const float* b, long rows, int c, int dtype, hipStream_t st, int relu) {
  if (!y || !b || rows <= 0 || c <= 0) return hipErrorInvalidValue;
  const size_t total = (size_t)rows * c;
  ACC_DISPATCH(dtype, hipLaunchKernelGGL(bias_add_kernel<T>, dim3(grid_for(total)), dim3(THREADS), 0, st, (T*)y, b,
                                         total, c, relu));
  return hipGetLastError();
}

size_t relu_bias_workspace_bytes(int c) { return (size_t)RB_MAX_SLABS * c * sizeof(double); }

hipError_t relu_bias_backward(void* dy, const void* y, float* db, long rows, int c, void* workspace, int dtype,
                              hipStream_t st) {
  if (!dy || !db || !workspace || rows <= 0 || c <= 0 || (c & 3)) return hipErrorInvalidValue;
  // threads along the channels first (four channels each), the rest of the workgroup along rows
  const int cgroups = c / 4;
  const int tpr = cgroups < 64 ? cgroups : 64;
  const int rpi = THREADS / tpr;
  const int col_slices = (cgroups + tpr - 1) / tpr;
  // enough slabs to fill the chip, at least 4 trips of the workgroup per slab
  long slabs = (rows + (long)rpi * 4 - 1) / ((long)rpi * 4);
  const long cap = RB_MAX_SLABS / col_slices > 0 ? RB_MAX_SLABS / col_slices : 1;
  if (slabs > cap) slabs = cap;
  if (slabs < 1) slabs = 1;
  const long rows_per_slab = (rows + slabs - 1) / slabs;
  slabs = (rows + rows_per_slab - 1) / rows_per_slab;
  ACC_DISPATCH(dtype, hipLaunchKernelGGL(relu_bias_bwd_kernel<T>, dim3((unsigned)slabs, col_slices), dim3(THREADS), 0, st,
                                         (T*)dy, (const T*)y, (double*)workspace, rows, c, tpr, rpi, rows_per_slab));
  hipLaunchKernelGGL(slab_sum_kernel, dim3((c + THREADS - 1) / THREADS), dim3(THREADS), 0, st, (const double*)workspace,
                     db, (int)slabs, c);
  return hipGetLastError();
}

hipError_t relu_mask(void* dy, const void* y, size_t count, int dtype, hipStream_t st) {
  if (!dy || !y || count == 0) return hipErrorInvalidValue;
  ACC_DISPATCH(dtype, hipLaunchKernelGGL(relu_mask_kernel<T>, dim3(grid_for(count)), dim3(THREADS), 0, st, (T*)dy,
                                         (const T*)y, count));
  return hipGetLastError();
}

hipError_t column_sum(const void* dy, float* db, long rows, int c, int dtype, hipStream_t st) {
  if (!dy || !db || rows <= 0 || c <= 0) return hipErrorInvalidValue;
  ACC_DISPATCH(dtype, hipLaunchKernelGGL(column_sum_kernel<T>, dim3((c + THREADS - 1) / THREADS), dim3(THREADS), 0, st,
                                         (const T*)dy, db, rows, c));
  return hipGetLastError();
}

hipError_t softmax_ce_forward(const void* z, const int32_t* labels, float* loss_rows, float* loss,
                              int n, int classes, int dtype, hipStream_t st) {
  if (!z || !labels || !loss_rows || !loss || n <= 0 || classes <= 0) return hipErrorInvalidValue;
  ACC_DISPATCH(dtype, hipLaunchKernelGGL(softmax_ce_kernel<T>, dim3(n), dim3(THREADS), 0, st, (const T*)z, labels,
                                         loss_rows, (T*)nullptr, n, classes));
  hipLaunchKernelGGL(loss_mean_kernel, dim3(1), dim3(64), 0, st, loss_rows, loss, n);
  return hipGetLastError();
}

hipError_t softmax_ce_backward(const void* z, const int32_t* labels, void* dz, int n, int classes, int dtype,
                               hipStream_t st) {
  if (!z || !labels || !dz || n <= 0 || classes <= 0) return hipErrorInvalidValue;
  ACC_DISPATCH(dtype, hipLaunchKernelGGL(softmax_ce_kernel<T>, dim3(n), dim3(THREADS), 0, st, (const T*)z, labels,
                                         (float*)nullptr, (T*)dz, n, classes));
  return hipGetLastError();
}

hipError_t sgd_update(float* w, const float* g, float lr, size_t count, void* w_bf16, hipStream_t st) {
  if (!w || !g) return hipErrorInvalidValue;
  if (count == 0) return hipSuccess;
  hipLaunchKernelGGL(sgd_kernel, dim3(grid_for(count)), dim3(THREADS), 0, st, w, g, lr, count, (bf16_t*)w_bf16);
  return hipGetLastError();
}

hipError_t fill_zero(float* p, size_t count, hipStream_t st) {
  if (!p) return hipErrorInvalidValue;
  if (count == 0) return hipSuccess;
  hipLaunchKernelGGL(fill_zero_kernel, dim3(grid_for(count)), dim3(THREADS), 0, st, p, count);
  return hipGetLastError();
}

}  // namespace acc
