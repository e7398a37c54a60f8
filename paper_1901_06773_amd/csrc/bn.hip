// Batch normalisation with minibatch statistics over an NHWC tensor viewed as
// rows x c, fused with ReLU and with the residual add of a bottleneck block.
//
// The work is bandwidth bound, so every kernel reads whole float4 channel groups of
// consecutive rows (a wave covers 1 KiB of contiguous memory per load).  Reductions
// over rows run in two fixed-order stages (per-slab partials in double, then one
// wave per channel adds the slabs in a fixed order): no atomics, results do not depend
// on timing or addresses.
//
// workspace layout (bn_workspace_bytes): double part[2][MAX_SLABS][c] | float coef[4][c]
// (partial sums a convolution launch hands over instead are floats: fp32 sums over 32 rows each)
#include "kernels.h"
#include "dtype.h"

namespace acc {
namespace {

constexpr int MAX_SLABS = kBnMaxSlabs;   // row slabs of the reduction grid (upper bound)
constexpr int ROWS_PER_THREAD = 4;  // rows a thread of the reduction sums at least (else fewer slabs)
constexpr int THREADS = 256;
constexpr int FIN_CH = THREADS / 64;  // the finishing kernels give every channel one wave

struct ReduceShape {
  int tpr;        // threads across one row (each owns 4 channels), at most 64
  int rpi;        // rows per iteration of a block
  int col_slices; // grid.y: slices of 4 * tpr channels
};

__host__ __device__ inline ReduceShape reduce_shape(int c) {
  ReduceShape s;
  const int cg = c / 4;
  s.tpr = cg < 64 ? cg : 64;
  // tpr need not divide 256: the leftover threads idle
  s.rpi = THREADS / s.tpr;
  s.col_slices = (cg + s.tpr - 1) / s.tpr;
  return s;
}

// Sums over the rows of one slab, per channel, of up to two quantities.
// MODE 0: (x, x*x).   MODE 1: (g, g*xhat) with g = dy * [y > 0] (y optional).
template <int MODE, class T>
__global__ __launch_bounds__(THREADS) void bn_reduce_kernel(const T* __restrict__ x,
                                                            const T* __restrict__ dy,
                                                            const T* __restrict__ y,
                                                            const float* __restrict__ mean,
                                                            const float* __restrict__ istd,
                                                            double* __restrict__ part, long rows,
                                                            int c, int tpr, int rpi, int slabs) {
  __shared__ double red[2][THREADS][4];
  const int tid = threadIdx.x;
  const int lane_r = tid / tpr;            // which row of the iteration
  const int lane_c = tid - lane_r * tpr;   // which channel group
  const int cg = blockIdx.y * tpr + lane_c;
  const bool active = lane_r < rpi && cg * 4 < c;
  const long rows_per_slab = (rows + slabs - 1) / slabs;
  const long r_lo = (long)blockIdx.x * rows_per_slab;
  const long r_hi = r_lo + rows_per_slab < rows ? r_lo + rows_per_slab : rows;

  double s0[4] = {0, 0, 0, 0}, s1[4] = {0, 0, 0, 0};
  if (active) {
    float mu[4] = {0, 0, 0, 0}, is[4] = {0, 0, 0, 0};
    if (MODE == 1) {
      const float4 m4 = *reinterpret_cast<const float4*>(mean + cg * 4);
      const float4 i4 = *reinterpret_cast<const float4*>(istd + cg * 4);
      mu[0] = m4.x; mu[1] = m4.y; mu[2] = m4.z; mu[3] = m4.w;
      is[0] = i4.x; is[1] = i4.y; is[2] = i4.z; is[3] = i4.w;
    }
    auto add_row = [&](const float (&xs)[4], const float (&gv)[4], const float (&ys)[4]) {
      if (MODE == 0) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const double d = (double)xs[j];
          s0[j] += d;
          s1[j] += d * d;
        }
      } else {
        float gs[4] = {gv[0], gv[1], gv[2], gv[3]};
        if (y) {
#pragma unroll
          for (int j = 0; j < 4; ++j) gs[j] = ys[j] > 0.f ? gs[j] : 0.f;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const double gd = (double)gs[j];
          s0[j] += gd;
          s1[j] += gd * (double)((xs[j] - mu[j]) * is[j]);
        }
      }
    };
    // four rows per trip: all their loads are issued before the first sum needs one
    constexpr int U = 4;
    long r = r_lo + lane_r;
    for (; r + (long)(U - 1) * rpi < r_hi; r += (long)U * rpi) {
      float xv[U][4], gv[U][4] = {}, yv[U][4] = {};
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const size_t off = (size_t)(r + (long)u * rpi) * c + (size_t)cg * 4;
        Elem<T>::load4(x + off, xv[u]);
        if (MODE == 1) Elem<T>::load4(dy + off, gv[u]);
        if (MODE == 1 && y) Elem<T>::load4(y + off, yv[u]);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) add_row(xv[u], gv[u], yv[u]);
    }
    for (; r < r_hi; r += rpi) {
      const size_t off = (size_t)r * c + (size_t)cg * 4;
      float xv[4], gv[4] = {}, yv[4] = {};
      Elem<T>::load4(x + off, xv);
      if (MODE == 1) Elem<T>::load4(dy + off, gv);
      if (MODE == 1 && y) Elem<T>::load4(y + off, yv);
      add_row(xv, gv, yv);
    }
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    red[0][tid][j] = s0[j];
    red[1][tid][j] = s1[j];
  }
  __syncthreads();
  // the first row of threads adds the other rows in order
  if (lane_r == 0 && cg * 4 < c) {
    for (int rr = 1; rr < rpi; ++rr) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        s0[j] += red[0][rr * tpr + lane_c][j];
        s1[j] += red[1][rr * tpr + lane_c][j];
      }
    }
    double* p0 = part + ((size_t)0 * MAX_SLABS + blockIdx.x) * c + (size_t)cg * 4;
    double* p1 = part + ((size_t)1 * MAX_SLABS + blockIdx.x) * c + (size_t)cg * 4;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      p0[j] = s0[j];
      p1[j] = s1[j];
    }
  }
}

// Adds the slab partials of one channel per wave in a fixed order: lane l adds slabs l,
// l+64, ..., then a butterfly over the wave adds the lanes (every lane ends with the same sum).
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

template <class P>
__device__ __forceinline__ void sum_partials(const P* __restrict__ part, int c, int slabs, int ch,
                                             int lane, double* out0, double* out1, int stride) {
  // every load of the lane is issued before the first sum: the partials were written by
  // other compute units a moment ago, so each access pays a full trip to memory
  constexpr int PER_LANE = MAX_SLABS / 64;
  double v0[PER_LANE], v1[PER_LANE];
  const P* p0 = part + (ch < c ? ch : 0);
  const P* p1 = p0 + (size_t)stride * c;      // part[2][stride][c]
#pragma unroll
  for (int u = 0; u < PER_LANE; ++u) {
    const int k = lane + 64 * u;
    const bool ok = ch < c && k < slabs;
    const size_t at = ok ? (size_t)k * c : 0;   // slab 0 always exists; its value is dropped
    const P w0 = p0[at], w1 = p1[at];
    v0[u] = ok ? (double)w0 : 0.0;
    v1[u] = ok ? (double)w1 : 0.0;
  }
  double a0 = 0.0, a1 = 0.0;
#pragma unroll
  for (int u = 0; u < PER_LANE; ++u) { a0 += v0[u]; a1 += v1[u]; }
  *out0 = wave_sum(a0);
  *out1 = wave_sum(a1);
}

// forward:  mean, istd; coef[0] = scale = gamma*istd, coef[1] = mean, coef[2] = beta
template <class P>
__global__ __launch_bounds__(THREADS) void bn_fwd_finish_kernel(
    const P* __restrict__ part, const float* __restrict__ gamma, const float* __restrict__ beta,
    float* __restrict__ mean, float* __restrict__ istd, float* __restrict__ coef, long rows, int c,
    float eps, int slabs, int stride) {
  const int ch = blockIdx.x * FIN_CH + threadIdx.x / 64, lane = threadIdx.x & 63;
  // the channel's parameters are fetched beside the partial sums, not after them
  const float gam = gamma[ch < c ? ch : 0], bet = beta[ch < c ? ch : 0];
  double sum, ss;
  sum_partials(part, c, slabs, ch, lane, &sum, &ss, stride);
  if (lane != 0 || ch >= c) return;
  const double m = (double)rows;
  const double mu = sum / m;
  double var = ss / m - mu * mu;
  if (var < 0.0) var = 0.0;
  const double is = 1.0 / sqrt(var + (double)eps);
  mean[ch] = (float)mu;
  istd[ch] = (float)is;
  const double scale = (double)gam * is;
  coef[ch] = (float)scale;
  coef[c + ch] = (float)mu;
  coef[2 * c + ch] = bet;
}

// backward: dbeta, dgamma; coef[0] = a = gamma*istd, coef[1] = dbeta/m, coef[2] = dgamma/m
template <class P>
__global__ __launch_bounds__(THREADS) void bn_bwd_finish_kernel(
    const P* __restrict__ part, const float* __restrict__ gamma, const float* __restrict__ istd,
    float* __restrict__ dgamma, float* __restrict__ dbeta, float* __restrict__ coef, long rows, int c,
    int slabs, int stride) {
  const int ch = blockIdx.x * FIN_CH + threadIdx.x / 64, lane = threadIdx.x & 63;
  const float gam = gamma[ch < c ? ch : 0], is = istd[ch < c ? ch : 0];
  double db, dg;
  sum_partials(part, c, slabs, ch, lane, &db, &dg, stride);
  if (lane != 0 || ch >= c) return;
  dbeta[ch] = (float)db;
  dgamma[ch] = (float)dg;
  const double m = (double)rows;
  coef[ch] = gam * is;
  coef[c + ch] = (float)(db / m);
  coef[2 * c + ch] = (float)(dg / m);
}

// y = relu?((x-mean)*scale + beta (+ res)), float4 per thread, grid-stride.  Subtracting the
// mean first keeps the result exact where x equals the mean (a channel of constant values).
template <class T>
__global__ __launch_bounds__(THREADS) void bn_apply_kernel(const T* __restrict__ x,
                                                           const T* __restrict__ res,
                                                           const float* __restrict__ coef,
                                                           T* __restrict__ y, size_t n4, int c,
                                                           int relu) {
  const int cg = c >> 2;
  for (size_t i = (size_t)blockIdx.x * THREADS + threadIdx.x; i < n4; i += (size_t)gridDim.x * THREADS) {
    const int g = (int)(i % cg);
    float xv[4], o[4];
    Elem<T>::load4(x + i * 4, xv);
    const float4 sc = reinterpret_cast<const float4*>(coef)[g];
    const float4 mu = reinterpret_cast<const float4*>(coef + c)[g];
    const float4 be = reinterpret_cast<const float4*>(coef + 2 * c)[g];
    o[0] = fmaf(xv[0] - mu.x, sc.x, be.x);
    o[1] = fmaf(xv[1] - mu.y, sc.y, be.y);
    o[2] = fmaf(xv[2] - mu.z, sc.z, be.z);
    o[3] = fmaf(xv[3] - mu.w, sc.w, be.w);
    if (res) {
      float rv[4];
      Elem<T>::load4(res + i * 4, rv);
#pragma unroll
      for (int j = 0; j < 4; ++j) o[j] += rv[j];
    }
    if (relu) {
#pragma unroll
      for (int j = 0; j < 4; ++j) o[j] = fmaxf(o[j], 0.f);
    }
    Elem<T>::store4(y + i * 4, o);
  }
}

// dx = a*(g - dbeta/m - xhat*dgamma/m), g = dy*[y>0]; optionally stores g (may alias dy)
template <class T>
__global__ __launch_bounds__(THREADS) void bn_bwd_apply_kernel(
    const T* __restrict__ x, const T* dy, const T* __restrict__ y,
    const float* __restrict__ mean, const float* __restrict__ istd, const float* __restrict__ coef,
    T* __restrict__ dx, T* g_out, size_t n4, int c) {
  const int cg = c >> 2;
  for (size_t i = (size_t)blockIdx.x * THREADS + threadIdx.x; i < n4; i += (size_t)gridDim.x * THREADS) {
    const int g = (int)(i % cg);
    float xv[4], gv[4], o[4];
    Elem<T>::load4(x + i * 4, xv);
    Elem<T>::load4(dy + i * 4, gv);
    if (y) {
      float yv[4];
      Elem<T>::load4(y + i * 4, yv);
#pragma unroll
      for (int j = 0; j < 4; ++j) gv[j] = yv[j] > 0.f ? gv[j] : 0.f;
    }
    const float4 mu = reinterpret_cast<const float4*>(mean)[g];
    const float4 is = reinterpret_cast<const float4*>(istd)[g];
    const float4 a = reinterpret_cast<const float4*>(coef)[g];
    const float4 c1 = reinterpret_cast<const float4*>(coef + c)[g];
    const float4 c2 = reinterpret_cast<const float4*>(coef + 2 * c)[g];
    o[0] = a.x * (gv[0] - c1.x - (xv[0] - mu.x) * is.x * c2.x);
    o[1] = a.y * (gv[1] - c1.y - (xv[1] - mu.y) * is.y * c2.y);
    o[2] = a.z * (gv[2] - c1.z - (xv[2] - mu.z) * is.z * c2.z);
    o[3] = a.w * (gv[3] - c1.w - (xv[3] - mu.w) * is.w * c2.w);
    Elem<T>::store4(dx + i * 4, o);
    if (g_out) Elem<T>::store4(g_out + i * 4, gv);
  }
}

// ---- finish + apply in one launch, for reductions with few slabs
//
// The finishing kernels above are two dependent trips to memory and a launch of their own
// between the sums and the apply pass.  Where the sums come in few slabs, every workgroup of
// the apply pass adds the slabs of its own 32 channels itself (same order in every workgroup,
// so all of them arrive at the same coefficients) while its first rows are on their way, one
// thread per channel works out the coefficients, and the workgroups of the first row slab
// also store the per-channel results.  A workgroup covers a column slice of 32 channels
// (8 threads x 4 channels across a row) and 32 rows per trip, four trips in flight.
constexpr int SL_TPR = 8;                   // threads across the 32 channels of a slice
constexpr int SL_CH = SL_TPR * 4;
constexpr int SL_ROWS = THREADS / SL_TPR;   // rows per trip
constexpr int SL_BATCH = 16;                // 16-byte partial loads a thread has in flight
constexpr int SL_U = 4;                     // rows of a thread in flight in the apply loop
constexpr int SL_WGS = 256;                 // workgroups of a launch, about: one per CU.  Every workgroup re-reads its
                                            // slice's partials, and in the step the kernel shares the chip with a weight
                                            // gradient (ResNet-152 at minibatch 41, images/s at 192 / 256 / 320 / 384 /
                                            // 512 / 768 / 1024: 1215 / 1233 / 1216 / 1218 / 1223 / 1219 / 1218)
constexpr int kSliceMaxSlabs = 512;         // beyond: the separate finishing launch
constexpr long kSliceMaxRows = 16384;       // ... and, with 2-byte storage, larger tensors: a slice's row segment is 64 bytes
                                            // there (ResNet-152 bf16 at minibatch 512: 3320 with, 3909 images/s without the
                                            // slice kernels; fp32 at minibatch 128: 1326 with, 1310 without)
template <class T> __host__ __device__ constexpr bool slice_takes(long rows, int slabs) {
  return slabs <= kSliceMaxSlabs && (sizeof(T) == 4 || rows <= kSliceMaxRows);
}
constexpr int kSlicePhasesMax = 16;

struct SliceScratch {
  double red[2][kSlicePhasesMax][SL_CH];
  double tot[2][SL_CH];
  float coef[3][SL_CH];
};

// tot[q][j] = sum over the slabs of part[q][slab][ch0 + j].  A 16-byte load covers VEC
// neighbouring channels of one slab; thread (col, plane, phase) adds the slabs phase,
// phase + PHASES, ... of its channels, then 64 threads add the phases in order.
template <class P>
__device__ __forceinline__ void slice_sums(const P* __restrict__ part, int c, int slabs, int stride, int ch0,
                                           SliceScratch& sh) {
  constexpr int VEC = 16 / sizeof(P), COLS = SL_CH / VEC, PHASES = THREADS / (2 * COLS);
  static_assert(PHASES <= kSlicePhasesMax, "scratch");
  struct alignas(16) Vec { P v[VEC]; };
  const int tid = threadIdx.x;
  const int col = tid % COLS, plane = (tid / COLS) & 1, phase = tid / (2 * COLS);
  const int ch = ch0 + col * VEC;
  const bool ch_ok = ch < c;                // c is a multiple of 4: the VEC channels exist together
  const P* p = part + (size_t)plane * stride * c + (ch_ok ? ch : 0);
  double a[VEC];
#pragma unroll
  for (int j = 0; j < VEC; ++j) a[j] = 0.0;
  for (int base = 0; base < slabs; base += PHASES * SL_BATCH) {
    Vec v[SL_BATCH];
#pragma unroll
    for (int u = 0; u < SL_BATCH; ++u) {
      const int k = base + phase + PHASES * u;
      v[u] = *reinterpret_cast<const Vec*>(p + (k < slabs ? (size_t)k * c : 0));   // slab 0 always exists
    }
#pragma unroll
    for (int u = 0; u < SL_BATCH; ++u) {
      const bool ok = ch_ok && base + phase + PHASES * u < slabs;
#pragma unroll
      for (int j = 0; j < VEC; ++j) a[j] += ok ? (double)v[u].v[j] : 0.0;
    }
  }
#pragma unroll
  for (int j = 0; j < VEC; ++j) sh.red[plane][phase][col * VEC + j] = a[j];
  __syncthreads();
  if (tid < 2 * SL_CH) {
    const int q = tid / SL_CH, j = tid % SL_CH;
    double t = 0.0;
#pragma unroll
    for (int ph = 0; ph < PHASES; ++ph) t += sh.red[q][ph][j];
    sh.tot[q][j] = t;
  }
  __syncthreads();
}

template <class T, class P>
__global__ __launch_bounds__(THREADS) void bn_fwd_slice_kernel(
    const T* __restrict__ x, const T* __restrict__ res, const P* __restrict__ part,
    const float* __restrict__ gamma, const float* __restrict__ beta, float* __restrict__ mean,
    float* __restrict__ istd, T* __restrict__ y, long rows, int c, int relu, float eps, int slabs, int stride,
    long rows_per_wg) {
  __shared__ SliceScratch sh;
  const int ch0 = blockIdx.y * SL_CH;
  const int lane_c = threadIdx.x % SL_TPR, lane_r = threadIdx.x / SL_TPR;
  const int ch = ch0 + lane_c * 4;
  const bool active = ch < c;
  float bet[4] = {0, 0, 0, 0};
  if (active) {
    const float4 b4 = *reinterpret_cast<const float4*>(beta + ch);
    bet[0] = b4.x; bet[1] = b4.y; bet[2] = b4.z; bet[3] = b4.w;
  }
  const long r_lo = (long)blockIdx.x * rows_per_wg;
  const long r_hi = r_lo + rows_per_wg < rows ? r_lo + rows_per_wg : rows;
  float xv[SL_U][4], rv[SL_U][4] = {};
  auto load_trip = [&](long r) {
#pragma unroll
    for (int u = 0; u < SL_U; ++u) {
      const long ru = r + (long)u * SL_ROWS;
      if (active && ru < r_hi) {
        const size_t off = (size_t)ru * c + ch;
        Elem<T>::load4(x + off, xv[u]);
        if (res) Elem<T>::load4(res + off, rv[u]);
      }
    }
  };
  load_trip(r_lo + lane_r);   // requested before the sums, so that they travel meanwhile
  slice_sums(part, c, slabs, stride, ch0, sh);
  if (threadIdx.x < SL_CH && ch0 + threadIdx.x < c) {
    const int j = threadIdx.x;
    const double m = (double)rows;
    const double mean_d = sh.tot[0][j] / m;
    double var = sh.tot[1][j] / m - mean_d * mean_d;
    if (var < 0.0) var = 0.0;
    const double is_d = 1.0 / sqrt(var + (double)eps);
    sh.coef[0][j] = (float)mean_d;
    sh.coef[1][j] = (float)((double)gamma[ch0 + j] * is_d);
    if (blockIdx.x == 0) {
      mean[ch0 + j] = (float)mean_d;
      istd[ch0 + j] = (float)is_d;
    }
  }
  __syncthreads();
  if (!active) return;
  float mu[4], sc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    mu[j] = sh.coef[0][lane_c * 4 + j];
    sc[j] = sh.coef[1][lane_c * 4 + j];
  }
  for (long r = r_lo + lane_r; r < r_hi; r += (long)SL_U * SL_ROWS) {
    if (r != r_lo + lane_r) load_trip(r);
#pragma unroll
    for (int u = 0; u < SL_U; ++u) {
      const long ru = r + (long)u * SL_ROWS;
      if (ru < r_hi) {
        float o[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          o[j] = fmaf(xv[u][j] - mu[j], sc[j], bet[j]);
          if (res) o[j] += rv[u][j];
          if (relu) o[j] = fmaxf(o[j], 0.f);
        }
        Elem<T>::store4(y + (size_t)ru * c + ch, o);
      }
    }
  }
}

template <class T, class P>
__global__ __launch_bounds__(THREADS) void bn_bwd_slice_kernel(
    const T* __restrict__ x, const T* dy, const T* __restrict__ y, const P* __restrict__ part,
    const float* __restrict__ gamma, const float* __restrict__ mean, const float* __restrict__ istd,
    float* __restrict__ dgamma, float* __restrict__ dbeta, T* __restrict__ dx, T* g_out, long rows, int c,
    int slabs, int stride, long rows_per_wg) {
  __shared__ SliceScratch sh;
  const int ch0 = blockIdx.y * SL_CH;
  const int lane_c = threadIdx.x % SL_TPR, lane_r = threadIdx.x / SL_TPR;
  const int ch = ch0 + lane_c * 4;
  const bool active = ch < c;
  float a[4] = {0, 0, 0, 0}, mu[4] = {0, 0, 0, 0}, is[4] = {0, 0, 0, 0};
  if (active) {
    const float4 g4 = *reinterpret_cast<const float4*>(gamma + ch);
    const float4 m4 = *reinterpret_cast<const float4*>(mean + ch);
    const float4 i4 = *reinterpret_cast<const float4*>(istd + ch);
    mu[0] = m4.x; mu[1] = m4.y; mu[2] = m4.z; mu[3] = m4.w;
    is[0] = i4.x; is[1] = i4.y; is[2] = i4.z; is[3] = i4.w;
    a[0] = g4.x * i4.x; a[1] = g4.y * i4.y; a[2] = g4.z * i4.z; a[3] = g4.w * i4.w;
  }
  const long r_lo = (long)blockIdx.x * rows_per_wg;
  const long r_hi = r_lo + rows_per_wg < rows ? r_lo + rows_per_wg : rows;
  float xv[SL_U][4], gv[SL_U][4], yv[SL_U][4] = {};
  auto load_trip = [&](long r) {
#pragma unroll
    for (int u = 0; u < SL_U; ++u) {
      const long ru = r + (long)u * SL_ROWS;
      if (active && ru < r_hi) {
        const size_t off = (size_t)ru * c + ch;
        Elem<T>::load4(x + off, xv[u]);
        Elem<T>::load4(dy + off, gv[u]);
        if (y) Elem<T>::load4(y + off, yv[u]);
      }
    }
  };
  load_trip(r_lo + lane_r);
  slice_sums(part, c, slabs, stride, ch0, sh);
  if (threadIdx.x < SL_CH && ch0 + threadIdx.x < c) {
    const int j = threadIdx.x;
    const double m = (double)rows;
    const double db_d = sh.tot[0][j], dg_d = sh.tot[1][j];
    sh.coef[0][j] = (float)(db_d / m);
    sh.coef[1][j] = (float)(dg_d / m);
    if (blockIdx.x == 0) {
      dbeta[ch0 + j] = (float)db_d;
      dgamma[ch0 + j] = (float)dg_d;
    }
  }
  __syncthreads();
  if (!active) return;
  float c1[4], c2[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    c1[j] = sh.coef[0][lane_c * 4 + j];
    c2[j] = sh.coef[1][lane_c * 4 + j];
  }
  for (long r = r_lo + lane_r; r < r_hi; r += (long)SL_U * SL_ROWS) {
    if (r != r_lo + lane_r) load_trip(r);
#pragma unroll
    for (int u = 0; u < SL_U; ++u) {
      const long ru = r + (long)u * SL_ROWS;
      if (ru < r_hi) {
        float o[4], g[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          g[j] = (!y || yv[u][j] > 0.f) ? gv[u][j] : 0.f;
          o[j] = a[j] * (g[j] - c1[j] - (xv[u][j] - mu[j]) * is[j] * c2[j]);
        }
        const size_t off = (size_t)ru * c + ch;
        Elem<T>::store4(dx + off, o);
        if (g_out) Elem<T>::store4(g_out + off, g);
      }
    }
  }
}

// grid of the slice kernels: about SL_WGS workgroups over all column slices, a whole number of
// SL_U-row trips per workgroup; a function of the shape only
inline dim3 slice_grid(long rows, int c, long* rows_per_wg) {
  const int slices = (c + SL_CH - 1) / SL_CH;
  const long slabs = SL_WGS / slices > 0 ? SL_WGS / slices : 1;
  const long trip = (long)SL_U * SL_ROWS;
  long per = (rows + slabs - 1) / slabs;
  per = (per + trip - 1) / trip * trip;
  *rows_per_wg = per;
  return dim3((unsigned)((rows + per - 1) / per), (unsigned)slices);
}

// slab count: a function of the shape only; at least ROWS_PER_THREAD rows per thread and
// slab, about 1024 workgroups over all column slices (the partials the finishing kernel has
// to read grow with slabs * c)
template <class T>
inline int slab_count(long rows, const ReduceShape& rs) {
  long s = (rows + (long)rs.rpi * ROWS_PER_THREAD - 1) / ((long)rs.rpi * ROWS_PER_THREAD);
  const long cap = MAX_SLABS / rs.col_slices > 0 ? MAX_SLABS / rs.col_slices : 1;
  if (s > cap) s = cap;
  // few enough for the slice kernels: then as few as one batch of their partial loads
  // (128 slabs of doubles), as long as that leaves a workgroup per compute unit
  if (slice_takes<T>(rows, (int)s)) {
    const long one_batch = 128 > 256 / rs.col_slices ? 128 : 256 / rs.col_slices;
    if (s > one_batch) s = one_batch;
  }
  if (s < 1) s = 1;
  return (int)s;
}

inline unsigned apply_grid(size_t n4) {
  const size_t blocks = (n4 + THREADS - 1) / THREADS;
  const size_t cap = 256 * 16;   // 16 workgroups per CU keep every XCD busy
  return (unsigned)(blocks < cap ? (blocks ? blocks : 1) : cap);
}

}  // namespace

size_t bn_workspace_bytes(int c) {
  return (size_t)2 * MAX_SLABS * c * sizeof(double) + (size_t)4 * c * sizeof(float);
}

namespace {

// finish + apply of the forward pass from `slabs` partial sums of type P
template <class T, class P>
void bn_forward_tail(const T* x, const float* gamma, const float* beta, const T* res, T* y, float* mean, float* istd,
                     long rows, int c, int relu, float eps, const P* sums, int slabs, int stride, float* coef,
                     hipStream_t st) {
  if (slice_takes<T>(rows, slabs)) {
    long per;
    const dim3 grid = slice_grid(rows, c, &per);
    hipLaunchKernelGGL((bn_fwd_slice_kernel<T, P>), grid, dim3(THREADS), 0, st, x, res, sums, gamma, beta, mean, istd,
                       y, rows, c, relu, eps, slabs, stride, per);
    return;
  }
  hipLaunchKernelGGL(bn_fwd_finish_kernel<P>, dim3((c + FIN_CH - 1) / FIN_CH), dim3(THREADS), 0, st, sums, gamma,
                     beta, mean, istd, coef, rows, c, eps, slabs, stride);
  const size_t n4 = (size_t)rows * c / 4;
  hipLaunchKernelGGL(bn_apply_kernel<T>, dim3(apply_grid(n4)), dim3(THREADS), 0, st, x, res, coef, y, n4, c, relu);
}

template <class T>
hipError_t bn_forward_t(const T* x, const float* gamma, const float* beta, const T* res, T* y, float* mean,
                        float* istd, long rows, int c, int relu, float eps, void* workspace, hipStream_t st,
                        const BnSums& ready) {
  double* part = static_cast<double*>(workspace);
  float* coef = reinterpret_cast<float*>(part + (size_t)2 * MAX_SLABS * c);
  if (ready.part) {   // the producer of x left the sums
    bn_forward_tail(x, gamma, beta, res, y, mean, istd, rows, c, relu, eps, ready.part, ready.slabs, ready.stride,
                    coef, st);
  } else {
    const ReduceShape rs = reduce_shape(c);
    const int slabs = slab_count<T>(rows, rs);
    hipLaunchKernelGGL((bn_reduce_kernel<0, T>), dim3(slabs, rs.col_slices), dim3(THREADS), 0, st, x, (const T*)nullptr,
                       (const T*)nullptr, nullptr, nullptr, part, rows, c, rs.tpr, rs.rpi, slabs);
    bn_forward_tail(x, gamma, beta, res, y, mean, istd, rows, c, relu, eps, (const double*)part, slabs, MAX_SLABS,
                    coef, st);
  }
  return hipGetLastError();
}

template <class T, class P>
void bn_backward_tail(const T* x, const T* dy, const T* y, const float* gamma, const float* mean, const float* istd,
                      T* dx, float* dgamma, float* dbeta, T* g_out, long rows, int c, const P* sums, int slabs,
                      int stride, float* coef, hipStream_t st) {
  if (slice_takes<T>(rows, slabs)) {
    long per;
    const dim3 grid = slice_grid(rows, c, &per);
    hipLaunchKernelGGL((bn_bwd_slice_kernel<T, P>), grid, dim3(THREADS), 0, st, x, dy, y, sums, gamma, mean, istd,
                       dgamma, dbeta, dx, g_out, rows, c, slabs, stride, per);
    return;
  }
  hipLaunchKernelGGL(bn_bwd_finish_kernel<P>, dim3((c + FIN_CH - 1) / FIN_CH), dim3(THREADS), 0, st, sums, gamma,
                     istd, dgamma, dbeta, coef, rows, c, slabs, stride);
  const size_t n4 = (size_t)rows * c / 4;
  hipLaunchKernelGGL(bn_bwd_apply_kernel<T>, dim3(apply_grid(n4)), dim3(THREADS), 0, st, x, dy, y, mean, istd,
                     coef, dx, g_out, n4, c);
}

template <class T>
hipError_t bn_backward_t(const T* x, const T* dy, const T* y, const float* gamma, const float* mean,
                         const float* istd, T* dx, float* dgamma, float* dbeta, T* g_out, long rows, int c,
                         void* workspace, hipStream_t st, const BnSums& ready) {
  double* part = static_cast<double*>(workspace);
  float* coef = reinterpret_cast<float*>(part + (size_t)2 * MAX_SLABS * c);
  if (ready.part) {   // the data gradient left the sums
    bn_backward_tail(x, dy, y, gamma, mean, istd, dx, dgamma, dbeta, g_out, rows, c, ready.part, ready.slabs,
                     ready.stride, coef, st);
  } else {
    const ReduceShape rs = reduce_shape(c);
    const int slabs = slab_count<T>(rows, rs);
    hipLaunchKernelGGL((bn_reduce_kernel<1, T>), dim3(slabs, rs.col_slices), dim3(THREADS), 0, st, x, dy, y, mean,
                       istd, part, rows, c, rs.tpr, rs.rpi, slabs);
    bn_backward_tail(x, dy, y, gamma, mean, istd, dx, dgamma, dbeta, g_out, rows, c, (const double*)part, slabs,
                     MAX_SLABS, coef, st);
  }
  return hipGetLastError();
}

}  // namespace

hipError_t bn_forward(const void* x, const float* gamma, const float* beta, const void* res, void* y,
                      float* mean, float* istd, long rows, int c, int relu, float eps, void* workspace,
                      int dtype, hipStream_t st, const BnSums* ready_sums) {
  if (!x || !gamma || !beta || !y || !mean || !istd || !workspace) return hipErrorInvalidValue;
  if (rows <= 0 || c <= 0 || (c & 3)) return hipErrorInvalidValue;
  const BnSums ready = ready_sums ? *ready_sums : BnSums{nullptr, 0, 0};
  if (ready.part && (ready.slabs <= 0 || ready.slabs > MAX_SLABS || ready.stride < ready.slabs)) return hipErrorInvalidValue;
  if (dtype == DT_F32)
    return bn_forward_t((const float*)x, gamma, beta, (const float*)res, (float*)y, mean, istd, rows, c, relu, eps,
                        workspace, st, ready);
  if (dtype == DT_BF16)
    return bn_forward_t((const bf16_t*)x, gamma, beta, (const bf16_t*)res, (bf16_t*)y, mean, istd, rows, c, relu,
                        eps, workspace, st, ready);
  return hipErrorInvalidValue;
}

hipError_t bn_backward(const void* x, const void* dy, const void* y, const float* gamma, const float* mean,
                       const float* istd, void* dx, float* dgamma, float* dbeta, void* g_out, long rows, int c,
                       void* workspace, int dtype, hipStream_t st, const BnSums* ready_sums) {
  if (!x || !dy || !gamma || !mean || !istd || !dx || !dgamma || !dbeta || !workspace)
    return hipErrorInvalidValue;
  if (rows <= 0 || c <= 0 || (c & 3)) return hipErrorInvalidValue;
  const BnSums ready = ready_sums ? *ready_sums : BnSums{nullptr, 0, 0};
  if (ready.part && (y || ready.slabs <= 0 || ready.slabs > MAX_SLABS || ready.stride < ready.slabs))
    return hipErrorInvalidValue;
  if (dtype == DT_F32)
    return bn_backward_t((const float*)x, (const float*)dy, (const float*)y, gamma, mean, istd, (float*)dx, dgamma,
                         dbeta, (float*)g_out, rows, c, workspace, st, ready);
  if (dtype == DT_BF16)
    return bn_backward_t((const bf16_t*)x, (const bf16_t*)dy, (const bf16_t*)y, gamma, mean, istd, (bf16_t*)dx,
                         dgamma, dbeta, (bf16_t*)g_out, rows, c, workspace, st, ready);
  return hipErrorInvalidValue;
}

}  // namespace acc
