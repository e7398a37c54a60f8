// Weight gradient of a convolution as a GEMM over the minibatch positions:
//
//   dw[co][j] = sum_m dy[m][co] * X[m][j],   m = (img,p,q),  j = (r,t,ci), ci fastest,
//   X[m][j] = x[img, p*stride+r-pad, q*stride+t-pad, ci]  (zero in the padding)
//
// Both operands are read along their contiguous channel axis and staged in LDS as
// [m][channel]; the fp32 MFMA (v_mfma_f32_32x32x2_f32) takes k = m.  The m range is cut
// into `splits` equal parts (grid.y); each part writes its own partial tile and a second
// kernel adds the parts in a fixed order, so the result is deterministic (no atomics).
#include "kernels.h"

#include <cstdlib>

namespace acc {
namespace {

typedef float v16f __attribute__((ext_vector_type(16)));
constexpr int BKM = 32;  // rows of m per chunk

__device__ __forceinline__ v16f mfma32x32x2(float a, float b, v16f c) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
#else
  return c;  // the host pass never runs this
#endif
}

// pixel offset (in pixels) of input position for GEMM row m and tap (kr,kt); -1 = padding
__device__ __forceinline__ int gather_pixel(const WgradGeom& g, int m, int kr, int kt) {
  const int pq = g.p * g.q;
  const int img = m / pq;
  const int rem = m - img * pq;
  const int p = rem / g.q;
  const int q = rem - p * g.q;
  const int iy = p * g.stride + kr - g.pad, ix = q * g.stride + kt - g.pad;
  if ((unsigned)iy >= (unsigned)g.h || (unsigned)ix >= (unsigned)g.wd) return -1;
  return (img * g.h + iy) * g.wd + ix;
}

// FAST: cin % BN == 0 (a tile's columns lie inside one tap), cout % 4 == 0, NHWC x.
template <int BM, int BN, bool FAST>
__global__ __launch_bounds__(256) void wgrad_kernel(WgradGeom g, int Mrows, int J, int tiles_j,
                                                     int chunks_per_split, float* out,
                                                     size_t split_stride) {
  constexpr int LDA = BM + 32, LDB = BN + 32;
  __shared__ __attribute__((aligned(16))) float As[BKM * LDA];
  __shared__ __attribute__((aligned(16))) float Bs[BKM * LDB];

  const int tile_co = blockIdx.x / tiles_j, tile_j = blockIdx.x - tile_co * tiles_j;
  const int co0 = tile_co * BM, j0 = tile_j * BN;
  const int split = blockIdx.y;
  const int chunk_lo = split * chunks_per_split;
  const int n_chunks_all = (Mrows + BKM - 1) / BKM;
  const int chunk_hi = min(chunk_lo + chunks_per_split, n_chunks_all);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  constexpr int WM = BM / 2, WN = BN / 2, FM = WM / 32, FN = WN / 32;
  const int wm0 = (wave >> 1) * WM, wn0 = (wave & 1) * WN;

  v16f acc[FM][FN];
#pragma unroll
  for (int a = 0; a < FM; ++a)
#pragma unroll
    for (int b = 0; b < FN; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  auto main_loop = [&](auto& load_chunk, auto& store_chunk) {
    if (chunk_lo >= chunk_hi) return;
    load_chunk(chunk_lo);
    store_chunk();
    __syncthreads();
    for (int kc = chunk_lo; kc < chunk_hi; ++kc) {
      const bool more = kc + 1 < chunk_hi;
      if (more) load_chunk(kc + 1);
#pragma unroll
      for (int kk = 0; kk < BKM; kk += 2) {
        float af[FM], bf[FN];
#pragma unroll
        for (int a = 0; a < FM; ++a) af[a] = As[(kk + (lane >> 5)) * LDA + wm0 + 32 * a + (lane & 31)];
#pragma unroll
        for (int b = 0; b < FN; ++b) bf[b] = Bs[(kk + (lane >> 5)) * LDB + wn0 + 32 * b + (lane & 31)];
#pragma unroll
        for (int a = 0; a < FM; ++a)
#pragma unroll
          for (int b = 0; b < FN; ++b) acc[a][b] = mfma32x32x2(af[a], bf[b], acc[a][b]);
      }
      __syncthreads();
      if (more) {
        store_chunk();
        __syncthreads();
      }
    }
  };

  if constexpr (FAST) {
    constexpr int ACPR = BM / 4, ARPP = 256 / ACPR, AI = BKM / ARPP;  // float4 per row, rows per pass
    constexpr int BCPR = BN / 4, BRPP = 256 / BCPR, BI = BKM / BRPP;
    const int acol = tid % ACPR, arow = tid / ACPR;
    const int bcol = tid % BCPR, brow = tid / BCPR;
    const int tap = j0 / g.cin, ci0 = j0 - tap * g.cin;
    const int kr = tap / g.s, kt = tap - kr * g.s;
    const bool direct = g.r == 1 && g.s == 1 && g.stride == 1 && g.pad == 0;
    const bool a_ok = co0 + acol * 4 < g.cout;
    float4 ra[AI], rb[BI];
    // position (image origin in pixels, p, q) of each gathered row; chunks are visited in
    // order, so the position advances by BKM rows per chunk without any division
    int r_org[BI], r_p[BI], r_q[BI];
    if (!direct) {
#pragma unroll
      for (int i = 0; i < BI; ++i) {
        const int m = chunk_lo * BKM + brow + BRPP * i;
        const int pq = g.p * g.q;
        const int img = m / pq, rem = m - img * pq;
        r_p[i] = rem / g.q;
        r_q[i] = rem - r_p[i] * g.q;
        r_org[i] = img * g.h * g.wd;
      }
    }
    auto load_chunk = [&](int kc) {
#pragma unroll
      for (int i = 0; i < AI; ++i) {
        const int m = kc * BKM + arow + ARPP * i;
        ra[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (a_ok && m < Mrows)
          ra[i] = *reinterpret_cast<const float4*>(g.dy + (size_t)m * g.cout + co0 + acol * 4);
      }
#pragma unroll
      for (int i = 0; i < BI; ++i) {
        const int m = kc * BKM + brow + BRPP * i;
        rb[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        int pix = m;
        if (!direct) {
          const int iy = r_p[i] * g.stride + kr - g.pad, ix = r_q[i] * g.stride + kt - g.pad;
          pix = ((unsigned)iy < (unsigned)g.h && (unsigned)ix < (unsigned)g.wd) ? r_org[i] + iy * g.wd + ix : -1;
          r_q[i] += BKM;
          while (r_q[i] >= g.q) {
            r_q[i] -= g.q;
            if (++r_p[i] == g.p) { r_p[i] = 0; r_org[i] += g.h * g.wd; }
          }
        }
        if (m < Mrows && pix >= 0)
          rb[i] = *reinterpret_cast<const float4*>(g.x + (size_t)pix * g.cin + ci0 + bcol * 4);
      }
    };
    auto store_chunk = [&]() {
#pragma unroll
      for (int i = 0; i < AI; ++i)
        *reinterpret_cast<float4*>(&As[(arow + ARPP * i) * LDA + acol * 4]) = ra[i];
#pragma unroll
      for (int i = 0; i < BI; ++i)
        *reinterpret_cast<float4*>(&Bs[(brow + BRPP * i) * LDB + bcol * 4]) = rb[i];
    };
    main_loop(load_chunk, store_chunk);
  } else {
    // one element per load: column tid % 64 is fixed per thread, rows tid/64 + 4*i
    static_assert(BM == 64 && BN == 64, "generic path is 64x64");
    constexpr int AI = BKM / 4;
    const int col = tid & 63, row0 = tid >> 6;
    const int co = co0 + col;
    const int j = j0 + col;
    const bool jok = j < J;
    const int jj = jok ? j : 0;
    const int tap = jj / g.cin, ci = jj - tap * g.cin;
    const int kr = tap / g.s, kt = tap - kr * g.s;
    float ra[AI], rb[AI];
    auto load_chunk = [&](int kc) {
#pragma unroll
      for (int i = 0; i < AI; ++i) {
        const int m = kc * BKM + row0 + 4 * i;
        const bool mok = m < Mrows;
        ra[i] = (mok && co < g.cout) ? g.dy[(size_t)m * g.cout + co] : 0.f;
        float v = 0.f;
        if (mok && jok) {
          const int pix = gather_pixel(g, m, kr, kt);
          if (pix >= 0) {
            if (g.x_nchw) {
              const int hw = g.h * g.wd;
              const int img = pix / hw, rem = pix - img * hw;
              v = g.x[((size_t)img * g.cin + ci) * hw + rem];
            } else {
              v = g.x[(size_t)pix * g.cin + ci];
            }
          }
        }
        rb[i] = v;
      }
    };
    auto store_chunk = [&]() {
#pragma unroll
      for (int i = 0; i < AI; ++i) {
        As[(row0 + 4 * i) * LDA + col] = ra[i];
        Bs[(row0 + 4 * i) * LDB + col] = rb[i];
      }
    };
    main_loop(load_chunk, store_chunk);
  }

  float* dst = out + (size_t)split * split_stride;
#pragma unroll
  for (int a = 0; a < FM; ++a)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int co = co0 + wm0 + 32 * a + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
      if (co >= g.cout) continue;
#pragma unroll
      for (int b = 0; b < FN; ++b) {
        const int j = j0 + wn0 + 32 * b + (lane & 31);
        if (j < J) dst[(size_t)co * J + j] = acc[a][b][v];
      }
    }
}

// dw[i] = part[0][i] + part[1][i] + ... in that order
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* part, float* dw, size_t count,
                                                             int splits) {
  const size_t i4 = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i4 >= count) return;
  if (i4 + 4 <= count && (count & 3) == 0) {
    float4 s = *reinterpret_cast<const float4*>(part + i4);
    for (int k = 1; k < splits; ++k) {
      const float4 v = *reinterpret_cast<const float4*>(part + (size_t)k * count + i4);
      s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    *reinterpret_cast<float4*>(dw + i4) = s;
  } else {
    for (size_t i = i4; i < count && i < i4 + 4; ++i) {
      float s = part[i];
      for (int k = 1; k < splits; ++k) s += part[(size_t)k * count + i];
      dw[i] = s;
    }
  }
}

struct WgradCfg {
  int bm, bn;
  bool fast;
  int tiles_co, tiles_j, splits, chunks_per_split;
};

WgradCfg choose(int n_img, int p, int q, int cin, int cout, int r, int s, bool x_nchw) {
  WgradCfg c;
  const long Mrows = (long)n_img * p * q;
  const long J = (long)r * s * cin;
  c.fast = !x_nchw && (cout % 4 == 0) && (cin % 64 == 0);
  static const int force64 = [] { const char* e = getenv("ACC_WGRAD_TILE64"); return e ? atoi(e) : 0; }();   // < 0: allow 128-wide tiles
  static const int target = [] { const char* e = getenv("ACC_WGRAD_TARGET"); return e ? atoi(e) : 1024; }();
  if (c.fast) {
    c.bn = (cin % 128 == 0 && force64 < 0) ? 128 : 64;
    c.bm = (cout >= 128 && force64 < 0) ? 128 : 64;
  } else {
    c.bm = c.bn = 64;
  }
  c.tiles_co = (cout + c.bm - 1) / c.bm;
  c.tiles_j = (int)((J + c.bn - 1) / c.bn);
  const long tiles = (long)c.tiles_co * c.tiles_j;
  const long chunks = (Mrows + BKM - 1) / BKM;
  long splits = (target + tiles - 1) / tiles;
  const long max_splits = chunks / 24 > 0 ? chunks / 24 : 1;
  if (splits > max_splits) splits = max_splits;
  if (splits > 1024) splits = 1024;
  if (splits < 1) splits = 1;
  c.chunks_per_split = (int)((chunks + splits - 1) / splits);
  c.splits = (int)((chunks + c.chunks_per_split - 1) / c.chunks_per_split);
  return c;
}

}  // namespace

int wgrad_splits(int n_img, int p, int q, int cin, int cout, int r, int s) {
  return choose(n_img, p, q, cin, cout, r, s, false).splits;
}

size_t wgrad_workspace_bytes(int n_img, int p, int q, int cin, int cout, int r, int s) {
  // the NCHW (image) variant never needs more than the NHWC one of the same shape
  const WgradCfg a = choose(n_img, p, q, cin, cout, r, s, false);
  const WgradCfg b = choose(n_img, p, q, cin, cout, r, s, true);
  const int splits = a.splits > b.splits ? a.splits : b.splits;
  if (splits <= 1) return 0;
  return (size_t)splits * cout * r * s * cin * sizeof(float);
}

hipError_t conv_wgrad(const WgradGeom& g, hipStream_t st, LaunchProbe* probe) {
  if (!g.x || !g.dy || !g.dw) return hipErrorInvalidValue;
  if (g.n_img <= 0 || g.h <= 0 || g.wd <= 0 || g.cin <= 0 || g.p <= 0 || g.q <= 0 || g.cout <= 0 ||
      g.r <= 0 || g.s <= 0 || g.stride <= 0 || g.pad < 0)
    return hipErrorInvalidValue;
  const long Mrows = (long)g.n_img * g.p * g.q;
  const long J = (long)g.r * g.s * g.cin;
  if (Mrows >= (1L << 31) || (long)g.n_img * g.h * g.wd >= (1L << 31) || J * g.cout >= (1L << 31))
    return hipErrorInvalidValue;
  const WgradCfg c = choose(g.n_img, g.p, g.q, g.cin, g.cout, g.r, g.s, g.x_nchw != 0);
  if (c.splits > 1 && !g.workspace) return hipErrorInvalidValue;
  if (c.splits > 65535) return hipErrorInvalidValue;
  float* out = c.splits > 1 ? g.workspace : g.dw;
  const size_t count = (size_t)g.cout * J;
  const dim3 grid(c.tiles_co * c.tiles_j, c.splits);
#define WG_LAUNCH(BM_, BN_, FAST_)                                                              \
  hipLaunchKernelGGL((wgrad_kernel<BM_, BN_, FAST_>), grid, dim3(256), 0, st, g, (int)Mrows,   \
                     (int)J, c.tiles_j, c.chunks_per_split, out, count)
  int v;
  if (probe && probe->before) (void)hipEventRecord(probe->before, st);
  if (!c.fast) { v = V_WGRAD_GENERIC; WG_LAUNCH(64, 64, false); }
  else if (c.bm == 128 && c.bn == 128) { v = V_WGRAD_128x128; WG_LAUNCH(128, 128, true); }
  else if (c.bm == 128 && c.bn == 64) { v = V_WGRAD_128x64; WG_LAUNCH(128, 64, true); }
  else if (c.bm == 64 && c.bn == 128) { v = V_WGRAD_64x128; WG_LAUNCH(64, 128, true); }
  else { v = V_WGRAD_64x64; WG_LAUNCH(64, 64, true); }
  if (probe && probe->after) (void)hipEventRecord(probe->after, st);
  if (probe) probe->variant = v;
#undef WG_LAUNCH
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (c.splits > 1) {
    const unsigned blocks = (unsigned)((count + 1023) / 1024);
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3(blocks), dim3(256), 0, st, g.workspace, g.dw, count,
                       c.splits);
    e = hipGetLastError();
  }
  return e;
}

}  // namespace acc
