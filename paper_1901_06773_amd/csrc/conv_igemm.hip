// Implicit-GEMM convolution on the fp32 matrix cores of gfx950
// (v_mfma_f32_32x32x2_f32), used for the forward pass and, with a flipped /
// transposed filter or a scattering epilogue, for the data gradient.
//
//   out[m][n] (+)= sum_k A[m][k] * W[n][k],   m = (img,p,q), k = (r,t,c), c fastest
//
// A is never materialised: each K-chunk of 32 lies inside one filter tap, so a tile
// row is 128 contiguous bytes of the NHWC input (or zeros in the padding).  A
// workgroup of 4 waves (2 x 2) owns a BM x BN tile; each wave a (BM/2) x (BN/2)
// sub-tile made of 32x32 MFMA blocks.  Operand tiles are staged through LDS (two chunks) as
// [row][k] with a 36-float pitch, so that one ds_read_b128 per lane feeds four
// consecutive MFMAs: lanes 0-31 hold k = 8g..8g+3, lanes 32-63 hold k = 8g+4..8g+7
// of their row (the pairing of k inside one MFMA is free, A and W use the same one).
// The next chunk's global loads are in flight while the current chunk is multiplied.
#include "kernels.h"

#include <cstdlib>

namespace acc {
namespace {

typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int BK = 32;
constexpr int LD = BK + 4;

__device__ __forceinline__ v16f mfma32x32x2(float a, float b, v16f c) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
#else
  return c;  // the host pass never runs this
#endif
}

struct RowPos {  // decoded GEMM row
  int pix;       // img * h * wd (pixel index of the image origin)
  int iy0, ix0;  // p*stride - pad, q*stride - pad
  int ok;
};

__device__ __forceinline__ RowPos decode_row(const ConvGeom& g, int m, int M) {
  RowPos rp;
  rp.ok = m < M;
  const int mm = rp.ok ? m : 0;
  const int pq = g.p * g.q;
  const int img = mm / pq;
  const int rem = mm - img * pq;
  const int p = rem / g.q;
  const int q = rem - p * g.q;
  rp.pix = img * g.h * g.wd;
  rp.iy0 = p * g.stride - g.pad;
  rp.ix0 = q * g.stride - g.pad;
  return rp;
}

__device__ __forceinline__ size_t out_row_offset(const ConvGeom& g, int m) {
  if (g.out_stride == 1 && g.out_h == g.p && g.out_w == g.q) return (size_t)m * g.n_out;
  const int pq = g.p * g.q;
  const int img = m / pq;
  const int rem = m - img * pq;
  const int p = rem / g.q;
  const int q = rem - p * g.q;
  return ((size_t)(img * g.out_h + p * g.out_stride) * g.out_w + q * g.out_stride) * g.n_out;
}

// FAST: c % 32 == 0, NHWC input.  Otherwise every element is decoded on its own
// (any c, K tail, NCHW input); used for the 3-channel stem and for tiny layers.
template <int BM, int BN, bool FAST>
__global__ __launch_bounds__(256) void igemm_kernel(ConvGeom g, int M, int K, int n_tiles_n,
                                                     int n_tiles) {
  __shared__ __attribute__((aligned(16))) float As[2 * BM * LD];
  __shared__ __attribute__((aligned(16))) float Bs[2 * BN * LD];

  // XCD-aware tile order: consecutive workgroup ids land on different XCDs, so give
  // each XCD a contiguous range of tiles (neighbouring tiles share operand rows in its L2).
  const int per_xcd = gridDim.x >> 3;
  const int tile = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (tile >= n_tiles) return;
  const int tile_m = tile / n_tiles_n, tile_n = tile - tile_m * n_tiles_n;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

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

  const int n_chunks = (K + BK - 1) / BK;

  // K loop shared by both loaders.  LDS holds two chunks and registers hold two more:
  // while chunk kc is multiplied out of one LDS half, chunk kc+1 moves from registers into
  // the other half and the global loads of chunk kc+3 are issued into the registers just
  // freed (chunk kc+2 is already on its way).  One barrier per chunk; a global load has
  // two whole chunks of MFMA work to complete before anything waits for it.
  auto compute_chunk = [&](int cur) {
    const float* as = As + cur * (BM * LD);
    const float* bs = Bs + cur * (BN * LD);
    float4 af[2][FM], bf[2][FN];
#pragma unroll
    for (int a = 0; a < FM; ++a)
      af[0][a] = *reinterpret_cast<const float4*>(&as[(wm0 + 32 * a + (lane & 31)) * LD + (lane >> 5) * 4]);
#pragma unroll
    for (int b = 0; b < FN; ++b)
      bf[0][b] = *reinterpret_cast<const float4*>(&bs[(wn0 + 32 * b + (lane & 31)) * LD + (lane >> 5) * 4]);
#pragma unroll
    for (int g8 = 0; g8 < 4; ++g8) {
      const int c = g8 & 1, nx = c ^ 1;
      if (g8 < 3) {   // fragments of the next k-group are fetched before this group's MFMAs
#pragma unroll
        for (int a = 0; a < FM; ++a)
          af[nx][a] = *reinterpret_cast<const float4*>(
              &as[(wm0 + 32 * a + (lane & 31)) * LD + (g8 + 1) * 8 + (lane >> 5) * 4]);
#pragma unroll
        for (int b = 0; b < FN; ++b)
          bf[nx][b] = *reinterpret_cast<const float4*>(
              &bs[(wn0 + 32 * b + (lane & 31)) * LD + (g8 + 1) * 8 + (lane >> 5) * 4]);
      }
#pragma unroll
      for (int a = 0; a < FM; ++a)
#pragma unroll
        for (int b = 0; b < FN; ++b) {
          acc[a][b] = mfma32x32x2(af[c][a].x, bf[c][b].x, acc[a][b]);
          acc[a][b] = mfma32x32x2(af[c][a].y, bf[c][b].y, acc[a][b]);
          acc[a][b] = mfma32x32x2(af[c][a].z, bf[c][b].z, acc[a][b]);
          acc[a][b] = mfma32x32x2(af[c][a].w, bf[c][b].w, acc[a][b]);
        }
    }
  };
  // load_chunk(set, kc) fills register set `set`; store_chunk(set, buf) moves it to LDS
  auto main_loop = [&](auto& load_chunk, auto& store_chunk) {
    load_chunk(0, 0);
    store_chunk(0, 0);
    if (n_chunks > 1) load_chunk(1, 1);
    if (n_chunks > 2) load_chunk(0, 2);
    __syncthreads();
    for (int kc = 0; kc < n_chunks; kc += 2) {
      // even chunk: the next one (odd) waits in register set 1
      if (kc + 1 < n_chunks) store_chunk(1, 1);
      if (kc + 3 < n_chunks) load_chunk(1, kc + 3);
      compute_chunk(0);
      __syncthreads();
      if (kc + 1 >= n_chunks) break;
      // odd chunk: the next one (even) waits in register set 0
      if (kc + 2 < n_chunks) store_chunk(0, 0);
      if (kc + 4 < n_chunks) load_chunk(0, kc + 4);
      compute_chunk(1);
      __syncthreads();
    }
  };

  if constexpr (FAST) {
    // Addresses are split into a per-lane 32-bit byte offset that never changes (the row's
    // pixel, shifted by the padding margin so that it is never negative) and a uniform
    // base that moves with the filter tap and the channel chunk, so the K loop spends no
    // vector instructions on addresses; whether a tap falls into the padding is one bit of
    // a per-row mask built once.
    constexpr int AI = BM / 32, BI = BN / 32;
    const int col4 = tid & 7, row0 = tid >> 3;
    const int margin = g.pad * g.wd + g.pad;               // pixels
    uint32_t a_voff[AI], a_mask[AI], b_voff[BI];
    bool wok[BI];
#pragma unroll
    for (int i = 0; i < AI; ++i) {
      const RowPos rp = decode_row(g, m0 + row0 + 32 * i, M);
      a_voff[i] = (uint32_t)(rp.pix + rp.iy0 * g.wd + rp.ix0 + margin) * (uint32_t)(g.c * 4) + col4 * 16;
      uint32_t mask = 0;
      for (int kr = 0; kr < g.r; ++kr)
        for (int kt = 0; kt < g.s; ++kt) {
          const bool ok = rp.ok && (unsigned)(rp.iy0 + kr) < (unsigned)g.h && (unsigned)(rp.ix0 + kt) < (unsigned)g.wd;
          mask |= (ok ? 1u : 0u) << (kr * g.s + kt);
        }
      a_mask[i] = mask;
    }
#pragma unroll
    for (int i = 0; i < BI; ++i) {
      const int n = n0 + row0 + 32 * i;
      wok[i] = n < g.n_out;
      b_voff[i] = (uint32_t)(wok[i] ? n : 0) * (uint32_t)(K * 4) + col4 * 16;
    }
    float4 ra[2][AI], rb[2][BI];
    int kr = 0, kt = 0, c0 = 0;  // tap and channel offset of the chunk being loaded (uniform)

    auto load_chunk = [&](int set, int kc) {
      const int tap = kr * g.s + kt;
      const char* abase = reinterpret_cast<const char*>(g.in) +
                          ((long)(kr * g.wd + kt - margin) * g.c + c0) * 4;
      const char* bbase = reinterpret_cast<const char*>(g.w) + (long)kc * (BK * 4);
#pragma unroll
      for (int i = 0; i < AI; ++i) {
        ra[set][i] = make_float4(0.f, 0.f, 0.f, 0.f);
        if ((a_mask[i] >> tap) & 1u) ra[set][i] = *reinterpret_cast<const float4*>(abase + a_voff[i]);
      }
#pragma unroll
      for (int i = 0; i < BI; ++i) {
        rb[set][i] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (wok[i]) rb[set][i] = *reinterpret_cast<const float4*>(bbase + b_voff[i]);
      }
      c0 += BK;
      if (c0 == g.c) {
        c0 = 0;
        if (++kt == g.s) { kt = 0; ++kr; }
      }
    };
    auto store_chunk = [&](int set, int buf) {
      float* as = As + buf * (BM * LD);
      float* bs = Bs + buf * (BN * LD);
#pragma unroll
      for (int i = 0; i < AI; ++i)
        *reinterpret_cast<float4*>(&as[(row0 + 32 * i) * LD + col4 * 4]) = ra[set][i];
#pragma unroll
      for (int i = 0; i < BI; ++i)
        *reinterpret_cast<float4*>(&bs[(row0 + 32 * i) * LD + col4 * 4]) = rb[set][i];
    };

    main_loop(load_chunk, store_chunk);
  } else {
    // one element per load: thread -> k column tid%32, rows tid/32 + 8*i
    constexpr int AI = BM / 8, BI = BN / 8;
    const int kcol = tid & 31, row0 = tid >> 5;
    RowPos rp[AI];
#pragma unroll
    for (int i = 0; i < AI; ++i) rp[i] = decode_row(g, m0 + row0 + 8 * i, M);
    float ra[2][AI], rb[2][BI];
    auto load_chunk = [&](int set, int kc) {
      const int k = kc * BK + kcol;
      const bool kok = k < K;
      const int kk = kok ? k : 0;
      const int tap = kk / g.c, c = kk - tap * g.c;
      const int kr = tap / g.s, kt = tap - kr * g.s;
#pragma unroll
      for (int i = 0; i < AI; ++i) {
        const int iy = rp[i].iy0 + kr, ix = rp[i].ix0 + kt;
        const bool ok = kok && rp[i].ok && (unsigned)iy < (unsigned)g.h && (unsigned)ix < (unsigned)g.wd;
        float v = 0.f;
        if (ok) {
          const int img = rp[i].pix / (g.h * g.wd);
          const size_t off = g.in_nchw ? ((size_t)(img * g.c + c) * g.h + iy) * g.wd + ix
                                       : (size_t)(rp[i].pix + iy * g.wd + ix) * g.c + c;
          v = g.in[off];
        }
        ra[set][i] = v;
      }
#pragma unroll
      for (int i = 0; i < BI; ++i) {
        const int n = n0 + row0 + 8 * i;
        rb[set][i] = (kok && n < g.n_out) ? g.w[(size_t)n * K + k] : 0.f;
      }
    };
    auto store_chunk = [&](int set, int buf) {
#pragma unroll
      for (int i = 0; i < AI; ++i) As[buf * (BM * LD) + (row0 + 8 * i) * LD + kcol] = ra[set][i];
#pragma unroll
      for (int i = 0; i < BI; ++i) Bs[buf * (BN * LD) + (row0 + 8 * i) * LD + kcol] = rb[set][i];
    };
    main_loop(load_chunk, store_chunk);
  }

  // epilogue: accumulator register v of a lane holds row 8*(v/4) + 4*(lane/32) + v%4,
  // column lane%32 of its 32x32 block
#pragma unroll
  for (int a = 0; a < FM; ++a)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int m = m0 + wm0 + 32 * a + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
      if (m >= M) continue;
      const size_t ro = out_row_offset(g, m);
#pragma unroll
      for (int b = 0; b < FN; ++b) {
        const int n = n0 + wn0 + 32 * b + (lane & 31);
        if (n >= g.n_out) continue;
        float val = acc[a][b][v];
        if (g.accumulate) val += g.out[ro + n];
        g.out[ro + n] = val;
      }
    }
}

template <int BM, int BN, bool FAST>
hipError_t launch(const ConvGeom& g, int M, int K, hipStream_t st, const LaunchProbe* probe) {
  const int tm = (M + BM - 1) / BM, tn = (g.n_out + BN - 1) / BN;
  const long tiles = (long)tm * tn;
  if (tiles <= 0 || tiles > (1L << 30)) return hipErrorInvalidValue;
  const int grid = (int)((tiles + 7) / 8 * 8);
  if (probe->before) (void)hipEventRecord(probe->before, st);
  hipLaunchKernelGGL((igemm_kernel<BM, BN, FAST>), dim3(grid), dim3(256), 0, st, g, M, K, tn,
                     (int)tiles);
  if (probe->after) (void)hipEventRecord(probe->after, st);
  return hipGetLastError();
}

}  // namespace

const char* conv_variant_name(int v) {
  static const char* names[V_COUNT] = {"igemm_kernel<128,128,fast>", "igemm_kernel<128,64,fast>",
                                       "igemm_kernel<64,64,fast>", "igemm_kernel<64,64,generic>",
                                       "wgrad_kernel<128,128,fast>", "wgrad_kernel<128,64,fast>",
                                       "wgrad_kernel<64,128,fast>", "wgrad_kernel<64,64,fast>",
                                       "wgrad_kernel<64,64,generic>"};
  return (v >= 0 && v < V_COUNT) ? names[v] : "?";
}

hipError_t conv_igemm(const ConvGeom& g, hipStream_t st, LaunchProbe* probe) {
  LaunchProbe local;
  if (!probe) probe = &local;
  int* variant = &probe->variant;
  if (!g.in || !g.w || !g.out) return hipErrorInvalidValue;
  if (g.n_img <= 0 || g.h <= 0 || g.wd <= 0 || g.c <= 0 || g.p <= 0 || g.q <= 0 || g.n_out <= 0 ||
      g.r <= 0 || g.s <= 0 || g.stride <= 0 || g.pad < 0 || g.out_stride <= 0)
    return hipErrorInvalidValue;
  // every gathered coordinate p*stride+r-pad is range-checked in the kernel; the output
  // pixel (p*out_stride, q*out_stride) must exist
  if ((g.p - 1) * g.out_stride >= g.out_h || (g.q - 1) * g.out_stride >= g.out_w)
    return hipErrorInvalidValue;
  const long M = (long)g.n_img * g.p * g.q;
  const long K = (long)g.r * g.s * g.c;
  if (M >= (1L << 31) || K >= (1L << 31) || (long)g.n_img * g.h * g.wd >= (1L << 31))
    return hipErrorInvalidValue;
  // fast loader: 32-channel chunks, at most 32 filter taps (one validity bit each), and
  // every per-lane byte offset below 2^32
  const bool fast = (g.c % BK == 0) && !g.in_nchw && g.r * g.s <= 32 &&
                    ((long)g.n_img * g.h * g.wd + 2L * g.pad * (g.wd + 1)) * g.c * 4 < (1L << 32) &&
                    (long)g.n_out * K * 4 < (1L << 32);
  if (!fast) { *variant = V_IGEMM_GENERIC; return launch<64, 64, false>(g, (int)M, (int)K, st, probe); }
  // Tile choice depends on the GEMM shape only (never on addresses or on the swap plan).
  // Measured on MI355X over the ResNet shapes at minibatch 32..256: 64x64 tiles beat
  // 128x64 and 128x128 everywhere (70.7 / 86 / 98 TFLOP/s against 56 / 76 / 88 and
  // 40 / 61 / 82): with M a multiple of 49 the larger tiles quantise badly over 256 CUs,
  // and four resident workgroups per CU hide the barrier of each 32-wide K chunk.
  static const int force = [] { const char* e = getenv("ACC_IGEMM_TILE"); return e ? atoi(e) : -1; }();
  if (force == 0) { *variant = V_IGEMM_128x128; return launch<128, 128, true>(g, (int)M, (int)K, st, probe); }
  if (force == 1) { *variant = V_IGEMM_128x64; return launch<128, 64, true>(g, (int)M, (int)K, st, probe); }
  *variant = V_IGEMM_64x64;
  return launch<64, 64, true>(g, (int)M, (int)K, st, probe);
}

}  // namespace acc
