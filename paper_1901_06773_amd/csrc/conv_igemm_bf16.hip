// Implicit-GEMM convolution for bf16 storage on the bf16 matrix cores of gfx950
// (v_mfma_f32_32x32x16_bf16), forward pass and data gradient of the layers that carry the work.
//
//   out[m][n] (+)= sum_k A[m][k] * W[n][k],   m = (img,p,q), k = (r,t,c), c fastest
//
// Same scheme as the 64 x 64 kernel of conv_igemm.hip (K-chunks of 128 bytes of a GEMM row go
// from global memory straight into LDS, rows unpadded with their 16-byte columns XORed by the
// row number, zero fill by offsets outside the buffer descriptor, two LDS stages), with a tile
// of 128 x 128 per workgroup and 64 x 64 per wave (2 x 2 MFMA blocks).  One bf16 MFMA does in 32
// cycles what sixteen fp32 ones do in 1024, so the 64 x 64 kernel, which reads 8 KB of LDS per
// wave and chunk for 4 MFMAs, is bound by LDS bandwidth at a fraction of the matrix peak; here a
// wave reads 16 KB for 16 MFMAs: every byte read from LDS feeds twice the arithmetic, every byte
// fetched from memory likewise.  64 KB of LDS per workgroup, two workgroups per CU.
#include "kernels.h"
#include "dtype.h"
#include "igemm_side.h"

namespace acc {
namespace {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef unsigned v4u __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

constexpr int TM = 128, TN = 128;        // tile of a workgroup
constexpr int CHUNK = 128;               // bytes of a GEMM row per K-chunk: 64 bf16
constexpr int BKE = CHUNK / 2;           // elements of K per chunk
constexpr int STAGE = TM * CHUNK;        // bytes of one operand's stage: 16 KB

__device__ __forceinline__ v16f mfma_bf16(const v4u& a, const v4u& b, v16f c) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, b), c, 0, 0, 0);
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
  rp.ix0 = q * g.stride - g.pad - g.pad_dx;
  return rp;
}

__device__ __forceinline__ size_t out_row_offset(const ConvGeom& g, int m) {
  const int pq = g.p * g.q;
  const int img = m / pq;
  const int rem = m - img * pq;
  const int p = rem / g.q;
  const int q = rem - p * g.q;
  return ((size_t)(img * g.out_h + g.out_y0 + p * g.out_stride) * g.out_w + g.out_x0 + q * g.out_stride) * g.n_out;
}

// ACT: the epilogue adds a bias and applies a ReLU (never together with accumulation)
template <bool ACT>
__global__ __launch_bounds__(256) void igemm_bf16_kernel(ConvGeom g, int M, int K, int n_tiles_n, int n_tiles,
                                                          int main_grid) {
  __shared__ __attribute__((aligned(1024))) char As[2 * STAGE];
  __shared__ __attribute__((aligned(1024))) char Bs[2 * STAGE];
  if ((int)blockIdx.x >= main_grid) {
    igemm_side_jobs<bf16_t>(g, (int)blockIdx.x - main_grid, As);
    return;
  }
#if defined(__HIP_DEVICE_COMPILE__)
  // XCD-aware tile order: each XCD gets a contiguous range of tiles (neighbours share operand rows in its L2)
  const int per_xcd = main_grid >> 3;
  const int tile = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (tile >= n_tiles) return;
  const int tile_m = tile / n_tiles_n, tile_n = tile - tile_m * n_tiles_n;
  const int m0 = tile_m * TM, n0 = tile_n * TN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave >> 1) * 64, wn0 = (wave & 1) * 64;

  v16f acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  const int n_chunks = K / BKE;                       // the launcher admits whole chunks only
  constexpr int CPR = CHUNK / 16;                     // 16-byte columns per row: 8
  constexpr int RPI = 4096 / CHUNK;                   // rows one load instruction of the 4 waves fills: 32
  constexpr int AI = TM / RPI, BI = TN / RPI;         // 4 and 4
  const int lrow = tid / CPR;                         // row of the lane's LDS slot within the first RPI rows
  const int lcol = (tid & (CPR - 1)) ^ (lrow & (CPR - 1));   // 16-byte column that belongs into that slot
  const int margin = g.pad * g.wd + g.pad + g.pad_dx; // pixels; the descriptor starts that far before the tensor
  constexpr uint32_t OUTSIDE = 0xFFFFFFF0u;           // beyond any descriptor range: reads as zero
  uint32_t a_voff[AI], a_mask[AI], b_voff[BI];
  const bool plain = g.r == 1 && g.s == 1 && g.stride == 1 && g.pad == 0 && g.pad_dx == 0 && g.p == g.h && g.q == g.wd;
#pragma unroll
  for (int i = 0; i < AI; ++i) {
    if (plain) {      // 1x1, stride 1, no padding: GEMM row m is pixel m
      const int m = m0 + lrow + RPI * i;
      a_voff[i] = (uint32_t)(m < M ? m : 0) * (uint32_t)(g.c * 2) + lcol * 16;
      a_mask[i] = m < M ? 1u : 0u;
      continue;
    }
    const RowPos rp = decode_row(g, m0 + lrow + RPI * i, M);
    a_voff[i] = (uint32_t)(rp.pix + rp.iy0 * g.wd + rp.ix0 + margin) * (uint32_t)(g.c * 2) + lcol * 16;
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
    const int n = n0 + lrow + RPI * i;
    b_voff[i] = (uint32_t)(n < g.n_out ? n : 0) * (uint32_t)(K * 2) + lcol * 16;   // beyond n_out: filter 0, never stored
  }
  const size_t margin_bytes = (size_t)margin * g.c * 2;
  const size_t a_bytes = margin_bytes + (size_t)g.n_img * g.h * g.wd * g.c * 2;
  __amdgpu_buffer_rsrc_t rs_a = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<char*>(reinterpret_cast<const char*>(g.in)) - margin_bytes, 0, (int)(uint32_t)a_bytes, 0x00020000);
  __amdgpu_buffer_rsrc_t rs_b = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<void*>(g.w), 0, (int)(uint32_t)((size_t)g.n_out * K * 2), 0x00020000);
  typedef __attribute__((address_space(3))) void* lds_ptr;
  const int uwave = __builtin_amdgcn_readfirstlane(wave);
  const uint32_t lds_a = (uint32_t)(size_t)As + uwave * 1024, lds_b = (uint32_t)(size_t)Bs + uwave * 1024;
  int kr = 0, kt = 0, c0 = 0;     // tap and channel offset of the chunk whose loads are issued next (uniform)
  auto issue = [&](int kc, int buf) {
    const int tap = kr * g.s + kt;
    const int soff_a = ((kr * g.wd + kt) * g.c + c0) * 2;
    const int soff_b = kc * CHUNK;
#pragma unroll
    for (int i = 0; i < AI; ++i) {
      const uint32_t voff = ((a_mask[i] >> tap) & 1u) ? a_voff[i] : OUTSIDE;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_a, (lds_ptr)(size_t)(lds_a + buf * STAGE + i * 4096), 16, voff, soff_a, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < BI; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_b, (lds_ptr)(size_t)(lds_b + buf * STAGE + i * 4096), 16, b_voff[i], soff_b, 0, 0);
    c0 += BKE;
    if (c0 == g.c) {
      c0 = 0;
      if (++kt == g.s) { kt = 0; ++kr; }
    }
  };
  // fragment of a row: 16-byte column c16 sits in slot c16 ^ (row % 8); the lane's rows differ by
  // multiples of 32, so the XOR term is the same for both of its blocks
  const int ra = wm0 + (lane & 31), rb = wn0 + (lane & 31);
  const int xa = ra & (CPR - 1), xb = rb & (CPR - 1);
  auto compute = [&](int buf) {
    const char* as = As + buf * STAGE + ra * CHUNK;
    const char* bs = Bs + buf * STAGE + rb * CHUNK;
#pragma unroll
    for (int g8 = 0; g8 < CPR / 2; ++g8) {
      const int c16 = g8 * 2 + (lane >> 5);
      v4u a[2], b[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        a[i] = *reinterpret_cast<const v4u*>(as + i * 32 * CHUNK + ((c16 ^ xa) << 4));
        b[i] = *reinterpret_cast<const v4u*>(bs + i * 32 * CHUNK + ((c16 ^ xb) << 4));
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = mfma_bf16(b[j], a[i], acc[i][j]);   // transposed block, see the epilogue
    }
  };
  // The barrier that opens chunk kc says two things: every wave's part of chunk kc has landed
  // in LDS (each wave waits for its own loads first), and every wave is done with chunk kc-1,
  // whose stage the loads of chunk kc+1 may now overwrite.
  issue(0, 0);
  int kc = 0;
  for (; kc + 2 <= n_chunks; kc += 2) {
    __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0): this wave's loads are in LDS
    __syncthreads();
    issue(kc + 1, 1);
    compute(0);
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
    if (kc + 2 < n_chunks) issue(kc + 2, 0);
    compute(1);
  }
  if (kc < n_chunks) {
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
    compute(0);
  }

  // Epilogue.  The blocks were accumulated transposed (filter fragment first): register v of a
  // lane holds output channel 8*(v/4) + 4*(lane/32) + v%4 of GEMM row lane%32 of its block, i.e.
  // four consecutive channels of one row per group of four registers.  They are staged in LDS,
  // one region per wave, and the wave reads whole rows back: eight channels per lane, 128
  // contiguous bytes of a row per eight lanes, one 16-byte store each.  Plain results are rounded
  // to bf16 before staging (8-byte LDS writes, one pass over the wave's 64 rows); results that
  // get a bias and a ReLU, or are added to what the tensor holds, are staged in fp32 (two passes
  // of 32 rows) so that they are rounded once, after the addition.
  __syncthreads();                                   // every wave is done reading the last chunk
  char* stg = (wave < 2 ? As : Bs) + (wave & 1) * STAGE;        // 16 KB per wave
  const bool dense = g.out_stride == 1 && g.out_h == g.p && g.out_w == g.q;
  const int c8 = lane & 7;                           // the lane's piece of a row: channels 8*c8 .. 8*c8+7
  const int n = n0 + wn0 + 8 * c8;
  const bool n_ok = n < g.n_out;                     // (n_out is a multiple of 8: a piece is stored whole or not at all)
  typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
  typedef float v2f __attribute__((ext_vector_type(2)));
  auto pack2 = [](float a, float b) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v2f{a, b}, v2bf));   // round to nearest even
  };
  if (!ACT && !g.accumulate) {
    constexpr int EP = 144;                          // bytes per staged row: 128 + 16 (rows on different banks)
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const v16f& c = acc[i][j];
          uint2 pk;
          pk.x = pack2(c[4 * q4], c[4 * q4 + 1]);
          pk.y = pack2(c[4 * q4 + 2], c[4 * q4 + 3]);
          const int row = 32 * i + (lane & 31), col = 32 * j + 8 * q4 + 4 * (lane >> 5);
          *reinterpret_cast<uint2*>(stg + row * EP + col * 2) = pk;
        }
    if (!n_ok) return;
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int row = (lane >> 3) + 8 * it;
      const int m = m0 + wm0 + row;
      if (m >= M) continue;
      const v4u piece = *reinterpret_cast<const v4u*>(stg + row * EP + c8 * 16);
      bf16_t* o = static_cast<bf16_t*>(g.out) + (dense ? (size_t)m * g.n_out : out_row_offset(g, m)) + n;
      *reinterpret_cast<v4u*>(o) = piece;
    }
    return;
  }
  float bias8[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if constexpr (ACT) {
    if (g.bias && n_ok) {
#pragma unroll
      for (int e = 0; e < 8; ++e) bias8[e] = g.bias[n + e];
    }
  }
  constexpr int EPF = 272;                           // bytes per staged fp32 row: 256 + 16
#pragma unroll
  for (int i = 0; i < 2; ++i) {
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const v16f& c = acc[i][j];
        const int row = lane & 31, col = 32 * j + 8 * q4 + 4 * (lane >> 5);
        *reinterpret_cast<float4*>(stg + row * EPF + col * 4) = make_float4(c[4 * q4], c[4 * q4 + 1], c[4 * q4 + 2], c[4 * q4 + 3]);
      }
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const int row = (lane >> 3) + 8 * it;
      const int m = m0 + wm0 + 32 * i + row;
      if (m >= M || !n_ok) continue;
      const float4 lo = *reinterpret_cast<const float4*>(stg + row * EPF + c8 * 32);
      const float4 hi = *reinterpret_cast<const float4*>(stg + row * EPF + c8 * 32 + 16);
      float f[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
      bf16_t* o = static_cast<bf16_t*>(g.out) + (dense ? (size_t)m * g.n_out : out_row_offset(g, m)) + n;
      if constexpr (ACT) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          f[e] += bias8[e];
          if (g.relu) f[e] = fmaxf(f[e], 0.f);
        }
      } else {
        const v4u old = *reinterpret_cast<const v4u*>(o);
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          f[2 * w] += __uint_as_float(old[w] << 16);
          f[2 * w + 1] += __uint_as_float(old[w] & 0xffff0000u);
        }
      }
      v4u res;
#pragma unroll
      for (int w = 0; w < 4; ++w) res[w] = pack2(f[2 * w], f[2 * w + 1]);
      *reinterpret_cast<v4u*>(o) = res;
    }
  }
#else
  (void)Bs; (void)&mfma_bf16; (void)&decode_row; (void)&out_row_offset;
#endif
}

}  // namespace

bool conv_igemm_bf16_takes(const ConvGeom& g, long M, long K) {
  if (g.dtype != DT_BF16) return false;
  // whole 64-channel chunks inside one tap, at most 32 taps, both operands within 32-bit byte ranges
  // (the last bytes stay free for the offset that stands for "outside"), 16-byte aligned tensors;
  // at least 128 output channels and enough rows that 128 x 128 tiles fill the chip; no fused
  // batch-norm sums (those belong to fp32 storage)
  const long margin_px = (long)g.pad * g.wd + g.pad + g.pad_dx;
  if (g.c % BKE != 0 || g.r * g.s > 32 || g.n_out < TN || g.n_out % 8 != 0 || g.stats || g.bnb.sums) return false;
  if ((margin_px + (long)g.n_img * g.h * g.wd) * g.c * 2 > 0xFFFFFF00L || (long)g.n_out * K * 2 > 0xFFFFFF00L) return false;
  if ((reinterpret_cast<uintptr_t>(g.in) & 15) || (reinterpret_cast<uintptr_t>(g.w) & 15) ||
      (reinterpret_cast<uintptr_t>(g.out) & 15)) return false;
  const long tiles = ((M + TM - 1) / TM) * ((g.n_out + TN - 1) / TN);
  return tiles >= 256;
}

hipError_t conv_igemm_bf16(const ConvGeom& g, int M, int K, hipStream_t st, const LaunchProbe* probe) {
  const int tm = (M + TM - 1) / TM, tn = (g.n_out + TN - 1) / TN;
  const long tiles = (long)tm * tn;
  if (tiles <= 0 || tiles > (1L << 30) || K % BKE != 0) return hipErrorInvalidValue;
  const int main_grid = (int)((tiles + 7) / 8 * 8);
  long side_blocks = 0;
  if (g.side.count) {
    if (!g.side.part || !g.side.dw || g.side.splits < 1) return hipErrorInvalidValue;
    side_blocks = (long)((g.side.count + 1023) / 1024);
  }
  if ((g.bias || g.relu) && g.accumulate) return hipErrorInvalidValue;
  if (g.flip.wt) {
    if (!g.flip.w || g.flip.cout <= 0 || g.flip.cin <= 0 || g.flip.r <= 0 || g.flip.s <= 0) return hipErrorInvalidValue;
    side_blocks += (long)((g.flip.cin + 31) / 32) * ((g.flip.cout + 31) / 32) * g.flip.r * g.flip.s;
  }
  if (main_grid + side_blocks > (1L << 30)) return hipErrorInvalidValue;
  if (probe && probe->before) (void)hipEventRecord(probe->before, st);
  const dim3 grid((unsigned)(main_grid + side_blocks));
  if (g.bias || g.relu)
    hipLaunchKernelGGL(igemm_bf16_kernel<true>, grid, dim3(256), 0, st, g, M, K, tn, (int)tiles, main_grid);
  else
    hipLaunchKernelGGL(igemm_bf16_kernel<false>, grid, dim3(256), 0, st, g, M, K, tn, (int)tiles, main_grid);
  if (probe && probe->after) (void)hipEventRecord(probe->after, st);
  return hipGetLastError();
}

}  // namespace acc
