// Implicit-GEMM convolution on the fp32 matrix cores of gfx950
// (v_mfma_f32_32x32x2_f32), used for the forward pass and, with a flipped /
// transposed filter or a scattering epilogue, for the data gradient.
//
//   out[m][n] (+)= sum_k A[m][k] * W[n][k],   m = (img,p,q), k = (r,t,c), c fastest
//
// A is never materialised: each K-chunk of 32 lies inside one filter tap, so a tile
// row is 128 contiguous bytes of the NHWC input (or zeros in the padding).  A
// workgroup of 4 waves (2 x 2) owns a 64 x 64 tile, each wave one 32x32 MFMA block.
// Operand tiles are staged through LDS (two chunks) as [row][k], so that one ds_read_b128
// per lane feeds four consecutive MFMAs: lanes 0-31 hold k = 8g..8g+3, lanes 32-63 hold
// k = 8g+4..8g+7 of their row (the pairing of k inside one MFMA is free, A and W use the
// same one).  Two loaders fill LDS, see below: straight from global memory (the layers that
// carry the work), or element by element through registers (odd shapes).
//
// Tile shape (measured on MI355X over the ResNet shapes at minibatch 32..256): 64x64
// beats 128x64 and 128x128 everywhere (70.7 / 86 / 98 TFLOP/s against 56 / 76 / 88 and
// 40 / 61 / 82): with M a multiple of 49 the larger tiles quantise badly over 256 CUs,
// and four resident workgroups per CU hide the one barrier per chunk.  A 64x128 variant of the
// direct loader (each wave two 32x32 blocks on shared input fragments, 48 KB of LDS, three
// workgroups per CU) for the 1x1 expansions lost as well: igemm 92.8 against 98.7 TFLOP/s over
// a ResNet-152 step at minibatch 41 when used from three tiles per CU on, 97.5 from six on.
#include "kernels.h"
#include "dtype.h"
#include "igemm_side.h"

namespace acc {
namespace {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));   // native vector: staging stays in registers

// A K-chunk is 128 bytes of a GEMM row: 32 fp32 or 64 bf16 elements.  The loaders and the
// LDS layout work on bytes and are the same for both; only the matrix instruction differs
// (16 x v_mfma_f32_32x32x2_f32 or 4 x v_mfma_f32_32x32x16_bf16 per chunk and wave).
constexpr int CHUNK_BYTES = 128;
constexpr int LD = CHUNK_BYTES / 4 + 4;      // LDS row pitch in 4-byte words (16 bytes of padding)
constexpr int BM = 64, BN = 64;
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

__device__ __forceinline__ v16f mfma32x32x16bf(const float4& a, const float4& b, v16f c) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, b), c, 0, 0, 0);
#else
  return c;  // the host pass never runs this
#endif
}

__device__ __forceinline__ v16f mfma32x32x2(float a, float b, v16f c) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
#else
  return c;  // the host pass never runs this
#endif
}

__device__ __forceinline__ void sched_fence() {
#if defined(__HIP_DEVICE_COMPILE__)
  __builtin_amdgcn_sched_barrier(0);   // the instruction scheduler moves nothing across this point
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
  if (g.out_stride == 1 && g.out_h == g.p && g.out_w == g.q) return (size_t)m * g.n_out;
  const int pq = g.p * g.q;
  const int img = m / pq;
  const int rem = m - img * pq;
  const int p = rem / g.q;
  const int q = rem - p * g.q;
  return ((size_t)(img * g.out_h + g.out_y0 + p * g.out_stride) * g.out_w + g.out_x0 + q * g.out_stride) * g.n_out;
}

// Loaders.  L_DIRECT: c a multiple of the chunk (32 fp32 / 64 bf16 channels), NHWC input, at
// most 32 filter taps, both operands within 32-bit byte ranges.  L_GENERIC: every element is
// decoded on its own and staged through registers (any c, K tail); used for the 3-channel
// stem and for tiny layers.
//
// L_DIRECT moves the chunks from global memory straight into LDS (buffer_load_dwordx4 ... lds:
// a wave's 64 lanes fill 1024 consecutive LDS bytes, eight 128-byte rows), so no staging
// registers, no LDS store instructions and no zeroing pass: a lane whose tap falls into the
// padding (or whose row lies beyond M) is given an offset beyond the buffer descriptor's
// range and the hardware delivers zeros.  Rows are unpadded (pitch 128 bytes); the 16-byte
// columns of a row are permuted by XOR with the row number (the lane fetches the column that
// belongs into its slot), which keeps the fragment reads free of bank conflicts.  Two LDS
// stages: the loads of chunk kc+1 are issued right after the barrier that opens chunk kc
// and have its whole MFMA work to land.
enum { L_GENERIC = 0, L_DIRECT = 2 };
// Chunk of L_DIRECT in bytes of a GEMM row (128 or 256; the loader and the fragment reads are
// written for both).  256-byte chunks in fp32 (one barrier per 32 MFMAs of a wave, 64 KB of
// LDS per workgroup) measured 127 against 121 TFLOP/s in a bare copy of the loop at two
// workgroups per CU, but lost in the kernel itself: no third workgroup fits beside two, so a
// tile's prologue and epilogue overlap nothing (256->256 3x3 at 4 tiles per CU 106 against
// 115 TFLOP/s, ResNet-152 step 1039 against 1165 images/s), and the weight-gradient kernel
// finds no LDS beside it.  Chosen per launch, for forward products with at most two tiles per CU only (nothing
// beside them, LDS to spare), it changed nothing either: 256->256 3x3 at 14 x 14 and minibatch 41 83.2 against
// 82.5 us, 1024->256 1x1 41.4 against 41.1 us.
__host__ __device__ constexpr int direct_chunk_bytes(int) { return 128; }

// KS = 2: a workgroup of 8 waves, two groups of 4 that each keep the whole 64 x 64 tile and take every
// second K-chunk (own LDS stages, 64 KB per workgroup); group 1 hands its accumulators over through LDS
// at the end and group 0 writes the tile.  For launches with at most one tile per compute unit (the 7 x 7
// layers of a ResNet at small minibatches), where the 4-wave kernel leaves every SIMD with a single wave:
// 512->512 3x3 at 7 x 7, minibatch 41 (256 tiles) 98 -> 85 us, 2048->512 1x1 47 -> 42 us.  With two tiles
// per compute unit it gains nothing (256->256 3x3 at 14 x 14: 82.7 -> 82.3 us; 1024->256 1x1 40.5 -> 41.7):
// the two groups pass the same barriers, so they wait together where two workgroups would not.
template <int LOADER, class T, bool ACT, int KS = 1>
__global__ __launch_bounds__(256 * KS) void igemm_kernel(ConvGeom g, int M, int K, int n_tiles_n, int n_tiles,
                                                          int main_grid) {
  constexpr bool DIRECT = LOADER == L_DIRECT;
  static_assert(KS == 1 || (KS == 2 && DIRECT && !ACT), "the split serves the direct loader only");
  constexpr int ES = sizeof(T);
  constexpr int DCHUNK = direct_chunk_bytes(ES);
  constexpr int BK = (DIRECT ? DCHUNK : CHUNK_BYTES) / ES;       // elements of K per chunk
  constexpr int LDD = DCHUNK / 4;            // LDS row pitch of L_DIRECT in words
  constexpr int PITCH = DIRECT ? LDD : LD;
  __shared__ __attribute__((aligned(1024))) float As[KS * 2 * BM * PITCH];
  __shared__ __attribute__((aligned(1024))) float Bs[KS * 2 * BN * PITCH];

  if ((int)blockIdx.x >= main_grid) {
    // the side jobs are written for 256 threads (the second group's waves leave; a barrier counts
    // the waves that are still there)
    if (KS == 1 || threadIdx.x < 256) igemm_side_jobs<T>(g, (int)blockIdx.x - main_grid, As);
    return;
  }

  // Forward products and data gradients are the critical path of an iteration; a weight gradient may run
  // beside them on a stream of its own (default wave priority) and has two layers' time to finish.  Where
  // waves of both want to issue, these go first: ResNet-152 at minibatch 41 1227 -> 1247 images/s.  (The same
  // in the batch-norm kernels took the gain away again, 1233: bandwidth-bound waves that win every issue
  // slot only keep the matrix cores from the weight gradient.)
#if defined(__HIP_DEVICE_COMPILE__)
  __builtin_amdgcn_s_setprio(3);
#endif
  // XCD-aware tile order: consecutive workgroup ids land on different XCDs, so give
  // each XCD a contiguous range of tiles (neighbouring tiles share operand rows in its L2).
  const int per_xcd = main_grid >> 3;
  const int tile = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (tile >= n_tiles) return;
  const int tile_m = tile / n_tiles_n, tile_n = tile - tile_m * n_tiles_n;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  // thread, wave: within the group of 4 waves; ugrp: the group (wave-uniform)
  const int tid = KS == 1 ? (int)threadIdx.x : (int)(threadIdx.x & 255), lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave >> 1) * 32, wn0 = (wave & 1) * 32;
#if defined(__HIP_DEVICE_COMPILE__)
  const int ugrp = KS == 1 ? 0 : __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 8));
#else
  const int ugrp = 0;
#endif

  v16f acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;

  const int n_chunks = (K + BK - 1) / BK;

  // One chunk out of LDS half `cur`: 4 k-groups of 8, the fragments of the next group
  // are fetched before the MFMAs of the current one.
  // first fragments of a chunk; fetched early so that their LDS latency hides behind the
  // stores and global loads of the half-iteration
  auto first_frag = [&](int cur, float4& a0, float4& b0) {
    const float* as = As + cur * (BM * LD) + (wm0 + (lane & 31)) * LD + (lane >> 5) * 4;
    const float* bs = Bs + cur * (BN * LD) + (wn0 + (lane & 31)) * LD + (lane >> 5) * 4;
    a0 = *reinterpret_cast<const float4*>(as);
    b0 = *reinterpret_cast<const float4*>(bs);
  };
  auto compute_chunk2 = [&](int cur, const float4& a0, const float4& b0) {
    const float* as = As + cur * (BM * LD) + (wm0 + (lane & 31)) * LD + (lane >> 5) * 4;
    const float* bs = Bs + cur * (BN * LD) + (wn0 + (lane & 31)) * LD + (lane >> 5) * 4;
    float4 af[2], bf[2];
    af[0] = a0;
    bf[0] = b0;
#pragma unroll
    for (int g8 = 0; g8 < 4; ++g8) {
      const int c = g8 & 1, nx = c ^ 1;
      if (g8 < 3) {
        af[nx] = *reinterpret_cast<const float4*>(as + (g8 + 1) * 8);
        bf[nx] = *reinterpret_cast<const float4*>(bs + (g8 + 1) * 8);
      }
      if constexpr (ES == 4) {
        acc = mfma32x32x2(af[c].x, bf[c].x, acc);
        acc = mfma32x32x2(af[c].y, bf[c].y, acc);
        acc = mfma32x32x2(af[c].z, bf[c].z, acc);
        acc = mfma32x32x2(af[c].w, bf[c].w, acc);
      } else {
        acc = mfma32x32x16bf(af[c], bf[c], acc);   // 16 bytes per lane = 8 bf16 of K
      }
    }
  };
  auto compute_chunk = [&](int cur) {
    float4 a0, b0;
    first_frag(cur, a0, b0);
    compute_chunk2(cur, a0, b0);
  };

  // K loop of the register-staged (per-element) loader.  LDS holds two chunks and registers hold two more:
  // while chunk kc is multiplied out of one LDS half, chunk kc+1 moves from registers
  // into the other half and the global loads of chunk kc+3 are issued into the registers
  // just freed (chunk kc+2 is already on its way).  One barrier per chunk; a global load
  // has two whole chunks of MFMA work to complete before anything waits for it.
  // load(ra, rb, tap, kc) fills a register set; store(ra, rb, tap, buf) moves it to LDS.
  // The sets are passed as arguments (not captured) so that they stay in registers.
  auto main_loop = [&](auto& load, auto& store, auto& ra0, auto& rb0, auto& ra1, auto& rb1) {
    int tap0 = 0, tap1 = 0;
    int kc = 0;
    load(ra0, rb0, tap0, 0);
    store(ra0, rb0, tap0, 0);
    // sched_fence(): nothing that consumes a register set (the zeroing of padded taps, the
    // LDS stores) may be hoisted above the MFMA work of the half-iteration before it, or
    // the wait for its loads would move up with it and shorten the prefetch distance.
    if (n_chunks >= 5) {
      // Steady state with every load unconditional: the number of loads in flight is the
      // same on every path, so the wait before a store leaves the younger set in flight.
      load(ra1, rb1, tap1, 1);
      load(ra0, rb0, tap0, 2);
      __syncthreads();
      for (; kc + 4 < n_chunks; kc += 2) {
        // the first fragments of the chunk are fetched before the stores and loads of this
        // half-iteration, which then cover their LDS latency
        float4 fa, fb;
        sched_fence();
        first_frag(0, fa, fb);
        sched_fence();
        store(ra1, rb1, tap1, 1);          // chunk kc+1
        load(ra1, rb1, tap1, kc + 3);
        sched_fence();
        compute_chunk2(0, fa, fb);
        __syncthreads();
        sched_fence();
        first_frag(1, fa, fb);
        sched_fence();
        store(ra0, rb0, tap0, 0);          // chunk kc+2
        load(ra0, rb0, tap0, kc + 4);
        sched_fence();
        compute_chunk2(1, fa, fb);
        __syncthreads();
      }
    } else {
      if (n_chunks > 1) load(ra1, rb1, tap1, 1);
      if (n_chunks > 2) load(ra0, rb0, tap0, 2);
      __syncthreads();
    }
    // drain (and short K): loads only while chunks remain
    for (; kc < n_chunks; kc += 2) {
      sched_fence();
      if (kc + 1 < n_chunks) store(ra1, rb1, tap1, 1);
      if (kc + 3 < n_chunks) load(ra1, rb1, tap1, kc + 3);
      sched_fence();
      compute_chunk(0);
      __syncthreads();
      if (kc + 1 >= n_chunks) break;
      sched_fence();
      if (kc + 2 < n_chunks) store(ra0, rb0, tap0, 0);
      if (kc + 4 < n_chunks) load(ra0, rb0, tap0, kc + 4);
      sched_fence();
      compute_chunk(1);
      __syncthreads();
    }
  };

  // A dense result that is added to what the tensor holds (the data gradient that joins a shortcut's
  // gradient): the sixteen old values of the lane are requested before the K loop and arrive during it.
  // In the epilogue their latency had nothing to hide behind: these launches have 2 to 8 chunks of K
  // and moved 2.0-2.5 TB/s.
  float old[16];
  bool have_old = false;
  if constexpr (DIRECT && !ACT) {
    const int n_pre = n0 + wn0 + (lane & 31);
    if (g.accumulate && g.out_stride == 1 && g.out_h == g.p && g.out_w == g.q && n_pre < g.n_out && ugrp == 0) {
      have_old = true;
      const int mb = m0 + wm0 + 4 * (lane >> 5);
      const int left = m0 + BM <= M ? 64 : M - mb;
      const T* o0 = static_cast<const T*>(g.out) + (size_t)(mb < M ? mb : 0) * g.n_out + n_pre;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int dr = 8 * (v >> 2) + (v & 3);
        old[v] = dr < left ? Elem<T>::load(o0 + (size_t)dr * g.n_out) : 0.f;
      }
    }
  }
  if constexpr (DIRECT) {
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr int CPR = DCHUNK / 16;                    // 16-byte columns per row: 8 or 16
    constexpr int RPI = 4096 / DCHUNK;                  // rows one load instruction of the 4 waves fills: 32 or 16
    constexpr int AI = BM / RPI, BI = BN / RPI;
    const int lrow = tid / CPR;                         // row of the lane's LDS slot within the first RPI rows
    const int lcol = (tid & (CPR - 1)) ^ (lrow & (CPR - 1));   // 16-byte column that belongs into that slot
    const int margin = g.pad * g.wd + g.pad + g.pad_dx; // pixels; the descriptor starts that far before the tensor
    constexpr uint32_t OUTSIDE = 0xFFFFFFF0u;           // beyond any descriptor range: reads as zero
    uint32_t a_voff[AI], a_mask[AI], b_voff[BI];
    // 1x1, stride 1, no padding (two launches in three): GEMM row m is pixel m, nothing to decode
    const bool plain = g.r == 1 && g.s == 1 && g.stride == 1 && g.pad == 0 && g.pad_dx == 0 && g.p == g.h && g.q == g.wd;
#pragma unroll
    for (int i = 0; i < AI; ++i) {
      if (plain) {
        const int m = m0 + lrow + RPI * i;
        a_voff[i] = (uint32_t)(m < M ? m : 0) * (uint32_t)(g.c * ES) + lcol * 16;
        a_mask[i] = m < M ? 1u : 0u;
        continue;
      }
      const RowPos rp = decode_row(g, m0 + lrow + RPI * i, M);
      a_voff[i] = (uint32_t)(rp.pix + rp.iy0 * g.wd + rp.ix0 + margin) * (uint32_t)(g.c * ES) + lcol * 16;
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
      b_voff[i] = (uint32_t)(n < g.n_out ? n : 0) * (uint32_t)(K * ES) + lcol * 16;   // beyond n_out: filter 0, never stored
    }
    const size_t margin_bytes = (size_t)margin * g.c * ES;
    const size_t a_bytes = margin_bytes + (size_t)g.n_img * g.h * g.wd * g.c * ES;
    __amdgpu_buffer_rsrc_t rs_a = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<char*>(reinterpret_cast<const char*>(g.in)) - margin_bytes, 0, (int)(uint32_t)a_bytes, 0x00020000);
    __amdgpu_buffer_rsrc_t rs_b = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void*>(g.w), 0, (int)(uint32_t)((size_t)g.n_out * K * ES), 0x00020000);
    typedef __attribute__((address_space(3))) void* lds_ptr;
    const int uwave = __builtin_amdgcn_readfirstlane(wave);
    const uint32_t lds_a = (uint32_t)(size_t)As + ugrp * (2 * BM * DCHUNK) + uwave * 1024;
    const uint32_t lds_b = (uint32_t)(size_t)Bs + ugrp * (2 * BN * DCHUNK) + uwave * 1024;
    int kr = 0, kt = 0, c0 = 0;     // tap and channel offset of the chunk whose loads are issued next (uniform)
    auto advance = [&]() {
      c0 += BK;
      if (c0 == g.c) {
        c0 = 0;
        if (++kt == g.s) { kt = 0; ++kr; }
      }
    };
    auto issue = [&](int kc, int buf) {
      const int tap = kr * g.s + kt;
      const int soff_a = ((kr * g.wd + kt) * g.c + c0) * ES;
      const int soff_b = kc * DCHUNK;
#pragma unroll
      for (int i = 0; i < AI; ++i) {
        const uint32_t voff = ((a_mask[i] >> tap) & 1u) ? a_voff[i] : OUTSIDE;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_a, (lds_ptr)(size_t)(lds_a + buf * (BM * DCHUNK) + i * 4096),
                                                 16, voff, soff_a, 0, 0);
      }
#pragma unroll
      for (int i = 0; i < BI; ++i)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_b, (lds_ptr)(size_t)(lds_b + buf * (BN * DCHUNK) + i * 4096),
                                                 16, b_voff[i], soff_b, 0, 0);
#pragma unroll
      for (int s = 0; s < KS; ++s) advance();   // a group's next chunk is KS further on
    };
    // fragment of a row: 16-byte column c16 sits in slot c16 ^ (row % CPR)
    const int ra_ = wm0 + (lane & 31), rb_ = wn0 + (lane & 31);
    // One chunk out of LDS stage `buf`.  A group = two 16-byte columns of a row (lanes 0-31 / 32-63) = four
    // MFMAs.  The reads of group g + 1 are issued between the MFMAs of group g, and the last group's MFMAs are
    // held back (pa, pb) until the next chunk's barrier has been passed and its first reads are on their way:
    // the matrix cores have work queued while the wave waits at the barrier and for LDS.  The products are
    // added in the same order as ever.  The next chunk's global loads are issued after the held-back MFMAs, so
    // that nothing stands between the barrier and queued matrix work.  (Measured against "all eight reads
    // first, then sixteen MFMAs", 256->256 3x3 at 14 x 14, minibatch 41: 82.6 -> 79.8 us with the interleaved
    // reads, 79.4 with the held-back group, 78.6 with the loads behind it; two held-back groups: 79.7; the four loads
    // spread over the four groups instead of issued together: 82.3.  With no loads at all after the second chunk
    // the same launch takes 71.3 us: the global -> LDS traffic costs a tenth of the kernel.)
    float4 pa = make_float4(0.f, 0.f, 0.f, 0.f), pb = pa;
    auto mm = [&](const float4& a, const float4& b, int half) {
      if constexpr (ES == 4) {
        if (half != 1) {
          acc = mfma32x32x2(a.x, b.x, acc);
          acc = mfma32x32x2(a.y, b.y, acc);
        }
        if (half != 0) {
          acc = mfma32x32x2(a.z, b.z, acc);
          acc = mfma32x32x2(a.w, b.w, acc);
        }
      } else {
        if (half != 0) acc = mfma32x32x16bf(a, b, acc);
      }
    };
    auto compute_direct = [&](int buf, bool prev, int next_kc = -1) {
      const float* as = As + (ugrp * 2 + buf) * (BM * LDD) + ra_ * LDD;
      const float* bs = Bs + (ugrp * 2 + buf) * (BN * LDD) + rb_ * LDD;
      constexpr int NG = CPR / 2;
      float4 af[NG], bf[NG];
      auto rd = [&](int g8) {
        const int c16 = g8 * 2 + (lane >> 5);
        af[g8] = *reinterpret_cast<const float4*>(as + ((c16 ^ (ra_ & (CPR - 1))) << 2));
        bf[g8] = *reinterpret_cast<const float4*>(bs + ((c16 ^ (rb_ & (CPR - 1))) << 2));
      };
      rd(0);
      __builtin_amdgcn_sched_barrier(0);
      if (prev) mm(pa, pb, 2);
      __builtin_amdgcn_sched_barrier(0);
      if (next_kc >= 0) issue(next_kc, buf ^ 1);   // the next chunk's loads, once the matrix cores have work queued
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int g8 = 0; g8 + 1 < NG; ++g8) {
        mm(af[g8], bf[g8], 0);
        __builtin_amdgcn_sched_barrier(0);
        rd(g8 + 1);
        __builtin_amdgcn_sched_barrier(0);
        mm(af[g8], bf[g8], 1);
        __builtin_amdgcn_sched_barrier(0);
      }
      pa = af[NG - 1];
      pb = bf[NG - 1];
      __builtin_amdgcn_sched_barrier(0);      // nothing of the next chunk's wait and barrier moves up among them
    };
    // The barrier that opens chunk kc says two things: every wave's part of chunk kc has
    // landed in LDS (each wave waits for its own loads first), and every wave is done with
    // chunk kc-1, whose stage the loads of chunk kc+1 may now overwrite.
    if constexpr (KS == 2) {
      // group u takes the chunks u, u + 2, ...: `mine` of them; both groups pass the same barriers
      // (those of group 0, which has the odd chunk), a group without a chunk left only waits
      const int mine = (n_chunks + 1 - ugrp) >> 1, rounds = (n_chunks + 1) >> 1;
      if (ugrp) advance();
      if (mine > 0) issue(ugrp, 0);
      int j = 0;
      for (; j + 2 <= rounds; j += 2) {
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
        if (j < mine) compute_direct(0, j > 0, j + 1 < mine ? ugrp + 2 * (j + 1) : -1);
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
        if (j + 1 < mine) compute_direct(1, true, j + 2 < mine ? ugrp + 2 * (j + 2) : -1);
      }
      if (j < rounds) {
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
        if (j < mine) compute_direct(0, j > 0);
      }
      if (mine > 0) mm(pa, pb, 2);
      // group 1's sums go to group 0 through LDS (16 KB over stage 0 of As, which nobody reads any more)
      __syncthreads();
      float* red = As + (wave * 16) * 64 + lane;
      if (ugrp == 1) {
#pragma unroll
        for (int v = 0; v < 16; ++v) red[v * 64] = acc[v];
      }
      __syncthreads();
      if (ugrp == 1) return;
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[v] += red[v * 64];
    } else {
    issue(0, 0);
    int kc = 0;
    for (; kc + 2 <= n_chunks; kc += 2) {     // whole pairs of chunks: stage 0, then stage 1
      __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0): this wave's loads are in LDS
      __syncthreads();
      compute_direct(0, kc > 0, kc + 1);
      __builtin_amdgcn_s_waitcnt(0x0F70);
      __syncthreads();
      compute_direct(1, true, kc + 2 < n_chunks ? kc + 2 : -1);
    }
    if (kc < n_chunks) {                      // an odd number of chunks: the last one sits in stage 0
      __builtin_amdgcn_s_waitcnt(0x0F70);
      __syncthreads();
      compute_direct(0, kc > 0);
    }
    mm(pa, pb, 2);                            // n_chunks >= 1
    }
#endif
  } else {
    // one element per load: thread -> k column tid % BK, rows tid / BK + RP * i
    constexpr int RP = 256 / BK;                 // rows per pass
    constexpr int AI = BM / RP, BI = BN / RP;
    constexpr int LDE = LD * 4 / ES;             // LDS row pitch in elements
    const int kcol = tid & (BK - 1), row0 = tid / BK;
    const T* in = static_cast<const T*>(g.in);
    const T* wp = static_cast<const T*>(g.w);
    T* AsE = reinterpret_cast<T*>(As);
    T* BsE = reinterpret_cast<T*>(Bs);
    RowPos rp[AI];
#pragma unroll
    for (int i = 0; i < AI; ++i) rp[i] = decode_row(g, m0 + row0 + RP * i, M);
    struct RegsA { T v[AI]; } ra0, ra1;
    struct RegsB { T v[BI]; } rb0, rb1;
    auto load_chunk = [&](RegsA& ra, RegsB& rb, int&, int kc) {
      const int k = kc * BK + kcol;
      const bool kok = k < K;
      const int kk = kok ? k : 0;
      const int tap = kk / g.c, c = kk - tap * g.c;
      const int kr = tap / g.s, kt = tap - kr * g.s;
#pragma unroll
      for (int i = 0; i < AI; ++i) {
        const int iy = rp[i].iy0 + kr, ix = rp[i].ix0 + kt;
        const bool ok = kok && rp[i].ok && (unsigned)iy < (unsigned)g.h && (unsigned)ix < (unsigned)g.wd;
        ra.v[i] = ok ? in[(size_t)(rp[i].pix + iy * g.wd + ix) * g.c + c] : T(0);
      }
#pragma unroll
      for (int i = 0; i < BI; ++i) {
        const int n = n0 + row0 + RP * i;
        rb.v[i] = (kok && n < g.n_out) ? wp[(size_t)n * K + k] : T(0);
      }
    };
    auto store_chunk = [&](const RegsA& ra, const RegsB& rb, int, int buf) {
#pragma unroll
      for (int i = 0; i < AI; ++i) AsE[buf * (BM * LDE) + (row0 + RP * i) * LDE + kcol] = ra.v[i];
#pragma unroll
      for (int i = 0; i < BI; ++i) BsE[buf * (BN * LDE) + (row0 + RP * i) * LDE + kcol] = rb.v[i];
    };
    main_loop(load_chunk, store_chunk, ra0, rb0, ra1, rb1);
  }

  // epilogue: accumulator register v of a lane holds row 8*(v/4) + 4*(lane/32) + v%4,
  // column lane%32 of its 32x32 block
  const int n = n0 + wn0 + (lane & 31);
  if (!ACT && g.stats) {
    // sums of the column and of its squares over the wave's 32 rows (rows beyond M are exact
    // zeros: their operand rows were zero), for the batch norm that follows: its slab
    // tile_m * 2 + (0 or 1).  Fixed order: the lane's 16 values, then the partner lane.
    float sum = 0.f, sq = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      sum += acc[v];
      sq = fmaf(acc[v], acc[v], sq);
    }
    sum += __shfl_xor(sum, 32);
    sq += __shfl_xor(sq, 32);
    if (lane < 32 && n < g.n_out) {
      const size_t slab = (size_t)tile_m * 2 + (wave >> 1);
      g.stats[slab * g.n_out + n] = sum;
      g.stats[((size_t)g.stats_stride + slab) * g.n_out + n] = sq;
    }
  }
  if (!ACT && g.bnb.sums) {
    // Data gradient whose result is the gradient of a batch norm's ReLU output: mask it with
    // [y > 0] and leave the sums of g and g * xhat over the wave's 32 rows for that batch
    // norm's backward pass (dense output: element (m, n) of x and y sits at m * n_out + n).
    // (Fetching y and x before the K loop instead, to hide their latency, measured slower with
    // the weight-gradient stream beside: 1141 against 1164 images/s; in an instance of its own, so that
    // the other launches keep their registers, and behind the first chunk's loads: 1260 against 1268.)
    const bool col = n < g.n_out;
    const float mu = col ? g.bnb.mean[n] : 0.f, is = col ? g.bnb.istd[n] : 0.f;
    // the lane's first row; its other rows lie dr = 8*(v/4) + v%4 rows further on, a distance
    // that is the same for every lane (one scalar product per v, no per-lane 64-bit multiply)
    const int mb = m0 + wm0 + 4 * (lane >> 5);
    const int left = !col ? 0 : m0 + BM <= M ? 64 : M - mb;   // rows of the lane that exist, counted from mb
    const size_t at0 = (size_t)(mb < M ? mb : 0) * g.n_out + (col ? n : 0);
    const T* bx = static_cast<const T*>(g.bnb.x) + at0;
    const T* by = static_cast<const T*>(g.bnb.y) + at0;
    float s0 = 0.f, s1 = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int dr = 8 * (v >> 2) + (v & 3);
      float gv = 0.f, xh = 0.f;
      if (dr < left) {
        const size_t at = (size_t)dr * g.n_out;
        gv = Elem<T>::load(by + at) > 0.f ? acc[v] : 0.f;
        xh = (Elem<T>::load(bx + at) - mu) * is;
      }
      acc[v] = gv;
      s0 += gv;
      s1 = fmaf(gv, xh, s1);
    }
    s0 += __shfl_xor(s0, 32);
    s1 += __shfl_xor(s1, 32);
    if (lane < 32 && col) {
      const size_t slab = (size_t)tile_m * 2 + (wave >> 1);
      g.bnb.sums[slab * g.n_out + n] = s0;
      g.bnb.sums[((size_t)g.bnb.stride + slab) * g.n_out + n] = s1;
    }
  }
  if (n >= g.n_out) return;
  // ACT: the instantiation whose epilogue adds a bias and applies a ReLU (it never accumulates)
  float bias_n = 0.f;
  if constexpr (ACT) bias_n = g.bias ? g.bias[n] : 0.f;
  if (g.out_stride == 1 && g.out_h == g.p && g.out_w == g.q) {
    // dense result (every forward pass, every stride-1 data gradient): row m at m * n_out.  One
    // pointer per lane, the sixteen rows at distances that are the same for every lane.
    const int mb = m0 + wm0 + 4 * (lane >> 5);
    const int left = m0 + BM <= M ? 64 : M - mb;      // a whole tile (all but the last row tile): no row is tested
    T* o0 = static_cast<T*>(g.out) + (size_t)(mb < M ? mb : 0) * g.n_out + n;
    if (m0 + BM <= M && !(!ACT && g.accumulate)) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        float val = acc[v];
        if constexpr (ACT) {
          val += bias_n;
          if (g.relu) val = fmaxf(val, 0.f);
        }
        Elem<T>::store(o0 + (size_t)(8 * (v >> 2) + (v & 3)) * g.n_out, val);
      }
      return;
    }
    if (!ACT && g.accumulate) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int dr = 8 * (v >> 2) + (v & 3);
        if (dr >= left) continue;
        T* o = o0 + (size_t)dr * g.n_out;
        Elem<T>::store(o, acc[v] + (have_old ? old[v] : Elem<T>::load(o)));
      }
    } else {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int dr = 8 * (v >> 2) + (v & 3);
        if (dr >= left) continue;
        float val = acc[v];
        if constexpr (ACT) {
          val += bias_n;
          if (g.relu) val = fmaxf(val, 0.f);
        }
        Elem<T>::store(o0 + (size_t)dr * g.n_out, val);
      }
    }
    return;
  }
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int m = m0 + wm0 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
    if (m >= M) continue;
    T* o = static_cast<T*>(g.out) + out_row_offset(g, m) + n;
    float val = acc[v];
    if constexpr (ACT) {
      val += bias_n;
      if (g.relu) val = fmaxf(val, 0.f);
    } else {
      if (g.accumulate) val += Elem<T>::load(o);
    }
    Elem<T>::store(o, val);
  }
}

template <int LOADER, class T>
hipError_t launch(const ConvGeom& g, int M, int K, hipStream_t st, LaunchProbe* probe) {
  const int tm = (M + BM - 1) / BM, tn = (g.n_out + BN - 1) / BN;
  const long tiles = (long)tm * tn;
  if (tiles <= 0 || tiles > (1L << 30)) return hipErrorInvalidValue;
  const int main_grid = (int)((tiles + 7) / 8 * 8);
  long side_blocks = 0;
  if (g.side.count) {
    if (!g.side.part || !g.side.dw || g.side.splits < 1) return hipErrorInvalidValue;
    side_blocks = (long)((g.side.count + 1023) / 1024);
  }
  if ((g.bias || g.relu) && (g.accumulate || g.stats || g.bnb.sums)) return hipErrorInvalidValue;
  if (g.stats) {
    // dense fp32 result only, and no more slabs than the batch-norm workspace holds
    if (g.dtype != DT_F32 || g.accumulate || g.out_stride != 1 || g.out_h != g.p || g.out_w != g.q ||
        conv_stat_slabs((long)g.n_img * g.p * g.q) > g.stats_stride)
      return hipErrorInvalidValue;
  }
  if (g.bnb.sums) {
    if (!g.bnb.x || !g.bnb.y || !g.bnb.mean || !g.bnb.istd || g.dtype != DT_F32 || g.accumulate || g.out_stride != 1 ||
        g.out_h != g.p || g.out_w != g.q || conv_stat_slabs((long)g.n_img * g.p * g.q) > g.bnb.stride)
      return hipErrorInvalidValue;
  }
  if (g.flip.wt) {
    if (!g.flip.w || g.flip.cout <= 0 || g.flip.cin <= 0 || g.flip.r <= 0 || g.flip.s <= 0) return hipErrorInvalidValue;
    side_blocks += (long)((g.flip.cin + 31) / 32) * ((g.flip.cout + 31) / 32) * g.flip.r * g.flip.s;
  }
  if (main_grid + side_blocks > (1L << 30)) return hipErrorInvalidValue;
  const dim3 grid((unsigned)(main_grid + side_blocks));
  // at most one tile per compute unit and at least eight chunks of K: two groups of waves per tile
  // (a function of the shape only)
  constexpr int BKE = direct_chunk_bytes((int)sizeof(T)) / (int)sizeof(T);
  const bool split = LOADER == L_DIRECT && sizeof(T) == 4 && !(g.bias || g.relu) && tiles <= 256 && K >= 8 * BKE;
  if (split) probe->variant = V_IGEMM_DIRECT_2G;
  if (probe->before) (void)hipEventRecord(probe->before, st);
  if (g.bias || g.relu)
    hipLaunchKernelGGL((igemm_kernel<LOADER, T, true>), grid, dim3(256), 0, st, g, M, K, tn, (int)tiles, main_grid);
  else if constexpr (LOADER == L_DIRECT && sizeof(T) == 4) {
    if (split)
      hipLaunchKernelGGL((igemm_kernel<LOADER, T, false, 2>), grid, dim3(512), 0, st, g, M, K, tn, (int)tiles, main_grid);
    else
      hipLaunchKernelGGL((igemm_kernel<LOADER, T, false>), grid, dim3(256), 0, st, g, M, K, tn, (int)tiles, main_grid);
  } else
    hipLaunchKernelGGL((igemm_kernel<LOADER, T, false>), grid, dim3(256), 0, st, g, M, K, tn, (int)tiles, main_grid);
  if (probe->after) (void)hipEventRecord(probe->after, st);
  return hipGetLastError();
}

}  // namespace

const char* conv_variant_name(int v) {
  static const char* names[V_COUNT] = {"igemm_kernel<fast>", "igemm_kernel<generic>", "wgrad_kernel<fast>",
                                       "wgrad_kernel<generic>", "igemm_kernel<direct>", "wgrad_kernel<direct>",
                                       "wgrad_bf16_kernel", "igemm_bf16_kernel", "igemm_kernel<direct, two groups>"};
  return (v >= 0 && v < V_COUNT) ? names[v] : "?";
}

hipError_t conv_igemm(const ConvGeom& g, hipStream_t st, LaunchProbe* probe) {
  LaunchProbe local;
  if (!probe) probe = &local;
  if (!g.in || !g.w || !g.out) return hipErrorInvalidValue;
  if (g.n_img <= 0 || g.h <= 0 || g.wd <= 0 || g.c <= 0 || g.p <= 0 || g.q <= 0 || g.n_out <= 0 ||
      g.r <= 0 || g.s <= 0 || g.stride <= 0 || g.pad < 0 || g.pad + g.pad_dx < 0 || g.out_stride <= 0 ||
      g.out_y0 < 0 || g.out_x0 < 0)
    return hipErrorInvalidValue;
  // every gathered coordinate p*stride+r-pad is range-checked in the kernel; the output
  // pixel (out_y0 + p*out_stride, out_x0 + q*out_stride) must exist
  if (g.out_y0 + (long)(g.p - 1) * g.out_stride >= g.out_h || g.out_x0 + (long)(g.q - 1) * g.out_stride >= g.out_w)
    return hipErrorInvalidValue;
  const long M = (long)g.n_img * g.p * g.q;
  const long K = (long)g.r * g.s * g.c;
  if (M >= (1L << 31) || K >= (1L << 31) || (long)g.n_img * g.h * g.wd >= (1L << 31))
    return hipErrorInvalidValue;
  if (g.dtype != DT_F32 && g.dtype != DT_BF16) return hipErrorInvalidValue;
  if ((g.bias || g.relu) && (g.accumulate || g.stats || g.bnb.sums)) return hipErrorInvalidValue;
  if (conv_igemm_bf16_takes(g, M, K)) {    // bf16 storage, large layers: 128 x 128 tiles
    probe->variant = V_IGEMM_BF16;
    return conv_igemm_bf16(g, (int)M, (int)K, st, probe);
  }
  const long es = (long)dt_size(g.dtype);
  // The direct loader addresses both operands through buffer descriptors: 32-bit ranges, the
  // last bytes kept free for the offset that stands for "outside"; 16-byte loads want aligned
  // tensors.  The choice depends on the shape and the alignment only, never on the swap plan
  // (pool offsets are multiples of 256).
  const long margin_px = (long)g.pad * g.wd + g.pad + g.pad_dx;
  const bool direct = (g.c % (direct_chunk_bytes((int)es) / es) == 0) && g.r * g.s <= 32 &&
                      (margin_px + (long)g.n_img * g.h * g.wd) * g.c * es <= 0xFFFFFF00L &&
                      (long)g.n_out * K * es <= 0xFFFFFF00L &&
                      (reinterpret_cast<uintptr_t>(g.in) & 15) == 0 && (reinterpret_cast<uintptr_t>(g.w) & 15) == 0;
  probe->variant = direct ? V_IGEMM_DIRECT : V_IGEMM_GENERIC;
  if (g.dtype == DT_F32)
    return direct ? launch<L_DIRECT, float>(g, (int)M, (int)K, st, probe) : launch<L_GENERIC, float>(g, (int)M, (int)K, st, probe);
  return direct ? launch<L_DIRECT, bf16_t>(g, (int)M, (int)K, st, probe) : launch<L_GENERIC, bf16_t>(g, (int)M, (int)K, st, probe);
}

}  // namespace acc
