// Weight gradient of a convolution as a GEMM over the minibatch positions:
//
//   dw[co][j] = sum_m dy[m][co] * X[m][j],   m = (img,p,q),  j = (r,t,ci), ci fastest,
//   X[m][j] = x[img, p*stride+r-pad, q*stride+t-pad, ci]  (zero in the padding)
//
// Both operands are read along their contiguous channel axis and staged in LDS as
// [m][channel]; the fp32 MFMA (v_mfma_f32_32x32x2_f32) takes k = m.  A workgroup of 4
// waves owns a 64 x 64 tile of dw; the m range is cut into `splits` equal parts
// (grid.y); each part writes its own partial tile and a second kernel adds the parts in
// a fixed order, so the result is deterministic (no atomics).
//
// Pipeline as in the forward kernel: two chunks of 32 rows in LDS, two more in
// registers, every steady-state load unconditional (rows beyond the range and padded taps
// read a stand-in address and are zeroed on the way into LDS), one barrier per chunk.
// 64x64 tiles measured best on MI355X (ResNet shapes, minibatch 32 / 256: 66 / 91
// TFLOP/s against 48 / 86 with 128-wide tiles).
#include <cstdlib>

#include "kernels.h"
#include "dtype.h"

namespace acc {
namespace {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef unsigned v2u __attribute__((ext_vector_type(2)));

// four consecutive elements as they come from memory, and as the fp32 values the MFMA takes
// (bf16 operands are widened on the way into LDS: their products are exact in fp32, so the
// result is that of a bf16 product accumulated in fp32)
template <class T> struct Quad;
template <> struct Quad<float> {
  typedef v4f raw;
  static __device__ __forceinline__ v4f widen(const raw& r) { return r; }
};
template <> struct Quad<bf16_t> {
  typedef v2u raw;
  static __device__ __forceinline__ v4f widen(const raw& r) {
    return v4f{__uint_as_float(r.x << 16), __uint_as_float(r.x & 0xffff0000u), __uint_as_float(r.y << 16),
               __uint_as_float(r.y & 0xffff0000u)};
  }
};
constexpr int BKM = 32;          // rows of m per chunk
constexpr int BM = 64, BN = 64;  // tile of dw: output channels x filter columns
constexpr int LDT = 64 + 32;     // LDS pitch: lanes 32-63 read the next row on other banks

__device__ __forceinline__ v16f mfma32x32x2(float a, float b, v16f c) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
#else
  return c;  // the host pass never runs this
#endif
}

__device__ __forceinline__ void sched_fence() {
#if defined(__HIP_DEVICE_COMPILE__)
  __builtin_amdgcn_sched_barrier(0);
#endif
}

// pixel index of the input position for GEMM row m and tap (kr,kt); -1 = padding
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

// Side jobs of a weight-gradient launch (workgroups appended behind the tiles): first the
// blocks that add up 1024 elements each of an earlier weight gradient's parts, in their fixed
// order; then the blocks that write one 32 x 32 (co, ci) block each of one tap of the flipped,
// transposed filter.  scratch: at least 32 x 33 elements of LDS.
template <class T>
__device__ __forceinline__ void side_jobs(const WgradGeom& g, int id, float* scratch) {
  const ReduceJob& rj = g.side;
  const int reduce_blocks = (int)((rj.count + 1023) / 1024);
  if (id < reduce_blocks) {
    const size_t i4 = ((size_t)id * 256 + threadIdx.x) * 4;
    if (i4 >= rj.count) return;
    if (i4 + 4 <= rj.count && (rj.count & 3) == 0) {
      float4 sum = *reinterpret_cast<const float4*>(rj.part + i4);
      // eight parts fetched at a time, added in their order: with hundreds of parts (few tiles, many
      // cuts of the minibatch range) one load waiting for the sum before it is a chain of latencies
      int k = 1;
      for (; k + 8 <= rj.splits; k += 8) {
        float4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const float4*>(rj.part + (size_t)(k + u) * rj.count + i4);
#pragma unroll
        for (int u = 0; u < 8; ++u) { sum.x += v[u].x; sum.y += v[u].y; sum.z += v[u].z; sum.w += v[u].w; }
      }
      for (; k < rj.splits; ++k) {
        const float4 v = *reinterpret_cast<const float4*>(rj.part + (size_t)k * rj.count + i4);
        sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
      }
      *reinterpret_cast<float4*>(rj.dw + i4) = sum;
    } else {
      for (size_t i = i4; i < rj.count && i < i4 + 4; ++i) {
        float sum = rj.part[i];
        for (int k = 1; k < rj.splits; ++k) sum += rj.part[(size_t)k * rj.count + i];
        rj.dw[i] = sum;
      }
    }
    return;
  }
  id -= reduce_blocks;
  if (!g.flip_wt) return;
  const int bx = (g.cin + 31) / 32, by = (g.cout + 31) / 32;
  const int tap = id / (bx * by), rem = id - tap * (bx * by);
  const int co0f = (rem / bx) * 32, ci0f = (rem - (rem / bx) * bx) * 32;
  const int kr = g.r - 1 - tap / g.s, kt = g.s - 1 - tap % g.s;
  const int src_tap = kr * g.s + kt;
  T (*tile)[33] = reinterpret_cast<T (*)[33]>(scratch);
  const T* fw = static_cast<const T*>(g.flip_w);
  T* fwt = static_cast<T*>(g.flip_wt);
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  for (int i = ty; i < 32; i += 8) {
    const int co = co0f + i, ci = ci0f + tx;
    tile[i][tx] = (co < g.cout && ci < g.cin) ? fw[((size_t)co * g.r * g.s + src_tap) * g.cin + ci] : T(0);
  }
  __syncthreads();
  for (int i = ty; i < 32; i += 8) {
    const int ci = ci0f + i, co = co0f + tx;
    if (ci < g.cin && co < g.cout) fwt[((size_t)ci * g.r * g.s + tap) * g.cout + co] = tile[tx][i];
  }
}

// L_FAST, L_DIRECT: cin % 64 == 0 (a tile's columns lie inside one tap), cout % 4 == 0, byte
// offsets below 2^32.  L_DIRECT (fp32 storage only: bf16 operands are widened on their way
// into LDS, which needs the registers) moves the chunks from global memory straight into LDS
// (buffer_load_dwordx4 ... lds: a wave fills four 256-byte rows), rows beyond the range,
// padded taps and columns beyond cout as offsets outside the buffer descriptor, which read as
// zero.  Rows are unpadded; odd rows hold their two 128-byte halves swapped (the lane fetches
// the half that belongs into its slot), so that the two rows one MFMA operand is read from
// lie on different banks.  Two LDS stages, as in the forward kernel's direct loader.
enum { L_GENERIC = 0, L_FAST = 1, L_DIRECT = 2 };

template <int LOADER, class T>
__global__ __launch_bounds__(256) void wgrad_kernel(WgradGeom g, int Mrows, int J, int tiles_j, int tiles,
                                                     int splits, int chunks_per_split, float* out,
                                                     size_t split_stride, int main_grid) {
  constexpr bool FAST = LOADER == L_FAST, DIRECT = LOADER == L_DIRECT;
  constexpr int PITCH = DIRECT ? 64 : LDT;
  __shared__ __attribute__((aligned(256))) float As[2 * BKM * PITCH];
  __shared__ __attribute__((aligned(256))) float Bs[2 * BKM * PITCH];

  if ((int)blockIdx.x >= main_grid) {
    side_jobs<T>(g, (int)blockIdx.x - main_grid, As);
    return;
  }

  // XCD-aware order: consecutive workgroup ids land on different XCDs, so each XCD gets a
  // contiguous range of (split, tile) pairs: the tiles of one split read the same rows of
  // x and dy and find them in that XCD's L2 instead of fetching them once per XCD.
  const int per_xcd = main_grid >> 3;
  const int work = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (work >= tiles * splits) return;
  const int split = work / tiles, tile = work - split * tiles;
  const int tile_co = tile / tiles_j, tile_j = tile - tile_co * tiles_j;
  const int co0 = tile_co * BM, j0 = tile_j * BN;
  const int chunk_lo = split * chunks_per_split;
  const int n_chunks_all = (Mrows + BKM - 1) / BKM;
  const int chunk_hi = min(chunk_lo + chunks_per_split, n_chunks_all);
  const int n_chunks = chunk_hi - chunk_lo;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave >> 1) * 32, wn0 = (wave & 1) * 32;

  v16f acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;

  auto compute_chunk = [&](int cur) {
    const float* as = As + cur * (BKM * LDT) + (lane >> 5) * LDT + wm0 + (lane & 31);
    const float* bs = Bs + cur * (BKM * LDT) + (lane >> 5) * LDT + wn0 + (lane & 31);
#pragma unroll
    for (int kk = 0; kk < BKM; kk += 2) acc = mfma32x32x2(as[kk * LDT], bs[kk * LDT], acc);
  };
  // The same with the first four operand pairs fetched by the caller, early enough for the
  // stores and global loads of the half-iteration to cover their LDS latency.
  constexpr int EARLY = 4;
  auto first_frag = [&](int cur, float (&a)[EARLY], float (&b)[EARLY]) {
    const float* as = As + cur * (BKM * LDT) + (lane >> 5) * LDT + wm0 + (lane & 31);
    const float* bs = Bs + cur * (BKM * LDT) + (lane >> 5) * LDT + wn0 + (lane & 31);
#pragma unroll
    for (int u = 0; u < EARLY; ++u) { a[u] = as[2 * u * LDT]; b[u] = bs[2 * u * LDT]; }
  };
  auto compute_chunk2 = [&](int cur, const float (&a)[EARLY], const float (&b)[EARLY]) {
    const float* as = As + cur * (BKM * LDT) + (lane >> 5) * LDT + wm0 + (lane & 31);
    const float* bs = Bs + cur * (BKM * LDT) + (lane >> 5) * LDT + wn0 + (lane & 31);
#pragma unroll
    for (int u = 0; u < EARLY; ++u) acc = mfma32x32x2(a[u], b[u], acc);
#pragma unroll
    for (int kk = 2 * EARLY; kk < BKM; kk += 2) acc = mfma32x32x2(as[kk * LDT], bs[kk * LDT], acc);
  };

  // same schedule as the forward kernel: chunk c (relative to chunk_lo) lives in LDS half
  // c & 1; chunks c+1 and c+2 wait in the two register sets
  auto main_loop = [&](auto& load, auto& store, auto& r0, auto& r1) {
    if (n_chunks <= 0) return;
    int kc = 0;
    load(r0, 0);
    store(r0, 0);
    if (n_chunks >= 5) {
      load(r1, 1);
      load(r0, 2);
      __syncthreads();
      for (; kc + 4 < n_chunks; kc += 2) {
        float fa[EARLY], fb[EARLY];
        sched_fence();
        first_frag(0, fa, fb);
        sched_fence();
        store(r1, 1);
        load(r1, kc + 3);
        sched_fence();
        compute_chunk2(0, fa, fb);
        __syncthreads();
        sched_fence();
        first_frag(1, fa, fb);
        sched_fence();
        store(r0, 0);
        load(r0, kc + 4);
        sched_fence();
        compute_chunk2(1, fa, fb);
        __syncthreads();
      }
    } else {
      if (n_chunks > 1) load(r1, 1);
      if (n_chunks > 2) load(r0, 2);
      __syncthreads();
    }
    for (; kc < n_chunks; kc += 2) {
      sched_fence();
      if (kc + 1 < n_chunks) store(r1, 1);
      if (kc + 3 < n_chunks) load(r1, kc + 3);
      sched_fence();
      compute_chunk(0);
      __syncthreads();
      if (kc + 1 >= n_chunks) break;
      sched_fence();
      if (kc + 2 < n_chunks) store(r0, 0);
      if (kc + 4 < n_chunks) load(r0, kc + 4);
      sched_fence();
      compute_chunk(1);
      __syncthreads();
    }
  };

  if constexpr (DIRECT) {
#if defined(__HIP_DEVICE_COMPILE__)
    static_assert(!DIRECT || sizeof(T) == 4, "the direct loader copies raw fp32 rows");
    // lane -> LDS slot: row tid/16 (+16 on the second pass), 16-byte column tid%16; the slot of
    // an odd row holds the column of the other half
    const int row = tid >> 4;
    const int col4 = (tid & 15) ^ ((row & 1) << 3);
    const int tap = j0 / g.cin, ci0 = j0 - tap * g.cin;
    const int kr = tap / g.s, kt = tap - kr * g.s;
    const bool plain = g.r == 1 && g.s == 1 && g.stride == 1 && g.pad == 0;
    const bool a_col_ok = co0 + col4 * 4 < g.cout;
    constexpr uint32_t OUTSIDE = 0xFFFFFFF0u;
    uint32_t a_lane[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) a_lane[i] = (uint32_t)(row + 16 * i) * (uint32_t)(g.cout * 4) + (uint32_t)(co0 + col4 * 4) * 4;
    const uint32_t b_lane = (uint32_t)(ci0 + col4 * 4) * 4;
    int r_org[2] = {0, 0}, r_p[2] = {0, 0}, r_q[2] = {0, 0};
    const float inv_q = 1.0f / (float)g.q, inv_p = 1.0f / (float)g.p;
    if (!plain) {
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int m = chunk_lo * BKM + row + 16 * i;
        const int pq = g.p * g.q;
        const int img = m / pq, rem = m - img * pq;
        r_p[i] = rem / g.q;
        r_q[i] = rem - r_p[i] * g.q;
        r_org[i] = img * g.h * g.wd;
      }
    }
    __amdgpu_buffer_rsrc_t rs_a = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void*>(g.dy), 0, (int)(uint32_t)((size_t)Mrows * g.cout * 4), 0x00020000);
    __amdgpu_buffer_rsrc_t rs_b = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void*>(g.x), 0, (int)(uint32_t)((size_t)g.n_img * g.h * g.wd * g.cin * 4), 0x00020000);
    typedef __attribute__((address_space(3))) void* lds_ptr;
    const int uwave = __builtin_amdgcn_readfirstlane(wave);
    const uint32_t lds_a = (uint32_t)(size_t)As + uwave * 1024, lds_b = (uint32_t)(size_t)Bs + uwave * 1024;
    // loads of chunk kc (relative to chunk_lo) into stage buf; chunks are issued in order, so the
    // gathered position advances by BKM rows per call without any division
    auto issue = [&](int kc, int buf) {
      const int mbase = (chunk_lo + kc) * BKM;
      const int soff_a = (int)((uint32_t)mbase * (uint32_t)(g.cout * 4));   // below 2^32 (launcher)
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int m = mbase + row + 16 * i;
        const bool mok = m < Mrows;
        const uint32_t va = (mok && a_col_ok) ? a_lane[i] : OUTSIDE;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_a, (lds_ptr)(size_t)(lds_a + buf * (BKM * 256) + i * (16 * 256)), 16, va,
                                                 soff_a, 0, 0);
        int pix = m;
        if (!plain) {
          const int iy = r_p[i] * g.stride + kr - g.pad, ix = r_q[i] * g.stride + kt - g.pad;
          pix = ((unsigned)iy < (unsigned)g.h && (unsigned)ix < (unsigned)g.wd) ? r_org[i] + iy * g.wd + ix : -1;
          // 32 positions on, without a loop that runs differently in every lane: the number of
          // rows and of images passed are small quotients, exact in float with the half added
          const int xq = r_q[i] + BKM;
          const int wq = (int)(((float)xq + 0.5f) * inv_q);
          r_q[i] = xq - wq * g.q;
          const int xp = r_p[i] + wq;
          const int wp = (int)(((float)xp + 0.5f) * inv_p);
          r_p[i] = xp - wp * g.p;
          r_org[i] += wp * (g.h * g.wd);
        }
        const uint32_t vb = (mok && pix >= 0) ? (uint32_t)pix * (uint32_t)(g.cin * 4) + b_lane : OUTSIDE;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_b, (lds_ptr)(size_t)(lds_b + buf * (BKM * 256) + i * (16 * 256)), 16, vb,
                                                 0, 0, 0);
      }
    };
    // operand of MFMA step kk: lanes 0-31 row kk (even), lanes 32-63 row kk+1 (odd: halves swapped)
    const int half = lane >> 5;
    const float* a_rd = As + half * 64 + ((wm0 + (lane & 31)) ^ (half << 5));
    const float* b_rd = Bs + half * 64 + ((wn0 + (lane & 31)) ^ (half << 5));
    // Groups of four MFMAs (eight rows of the chunk): the operands of group g + 1 are read between the MFMAs
    // of group g, and the last group's MFMAs are held back (pa, pb) until the next chunk's barrier has been
    // passed and its first reads are on their way.  Same order of additions.
    constexpr int NG = BKM / 8;
    float pa[4] = {0.f, 0.f, 0.f, 0.f}, pb[4] = {0.f, 0.f, 0.f, 0.f};
    auto mm4 = [&](const float (&a)[4], const float (&b)[4], int half) {
      if (half != 1) {
        acc = mfma32x32x2(a[0], b[0], acc);
        acc = mfma32x32x2(a[1], b[1], acc);
      }
      if (half != 0) {
        acc = mfma32x32x2(a[2], b[2], acc);
        acc = mfma32x32x2(a[3], b[3], acc);
      }
    };
    auto compute_direct = [&](int buf, bool prev) {
      const float* as = a_rd + buf * (BKM * 64);
      const float* bs = b_rd + buf * (BKM * 64);
      float af[NG][4], bf[NG][4];
      auto rd = [&](int g) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          af[g][u] = as[(g * 8 + u * 2) * 64];
          bf[g][u] = bs[(g * 8 + u * 2) * 64];
        }
      };
      rd(0);
      __builtin_amdgcn_sched_barrier(0);
      if (prev) mm4(pa, pb, 2);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int g = 0; g + 1 < NG; ++g) {
        mm4(af[g], bf[g], 0);
        __builtin_amdgcn_sched_barrier(0);
        rd(g + 1);
        __builtin_amdgcn_sched_barrier(0);
        mm4(af[g], bf[g], 1);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) { pa[u] = af[NG - 1][u]; pb[u] = bf[NG - 1][u]; }
      __builtin_amdgcn_sched_barrier(0);
    };
    if (n_chunks > 0) {
      issue(0, 0);
      int kc = 0;
      for (; kc + 2 <= n_chunks; kc += 2) {     // whole pairs of chunks: stage 0, then stage 1
        __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0): this wave's part of chunk kc is in LDS
        __syncthreads();                        // everybody's is, and chunk kc-1 has been read by all
        issue(kc + 1, 1);
        compute_direct(0, kc > 0);
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
        if (kc + 2 < n_chunks) issue(kc + 2, 0);
        compute_direct(1, true);
      }
      if (kc < n_chunks) {                      // an odd number of chunks: the last one sits in stage 0
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
        compute_direct(0, kc > 0);
      }
      mm4(pa, pb, 2);
    }
#endif
  } else if constexpr (FAST) {
    // 16 float4 per 64-wide row, 16 rows per pass, 2 passes per operand and chunk
    const int col4 = tid & 15, row = tid >> 4;
    const int tap = j0 / g.cin, ci0 = j0 - tap * g.cin;
    const int kr = tap / g.s, kt = tap - kr * g.s;
    const bool direct = g.r == 1 && g.s == 1 && g.stride == 1 && g.pad == 0;
    const bool a_col_ok = co0 + col4 * 4 < g.cout;
    constexpr int ES = sizeof(T);
    typedef typename Quad<T>::raw raw;
    const uint32_t a_lane = (uint32_t)(a_col_ok ? co0 + col4 * 4 : 0) * ES;
    const uint32_t b_lane = (uint32_t)(ci0 + col4 * 4) * ES;
    struct Regs {
      raw a[2], b[2];
      uint32_t ok;   // bit i: a[i] valid, bit 2+i: b[i] valid
    } r0, r1;
    // position of each gathered row; chunks are visited in order, so the position advances
    // by BKM rows per chunk without any division
    int r_org[2] = {0, 0}, r_p[2] = {0, 0}, r_q[2] = {0, 0};
    if (!direct) {
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int m = chunk_lo * BKM + row + 16 * i;
        const int pq = g.p * g.q;
        const int img = m / pq, rem = m - img * pq;
        r_p[i] = rem / g.q;
        r_q[i] = rem - r_p[i] * g.q;
        r_org[i] = img * g.h * g.wd;
      }
    }
    // Unconditional loads: a row beyond Mrows, a padded tap or a column beyond cout reads
    // element 0 of its tensor and is zeroed when the chunk moves to LDS.
    auto load_chunk = [&](Regs& r, int kc) {
      const int mbase = (chunk_lo + kc) * BKM;
      const char* abase = reinterpret_cast<const char*>(g.dy);
      const char* bbase = reinterpret_cast<const char*>(g.x);
      uint32_t ok = 0;
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int m = mbase + row + 16 * i;
        const bool mok = m < Mrows;
        const uint32_t mm = mok ? (uint32_t)m : 0u;
        ok |= (mok && a_col_ok ? 1u : 0u) << i;
        r.a[i] = *reinterpret_cast<const raw*>(abase + (mm * (uint32_t)(g.cout * ES) + a_lane));
        int pix = (int)mm;
        if (!direct) {
          const int iy = r_p[i] * g.stride + kr - g.pad, ix = r_q[i] * g.stride + kt - g.pad;
          pix = ((unsigned)iy < (unsigned)g.h && (unsigned)ix < (unsigned)g.wd) ? r_org[i] + iy * g.wd + ix : -1;
          r_q[i] += BKM;
          while (r_q[i] >= g.q) {
            r_q[i] -= g.q;
            if (++r_p[i] == g.p) { r_p[i] = 0; r_org[i] += g.h * g.wd; }
          }
        }
        const bool bok = mok && pix >= 0;
        ok |= (bok ? 1u : 0u) << (2 + i);
        r.b[i] = *reinterpret_cast<const raw*>(bbase + ((uint32_t)(bok ? pix : 0) * (uint32_t)(g.cin * ES) + b_lane));
      }
      r.ok = ok;
    };
    auto store_chunk = [&](const Regs& r, int buf) {
      float* as = As + buf * (BKM * LDT);
      float* bs = Bs + buf * (BKM * LDT);
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        v4f a = Quad<T>::widen(r.a[i]), b = Quad<T>::widen(r.b[i]);
        if (!((r.ok >> i) & 1u)) a = v4f{0.f, 0.f, 0.f, 0.f};
        if (!((r.ok >> (2 + i)) & 1u)) b = v4f{0.f, 0.f, 0.f, 0.f};
        *reinterpret_cast<v4f*>(&as[(row + 16 * i) * LDT + col4 * 4]) = a;
        *reinterpret_cast<v4f*>(&bs[(row + 16 * i) * LDT + col4 * 4]) = b;
      }
    };
    main_loop(load_chunk, store_chunk, r0, r1);
  } else {
    // one element per load: column tid % 64 is fixed per thread, rows tid/64 + 4*i
    constexpr int AI = BKM / 4;
    const int col = tid & 63, row0 = tid >> 6;
    const int co = co0 + col;
    const int j = j0 + col;
    const bool jok = j < J;
    const int jj = jok ? j : 0;
    const int tap = jj / g.cin, ci = jj - tap * g.cin;
    const int kr = tap / g.s, kt = tap - kr * g.s;
    struct Regs { float a[AI], b[AI]; } r0, r1;
    // Output position (image origin, p, q) of each of the thread's rows, worked out once and then
    // moved on by the 32 rows of a chunk (chunks are loaded in order): two small quotients,
    // exact in float with the half added for p, q <= 4096, instead of two integer divisions
    // per element, which cost this loader more than its MFMAs (the 3-channel stem).
    const bool stepwise = g.p <= 4096 && g.q <= 4096;
    const float inv_q = 1.0f / (float)g.q, inv_p = 1.0f / (float)g.p;
    int r_org[AI], r_p[AI], r_q[AI];
#pragma unroll
    for (int i = 0; i < AI; ++i) {
      const int m = chunk_lo * BKM + row0 + 4 * i;
      const int pq = g.p * g.q;
      const int img = m / pq, rem = m - img * pq;
      r_p[i] = rem / g.q;
      r_q[i] = rem - r_p[i] * g.q;
      r_org[i] = img * g.h * g.wd;
    }
    auto load_chunk = [&](Regs& r, int kc) {
#pragma unroll
      for (int i = 0; i < AI; ++i) {
        const int m = (chunk_lo + kc) * BKM + row0 + 4 * i;
        const bool mok = m < Mrows;
        r.a[i] = (mok && co < g.cout) ? Elem<T>::load(static_cast<const T*>(g.dy) + (size_t)m * g.cout + co) : 0.f;
        float v = 0.f;
        if (mok && jok) {
          int pix;
          if (stepwise) {
            const int iy = r_p[i] * g.stride + kr - g.pad, ix = r_q[i] * g.stride + kt - g.pad;
            pix = ((unsigned)iy < (unsigned)g.h && (unsigned)ix < (unsigned)g.wd) ? r_org[i] + iy * g.wd + ix : -1;
          } else {
            pix = gather_pixel(g, m, kr, kt);
          }
          if (pix >= 0) v = Elem<T>::load(static_cast<const T*>(g.x) + (size_t)pix * g.cin + ci);
        }
        r.b[i] = v;
        if (stepwise) {
          const int xq = r_q[i] + BKM;
          const int wq = (int)(((float)xq + 0.5f) * inv_q);
          r_q[i] = xq - wq * g.q;
          const int xp = r_p[i] + wq;
          const int wp = (int)(((float)xp + 0.5f) * inv_p);
          r_p[i] = xp - wp * g.p;
          r_org[i] += wp * (g.h * g.wd);
        }
      }
    };
    auto store_chunk = [&](const Regs& r, int buf) {
#pragma unroll
      for (int i = 0; i < AI; ++i) {
        As[buf * (BKM * LDT) + (row0 + 4 * i) * LDT + col] = r.a[i];
        Bs[buf * (BKM * LDT) + (row0 + 4 * i) * LDT + col] = r.b[i];
      }
    };
    main_loop(load_chunk, store_chunk, r0, r1);
  }

  float* dst = out + (size_t)split * split_stride;
  const int jcol = j0 + wn0 + (lane & 31);
  if (jcol >= J) return;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int co = co0 + wm0 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
    if (co < g.cout) dst[(size_t)co * J + jcol] = acc[v];
  }
}


// ---------------------------------------------------------------------------------------------
// bf16 storage on the bf16 matrix cores (v_mfma_f32_32x32x16_bf16).  The instruction wants eight
// consecutive values of the reduction index per lane; here that index is the minibatch position
// m, and memory is contiguous along channels.  So every thread loads an 8 x 8 block (eight rows
// of m, sixteen bytes = eight channels each), transposes it in registers (32 byte permutes) and
// writes eight 16-byte vectors "channel c, rows m..m+7" into LDS, where a fragment read is one
// ds_read_b128 per lane again.  A workgroup of 4 waves owns a 128 x 128 tile of dw, each wave
// 64 x 64 (2 x 2 MFMA blocks: 16 MFMAs per 16 fragment reads and chunk of 64 rows), two LDS
// stages of 32 KB, the global loads of the next chunk in flight during the MFMAs of this one.
// Waves 0-1 stage dy, waves 2-3 gather x.  LDS layout per stage and operand: [8 row groups][128
// channels] of 16 bytes, a channel's position inside its group of eight XORed with
// (group >> 1) & 7: the eight vectors a thread writes with one instruction land on different
// banks, and so do the 32 consecutive channels a half-wave reads.
// Needs cin % 8 == 0 (the eight channels a thread stages lie inside one filter tap; the tap is the
// thread's own, a tile's 128 columns may span several) and cout % 8 == 0.
constexpr int WB_BM = 128, WB_BN = 128, WB_BK = 64;
typedef unsigned v4u __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

__device__ __forceinline__ v16f mfma32x32x16bf(const v4u& a, const v4u& b, v16f c) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, b), c, 0, 0, 0);
#else
  return c;  // the host pass never runs this
#endif
}

__device__ __forceinline__ int wb_slot(int kg, int ch) {   // 16-byte slot of (row group, channel) inside a stage
  const int o = ch >> 3;
  return kg * WB_BM + (o << 3) + ((ch & 7) ^ ((o >> 1) & 7));
}

__global__ __launch_bounds__(256) void wgrad_bf16_kernel(WgradGeom g, int Mrows, int J, int tiles_j, int tiles,
                                                          int splits, int chunks_per_split, float* out,
                                                          size_t split_stride, int main_grid) {
  __shared__ __attribute__((aligned(1024))) v4u As[2 * 8 * WB_BM];
  __shared__ __attribute__((aligned(1024))) v4u Bs[2 * 8 * WB_BN];
  if ((int)blockIdx.x >= main_grid) {
    side_jobs<bf16_t>(g, (int)blockIdx.x - main_grid, reinterpret_cast<float*>(As));
    return;
  }
#if defined(__HIP_DEVICE_COMPILE__)
  const int per_xcd = main_grid >> 3;
  const int work = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (work >= tiles * splits) return;
  const int split = work / tiles, tile = work - split * tiles;
  const int tile_co = tile / tiles_j, tile_j = tile - tile_co * tiles_j;
  const int co0 = tile_co * WB_BM, j0 = tile_j * WB_BN;
  const int chunk_lo = split * chunks_per_split;
  const int n_chunks_all = (Mrows + WB_BK - 1) / WB_BK;
  const int n_chunks = min(chunk_lo + chunks_per_split, n_chunks_all) - chunk_lo;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave >> 1) * 64, wn0 = (wave & 1) * 64;

  v16f acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  // ---- staging role of the thread: operand (uniform per wave), row group, group of eight channels
  const bool role_b = tid >= 128;
  const int u = tid & 127, oct = u & 15, kg = u >> 4;
  const int jt = j0 + oct * 8;                 // first of the thread's eight columns of dw
  const bool b_col_ok = jt < J;
  const int tap = (b_col_ok ? jt : 0) / g.cin, ci0 = (b_col_ok ? jt : 0) - tap * g.cin;
  const int kr = tap / g.s, kt = tap - kr * g.s;
  const bool plain = g.r == 1 && g.s == 1 && g.stride == 1 && g.pad == 0;
  constexpr uint32_t OUTSIDE = 0xFFFFFFF0u;   // beyond the descriptor's range: reads as zero
  const bool a_col_ok = co0 + oct * 8 < g.cout;
  const uint32_t a_lane = (uint32_t)(co0 + oct * 8) * 2u, b_lane = (uint32_t)ci0 * 2u;
  __amdgpu_buffer_rsrc_t rs = role_b
      ? __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(g.x), 0, (int)(uint32_t)((size_t)g.n_img * g.h * g.wd * g.cin * 2), 0x00020000)
      : __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(g.dy), 0, (int)(uint32_t)((size_t)Mrows * g.cout * 2), 0x00020000);
  v4u R[8];
  auto load = [&](int kc) {
    const int m0 = (chunk_lo + kc) * WB_BK + kg * 8;
    if (!role_b) {
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        const int m = m0 + r;
        const uint32_t voff = (m < Mrows && a_col_ok) ? (uint32_t)m * (uint32_t)(g.cout * 2) + a_lane : OUTSIDE;
        R[r] = __builtin_amdgcn_raw_buffer_load_b128(rs, voff, 0, 0);
      }
    } else {
      int p = 0, q = 0, org = 0;
      if (!plain) {
        const int pq = g.p * g.q;
        const int mm = m0 < Mrows ? m0 : 0;
        const int img = mm / pq, rem = mm - img * pq;
        p = rem / g.q;
        q = rem - p * g.q;
        org = img * g.h * g.wd;
      }
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        const int m = m0 + r;
        int pix = m;
        if (!plain) {
          const int iy = p * g.stride + kr - g.pad, ix = q * g.stride + kt - g.pad;
          pix = ((unsigned)iy < (unsigned)g.h && (unsigned)ix < (unsigned)g.wd) ? org + iy * g.wd + ix : -1;
          if (++q == g.q) { q = 0; if (++p == g.p) { p = 0; org += g.h * g.wd; } }
        }
        const uint32_t voff = (m < Mrows && pix >= 0 && b_col_ok) ? (uint32_t)pix * (uint32_t)(g.cin * 2) + b_lane : OUTSIDE;
        R[r] = __builtin_amdgcn_raw_buffer_load_b128(rs, voff, 0, 0);
      }
    }
  };
  // 8 x 8 transpose of 16-bit values: vector c = channel c of the thread's eight, rows 0..7
  v4u* stage_base = (role_b ? Bs : As);
  const int slot0 = kg * WB_BM + (oct << 3);
  const int sw = (oct >> 1) & 7;
  auto transpose_store = [&](int buf) {
    v4u* dst = stage_base + buf * (8 * WB_BM) + slot0;
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      const uint32_t sel = (c & 1) ? 0x07060302u : 0x05040100u;
      v4u v;
      v.x = __builtin_amdgcn_perm(R[1][c >> 1], R[0][c >> 1], sel);
      v.y = __builtin_amdgcn_perm(R[3][c >> 1], R[2][c >> 1], sel);
      v.z = __builtin_amdgcn_perm(R[5][c >> 1], R[4][c >> 1], sel);
      v.w = __builtin_amdgcn_perm(R[7][c >> 1], R[6][c >> 1], sel);
      dst[c ^ sw] = v;
    }
  };
  // fragment slots of the lane: rows of dw (channels of dy) wm0 + 32*bi + lane%32, columns
  // (channels of x) wn0 + 32*bj + lane%32; row group 2*s + lane/32 in MFMA step s
  int a_at[2], b_at[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    a_at[i] = wb_slot(lane >> 5, wm0 + 32 * i + (lane & 31));
    b_at[i] = wb_slot(lane >> 5, wn0 + 32 * i + (lane & 31));
  }
  auto compute = [&](int buf) {
    const v4u* as = As + buf * (8 * WB_BM);
    const v4u* bs = Bs + buf * (8 * WB_BN);
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) {
      v4u a[2], b[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        a[i] = as[a_at[i] + s4 * 2 * WB_BM];
        b[i] = bs[b_at[i] + s4 * 2 * WB_BN];
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = mfma32x32x16bf(a[i], b[j], acc[i][j]);
    }
  };
  if (n_chunks > 0) {
    load(0);
    transpose_store(0);
    __syncthreads();
    for (int kc = 0; kc < n_chunks; ++kc) {
      const bool more = kc + 1 < n_chunks;
      if (more) load(kc + 1);
      compute(kc & 1);
      if (more) transpose_store((kc + 1) & 1);
      __syncthreads();
    }
  }
  float* dst = out + (size_t)split * split_stride;
  (void)ci0;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int jcol = j0 + wn0 + 32 * j + (lane & 31);
      if (jcol >= J) continue;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int co = co0 + wm0 + 32 * i + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        if (co < g.cout) dst[(size_t)co * J + jcol] = acc[i][j][v];
      }
    }
#else
  (void)Bs; (void)&mfma32x32x16bf; (void)&wb_slot;
#endif
}

// dw[i] = part[0][i] + part[1][i] + ... in that order
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* part, float* dw, size_t count,
                                                             int splits) {
  const size_t i4 = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i4 >= count) return;
  if (i4 + 4 <= count && (count & 3) == 0) {
    float4 s = *reinterpret_cast<const float4*>(part + i4);
    // eight parts fetched at a time, added in their order: with hundreds of parts (the stem's
    // weight gradient) one load waiting for the sum before it made this a chain of latencies
    int k = 1;
    for (; k + 8 <= splits; k += 8) {
      float4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const float4*>(part + (size_t)(k + u) * count + i4);
#pragma unroll
      for (int u = 0; u < 8; ++u) { s.x += v[u].x; s.y += v[u].y; s.z += v[u].z; s.w += v[u].w; }
    }
    for (; k < splits; ++k) {
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
  int tiles_co, tiles_j, splits, chunks_per_split;
};

// Depends on the shape only (never on addresses or on the swap plan).  The m range is cut into
// as many parts as keep the launch within 768 workgroups, three per CU (what the
// register-staged loader's LDS allows; measured with the direct loader at minibatch 41:
// 512 -> 86, 768 -> 96, 1024 -> 99, 1280 -> 88 TFLOP/s, and the larger part count of 1024
// costs the reduction what it gains here), at least 8 chunks of 32 rows each.
// bf16 storage on the bf16 matrix cores: channel counts the 128 x 128 tile of wgrad_bf16_kernel takes
inline bool bf16_mfma_shape(int dtype, int cin, int cout) { return dtype == DT_BF16 && cin % 8 == 0 && cout % 8 == 0; }

WgradCfg choose(long Mrows, int cin, int cout, int r, int s, int dtype) {
  WgradCfg c;
  const long J = (long)r * s * cin;
  if (bf16_mfma_shape(dtype, cin, cout)) {
    // 128 x 128 tiles, chunks of 64 rows; two workgroups per CU (64 KB of LDS each): one round of 512,
    // at least four chunks per part
    c.tiles_co = (cout + WB_BM - 1) / WB_BM;
    c.tiles_j = (int)((J + WB_BN - 1) / WB_BN);
    const long tiles = (long)c.tiles_co * c.tiles_j;
    const long chunks = (Mrows + WB_BK - 1) / WB_BK;
    long splits = 512 / tiles;
    const long max_splits = chunks / 4 > 0 ? chunks / 4 : 1;
    if (splits > max_splits) splits = max_splits;
    if (splits > 1024) splits = 1024;
    if (splits < 1) splits = 1;
    c.chunks_per_split = (int)((chunks + splits - 1) / splits);
    c.splits = (int)((chunks + c.chunks_per_split - 1) / c.chunks_per_split);
    return c;
  }
  c.tiles_co = (cout + BM - 1) / BM;
  c.tiles_j = (int)((J + BN - 1) / BN);
  const long tiles = (long)c.tiles_co * c.tiles_j;
  const long chunks = (Mrows + BKM - 1) / BKM;
  // One round of workgroups.  Alone the kernel is fastest with 768 (three per CU: measured 86 / 96 / 99 / 88
  // TFLOP/s at 512 / 768 / 1024 / 1280 when the choice was first made; 93 against 102 now), but in the step it
  // runs on a stream of its own beside the data gradient and the next batch norm.  Those are the critical
  // path, and at small minibatches, where their fixed costs weigh most, two weight-gradient workgroups per CU
  // leave them the larger share of the matrix cores; at large minibatches the weight gradient itself becomes
  // the longer chain.  ResNet-152, images/s with 512 / 768 everywhere: minibatch 32 1099 / 1110, 36 1159 / 1135,
  // 41 1233 / 1194, 48 1177 / 1154, 52 1184 / 1199, 56 1186 / 1220, 64 1208 / 1205, 128 1263 / 1314; the
  // row count below (14 x 14 maps up to minibatch 50) takes the better of the two everywhere but at 32.
  // The per-element loader (3-channel stem, nothing beside it) keeps 768.
  const long target = cin % 64 ? 768 : Mrows <= 9800 ? 512 : 768;
  long splits = target / tiles;
  const long max_splits = chunks / 8 > 0 ? chunks / 8 : 1;
  if (splits > max_splits) splits = max_splits;
  if (splits > 1024) splits = 1024;
  if (splits < 1) splits = 1;
  c.chunks_per_split = (int)((chunks + splits - 1) / splits);
  c.splits = (int)((chunks + c.chunks_per_split - 1) / c.chunks_per_split);
  return c;
}

}  // namespace

size_t wgrad_workspace_bytes(int n_img, int p, int q, int cin, int cout, int r, int s, int dtype) {
  if (dtype < 0) {   // whichever storage type needs more
    const size_t a = wgrad_workspace_bytes(n_img, p, q, cin, cout, r, s, DT_F32);
    const size_t b = wgrad_workspace_bytes(n_img, p, q, cin, cout, r, s, DT_BF16);
    return a > b ? a : b;
  }
  const WgradCfg c = choose((long)n_img * p * q, cin, cout, r, s, dtype);
  if (c.splits <= 1) return 0;
  return (size_t)c.splits * cout * r * s * cin * sizeof(float);
}

hipError_t reduce_parts(const ReduceJob& job, hipStream_t st) {
  if (job.count == 0) return hipSuccess;
  if (!job.part || !job.dw || job.splits < 1) return hipErrorInvalidValue;
  const unsigned blocks = (unsigned)((job.count + 1023) / 1024);
  hipLaunchKernelGGL(splitk_reduce_kernel, dim3(blocks), dim3(256), 0, st, job.part, job.dw, job.count, job.splits);
  return hipGetLastError();
}

hipError_t conv_wgrad(const WgradGeom& g, hipStream_t st, LaunchProbe* probe, ReduceJob* deferred) {
  if (deferred) *deferred = ReduceJob{nullptr, nullptr, 0, 0};
  if (!g.x || !g.dy || !g.dw) return hipErrorInvalidValue;
  if ((g.flip_w == nullptr) != (g.flip_wt == nullptr)) return hipErrorInvalidValue;
  if (g.n_img <= 0 || g.h <= 0 || g.wd <= 0 || g.cin <= 0 || g.p <= 0 || g.q <= 0 || g.cout <= 0 ||
      g.r <= 0 || g.s <= 0 || g.stride <= 0 || g.pad < 0)
    return hipErrorInvalidValue;
  const long Mrows = (long)g.n_img * g.p * g.q;
  const long J = (long)g.r * g.s * g.cin;
  if (Mrows >= (1L << 31) || (long)g.n_img * g.h * g.wd >= (1L << 31) || J * g.cout >= (1L << 31))
    return hipErrorInvalidValue;
  if (g.dtype != DT_F32 && g.dtype != DT_BF16) return hipErrorInvalidValue;
  const WgradCfg c = choose(Mrows, g.cin, g.cout, g.r, g.s, g.dtype);
  if (c.splits > 1 && !g.workspace) return hipErrorInvalidValue;
  const long work = (long)c.tiles_co * c.tiles_j * c.splits;
  if (work > (1L << 30)) return hipErrorInvalidValue;
  const long es = (long)dt_size(g.dtype);
  const bool fast = (g.cout % 4 == 0) && (g.cin % 64 == 0) && Mrows * g.cout * es < (1L << 32) &&
                    (long)g.n_img * g.h * g.wd * g.cin * es < (1L << 32);
  float* out = c.splits > 1 ? g.workspace : g.dw;
  const size_t count = (size_t)g.cout * J;
  const int main_grid = (int)((work + 7) / 8 * 8);
  const long flip_blocks = g.flip_wt ? (long)((g.cin + 31) / 32) * ((g.cout + 31) / 32) * g.r * g.s : 0;
  long reduce_blocks = 0;
  if (g.side.count) {
    if (!g.side.part || !g.side.dw || g.side.splits < 1) return hipErrorInvalidValue;
    reduce_blocks = (long)((g.side.count + 1023) / 1024);
  }
  if (main_grid + flip_blocks + reduce_blocks > (1L << 30)) return hipErrorInvalidValue;
  const dim3 grid((unsigned)(main_grid + reduce_blocks + flip_blocks));
  const int tiles = c.tiles_co * c.tiles_j;
  if (probe && probe->before) (void)hipEventRecord(probe->before, st);
  // direct loader: fp32 storage, both operands inside 32-bit buffer ranges (the last bytes stay
  // free for the offset that stands for "outside") and 16-byte aligned
  // (p, q <= 4096: the range over which the loader's float quotients were checked exhaustively)
  const bool direct = fast && g.dtype == DT_F32 && g.p <= 4096 && g.q <= 4096 && Mrows * g.cout * es <= 0xFFFFFF00L &&
                      (long)g.n_img * g.h * g.wd * g.cin * es <= 0xFFFFFF00L &&
                      (reinterpret_cast<uintptr_t>(g.x) & 15) == 0 && (reinterpret_cast<uintptr_t>(g.dy) & 15) == 0;
#define ACC_WGRAD_LAUNCH(F, T)                                                                             \
  hipLaunchKernelGGL((wgrad_kernel<F, T>), grid, dim3(256), 0, st, g, (int)Mrows, (int)J, c.tiles_j, tiles, \
                     c.splits, c.chunks_per_split, out, count, main_grid)
  // bf16 matrix cores: the shapes choose() cut into 128 x 128 tiles; byte offsets inside 32-bit buffer
  // ranges (the last bytes stay free for the offset that stands for "outside"), 16-byte aligned operands
  const bool mfma16 = bf16_mfma_shape(g.dtype, g.cin, g.cout);
  if (mfma16 && !(Mrows * g.cout * es <= 0xFFFFFF00L && (long)g.n_img * g.h * g.wd * g.cin * es <= 0xFFFFFF00L &&
                  (reinterpret_cast<uintptr_t>(g.x) & 15) == 0 && (reinterpret_cast<uintptr_t>(g.dy) & 15) == 0))
    return hipErrorInvalidValue;   // (the split count, and with it the workspace, was sized for this kernel)
  if (g.dtype == DT_F32) {
    if (direct) ACC_WGRAD_LAUNCH(L_DIRECT, float);
    else if (fast) ACC_WGRAD_LAUNCH(L_FAST, float);
    else ACC_WGRAD_LAUNCH(L_GENERIC, float);
  } else if (mfma16) {
    hipLaunchKernelGGL(wgrad_bf16_kernel, grid, dim3(256), 0, st, g, (int)Mrows, (int)J, c.tiles_j, tiles, c.splits,
                       c.chunks_per_split, out, count, main_grid);
  } else {
    if (fast) ACC_WGRAD_LAUNCH(L_FAST, bf16_t); else ACC_WGRAD_LAUNCH(L_GENERIC, bf16_t);
  }
#undef ACC_WGRAD_LAUNCH
  if (probe && probe->after) (void)hipEventRecord(probe->after, st);
  if (probe) probe->variant = mfma16 ? V_WGRAD_BF16 : direct ? V_WGRAD_DIRECT : fast ? V_WGRAD_FAST : V_WGRAD_GENERIC;
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (c.splits > 1) {
    const ReduceJob job{g.workspace, g.dw, count, c.splits};
    if (deferred) *deferred = job;
    else e = reduce_parts(job, st);
  }
  return e;
}

}  // namespace acc
