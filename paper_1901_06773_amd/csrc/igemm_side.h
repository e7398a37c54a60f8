// Side jobs of an implicit-GEMM launch: workgroups appended behind the tiles that do small,
// independent work which would otherwise cost a launch of its own.
#pragma once
#include <hip/hip_runtime.h>

#include "kernels.h"

namespace acc {

// id: index of the workgroup among the side-job workgroups.  First the blocks that add up 1024
// elements each of a weight gradient's parts, in their fixed order; then the blocks that write
// one 32 x 32 (co, ci) block each of one tap of a flipped, transposed filter.
// scratch: at least 32 x 33 elements of T in LDS.
template <class T>
__device__ __forceinline__ void igemm_side_jobs(const ConvGeom& g, int id, void* scratch) {
  const ReduceJob& j = g.side;
  const int reduce_blocks = (int)((j.count + 1023) / 1024);
  if (id >= reduce_blocks) {
    const FlipJob& f = g.flip;
    id -= reduce_blocks;
    const int bx = (f.cin + 31) / 32, by = (f.cout + 31) / 32;
    const int tap = id / (bx * by), rem = id - tap * (bx * by);
    if (tap >= f.r * f.s) return;
    const int co0f = (rem / bx) * 32, ci0f = (rem - (rem / bx) * bx) * 32;
    const int kr = f.r - 1 - tap / f.s, kt = f.s - 1 - tap % f.s;
    const int src_tap = kr * f.s + kt;
    T (*tile)[33] = reinterpret_cast<T (*)[33]>(scratch);
    const T* fw = static_cast<const T*>(f.w);
    T* fwt = static_cast<T*>(f.wt);
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    for (int i = ty; i < 32; i += 8) {
      const int co = co0f + i, ci = ci0f + tx;
      tile[i][tx] = (co < f.cout && ci < f.cin) ? fw[((size_t)co * f.r * f.s + src_tap) * f.cin + ci] : T(0);
    }
    __syncthreads();
    for (int i = ty; i < 32; i += 8) {
      const int ci = ci0f + i, co = co0f + tx;
      if (ci < f.cin && co < f.cout) fwt[((size_t)ci * f.r * f.s + tap) * f.cout + co] = tile[tx][i];
    }
    return;
  }
  const size_t i4 = ((size_t)id * 256 + threadIdx.x) * 4;
  if (i4 >= j.count) return;
  if (i4 + 4 <= j.count && (j.count & 3) == 0) {
    float4 sum = *reinterpret_cast<const float4*>(j.part + i4);
    // eight parts fetched at a time, added in their order: with hundreds of parts (few tiles, many
    // cuts of the minibatch range) one load waiting for the sum before it is a chain of latencies
    int k = 1;
    for (; k + 8 <= j.splits; k += 8) {
      float4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const float4*>(j.part + (size_t)(k + u) * j.count + i4);
#pragma unroll
      for (int u = 0; u < 8; ++u) { sum.x += v[u].x; sum.y += v[u].y; sum.z += v[u].z; sum.w += v[u].w; }
    }
    for (; k < j.splits; ++k) {
      const float4 v = *reinterpret_cast<const float4*>(j.part + (size_t)k * j.count + i4);
      sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
    }
    *reinterpret_cast<float4*>(j.dw + i4) = sum;
  } else {
    for (size_t i = i4; i < j.count && i < i4 + 4; ++i) {
      float sum = j.part[i];
      for (int k = 1; k < j.splits; ++k) sum += j.part[(size_t)k * j.count + i];
      j.dw[i] = sum;
    }
  }
}

}  // namespace acc
