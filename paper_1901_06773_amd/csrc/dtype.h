// Storage types of activations and activation gradients: fp32, or bf16 with fp32
// arithmetic (bf16 = the upper 16 bits of an fp32, rounded to nearest even).  Weights keep an
// fp32 master copy; batch-norm statistics, weight gradients and the loss stay fp32.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

namespace acc {

enum { DT_F32 = 0, DT_BF16 = 1 };   // same values as ACC_F32 / ACC_BF16 of the C ABI
inline size_t dt_size(int dt) { return dt == DT_BF16 ? 2 : 4; }

typedef uint16_t bf16_t;

__host__ __device__ inline float bf16_to_float(bf16_t h) {
  union { uint32_t u; float f; } c;
  c.u = (uint32_t)h << 16;
  return c.f;
}

__host__ __device__ inline bf16_t float_to_bf16(float f) {
  union { uint32_t u; float f; } c;
  c.f = f;
  if ((c.u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)0x7fc0;   // NaN stays NaN
  c.u += 0x7fffu + ((c.u >> 16) & 1u);                            // round to nearest even
  return (bf16_t)(c.u >> 16);
}

// One element / four consecutive elements as floats.
template <class T> struct Elem;
template <> struct Elem<float> {
  static __device__ __forceinline__ float load(const float* p) { return *p; }
  static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
  static __device__ __forceinline__ void load4(const float* p, float (&v)[4]) {
    const float4 q = *reinterpret_cast<const float4*>(p);
    v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
  }
  static __device__ __forceinline__ void store4(float* p, const float (&v)[4]) {
    *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  }
};
template <> struct Elem<bf16_t> {
  static __device__ __forceinline__ float load(const bf16_t* p) { return bf16_to_float(*p); }
  static __device__ __forceinline__ void store(bf16_t* p, float v) { *p = float_to_bf16(v); }
  static __device__ __forceinline__ void load4(const bf16_t* p, float (&v)[4]) {
    const uint2 q = *reinterpret_cast<const uint2*>(p);
    v[0] = __uint_as_float(q.x << 16); v[1] = __uint_as_float(q.x & 0xffff0000u);
    v[2] = __uint_as_float(q.y << 16); v[3] = __uint_as_float(q.y & 0xffff0000u);
  }
  static __device__ __forceinline__ void store4(bf16_t* p, const float (&v)[4]) {
    uint2 q;
    q.x = (uint32_t)float_to_bf16(v[0]) | ((uint32_t)float_to_bf16(v[1]) << 16);
    q.y = (uint32_t)float_to_bf16(v[2]) | ((uint32_t)float_to_bf16(v[3]) << 16);
    *reinterpret_cast<uint2*>(p) = q;
  }
};

}  // namespace acc
