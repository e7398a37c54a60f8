// Stand-in for the HIP runtime header, for a HOST-ONLY build of the planner and the executor
// (graph.cpp, plan.cpp, engine.hip compiled as plain C++ with g++ under AddressSanitizer /
// UBSan).  No GPU is involved: streams and events are bookkeeping objects on the heap, copies
// only check their address ranges, kernel launches are counted.  TEST INFRASTRUCTURE: nothing
// in the product builds against this file.
#pragma once
#include <cstddef>
#include <cstdint>
#include <cstring>

#define __global__
#define __device__
#define __host__
#define __forceinline__ inline
#define __launch_bounds__(...)
#define __restrict__

typedef enum {
  hipSuccess = 0,
  hipErrorInvalidValue = 1,
  hipErrorOutOfMemory = 2,
  hipErrorInvalidDevice = 101,
  hipErrorInvalidSymbol = 13,
  hipErrorNotReady = 600,
  hipErrorUnknown = 999
} hipError_t;

typedef enum {
  hipMemcpyHostToHost = 0,
  hipMemcpyHostToDevice = 1,
  hipMemcpyDeviceToHost = 2,
  hipMemcpyDeviceToDevice = 3
} hipMemcpyKind;

struct stub_stream;
struct stub_event;
typedef stub_stream* hipStream_t;
typedef stub_event* hipEvent_t;

enum { hipEventDefault = 0, hipEventDisableTiming = 2, hipHostMallocDefault = 0 };

struct dim3 {
  unsigned x, y, z;
  dim3(unsigned a = 1, unsigned b = 1, unsigned c = 1) : x(a), y(b), z(c) {}
};
struct float4 { float x, y, z, w; };
struct uint2 { unsigned x, y; };
inline float4 make_float4(float a, float b, float c, float d) { return float4{a, b, c, d}; }
inline float __uint_as_float(unsigned u) { float f; std::memcpy(&f, &u, 4); return f; }
static const dim3 blockIdx, threadIdx, blockDim, gridDim;
template <class T> inline T __shfl_xor(T v, int) { return v; }
template <class T> inline T atomicMax(T* p, T v) { T o = *p; if (v > o) *p = v; return o; }
template <class T> inline T atomicAdd(T* p, T v) { T o = *p; *p = o + v; return o; }

hipError_t hipEventCreate(hipEvent_t* e);
hipError_t hipEventCreateWithFlags(hipEvent_t* e, unsigned flags);
hipError_t hipEventDestroy(hipEvent_t e);
hipError_t hipEventRecord(hipEvent_t e, hipStream_t s);
hipError_t hipEventSynchronize(hipEvent_t e);
hipError_t hipEventElapsedTime(float* ms, hipEvent_t a, hipEvent_t b);
hipError_t hipStreamWaitEvent(hipStream_t s, hipEvent_t e, unsigned flags);
hipError_t hipStreamSynchronize(hipStream_t s);
hipError_t hipMemcpyAsync(void* dst, const void* src, size_t bytes, hipMemcpyKind kind, hipStream_t s);
hipError_t hipHostMalloc(void** p, size_t bytes, unsigned flags);
hipError_t hipHostFree(void* p);
hipError_t hipGetLastError();
const char* hipGetErrorString(hipError_t e);

struct stub_graph;
typedef stub_graph* hipGraph_t;
typedef stub_graph* hipGraphExec_t;
typedef struct hipGraphNode_st* hipGraphNode_t;
enum hipStreamCaptureMode { hipStreamCaptureModeGlobal = 0, hipStreamCaptureModeThreadLocal = 1, hipStreamCaptureModeRelaxed = 2 };
hipError_t hipStreamBeginCapture(hipStream_t s, hipStreamCaptureMode mode);
hipError_t hipStreamEndCapture(hipStream_t s, hipGraph_t* graph);
hipError_t hipGraphInstantiate(hipGraphExec_t* exec, hipGraph_t graph, hipGraphNode_t* error_node, char* log, size_t log_bytes);
hipError_t hipGraphLaunch(hipGraphExec_t exec, hipStream_t s);
hipError_t hipGraphExecDestroy(hipGraphExec_t exec);
hipError_t hipGraphDestroy(hipGraph_t graph);

void stub_count_launch(const char* kernel, hipStream_t s);
#define hipLaunchKernelGGL(kernel, grid, block, shmem, stream, ...) stub_count_launch(#kernel, (stream))
