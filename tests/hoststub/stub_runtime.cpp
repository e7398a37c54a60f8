// Host-only stand-ins for the HIP runtime calls and for the kernel launchers that the executor
// (engine.hip) uses.  They do no arithmetic and move no data: they check what a missing wait,
// a stale event or a wrong offset would break.
//   * every event must be alive when used (AddressSanitizer catches the rest), and a wait on
//     an event (hipStreamWaitEvent, hipEventSynchronize, hipEventElapsedTime) must find it
//     recorded in the current iteration ("epoch"): a wait on last iteration's record would
//     order nothing;
//   * hipEventElapsedTime needs two events created with timing;
//   * the device side of every copy and every tensor pointer handed to a kernel launcher must
//     lie inside the device pool, the host side of a swap copy inside the pinned arena.
// TEST INFRASTRUCTURE (see hip/hip_runtime.h beside this file).
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <map>
#include <set>
#include <string>

#include "../../paper_1901_06773_amd/csrc/dtype.h"
#include "../../paper_1901_06773_amd/csrc/kernels.h"
#include "stub_runtime.h"

struct stub_stream { int id; long ops; };
struct stub_event { unsigned flags; int epoch; long records; stub_stream* on; };

namespace {
StubCounters g;
std::set<stub_event*> g_events;
char* g_pool = nullptr; size_t g_pool_bytes = 0;
char* g_arena = nullptr; size_t g_arena_bytes = 0;
int g_epoch = 1;
bool g_capture = false;

bool in_pool(const void* p, size_t bytes) {
  const char* q = static_cast<const char*>(p);
  return q >= g_pool && q + bytes <= g_pool + g_pool_bytes;
}
bool touches_pool(const void* p) {
  const char* q = static_cast<const char*>(p);
  return q >= g_pool && q < g_pool + g_pool_bytes;
}
bool touches_arena(const void* p) {
  const char* q = static_cast<const char*>(p);
  return q >= g_arena && q < g_arena + g_arena_bytes;
}
void complain(const char* what) {
  if (g.first_complaint[0] == 0) snprintf(g.first_complaint, sizeof g.first_complaint, "%s", what);
}
bool alive(hipEvent_t e, const char* where) {
  if (!e || !g_events.count(e)) { ++g.dead_event_uses; complain(where); return false; }
  return true;
}
void need_fresh(hipEvent_t e, const char* where) {
  if (!alive(e, where)) return;
  if (e->records == 0) { ++g.waits_on_unrecorded; complain(where); }
  else if (e->epoch != g_epoch) { ++g.waits_on_stale; complain(where); }
}
void dev(const void* p, const char* where) {
  if (p && !touches_pool(p)) { ++g.pointers_outside_pool; complain(where); }
}
}  // namespace

StubCounters& stub_counters() { return g; }
void stub_set_regions(void* pool, size_t pool_bytes, void* arena, size_t arena_bytes) {
  g_pool = static_cast<char*>(pool); g_pool_bytes = pool_bytes;
  g_arena = static_cast<char*>(arena); g_arena_bytes = arena_bytes;
}
void stub_new_epoch() { ++g_epoch; }
hipStream_t stub_make_stream(int id) { return new stub_stream{id, 0}; }
void stub_free_stream(hipStream_t s) { delete s; }
long stub_live_events() { return (long)g_events.size(); }

hipError_t hipEventCreateWithFlags(hipEvent_t* e, unsigned flags) {
  *e = new stub_event{flags, 0, 0, nullptr};
  g_events.insert(*e);
  ++g.events_created;
  if ((long)g_events.size() > g.max_live_events) g.max_live_events = (long)g_events.size();
  return hipSuccess;
}
hipError_t hipEventCreate(hipEvent_t* e) { return hipEventCreateWithFlags(e, hipEventDefault); }
hipError_t hipEventDestroy(hipEvent_t e) {
  if (!alive(e, "hipEventDestroy of a dead event")) return hipErrorInvalidValue;
  g_events.erase(e);
  delete e;
  ++g.events_destroyed;
  return hipSuccess;
}
hipError_t hipEventRecord(hipEvent_t e, hipStream_t s) {
  if (!alive(e, "hipEventRecord on a dead event")) return hipErrorInvalidValue;
  if (!s) { ++g.null_streams; complain("hipEventRecord on the null stream"); }
  e->epoch = g_epoch; e->records++; e->on = s;
  if (s) s->ops++;
  ++g.records;
  return hipSuccess;
}
hipError_t hipEventSynchronize(hipEvent_t e) {
  need_fresh(e, "hipEventSynchronize");
  if (g_capture) { ++g.sync_in_capture; complain("hipEventSynchronize while a stream is capturing"); }
  ++g.host_waits;
  return hipSuccess;
}
hipError_t hipEventElapsedTime(float* ms, hipEvent_t a, hipEvent_t b) {
  need_fresh(a, "hipEventElapsedTime (first event)");
  need_fresh(b, "hipEventElapsedTime (second event)");
  if (a && b && g_events.count(a) && g_events.count(b) && ((a->flags | b->flags) & hipEventDisableTiming)) {
    ++g.elapsed_on_untimed; complain("hipEventElapsedTime on an event created without timing");
  }
  *ms = 0.01f;
  ++g.elapsed_reads;
  return hipSuccess;
}
hipError_t hipStreamWaitEvent(hipStream_t s, hipEvent_t e, unsigned) {
  need_fresh(e, "hipStreamWaitEvent");
  if (!s) { ++g.null_streams; complain("hipStreamWaitEvent on the null stream"); }
  else {
    if (e && g_events.count(e) && e->on == s) ++g.waits_on_own_stream;   // harmless, but says the plan is confused
    s->ops++;
  }
  ++g.stream_waits;
  return hipSuccess;
}
hipError_t hipStreamSynchronize(hipStream_t s) {
  if (!s) ++g.null_streams;
  if (g_capture) { ++g.sync_in_capture; complain("hipStreamSynchronize while a stream is capturing"); }
  return hipSuccess;
}
hipError_t hipMemcpyAsync(void* dst, const void* src, size_t bytes, hipMemcpyKind kind, hipStream_t s) {
  if (!s) { ++g.null_streams; complain("hipMemcpyAsync on the null stream"); }
  else s->ops++;
  ++g.copies;
  g.copy_bytes += bytes;
  const bool dst_dev = kind == hipMemcpyHostToDevice || kind == hipMemcpyDeviceToDevice;
  const bool src_dev = kind == hipMemcpyDeviceToHost || kind == hipMemcpyDeviceToDevice;
  if (dst_dev && !in_pool(dst, bytes)) { ++g.copies_out_of_range; complain("copy: device destination outside the pool"); }
  if (src_dev && !in_pool(src, bytes) && kind != hipMemcpyDeviceToDevice) { ++g.copies_out_of_range; complain("copy: device source outside the pool"); }
  if (!dst_dev) {
    if (touches_pool(dst)) { ++g.copies_out_of_range; complain("copy: host destination inside the pool"); }
    if (touches_arena(dst) && !(static_cast<char*>(dst) + bytes <= g_arena + g_arena_bytes)) { ++g.copies_out_of_range; complain("copy: runs past the pinned arena"); }
  }
  if (!src_dev && touches_arena(src) && !(static_cast<const char*>(src) + bytes <= g_arena + g_arena_bytes)) {
    ++g.copies_out_of_range; complain("copy: reads past the pinned arena");
  }
  return hipSuccess;
}
struct stub_graph { int nodes; };
hipError_t hipStreamBeginCapture(hipStream_t s, hipStreamCaptureMode) {
  if (!s || g_capture) { ++g.null_streams; complain("hipStreamBeginCapture: null stream or nested capture"); return hipErrorInvalidValue; }
  g_capture = true;
  return hipSuccess;
}
hipError_t hipStreamEndCapture(hipStream_t, hipGraph_t* graph) {
  if (!g_capture) return hipErrorInvalidValue;
  g_capture = false;
  *graph = new stub_graph{0};
  return hipSuccess;
}
hipError_t hipGraphInstantiate(hipGraphExec_t* exec, hipGraph_t graph, hipGraphNode_t*, char*, size_t) {
  if (!graph) return hipErrorInvalidValue;
  *exec = new stub_graph{graph->nodes};
  return hipSuccess;
}
hipError_t hipGraphLaunch(hipGraphExec_t exec, hipStream_t s) {
  if (!exec || !s) { ++g.null_streams; complain("hipGraphLaunch: null graph or stream"); return hipErrorInvalidValue; }
  ++g.graph_launches;
  return hipSuccess;
}
hipError_t hipGraphExecDestroy(hipGraphExec_t exec) { delete exec; return hipSuccess; }
hipError_t hipGraphDestroy(hipGraph_t graph) { delete graph; return hipSuccess; }
hipError_t hipHostMalloc(void** p, size_t bytes, unsigned) { *p = calloc(1, bytes); return *p ? hipSuccess : hipErrorOutOfMemory; }
hipError_t hipHostFree(void* p) { free(p); return hipSuccess; }
hipError_t hipGetLastError() { return hipSuccess; }
const char* hipGetErrorString(hipError_t e) { return e == hipSuccess ? "no error" : "stub error"; }
void stub_count_launch(const char*, hipStream_t s) {
  ++g.launches;
  if (!s) { ++g.null_streams; complain("kernel launch on the null stream"); } else s->ops++;
}

// ---------------------------------------------------------------- kernel launchers (kernels.h)
namespace acc {

static void probe_events(LaunchProbe* probe, hipStream_t st, int variant) {
  if (!probe) return;
  probe->variant = variant;
  if (probe->before) (void)hipEventRecord(probe->before, st);
  if (probe->after) (void)hipEventRecord(probe->after, st);
}

bool conv_igemm_bf16_takes(const ConvGeom&, long, long) { return false; }
hipError_t conv_igemm_bf16(const ConvGeom&, int, int, hipStream_t, const LaunchProbe*) { return hipErrorInvalidValue; }
const char* conv_variant_name(int v) { return v == V_WGRAD_DIRECT ? "wgrad_kernel<stub>" : "igemm_kernel<stub>"; }

hipError_t conv_igemm(const ConvGeom& g_, hipStream_t st, LaunchProbe* probe) {
  dev(g_.in, "conv_igemm: input"); dev(g_.w, "conv_igemm: filter"); dev(g_.out, "conv_igemm: output");
  dev(g_.side.part, "conv_igemm: reduce parts"); dev(g_.side.dw, "conv_igemm: reduce target");
  dev(g_.flip.w, "conv_igemm: flip source"); dev(g_.flip.wt, "conv_igemm: flip target");
  dev(g_.stats, "conv_igemm: stats"); dev(g_.bnb.sums, "conv_igemm: bn backward sums");
  dev(g_.bnb.x, "conv_igemm: bn x"); dev(g_.bnb.y, "conv_igemm: bn y");
  const size_t es = dt_size(g_.dtype);
  if (!in_pool(g_.in, (size_t)g_.n_img * g_.h * g_.wd * g_.c * es)) { ++g.pointers_outside_pool; complain("conv_igemm: input runs past the pool"); }
  if (!in_pool(g_.out, (size_t)g_.n_img * g_.out_h * g_.out_w * g_.n_out * es)) { ++g.pointers_outside_pool; complain("conv_igemm: output runs past the pool"); }
  probe_events(probe, st, V_IGEMM_DIRECT);
  stub_count_launch("conv_igemm", st);
  return hipSuccess;
}
size_t wgrad_workspace_bytes(int n_img, int p, int q, int cin, int cout, int r, int s, int) {
  const long rows = (long)n_img * p * q;
  const long splits = rows >= 2048 ? 8 : rows >= 256 ? 2 : 1;     // any step function of the minibatch will do here
  return splits > 1 ? (size_t)splits * cout * r * s * cin * sizeof(float) : 0;
}
hipError_t conv_wgrad(const WgradGeom& g_, hipStream_t st, LaunchProbe* probe, ReduceJob* deferred) {
  dev(g_.x, "conv_wgrad: x"); dev(g_.dy, "conv_wgrad: dy"); dev(g_.dw, "conv_wgrad: dw"); dev(g_.workspace, "conv_wgrad: workspace");
  dev(g_.flip_w, "conv_wgrad: flip source"); dev(g_.flip_wt, "conv_wgrad: flip target");
  dev(g_.side.part, "conv_wgrad: reduce parts"); dev(g_.side.dw, "conv_wgrad: reduce target");
  const size_t need = wgrad_workspace_bytes(g_.n_img, g_.p, g_.q, g_.cin, g_.cout, g_.r, g_.s, g_.dtype);
  if (need && (!g_.workspace || !in_pool(g_.workspace, need))) { ++g.pointers_outside_pool; complain("conv_wgrad: workspace runs past the pool"); }
  if (deferred) *deferred = ReduceJob{nullptr, nullptr, 0, 0};
  if (need) {
    const ReduceJob job{g_.workspace, g_.dw, (size_t)g_.cout * g_.r * g_.s * g_.cin, (int)(need / ((size_t)g_.cout * g_.r * g_.s * g_.cin * 4))};
    if (deferred) *deferred = job; else stub_count_launch("reduce", st);
  }
  probe_events(probe, st, V_WGRAD_DIRECT);
  stub_count_launch("conv_wgrad", st);
  return hipSuccess;
}
hipError_t reduce_parts(const ReduceJob& job, hipStream_t st) {
  dev(job.part, "reduce_parts: parts"); dev(job.dw, "reduce_parts: target");
  stub_count_launch("reduce_parts", st);
  return hipSuccess;
}
hipError_t filter_flip_transpose(const void* w, void* wt, int, int, int, int, int, hipStream_t st) {
  dev(w, "flip: source"); dev(wt, "flip: target"); stub_count_launch("flip", st); return hipSuccess;
}
hipError_t filter_gather_transpose(const void* w, void* wt, int, int, int, int, int, const DgradPart&, int, hipStream_t st) {
  dev(w, "gather: source"); dev(wt, "gather: target"); stub_count_launch("gather", st); return hipSuccess;
}
size_t bn_workspace_bytes(int c) { return (size_t)2 * kBnMaxSlabs * c * sizeof(double) + (size_t)4 * c * sizeof(float); }
hipError_t bn_forward(const void* x, const float* gamma, const float* beta, const void* res, void* y, float* mean, float* istd,
                      long rows, int c, int, float, void* workspace, int dtype, hipStream_t st, const BnSums* ready) {
  dev(x, "bn_forward: x"); dev(gamma, "bn_forward: gamma"); dev(beta, "bn_forward: beta"); dev(res, "bn_forward: res");
  dev(y, "bn_forward: y"); dev(mean, "bn_forward: mean"); dev(istd, "bn_forward: istd"); dev(workspace, "bn_forward: workspace");
  if (ready) dev(ready->part, "bn_forward: ready sums");
  if (!in_pool(y, (size_t)rows * c * dt_size(dtype))) { ++g.pointers_outside_pool; complain("bn_forward: y runs past the pool"); }
  if (!in_pool(workspace, bn_workspace_bytes(c))) { ++g.pointers_outside_pool; complain("bn_forward: workspace runs past the pool"); }
  stub_count_launch("bn_forward", st);
  return hipSuccess;
}
hipError_t bn_backward(const void* x, const void* dy, const void* y, const float* gamma, const float* mean, const float* istd,
                       void* dx, float* dgamma, float* dbeta, void* g_out, long rows, int c, void* workspace, int dtype,
                       hipStream_t st, const BnSums* ready) {
  dev(x, "bn_backward: x"); dev(dy, "bn_backward: dy"); dev(y, "bn_backward: y"); dev(gamma, "bn_backward: gamma");
  dev(mean, "bn_backward: mean"); dev(istd, "bn_backward: istd"); dev(dx, "bn_backward: dx"); dev(dgamma, "bn_backward: dgamma");
  dev(dbeta, "bn_backward: dbeta"); dev(g_out, "bn_backward: g_out"); dev(workspace, "bn_backward: workspace");
  if (ready) dev(ready->part, "bn_backward: ready sums");
  if (!in_pool(dx, (size_t)rows * c * dt_size(dtype))) { ++g.pointers_outside_pool; complain("bn_backward: dx runs past the pool"); }
  stub_count_launch("bn_backward", st);
  return hipSuccess;
}
hipError_t maxpool_forward(const void* x, void* y, int, int, int, int, int, int, int, int, int, hipStream_t st) {
  dev(x, "maxpool_forward: x"); dev(y, "maxpool_forward: y"); stub_count_launch("maxpool_forward", st); return hipSuccess;
}
hipError_t maxpool_backward(const void* x, const void* dy, void* dx, int, int, int, int, int, int, int, int, int, int, hipStream_t st) {
  dev(x, "maxpool_backward: x"); dev(dy, "maxpool_backward: dy"); dev(dx, "maxpool_backward: dx");
  stub_count_launch("maxpool_backward", st); return hipSuccess;
}
hipError_t gap_forward(const void* x, void* y, int, int, int, int, hipStream_t st) {
  dev(x, "gap_forward: x"); dev(y, "gap_forward: y"); stub_count_launch("gap_forward", st); return hipSuccess;
}
hipError_t gap_backward(const void* dy, void* dx, int, int, int, int, int, hipStream_t st) {
  dev(dy, "gap_backward: dy"); dev(dx, "gap_backward: dx"); stub_count_launch("gap_backward", st); return hipSuccess;
}
hipError_t bias_add(void* y, const float* b, long, int, int, hipStream_t st, int) {
  dev(y, "bias_add: y"); dev(b, "bias_add: b"); stub_count_launch("bias_add", st); return hipSuccess;
}
size_t relu_bias_workspace_bytes(int c) { return (size_t)kBnMaxSlabs * c * sizeof(double); }
hipError_t relu_mask(void* dy, const void* y, size_t, int, hipStream_t st) {
  dev(dy, "relu_mask: dy"); dev(y, "relu_mask: y"); stub_count_launch("relu_mask", st); return hipSuccess;
}
hipError_t relu_bias_backward(void* dy, const void* y, float* db, long, int, void* workspace, int, hipStream_t st) {
  dev(dy, "relu_bias_backward: dy"); dev(y, "relu_bias_backward: y"); dev(db, "relu_bias_backward: db");
  dev(workspace, "relu_bias_backward: workspace"); stub_count_launch("relu_bias_backward", st); return hipSuccess;
}
hipError_t column_sum(const void* dy, float* db, long, int, int, hipStream_t st) {
  dev(dy, "column_sum: dy"); dev(db, "column_sum: db"); stub_count_launch("column_sum", st); return hipSuccess;
}
hipError_t softmax_ce_forward(const void* z, const int32_t* labels, float* rows, float* loss, int, int, int, hipStream_t st) {
  dev(z, "softmax_ce_forward: z"); dev(labels, "softmax_ce_forward: labels"); dev(rows, "softmax_ce_forward: rows");
  dev(loss, "softmax_ce_forward: loss"); stub_count_launch("softmax_ce_forward", st); return hipSuccess;
}
hipError_t softmax_ce_backward(const void* z, const int32_t* labels, void* dz, int, int, int, hipStream_t st) {
  dev(z, "softmax_ce_backward: z"); dev(labels, "softmax_ce_backward: labels"); dev(dz, "softmax_ce_backward: dz");
  stub_count_launch("softmax_ce_backward", st); return hipSuccess;
}
hipError_t sgd_update(float* w, const float* gr, float, size_t, void* w16, hipStream_t st) {
  dev(w, "sgd_update: w"); dev(gr, "sgd_update: g"); dev(w16, "sgd_update: w16"); stub_count_launch("sgd_update", st); return hipSuccess;
}
hipError_t fill_zero(float* p, size_t count, hipStream_t st) {
  dev(p, "fill_zero: p");
  if (!in_pool(p, count * 4)) { ++g.pointers_outside_pool; complain("fill_zero: runs past the pool"); }
  stub_count_launch("fill_zero", st);
  return hipSuccess;
}
hipError_t nchw_to_nhwc(const float* x, void* y, int, int, int, int, hipStream_t st) {
  dev(x, "nchw_to_nhwc: x"); dev(y, "nchw_to_nhwc: y"); stub_count_launch("nchw_to_nhwc", st); return hipSuccess;
}

}  // namespace acc
