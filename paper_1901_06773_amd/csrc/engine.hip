// Context, runtime memory manager and executor behind the C ABI (include/accudnn.h).
//
// The runtime of Sec. 5 of the paper: one buffer pool of the size of the budget, pinned
// host backing store, and three streams (compute, swap-out, swap-in).  The four operations
// allocate / release / offload / prefetch are resolved at plan time into pool offsets and
// event waits (plan.h); train_step() only walks the instruction list, so the host never
// blocks inside an iteration and the GPU-side order is the same on every run.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/accudnn.h"
#include "graph.h"
#include "kernels.h"
#include "dtype.h"
#include <cmath>
#include "plan.h"

using namespace acc;

namespace {
thread_local std::string g_create_error;
inline size_t al256(size_t b) { return (b + 255) & ~(size_t)255; }
double now_ms() {
  return std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now().time_since_epoch()).count();
}
}  // namespace

void acc::set_thread_error(const char* text) { g_create_error = text ? text : ""; }

struct acc_ctx {
  Graph g;
  CostModel cm;
  Plan plan;
  bool have_res = false;
  acc_resources res{};
  std::string err;
  hipStream_t s_c = nullptr, s_o = nullptr, s_i = nullptr;
  hipStream_t s_w = nullptr;           // optional: weight gradients run here beside the data gradients
  bool wgrad_overlap = true;           // use s_w when there is one (off: everything on s_c)
  std::vector<hipEvent_t> ev_fork, ev_wdone;   // per conv backward step: its dy is ready / its wgrad is done
  std::vector<char> wgrad_in_flight;   // per step: its wgrad went to s_w in this iteration
  std::vector<int> bn_ready_slabs;     // per step: a BN forward step finds its sums in its workspace (slab count)
  ReduceJob pending_reduce{nullptr, nullptr, 0, 0};   // parts of the last conv weight gradient, not added up yet
  hipStream_t pending_stream = nullptr;               // ... and the stream that gradient ran on
  hipEvent_t ev_flush = nullptr;
  // static part of the pool
  float* d_params = nullptr;
  float* d_grads = nullptr;
  uint16_t* d_params16 = nullptr;      // bf16 mode: the rounded copy of the weights the kernels read
  float* d_stats = nullptr;
  float* d_loss = nullptr;
  char* dyn = nullptr;
  size_t dyn_cap = 0;
  // events of the current plan
  std::vector<hipEvent_t> ev_step, ev_d2h, ev_h2d;
  std::vector<hipEvent_t> ev_window;   // one per kStepWindow compute steps: bounds the host's run-ahead
  std::vector<hipEvent_t> prof_a, prof_b, prof_copy_a, prof_copy_b;
  std::vector<double> obs_start, obs_end;   // per instruction of the plan that ran, seconds
  hipEvent_t ev_begin = nullptr, ev_end = nullptr;
  bool profiling = false;
  bool kernel_profiling = false;
  bool calibrating = false;     // input batch is synthesised on the device
  struct KProbe { int variant; double flops; hipEvent_t a, b; int step, role; double ms; };
  std::vector<KProbe> kprobes;  // one per convolution kernel launch of the last profiled step
  size_t kprobes_used = 0;
  hipEvent_t empty_pair[2 * 9] = {};  // event pairs with nothing between them: what a probe itself costs
  double probe_overhead_ms = 0.0;
  double k_ms[V_COUNT] = {}, k_flops[V_COUNT] = {};
  long k_launches[V_COUNT] = {};
  std::vector<double> step_ms;
  std::vector<size_t> cur_off;  // per tensor, while executing
  acc_stats stats{};
  float* h_loss = nullptr;      // pinned: [0] loss, then (as 64-bit words 1..2) what the poison scan found
  // The compute part of an iteration that swaps nothing, captured once per plan into a HIP graph
  // and replayed (acc_set_graph): everything between the input copies and the update kernel.
  bool use_graph = false;
  bool capturing = false;             // run_step is recording into the graph: the update kernel stays outside
  hipGraph_t graph = nullptr;
  hipGraphExec_t graph_exec = nullptr;
  void drop_graph() {
    if (graph_exec) (void)hipGraphExecDestroy(graph_exec);
    if (graph) (void)hipGraphDestroy(graph);
    graph_exec = nullptr;
    graph = nullptr;
  }
  // verification switches (acc_set_debug) and parity hooks (acc_capture_output)
  int debug_flags = 0;
  struct Capture { int tensor; void* dst; size_t cap; };
  std::vector<std::vector<Capture>> capture_at;   // per forward step: outputs to copy out after it
  std::vector<std::vector<Capture>> inject_at;    // per forward step: outputs to overwrite after it (dst = source)
  struct Block { size_t off, bytes; };
  std::vector<std::vector<Block>> poison_after_step;   // per step: blocks released once it has run
  std::vector<Block> poison_after_d2h;                 // per offload: the block its map leaves behind

  int fail(int code, const std::string& what) { err = what; return code; }
  int hipfail(hipError_t e, const char* what) {
    err = std::string(what) + ": " + hipGetErrorString(e);
    return ACC_EHIP;
  }
  // hands out an event pair for one kernel launch (kernel-level profiling only)
  LaunchProbe* next_probe(LaunchProbe* lp, double flops, int step, int role) {
    if (!kernel_profiling) return nullptr;
    if (kprobes_used == kprobes.size()) {
      KProbe kp{-1, 0.0, nullptr, nullptr, -1, 0, 0.0};
      if (hipEventCreate(&kp.a) != hipSuccess || hipEventCreate(&kp.b) != hipSuccess) return nullptr;
      kprobes.push_back(kp);
    }
    KProbe& kp = kprobes[kprobes_used++];
    kp.flops = flops;
    kp.variant = -1;
    kp.step = step;
    kp.role = role;
    kp.ms = 0.0;
    lp->before = kp.a;
    lp->after = kp.b;
    return lp;
  }
  void drop_events() {
    for (auto* v : {&ev_step, &ev_d2h, &ev_h2d, &ev_window, &prof_a, &prof_b, &prof_copy_a, &prof_copy_b}) {
      for (hipEvent_t e : *v) if (e) (void)hipEventDestroy(e);
      v->clear();
    }
  }
};

// Flow control of the executor.  The host could queue a whole iteration (a few thousand
// kernels, copies, event records and waits) long before the GPU gets to it.  Keeping the
// queues that deep buys nothing, so the host never runs more than kWindows * kStepWindow
// steps ahead of the compute stream, nor more than kCopyWindow copies ahead of either copy
// stream: it waits on an event of older work first.  The windows are far deeper than any
// dependency between the streams (the pool holds a few dozen maps at a time).
constexpr int kStepWindow = 32, kWindows = 3, kCopyWindow = 64;
// Event timing of steps and copies is refused for plans that swap more than this per
// iteration: such runs (ResNet-152, minibatch 224 and 256, all maps swapped, 36-41 GiB each
// way) ended in a crash of the process at its next HIP call, cause unknown; the same
// plans run fine untimed, and timed runs up to 20 GiB of swapped maps are fine.
#ifndef ACC_MAX_TIMED_SWAP_BYTES
#define ACC_MAX_TIMED_SWAP_BYTES ((size_t)24 << 30)   // (a host-only test build lifts it)
#endif
constexpr size_t kMaxTimedSwapBytes = ACC_MAX_TIMED_SWAP_BYTES;

#define HIPCHK(ctx, expr)                                  \
  do {                                                     \
    hipError_t e_ = (expr);                                \
    if (e_ != hipSuccess) return (ctx)->hipfail(e_, #expr); \
  } while (0)

// ------------------------------------------------------------------ weight layout helpers
namespace {

// host OIHW <-> device O-H-W-I
void oihw_to_ohwi(const float* src, float* dst, int o, int i, int r, int s) {
  for (int a = 0; a < o; ++a)
    for (int b = 0; b < i; ++b)
      for (int y = 0; y < r; ++y)
        for (int x = 0; x < s; ++x)
          dst[(((size_t)a * r + y) * s + x) * i + b] = src[(((size_t)a * i + b) * r + y) * s + x];
}
void ohwi_to_oihw(const float* src, float* dst, int o, int i, int r, int s) {
  for (int a = 0; a < o; ++a)
    for (int b = 0; b < i; ++b)
      for (int y = 0; y < r; ++y)
        for (int x = 0; x < s; ++x)
          dst[(((size_t)a * i + b) * r + y) * s + x] = src[(((size_t)a * r + y) * s + x) * i + b];
}

int param_io(acc_ctx* c, int layer, float* host, size_t n, bool to_device, bool grads) {
  if (!c) return ACC_EINVAL;
  if (!c->have_res) return c->fail(ACC_ESTATE, "context has no device resources");
  if (layer < 0 || layer >= (int)c->g.layers.size() || !host) return c->fail(ACC_EINVAL, "bad layer or pointer");
  const ParamSlot& ps = c->g.params[layer];
  if (ps.count == 0 || n != ps.count) return c->fail(ACC_EINVAL, "element count does not match the layer");
  const acc_layer& l = c->g.layers[layer];
  float* dev = (grads ? c->d_grads : c->d_params) + ps.offset;
  std::vector<float> tmp(n);
  // An FC layer over a map with h * w > 1 reads it flattened in the device's h, w, c order: its
  // weight rows are permuted like a filter of that size (the bias behind them stays).
  int fc_c = 0, fc_h = 1, fc_w = 1;
  if (l.kind == ACC_FC) {
    fc_c = l.in0 < 0 ? c->g.in_c : c->g.shape_c[l.in0];
    fc_h = l.in0 < 0 ? c->g.in_h : c->g.shape_h[l.in0];
    fc_w = l.in0 < 0 ? c->g.in_w : c->g.shape_w[l.in0];
  }
  const bool fc_map = l.kind == ACC_FC && fc_h * fc_w > 1;
  if (to_device) {
    if (l.kind == ACC_CONV) oihw_to_ohwi(host, tmp.data(), l.cout, l.cin, l.r, l.s);
    else if (fc_map) {
      oihw_to_ohwi(host, tmp.data(), l.cout, fc_c, fc_h, fc_w);
      std::memcpy(tmp.data() + (size_t)l.cout * l.cin, host + (size_t)l.cout * l.cin, l.cout * sizeof(float));
    }
    else std::memcpy(tmp.data(), host, n * sizeof(float));
    HIPCHK(c, hipMemcpyAsync(dev, tmp.data(), n * sizeof(float), hipMemcpyHostToDevice, c->s_c));
    HIPCHK(c, hipStreamSynchronize(c->s_c));
    if (!grads && c->d_params16) {   // bf16 mode: the kernels read the rounded copy
      std::vector<uint16_t> h16(n);
      for (size_t i = 0; i < n; ++i) h16[i] = float_to_bf16(tmp[i]);
      HIPCHK(c, hipMemcpyAsync(c->d_params16 + ps.offset, h16.data(), n * 2, hipMemcpyHostToDevice, c->s_c));
      HIPCHK(c, hipStreamSynchronize(c->s_c));
    }
  } else {
    HIPCHK(c, hipMemcpyAsync(tmp.data(), dev, n * sizeof(float), hipMemcpyDeviceToHost, c->s_c));
    HIPCHK(c, hipStreamSynchronize(c->s_c));
    if (l.kind == ACC_CONV) ohwi_to_oihw(tmp.data(), host, l.cout, l.cin, l.r, l.s);
    else if (fc_map) {
      ohwi_to_oihw(tmp.data(), host, l.cout, fc_c, fc_h, fc_w);
      std::memcpy(host + (size_t)l.cout * l.cin, tmp.data() + (size_t)l.cout * l.cin, l.cout * sizeof(float));
    }
    else std::memcpy(host, tmp.data(), n * sizeof(float));
  }
  return ACC_OK;
}

}  // namespace

// --------------------------------------------------------------------------- lifecycle
extern "C" int acc_create(const acc_layer* layers, int n_layers, int in_c, int in_h, int in_w, int dtype,
                          const acc_resources* res, acc_ctx** out) {
  if (!out) { g_create_error = "out is null"; return ACC_EINVAL; }
  *out = nullptr;
  if (dtype != ACC_F32 && dtype != ACC_BF16) { g_create_error = "dtype must be ACC_F32 or ACC_BF16"; return ACC_EINVAL; }
  acc_ctx* c = new (std::nothrow) acc_ctx();
  if (!c) { g_create_error = "out of host memory"; return ACC_EHOSTMEM; }
  std::string err;
  if (!c->g.build(layers, n_layers, in_c, in_h, in_w, dtype, &err)) {
    g_create_error = err;
    delete c;
    return ACC_EINVAL;
  }
  if (res) {
    if (!res->pool || !res->host || !res->s_compute || !res->s_out || !res->s_in ||
        ((uintptr_t)res->pool & 255) || ((uintptr_t)res->host & 255)) {
      g_create_error = "resources: null or not 256-byte aligned";
      delete c;
      return ACC_EINVAL;
    }
    if (res->s_compute == res->s_out || res->s_compute == res->s_in || res->s_out == res->s_in) {
      g_create_error = "resources: the three streams must differ";
      delete c;
      return ACC_EINVAL;
    }
    const size_t stat = c->g.static_bytes();
    if (res->pool_bytes < stat + 256) {
      g_create_error = "pool smaller than parameters + gradients";
      delete c;
      return ACC_EPOOL;
    }
    c->res = *res;
    c->have_res = true;
    c->s_c = (hipStream_t)res->s_compute;
    c->s_o = (hipStream_t)res->s_out;
    c->s_i = (hipStream_t)res->s_in;
    c->s_w = (hipStream_t)res->s_wgrad;
    if (c->s_w && (c->s_w == c->s_c || c->s_w == c->s_o || c->s_w == c->s_i)) {
      g_create_error = "resources: the weight-gradient stream must differ from the other three";
      delete c;
      return ACC_EINVAL;
    }
    char* p = (char*)res->pool;
    const size_t pb = al256(c->g.param_elems * sizeof(float));
    c->d_params = (float*)p; p += pb;
    c->d_grads = (float*)p; p += pb;
    if (dtype == ACC_BF16) { c->d_params16 = (uint16_t*)p; p += al256(c->g.param_elems * 2); }
    c->d_stats = (float*)p; p += al256(c->g.stat_elems * sizeof(float));
    c->d_loss = (float*)p; p += 256;
    c->dyn = p;
    c->dyn_cap = (res->pool_bytes - stat) & ~(size_t)255;
    hipError_t e = fill_zero(c->d_params, (pb * 2) / sizeof(float), c->s_c);
    if (e == hipSuccess) e = hipStreamSynchronize(c->s_c);
    if (e == hipSuccess) e = hipHostMalloc((void**)&c->h_loss, 256, hipHostMallocDefault);
    if (e == hipSuccess) e = hipEventCreate(&c->ev_begin);
    if (e == hipSuccess) e = hipEventCreate(&c->ev_end);
    if (c->s_w && e == hipSuccess) e = hipEventCreateWithFlags(&c->ev_flush, hipEventDisableTiming);
    if (c->s_w) {
      const size_t ns = c->g.steps.size();
      c->ev_fork.assign(ns, nullptr);
      c->ev_wdone.assign(ns, nullptr);
      c->wgrad_in_flight.assign(ns, 0);
      for (size_t j = 0; j < ns && e == hipSuccess; ++j) {
        if (c->g.steps[j].wgrad_join < 0) continue;
        e = hipEventCreateWithFlags(&c->ev_fork[j], hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ev_wdone[j], hipEventDisableTiming);
      }
    }
    if (e != hipSuccess) {
      g_create_error = std::string("device setup: ") + hipGetErrorString(e);
      acc_destroy(c);   // also releases the events and the pinned scalar made so far
      return ACC_EHIP;
    }
  }
  *out = c;
  return ACC_OK;
}

extern "C" void acc_destroy(acc_ctx* c) {
  if (!c) return;
  if (c->have_res) {
    (void)hipStreamSynchronize(c->s_c);
    (void)hipStreamSynchronize(c->s_o);
    (void)hipStreamSynchronize(c->s_i);
    if (c->s_w) (void)hipStreamSynchronize(c->s_w);
    c->drop_events();
    c->drop_graph();
    for (auto* v : {&c->ev_fork, &c->ev_wdone})
      for (hipEvent_t e : *v) if (e) (void)hipEventDestroy(e);
    for (auto& kp : c->kprobes) { (void)hipEventDestroy(kp.a); (void)hipEventDestroy(kp.b); }
    for (hipEvent_t e : c->empty_pair) if (e) (void)hipEventDestroy(e);
    if (c->ev_flush) (void)hipEventDestroy(c->ev_flush);
    if (c->ev_begin) (void)hipEventDestroy(c->ev_begin);
    if (c->ev_end) (void)hipEventDestroy(c->ev_end);
    if (c->h_loss) (void)hipHostFree(c->h_loss);
  }
  delete c;
}

extern "C" const char* acc_last_error(const acc_ctx* c) { return c ? c->err.c_str() : g_create_error.c_str(); }
extern "C" const char* acc_step_kind_name(int kind) { return step_kind_name(kind); }

extern "C" int acc_set_weights(acc_ctx* c, int layer, const float* w, size_t n) {
  return param_io(c, layer, const_cast<float*>(w), n, true, false);
}
extern "C" int acc_get_weights(acc_ctx* c, int layer, float* w, size_t n) { return param_io(c, layer, w, n, false, false); }
extern "C" int acc_get_grads(acc_ctx* c, int layer, float* g, size_t n) { return param_io(c, layer, g, n, false, true); }
extern "C" int acc_param_count(const acc_ctx* c, int layer, size_t* n) {
  if (!c || !n || layer < 0 || layer >= (int)c->g.layers.size()) return ACC_EINVAL;
  *n = c->g.params[layer].count;
  return ACC_OK;
}

// -------------------------------------------------------------------------- cost model
extern "C" int acc_set_cost_model(acc_ctx* c, double flops_per_s, double bytes_per_s, double launch_s,
                                  double d2h, double h2d, double copy_latency_s) {
  if (!c) return ACC_EINVAL;
  if (!(flops_per_s > 0) || !(bytes_per_s > 0) || launch_s < 0 || !(d2h > 0) || !(h2d > 0) || copy_latency_s < 0)
    return c->fail(ACC_EINVAL, "cost model parameters must be positive");
  c->cm.flops_per_s = flops_per_s; c->cm.bytes_per_s = bytes_per_s; c->cm.launch_s = launch_s;
  c->cm.d2h_bps = d2h; c->cm.h2d_bps = h2d; c->cm.copy_latency_s = copy_latency_s;
  c->cm.ks.clear(); c->cm.table.clear(); c->cm.fixed.clear();
  return ACC_OK;
}

extern "C" int acc_set_step_times(acc_ctx* c, const double* seconds, int n) {
  if (!c) return ACC_EINVAL;
  if (n == 0) { c->cm.fixed.clear(); return ACC_OK; }
  if (!seconds || n != (int)c->g.steps.size()) return c->fail(ACC_EINVAL, "need one time per step");
  for (int i = 0; i < n; ++i) if (!(seconds[i] >= 0)) return c->fail(ACC_EINVAL, "negative step time");
  c->cm.fixed.assign(seconds, seconds + n);
  return ACC_OK;
}

extern "C" int acc_get_calibration(const acc_ctx* c, int* ks, int max_k, double* seconds, size_t max_seconds,
                                   double* link) {
  if (!c) return ACC_EINVAL;
  const int nk = (int)c->cm.ks.size();
  const size_t ns = c->g.steps.size();
  if (link) { link[0] = c->cm.d2h_bps; link[1] = c->cm.h2d_bps; link[2] = c->cm.copy_latency_s; }
  if (ks) {
    if (max_k < nk) return ACC_EINVAL;
    for (int i = 0; i < nk; ++i) ks[i] = c->cm.ks[i];
  }
  if (seconds) {
    if (max_seconds < nk * ns) return ACC_EINVAL;
    for (int i = 0; i < nk; ++i)
      for (size_t j = 0; j < ns; ++j) seconds[i * ns + j] = c->cm.table[i][j];
  }
  return nk;
}

extern "C" int acc_set_calibration(acc_ctx* c, const int* ks, int nk, const double* seconds, const double* link) {
  if (!c) return ACC_EINVAL;
  if (!ks || !seconds || nk <= 0) return c->fail(ACC_EINVAL, "need at least one measured minibatch");
  const size_t ns = c->g.steps.size();
  for (int i = 0; i < nk; ++i)
    if (ks[i] <= 0 || (i > 0 && ks[i] <= ks[i - 1])) return c->fail(ACC_EINVAL, "minibatches must be positive and ascending");
  for (size_t i = 0; i < nk * ns; ++i)
    if (!(seconds[i] >= 0)) return c->fail(ACC_EINVAL, "negative step time");
  if (link && (!(link[0] > 0) || !(link[1] > 0) || !(link[2] >= 0))) return c->fail(ACC_EINVAL, "bad link figures");
  c->cm.fixed.clear();
  c->cm.ks.assign(ks, ks + nk);
  c->cm.table.assign(nk, std::vector<double>());
  for (int i = 0; i < nk; ++i) c->cm.table[i].assign(seconds + i * ns, seconds + (i + 1) * ns);
  if (link) { c->cm.d2h_bps = link[0]; c->cm.h2d_bps = link[1]; c->cm.copy_latency_s = link[2]; }
  c->plan.valid = false;
  return ACC_OK;
}

// ---------------------------------------------------------------------------- planning
namespace {

int install_plan(acc_ctx* c, Plan&& p, acc_plan_summary* out, double t0) {
  if (c->have_res) {
    if (p.budget > c->res.pool_bytes) return c->fail(ACC_EPOOL, "budget exceeds the pool");
    if (p.host_bytes > c->res.host_bytes) return c->fail(ACC_EHOSTMEM, "pinned host arena smaller than the swapped maps");
    HIPCHK(c, hipStreamSynchronize(c->s_c));
    HIPCHK(c, hipStreamSynchronize(c->s_o));
    HIPCHK(c, hipStreamSynchronize(c->s_i));
    if (c->s_w) HIPCHK(c, hipStreamSynchronize(c->s_w));
    c->drop_events();
    c->drop_graph();                      // a graph holds the pool offsets of the plan it was captured under
    const int ns = (int)c->g.steps.size();
    c->ev_step.assign(ns, nullptr);
    for (const Instr& in : p.instrs)
      if (in.op == I_COMPUTE && in.record)
        HIPCHK(c, hipEventCreateWithFlags(&c->ev_step[in.arg], hipEventDisableTiming));
    c->ev_d2h.assign(p.n_d2h, nullptr);
    c->ev_h2d.assign(p.n_h2d, nullptr);
    for (auto& e : c->ev_d2h) HIPCHK(c, hipEventCreateWithFlags(&e, hipEventDisableTiming));
    for (auto& e : c->ev_h2d) HIPCHK(c, hipEventCreateWithFlags(&e, hipEventDisableTiming));
    c->ev_window.assign(ns / kStepWindow + 1, nullptr);
    for (auto& e : c->ev_window) HIPCHK(c, hipEventCreateWithFlags(&e, hipEventDisableTiming));
  }
  c->plan = std::move(p);
  c->obs_start.clear(); c->obs_end.clear();   // observations belong to the plan they ran under
  c->stats = acc_stats{};
  {
    // Where the plan releases memory (for the poison mode): a tensor's block is free once the
    // last step that touches it has run; the block a swapped map is produced in is free once
    // its offload has finished, and the block it comes back into after its last use.
    const Plan& P = c->plan;
    const int ns = (int)c->g.steps.size();
    c->poison_after_step.assign(ns, {});
    c->poison_after_d2h.assign(P.n_d2h, {0, 0});
    for (int t = 0; t < (int)c->g.tensors.size(); ++t) {
      const Tensor& T = c->g.tensors[t];
      if (!P.tbytes[t] || T.last < 0 || T.last >= ns) continue;
      c->poison_after_step[T.last].push_back({P.swapped[t] ? P.off2[t] : P.off1[t], P.tbytes[t]});
    }
    for (const Instr& in : P.instrs)
      if (in.op == I_OFFLOAD) c->poison_after_d2h[in.seq] = {P.off1[in.arg], P.tbytes[in.arg]};
  }
  if (out) {
    const Plan& P = c->plan;
    std::memset(out, 0, sizeof *out);
    out->n_steps = (int)c->g.steps.size();
    out->n_maps = (int)c->g.maps.size();
    out->n_swapped = P.n_swapped;
    out->n_instr = (int)P.instrs.size();
    out->bytes_swapped = P.bytes_swapped;
    for (int t : c->g.maps) out->bytes_maps += P.tbytes[t];
    out->static_bytes = c->g.static_bytes();
    out->peak_bytes = out->static_bytes + P.dyn_peak;
    std::vector<uint8_t> all(c->g.tensors.size(), 0), none(c->g.tensors.size(), 0);
    for (int t : c->g.maps) all[t] = 1;
    out->layer_peak_bytes = out->static_bytes + live_peak(c->g, P.k, all);
    out->noswap_peak_bytes = out->static_bytes + live_peak(c->g, P.k, none);
    out->host_bytes = P.host_bytes;
    out->t_compute = P.t_compute;
    out->t_iter = P.t_iter;
    out->t_stall = P.t_stall;
    out->plan_ms = now_ms() - t0;
  }
  return ACC_OK;
}

}  // namespace

extern "C" int acc_plan_swaps(acc_ctx* c, int minibatch, size_t budget_bytes, int mode, acc_plan_summary* out) {
  if (!c) return ACC_EINVAL;
  const double t0 = now_ms();
  if (minibatch <= 0) return c->fail(ACC_EINVAL, "minibatch must be positive");
  c->plan.valid = false;
  Plan p;
  std::string why;
  const int rc = make_plan(c->g, c->cm, minibatch, budget_bytes, mode, &p, &why);
  if (rc != ACC_OK) return c->fail(rc, why);
  return install_plan(c, std::move(p), out, t0);
}

extern "C" int acc_plan_explicit(acc_ctx* c, int minibatch, size_t budget_bytes, const uint8_t* swap, int n_maps,
                                 acc_plan_summary* out) {
  if (!c) return ACC_EINVAL;
  const double t0 = now_ms();
  if (minibatch <= 0 || !swap || n_maps != (int)c->g.maps.size()) return c->fail(ACC_EINVAL, "need one flag per map");
  c->plan.valid = false;
  std::vector<uint8_t> sw(c->g.tensors.size(), 0);
  for (int i = 0; i < n_maps; ++i) sw[c->g.maps[i]] = swap[i] ? 1 : 0;
  Plan p;
  std::string why;
  if (!build_plan(c->g, minibatch, budget_bytes, sw, PlanOptions(), &p, &why)) return c->fail(ACC_EUNTRAINABLE, why);
  simulate(c->g, c->cm, &p);
  p.mode = -1;
  return install_plan(c, std::move(p), out, t0);
}

extern "C" int acc_tune_minibatch(acc_ctx* c, size_t budget_bytes, int k_lo, int k_hi, acc_tune_result* out,
                                  acc_plan_summary* plan_out) {
  if (!c) return ACC_EINVAL;
  const double t0 = now_ms();
  if (k_lo <= 0 || k_hi < k_lo || !out) return c->fail(ACC_EINVAL, "need 0 < k_lo <= k_hi and a result struct");
  c->plan.valid = false;
  const int nt = (int)c->g.tensors.size();
  std::vector<uint8_t> none(nt, 0), all(nt, 0);
  for (int t : c->g.maps) all[t] = 1;
  auto feasible = [&](int k, const std::vector<uint8_t>& sw) {
    if (budget_bytes < c->g.static_bytes() + 256) return false;
    Plan p;
    std::string why;
    return build_plan(c->g, k, budget_bytes, sw, PlanOptions(), &p, &why);
  };
  auto largest = [&](const std::vector<uint8_t>& sw) {   // feasibility is monotone in k (Eq. 4)
    if (!feasible(k_lo, sw)) return 0;
    int lo = k_lo, hi = k_hi;
    while (lo < hi) {
      const int mid = lo + (hi - lo + 1) / 2;
      if (feasible(mid, sw)) lo = mid; else hi = mid - 1;
    }
    return lo;
  };
  const int k_max = largest(all);
  if (k_max == 0) return c->fail(ACC_EUNTRAINABLE, "the smallest minibatch of the range does not train under the budget");
  const int k_fit = largest(none);
  std::vector<int> cand;
  for (int k = k_lo; k <= k_fit; ++k) cand.push_back(k);
  for (double x = std::max(k_fit, k_lo - 1) + 1.0; x <= k_max; x = std::max(x + 1.0, x * 1.15)) cand.push_back((int)x);
  if (cand.empty() || cand.back() != k_max) cand.push_back(k_max);
  int best_k = 0, n_eval = 0;
  double best_rate = -1.0;
  for (int k : cand) {
    Plan p;
    std::string why;
    if (make_plan(c->g, c->cm, k, budget_bytes, ACC_PLAN_DYNAMIC, &p, &why) != ACC_OK) continue;
    ++n_eval;
    const double rate = p.t_iter > 0 ? k / p.t_iter : 0.0;
    if (rate >= best_rate) { best_rate = rate; best_k = k; }
  }
  if (best_k == 0) return c->fail(ACC_EUNTRAINABLE, "no minibatch of the range could be planned");
  Plan p;
  std::string why;
  const int rc = make_plan(c->g, c->cm, best_k, budget_bytes, ACC_PLAN_DYNAMIC, &p, &why);
  if (rc != ACC_OK) return c->fail(rc, why);
  out->k_best = best_k;
  out->k_trainable_max = k_max;
  out->k_noswap_max = k_fit;
  out->n_evaluated = n_eval;
  out->images_per_s = best_rate;
  out->t_iter = p.t_iter;
  out->t_stall = p.t_stall;
  const int rc2 = install_plan(c, std::move(p), plan_out, t0);
  out->tune_ms = now_ms() - t0;
  return rc2;
}

extern "C" double acc_adaptive_lr(double lr_base, double cvx, double q) {
  if (!(cvx > 0) || !(lr_base > 0) || !(lr_base * cvx < 1) || !(q > 0)) return std::nan("");
  return (1.0 - std::pow(1.0 - lr_base * cvx, q)) / cvx;
}

extern "C" int acc_get_step_count(const acc_ctx* c) { return c ? (int)c->g.steps.size() : ACC_EINVAL; }
extern "C" int acc_get_tensor_count(const acc_ctx* c) { return c ? (int)c->g.tensors.size() : ACC_EINVAL; }

extern "C" int acc_get_step_info(const acc_ctx* c, int step, acc_step_info* out) {
  if (!c || !out || step < 0 || step >= (int)c->g.steps.size()) return ACC_EINVAL;
  const Step& s = c->g.steps[step];
  std::memset(out, 0, sizeof *out);
  out->kind = s.kind; out->layer = s.layer; out->backward = s.phase;
  const int k = c->plan.valid ? c->plan.k : 1;
  out->flops = s.flops_per_image * k;
  if (c->plan.valid) {
    out->t_compute = c->plan.t_cost[step]; out->t_ready = c->plan.t_ready[step];
    out->t_start = c->plan.t_start[step]; out->t_end = c->plan.t_end[step];
  }
  return ACC_OK;
}

extern "C" int acc_get_tensor_info(const acc_ctx* c, int t, acc_tensor_info* out) {
  if (!c || !out || t < 0 || t >= (int)c->g.tensors.size()) return ACC_EINVAL;
  const Tensor& T = c->g.tensors[t];
  std::memset(out, 0, sizeof *out);
  out->kind = T.kind; out->producer_step = T.producer; out->last_fwd_step = T.last_fwd;
  out->first_bwd_step = T.first_bwd; out->last_step = T.last; out->is_map = T.is_map;
  if (c->plan.valid) {
    const size_t stat = c->g.static_bytes();
    out->swapped = c->plan.swapped[t]; out->bytes = c->plan.tbytes[t];
    out->offset = stat + c->plan.off1[t]; out->offset2 = stat + c->plan.off2[t]; out->host_offset = c->plan.host_off[t];
  } else {
    out->bytes = c->g.bytes(t, 1);
  }
  return ACC_OK;
}

extern "C" int acc_get_step_io(const acc_ctx* c, int step, int32_t* reads, int max_reads, int32_t* writes, int max_writes) {
  if (!c || step < 0 || step >= (int)c->g.steps.size()) return ACC_EINVAL;
  const Step& s = c->g.steps[step];
  if ((int)s.reads.size() > max_reads || (int)s.writes.size() > max_writes) return ACC_EINVAL;
  for (size_t i = 0; i < s.reads.size(); ++i) reads[i] = s.reads[i];
  for (size_t i = 0; i < s.writes.size(); ++i) writes[i] = s.writes[i];
  return (int)(s.reads.size() * 256 + s.writes.size());
}

extern "C" int acc_get_instr_count(const acc_ctx* c) {
  if (!c) return ACC_EINVAL;
  return c->plan.valid ? (int)c->plan.instrs.size() : 0;
}

extern "C" int acc_get_instr(const acc_ctx* c, int i, acc_instr* out) {
  if (!c || !out || !c->plan.valid || i < 0 || i >= (int)c->plan.instrs.size()) return ACC_EINVAL;
  const Instr& in = c->plan.instrs[i];
  out->op = in.op; out->arg = in.arg; out->wait_step = in.wait_step; out->wait_d2h = in.wait_d2h;
  out->wait_h2d = in.wait_h2d; out->seq = in.seq; out->record = in.record ? 1 : 0; out->reserved = 0;
  return ACC_OK;
}

// ---------------------------------------------------------------------------- executor
namespace {

hipError_t fill_pseudo_input(acc_ctx* c, float* p, size_t count);

// Poison patterns of the verification mode: a word that is a NaN as fp32, as two bf16 values
// and (two of them) as a double, so that a kernel that reads memory nobody has written for
// it yields NaN.  kNeverWritten marks the dynamic region before the iteration, kReleased a
// block whose tensor has had its last use.
constexpr uint32_t kNeverWritten = 0x7FF87FF8u, kReleased = 0x7FF97FF9u;

__global__ void fill_word_kernel(uint32_t* __restrict__ p, size_t words, uint32_t v) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < words; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

// out[0] = 1 + index of the last word that differs from `untouched` (0 if none), out[1] = how
// many words differ.  out must be zero before the launch.
__global__ void written_extent_kernel(const uint32_t* __restrict__ p, size_t words, uint32_t untouched,
                                      unsigned long long* __restrict__ out) {
  unsigned long long hi = 0, cnt = 0;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < words; i += (size_t)gridDim.x * blockDim.x)
    if (p[i] != untouched) { hi = i + 1; ++cnt; }
  for (int o = 32; o > 0; o >>= 1) {
    const unsigned long long h2 = __shfl_xor(hi, o), c2 = __shfl_xor(cnt, o);
    hi = h2 > hi ? h2 : hi;
    cnt += c2;
  }
  if ((threadIdx.x & 63) == 0 && cnt) {
    atomicMax(out, hi);
    atomicAdd(out + 1, cnt);
  }
}

hipError_t fill_words(void* p, size_t bytes, uint32_t v, hipStream_t st) {
  if (!bytes) return hipSuccess;
  const size_t words = bytes / 4;
  const size_t blocks = std::min<size_t>((words + 255) / 256, 256 * 16);
  hipLaunchKernelGGL(fill_word_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (uint32_t*)p, words, v);
  return hipGetLastError();
}

// launches the kernels of one step on the compute stream
// Adds up the parts of the last conv weight gradient on the stream it ran on; the compute
// stream then waits for that stream (the update reads the result).
hipError_t flush_pending_reduce(acc_ctx* c) {
  if (!c->pending_reduce.count) return hipSuccess;
  hipError_t e = reduce_parts(c->pending_reduce, c->pending_stream);
  c->pending_reduce = ReduceJob{nullptr, nullptr, 0, 0};
  if (e != hipSuccess || c->pending_stream == c->s_c) return e;
  if ((e = hipEventRecord(c->ev_flush, c->pending_stream)) != hipSuccess) return e;
  return hipStreamWaitEvent(c->s_c, c->ev_flush, 0);
}

hipError_t run_step(acc_ctx* c, int j, float lr) {
  const Graph& g = c->g;
  const Step& s = g.steps[j];
  const int k = c->plan.k;
  auto ptr = [&](int t) -> float* { return t < 0 ? nullptr : (float*)(c->dyn + c->cur_off[t]); };
  const int dt = g.dtype;
  const size_t es = dt_size(dt);
  auto T = [&](int t) -> const Tensor& { return g.tensors[t]; };
  hipStream_t st = c->s_c;
  const acc_layer* l = s.layer >= 0 ? &g.layers[s.layer] : nullptr;
  float* w = s.layer >= 0 ? c->d_params + g.params[s.layer].offset : nullptr;
  float* dw = s.layer >= 0 ? c->d_grads + g.params[s.layer].offset : nullptr;
  // the filter copy the convolution kernels read: the fp32 weights themselves, or their bf16 copy
  const void* wk = s.layer < 0 ? nullptr
                   : dt == ACC_BF16 ? (const void*)(c->d_params16 + g.params[s.layer].offset) : (const void*)w;
  auto igemm = [&](const ConvGeom& cg, double flops) {
    LaunchProbe lp;
    LaunchProbe* pp = c->next_probe(&lp, flops, j, s.phase == 1 ? 1 : 0);
    const hipError_t e = conv_igemm(cg, st, pp);
    if (pp) c->kprobes[c->kprobes_used - 1].variant = lp.variant;
    return e;
  };
  auto wgrad = [&](const WgradGeom& wg, double flops, ReduceJob* deferred, hipStream_t on = nullptr) {
    LaunchProbe lp;
    LaunchProbe* pp = c->next_probe(&lp, flops, j, 2);
    const hipError_t e = conv_wgrad(wg, on ? on : st, pp, deferred);
    if (pp) c->kprobes[c->kprobes_used - 1].variant = lp.variant;
    return e;
  };
  // algorithmic flops of one of the three GEMMs of a convolution at this minibatch
  const double conv_flops = s.flops_per_image * k / (s.phase == 1 && s.dx >= 0 ? 2.0 : 1.0);
  switch (s.kind) {
    case K_INPUT_F:
      return nchw_to_nhwc(ptr(s.x), ptr(s.y), k, g.in_c, g.in_h * g.in_w, dt, st);
    case K_CONV_F: {
      ConvGeom cg{};
      cg.in = ptr(s.x); cg.w = wk; cg.out = ptr(s.y); cg.dtype = dt;
      cg.n_img = k; cg.h = T(s.x).h; cg.wd = T(s.x).w; cg.c = l->cin;
      cg.p = T(s.y).h; cg.q = T(s.y).w; cg.n_out = l->cout;
      cg.r = l->r; cg.s = l->s; cg.stride = l->stride; cg.pad = l->pad;
      cg.out_h = cg.p; cg.out_w = cg.q; cg.out_stride = 1; cg.accumulate = 0;
      if (s.bias_layer >= 0) {   // conv + bias (+ ReLU) in one launch
        cg.bias = c->d_params + g.params[s.bias_layer].offset;
        cg.relu = s.relu ? 1 : 0;
      }
      // the batch norm that follows takes its sums from this launch (fp32 storage; with bf16
      // the statistics are those of the rounded values) unless there are more 32-row blocks
      // than its finishing pass adds up
      if (s.stats >= 0) {
        const long rows = (long)k * cg.p * cg.q;
        const long slabs = conv_stat_slabs(rows);
        const long stride = (long)k * 2 * (((long)cg.p * cg.q + 63) / 64);
        const bool fused = slabs <= kBnMaxSlabs && (size_t)2 * stride * l->cout * sizeof(float) <= c->plan.tbytes[s.stats];
        c->bn_ready_slabs[s.stats_for] = fused ? (int)slabs : 0;
        if (fused) { cg.stats = (float*)ptr(s.stats); cg.stats_stride = (int)stride; }
      }
      return igemm(cg, conv_flops);
    }
    case K_BN_F: {
      float* stat = c->d_stats + g.params[s.layer].stat_offset;
      BnSums ready{nullptr, 0, 0};
      if (s.stats >= 0 && c->bn_ready_slabs[j] > 0) {
        ready.part = (const float*)ptr(s.stats);
        ready.slabs = c->bn_ready_slabs[j];
        ready.stride = (int)((long)k * 2 * (((long)T(s.x).h * T(s.x).w + 63) / 64));
      }
      return bn_forward(ptr(s.x), w, w + l->cin, ptr(s.res), ptr(s.y), stat, stat + l->cin,
                        (long)k * T(s.x).h * T(s.x).w, l->cin, s.relu, 1e-5f, ptr(s.ws), dt, st,
                        ready.part ? &ready : nullptr);
    }
    case K_MAXPOOL_F:
      return maxpool_forward(ptr(s.x), ptr(s.y), k, T(s.x).h, T(s.x).w, T(s.x).c, l->r, l->s, l->stride, l->pad, dt, st);
    case K_GAP_F:
      return gap_forward(ptr(s.x), ptr(s.y), k, T(s.x).h * T(s.x).w, T(s.x).c, dt, st);
    case K_FC_F: {
      ConvGeom cg{};
      cg.in = ptr(s.x); cg.w = wk; cg.out = ptr(s.y); cg.dtype = dt;
      cg.n_img = k; cg.h = 1; cg.wd = 1; cg.c = l->cin; cg.p = 1; cg.q = 1; cg.n_out = l->cout;
      cg.r = 1; cg.s = 1; cg.stride = 1; cg.pad = 0; cg.out_h = 1; cg.out_w = 1; cg.out_stride = 1;
      hipError_t e = igemm(cg, conv_flops);
      if (e != hipSuccess) return e;
      return bias_add(ptr(s.y), w + (size_t)l->cout * l->cin, k, l->cout, dt, st, s.relu ? 1 : 0);
    }
    case K_LOSS_F:
      return softmax_ce_forward(ptr(s.x), (const int32_t*)ptr(g.t_labels), ptr(s.ws), c->d_loss, k, g.classes, dt, st);
    case K_LOSS_B:
      return softmax_ce_backward(ptr(s.x), (const int32_t*)ptr(g.t_labels), ptr(s.dx), k, g.classes, dt, st);
    case K_FC_B: {
      if (s.relu) {   // FC + ReLU: mask the gradient with [y > 0] first
        const hipError_t em = relu_mask(ptr(s.dy), ptr(s.y), (size_t)k * l->cout, dt, st);
        if (em != hipSuccess) return em;
      }
      WgradGeom wg{};
      wg.x = ptr(s.x); wg.dy = ptr(s.dy); wg.dw = dw; wg.dtype = dt;
      wg.n_img = k; wg.h = 1; wg.wd = 1; wg.cin = l->cin; wg.p = 1; wg.q = 1; wg.cout = l->cout;
      wg.r = 1; wg.s = 1; wg.stride = 1; wg.pad = 0; wg.workspace = ptr(s.ws2);
      // the transposed filter for the data gradient is written by extra workgroups of the
      // weight-gradient launch; the parts of the weight gradient are added up by extra
      // workgroups of the data-gradient launch
      wg.flip_w = wk; wg.flip_wt = ptr(s.ws);
      ReduceJob job;
      hipError_t e = wgrad(wg, conv_flops, &job);
      if (e != hipSuccess) return e;
      e = column_sum(ptr(s.dy), dw + (size_t)l->cout * l->cin, k, l->cout, dt, st);
      if (e != hipSuccess) return e;
      ConvGeom cg{};
      cg.side = job;
      cg.in = ptr(s.dy); cg.w = ptr(s.ws); cg.out = ptr(s.dx); cg.dtype = dt;
      cg.n_img = k; cg.h = 1; cg.wd = 1; cg.c = l->cout; cg.p = 1; cg.q = 1; cg.n_out = l->cin;
      cg.r = 1; cg.s = 1; cg.stride = 1; cg.pad = 0; cg.out_h = 1; cg.out_w = 1; cg.out_stride = 1;
      cg.accumulate = s.dx_accumulate;
      return igemm(cg, conv_flops);
    }
    case K_GAP_B:
      return gap_backward(ptr(s.dy), ptr(s.dx), k, T(s.dx).h * T(s.dx).w, T(s.dx).c, s.dx_accumulate, dt, st);
    case K_MAXPOOL_B:
      return maxpool_backward(ptr(s.x), ptr(s.dy), ptr(s.dx), k, T(s.x).h, T(s.x).w, T(s.x).c, l->r, l->s,
                              l->stride, l->pad, s.dx_accumulate, dt, st);
    case K_BN_B: {
      float* stat = c->d_stats + g.params[s.layer].stat_offset;
      if (s.bnb >= 0 && c->bn_ready_slabs[j] > 0) {
        // the data gradient before this step masked dy and left the sums
        BnSums ready{(const float*)ptr(s.bnb), c->bn_ready_slabs[j],
                     (int)((long)k * 2 * (((long)T(s.x).h * T(s.x).w + 63) / 64))};
        return bn_backward(ptr(s.x), ptr(s.dy), nullptr, w, stat, stat + l->cin, ptr(s.dx), dw, dw + l->cin, nullptr,
                           (long)k * T(s.x).h * T(s.x).w, l->cin, ptr(s.ws), dt, st, &ready);
      }
      return bn_backward(ptr(s.x), ptr(s.dy), ptr(s.y), w, stat, stat + l->cin, ptr(s.dx), dw, dw + l->cin,
                         s.g_inplace ? ptr(s.dy) : nullptr, (long)k * T(s.x).h * T(s.x).w, l->cin, ptr(s.ws), dt, st);
    }
    case K_CONV_B: {
      const int h = T(s.x).h, wd = T(s.x).w, ho = T(s.dy).h, wo = T(s.dy).w;
      if (s.bias_layer >= 0) {
        // conv + bias (+ ReLU): mask the gradient with [y > 0] in place and sum it per channel
        // (the bias gradient) before the two GEMMs read it
        float* db = c->d_grads + g.params[s.bias_layer].offset;
        const hipError_t eb = relu_bias_backward(ptr(s.dy), s.relu ? ptr(s.y) : nullptr, db, (long)k * ho * wo, l->cout,
                                                 ptr(s.ws3), dt, st);
        if (eb != hipSuccess) return eb;
      }
      WgradGeom wg{};
      wg.x = ptr(s.x); wg.dy = ptr(s.dy); wg.dw = dw; wg.dtype = dt;
      wg.n_img = k; wg.h = h; wg.wd = wd; wg.cin = l->cin; wg.p = ho; wg.q = wo; wg.cout = l->cout;
      wg.r = l->r; wg.s = l->s; wg.stride = l->stride; wg.pad = l->pad;
      wg.workspace = ptr(s.ws2);
      if (s.dx < 0) return wgrad(wg, conv_flops, nullptr);   // first layer: no data gradient
      const bool split = l->stride > 1 && (l->r > 1 || l->s > 1 || l->pad > 0);
      // The weight gradient reads x and dy and writes only its own partial sums and dw, so it
      // may run beside the steps that follow: on the weight-gradient stream if there is one
      // (not while single kernels are being timed), joined kWgradLag conv steps later.
      const bool aside = c->s_w && c->wgrad_overlap && !c->kernel_profiling && s.wgrad_join >= 0;
      const hipStream_t sw = aside ? c->s_w : st;
      hipError_t e;
      if (aside) {
        if ((e = hipEventRecord(c->ev_fork[j], st)) != hipSuccess) return e;        // dy (and x) are ready
        if ((e = hipStreamWaitEvent(sw, c->ev_fork[j], 0)) != hipSuccess) return e;
      }
      // the parts of the previous conv weight gradient (same stream) are added up by extra
      // workgroups of this launch; this one's by the next, the last one's before the update
      if (c->pending_reduce.count && c->pending_stream != sw) {
        if ((e = flush_pending_reduce(c)) != hipSuccess) return e;
      }
      wg.side = c->pending_reduce;
      ReduceJob job;
      if ((e = wgrad(wg, conv_flops, &job, sw)) != hipSuccess) return e;
      c->pending_reduce = job;
      c->pending_stream = sw;
      if (aside) {
        if ((e = hipEventRecord(c->ev_wdone[j], sw)) != hipSuccess) return e;
        c->wgrad_in_flight[j] = 1;
      }
      // the flipped, transposed filter: written by the previous conv backward step's launch,
      // unless this is the first one
      if (s.flips_itself && (e = filter_flip_transpose(wk, ptr(s.ws), l->cout, l->cin, l->r, l->s, dt, st)) != hipSuccess)
        return e;
      ConvGeom cg{};
      if (s.flip_for >= 0) {   // ... and the next one's rides on this step's launch
        const Step& nx = g.steps[s.flip_for];
        const acc_layer& nl = g.layers[nx.layer];
        const float* nw = c->d_params + g.params[nx.layer].offset;
        cg.flip.w = dt == ACC_BF16 ? (const void*)(c->d_params16 + g.params[nx.layer].offset) : (const void*)nw;
        cg.flip.wt = ptr(nx.ws);
        cg.flip.cout = nl.cout; cg.flip.cin = nl.cin; cg.flip.r = nl.r; cg.flip.s = nl.s;
      }
      cg.in = ptr(s.dy); cg.w = ptr(s.ws); cg.out = ptr(s.dx); cg.dtype = dt;
      cg.n_img = k; cg.h = ho; cg.wd = wo; cg.c = l->cout; cg.n_out = l->cin;
      cg.r = l->r; cg.s = l->s; cg.stride = 1; cg.accumulate = s.dx_accumulate;
      cg.out_h = h; cg.out_w = wd;
      if (split) {
        // strided and larger than 1x1: one stride-1 convolution per residue class of the dx
        // position, each with its own sub-filter; the first launch carries the side job
        DgradPart parts[kMaxDgradParts];
        bool covers_all = false;
        size_t wt_bytes = 0;
        const int np = dgrad_split(h, wd, l->cin, l->cout, l->r, l->s, l->stride, l->pad, (int)es, parts, &covers_all,
                                   &wt_bytes);
        if (np <= 0 || wt_bytes > T(s.ws).bytes_fixed) return hipErrorInvalidValue;
        if (!covers_all && !s.dx_accumulate) {
          e = fill_zero(ptr(s.dx), (size_t)k * h * wd * l->cin * es / 4, st);
          if (e != hipSuccess) return e;
        }
        double work = 0;
        for (int i = 0; i < np; ++i) work += (double)parts[i].p * parts[i].q * parts[i].nr * parts[i].ns;
        for (int i = 0; i < np; ++i) {
          const DgradPart& pt = parts[i];
          e = filter_gather_transpose(wk, ptr(s.ws), l->cout, l->cin, l->r, l->s, l->stride, pt, dt, st);
          if (e != hipSuccess) return e;
          cg.w = (const char*)ptr(s.ws) + pt.wt_offset;
          cg.p = pt.p; cg.q = pt.q; cg.r = pt.nr; cg.s = pt.ns;
          cg.pad = pt.pad_y; cg.pad_dx = pt.pad_x - pt.pad_y;
          cg.out_stride = l->stride; cg.out_y0 = pt.y0; cg.out_x0 = pt.x0;
          e = igemm(cg, conv_flops * ((double)pt.p * pt.q * pt.nr * pt.ns / work));
          if (e != hipSuccess) return e;
          cg.flip = FlipJob{};         // the side job went with the first part
        }
        return hipSuccess;
      }
      if (l->stride == 1) {
        cg.p = h; cg.q = wd; cg.pad = l->r - 1 - l->pad; cg.out_stride = 1;
        // the batch norm whose ReLU output was this convolution's input gets its backward sums
        // (and the masked gradient) from this launch, unless there are more 32-row blocks than
        // its finishing pass adds up
        if (s.bnb >= 0) {
          const Step& bb = g.steps[s.bnb_for];
          const long rows = (long)k * h * wd;
          const long slabs = conv_stat_slabs(rows);
          const long stride = (long)k * 2 * (((long)h * wd + 63) / 64);
          const bool fused = slabs <= kBnMaxSlabs && (size_t)2 * stride * l->cin * sizeof(float) <= c->plan.tbytes[s.bnb];
          c->bn_ready_slabs[s.bnb_for] = fused ? (int)slabs : 0;
          if (fused) {
            const float* stat = c->d_stats + g.params[bb.layer].stat_offset;
            cg.bnb = BnBackwardSums{ptr(bb.x), ptr(s.x), stat, stat + l->cin, (float*)ptr(s.bnb), (int)stride};
          }
        }
      } else {  // 1x1, pad 0: dense product on the strided positions, zeros elsewhere
        cg.p = ho; cg.q = wo; cg.pad = 0; cg.out_stride = l->stride;
        if (!s.dx_accumulate) {
          e = fill_zero(ptr(s.dx), (size_t)k * h * wd * l->cin * es / 4, st);   // whole words: cin is even
          if (e != hipSuccess) return e;
        }
      }
      return igemm(cg, conv_flops);
    }
    case K_SGD:
      if (hipError_t e = flush_pending_reduce(c); e != hipSuccess) return e;
      if (c->capturing) return hipSuccess;   // the learning rate is an argument: the update is launched after the graph
      return sgd_update(c->d_params, c->d_grads, lr, g.param_elems, c->d_params16, st);
  }
  return hipErrorInvalidValue;
}

}  // namespace

extern "C" int acc_train_step(acc_ctx* c, const float* images, int images_loc, const int32_t* labels, float lr,
                              float* loss_out) {
  if (!c) return ACC_EINVAL;
  if (!c->have_res) return c->fail(ACC_ESTATE, "context has no device resources");
  if (!c->plan.valid) return c->fail(ACC_ESTATE, "call acc_plan_swaps first");
  if (!c->calibrating && (!images || !labels)) return c->fail(ACC_EINVAL, "images / labels are null");
  if (images_loc != ACC_LOC_HOST && images_loc != ACC_LOC_DEVICE) return c->fail(ACC_EINVAL, "bad images_loc");
  const Plan& P = c->plan;
  const Graph& g = c->g;
  const int ns = (int)g.steps.size();
  const double t_host0 = now_ms();
  c->cur_off = P.off1;
  if ((c->profiling || c->kernel_profiling) && P.host_bytes > kMaxTimedSwapBytes)
    return c->fail(ACC_ESTATE, "profiling is switched off for plans that swap more than 24 GiB per iteration");
  if (c->profiling) {
    if ((int)c->prof_a.size() != ns) {
      c->prof_a.assign(ns, nullptr); c->prof_b.assign(ns, nullptr);
      for (int j = 0; j < ns; ++j) { HIPCHK(c, hipEventCreate(&c->prof_a[j])); HIPCHK(c, hipEventCreate(&c->prof_b[j])); }
    }
    const size_t nc = P.n_d2h + P.n_h2d;
    if (c->prof_copy_a.size() != nc) {
      for (hipEvent_t e : c->prof_copy_a) (void)hipEventDestroy(e);
      for (hipEvent_t e : c->prof_copy_b) (void)hipEventDestroy(e);
      c->prof_copy_a.assign(nc, nullptr); c->prof_copy_b.assign(nc, nullptr);
      for (size_t i = 0; i < nc; ++i) { HIPCHK(c, hipEventCreate(&c->prof_copy_a[i])); HIPCHK(c, hipEventCreate(&c->prof_copy_b[i])); }
    }
  }
  if (!c->calibrating) {
    // a label indexes the logits: one outside [0, classes) must not reach the loss kernel
    for (int i = 0; i < P.k; ++i)
      if (labels[i] < 0 || labels[i] >= g.classes) return c->fail(ACC_EINVAL, "label outside [0, classes)");
  }
  for (const auto* table : {&c->capture_at, &c->inject_at})
    for (const auto& list : *table)
      for (const acc_ctx::Capture& cp : list)
        if (cp.cap < (size_t)P.k * g.tensors[cp.tensor].bytes_per_image)
          return c->fail(ACC_EINVAL, "a capture / injection buffer is smaller than the layer's output at this minibatch");
  const bool poison = (c->debug_flags & ACC_DEBUG_POISON) != 0;
  unsigned long long* d_scan = (unsigned long long*)((char*)c->d_loss + 16);
  if (poison) {
    // nothing in the dynamic region or in the host arena is valid before the iteration
    hipError_t e = fill_words(c->dyn, c->dyn_cap, kNeverWritten, c->s_c);
    if (e == hipSuccess) e = fill_zero((float*)d_scan, 4, c->s_c);
    if (e != hipSuccess) return c->hipfail(e, "poison fill");
    HIPCHK(c, hipStreamSynchronize(c->s_c));
    uint32_t* hw = (uint32_t*)c->res.host;
    std::fill(hw, hw + P.host_bytes / 4, kNeverWritten);
  }
  uint64_t bytes_out = 0, bytes_in = 0;
  c->bn_ready_slabs.assign(ns, 0);
  std::fill(c->wgrad_in_flight.begin(), c->wgrad_in_flight.end(), 0);   // (a failed step may have left some set)
  c->pending_reduce = ReduceJob{nullptr, nullptr, 0, 0};
  c->kprobes_used = 0;
  if (c->kernel_profiling) {
    // the time between two events with no kernel between them is taken off every probe
    for (hipEvent_t& e : c->empty_pair) {
      if (!e) HIPCHK(c, hipEventCreate(&e));
      HIPCHK(c, hipEventRecord(e, c->s_c));
    }
  }
  HIPCHK(c, hipEventRecord(c->ev_begin, c->s_c));
  // Graph mode: an iteration that swaps nothing is the same sequence of launches every time, with the
  // same addresses; only the input copies (their source is the caller's) and the update kernel (the
  // learning rate is its argument) stay outside the graph.
  bool no_hooks = true;
  for (const auto* table : {&c->capture_at, &c->inject_at})
    for (const auto& list : *table) no_hooks = no_hooks && list.empty();
  const bool graph_mode = c->use_graph && P.n_swapped == 0 && P.n_d2h == 0 && !c->profiling && !c->kernel_profiling &&
                          !poison && !c->calibrating && no_hooks;
  bool graph_started = false, graph_replayed = false;
  auto abort_capture = [&]() {
    hipGraph_t dead = nullptr;
    (void)hipStreamEndCapture(c->s_c, &dead);
    if (dead) (void)hipGraphDestroy(dead);
    c->capturing = false;
    c->drop_graph();
    (void)hipGetLastError();
  };
  int n_compute = 0;
  double t_waited = 0.0;     // host time spent blocked on the flow-control windows (the GPU is behind, not the host)
  auto window_wait = [&](hipEvent_t e) {
    const double t0w = now_ms();
    const hipError_t r = hipEventSynchronize(e);
    t_waited += now_ms() - t0w;
    return r;
  };
  for (const Instr& in : P.instrs) {
    if ((in.op == I_LOAD_INPUT || in.op == I_PREFETCH) && in.seq >= kCopyWindow)
      HIPCHK(c, window_wait(c->ev_h2d[in.seq - kCopyWindow]));
    if (in.op == I_OFFLOAD && in.seq >= kCopyWindow)
      HIPCHK(c, window_wait(c->ev_d2h[in.seq - kCopyWindow]));
    if (in.op == I_COMPUTE && n_compute % kStepWindow == 0 && n_compute / kStepWindow >= kWindows)
      HIPCHK(c, window_wait(c->ev_window[n_compute / kStepWindow - kWindows]));
    switch (in.op) {
      case I_LOAD_INPUT: {
        void* dst = c->dyn + c->cur_off[in.arg];
        if (c->calibrating) {
          if (in.arg == g.t_stage) {
            hipError_t e = fill_pseudo_input(c, (float*)dst, (size_t)P.k * g.in_c * g.in_h * g.in_w);
            if (e != hipSuccess) return c->hipfail(e, "fill_pseudo_input");
          } else {
            hipError_t e = fill_zero((float*)dst, (size_t)P.k, c->s_i);
            if (e != hipSuccess) return c->hipfail(e, "fill_zero(labels)");
          }
        } else if (in.arg == g.t_stage) {
          const size_t bytes = (size_t)P.k * g.in_c * g.in_h * g.in_w * sizeof(float);
          HIPCHK(c, hipMemcpyAsync(dst, images, bytes,
                                   images_loc == ACC_LOC_HOST ? hipMemcpyHostToDevice : hipMemcpyDeviceToDevice, c->s_i));
        } else {
          HIPCHK(c, hipMemcpyAsync(dst, labels, (size_t)P.k * sizeof(int32_t), hipMemcpyHostToDevice, c->s_i));
        }
        HIPCHK(c, hipEventRecord(c->ev_h2d[in.seq], c->s_i));
        break;
      }
      case I_COMPUTE: {
        if (graph_mode) {
          if (!graph_started) {
            graph_started = true;
            // every input copy has been issued (they head the list); the graph starts behind them
            for (int q = 0; q < P.n_h2d; ++q) HIPCHK(c, hipStreamWaitEvent(c->s_c, c->ev_h2d[q], 0));
            if (c->graph_exec) {
              HIPCHK(c, hipGraphLaunch(c->graph_exec, c->s_c));
              graph_replayed = true;
            } else {
              HIPCHK(c, hipStreamBeginCapture(c->s_c, hipStreamCaptureModeThreadLocal));
              c->capturing = true;
            }
          }
          if (graph_replayed) break;
          hipError_t e = hipSuccess;
          for (int jw : g.steps[in.arg].joins)
            if (c->s_w && c->wgrad_in_flight[jw] && e == hipSuccess) {
              e = hipStreamWaitEvent(c->s_c, c->ev_wdone[jw], 0);
              c->wgrad_in_flight[jw] = 0;
            }
          if (e == hipSuccess) e = run_step(c, in.arg, lr);
          if (e != hipSuccess) {
            abort_capture();
            char buf[96];
            snprintf(buf, sizeof buf, "step %d (%s), while capturing", in.arg, step_kind_name(g.steps[in.arg].kind));
            return c->hipfail(e, buf);
          }
          break;
        }
        if (in.wait_d2h >= 0) HIPCHK(c, hipStreamWaitEvent(c->s_c, c->ev_d2h[in.wait_d2h], 0));
        if (in.wait_h2d >= 0) HIPCHK(c, hipStreamWaitEvent(c->s_c, c->ev_h2d[in.wait_h2d], 0));
        if (c->profiling) HIPCHK(c, hipEventRecord(c->prof_a[in.arg], c->s_c));
        // weight gradients that went to their own stream and must be complete before this step
        // (their operands may be released after it; the update reads their results)
        for (int jw : g.steps[in.arg].joins)
          if (c->s_w && c->wgrad_in_flight[jw]) {
            HIPCHK(c, hipStreamWaitEvent(c->s_c, c->ev_wdone[jw], 0));
            c->wgrad_in_flight[jw] = 0;
          }
        hipError_t e = run_step(c, in.arg, lr);
        if (e != hipSuccess) {
          char buf[96];
          snprintf(buf, sizeof buf, "step %d (%s)", in.arg, step_kind_name(g.steps[in.arg].kind));
          (void)hipStreamSynchronize(c->s_c); (void)hipStreamSynchronize(c->s_o); (void)hipStreamSynchronize(c->s_i);
          if (c->s_w) (void)hipStreamSynchronize(c->s_w);
          return c->hipfail(e, buf);
        }
        if (c->profiling) HIPCHK(c, hipEventRecord(c->prof_b[in.arg], c->s_c));
        if (in.arg < (int)c->capture_at.size())
          for (const acc_ctx::Capture& cp : c->capture_at[in.arg])
            HIPCHK(c, hipMemcpyAsync(cp.dst, c->dyn + c->cur_off[cp.tensor], (size_t)P.k * g.tensors[cp.tensor].bytes_per_image,
                                     hipMemcpyDeviceToHost, c->s_c));
        if (in.arg < (int)c->inject_at.size())
          for (const acc_ctx::Capture& ip : c->inject_at[in.arg])
            HIPCHK(c, hipMemcpyAsync(c->dyn + c->cur_off[ip.tensor], ip.dst, (size_t)P.k * g.tensors[ip.tensor].bytes_per_image,
                                     hipMemcpyHostToDevice, c->s_c));
        if (poison)
          for (const acc_ctx::Block& b : c->poison_after_step[in.arg]) {
            const hipError_t ep = fill_words(c->dyn + b.off, b.bytes, kReleased, c->s_c);
            if (ep != hipSuccess) return c->hipfail(ep, "poison fill");
          }
        if (in.record) HIPCHK(c, hipEventRecord(c->ev_step[in.arg], c->s_c));
        if (++n_compute % kStepWindow == 0) HIPCHK(c, hipEventRecord(c->ev_window[n_compute / kStepWindow - 1], c->s_c));
        break;
      }
      case I_OFFLOAD: {
        HIPCHK(c, hipStreamWaitEvent(c->s_o, c->ev_step[in.wait_step], 0));
        if (c->profiling) HIPCHK(c, hipEventRecord(c->prof_copy_a[in.seq], c->s_o));
        HIPCHK(c, hipMemcpyAsync((char*)c->res.host + P.host_off[in.arg], c->dyn + P.off1[in.arg], P.tbytes[in.arg],
                                 hipMemcpyDeviceToHost, c->s_o));
        if (c->profiling) HIPCHK(c, hipEventRecord(c->prof_copy_b[in.seq], c->s_o));
        if (poison) {
          const acc_ctx::Block& b = c->poison_after_d2h[in.seq];
          const hipError_t ep = fill_words(c->dyn + b.off, b.bytes, kReleased, c->s_o);
          if (ep != hipSuccess) return c->hipfail(ep, "poison fill");
        }
        HIPCHK(c, hipEventRecord(c->ev_d2h[in.seq], c->s_o));
        bytes_out += P.tbytes[in.arg];
        break;
      }
      case I_PREFETCH: {
        if (in.wait_step >= 0) HIPCHK(c, hipStreamWaitEvent(c->s_i, c->ev_step[in.wait_step], 0));
        if (in.wait_d2h >= 0) HIPCHK(c, hipStreamWaitEvent(c->s_i, c->ev_d2h[in.wait_d2h], 0));
        if (c->profiling) HIPCHK(c, hipEventRecord(c->prof_copy_a[P.n_d2h + in.seq], c->s_i));
        HIPCHK(c, hipMemcpyAsync(c->dyn + P.off2[in.arg], (char*)c->res.host + P.host_off[in.arg], P.tbytes[in.arg],
                                 hipMemcpyHostToDevice, c->s_i));
        if (c->profiling) HIPCHK(c, hipEventRecord(c->prof_copy_b[P.n_d2h + in.seq], c->s_i));
        HIPCHK(c, hipEventRecord(c->ev_h2d[in.seq], c->s_i));
        c->cur_off[in.arg] = P.off2[in.arg];
        bytes_in += P.tbytes[in.arg];
        break;
      }
    }
  }
  if (graph_mode && graph_started) {
    if (c->capturing) {
      // every weight gradient was joined by the last step; close, instantiate and run the recording
      hipError_t e = hipStreamEndCapture(c->s_c, &c->graph);
      c->capturing = false;
      if (e == hipSuccess) e = hipGraphInstantiate(&c->graph_exec, c->graph, nullptr, nullptr, 0);
      if (e != hipSuccess) {
        c->drop_graph();
        (void)hipGetLastError();
        return c->hipfail(e, "graph capture");
      }
      HIPCHK(c, hipGraphLaunch(c->graph_exec, c->s_c));
    }
    const hipError_t eu = sgd_update(c->d_params, c->d_grads, lr, g.param_elems, c->d_params16, c->s_c);
    if (eu != hipSuccess) return c->hipfail(eu, "sgd_update");
  }
  HIPCHK(c, hipMemcpyAsync(c->h_loss, c->d_loss, sizeof(float), hipMemcpyDeviceToHost, c->s_c));
  HIPCHK(c, hipEventRecord(c->ev_end, c->s_c));
  const double t_issued = now_ms();
  HIPCHK(c, hipStreamSynchronize(c->s_c));
  HIPCHK(c, hipStreamSynchronize(c->s_o));
  HIPCHK(c, hipStreamSynchronize(c->s_i));
  if (c->s_w) HIPCHK(c, hipStreamSynchronize(c->s_w));
  const double t_done = now_ms();
  if (loss_out) *loss_out = *c->h_loss;
  c->stats.step_ms = t_done - t_host0;
  c->stats.host_issue_ms = t_issued - t_host0;
  c->stats.host_wait_ms = t_waited;
  // without the poison mode: where the plan's highest block ends (an offset, not a sum of sizes)
  c->stats.peak_pool_bytes = g.static_bytes() + P.dyn_top;
  c->stats.touched_pool_bytes = 0;
  c->stats.peak_is_measured = 0;
  if (poison) {
    // the highest byte of the pool that anything wrote during the iteration, and how many bytes
    // were written at all: every word that no longer holds the pattern of before the iteration
    hipLaunchKernelGGL(written_extent_kernel, dim3(256 * 8), dim3(256), 0, c->s_c, (const uint32_t*)c->dyn,
                       c->dyn_cap / 4, kNeverWritten, d_scan);
    HIPCHK(c, hipGetLastError());
    unsigned long long* h_scan = (unsigned long long*)((char*)c->h_loss + 16);
    HIPCHK(c, hipMemcpyAsync(h_scan, d_scan, 16, hipMemcpyDeviceToHost, c->s_c));
    HIPCHK(c, hipStreamSynchronize(c->s_c));
    c->stats.peak_pool_bytes = g.static_bytes() + (uint64_t)h_scan[0] * 4;
    c->stats.touched_pool_bytes = g.static_bytes() + (uint64_t)h_scan[1] * 4;
    c->stats.peak_is_measured = 1;
    if (c->stats.peak_pool_bytes > P.budget)
      return c->fail(ACC_EPOOL, "the iteration wrote beyond the budget (found by the poison scan)");
  }
  c->stats.bytes_out = bytes_out;
  c->stats.bytes_in = bytes_in;
  c->stats.steps_run += 1;
  c->stats.d2h_ms = c->stats.h2d_ms = 0;
  if (c->kernel_profiling) {
    for (int v = 0; v < V_COUNT; ++v) { c->k_ms[v] = 0; c->k_flops[v] = 0; c->k_launches[v] = 0; }
    float gaps[9];
    for (int i = 0; i < 9; ++i) HIPCHK(c, hipEventElapsedTime(&gaps[i], c->empty_pair[2 * i], c->empty_pair[2 * i + 1]));
    std::sort(gaps, gaps + 9);
    c->probe_overhead_ms = gaps[4];
    for (size_t i = 0; i < c->kprobes_used; ++i) {
      acc_ctx::KProbe& kp = c->kprobes[i];
      if (kp.variant < 0 || kp.variant >= V_COUNT) continue;
      float ms = 0;
      HIPCHK(c, hipEventElapsedTime(&ms, kp.a, kp.b));
      kp.ms = std::max(0.0, (double)ms - c->probe_overhead_ms);
      c->k_ms[kp.variant] += kp.ms;
      c->k_flops[kp.variant] += kp.flops;
      c->k_launches[kp.variant] += 1;
    }
  }
  if (c->profiling) {
    c->step_ms.assign(ns, 0.0);
    for (int j = 0; j < ns; ++j) {
      float ms = 0;
      HIPCHK(c, hipEventElapsedTime(&ms, c->prof_a[j], c->prof_b[j]));
      c->step_ms[j] = ms;
    }
    for (const Instr& in : P.instrs) {
      if (in.op != I_OFFLOAD && in.op != I_PREFETCH) continue;
      const size_t idx = in.op == I_OFFLOAD ? (size_t)in.seq : (size_t)P.n_d2h + in.seq;
      float ms = 0;
      HIPCHK(c, hipEventElapsedTime(&ms, c->prof_copy_a[idx], c->prof_copy_b[idx]));
      (in.op == I_OFFLOAD ? c->stats.d2h_ms : c->stats.h2d_ms) += ms;
    }
    // observed timeline: every timed instruction against the first event of the iteration
    c->obs_start.assign(P.instrs.size(), -1.0);
    c->obs_end.assign(P.instrs.size(), -1.0);
    for (size_t i = 0; i < P.instrs.size(); ++i) {
      const Instr& in = P.instrs[i];
      hipEvent_t a = nullptr, b = nullptr;
      if (in.op == I_COMPUTE) { a = c->prof_a[in.arg]; b = c->prof_b[in.arg]; }
      else if (in.op == I_OFFLOAD) { a = c->prof_copy_a[in.seq]; b = c->prof_copy_b[in.seq]; }
      else if (in.op == I_PREFETCH) { a = c->prof_copy_a[P.n_d2h + in.seq]; b = c->prof_copy_b[P.n_d2h + in.seq]; }
      if (!a) continue;
      float ms0 = 0, ms1 = 0;
      HIPCHK(c, hipEventElapsedTime(&ms0, c->ev_begin, a));
      HIPCHK(c, hipEventElapsedTime(&ms1, c->ev_begin, b));
      c->obs_start[i] = ms0 * 1e-3;
      c->obs_end[i] = ms1 * 1e-3;
    }
  }
  return ACC_OK;
}

extern "C" int acc_get_timeline(acc_ctx* c, int which, acc_timeline_entry* out, int max_entries) {
  if (!c || !out || (which != 0 && which != 1)) return ACC_EINVAL;
  const Plan& P = c->plan;
  if (!P.valid) return c->fail(ACC_ESTATE, "call acc_plan_swaps first");
  const size_t n = P.instrs.size();
  if ((size_t)(max_entries < 0 ? 0 : max_entries) < n) return c->fail(ACC_EINVAL, "max_entries is smaller than the instruction count");
  const std::vector<double>& t0 = which == 0 ? P.i_start : c->obs_start;
  const std::vector<double>& t1 = which == 0 ? P.i_end : c->obs_end;
  if (t0.size() != n || t1.size() != n)
    return c->fail(ACC_ESTATE, which == 0 ? "the plan has not been simulated" : "no profiled step of this plan yet");
  for (size_t i = 0; i < n; ++i) {
    const Instr& in = P.instrs[i];
    out[i].op = in.op; out[i].arg = in.arg;
    out[i].bytes = in.op == I_COMPUTE ? 0 : P.tbytes[in.arg];
    out[i].t_start = t0[i]; out[i].t_end = t1[i];
  }
  return (int)n;
}

extern "C" int acc_get_stats(acc_ctx* c, acc_stats* out) {
  if (!c || !out) return ACC_EINVAL;
  *out = c->stats;
  return ACC_OK;
}

extern "C" int acc_set_debug(acc_ctx* c, int flags) {
  if (!c) return ACC_EINVAL;
  if (flags & ~ACC_DEBUG_POISON) return c->fail(ACC_EINVAL, "unknown debug flag");
  if (flags && !c->have_res) return c->fail(ACC_ESTATE, "context has no device resources");
  c->debug_flags = flags;
  return ACC_OK;
}

namespace {
int register_hook(acc_ctx* c, std::vector<std::vector<acc_ctx::Capture>>* table, int layer, void* host, size_t bytes) {
  if (!c) return ACC_EINVAL;
  if (!c->have_res) return c->fail(ACC_ESTATE, "context has no device resources");
  const int ns = (int)c->g.steps.size();
  if (layer == -1 && !host) { table->clear(); return ACC_OK; }
  if (layer < 0 || layer >= (int)c->g.layers.size()) return c->fail(ACC_EINVAL, "bad layer");
  const int t = c->g.act_of_layer[layer];
  if (t < 0) return c->fail(ACC_EINVAL, "the output of this layer is not stored (fused into the next layer's step)");
  const int j = c->g.tensors[t].producer;
  if (j < 0 || j >= c->g.n_fwd) return c->fail(ACC_EINVAL, "the output of this layer has no forward step");
  if ((int)table->size() != ns) table->assign(ns, {});
  auto& list = (*table)[j];
  list.erase(std::remove_if(list.begin(), list.end(), [&](const acc_ctx::Capture& cp) { return cp.tensor == t; }), list.end());
  if (host) list.push_back({t, host, bytes});
  return ACC_OK;
}
}  // namespace

extern "C" int acc_capture_output(acc_ctx* c, int layer, void* host_dst, size_t bytes) {
  return register_hook(c, c ? &c->capture_at : nullptr, layer, host_dst, bytes);
}

extern "C" int acc_inject_output(acc_ctx* c, int layer, const void* host_src, size_t bytes) {
  return register_hook(c, c ? &c->inject_at : nullptr, layer, const_cast<void*>(host_src), bytes);
}

extern "C" int acc_set_wgrad_overlap(acc_ctx* c, int on) {
  if (!c) return ACC_EINVAL;
  if (c->wgrad_overlap != (on != 0)) c->drop_graph();   // the recording holds the streams' fork and join
  c->wgrad_overlap = on != 0;
  return ACC_OK;
}

extern "C" int acc_set_graph(acc_ctx* c, int on) {
  if (!c) return ACC_EINVAL;
  if (on && !c->have_res) return c->fail(ACC_ESTATE, "context has no device resources");
  c->use_graph = on != 0;
  if (!on) c->drop_graph();
  return ACC_OK;
}

extern "C" int acc_set_profiling(acc_ctx* c, int level) {
  if (!c) return ACC_EINVAL;
  c->profiling = level == 1 || level == 3;
  c->kernel_profiling = level == 2 || level == 3;
  return ACC_OK;
}

extern "C" int acc_get_kernel_profile(acc_ctx* c, acc_kernel_profile* out, int max_entries) {
  if (!c || !out || max_entries < 0) return ACC_EINVAL;
  int n = 0;
  for (int v = 0; v < V_COUNT && n < max_entries; ++v) {
    if (!c->k_launches[v]) continue;
    std::memset(&out[n], 0, sizeof out[n]);
    snprintf(out[n].name, sizeof out[n].name, "%s", conv_variant_name(v));
    out[n].launches = (int32_t)c->k_launches[v];
    out[n].ms = c->k_ms[v];
    out[n].flops = c->k_flops[v];
    ++n;
  }
  return n;
}

extern "C" int acc_get_launch_profile(acc_ctx* c, acc_launch_profile* out, int max_entries) {
  if (!c || max_entries < 0 || (!out && max_entries > 0)) return ACC_EINVAL;
  int n = 0;
  for (size_t i = 0; i < c->kprobes_used; ++i) {
    const acc_ctx::KProbe& kp = c->kprobes[i];
    if (kp.variant < 0 || kp.variant >= V_COUNT) continue;
    if (n < max_entries) {
      out[n].step = kp.step;
      out[n].layer = kp.step >= 0 ? c->g.steps[kp.step].layer : -1;
      out[n].role = kp.role;
      out[n].variant = kp.variant;
      out[n].ms = kp.ms;
      out[n].flops = kp.flops;
    }
    ++n;
  }
  return n;
}

extern "C" int acc_get_step_times_ms(acc_ctx* c, double* ms, int n) {
  if (!c || !ms) return ACC_EINVAL;
  if (n != (int)c->g.steps.size() || c->step_ms.size() != (size_t)n) return c->fail(ACC_ESTATE, "no profiled step yet");
  std::copy(c->step_ms.begin(), c->step_ms.end(), ms);
  return ACC_OK;
}

// ------------------------------------------------------------------------- calibration
namespace {

__global__ void pseudo_input_kernel(float* p, size_t count) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (size_t)gridDim.x * blockDim.x) {
    uint32_t h = (uint32_t)i * 2654435761u;
    h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
    p[i] = (float)(int32_t)h * (1.0f / 2147483648.0f);   // in [-1, 1)
  }
}

hipError_t fill_pseudo_input(acc_ctx* c, float* p, size_t count) {
  hipLaunchKernelGGL(pseudo_input_kernel, dim3(2048), dim3(256), 0, c->s_i, p, count);
  return hipGetLastError();
}

}  // namespace

extern "C" int acc_calibrate(acc_ctx* c, const int* ks, int nk) {
  if (!c) return ACC_EINVAL;
  if (!c->have_res) return c->fail(ACC_ESTATE, "context has no device resources");
  if (!ks || nk <= 0) return c->fail(ACC_EINVAL, "need at least one minibatch size");
  std::vector<int> kk(ks, ks + nk);
  std::sort(kk.begin(), kk.end());
  kk.erase(std::unique(kk.begin(), kk.end()), kk.end());
  if (kk[0] <= 0) return c->fail(ACC_EINVAL, "minibatch must be positive");
  const int ns = (int)c->g.steps.size();

  // dynamic information 2: transfer rates on the side streams (Eq. 5's Bandwidth_avail)
  {
    size_t big = std::min<size_t>((size_t)256 << 20, std::min(c->dyn_cap, c->res.host_bytes));
    big &= ~(size_t)255;
    const size_t small = std::min<size_t>((size_t)1 << 20, big);
    if (big >= ((size_t)8 << 20)) {
      hipEvent_t a, b;
      HIPCHK(c, hipEventCreate(&a));
      HIPCHK(c, hipEventCreate(&b));
      double t[2][2];
      for (int dir = 0; dir < 2; ++dir) {
        hipStream_t st = dir == 0 ? c->s_o : c->s_i;
        for (int sz = 0; sz < 2; ++sz) {
          const size_t bytes = sz == 0 ? small : big;
          float best = 1e30f;
          for (int rep = 0; rep < 3; ++rep) {
            HIPCHK(c, hipEventRecord(a, st));
            if (dir == 0) HIPCHK(c, hipMemcpyAsync(c->res.host, c->dyn, bytes, hipMemcpyDeviceToHost, st));
            else HIPCHK(c, hipMemcpyAsync(c->dyn, c->res.host, bytes, hipMemcpyHostToDevice, st));
            HIPCHK(c, hipEventRecord(b, st));
            HIPCHK(c, hipStreamSynchronize(st));
            float ms = 0;
            HIPCHK(c, hipEventElapsedTime(&ms, a, b));
            best = std::min(best, ms);
          }
          t[dir][sz] = best * 1e-3;
        }
      }
      (void)hipEventDestroy(a);
      (void)hipEventDestroy(b);
      const double bw_o = (double)(big - small) / std::max(1e-9, t[0][1] - t[0][0]);
      const double bw_i = (double)(big - small) / std::max(1e-9, t[1][1] - t[1][0]);
      c->cm.d2h_bps = bw_o;
      c->cm.h2d_bps = bw_i;
      const double lat = 0.5 * ((t[0][0] - small / bw_o) + (t[1][0] - small / bw_i));
      c->cm.copy_latency_s = std::max(0.0, lat);
    }
  }

  // dynamic information 1: per-step compute time, taken from real iterations at every
  // requested minibatch that trains in this pool without swapping.  A larger minibatch is
  // not run here: its step times follow from the largest measured one in proportion to
  // the minibatch (Eq. 1; throughput has saturated by then, Sec. 3.3.1), so if any request
  // is too large the largest minibatch that does fit is measured as well.
  const bool was_prof = c->profiling;
  std::vector<int> ok_ks;
  std::vector<std::vector<double>> table;
  c->cm.fixed.clear();
  auto fits = [&](int k) {
    Plan p;
    std::string why;
    return make_plan(c->g, c->cm, k, c->res.pool_bytes, ACC_PLAN_NONE, &p, &why) == ACC_OK;
  };
  std::vector<int> run_ks;
  bool some_too_large = false;
  for (int k : kk) {
    if (fits(k)) run_ks.push_back(k);
    else some_too_large = true;
  }
  if (some_too_large && fits(1)) {
    int lo = 1, hi = kk.back();
    while (lo < hi) {
      const int mid = lo + (hi - lo + 1) / 2;
      if (fits(mid)) lo = mid; else hi = mid - 1;
    }
    run_ks.push_back(lo);
    std::sort(run_ks.begin(), run_ks.end());
    run_ks.erase(std::unique(run_ks.begin(), run_ks.end()), run_ks.end());
  }
  for (int k : run_ks) {
    Plan p;
    std::string why;
    int rc = make_plan(c->g, c->cm, k, c->res.pool_bytes, ACC_PLAN_NONE, &p, &why);
    if (rc != ACC_OK) continue;
    rc = install_plan(c, std::move(p), nullptr, now_ms());
    if (rc != ACC_OK) return rc;
    c->calibrating = true;
    c->profiling = true;
    std::vector<double> best(ns, 1e30);
    int rc2 = ACC_OK;
    for (int it = 0; it < 3 && rc2 == ACC_OK; ++it) {
      float loss;
      rc2 = acc_train_step(c, nullptr, ACC_LOC_DEVICE, nullptr, 0.0f, &loss);
      if (rc2 == ACC_OK && it > 0)
        for (int j = 0; j < ns; ++j) best[j] = std::min(best[j], c->step_ms[j] * 1e-3);
    }
    c->calibrating = false;
    c->profiling = was_prof;
    if (rc2 != ACC_OK) return rc2;
    ok_ks.push_back(k);
    table.push_back(best);
  }
  c->plan.valid = false;
  if (ok_ks.empty()) return c->fail(ACC_EPOOL, "not even one image trains in this pool without swapping");
  c->cm.ks = ok_ks;
  c->cm.table = table;
  return ACC_OK;
}
