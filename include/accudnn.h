/*
 * accudnn.h - C ABI of the MI355X-native training-step library.
 *
 * One context trains one network on one GPU under a device-memory budget.  That is
 * the problem of Sec. 2 (overall architecture): a network, a machine and a memory
 * budget come in; a swapping strategy and a minibatch come out and are then executed.
 * The layer list is unfolded into 2N steps (Sec. 3.1), feature maps are the swap
 * targets, and the runtime knows four operations: allocate, release, offload,
 * prefetch (Sec. 3.1, Sec. 5).
 *
 * Conventions
 *  - Every function returns ACC_OK (0) or a negative acc_status; nothing throws
 *    or aborts.  acc_last_error() gives the text of the last failure of a context.
 *  - "host" pointers are ordinary or pinned host memory, "device" pointers are
 *    HIP device memory.  The caller owns every buffer it passes in and keeps the
 *    pool, the host arena and the streams alive until acc_destroy().
 *  - The library calls no hipMalloc: all device data (weights, gradients, feature
 *    maps, workspace, the input batch) lives inside the caller's pool, so the
 *    budget is a hard cap by construction (Sec. 5: one buffer pool of the size of
 *    the budget, sub-allocated at run time).
 *  - Activations are NHWC fp32 on the device, filters O-H-W-I; the host-side
 *    weight interface uses the framework-neutral OIHW order and converts.
 *  - One context per thread; calls on one context must not overlap.
 */
#ifndef ACCUDNN_H
#define ACCUDNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  ACC_OK = 0,
  ACC_EINVAL = -1,       /* malformed argument or unsupported network topology        */
  ACC_EUNTRAINABLE = -2, /* budget below the layer-wise peak: k > k_max (Algorithm 2) */
  ACC_EPOOL = -3,        /* pool smaller than budget / static data do not fit         */
  ACC_EHOSTMEM = -4,     /* pinned host arena too small for the swapped maps          */
  ACC_EHIP = -5,         /* a HIP call failed; text in acc_last_error()               */
  ACC_ESTATE = -6        /* call out of order (e.g. train_step before plan_swaps)     */
} acc_status;

/* layer kinds of a network record */
enum { ACC_CONV = 0, ACC_BN = 1, ACC_RELU = 2, ACC_ADD = 3, ACC_MAXPOOL = 4, ACC_GAP = 5,
       ACC_FC = 6, ACC_SOFTMAX_CE = 7, ACC_BIAS = 8 };
enum { ACC_F32 = 0, ACC_BF16 = 1 };
/* planner modes: keep everything / swap every feature map (the "naive" strategy of
 * Sec. 3.1) / performance-model-guided choice (the "dynamic" strategy, Sec. 3.1, 3.4, 4.1) */
enum { ACC_PLAN_NONE = 0, ACC_PLAN_NAIVE_ALL = 1, ACC_PLAN_DYNAMIC = 2 };
enum { ACC_LOC_HOST = 0, ACC_LOC_DEVICE = 1 };

/* One layer, in execution order.  in0/in1: index of the producing layer, -1 = the
 * network input.  conv: cin,cout,r,s,stride,pad (no bias).  bias: cin channels, one
 * parameter each, added per channel.  bn: cin channels, parameters [gamma|beta], eps 1e-5,
 * minibatch statistics.  maxpool: r,s,stride,pad.  fc: cin,cout, parameters
 * [W cout x cin | b cout]; cin = all elements of the input map of one image (a map larger
 * than 1x1 is flattened in c, h, w order, as OIHW filters are).  softmax_ce: in0 = logits.
 * Element-wise layers are executed fused into the step of their producer, so they must
 * appear in one of these patterns (acc_create returns ACC_EINVAL otherwise):
 * bn -> relu, bn -> add -> relu, conv -> bias [-> relu], fc -> relu. */
typedef struct {
  int32_t kind, in0, in1, cin, cout, r, s, stride, pad;
} acc_layer;

/* Device pool, pinned host arena and the three streams of Sec. 5 (compute,
 * swap-out, swap-in; hipStream_t passed as void*).  With a NULL acc_resources the
 * context is planning-only: everything but calibrate / train_step / weights works.
 * s_wgrad (may be NULL) is a fourth stream, different from the other three: the weight
 * gradient of a convolution then runs there, beside the data gradient and the steps that
 * follow on the compute stream, and is joined two convolutions later; results are the same
 * bit for bit.  All streams at the default priority. */
typedef struct {
  void* pool;        /* device */
  size_t pool_bytes;
  void* host;        /* pinned host */
  size_t host_bytes;
  void* s_compute;
  void* s_out;
  void* s_in;
  void* s_wgrad;
} acc_resources;

typedef struct {
  int32_t n_steps;          /* 2N (+1 for the weight update)                              */
  int32_t n_maps;           /* feature maps that live from forward into backward          */
  int32_t n_swapped;        /* of those, how many are offloaded and prefetched            */
  int32_t n_instr;          /* length of the instruction list the executor runs           */
  uint64_t bytes_swapped;   /* per direction, per step                                    */
  uint64_t bytes_maps;      /* retention set at this minibatch                            */
  uint64_t static_bytes;    /* weights, gradients, saved statistics, scratch              */
  uint64_t peak_bytes;      /* predicted pool high-water mark, static part included       */
  uint64_t layer_peak_bytes;/* M_peak(k): high-water mark with every map swapped          */
  uint64_t noswap_peak_bytes;/* high-water mark with no map swapped                       */
  uint64_t host_bytes;      /* pinned host bytes the plan uses                            */
  double t_compute;         /* Eq. 2: sum of per-step compute times, seconds              */
  double t_iter;            /* predicted iteration time with stalls, seconds              */
  double t_stall;           /* predicted total stall, seconds                             */
  double plan_ms;           /* wall time spent planning                                   */
} acc_plan_summary;

typedef struct {
  int32_t kind;             /* internal step kind (see acc_step_kind_name)                */
  int32_t layer;            /* layer record this step belongs to                          */
  int32_t backward;         /* 0 forward, 1 backward, 2 update                            */
  int32_t reserved;
  double flops;             /* at the planned minibatch (Eq. 1: linear in k)              */
  double t_compute;         /* cost-model time, seconds                                   */
  double t_ready;           /* Algorithm 1: data on the GPU and memory allocated          */
  double t_start, t_end;    /* simulated execution on the compute stream                  */
} acc_step_info;

typedef struct {
  int32_t kind;             /* 0 activation, 1 gradient, 2 workspace, 3 input staging     */
  int32_t producer_step, last_fwd_step, first_bwd_step, last_step;
  int32_t is_map;           /* lives from forward into backward (swappable)               */
  int32_t swapped;
  int32_t reserved;
  uint64_t bytes;           /* at the planned minibatch                                   */
  uint64_t offset;          /* pool offset of the (first) allocation                      */
  uint64_t offset2;         /* pool offset after prefetch, if swapped                     */
  uint64_t host_offset;     /* slot in the pinned arena, if swapped                       */
} acc_tensor_info;

typedef struct {
  double step_ms;           /* last train_step: host clock, entry to completion           */
  double host_issue_ms;     /* last train_step: host time from entry until all work is issued,
                               host_wait_ms included                                     */
  uint64_t peak_pool_bytes; /* pool offset where the highest byte in use ends, static part
                               included.  With ACC_DEBUG_POISON: measured (the highest word
                               that anything wrote during the iteration); otherwise the end
                               of the highest block of the plan                           */
  uint64_t bytes_out, bytes_in; /* offloaded / prefetched in the last step                */
  double d2h_ms, h2d_ms;    /* summed copy durations (only when profiling is enabled)     */
  uint64_t steps_run;
  uint64_t touched_pool_bytes; /* ACC_DEBUG_POISON: bytes of the pool written at least once
                               during the iteration, static part included; else 0         */
  int32_t peak_is_measured; /* 1 if peak_pool_bytes comes from the poison scan            */
  int32_t reserved;
  double host_wait_ms;      /* of host_issue_ms: time the host stood still because it was a full
                               window of steps or copies ahead of the GPU (it issues no further
                               ahead than that); host_issue_ms - host_wait_ms is what issuing
                               the iteration costs the host                               */
} acc_stats;

typedef struct acc_ctx acc_ctx;

/* ---- context ---------------------------------------------------------------------- */
/* Builds the fused step list and the tensor table (static information of Sec. 3.2).
 * With resources: places weights / gradients / statistics at the bottom of the pool.
 * dtype: ACC_F32, or ACC_BF16 = activations, activation gradients and the copy of the
 * weights that the kernels read are stored as bf16 (half the bytes to keep and to swap),
 * products accumulate in fp32, master weights, weight gradients, batch-norm parameters and
 * statistics and the loss stay fp32; images and weights cross the boundary as fp32 either way. */
int acc_create(const acc_layer* layers, int n_layers, int in_c, int in_h, int in_w, int dtype,
               const acc_resources* res, acc_ctx** out);
void acc_destroy(acc_ctx* ctx);
const char* acc_last_error(const acc_ctx* ctx);   /* ctx may be NULL: this thread's last error of acc_create or of a call without a context */
const char* acc_step_kind_name(int kind);

/* Parameters and their gradients are the memory objects that never leave the GPU (Sec. 3.1:
 * feature maps are the swap targets; M_para of Algorithm 2).  fp32 master weights of one
 * layer, host side, OIHW / [gamma|beta] / [W|b]; n = element count and must match.
 * Blocking.  get_grads returns d(loss)/d(weights) of the last step (a parity hook: the
 * abstract's claim that swapping costs no accuracy is checked on these, bit for bit). */
int acc_set_weights(acc_ctx* ctx, int layer, const float* host_w, size_t n);
int acc_get_weights(acc_ctx* ctx, int layer, float* host_w, size_t n);
int acc_get_grads(acc_ctx* ctx, int layer, float* host_g, size_t n);
int acc_param_count(const acc_ctx* ctx, int layer, size_t* n);

/* ---- cost model (dynamic information, Sec. 3.2; Eq. 2 and Eq. 5) ------------------- */
/* Measures the link (D2H / H2D copies of two sizes on the side streams) and every step's
 * kernels (events on the compute stream, three iterations on a synthetic batch, weights
 * untouched) at each minibatch of ks[] that trains in the pool without swapping.  If some
 * of ks[] are too large for that, the largest minibatch that does fit is measured too and
 * the planner scales its times in proportion (Eq. 1, Sec. 3.3.1).  Needs resources;
 * ACC_EPOOL if not even one image fits. */
int acc_calibrate(acc_ctx* ctx, const int* ks, int nk);
/* Synthetic cost model for planning without a GPU: step time = launch_s + flops /
 * flops_per_s + bytes / bytes_per_s (flops for conv/fc steps, touched bytes for the
 * rest); copies run at d2h / h2d bytes per second plus copy_latency_s each. */
int acc_set_cost_model(acc_ctx* ctx, double flops_per_s, double bytes_per_s, double launch_s,
                       double d2h_bytes_per_s, double h2d_bytes_per_s, double copy_latency_s);
/* Overrides the cost of single steps (seconds, at the minibatch given to the next
 * plan_swaps); n must equal the step count.  Used to test Algorithm 1 on hand-built cases. */
int acc_set_step_times(acc_ctx* ctx, const double* seconds, int n);
/* Reads back / installs the measured table of acc_calibrate, so that a calibration can be
 * kept and a planning-only context can plan with it: ks[nk] ascending minibatches,
 * seconds[nk][n_steps] row-major, link[3] = D2H bytes/s, H2D bytes/s, latency per copy (s).
 * get: returns nk (0 if nothing was measured) or ACC_EINVAL if max_k / max_seconds are too
 * small; any output pointer may be null.  Between two measured minibatches the planner
 * interpolates linearly in k; beyond the largest it scales in proportion (Sec. 3.3.1:
 * throughput saturates), below the smallest it scales down to no less than the launch cost. */
int acc_get_calibration(const acc_ctx* ctx, int* ks, int max_k, double* seconds, size_t max_seconds,
                        double* link);
int acc_set_calibration(acc_ctx* ctx, const int* ks, int nk, const double* seconds, const double* link);

/* ---- planning (Algorithm 1, Eq. 4-6, body of Algorithm 2) ------------------------- */
int acc_plan_swaps(acc_ctx* ctx, int minibatch, size_t budget_bytes, int mode,
                   acc_plan_summary* out);
/* ---- efficiency-optimal minibatch (Sec. 4.1: Eq. 7, Algorithm 2; Sec. 4.2: Eq. 9) --- */
typedef struct {
  int32_t k_best;           /* minibatch with the highest predicted images/s              */
  int32_t k_trainable_max;  /* k_max: largest minibatch in [k_lo, k_hi] that trains at all  */
  int32_t k_noswap_max;     /* largest minibatch in range that needs no swap (0 if none)   */
  int32_t n_evaluated;      /* minibatches that were planned and timed by the model       */
  double images_per_s;      /* k_best / t_iter(k_best), predicted                         */
  double t_iter;            /* predicted iteration time at k_best, seconds                */
  double t_stall;           /* predicted stall at k_best, seconds                         */
  double tune_ms;           /* wall time of the search                                    */
} acc_tune_result;
/* Minimises the predicted time per image, t_iter(k) / k (Eq. 3 for one GPU), over the
 * minibatches of [k_lo, k_hi] that train under the budget (Eq. 4), each with its own swap
 * plan, and installs the plan of the winner (as acc_plan_swaps(k_best, DYNAMIC) would).
 * Algorithm 2 walks down from k_max and stops at the first minibatch without a stall
 * (Eq. 6); that is the optimum when throughput only grows with k.  Here the measured
 * step times decide instead (on this GPU tile quantisation makes throughput uneven in
 * k), and a plan with stalls is admitted at its predicted time.  Every minibatch that
 * needs no swap is evaluated; above that, where one plan costs ~0.1 s, a geometric grid
 * (ratio 1.15) up to k_max.  Ties go to the larger minibatch.
 * ACC_EUNTRAINABLE if not even k_lo trains under the budget. */
int acc_tune_minibatch(acc_ctx* ctx, size_t budget_bytes, int k_lo, int k_hi, acc_tune_result* out,
                       acc_plan_summary* plan_out);
/* Eq. 9: the learning rate that keeps the convergence rate when the minibatch grows by
 * the factor q = k_best / k_base: (1 - (1 - lr_base * c)^q) / c, c = convexity constant
 * of the objective (0 < lr_base * c < 1).  Returns NaN for arguments outside that range. */
double acc_adaptive_lr(double lr_base, double c, double q);

/* Plans with an explicit swap decision per map (maps in producer order; 1 = swap). */
int acc_plan_explicit(acc_ctx* ctx, int minibatch, size_t budget_bytes, const uint8_t* swap,
                      int n_maps, acc_plan_summary* out);
int acc_get_step_count(const acc_ctx* ctx);
int acc_get_tensor_count(const acc_ctx* ctx);
int acc_get_step_info(const acc_ctx* ctx, int step, acc_step_info* out);
int acc_get_tensor_info(const acc_ctx* ctx, int tensor, acc_tensor_info* out);
/* tensors a step reads / writes (ids into the tensor table); returns the count or <0 */
int acc_get_step_io(const acc_ctx* ctx, int step, int32_t* reads, int max_reads, int32_t* writes,
                    int max_writes);

/* The instruction list of the current plan, in issue order.  op: 0 load input (swap-in
 * stream), 1 compute step (compute stream), 2 offload (swap-out stream), 3 prefetch
 * (swap-in stream).  arg: tensor id, or step index for op 1.  wait_*: the instruction first
 * waits for the event recorded after that compute step / after the offload resp. prefetch
 * (or input load) with that sequence number; -1 = none.  seq: own sequence number among
 * offloads resp. among prefetches and input loads.  record: op 1 records its step event. */
typedef struct {
  int32_t op, arg, wait_step, wait_d2h, wait_h2d, seq, record, reserved;
} acc_instr;
int acc_get_instr_count(const acc_ctx* ctx);
int acc_get_instr(const acc_ctx* ctx, int index, acc_instr* out);

/* One entry per instruction of the current plan, in issue order: when it runs on its own
 * stream, in seconds after the start of the iteration.  which = 0: as Algorithm 1's
 * simulation predicts with the current cost model; which = 1: as observed in the last
 * train_step that ran with profiling level 1 or 3 (events around every step and copy, read
 * against the first event of the iteration on the compute stream; input loads are not timed
 * and report -1 / -1).  Returns the number of entries, ACC_EINVAL if max_entries is too small,
 * ACC_ESTATE if there is no plan resp. no profiled step. */
typedef struct {
  int32_t op, arg;          /* as in acc_instr                                            */
  uint64_t bytes;           /* copies: bytes moved; compute steps: 0                      */
  double t_start, t_end;
} acc_timeline_entry;
int acc_get_timeline(acc_ctx* ctx, int which, acc_timeline_entry* out, int max_entries);

/* ---- execution (runtime memory manager, Sec. 5; the 2N steps of Sec. 3.1) ------------- */
/* One iteration as Sec. 2 describes its last stage and Sec. 5 its runtime: the 2N steps in
 * order on the compute stream, offloads (then release) on the swap-out stream, allocate and
 * prefetch on the swap-in stream, the input batch being the first layer's prefetch
 * (Algorithm 1, j = 1); then the weight update.
 * One forward / backward / SGD step at the planned minibatch.  images: fp32 NCHW,
 * pinned host (ACC_LOC_HOST) or device (ACC_LOC_DEVICE); labels: int32, host.  Blocks
 * until the step is done; *loss_out is the mean cross-entropy at the pre-update weights. */
int acc_train_step(acc_ctx* ctx, const float* images, int images_loc, const int32_t* labels,
                   float lr, float* loss_out);
/* What the last iteration did (Sec. 6.2.2 and 6.2.3 verify the memory and the transfer model
 * on such figures: bytes in the pool, bytes over the link, copy durations). */
int acc_get_stats(acc_ctx* ctx, acc_stats* out);
/* Verification mode of the swap engine (Sec. 5's four operations, checked at run time).
 * ACC_DEBUG_POISON: before every iteration the dynamic part of the pool and the used part of
 * the host arena are filled with a NaN pattern; every block is filled with a second NaN
 * pattern at the moment the plan releases it (after the last step that uses its tensor, on
 * the compute stream; after the offload copy of a swapped map, on the swap-out stream).  A
 * kernel or copy that runs before the data it needs has arrived, or after its block has been
 * given away, then reads NaNs, and the loss or some gradient is not finite; a correct plan
 * gives the same bits as without the mode.  After the iteration the pool is scanned:
 * acc_stats.peak_pool_bytes / touched_pool_bytes are then measured, and a write beyond the
 * budget makes acc_train_step return ACC_EPOOL.  Slow (two passes over the pool per
 * iteration); flags = 0 switches it off. */
enum { ACC_DEBUG_POISON = 1 };
int acc_set_debug(acc_ctx* ctx, int flags);
/* Parity hook: after the forward step that produces the stored output of `layer`, the next
 * iterations copy it to host_dst (bytes >= minibatch * elements per image * element size,
 * checked at acc_train_step; device layout NHWC in the context's storage type), complete when
 * acc_train_step returns.  Stored outputs are those of a convolution that feeds a batch norm,
 * of conv + bias (+ ReLU), of bn + ReLU and bn + add + ReLU (at the ReLU layer), of max-pool,
 * global average pooling and FC; a layer fused away (a bn before its ReLU) is ACC_EINVAL.
 * host_dst = NULL stops capturing that layer; layer = -1 with NULL stops all.  The pointer
 * must stay valid while it is registered (pinned memory keeps the copy asynchronous). */
int acc_capture_output(acc_ctx* ctx, int layer, void* host_dst, size_t bytes);
/* Parity hook, the other way round: after the forward step that produces the stored output of
 * `layer` (and after a capture of it), the next iterations overwrite it with host_src (same
 * layout and size rule).  The rest of the iteration then runs on those values: with the
 * outputs of an independent forward pass injected, the backward pass takes its discrete
 * decisions (ReLU masks, max-pool winners) from the same numbers as that pass, and its
 * gradients can be compared layer by layer without the noise of decisions that differ where
 * a value lies within rounding of zero.  Same registration rules as acc_capture_output. */
int acc_inject_output(acc_ctx* ctx, int layer, const void* host_src, size_t bytes);
/* on = 0: weight gradients run on the compute stream even if the context has a stream for
 * them (for measurements); on != 0 (default): they use it. */
int acc_set_wgrad_overlap(acc_ctx* ctx, int on);
/* on != 0: an iteration whose plan swaps nothing is recorded once into a HIP graph (stream capture
 * of the compute stream and, through its fork / join events, of the weight-gradient stream) and
 * replayed from then on: one graph launch instead of about a thousand kernel launches and event
 * calls per iteration.  The input copies and the update kernel (the learning rate is its argument)
 * stay outside the recording.  Same kernels, same order, same bits.  Plans that swap, profiling,
 * the verification mode and capture / injection hooks run the ordinary way whatever this says; a
 * new plan or a change of acc_set_wgrad_overlap discards the recording.  Default: off. */
int acc_set_graph(acc_ctx* ctx, int on);
/* level 0: off.  1: timing events around every step and every copy.  2: timing events
 * directly around every convolution kernel launch (while this is on, weight gradients run on
 * the compute stream, so that every kernel is timed alone).  3: both.  Events cost host time. */
int acc_set_profiling(acc_ctx* ctx, int level);
/* Per convolution kernel instance, summed over the last train_step run at level 2 or 3:
 * launches, milliseconds between the events around the launches, algorithmic flops
 * (2 * k*Ho*Wo * Cout * Cin*R*S per GEMM).  Returns the number of entries written. */
typedef struct {
  char name[48];
  int32_t launches;
  int32_t reserved;
  double ms;
  double flops;
} acc_kernel_profile;
int acc_get_kernel_profile(acc_ctx* ctx, acc_kernel_profile* out, int max_entries);
/* One entry per convolution-kernel launch of the last train_step run at level 2 or 3, in issue
 * order: the step and layer record it belongs to, its role (0 forward product, 1 data gradient,
 * 2 weight gradient; FC layers use the same kernels), which kernel instance ran (index of
 * acc_get_kernel_profile's names in V_* order), milliseconds between the events around the
 * launch and its algorithmic flops.  Returns the number of launches (which may exceed
 * max_entries: then only the first max_entries were written). */
typedef struct {
  int32_t step, layer, role, variant;
  double ms, flops;
} acc_launch_profile;
int acc_get_launch_profile(acc_ctx* ctx, acc_launch_profile* out, int max_entries);
/* per-step kernel time of the last profiled train_step, milliseconds; n = step count */
int acc_get_step_times_ms(acc_ctx* ctx, double* ms, int n);

/* ---- single operations on caller-owned device buffers (parity and roofline) ------- */
/* All pointers device; x / y / dy / dx / res / g_out NHWC and w (O-H-W-I) are stored as
 * `dtype` says (ACC_F32, or ACC_BF16 = the upper half of an fp32, round to nearest even);
 * dw (O-H-W-I), gamma, beta, mean, istd, dgamma, dbeta are always fp32.  Arithmetic is fp32
 * (bf16 products accumulate in fp32).  stream is a hipStream_t.  workspace may be NULL when
 * workspace_bytes is 0; query the need with acc_op_conv_workspace().  accumulate != 0 adds
 * into dx instead of overwriting.  Every pointer must be 16-byte aligned (the kernels move
 * 16 bytes at a time); a misaligned one is ACC_EINVAL, like any other bad argument, and
 * nothing is launched. */
size_t acc_op_conv_workspace(int n, int h, int w, int cin, int cout, int r, int s, int stride,
                             int pad);
int acc_op_conv_fwd(const void* x, const void* w, void* y, int n, int h, int wd, int cin,
                    int cout, int r, int s, int stride, int pad, int dtype, void* stream);
int acc_op_conv_dgrad(const void* dy, const void* w, void* dx, int n, int h, int wd, int cin,
                      int cout, int r, int s, int stride, int pad, int accumulate,
                      void* workspace, size_t workspace_bytes, int dtype, void* stream);
int acc_op_conv_wgrad(const void* x, const void* dy, float* dw, int n, int h, int wd, int cin,
                      int cout, int r, int s, int stride, int pad, void* workspace,
                      size_t workspace_bytes, int dtype, void* stream);
/* y = relu?(gamma*(x-mean)*istd + beta (+ res)); saves mean / istd (c floats each).
 * workspace: acc_op_bn_workspace(c) bytes. */
size_t acc_op_bn_workspace(int c);
int acc_op_bn_fwd(const void* x, const float* gamma, const float* beta, const void* res,
                  void* y, float* mean, float* istd, int rows, int c, int relu, float eps,
                  void* workspace, int dtype, void* stream);
/* dy is masked by (y > 0) when y != NULL (fused ReLU); when g_out != NULL the masked
 * gradient is also written there (it may alias dy). */
int acc_op_bn_bwd(const void* x, const void* dy, const void* y, const float* gamma,
                  const float* mean, const float* istd, void* dx, float* dgamma, float* dbeta,
                  void* g_out, int rows, int c, void* workspace, int dtype, void* stream);

/* The parameter-free layers of the evaluated networks (Sec. 6.1: residual networks, VGG-16), which the
 * unfolded iteration of Sec. 3.1 runs like any other step; the paper does not define them, the
 * definitions are the textbook ones.  Max-pool over r x r windows (padding never wins, the first maximum
 * in row-major window order takes the gradient; c a multiple of 4); mean over the hw positions of an
 * image; softmax cross-entropy: loss_rows[i] = logsumexp(z_i) - z_i[label_i] (NaN for a label outside
 * [0, classes)), *loss = their mean, dz = (softmax(z) - onehot) / n; loss_rows and dz may each be NULL
 * (then loss, too, is not written).  labels, loss_rows (n floats) and loss (1 float) are device memory. */
int acc_op_maxpool_fwd(const void* x, void* y, int n, int h, int wd, int c, int r, int stride, int pad,
                       int dtype, void* stream);
int acc_op_maxpool_bwd(const void* x, const void* dy, void* dx, int n, int h, int wd, int c, int r,
                       int stride, int pad, int accumulate, int dtype, void* stream);
int acc_op_gap_fwd(const void* x, void* y, int n, int hw, int c, int dtype, void* stream);
int acc_op_gap_bwd(const void* dy, void* dx, int n, int hw, int c, int accumulate, int dtype, void* stream);
int acc_op_softmax_ce(const void* z, const int32_t* labels, float* loss_rows, float* loss, void* dz, int n,
                      int classes, int dtype, void* stream);


/* ---- for callers that cannot allocate --------------------------------------------- */
/* acc_op_bn_fwd() without the workspace argument, for code that may not call hipMalloc or
 * hand a workspace through: kernels under HIP graph capture, serving loops, harnesses that
 * forbid allocation.  The reduction workspace is a device array built into the library
 * (ACC_NOALLOC_BN_MAX_C channels: 32.03 MiB per GPU, held until the process ends); the call
 * allocates and frees nothing, on the host or on the device.  Same arguments, kernels and
 * results as acc_op_bn_fwd(); stream must belong to the current device.  c above
 * ACC_NOALLOC_BN_MAX_C is ACC_EINVAL (text in acc_last_error(NULL)) and nothing is launched.
 * All calls on one GPU share the array: calls that overlap there (different streams with no
 * event between them, or different threads) race; nothing needs to be cleared between calls. */
#define ACC_NOALLOC_BN_MAX_C 2048
int acc_op_bn_fwd_noalloc(const void* x, const float* gamma, const float* beta, const void* res,
                          void* y, float* mean, float* istd, int rows, int c, int relu, float eps,
                          int dtype, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ACCUDNN_H */
