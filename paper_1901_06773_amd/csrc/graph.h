// Static information of the planner (Sec. 3.2 of the paper): the network unfolded into
// 2N steps (Sec. 3.1), the memory objects each step reads and writes, their sizes as a
// linear function of the minibatch, FLOPs per step (Eq. 1), and their lifetimes.  The
// global memory-object access pattern (GMAP) is the per-step read/write lists below.
// Host code only; no device calls.
#pragma once
#include <cstddef>
#include <cstdint>
#include <string>
#include <vector>

#include "../../include/accudnn.h"

namespace acc {

enum StepKind {
  K_INPUT_F = 0,   // NCHW minibatch -> NHWC
  K_CONV_F, K_BN_F, K_MAXPOOL_F, K_GAP_F, K_FC_F, K_LOSS_F,
  K_LOSS_B, K_FC_B, K_GAP_B, K_MAXPOOL_B, K_BN_B, K_CONV_B, K_SGD,
  K_COUNT
};

enum TensorKind { T_ACT = 0, T_GRAD = 1, T_WORK = 2, T_INPUT = 3 };

struct Tensor {
  int kind = T_ACT;
  int c = 0, h = 0, w = 0;            // per image, NHWC (input image: NCHW)
  size_t bytes_per_image = 0;         // bytes(k) = align256(bytes_fixed + k * bytes_per_image)
  size_t bytes_fixed = 0;
  int layer = -1;                     // layer record whose output this is (activations)
  int wgrad_layer = -1;               // >= 0: split-K workspace of that conv/fc layer's weight
                                      // gradient; its size is a step function of k
  // lifetimes in step indices, filled by finalize()
  int producer = -1, last_fwd = -1, first_bwd = -1, last = -1;
  bool is_map = false;                // alive in forward and needed again in backward
};

struct Step {
  int kind = 0;
  int layer = -1;        // conv / bn / fc / pool layer record
  int phase = 0;         // 0 forward, 1 backward, 2 update
  // tensor ids (-1 = unused)
  int x = -1, y = -1, res = -1, dy = -1, dx = -1, ws = -1, ws2 = -1;
  bool relu = false, dx_accumulate = false, g_inplace = false, x_is_image = false;
  int bias_layer = -1;   // conv steps: the per-channel bias layer fused into them (with relu: conv + bias + ReLU)
  int ws3 = -1;          // conv backward with a fused bias: slab sums of the (masked) gradient
  double flops_per_image = 0;   // conv / fc steps
  double bytes_per_image = 0;   // HBM bytes the step touches, per image
  double bytes_fixed = 0;
  std::vector<int> reads, writes;     // GMAP: memory objects touched (scratch included in writes)
  // Conv backward steps with a data gradient: the weight gradient may run on a stream of its
  // own beside the steps that follow.  wgrad_join: the step before which it must be complete
  // (its operands x, dy and its partial sums stay allocated until then: they are among that
  // step's reads; the partial sums one conv backward step longer, because they are added up
  // on the side of the next weight-gradient launch); joins: the steps whose weight gradients
  // this step waits for;
  // flip_for: the later conv backward step whose flipped filter this step's data-gradient
  // launch writes on the side (-1: none); flips_itself: nobody did it for this step.
  // Conv forward steps whose result goes into a batch norm (fp32 storage): stats_for is that
  // step, stats the tensor in which the conv launch leaves the per-channel partial sums for
  // it (set on both steps).
  int stats_for = -1, stats = -1;
  // Conv backward steps (fp32 storage, stride 1) whose data gradient is the gradient of a
  // batch norm's ReLU output, that batch norm's backward being the next step: bnb_for is that
  // step, bnb the tensor in which the data-gradient launch leaves the sums of the masked
  // gradient g and of g * xhat for it (set on both steps); the launch also applies the mask.
  int bnb_for = -1, bnb = -1;
  int wgrad_join = -1;
  std::vector<int> joins;
  int flip_for = -1;
  bool flips_itself = false;
};

// A weight gradient is joined this many conv backward steps after its own: a wait for an
// event that was signalled long ago costs next to nothing on the waiting stream, a wait for
// a fresh one stalls it (measured at the ResNet-152 headline: joined one conv step later
// 1026 images/s, slower than without the second stream; two to six steps later 1118-1123).
constexpr int kWgradLag = 2;

struct ParamSlot {       // static device data of a layer
  size_t count = 0;      // elements
  size_t offset = 0;     // element offset into the parameter (and gradient) region
  size_t stat_offset = 0;// bn: element offset of mean|istd in the statistics region
};

struct Graph {
  std::vector<acc_layer> layers;
  int in_c = 0, in_h = 0, in_w = 0, classes = 0;
  std::vector<Tensor> tensors;
  std::vector<Step> steps;
  int n_fwd = 0;                      // steps [0, n_fwd) are forward
  std::vector<ParamSlot> params;      // per layer
  size_t param_elems = 0, stat_elems = 0;
  int t_stage = -1, t_image = -1, t_labels = -1;   // NCHW staging copy, NHWC images, labels
  std::vector<int> maps;              // tensor ids with is_map, in producer order
  std::vector<int> act_of_layer;      // tensor holding a layer's output, -1 if fused away

  // Builds everything from the layer records; on failure returns false and sets err.
  int dtype = 0;                      // ACC_F32 / ACC_BF16: storage of activations and their gradients
  bool build(const acc_layer* recs, int n, int in_c, int in_h, int in_w, int dtype, std::string* err);
  size_t static_bytes() const;        // params + grads + statistics + scalars, 256-aligned parts
  size_t bytes(int tensor, int k) const;   // 256-aligned size of a memory object at minibatch k
  void conv_dims(int layer, int* h, int* w, int* ho, int* wo) const;  // input / output size
  std::vector<int> shape_c, shape_h, shape_w;   // per layer output shape
};

const char* step_kind_name(int kind);

}  // namespace acc
