// Static analyzer (Sec. 3.2, "static information"): walks the layer records once and
// produces the 2N-step unfolding of Sec. 3.1 with its memory-object access pattern,
// object sizes proportional to the minibatch, and FLOPs per step (Eq. 1).
//
// Fusions chosen for a bandwidth-bound GPU: BN+ReLU and BN+add+ReLU are one step each,
// so pre-activation tensors are never stored.  What lives from forward into backward
// (the swappable feature maps) is every convolution input and every BN input.
#include "graph.h"

#include <algorithm>
#include <cstdio>

#include "kernels.h"

namespace acc {

const char* step_kind_name(int kind) {
  static const char* names[K_COUNT] = {"input_fwd", "conv_fwd", "bn_fwd", "maxpool_fwd", "gap_fwd", "fc_fwd",
                                       "loss_fwd", "loss_bwd", "fc_bwd", "gap_bwd", "maxpool_bwd",
                                       "bn_bwd", "conv_bwd", "sgd"};
  return (kind >= 0 && kind < K_COUNT) ? names[kind] : "?";
}

static inline int conv_out(int in, int r, int stride, int pad) { return (in + 2 * pad - r) / stride + 1; }

static std::string fmt(const char* f, int a, const char* what) {
  char buf[256];
  snprintf(buf, sizeof buf, f, a, what);
  return buf;
}

void Graph::conv_dims(int layer, int* h, int* w, int* ho, int* wo) const {
  const acc_layer& l = layers[layer];
  *h = l.in0 < 0 ? in_h : shape_h[l.in0];
  *w = l.in0 < 0 ? in_w : shape_w[l.in0];
  *ho = shape_h[layer];
  *wo = shape_w[layer];
}

size_t Graph::bytes(int t, int k) const {
  const Tensor& T = tensors[t];
  size_t b;
  if (T.wgrad_layer >= 0) {
    const acc_layer& l = layers[T.wgrad_layer];
    if (l.kind == ACC_FC) {
      b = wgrad_workspace_bytes(k, 1, 1, l.cin, l.cout, 1, 1, dtype);
    } else {
      int h, w, ho, wo;
      conv_dims(T.wgrad_layer, &h, &w, &ho, &wo);
      b = wgrad_workspace_bytes(k, ho, wo, l.cin, l.cout, l.r, l.s, dtype);
    }
    if (b == 0) b = 256;   // keep the object in the access pattern even when no split is used
  } else {
    b = T.bytes_fixed + (size_t)k * T.bytes_per_image;
  }
  return (b + 255) & ~(size_t)255;
}

size_t Graph::static_bytes() const {
  auto al = [](size_t b) { return (b + 255) & ~(size_t)255; };
  // weights, gradients (fp32), in bf16 mode the rounded copy of the weights, statistics, loss
  return 2 * al(param_elems * sizeof(float)) + (dtype == ACC_BF16 ? al(param_elems * 2) : 0) +
         al(stat_elems * sizeof(float)) + 256;
}

bool Graph::build(const acc_layer* recs, int n, int ic, int ih, int iw, int dt, std::string* err) {
  *this = Graph();
  dtype = dt;
  const size_t es = dt == ACC_BF16 ? 2 : 4;   // bytes per stored activation element
  if (!recs || n <= 0 || ic <= 0 || ih <= 0 || iw <= 0) { *err = "empty network or input"; return false; }
  layers.assign(recs, recs + n);
  in_c = ic; in_h = ih; in_w = iw;
  shape_c.assign(n, 0); shape_h.assign(n, 0); shape_w.assign(n, 0);
  act_of_layer.assign(n, -1);
  params.assign(n, ParamSlot());

  auto in_shape = [&](int id, int* c, int* h, int* w) {
    if (id < 0) { *c = in_c; *h = in_h; *w = in_w; }
    else { *c = shape_c[id]; *h = shape_h[id]; *w = shape_w[id]; }
  };
  // ---- shapes, consumers, parameter slots
  std::vector<std::vector<int>> consumers(n);
  int loss_layer = -1;
  for (int i = 0; i < n; ++i) {
    const acc_layer& l = layers[i];
    if (l.in0 >= i || l.in1 >= i || l.in0 < -1 || l.in1 < -1) { *err = fmt("layer %d: %s", i, "input index out of order"); return false; }
    int c, h, w;
    in_shape(l.in0, &c, &h, &w);
    if (l.in0 >= 0) consumers[l.in0].push_back(i);
    switch (l.kind) {
      case ACC_CONV:
        if (l.cin != c || l.cout <= 0 || l.r <= 0 || l.s != l.r || l.stride <= 0 || l.pad < 0 ||
            l.pad >= l.r || h + 2 * l.pad < l.r || w + 2 * l.pad < l.s) { *err = fmt("layer %d: %s", i, "bad convolution (square filters, pad < r)"); return false; }
        shape_c[i] = l.cout; shape_h[i] = conv_out(h, l.r, l.stride, l.pad); shape_w[i] = conv_out(w, l.s, l.stride, l.pad);
        params[i].count = (size_t)l.cout * l.cin * l.r * l.s;
        break;
      case ACC_BN:
        if (l.cin != c || (c & 3)) { *err = fmt("layer %d: %s", i, "bn channels must match and be a multiple of 4"); return false; }
        shape_c[i] = c; shape_h[i] = h; shape_w[i] = w;
        params[i].count = 2 * (size_t)c;
        break;
      case ACC_RELU:
        shape_c[i] = c; shape_h[i] = h; shape_w[i] = w;
        break;
      case ACC_BIAS:
        if (l.cin != c || (c & 3)) { *err = fmt("layer %d: %s", i, "bias channels must match and be a multiple of 4"); return false; }
        shape_c[i] = c; shape_h[i] = h; shape_w[i] = w;
        params[i].count = (size_t)c;
        break;
      case ACC_ADD: {
        int c1, h1, w1;
        in_shape(l.in1, &c1, &h1, &w1);
        if (c1 != c || h1 != h || w1 != w) { *err = fmt("layer %d: %s", i, "add shapes differ"); return false; }
        if (l.in1 >= 0) consumers[l.in1].push_back(i);
        shape_c[i] = c; shape_h[i] = h; shape_w[i] = w;
        break;
      }
      case ACC_MAXPOOL:
        if (l.r <= 0 || l.s <= 0 || l.stride <= 0 || l.pad < 0 || l.pad >= l.r || l.pad >= l.s || (c & 3) ||
            h + 2 * l.pad < l.r || w + 2 * l.pad < l.s) { *err = fmt("layer %d: %s", i, "bad max-pool"); return false; }
        shape_c[i] = c; shape_h[i] = conv_out(h, l.r, l.stride, l.pad); shape_w[i] = conv_out(w, l.s, l.stride, l.pad);
        break;
      case ACC_GAP:
        shape_c[i] = c; shape_h[i] = 1; shape_w[i] = 1;
        break;
      case ACC_FC:
        // a map with h * w > 1 is flattened (on the device in h, w, c order; weights are permuted on their way in)
        if (l.cin != c * h * w || l.cout <= 0) { *err = fmt("layer %d: %s", i, "fc input must have cin elements per image"); return false; }
        shape_c[i] = l.cout; shape_h[i] = 1; shape_w[i] = 1;
        params[i].count = (size_t)l.cout * l.cin + l.cout;
        break;
      case ACC_SOFTMAX_CE:
        if (l.in0 < 0 || h != 1 || w != 1 || loss_layer >= 0) { *err = fmt("layer %d: %s", i, "one softmax_ce over a 1x1 map"); return false; }
        shape_c[i] = 1; shape_h[i] = 1; shape_w[i] = 1;
        loss_layer = i;
        classes = c;
        break;
      default:
        *err = fmt("layer %d: %s", i, "unknown kind");
        return false;
    }
  }
  if (loss_layer != n - 1) { *err = "the last layer must be softmax_ce"; return false; }
  for (int i = 0; i < n; ++i) {
    params[i].offset = param_elems;
    param_elems += (params[i].count + 63) & ~(size_t)63;
    if (layers[i].kind == ACC_BN) {
      params[i].stat_offset = stat_elems;
      stat_elems += (2 * (size_t)layers[i].cin + 63) & ~(size_t)63;
    }
  }

  // ---- tensors
  auto new_tensor = [&](int kind, int c, int h, int w, size_t per_image, size_t fixed, int layer) {
    Tensor t;
    t.kind = kind; t.c = c; t.h = h; t.w = w;
    t.bytes_per_image = per_image; t.bytes_fixed = fixed; t.layer = layer;
    tensors.push_back(t);
    return (int)tensors.size() - 1;
  };
  auto new_act = [&](int layer) {
    return new_tensor(T_ACT, shape_c[layer], shape_h[layer], shape_w[layer],
                      (size_t)shape_c[layer] * shape_h[layer] * shape_w[layer] * es, 0, layer);
  };
  t_stage = new_tensor(T_INPUT, in_c, in_h, in_w, (size_t)in_c * in_h * in_w * 4, 0, -1);
  t_labels = new_tensor(T_INPUT, 1, 1, 1, 4, 0, -1);
  t_image = new_tensor(T_ACT, in_c, in_h, in_w, (size_t)in_c * in_h * in_w * es, 0, -1);
  auto act_in = [&](int id) { return id < 0 ? t_image : act_of_layer[id]; };
  auto elems = [&](int t) { return (double)tensors[t].c * tensors[t].h * tensors[t].w; };

  // ---- forward steps
  {
    Step s;
    s.kind = K_INPUT_F;
    s.x = t_stage; s.y = t_image;
    s.bytes_per_image = (4.0 + es) * in_c * in_h * in_w;
    s.reads = {t_stage};
    s.writes = {t_image};
    steps.push_back(s);
  }
  std::vector<char> fused(n, 0);       // layer absorbed into an earlier step
  std::vector<int> step_of_layer(n, -1);
  for (int i = 0; i < n; ++i) {
    const acc_layer& l = layers[i];
    if (fused[i]) continue;
    Step s;
    s.layer = i;
    s.phase = 0;
    if (l.kind != ACC_ADD && l.kind != ACC_RELU) {
      s.x = act_in(l.in0);
      if (s.x < 0) { *err = fmt("layer %d: %s", i, "reads a tensor that was fused away"); return false; }
    }
    switch (l.kind) {
      case ACC_CONV: {
        s.kind = K_CONV_F;
        s.x_is_image = l.in0 < 0;
        int out_layer = i;
        if (consumers[i].size() == 1 && layers[consumers[i][0]].kind == ACC_BIAS) {
          // conv -> bias (-> ReLU): one step, the bias and the ReLU sit in the epilogue
          const int bl = consumers[i][0];
          s.bias_layer = bl;
          out_layer = bl;
          fused[bl] = 1;
          if (consumers[bl].size() == 1 && layers[consumers[bl][0]].kind == ACC_RELU) {
            s.relu = true;
            out_layer = consumers[bl][0];
            fused[out_layer] = 1;
          }
        }
        s.y = new_act(out_layer);
        act_of_layer[i] = act_of_layer[out_layer] = s.y;
        if (s.bias_layer >= 0) act_of_layer[s.bias_layer] = s.y;
        s.flops_per_image = 2.0 * shape_h[i] * shape_w[i] * l.cout * l.cin * l.r * l.s;
        s.bytes_per_image = (double)es * (elems(s.x) + elems(s.y));
        s.bytes_fixed = 4.0 * params[i].count;
        break;
      }
      case ACC_BN: {
        s.kind = K_BN_F;
        int out_layer = i;
        if (consumers[i].size() == 1) {
          const int c0 = consumers[i][0];
          if (layers[c0].kind == ACC_RELU) {
            s.relu = true; out_layer = c0; fused[c0] = 1;
          } else if (layers[c0].kind == ACC_ADD && consumers[c0].size() == 1 &&
                     layers[consumers[c0][0]].kind == ACC_RELU) {
            const int other = layers[c0].in0 == i ? layers[c0].in1 : layers[c0].in0;
            if (other < i && other != i && act_in(other) >= 0) {
              s.relu = true; s.res = act_in(other);
              out_layer = consumers[c0][0];
              fused[c0] = 1; fused[out_layer] = 1;
            }
          }
        }
        s.y = new_act(out_layer);
        act_of_layer[out_layer] = s.y;
        s.ws = new_tensor(T_WORK, 0, 0, 0, 0, bn_workspace_bytes(l.cin), i);
        s.bytes_per_image = (double)es * elems(s.x) * (s.res >= 0 ? 4 : 3);
        break;
      }
      case ACC_RELU:
      case ACC_ADD:
      case ACC_BIAS:
        *err = fmt("layer %d: %s", i, "only BN->ReLU, BN->add->ReLU, conv->bias(->ReLU) and FC->ReLU patterns are supported");
        return false;
      case ACC_MAXPOOL:
        s.kind = K_MAXPOOL_F;
        s.y = act_of_layer[i] = new_act(i);
        s.bytes_per_image = (double)es * (elems(s.x) + elems(s.y));
        break;
      case ACC_GAP:
        s.kind = K_GAP_F;
        s.y = act_of_layer[i] = new_act(i);
        s.bytes_per_image = (double)es * (elems(s.x) + elems(s.y));
        break;
      case ACC_FC:
        s.kind = K_FC_F;
        {
          int out_layer = i;
          if (consumers[i].size() == 1 && layers[consumers[i][0]].kind == ACC_RELU) {
            s.relu = true;
            out_layer = consumers[i][0];
            fused[out_layer] = 1;
          }
          s.y = new_act(out_layer);
          act_of_layer[i] = act_of_layer[out_layer] = s.y;
        }
        s.flops_per_image = 2.0 * l.cin * l.cout;
        s.bytes_per_image = (double)es * (elems(s.x) + elems(s.y));
        s.bytes_fixed = 4.0 * params[i].count;
        break;
      case ACC_SOFTMAX_CE:
        s.kind = K_LOSS_F;
        s.ws = new_tensor(T_WORK, 0, 0, 0, 4, 0, i);   // per-sample losses
        s.bytes_per_image = (double)es * elems(s.x);
        break;
    }
    s.reads.push_back(s.x);
    if (s.res >= 0) s.reads.push_back(s.res);
    if (l.kind == ACC_SOFTMAX_CE) s.reads.push_back(t_labels);
    if (s.y >= 0) s.writes.push_back(s.y);
    if (s.ws >= 0) s.writes.push_back(s.ws);
    step_of_layer[i] = (int)steps.size();
    steps.push_back(s);
  }
  n_fwd = (int)steps.size();
  // A convolution whose output feeds the next step's batch norm hands it the per-channel sums
  // of every block of 32 rows (fp32 storage): part[2][stride][cout] floats with
  // stride = k * 2 * ceil(Ho*Wo / 64) >= 2 * ceil(k*Ho*Wo / 64) blocks.
  if (dtype == ACC_F32)
    for (int j = 0; j + 1 < n_fwd; ++j) {
      if (steps[j].kind != K_CONV_F || steps[j + 1].kind != K_BN_F || steps[j + 1].x != steps[j].y) continue;
      const Tensor& y = tensors[steps[j].y];
      const size_t per_image = (size_t)2 * 2 * (((size_t)y.h * y.w + 63) / 64) * y.c * sizeof(float);
      const int t = new_tensor(T_WORK, 0, 0, 0, per_image, 0, steps[j].layer);
      steps[j].stats_for = j + 1;
      steps[j].stats = t;
      steps[j + 1].stats = t;
      steps[j].writes.push_back(t);
      steps[j + 1].reads.push_back(t);
    }

  // ---- backward steps: reverse order; grad_of[t] is the tensor holding d(loss)/d(t)
  std::vector<int> grad_of(tensors.size() + 4 * n, -1);
  auto grad_for_write = [&](int act, bool* accumulate) {
    if ((int)grad_of.size() <= act) grad_of.resize(act + 1, -1);
    if (grad_of[act] >= 0) { *accumulate = true; return grad_of[act]; }
    *accumulate = false;
    const Tensor a = tensors[act];
    const int g = new_tensor(T_GRAD, a.c, a.h, a.w, a.bytes_per_image, 0, a.layer);
    grad_of[act] = g;
    return g;
  };
  for (int si = n_fwd - 1; si >= 0; --si) {
    const Step f = steps[si];
    if (f.kind == K_INPUT_F) continue;
    const acc_layer& l = layers[f.layer];
    Step b;
    b.layer = f.layer;
    b.phase = 1;
    b.x = f.x;
    if (f.kind != K_LOSS_F) {
      if (f.y >= (int)grad_of.size() || grad_of[f.y] < 0) {
        *err = fmt("layer %d: %s", f.layer, "output does not reach the loss");
        return false;
      }
      b.dy = grad_of[f.y];
    }
    switch (f.kind) {
      case K_LOSS_F:
        b.kind = K_LOSS_B;
        b.dx = grad_for_write(f.x, &b.dx_accumulate);
        if (b.dx_accumulate) { *err = "logits feed more than the loss"; return false; }
        b.reads = {f.x, t_labels};
        b.writes = {b.dx};
        b.bytes_per_image = 8.0 * elems(f.x);
        break;
      case K_FC_F:
        b.kind = K_FC_B;
        b.dx = grad_for_write(f.x, &b.dx_accumulate);
        b.ws = new_tensor(T_WORK, 0, 0, 0, 0, (size_t)l.cin * l.cout * es, f.layer);
        b.ws2 = new_tensor(T_WORK, 0, 0, 0, 0, 0, f.layer);
        tensors[b.ws2].wgrad_layer = f.layer;
        b.flops_per_image = 4.0 * l.cin * l.cout;
        b.bytes_per_image = (double)es * (2 * elems(f.x) + elems(f.y));
        b.bytes_fixed = 12.0 * params[f.layer].count;
        b.reads = {f.x, b.dy};
        if (b.dx_accumulate) b.reads.push_back(b.dx);
        b.writes = {b.dx, b.ws, b.ws2};
        if (f.relu) {   // the gradient is masked with [y > 0] first (in place)
          b.relu = true;
          b.y = f.y;
          b.reads.push_back(b.y);
          b.writes.push_back(b.dy);
        }
        break;
      case K_GAP_F:
        b.kind = K_GAP_B;
        b.dx = grad_for_write(f.x, &b.dx_accumulate);
        b.reads = {b.dy};
        if (b.dx_accumulate) b.reads.push_back(b.dx);
        b.writes = {b.dx};
        b.bytes_per_image = (double)es * (elems(f.x) + elems(f.y));
        break;
      case K_MAXPOOL_F:
        b.kind = K_MAXPOOL_B;
        b.dx = grad_for_write(f.x, &b.dx_accumulate);
        b.reads = {f.x, b.dy};
        if (b.dx_accumulate) b.reads.push_back(b.dx);
        b.writes = {b.dx};
        b.bytes_per_image = (double)es * (2 * elems(f.x) + elems(f.y));
        break;
      case K_BN_F: {
        b.kind = K_BN_B;
        b.relu = f.relu;
        b.res = f.res;
        if (f.relu) b.y = f.y;
        b.dx = grad_for_write(f.x, &b.dx_accumulate);
        if (b.dx_accumulate) { *err = fmt("layer %d: %s", f.layer, "bn input has a second consumer"); return false; }
        b.ws = new_tensor(T_WORK, 0, 0, 0, 0, bn_workspace_bytes(l.cin), f.layer);
        b.reads = {f.x, b.dy};
        if (b.y >= 0) b.reads.push_back(b.y);
        b.writes = {b.dx, b.ws};
        if (f.res >= 0 && f.res != t_image) {
          // the masked gradient is also the gradient of the shortcut operand: it is written
          // in place over dy, and that buffer becomes the shortcut's gradient tensor
          if ((int)grad_of.size() <= f.res) grad_of.resize(f.res + 1, -1);
          if (grad_of[f.res] >= 0) {
            *err = fmt("layer %d: %s", f.layer, "shortcut operand already has a gradient (unsupported topology)");
            return false;
          }
          grad_of[f.res] = b.dy;
          b.g_inplace = true;
          b.writes.push_back(b.dy);
        }
        b.bytes_per_image = (double)es * elems(f.x) * (2 * (f.relu ? 3 : 2) + 1 + (f.res >= 0 ? 1 : 0));
        break;
      }
      case K_CONV_F: {
        b.kind = K_CONV_B;
        b.x_is_image = f.x_is_image;
        const bool need_dx = !f.x_is_image;
        if (need_dx) {
          size_t filter_bytes = params[f.layer].count * es;
          if (l.stride > 1 && (l.r > 1 || l.s > 1 || l.pad > 0)) {
            // cut by the residue of the dx position: one sub-filter per class, aligned one by one
            DgradPart parts[kMaxDgradParts];
            if (dgrad_split(tensors[f.x].h, tensors[f.x].w, l.cin, l.cout, l.r, l.s, l.stride, l.pad, (int)es, parts,
                            nullptr, &filter_bytes) < 0) {
              *err = fmt("layer %d: %s", f.layer, "data gradient of this strided convolution is not supported");
              return false;
            }
          }
          b.dx = grad_for_write(f.x, &b.dx_accumulate);
          b.ws = new_tensor(T_WORK, 0, 0, 0, 0, filter_bytes, f.layer);
        }
        b.ws2 = new_tensor(T_WORK, 0, 0, 0, 0, 0, f.layer);
        tensors[b.ws2].wgrad_layer = f.layer;
        b.flops_per_image = f.flops_per_image * (need_dx ? 2 : 1);
        b.bytes_per_image = (double)es * (elems(f.x) * (need_dx ? 2 : 1) + 2 * elems(f.y));
        b.bytes_fixed = 4.0 * params[f.layer].count * (need_dx ? 4 : 1);
        b.reads = {f.x, b.dy};
        if (need_dx && b.dx_accumulate) b.reads.push_back(b.dx);
        if (need_dx) { b.writes.push_back(b.dx); b.writes.push_back(b.ws); }
        b.writes.push_back(b.ws2);
        if (f.bias_layer >= 0) {
          // conv + bias (+ ReLU): the gradient is masked with [y > 0] in place and summed per
          // channel (the bias gradient) before the two GEMMs
          b.bias_layer = f.bias_layer;
          b.relu = f.relu;
          b.ws3 = new_tensor(T_WORK, 0, 0, 0, 0, relu_bias_workspace_bytes(l.cout), f.layer);
          if (f.relu) { b.y = f.y; b.reads.push_back(b.y); }
          b.writes.push_back(b.dy);
          b.writes.push_back(b.ws3);
        }
        break;
      }
      default:
        *err = "internal: unexpected forward step";
        return false;
    }
    steps.push_back(b);
  }
  {
    Step u;
    u.kind = K_SGD;
    u.phase = 2;
    u.bytes_fixed = 12.0 * param_elems;
    steps.push_back(u);
  }

  // ---- the data gradient of a stride-1 convolution hands the batch norm before it (the one
  //      whose ReLU output is the convolution's only input) the sums its backward pass needs
  if (dtype == ACC_F32)
    for (int j = n_fwd; j + 1 < (int)steps.size(); ++j) {
      Step& cb = steps[j];
      Step& bb = steps[j + 1];
      if (cb.kind != K_CONV_B || cb.dx < 0 || cb.dx_accumulate || bb.kind != K_BN_B) continue;
      const acc_layer& cl = layers[cb.layer];
      // (Not for a batch norm with a shortcut operand, whose dy this convolution adds onto:
      // the 1x1 data gradient before it has 8 chunks per tile, and three more strided reads
      // per output element in its epilogue cost it about what the batch norm's own pass over
      // dy saves: 1.4 ms saved and 1.0 ms added per ResNet-152 step, 0.3 % in all, with the
      // convolution kernel 5 % slower for it.)
      if (cl.stride != 1 || bb.dy != cb.dx || !bb.relu || bb.res >= 0 || bb.g_inplace || bb.y != cb.x) continue;
      const Tensor& bx = tensors[bb.x];
      const size_t per_image = (size_t)2 * 2 * (((size_t)bx.h * bx.w + 63) / 64) * bx.c * sizeof(float);
      const int t = new_tensor(T_WORK, 0, 0, 0, per_image, 0, bb.layer);
      cb.bnb_for = j + 1;
      cb.bnb = t;
      bb.bnb = t;
      cb.writes.push_back(t);
      if (std::find(cb.reads.begin(), cb.reads.end(), bb.x) == cb.reads.end()) cb.reads.push_back(bb.x);
      bb.reads.push_back(t);
    }

  // ---- weight gradients beside the data gradients: join points, operands kept until then,
  //      and the flipped filter of the next conv backward step written one step early
  {
    const int sgd = (int)steps.size() - 1;
    std::vector<int> convb;
    for (int j = 0; j < (int)steps.size(); ++j)
      if (steps[j].kind == K_CONV_B && steps[j].dx >= 0) convb.push_back(j);
    auto add_unique = [](std::vector<int>& v, int t) {
      if (t >= 0 && std::find(v.begin(), v.end(), t) == v.end()) v.push_back(t);
    };
    for (size_t i = 0; i < convb.size(); ++i) {
      Step& s = steps[convb[i]];
      const int join = i + kWgradLag < convb.size() ? convb[i + kWgradLag] : sgd;
      s.wgrad_join = join;
      steps[join].joins.push_back(convb[i]);
      for (int t : {s.x, s.dy, s.ws2}) add_unique(steps[join].reads, t);
      // the parts are added up on the side of the next weight-gradient launch: they live until
      // that one is joined
      const int join_next = i + 1 + kWgradLag < convb.size() ? convb[i + 1 + kWgradLag] : sgd;
      add_unique(steps[join_next].reads, s.ws2);
      const acc_layer& l = layers[s.layer];
      const bool split = l.stride > 1 && (l.r > 1 || l.s > 1 || l.pad > 0);
      if (split) continue;                       // writes its sub-filters itself
      if (i == 0) { s.flips_itself = true; continue; }
      Step& prev = steps[convb[i - 1]];
      prev.flip_for = convb[i];
      add_unique(prev.writes, s.ws);
      add_unique(s.reads, s.ws);
    }
  }

  // ---- lifetimes
  const int ns = (int)steps.size();
  for (int j = 0; j < ns; ++j) {
    auto touch = [&](int t, bool write) {
      Tensor& T = tensors[t];
      if (T.producer < 0 && write) T.producer = j;
      if (j < n_fwd) T.last_fwd = j;
      else if (T.first_bwd < 0) T.first_bwd = j;
      T.last = j;
    };
    for (int t : steps[j].writes) touch(t, true);
    for (int t : steps[j].reads) touch(t, false);
  }
  tensors[t_stage].producer = -1;
  tensors[t_labels].producer = -1;
  for (size_t t = 0; t < tensors.size(); ++t) {
    Tensor& T = tensors[t];
    if (T.last < 0) { *err = "internal: unused tensor"; return false; }
    const bool crosses = T.last_fwd >= 0 && T.first_bwd >= 0;
    T.is_map = crosses && T.kind == T_ACT;
    if (T.is_map) maps.push_back((int)t);
  }
  std::stable_sort(maps.begin(), maps.end(),
                   [&](int a, int b) { return tensors[a].producer < tensors[b].producer; });
  return true;
}

}  // namespace acc
