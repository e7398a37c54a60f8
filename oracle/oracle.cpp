// CPU oracle: one SGD training step of a layer list (ResNets, VGG), written out as the
// plain definitions of its layers.  TEST INFRASTRUCTURE ONLY: the product path
// never links, loads or calls this file; it shares no code with the HIP library.
//
// What it computes is the quantity the paper's runtime must leave unchanged:
// swapping feature maps out and back in moves bytes and never alters values
// (abstract: no accuracy loss; Sec. 3.1: the four operations allocate / release /
// offload / prefetch are copies), so the result of a training iteration is the
// textbook forward / backward / SGD step of the network.
//
// Conventions: NCHW activations, OIHW filters, cross-correlation with zero
// padding and no bias (a per-channel bias is a layer of its own), batch-norm with minibatch statistics (biased variance,
// eps passed in), first-maximum tie-break in max-pooling, ReLU'(0) = 0.
// Storage type T is float or double; every reduction (dot products, means,
// sums over the minibatch, log-sum-exp) is accumulated in double and rounded to
// T once.  There is no blocking, no fusion and no reordering beyond choosing
// which loop is outermost.
//
// Parity status: every function here is pinned by tests/test_oracle_*.py
// (closed forms, adjoint identities, library special cases, brute force,
// central finite differences of the double build).
#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>

namespace {

enum Kind { CONV = 0, BN = 1, RELU = 2, ADD = 3, MAXPOOL = 4, GAP = 5, FC = 6, SOFTMAX_CE = 7, BIAS = 8 };

struct LayerRec {  // same field order as the int32[9] record handed in
  int kind, in0, in1, cin, cout, r, s, stride, pad;
};

inline int out_dim(int in, int r, int stride, int pad) { return (in + 2 * pad - r) / stride + 1; }

// Output positions o in [lo, hi) are exactly those whose input coordinate
// o*stride + tap - pad falls inside [0, in): the zero padding contributes nothing.
inline void inside(int tap, int pad, int stride, int in, int out, int* lo, int* hi) {
  int a = 0, b = out;
  while (a < out && a * stride + tap - pad < 0) ++a;
  while (b > a && (b - 1) * stride + tap - pad >= in) --b;
  *lo = a;
  *hi = b;
}

// ---------------------------------------------------------------- convolution
// y[n,co,oy,ox] = sum_{ci,r,t} x[n,ci,oy*stride+r-pad,ox*stride+t-pad] * w[co,ci,r,t]
template <class T>
void conv_fwd(const T* x, const T* w, T* y, int n, int cin, int h, int wd, int cout, int r, int s,
              int stride, int pad) {
  const int ho = out_dim(h, r, stride, pad), wo = out_dim(wd, s, stride, pad);
#pragma omp parallel for collapse(2) schedule(static)
  for (int in = 0; in < n; ++in)
    for (int co = 0; co < cout; ++co) {
      std::vector<double> acc((size_t)ho * wo, 0.0);
      for (int ci = 0; ci < cin; ++ci)
        for (int kr = 0; kr < r; ++kr)
          for (int kt = 0; kt < s; ++kt) {
            const double wv = (double)w[(((size_t)co * cin + ci) * r + kr) * s + kt];
            int oy0, oy1, ox0, ox1;
            inside(kr, pad, stride, h, ho, &oy0, &oy1);
            inside(kt, pad, stride, wd, wo, &ox0, &ox1);
            for (int oy = oy0; oy < oy1; ++oy) {
              const int iy = oy * stride + kr - pad;
              const T* xrow = x + (((size_t)in * cin + ci) * h + iy) * wd + (kt - pad);
              double* arow = acc.data() + (size_t)oy * wo;
              for (int ox = ox0; ox < ox1; ++ox) arow[ox] += (double)xrow[ox * stride] * wv;
            }
          }
      T* yp = y + ((size_t)in * cout + co) * ho * wo;
      for (size_t i = 0; i < (size_t)ho * wo; ++i) yp[i] = (T)acc[i];
    }
}

// Adjoint of conv_fwd with respect to x:
// dx[n,ci,iy,ix] += sum over (co,r,t,oy,ox) with iy = oy*stride+r-pad, ix = ox*stride+t-pad
//                   of dy[n,co,oy,ox] * w[co,ci,r,t]
template <class T>
void conv_dgrad(const T* dy, const T* w, T* dx, int n, int cin, int h, int wd, int cout, int r,
                int s, int stride, int pad) {
  const int ho = out_dim(h, r, stride, pad), wo = out_dim(wd, s, stride, pad);
#pragma omp parallel for collapse(2) schedule(static)
  for (int in = 0; in < n; ++in)
    for (int ci = 0; ci < cin; ++ci) {
      std::vector<double> acc((size_t)h * wd, 0.0);
      for (int co = 0; co < cout; ++co)
        for (int kr = 0; kr < r; ++kr)
          for (int kt = 0; kt < s; ++kt) {
            const double wv = (double)w[(((size_t)co * cin + ci) * r + kr) * s + kt];
            int oy0, oy1, ox0, ox1;
            inside(kr, pad, stride, h, ho, &oy0, &oy1);
            inside(kt, pad, stride, wd, wo, &ox0, &ox1);
            for (int oy = oy0; oy < oy1; ++oy) {
              const int iy = oy * stride + kr - pad;
              const T* dyrow = dy + (((size_t)in * cout + co) * ho + oy) * wo;
              double* arow = acc.data() + (size_t)iy * wd + (kt - pad);
              for (int ox = ox0; ox < ox1; ++ox) arow[ox * stride] += (double)dyrow[ox] * wv;
            }
          }
      T* dxp = dx + ((size_t)in * cin + ci) * h * wd;
      for (size_t i = 0; i < (size_t)h * wd; ++i) dxp[i] = (T)((double)dxp[i] + acc[i]);
    }
}

// Adjoint of conv_fwd with respect to w:
// dw[co,ci,r,t] += sum_{n,oy,ox} dy[n,co,oy,ox] * x[n,ci,oy*stride+r-pad,ox*stride+t-pad]
template <class T>
void conv_wgrad(const T* x, const T* dy, T* dw, int n, int cin, int h, int wd, int cout, int r,
                int s, int stride, int pad) {
  const int ho = out_dim(h, r, stride, pad), wo = out_dim(wd, s, stride, pad);
#pragma omp parallel for collapse(2) schedule(static)
  for (int co = 0; co < cout; ++co)
    for (int ci = 0; ci < cin; ++ci)
      for (int kr = 0; kr < r; ++kr)
        for (int kt = 0; kt < s; ++kt) {
          int oy0, oy1, ox0, ox1;
          inside(kr, pad, stride, h, ho, &oy0, &oy1);
          inside(kt, pad, stride, wd, wo, &ox0, &ox1);
          double acc = 0.0;
          for (int in = 0; in < n; ++in)
            for (int oy = oy0; oy < oy1; ++oy) {
              const int iy = oy * stride + kr - pad;
              const T* xrow = x + (((size_t)in * cin + ci) * h + iy) * wd + (kt - pad);
              const T* dyrow = dy + (((size_t)in * cout + co) * ho + oy) * wo;
              for (int ox = ox0; ox < ox1; ++ox) acc += (double)dyrow[ox] * (double)xrow[ox * stride];
            }
          T& d = dw[(((size_t)co * cin + ci) * r + kr) * s + kt];
          d = (T)((double)d + acc);
        }
}

// ----------------------------------------------------------------- batch norm
// mean_c = (1/m) sum x, var_c = (1/m) sum (x-mean_c)^2 (biased), m = n*hw,
// istd_c = 1/sqrt(var_c+eps), y = gamma_c*(x-mean_c)*istd_c + beta_c.
template <class T>
void bn_fwd(const T* x, const T* gamma, const T* beta, T* y, double* mean, double* istd, int n,
            int c, int hw, double eps) {
  const double m = (double)n * hw;
#pragma omp parallel for schedule(static)
  for (int ch = 0; ch < c; ++ch) {
    double sum = 0.0;
    for (int in = 0; in < n; ++in) {
      const T* p = x + ((size_t)in * c + ch) * hw;
      for (int i = 0; i < hw; ++i) sum += (double)p[i];
    }
    const double mu = sum / m;
    double ss = 0.0;
    for (int in = 0; in < n; ++in) {
      const T* p = x + ((size_t)in * c + ch) * hw;
      for (int i = 0; i < hw; ++i) {
        const double d = (double)p[i] - mu;
        ss += d * d;
      }
    }
    const double is = 1.0 / std::sqrt(ss / m + eps);
    mean[ch] = mu;
    istd[ch] = is;
    for (int in = 0; in < n; ++in) {
      const T* p = x + ((size_t)in * c + ch) * hw;
      T* q = y + ((size_t)in * c + ch) * hw;
      for (int i = 0; i < hw; ++i)
        q[i] = (T)((double)gamma[ch] * (((double)p[i] - mu) * is) + (double)beta[ch]);
    }
  }
}

// xhat = (x-mean)*istd; dbeta = sum dy; dgamma = sum dy*xhat;
// dx += gamma*istd*(dy - dbeta/m - xhat*dgamma/m).
template <class T>
void bn_bwd(const T* x, const T* dy, const T* gamma, const double* mean, const double* istd, T* dx,
            T* dgamma, T* dbeta, int n, int c, int hw) {
  const double m = (double)n * hw;
#pragma omp parallel for schedule(static)
  for (int ch = 0; ch < c; ++ch) {
    const double mu = mean[ch], is = istd[ch];
    double db = 0.0, dg = 0.0;
    for (int in = 0; in < n; ++in) {
      const T* p = x + ((size_t)in * c + ch) * hw;
      const T* g = dy + ((size_t)in * c + ch) * hw;
      for (int i = 0; i < hw; ++i) {
        db += (double)g[i];
        dg += (double)g[i] * (((double)p[i] - mu) * is);
      }
    }
    dgamma[ch] = (T)((double)dgamma[ch] + dg);
    dbeta[ch] = (T)((double)dbeta[ch] + db);
    const double a = (double)gamma[ch] * is;
    for (int in = 0; in < n; ++in) {
      const T* p = x + ((size_t)in * c + ch) * hw;
      const T* g = dy + ((size_t)in * c + ch) * hw;
      T* q = dx + ((size_t)in * c + ch) * hw;
      for (int i = 0; i < hw; ++i) {
        const double xh = ((double)p[i] - mu) * is;
        q[i] = (T)((double)q[i] + a * ((double)g[i] - db / m - xh * dg / m));
      }
    }
  }
}

// ------------------------------------------------- ReLU, add, pooling, FC, loss
template <class T>
void relu_fwd(const T* x, T* y, size_t cnt) {
  for (size_t i = 0; i < cnt; ++i) y[i] = x[i] > (T)0 ? x[i] : (T)0;
}
template <class T>
void relu_bwd(const T* y, const T* dy, T* dx, size_t cnt) {
  for (size_t i = 0; i < cnt; ++i)
    if (y[i] > (T)0) dx[i] = (T)((double)dx[i] + (double)dy[i]);
}

// Max over the window positions that fall inside the image; the first maximum in
// (r, t) scan order wins.  arg holds the flat input offset iy*w+ix of the winner.
template <class T>
void maxpool_fwd(const T* x, T* y, int32_t* arg, int n, int c, int h, int wd, int r, int s,
                 int stride, int pad) {
  const int ho = out_dim(h, r, stride, pad), wo = out_dim(wd, s, stride, pad);
#pragma omp parallel for schedule(static)
  for (int pl = 0; pl < n * c; ++pl) {
    const T* xp = x + (size_t)pl * h * wd;
    for (int oy = 0; oy < ho; ++oy)
      for (int ox = 0; ox < wo; ++ox) {
        bool have = false;
        T best = (T)0;
        int where = -1;
        for (int kr = 0; kr < r; ++kr)
          for (int kt = 0; kt < s; ++kt) {
            const int iy = oy * stride + kr - pad, ix = ox * stride + kt - pad;
            if (iy < 0 || iy >= h || ix < 0 || ix >= wd) continue;
            const T v = xp[(size_t)iy * wd + ix];
            if (!have || v > best) {
              have = true;
              best = v;
              where = iy * wd + ix;
            }
          }
        y[((size_t)pl * ho + oy) * wo + ox] = best;
        arg[((size_t)pl * ho + oy) * wo + ox] = where;
      }
  }
}
template <class T>
void maxpool_bwd(const T* dy, const int32_t* arg, T* dx, int n, int c, int h, int wd, int ho,
                 int wo) {
#pragma omp parallel for schedule(static)
  for (int pl = 0; pl < n * c; ++pl) {
    T* dxp = dx + (size_t)pl * h * wd;
    for (int i = 0; i < ho * wo; ++i) {
      const int a = arg[(size_t)pl * ho * wo + i];
      if (a >= 0) dxp[a] = (T)((double)dxp[a] + (double)dy[(size_t)pl * ho * wo + i]);
    }
  }
}

template <class T>
void gap_fwd(const T* x, T* y, int n, int c, int hw) {
  for (int pl = 0; pl < n * c; ++pl) {
    double sum = 0.0;
    for (int i = 0; i < hw; ++i) sum += (double)x[(size_t)pl * hw + i];
    y[pl] = (T)(sum / hw);
  }
}
template <class T>
void gap_bwd(const T* dy, T* dx, int n, int c, int hw) {
  for (int pl = 0; pl < n * c; ++pl)
    for (int i = 0; i < hw; ++i) {
      T& d = dx[(size_t)pl * hw + i];
      d = (T)((double)d + (double)dy[pl] / hw);
    }
}

// y[n,o] = sum_i W[o,i]*x[n,i] + b[o];  param = [W (cout x cin) | b (cout)].
template <class T>
void fc_fwd(const T* x, const T* param, T* y, int n, int cin, int cout) {
  const T* b = param + (size_t)cout * cin;
#pragma omp parallel for schedule(static)
  for (int in = 0; in < n; ++in)
    for (int o = 0; o < cout; ++o) {
      double acc = 0.0;
      for (int i = 0; i < cin; ++i) acc += (double)param[(size_t)o * cin + i] * (double)x[(size_t)in * cin + i];
      y[(size_t)in * cout + o] = (T)(acc + (double)b[o]);
    }
}
template <class T>
void fc_bwd(const T* x, const T* param, const T* dy, T* dx, T* dparam, int n, int cin, int cout) {
  T* db = dparam + (size_t)cout * cin;
#pragma omp parallel for schedule(static)
  for (int o = 0; o < cout; ++o) {
    double sb = 0.0;
    for (int in = 0; in < n; ++in) sb += (double)dy[(size_t)in * cout + o];
    db[o] = (T)((double)db[o] + sb);
    for (int i = 0; i < cin; ++i) {
      double acc = 0.0;
      for (int in = 0; in < n; ++in) acc += (double)dy[(size_t)in * cout + o] * (double)x[(size_t)in * cin + i];
      T& d = dparam[(size_t)o * cin + i];
      d = (T)((double)d + acc);
    }
  }
#pragma omp parallel for schedule(static)
  for (int in = 0; in < n; ++in)
    for (int i = 0; i < cin; ++i) {
      double acc = 0.0;
      for (int o = 0; o < cout; ++o) acc += (double)dy[(size_t)in * cout + o] * (double)param[(size_t)o * cin + i];
      T& d = dx[(size_t)in * cin + i];
      d = (T)((double)d + acc);
    }
}

// loss = (1/n) sum_i [ log sum_j exp(z[i,j]) - z[i,label_i] ] (max-subtracted);
// dz[i,j] = (softmax(z_i)[j] - [j == label_i]) / n.
template <class T>
double softmax_ce(const T* z, const int32_t* label, T* dz, int n, int classes) {
  double loss = 0.0;
  for (int i = 0; i < n; ++i) {
    const T* zi = z + (size_t)i * classes;
    double mx = (double)zi[0];
    for (int j = 1; j < classes; ++j) mx = std::fmax(mx, (double)zi[j]);
    double se = 0.0;
    for (int j = 0; j < classes; ++j) se += std::exp((double)zi[j] - mx);
    const double lse = mx + std::log(se);
    loss += lse - (double)zi[label[i]];
    if (dz)
      for (int j = 0; j < classes; ++j) {
        const double p = std::exp((double)zi[j] - lse);
        dz[(size_t)i * classes + j] = (T)((p - (j == label[i] ? 1.0 : 0.0)) / n);
      }
  }
  return loss / n;
}

// --------------------------------------------------------------- whole network
struct Shape {
  int c, h, w;
  size_t per_image() const { return (size_t)c * h * w; }
};

// Executes the layer list in order, then its reverse, then theta <- theta - lr*grad.
// params[i] / grads[i]: one array per layer (conv OIHW; bn [gamma|beta]; fc [W|b]).
// grads and acts may be null; grads[i] receives d(loss)/d(params[i]) for the
// pre-update parameters, acts[i] the forward output of layer i.
// Returns 0, or -(1+i) if layer record i is malformed.
template <class T>
int train_step(const int32_t* recs, int nl, int in_c, int in_h, int in_w, int k, T** params,
               T** grads, T** acts, const T* images, const int32_t* labels, double lr, double eps,
               double* loss_out) {
  const LayerRec* L = reinterpret_cast<const LayerRec*>(recs);
  std::vector<Shape> shp(nl);
  std::vector<std::vector<T>> out(nl), gout(nl), gpar(nl);
  std::vector<std::vector<double>> mean(nl), istd(nl);
  std::vector<std::vector<int32_t>> arg(nl);
  auto in_shape = [&](int id) { return id < 0 ? Shape{in_c, in_h, in_w} : shp[id]; };
  auto in_data = [&](int id) -> const T* { return id < 0 ? images : out[id].data(); };
  double loss = 0.0;

  // forward
  for (int i = 0; i < nl; ++i) {
    const LayerRec& l = L[i];
    if (l.in0 >= i || l.in1 >= i) return -(1 + i);
    const Shape a = in_shape(l.in0);
    const T* x = in_data(l.in0);
    switch (l.kind) {
      case CONV:
        if (a.c != l.cin) return -(1 + i);
        shp[i] = {l.cout, out_dim(a.h, l.r, l.stride, l.pad), out_dim(a.w, l.s, l.stride, l.pad)};
        out[i].assign(k * shp[i].per_image(), (T)0);
        conv_fwd(x, params[i], out[i].data(), k, l.cin, a.h, a.w, l.cout, l.r, l.s, l.stride, l.pad);
        break;
      case BN:
        if (a.c != l.cin) return -(1 + i);
        shp[i] = a;
        out[i].assign(k * a.per_image(), (T)0);
        mean[i].assign(a.c, 0.0);
        istd[i].assign(a.c, 0.0);
        bn_fwd(x, params[i], params[i] + a.c, out[i].data(), mean[i].data(), istd[i].data(), k, a.c,
               a.h * a.w, eps);
        break;
      case RELU:
        shp[i] = a;
        out[i].assign(k * a.per_image(), (T)0);
        relu_fwd(x, out[i].data(), out[i].size());
        break;
      case BIAS: {
        // y[n,c,h,w] = x[n,c,h,w] + b[c]
        if (a.c != l.cin) return -(1 + i);
        shp[i] = a;
        out[i].resize(k * a.per_image());
        const size_t hw = (size_t)a.h * a.w;
        for (size_t e = 0; e < out[i].size(); ++e) out[i][e] = (T)((double)x[e] + (double)params[i][(e / hw) % a.c]);
        break;
      }
      case ADD: {
        const Shape b = in_shape(l.in1);
        if (a.c != b.c || a.h != b.h || a.w != b.w) return -(1 + i);
        shp[i] = a;
        out[i].resize(k * a.per_image());
        const T* x1 = in_data(l.in1);
        for (size_t e = 0; e < out[i].size(); ++e) out[i][e] = x[e] + x1[e];
        break;
      }
      case MAXPOOL:
        shp[i] = {a.c, out_dim(a.h, l.r, l.stride, l.pad), out_dim(a.w, l.s, l.stride, l.pad)};
        out[i].assign(k * shp[i].per_image(), (T)0);
        arg[i].assign(out[i].size(), -1);
        maxpool_fwd(x, out[i].data(), arg[i].data(), k, a.c, a.h, a.w, l.r, l.s, l.stride, l.pad);
        break;
      case GAP:
        shp[i] = {a.c, 1, 1};
        out[i].assign((size_t)k * a.c, (T)0);
        gap_fwd(x, out[i].data(), k, a.c, a.h * a.w);
        break;
      case FC:
        if ((int)a.per_image() != l.cin) return -(1 + i);
        shp[i] = {l.cout, 1, 1};
        out[i].assign((size_t)k * l.cout, (T)0);
        fc_fwd(x, params[i], out[i].data(), k, l.cin, l.cout);
        break;
      case SOFTMAX_CE:
        shp[i] = {1, 1, 1};
        if (l.in0 < 0) return -(1 + i);
        gout[l.in0].assign(out[l.in0].size(), (T)0);
        loss = softmax_ce(x, labels, gout[l.in0].data(), k, (int)a.per_image());
        out[i].assign(1, (T)loss);
        break;
      default:
        return -(1 + i);
    }
  }
  if (loss_out) *loss_out = loss;
  if (acts)
    for (int i = 0; i < nl; ++i)
      if (acts[i]) std::memcpy(acts[i], out[i].data(), out[i].size() * sizeof(T));

  // backward: gout[i] = d(loss)/d(out[i]), summed over the consumers of out[i]
  auto grad_of = [&](int id) -> T* {
    if (id < 0) return nullptr;  // the gradient of the images is not needed
    if (gout[id].empty()) gout[id].assign(out[id].size(), (T)0);
    return gout[id].data();
  };
  for (int i = nl - 1; i >= 0; --i) {
    const LayerRec& l = L[i];
    if (l.kind == SOFTMAX_CE) continue;
    if (gout[i].empty()) continue;  // output unused by the loss
    const Shape a = in_shape(l.in0);
    const T* x = in_data(l.in0);
    const T* dy = gout[i].data();
    T* dx = grad_of(l.in0);
    switch (l.kind) {
      case CONV:
        gpar[i].assign((size_t)l.cout * l.cin * l.r * l.s, (T)0);
        conv_wgrad(x, dy, gpar[i].data(), k, l.cin, a.h, a.w, l.cout, l.r, l.s, l.stride, l.pad);
        if (dx) conv_dgrad(dy, params[i], dx, k, l.cin, a.h, a.w, l.cout, l.r, l.s, l.stride, l.pad);
        break;
      case BN: {
        gpar[i].assign(2 * (size_t)a.c, (T)0);
        std::vector<T> scratch;
        if (!dx) { scratch.assign(out[i].size(), (T)0); dx = scratch.data(); }
        bn_bwd(x, dy, params[i], mean[i].data(), istd[i].data(), dx, gpar[i].data(),
               gpar[i].data() + a.c, k, a.c, a.h * a.w);
        break;
      }
      case RELU:
        if (dx) relu_bwd(out[i].data(), dy, dx, out[i].size());
        break;
      case BIAS: {
        // db[c] = sum over n, h, w of dy; dx += dy
        gpar[i].assign((size_t)a.c, (T)0);
        const size_t hw = (size_t)a.h * a.w;
        std::vector<double> db((size_t)a.c, 0.0);
        for (size_t e = 0; e < out[i].size(); ++e) db[(e / hw) % a.c] += (double)dy[e];
        for (int c = 0; c < a.c; ++c) gpar[i][c] = (T)db[c];
        if (dx)
          for (size_t e = 0; e < out[i].size(); ++e) dx[e] = (T)((double)dx[e] + (double)dy[e]);
        break;
      }
      case ADD: {
        T* dx1 = grad_of(l.in1);
        for (size_t e = 0; e < out[i].size(); ++e) {
          if (dx) dx[e] = (T)((double)dx[e] + (double)dy[e]);
          if (dx1) dx1[e] = (T)((double)dx1[e] + (double)dy[e]);
        }
        break;
      }
      case MAXPOOL:
        if (dx) maxpool_bwd(dy, arg[i].data(), dx, k, a.c, a.h, a.w, shp[i].h, shp[i].w);
        break;
      case GAP:
        if (dx) gap_bwd(dy, dx, k, a.c, a.h * a.w);
        break;
      case FC: {
        gpar[i].assign((size_t)l.cout * l.cin + l.cout, (T)0);
        std::vector<T> scratch;
        if (!dx) { scratch.assign((size_t)k * l.cin, (T)0); dx = scratch.data(); }
        fc_bwd(x, params[i], dy, dx, gpar[i].data(), k, l.cin, l.cout);
        break;
      }
      default:
        break;
    }
    std::vector<T>().swap(gout[i]);
  }

  // plain SGD on every parameter (Sec. 4.2 discusses only the learning rate; no
  // momentum or weight decay is part of the step)
  for (int i = 0; i < nl; ++i) {
    if (grads && grads[i] && !gpar[i].empty())
      std::memcpy(grads[i], gpar[i].data(), gpar[i].size() * sizeof(T));
    for (size_t e = 0; e < gpar[i].size(); ++e)
      params[i][e] = (T)((double)params[i][e] - lr * (double)gpar[i][e]);
  }
  return 0;
}

}  // namespace

#define ORACLE_API(T, SFX)                                                                          \
  void oracle_conv_fwd_##SFX(const T* x, const T* w, T* y, int n, int cin, int h, int wd, int cout, \
                             int r, int s, int stride, int pad) {                                   \
    conv_fwd<T>(x, w, y, n, cin, h, wd, cout, r, s, stride, pad);                                   \
  }                                                                                                 \
  void oracle_conv_dgrad_##SFX(const T* dy, const T* w, T* dx, int n, int cin, int h, int wd,       \
                               int cout, int r, int s, int stride, int pad) {                       \
    conv_dgrad<T>(dy, w, dx, n, cin, h, wd, cout, r, s, stride, pad);                               \
  }                                                                                                 \
  void oracle_conv_wgrad_##SFX(const T* x, const T* dy, T* dw, int n, int cin, int h, int wd,       \
                               int cout, int r, int s, int stride, int pad) {                       \
    conv_wgrad<T>(x, dy, dw, n, cin, h, wd, cout, r, s, stride, pad);                               \
  }                                                                                                 \
  void oracle_bn_fwd_##SFX(const T* x, const T* gamma, const T* beta, T* y, double* mean,           \
                           double* istd, int n, int c, int hw, double eps) {                        \
    bn_fwd<T>(x, gamma, beta, y, mean, istd, n, c, hw, eps);                                        \
  }                                                                                                 \
  void oracle_bn_bwd_##SFX(const T* x, const T* dy, const T* gamma, const double* mean,             \
                           const double* istd, T* dx, T* dgamma, T* dbeta, int n, int c, int hw) {  \
    bn_bwd<T>(x, dy, gamma, mean, istd, dx, dgamma, dbeta, n, c, hw);                               \
  }                                                                                                 \
  void oracle_relu_fwd_##SFX(const T* x, T* y, size_t cnt) { relu_fwd<T>(x, y, cnt); }              \
  void oracle_relu_bwd_##SFX(const T* y, const T* dy, T* dx, size_t cnt) {                          \
    relu_bwd<T>(y, dy, dx, cnt);                                                                    \
  }                                                                                                 \
  void oracle_maxpool_fwd_##SFX(const T* x, T* y, int32_t* arg, int n, int c, int h, int wd, int r, \
                                int s, int stride, int pad) {                                       \
    maxpool_fwd<T>(x, y, arg, n, c, h, wd, r, s, stride, pad);                                      \
  }                                                                                                 \
  void oracle_maxpool_bwd_##SFX(const T* dy, const int32_t* arg, T* dx, int n, int c, int h,        \
                                int wd, int ho, int wo) {                                           \
    maxpool_bwd<T>(dy, arg, dx, n, c, h, wd, ho, wo);                                               \
  }                                                                                                 \
  void oracle_gap_fwd_##SFX(const T* x, T* y, int n, int c, int hw) { gap_fwd<T>(x, y, n, c, hw); } \
  void oracle_gap_bwd_##SFX(const T* dy, T* dx, int n, int c, int hw) {                             \
    gap_bwd<T>(dy, dx, n, c, hw);                                                                   \
  }                                                                                                 \
  void oracle_fc_fwd_##SFX(const T* x, const T* param, T* y, int n, int cin, int cout) {            \
    fc_fwd<T>(x, param, y, n, cin, cout);                                                           \
  }                                                                                                 \
  void oracle_fc_bwd_##SFX(const T* x, const T* param, const T* dy, T* dx, T* dparam, int n,        \
                           int cin, int cout) {                                                     \
    fc_bwd<T>(x, param, dy, dx, dparam, n, cin, cout);                                              \
  }                                                                                                 \
  double oracle_softmax_ce_##SFX(const T* z, const int32_t* label, T* dz, int n, int classes) {     \
    return softmax_ce<T>(z, label, dz, n, classes);                                                 \
  }                                                                                                 \
  int oracle_train_step_##SFX(const int32_t* recs, int nl, int in_c, int in_h, int in_w, int k,     \
                              T** params, T** grads, T** acts, const T* images,                     \
                              const int32_t* labels, double lr, double eps, double* loss_out) {     \
    return train_step<T>(recs, nl, in_c, in_h, in_w, k, params, grads, acts, images, labels, lr,    \
                         eps, loss_out);                                                            \
  }

extern "C" {
ORACLE_API(float, f32)
ORACLE_API(double, f64)
}
