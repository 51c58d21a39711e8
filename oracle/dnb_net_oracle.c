/*
 * dnb_net_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain float64 CPU reference of a whole CIFAR-shaped DenseNet-BC training step
 * (forward, mean softmax cross-entropy, reverse-mode gradients of every
 * parameter): the glue around the dense blocks of dnb_oracle.c.  Shares no code
 * with the GPU library.
 *
 * Network (paper Section 2, "DenseNet Architecture": dense blocks joined by
 * transition layers; Section 5 trains the BC form on 32x32 inputs.  The paper
 * defers the remaining details to the original DenseNet description; readings
 * listed in the design notes):
 *   stem      3x3 conv, pad 1, 3 -> 2k channels, no bias, no BN/ReLU
 *   3 x       dense block of (L-4)/6 bottleneck layers (dnbo_block_naive)
 *   between   transition: BN -> ReLU -> 1x1 conv (C -> floor(C/2)) -> 2x2 average pool, stride 2
 *   tail      BN -> ReLU -> global average pool -> linear (+bias) to `classes`
 *   loss      mean over the batch of -log softmax(logits)[label]
 * BN is train-mode (batch statistics, biased variance, eps inside the root).
 *
 * Parameter pack (float64 here, fp32 on the GPU; gradients same layout):
 *   stem W[2k][3][3][3]
 *   block1 | trans1: g[C] b[C] W[C/2][C] | block2 | trans2 | block3
 *   tail: g[C] b[C] Wl[classes][C] bl[classes]
 * with each block in dnb_oracle.c's own pack layout.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
  int32_t n, c0, h, w, layers, growth, bottleneck;
  double eps;
} dnbo_desc;
typedef struct { int64_t peak_elems, stored_elems, live_elems; } dnbo_mem;

/* primitives and the block from dnb_oracle.c */
void dnbo_bn_forward(const double* u, int64_t n, int64_t c, int64_t hw, const double* gamma,
                     const double* beta, double eps, double* z, double* mean, double* var);
void dnbo_bn_backward(const double* u, const double* dz, int64_t n, int64_t c, int64_t hw,
                      const double* gamma, const double* mean, const double* var, double eps,
                      double* du, double* dgamma, double* dbeta);
void dnbo_relu_inplace(double* z, int64_t count);
void dnbo_relu_backward(const double* a, const double* da, double* dz, int64_t count);
void dnbo_conv_forward(const double* in, const double* wgt, int64_t n, int64_t ci, int64_t co,
                       int64_t h, int64_t w, int64_t ks, double* out);
void dnbo_conv_dgrad(const double* dout, const double* wgt, int64_t n, int64_t ci, int64_t co,
                     int64_t h, int64_t w, int64_t ks, double* din);
void dnbo_conv_wgrad(const double* in, const double* dout, int64_t n, int64_t ci, int64_t co,
                     int64_t h, int64_t w, int64_t ks, double* dwgt);
int64_t dnbo_param_count(const dnbo_desc* d);
int dnbo_block_naive(const dnbo_desc* d, const double* x0, const double* params, const double* dy,
                     double* y, double* dx0, double* dparams, dnbo_mem* mem);
/* the block with its ReLU decisions written out (mode 0) or imposed (mode 1), and the two
 * element-wise routines it uses for that */
int dnbo_block_naive_masks(const dnbo_desc* d, const double* x0, const double* params, const double* dy,
                           double* y, double* dx0, double* dparams, dnbo_mem* mem, int mode, uint8_t* m1,
                           uint8_t* m2, double* stats, int bf16_storage);
void dnbo_relu_with_decisions(double* z, int64_t n, int64_t c, int64_t hw, const double* gamma,
                              const double* beta, uint8_t* mask, int mode, double* stat);
void dnbo_relu_backward_decisions(const uint8_t* mask, const double* da, double* dz, int64_t count);

typedef struct {
  int32_t n, image;   /* batch, input height = width (3 channels) */
  int32_t depth;      /* L = 6*per + 4 */
  int32_t growth;     /* k; bottleneck width 4k, stem width 2k */
  int32_t classes;
  double eps;
} dnbo_net_desc;

/* ---------------------------------------------------------------- glue primitives */

/* 2x2 average pooling, stride 2 (h, w even): out (n,c,h/2,w/2). */
void dnbo_avgpool2(const double* in, int64_t n, int64_t c, int64_t h, int64_t w, double* out) {
  const int64_t ho = h / 2, wo = w / 2;
  for (int64_t p = 0; p < n * c; ++p)
    for (int64_t y = 0; y < ho; ++y)
      for (int64_t x = 0; x < wo; ++x) {
        const double* s = in + p * h * w + (2 * y) * w + 2 * x;
        out[p * ho * wo + y * wo + x] = 0.25 * (s[0] + s[1] + s[w] + s[w + 1]);
      }
}

/* Adjoint: every input pixel receives a quarter of its window's gradient. */
void dnbo_avgpool2_backward(const double* dout, int64_t n, int64_t c, int64_t h, int64_t w, double* din) {
  const int64_t ho = h / 2, wo = w / 2;
  for (int64_t p = 0; p < n * c; ++p)
    for (int64_t y = 0; y < h; ++y)
      for (int64_t x = 0; x < w; ++x)
        din[p * h * w + y * w + x] = 0.25 * dout[p * ho * wo + (y / 2) * wo + (x / 2)];
}

/* Global average pool: out (n,c) = mean over hw. */
void dnbo_global_avgpool(const double* in, int64_t n, int64_t c, int64_t hw, double* out) {
  for (int64_t p = 0; p < n * c; ++p) {
    double s = 0.0;
    for (int64_t q = 0; q < hw; ++q) s += in[p * hw + q];
    out[p] = s / (double)hw;
  }
}

void dnbo_global_avgpool_backward(const double* dout, int64_t n, int64_t c, int64_t hw, double* din) {
  for (int64_t p = 0; p < n * c; ++p)
    for (int64_t q = 0; q < hw; ++q) din[p * hw + q] = dout[p] / (double)hw;
}

/* logits (n,classes) = f (n,c) . Wl^T + bl */
void dnbo_linear(const double* f, const double* wl, const double* bl, int64_t n, int64_t c, int64_t classes,
                 double* logits) {
  for (int64_t i = 0; i < n; ++i)
    for (int64_t o = 0; o < classes; ++o) {
      double s = bl[o];
      for (int64_t j = 0; j < c; ++j) s += wl[o * c + j] * f[i * c + j];
      logits[i * classes + o] = s;
    }
}

void dnbo_linear_backward(const double* f, const double* wl, const double* dlogits, int64_t n, int64_t c,
                          int64_t classes, double* df, double* dwl, double* dbl) {
  for (int64_t i = 0; i < n; ++i)
    for (int64_t j = 0; j < c; ++j) {
      double s = 0.0;
      for (int64_t o = 0; o < classes; ++o) s += dlogits[i * classes + o] * wl[o * c + j];
      df[i * c + j] = s;
    }
  for (int64_t o = 0; o < classes; ++o) {
    double sb = 0.0;
    for (int64_t i = 0; i < n; ++i) sb += dlogits[i * classes + o];
    dbl[o] = sb;
    for (int64_t j = 0; j < c; ++j) {
      double s = 0.0;
      for (int64_t i = 0; i < n; ++i) s += dlogits[i * classes + o] * f[i * c + j];
      dwl[o * c + j] = s;
    }
  }
}

/* Mean softmax cross-entropy and its gradient w.r.t. the logits:
 * loss = -(1/n) sum_i log softmax(logits_i)[label_i];  dlogits = (softmax - onehot)/n. */
double dnbo_softmax_xent(const double* logits, const int32_t* labels, int64_t n, int64_t classes,
                         double* dlogits) {
  double loss = 0.0;
  for (int64_t i = 0; i < n; ++i) {
    const double* z = logits + i * classes;
    double mx = z[0];
    for (int64_t o = 1; o < classes; ++o) mx = z[o] > mx ? z[o] : mx;
    double se = 0.0;
    for (int64_t o = 0; o < classes; ++o) se += exp(z[o] - mx);
    const double lse = mx + log(se);
    loss += lse - z[labels[i]];
    if (dlogits)
      for (int64_t o = 0; o < classes; ++o)
        dlogits[i * classes + o] = (exp(z[o] - lse) - (o == labels[i] ? 1.0 : 0.0)) / (double)n;
  }
  return loss / (double)n;
}

/* ---------------------------------------------------------------- the network */

static dnbo_desc block_desc(const dnbo_net_desc* d, int b, int64_t* c_in_out) {
  const int per = (d->depth - 4) / 6;
  int64_t c = 2 * d->growth, s = d->image;
  for (int i = 0; i < b; ++i) { c = (c + (int64_t)per * d->growth) / 2; s /= 2; }
  dnbo_desc bd = {d->n, (int32_t)c, (int32_t)s, (int32_t)s, per, d->growth, 4 * d->growth, d->eps};
  if (c_in_out) *c_in_out = c + (int64_t)per * d->growth;
  return bd;
}

/* Offsets into the pack: stem, then per block b: block params, then (b < 2) transition g, b, W;
 * then tail g, b, Wl, bl.  which: 0 stem | 1+3b block b | 2+3b trans b (g) | 10 tail g. */
int64_t dnbo_net_param_count(const dnbo_net_desc* d) {
  int64_t t = (int64_t)2 * d->growth * 27;
  for (int b = 0; b < 3; ++b) {
    int64_t cout;
    dnbo_desc bd = block_desc(d, b, &cout);
    t += dnbo_param_count(&bd);
    if (b < 2) t += 2 * cout + (cout / 2) * cout;
    else t += 2 * cout + (int64_t)d->classes * cout + d->classes;
  }
  return t;
}

int64_t dnbo_net_block_param_offset(const dnbo_net_desc* d, int b) {
  int64_t t = (int64_t)2 * d->growth * 27;
  for (int i = 0; i < b; ++i) {
    int64_t cout;
    dnbo_desc bd = block_desc(d, i, &cout);
    t += dnbo_param_count(&bd) + 2 * cout + (cout / 2) * cout;
  }
  return t;
}

/* Bytes of the network's ReLU decisions, in the order they are laid out: for block b = 0, 1, 2
 * the block's first-BN decisions (all layers), its second-BN decisions (all layers), then the
 * decisions of the BN+ReLU that follows the block (transition b or the tail), (n, C_out_b, hw). */
int64_t dnbo_net_decision_count(const dnbo_net_desc* d) {
  int64_t t = 0;
  for (int b = 0; b < 3; ++b) {
    int64_t cout;
    dnbo_desc bd = block_desc(d, b, &cout);
    const int64_t P = (int64_t)bd.n * bd.h * bd.w;
    int64_t sigma = 0;
    for (int l = 1; l <= bd.layers; ++l) sigma += bd.c0 + (int64_t)(l - 1) * bd.growth;
    t += (sigma + (int64_t)bd.layers * bd.bottleneck + cout) * P;
  }
  return t;
}

static double net_step_impl(const dnbo_net_desc* d, const double* x, const int32_t* labels, const double* params,
                            double* dparams, double* logits_out, int use_masks, int mode, uint8_t* masks, double* stats);

/* One training step.  x (n,3,image,image), labels (n).  Returns the loss; writes dparams (whole
 * pack) and, if logits_out != NULL, the logits (n,classes). */
double dnbo_net_step(const dnbo_net_desc* d, const double* x, const int32_t* labels, const double* params,
                     double* dparams, double* logits_out) {
  return net_step_impl(d, x, labels, params, dparams, logits_out, 0, 0, NULL, NULL);
}

/* The same step with every ReLU decision written to `masks` (mode 0) or taken from it (mode 1);
 * layout as for dnbo_net_decision_count.  stats (mode 1, 2 doubles): how many of the given
 * decisions differ from the step's own, and the largest margin |z| / sqrt(gamma^2 + beta^2) among
 * those (see dnb_oracle.c). */
double dnbo_net_step_masks(const dnbo_net_desc* d, const double* x, const int32_t* labels, const double* params,
                           double* dparams, double* logits_out, int mode, uint8_t* masks, double* stats) {
  return net_step_impl(d, x, labels, params, dparams, logits_out, 1, mode, masks, stats);
}

static double net_step_impl(const dnbo_net_desc* d, const double* x, const int32_t* labels, const double* params,
                            double* dparams, double* logits_out, int use_masks, int mode, uint8_t* masks, double* stats) {
  uint8_t *mb1[3], *mb2[3], *mg[3]; /* where block b's and its following BN's decisions sit */
  double st_acc[2] = {0.0, 0.0};
  const int64_t n = d->n, k = d->growth, S = d->image;
  const double* stemW = params;
  double* dstemW = dparams;
  /* ---- forward */
  double* feat[3];   /* block inputs  */
  double* yb[3];     /* block outputs */
  double* tz[3];     /* BN output after ReLU of transition b / tail */
  double* tmu[3];
  double* tvar[3];
  double* tconv[2];  /* transition conv outputs (before pooling) */
  dnbo_desc bd[3];
  int64_t cout[3];
  feat[0] = (double*)malloc((size_t)(n * 2 * k * S * S) * sizeof(double));
  dnbo_conv_forward(x, stemW, n, 3, 2 * k, S, S, 3, feat[0]);
  {
    uint8_t* mp = masks;
    for (int b = 0; b < 3; ++b) {
      bd[b] = block_desc(d, b, &cout[b]);
      const int64_t P = n * bd[b].h * bd[b].w;
      int64_t sigma = 0;
      for (int l = 1; l <= bd[b].layers; ++l) sigma += bd[b].c0 + (int64_t)(l - 1) * bd[b].growth;
      mb1[b] = mp; mp += use_masks ? sigma * P : 0;
      mb2[b] = mp; mp += use_masks ? (int64_t)bd[b].layers * bd[b].bottleneck * P : 0;
      mg[b] = mp;  mp += use_masks ? cout[b] * P : 0;
    }
  }
  for (int b = 0; b < 3; ++b) {
    const int64_t hw = (int64_t)bd[b].h * bd[b].w;
    const double* bp = params + dnbo_net_block_param_offset(d, b);
    yb[b] = (double*)malloc((size_t)(n * cout[b] * hw) * sizeof(double));
    if (use_masks) {
      double bst[4];
      dnbo_block_naive_masks(&bd[b], feat[b], bp, NULL, yb[b], NULL, NULL, NULL, mode, mb1[b], mb2[b], bst, 0);
      if (mode == 1) {
        st_acc[0] += bst[0] + bst[2];
        if (bst[1] > st_acc[1]) st_acc[1] = bst[1];
        if (bst[3] > st_acc[1]) st_acc[1] = bst[3];
      }
    } else {
      dnbo_block_naive(&bd[b], feat[b], bp, NULL, yb[b], NULL, NULL, NULL);
    }
    const double* tp = bp + dnbo_param_count(&bd[b]);  /* g, b, then W or Wl, bl */
    tz[b] = (double*)malloc((size_t)(n * cout[b] * hw) * sizeof(double));
    tmu[b] = (double*)malloc((size_t)cout[b] * sizeof(double));
    tvar[b] = (double*)malloc((size_t)cout[b] * sizeof(double));
    dnbo_bn_forward(yb[b], n, cout[b], hw, tp, tp + cout[b], d->eps, tz[b], tmu[b], tvar[b]);
    if (use_masks)
      dnbo_relu_with_decisions(tz[b], n, cout[b], hw, tp, tp + cout[b], mg[b], mode, st_acc);
    else
      dnbo_relu_inplace(tz[b], n * cout[b] * hw);
    if (b < 2) {
      const int64_t ch = cout[b] / 2;
      tconv[b] = (double*)malloc((size_t)(n * ch * hw) * sizeof(double));
      dnbo_conv_forward(tz[b], tp + 2 * cout[b], n, cout[b], ch, bd[b].h, bd[b].w, 1, tconv[b]);
      feat[b + 1] = (double*)malloc((size_t)(n * ch * hw / 4) * sizeof(double));
      dnbo_avgpool2(tconv[b], n, ch, bd[b].h, bd[b].w, feat[b + 1]);
    }
  }
  const int64_t C = cout[2], hw2 = (int64_t)bd[2].h * bd[2].w;
  const double* tailp = params + dnbo_net_block_param_offset(d, 2) + dnbo_param_count(&bd[2]);
  const double* Wl = tailp + 2 * C;
  const double* bl = Wl + (int64_t)d->classes * C;
  double* pooled = (double*)malloc((size_t)(n * C) * sizeof(double));
  dnbo_global_avgpool(tz[2], n, C, hw2, pooled);
  double* logits = (double*)malloc((size_t)(n * d->classes) * sizeof(double));
  dnbo_linear(pooled, Wl, bl, n, C, d->classes, logits);
  double* dlogits = (double*)malloc((size_t)(n * d->classes) * sizeof(double));
  const double loss = dnbo_softmax_xent(logits, labels, n, d->classes, dparams ? dlogits : NULL);
  if (logits_out) memcpy(logits_out, logits, (size_t)(n * d->classes) * sizeof(double));

  /* ---- backward */
  if (dparams) {
    double* dtail = dparams + (tailp - params);
    double* dpooled = (double*)malloc((size_t)(n * C) * sizeof(double));
    dnbo_linear_backward(pooled, Wl, dlogits, n, C, d->classes, dpooled, dtail + 2 * C,
                         dtail + 2 * C + (int64_t)d->classes * C);
    double* g = (double*)malloc((size_t)(n * C * hw2) * sizeof(double)); /* gradient w.r.t. tz[2], then yb[2] */
    dnbo_global_avgpool_backward(dpooled, n, C, hw2, g);
    free(dpooled);
    for (int b = 2; b >= 0; --b) {
      const int64_t hw = (int64_t)bd[b].h * bd[b].w;
      const int64_t boff = dnbo_net_block_param_offset(d, b);
      const double* tp = params + boff + dnbo_param_count(&bd[b]);
      double* dtp = dparams + boff + dnbo_param_count(&bd[b]);
      /* g = gradient of the BN+ReLU output of this block's transition / tail */
      if (use_masks && mode == 1)
        dnbo_relu_backward_decisions(mg[b], g, g, n * cout[b] * hw);
      else
        dnbo_relu_backward(tz[b], g, g, n * cout[b] * hw);
      dnbo_bn_backward(yb[b], g, n, cout[b], hw, tp, tmu[b], tvar[b], d->eps, g, dtp, dtp + cout[b]);
      /* g = gradient of the block output */
      const int64_t cin = bd[b].c0;
      double* dfeat = (double*)malloc((size_t)(n * cin * hw) * sizeof(double));
      double* ydummy = (double*)malloc((size_t)(n * cout[b] * hw) * sizeof(double));
      if (use_masks && mode == 1) {
        double bst[4];  /* (the forward pass above has already counted this block's disagreements) */
        dnbo_block_naive_masks(&bd[b], feat[b], params + boff, g, ydummy, dfeat, dparams + boff, NULL, 1, mb1[b], mb2[b], bst, 0);
      } else {
        dnbo_block_naive(&bd[b], feat[b], params + boff, g, ydummy, dfeat, dparams + boff, NULL);
      }
      free(ydummy);
      free(g);
      if (b == 0) {
        dnbo_conv_wgrad(x, dfeat, n, 3, 2 * k, S, S, 3, dstemW);
        free(dfeat);
      } else {
        /* through the previous transition: pool backward, 1x1 conv backward */
        const int64_t hp = bd[b - 1].h, wp = bd[b - 1].w, cp = cout[b - 1], ch = cp / 2;
        const double* tpp = params + dnbo_net_block_param_offset(d, b - 1) + dnbo_param_count(&bd[b - 1]);
        double* dtpp = dparams + (tpp - params);
        double* dconv = (double*)malloc((size_t)(n * ch * hp * wp) * sizeof(double));
        dnbo_avgpool2_backward(dfeat, n, ch, hp, wp, dconv);
        free(dfeat);
        dnbo_conv_wgrad(tz[b - 1], dconv, n, cp, ch, hp, wp, 1, dtpp + 2 * cp);
        g = (double*)malloc((size_t)(n * cp * hp * wp) * sizeof(double));
        dnbo_conv_dgrad(dconv, tpp + 2 * cp, n, cp, ch, hp, wp, 1, g);
        free(dconv);
      }
    }
  }
  for (int b = 0; b < 3; ++b) { free(feat[b]); free(yb[b]); free(tz[b]); free(tmu[b]); free(tvar[b]); }
  free(tconv[0]); free(tconv[1]); free(pooled); free(logits); free(dlogits);
  if (use_masks && mode == 1 && stats) { stats[0] = st_acc[0]; stats[1] = st_acc[1]; }
  return loss;
}
