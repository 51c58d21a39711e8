/*
 * dnb_inet_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain float64 CPU reference of one training step (forward + backward) of an ImageNet-shaped
 * DenseNet-BC built around four dense blocks of dnb_oracle.c (paper, Section 2, "DenseNet
 * Architecture": dense blocks joined by pooling layers; Section 5's ImageNet models have four
 * dense blocks):
 *   stem      7x7 conv, stride 2, pad 3, 3 -> 2k channels, no bias; BN -> ReLU;
 *             3x3 max pool, stride 2, pad 1
 *   4 x       dense block of layers[b] bottleneck layers (B = 4k)
 *   between   transition: BN -> ReLU -> 1x1 conv (C -> C/2) -> 2x2 average pool, stride 2
 *   tail      BN -> ReLU -> global average pool -> linear (+bias) to `classes`
 *   loss      mean softmax cross-entropy
 * BN is train-mode batch statistics as in the blocks.  Shares no code with the GPU library.
 *
 * Two kinds of integer decided by floating point occur: the ReLU decisions (see dnb_oracle.c)
 * and the position of the maximum inside each pooling window.  Ties (frequent among values stored
 * with an 8-bit significand) go to the first position in scan order (row by row inside the
 * window).  Both kinds can be written out or imposed (mode 0 / 1); imposed decisions that differ
 * from the step's own are counted and their margin reported.
 *
 * bf16_storage != 0 rounds every tensor that the bf16 path keeps in memory to bfloat16 where it is
 * produced (stem output, pooled features, transition conv outputs and inputs, the gradients
 * between the pieces), as dnbo_block_naive_bf16 does inside the blocks: it measures what bf16
 * storage costs by itself.
 *
 * Parameter pack (doubles; gradients in the same layout):
 *   stem W[2k][3][7][7]  g[2k] b[2k] | block 0 | trans 0: g[C] b[C] W[C/2][C] | block 1 | trans 1 |
 *   block 2 | trans 2 | block 3 | tail: g[C] b[C] Wl[classes][C] bl[classes]
 * Layout NCHW, row-major.
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

/* from dnb_oracle.c and dnb_net_oracle.c */
void dnbo_bn_forward(const double* u, int64_t n, int64_t c, int64_t hw, const double* gamma,
                     const double* beta, double eps, double* z, double* mean, double* var);
void dnbo_bn_backward(const double* u, const double* dz, int64_t n, int64_t c, int64_t hw,
                      const double* gamma, const double* mean, const double* var, double eps,
                      double* du, double* dgamma, double* dbeta);
void dnbo_relu_inplace(double* z, int64_t count);
void dnbo_relu_backward(const double* a, const double* da, double* dz, int64_t count);
void dnbo_relu_with_decisions(double* z, int64_t n, int64_t c, int64_t hw, const double* gamma,
                              const double* beta, uint8_t* mask, int mode, double* stat);
void dnbo_relu_backward_decisions(const uint8_t* mask, const double* da, double* dz, int64_t count);
void dnbo_conv_forward(const double* in, const double* wgt, int64_t n, int64_t ci, int64_t co,
                       int64_t h, int64_t w, int64_t ks, double* out);
void dnbo_conv_dgrad(const double* dout, const double* wgt, int64_t n, int64_t ci, int64_t co,
                     int64_t h, int64_t w, int64_t ks, double* din);
void dnbo_conv_wgrad(const double* in, const double* dout, int64_t n, int64_t ci, int64_t co,
                     int64_t h, int64_t w, int64_t ks, double* dwgt);
int64_t dnbo_param_count(const dnbo_desc* d);
int dnbo_block_naive(const dnbo_desc* d, const double* x0, const double* params, const double* dy,
                     double* y, double* dx0, double* dparams, dnbo_mem* mem);
int dnbo_block_naive_bf16(const dnbo_desc* d, const double* x0, const double* params, const double* dy,
                          double* y, double* dx0, double* dparams, dnbo_mem* mem);
int dnbo_block_naive_masks(const dnbo_desc* d, const double* x0, const double* params, const double* dy,
                           double* y, double* dx0, double* dparams, dnbo_mem* mem, int mode, uint8_t* m1,
                           uint8_t* m2, double* stats, int bf16_storage);
double dnbo_round_bf16(double v);
void dnbo_avgpool2(const double* in, int64_t n, int64_t c, int64_t h, int64_t w, double* out);
void dnbo_avgpool2_backward(const double* dout, int64_t n, int64_t c, int64_t h, int64_t w, double* din);
void dnbo_global_avgpool(const double* in, int64_t n, int64_t c, int64_t hw, double* out);
void dnbo_global_avgpool_backward(const double* dout, int64_t n, int64_t c, int64_t hw, double* din);
void dnbo_linear(const double* f, const double* wl, const double* bl, int64_t n, int64_t c, int64_t classes,
                 double* logits);
void dnbo_linear_backward(const double* f, const double* wl, const double* dlogits, int64_t n, int64_t c,
                          int64_t classes, double* df, double* dwl, double* dbl);
double dnbo_softmax_xent(const double* logits, const int32_t* labels, int64_t n, int64_t classes,
                         double* dlogits);

typedef struct {
  int32_t n, image;      /* batch; input height = width (3 channels), a multiple of 32 */
  int32_t growth;        /* k; stem width 2k, bottleneck width 4k */
  int32_t layers[4];     /* bottleneck layers of the four dense blocks */
  int32_t classes;
  double eps;
} dnbo_inet_desc;

/* ------------------------------------------------------------------ primitives */

/* Cross-correlation with stride and zero padding, no bias.  in (n,ci,h,w), wgt (co,ci,ks,ks),
 * out (n,co,ho,wo) with ho = (h + 2 pad - ks) / stride + 1:
 *   out[b][o][y][x] = sum_{c,i,j} wgt[o][c][i][j] * in[b][c][y*stride + i - pad][x*stride + j - pad]. */
void dnbo_conv_forward_strided(const double* in, const double* wgt, int64_t n, int64_t ci, int64_t co, int64_t h,
                               int64_t w, int64_t ks, int64_t stride, int64_t pad, double* out) {
  const int64_t ho = (h + 2 * pad - ks) / stride + 1, wo = (w + 2 * pad - ks) / stride + 1;
#pragma omp parallel for collapse(2) schedule(static)
  for (int64_t b = 0; b < n; ++b)
    for (int64_t o = 0; o < co; ++o)
      for (int64_t y = 0; y < ho; ++y)
        for (int64_t x = 0; x < wo; ++x) {
          double s = 0.0;
          for (int64_t c = 0; c < ci; ++c)
            for (int64_t i = 0; i < ks; ++i) {
              const int64_t yy = y * stride + i - pad;
              if (yy < 0 || yy >= h) continue;
              for (int64_t j = 0; j < ks; ++j) {
                const int64_t xx = x * stride + j - pad;
                if (xx < 0 || xx >= w) continue;
                s += wgt[((o * ci + c) * ks + i) * ks + j] * in[((b * ci + c) * h + yy) * w + xx];
              }
            }
          out[((b * co + o) * ho + y) * wo + x] = s;
        }
}

/* Adjoint w.r.t. the weights: dwgt[o][c][i][j] = sum_{b,y,x} dout[b][o][y][x] * in[b][c][y*stride+i-pad][x*stride+j-pad]. */
void dnbo_conv_wgrad_strided(const double* in, const double* dout, int64_t n, int64_t ci, int64_t co, int64_t h,
                             int64_t w, int64_t ks, int64_t stride, int64_t pad, double* dwgt) {
  const int64_t ho = (h + 2 * pad - ks) / stride + 1, wo = (w + 2 * pad - ks) / stride + 1;
#pragma omp parallel for collapse(2) schedule(static)
  for (int64_t o = 0; o < co; ++o)
    for (int64_t c = 0; c < ci; ++c)
      for (int64_t i = 0; i < ks; ++i)
        for (int64_t j = 0; j < ks; ++j) {
          double s = 0.0;
          for (int64_t b = 0; b < n; ++b)
            for (int64_t y = 0; y < ho; ++y) {
              const int64_t yy = y * stride + i - pad;
              if (yy < 0 || yy >= h) continue;
              for (int64_t x = 0; x < wo; ++x) {
                const int64_t xx = x * stride + j - pad;
                if (xx < 0 || xx >= w) continue;
                s += dout[((b * co + o) * ho + y) * wo + x] * in[((b * ci + c) * h + yy) * w + xx];
              }
            }
          dwgt[((o * ci + c) * ks + i) * ks + j] = s;
        }
}

/* Adjoint w.r.t. the input (not on the training path -- the stem's input needs no gradient --
 * but it completes the adjoint identities the tests check). */
void dnbo_conv_dgrad_strided(const double* dout, const double* wgt, int64_t n, int64_t ci, int64_t co, int64_t h,
                             int64_t w, int64_t ks, int64_t stride, int64_t pad, double* din) {
  const int64_t ho = (h + 2 * pad - ks) / stride + 1, wo = (w + 2 * pad - ks) / stride + 1;
  memset(din, 0, (size_t)(n * ci * h * w) * sizeof(double));
#pragma omp parallel for collapse(2) schedule(static)
  for (int64_t b = 0; b < n; ++b)
    for (int64_t c = 0; c < ci; ++c)
      for (int64_t o = 0; o < co; ++o)
        for (int64_t y = 0; y < ho; ++y)
          for (int64_t x = 0; x < wo; ++x) {
            const double g = dout[((b * co + o) * ho + y) * wo + x];
            for (int64_t i = 0; i < ks; ++i) {
              const int64_t yy = y * stride + i - pad;
              if (yy < 0 || yy >= h) continue;
              for (int64_t j = 0; j < ks; ++j) {
                const int64_t xx = x * stride + j - pad;
                if (xx < 0 || xx >= w) continue;
                din[((b * ci + c) * h + yy) * w + xx] += g * wgt[((o * ci + c) * ks + i) * ks + j];
              }
            }
          }
}

/* 3x3 max pooling, stride 2, pad 1 (h, w even): out (n,c,h/2,w/2); positions outside the image do
 * not take part.  idx receives, per output, the window position 3*i + j of the maximum, the first
 * one in scan order among equals.  mode 1: the positions in idx are imposed instead (out = the
 * value there); positions that differ from the pool's own are counted in stat[0] and the largest
 * (own maximum - imposed value) * inv_rms[c] goes to stat[1] (an imposed position outside the image
 * counts with margin 1e30).  mode 0 writes idx; mode -1 ignores it. */
void dnbo_maxpool3s2(const double* in, int64_t n, int64_t c, int64_t h, int64_t w, double* out, uint8_t* idx, int mode,
                     const double* inv_rms, double* stat) {
  const int64_t ho = h / 2, wo = w / 2;
  double cnt = 0.0, worst = 0.0;
  for (int64_t p = 0; p < n * c; ++p) {
    const double* s = in + p * h * w;
    const double ir = inv_rms ? inv_rms[p % c] : 1.0;
    for (int64_t y = 0; y < ho; ++y)
      for (int64_t x = 0; x < wo; ++x) {
        double best = 0.0;
        int bi = -1;
        for (int i = 0; i < 3; ++i) {
          const int64_t yy = 2 * y + i - 1;
          if (yy < 0 || yy >= h) continue;
          for (int j = 0; j < 3; ++j) {
            const int64_t xx = 2 * x + j - 1;
            if (xx < 0 || xx >= w) continue;
            const double v = s[yy * w + xx];
            if (bi < 0 || v > best) { best = v; bi = 3 * i + j; }
          }
        }
        const int64_t o = (p * ho + y) * wo + x;
        if (mode == 1) {
          const int use = idx[o];
          const int64_t yy = 2 * y + use / 3 - 1, xx = 2 * x + use % 3 - 1;
          const int inside = use < 9 && yy >= 0 && yy < h && xx >= 0 && xx < w;
          const double v = inside ? s[yy * w + xx] : 0.0;
          if (use != bi) {
            const double m = inside ? (best - v) * ir : 1e30;
            cnt += 1.0;
            if (m > worst) worst = m;
          }
          out[o] = v;
        } else {
          out[o] = best;
          if (mode == 0) idx[o] = (uint8_t)bi;
        }
      }
  }
  if (stat && mode == 1) {
    stat[0] += cnt;
    if (worst > stat[1]) stat[1] = worst;
  }
}

/* Adjoint of the pooling with the positions in idx: every output's gradient goes to its maximum's position. */
void dnbo_maxpool3s2_backward(const double* dout, const uint8_t* idx, int64_t n, int64_t c, int64_t h, int64_t w,
                              double* din) {
  const int64_t ho = h / 2, wo = w / 2;
  memset(din, 0, (size_t)(n * c * h * w) * sizeof(double));
  for (int64_t p = 0; p < n * c; ++p)
    for (int64_t y = 0; y < ho; ++y)
      for (int64_t x = 0; x < wo; ++x) {
        const int64_t o = (p * ho + y) * wo + x;
        const int use = idx[o];
        const int64_t yy = 2 * y + use / 3 - 1, xx = 2 * x + use % 3 - 1;
        if (use < 9 && yy >= 0 && yy < h && xx >= 0 && xx < w) din[p * h * w + yy * w + xx] += dout[o];
      }
}

/* ------------------------------------------------------------------ the network */

static void quant(double* p, int64_t count, int on) {
  if (!on) return;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < count; ++i) p[i] = dnbo_round_bf16(p[i]);
}
static double* quant_copy(const double* src, int64_t count, int on) {
  double* q = (double*)malloc((size_t)(count > 0 ? count : 1) * sizeof(double));
  for (int64_t i = 0; i < count; ++i) q[i] = on ? dnbo_round_bf16(src[i]) : src[i];
  return q;
}

static dnbo_desc inet_block_desc(const dnbo_inet_desc* d, int b, int64_t* cout) {
  int64_t c = 2 * d->growth, s = d->image / 4;
  for (int i = 0; i < b; ++i) { c = (c + (int64_t)d->layers[i] * d->growth) / 2; s /= 2; }
  dnbo_desc bd = {d->n, (int32_t)c, (int32_t)s, (int32_t)s, d->layers[b], d->growth, 4 * d->growth, d->eps};
  if (cout) *cout = c + (int64_t)d->layers[b] * d->growth;
  return bd;
}

/* Offset of part `which` in the pack: 0 stem W, 1 stem g, 2 stem b; 3 + 4*b + {0: block b, 1: g, 2: b,
 * 3: W (transition) or Wl (tail)}; 19 tail bl.  *count receives its size. */
int64_t dnbo_inet_param_offset(const dnbo_inet_desc* d, int which, int64_t* count) {
  const int64_t cs = 2 * d->growth;
  int64_t off = 0, cnt = 0;
  if (which == 0) cnt = cs * 147;
  else if (which == 1) { off = cs * 147; cnt = cs; }
  else if (which == 2) { off = cs * 148; cnt = cs; }
  else {
    off = cs * 149;
    for (int b = 0; b < 4; ++b) {
      int64_t cout;
      dnbo_desc bd = inet_block_desc(d, b, &cout);
      const int64_t pb = dnbo_param_count(&bd);
      const int64_t wsz = b < 3 ? (cout / 2) * cout : (int64_t)d->classes * cout;
      if (which == 3 + 4 * b) { cnt = pb; break; }
      off += pb;
      if (which == 4 + 4 * b) { cnt = cout; break; }
      off += cout;
      if (which == 5 + 4 * b) { cnt = cout; break; }
      off += cout;
      if (which == 6 + 4 * b) { cnt = wsz; break; }
      off += wsz;
      if (b == 3) {
        if (which == 19) { cnt = d->classes; break; }
        return -1;
      }
    }
  }
  if (count) *count = cnt;
  return off;
}

int64_t dnbo_inet_param_count(const dnbo_inet_desc* d) {
  int64_t cnt = 0;
  const int64_t off = dnbo_inet_param_offset(d, 19, &cnt);
  return off + cnt;
}

/* Bytes of the ReLU decisions (stem BN, then per block: first-BN decisions of all layers, second-BN
 * decisions, the BN that follows the block) and of the pooling positions (n, 2k, image/4, image/4). */
void dnbo_inet_decision_counts(const dnbo_inet_desc* d, int64_t* relu, int64_t* pool) {
  const int64_t cs = 2 * d->growth, s2 = d->image / 2, s4 = d->image / 4;
  int64_t t = (int64_t)d->n * cs * s2 * s2;
  for (int b = 0; b < 4; ++b) {
    int64_t cout;
    dnbo_desc bd = inet_block_desc(d, b, &cout);
    const int64_t P = (int64_t)bd.n * bd.h * bd.w;
    int64_t sigma = 0;
    for (int l = 1; l <= bd.layers; ++l) sigma += bd.c0 + (int64_t)(l - 1) * bd.growth;
    t += (sigma + (int64_t)bd.layers * bd.bottleneck + cout) * P;
  }
  *relu = t;
  *pool = (int64_t)d->n * cs * s4 * s4;
}

/* One training step.  x (n,3,image,image), labels (n).  Returns the loss; writes dparams (whole pack,
 * may be NULL for forward only) and, if logits_out != NULL, the logits (n,classes).
 * mode -1: plain; 0: the step's ReLU decisions and pooling positions are written to masks / pool;
 * 1: they are imposed.  stats (mode 1, 4 doubles): differing ReLU decisions and their worst margin
 * (|z| / sqrt(gamma^2 + beta^2)), differing pooling positions and their worst margin ((own maximum -
 * imposed value) / sqrt(gamma^2 + beta^2) of the stem BN channel). */
double dnbo_inet_step(const dnbo_inet_desc* d, const double* x, const int32_t* labels, const double* params,
                      double* dparams, double* logits_out, int mode, uint8_t* masks, uint8_t* pool, double* stats,
                      int bf16_storage) {
  const int q = bf16_storage ? 1 : 0;
  const int64_t n = d->n, S = d->image, cs = 2 * d->growth, S2 = S / 2, S4 = S / 4;
  const int use = mode >= 0;
  double st_relu[2] = {0.0, 0.0}, st_pool[2] = {0.0, 0.0};
  int64_t cnt;
  const double* Ws = params + dnbo_inet_param_offset(d, 0, &cnt);
  const double* gs = params + dnbo_inet_param_offset(d, 1, &cnt);
  const double* bs = params + dnbo_inet_param_offset(d, 2, &cnt);
  uint8_t* mp = masks;

  /* ---- forward: stem */
  double* Wsq = quant_copy(Ws, cs * 147, q);
  double* s = (double*)malloc((size_t)(n * cs * S2 * S2) * sizeof(double));
  dnbo_conv_forward_strided(x, Wsq, n, 3, cs, S, S, 7, 2, 3, s);
  quant(s, n * cs * S2 * S2, q);
  double* a0 = (double*)malloc((size_t)(n * cs * S2 * S2) * sizeof(double));
  double* smu = (double*)malloc((size_t)cs * sizeof(double));
  double* svar = (double*)malloc((size_t)cs * sizeof(double));
  dnbo_bn_forward(s, n, cs, S2 * S2, gs, bs, d->eps, a0, smu, svar);
  uint8_t* m_stem = mp;
  if (use) { dnbo_relu_with_decisions(a0, n, cs, S2 * S2, gs, bs, m_stem, mode, st_relu); mp += n * cs * S2 * S2; }
  else dnbo_relu_inplace(a0, n * cs * S2 * S2);
  double* inv_rms = (double*)malloc((size_t)cs * sizeof(double));
  for (int64_t c = 0; c < cs; ++c) inv_rms[c] = 1.0 / (sqrt(gs[c] * gs[c] + bs[c] * bs[c]) + 1e-300);
  uint8_t* own_pool = NULL;
  uint8_t* pidx = pool;
  if (!use) { own_pool = (uint8_t*)malloc((size_t)(n * cs * S4 * S4)); pidx = own_pool; }
  double* feat[4];
  feat[0] = (double*)malloc((size_t)(n * cs * S4 * S4) * sizeof(double));
  dnbo_maxpool3s2(a0, n, cs, S2, S2, feat[0], pidx, mode == 1 ? 1 : 0, inv_rms, st_pool);
  quant(feat[0], n * cs * S4 * S4, q);

  /* ---- forward: blocks, transitions, tail */
  dnbo_desc bd[4];
  int64_t cout[4];
  double *yb[4], *tz[4], *tmu[4], *tvar[4], *tconv[3], *Wtq[3];
  uint8_t *mb1[4], *mb2[4], *mg[4];
  const double *bp[4], *tg[4], *tb[4], *tw[4];
  for (int b = 0; b < 4; ++b) {
    bd[b] = inet_block_desc(d, b, &cout[b]);
    const int64_t hw = (int64_t)bd[b].h * bd[b].w, P = n * hw;
    bp[b] = params + dnbo_inet_param_offset(d, 3 + 4 * b, &cnt);
    tg[b] = params + dnbo_inet_param_offset(d, 4 + 4 * b, &cnt);
    tb[b] = params + dnbo_inet_param_offset(d, 5 + 4 * b, &cnt);
    tw[b] = params + dnbo_inet_param_offset(d, 6 + 4 * b, &cnt);
    int64_t sigma = 0;
    for (int l = 1; l <= bd[b].layers; ++l) sigma += bd[b].c0 + (int64_t)(l - 1) * bd[b].growth;
    mb1[b] = mp; mp += use ? sigma * P : 0;
    mb2[b] = mp; mp += use ? (int64_t)bd[b].layers * bd[b].bottleneck * P : 0;
    mg[b] = mp;  mp += use ? cout[b] * P : 0;
    yb[b] = (double*)malloc((size_t)(cout[b] * P) * sizeof(double));
    if (use) {
      double bst[4];
      dnbo_block_naive_masks(&bd[b], feat[b], bp[b], NULL, yb[b], NULL, NULL, NULL, mode, mb1[b], mb2[b], bst, q);
      if (mode == 1) {
        st_relu[0] += bst[0] + bst[2];
        if (bst[1] > st_relu[1]) st_relu[1] = bst[1];
        if (bst[3] > st_relu[1]) st_relu[1] = bst[3];
      }
    } else if (q) {
      dnbo_block_naive_bf16(&bd[b], feat[b], bp[b], NULL, yb[b], NULL, NULL, NULL);
    } else {
      dnbo_block_naive(&bd[b], feat[b], bp[b], NULL, yb[b], NULL, NULL, NULL);
    }
    tz[b] = (double*)malloc((size_t)(cout[b] * P) * sizeof(double));
    tmu[b] = (double*)malloc((size_t)cout[b] * sizeof(double));
    tvar[b] = (double*)malloc((size_t)cout[b] * sizeof(double));
    dnbo_bn_forward(yb[b], n, cout[b], hw, tg[b], tb[b], d->eps, tz[b], tmu[b], tvar[b]);
    if (use) dnbo_relu_with_decisions(tz[b], n, cout[b], hw, tg[b], tb[b], mg[b], mode, st_relu);
    else dnbo_relu_inplace(tz[b], cout[b] * P);
    if (b < 3) {
      const int64_t ch = cout[b] / 2;
      quant(tz[b], cout[b] * P, q); /* the conv's operand */
      Wtq[b] = quant_copy(tw[b], ch * cout[b], q);
      tconv[b] = (double*)malloc((size_t)(ch * P) * sizeof(double));
      dnbo_conv_forward(tz[b], Wtq[b], n, cout[b], ch, bd[b].h, bd[b].w, 1, tconv[b]);
      quant(tconv[b], ch * P, q);
      feat[b + 1] = (double*)malloc((size_t)(ch * P / 4) * sizeof(double));
      dnbo_avgpool2(tconv[b], n, ch, bd[b].h, bd[b].w, feat[b + 1]);
      quant(feat[b + 1], ch * P / 4, q);
    }
  }
  const int64_t C = cout[3], hw3 = (int64_t)bd[3].h * bd[3].w;
  const double* bl = params + dnbo_inet_param_offset(d, 19, &cnt);
  double* pooled = (double*)malloc((size_t)(n * C) * sizeof(double));
  dnbo_global_avgpool(tz[3], n, C, hw3, pooled);
  double* logits = (double*)malloc((size_t)(n * d->classes) * sizeof(double));
  dnbo_linear(pooled, tw[3], bl, n, C, d->classes, logits);
  double* dlogits = (double*)malloc((size_t)(n * d->classes) * sizeof(double));
  const double loss = dnbo_softmax_xent(logits, labels, n, d->classes, dparams ? dlogits : NULL);
  if (logits_out) memcpy(logits_out, logits, (size_t)(n * d->classes) * sizeof(double));

  /* ---- backward */
  if (dparams) {
    double* dpooled = (double*)malloc((size_t)(n * C) * sizeof(double));
    dnbo_linear_backward(pooled, tw[3], dlogits, n, C, d->classes, dpooled, dparams + (tw[3] - params),
                         dparams + (bl - params));
    double* g = (double*)malloc((size_t)(n * C * hw3) * sizeof(double)); /* gradient w.r.t. tz[3], then yb[3] */
    dnbo_global_avgpool_backward(dpooled, n, C, hw3, g);
    quant(g, n * C * hw3, q);
    free(dpooled);
    for (int b = 3; b >= 0; --b) {
      const int64_t hw = (int64_t)bd[b].h * bd[b].w, P = n * hw;
      if (use && mode == 1) dnbo_relu_backward_decisions(mg[b], g, g, cout[b] * P);
      else dnbo_relu_backward(tz[b], g, g, cout[b] * P);
      dnbo_bn_backward(yb[b], g, n, cout[b], hw, tg[b], tmu[b], tvar[b], d->eps, g, dparams + (tg[b] - params),
                       dparams + (tb[b] - params));
      quant(g, cout[b] * P, q); /* the block's dy */
      double* dfeat = (double*)malloc((size_t)(bd[b].c0 * P) * sizeof(double));
      double* ydummy = (double*)malloc((size_t)(cout[b] * P) * sizeof(double));
      double* dbp = dparams + (bp[b] - params);
      if (use && mode == 1) {
        double bst[4];
        dnbo_block_naive_masks(&bd[b], feat[b], bp[b], g, ydummy, dfeat, dbp, NULL, 1, mb1[b], mb2[b], bst, q);
      } else if (q) {
        dnbo_block_naive_bf16(&bd[b], feat[b], bp[b], g, ydummy, dfeat, dbp, NULL);
      } else {
        dnbo_block_naive(&bd[b], feat[b], bp[b], g, ydummy, dfeat, dbp, NULL);
      }
      free(ydummy);
      free(g);
      g = NULL;
      if (b > 0) {
        /* through transition b-1: pooling backward, then the 1x1 conv's weight and data gradients */
        const int64_t hp = bd[b - 1].h, wp = bd[b - 1].w, cp = cout[b - 1], ch = cp / 2;
        double* dconv = (double*)malloc((size_t)(n * ch * hp * wp) * sizeof(double));
        dnbo_avgpool2_backward(dfeat, n, ch, hp, wp, dconv);
        quant(dconv, n * ch * hp * wp, q);
        dnbo_conv_wgrad(tz[b - 1], dconv, n, cp, ch, hp, wp, 1, dparams + (tw[b - 1] - params));
        g = (double*)malloc((size_t)(n * cp * hp * wp) * sizeof(double));
        dnbo_conv_dgrad(dconv, Wtq[b - 1], n, cp, ch, hp, wp, 1, g);
        quant(g, n * cp * hp * wp, q);
        free(dconv);
      } else {
        /* through the stem: pooling backward to the maxima's positions, BN+ReLU backward, weight gradient */
        double* da0 = (double*)malloc((size_t)(n * cs * S2 * S2) * sizeof(double));
        dnbo_maxpool3s2_backward(dfeat, pidx, n, cs, S2, S2, da0);
        quant(da0, n * cs * S2 * S2, q); /* kept in bf16 between the pooling's and the BN's backward */
        if (use && mode == 1) dnbo_relu_backward_decisions(m_stem, da0, da0, n * cs * S2 * S2);
        else dnbo_relu_backward(a0, da0, da0, n * cs * S2 * S2);
        dnbo_bn_backward(s, da0, n, cs, S2 * S2, gs, smu, svar, d->eps, da0, dparams + (gs - params), dparams + (bs - params));
        quant(da0, n * cs * S2 * S2, q);
        dnbo_conv_wgrad_strided(x, da0, n, 3, cs, S, S, 7, 2, 3, dparams + (Ws - params));
        free(da0);
      }
      free(dfeat);
    }
  }
  for (int b = 0; b < 4; ++b) { free(feat[b]); free(yb[b]); free(tz[b]); free(tmu[b]); free(tvar[b]); }
  for (int b = 0; b < 3; ++b) { free(tconv[b]); free(Wtq[b]); }
  free(Wsq); free(s); free(a0); free(smu); free(svar); free(inv_rms); free(own_pool);
  free(pooled); free(logits); free(dlogits);
  if (mode == 1 && stats) { stats[0] = st_relu[0]; stats[1] = st_relu[1]; stats[2] = st_pool[0]; stats[3] = st_pool[1]; }
  return loss;
}
