/*
 * dnb_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, obviously-correct CPU reference (float64 throughout) for one
 * DenseNet dense block, forward and reverse-mode gradients.  It exists so the
 * HIP path has something independent to be compared with; it shares no code,
 * header or table with the GPU library and is never used by the product path.
 * Only tests, the smoke check and the benchmark's cpu_baseline leg call it.
 *
 * What is computed (paper, Section 2 "The DenseNet Architecture"):
 *   x_l = H_l([x_0, x_1, ..., x_{l-1}])  with H_l = BN -> ReLU -> conv, the
 *   pre-activation order of Section 2 ("Pre-activation batch normalization"),
 *   optionally with the bottleneck BN -> ReLU -> 1x1 conv (to B channels)
 *   -> BN -> ReLU -> 3x3 conv (to k channels).
 *
 * Two schedules over the same arithmetic:
 *   dnbo_block_naive  -- Section 3 ("Naive Implementation"): every concat and
 *                        BN output is freshly allocated and kept for backward.
 *   dnbo_block_shared -- Section 4 ("Memory-Efficient Implementation"): concat
 *                        output goes to shared storage 1, BN+ReLU output to
 *                        shared storage 2 (and the bottleneck's second BN+ReLU
 *                        output to a third shared buffer); later layers
 *                        overwrite them; backward re-runs concat and BN to
 *                        re-populate them before ordinary back-propagation.
 *   Both track the peak number of live feature-map elements they allocate.
 *   dnbo_block_naive_masks -- the store-everything schedule with the ReLU decisions (z > 0, one
 *                        bit per pre-activation) either written out or taken from the caller.
 *                        A ReLU decision is an integer decided by floating point: a pre-activation
 *                        within rounding of zero falls on either side depending on the precision
 *                        of the arithmetic, and the gradient element behind it then changes by
 *                        its whole size.  A parity test therefore lets both sides take the
 *                        decision in the same precision (the kernel's): the block is evaluated in
 *                        float64 with the kernel's decisions, and every decision that differs
 *                        from the block's own is reported with its margin |z| / sqrt(gamma^2 +
 *                        beta^2) (the pre-activation in units of its channel's root mean square:
 *                        xhat has unit variance), so the test can check that only ties within
 *                        rounding differ.
 *   dnbo_block_naive_bf16 -- the store-everything schedule with every stored tensor rounded
 *                        to bfloat16 where it is produced (arithmetic still float64); the
 *                        reference for the bf16 path's gradients.  Pinned by a library
 *                        autograd construction with casts at the same points.
 *
 * Readings where the paper is silent (listed in the design notes too):
 *   BN uses train-mode batch statistics over (n,h,w), biased variance, eps
 *   inside the square root; ReLU derivative is 0 at z <= 0; convs are
 *   cross-correlations, stride 1, zero padding (ksize-1)/2, no bias; the block
 *   input x_0 is the first member of every concatenation, oldest first.
 *
 * Parity pins (tests/test_oracle_*.py): central finite differences of the
 * whole block, hand-enumerated tiny cases, BN closed-form invariants, conv
 * adjoint identities, textbook special cases, a float64 library cross-check,
 * and bit-equality of the two schedules.
 *
 * Layout: NCHW, row-major, double.  Parameter pack per layer, in order:
 *   bottleneck B>0 : g1[C_l] b1[C_l] W1[B][C_l] g2[B] b2[B] W3[k][B][3][3]
 *   bottleneck B=0 : g1[C_l] b1[C_l] W3[k][C_l][3][3]
 * with C_l = c0 + (l-1)*k for l = 1..m.  Gradients use the same layout.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
  int32_t n, c0, h, w;
  int32_t layers;     /* m */
  int32_t growth;     /* k */
  int32_t bottleneck; /* B; 0 = BN-ReLU-3x3 only */
  double eps;
} dnbo_desc;

typedef struct {
  int64_t peak_elems;   /* peak live feature-map elements (forward+backward)  */
  int64_t stored_elems; /* elements still live when forward returns           */
  int64_t live_elems;   /* running counter (internal)                         */
} dnbo_mem;

enum { DNBO_G1 = 0, DNBO_B1, DNBO_W1, DNBO_G2, DNBO_B2, DNBO_W3 };

/* ------------------------------------------------------------------ helpers */

static int64_t layer_cin(const dnbo_desc* d, int l /*1-based*/) {
  return (int64_t)d->c0 + (int64_t)(l - 1) * d->growth;
}

static int64_t layer_param_count(const dnbo_desc* d, int l) {
  int64_t c = layer_cin(d, l), k = d->growth, B = d->bottleneck;
  if (B > 0) return 2 * c + B * c + 2 * B + k * B * 9;
  return 2 * c + k * c * 9;
}

int64_t dnbo_param_count(const dnbo_desc* d) {
  int64_t t = 0;
  for (int l = 1; l <= d->layers; ++l) t += layer_param_count(d, l);
  return t;
}

/* Offset (in elements) of one parameter tensor; returns -1 if it does not
 * exist for this descriptor.  *count receives its element count. */
int64_t dnbo_param_offset(const dnbo_desc* d, int layer, int which, int64_t* count) {
  if (layer < 1 || layer > d->layers) return -1;
  int64_t off = 0;
  for (int l = 1; l < layer; ++l) off += layer_param_count(d, l);
  int64_t c = layer_cin(d, layer), k = d->growth, B = d->bottleneck, cnt = 0;
  if (B > 0) {
    switch (which) {
      case DNBO_G1: cnt = c; break;
      case DNBO_B1: off += c; cnt = c; break;
      case DNBO_W1: off += 2 * c; cnt = B * c; break;
      case DNBO_G2: off += 2 * c + B * c; cnt = B; break;
      case DNBO_B2: off += 2 * c + B * c + B; cnt = B; break;
      case DNBO_W3: off += 2 * c + B * c + 2 * B; cnt = k * B * 9; break;
      default: return -1;
    }
  } else {
    switch (which) {
      case DNBO_G1: cnt = c; break;
      case DNBO_B1: off += c; cnt = c; break;
      case DNBO_W3: off += 2 * c; cnt = k * c * 9; break;
      default: return -1;
    }
  }
  if (count) *count = cnt;
  return off;
}

static double* fm_alloc(dnbo_mem* mem, int64_t elems) {
  double* p = (double*)calloc((size_t)(elems > 0 ? elems : 1), sizeof(double));
  if (mem) {
    mem->live_elems += elems;
    if (mem->live_elems > mem->peak_elems) mem->peak_elems = mem->live_elems;
  }
  return p;
}

static void fm_free(dnbo_mem* mem, double* p, int64_t elems) {
  free(p);
  if (mem) mem->live_elems -= elems;
}

/* Storage-precision emulation (reading of the bf16 workloads: "bf16 activations/weights with
 * fp32 accumulation and fp32 BN statistics"): a value that the bf16 path keeps in memory is
 * rounded to the nearest bfloat16 (8-bit significand, round to nearest even) at the point
 * where it is stored; all arithmetic stays float64.  Used only by dnbo_block_naive_bf16. */
double dnbo_round_bf16(double v) {
  float f = (float)v;
  uint32_t u;
  memcpy(&u, &f, 4);
  if ((u & 0x7F800000u) == 0x7F800000u) return (double)f; /* inf / nan unchanged */
  u += 0x7FFFu + ((u >> 16) & 1u);
  u &= 0xFFFF0000u;
  memcpy(&f, &u, 4);
  return (double)f;
}

static void quantize(double* p, int64_t count, int on) {
  if (!on) return;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < count; ++i) p[i] = dnbo_round_bf16(p[i]);
}

static double* rounded_copy(const double* src, int64_t count, int on) {
  double* q = (double*)malloc((size_t)(count > 0 ? count : 1) * sizeof(double));
  for (int64_t i = 0; i < count; ++i) q[i] = on ? dnbo_round_bf16(src[i]) : src[i];
  return q;
}

/* ------------------------------------------------------------- primitives */

/* Batch normalisation, train mode (paper Section 2 cites Ioffe & Szegedy):
 * per channel c over all (n,h,w): mean, biased variance,
 * xhat = (u-mean)/sqrt(var+eps), z = gamma*xhat + beta.
 * u,z: (n,c,hw).  mean,var: (c).  z may not alias u. */
void dnbo_bn_forward(const double* u, int64_t n, int64_t c, int64_t hw, const double* gamma,
                     const double* beta, double eps, double* z, double* mean, double* var) {
  const double P = (double)(n * hw);
#pragma omp parallel for schedule(static)
  for (int64_t ch = 0; ch < c; ++ch) {
    double s = 0.0;
    for (int64_t i = 0; i < n; ++i) {
      const double* p = u + (i * c + ch) * hw;
      for (int64_t q = 0; q < hw; ++q) s += p[q];
    }
    const double mu = s / P;
    double ss = 0.0;
    for (int64_t i = 0; i < n; ++i) {
      const double* p = u + (i * c + ch) * hw;
      for (int64_t q = 0; q < hw; ++q) {
        const double dlt = p[q] - mu;
        ss += dlt * dlt;
      }
    }
    const double v = ss / P;
    const double istd = 1.0 / sqrt(v + eps);
    for (int64_t i = 0; i < n; ++i) {
      const double* p = u + (i * c + ch) * hw;
      double* o = z + (i * c + ch) * hw;
      for (int64_t q = 0; q < hw; ++q) o[q] = gamma[ch] * ((p[q] - mu) * istd) + beta[ch];
    }
    mean[ch] = mu;
    var[ch] = v;
  }
}

/* Reverse mode of dnbo_bn_forward.  dz: gradient w.r.t. z.
 * dbeta = sum dz; dgamma = sum dz*xhat;
 * du = gamma/sqrt(var+eps) * (dz - dbeta/P - xhat*dgamma/P). */
void dnbo_bn_backward(const double* u, const double* dz, int64_t n, int64_t c, int64_t hw,
                      const double* gamma, const double* mean, const double* var, double eps,
                      double* du, double* dgamma, double* dbeta) {
  const double P = (double)(n * hw);
#pragma omp parallel for schedule(static)
  for (int64_t ch = 0; ch < c; ++ch) {
    const double mu = mean[ch], istd = 1.0 / sqrt(var[ch] + eps);
    double sb = 0.0, sg = 0.0;
    for (int64_t i = 0; i < n; ++i) {
      const double* p = u + (i * c + ch) * hw;
      const double* g = dz + (i * c + ch) * hw;
      for (int64_t q = 0; q < hw; ++q) {
        sb += g[q];
        sg += g[q] * ((p[q] - mu) * istd);
      }
    }
    for (int64_t i = 0; i < n; ++i) {
      const double* p = u + (i * c + ch) * hw;
      const double* g = dz + (i * c + ch) * hw;
      double* o = du + (i * c + ch) * hw;
      for (int64_t q = 0; q < hw; ++q) {
        const double xh = (p[q] - mu) * istd;
        o[q] = gamma[ch] * istd * (g[q] - sb / P - xh * sg / P);
      }
    }
    dgamma[ch] = sg;
    dbeta[ch] = sb;
  }
}

/* In-place ReLU (Section 3: the non-linearity occurs in place). */
void dnbo_relu_inplace(double* z, int64_t count) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < count; ++i) z[i] = z[i] > 0.0 ? z[i] : 0.0;
}

/* dz = da where the (post-ReLU) activation a is > 0, else 0. */
void dnbo_relu_backward(const double* a, const double* da, double* dz, int64_t count) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < count; ++i) dz[i] = a[i] > 0.0 ? da[i] : 0.0;
}

/* Cross-correlation, stride 1, zero padding pad=(ks-1)/2, no bias.
 * in (n,ci,h,w), wgt (co,ci,ks,ks), out (n,co,h,w) is overwritten. */
void dnbo_conv_forward(const double* in, const double* wgt, int64_t n, int64_t ci, int64_t co,
                       int64_t h, int64_t w, int64_t ks, double* out) {
  const int64_t pad = (ks - 1) / 2;
#pragma omp parallel for collapse(2) schedule(static)
  for (int64_t b = 0; b < n; ++b) {
    for (int64_t o = 0; o < co; ++o) {
      double* op = out + (b * co + o) * h * w;
      for (int64_t q = 0; q < h * w; ++q) op[q] = 0.0;
      for (int64_t c = 0; c < ci; ++c) {
        const double* ip = in + (b * ci + c) * h * w;
        for (int64_t i = 0; i < ks; ++i) {
          for (int64_t j = 0; j < ks; ++j) {
            const double wv = wgt[((o * ci + c) * ks + i) * ks + j];
            for (int64_t y = 0; y < h; ++y) {
              const int64_t yy = y + i - pad;
              if (yy < 0 || yy >= h) continue;
              const int64_t x_lo = (pad - j) > 0 ? (pad - j) : 0;
              const int64_t x_hi = (w + pad - j) < w ? (w + pad - j) : w;
              for (int64_t x = x_lo; x < x_hi; ++x) op[y * w + x] += wv * ip[yy * w + x + j - pad];
            }
          }
        }
      }
    }
  }
}

/* Adjoint of dnbo_conv_forward w.r.t. its input: din (n,ci,h,w) overwritten. */
void dnbo_conv_dgrad(const double* dout, const double* wgt, int64_t n, int64_t ci, int64_t co,
                     int64_t h, int64_t w, int64_t ks, double* din) {
  const int64_t pad = (ks - 1) / 2;
#pragma omp parallel for collapse(2) schedule(static)
  for (int64_t b = 0; b < n; ++b) {
    for (int64_t c = 0; c < ci; ++c) {
      double* dp = din + (b * ci + c) * h * w;
      for (int64_t q = 0; q < h * w; ++q) dp[q] = 0.0;
      for (int64_t o = 0; o < co; ++o) {
        const double* gp = dout + (b * co + o) * h * w;
        for (int64_t i = 0; i < ks; ++i) {
          for (int64_t j = 0; j < ks; ++j) {
            const double wv = wgt[((o * ci + c) * ks + i) * ks + j];
            /* forward: out[y][x] += wv * in[y+i-pad][x+j-pad]
             * hence     din[y+i-pad][x+j-pad] += wv * dout[y][x] */
            for (int64_t y = 0; y < h; ++y) {
              const int64_t yy = y + i - pad;
              if (yy < 0 || yy >= h) continue;
              const int64_t x_lo = (pad - j) > 0 ? (pad - j) : 0;
              const int64_t x_hi = (w + pad - j) < w ? (w + pad - j) : w;
              for (int64_t x = x_lo; x < x_hi; ++x) dp[yy * w + x + j - pad] += wv * gp[y * w + x];
            }
          }
        }
      }
    }
  }
}

/* Adjoint of dnbo_conv_forward w.r.t. its weights: dwgt (co,ci,ks,ks) overwritten. */
void dnbo_conv_wgrad(const double* in, const double* dout, int64_t n, int64_t ci, int64_t co,
                     int64_t h, int64_t w, int64_t ks, double* dwgt) {
  const int64_t pad = (ks - 1) / 2;
#pragma omp parallel for collapse(2) schedule(static)
  for (int64_t o = 0; o < co; ++o) {
    for (int64_t c = 0; c < ci; ++c) {
      for (int64_t i = 0; i < ks; ++i) {
        for (int64_t j = 0; j < ks; ++j) {
          double s = 0.0;
          for (int64_t b = 0; b < n; ++b) {
            const double* ip = in + (b * ci + c) * h * w;
            const double* gp = dout + (b * co + o) * h * w;
            for (int64_t y = 0; y < h; ++y) {
              const int64_t yy = y + i - pad;
              if (yy < 0 || yy >= h) continue;
              const int64_t x_lo = (pad - j) > 0 ? (pad - j) : 0;
              const int64_t x_hi = (w + pad - j) < w ? (w + pad - j) : w;
              for (int64_t x = x_lo; x < x_hi; ++x) s += gp[y * w + x] * ip[yy * w + x + j - pad];
            }
          }
          dwgt[((o * ci + c) * ks + i) * ks + j] = s;
        }
      }
    }
  }
}

/* Channel-axis concatenation (Section 2, "Contiguous concatenation"):
 * copies srcs[0] (n,c0,hw), srcs[1..cnt-1] (n,k,hw) into dst (n,ctot,hw). */
static void concat_into(double* dst, double* const* srcs, int cnt, int64_t n, int64_t c0, int64_t k,
                        int64_t hw) {
  const int64_t ctot = c0 + (int64_t)(cnt - 1) * k;
  for (int64_t b = 0; b < n; ++b) {
    int64_t coff = 0;
    for (int s = 0; s < cnt; ++s) {
      const int64_t cs = (s == 0) ? c0 : k;
      memcpy(dst + (b * ctot + coff) * hw, srcs[s] + b * cs * hw, (size_t)(cs * hw) * sizeof(double));
      coff += cs;
    }
  }
}

/* Concat backward: add channel slices of du (n,ctot,hw) into each source's
 * gradient accumulator. */
static void concat_backward_add(const double* du, double* const* dsrcs, int cnt, int64_t n,
                                int64_t c0, int64_t k, int64_t hw) {
  const int64_t ctot = c0 + (int64_t)(cnt - 1) * k;
  for (int64_t b = 0; b < n; ++b) {
    int64_t coff = 0;
    for (int s = 0; s < cnt; ++s) {
      const int64_t cs = (s == 0) ? c0 : k;
      const double* p = du + (b * ctot + coff) * hw;
      double* g = dsrcs[s] + b * cs * hw;
      for (int64_t q = 0; q < cs * hw; ++q) g[q] += p[q];
      coff += cs;
    }
  }
}

static const double* par(const dnbo_desc* d, const double* params, int layer, int which) {
  int64_t cnt;
  int64_t off = dnbo_param_offset(d, layer, which, &cnt);
  return off < 0 ? NULL : params + off;
}
static double* dpar(const dnbo_desc* d, double* dparams, int layer, int which) {
  int64_t cnt;
  int64_t off = dnbo_param_offset(d, layer, which, &cnt);
  return off < 0 ? NULL : dparams + off;
}

/* Splits dy (n,c_out,hw) into per-feature gradient accumulators
 * gx[0] (n,c0,hw), gx[l] (n,k,hw). */
static void split_dy(const double* dy, double** gx, int m, int64_t n, int64_t c0, int64_t k,
                     int64_t hw) {
  const int64_t cout = c0 + (int64_t)m * k;
  for (int64_t b = 0; b < n; ++b) {
    int64_t coff = 0;
    for (int s = 0; s <= m; ++s) {
      const int64_t cs = (s == 0) ? c0 : k;
      memcpy(gx[s] + b * cs * hw, dy + (b * cout + coff) * hw, (size_t)(cs * hw) * sizeof(double));
      coff += cs;
    }
  }
}

/* ReLU decisions of a block: mode 0 writes the block's own (z > 0), mode 1 reads the caller's
 * and uses them in forward (a = z where the decision is 1, else 0) and backward.
 * m1: first BN of every layer, the layers' (n, C_l, hw) byte arrays one after the other;
 * m2: second BN (bottleneck only), m arrays of (n, B, hw).
 * stats (mode 1): [0] decisions of m1 that differ from the block's own, [1] the largest margin
 * |z| / sqrt(gamma^2 + beta^2) among them (z = gamma xhat + beta with xhat of unit variance, so
 * this is the distance from the decision boundary in units of the channel's root mean square
 * pre-activation), [2], [3] the same for m2. */
typedef struct {
  int mode;
  uint8_t* m1;
  uint8_t* m2;
  double* stats;
} dnbo_masks;

/* In-place ReLU of z = BN(u) under `mk` (see dnbo_masks); mask points at this tensor's bytes. */
void dnbo_relu_with_decisions(double* z, int64_t n, int64_t c, int64_t hw, const double* gamma,
                                const double* beta, uint8_t* mask, int mode, double* stat /* count, worst margin */) {
  double cnt = 0.0, worst = 0.0;
#pragma omp parallel for schedule(static) reduction(+ : cnt) reduction(max : worst)
  for (int64_t ch = 0; ch < c; ++ch) {
    const double rms = sqrt(gamma[ch] * gamma[ch] + beta[ch] * beta[ch]) + 1e-300;
    for (int64_t i = 0; i < n; ++i) {
      const int64_t base = (i * c + ch) * hw;
      for (int64_t q = 0; q < hw; ++q) {
        const int own = z[base + q] > 0.0;
        if (mode == 0) {
          mask[base + q] = (uint8_t)own;
          z[base + q] = own ? z[base + q] : 0.0;
        } else {
          const int use = mask[base + q] != 0;
          if (use != own) {
            const double margin = fabs(z[base + q]) / rms;
            cnt += 1.0;
            if (margin > worst) worst = margin;
          }
          z[base + q] = use ? z[base + q] : 0.0;
        }
      }
    }
  }
  if (stat && mode == 1) {
    stat[0] += cnt;
    if (worst > stat[1]) stat[1] = worst;
  }
}

void dnbo_relu_backward_decisions(const uint8_t* mask, const double* da, double* dz, int64_t count) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < count; ++i) dz[i] = mask[i] ? da[i] : 0.0;
}

/* ------------------------------------------------- schedule 1: store all */

/* Section 3.  Forward keeps, per layer: the concat output u_l, the BN+ReLU
 * output a_l (ReLU in place on the BN output), and with a bottleneck also
 * b_l and its BN+ReLU output a2_l; plus every x_l.  Backward is textbook
 * reverse mode, layers m..1, with one gradient accumulator per feature
 * (dense connectivity: the gradient of x_l is complete once every later
 * layer has been processed). */
static int block_naive_impl(const dnbo_desc* d, const double* x0, const double* params, const double* dy,
                            double* y, double* dx0, double* dparams, dnbo_mem* mem, int q /* bf16 storage */,
                            const dnbo_masks* mk /* may be NULL */) {
  const int m = d->layers;
  const int64_t n = d->n, c0 = d->c0, k = d->growth, B = d->bottleneck, H = d->h, W = d->w;
  const int64_t hw = H * W, P = n * hw, cout = c0 + m * k;
  if (mem) memset(mem, 0, sizeof(*mem));
  double** x = (double**)calloc((size_t)m + 1, sizeof(double*));
  double** u = (double**)calloc((size_t)m + 1, sizeof(double*));
  double** a = (double**)calloc((size_t)m + 1, sizeof(double*));
  double** b = (double**)calloc((size_t)m + 1, sizeof(double*));
  double** a2 = (double**)calloc((size_t)m + 1, sizeof(double*));
  double** mu1 = (double**)calloc((size_t)m + 1, sizeof(double*));
  double** v1 = (double**)calloc((size_t)m + 1, sizeof(double*));
  double** mu2 = (double**)calloc((size_t)m + 1, sizeof(double*));
  double** v2 = (double**)calloc((size_t)m + 1, sizeof(double*));
  double** W1q = (double**)calloc((size_t)m + 1, sizeof(double*)); /* weights as the convs read them */
  double** W3q = (double**)calloc((size_t)m + 1, sizeof(double*));

  /* where layer l's ReLU decisions sit inside mk->m1 / mk->m2 */
  int64_t* mo1 = (int64_t*)calloc((size_t)m + 2, sizeof(int64_t));
  for (int l = 1; l <= m; ++l) mo1[l + 1] = mo1[l] + layer_cin(d, l) * P;
  if (mk && mk->mode == 1 && mk->stats) memset(mk->stats, 0, 4 * sizeof(double));

  x[0] = (double*)x0; /* the caller's input is not ours to count */
  for (int l = 1; l <= m; ++l) {
    const int64_t c = layer_cin(d, l);
    u[l] = fm_alloc(mem, c * P);
    concat_into(u[l], x, l, n, c0, k, hw);
    a[l] = fm_alloc(mem, c * P);
    mu1[l] = (double*)calloc((size_t)c, sizeof(double));
    v1[l] = (double*)calloc((size_t)c, sizeof(double));
    dnbo_bn_forward(u[l], n, c, hw, par(d, params, l, DNBO_G1), par(d, params, l, DNBO_B1), d->eps,
                    a[l], mu1[l], v1[l]);
    if (mk)
      dnbo_relu_with_decisions(a[l], n, c, hw, par(d, params, l, DNBO_G1), par(d, params, l, DNBO_B1), mk->m1 + mo1[l],
                          mk->mode, mk->stats);
    else
      dnbo_relu_inplace(a[l], c * P);
    quantize(a[l], c * P, q);
    x[l] = fm_alloc(mem, k * P);
    int64_t nw3 = 0;
    dnbo_param_offset(d, l, DNBO_W3, &nw3);
    W3q[l] = rounded_copy(par(d, params, l, DNBO_W3), nw3, q);
    if (B > 0) {
      W1q[l] = rounded_copy(par(d, params, l, DNBO_W1), B * c, q);
      b[l] = fm_alloc(mem, B * P);
      dnbo_conv_forward(a[l], W1q[l], n, c, B, H, W, 1, b[l]);
      quantize(b[l], B * P, q);
      a2[l] = fm_alloc(mem, B * P);
      mu2[l] = (double*)calloc((size_t)B, sizeof(double));
      v2[l] = (double*)calloc((size_t)B, sizeof(double));
      dnbo_bn_forward(b[l], n, B, hw, par(d, params, l, DNBO_G2), par(d, params, l, DNBO_B2),
                      d->eps, a2[l], mu2[l], v2[l]);
      if (mk)
        dnbo_relu_with_decisions(a2[l], n, B, hw, par(d, params, l, DNBO_G2), par(d, params, l, DNBO_B2),
                            mk->m2 + (int64_t)(l - 1) * B * P, mk->mode, mk->stats ? mk->stats + 2 : NULL);
      else
        dnbo_relu_inplace(a2[l], B * P);
      quantize(a2[l], B * P, q);
      dnbo_conv_forward(a2[l], W3q[l], n, B, k, H, W, 3, x[l]);
    } else {
      dnbo_conv_forward(a[l], W3q[l], n, c, k, H, W, 3, x[l]);
    }
    quantize(x[l], k * P, q);
  }
  /* block output = concatenation of everything */
  concat_into(y, x, m + 1, n, c0, k, hw);
  if (mem) mem->stored_elems = mem->live_elems;

  if (dy) {
    const int64_t cmax = layer_cin(d, m);
    /* shared gradient storage (Section 4, "Shared storage for gradients"):
     * one accumulator slab for the features and one scratch per tensor kind */
    double** gx = (double**)calloc((size_t)m + 1, sizeof(double*));
    gx[0] = fm_alloc(mem, c0 * P);
    for (int l = 1; l <= m; ++l) gx[l] = fm_alloc(mem, k * P);
    double* da = fm_alloc(mem, cmax * P);  /* gradient of a_l / z1_l / u_l */
    double* da2 = B > 0 ? fm_alloc(mem, B * P) : NULL; /* gradient of a2_l / b_l */
    split_dy(dy, gx, m, n, c0, k, hw);
    for (int l = m; l >= 1; --l) {
      const int64_t c = layer_cin(d, l);
      /* the convs read the accumulated gradient of x_l as a rounded operand; the
       * accumulators themselves stay unrounded (they are fp32 on the bf16 path) */
      double* g = q ? rounded_copy(gx[l], k * P, 1) : gx[l];
      if (B > 0) {
        dnbo_conv_wgrad(a2[l], g, n, B, k, H, W, 3, dpar(d, dparams, l, DNBO_W3));
        dnbo_conv_dgrad(g, W3q[l], n, B, k, H, W, 3, da2);
        quantize(da2, B * P, q);
        if (mk && mk->mode == 1)
          dnbo_relu_backward_decisions(mk->m2 + (int64_t)(l - 1) * B * P, da2, da2, B * P);
        else
          dnbo_relu_backward(a2[l], da2, da2, B * P);
        dnbo_bn_backward(b[l], da2, n, B, hw, par(d, params, l, DNBO_G2), mu2[l], v2[l], d->eps,
                         da2, dpar(d, dparams, l, DNBO_G2), dpar(d, dparams, l, DNBO_B2));
        quantize(da2, B * P, q);
        dnbo_conv_wgrad(a[l], da2, n, c, B, H, W, 1, dpar(d, dparams, l, DNBO_W1));
        dnbo_conv_dgrad(da2, W1q[l], n, c, B, H, W, 1, da);
      } else {
        dnbo_conv_wgrad(a[l], g, n, c, k, H, W, 3, dpar(d, dparams, l, DNBO_W3));
        dnbo_conv_dgrad(g, W3q[l], n, c, k, H, W, 3, da);
      }
      quantize(da, c * P, q);
      if (q) free(g);
      if (mk && mk->mode == 1)
        dnbo_relu_backward_decisions(mk->m1 + mo1[l], da, da, c * P);
      else
        dnbo_relu_backward(a[l], da, da, c * P);
      dnbo_bn_backward(u[l], da, n, c, hw, par(d, params, l, DNBO_G1), mu1[l], v1[l], d->eps, da,
                       dpar(d, dparams, l, DNBO_G1), dpar(d, dparams, l, DNBO_B1));
      concat_backward_add(da, gx, l, n, c0, k, hw);
    }
    memcpy(dx0, gx[0], (size_t)(c0 * P) * sizeof(double));
    quantize(dx0, c0 * P, q);
    fm_free(mem, da, cmax * P);
    if (da2) fm_free(mem, da2, B * P);
    fm_free(mem, gx[0], c0 * P);
    for (int l = 1; l <= m; ++l) fm_free(mem, gx[l], k * P);
    free(gx);
  }
  for (int l = 1; l <= m; ++l) {
    const int64_t c = layer_cin(d, l);
    fm_free(mem, u[l], c * P);
    fm_free(mem, a[l], c * P);
    fm_free(mem, x[l], k * P);
    if (B > 0) {
      fm_free(mem, b[l], B * P);
      fm_free(mem, a2[l], B * P);
      free(mu2[l]);
      free(v2[l]);
    }
    free(mu1[l]);
    free(v1[l]);
    free(W1q[l]);
    free(W3q[l]);
  }
  free(x); free(u); free(a); free(b); free(a2); free(mu1); free(v1); free(mu2); free(v2);
  free(W1q); free(W3q); free(mo1);
  (void)cout;
  return 0;
}

int dnbo_block_naive(const dnbo_desc* d, const double* x0, const double* params, const double* dy,
                     double* y, double* dx0, double* dparams, dnbo_mem* mem) {
  return block_naive_impl(d, x0, params, dy, y, dx0, dparams, mem, 0, NULL);
}

/* The store-everything block with its ReLU decisions written to m1 / m2 (mode 0) or taken from
 * them (mode 1); layout and stats as described at dnbo_masks.  m2 may be NULL without a bottleneck.
 * bf16_storage != 0: with the storage rounding of dnbo_block_naive_bf16 on top (its distance from
 * the unrounded block under the same decisions is what bf16 storage costs by itself). */
int dnbo_block_naive_masks(const dnbo_desc* d, const double* x0, const double* params, const double* dy,
                           double* y, double* dx0, double* dparams, dnbo_mem* mem, int mode, uint8_t* m1,
                           uint8_t* m2, double* stats, int bf16_storage) {
  dnbo_masks mk = {mode, m1, m2, stats};
  return block_naive_impl(d, x0, params, dy, y, dx0, dparams, mem, bf16_storage ? 1 : 0, &mk);
}

/* The same block with bf16 storage emulated: every tensor the bf16 path keeps in memory or
 * feeds to a convolution as an operand is rounded to bfloat16 where it is produced -- the
 * BN+ReLU outputs, the conv weights as read by forward and data-gradient convs, the conv
 * outputs b_l and x_l (whose batch statistics are then those of the rounded values), the
 * gradient of x_l as a conv operand, the data gradients leaving each conv and the bottleneck
 * BN, and dx0.  Gradient accumulators, statistics and parameter gradients are not rounded.
 * It separates storage quantisation from algorithmic error: ReLU masks decided on rounded
 * values can flip, which moves a sum of random-sign gradient terms by far more than the
 * rounding itself.  x0 and dy should already hold bf16-representable values. */
int dnbo_block_naive_bf16(const dnbo_desc* d, const double* x0, const double* params, const double* dy,
                          double* y, double* dx0, double* dparams, dnbo_mem* mem) {
  return block_naive_impl(d, x0, params, dy, y, dx0, dparams, mem, 1, NULL);
}

/* ------------------------------------------- schedule 0: shared storage */

/* Section 4.  S1 holds the concat output, S2 the BN+ReLU output, S3 (with a
 * bottleneck) the second BN+ReLU output; each is one allocation sized for the
 * widest layer and overwritten by every layer.  Only the conv outputs (b_l,
 * x_l) persist.  Backward, for l = m..1, first re-runs concat and BN to put
 * layer l's data back into S1/S2/S3, then back-propagates as usual. */
int dnbo_block_shared(const dnbo_desc* d, const double* x0, const double* params, const double* dy,
                      double* y, double* dx0, double* dparams, dnbo_mem* mem) {
  const int m = d->layers;
  const int64_t n = d->n, c0 = d->c0, k = d->growth, B = d->bottleneck, H = d->h, W = d->w;
  const int64_t hw = H * W, P = n * hw, cmax = layer_cin(d, m);
  if (mem) memset(mem, 0, sizeof(*mem));
  double** x = (double**)calloc((size_t)m + 1, sizeof(double*));
  double** b = (double**)calloc((size_t)m + 1, sizeof(double*));
  double* mu1 = (double*)calloc((size_t)cmax, sizeof(double));
  double* v1 = (double*)calloc((size_t)cmax, sizeof(double));
  double* mu2 = (double*)calloc((size_t)(B > 0 ? B : 1), sizeof(double));
  double* v2 = (double*)calloc((size_t)(B > 0 ? B : 1), sizeof(double));
  double* S1 = fm_alloc(mem, cmax * P);
  double* S2 = fm_alloc(mem, cmax * P);
  double* S3 = B > 0 ? fm_alloc(mem, B * P) : NULL;

  x[0] = (double*)x0;
  for (int l = 1; l <= m; ++l) {
    const int64_t c = layer_cin(d, l);
    concat_into(S1, x, l, n, c0, k, hw);
    dnbo_bn_forward(S1, n, c, hw, par(d, params, l, DNBO_G1), par(d, params, l, DNBO_B1), d->eps,
                    S2, mu1, v1);
    dnbo_relu_inplace(S2, c * P);
    x[l] = fm_alloc(mem, k * P);
    if (B > 0) {
      b[l] = fm_alloc(mem, B * P);
      dnbo_conv_forward(S2, par(d, params, l, DNBO_W1), n, c, B, H, W, 1, b[l]);
      dnbo_bn_forward(b[l], n, B, hw, par(d, params, l, DNBO_G2), par(d, params, l, DNBO_B2),
                      d->eps, S3, mu2, v2);
      dnbo_relu_inplace(S3, B * P);
      dnbo_conv_forward(S3, par(d, params, l, DNBO_W3), n, B, k, H, W, 3, x[l]);
    } else {
      dnbo_conv_forward(S2, par(d, params, l, DNBO_W3), n, c, k, H, W, 3, x[l]);
    }
  }
  concat_into(y, x, m + 1, n, c0, k, hw);
  if (mem) mem->stored_elems = mem->live_elems;

  if (dy) {
    double** gx = (double**)calloc((size_t)m + 1, sizeof(double*));
    gx[0] = fm_alloc(mem, c0 * P);
    for (int l = 1; l <= m; ++l) gx[l] = fm_alloc(mem, k * P);
    double* da = fm_alloc(mem, cmax * P);
    double* da2 = B > 0 ? fm_alloc(mem, B * P) : NULL;
    split_dy(dy, gx, m, n, c0, k, hw);
    for (int l = m; l >= 1; --l) {
      const int64_t c = layer_cin(d, l);
      /* the additional step: re-populate the shared storage for layer l */
      concat_into(S1, x, l, n, c0, k, hw);
      dnbo_bn_forward(S1, n, c, hw, par(d, params, l, DNBO_G1), par(d, params, l, DNBO_B1), d->eps,
                      S2, mu1, v1);
      dnbo_relu_inplace(S2, c * P);
      if (B > 0) {
        dnbo_bn_forward(b[l], n, B, hw, par(d, params, l, DNBO_G2), par(d, params, l, DNBO_B2),
                        d->eps, S3, mu2, v2);
        dnbo_relu_inplace(S3, B * P);
        /* regular back-propagation from here on */
        dnbo_conv_wgrad(S3, gx[l], n, B, k, H, W, 3, dpar(d, dparams, l, DNBO_W3));
        dnbo_conv_dgrad(gx[l], par(d, params, l, DNBO_W3), n, B, k, H, W, 3, da2);
        dnbo_relu_backward(S3, da2, da2, B * P);
        dnbo_bn_backward(b[l], da2, n, B, hw, par(d, params, l, DNBO_G2), mu2, v2, d->eps, da2,
                         dpar(d, dparams, l, DNBO_G2), dpar(d, dparams, l, DNBO_B2));
        dnbo_conv_wgrad(S2, da2, n, c, B, H, W, 1, dpar(d, dparams, l, DNBO_W1));
        dnbo_conv_dgrad(da2, par(d, params, l, DNBO_W1), n, c, B, H, W, 1, da);
      } else {
        dnbo_conv_wgrad(S2, gx[l], n, c, k, H, W, 3, dpar(d, dparams, l, DNBO_W3));
        dnbo_conv_dgrad(gx[l], par(d, params, l, DNBO_W3), n, c, k, H, W, 3, da);
      }
      dnbo_relu_backward(S2, da, da, c * P);
      dnbo_bn_backward(S1, da, n, c, hw, par(d, params, l, DNBO_G1), mu1, v1, d->eps, da,
                       dpar(d, dparams, l, DNBO_G1), dpar(d, dparams, l, DNBO_B1));
      concat_backward_add(da, gx, l, n, c0, k, hw);
    }
    memcpy(dx0, gx[0], (size_t)(c0 * P) * sizeof(double));
    fm_free(mem, da, cmax * P);
    if (da2) fm_free(mem, da2, B * P);
    fm_free(mem, gx[0], c0 * P);
    for (int l = 1; l <= m; ++l) fm_free(mem, gx[l], k * P);
    free(gx);
  }
  for (int l = 1; l <= m; ++l) {
    fm_free(mem, x[l], k * P);
    if (B > 0) fm_free(mem, b[l], B * P);
  }
  fm_free(mem, S1, cmax * P);
  fm_free(mem, S2, cmax * P);
  if (S3) fm_free(mem, S3, B * P);
  free(x); free(b); free(mu1); free(v1); free(mu2); free(v2);
  return 0;
}

/* Forward only, exposing one layer's intermediates for invariant tests:
 * writes the layer's concat input u (n,C_l,hw) and pre-affine normalised
 * values xhat (n,C_l,hw) of the first BN.  Buffers sized by the caller. */
int dnbo_block_probe_layer(const dnbo_desc* d, const double* x0, const double* params, int layer,
                           double* u_out, double* xhat_out) {
  const int m = d->layers;
  if (layer < 1 || layer > m) return -1;
  const int64_t n = d->n, c0 = d->c0, k = d->growth, H = d->h, W = d->w, hw = H * W;
  const int64_t P = n * hw, cout = c0 + (int64_t)m * k;
  double* y = (double*)calloc((size_t)(cout * P), sizeof(double));
  dnbo_block_naive(d, x0, params, NULL, y, NULL, NULL, NULL);
  const int64_t c = layer_cin(d, layer);
  for (int64_t b = 0; b < n; ++b)
    memcpy(u_out + b * c * hw, y + b * cout * hw, (size_t)(c * hw) * sizeof(double));
  double* ones = (double*)calloc((size_t)c, sizeof(double));
  double* zeros = (double*)calloc((size_t)c, sizeof(double));
  double* mu = (double*)calloc((size_t)c, sizeof(double));
  double* v = (double*)calloc((size_t)c, sizeof(double));
  for (int64_t i = 0; i < c; ++i) ones[i] = 1.0;
  dnbo_bn_forward(u_out, n, c, hw, ones, zeros, d->eps, xhat_out, mu, v);
  free(ones); free(zeros); free(mu); free(v); free(y);
  return 0;
}

int dnbo_num_threads(void) {
#ifdef _OPENMP
  extern int omp_get_max_threads(void);
  return omp_get_max_threads();
#else
  return 1;
#endif
}
