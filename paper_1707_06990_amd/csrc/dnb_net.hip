// Whole training step of a CIFAR-shaped DenseNet-BC (fp32, NCHW): the glue around the dense
// blocks -- stem conv, transitions (BN -> ReLU -> 1x1 conv -> 2x2 average pool), tail
// (BN -> ReLU -> global average pool -> linear) and the mean softmax cross-entropy, forward and
// backward -- built from the block library's own kernels plus the small kernels in this file.
// Paper: Section 2 ("DenseNet Architecture": dense blocks joined by transition layers); the
// workloads of Section 5 are such networks.  The dense blocks run under the descriptor's
// schedule; the glue keeps its few BN+ReLU outputs (three per network, constant in depth).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <new>
#include <vector>

#include "../../include/dnb.h"
#include "dnb_internal.h"

namespace dnb {
namespace {

constexpr int kT = 256;

// out (n*c, h/2, w/2) = mean of each 2x2 window.
__global__ __launch_bounds__(kT) void k_avgpool2(const float* __restrict__ in, float* __restrict__ out,
                                                 int64_t planes, int h, int w) {
  const int ho = h >> 1, wo = w >> 1;
  const int64_t total = planes * ho * wo;
  for (int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x; i < total; i += (int64_t)gridDim.x * kT) {
    const int x = (int)(i % wo);
    const int64_t r = i / wo;
    const int y = (int)(r % ho);
    const int64_t p = r / ho;
    const float* s = in + (p * h + 2 * y) * w + 2 * x;
    out[i] = 0.25f * ((s[0] + s[1]) + (s[w] + s[w + 1]));
  }
}

// din (n*c, h, w): every pixel gets a quarter of its window's gradient.
__global__ __launch_bounds__(kT) void k_avgpool2_bwd(const float* __restrict__ dout, float* __restrict__ din,
                                                     int64_t planes, int h, int w) {
  const int ho = h >> 1, wo = w >> 1;
  const int64_t total = planes * h * w;
  for (int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x; i < total; i += (int64_t)gridDim.x * kT) {
    const int x = (int)(i % w);
    const int64_t r = i / w;
    const int y = (int)(r % h);
    const int64_t p = r / h;
    din[i] = 0.25f * dout[(p * ho + (y >> 1)) * wo + (x >> 1)];
  }
}

// One wave per (image, channel) plane: out[p] = mean over hw (lane-strided sums, butterfly).
__global__ __launch_bounds__(kT) void k_global_avgpool(const float* __restrict__ in, float* __restrict__ out,
                                                       int64_t planes, int hw) {
  const int64_t p = (int64_t)blockIdx.x * (kT / 64) + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (p >= planes) return;
  float s = 0.f;
  for (int q = lane; q < hw; q += 64) s += in[p * hw + q];
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) s += __shfl_xor(s, off, 64);
  if (lane == 0) out[p] = s / (float)hw;
}

__global__ __launch_bounds__(kT) void k_global_avgpool_bwd(const float* __restrict__ dout, float* __restrict__ din,
                                                           int64_t planes, int hw) {
  const int64_t total = planes * hw;
  const float inv = 1.0f / (float)hw;
  for (int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x; i < total; i += (int64_t)gridDim.x * kT)
    din[i] = dout[i / hw] * inv;
}

// logits[i][o] = bl[o] + sum_j Wl[o][j] f[i][j]; one wave per (i, o).
__global__ __launch_bounds__(kT) void k_linear(const float* __restrict__ f, const float* __restrict__ wl,
                                               const float* __restrict__ bl, float* __restrict__ logits, int n,
                                               int c, int classes) {
  const int idx = blockIdx.x * (kT / 64) + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (idx >= n * classes) return;
  const int i = idx / classes, o = idx - i * classes;
  float s = 0.f;
  for (int j = lane; j < c; j += 64) s = __fmaf_rn(wl[(int64_t)o * c + j], f[(int64_t)i * c + j], s);
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) s += __shfl_xor(s, off, 64);
  if (lane == 0) logits[idx] = s + bl[o];
}

// Per sample: log-sum-exp, loss term, dlogits = (softmax - onehot)/n.  One workgroup; each wave takes
// samples wave, wave + 4, ... and its lanes stride over the classes (butterfly maximum and sum, so
// every lane holds the same values).  Then the loss terms are added in sample order by thread 0 (n
// is a batch size: a few hundred at most).
__global__ __launch_bounds__(kT) void k_softmax_xent(const float* __restrict__ logits,
                                                     const int32_t* __restrict__ labels, float* __restrict__ dlogits,
                                                     float* __restrict__ terms, float* __restrict__ loss, int n,
                                                     int classes) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int i = wave; i < n; i += kT / 64) {
    const float* z = logits + (int64_t)i * classes;
    float mx = -3.4e38f;
    for (int o = lane; o < classes; o += 64) mx = fmaxf(mx, z[o]);
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
    float se = 0.f;
    for (int o = lane; o < classes; o += 64) se += expf(z[o] - mx);
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) se += __shfl_xor(se, off, 64);
    const float lse = mx + logf(se);
    const int lab = labels[i];
    const bool valid = lab >= 0 && lab < classes;  // a sample with a label out of range adds nothing
    if (lane == 0) terms[i] = valid ? lse - z[lab] : 0.f;
    for (int o = lane; o < classes; o += 64)
      dlogits[(int64_t)i * classes + o] = valid ? (expf(z[o] - lse) - (o == lab ? 1.f : 0.f)) / (float)n : 0.f;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    float s = 0.f;
    for (int i = 0; i < n; ++i) s += terms[i];
    *loss = s / (float)n;
  }
}

// df[i][j] = sum_o dlogits[i][o] Wl[o][j].  A workgroup owns 64 columns j for a group of 8 samples; its 16
// waves take a sixteenth of the classes each (a weight row segment is one coalesced 256-byte read per wave
// and class, used for the 8 samples; the dlogits reads are the same for the whole wave), four classes'
// loads issued before the first is used.  The waves' sums are added through LDS in wave order.
// grid (ceil(c/64), ceil(n/8)), 1024 threads.
constexpr int kLbdWaves = 16;
__global__ __launch_bounds__(64 * kLbdWaves) void k_linear_bwd_data(const float* __restrict__ dlogits,
                                                                    const float* __restrict__ wl, float* __restrict__ df,
                                                                    int n, int c, int classes) {
  __shared__ float sh[kLbdWaves - 1][8][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j = blockIdx.x * 64 + lane, jc = min(j, c - 1), i0 = blockIdx.y * 8;
  const int per = (classes + kLbdWaves - 1) / kLbdWaves, o0 = wave * per, o1 = min(classes, o0 + per);
  const float* drow[8];
#pragma unroll
  for (int u = 0; u < 8; ++u) drow[u] = dlogits + (int64_t)min(i0 + u, n - 1) * classes;  // rows past n: computed, not stored
  float acc[8];
#pragma unroll
  for (int u = 0; u < 8; ++u) acc[u] = 0.f;
  for (int o = o0; o < o1; o += 4) {
    float w[4];
    int oo[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      oo[v] = min(o + v, o1 - 1);
      w[v] = wl[(int64_t)oo[v] * c + jc];
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const float wv = o + v < o1 ? w[v] : 0.f;
#pragma unroll
      for (int u = 0; u < 8; ++u) acc[u] = __fmaf_rn(drow[u][oo[v]], wv, acc[u]);
    }
  }
  if (wave > 0) {
#pragma unroll
    for (int u = 0; u < 8; ++u) sh[wave - 1][u][lane] = acc[u];
  }
  __syncthreads();
  if (wave == 0 && j < c) {
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      float t = acc[u];
      for (int w2 = 0; w2 < kLbdWaves - 1; ++w2) t += sh[w2][u][lane];
      if (i0 + u < n) df[(int64_t)(i0 + u) * c + j] = t;
    }
  }
}

// dWl[o][j] = sum_i dlogits[i][o] f[i][j] (thread per (o, j)); dbl[o] = sum_i dlogits[i][o] (j == 0).
__global__ __launch_bounds__(kT) void k_linear_bwd_weights(const float* __restrict__ dlogits,
                                                           const float* __restrict__ f, float* __restrict__ dwl,
                                                           float* __restrict__ dbl, int n, int c, int classes) {
  const int idx = blockIdx.x * kT + threadIdx.x;
  if (idx >= classes * c) return;
  const int o = idx / c, j = idx - o * c;
  float s = 0.f, sb = 0.f;
  for (int i = 0; i < n; ++i) {
    const float d = dlogits[(int64_t)i * classes + o];
    s = __fmaf_rn(d, f[(int64_t)i * c + j], s);
    sb += d;
  }
  dwl[idx] = s;
  if (j == 0) dbl[o] = sb;
}

inline unsigned grid_for(int64_t items, int per_block, unsigned cap = 65535u * 16u) {
  int64_t g = (items + per_block - 1) / per_block;
  if (g < 1) g = 1;
  if (g > (int64_t)cap) g = cap;
  return (unsigned)g;
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

#define DNB_TRYH(expr)                                \
  do {                                                \
    if ((expr) != hipSuccess) return DNB_E_LAUNCH;    \
  } while (0)
#define DNB_TRYS(expr)                                \
  do {                                                \
    const int rc_ = (expr);                           \
    if (rc_ != DNB_OK) return rc_;                    \
  } while (0)

}  // namespace
}  // namespace dnb

namespace dnb {
// The classifier head shared by the two network steps: logits = pooled . Wl^T + bl, mean softmax
// cross-entropy with its gradient (all fp32), and the head's backward pass.
hipError_t launch_head_forward(const float* pooled, const float* wl, const float* bl, const int32_t* labels, float* logits,
                               float* dlogits, float* terms, float* loss, int n, int c, int classes, hipStream_t st) {
  hipLaunchKernelGGL(k_linear, dim3(grid_for((int64_t)n * classes, kT / 64)), dim3(kT), 0, st, pooled, wl, bl, logits, n, c,
                     classes);
  hipLaunchKernelGGL(k_softmax_xent, dim3(1), dim3(kT), 0, st, logits, labels, dlogits, terms, loss, n, classes);
  return hipGetLastError();
}

hipError_t launch_head_backward(const float* dlogits, const float* pooled, const float* wl, float* dpooled, float* dwl,
                                float* dbl, int n, int c, int classes, hipStream_t st) {
  hipLaunchKernelGGL(k_linear_bwd_data, dim3((unsigned)((c + 63) / 64), (unsigned)((n + 7) / 8)), dim3(64 * kLbdWaves), 0, st,
                     dlogits, wl, dpooled, n, c, classes);
  hipLaunchKernelGGL(k_linear_bwd_weights, dim3(grid_for((int64_t)classes * c, kT)), dim3(kT), 0, st, dlogits, pooled, dwl,
                     dbl, n, c, classes);
  return hipGetLastError();
}
}  // namespace dnb

using namespace dnb;

struct dnb_net {
  dnb_net_desc d;
  dnb_block* blk[3];
  dnb_block_desc bd[3];
  int cout[3];                       // channels leaving block b
  size_t p_stem, p_block[3], p_g[3], p_b[3], p_w[3], p_bl, p_count;  // offsets in the pack (floats)
  // workspace offsets (bytes)
  size_t o_feat[3], o_y[3], o_ws[3], o_tz[3], o_mean[3], o_istd[3];
  size_t o_tconv, o_gy, o_dtz, o_dconv, o_dfeat, o_part, o_pack[2];
  size_t o_pooled, o_logits, o_dlogits, o_terms, o_dpooled;
  size_t ws_bytes, glue_feature_bytes;
  struct Piece { const char* name; int index; size_t offset, bytes; };
  std::vector<Piece> layout;  // every carved piece of the workspace, in carve order
};

extern "C" {

int dnb_op_head_forward(const void* pooled, const void* wl, const void* bl, const int32_t* labels, void* logits,
                        void* dlogits, void* terms, float* loss, int64_t n, int64_t c, int64_t classes, void* stream) {
  if (!pooled || !wl || !bl || !labels || !logits || !dlogits || !terms || !loss) return DNB_E_NULL;
  if (n < 1 || c < 1 || classes < 1 || n > 4096 || classes > 65536 || c > ((int64_t)1 << 20)) return DNB_E_RANGE;
  if (launch_head_forward((const float*)pooled, (const float*)wl, (const float*)bl, labels, (float*)logits, (float*)dlogits,
                          (float*)terms, loss, (int)n, (int)c, (int)classes, (hipStream_t)stream) != hipSuccess)
    return DNB_E_LAUNCH;
  return DNB_OK;
}

int dnb_op_head_backward(const void* dlogits, const void* pooled, const void* wl, void* dpooled, void* dwl, void* dbl,
                         int64_t n, int64_t c, int64_t classes, void* stream) {
  if (!dlogits || !pooled || !wl || !dpooled || !dwl || !dbl) return DNB_E_NULL;
  if (n < 1 || c < 1 || classes < 1 || n > 4096 || classes > 65536 || c > ((int64_t)1 << 20)) return DNB_E_RANGE;
  if (launch_head_backward((const float*)dlogits, (const float*)pooled, (const float*)wl, (float*)dpooled, (float*)dwl,
                           (float*)dbl, (int)n, (int)c, (int)classes, (hipStream_t)stream) != hipSuccess)
    return DNB_E_LAUNCH;
  return DNB_OK;
}

int dnb_net_create(const dnb_net_desc* desc, dnb_net** out) {
  if (!desc || !out) return DNB_E_NULL;
  const dnb_net_desc& d = *desc;
  if (d.n < 1 || d.image < 4 || d.growth < 1 || d.classes < 1 || d.depth < 10 || (d.depth - 4) % 6 != 0)
    return DNB_E_BADDESC;
  if (d.image % 4 != 0 || !(d.eps >= 0.f)) return DNB_E_BADDESC;  // two 2x2 poolings
  if (d.n > 4096 || d.classes > 65536) return DNB_E_RANGE;
  dnb_net* net = new (std::nothrow) dnb_net();
  if (!net) return DNB_E_NOMEM;
  net->d = d;
  for (int b = 0; b < 3; ++b) net->blk[b] = nullptr;
  const int per = (d.depth - 4) / 6, k = d.growth;
  int c = 2 * k, s = d.image;
  size_t po = (size_t)2 * k * 27;
  net->p_stem = 0;
  for (int b = 0; b < 3; ++b) {
    dnb_block_desc bd{};
    bd.n = d.n; bd.c0 = c; bd.h = s; bd.w = s; bd.layers = per; bd.growth = k; bd.bottleneck = 4 * k;
    bd.dtype = DNB_F32; bd.layout = DNB_NCHW; bd.schedule = d.schedule; bd.eps = d.eps;
    const int rc = dnb_block_create(&bd, &net->blk[b]);
    if (rc != DNB_OK) { dnb_net_destroy(net); return rc; }
    net->bd[b] = bd;
    net->cout[b] = c + per * k;
    net->p_block[b] = po;
    po += dnb_block_param_count(net->blk[b]);
    const size_t co = (size_t)net->cout[b];
    net->p_g[b] = po; net->p_b[b] = po + co; net->p_w[b] = po + 2 * co;
    if (b < 2) {
      po += 2 * co + (co / 2) * co;
      c = (int)(co / 2);
      s /= 2;
    } else {
      net->p_bl = po + 2 * co + (size_t)d.classes * co;
      po += 2 * co + (size_t)d.classes * co + (size_t)d.classes;
    }
  }
  net->p_count = po;

  // ---- workspace plan
  size_t off = 0, glue = 0;
  auto carve = [&](size_t bytes, bool feature_map, const char* name, int index = 0) {
    const size_t o = off;
    off = align_up(off + bytes, 256);
    if (feature_map) glue += bytes;
    net->layout.push_back(dnb_net::Piece{name, index, o, bytes});
    return o;
  };
  size_t part = 0, pmax = 0;
  for (int b = 0; b < 3; ++b) {
    const dnb_block_desc& bd = net->bd[b];
    const size_t hw = (size_t)bd.h * bd.w, P = hw * d.n, co = (size_t)net->cout[b];
    net->o_feat[b] = carve((size_t)bd.c0 * P * 4, true, "feat", b);
    net->o_y[b] = carve(co * P * 4, true, "y", b);
    net->o_ws[b] = carve(dnb_block_workspace_bytes(net->blk[b]), false, "block_ws", b);
    net->o_tz[b] = carve(co * P * 4, true, "tz", b);
    net->o_mean[b] = carve(co * 4, false, "mean", b);
    net->o_istd[b] = carve(co * 4, false, "istd", b);
    if (co * P > pmax) pmax = co * P;
    auto need = [&](size_t f) { if (f > part) part = f; };
    need(bn_stats_partial_floats(d.n, (int)co, (int)hw));
    need(bn_bwd_partial_floats(d.n, (int)co, (int)hw));
    if (b < 2) {
      need(conv_wgrad_partial_floats(d.n, (int)co, (int)(co / 2), bd.h, bd.w, 1));
      net->o_pack[b] = carve(packed_weight_floats((int)(co / 2), (int)co, 1) * 4 * 2, false, "pack", b);  // forward + transposed
    }
  }
  {
    const size_t S = (size_t)d.image;
    size_t f = conv_wgrad_partial_floats(d.n, 3, 2 * k, (int)S, (int)S, 9);
    if (f > part) part = f;
  }
  // Buffers reused by every block / transition are sized for their largest user, computed (not
  // assumed): with more than 14 layers per block the input of block 1 is larger than that of block 0.
  size_t conv_max = 0, feat_max = 0;
  for (int b = 0; b < 3; ++b) {
    const dnb_block_desc& bd = net->bd[b];
    const size_t P = (size_t)d.n * bd.h * bd.w;
    if ((size_t)bd.c0 * P > feat_max) feat_max = (size_t)bd.c0 * P;
    if (b < 2 && (size_t)(net->cout[b] / 2) * P > conv_max) conv_max = (size_t)(net->cout[b] / 2) * P;
  }
  net->o_tconv = carve(conv_max * 4, true, "tconv");  // a transition's 1x1 output before pooling
  net->o_gy = carve(pmax * 4, true, "gy");         // gradient of a block output
  net->o_dtz = carve(pmax * 4, true, "dtz");        // gradient of a transition's BN+ReLU output
  net->o_dconv = carve(conv_max * 4, true, "dconv");  // gradient of a transition's conv output
  net->o_dfeat = carve(feat_max * 4, true, "dfeat");  // gradient of a block input
  net->o_part = carve(part * 4, false, "part");
  const size_t C = (size_t)net->cout[2];
  net->o_pooled = carve((size_t)d.n * C * 4, false, "pooled");
  net->o_dpooled = carve((size_t)d.n * C * 4, false, "dpooled");
  net->o_logits = carve((size_t)d.n * d.classes * 4, false, "logits");
  net->o_dlogits = carve((size_t)d.n * d.classes * 4, false, "dlogits");
  net->o_terms = carve((size_t)d.n * 4, false, "terms");
  net->ws_bytes = off;
  net->glue_feature_bytes = glue;
  *out = net;
  return DNB_OK;
}

void dnb_net_destroy(dnb_net* net) {
  if (!net) return;
  for (int b = 0; b < 3; ++b)
    if (net->blk[b]) dnb_block_destroy(net->blk[b]);
  delete net;
}

size_t dnb_net_param_count(const dnb_net* net) { return net ? net->p_count : 0; }

int dnb_net_workspace_piece(const dnb_net* net, int i, const char** name, int* index, size_t* offset, size_t* bytes) {
  if (!net || !name || !index || !offset || !bytes) return DNB_E_NULL;
  if (i < 0 || (size_t)i >= net->layout.size()) return DNB_E_RANGE;
  const dnb_net::Piece& p = net->layout[(size_t)i];
  *name = p.name; *index = p.index; *offset = p.offset; *bytes = p.bytes;
  return DNB_OK;
}
size_t dnb_net_workspace_bytes(const dnb_net* net) { return net ? net->ws_bytes : 0; }

size_t dnb_net_peak_bytes(const dnb_net* net) {
  if (!net) return 0;
  size_t t = net->glue_feature_bytes;
  for (int b = 0; b < 3; ++b) {
    // the block's x_l live inside the y buffer already counted as glue
    const dnb_block_desc& bd = net->bd[b];
    t += dnb_block_peak_bytes(net->blk[b]) - (size_t)bd.layers * bd.growth * bd.n * bd.h * bd.w * 4;
  }
  return t;
}

int dnb_net_param_offset(const dnb_net* net, int part, size_t* offset, size_t* count) {
  if (!net || !offset || !count) return DNB_E_NULL;
  const dnb_net_desc& d = net->d;
  size_t o = 0, n = 0;
  if (part == DNB_NP_STEM) { o = 0; n = (size_t)2 * d.growth * 27; }
  else if (part >= DNB_NP_BLOCK0 && part <= DNB_NP_BLOCK0 + 2) {
    const int b = part - DNB_NP_BLOCK0;
    o = net->p_block[b]; n = dnb_block_param_count(net->blk[b]);
  } else if (part >= DNB_NP_TRANS0_G && part < DNB_NP_TRANS0_G + 6) {
    const int b = (part - DNB_NP_TRANS0_G) / 3, which = (part - DNB_NP_TRANS0_G) % 3;
    const size_t co = (size_t)net->cout[b];
    o = which == 0 ? net->p_g[b] : which == 1 ? net->p_b[b] : net->p_w[b];
    n = which < 2 ? co : (co / 2) * co;
  } else if (part == DNB_NP_TAIL_G) { o = net->p_g[2]; n = (size_t)net->cout[2]; }
  else if (part == DNB_NP_TAIL_B) { o = net->p_b[2]; n = (size_t)net->cout[2]; }
  else if (part == DNB_NP_TAIL_WL) { o = net->p_w[2]; n = (size_t)d.classes * net->cout[2]; }
  else if (part == DNB_NP_TAIL_BL) { o = net->p_bl; n = (size_t)d.classes; }
  else return DNB_E_RANGE;
  *offset = o;
  *count = n;
  return DNB_OK;
}

size_t dnb_net_relu_decision_bytes(const dnb_net* net) {
  if (!net) return 0;
  size_t t = 0;
  for (int b = 0; b < 3; ++b) {
    const dnb_block_desc& bd = net->bd[b];
    t += dnb_block_relu_decision_bytes(net->blk[b], 1) + dnb_block_relu_decision_bytes(net->blk[b], 2) +
         (size_t)net->cout[b] * bd.n * bd.h * bd.w;
  }
  return t;
}

int dnb_net_relu_decisions(dnb_net* net, const void* paramsv, const void* wsv, void* outv, void* stream) {
  if (!net || !paramsv || !wsv || !outv) return DNB_E_NULL;
  const float* params = (const float*)paramsv;
  const char* ws = (const char*)wsv;
  unsigned char* out = (unsigned char*)outv;
  for (int b = 0; b < 3; ++b) {
    const dnb_block_desc& bd = net->bd[b];
    const int hw = bd.h * bd.w, co = net->cout[b];
    const size_t n1 = dnb_block_relu_decision_bytes(net->blk[b], 1), n2 = dnb_block_relu_decision_bytes(net->blk[b], 2);
    const float* y = (const float*)(ws + net->o_y[b]);
    DNB_TRYS(dnb_block_relu_decisions(net->blk[b], params + net->p_block[b], y, ws + net->o_ws[b], out, out + n1, stream));
    out += n1 + n2;
    DNB_TRYH(launch_relu_decisions(y, (int64_t)co * hw, bd.n, co, hw, params + net->p_g[b], params + net->p_b[b],
                                   (const float*)(ws + net->o_mean[b]), (const float*)(ws + net->o_istd[b]), out,
                                   (hipStream_t)stream));
    out += (size_t)co * bd.n * hw;
  }
  return DNB_OK;
}

int dnb_net_set_concurrency(dnb_net* net, int enable) {
  if (!net) return DNB_E_NULL;
  for (int b = 0; b < 3; ++b) DNB_TRYS(dnb_block_set_concurrency(net->blk[b], enable));
  return DNB_OK;
}

int dnb_net_forward(dnb_net* net, const void* xv, const int32_t* labels, const void* paramsv, float* loss,
                    float* logits_out, void* wsv, void* stream) {
  if (!net || !xv || !labels || !paramsv || !loss || !wsv) return DNB_E_NULL;
  if (misaligned(xv) || (reinterpret_cast<uintptr_t>(paramsv) & 3u) || misaligned(wsv)) return DNB_E_ALIGN;
  hipStream_t st = (hipStream_t)stream;
  const dnb_net_desc& d = net->d;
  const float* x = (const float*)xv;
  const float* params = (const float*)paramsv;
  char* ws = (char*)wsv;
  const int n = d.n, k = d.growth, S = d.image;
  float* part = (float*)(ws + net->o_part);
  float* feat0 = (float*)(ws + net->o_feat[0]);
  // stem: 3x3 conv, 3 -> 2k channels
  DNB_TRYH(launch_conv_igemm(x, (int64_t)3 * S * S, WeightView{params + net->p_stem, 27, 9, 0}, nullptr, feat0,
                             (int64_t)2 * k * S * S, n, 3, 2 * k, S, S, 9, nullptr, st));
  for (int b = 0; b < 3; ++b) {
    const dnb_block_desc& bd = net->bd[b];
    const int hw = bd.h * bd.w, co = net->cout[b];
    float* feat = (float*)(ws + net->o_feat[b]);
    float* y = (float*)(ws + net->o_y[b]);
    float* tz = (float*)(ws + net->o_tz[b]);
    float* mean = (float*)(ws + net->o_mean[b]);
    float* istd = (float*)(ws + net->o_istd[b]);
    DNB_TRYS(dnb_block_forward(net->blk[b], feat, params + net->p_block[b], y, ws + net->o_ws[b], stream));
    // BN -> ReLU of the block output (kept for the backward pass)
    DNB_TRYH(launch_bn_stats(y, (int64_t)co * hw, n, co, hw, d.eps, mean, istd, part, st));
    DNB_TRYH(launch_bn_relu(y, (int64_t)co * hw, tz, (int64_t)co * hw, nullptr, 0, n, co, hw, params + net->p_g[b],
                            params + net->p_b[b], StatsSrc{mean, istd, nullptr, 0, 0, 0, d.eps}, st));
    if (b < 2) {
      const int ch = co / 2;
      const float* W = params + net->p_w[b];
      float* pk = (float*)(ws + net->o_pack[b]);
      float* pkt = pk + packed_weight_floats(ch, co, 1);
      float* tconv = (float*)(ws + net->o_tconv);
      DNB_TRYH(launch_pack_weights(WeightView{W, co, 1, 0}, ch, co, 1, pk, st));
      DNB_TRYH(launch_pack_weights(WeightView{W, 1, co, 0}, co, ch, 1, pkt, st));  // for the data gradient
      DNB_TRYH(launch_conv_igemm(tz, (int64_t)co * hw, WeightView{W, co, 1, 0}, pk, tconv, (int64_t)ch * hw, n, co,
                                 ch, bd.h, bd.w, 1, nullptr, st));
      float* next = (float*)(ws + net->o_feat[b + 1]);
      const int64_t planes = (int64_t)n * ch;
      hipLaunchKernelGGL(k_avgpool2, dim3(grid_for(planes * (hw / 4), kT)), dim3(kT), 0, st, tconv, next, planes,
                         bd.h, bd.w);
      DNB_TRYH(hipGetLastError());
    } else {
      float* pooled = (float*)(ws + net->o_pooled);
      float* logits = (float*)(ws + net->o_logits);
      const int64_t planes = (int64_t)n * co;
      hipLaunchKernelGGL(k_global_avgpool, dim3(grid_for(planes, kT / 64)), dim3(kT), 0, st, tz, pooled, planes, hw);
      DNB_TRYH(hipGetLastError());
      DNB_TRYH(launch_head_forward(pooled, params + net->p_w[2], params + net->p_bl, labels, logits,
                                   (float*)(ws + net->o_dlogits), (float*)(ws + net->o_terms), loss, n, co, d.classes, st));
      if (logits_out)
        DNB_TRYH(launch_copy_slab(logits, (int64_t)n * d.classes, logits_out, (int64_t)n * d.classes, 1,
                                  (int64_t)n * d.classes, st));
    }
  }
  return DNB_OK;
}

int dnb_net_backward(dnb_net* net, const void* xv, const void* paramsv, void* dparamsv, void* wsv, void* stream) {
  if (!net || !xv || !paramsv || !dparamsv || !wsv) return DNB_E_NULL;
  if (misaligned(xv) || (reinterpret_cast<uintptr_t>(paramsv) & 3u) || (reinterpret_cast<uintptr_t>(dparamsv) & 3u) ||
      misaligned(wsv))
    return DNB_E_ALIGN;
  hipStream_t st = (hipStream_t)stream;
  const dnb_net_desc& d = net->d;
  const float* x = (const float*)xv;
  const float* params = (const float*)paramsv;
  float* dparams = (float*)dparamsv;
  char* ws = (char*)wsv;
  const int n = d.n, k = d.growth, S = d.image;
  float* part = (float*)(ws + net->o_part);
  float* gy = (float*)(ws + net->o_gy);
  float* dtz = (float*)(ws + net->o_dtz);
  float* dconv = (float*)(ws + net->o_dconv);
  float* dfeat = (float*)(ws + net->o_dfeat);
  {  // head: linear backward, global average pool backward
    const int C = net->cout[2], hw = net->bd[2].h * net->bd[2].w;
    const float* dlogits = (const float*)(ws + net->o_dlogits);
    const float* pooled = (const float*)(ws + net->o_pooled);
    float* dpooled = (float*)(ws + net->o_dpooled);
    DNB_TRYH(launch_head_backward(dlogits, pooled, params + net->p_w[2], dpooled, dparams + net->p_w[2],
                                  dparams + net->p_bl, n, C, d.classes, st));
    hipLaunchKernelGGL(k_global_avgpool_bwd, dim3(grid_for((int64_t)n * C * hw, kT * 4)), dim3(kT), 0, st, dpooled,
                       dtz, (int64_t)n * C, hw);
    DNB_TRYH(hipGetLastError());
  }
  for (int b = 2; b >= 0; --b) {
    const dnb_block_desc& bd = net->bd[b];
    const int hw = bd.h * bd.w, co = net->cout[b];
    const float* y = (const float*)(ws + net->o_y[b]);
    const float* mean = (const float*)(ws + net->o_mean[b]);
    const float* istd = (const float*)(ws + net->o_istd[b]);
    // BN+ReLU backward of the transition / tail: gradient of the block output
    DNB_TRYH(launch_bn_relu_bwd(y, (int64_t)co * hw, dtz, (int64_t)co * hw, gy, (int64_t)co * hw, false, n, co, hw,
                                params + net->p_g[b], params + net->p_b[b], mean, istd, dparams + net->p_g[b],
                                dparams + net->p_b[b], part, st));
    DNB_TRYS(dnb_block_backward(net->blk[b], params + net->p_block[b], y, gy, dfeat, dparams + net->p_block[b],
                                ws + net->o_ws[b], stream));
    if (b == 0) {
      DNB_TRYH(launch_conv_wgrad(x, (int64_t)3 * S * S, dfeat, (int64_t)2 * k * S * S, dparams + net->p_stem, n, 3,
                                 2 * k, S, S, 9, part, nullptr, st));
    } else {
      // through transition b-1: pool backward, then the 1x1 conv's weight and data gradients
      const dnb_block_desc& pd = net->bd[b - 1];
      const int hwp = pd.h * pd.w, cp = net->cout[b - 1], ch = cp / 2;
      const float* W = params + net->p_w[b - 1];
      const float* tzp = (const float*)(ws + net->o_tz[b - 1]);
      const float* pkt = (const float*)(ws + net->o_pack[b - 1]) + packed_weight_floats(ch, cp, 1);
      const int64_t planes = (int64_t)n * ch;
      hipLaunchKernelGGL(k_avgpool2_bwd, dim3(grid_for(planes * hwp, kT * 4)), dim3(kT), 0, st, dfeat, dconv, planes,
                         pd.h, pd.w);
      DNB_TRYH(hipGetLastError());
      DNB_TRYH(launch_conv_wgrad(tzp, (int64_t)cp * hwp, dconv, (int64_t)ch * hwp, dparams + net->p_w[b - 1], n, cp,
                                 ch, pd.h, pd.w, 1, part, nullptr, st));
      DNB_TRYH(launch_conv_igemm(dconv, (int64_t)ch * hwp, WeightView{W, 1, cp, 0}, pkt, dtz, (int64_t)cp * hwp, n, ch,
                                 cp, pd.h, pd.w, 1, nullptr, st));
    }
  }
  return DNB_OK;
}

}  // extern "C"
