// Host side of the dense-block library: descriptor validation, the workspace plan
// (which buffer lives where, and the exact feature-map byte accounting), the two
// schedules' kernel sequences, and the C ABI.  No device memory is allocated here.
#include <new>
#include <vector>

#include "../../include/dnb.h"
#include "dnb_internal.h"
#include "dnb_stats.h"

using namespace dnb;

struct dnb_block {
  dnb_block_desc d;
  int64_t hw, P;
  int cm, cout;
  size_t esz;
  // byte offsets into the workspace
  std::vector<size_t> off_b;                 // b_l, kept 1x1 conv outputs
  std::vector<size_t> off_u, off_a, off_a2;  // per layer: storage 1/2/3 (shared schedule: all equal)
  size_t off_G, off_dS2, off_dS3;
  size_t off_stat_y;                         // mean[C_out], istd[C_out]
  std::vector<size_t> off_stat_b;            // per layer mean[B], istd[B]
  std::vector<size_t> off_fold1, off_fold2;  // fused schedule: per layer folded (scale, shift) of BN1 / BN2
  size_t off_part;                           // reduction partials of the main chain (BN)
  size_t partA_floats, partB_floats;         // size of one weight-gradient partial buffer
  size_t off_partA, off_partB;               // partials of the 3x3 / 1x1 weight gradients
  // with concurrency on, backward runs three chains: the data-gradient chain on the caller's
  // stream and the two weight-gradient chains on these helper streams (created at the first
  // such backward call); off, everything runs on the caller's stream
  int concurrency;
  bool streams_ready;
  hipStream_t sA, sB;
  std::vector<hipEvent_t> ev;                // per layer: main done, db ready, S1/S2 ready, wgrad1 done
  hipEvent_t ev_start, ev_endA, ev_endB;
  std::vector<hipEvent_t> evc;  // bf16: two more events per layer (BN1 reduction done, slab share done)
  size_t off_pack;                           // packed weights of all layers
  std::vector<size_t> pk;                    // per layer: float offset of its packed weights
  std::vector<size_t> poff;                  // parameter offsets (elements) per layer
  size_t pcount;
  dnb_block_memory mem;
};

namespace {

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline int c_in(const dnb_block_desc& d, int l) { return d.c0 + (l - 1) * d.growth; }

// Per layer: g1[C] b1[C] W1[B][C] g2[B] b2[B] W3[k][B][3][3]; without a bottleneck (B = 0) the
// 3x3 conv reads the concatenation directly: g1[C] b1[C] W3[k][C][3][3].
size_t layer_params(const dnb_block_desc& d, int l) {
  const size_t c = (size_t)c_in(d, l), B = (size_t)d.bottleneck, k = (size_t)d.growth;
  if (B == 0) return 2 * c + k * c * 9;
  return 2 * c + B * c + 2 * B + k * B * 9;
}

inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }
// parameter packs are read and written with scalar accesses only (layer offsets inside a pack
// are not multiples of 16 bytes anyway): float alignment is enough
inline bool misaligned4(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 3u) != 0; }

#define DNB_TRY(expr)                                 \
  do {                                                \
    if ((expr) != hipSuccess) return DNB_E_LAUNCH;    \
  } while (0)

struct LayerParams {
  const float *g1, *b1, *W1, *g2, *b2, *W3;
};
struct LayerGrads {
  float *g1, *b1, *W1, *g2, *b2, *W3;
};

template <typename T, typename P>
T layer_ptrs(const dnb_block* b, P* base, int l) {
  const size_t c = (size_t)c_in(b->d, l), B = (size_t)b->d.bottleneck;
  P* p = base + b->poff[l];
  T r;
  r.g1 = p; r.b1 = p + c; r.W1 = p + 2 * c; r.g2 = p + 2 * c + B * c; r.b2 = r.g2 + B; r.W3 = r.b2 + B;
  return r;  // (B = 0: W1, g2, b2 are empty and W3 starts right after b1)
}


// ReLU decisions as the kernels take them: fma(u, scale, shift) > 0 with (scale, shift) folded by
// bn_fold from the cached statistics -- the one expression every forward, recomputing and backward
// kernel evaluates.  One byte per pre-activation, in the tensor's own layout: element (img, ch, q)
// of u sits at u[img*s_img + ch*s_ch + q*s_px]; `nhwc` picks the order of the compact output.
template <typename T>
__global__ __launch_bounds__(256) void k_relu_decisions(const T* __restrict__ u, int64_t s_img, int64_t s_ch,
                                                        int64_t s_px, int n, int c, int hw, int nhwc,
                                                        const float* __restrict__ gamma, const float* __restrict__ beta,
                                                        const float* __restrict__ mean, const float* __restrict__ istd,
                                                        unsigned char* __restrict__ out) {
  const int64_t total = (int64_t)n * c * hw;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    int img, ch, q;
    if (nhwc) { ch = (int)(i % c); const int64_t r = i / c; q = (int)(r % hw); img = (int)(r / hw); }
    else      { q = (int)(i % hw); const int64_t r = i / hw; ch = (int)(r % c); img = (int)(r / c); }
    float scale, shift;
    bn_fold(gamma[ch], beta[ch], mean[ch], istd[ch], scale, shift);
    const T raw = u[(int64_t)img * s_img + (int64_t)ch * s_ch + (int64_t)q * s_px];
    float v;
    if (sizeof(T) == 2) v = __uint_as_float((unsigned)raw << 16);  // bf16 bits
    else v = (float)raw;
    out[i] = __fmaf_rn(v, scale, shift) > 0.f ? 1 : 0;
  }
}

}  // namespace

namespace dnb {
hipError_t launch_relu_decisions(const float* u, int64_t stride, int n, int c, int hw, const float* gamma,
                                 const float* beta, const float* mean, const float* istd, unsigned char* out,
                                 hipStream_t st) {
  const int64_t total = (int64_t)n * c * hw;
  int64_t g = (total + 256 * 8 - 1) / (256 * 8);
  if (g < 1) g = 1;
  if (g > 65535) g = 65535;
  hipLaunchKernelGGL(k_relu_decisions<float>, dim3((unsigned)g), dim3(256), 0, st, u, stride, (int64_t)hw, (int64_t)1, n,
                     c, hw, 0, gamma, beta, mean, istd, out);
  return hipGetLastError();
}

hipError_t launch_relu_decisions_rows(const void* u, int64_t ld, int64_t P, int c, const float* gamma, const float* beta,
                                      const float* mean, const float* istd, unsigned char* out, hipStream_t st) {
  if (P >= ((int64_t)1 << 31)) return hipErrorInvalidValue;
  const int64_t total = P * c;
  int64_t g = (total + 256 * 8 - 1) / (256 * 8);
  if (g < 1) g = 1;
  if (g > 65535) g = 65535;
  hipLaunchKernelGGL(k_relu_decisions<unsigned short>, dim3((unsigned)g), dim3(256), 0, st, (const unsigned short*)u,
                     (int64_t)0, (int64_t)1, ld, 1, c, (int)P, 1, gamma, beta, mean, istd, out);
  return hipGetLastError();
}
}  // namespace dnb

namespace {

// ---- bf16 / NHWC.  x0, y, dy, dx0 and the kept b_l are bf16 with channels contiguous; y's pixel
// stride is C_out, so layer l reads y[..., :C_l] in place and writes its k new channels into
// y[..., C_l:C_l+k].  The gradient slab G is fp32 (it is accumulated into up to m times); dS2 /
// dS3 are bf16.  Fused schedule: BN+ReLU inside the convolutions' operand loads.  Shared and
// store-everything schedules (Sections 4 and 3): the concatenation is copied to storage 1, its
// BN+ReLU written to storage 2, the bottleneck's to storage 3, and the convolutions read those;
// the values are the ones the fused schedule forms on the fly, so all three give the same bits.
int forward_bf16(dnb_block* b, const void* x0, const float* params, void* yv, char* ws, hipStream_t st) {
  const dnb_block_desc& d = b->d;
  const int n = d.n, m = d.layers, k = d.growth, B = d.bottleneck, cout = b->cout;
  const int64_t P = b->P;
  unsigned short* y = (unsigned short*)yv;
  float* mean_y = (float*)(ws + b->off_stat_y);
  float* istd_y = mean_y + cout;
  float* part = (float*)(ws + b->off_part);
  unsigned short* pack = (unsigned short*)(ws + b->off_pack);
  const size_t B16 = (size_t)((B + 15) & ~15), k16 = (size_t)((k + 15) & ~15), B32 = (size_t)((B + 31) & ~31);
  DNB_TRY(nhwc::pack_block_weights(params, pack, d.c0, k, B, m, st));
  DNB_TRY(nhwc::copy_rows(x0, d.c0, y, cout, P, d.c0, st));
  int freshT = 0;
  DNB_TRY(nhwc::stats_partial(y, cout, P, d.c0, part, &freshT, st));
  int fresh_lo = 0, fresh_hi = d.c0;
  for (int l = 1; l <= m; ++l) {
    const int c = c_in(d, l);
    const LayerParams p = layer_ptrs<LayerParams, const float>(b, params, l);
    unsigned short* bl = (unsigned short*)(ws + b->off_b[l]);
    float* mean_b = (float*)(ws + b->off_stat_b[l]);
    float* istd_b = mean_b + B;
    float2* fold1 = (float2*)(ws + b->off_fold1[l]);
    float2* fold2 = (float2*)(ws + b->off_fold2[l]);
    const size_t c16 = (size_t)((c + 15) & ~15), c32 = (size_t)((c + 31) & ~31);
    const unsigned short* pk1 = pack + b->pk[l];                   // 1x1 forward
    const unsigned short* pk3 = pk1 + B16 * c32 + c16 * B32;       // 3x3 forward
    int T1 = 0, T3 = 0;
    DNB_TRY(launch_bn_fold(p.g1, p.b1, mean_y, istd_y, part, freshT, fresh_lo, fresh_hi, d.eps, c, fold1, st));
    if (d.schedule == DNB_SCHED_FUSED) {
      DNB_TRY(nhwc::conv(y, cout, false, pk1, bl, B, n, c, B, d.h, d.w, 1, fold1, part, &T1, st));
      DNB_TRY(launch_bn_fold(p.g2, p.b2, mean_b, istd_b, part, T1, 0, B, d.eps, B, fold2, st));
      DNB_TRY(nhwc::conv(bl, B, false, pk3, y + c, cout, n, B, k, d.h, d.w, 9, fold2, part, &T3, st));
    } else {
      void* S1 = ws + b->off_u[l];
      void* S2 = ws + b->off_a[l];
      void* S3 = ws + b->off_a2[l];
      DNB_TRY(nhwc::bn_relu_rows(y, cout, fold1, S2, c, S1, c, P, c, st));  // concat -> storage 1, BN+ReLU -> storage 2
      DNB_TRY(nhwc::conv(S2, c, false, pk1, bl, B, n, c, B, d.h, d.w, 1, nullptr, part, &T1, st));
      DNB_TRY(launch_bn_fold(p.g2, p.b2, mean_b, istd_b, part, T1, 0, B, d.eps, B, fold2, st));
      DNB_TRY(nhwc::bn_relu_rows(bl, B, fold2, S3, B, nullptr, 0, P, B, st));
      DNB_TRY(nhwc::conv(S3, B, false, pk3, y + c, cout, n, B, k, d.h, d.w, 9, nullptr, part, &T3, st));
    }
    freshT = T3; fresh_lo = c; fresh_hi = c + k;
  }
  (void)k16;
  return DNB_OK;
}

// The helper streams and the events of the concurrent backward pass, created on first use
// (default priority; four events per layer: main chain done, db_l ready, storage 1/2 ready,
// 1x1 weight gradient done; the bf16 path has two more events per layer and uses one helper stream).
// Destroys whatever of the helper streams and events exists (handles are null until created).
void release_helper_streams(dnb_block* b) {
  for (hipEvent_t e : b->ev) if (e) (void)hipEventDestroy(e);
  for (hipEvent_t e : b->evc) if (e) (void)hipEventDestroy(e);
  b->ev.clear();
  b->evc.clear();
  for (hipEvent_t* e : {&b->ev_start, &b->ev_endA, &b->ev_endB}) {
    if (*e) (void)hipEventDestroy(*e);
    *e = nullptr;
  }
  for (hipStream_t* s : {&b->sA, &b->sB}) {
    if (*s) (void)hipStreamDestroy(*s);
    *s = nullptr;
  }
  b->streams_ready = false;
}

int ensure_helper_streams(dnb_block* b) {
  if (b->streams_ready) return DNB_OK;
  bool ok = hipStreamCreateWithFlags(&b->sA, hipStreamNonBlocking) == hipSuccess &&
            hipStreamCreateWithFlags(&b->sB, hipStreamNonBlocking) == hipSuccess;
  b->ev.assign((size_t)4 * (b->d.layers + 2), nullptr);
  b->evc.assign((size_t)2 * (b->d.layers + 2), nullptr);
  for (auto& e : b->ev) ok = ok && hipEventCreateWithFlags(&e, hipEventDisableTiming) == hipSuccess;
  for (auto& e : b->evc) ok = ok && hipEventCreateWithFlags(&e, hipEventDisableTiming) == hipSuccess;
  for (hipEvent_t* e : {&b->ev_start, &b->ev_endA, &b->ev_endB})
    ok = ok && hipEventCreateWithFlags(e, hipEventDisableTiming) == hipSuccess;
  if (!ok) {  // nothing half-made is kept: the next call starts over
    release_helper_streams(b);
    return DNB_E_LAUNCH;
  }
  b->streams_ready = true;
  return DNB_OK;
}

int backward_bf16(dnb_block* b, const float* params, const void* yv, const void* dy, void* dx0, float* dparams,
                  char* ws, hipStream_t st) {
  const dnb_block_desc& d = b->d;
  const int n = d.n, m = d.layers, k = d.growth, B = d.bottleneck, cout = b->cout;
  const int64_t P = b->P;
  const unsigned short* y = (const unsigned short*)yv;
  float* mean_y = (float*)(ws + b->off_stat_y);
  float* istd_y = mean_y + cout;
  float* part = (float*)(ws + b->off_part);
  float* partA = (float*)(ws + b->off_partA);
  float* partB = (float*)(ws + b->off_partB);
  float* G = (float*)(ws + b->off_G);
  unsigned short* dS2 = (unsigned short*)(ws + b->off_dS2);
  unsigned short* dS3 = (unsigned short*)(ws + b->off_dS3);
  const unsigned short* pack = (const unsigned short*)(ws + b->off_pack);
  const size_t B16 = (size_t)((B + 15) & ~15), k16 = (size_t)((k + 15) & ~15), B32 = (size_t)((B + 31) & ~31);
  // Two chains.  Only the data-gradient chain (dgrad 3x3 -> BN2 bwd -> dgrad 1x1 -> BN1 reduction
  // -> BN1 element-wise pass on the k channels of x_{l-1}) carries the dependence from layer l to
  // layer l-1: the next layer down reads nothing of the slab but that slice.  With concurrency on,
  // the two weight gradients (with their sums) and the rest of BN1's element-wise pass (channels
  // below x_{l-1}, the bulk of its traffic) run on a helper stream, ordered by events where buffers
  // are shared: the 3x3 weight gradient needs the slab's slice g_l complete (layer l+1's share on
  // the main chain), the 1x1 needs db_l in dS3, which the next layer's 3x3 data gradient
  // overwrites, and the helper's share of BN1 reads dS2, which the next layer's 1x1 data gradient
  // overwrites.  Every slab element still receives its layers' contributions in the order m, m-1,
  // ...: the helper adds them in stream order and the main chain's share of layer l waits for the
  // helper's share of layer l+1, so serial and concurrent runs give the same bits.  The slices of
  // the fp32 slab that the two chains touch at the same time are disjoint channel ranges.
  //
  // One helper stream, and at every fork the main chain's launch issued first: a captured graph
  // keeps the first successor of a node on the node's hardware queue, and a change of queue costs
  // the main chain about 10 us.  Measured per step of the DenseNet-161-shaped blocks: this order
  // 13.9 ms; three helper streams with the helpers' launches first 14.4 ms (the main chain then
  // changes queue twice per layer); three helper streams with the main chain's launches first
  // 19.9 ms (the graph puts all helpers on one queue in an order that makes the main chain wait).
  if (d.schedule != DNB_SCHED_FUSED) {
    // Materialised schedules, in program order on the caller's stream.  Shared (Section 4): before
    // a layer's back-propagation its storage 3, then storage 1 and 2, are re-populated from the
    // kept conv outputs and the cached folded statistics; store-everything keeps them per layer.
    const bool recompute = d.schedule == DNB_SCHED_SHARED;
    DNB_TRY(nhwc::bf16_to_f32(dy, G, P * cout, st));
    for (int l = m; l >= 1; --l) {
      const int c = c_in(d, l);
      const LayerParams p = layer_ptrs<LayerParams, const float>(b, params, l);
      const LayerGrads gp = layer_ptrs<LayerGrads, float>(b, dparams, l);
      const unsigned short* bl = (const unsigned short*)(ws + b->off_b[l]);
      float* mean_b = (float*)(ws + b->off_stat_b[l]);
      float* istd_b = mean_b + B;
      const float2* fold1 = (const float2*)(ws + b->off_fold1[l]);
      const float2* fold2 = (const float2*)(ws + b->off_fold2[l]);
      unsigned short* S1 = (unsigned short*)(ws + b->off_u[l]);
      unsigned short* S2 = (unsigned short*)(ws + b->off_a[l]);
      unsigned short* S3 = (unsigned short*)(ws + b->off_a2[l]);
      const size_t c16 = (size_t)((c + 15) & ~15), c32 = (size_t)((c + 31) & ~31);
      const unsigned short* pk1t = pack + b->pk[l] + B16 * c32;
      const unsigned short* pk3t = pack + b->pk[l] + B16 * c32 + c16 * B32 + 9 * k16 * B32;
      const float* gl = G + c;
      if (recompute) DNB_TRY(nhwc::bn_relu_rows(bl, B, fold2, S3, B, nullptr, 0, P, B, st));
      DNB_TRY(nhwc::wgrad(S3, B, gl, cout, true, partA, gp.W3, n, B, k, d.h, d.w, 9, nullptr, st));
      DNB_TRY(nhwc::conv(gl, cout, true, pk3t, dS3, B, n, k, B, d.h, d.w, 9, nullptr, nullptr, nullptr, st));
      DNB_TRY(nhwc::bn_relu_bwd(bl, B, dS3, B, dS3, B, nullptr, 0, P, B, p.g2, p.b2, mean_b, istd_b, gp.g2, gp.b2,
                                part, st));
      if (recompute) DNB_TRY(nhwc::bn_relu_rows(y, cout, fold1, S2, c, S1, c, P, c, st));
      DNB_TRY(nhwc::wgrad(S2, c, dS3, B, false, partB, gp.W1, n, c, B, d.h, d.w, 1, nullptr, st));
      DNB_TRY(nhwc::conv(dS3, B, false, pk1t, dS2, c, n, B, c, d.h, d.w, 1, nullptr, nullptr, nullptr, st));
      // BN1+ReLU backward reads the concatenated features from storage 1; concat backward adds into the slab
      DNB_TRY(nhwc::bn_relu_bwd_reduce(S1, c, dS2, c, P, c, p.g1, p.b1, mean_y, istd_y, gp.g1, gp.b1, part, st));
      DNB_TRY(nhwc::bn_relu_bwd_apply(S1, c, dS2, c, nullptr, 0, G, cout, P, c, p.g1, p.b1, mean_y, istd_y, gp.g1, gp.b1,
                                      st));
    }
    DNB_TRY(nhwc::f32_rows_to_bf16(G, cout, dx0, P, d.c0, st));
    return DNB_OK;
  }
  const bool conc = b->concurrency != 0;
  if (conc) {
    const int rc = ensure_helper_streams(b);
    if (rc != DNB_OK) return rc;
  }
  hipStream_t sH = conc ? b->sA : st;
  enum { EV_MAIN = 0, EV_DB = 1, EV_WG1 = 3, EV_RED = 0, EV_REST = 1 };
  auto ev = [&](int l, int which) -> hipEvent_t { return conc ? b->ev[(size_t)4 * l + which] : nullptr; };
  auto evc = [&](int l, int which) -> hipEvent_t { return conc ? b->evc[(size_t)2 * l + which] : nullptr; };
  auto record = [&](hipEvent_t e, hipStream_t s) { return conc ? hipEventRecord(e, s) : hipSuccess; };
  auto wait = [&](hipStream_t s, hipEvent_t e) { return conc ? hipStreamWaitEvent(s, e, 0) : hipSuccess; };

  DNB_TRY(nhwc::bf16_to_f32(dy, G, P * cout, st));
  DNB_TRY(record(conc ? b->ev_start : nullptr, st));
  DNB_TRY(wait(sH, conc ? b->ev_start : nullptr));
  for (int l = m; l >= 1; --l) {
    const int c = c_in(d, l);
    const LayerParams p = layer_ptrs<LayerParams, const float>(b, params, l);
    const LayerGrads gp = layer_ptrs<LayerGrads, float>(b, dparams, l);
    const unsigned short* bl = (const unsigned short*)(ws + b->off_b[l]);
    float* mean_b = (float*)(ws + b->off_stat_b[l]);
    float* istd_b = mean_b + B;
    const float2* fold1 = (const float2*)(ws + b->off_fold1[l]);
    const float2* fold2 = (const float2*)(ws + b->off_fold2[l]);
    const size_t c16 = (size_t)((c + 15) & ~15), c32 = (size_t)((c + 31) & ~31);
    const unsigned short* pk1t = pack + b->pk[l] + B16 * c32;                         // 1x1 data gradient
    const unsigned short* pk3t = pack + b->pk[l] + B16 * c32 + c16 * B32 + 9 * k16 * B32;  // 3x3 data gradient
    const float* gl = G + c;  // gradient of x_l (fp32, pixel stride C_out), complete at this point

    // ---- main chain: 3x3 data gradient; dS3 is still read by layer l+1's 1x1 weight gradient
    if (l < m) DNB_TRY(wait(st, ev(l + 1, EV_WG1)));
    DNB_TRY(nhwc::conv(gl, cout, true, pk3t, dS3, B, n, k, B, d.h, d.w, 9, nullptr, nullptr, nullptr, st));

    // ---- helper: 3x3 weight gradient (BN2+ReLU of b_l recomputed in the operand staging)
    if (l < m) DNB_TRY(wait(sH, ev(l + 1, EV_MAIN)));
    DNB_TRY(nhwc::wgrad(bl, B, gl, cout, true, partA, gp.W3, n, B, k, d.h, d.w, 9, fold2, sH));

    // ---- main chain, continued: BN2 backward, then the 1x1 data gradient (dS2 and the slab's
    // lower channels are the helper's until its share of layer l+1 is done)
    DNB_TRY(nhwc::bn_relu_bwd(bl, B, dS3, B, dS3, B, nullptr, 0, P, B, p.g2, p.b2, mean_b, istd_b, gp.g2, gp.b2,
                              part, st));
    DNB_TRY(record(ev(l, EV_DB), st));
    if (l < m) DNB_TRY(wait(st, evc(l + 1, EV_REST)));
    DNB_TRY(nhwc::conv(dS3, B, false, pk1t, dS2, c, n, B, c, d.h, d.w, 1, nullptr, nullptr, nullptr, st));

    // ---- helper: 1x1 weight gradient (BN1+ReLU of y[..., :C_l] recomputed in the operand staging)
    DNB_TRY(wait(sH, ev(l, EV_DB)));
    DNB_TRY(nhwc::wgrad(y, cout, dS3, B, false, partB, gp.W1, n, c, B, d.h, d.w, 1, fold1, sH));
    DNB_TRY(record(ev(l, EV_WG1), sH));

    // ---- main chain, continued: BN1's reduction, and BN1's element-wise pass with the concat
    // backward (accumulate into the slab) on the k channels of x_{l-1}.  The channels below go to
    // the helper; layer 1 has only those (x_0); on one stream the pass is one launch.
    DNB_TRY(nhwc::bn_relu_bwd_reduce(y, cout, dS2, c, P, c, p.g1, p.b1, mean_y, istd_y, gp.g1, gp.b1, part, st));
    DNB_TRY(record(evc(l, EV_RED), st));
    const int lo = !conc ? 0 : (l >= 2 ? c - k : c);
    if (lo < c)
      DNB_TRY(nhwc::bn_relu_bwd_apply(y + lo, cout, dS2 + lo, c, nullptr, 0, G + lo, cout, P, c - lo, p.g1 + lo,
                                      p.b1 + lo, mean_y + lo, istd_y + lo, gp.g1 + lo, gp.b1 + lo, st));
    DNB_TRY(record(ev(l, EV_MAIN), st));

    // ---- helper: the same pass on the channels below
    DNB_TRY(wait(sH, evc(l, EV_RED)));
    if (lo > 0)
      DNB_TRY(nhwc::bn_relu_bwd_apply(y, cout, dS2, c, nullptr, 0, G, cout, P, lo, p.g1, p.b1, mean_y, istd_y, gp.g1,
                                      gp.b1, sH));
    DNB_TRY(record(evc(l, EV_REST), sH));
  }
  if (conc) {  // join: the caller's stream is done only when the helper chain is
    DNB_TRY(hipEventRecord(b->ev_endA, sH));
    DNB_TRY(hipStreamWaitEvent(st, b->ev_endA, 0));
  }
  DNB_TRY(nhwc::f32_rows_to_bf16(G, cout, dx0, P, d.c0, st));
  return DNB_OK;
}

// ---- fp32 NCHW without a bottleneck: each layer is BN -> ReLU -> 3x3 conv on the concatenation
// (the composite function as first defined, Section 2 "Dense connectivity").  Storage 1 and 2 are
// used exactly as with a bottleneck; there is no storage 3 and no kept b_l.  The generic
// implicit-GEMM kernels take the wide 3x3 (C_l input channels); everything runs in program order
// on the caller's stream.
int forward_plain3x3(dnb_block* b, const float* x0, const float* params, float* y, char* ws, hipStream_t st) {
  const dnb_block_desc& d = b->d;
  const int n = d.n, m = d.layers, k = d.growth, hw = (int)b->hw;
  const int64_t ys = (int64_t)b->cout * hw;
  float* mean_y = (float*)(ws + b->off_stat_y);
  float* istd_y = mean_y + b->cout;
  float* part = (float*)(ws + b->off_part);
  DNB_TRY(launch_copy_slab(x0, (int64_t)d.c0 * hw, y, ys, n, (int64_t)d.c0 * hw, st));
  int freshT = 0;
  DNB_TRY(launch_bn_stats_partial(y, ys, n, d.c0, hw, part, &freshT, st));
  int fresh_lo = 0, fresh_hi = d.c0;
  for (int l = 1; l <= m; ++l) {
    const int c = c_in(d, l);
    const LayerParams p = layer_ptrs<LayerParams, const float>(b, params, l);
    float* S1 = (float*)(ws + b->off_u[l]);
    float* S2 = (float*)(ws + b->off_a[l]);
    float* xl = y + (int64_t)c * hw;
    DNB_TRY(launch_bn_relu(y, ys, S2, (int64_t)c * hw, S1, (int64_t)c * hw, n, c, hw, p.g1, p.b1,
                           StatsSrc{mean_y, istd_y, part, freshT, fresh_lo, fresh_hi, d.eps}, st));
    DNB_TRY(launch_conv_igemm(S2, (int64_t)c * hw, WeightView{p.W3, (int64_t)c * 9, 9, 0}, nullptr, xl, ys,
                              n, c, k, d.h, d.w, 9, nullptr, st));
    if (l < m) DNB_TRY(launch_bn_stats_partial(xl, ys, n, k, hw, part, &freshT, st));
    fresh_lo = c; fresh_hi = c + k;
  }
  return DNB_OK;
}

int backward_plain3x3(dnb_block* b, const float* params, const float* y, const float* dy, float* dx0,
                      float* dparams, char* ws, hipStream_t st) {
  const dnb_block_desc& d = b->d;
  const int n = d.n, m = d.layers, k = d.growth, hw = (int)b->hw;
  const bool recompute = d.schedule == DNB_SCHED_SHARED;
  const int64_t ys = (int64_t)b->cout * hw;
  float* mean_y = (float*)(ws + b->off_stat_y);
  float* istd_y = mean_y + b->cout;
  float* part = (float*)(ws + b->off_part);
  float* partA = (float*)(ws + b->off_partA);
  float* G = (float*)(ws + b->off_G);
  float* dS2 = (float*)(ws + b->off_dS2);
  DNB_TRY(launch_copy_slab(dy, ys, G, ys, n, ys, st));
  for (int l = m; l >= 1; --l) {
    const int c = c_in(d, l);
    const LayerParams p = layer_ptrs<LayerParams, const float>(b, params, l);
    const LayerGrads gp = layer_ptrs<LayerGrads, float>(b, dparams, l);
    float* S1 = (float*)(ws + b->off_u[l]);
    float* S2 = (float*)(ws + b->off_a[l]);
    float* gl = G + (int64_t)c * hw;
    if (recompute)  // re-populate storage 1 and 2 for this layer
      DNB_TRY(launch_bn_relu(y, ys, S2, (int64_t)c * hw, S1, (int64_t)c * hw, n, c, hw, p.g1, p.b1,
                             StatsSrc{mean_y, istd_y, nullptr, 0, 0, 0, d.eps}, st));
    DNB_TRY(launch_conv_wgrad(S2, (int64_t)c * hw, gl, ys, gp.W3, n, c, k, d.h, d.w, 9, partA, nullptr, st));
    DNB_TRY(launch_conv_igemm(gl, ys, WeightView{p.W3, 9, (int64_t)c * 9, 1}, nullptr, dS2, (int64_t)c * hw,
                              n, k, c, d.h, d.w, 9, nullptr, st));
    DNB_TRY(launch_bn_relu_bwd(S1, (int64_t)c * hw, dS2, (int64_t)c * hw, G, ys, true, n, c, hw, p.g1, p.b1,
                               mean_y, istd_y, gp.g1, gp.b1, part, st));
  }
  DNB_TRY(launch_copy_slab(G, ys, dx0, (int64_t)d.c0 * hw, n, (int64_t)d.c0 * hw, st));
  return DNB_OK;
}

}  // namespace

extern "C" {

const char* dnb_status_string(int status) {
  switch (status) {
    case DNB_OK: return "ok";
    case DNB_E_BADDESC: return "invalid block descriptor";
    case DNB_E_NULL: return "null pointer argument";
    case DNB_E_ALIGN: return "pointer not 16-byte aligned";
    case DNB_E_LAUNCH: return "kernel launch failed";
    case DNB_E_UNSUPPORTED: return "dtype/layout/schedule combination not built";
    case DNB_E_RANGE: return "argument out of range";
    case DNB_E_NOMEM: return "host allocation failed";
    default: return "unknown status";
  }
}

int dnb_block_create(const dnb_block_desc* desc, dnb_block** out) {
  if (!desc || !out) return DNB_E_NULL;
  const dnb_block_desc& d = *desc;
  if (d.n < 1 || d.c0 < 1 || d.h < 1 || d.w < 1 || d.layers < 1 || d.growth < 1 || d.bottleneck < 0)
    return DNB_E_BADDESC;
  if (!(d.eps >= 0.f)) return DNB_E_BADDESC;
  if (d.dtype != DNB_F32 && d.dtype != DNB_BF16) return DNB_E_BADDESC;
  if (d.layout != DNB_NCHW && d.layout != DNB_NHWC) return DNB_E_BADDESC;
  if (d.schedule != DNB_SCHED_SHARED && d.schedule != DNB_SCHED_STORE_ALL && d.schedule != DNB_SCHED_FUSED)
    return DNB_E_BADDESC;
  // built combinations: fp32 + NCHW, bf16 + NHWC (all schedules each)
  const bool bf16 = d.dtype == DNB_BF16;
  if (bf16 ? (d.layout != DNB_NHWC) : (d.layout != DNB_NCHW)) return DNB_E_UNSUPPORTED;
  // no bottleneck (BN-ReLU-3x3 on the concatenation): fp32, materialised schedules
  if (d.bottleneck == 0 && (bf16 || d.schedule == DNB_SCHED_FUSED)) return DNB_E_UNSUPPORTED;
  // bf16 kernels move 8 channels (16 bytes) at a time
  if (bf16 && (d.c0 % 8 || d.growth % 8 || d.bottleneck % 8)) return DNB_E_UNSUPPORTED;
  // ... and the 3x3 double-buffers 64 pixels + halo x 64 channels in 64 KB of LDS, with the folded
  // BN parameters of its input channels behind them in the fused schedule (the 1x1 likewise, with
  // no halo and the widest layer's channels): shapes beyond that are refused here, not at launch
  if (bf16) {
    const size_t fold3 = d.schedule == DNB_SCHED_FUSED ? (size_t)d.bottleneck * 8 : 0;
    const size_t fold1 = d.schedule == DNB_SCHED_FUSED ? (size_t)(d.c0 + (d.layers - 1) * d.growth) * 8 : 0;
    if ((size_t)2 * (64 + 2 * (d.w + 1)) * 72 * 2 + fold3 > 64 * 1024 || 64 + 2 * (d.w + 1) > 256) return DNB_E_UNSUPPORTED;
    if ((size_t)2 * 64 * 72 * 2 + fold1 > 64 * 1024) return DNB_E_UNSUPPORTED;
  }
  // the fp32 fused schedule exists only in the 16-byte-vector kernels (pixel rows a multiple of 4)
  if (!bf16 && d.schedule == DNB_SCHED_FUSED) {
    // ... and its 3x3 stages all B channels of a 64-pixel tile (+ halo) in 64 KB of LDS
    int pitch = (64 + 2 * d.w + 8 + 31) / 32 * 32 + 4;
    if (pitch - 32 >= 64 + 2 * d.w + 8) pitch -= 32;
    if (d.w % 4 != 0 || (size_t)((d.bottleneck + 3) & ~3) * pitch * sizeof(float) > 64 * 1024)
      return DNB_E_UNSUPPORTED;
    // ... and its weight gradients (BN+ReLU in their operand loads) need the fast kernels' tile plans
    if (d.h * d.w % 4 != 0 || conv_wgrad_fast_partial_floats(d.n, d.bottleneck, d.growth, d.h, d.w, 9) == 0 ||
        conv_wgrad_fast_partial_floats(d.n, d.c0, d.bottleneck, d.h, d.w, 1) == 0)
      return DNB_E_UNSUPPORTED;
  }
  const int64_t hw = (int64_t)d.h * d.w, P = hw * d.n;
  const int64_t cout = (int64_t)d.c0 + (int64_t)d.layers * d.growth;
  if (cout * P >= (int64_t)1 << 31 || (int64_t)d.bottleneck * P >= (int64_t)1 << 31) return DNB_E_RANGE;
  if (!bf16 && d.schedule != DNB_SCHED_FUSED) {
    // the materialised fp32 schedules fall back to the any-shape kernels: their 3x3 tiles (64 pixels
    // plus a halo of two rows) must fit LDS, else the shape is refused here rather than at launch
    const int cin3 = d.bottleneck > 0 ? d.bottleneck : d.c0 + (d.layers - 1) * d.growth;
    if (!conv_generic_fits(d.n, cin3, d.growth, d.h, d.w, 9)) return DNB_E_UNSUPPORTED;
  }

  dnb_block* b = new (std::nothrow) dnb_block();
  if (!b) return DNB_E_NOMEM;
  b->d = d;
  b->hw = hw;
  b->P = P;
  const int m = d.layers, k = d.growth, B = d.bottleneck;
  b->cm = c_in(d, m);
  b->cout = (int)cout;
  b->esz = bf16 ? 2 : 4;
  const size_t Ps = (size_t)P * b->esz;
  const size_t Pg = (size_t)P * 4;  // the gradient slab G is fp32 for both storage types

  b->poff.assign(m + 2, 0);
  size_t po = 0;
  for (int l = 1; l <= m; ++l) { b->poff[l] = po; po += layer_params(d, l); }
  b->pcount = po;

  // ---- workspace plan; every buffer starts on a 256-byte boundary
  size_t off = 0, fm_exact = 0;
  auto carve = [&](size_t bytes, bool feature_map) {
    const size_t o = off;
    off = align_up(off + bytes, 256);
    if (feature_map) fm_exact += bytes;
    return o;
  };
  b->off_b.assign(m + 1, 0);
  b->off_u.assign(m + 1, 0);
  b->off_a.assign(m + 1, 0);
  b->off_a2.assign(m + 1, 0);
  b->off_stat_b.assign(m + 1, 0);
  dnb_block_memory& mem = b->mem;
  mem = dnb_block_memory{};
  size_t sigma_c = 0;
  for (int l = 1; l <= m; ++l) sigma_c += (size_t)c_in(d, l);
  for (int l = 1; l <= m; ++l) b->off_b[l] = carve((size_t)B * Ps, true);
  if (d.schedule == DNB_SCHED_FUSED) {
    // nothing of storage 1/2/3 is materialised: BN+ReLU is applied inside the conv operand loads
    mem.stored_fwd_bytes = (uint64_t)((size_t)m * B + (size_t)m * k) * Ps;
    mem.shared_fwd_bytes = 0;
  } else if (d.schedule == DNB_SCHED_SHARED) {
    const size_t s1 = carve((size_t)b->cm * Ps, true), s2 = carve((size_t)b->cm * Ps, true),
                 s3 = carve((size_t)B * Ps, true);
    for (int l = 1; l <= m; ++l) { b->off_u[l] = s1; b->off_a[l] = s2; b->off_a2[l] = s3; }
    mem.stored_fwd_bytes = (uint64_t)((size_t)m * B + (size_t)m * k) * Ps;
    mem.shared_fwd_bytes = (uint64_t)(2 * (size_t)b->cm + B) * Ps;
  } else {
    for (int l = 1; l <= m; ++l) {
      b->off_u[l] = carve((size_t)c_in(d, l) * Ps, true);
      b->off_a[l] = carve((size_t)c_in(d, l) * Ps, true);
      b->off_a2[l] = carve((size_t)B * Ps, true);
    }
    mem.stored_fwd_bytes = (uint64_t)(2 * sigma_c + (size_t)m * (2 * B + k)) * Ps;
    mem.shared_fwd_bytes = 0;
  }
  b->off_G = carve((size_t)cout * Pg, true);
  b->off_dS2 = carve((size_t)b->cm * Ps, true);
  b->off_dS3 = carve((size_t)B * Ps, true);
  mem.grad_bytes = (uint64_t)((size_t)cout * Pg + ((size_t)b->cm + B) * Ps);
  mem.peak_bytes = mem.stored_fwd_bytes + mem.shared_fwd_bytes + mem.grad_bytes;
  // the x_l part of `stored` lives in the caller's y, everything else was carved above
  if (fm_exact + (size_t)m * k * Ps != mem.peak_bytes) { delete b; return DNB_E_BADDESC; }

  b->off_stat_y = carve((size_t)cout * 2 * sizeof(float), false);
  for (int l = 1; l <= m; ++l) b->off_stat_b[l] = carve((size_t)B * 2 * sizeof(float), false);
  mem.stats_bytes = (uint64_t)((size_t)cout * 2 + (size_t)m * B * 2) * sizeof(float);
  b->off_fold1.assign(m + 1, 0);
  b->off_fold2.assign(m + 1, 0);
  if (d.schedule == DNB_SCHED_FUSED || bf16) {  // (bf16 keeps the folded statistics in every schedule)
    for (int l = 1; l <= m; ++l) {
      b->off_fold1[l] = carve((size_t)c_in(d, l) * 2 * sizeof(float), false);
      b->off_fold2[l] = carve((size_t)B * 2 * sizeof(float), false);
      mem.stats_bytes += (uint64_t)((size_t)c_in(d, l) + B) * 2 * sizeof(float);
    }
  }

  size_t part = 0, partA = 0, partB = 0;
  auto need = [&](size_t floats) { if (floats > part) part = floats; };
  b->pk.assign(m + 2, 0);
  size_t pack = 0;  // in floats
  if (bf16) {
    need(nhwc::stats_partial_floats(P, d.c0));
    need(nhwc::conv_stats_partial_floats(d.n, B, d.h, d.w));
    need(nhwc::conv_stats_partial_floats(d.n, k, d.h, d.w));
    need(nhwc::bn_bwd_partial_floats(P, B));
    size_t pe = 0;  // bf16 elements
    for (int l = 1; l <= m; ++l) {
      need(nhwc::bn_bwd_partial_floats(P, c_in(d, l)));
      const size_t f = nhwc::wgrad_partial_floats(d.n, c_in(d, l), B, d.h, d.w, 1);
      if (f > partB) partB = f;
      b->pk[l] = pe;
      pe += nhwc::packed_layer_elems(c_in(d, l), k, B);
    }
    partA = nhwc::wgrad_partial_floats(d.n, B, k, d.h, d.w, 9);
    pack = (pe + 1) / 2;
  } else {
    need(bn_stats_partial_floats(d.n, d.c0, (int)hw));
    need(bn_stats_partial_floats(d.n, k, (int)hw));
    if (B > 0) {
      need(bn_stats_partial_floats(d.n, B, (int)hw));
      need(bn_bwd_partial_floats(d.n, B, (int)hw));
      need(conv_stats_partial_floats(d.n, B, d.h, d.w));  // epilogue statistics of the two convs
    }
    need(conv_stats_partial_floats(d.n, k, d.h, d.w));
    for (int l = 1; l <= m; ++l) {
      need(bn_bwd_partial_floats(d.n, c_in(d, l), (int)hw));
      const size_t f = B > 0 ? conv_wgrad_partial_floats(d.n, c_in(d, l), B, d.h, d.w, 1) : 0;
      if (f > partB) partB = f;
    }
    if (B == 0) {
      for (int l = 1; l <= m; ++l) {
        const size_t f = conv_wgrad_partial_floats(d.n, c_in(d, l), k, d.h, d.w, 9);
        if (f > partA) partA = f;
      }
    } else {
      partA = conv_wgrad_partial_floats(d.n, B, k, d.h, d.w, 9);
      for (int l = 1; l <= m; ++l) { b->pk[l] = pack; pack += packed_layer_floats(c_in(d, l), k, B); }
    }
  }
  mem.scratch_bytes = (uint64_t)(part + (bf16 ? 1 : 2) * (partA + partB) + pack) * sizeof(float);
  b->off_part = carve(part * sizeof(float), false);
  // fp32: two buffers each, used alternately by consecutive layers (a layer's partials are
  // summed by extra workgroups of the next layer's weight-gradient launch)
  b->partA_floats = partA;
  b->partB_floats = partB;
  const size_t nbuf = bf16 ? 1 : 2;
  b->off_partA = carve(nbuf * partA * sizeof(float), false);
  b->off_partB = carve(nbuf * partB * sizeof(float), false);
  b->off_pack = carve(pack * sizeof(float), false);
  // measured on MI355X: with the weight gradients on helper streams the fp32 step is slower
  // (idle time between dependent launches of different streams outweighs the overlap), the
  // bf16 step, whose helper chains carry long kernels, a fifth faster
  b->concurrency = d.dtype == DNB_BF16 ? 1 : 0;
  b->streams_ready = false;
  b->sA = b->sB = nullptr;
  b->ev_start = b->ev_endA = b->ev_endB = nullptr;
  mem.workspace_bytes = (uint64_t)off;
  *out = b;
  return DNB_OK;
}

void dnb_block_destroy(dnb_block* b) {
  if (!b) return;
  release_helper_streams(b);
  delete b;
}

int dnb_block_set_concurrency(dnb_block* b, int enable) {
  if (!b) return DNB_E_NULL;
  b->concurrency = enable ? 1 : 0;
  return DNB_OK;
}

size_t dnb_block_peak_bytes(const dnb_block* b) { return b ? (size_t)b->mem.peak_bytes : 0; }
size_t dnb_block_workspace_bytes(const dnb_block* b) { return b ? (size_t)b->mem.workspace_bytes : 0; }

int dnb_block_memory_breakdown(const dnb_block* b, dnb_block_memory* out) {
  if (!b || !out) return DNB_E_NULL;
  *out = b->mem;
  return DNB_OK;
}

size_t dnb_block_param_count(const dnb_block* b) { return b ? b->pcount : 0; }
size_t dnb_block_param_bytes(const dnb_block* b) { return b ? b->pcount * sizeof(float) : 0; }

size_t dnb_block_relu_decision_bytes(const dnb_block* b, int which) {
  if (!b) return 0;
  size_t sigma_c = 0;
  for (int l = 1; l <= b->d.layers; ++l) sigma_c += (size_t)c_in(b->d, l);
  if (which == 1) return sigma_c * (size_t)b->P;
  if (which == 2) return (size_t)b->d.layers * (size_t)b->d.bottleneck * (size_t)b->P;
  return 0;
}

int dnb_block_relu_decisions(dnb_block* b, const void* paramsv, const void* yv, const void* wsv, void* d1v, void* d2v,
                             void* stream) {
  if (!b || !paramsv || !yv || !wsv || !d1v || (b->d.bottleneck > 0 && !d2v)) return DNB_E_NULL;
  if (misaligned4(paramsv) || misaligned(yv) || misaligned(wsv)) return DNB_E_ALIGN;
  const dnb_block_desc& d = b->d;
  hipStream_t st = (hipStream_t)stream;
  const bool nhwc = d.layout == DNB_NHWC;
  const int n = d.n, m = d.layers, B = d.bottleneck, hw = (int)b->hw, cout = b->cout;
  const float* params = (const float*)paramsv;
  const char* ws = (const char*)wsv;
  const float* mean_y = (const float*)(ws + b->off_stat_y);
  const float* istd_y = mean_y + cout;
  unsigned char* d1 = (unsigned char*)d1v;
  unsigned char* d2 = (unsigned char*)d2v;
  auto launch = [&](const void* u, int64_t s_img, int64_t s_ch, int64_t s_px, int c, const float* g, const float* be,
                    const float* mu, const float* is, unsigned char* out) {
    const int64_t total = (int64_t)n * c * hw;
    const unsigned grid = (unsigned)((total + 256 * 8 - 1) / (256 * 8) < 1 ? 1 : (total + 256 * 8 - 1) / (256 * 8) > 65535 ? 65535 : (total + 256 * 8 - 1) / (256 * 8));
    if (d.dtype == DNB_BF16)
      hipLaunchKernelGGL(k_relu_decisions<unsigned short>, dim3(grid), dim3(256), 0, st, (const unsigned short*)u, s_img,
                         s_ch, s_px, n, c, hw, nhwc ? 1 : 0, g, be, mu, is, out);
    else
      hipLaunchKernelGGL(k_relu_decisions<float>, dim3(grid), dim3(256), 0, st, (const float*)u, s_img, s_ch, s_px, n,
                         c, hw, nhwc ? 1 : 0, g, be, mu, is, out);
    return hipGetLastError();
  };
  size_t o1 = 0;
  for (int l = 1; l <= m; ++l) {
    const int c = c_in(d, l);
    const LayerParams p = layer_ptrs<LayerParams, const float>(b, params, l);
    // the layer's concatenated input is y[:, :C_l] in place
    if (nhwc) DNB_TRY(launch(yv, (int64_t)hw * cout, 1, cout, c, p.g1, p.b1, mean_y, istd_y, d1 + o1));
    else      DNB_TRY(launch(yv, (int64_t)cout * hw, hw, 1, c, p.g1, p.b1, mean_y, istd_y, d1 + o1));
    o1 += (size_t)c * (size_t)b->P;
    if (B > 0) {
      const void* bl = ws + b->off_b[l];
      const float* mean_b = (const float*)(ws + b->off_stat_b[l]);
      if (nhwc) DNB_TRY(launch(bl, (int64_t)hw * B, 1, B, B, p.g2, p.b2, mean_b, mean_b + B, d2 + (size_t)(l - 1) * B * b->P));
      else      DNB_TRY(launch(bl, (int64_t)B * hw, hw, 1, B, p.g2, p.b2, mean_b, mean_b + B, d2 + (size_t)(l - 1) * B * b->P));
    }
  }
  return DNB_OK;
}

int dnb_block_param_offset(const dnb_block* b, int layer, int which, size_t* offset, size_t* count) {
  if (!b || !offset || !count) return DNB_E_NULL;
  if (layer < 1 || layer > b->d.layers || which < DNB_P_G1 || which > DNB_P_W3) return DNB_E_RANGE;
  const size_t c = (size_t)c_in(b->d, layer), B = (size_t)b->d.bottleneck, k = (size_t)b->d.growth;
  size_t o = b->poff[layer], n = 0;
  switch (which) {
    case DNB_P_G1: n = c; break;
    case DNB_P_B1: o += c; n = c; break;
    case DNB_P_W1: o += 2 * c; n = B * c; break;
    case DNB_P_G2: o += 2 * c + B * c; n = B; break;
    case DNB_P_B2: o += 2 * c + B * c + B; n = B; break;
    default: o += 2 * c + B * c + 2 * B; n = k * (B ? B : c) * 9; break;
  }
  *offset = o;
  *count = n;
  return DNB_OK;
}

int dnb_block_forward(dnb_block* b, const void* x0v, const void* paramsv, void* yv, void* wsv,
                      void* stream) {
  if (!b || !x0v || !paramsv || !yv || !wsv) return DNB_E_NULL;
  if (misaligned(x0v) || misaligned4(paramsv) || misaligned(yv) || misaligned(wsv)) return DNB_E_ALIGN;
  hipStream_t st = (hipStream_t)stream;
  const dnb_block_desc& d = b->d;
  if (d.dtype == DNB_BF16) return forward_bf16(b, x0v, (const float*)paramsv, yv, (char*)wsv, st);
  if (d.bottleneck == 0)
    return forward_plain3x3(b, (const float*)x0v, (const float*)paramsv, (float*)yv, (char*)wsv, st);
  const int n = d.n, m = d.layers, k = d.growth, B = d.bottleneck, hw = (int)b->hw;
  const float* x0 = (const float*)x0v;
  const float* params = (const float*)paramsv;
  float* y = (float*)yv;
  char* ws = (char*)wsv;
  const int64_t ys = (int64_t)b->cout * hw;  // image stride of y
  float* mean_y = (float*)(ws + b->off_stat_y);
  float* istd_y = mean_y + b->cout;
  float* part = (float*)(ws + b->off_part);

  // y[:, 0:c0] = x0, and the statistics of those channels (every later layer reuses them:
  // a channel's batch statistics do not depend on which layer consumes it)
  float* pack = (float*)(ws + b->off_pack);
  const size_t B16 = (size_t)((B + 15) & ~15), k16 = (size_t)((k + 15) & ~15);
  DNB_TRY(launch_pack_block_weights(params, pack, d.c0, k, B, m, st));
  DNB_TRY(launch_copy_slab(x0, (int64_t)d.c0 * hw, y, ys, n, (int64_t)d.c0 * hw, st));
  // Statistics exist first as partials in `part` -- from the statistics kernel (block input) or
  // from the epilogue of the convolution that produced the feature -- and are merged by the
  // first kernel that needs them; `fresh` tracks which channels of y still only have partials.
  const bool fused = d.schedule == DNB_SCHED_FUSED;
  int freshT = 0;
  DNB_TRY(launch_bn_stats_partial(y, ys, n, d.c0, hw, part, &freshT, st));
  int fresh_lo = 0, fresh_hi = d.c0;
  for (int l = 1; l <= m; ++l) {
    const int c = c_in(d, l);
    const LayerParams p = layer_ptrs<LayerParams, const float>(b, params, l);
    float* S1 = (float*)(ws + b->off_u[l]);
    float* S2 = (float*)(ws + b->off_a[l]);
    float* S3 = (float*)(ws + b->off_a2[l]);
    float* bl = (float*)(ws + b->off_b[l]);
    float* mean_b = (float*)(ws + b->off_stat_b[l]);
    float* istd_b = mean_b + B;
    float2* fold1 = (float2*)(ws + b->off_fold1[l]);
    float2* fold2 = (float2*)(ws + b->off_fold2[l]);
    const size_t c16 = (size_t)((c + 15) & ~15);
    const float* pk1 = pack + b->pk[l];               // 1x1 forward
    const float* pk3 = pk1 + 2 * B16 * c16;           // 3x3 forward
    float* xl = y + (int64_t)c * hw;  // x_l goes straight into its channel range of y
    ConvExtras e1{nullptr, part, 0, false}, e3{nullptr, part, 0, false};
    if (fused) {
      // BN1+ReLU is applied in the 1x1's operand load, BN2+ReLU while the 3x3 stages its tile
      DNB_TRY(launch_bn_fold(p.g1, p.b1, mean_y, istd_y, part, freshT, fresh_lo, fresh_hi, d.eps, c,
                             fold1, st));
      e1.fold = fold1;
      DNB_TRY(launch_conv_igemm(y, ys, WeightView{p.W1, c, 1, 0}, pk1, bl, (int64_t)B * hw, n, c, B,
                                d.h, d.w, 1, &e1, st));
      DNB_TRY(launch_bn_fold(p.g2, p.b2, mean_b, istd_b, part, e1.stats_T, 0, B, d.eps, B, fold2, st));
      e3.fold = fold2;
      DNB_TRY(launch_conv_igemm(bl, (int64_t)B * hw, WeightView{p.W3, (int64_t)B * 9, 9, 0}, pk3, xl, ys,
                                n, B, k, d.h, d.w, 9, &e3, st));
      freshT = e3.stats_T;
    } else {
      // concat -> storage 1 and BN+ReLU -> storage 2, one pass over the features
      DNB_TRY(launch_bn_relu(y, ys, S2, (int64_t)c * hw, S1, (int64_t)c * hw, n, c, hw, p.g1, p.b1,
                             StatsSrc{mean_y, istd_y, part, freshT, fresh_lo, fresh_hi, d.eps}, st));
      DNB_TRY(launch_conv_igemm(S2, (int64_t)c * hw, WeightView{p.W1, c, 1, 0}, pk1, bl, (int64_t)B * hw,
                                n, c, B, d.h, d.w, 1, &e1, st));
      int bT = e1.stats_T;
      if (!e1.used_fast) DNB_TRY(launch_bn_stats_partial(bl, (int64_t)B * hw, n, B, hw, part, &bT, st));
      DNB_TRY(launch_bn_relu(bl, (int64_t)B * hw, S3, (int64_t)B * hw, nullptr, 0, n, B, hw, p.g2, p.b2,
                             StatsSrc{mean_b, istd_b, part, bT, 0, B, d.eps}, st));
      if (l == m) e3.stats_part = nullptr;  // nobody normalises x_m inside the block
      DNB_TRY(launch_conv_igemm(S3, (int64_t)B * hw, WeightView{p.W3, (int64_t)B * 9, 9, 0}, pk3, xl, ys,
                                n, B, k, d.h, d.w, 9, &e3, st));
      freshT = e3.stats_T;
      if (l < m && !e3.used_fast) DNB_TRY(launch_bn_stats_partial(xl, ys, n, k, hw, part, &freshT, st));
    }
    fresh_lo = c; fresh_hi = c + k;
  }
  return DNB_OK;
}

int dnb_block_backward(dnb_block* b, const void* paramsv, const void* yv, const void* dyv,
                       void* dx0v, void* dparamsv, void* wsv, void* stream) {
  if (!b || !paramsv || !yv || !dyv || !dx0v || !dparamsv || !wsv) return DNB_E_NULL;
  if (misaligned4(paramsv) || misaligned(yv) || misaligned(dyv) || misaligned(dx0v) ||
      misaligned4(dparamsv) || misaligned(wsv))
    return DNB_E_ALIGN;
  hipStream_t st = (hipStream_t)stream;
  const dnb_block_desc& d = b->d;
  if (d.dtype == DNB_BF16)
    return backward_bf16(b, (const float*)paramsv, yv, dyv, dx0v, (float*)dparamsv, (char*)wsv, st);
  if (d.bottleneck == 0)
    return backward_plain3x3(b, (const float*)paramsv, (const float*)yv, (const float*)dyv, (float*)dx0v,
                             (float*)dparamsv, (char*)wsv, st);
  const int n = d.n, m = d.layers, k = d.growth, B = d.bottleneck, hw = (int)b->hw;
  const bool recompute = d.schedule == DNB_SCHED_SHARED;
  const bool fused = d.schedule == DNB_SCHED_FUSED;
  const float* params = (const float*)paramsv;
  const float* y = (const float*)yv;
  float* dparams = (float*)dparamsv;
  char* ws = (char*)wsv;
  const int64_t ys = (int64_t)b->cout * hw;
  float* mean_y = (float*)(ws + b->off_stat_y);
  float* istd_y = mean_y + b->cout;
  float* part = (float*)(ws + b->off_part);
  float* G = (float*)(ws + b->off_G);      // gradient slab, same shape as y
  float* dS2 = (float*)(ws + b->off_dS2);  // gradient of storage 2 (widest layer)
  float* dS3 = (float*)(ws + b->off_dS3);  // gradient of storage 3, then of b_l

  const float* pack = (const float*)(ws + b->off_pack);  // packed by the forward pass
  const size_t B16 = (size_t)((B + 15) & ~15), k16 = (size_t)((k + 15) & ~15);
  float* partA = (float*)(ws + b->off_partA);
  float* partB = (float*)(ws + b->off_partB);

  // Three chains.  Only the data-gradient chain (dgrad 3x3 -> BN2 bwd -> dgrad 1x1 -> BN1 bwd)
  // carries the dependence from layer l to layer l-1; the weight gradients, and the
  // recomputation that feeds only them, hang off it.  With concurrency on they run on two
  // helper streams, ordered by events exactly where buffers are shared:
  //   A: [recompute storage 3] -> wgrad 3x3 -> sum        (needs g_l complete)
  //   B: [recompute storage 1,2] -> wgrad 1x1 -> sum      (needs db_l; storage 1 also feeds BN1 bwd)
  // In the fused schedule there is nothing to recompute and both weight gradients go out as one
  // paired launch on a single helper stream, issued after the main chain's 1x1 data gradient so
  // that a captured graph keeps the main chain on its hardware queue (5.88 ms per DenseNet-BC-100
  // step against 6.53 ms with two helper streams and separate launches).
  // With concurrency off (the fp32 default, 5.56 ms) the same kernels run on the caller's stream,
  // and the leaves are gathered: a layer's two weight gradients, the previous layer's partial
  // sums and the reduction pass of BN1's backward go out as one launch just before BN1's apply
  // pass; every wait of the main chain for another queue costs about 10 us, more than the
  // overlap buys at these kernel sizes.
  const bool conc = b->concurrency != 0;
  if (conc) {
    const int rc = ensure_helper_streams(b);
    if (rc != DNB_OK) return rc;
  }
  // fused schedule with concurrency on: one helper stream carries each layer's paired weight
  // gradients (there are no recomputation kernels to share buffers with)
  const bool oneh = conc && fused;
  hipStream_t sA = conc ? b->sA : st, sB = conc ? (oneh ? b->sA : b->sB) : st;
  enum { EV_MAIN = 0, EV_DB = 1, EV_S12 = 2, EV_WG1 = 3 };
  auto ev = [&](int l, int which) -> hipEvent_t { return conc ? b->ev[(size_t)4 * l + which] : nullptr; };
  auto record = [&](hipEvent_t e, hipStream_t s) { return conc ? hipEventRecord(e, s) : hipSuccess; };
  auto wait = [&](hipStream_t s, hipEvent_t e) { return conc ? hipStreamWaitEvent(s, e, 0) : hipSuccess; };

  PendingSum pendA, pendB, nextA, nextB;
  DNB_TRY(launch_copy_slab((const float*)dyv, ys, G, ys, n, ys, st));
  DNB_TRY(record(conc ? b->ev_start : nullptr, st));
  DNB_TRY(wait(sA, conc ? b->ev_start : nullptr));
  DNB_TRY(wait(sB, conc ? b->ev_start : nullptr));
  for (int l = m; l >= 1; --l) {
    const int c = c_in(d, l);
    const LayerParams p = layer_ptrs<LayerParams, const float>(b, params, l);
    const LayerGrads gp = layer_ptrs<LayerGrads, float>(b, dparams, l);
    float* S1 = (float*)(ws + b->off_u[l]);
    float* S2 = (float*)(ws + b->off_a[l]);
    float* S3 = (float*)(ws + b->off_a2[l]);
    float* bl = (float*)(ws + b->off_b[l]);
    float* mean_b = (float*)(ws + b->off_stat_b[l]);
    float* istd_b = mean_b + B;
    float* gl = G + (int64_t)c * hw;  // complete gradient of x_l: all later layers have added theirs
    const size_t c16 = (size_t)((c + 15) & ~15);
    const float* pk1t = pack + b->pk[l] + B16 * c16;                    // 1x1 data gradient
    const float* pk3t = pack + b->pk[l] + 2 * B16 * c16 + 9 * k16 * B16;  // 3x3 data gradient

    // ---- chain A: storage 3 and the 3x3 weight gradient.  g_l is complete once layer l+1's
    // BN1 backward has run; storage 3 is free because the previous wgrad ran on this stream.
    if (l < m) DNB_TRY(wait(sA, ev(l + 1, EV_MAIN)));
    if (recompute)  // re-populate storage 3 from the kept b_l and its cached statistics
      DNB_TRY(launch_bn_relu(bl, (int64_t)B * hw, S3, (int64_t)B * hw, nullptr, 0, n, B, hw, p.g2,
                             p.b2, StatsSrc{mean_b, istd_b, nullptr, 0, 0, 0, d.eps}, sA));
    // (the sum of this launch's partials is left to the next layer's launch on this chain).
    // On one stream the 3x3 weight gradient waits for the 1x1's launch below and shares it.
    float* pA = partA + (size_t)(l & 1) * b->partA_floats;
    const float* in3 = fused ? bl : S3;
    const float2* f3 = fused ? (const float2*)(ws + b->off_fold2[l]) : nullptr;
    if (conc && !oneh) {  // (fused: BN2+ReLU of b_l is applied while the kernel stages its tile)
      DNB_TRY(launch_conv_wgrad(in3, (int64_t)B * hw, gl, ys, gp.W3, n, B, k, d.h, d.w, 9, pA, f3, sA, nullptr, nullptr,
                                nullptr, &pendA, &nextA));
      pendA = nextA;
    }

    // ---- chain B, first half: storage 1 and 2.  Storage 1 was last read by layer l+1's BN1
    // backward on the main chain; storage 2 by the previous wgrad on this stream.
    if (l < m) DNB_TRY(wait(sB, ev(l + 1, EV_MAIN)));
    if (recompute)  // re-populate storage 1 and 2 for this layer
      DNB_TRY(launch_bn_relu(y, ys, S2, (int64_t)c * hw, S1, (int64_t)c * hw, n, c, hw, p.g1, p.b1,
                             StatsSrc{mean_y, istd_y, nullptr, 0, 0, 0, d.eps}, sB));
    DNB_TRY(record(ev(l, EV_S12), sB));

    // ---- main chain.  dS3 doubles as db_{l+1}, which chain B's wgrad of layer l+1 still reads.
    if (l < m) DNB_TRY(wait(st, ev(l + 1, EV_WG1)));
    DNB_TRY(launch_conv_igemm(gl, ys, WeightView{p.W3, 9, (int64_t)B * 9, 1}, pk3t, dS3, (int64_t)B * hw,
                              n, k, B, d.h, d.w, 9, nullptr, st));
    DNB_TRY(launch_bn_relu_bwd(bl, (int64_t)B * hw, dS3, (int64_t)B * hw, dS3, (int64_t)B * hw, false,
                               n, B, hw, p.g2, p.b2, mean_b, istd_b, gp.g2, gp.b2, part, st));
    DNB_TRY(record(ev(l, EV_DB), st));

    // ---- chain B, second half: the 1x1 weight gradient from storage 2 and db_l
    DNB_TRY(wait(sB, ev(l, EV_DB)));
    float* pB = partB + (size_t)(l & 1) * b->partB_floats;
    const float* in1 = fused ? y : S2;
    const int64_t in1s = fused ? ys : (int64_t)c * hw;
    const float2* f1 = fused ? (const float2*)(ws + b->off_fold1[l]) : nullptr;
    if (conc && !oneh) {  // (fused: BN1+ReLU of the concatenated features is applied in the operand load)
      DNB_TRY(launch_conv_wgrad(in1, in1s, dS3, (int64_t)B * hw, gp.W1, n, c, B, d.h, d.w, 1, pB, f1, sB, nullptr,
                                nullptr, nullptr, &pendB, &nextB));
      pendB = nextB;
    }
    if (!oneh) DNB_TRY(record(ev(l, EV_WG1), sB));

    // ---- main chain, continued
    DNB_TRY(launch_conv_igemm(dS3, (int64_t)B * hw, WeightView{p.W1, 1, c, 0}, pk1t, dS2, (int64_t)c * hw,
                              n, B, c, d.h, d.w, 1, nullptr, st));
    if (oneh) {  // issued after the main chain's launch: the main chain keeps its hardware queue in a captured graph
      DNB_TRY(launch_conv_wgrad_pair(in1, in1s, dS3, (int64_t)B * hw, gp.W1, c, pB, f1, in3, (int64_t)B * hw, gl, ys,
                                     gp.W3, k, pA, f3, n, B, d.h, d.w, sA, &pendB, &pendA, nullptr, nullptr));
      DNB_TRY(record(ev(l, EV_WG1), sA));
    }
    DNB_TRY(wait(st, ev(l, EV_S12)));
    // BN1+ReLU backward, then concat backward: add the slice gradients into the slab
    // (the fused schedule reads the concatenated features in place from y)
    const float* x1 = fused ? y : S1;
    const int64_t x1s = fused ? ys : (int64_t)c * hw;
    int passes = 3;
    if (!conc) {
      // one stream: the layer's two weight gradients (leaves of the dependence graph: db_l in dS3
      // and g_l stay untouched until the next layer), the previous layer's partial sums and the
      // reduction pass of this BN backward share one launch
      BnBwdPartialArgs bn;
      const bool has_bn = bn_bwd_partial_plan(x1, x1s, dS2, (int64_t)c * hw, n, c, hw, p.g1, p.b1, mean_y, istd_y, part, &bn);
      bool bn_done = false;
      DNB_TRY(launch_conv_wgrad_pair(in1, in1s, dS3, (int64_t)B * hw, gp.W1, c, pB, f1, in3, (int64_t)B * hw, gl, ys,
                                     gp.W3, k, pA, f3, n, B, d.h, d.w, st, &pendB, &pendA, has_bn ? &bn : nullptr,
                                     &bn_done));
      if (bn_done) passes = 2;
    }
    DNB_TRY(launch_bn_relu_bwd(x1, x1s, dS2, (int64_t)c * hw, G, ys, true, n, c, hw, p.g1, p.b1, mean_y, istd_y, gp.g1,
                               gp.b1, part, st, passes));
    DNB_TRY(record(ev(l, EV_MAIN), st));
  }
  // the first layer's weight-gradient partials have no later launch to ride on
  DNB_TRY(launch_pending_sum(&pendA, sA));
  DNB_TRY(launch_pending_sum(&pendB, sB));
  if (conc) {  // join: the caller's stream is done only when both helper chains are
    DNB_TRY(hipEventRecord(b->ev_endA, sA));
    DNB_TRY(hipEventRecord(b->ev_endB, sB));
    DNB_TRY(hipStreamWaitEvent(st, b->ev_endA, 0));
    DNB_TRY(hipStreamWaitEvent(st, b->ev_endB, 0));
  }
  DNB_TRY(launch_copy_slab(G, ys, (float*)dx0v, (int64_t)d.c0 * hw, n, (int64_t)d.c0 * hw, st));
  return DNB_OK;
}

// ------------------------------------------------------------------ single operations

int dnb_op_copy_slab(const void* src, int64_t src_stride, void* dst, int64_t dst_stride, int64_t n,
                     int64_t len, void* stream) {
  if (!src || !dst) return DNB_E_NULL;
  if (n < 0 || len < 0 || n > 65535) return DNB_E_RANGE;
  DNB_TRY(launch_copy_slab((const float*)src, src_stride, (float*)dst, dst_stride, (int)n, len,
                           (hipStream_t)stream));
  return DNB_OK;
}

size_t dnb_op_bn_scratch_bytes(int64_t n, int64_t c, int64_t hw) {
  const size_t a = bn_stats_partial_floats((int)n, (int)c, (int)hw);
  const size_t b = bn_bwd_partial_floats((int)n, (int)c, (int)hw);
  return (a > b ? a : b) * sizeof(float);
}

int dnb_op_bn_stats(const void* x, int64_t stride, int64_t n, int64_t c, int64_t hw, float eps,
                    void* mean, void* istd, void* scratch, void* stream) {
  if (!x || !mean || !istd || !scratch) return DNB_E_NULL;
  if (n < 1 || c < 1 || hw < 1 || c > 65535) return DNB_E_RANGE;
  DNB_TRY(launch_bn_stats((const float*)x, stride, (int)n, (int)c, (int)hw, eps, (float*)mean,
                          (float*)istd, (float*)scratch, (hipStream_t)stream));
  return DNB_OK;
}

int dnb_op_bn_relu(const void* x, int64_t x_stride, void* out, int64_t out_stride, int64_t n,
                   int64_t c, int64_t hw, const void* gamma, const void* beta, const void* mean,
                   const void* istd, void* stream) {
  if (!x || !out || !gamma || !beta || !mean || !istd) return DNB_E_NULL;
  if (n < 1 || c < 1 || hw < 1) return DNB_E_RANGE;
  DNB_TRY(launch_bn_relu((const float*)x, x_stride, (float*)out, out_stride, nullptr, 0, (int)n, (int)c,
                         (int)hw, (const float*)gamma, (const float*)beta,
                         StatsSrc{(float*)mean, (float*)istd, nullptr, 0, 0, 0, 0.f}, (hipStream_t)stream));
  return DNB_OK;
}

int dnb_op_bn_relu_backward(const void* x, int64_t x_stride, const void* dact, int64_t dact_stride,
                            void* du, int64_t du_stride, int accumulate, int64_t n, int64_t c,
                            int64_t hw, const void* gamma, const void* beta, const void* mean,
                            const void* istd, void* dgamma, void* dbeta, void* scratch, void* stream) {
  if (!x || !dact || !du || !gamma || !beta || !mean || !istd || !dgamma || !dbeta || !scratch)
    return DNB_E_NULL;
  if (n < 1 || c < 1 || hw < 1 || c > 65535) return DNB_E_RANGE;
  DNB_TRY(launch_bn_relu_bwd((const float*)x, x_stride, (const float*)dact, dact_stride, (float*)du,
                             du_stride, accumulate != 0, (int)n, (int)c, (int)hw, (const float*)gamma,
                             (const float*)beta, (const float*)mean, (const float*)istd,
                             (float*)dgamma, (float*)dbeta, (float*)scratch, (hipStream_t)stream));
  return DNB_OK;
}

int dnb_op_bn_relu_backward_apply(const void* x, int64_t x_stride, const void* dact, int64_t dact_stride,
                                  void* du, int64_t du_stride, int accumulate, int64_t n, int64_t c,
                                  int64_t hw, const void* gamma, const void* beta, const void* mean,
                                  const void* istd, void* dgamma, void* dbeta, const void* scratch,
                                  void* ev_start, void* ev_stop, void* stream) {
  if (!x || !dact || !du || !gamma || !beta || !mean || !istd || !dgamma || !dbeta || !scratch)
    return DNB_E_NULL;
  if (n < 1 || c < 1 || hw < 1 || c > 65535) return DNB_E_RANGE;
  DNB_TRY(launch_bn_relu_bwd((const float*)x, x_stride, (const float*)dact, dact_stride, (float*)du,
                             du_stride, accumulate != 0, (int)n, (int)c, (int)hw, (const float*)gamma,
                             (const float*)beta, (const float*)mean, (const float*)istd,
                             (float*)dgamma, (float*)dbeta, (float*)const_cast<void*>(scratch),
                             (hipStream_t)stream, 2, (hipEvent_t)ev_start, (hipEvent_t)ev_stop));
  return DNB_OK;
}

static int conv_args_ok(int64_t n, int64_t cin, int64_t cout, int64_t h, int64_t w, int ks) {
  if (ks != 1 && ks != 3) return DNB_E_UNSUPPORTED;
  if (n < 1 || cin < 1 || cout < 1 || h < 1 || w < 1 || n > 65535) return DNB_E_RANGE;
  if (cin * h * w >= ((int64_t)1 << 31) || cout * h * w >= ((int64_t)1 << 31)) return DNB_E_RANGE;
  return DNB_OK;
}

size_t dnb_op_conv_scratch_bytes(int64_t cin, int64_t cout, int ks) {
  if ((ks != 1 && ks != 3) || cin < 1 || cout < 1 || cin > (1 << 20) || cout > (1 << 20)) return 0;
  return packed_weight_floats((int)cout, (int)cin, ks * ks) * sizeof(float);
}

int dnb_op_conv_forward(const void* x, int64_t x_stride, const void* wgt, void* out,
                        int64_t out_stride, int64_t n, int64_t cin, int64_t cout, int64_t h,
                        int64_t w, int ks, void* scratch, void* stream) {
  if (!x || !wgt || !out || !scratch) return DNB_E_NULL;
  const int rc = conv_args_ok(n, cin, cout, h, w, ks);
  if (rc) return rc;
  const int taps = ks * ks;
  const WeightView wv{(const float*)wgt, cin * taps, taps, 0};
  DNB_TRY(launch_pack_weights(wv, (int)cout, (int)cin, taps, (float*)scratch, (hipStream_t)stream));
  DNB_TRY(launch_conv_igemm((const float*)x, x_stride, wv, (const float*)scratch, (float*)out, out_stride,
                            (int)n, (int)cin, (int)cout, (int)h, (int)w, taps, nullptr, (hipStream_t)stream));
  return DNB_OK;
}

size_t dnb_op_conv_stats_bytes(int64_t n, int64_t cout, int64_t h, int64_t w) {
  if (n < 1 || cout < 1 || h < 1 || w < 1 || n > 65535 || cout > 65535 || h > 4096 || w > 4096) return 0;
  return conv_stats_partial_floats((int)n, (int)cout, (int)h, (int)w) * sizeof(float);
}

int dnb_op_conv_bnrelu_forward(const void* x, int64_t x_stride, const void* wgt, const void* fold, void* out,
                               int64_t out_stride, void* stats, int* tiles, int64_t n, int64_t cin, int64_t cout,
                               int64_t h, int64_t w, int ks, void* scratch, int prepacked, void* ev_start,
                               void* ev_stop, void* stream) {
  if (!x || !wgt || !fold || !out || !stats || !tiles || !scratch) return DNB_E_NULL;
  const int rc = conv_args_ok(n, cin, cout, h, w, ks);
  if (rc) return rc;
  const int taps = ks * ks;
  const WeightView wv{(const float*)wgt, cin * taps, taps, 0};
  if (!conv_fast_ok((const float*)x, x_stride, (const float*)out, out_stride, (int)h, (int)w, taps))
    return DNB_E_UNSUPPORTED;
  if (!prepacked) DNB_TRY(launch_pack_weights(wv, (int)cout, (int)cin, taps, (float*)scratch, (hipStream_t)stream));
  ConvExtras ex{(const float2*)fold, (float*)stats, 0, false, (hipEvent_t)ev_start, (hipEvent_t)ev_stop};
  DNB_TRY(launch_conv_igemm((const float*)x, x_stride, wv, (const float*)scratch, (float*)out, out_stride,
                            (int)n, (int)cin, (int)cout, (int)h, (int)w, taps, &ex, (hipStream_t)stream));
  if (!ex.used_fast) return DNB_E_UNSUPPORTED;
  *tiles = ex.stats_T;
  return DNB_OK;
}

int dnb_op_conv_dgrad(const void* dout, int64_t dout_stride, const void* wgt, void* din,
                      int64_t din_stride, int64_t n, int64_t cin, int64_t cout, int64_t h, int64_t w,
                      int ks, void* scratch, void* stream) {
  if (!dout || !wgt || !din || !scratch) return DNB_E_NULL;
  const int rc = conv_args_ok(n, cin, cout, h, w, ks);
  if (rc) return rc;
  const int taps = ks * ks;
  // the data gradient is a convolution of dout with the weights transposed and flipped
  const WeightView wv{(const float*)wgt, taps, cin * taps, taps == 9 ? 1 : 0};
  DNB_TRY(launch_pack_weights(wv, (int)cin, (int)cout, taps, (float*)scratch, (hipStream_t)stream));
  DNB_TRY(launch_conv_igemm((const float*)dout, dout_stride, wv, (const float*)scratch, (float*)din,
                            din_stride, (int)n, (int)cout, (int)cin, (int)h, (int)w, taps, nullptr,
                            (hipStream_t)stream));
  return DNB_OK;
}

size_t dnb_op_conv_wgrad_scratch_bytes(int64_t n, int64_t cin, int64_t cout, int64_t h, int64_t w,
                                       int ks) {
  if (conv_args_ok(n, cin, cout, h, w, ks)) return 0;
  return conv_wgrad_partial_floats((int)n, (int)cin, (int)cout, (int)h, (int)w, ks * ks) * sizeof(float);
}

int dnb_op_conv_wgrad(const void* x, int64_t x_stride, const void* dout, int64_t dout_stride,
                      void* dwgt, int64_t n, int64_t cin, int64_t cout, int64_t h, int64_t w, int ks,
                      void* scratch, void* stream) {
  if (!x || !dout || !dwgt || !scratch) return DNB_E_NULL;
  const int rc = conv_args_ok(n, cin, cout, h, w, ks);
  if (rc) return rc;
  DNB_TRY(launch_conv_wgrad((const float*)x, x_stride, (const float*)dout, dout_stride, (float*)dwgt,
                            (int)n, (int)cin, (int)cout, (int)h, (int)w, ks * ks, (float*)scratch, nullptr,
                            (hipStream_t)stream));
  return DNB_OK;
}

int dnb_op_conv_bnrelu_wgrad(const void* x, int64_t x_stride, const void* fold, const void* dout,
                             int64_t dout_stride, void* dwgt, int64_t n, int64_t cin, int64_t cout, int64_t h,
                             int64_t w, int ks, void* scratch, void* ev_start, void* ev_stop, void* stream) {
  if (!x || !fold || !dout || !dwgt || !scratch) return DNB_E_NULL;
  const int rc = conv_args_ok(n, cin, cout, h, w, ks);
  if (rc) return rc;
  bool fast = false;
  const hipError_t e = launch_conv_wgrad((const float*)x, x_stride, (const float*)dout, dout_stride, (float*)dwgt,
                                         (int)n, (int)cin, (int)cout, (int)h, (int)w, ks * ks, (float*)scratch,
                                         (const float2*)fold, (hipStream_t)stream, (hipEvent_t)ev_start,
                                         (hipEvent_t)ev_stop, &fast);
  if (!fast) return DNB_E_UNSUPPORTED;  // only the 16-byte-vector kernels have the prologue
  return e == hipSuccess ? DNB_OK : DNB_E_LAUNCH;
}

size_t dnb_op_layer_wgrads_scratch_bytes(int64_t n, int64_t cin, int64_t B, int64_t k, int64_t h, int64_t w) {
  if (n < 1 || cin < 1 || B < 1 || k < 1 || h < 1 || w < 1) return 0;
  const size_t f = conv_wgrad_partial_floats((int)n, (int)cin, (int)B, (int)h, (int)w, 1) +
                   conv_wgrad_partial_floats((int)n, (int)B, (int)k, (int)h, (int)w, 9) +
                   bn_bwd_partial_floats((int)n, (int)cin, (int)(h * w)) + 16;
  return f * sizeof(float);
}

size_t dnb_op_layer_wgrads_bn_partials_offset(int64_t n, int64_t cin, int64_t B, int64_t k, int64_t h, int64_t w) {
  if (n < 1 || cin < 1 || B < 1 || k < 1 || h < 1 || w < 1) return 0;
  const size_t f = ((conv_wgrad_partial_floats((int)n, (int)cin, (int)B, (int)h, (int)w, 1) + 3) & ~(size_t)3) +
                   ((conv_wgrad_partial_floats((int)n, (int)B, (int)k, (int)h, (int)w, 9) + 3) & ~(size_t)3);
  return f * sizeof(float);
}

int dnb_op_layer_wgrads(const void* x1, int64_t x1_stride, const void* fold1, const void* db, void* dw1, int64_t cin,
                        const void* bact, const void* fold2, const void* g, int64_t g_stride, void* dw3, int64_t n,
                        int64_t B, int64_t k, int64_t h, int64_t w, const void* bn_dact, const void* bn_gamma,
                        const void* bn_beta, const void* bn_mean, const void* bn_istd, void* scratch, void* ev_start,
                        void* ev_stop, void* stream) {
  if (!x1 || !fold1 || !db || !dw1 || !bact || !fold2 || !g || !dw3 || !scratch) return DNB_E_NULL;
  if (bn_dact && (!bn_gamma || !bn_beta || !bn_mean || !bn_istd)) return DNB_E_NULL;
  int rc = conv_args_ok(n, cin, B, h, w, 1);
  if (rc) return rc;
  rc = conv_args_ok(n, B, k, h, w, 3);
  if (rc) return rc;
  const int hw = (int)(h * w);
  float* part1 = (float*)scratch;
  float* part3 = part1 + ((conv_wgrad_partial_floats((int)n, (int)cin, (int)B, (int)h, (int)w, 1) + 3) & ~(size_t)3);
  float* partbn = part3 + ((conv_wgrad_partial_floats((int)n, (int)B, (int)k, (int)h, (int)w, 9) + 3) & ~(size_t)3);
  BnBwdPartialArgs bn;
  bool has_bn = false;
  if (bn_dact) {
    has_bn = bn_bwd_partial_plan((const float*)x1, x1_stride, (const float*)bn_dact, cin * hw, (int)n, (int)cin, hw,
                                 (const float*)bn_gamma, (const float*)bn_beta, (const float*)bn_mean,
                                 (const float*)bn_istd, partbn, &bn);
    if (!has_bn) return DNB_E_UNSUPPORTED;
  }
  PendingSum p1, p3;
  bool paired = false, bn_done = false;
  hipStream_t st = (hipStream_t)stream;
  hipError_t e = launch_conv_wgrad_pair((const float*)x1, x1_stride, (const float*)db, B * hw, (float*)dw1, (int)cin,
                                        part1, (const float2*)fold1, (const float*)bact, B * hw, (const float*)g,
                                        g_stride, (float*)dw3, (int)k, part3, (const float2*)fold2, (int)n, (int)B,
                                        (int)h, (int)w, st, &p1, &p3, has_bn ? &bn : nullptr, &bn_done,
                                        (hipEvent_t)ev_start, (hipEvent_t)ev_stop, &paired);
  if (e == hipSuccess) e = launch_pending_sum(&p1, st);
  if (e == hipSuccess) e = launch_pending_sum(&p3, st);
  if (e != hipSuccess) return DNB_E_LAUNCH;
  return paired ? DNB_OK : DNB_E_UNSUPPORTED;  // (the two gradients are complete either way)
}

// ---- single operations of the bf16 / NHWC path

size_t dnb_op_nhwc_scratch_bytes(int64_t n, int64_t cin, int64_t cout, int64_t h, int64_t w, int ks) {
  if ((ks != 1 && ks != 3) || n < 1 || cin < 1 || cout < 1 || h < 1 || w < 1) return 0;
  const size_t a = nhwc::packed_weight_elems((int)cout, (int)cin, ks * ks) * 2;
  const size_t b = nhwc::packed_weight_elems((int)cin, (int)cout, ks * ks) * 2;
  const size_t c = nhwc::wgrad_partial_floats((int)n, (int)cin, (int)cout, (int)h, (int)w, ks * ks) * 4;
  const size_t d = nhwc::bn_bwd_partial_floats(n * h * w, (int)(cin > cout ? cin : cout)) * 4;
  size_t m = a > b ? a : b;
  if (c > m) m = c;
  if (d > m) m = d;
  return m + 256;
}

static int nhwc_args_ok(int64_t n, int64_t cin, int64_t cout, int64_t h, int64_t w, int ks) {
  if (ks != 1 && ks != 3) return DNB_E_UNSUPPORTED;
  if (n < 1 || cin < 1 || cout < 1 || h < 1 || w < 1 || n > 65535) return DNB_E_RANGE;
  if (cin % 8 || cout % 8) return DNB_E_UNSUPPORTED;
  if ((size_t)(64 + 2 * (w + 1)) * 80 > 64 * 1024) return DNB_E_UNSUPPORTED;
  return DNB_OK;
}

// The NHWC kernels move 16 bytes per lane: tensors start on 16-byte boundaries and a pixel
// stride is a whole number of such vectors that covers the channels used (8 bf16 or 4 fp32 each).
static int nhwc_tensor_ok(const void* p, int64_t ld, int64_t c, bool f32) {
  if (misaligned(p)) return DNB_E_ALIGN;
  if (ld < c || ld % (f32 ? 4 : 8)) return DNB_E_RANGE;
  return DNB_OK;
}
#define DNB_NHWC_CHECK(p, ld, c, f32)                       \
  do {                                                      \
    const int rc_ = nhwc_tensor_ok((p), (ld), (c), (f32));  \
    if (rc_) return rc_;                                    \
  } while (0)

int dnb_op_nhwc_conv_forward(const void* x, int64_t x_ld, const void* wgt, void* out, int64_t out_ld, int64_t n,
                             int64_t cin, int64_t cout, int64_t h, int64_t w, int ks, void* scratch, void* stream) {
  if (!x || !wgt || !out || !scratch) return DNB_E_NULL;
  const int rc = nhwc_args_ok(n, cin, cout, h, w, ks);
  if (rc) return rc;
  DNB_NHWC_CHECK(x, x_ld, cin, false);
  DNB_NHWC_CHECK(out, out_ld, cout, false);
  if (misaligned4(wgt) || misaligned(scratch)) return DNB_E_ALIGN;
  const int taps = ks * ks;
  DNB_TRY(nhwc::pack_weights(WeightView{(const float*)wgt, cin * taps, taps, 0}, (int)cout, (int)cin, taps, scratch,
                             (hipStream_t)stream));
  DNB_TRY(nhwc::conv(x, x_ld, false, scratch, out, out_ld, (int)n, (int)cin, (int)cout, (int)h, (int)w, taps, nullptr,
                     nullptr, nullptr, (hipStream_t)stream));
  return DNB_OK;
}

int dnb_op_nhwc_conv_dgrad(const void* dout, int64_t dout_ld, int dout_is_f32, const void* wgt, void* din,
                           int64_t din_ld, int64_t n, int64_t cin, int64_t cout, int64_t h, int64_t w, int ks,
                           void* scratch, void* stream) {
  if (!dout || !wgt || !din || !scratch) return DNB_E_NULL;
  const int rc = nhwc_args_ok(n, cin, cout, h, w, ks);
  if (rc) return rc;
  DNB_NHWC_CHECK(dout, dout_ld, cout, dout_is_f32 != 0);
  DNB_NHWC_CHECK(din, din_ld, cin, false);
  if (misaligned4(wgt) || misaligned(scratch)) return DNB_E_ALIGN;
  const int taps = ks * ks;
  DNB_TRY(nhwc::pack_weights(WeightView{(const float*)wgt, taps, cin * taps, taps == 9 ? 1 : 0}, (int)cin, (int)cout,
                             taps, scratch, (hipStream_t)stream));
  DNB_TRY(nhwc::conv(dout, dout_ld, dout_is_f32 != 0, scratch, din, din_ld, (int)n, (int)cout, (int)cin, (int)h, (int)w,
                     taps, nullptr, nullptr, nullptr, (hipStream_t)stream));
  return DNB_OK;
}

int dnb_op_nhwc_conv_wgrad(const void* x, int64_t x_ld, const void* dout, int64_t dout_ld, int dout_is_f32, void* dwgt,
                           int64_t n, int64_t cin, int64_t cout, int64_t h, int64_t w, int ks, void* scratch,
                           void* stream) {
  if (!x || !dout || !dwgt || !scratch) return DNB_E_NULL;
  const int rc = nhwc_args_ok(n, cin, cout, h, w, ks);
  if (rc) return rc;
  DNB_NHWC_CHECK(x, x_ld, cin, false);
  DNB_NHWC_CHECK(dout, dout_ld, cout, dout_is_f32 != 0);
  if (misaligned4(dwgt) || misaligned(scratch)) return DNB_E_ALIGN;
  DNB_TRY(nhwc::wgrad(x, x_ld, dout, dout_ld, dout_is_f32 != 0, (float*)scratch, (float*)dwgt, (int)n, (int)cin,
                      (int)cout, (int)h, (int)w, ks * ks, nullptr, (hipStream_t)stream));
  return DNB_OK;
}

int dnb_op_nhwc_bn_relu_backward(const void* x, int64_t x_ld, const void* dact, int64_t dact_ld, void* du_bf16,
                                 int64_t du_ld, void* du_accum_f32, int64_t acc_ld, int64_t pixels, int64_t c,
                                 const void* gamma, const void* beta, const void* mean, const void* istd,
                                 void* dgamma, void* dbeta, void* scratch, void* stream) {
  if (!x || !dact || (!du_bf16 && !du_accum_f32) || !gamma || !beta || !mean || !istd || !dgamma || !dbeta || !scratch)
    return DNB_E_NULL;
  if (pixels < 1 || c < 8 || c % 8) return DNB_E_RANGE;
  DNB_NHWC_CHECK(x, x_ld, c, false);
  DNB_NHWC_CHECK(dact, dact_ld, c, false);
  if (du_accum_f32)
    DNB_NHWC_CHECK(du_accum_f32, acc_ld, c, true);
  else
    DNB_NHWC_CHECK(du_bf16, du_ld, c, false);
  if (misaligned4(gamma) || misaligned4(beta) || misaligned4(mean) || misaligned4(istd) || misaligned4(dgamma) ||
      misaligned4(dbeta) || misaligned(scratch))
    return DNB_E_ALIGN;
  DNB_TRY(nhwc::bn_relu_bwd(x, x_ld, dact, dact_ld, du_bf16, du_ld, (float*)du_accum_f32, acc_ld, pixels, (int)c,
                            (const float*)gamma, (const float*)beta, (const float*)mean, (const float*)istd,
                            (float*)dgamma, (float*)dbeta, (float*)scratch, (hipStream_t)stream));
  return DNB_OK;
}

}  // extern "C"
