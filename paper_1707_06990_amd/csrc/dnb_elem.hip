// Element-wise and per-channel reduction kernels of the dense block (fp32, NCHW):
// concatenation copy, BN batch statistics, BN-apply+ReLU (also used for the
// backward pass's recomputation), and BN+ReLU backward.  All are HBM-bound:
// 16-byte accesses along the contiguous pixel axis, one pass over the data per
// kernel, wave-level butterfly reductions and LDS only to combine the waves of a
// workgroup.
#include <hip/hip_ext.h>

#include <mutex>

#include "../../include/dnb.h"
#include "dnb_internal.h"
#include "dnb_stats.h"

namespace dnb {

namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ float wave_sum(float v) { return bnb_wave_sum(v); }
__device__ __forceinline__ float block_sum(float v, float* red) { return bnb_block_sum(v, red); }

template <int V>
struct Vec;
template <>
struct Vec<4> {
  using T = float4;
  static __device__ __forceinline__ void ld(const float* p, float (&v)[4]) {
    const float4 t = *reinterpret_cast<const float4*>(p);
    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
  }
  static __device__ __forceinline__ void st(float* p, const float (&v)[4]) {
    *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  }
};
template <>
struct Vec<1> {
  static __device__ __forceinline__ void ld(const float* p, float (&v)[1]) { v[0] = *p; }
  static __device__ __forceinline__ void st(float* p, const float (&v)[1]) { *p = v[0]; }
};

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline unsigned grid_for(int64_t items, int per_block, unsigned cap = 0x7fffffffu) {
  int64_t g = (items + per_block - 1) / per_block;
  if (g < 1) g = 1;
  if (g > (int64_t)cap) g = cap;
  return (unsigned)g;
}

// ----------------------------------------------------------------------------- copy

template <int V>
__global__ __launch_bounds__(kThreads) void k_copy_slab(const float* __restrict__ src,
                                                        int64_t src_stride, float* __restrict__ dst,
                                                        int64_t dst_stride, int64_t lenv) {
  const int img = blockIdx.y;
  const float* s = src + (int64_t)img * src_stride;
  float* d = dst + (int64_t)img * dst_stride;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < lenv;
       i += (int64_t)gridDim.x * kThreads) {
    float v[V];
    Vec<V>::ld(s + i * V, v);
    Vec<V>::st(d + i * V, v);
  }
}

// ----------------------------------------------------------------------------- row iteration

// A workgroup of the BN kernels below owns ONE channel and a range of images: its elements are
// (RowIter, which walks rows of hw contiguous floats, one per image, is in dnb_stats.h)

// ----------------------------------------------------------------------------- BN statistics

// grid (c, splits): workgroup (ch, s) reduces images [s*ipb, min(n,(s+1)*ipb)) of channel ch
// to (count, mean, M2) with a two-pass sum (second pass hits L2), so no cancellation.
template <int V>
__global__ __launch_bounds__(kThreads) void k_bn_stats_partial(const float* __restrict__ x,
                                                               int64_t stride, int n, int hw,
                                                               int ipb, float* __restrict__ part) {
  __shared__ float red[kThreads / 64];
  const int ch = blockIdx.x, s = blockIdx.y, splits = gridDim.y;
  const int n0 = s * ipb, n1 = min(n, n0 + ipb), ni = n1 - n0;
  const int hwv = hw / V;
  const float* xc = x + (int64_t)n0 * stride + (int64_t)ch * hw;
  float acc = 0.f;
  for (RowIter it(hwv, threadIdx.x, blockDim.x); it.img < ni; it.next()) {
    float t[V];
    Vec<V>::ld(xc + (int64_t)it.img * stride + (int64_t)it.q * V, t);
#pragma unroll
    for (int e = 0; e < V; ++e) acc += t[e];
  }
  const float cnt = (float)ni * (float)hw;
  const float mu = block_sum(acc, red) / cnt;
  float m2 = 0.f;
  for (RowIter it(hwv, threadIdx.x, blockDim.x); it.img < ni; it.next()) {
    float t[V];
    Vec<V>::ld(xc + (int64_t)it.img * stride + (int64_t)it.q * V, t);
#pragma unroll
    for (int e = 0; e < V; ++e) {
      const float d = t[e] - mu;
      m2 = __fmaf_rn(d, d, m2);
    }
  }
  m2 = block_sum(m2, red);
  if (threadIdx.x == 0) {
    float* p = part + ((int64_t)ch * splits + s) * 3;
    p[0] = cnt; p[1] = mu; p[2] = m2;
  }
}

// Finalised statistics of channel ch for the calling workgroup.  Channels in
// [fresh_lo, fresh_hi) still only have partials ([splits][3] per channel, from the statistics
// kernel or a convolution epilogue): the workgroup merges them; the one with blockIdx.y == 0
// also stores mean / inverse std so later kernels read them.  Returns (mean, istd) to every thread.
__device__ __forceinline__ void channel_stats(int ch, float* mean, float* istd, const float* part,
                                              int splits, int fresh_lo, int fresh_hi, float eps,
                                              float* sh, float& mu, float& is) {
  if (ch >= fresh_lo && ch < fresh_hi) {  // workgroup-uniform branch
    const Stat3 r = stat_merge_block(part + (int64_t)(ch - fresh_lo) * splits * 3, splits, sh);
    mu = r.m;
    is = bn_istd(r.m2, r.c, eps);
    if (blockIdx.y == 0 && threadIdx.x == 0) { mean[ch] = mu; istd[ch] = is; }
  } else {
    mu = mean[ch];
    is = istd[ch];
  }
}

// One wave per channel merges the partials; used by the stand-alone statistics entry point.
__global__ __launch_bounds__(64) void k_bn_stats_finalize(const float* __restrict__ part, int c, int splits,
                                                          float eps, float* __restrict__ mean,
                                                          float* __restrict__ istd) {
  __shared__ float sh[3];
  const int ch = blockIdx.x;
  const Stat3 r = stat_merge_block(part + (int64_t)ch * splits * 3, splits, sh);
  if (threadIdx.x == 0) {
    mean[ch] = r.m;
    istd[ch] = bn_istd(r.m2, r.c, eps);
  }
}

// ----------------------------------------------------------------------------- BN apply + ReLU

// grid (c, splits).  out = max(0, fma(x, scale, shift)); COPY also writes the raw x (the
// concatenation into storage 1 and its BN+ReLU into storage 2 in one pass over the features).
template <int V, bool COPY>
__global__ __launch_bounds__(kThreads) void k_bn_relu(
    const float* __restrict__ x, int64_t x_stride, float* __restrict__ out, int64_t out_stride,
    float* __restrict__ copy_out, int64_t copy_stride, int n, int hw, int ipb,
    const float* __restrict__ gamma, const float* __restrict__ beta, float* mean, float* istd,
    const float* __restrict__ part, int splits, int fresh_lo, int fresh_hi, float eps) {
  __shared__ float sh[3 * kThreads / 64];
  const int ch = blockIdx.x, n0 = blockIdx.y * ipb, ni = min(n, n0 + ipb) - n0;
  float mu, is, scale, shift;
  channel_stats(ch, mean, istd, part, splits, fresh_lo, fresh_hi, eps, sh, mu, is);
  bn_fold(gamma[ch], beta[ch], mu, is, scale, shift);
  const int hwv = hw / V;
  const int64_t inner = (int64_t)ch * hw;
  const float* xp = x + (int64_t)n0 * x_stride + inner;
  float* op = out + (int64_t)n0 * out_stride + inner;
  float* cp = COPY ? copy_out + (int64_t)n0 * copy_stride + inner : nullptr;
  for (RowIter it(hwv, threadIdx.x, blockDim.x); it.img < ni; it.next()) {
    float t[V], r[V];
    Vec<V>::ld(xp + (int64_t)it.img * x_stride + (int64_t)it.q * V, t);
#pragma unroll
    for (int e = 0; e < V; ++e) r[e] = fmaxf(__fmaf_rn(t[e], scale, shift), 0.f);
    Vec<V>::st(op + (int64_t)it.img * out_stride + (int64_t)it.q * V, r);
    if (COPY) Vec<V>::st(cp + (int64_t)it.img * copy_stride + (int64_t)it.q * V, t);
  }
}

// ----------------------------------------------------------------------------- BN + ReLU backward

// grid (c, splits): partial sums of dz and dz*xhat over a range of images.
template <int V>
__global__ __launch_bounds__(kThreads) void k_bn_bwd_partial(
    const float* __restrict__ x, int64_t x_stride, const float* __restrict__ dact,
    int64_t dact_stride, int n, int hw, int ipb, const float* __restrict__ gamma,
    const float* __restrict__ beta, const float* __restrict__ mean, const float* __restrict__ istd,
    float* __restrict__ part) {
  if (V == 4) {  // the vector form lives in dnb_stats.h: the weight-gradient launch can carry it too
    const BnBwdPartialArgs A{x, x_stride, dact, dact_stride, n, hw, ipb, gamma, beta, mean, istd, part,
                             (int)gridDim.x, (int)gridDim.y};
    bn_bwd_partial_body4(A, blockIdx.x, blockIdx.y);
    return;
  }
  __shared__ float red[kThreads / 64];
  const int ch = blockIdx.x, s = blockIdx.y, splits = gridDim.y;
  const int n0 = s * ipb, ni = min(n, n0 + ipb) - n0;
  float scale, shift;
  const float mu = mean[ch], is = istd[ch];
  bn_fold(gamma[ch], beta[ch], mu, is, scale, shift);
  const int64_t inner = (int64_t)ch * hw;
  const float* xp = x + (int64_t)n0 * x_stride + inner;
  const float* gp = dact + (int64_t)n0 * dact_stride + inner;
  float sb = 0.f, sg = 0.f;
  for (RowIter it(hw, threadIdx.x, blockDim.x); it.img < ni; it.next()) {
    const float t = xp[(int64_t)it.img * x_stride + it.q], g = gp[(int64_t)it.img * dact_stride + it.q];
    const float dz = __fmaf_rn(t, scale, shift) > 0.f ? g : 0.f;
    sb += dz;
    sg = __fmaf_rn(dz, (t - mu) * is, sg);
  }
  sb = block_sum(sb, red);
  sg = block_sum(sg, red);
  if (threadIdx.x == 0) {
    float* p = part + ((int64_t)ch * splits + s) * 2;
    p[0] = sb; p[1] = sg;
  }
}

// grid (c, splits).  Adds up the channel's partial sums (wave butterfly, every workgroup gets
// the same bits), then du = scale*(dz - dbeta/P - xhat*dgamma/P).  Split 0 stores dgamma/dbeta.
template <int V, bool ACC>
__global__ __launch_bounds__(kThreads) void k_bn_bwd_apply(
    const float* __restrict__ x, int64_t x_stride, const float* dact /* may alias du */,
    int64_t dact_stride, float* du, int64_t du_stride, int n, int hw, int ipb, float inv_p,
    const float* __restrict__ gamma, const float* __restrict__ beta,
    const float* __restrict__ mean, const float* __restrict__ istd,
    const float* __restrict__ part, int psplits, float* __restrict__ dgamma, float* __restrict__ dbeta) {
  __shared__ float sh[2];
  const int ch = blockIdx.x, n0 = blockIdx.y * ipb, ni = min(n, n0 + ipb) - n0;
  // Everything that does not depend on the sums is requested before the barrier below: the
  // channel's constants and the thread's first four positions (behind the barrier each would
  // cost one more memory round trip, which is what a small slab's launch consists of).
  const float mu = mean[ch], is = istd[ch], ga = gamma[ch], be = beta[ch];
  const int hwv = hw / V;
  const int64_t inner = (int64_t)ch * hw;
  const float* xp = x + (int64_t)n0 * x_stride + inner;
  const float* gp = dact + (int64_t)n0 * dact_stride + inner;
  float* dp = du + (int64_t)n0 * du_stride + inner;
  RowIter it(hwv, threadIdx.x, blockDim.x);
  float t[4][V], g[4][V], r[4][V];
  float* d[4];
  bool ok[4];
  // four positions per pass, all loads issued before the first is consumed (as in the partial
  // kernel; a position past the range repeats the last image's and is not stored); dact may
  // alias du: a thread reads its four positions before it writes them
  auto request = [&]() {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      ok[u] = it.img < ni;
      const int im = ok[u] ? it.img : ni - 1;
      const int64_t qo = (int64_t)it.q * V;
      Vec<V>::ld(xp + (int64_t)im * x_stride + qo, t[u]);
      Vec<V>::ld(gp + (int64_t)im * dact_stride + qo, g[u]);
      d[u] = dp + (int64_t)im * du_stride + qo;
      if (ACC) Vec<V>::ld(d[u], r[u]);
      it.next();
    }
  };
  request();
  if (threadIdx.x < 64) {
    const int lane = threadIdx.x;
    float sb = 0.f, sg = 0.f;
    if (lane < psplits) {
      const float* p = part + ((int64_t)ch * psplits + lane) * 2;
      sb = p[0]; sg = p[1];
    }
    sb = wave_sum(sb);
    sg = wave_sum(sg);
    if (lane == 0) {
      sh[0] = sb; sh[1] = sg;
      if (blockIdx.y == 0) { dbeta[ch] = sb; dgamma[ch] = sg; }
    }
  }
  __syncthreads();
  const float mb = sh[0] * inv_p, mg = sh[1] * inv_p;
  float scale, shift;
  bn_fold(ga, be, mu, is, scale, shift);
  for (;;) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (ok[u]) {
#pragma unroll
        for (int e = 0; e < V; ++e) {
          const float dz = __fmaf_rn(t[u][e], scale, shift) > 0.f ? g[u][e] : 0.f;
          const float xh = (t[u][e] - mu) * is;
          const float v = scale * (dz - mb - xh * mg);
          r[u][e] = ACC ? r[u][e] + v : v;
        }
        Vec<V>::st(d[u], r[u]);
      }
    }
    if (!(it.img < ni)) break;
    request();
  }
}

// Image splits for a (n, c, hw) slab: enough workgroups to cover the chip a few times over,
// at least ~4 KB per workgroup, at most 64 (one wave merges a channel's partials).
int splits_for(int n, int c, int hw) {
  int s = (1024 + c - 1) / c;
  const int min_ipb = (1024 + hw - 1) / hw;
  const int cap = (n + min_ipb - 1) / min_ipb;
  if (s > cap) s = cap;
  if (s > n) s = n;
  if (s > 64) s = 64;
  if (s < 1) s = 1;
  return s;
}

struct Split { int ipb, gs; };
Split split_plan(int n, int c, int hw) {
  const int s = splits_for(n, c, hw);
  Split p;
  p.ipb = (n + s - 1) / s;
  p.gs = (n + p.ipb - 1) / p.ipb;  // every split non-empty
  return p;
}

}  // namespace

// ============================================================================ launchers

hipError_t launch_copy_slab(const float* src, int64_t src_stride, float* dst, int64_t dst_stride,
                            int n, int64_t len, hipStream_t st) {
  if (n <= 0 || len <= 0) return hipSuccess;
  const bool v4 = (len % 4 == 0) && (src_stride % 4 == 0) && (dst_stride % 4 == 0) &&
                  aligned16(src) && aligned16(dst);
  const int64_t lenv = v4 ? len / 4 : len;
  dim3 grid(grid_for(lenv, kThreads * 4, 4096), (unsigned)n);
  if (v4)
    hipLaunchKernelGGL(k_copy_slab<4>, grid, dim3(kThreads), 0, st, src, src_stride, dst, dst_stride, lenv);
  else
    hipLaunchKernelGGL(k_copy_slab<1>, grid, dim3(kThreads), 0, st, src, src_stride, dst, dst_stride, lenv);
  return hipGetLastError();
}

size_t bn_stats_partial_floats(int n, int c, int hw) { return (size_t)c * splits_for(n, c, hw) * 3; }

hipError_t launch_bn_stats_partial(const float* x, int64_t stride, int n, int c, int hw,
                                   float* partials, int* splits, hipStream_t st) {
  const Split p = split_plan(n, c, hw);
  *splits = p.gs;
  if (c <= 0) return hipSuccess;
  const bool v4 = (hw % 4 == 0) && (stride % 4 == 0) && aligned16(x);
  dim3 grid((unsigned)c, (unsigned)p.gs);
  if (v4)
    hipLaunchKernelGGL(k_bn_stats_partial<4>, grid, dim3(kThreads), 0, st, x, stride, n, hw, p.ipb, partials);
  else
    hipLaunchKernelGGL(k_bn_stats_partial<1>, grid, dim3(kThreads), 0, st, x, stride, n, hw, p.ipb, partials);
  return hipGetLastError();
}

hipError_t launch_bn_stats(const float* x, int64_t stride, int n, int c, int hw, float eps,
                           float* mean, float* istd, float* partials, hipStream_t st) {
  if (c <= 0) return hipSuccess;
  int splits = 0;
  hipError_t e = launch_bn_stats_partial(x, stride, n, c, hw, partials, &splits, st);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_bn_stats_finalize, dim3((unsigned)c), dim3(64), 0, st, partials, c, splits, eps, mean, istd);
  return hipGetLastError();
}

hipError_t launch_bn_relu(const float* x, int64_t x_stride, float* out, int64_t out_stride,
                          float* copy_out, int64_t copy_stride, int n, int c, int hw,
                          const float* gamma, const float* beta, StatsSrc s, hipStream_t st) {
  if (n <= 0 || c <= 0 || hw <= 0) return hipSuccess;
  const bool v4 = (hw % 4 == 0) && (x_stride % 4 == 0) && (out_stride % 4 == 0) && aligned16(x) &&
                  aligned16(out) && (!copy_out || ((copy_stride % 4 == 0) && aligned16(copy_out)));
  const Split p = split_plan(n, c, hw);
  dim3 grid((unsigned)c, (unsigned)p.gs);
#define DNB_LAUNCH_BNRELU(V, C)                                                                     \
  hipLaunchKernelGGL((k_bn_relu<V, C>), grid, dim3(kThreads), 0, st, x, x_stride, out, out_stride, \
                     copy_out, copy_stride, n, hw, p.ipb, gamma, beta, s.mean, s.istd, s.part,    \
                     s.splits, s.fresh_lo, s.fresh_hi, s.eps)
  if (v4) { if (copy_out) DNB_LAUNCH_BNRELU(4, true); else DNB_LAUNCH_BNRELU(4, false); }
  else    { if (copy_out) DNB_LAUNCH_BNRELU(1, true); else DNB_LAUNCH_BNRELU(1, false); }
#undef DNB_LAUNCH_BNRELU
  return hipGetLastError();
}

size_t bn_bwd_partial_floats(int n, int c, int hw) { return (size_t)c * splits_for(n, c, hw) * 2; }

bool bn_bwd_partial_plan(const float* x, int64_t x_stride, const float* dact, int64_t dact_stride, int n, int c,
                         int hw, const float* gamma, const float* beta, const float* mean, const float* istd,
                         float* partials, BnBwdPartialArgs* out) {
  if (n <= 0 || c <= 0 || hw <= 0) return false;
  if (hw % 4 || x_stride % 4 || dact_stride % 4 || !aligned16(x) || !aligned16(dact)) return false;
  const Split p = split_plan(n, c, hw);
  *out = BnBwdPartialArgs{x, x_stride, dact, dact_stride, n, hw, p.ipb, gamma, beta, mean, istd, partials, c, p.gs};
  return true;
}

hipError_t launch_bn_relu_bwd(const float* x, int64_t x_stride, const float* dact,
                              int64_t dact_stride, float* du, int64_t du_stride, bool accumulate,
                              int n, int c, int hw, const float* gamma, const float* beta,
                              const float* mean, const float* istd, float* dgamma, float* dbeta,
                              float* partials, hipStream_t st, int passes, hipEvent_t ev_start,
                              hipEvent_t ev_stop) {
  if (n <= 0 || c <= 0 || hw <= 0) return hipSuccess;
  const Split p = split_plan(n, c, hw);
  const bool v4 = (hw % 4 == 0) && (x_stride % 4 == 0) && (dact_stride % 4 == 0) &&
                  (du_stride % 4 == 0) && aligned16(x) && aligned16(dact) && aligned16(du);
  dim3 grid((unsigned)c, (unsigned)p.gs);
  if (passes & 1) {
    if (v4)
      hipLaunchKernelGGL(k_bn_bwd_partial<4>, grid, dim3(kThreads), 0, st, x, x_stride, dact, dact_stride,
                         n, hw, p.ipb, gamma, beta, mean, istd, partials);
    else
      hipLaunchKernelGGL(k_bn_bwd_partial<1>, grid, dim3(kThreads), 0, st, x, x_stride, dact, dact_stride,
                         n, hw, p.ipb, gamma, beta, mean, istd, partials);
  }
  if (!(passes & 2)) return hipGetLastError();
  const float inv_p = 1.0f / ((float)n * (float)hw);
  // (the Ext launch stamps the two optional events right at the kernel's start and end)
#define DNB_LAUNCH_BNBWD(V, A)                                                                      \
  hipExtLaunchKernelGGL((k_bn_bwd_apply<V, A>), grid, dim3(kThreads), 0, st, ev_start, ev_stop, 0, \
                        x, x_stride, dact, dact_stride, du, du_stride, n, hw, p.ipb, inv_p, gamma, \
                        beta, mean, istd, (const float*)partials, p.gs, dgamma, dbeta)
  if (v4) { if (accumulate) DNB_LAUNCH_BNBWD(4, true); else DNB_LAUNCH_BNBWD(4, false); }
  else    { if (accumulate) DNB_LAUNCH_BNBWD(1, true); else DNB_LAUNCH_BNBWD(1, false); }
#undef DNB_LAUNCH_BNBWD
  return hipGetLastError();
}

}  // namespace dnb

// ---- BN statistics for callers that cannot allocate device memory (code under HIP graph
// capture, serving loops, harnesses that forbid it): same kernels as dnb_op_bn_stats, with the
// split-reduction partials in a file-scope device array instead of a caller's buffer.  Every GPU
// the library runs on holds its own copy of the array (at its own address) until the process ends.
namespace {
constexpr size_t kStaticScratchFloats = (size_t)1 << 16;  // 256 KiB
__device__ __align__(256) float scratch[kStaticScratchFloats];
constexpr int kMaxDevices = 64;
float* g_scratch_ptr[kMaxDevices];  // device address of `scratch` per device; null until looked up
std::mutex g_scratch_mutex;

// The array's name is only a host-side stand-in: its device address is looked up once per device,
// with that device current, and that pointer is what kernels and copies get.
int static_scratch(float** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return DNB_E_LAUNCH;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return DNB_E_LAUNCH;
    g_scratch_ptr[dev] = (float*)p;
  }
  *out = g_scratch_ptr[dev];
  return DNB_OK;
}
}  // namespace

extern "C" int dnb_op_bn_stats_static(const void* x, int64_t stride, int64_t n, int64_t c, int64_t hw, float eps,
                                      void* mean, void* istd, void* stream) {
  if (!x || !mean || !istd) return DNB_E_NULL;
  if (n < 1 || c < 1 || hw < 1 || c > 65535 || n > 65535 || hw > ((int64_t)1 << 30)) return DNB_E_RANGE;
  if (dnb::bn_stats_partial_floats((int)n, (int)c, (int)hw) > kStaticScratchFloats) return DNB_E_RANGE;
  float* part = nullptr;
  const int rc = static_scratch(&part);
  if (rc != DNB_OK) return rc;
  // every (channel, split) slot the finalisation reads is written by the partial kernel of this
  // call, so nothing of an earlier call's contents has to be cleared
  if (dnb::launch_bn_stats((const float*)x, stride, (int)n, (int)c, (int)hw, eps, (float*)mean, (float*)istd, part,
                           (hipStream_t)stream) != hipSuccess)
    return DNB_E_LAUNCH;
  return DNB_OK;
}
