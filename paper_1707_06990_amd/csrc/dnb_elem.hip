// Element-wise and per-channel reduction kernels of the dense block (fp32, NCHW):
// concatenation copy, BN batch statistics, BN-apply+ReLU (also used for the
// backward pass's recomputation), and BN+ReLU backward.  All are HBM-bound:
// 16-byte accesses along the contiguous pixel axis, one pass over the data per
// kernel, wave-level butterfly reductions and LDS only to combine the waves of a
// workgroup.
#include "dnb_internal.h"

namespace dnb {

namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ float wave_sum(float v) {
  // butterfly over the 64 lanes of a wavefront: every lane ends with the same total
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// Sum over the workgroup; the result is returned to every thread.  `red` holds one
// float per wave.  Safe to call repeatedly (barrier before reuse).
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  const int wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[wave] = v;
  __syncthreads();
  float t = 0.f;
  for (int i = 0; i < nw; ++i) t += red[i];
  return t;
}

// The one place BN's affine map is folded into (scale, shift); forward, recomputation
// and backward all call it so the ReLU mask is reproduced bit for bit.
__device__ __forceinline__ void bn_fold(float gamma, float beta, float mean, float istd,
                                        float& scale, float& shift) {
  scale = __fmul_rn(gamma, istd);
  shift = __fmaf_rn(-mean, scale, beta);
}

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

// ----------------------------------------------------------------------------- BN statistics

// grid (c, splits): workgroup (ch, s) reduces images [s*ipb, min(n,(s+1)*ipb)) of channel ch
// to (count, mean, M2) with a two-pass sum (second pass hits L2), so no cancellation.
template <int V>
__global__ __launch_bounds__(kThreads) void k_bn_stats_partial(const float* __restrict__ x,
                                                               int64_t stride, int n, int hw,
                                                               int ipb, float* __restrict__ part) {
  __shared__ float red[kThreads / 64];
  const int ch = blockIdx.x, s = blockIdx.y, splits = gridDim.y;
  const int n0 = s * ipb, n1 = min(n, n0 + ipb);
  const int hwv = hw / V;
  const int total = (n1 - n0) * hwv;
  const float* xc = x + (int64_t)ch * hw;
  float acc = 0.f;
  for (int v = threadIdx.x; v < total; v += blockDim.x) {
    const int img = v / hwv, q = v - img * hwv;
    float t[V];
    Vec<V>::ld(xc + (int64_t)(n0 + img) * stride + (int64_t)q * V, t);
#pragma unroll
    for (int e = 0; e < V; ++e) acc += t[e];
  }
  const float cnt = (float)((n1 - n0) * hw);
  const float mu = block_sum(acc, red) / cnt;
  float m2 = 0.f;
  for (int v = threadIdx.x; v < total; v += blockDim.x) {
    const int img = v / hwv, q = v - img * hwv;
    float t[V];
    Vec<V>::ld(xc + (int64_t)(n0 + img) * stride + (int64_t)q * V, t);
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

// One thread per channel merges the splits in index order (pairwise update of
// count/mean/M2), then mean and 1/sqrt(M2/P + eps).
__global__ void k_bn_stats_finalize(const float* __restrict__ part, int c, int splits, float eps,
                                    float* __restrict__ mean, float* __restrict__ istd) {
  const int ch = blockIdx.x * blockDim.x + threadIdx.x;
  if (ch >= c) return;
  const float* p = part + (int64_t)ch * splits * 3;
  float cnt = p[0], mu = p[1], m2 = p[2];
  for (int s = 1; s < splits; ++s) {
    const float cb = p[3 * s], mb = p[3 * s + 1], m2b = p[3 * s + 2];
    const float tot = cnt + cb, d = mb - mu;
    mu = mu + d * (cb / tot);
    m2 = m2 + m2b + d * d * (cnt * cb / tot);
    cnt = tot;
  }
  mean[ch] = mu;
  istd[ch] = 1.0f / sqrtf(m2 / cnt + eps);
}

// ----------------------------------------------------------------------------- BN apply + ReLU

template <int V, bool COPY>
__global__ __launch_bounds__(kThreads) void k_bn_relu(
    const float* __restrict__ x, int64_t x_stride, float* __restrict__ out, int64_t out_stride,
    float* __restrict__ copy_out, int64_t copy_stride, int c, int hw, int64_t total /*vectors*/,
    const float* __restrict__ gamma, const float* __restrict__ beta, const float* __restrict__ mean,
    const float* __restrict__ istd) {
  const int hwv = hw / V;
  for (int64_t v = (int64_t)blockIdx.x * kThreads + threadIdx.x; v < total;
       v += (int64_t)gridDim.x * kThreads) {
    const int row = (int)(v / hwv), q = (int)(v - (int64_t)row * hwv);
    const int img = row / c, ch = row - img * c;
    float scale, shift;
    bn_fold(gamma[ch], beta[ch], mean[ch], istd[ch], scale, shift);
    const int64_t inner = (int64_t)ch * hw + (int64_t)q * V;
    float t[V], r[V];
    Vec<V>::ld(x + (int64_t)img * x_stride + inner, t);
#pragma unroll
    for (int e = 0; e < V; ++e) r[e] = fmaxf(__fmaf_rn(t[e], scale, shift), 0.f);
    Vec<V>::st(out + (int64_t)img * out_stride + inner, r);
    if (COPY) Vec<V>::st(copy_out + (int64_t)img * copy_stride + inner, t);
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
  __shared__ float red[kThreads / 64];
  const int ch = blockIdx.x, s = blockIdx.y, splits = gridDim.y;
  const int n0 = s * ipb, n1 = min(n, n0 + ipb);
  const int hwv = hw / V;
  const int total = (n1 - n0) * hwv;
  float scale, shift;
  const float mu = mean[ch], is = istd[ch];
  bn_fold(gamma[ch], beta[ch], mu, is, scale, shift);
  float sb = 0.f, sg = 0.f;
  for (int v = threadIdx.x; v < total; v += blockDim.x) {
    const int img = v / hwv, q = v - img * hwv;
    const int64_t inner = (int64_t)ch * hw + (int64_t)q * V;
    float t[V], g[V];
    Vec<V>::ld(x + (int64_t)(n0 + img) * x_stride + inner, t);
    Vec<V>::ld(dact + (int64_t)(n0 + img) * dact_stride + inner, g);
#pragma unroll
    for (int e = 0; e < V; ++e) {
      const float dz = __fmaf_rn(t[e], scale, shift) > 0.f ? g[e] : 0.f;
      sb += dz;
      sg = __fmaf_rn(dz, (t[e] - mu) * is, sg);
    }
  }
  sb = block_sum(sb, red);
  sg = block_sum(sg, red);
  if (threadIdx.x == 0) {
    float* p = part + ((int64_t)ch * splits + s) * 2;
    p[0] = sb; p[1] = sg;
  }
}

__global__ void k_bn_bwd_finalize(const float* __restrict__ part, int c, int splits,
                                  float* __restrict__ dgamma, float* __restrict__ dbeta) {
  const int ch = blockIdx.x * blockDim.x + threadIdx.x;
  if (ch >= c) return;
  const float* p = part + (int64_t)ch * splits * 2;
  float sb = 0.f, sg = 0.f;
  for (int s = 0; s < splits; ++s) { sb += p[2 * s]; sg += p[2 * s + 1]; }
  dbeta[ch] = sb;
  dgamma[ch] = sg;
}

template <int V, bool ACC>
__global__ __launch_bounds__(kThreads) void k_bn_bwd_apply(
    const float* __restrict__ x, int64_t x_stride, const float* dact /* may alias du */,
    int64_t dact_stride, float* du, int64_t du_stride, int c, int hw, int64_t total,
    float inv_p, const float* __restrict__ gamma, const float* __restrict__ beta,
    const float* __restrict__ mean, const float* __restrict__ istd,
    const float* __restrict__ dgamma, const float* __restrict__ dbeta) {
  const int hwv = hw / V;
  for (int64_t v = (int64_t)blockIdx.x * kThreads + threadIdx.x; v < total;
       v += (int64_t)gridDim.x * kThreads) {
    const int row = (int)(v / hwv), q = (int)(v - (int64_t)row * hwv);
    const int img = row / c, ch = row - img * c;
    const float mu = mean[ch], is = istd[ch];
    float scale, shift;
    bn_fold(gamma[ch], beta[ch], mu, is, scale, shift);
    const float mb = dbeta[ch] * inv_p, mg = dgamma[ch] * inv_p;
    const int64_t inner = (int64_t)ch * hw + (int64_t)q * V;
    float t[V], g[V], r[V];
    Vec<V>::ld(x + (int64_t)img * x_stride + inner, t);
    Vec<V>::ld(dact + (int64_t)img * dact_stride + inner, g);
    float* dp = du + (int64_t)img * du_stride + inner;
    if (ACC) Vec<V>::ld(dp, r);
#pragma unroll
    for (int e = 0; e < V; ++e) {
      const float dz = __fmaf_rn(t[e], scale, shift) > 0.f ? g[e] : 0.f;
      const float xh = (t[e] - mu) * is;
      const float d = scale * (dz - mb - xh * mg);
      r[e] = ACC ? r[e] + d : d;
    }
    Vec<V>::st(dp, r);
  }
}

int splits_for(int n, int c) {
  // enough workgroups to cover the chip (256 CUs) a few times over, at least one image each
  int s = (1024 + c - 1) / c;
  if (s > n) s = n;
  if (s < 1) s = 1;
  return s;
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

int bn_stats_splits(int n, int c, int hw) { (void)hw; return splits_for(n, c); }
size_t bn_stats_partial_floats(int n, int c, int hw) { return (size_t)c * bn_stats_splits(n, c, hw) * 3; }

hipError_t launch_bn_stats(const float* x, int64_t stride, int n, int c, int hw, float eps,
                           float* mean, float* istd, float* partials, hipStream_t st) {
  if (c <= 0) return hipSuccess;
  const int splits = bn_stats_splits(n, c, hw);
  const int ipb = (n + splits - 1) / splits;
  const int gs = (n + ipb - 1) / ipb;  // every split non-empty
  const bool v4 = (hw % 4 == 0) && (stride % 4 == 0) && aligned16(x);
  const int work = ipb * (v4 ? hw / 4 : hw);
  const int threads = work <= 64 ? 64 : (work <= 128 ? 128 : kThreads);
  dim3 grid((unsigned)c, (unsigned)gs);
  if (v4)
    hipLaunchKernelGGL(k_bn_stats_partial<4>, grid, dim3(threads), 0, st, x, stride, n, hw, ipb, partials);
  else
    hipLaunchKernelGGL(k_bn_stats_partial<1>, grid, dim3(threads), 0, st, x, stride, n, hw, ipb, partials);
  hipLaunchKernelGGL(k_bn_stats_finalize, dim3((c + 63) / 64), dim3(64), 0, st, partials, c, gs, eps, mean, istd);
  return hipGetLastError();
}

hipError_t launch_bn_relu(const float* x, int64_t x_stride, float* out, int64_t out_stride,
                          float* copy_out, int64_t copy_stride, int n, int c, int hw,
                          const float* gamma, const float* beta, const float* mean,
                          const float* istd, hipStream_t st) {
  if (n <= 0 || c <= 0 || hw <= 0) return hipSuccess;
  const bool v4 = (hw % 4 == 0) && (x_stride % 4 == 0) && (out_stride % 4 == 0) && aligned16(x) &&
                  aligned16(out) && (!copy_out || ((copy_stride % 4 == 0) && aligned16(copy_out)));
  const int64_t total = (int64_t)n * c * (v4 ? hw / 4 : hw);
  dim3 grid(grid_for(total, kThreads * 2, 65535 * 4));
#define DNB_LAUNCH_BNRELU(V, C)                                                                     \
  hipLaunchKernelGGL((k_bn_relu<V, C>), grid, dim3(kThreads), 0, st, x, x_stride, out, out_stride, \
                     copy_out, copy_stride, c, hw, total, gamma, beta, mean, istd)
  if (v4) { if (copy_out) DNB_LAUNCH_BNRELU(4, true); else DNB_LAUNCH_BNRELU(4, false); }
  else    { if (copy_out) DNB_LAUNCH_BNRELU(1, true); else DNB_LAUNCH_BNRELU(1, false); }
#undef DNB_LAUNCH_BNRELU
  return hipGetLastError();
}

size_t bn_bwd_partial_floats(int n, int c, int hw) { (void)hw; return (size_t)c * splits_for(n, c) * 2; }

hipError_t launch_bn_relu_bwd(const float* x, int64_t x_stride, const float* dact,
                              int64_t dact_stride, float* du, int64_t du_stride, bool accumulate,
                              int n, int c, int hw, const float* gamma, const float* beta,
                              const float* mean, const float* istd, float* dgamma, float* dbeta,
                              float* partials, hipStream_t st) {
  if (n <= 0 || c <= 0 || hw <= 0) return hipSuccess;
  const int splits = splits_for(n, c);
  const int ipb = (n + splits - 1) / splits;
  const int gs = (n + ipb - 1) / ipb;
  const bool v4 = (hw % 4 == 0) && (x_stride % 4 == 0) && (dact_stride % 4 == 0) &&
                  (du_stride % 4 == 0) && aligned16(x) && aligned16(dact) && aligned16(du);
  const int work = ipb * (v4 ? hw / 4 : hw);
  const int threads = work <= 64 ? 64 : (work <= 128 ? 128 : kThreads);
  dim3 rgrid((unsigned)c, (unsigned)gs);
  if (v4)
    hipLaunchKernelGGL(k_bn_bwd_partial<4>, rgrid, dim3(threads), 0, st, x, x_stride, dact, dact_stride,
                       n, hw, ipb, gamma, beta, mean, istd, partials);
  else
    hipLaunchKernelGGL(k_bn_bwd_partial<1>, rgrid, dim3(threads), 0, st, x, x_stride, dact, dact_stride,
                       n, hw, ipb, gamma, beta, mean, istd, partials);
  hipLaunchKernelGGL(k_bn_bwd_finalize, dim3((c + 63) / 64), dim3(64), 0, st, partials, c, gs, dgamma, dbeta);
  const int64_t total = (int64_t)n * c * (v4 ? hw / 4 : hw);
  const float inv_p = 1.0f / ((float)n * (float)hw);
  dim3 grid(grid_for(total, kThreads * 2, 65535 * 4));
#define DNB_LAUNCH_BNBWD(V, A)                                                                      \
  hipLaunchKernelGGL((k_bn_bwd_apply<V, A>), grid, dim3(kThreads), 0, st, x, x_stride, dact,       \
                     dact_stride, du, du_stride, c, hw, total, inv_p, gamma, beta, mean, istd,     \
                     dgamma, dbeta)
  if (v4) { if (accumulate) DNB_LAUNCH_BNBWD(4, true); else DNB_LAUNCH_BNBWD(4, false); }
  else    { if (accumulate) DNB_LAUNCH_BNBWD(1, true); else DNB_LAUNCH_BNBWD(1, false); }
#undef DNB_LAUNCH_BNBWD
  return hipGetLastError();
}

}  // namespace dnb
