// Device helpers shared by the kernel files: BN's folded affine map and the deterministic
// merging of (count, mean, M2) partial statistics.
#pragma once

#include <hip/hip_runtime.h>

namespace dnb {

// The one place BN's affine map is folded into (scale, shift); forward, recomputation
// and backward all call it so the ReLU mask is reproduced bit for bit.
__device__ __forceinline__ void bn_fold(float gamma, float beta, float mean, float istd,
                                        float& scale, float& shift) {
  scale = __fmul_rn(gamma, istd);
  shift = __fmaf_rn(-mean, scale, beta);
}

__device__ __forceinline__ float bn_istd(float m2, float cnt, float eps) {
  return __fdiv_rn(1.0f, __fsqrt_rn(__fadd_rn(__fdiv_rn(m2, cnt), eps)));
}

struct Stat3 {
  float c, m, m2;  // count, mean, sum of squared deviations from the mean
};

// Pairwise update: statistics of the union of two disjoint sets (a first, then b).
__device__ __forceinline__ Stat3 stat_combine(Stat3 a, Stat3 b) {
  if (b.c == 0.f) return a;
  if (a.c == 0.f) return b;
  const float tot = __fadd_rn(a.c, b.c), d = __fsub_rn(b.m, a.m);
  Stat3 r;
  r.c = tot;
  r.m = __fmaf_rn(d, __fdiv_rn(b.c, tot), a.m);
  r.m2 = __fadd_rn(__fadd_rn(a.m2, b.m2), __fmul_rn(__fmul_rn(d, d), __fdiv_rn(__fmul_rn(a.c, b.c), tot)));
  return r;
}

// Butterfly over the 64 lanes; both lanes of a pair evaluate combine(lower lane, upper lane),
// so every lane ends with the same bits.
__device__ __forceinline__ Stat3 stat_merge_wave(Stat3 v) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    Stat3 o;
    o.c = __shfl_xor(v.c, off, 64); o.m = __shfl_xor(v.m, off, 64); o.m2 = __shfl_xor(v.m2, off, 64);
    v = (lane & off) ? stat_combine(o, v) : stat_combine(v, o);
  }
  return v;
}

// Merges T partials stored as [T][3] floats with the whole workgroup (blockDim a multiple of
// 64, at most 1024): thread t folds partials t, t+blockDim, ... in order, then waves, then the
// per-wave results in wave order.  `sh` needs 3 floats per wave.  Result in every thread.
__device__ __forceinline__ Stat3 stat_merge_block(const float* __restrict__ p, int T, float* sh) {
  Stat3 v{0.f, 0.f, 0.f};
  // four of the thread's partials are requested before the first is folded in (a fold per load
  // would wait out one memory latency per partial); loads past T repeat the last partial and
  // enter as empty sets, which stat_combine passes through unchanged
  const int bd = blockDim.x;
  for (int i = threadIdx.x; i < T; i += 4 * bd) {
    Stat3 o[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int q = min(i + u * bd, T - 1);
      o[u] = Stat3{p[3 * q], p[3 * q + 1], p[3 * q + 2]};
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (i + u * bd >= T) o[u] = Stat3{0.f, 0.f, 0.f};
      v = stat_combine(v, o[u]);
    }
  }
  v = stat_merge_wave(v);
  const int wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) { sh[3 * wave] = v.c; sh[3 * wave + 1] = v.m; sh[3 * wave + 2] = v.m2; }
  __syncthreads();
  Stat3 r{sh[0], sh[1], sh[2]};
  for (int w = 1; w < nw; ++w) r = stat_combine(r, Stat3{sh[3 * w], sh[3 * w + 1], sh[3 * w + 2]});
  return r;
}


// ---- pieces of the fp32 BN+ReLU backward reduction shared by its own kernel and by the launch
// that carries it beside the weight gradients (same code, same bits)

__device__ __forceinline__ float bnb_wave_sum(float v) {
  // butterfly over the 64 lanes of a wavefront: every lane ends with the same total
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// Sum over the workgroup; the result is returned to every thread.  `red` holds one
// float per wave.  Safe to call repeatedly (barrier before reuse).
__device__ __forceinline__ float bnb_block_sum(float v, float* red) {
  v = bnb_wave_sum(v);
  const int wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[wave] = v;
  __syncthreads();
  float t = 0.f;
  for (int i = 0; i < nw; ++i) t += red[i];
  return t;
}

// rows of hw contiguous floats, one per image: walks (image, vector-in-row) pairs with a stride
// of blockDim threads without a division per element
struct RowIter {
  int img, q, dimg, dq, hwv;
  __device__ __forceinline__ RowIter(int hwv_, int tid, int nthr) : hwv(hwv_) {
    img = tid / hwv_; q = tid - img * hwv_;
    dimg = nthr / hwv_; dq = nthr - dimg * hwv_;
  }
  __device__ __forceinline__ void next() {
    img += dimg; q += dq;
    if (q >= hwv) { q -= hwv; ++img; }
  }
};

struct BnBwdPartialArgs {
  const float* x; int64_t x_stride; const float* dact; int64_t dact_stride;
  int n, hw, ipb;
  const float *gamma, *beta, *mean, *istd;
  float* part;
  int c, splits;  // grid of the reduction: channels x image splits
};

// Workgroup (ch, s): partial sums of dz and dz*xhat over images [s*ipb, (s+1)*ipb) of channel ch,
// 16-byte accesses (hw and the strides multiples of 4, 16-byte aligned), 256 threads.
__device__ __forceinline__ void bn_bwd_partial_body4(const BnBwdPartialArgs& A, int ch, int s) {
  __shared__ float red[4];
  const int n0 = s * A.ipb, ni = min(A.n, n0 + A.ipb) - n0;
  const int hwv = A.hw / 4;
  float scale, shift;
  const float mu = A.mean[ch], is = A.istd[ch];
  bn_fold(A.gamma[ch], A.beta[ch], mu, is, scale, shift);
  const int64_t inner = (int64_t)ch * A.hw;
  const float* xp = A.x + (int64_t)n0 * A.x_stride + inner;
  const float* gp = A.dact + (int64_t)n0 * A.dact_stride + inner;
  float sb = 0.f, sg = 0.f;
  // four positions per pass: all eight loads are issued (unconditionally; a position past the
  // range repeats the last image's) before the first is consumed
  for (RowIter it(hwv, threadIdx.x, blockDim.x); it.img < ni;) {
    float4 t[4], g[4];
    bool ok[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      ok[u] = it.img < ni;
      const int im = ok[u] ? it.img : ni - 1;
      t[u] = *reinterpret_cast<const float4*>(xp + (int64_t)im * A.x_stride + (int64_t)it.q * 4);
      g[u] = *reinterpret_cast<const float4*>(gp + (int64_t)im * A.dact_stride + (int64_t)it.q * 4);
      it.next();
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (ok[u]) {
        const float tv[4] = {t[u].x, t[u].y, t[u].z, t[u].w}, gv[4] = {g[u].x, g[u].y, g[u].z, g[u].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float dz = __fmaf_rn(tv[e], scale, shift) > 0.f ? gv[e] : 0.f;
          sb += dz;
          sg = __fmaf_rn(dz, (tv[e] - mu) * is, sg);
        }
      }
    }
  }
  sb = bnb_block_sum(sb, red);
  sg = bnb_block_sum(sg, red);
  if (threadIdx.x == 0) {
    float* p = A.part + ((int64_t)ch * A.splits + s) * 2;
    p[0] = sb; p[1] = sg;
  }
}

}  // namespace dnb
