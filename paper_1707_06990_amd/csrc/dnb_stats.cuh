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
  for (int i = threadIdx.x; i < T; i += blockDim.x) {
    Stat3 o{p[3 * i], p[3 * i + 1], p[3 * i + 2]};
    v = stat_combine(v, o);
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

}  // namespace dnb
