// Whole training step of an ImageNet-shaped DenseNet-BC (bf16 feature maps, NHWC, fp32 accumulation
// and statistics): the glue around four dense blocks -- 7x7 stride-2 stem conv, BN -> ReLU, 3x3
// stride-2 max pool, transitions (BN -> ReLU -> 1x1 conv -> 2x2 average pool), tail (BN -> ReLU ->
// global average pool -> linear) and the mean softmax cross-entropy, forward and backward -- built
// from the bf16 block library's own kernels plus the small kernels in this file.
// Paper: Section 2 ("DenseNet Architecture": dense blocks joined by pooling layers); the ImageNet
// models of Section 5 have four dense blocks.  The glue keeps its few feature maps (one stem
// output, one BN+ReLU-input per block: constant in depth); the dense blocks run under the
// descriptor's schedule.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <new>
#include <vector>

#include "../../include/dnb.h"
#include "dnb_internal.h"

namespace dnb {
namespace {

typedef unsigned short u16;
__device__ __forceinline__ float bf2f(u16 v) { return __uint_as_float((unsigned)v << 16); }
__device__ __forceinline__ u16 f2bf(float f) {  // round to nearest even (hardware conversion)
  const __bf16 b = (__bf16)f;
  return __builtin_bit_cast(u16, b);
}
union V8 {
  uint4 q;
  u16 h[8];
};

constexpr int kTile = 8;                  // output pixels per tile side of the stem kernels
constexpr int kPatch = 2 * kTile + 5;     // input rows / columns a tile of the 7x7 stride-2 conv touches (21)
constexpr int kTaps = 147;                // 3 channels x 7 x 7

// Stages the input patch of output tile (ty, tx) of image img: rows 2*ty*8 - 3 .. + 20, same for
// columns, 3 channels, zero outside the image.  patch[(r*21 + q)*3 + ci].
__device__ __forceinline__ void stage_patch(const u16* __restrict__ x, int S, int img, int ty, int tx, float* patch) {
  const int y0 = 2 * ty * kTile - 3, x0 = 2 * tx * kTile - 3;
  for (int i = threadIdx.x; i < kPatch * kPatch * 3; i += blockDim.x) {
    const int r = i / (kPatch * 3), rem = i - r * (kPatch * 3);
    const int q = rem / 3, ci = rem - q * 3;
    const int yy = y0 + r, xx = x0 + q;
    float v = 0.f;
    if (yy >= 0 && yy < S && xx >= 0 && xx < S) v = bf2f(x[(((int64_t)img * S + yy) * S + xx) * 3 + ci]);
    patch[i] = v;
  }
}

// The stem conv's weights as its kernel reads them: Wt[t][c] = W (C, 3, 7, 7) rounded to bf16 (as every
// conv of this path reads its weights), tap-major with t = (ky*7 + kx)*3 + ci.
__global__ __launch_bounds__(256) void k_stem_pack_w(const float* __restrict__ W, float* __restrict__ Wt, int C) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= kTaps * C) return;
  const int t = i / C, c = i - t * C;
  const int ci = t % 3, kk = t / 3, ky = kk / 7, kx = kk - ky * 7;
  Wt[i] = bf2f(f2bf(W[((c * 3 + ci) * 7 + ky) * 7 + kx]));
}

// Stem convolution: out (n, S/2, S/2, C) bf16 = conv7x7 stride 2 pad 3 of x (n, S, S, 3) bf16 with the
// packed weights Wt (147, C); fp32 accumulation.  One workgroup per 8x8 output tile with the 21x21x3
// input patch in LDS; a thread owns one pixel and C/4 = 4*NV channels.  Each wave is one channel
// group, so its weight addresses are the same for all lanes: they are read through the scalar
// cache straight into the FMAs' scalar operand, and LDS serves only the one patch value per tap
// (with the weights in LDS as well, six 16-byte broadcast reads per 24 FMAs kept the CU's one LDS
// twice as busy as its four vector units: 394 us per launch at C = 96, batch 32).
// grid (tiles, n), 256 threads.
template <int NV>
__global__ __launch_bounds__(256) void k_stem_conv7(const u16* __restrict__ x, const float* __restrict__ Wt,
                                                    u16* __restrict__ out, int S) {
  constexpr int C = 16 * NV, CPG = 4 * NV;
  extern __shared__ float lds[];
  float* patch = lds;                  // [21*21*3]
  const int So = S / 2, tiles = So / kTile;
  const int img = blockIdx.y, ty = blockIdx.x / tiles, tx = blockIdx.x - ty * tiles;
  stage_patch(x, S, img, ty, tx, patch);
  __syncthreads();
  const int p = threadIdx.x & 63, py = p >> 3, px = p & 7;
  const int grp = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // the same for the whole wave
  float4 acc[NV];
#pragma unroll
  for (int q = 0; q < NV; ++q) acc[q] = make_float4(0.f, 0.f, 0.f, 0.f);
  const float* pb = patch + ((2 * py) * kPatch + 2 * px) * 3;
  const float* wb = Wt + grp * CPG;
  for (int ky = 0; ky < 7; ++ky) {
#pragma unroll
    for (int kxc = 0; kxc < 21; ++kxc) {   // (kx, ci) pairs are contiguous in the patch row and in t
      const float v = pb[ky * kPatch * 3 + kxc];
      const float* wr = wb + (ky * 21 + kxc) * C;
#pragma unroll
      for (int q = 0; q < NV; ++q) {
        const float4 w4 = *reinterpret_cast<const float4*>(wr + 4 * q);
        acc[q].x = __fmaf_rn(v, w4.x, acc[q].x); acc[q].y = __fmaf_rn(v, w4.y, acc[q].y);
        acc[q].z = __fmaf_rn(v, w4.z, acc[q].z); acc[q].w = __fmaf_rn(v, w4.w, acc[q].w);
      }
    }
  }
  const int oy = ty * kTile + py, ox = tx * kTile + px;
  u16* o = out + (((int64_t)img * So + oy) * So + ox) * C + grp * CPG;
#pragma unroll
  for (int q = 0; q < NV; ++q) {
    uint2 pk;
    pk.x = (unsigned)f2bf(acc[q].x) | ((unsigned)f2bf(acc[q].y) << 16);
    pk.y = (unsigned)f2bf(acc[q].z) | ((unsigned)f2bf(acc[q].w) << 16);
    *reinterpret_cast<uint2*>(o + 4 * q) = pk;
  }
}

// Stem weight gradient: dW (C, 3, 7, 7) = sum over output pixels of g (n, S/2, S/2, C) bf16 times the
// input patch.  A workgroup walks over 8x8 output tiles (tile = blockIdx.x, += gridDim.x), staging
// the tile's gradients and input patch in LDS; a thread keeps 4 channels x TPC taps of the result in
// registers over all its tiles and stores them into its workgroup's partial, OIHW order
// ([gridDim.x][C*147] floats, summed afterwards in a fixed order).  C/4 channel quads x 256/(C/4)
// tap chunks of TPC taps.
template <int C, int TPC>
__global__ __launch_bounds__(256) void k_stem_wgrad7(const u16* __restrict__ x, const u16* __restrict__ g,
                                                     float* __restrict__ part, int S, int n) {
  constexpr int QUADS = C / 4, CHUNKS = 256 / QUADS;
  static_assert(CHUNKS * TPC >= kTaps, "the tap chunks cover all 147 taps");
  extern __shared__ float lds[];
  float* gl = lds;                       // [64][C]
  float* patch = lds + 64 * C;           // [21*21*3]
  const int So = S / 2, tiles = So / kTile, per_img = tiles * tiles, total = per_img * n;
  const int quad = threadIdx.x % QUADS, chunk = threadIdx.x / QUADS;
  const bool active = chunk < CHUNKS;
  int off[TPC];
  bool live[TPC];
#pragma unroll
  for (int tt = 0; tt < TPC; ++tt) {
    const int t = chunk * TPC + tt;        // OIHW tap index (ci*7 + ky)*7 + kx
    live[tt] = active && t < kTaps;
    const int tc = live[tt] ? t : 0;
    const int ci = tc / 49, r = tc - ci * 49, ky = r / 7, kx = r - ky * 7;
    off[tt] = (ky * kPatch + kx) * 3 + ci;
  }
  float4 acc[TPC];
#pragma unroll
  for (int tt = 0; tt < TPC; ++tt) acc[tt] = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int tile = blockIdx.x; tile < total; tile += gridDim.x) {
    const int img = tile / per_img, r = tile - img * per_img, ty = r / tiles, tx = r - ty * tiles;
    __syncthreads();  // the previous tile's reads are done
    stage_patch(x, S, img, ty, tx, patch);
    for (int i = threadIdx.x; i < 64 * (C / 8); i += 256) {
      const int p = i / (C / 8), v = i - p * (C / 8);
      const int oy = ty * kTile + (p >> 3), ox = tx * kTile + (p & 7);
      V8 raw;
      raw.q = *reinterpret_cast<const uint4*>(g + (((int64_t)img * So + oy) * So + ox) * C + 8 * v);
#pragma unroll
      for (int e = 0; e < 8; ++e) gl[p * C + 8 * v + e] = bf2f(raw.h[e]);
    }
    __syncthreads();
    if (active) {
      for (int p = 0; p < 64; ++p) {
        const float4 g4 = *reinterpret_cast<const float4*>(gl + p * C + 4 * quad);
        const float* pb = patch + ((2 * (p >> 3)) * kPatch + 2 * (p & 7)) * 3;
#pragma unroll
        for (int tt = 0; tt < TPC; ++tt) {
          const float v = pb[off[tt]];
          acc[tt].x = __fmaf_rn(g4.x, v, acc[tt].x); acc[tt].y = __fmaf_rn(g4.y, v, acc[tt].y);
          acc[tt].z = __fmaf_rn(g4.z, v, acc[tt].z); acc[tt].w = __fmaf_rn(g4.w, v, acc[tt].w);
        }
      }
    }
  }
  float* po = part + (int64_t)blockIdx.x * (C * kTaps);
#pragma unroll
  for (int tt = 0; tt < TPC; ++tt) {
    if (live[tt]) {
      const int t = chunk * TPC + tt;
      po[(4 * quad + 0) * kTaps + t] = acc[tt].x;
      po[(4 * quad + 1) * kTaps + t] = acc[tt].y;
      po[(4 * quad + 2) * kTaps + t] = acc[tt].z;
      po[(4 * quad + 3) * kTaps + t] = acc[tt].w;
    }
  }
}

// BN+ReLU (folded scale, shift per channel) and 3x3 stride-2 pad-1 max pooling in one pass:
// out (n, H/2, W/2, C) bf16 = max over the window of max(0, fma(s, scale, shift)), positions outside
// the image left out; pos receives the window position 3*i + j of the maximum, the first in scan
// order among equals.  A thread owns one output pixel and 8 channels.
__global__ __launch_bounds__(256) void k_maxpool_bnrelu(const u16* __restrict__ s, const float2* __restrict__ fold,
                                                        u16* __restrict__ out, unsigned char* __restrict__ pos, int n,
                                                        int H, int W, int C) {
  const int Ho = H / 2, Wo = W / 2, cv = C / 8;
  const int64_t total = (int64_t)n * Ho * Wo * cv;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int v = (int)(i % cv);
    int64_t r = i / cv;
    const int ox = (int)(r % Wo); r /= Wo;
    const int oy = (int)(r % Ho);
    const int img = (int)(r / Ho);
    float sc[8], sh[8], best[8];
    int bi[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float2 f = fold[8 * v + e];
      sc[e] = f.x; sh[e] = f.y; best[e] = 0.f; bi[e] = -1;
    }
#pragma unroll
    for (int wi = 0; wi < 3; ++wi) {
      const int yy = 2 * oy + wi - 1;
      if (yy < 0 || yy >= H) continue;
#pragma unroll
      for (int wj = 0; wj < 3; ++wj) {
        const int xx = 2 * ox + wj - 1;
        if (xx < 0 || xx >= W) continue;
        V8 raw;
        raw.q = *reinterpret_cast<const uint4*>(s + (((int64_t)img * H + yy) * W + xx) * C + 8 * v);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float a = fmaxf(__fmaf_rn(bf2f(raw.h[e]), sc[e], sh[e]), 0.f);
          if (bi[e] < 0 || a > best[e]) { best[e] = a; bi[e] = 3 * wi + wj; }
        }
      }
    }
    V8 o;
    unsigned char pb[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { o.h[e] = f2bf(best[e]); pb[e] = (unsigned char)bi[e]; }
    const int64_t ob = (((int64_t)img * Ho + oy) * Wo + ox) * C + 8 * v;
    *reinterpret_cast<uint4*>(out + ob) = o.q;
    *reinterpret_cast<uint2*>(pos + ob) = *reinterpret_cast<const uint2*>(pb);
  }
}

// Adjoint of the pooling: din (n, H, W, C) bf16; an input position receives the gradients of the (at
// most four) windows whose maximum it is, added in window scan order in fp32.  Gather form: no atomics.
__global__ __launch_bounds__(256) void k_maxpool_bwd(const u16* __restrict__ dout, const unsigned char* __restrict__ pos,
                                                     u16* __restrict__ din, int n, int H, int W, int C) {
  const int Ho = H / 2, Wo = W / 2, cv = C / 8;
  const int64_t total = (int64_t)n * H * W * cv;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int v = (int)(i % cv);
    int64_t r = i / cv;
    const int x = (int)(r % W); r /= W;
    const int y = (int)(r % H);
    const int img = (int)(r / H);
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    // windows (oy, ox) that contain (y, x): 2*oy + wi - 1 = y with wi in 0..2
    for (int oy = (y - 1 + 1) / 2; oy <= (y + 1) / 2; ++oy) {
      const int wi = y - 2 * oy + 1;
      if (oy < 0 || oy >= Ho || wi < 0 || wi > 2) continue;
      for (int ox = x / 2; ox <= (x + 1) / 2; ++ox) {
        const int wj = x - 2 * ox + 1;
        if (ox < 0 || ox >= Wo || wj < 0 || wj > 2) continue;
        const int64_t ob = (((int64_t)img * Ho + oy) * Wo + ox) * C + 8 * v;
        V8 gq;
        gq.q = *reinterpret_cast<const uint4*>(dout + ob);
        unsigned char pb[8];
        *reinterpret_cast<uint2*>(pb) = *reinterpret_cast<const uint2*>(pos + ob);
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (pb[e] == 3 * wi + wj) acc[e] += bf2f(gq.h[e]);
      }
    }
    V8 o;
#pragma unroll
    for (int e = 0; e < 8; ++e) o.h[e] = f2bf(acc[e]);
    *reinterpret_cast<uint4*>(din + (((int64_t)img * H + y) * W + x) * C + 8 * v) = o.q;
  }
}

// 2x2 average pooling, stride 2: out (n, H/2, W/2, C) bf16; and its adjoint.
__global__ __launch_bounds__(256) void k_avgpool2_rows(const u16* __restrict__ in, u16* __restrict__ out, int n, int H,
                                                       int W, int C) {
  const int Ho = H / 2, Wo = W / 2, cv = C / 8;
  const int64_t total = (int64_t)n * Ho * Wo * cv;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int v = (int)(i % cv);
    int64_t r = i / cv;
    const int ox = (int)(r % Wo); r /= Wo;
    const int oy = (int)(r % Ho);
    const int img = (int)(r / Ho);
    const u16* b = in + (((int64_t)img * H + 2 * oy) * W + 2 * ox) * C + 8 * v;
    V8 a, bb, c, d, o;
    a.q = *reinterpret_cast<const uint4*>(b);
    bb.q = *reinterpret_cast<const uint4*>(b + C);
    c.q = *reinterpret_cast<const uint4*>(b + (int64_t)W * C);
    d.q = *reinterpret_cast<const uint4*>(b + (int64_t)W * C + C);
#pragma unroll
    for (int e = 0; e < 8; ++e)
      o.h[e] = f2bf(0.25f * ((bf2f(a.h[e]) + bf2f(bb.h[e])) + (bf2f(c.h[e]) + bf2f(d.h[e]))));
    *reinterpret_cast<uint4*>(out + (((int64_t)img * Ho + oy) * Wo + ox) * C + 8 * v) = o.q;
  }
}

__global__ __launch_bounds__(256) void k_avgpool2_rows_bwd(const u16* __restrict__ dout, u16* __restrict__ din, int n,
                                                           int H, int W, int C) {
  const int Ho = H / 2, Wo = W / 2, cv = C / 8;
  const int64_t total = (int64_t)n * H * W * cv;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int v = (int)(i % cv);
    int64_t r = i / cv;
    const int x = (int)(r % W); r /= W;
    const int y = (int)(r % H);
    const int img = (int)(r / H);
    V8 gq, o;
    gq.q = *reinterpret_cast<const uint4*>(dout + (((int64_t)img * Ho + (y >> 1)) * Wo + (x >> 1)) * C + 8 * v);
#pragma unroll
    for (int e = 0; e < 8; ++e) o.h[e] = f2bf(0.25f * bf2f(gq.h[e]));
    *reinterpret_cast<uint4*>(din + (((int64_t)img * H + y) * W + x) * C + 8 * v) = o.q;
  }
}

// Tail: pooled (n, C) fp32 = mean over the hw pixels of max(0, fma(y, scale, shift)); a thread owns one
// image and 8 channels and adds its pixels in order.
__global__ __launch_bounds__(256) void k_global_avgpool_bnrelu(const u16* __restrict__ y, const float2* __restrict__ fold,
                                                               float* __restrict__ pooled, int n, int hw, int C) {
  const int cv = C / 8;
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= n * cv) return;
  const int img = i / cv, v = i - img * cv;
  float sc[8], sh[8], acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const float2 f = fold[8 * v + e];
    sc[e] = f.x; sh[e] = f.y; acc[e] = 0.f;
  }
  for (int q = 0; q < hw; ++q) {
    V8 raw;
    raw.q = *reinterpret_cast<const uint4*>(y + ((int64_t)img * hw + q) * C + 8 * v);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] += fmaxf(__fmaf_rn(bf2f(raw.h[e]), sc[e], sh[e]), 0.f);
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) pooled[(int64_t)img * C + 8 * v + e] = acc[e] / (float)hw;
}

// dtz (n, hw, C) bf16 = dpooled (n, C) / hw: the adjoint of the global average pool
__global__ __launch_bounds__(256) void k_global_avgpool_rows_bwd(const float* __restrict__ dpooled, u16* __restrict__ dtz,
                                                                 int n, int hw, int C) {
  const int cv = C / 8;
  const int64_t total = (int64_t)n * hw * cv;
  const float inv = 1.0f / (float)hw;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int v = (int)(i % cv);
    const int64_t p = i / cv;
    const int img = (int)(p / hw);
    V8 o;
#pragma unroll
    for (int e = 0; e < 8; ++e) o.h[e] = f2bf(dpooled[(int64_t)img * C + 8 * v + e] * inv);
    *reinterpret_cast<uint4*>(dtz + p * C + 8 * v) = o.q;
  }
}

inline unsigned grid_for(int64_t items, int per_block, unsigned cap = 65535u * 8u) {
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

constexpr int kStemWgradWorkgroups = 512;

// Wt: scratch of 147*C floats for the packed weights
hipError_t launch_stem_conv(const u16* x, const float* W, float* Wt, u16* out, int n, int S, int C, hipStream_t st) {
  const int tiles = (S / 2) / kTile;
  const dim3 grid((unsigned)(tiles * tiles), (unsigned)n);
  const size_t lds = (size_t)kPatch * kPatch * 3 * sizeof(float);
  hipLaunchKernelGGL(k_stem_pack_w, dim3((unsigned)((kTaps * C + 255) / 256)), dim3(256), 0, st, W, Wt, C);
  switch (C / 16) {
    case 1: hipLaunchKernelGGL(k_stem_conv7<1>, grid, dim3(256), lds, st, x, Wt, out, S); break;
    case 2: hipLaunchKernelGGL(k_stem_conv7<2>, grid, dim3(256), lds, st, x, Wt, out, S); break;
    case 4: hipLaunchKernelGGL(k_stem_conv7<4>, grid, dim3(256), lds, st, x, Wt, out, S); break;
    case 6: hipLaunchKernelGGL(k_stem_conv7<6>, grid, dim3(256), lds, st, x, Wt, out, S); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

int stem_wgrad_groups(int n, int S) {
  const int tiles = (S / 2) / kTile, total = tiles * tiles * n;
  return total < kStemWgradWorkgroups ? total : kStemWgradWorkgroups;
}

hipError_t launch_stem_wgrad(const u16* x, const u16* g, float* part, float* dW, int n, int S, int C, hipStream_t st) {
  const int G = stem_wgrad_groups(n, S);
  const size_t lds = ((size_t)64 * C + kPatch * kPatch * 3) * sizeof(float);
  switch (C) {
    case 16: hipLaunchKernelGGL((k_stem_wgrad7<16, 3>), dim3(G), dim3(256), lds, st, x, g, part, S, n); break;
    case 32: hipLaunchKernelGGL((k_stem_wgrad7<32, 5>), dim3(G), dim3(256), lds, st, x, g, part, S, n); break;
    case 64: hipLaunchKernelGGL((k_stem_wgrad7<64, 10>), dim3(G), dim3(256), lds, st, x, g, part, S, n); break;
    case 96: hipLaunchKernelGGL((k_stem_wgrad7<96, 15>), dim3(G), dim3(256), lds, st, x, g, part, S, n); break;
    default: return hipErrorInvalidValue;
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_sum_partials(part, G, (int64_t)C * kTaps, dW, st);
}

}  // namespace
}  // namespace dnb

using namespace dnb;

struct dnb_inet {
  dnb_inet_desc d;
  dnb_block* blk[4];
  dnb_block_desc bd[4];
  int cs, cout[4];
  // offsets in the pack (floats)
  size_t p_stem_w, p_stem_g, p_stem_b, p_block[4], p_g[4], p_b[4], p_w[4], p_bl, p_count;
  // workspace offsets (bytes)
  size_t o_s, o_pos, o_fold_s, o_stat_s;
  size_t o_feat[4], o_y[4], o_ws[4], o_stat[4], o_fold[4], o_pack[3], o_tconv;
  size_t o_gy, o_dtz, o_dconv, o_dfeat, o_da0, o_part, o_stem_wt;
  size_t o_pooled, o_dpooled, o_logits, o_dlogits, o_terms;
  size_t ws_bytes, glue_feature_bytes;
};

extern "C" {

int dnb_inet_create(const dnb_inet_desc* desc, dnb_inet** out) {
  if (!desc || !out) return DNB_E_NULL;
  const dnb_inet_desc& d = *desc;
  if (d.n < 1 || d.image < 32 || d.image % 32 != 0 || d.growth < 1 || d.classes < 1 || !(d.eps >= 0.f)) return DNB_E_BADDESC;
  for (int b = 0; b < 4; ++b)
    if (d.layers[b] < 1) return DNB_E_BADDESC;
  if (d.schedule != DNB_SCHED_SHARED && d.schedule != DNB_SCHED_STORE_ALL && d.schedule != DNB_SCHED_FUSED) return DNB_E_BADDESC;
  if (d.n > 4096 || d.classes > 65536 || d.image > 1024) return DNB_E_RANGE;
  const int cs = 2 * d.growth;
  // the stem kernels are built for 16, 32, 64 and 96 output channels (k = 8, 16, 32, 48)
  if (cs != 16 && cs != 32 && cs != 64 && cs != 96) return DNB_E_UNSUPPORTED;
  dnb_inet* net = new (std::nothrow) dnb_inet();
  if (!net) return DNB_E_NOMEM;
  net->d = d;
  net->cs = cs;
  for (int b = 0; b < 4; ++b) net->blk[b] = nullptr;
  const int k = d.growth;
  int c = cs, s = d.image / 4;
  net->p_stem_w = 0;
  net->p_stem_g = (size_t)cs * kTaps;
  net->p_stem_b = net->p_stem_g + cs;
  size_t po = net->p_stem_b + cs;
  for (int b = 0; b < 4; ++b) {
    dnb_block_desc bd{};
    bd.n = d.n; bd.c0 = c; bd.h = s; bd.w = s; bd.layers = d.layers[b]; bd.growth = k; bd.bottleneck = 4 * k;
    bd.dtype = DNB_BF16; bd.layout = DNB_NHWC; bd.schedule = d.schedule; bd.eps = d.eps;
    const int rc = dnb_block_create(&bd, &net->blk[b]);
    if (rc != DNB_OK) { dnb_inet_destroy(net); return rc; }
    net->bd[b] = bd;
    net->cout[b] = c + d.layers[b] * k;
    const size_t co = (size_t)net->cout[b];
    if (b < 3 && co % 16 != 0) { dnb_inet_destroy(net); return DNB_E_UNSUPPORTED; }  // C/2 channels in 8-channel vectors
    net->p_block[b] = po;
    po += dnb_block_param_count(net->blk[b]);
    net->p_g[b] = po; net->p_b[b] = po + co; net->p_w[b] = po + 2 * co;
    if (b < 3) {
      po += 2 * co + (co / 2) * co;
      c = (int)(co / 2);
      s /= 2;
    } else {
      net->p_bl = po + 2 * co + (size_t)d.classes * co;
      po += 2 * co + (size_t)d.classes * co + (size_t)d.classes;
    }
  }
  net->p_count = po;

  // ---- workspace plan: every shared buffer is sized for its largest user
  size_t off = 0, glue = 0;
  auto carve = [&](size_t bytes, bool feature_map) {
    const size_t o = off;
    off = align_up(off + bytes, 256);
    if (feature_map) glue += bytes;
    return o;
  };
  const size_t S2 = (size_t)d.image / 2, S4 = (size_t)d.image / 4;
  const size_t Ps = (size_t)d.n * S2 * S2;
  net->o_s = carve(Ps * cs * 2, true);
  net->o_pos = carve((size_t)d.n * S4 * S4 * cs, true);
  net->o_fold_s = carve((size_t)cs * 8, false);
  net->o_stat_s = carve((size_t)cs * 8, false);
  size_t part = nhwc::stats_partial_floats((int64_t)Ps, cs), pmax = 0, conv_max = 0, feat_max = 0;
  auto need = [&](size_t f) { if (f > part) part = f; };
  need(nhwc::bn_bwd_partial_floats((int64_t)Ps, cs));
  need((size_t)stem_wgrad_groups(d.n, d.image) * cs * kTaps);
  for (int b = 0; b < 4; ++b) {
    const dnb_block_desc& bd = net->bd[b];
    const size_t hw = (size_t)bd.h * bd.w, P = hw * d.n, co = (size_t)net->cout[b];
    net->o_feat[b] = carve((size_t)bd.c0 * P * 2, true);
    net->o_y[b] = carve(co * P * 2, true);
    net->o_ws[b] = carve(dnb_block_workspace_bytes(net->blk[b]), false);
    net->o_stat[b] = carve(co * 8, false);
    net->o_fold[b] = carve(co * 8, false);
    if (co * P > pmax) pmax = co * P;
    if ((size_t)bd.c0 * P > feat_max) feat_max = (size_t)bd.c0 * P;
    need(nhwc::stats_partial_floats((int64_t)P, (int)co));
    need(nhwc::bn_bwd_partial_floats((int64_t)P, (int)co));
    if (b < 3) {
      const size_t ch = co / 2;
      if (ch * P > conv_max) conv_max = ch * P;
      need(nhwc::conv_stats_partial_floats(d.n, (int)ch, bd.h, bd.w));
      need(nhwc::wgrad_partial_floats(d.n, (int)co, (int)ch, bd.h, bd.w, 1));
      net->o_pack[b] = carve((nhwc::packed_weight_elems((int)ch, (int)co, 1) + nhwc::packed_weight_elems((int)co, (int)ch, 1)) * 2 + 256,
                             false);
    }
  }
  net->o_tconv = carve(conv_max * 2, true);   // a transition's 1x1 output before pooling
  net->o_gy = carve(pmax * 2, true);          // gradient of a block output
  net->o_dtz = carve(pmax * 2, true);         // gradient of a transition's / the tail's BN+ReLU output
  net->o_dconv = carve(conv_max * 2, true);   // gradient of a transition's conv output
  net->o_dfeat = carve(feat_max * 2, true);   // gradient of a block input
  net->o_da0 = carve(Ps * cs * 2, true);      // gradient of the stem's BN+ReLU output, then of the stem conv's output
  net->o_part = carve(part * 4, false);
  net->o_stem_wt = carve((size_t)kTaps * cs * 4, false);
  const size_t C = (size_t)net->cout[3];
  net->o_pooled = carve((size_t)d.n * C * 4, false);
  net->o_dpooled = carve((size_t)d.n * C * 4, false);
  net->o_logits = carve((size_t)d.n * d.classes * 4, false);
  net->o_dlogits = carve((size_t)d.n * d.classes * 4, false);
  net->o_terms = carve((size_t)d.n * 4, false);
  net->ws_bytes = off;
  net->glue_feature_bytes = glue;
  *out = net;
  return DNB_OK;
}

void dnb_inet_destroy(dnb_inet* net) {
  if (!net) return;
  for (int b = 0; b < 4; ++b)
    if (net->blk[b]) dnb_block_destroy(net->blk[b]);
  delete net;
}

size_t dnb_inet_param_count(const dnb_inet* net) { return net ? net->p_count : 0; }
size_t dnb_inet_workspace_bytes(const dnb_inet* net) { return net ? net->ws_bytes : 0; }

size_t dnb_inet_peak_bytes(const dnb_inet* net) {
  if (!net) return 0;
  size_t t = net->glue_feature_bytes;
  for (int b = 0; b < 4; ++b) {
    const dnb_block_desc& bd = net->bd[b];  // the block's x_l live inside the y buffer already counted as glue
    t += dnb_block_peak_bytes(net->blk[b]) - (size_t)bd.layers * bd.growth * bd.n * bd.h * bd.w * 2;
  }
  return t;
}

int dnb_inet_param_offset(const dnb_inet* net, int part, size_t* offset, size_t* count) {
  if (!net || !offset || !count) return DNB_E_NULL;
  const dnb_inet_desc& d = net->d;
  const size_t cs = (size_t)net->cs;
  size_t o = 0, n = 0;
  if (part == DNB_IP_STEM_W) { o = net->p_stem_w; n = cs * kTaps; }
  else if (part == DNB_IP_STEM_G) { o = net->p_stem_g; n = cs; }
  else if (part == DNB_IP_STEM_B) { o = net->p_stem_b; n = cs; }
  else if (part >= DNB_IP_BLOCK0 && part < DNB_IP_BLOCK0 + 16) {
    const int b = (part - DNB_IP_BLOCK0) / 4, which = (part - DNB_IP_BLOCK0) % 4;
    const size_t co = (size_t)net->cout[b];
    if (which == 0) { o = net->p_block[b]; n = dnb_block_param_count(net->blk[b]); }
    else if (which == 1) { o = net->p_g[b]; n = co; }
    else if (which == 2) { o = net->p_b[b]; n = co; }
    else { o = net->p_w[b]; n = b < 3 ? (co / 2) * co : (size_t)d.classes * co; }
  } else if (part == DNB_IP_TAIL_BL) { o = net->p_bl; n = (size_t)d.classes; }
  else return DNB_E_RANGE;
  *offset = o;
  *count = n;
  return DNB_OK;
}

int dnb_inet_set_concurrency(dnb_inet* net, int enable) {
  if (!net) return DNB_E_NULL;
  for (int b = 0; b < 4; ++b) DNB_TRYS(dnb_block_set_concurrency(net->blk[b], enable));
  return DNB_OK;
}

int dnb_inet_forward(dnb_inet* net, const void* xv, const int32_t* labels, const void* paramsv, float* loss,
                     float* logits_out, void* wsv, void* stream) {
  if (!net || !xv || !labels || !paramsv || !loss || !wsv) return DNB_E_NULL;
  if ((reinterpret_cast<uintptr_t>(xv) & 1u) || (reinterpret_cast<uintptr_t>(paramsv) & 3u) || misaligned(wsv)) return DNB_E_ALIGN;
  hipStream_t st = (hipStream_t)stream;
  const dnb_inet_desc& d = net->d;
  const u16* x = (const u16*)xv;
  const float* params = (const float*)paramsv;
  char* ws = (char*)wsv;
  const int n = d.n, S = d.image, S2 = S / 2, cs = net->cs;
  const int64_t Ps = (int64_t)n * S2 * S2;
  float* part = (float*)(ws + net->o_part);
  // stem: conv, batch statistics, BN+ReLU and max pool in one pass
  u16* s = (u16*)(ws + net->o_s);
  float* mean_s = (float*)(ws + net->o_stat_s);
  float2* fold_s = (float2*)(ws + net->o_fold_s);
  DNB_TRYH(launch_stem_conv(x, params + net->p_stem_w, (float*)(ws + net->o_stem_wt), s, n, S, cs, st));
  int T = 0;
  DNB_TRYH(nhwc::stats_partial(s, cs, Ps, cs, part, &T, st));
  DNB_TRYH(launch_bn_fold(params + net->p_stem_g, params + net->p_stem_b, mean_s, mean_s + cs, part, T, 0, cs, d.eps, cs,
                          fold_s, st));
  hipLaunchKernelGGL(k_maxpool_bnrelu, dim3(grid_for((int64_t)n * (S2 / 2) * (S2 / 2) * (cs / 8), 256)), dim3(256), 0, st, s,
                     fold_s, (u16*)(ws + net->o_feat[0]), (unsigned char*)(ws + net->o_pos), n, S2, S2, cs);
  DNB_TRYH(hipGetLastError());
  for (int b = 0; b < 4; ++b) {
    const dnb_block_desc& bd = net->bd[b];
    const int hw = bd.h * bd.w, co = net->cout[b];
    const int64_t P = (int64_t)n * hw;
    u16* feat = (u16*)(ws + net->o_feat[b]);
    u16* y = (u16*)(ws + net->o_y[b]);
    float* mean = (float*)(ws + net->o_stat[b]);
    float2* fold = (float2*)(ws + net->o_fold[b]);
    DNB_TRYS(dnb_block_forward(net->blk[b], feat, params + net->p_block[b], y, ws + net->o_ws[b], stream));
    // BN of the block output: statistics, folded (scale, shift); the BN+ReLU itself is applied by its consumer
    DNB_TRYH(nhwc::stats_partial(y, co, P, co, part, &T, st));
    DNB_TRYH(launch_bn_fold(params + net->p_g[b], params + net->p_b[b], mean, mean + co, part, T, 0, co, d.eps, co, fold, st));
    if (b < 3) {
      const int ch = co / 2;
      const float* W = params + net->p_w[b];
      u16* pk = (u16*)(ws + net->o_pack[b]);
      u16* pkt = pk + ((nhwc::packed_weight_elems(ch, co, 1) + 7) & ~(size_t)7);
      u16* tconv = (u16*)(ws + net->o_tconv);
      DNB_TRYH(nhwc::pack_weights(WeightView{W, co, 1, 0}, ch, co, 1, pk, st));
      DNB_TRYH(nhwc::pack_weights(WeightView{W, 1, co, 0}, co, ch, 1, pkt, st));  // for the data gradient
      int Tc = 0;
      DNB_TRYH(nhwc::conv(y, co, false, pk, tconv, ch, n, co, ch, bd.h, bd.w, 1, fold, part, &Tc, st));
      hipLaunchKernelGGL(k_avgpool2_rows, dim3(grid_for((int64_t)n * (hw / 4) * (ch / 8), 256)), dim3(256), 0, st, tconv,
                         (u16*)(ws + net->o_feat[b + 1]), n, bd.h, bd.w, ch);
      DNB_TRYH(hipGetLastError());
    } else {
      float* pooled = (float*)(ws + net->o_pooled);
      float* logits = (float*)(ws + net->o_logits);
      hipLaunchKernelGGL(k_global_avgpool_bnrelu, dim3(grid_for((int64_t)n * (co / 8), 256)), dim3(256), 0, st, y, fold, pooled,
                         n, hw, co);
      DNB_TRYH(hipGetLastError());
      DNB_TRYH(launch_head_forward(pooled, params + net->p_w[3], params + net->p_bl, labels, logits,
                                   (float*)(ws + net->o_dlogits), (float*)(ws + net->o_terms), loss, n, co, d.classes, st));
      if (logits_out)
        DNB_TRYH(launch_copy_slab(logits, (int64_t)n * d.classes, logits_out, (int64_t)n * d.classes, 1,
                                  (int64_t)n * d.classes, st));
    }
  }
  return DNB_OK;
}

int dnb_inet_backward(dnb_inet* net, const void* xv, const void* paramsv, void* dparamsv, void* wsv, void* stream) {
  if (!net || !xv || !paramsv || !dparamsv || !wsv) return DNB_E_NULL;
  if ((reinterpret_cast<uintptr_t>(xv) & 1u) || (reinterpret_cast<uintptr_t>(paramsv) & 3u) ||
      (reinterpret_cast<uintptr_t>(dparamsv) & 3u) || misaligned(wsv))
    return DNB_E_ALIGN;
  hipStream_t st = (hipStream_t)stream;
  const dnb_inet_desc& d = net->d;
  const u16* x = (const u16*)xv;
  const float* params = (const float*)paramsv;
  float* dparams = (float*)dparamsv;
  char* ws = (char*)wsv;
  const int n = d.n, S = d.image, S2 = S / 2, cs = net->cs;
  const int64_t Ps = (int64_t)n * S2 * S2;
  float* part = (float*)(ws + net->o_part);
  u16* gy = (u16*)(ws + net->o_gy);
  u16* dtz = (u16*)(ws + net->o_dtz);
  u16* dconv = (u16*)(ws + net->o_dconv);
  u16* dfeat = (u16*)(ws + net->o_dfeat);
  {  // head: linear backward, global average pool backward
    const int C = net->cout[3], hw = net->bd[3].h * net->bd[3].w;
    float* dpooled = (float*)(ws + net->o_dpooled);
    DNB_TRYH(launch_head_backward((const float*)(ws + net->o_dlogits), (const float*)(ws + net->o_pooled), params + net->p_w[3],
                                  dpooled, dparams + net->p_w[3], dparams + net->p_bl, n, C, d.classes, st));
    hipLaunchKernelGGL(k_global_avgpool_rows_bwd, dim3(grid_for((int64_t)n * hw * (C / 8), 256)), dim3(256), 0, st, dpooled, dtz,
                       n, hw, C);
    DNB_TRYH(hipGetLastError());
  }
  for (int b = 3; b >= 0; --b) {
    const dnb_block_desc& bd = net->bd[b];
    const int hw = bd.h * bd.w, co = net->cout[b];
    const int64_t P = (int64_t)n * hw;
    const u16* y = (const u16*)(ws + net->o_y[b]);
    const float* mean = (const float*)(ws + net->o_stat[b]);
    // BN+ReLU backward of the transition / tail: gradient of the block output
    DNB_TRYH(nhwc::bn_relu_bwd(y, co, dtz, co, gy, co, nullptr, 0, P, co, params + net->p_g[b], params + net->p_b[b], mean,
                               mean + co, dparams + net->p_g[b], dparams + net->p_b[b], part, st));
    DNB_TRYS(dnb_block_backward(net->blk[b], params + net->p_block[b], y, gy, dfeat, dparams + net->p_block[b],
                                ws + net->o_ws[b], stream));
    if (b > 0) {
      // through transition b-1: pool backward, then the 1x1 conv's weight and data gradients
      const dnb_block_desc& pd = net->bd[b - 1];
      const int hwp = pd.h * pd.w, cp = net->cout[b - 1], ch = cp / 2;
      const u16* yp = (const u16*)(ws + net->o_y[b - 1]);
      const float2* foldp = (const float2*)(ws + net->o_fold[b - 1]);
      const u16* pkt = (const u16*)(ws + net->o_pack[b - 1]) + ((nhwc::packed_weight_elems(ch, cp, 1) + 7) & ~(size_t)7);
      hipLaunchKernelGGL(k_avgpool2_rows_bwd, dim3(grid_for((int64_t)n * hwp * (ch / 8), 256)), dim3(256), 0, st, dfeat, dconv,
                         n, pd.h, pd.w, ch);
      DNB_TRYH(hipGetLastError());
      DNB_TRYH(nhwc::wgrad(yp, cp, dconv, ch, false, part, dparams + net->p_w[b - 1], n, cp, ch, pd.h, pd.w, 1, foldp, st));
      DNB_TRYH(nhwc::conv(dconv, ch, false, pkt, dtz, cp, n, ch, cp, pd.h, pd.w, 1, nullptr, nullptr, nullptr, st));
    } else {
      // through the stem: pool backward to the maxima's positions, BN+ReLU backward, weight gradient
      u16* da0 = (u16*)(ws + net->o_da0);
      const u16* s = (const u16*)(ws + net->o_s);
      const float* mean_s = (const float*)(ws + net->o_stat_s);
      hipLaunchKernelGGL(k_maxpool_bwd, dim3(grid_for(Ps * (cs / 8), 256)), dim3(256), 0, st, dfeat,
                         (const unsigned char*)(ws + net->o_pos), da0, n, S2, S2, cs);
      DNB_TRYH(hipGetLastError());
      DNB_TRYH(nhwc::bn_relu_bwd(s, cs, da0, cs, da0, cs, nullptr, 0, Ps, cs, params + net->p_stem_g, params + net->p_stem_b,
                                 mean_s, mean_s + cs, dparams + net->p_stem_g, dparams + net->p_stem_b, part, st));
      DNB_TRYH(launch_stem_wgrad(x, da0, part, dparams + net->p_stem_w, n, S, cs, st));
    }
  }
  return DNB_OK;
}

size_t dnb_inet_relu_decision_bytes(const dnb_inet* net) {
  if (!net) return 0;
  const size_t S2 = (size_t)net->d.image / 2;
  size_t t = (size_t)net->d.n * S2 * S2 * net->cs;
  for (int b = 0; b < 4; ++b) {
    const dnb_block_desc& bd = net->bd[b];
    t += dnb_block_relu_decision_bytes(net->blk[b], 1) + dnb_block_relu_decision_bytes(net->blk[b], 2) +
         (size_t)net->cout[b] * bd.n * bd.h * bd.w;
  }
  return t;
}

size_t dnb_inet_pool_position_bytes(const dnb_inet* net) {
  if (!net) return 0;
  const size_t S4 = (size_t)net->d.image / 4;
  return (size_t)net->d.n * S4 * S4 * net->cs;
}

int dnb_inet_decisions(dnb_inet* net, const void* paramsv, const void* wsv, void* reluv, void* poolv, void* stream) {
  if (!net || !paramsv || !wsv || !reluv || !poolv) return DNB_E_NULL;
  hipStream_t st = (hipStream_t)stream;
  const float* params = (const float*)paramsv;
  const char* ws = (const char*)wsv;
  unsigned char* out = (unsigned char*)reluv;
  const int n = net->d.n, S2 = net->d.image / 2, cs = net->cs;
  const int64_t Ps = (int64_t)n * S2 * S2;
  const float* mean_s = (const float*)(ws + net->o_stat_s);
  DNB_TRYH(launch_relu_decisions_rows(ws + net->o_s, cs, Ps, cs, params + net->p_stem_g, params + net->p_stem_b, mean_s,
                                      mean_s + cs, out, st));
  out += Ps * cs;
  for (int b = 0; b < 4; ++b) {
    const dnb_block_desc& bd = net->bd[b];
    const int co = net->cout[b];
    const int64_t P = (int64_t)n * bd.h * bd.w;
    const size_t n1 = dnb_block_relu_decision_bytes(net->blk[b], 1), n2 = dnb_block_relu_decision_bytes(net->blk[b], 2);
    const void* y = ws + net->o_y[b];
    DNB_TRYS(dnb_block_relu_decisions(net->blk[b], params + net->p_block[b], y, ws + net->o_ws[b], out, out + n1, stream));
    out += n1 + n2;
    const float* mean = (const float*)(ws + net->o_stat[b]);
    DNB_TRYH(launch_relu_decisions_rows(y, co, P, co, params + net->p_g[b], params + net->p_b[b], mean, mean + co, out, st));
    out += (size_t)co * P;
  }
  DNB_TRYH(hipMemcpyAsync(poolv, ws + net->o_pos, dnb_inet_pool_position_bytes(net), hipMemcpyDeviceToDevice, st));
  return DNB_OK;
}

// ---- the glue kernels as single operations

static int stem_shape_ok(int64_t n, int64_t image, int64_t channels) {
  if (n < 1 || image < 32 || image % 32 != 0) return DNB_E_BADDESC;
  if (n > 4096 || image > 1024) return DNB_E_RANGE;
  if (channels != 16 && channels != 32 && channels != 64 && channels != 96) return DNB_E_UNSUPPORTED;
  return DNB_OK;
}

size_t dnb_op_stem_scratch_bytes(int64_t n, int64_t image, int64_t channels) {
  if (stem_shape_ok(n, image, channels) != DNB_OK) return 0;
  const size_t wt = (size_t)kTaps * channels * 4;
  const size_t part = (size_t)stem_wgrad_groups((int)n, (int)image) * channels * kTaps * 4;
  return wt > part ? wt : part;
}

int dnb_op_stem_conv7(const void* x, const void* w, void* out, int64_t n, int64_t image, int64_t channels, void* scratch,
                      void* stream) {
  if (!x || !w || !out || !scratch) return DNB_E_NULL;
  const int rc = stem_shape_ok(n, image, channels);
  if (rc != DNB_OK) return rc;
  if ((reinterpret_cast<uintptr_t>(x) & 1u) || (reinterpret_cast<uintptr_t>(w) & 3u) || misaligned(out) || misaligned(scratch))
    return DNB_E_ALIGN;
  DNB_TRYH(launch_stem_conv((const u16*)x, (const float*)w, (float*)scratch, (u16*)out, (int)n, (int)image, (int)channels,
                            (hipStream_t)stream));
  return DNB_OK;
}

int dnb_op_stem_wgrad7(const void* x, const void* g, void* dw, int64_t n, int64_t image, int64_t channels, void* scratch,
                       void* stream) {
  if (!x || !g || !dw || !scratch) return DNB_E_NULL;
  const int rc = stem_shape_ok(n, image, channels);
  if (rc != DNB_OK) return rc;
  if ((reinterpret_cast<uintptr_t>(x) & 1u) || misaligned(g) || (reinterpret_cast<uintptr_t>(dw) & 3u) || misaligned(scratch))
    return DNB_E_ALIGN;
  DNB_TRYH(launch_stem_wgrad((const u16*)x, (const u16*)g, (float*)scratch, (float*)dw, (int)n, (int)image, (int)channels,
                             (hipStream_t)stream));
  return DNB_OK;
}

static int pool_shape_ok(int64_t n, int64_t h, int64_t w, int64_t c) {
  if (n < 1 || h < 2 || w < 2 || c < 8 || h % 2 || w % 2 || c % 8) return DNB_E_BADDESC;
  if (n > 4096 || h > 4096 || w > 4096 || c > 65536) return DNB_E_RANGE;
  return DNB_OK;
}

int dnb_op_maxpool3s2_bnrelu(const void* s, const void* fold, void* out, void* pos, int64_t n, int64_t h, int64_t w,
                             int64_t c, void* stream) {
  if (!s || !fold || !out || !pos) return DNB_E_NULL;
  const int rc = pool_shape_ok(n, h, w, c);
  if (rc != DNB_OK) return rc;
  if (misaligned(s) || (reinterpret_cast<uintptr_t>(fold) & 7u) || misaligned(out) || (reinterpret_cast<uintptr_t>(pos) & 7u))
    return DNB_E_ALIGN;
  hipLaunchKernelGGL(k_maxpool_bnrelu, dim3(grid_for(n * (h / 2) * (w / 2) * (c / 8), 256)), dim3(256), 0, (hipStream_t)stream,
                     (const u16*)s, (const float2*)fold, (u16*)out, (unsigned char*)pos, (int)n, (int)h, (int)w, (int)c);
  DNB_TRYH(hipGetLastError());
  return DNB_OK;
}

int dnb_op_maxpool3s2_backward(const void* dout, const void* pos, void* din, int64_t n, int64_t h, int64_t w, int64_t c,
                               void* stream) {
  if (!dout || !pos || !din) return DNB_E_NULL;
  const int rc = pool_shape_ok(n, h, w, c);
  if (rc != DNB_OK) return rc;
  if (misaligned(dout) || (reinterpret_cast<uintptr_t>(pos) & 7u) || misaligned(din)) return DNB_E_ALIGN;
  hipLaunchKernelGGL(k_maxpool_bwd, dim3(grid_for(n * h * w * (c / 8), 256)), dim3(256), 0, (hipStream_t)stream,
                     (const u16*)dout, (const unsigned char*)pos, (u16*)din, (int)n, (int)h, (int)w, (int)c);
  DNB_TRYH(hipGetLastError());
  return DNB_OK;
}

}  // extern "C"
