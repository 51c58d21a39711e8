// bf16 / NHWC kernels of the dense block (feature maps stored as bf16, channels contiguous;
// fp32 accumulation, fp32 BN statistics, fp32 parameters and parameter gradients, fp32 gradient
// slab).  Every step of the fused schedule, built around v_mfma_f32_16x16x32_bf16 with output
// channels on M and pixels on N, so a lane's operand is 8 consecutive channels of one pixel
// (16 bytes of NHWC) and an accumulator holds 4 consecutive channels of one pixel (one 8-byte
// NHWC store).
//
// Convolutions (forward / data gradient): the workgroup stages a 64-pixel tile (+ one image row
// of halo for 3x3) of a 64-channel chunk in LDS, double-buffered, applying the BN+ReLU prologue
// once per element; its four waves split the output-channel tiles and take packed bf16 weights
// from L2 through register rings.  Weight gradients contract over pixels, which NHWC keeps on
// the slow axis, so both operands are transposed on their way into LDS ([channel][pixel]); the
// 3x3 stages a row tile once and reads its nine taps as shifted fragments.
#include "dnb_internal.h"
#include "dnb_stats.h"

namespace dnb {
namespace nhwc {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned short u16;

__device__ __forceinline__ float bf2f(u16 v) { return __uint_as_float((unsigned)v << 16); }
// round to nearest even (the hardware conversion of gfx950)
__device__ __forceinline__ u16 f2bf(float f) {
  const __bf16 b = (__bf16)f;
  return __builtin_bit_cast(u16, b);
}

union V8 {          // 8 bf16 = 16 bytes
  uint4 q;
  u16 h[8];
  bf16x8 v;
};

__device__ __forceinline__ f32x4 mfma_bf16(const V8& a, const V8& b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, b.v, c, 0, 0, 0);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// ----------------------------------------------------------------------------- small kernels

// dst[p][0:c] = src[p][0:c] (bf16, c % 8 == 0), pixel strides in elements
__global__ __launch_bounds__(256) void k_copy_rows(const u16* __restrict__ src, int64_t sld,
                                                   u16* __restrict__ dst, int64_t dld, int64_t P, int cv) {
  const int64_t total = P * cv;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int64_t p = i / cv;
    const int v = (int)(i - p * cv);
    *reinterpret_cast<uint4*>(dst + p * dld + 8 * v) = *reinterpret_cast<const uint4*>(src + p * sld + 8 * v);
  }
}

// out[p][0:c] = bf16(max(0, fma(x[p][ch], scale_ch, shift_ch))) with (scale, shift) = fold[ch]: BN+ReLU
// into shared storage 2 exactly as the fused schedule's convolutions apply it in their operand
// loads; copy (may be null) receives the raw features (the concatenation into shared storage 1).
__global__ __launch_bounds__(256) void k_bn_relu_rows(const u16* __restrict__ x, int64_t ld,
                                                      const float2* __restrict__ fold, u16* __restrict__ out,
                                                      int64_t old, u16* __restrict__ copy, int64_t cld, int64_t P,
                                                      int cv) {
  const int64_t total = P * cv;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int64_t p = i / cv;
    const int v = (int)(i - p * cv);
    V8 r, o;
    r.q = *reinterpret_cast<const uint4*>(x + p * ld + 8 * v);
    const float4* f4 = reinterpret_cast<const float4*>(fold + 8 * v);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float4 f = f4[e];  // two channels' (scale, shift)
      o.h[2 * e] = f2bf(fmaxf(__fmaf_rn(bf2f(r.h[2 * e]), f.x, f.y), 0.f));
      o.h[2 * e + 1] = f2bf(fmaxf(__fmaf_rn(bf2f(r.h[2 * e + 1]), f.z, f.w), 0.f));
    }
    *reinterpret_cast<uint4*>(out + p * old + 8 * v) = o.q;
    if (copy) *reinterpret_cast<uint4*>(copy + p * cld + 8 * v) = r.q;
  }
}

// G (fp32, [P][c]) = dy (bf16, [P][c])
__global__ __launch_bounds__(256) void k_bf16_to_f32(const u16* __restrict__ src, float* __restrict__ dst,
                                                     int64_t total8) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total8; i += (int64_t)gridDim.x * 256) {
    V8 s;
    s.q = *reinterpret_cast<const uint4*>(src + 8 * i);
    float4 a = make_float4(bf2f(s.h[0]), bf2f(s.h[1]), bf2f(s.h[2]), bf2f(s.h[3]));
    float4 b = make_float4(bf2f(s.h[4]), bf2f(s.h[5]), bf2f(s.h[6]), bf2f(s.h[7]));
    *reinterpret_cast<float4*>(dst + 8 * i) = a;
    *reinterpret_cast<float4*>(dst + 8 * i + 4) = b;
  }
}

// dst (bf16, [P][c]) = src (fp32, [P][ld]) first c channels
__global__ __launch_bounds__(256) void k_f32_rows_to_bf16(const float* __restrict__ src, int64_t sld,
                                                          u16* __restrict__ dst, int64_t P, int cv) {
  const int64_t total = P * cv;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int64_t p = i / cv;
    const int v = (int)(i - p * cv);
    const float4 a = *reinterpret_cast<const float4*>(src + p * sld + 8 * v);
    const float4 b = *reinterpret_cast<const float4*>(src + p * sld + 8 * v + 4);
    V8 o;
    o.h[0] = f2bf(a.x); o.h[1] = f2bf(a.y); o.h[2] = f2bf(a.z); o.h[3] = f2bf(a.w);
    o.h[4] = f2bf(b.x); o.h[5] = f2bf(b.y); o.h[6] = f2bf(b.z); o.h[7] = f2bf(b.w);
    *reinterpret_cast<uint4*>(dst + p * (int64_t)(8 * cv) + 8 * v) = o.q;
  }
}

// Statistics partials of c channels over pixel range split s: part[(ch*S + s)*3] = (count, mean, M2).
// Thread = (8-channel vector, pixel row): 32 vectors x 8 rows per workgroup, 16-byte loads.  Each
// thread sums deviations from its first value (no cancellation for |mean| >> std), converts to
// (count, mean, M2) and the 8 rows are combined in row order.  grid (vector groups, splits).
__global__ __launch_bounds__(256) void k_stats_partial(const u16* __restrict__ x, int64_t ld, int64_t P,
                                                       int c, int ppb, float* __restrict__ part) {
  __shared__ float red[3][8][256];
  const int cvl = threadIdx.x & 31, pr = threadIdx.x >> 5;
  const int ch0 = (blockIdx.x * 32 + cvl) * 8, s = blockIdx.y, S = gridDim.y;
  const int64_t p0 = (int64_t)s * ppb, p1 = min(P, p0 + ppb);
  const bool ok = ch0 < c;
  float K[8], sd[8], sq[8];
  float cnt = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) K[e] = sd[e] = sq[e] = 0.f;
  if (ok) {
    int64_t p = p0 + pr;
    if (p < p1) {
      V8 v;
      v.q = *reinterpret_cast<const uint4*>(x + p * ld + ch0);
#pragma unroll
      for (int e = 0; e < 8; ++e) K[e] = bf2f(v.h[e]);
      cnt = 1.f;
      p += 8;
    }
    for (; p < p1; p += 8) {
      V8 v;
      v.q = *reinterpret_cast<const uint4*>(x + p * ld + ch0);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float d = bf2f(v.h[e]) - K[e];
        sd[e] += d;
        sq[e] = __fmaf_rn(d, d, sq[e]);
      }
      cnt += 1.f;
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const float md = cnt > 0.f ? sd[e] / cnt : 0.f;
    red[0][e][threadIdx.x] = cnt;
    red[1][e][threadIdx.x] = K[e] + md;
    red[2][e][threadIdx.x] = fmaxf(0.f, __fmaf_rn(-sd[e], md, sq[e]));
  }
  __syncthreads();
  if (pr == 0 && ok) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      Stat3 a{red[0][e][cvl], red[1][e][cvl], red[2][e][cvl]};
      for (int r = 1; r < 8; ++r)
        a = stat_combine(a, Stat3{red[0][e][r * 32 + cvl], red[1][e][r * 32 + cvl], red[2][e][r * 32 + cvl]});
      float* o = part + ((int64_t)(ch0 + e) * S + s) * 3;
      o[0] = a.c; o[1] = a.m; o[2] = a.m2;
    }
  }
}

// Packed bf16 weights: [taps][M16][K32] (K padded to a multiple of 32, zero filled), K natural order.
__global__ __launch_bounds__(256) void k_pack_block_weights(const float* __restrict__ params,
                                                            u16* __restrict__ packed, int c0, int k, int B) {
  const int l = blockIdx.y + 1;
  const int B16 = (B + 15) & ~15, k16 = (k + 15) & ~15, B32 = (B + 31) & ~31, k32 = (k + 31) & ~31;
  int64_t poff = 0, koff = 0;
  for (int i = 1; i < l; ++i) {
    const int c = c0 + (i - 1) * k, c16 = (c + 15) & ~15, c32 = (c + 31) & ~31;
    poff += 2 * (int64_t)c + (int64_t)B * c + 2 * B + 9 * (int64_t)k * B;
    koff += (int64_t)B16 * c32 + (int64_t)c16 * B32 + 9 * (int64_t)k16 * B32 + 9 * (int64_t)B16 * k32;
  }
  const int C = c0 + (l - 1) * k, C16 = (C + 15) & ~15, C32 = (C + 31) & ~31;
  const float* W1 = params + poff + 2 * C;
  const float* W3 = W1 + (int64_t)B * C + 2 * B;
  u16* A = packed + koff;
  const int64_t n1 = (int64_t)B16 * C32, n2 = (int64_t)C16 * B32, n3 = 9 * (int64_t)k16 * B32,
                n4 = 9 * (int64_t)B16 * k32, total = n1 + n2 + n3 + n4;
  for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * 256) {
    float v = 0.f;
    if (idx < n1) {                       // 1x1 forward  [B16][C32]
      const int m = (int)(idx / C32), c = (int)(idx % C32);
      if (m < B && c < C) v = W1[(int64_t)m * C + c];
    } else if (idx < n1 + n2) {           // 1x1 dgrad    [C16][B32]
      const int64_t e = idx - n1;
      const int cc = (int)(e / B32), o = (int)(e % B32);
      if (cc < C && o < B) v = W1[(int64_t)o * C + cc];
    } else if (idx < n1 + n2 + n3) {      // 3x3 forward  [9][k16][B32]
      const int64_t e = idx - n1 - n2;
      const int t = (int)(e / (k16 * B32)), rem = (int)(e % (k16 * B32));
      const int mm = rem / B32, c = rem % B32;
      if (mm < k && c < B) v = W3[((int64_t)mm * B + c) * 9 + t];
    } else {                              // 3x3 dgrad    [9][B16][k32], transposed and flipped
      const int64_t e = idx - n1 - n2 - n3;
      const int t = (int)(e / (B16 * k32)), rem = (int)(e % (B16 * k32));
      const int cc = rem / k32, o = rem % k32;
      if (cc < B && o < k) v = W3[((int64_t)o * B + cc) * 9 + (8 - t)];
    }
    A[idx] = f2bf(v);
  }
}

// One convolution's weights: [taps][M16][K32] from element (m, c, t) at w[m*sm + c*sc + (flip ? taps-1-t : t)].
__global__ __launch_bounds__(256) void k_pack_weights(const float* __restrict__ w, int64_t sm, int64_t sc, int flip,
                                                      int cout, int cin, int taps, u16* __restrict__ outp) {
  const int M16 = (cout + 15) & ~15, K32 = (cin + 31) & ~31;
  const int64_t total = (int64_t)taps * M16 * K32;
  for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * 256) {
    const int c = (int)(idx % K32);
    const int64_t rem = idx / K32;
    const int m = (int)(rem % M16), t = (int)(rem / M16);
    const float v = (m < cout && c < cin) ? w[(int64_t)m * sm + (int64_t)c * sc + (flip ? taps - 1 - t : t)] : 0.f;
    outp[idx] = f2bf(v);
  }
}

// ----------------------------------------------------------------------------- conv fwd / dgrad

// out[q][m] = sum_{t,c} W(t,m,c) * act(in[q+shift(t)][c]),  act = BN+ReLU prologue or identity.
// 256 threads; a workgroup owns 64 pixels -- for the 1x1 a flat range of all n*h*w pixels (grid.x
// tiles, grid.z = 1), for the 3x3 a range of one image (grid.z = images) plus one image row and
// one pixel of halo on both sides -- and the four waves split the output channels (MT M-tiles
// each).  Input channels are walked in chunks of 64 through two LDS buffers: the next chunk is
// requested from HBM before the current chunk's MFMAs are issued and written to the other
// buffer (BN+ReLU applied, rounded to bf16) after them: one barrier per chunk, load latency
// under the matrix work.  TIN = u16 (bf16) or float (the gradient slab).  STATS: per-tile
// (count, mean, M2) of the rounded outputs, as in the fp32 kernels: spart[(m*T + tile)*3].
template <int TAPS, int MT, typename TIN, bool PRO, bool STATS, bool RING>
__global__ __launch_bounds__(256) void k_conv(
    const TIN* __restrict__ in, int64_t in_ld, const u16* __restrict__ Wp, int M16, int K32,
    u16* __restrict__ out, int64_t out_ld, int cin, int cout, int H, int W, int64_t Ptot,
    const float2* __restrict__ fold, float* __restrict__ spart, int sT) {
  extern __shared__ u16 lds[];
  constexpr int KC = 64, PITCH = KC + 8;  // elements per staged pixel (144 bytes: spreads banks)
  constexpr int U = TAPS == 9 ? 8 : 2;    // 16-byte vectors per thread and chunk (3x3: W <= 95)
  const int HW = H * W;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j = lane & 15, g = lane >> 4;
  const int img = TAPS == 9 ? blockIdx.z : 0;
  const int64_t q0 = (int64_t)blockIdx.x * 64;
  const int64_t limit = TAPS == 9 ? (int64_t)HW : Ptot;  // pixels of the range q0 indexes
  const int halo = (TAPS == 9) ? W + 1 : 0;
  const int seg = 64 + 2 * halo, nvec = seg * 8, BUFE = seg * PITCH;
  const TIN* inb = in + (int64_t)img * HW * in_ld;
  const int mbase = (blockIdx.y * 4 + wave) * (MT * 16);
  const bool m_ok = mbase < M16;

  f32x4 acc[MT][4];
#pragma unroll
  for (int a = 0; a < MT; ++a)
#pragma unroll
    for (int t = 0; t < 4; ++t) acc[a][t] = (f32x4){0.f, 0.f, 0.f, 0.f};

  bool lok[4], rok[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int wc = (int)((q0 + t * 16 + j) % W);
    lok[t] = wc != 0;
    rok[t] = wc != W - 1;
  }

  // PRO: the folded BN (scale, shift) of all input channels is copied to LDS once, behind the two
  // tile buffers (the staging reads it for every vector it transforms)
  float* flds = reinterpret_cast<float*>(lds + 2 * BUFE);  // 2*BUFE*2 bytes is a multiple of 16
  if (PRO) {
    for (int i = tid; i < cin; i += 256) {
      const float2 fl = fold[i];
      flds[2 * i] = fl.x; flds[2 * i + 1] = fl.y;
    }
    __syncthreads();
  }

  struct Raw { uint4 a, b; };  // bf16: a only; float: 8 floats
  // Every load of the main loop is unconditional, at an address clamped into the tensor: the
  // number of loads in flight at each point is then the same on every path, and a use waits only
  // for its own load instead of for all of them.
  auto request = [&](int c0, Raw(&v)[U]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int idx = min(u * 256 + tid, nvec - 1);
      const int s = idx >> 3, ch = min(c0 + 8 * (idx & 7), cin - 8);  // cin % 8 == 0
      const int64_t q = min(max(q0 - halo + s, (int64_t)0), limit - 1);
      if (sizeof(TIN) == 2) {
        v[u].a = *reinterpret_cast<const uint4*>(reinterpret_cast<const u16*>(inb) + q * in_ld + ch);
      } else {
        const float* pf = reinterpret_cast<const float*>(inb) + q * in_ld + ch;
        v[u].a = *reinterpret_cast<const uint4*>(pf);
        v[u].b = *reinterpret_cast<const uint4*>(pf + 4);
      }
    }
  };
  auto deposit = [&](int c0, const Raw(&v)[U], int boff) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int idx = u * 256 + tid;
      if (idx < nvec) {
        const int s = idx >> 3, vv = idx & 7, ch = c0 + 8 * vv;
        const int64_t q = q0 - halo + s;
        V8 o;
        o.q = make_uint4(0u, 0u, 0u, 0u);
        if (q >= 0 && q < limit && ch < cin) {  // a vector is entirely in or out
          float f[8];
          if (sizeof(TIN) == 2) {
            V8 r;
            r.q = v[u].a;
#pragma unroll
            for (int e = 0; e < 8; ++e) f[e] = bf2f(r.h[e]);
          } else {
            f[0] = __uint_as_float(v[u].a.x); f[1] = __uint_as_float(v[u].a.y);
            f[2] = __uint_as_float(v[u].a.z); f[3] = __uint_as_float(v[u].a.w);
            f[4] = __uint_as_float(v[u].b.x); f[5] = __uint_as_float(v[u].b.y);
            f[6] = __uint_as_float(v[u].b.z); f[7] = __uint_as_float(v[u].b.w);
          }
          if (PRO) {
#pragma unroll
            for (int e = 0; e < 8; e += 2) {  // (scale, shift) pairs from their LDS copy, 16 bytes at a time
              const float4 fl = *reinterpret_cast<const float4*>(&flds[2 * (ch + e)]);
              f[e] = fmaxf(__fmaf_rn(f[e], fl.x, fl.y), 0.f);
              f[e + 1] = fmaxf(__fmaf_rn(f[e + 1], fl.z, fl.w), 0.f);
            }
          }
#pragma unroll
          for (int e = 0; e < 8; ++e) o.h[e] = f2bf(f[e]);
        }
        *reinterpret_cast<uint4*>(&lds[boff + s * PITCH + 8 * vv]) = o.q;
      }
    }
  };

  // packed weights of one (chunk, tap): MT M-tiles x 2 K-steps, 16 bytes per lane each.  They
  // come from L2 at best and, early in a launch, from HBM, so they are requested several steps
  // before their use, into a ring of register sets indexed statically: the 1x1 keeps four chunks
  // in flight (chunk loop unrolled by four), the 3x3 nine taps (MT == 1) or three.  Rows past M16
  // and K-steps past K32 are clamped: their products are never formed or never stored.
  struct WSet { uint4 w[MT][2]; };
  auto wload = [&](int c0, int t9, WSet& ws) {
#pragma unroll
    for (int a = 0; a < MT; ++a)
#pragma unroll
      for (int kk = 0; kk < 2; ++kk)
        ws.w[a][kk] = *reinterpret_cast<const uint4*>(Wp + ((int64_t)t9 * M16 + min(mbase + a * 16 + j, M16 - 1)) * K32 +
                                                      min(c0 + kk * 32, K32 - 32) + 8 * g);
  };
  // the MFMAs of one (chunk, tap) on the tile staged at boff
  auto mm = [&](int c0, int t9, int boff, const WSet& ws) {
    const int di = (TAPS == 9) ? t9 / 3 - 1 : 0, dj = (TAPS == 9) ? t9 % 3 - 1 : 0;
    const int ksteps = min(2, (K32 - c0) >> 5);
    if (m_ok) {
#pragma unroll
      for (int kk = 0; kk < 2; ++kk) {
        if (kk < ksteps) {
          V8 bfrag[4];
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            bfrag[t].q = *reinterpret_cast<const uint4*>(
                &lds[boff + (t * 16 + j + halo + di * W + dj) * PITCH + kk * 32 + 8 * g]);
            if ((dj < 0 && !lok[t]) || (dj > 0 && !rok[t])) bfrag[t].q = make_uint4(0u, 0u, 0u, 0u);
          }
#pragma unroll
          for (int a = 0; a < MT; ++a) {
            V8 w;
            w.q = ws.w[a][kk];
#pragma unroll
            for (int t = 0; t < 4; ++t) acc[a][t] = mfma_bf16(w, bfrag[t], acc[a][t]);
          }
        }
      }
    }
  };

  const int clast = ((cin - 1) / KC) * KC;  // start of the last chunk
  if (RING) {  // 1x1 with many chunks
    // chunk x lives in ring slot x % 4 (activations and weights alike): step s multiplies chunk
    // c, requests chunk c+4 into the slots it has just freed and deposits chunk c+1
    Raw r[4][U];
    WSet wt[4];
    request(0, r[0]);
    wload(0, 0, wt[0]);
#pragma unroll
    for (int x = 1; x < 4; ++x) {
      wload(min(x * KC, clast), 0, wt[x]);
      request(min(x * KC, clast), r[x]);
    }
    deposit(0, r[0], 0);
    __syncthreads();
    // The loop always runs whole groups of four steps: steps past the last chunk load (clamped),
    // deposit and synchronise like the others and only skip the MFMAs, so the sequence of loads
    // and of waits for them is the same on every path.
    for (int cb = 0; cb < cin; cb += 4 * KC) {
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const int c0 = cb + s * KC, cn = min(c0 + 4 * KC, clast);
        if (c0 < cin) mm(c0, 0, (s & 1) * BUFE, wt[s]);
        wload(cn, 0, wt[s]);
        request(cn, r[s]);
        deposit(min(c0 + KC, clast), r[(s + 1) & 3], ((s & 1) ^ 1) * BUFE);
        __syncthreads();
      }
    }
  } else {
    constexpr int WD = TAPS == 1 ? 1 : (MT == 1 ? 9 : 3);
    Raw va[U];
    {
      Raw v[U];
      request(0, v);
      request(min(KC, clast), va);
      deposit(0, v, 0);
    }
    WSet wt[WD];
#pragma unroll
    for (int s = 0; s < WD; ++s) wload(0, s, wt[s]);
    __syncthreads();
    int it = 0;
    for (int c0 = 0; c0 < cin; c0 += KC, ++it) {
      const int boff = (it & 1) * BUFE;
      const int cn = min(c0 + KC, clast);
#pragma unroll
      for (int t9 = 0; t9 < TAPS; ++t9) {
        mm(c0, t9, boff, wt[t9 % WD]);
        if (t9 + WD < TAPS) wload(c0, t9 + WD, wt[t9 % WD]);
        else wload(cn, t9 + WD - TAPS, wt[t9 % WD]);
      }
      if (c0 + KC < cin) deposit(c0 + KC, va, ((it & 1) ^ 1) * BUFE);
      request(min(c0 + 2 * KC, clast), va);  // in flight across the barrier and the next chunk's MFMAs
      __syncthreads();
    }
  }

  if (!m_ok) return;
  const int tile_px = (int)min((int64_t)64, limit - q0);
  const int tile_id = TAPS == 9 ? img * gridDim.x + blockIdx.x : blockIdx.x;
#pragma unroll
  for (int a = 0; a < MT; ++a) {
    if (mbase + a * 16 >= M16) continue;
    // round to bf16 first: statistics describe exactly what is stored
    float rv[4][4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) rv[t][r] = bf2f(f2bf(acc[a][t][r]));
    if (STATS) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        float s = 0.f;
#pragma unroll
        for (int t = 0; t < 4; ++t) s += (q0 + t * 16 + j < limit) ? rv[t][r] : 0.f;
#pragma unroll
        for (int off = 1; off < 16; off <<= 1) s += __shfl_xor(s, off, 64);
        const float mu = s / (float)tile_px;
        float m2 = 0.f;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const float d = rv[t][r] - mu;
          m2 += (q0 + t * 16 + j < limit) ? d * d : 0.f;
        }
#pragma unroll
        for (int off = 1; off < 16; off <<= 1) m2 += __shfl_xor(m2, off, 64);
        const int m = mbase + a * 16 + 4 * g + r;
        if (j == 0 && m < cout) {
          float* p = spart + ((int64_t)m * sT + tile_id) * 3;
          p[0] = (float)tile_px; p[1] = mu; p[2] = m2;
        }
      }
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int64_t q = q0 + t * 16 + j;
      const int m = mbase + a * 16 + 4 * g;
      if (q < limit && m < cout) {  // cout % 4 == 0 on this path
        u16* o = out + ((int64_t)img * HW + q) * out_ld + m;
        uint2 pk;
        pk.x = (unsigned)f2bf(acc[a][t][0]) | ((unsigned)f2bf(acc[a][t][1]) << 16);
        pk.y = (unsigned)f2bf(acc[a][t][2]) | ((unsigned)f2bf(acc[a][t][3]) << 16);
        *reinterpret_cast<uint2*>(o) = pk;
      }
    }
  }
}

// ----------------------------------------------------------------------------- weight gradient

// dW[m][c][t] = sum_{img,q} g[q][m] * act(a[q+shift(t)][c]).  grid (pixel splits, c groups of 64,
// m groups of 64).  Per 64-pixel tile and tap the workgroup stages gT[m][pixel] and aT[c][pixel]
// (transposed, prologue and edge masks applied) in LDS; wave w owns m-tile w of the group and
// all four c-tiles.  part[split][m][c][t] fp32.
template <int TAPS, typename TG, bool PRO>
__global__ __launch_bounds__(256) void k_wgrad(
    const u16* __restrict__ a, int64_t a_ld, const TG* __restrict__ gout, int64_t g_ld,
    float* __restrict__ part, int cin, int cout, int n, int H, int W, int tiles_per_img,
    int tiles_per_split, const float2* __restrict__ fold) {
  __shared__ u16 gT[64 * 72];  // [m][pixel], pitch 72 elements (144 bytes)
  __shared__ u16 aT[64 * 72];  // [c][pixel]
  constexpr int PT = 72;
  const int HW = H * W;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j = lane & 15, g = lane >> 4;
  const int c0 = blockIdx.y * 64, m0 = blockIdx.z * 64;
  const int total_tiles = n * tiles_per_img;
  const int t_begin = blockIdx.x * tiles_per_split, t_end = min(total_tiles, t_begin + tiles_per_split);

  f32x4 acc[TAPS][4];
#pragma unroll
  for (int t = 0; t < TAPS; ++t)
#pragma unroll
    for (int y = 0; y < 4; ++y) acc[t][y] = (f32x4){0.f, 0.f, 0.f, 0.f};

  for (int tile = t_begin; tile < t_end; ++tile) {
    const int img = tile / tiles_per_img, q0 = (tile - img * tiles_per_img) * 64;
    const u16* ab = a + (int64_t)img * HW * a_ld;
    const TG* gb = gout + (int64_t)img * HW * g_ld;
    __syncthreads();
    // gT: thread = (pixel s, 8-channel vector v of the 64 m's)
    for (int idx = tid; idx < 64 * 8; idx += 256) {
      const int s = idx >> 3, v = idx & 7;
      const int q = q0 + s, m = m0 + 8 * v;
      u16 h[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) h[e] = 0;
      if (q < HW && m < cout) {  // cout % 8 == 0
        if (sizeof(TG) == 2) {
          V8 r;
          r.q = *reinterpret_cast<const uint4*>(reinterpret_cast<const u16*>(gb) + (int64_t)q * g_ld + m);
#pragma unroll
          for (int e = 0; e < 8; ++e) h[e] = r.h[e];
        } else {
          const float* pf = reinterpret_cast<const float*>(gb) + (int64_t)q * g_ld + m;
          const float4 x = *reinterpret_cast<const float4*>(pf), y = *reinterpret_cast<const float4*>(pf + 4);
          h[0] = f2bf(x.x); h[1] = f2bf(x.y); h[2] = f2bf(x.z); h[3] = f2bf(x.w);
          h[4] = f2bf(y.x); h[5] = f2bf(y.y); h[6] = f2bf(y.z); h[7] = f2bf(y.w);
        }
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) gT[(8 * v + e) * PT + s] = h[e];
    }
#pragma unroll
    for (int t9 = 0; t9 < TAPS; ++t9) {  // unrolled: acc[t9] must stay in registers
      const int di = (TAPS == 9) ? t9 / 3 - 1 : 0, dj = (TAPS == 9) ? t9 % 3 - 1 : 0;
      if (t9 > 0) __syncthreads();
      for (int idx = tid; idx < 64 * 8; idx += 256) {
        const int s = idx >> 3, v = idx & 7;
        const int q = q0 + s, ch = c0 + 8 * v;
        const int wc = q % W, qq = q + di * W + dj;
        u16 h[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) h[e] = 0;
        const bool ok = q < HW && ch < cin && qq >= 0 && qq < HW && !(dj < 0 && wc == 0) && !(dj > 0 && wc == W - 1);
        if (ok) {
          V8 r;
          r.q = *reinterpret_cast<const uint4*>(ab + (int64_t)qq * a_ld + ch);
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            if (PRO) {
              const float2 fl = fold[ch + e];
              h[e] = f2bf(fmaxf(__fmaf_rn(bf2f(r.h[e]), fl.x, fl.y), 0.f));
            } else {
              h[e] = r.h[e];
            }
          }
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) aT[(8 * v + e) * PT + s] = h[e];
      }
      __syncthreads();
      // 64 pixels = 2 K-steps of 32
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        V8 af;
        af.q = *reinterpret_cast<const uint4*>(&gT[(wave * 16 + j) * PT + ks * 32 + 8 * g]);
#pragma unroll
        for (int y = 0; y < 4; ++y) {
          V8 bf;
          bf.q = *reinterpret_cast<const uint4*>(&aT[(y * 16 + j) * PT + ks * 32 + 8 * g]);
          acc[t9][y] = mfma_bf16(af, bf, acc[t9][y]);
        }
      }
    }
  }

  float* pb = part + (int64_t)blockIdx.x * cout * cin * TAPS;
#pragma unroll
  for (int t9 = 0; t9 < TAPS; ++t9)
#pragma unroll
    for (int y = 0; y < 4; ++y) {
      const int c = c0 + y * 16 + j;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int m = m0 + wave * 16 + 4 * g + r;
        if (m < cout && c < cin) pb[((int64_t)m * cin + c) * TAPS + t9] = acc[t9][y][r];
      }
    }
}

// 3x3 weight gradient with the activation tile staged once.  A tile is R image rows of one image;
// aT[c][row][x] holds rows r0-1 .. r0+R of the (prologue-applied) activations, pixel-contiguous
// per channel with 8 zero pixels on either side of each row, so a tap is the same tile read at a
// shifted position: the centre column is one aligned 16-byte read, the left and right columns
// are that read funnel-shifted by one element with the neighbouring dword.  gT[m][row][x] holds
// the gradient tile.  A K-step is four 8-pixel row fragments (one per lane group).  Rows of both
// arrays are permuted (channel 8v+e sits in row v+8e) so that the staging stores of one wave
// spread over all banks.  Everything the staging loops do not write stays zero from the initial
// fill: the row margins, fragments past the tile, channels past cin / cout.
constexpr int WG3_AP = 328, WG3_GP = 136;  // row pitches, both = 8 (mod 64) elements
constexpr int WG3_ROWPIX = 320;            // (R+2) * (8*FR+16) must fit in this
constexpr int WG3_BLOCK = 64 * 64 * 9;     // partial floats per (split, c group, m group)
struct Wg3Geom {
  bool ok;
  int R, FR, tpi;
};
static Wg3Geom wg3_geom(int h, int w) {
  Wg3Geom q{};
  q.FR = (w + 7) / 8;
  const int XP = q.FR * 8 + 16;
  if (3 * XP > WG3_ROWPIX) return q;
  int R = WG3_ROWPIX / XP - 2;
  if (R > 16 / q.FR) R = 16 / q.FR;
  if (R > h) R = h;
  q.R = R;
  q.tpi = (h + R - 1) / R;
  q.ok = true;
  return q;
}

template <typename TG, bool PRO>
__global__ __launch_bounds__(512) void k_wgrad3(
    const u16* __restrict__ a, int64_t a_ld, const TG* __restrict__ gout, int64_t g_ld,
    float* __restrict__ part, int cin, int cout, int n, int H, int W, int R, int FR, int tiles_per_img,
    int tiles_per_split, const float2* __restrict__ fold) {
  constexpr int AP = WG3_AP, GP = WG3_GP;
  __shared__ __attribute__((aligned(16))) u16 aT[64 * AP];
  __shared__ __attribute__((aligned(16))) u16 gT[64 * GP];
  const int RW = FR * 8, XP = RW + 16, F = R * FR, KS = (F + 3) >> 2;
  // eight waves: wave & 3 = m-tile of the group, wave >> 2 = which pair of the four c-tiles
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, mw = wave & 3, yh = wave >> 2;
  const int j = lane & 15, g = lane >> 4, v = tid & 7;
  const int c0 = blockIdx.y * 64, m0 = blockIdx.z * 64;
  const int total_tiles = n * tiles_per_img;
  const int t_begin = blockIdx.x * tiles_per_split, t_end = min(total_tiles, t_begin + tiles_per_split);

  for (int i = tid; i < 64 * AP / 8; i += 512) reinterpret_cast<uint4*>(aT)[i] = make_uint4(0u, 0u, 0u, 0u);
  for (int i = tid; i < 64 * GP / 8; i += 512) reinterpret_cast<uint4*>(gT)[i] = make_uint4(0u, 0u, 0u, 0u);

  const int chv = c0 + 8 * v, mv = m0 + 8 * v;
  const bool ch_ok = chv < cin, m_ok = mv < cout;  // cin % 8 == 0, cout % 8 == 0
  const int chl = ch_ok ? chv : 0, ml = m_ok ? mv : 0;  // load addresses stay inside the tensors
  float fs[8], fb[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    fs[e] = 0.f;
    fb[e] = 0.f;
    if (PRO) {
      const float2 fl = fold[chl + e];
      fs[e] = fl.x;
      fb[e] = fl.y;
    }
  }
  int boff[4];  // per K-step: offset of this lane group's fragment inside an aT row block
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const int f = 4 * s + g, fv = f < F ? f : 0;  // fragments past the tile meet zeros in gT
    const int r = fv / FR;
    boff[s] = r * XP + (fv - r * FR) * 8;
  }

  f32x4 acc[9][2];
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int y = 0; y < 2; ++y) acc[t][y] = (f32x4){0.f, 0.f, 0.f, 0.f};

  // Software pipeline: the global loads of tile i+1 are issued before the MFMA phase of tile i
  // and deposited (prologue, bf16 rounding, transposing 2-byte stores) after it.  Every load is
  // unconditional at a clamped in-range address, so none of them waits for another; what lies
  // outside the image or the tile is replaced by zero when it is deposited.
  const int na = (R + 2) * RW * 8, ng = R * RW * 8;  // at most 5 and 2 vectors per thread
  uint4 ra[5], rg[2];  // kept as whole vectors across the MFMA phase; taken apart only in deposit
  float4 rgl[2], rgh[2];
  auto issue = [&](int tile) {
    const int img = tile / tiles_per_img, r0 = (tile - img * tiles_per_img) * R;
    const u16* ab = a + (int64_t)img * H * W * a_ld + chl;
    const TG* gb = gout + (int64_t)img * H * W * g_ld + ml;
#pragma unroll
    for (int u = 0; u < 5; ++u) {
      const int pos = (tid + 512 * u) >> 3;
      const int rr = pos / RW, x = min(pos - rr * RW, W - 1), ir = min(max(r0 - 1 + rr, 0), H - 1);
      ra[u] = *reinterpret_cast<const uint4*>(ab + ((int64_t)ir * W + x) * a_ld);
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int pos = (tid + 512 * u) >> 3;
      const int r = pos / RW, x = min(pos - r * RW, W - 1), ir = min(r0 + r, H - 1);
      const int64_t q = (int64_t)ir * W + x;
      if (sizeof(TG) == 2) {
        rg[u] = *reinterpret_cast<const uint4*>(reinterpret_cast<const u16*>(gb) + q * g_ld);
      } else {
        const float* pf = reinterpret_cast<const float*>(gb) + q * g_ld;
        rgl[u] = *reinterpret_cast<const float4*>(pf);
        rgh[u] = *reinterpret_cast<const float4*>(pf + 4);
      }
    }
  };
  auto deposit = [&](int tile) {
    const int img = tile / tiles_per_img, r0 = (tile - img * tiles_per_img) * R;
#pragma unroll
    for (int u = 0; u < 5; ++u) {
      const int idx = tid + 512 * u, pos = idx >> 3;
      const int rr = pos / RW, x = pos - rr * RW, ir = r0 - 1 + rr;
      if (ch_ok && idx < na) {
        const bool in = ir >= 0 && ir < H && x < W;
        const int dst = rr * XP + 8 + x;
        V8 t;
        t.q = ra[u];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          u16 hv = t.h[e];
          if (PRO) hv = f2bf(fmaxf(__fmaf_rn(bf2f(hv), fs[e], fb[e]), 0.f));
          aT[(v + 8 * e) * AP + dst] = in ? hv : (u16)0;
        }
      }
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int idx = tid + 512 * u, pos = idx >> 3;
      const int r = pos / RW, x = pos - r * RW, ir = r0 + r;
      if (m_ok && idx < ng) {
        const bool in = ir < H && x < W;
        V8 t;
        if (sizeof(TG) == 2) {
          t.q = rg[u];
        } else {
          t.h[0] = f2bf(rgl[u].x); t.h[1] = f2bf(rgl[u].y); t.h[2] = f2bf(rgl[u].z); t.h[3] = f2bf(rgl[u].w);
          t.h[4] = f2bf(rgh[u].x); t.h[5] = f2bf(rgh[u].y); t.h[6] = f2bf(rgh[u].z); t.h[7] = f2bf(rgh[u].w);
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) gT[(v + 8 * e) * GP + pos] = in ? t.h[e] : (u16)0;
      }
    }
  };

  if (t_begin < t_end) issue(t_begin);
  for (int tile = t_begin; tile < t_end; ++tile) {
    __syncthreads();  // the previous tile's fragment reads (first pass: the zero fill) are done
    deposit(tile);
    __syncthreads();
    if (tile + 1 < t_end) issue(tile + 1);
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      if (s < KS) {
        V8 af;
        af.q = *reinterpret_cast<const uint4*>(&gT[(mw * 16 + j) * GP + (4 * s + g) * 8]);
        const int lb = (yh * 32 + j) * AP + boff[s] + 8;
        uint4 cq[6];
        unsigned pv[6], nx[6];
#pragma unroll
        for (int i = 0; i < 6; ++i) {  // i = c-tile of the pair * 3 + image row offset + 1
          const int base = lb + (i / 3) * 16 * AP + (i % 3) * XP;
          cq[i] = *reinterpret_cast<const uint4*>(&aT[base]);
          pv[i] = *reinterpret_cast<const unsigned*>(&aT[base - 2]);
          nx[i] = *reinterpret_cast<const unsigned*>(&aT[base + 8]);
        }
#pragma unroll
        for (int i = 0; i < 6; ++i) {
          const int y = i / 3, d = i % 3;
          V8 cur, lf, rf;
          cur.q = cq[i];
          const unsigned s0 = __builtin_amdgcn_alignbit(cur.q.y, cur.q.x, 16);
          const unsigned s1 = __builtin_amdgcn_alignbit(cur.q.z, cur.q.y, 16);
          const unsigned s2 = __builtin_amdgcn_alignbit(cur.q.w, cur.q.z, 16);
          lf.q = make_uint4(__builtin_amdgcn_alignbit(cur.q.x, pv[i], 16), s0, s1, s2);
          rf.q = make_uint4(s0, s1, s2, __builtin_amdgcn_alignbit(nx[i], cur.q.w, 16));
          acc[d * 3 + 0][y] = mfma_bf16(af, lf, acc[d * 3 + 0][y]);
          acc[d * 3 + 1][y] = mfma_bf16(af, cur, acc[d * 3 + 1][y]);
          acc[d * 3 + 2][y] = mfma_bf16(af, rf, acc[d * 3 + 2][y]);
        }
      }
    }
  }

  // partials in accumulator order: [split][c group][m group][wave][tap][c-tile of the pair][lane][4]
  float* pb = part + (((int64_t)blockIdx.x * gridDim.y + blockIdx.y) * gridDim.z + blockIdx.z) * WG3_BLOCK +
              (int64_t)wave * 18 * 256 + lane * 4;
#pragma unroll
  for (int t9 = 0; t9 < 9; ++t9)
#pragma unroll
    for (int y = 0; y < 2; ++y)
      *reinterpret_cast<float4*>(pb + (t9 * 2 + y) * 256) = make_float4(acc[t9][y][0], acc[t9][y][1], acc[t9][y][2], acc[t9][y][3]);
}

// Sums the splits of k_wgrad3's partials and writes dW[m][c][tap].  A workgroup covers 64
// accumulator quads; its four 64-thread groups each sum every fourth split (loads batched four
// deep), and the four results are added in group order.
__global__ __launch_bounds__(256) void k_sum_wgrad3(const float* __restrict__ part, int S, int gy, int gz, int cin,
                                                    int cout, float* __restrict__ dw) {
  __shared__ float4 red[3][64];
  const int64_t per_split = (int64_t)gy * gz * WG3_BLOCK;
  const int t = threadIdx.x & 63, sg = threadIdx.x >> 6;
  const int64_t i = ((int64_t)blockIdx.x * 64 + t) * 4;  // per_split is a multiple of 256
  float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
  const float* p = part + i;
  int s = sg;
  for (; s + 12 < S; s += 16) {
    const float4 a0 = *reinterpret_cast<const float4*>(p + (int64_t)s * per_split);
    const float4 a1 = *reinterpret_cast<const float4*>(p + (int64_t)(s + 4) * per_split);
    const float4 a2 = *reinterpret_cast<const float4*>(p + (int64_t)(s + 8) * per_split);
    const float4 a3 = *reinterpret_cast<const float4*>(p + (int64_t)(s + 12) * per_split);
    sum.x += a0.x; sum.y += a0.y; sum.z += a0.z; sum.w += a0.w;
    sum.x += a1.x; sum.y += a1.y; sum.z += a1.z; sum.w += a1.w;
    sum.x += a2.x; sum.y += a2.y; sum.z += a2.z; sum.w += a2.w;
    sum.x += a3.x; sum.y += a3.y; sum.z += a3.z; sum.w += a3.w;
  }
  for (; s < S; s += 4) {
    const float4 a0 = *reinterpret_cast<const float4*>(p + (int64_t)s * per_split);
    sum.x += a0.x; sum.y += a0.y; sum.z += a0.z; sum.w += a0.w;
  }
  if (sg > 0) red[sg - 1][t] = sum;
  __syncthreads();
  if (sg > 0) return;
#pragma unroll
  for (int q = 0; q < 3; ++q) {
    const float4 o = red[q][t];
    sum.x += o.x; sum.y += o.y; sum.z += o.z; sum.w += o.w;
  }
  const int blk = (int)(i / WG3_BLOCK), rem = (int)(i - (int64_t)blk * WG3_BLOCK);
  const int by = blk / gz, bz = blk - by * gz;
  const int lane = (rem >> 2) & 63, ty = rem >> 8;  // ty = (wave*9 + tap)*2 + c-tile of the pair
  const int wave = ty / 18, t9 = (ty - wave * 18) >> 1, y = 2 * (wave >> 2) + (ty & 1);
  const int j = lane & 15, g = lane >> 4;
  const int rc = y * 16 + j, c = by * 64 + 8 * (rc & 7) + (rc >> 3);
  if (c >= cin) return;
  const float o4[4] = {sum.x, sum.y, sum.z, sum.w};
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int rm = (wave & 3) * 16 + 4 * g + r, m = bz * 64 + 8 * (rm & 7) + (rm >> 3);
    if (m < cout) dw[((int64_t)m * cin + c) * 9 + t9] = o4[r];
  }
}

// 1x1 weight gradient, bf16 gradient operand.  A workgroup (eight waves) owns up to 256 input
// channels and up to 192 output channels, so the activations are read once when cout <= 192 and
// the gradient once per 256 input channels.  A tile is 32 pixels of the flattened pixel axis (one
// K-step); both operands are staged transposed, rows permuted inside each block of 64 channels
// (channel 8v+e in row v+8e) so that the 2-byte staging stores of a wave spread over all banks.
// Wave (mh, cq) accumulates m-tiles mh, mh+2, .. and c-tiles cq, cq+4, ...  The next tile's loads
// are issued, unconditionally at clamped addresses, before the MFMA phase.
constexpr int WG1_PT = 40, WG1_CG = 256, WG1_MG = 192, WG1_BLOCK = WG1_CG * WG1_MG;

template <bool PRO>
__global__ __launch_bounds__(512) void k_wgrad1(
    const u16* __restrict__ a, int64_t a_ld, const u16* __restrict__ gout, int64_t g_ld,
    float* __restrict__ part, int cin, int cout, int64_t P, int tiles_per_split, const float2* __restrict__ fold) {
  constexpr int PT = WG1_PT;
  __shared__ __attribute__((aligned(16))) u16 aT[WG1_CG * PT];
  __shared__ __attribute__((aligned(16))) u16 gT[WG1_MG * PT];
  __shared__ __attribute__((aligned(16))) float2 fl[WG1_CG];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, mh = wave & 1, cq = wave >> 1;
  const int j = lane & 15, g = lane >> 4, v = lane & 7, pl = lane >> 3;
  const int c0 = blockIdx.y * WG1_CG, m0 = blockIdx.z * WG1_MG;
  const int64_t tiles = (P + 31) / 32;
  const int64_t t_begin = (int64_t)blockIdx.x * tiles_per_split;
  const int64_t t_end = min(tiles, t_begin + tiles_per_split);
  if (PRO) {
    for (int i = tid; i < WG1_CG; i += 512) fl[i] = c0 + i < cin ? fold[c0 + i] : make_float2(0.f, 0.f);
  }

  // staging units of 64 lanes = (8 pixels) x (8 channel vectors): 16 for the activations, 12 for
  // the gradient; wave w takes units w and w + 8
  int a_row[2], a_px[2], g_row[2], g_px[2];
  bool a_ok[2], g_ok[2], g_unit[2];
  const u16* a_src[2];
  const u16* g_src[2];
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int unit = wave + 8 * u, blk = unit >> 2, pg = unit & 3;
    const int ch = c0 + blk * 64 + 8 * v, m = m0 + blk * 64 + 8 * v;
    a_ok[u] = ch < cin;  // cin % 8 == 0, cout % 8 == 0
    a_row[u] = blk * 64 + v;
    a_px[u] = pg * 8 + pl;
    a_src[u] = a + (a_ok[u] ? ch : 0);
    g_unit[u] = unit < 12;
    g_ok[u] = g_unit[u] && m < cout;
    g_row[u] = blk * 64 + v;
    g_px[u] = pg * 8 + pl;
    g_src[u] = gout + (g_ok[u] ? m : 0);
  }

  f32x4 acc[6][4];
#pragma unroll
  for (int i = 0; i < 6; ++i)
#pragma unroll
    for (int k = 0; k < 4; ++k) acc[i][k] = (f32x4){0.f, 0.f, 0.f, 0.f};

  uint4 ra[2], rg[2];
  auto issue = [&](int64_t tile) {
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int64_t pa = min(tile * 32 + a_px[u], P - 1), pg = min(tile * 32 + g_px[u], P - 1);
      ra[u] = *reinterpret_cast<const uint4*>(a_src[u] + pa * a_ld);
      rg[u] = *reinterpret_cast<const uint4*>(g_src[u] + pg * g_ld);
    }
  };
  auto deposit = [&](int64_t tile) {
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const bool in = a_ok[u] && tile * 32 + a_px[u] < P;
      V8 t;
      t.q = ra[u];
      float2 f8[8];
      if (PRO) {
        const float4* fp = reinterpret_cast<const float4*>(&fl[(a_row[u] & ~63) + 8 * v]);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float4 q = fp[e];
          f8[2 * e] = make_float2(q.x, q.y);
          f8[2 * e + 1] = make_float2(q.z, q.w);
        }
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        u16 hv = t.h[e];
        if (PRO) hv = f2bf(fmaxf(__fmaf_rn(bf2f(hv), f8[e].x, f8[e].y), 0.f));
        aT[(a_row[u] + 8 * e) * PT + a_px[u]] = in ? hv : (u16)0;
      }
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      if (g_unit[u]) {
        const bool in = g_ok[u] && tile * 32 + g_px[u] < P;
        V8 t;
        t.q = rg[u];
#pragma unroll
        for (int e = 0; e < 8; ++e) gT[(g_row[u] + 8 * e) * PT + g_px[u]] = in ? t.h[e] : (u16)0;
      }
    }
  };

  if (t_begin < t_end) issue(t_begin);
  __syncthreads();  // fold parameters are in LDS
  for (int64_t tile = t_begin; tile < t_end; ++tile) {
    deposit(tile);
    __syncthreads();
    if (tile + 1 < t_end) issue(tile + 1);
    // every row of both arrays is deposited each tile (zeros past cin / cout), so all 24 products
    // are formed unguarded
    V8 af[6], bf[4];
#pragma unroll
    for (int i = 0; i < 6; ++i) af[i].q = *reinterpret_cast<const uint4*>(&gT[((mh + 2 * i) * 16 + j) * PT + 8 * g]);
#pragma unroll
    for (int k = 0; k < 4; ++k) bf[k].q = *reinterpret_cast<const uint4*>(&aT[((cq + 4 * k) * 16 + j) * PT + 8 * g]);
#pragma unroll
    for (int i = 0; i < 6; ++i)
#pragma unroll
      for (int k = 0; k < 4; ++k) acc[i][k] = mfma_bf16(af[i], bf[k], acc[i][k]);
    __syncthreads();  // fragment reads done before the next tile is deposited
  }

  // partials in accumulator order: [split][c group][m group][wave][m-tile i][c-tile k][lane][4]
  float* pb = part + (((int64_t)blockIdx.x * gridDim.y + blockIdx.y) * gridDim.z + blockIdx.z) * WG1_BLOCK +
              (int64_t)wave * 24 * 256 + lane * 4;
#pragma unroll
  for (int i = 0; i < 6; ++i)
#pragma unroll
    for (int k = 0; k < 4; ++k)
      *reinterpret_cast<float4*>(pb + (i * 4 + k) * 256) = make_float4(acc[i][k][0], acc[i][k][1], acc[i][k][2], acc[i][k][3]);
}

// Sums the splits of k_wgrad1's partials (same scheme as k_sum_wgrad3) and writes dW[m][c].
__global__ __launch_bounds__(256) void k_sum_wgrad1(const float* __restrict__ part, int S, int gy, int gz, int cin,
                                                    int cout, float* __restrict__ dw) {
  __shared__ float4 red[3][64];
  const int64_t per_split = (int64_t)gy * gz * WG1_BLOCK;
  const int t = threadIdx.x & 63, sg = threadIdx.x >> 6;
  const int64_t i = ((int64_t)blockIdx.x * 64 + t) * 4;
  const int blk = (int)(i / WG1_BLOCK), rem = (int)(i - (int64_t)blk * WG1_BLOCK);
  const int by = blk / gz, bz = blk - by * gz;
  const int lane = (rem >> 2) & 63, ty = rem >> 8;  // ty = wave*24 + i*4 + k
  const int wave = ty / 24, ik = ty - wave * 24, mt = (wave & 1) + 2 * (ik >> 2), ct = (wave >> 1) + 4 * (ik & 3);
  // the 64 quads of a workgroup share (wave, m-tile, c-tile): uniform early exit for tiles whose
  // whole block of 64 (the unit of the row permutation) lies past the tensor
  if (bz * WG1_MG + (mt >> 2) * 64 >= cout || by * WG1_CG + (ct >> 2) * 64 >= cin) return;
  float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
  const float* p = part + i;
  int s = sg;
  for (; s + 12 < S; s += 16) {
    const float4 a0 = *reinterpret_cast<const float4*>(p + (int64_t)s * per_split);
    const float4 a1 = *reinterpret_cast<const float4*>(p + (int64_t)(s + 4) * per_split);
    const float4 a2 = *reinterpret_cast<const float4*>(p + (int64_t)(s + 8) * per_split);
    const float4 a3 = *reinterpret_cast<const float4*>(p + (int64_t)(s + 12) * per_split);
    sum.x += a0.x; sum.y += a0.y; sum.z += a0.z; sum.w += a0.w;
    sum.x += a1.x; sum.y += a1.y; sum.z += a1.z; sum.w += a1.w;
    sum.x += a2.x; sum.y += a2.y; sum.z += a2.z; sum.w += a2.w;
    sum.x += a3.x; sum.y += a3.y; sum.z += a3.z; sum.w += a3.w;
  }
  for (; s < S; s += 4) {
    const float4 a0 = *reinterpret_cast<const float4*>(p + (int64_t)s * per_split);
    sum.x += a0.x; sum.y += a0.y; sum.z += a0.z; sum.w += a0.w;
  }
  if (sg > 0) red[sg - 1][t] = sum;
  __syncthreads();
  if (sg > 0) return;
#pragma unroll
  for (int q = 0; q < 3; ++q) {
    const float4 o = red[q][t];
    sum.x += o.x; sum.y += o.y; sum.z += o.z; sum.w += o.w;
  }
  const int j = lane & 15, g = lane >> 4;
  const int rc = ct * 16 + j, c = by * WG1_CG + (rc & ~63) + 8 * (rc & 7) + ((rc & 63) >> 3);
  if (c >= cin) return;
  const float o4[4] = {sum.x, sum.y, sum.z, sum.w};
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int rm = mt * 16 + 4 * g + r, m = bz * WG1_MG + (rm & ~63) + 8 * (rm & 7) + ((rm & 63) >> 3);
    if (m < cout) dw[(int64_t)m * cin + c] = o4[r];
  }
}

// ----------------------------------------------------------------------------- BN + ReLU backward

// Thread = (pixel row pr, 8-channel vector cv); workgroup = 256 threads covering `rows` pixels per
// step x CV vectors (CV*rows = 256).  grid (channel-vector groups, pixel splits).
// part[(ch*S + s)*2] = (sum dz, sum dz*xhat) over the split's pixels.
__global__ __launch_bounds__(256) void k_bn_bwd_partial(
    const u16* __restrict__ x, int64_t x_ld, const u16* __restrict__ dact, int64_t d_ld, int64_t P,
    int c, int ppb, int lsh, const float* __restrict__ gamma, const float* __restrict__ beta,
    const float* __restrict__ mean, const float* __restrict__ istd, float* __restrict__ part) {
  __shared__ float red[2][8][256];
  // L = 1 << lsh channel vectors x 256/L pixel rows; four pixels per thread in flight
  const int L = 1 << lsh, rows = 256 >> lsh;
  const int cvl = threadIdx.x & (L - 1), pr = threadIdx.x >> lsh;
  const int ch0 = (blockIdx.x * L + cvl) * 8, s = blockIdx.y, S = gridDim.y;
  const int64_t p0 = (int64_t)s * ppb, p1 = min(P, p0 + ppb);
  float sb[8], sg[8], sc[8], sf[8], mu[8], is[8];
  const bool ok = ch0 < c;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    sb[e] = sg[e] = 0.f;
    if (ok) {
      mu[e] = mean[ch0 + e]; is[e] = istd[ch0 + e];
      bn_fold(gamma[ch0 + e], beta[ch0 + e], mu[e], is[e], sc[e], sf[e]);
    }
  }
  if (ok) {
    const u16* xp = x + ch0;
    const u16* dp = dact + ch0;
    for (int64_t pb = p0 + pr; pb < p1; pb += 4 * rows) {
      V8 xv[4], dv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {  // rows past the split are clamped here and skipped below
        const int64_t p = min(pb + u * rows, p1 - 1);
        xv[u].q = *reinterpret_cast<const uint4*>(xp + p * x_ld);
        dv[u].q = *reinterpret_cast<const uint4*>(dp + p * d_ld);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (pb + u * rows < p1) {
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float xf = bf2f(xv[u].h[e]);
            const float dz = __fmaf_rn(xf, sc[e], sf[e]) > 0.f ? bf2f(dv[u].h[e]) : 0.f;
            sb[e] += dz;
            sg[e] = __fmaf_rn(dz, (xf - mu[e]) * is[e], sg[e]);
          }
        }
      }
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) { red[0][e][threadIdx.x] = sb[e]; red[1][e][threadIdx.x] = sg[e]; }
  __syncthreads();
  // one thread per (sum, channel of the vector, vector): adds its 256/L pixel rows in order
  for (int q = threadIdx.x; q < 16 * L; q += 256) {
    const int cv = q & (L - 1), e = (q >> lsh) & 7, which = q >> (lsh + 3);
    const int ch = (blockIdx.x * L + cv) * 8 + e;
    if (ch < c) {
      float acc = 0.f;
      for (int r = 0; r < rows; ++r) acc += red[which][e][r * L + cv];
      part[((int64_t)ch * S + s) * 2 + which] = acc;
    }
  }
}

// dgamma/dbeta = sum of the S partials, one wave per channel: lane i adds partials i, i+64, ...
// in order, then a butterfly over the lanes (fixed order, every lane the same bits).
// (Measured alternative: with at most 32 partials per channel, every workgroup of the
// element-wise pass added them itself and this launch was left out for slabs of up to 8192
// pixels.  The reduction pass with fewer splits and the element-wise pass with that prologue
// each took 3-5 us longer, more than the 3 us launch they replaced: config 4 went from 15.0
// to 15.2 ms.)
__global__ __launch_bounds__(256) void k_bn_bwd_finalize(const float* __restrict__ part, int c, int S,
                                                         float* __restrict__ dgamma, float* __restrict__ dbeta) {
  const int ch = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (ch >= c) return;
  const float2* pp = reinterpret_cast<const float2*>(part) + (int64_t)ch * S;
  float b = 0.f, g = 0.f;
  for (int s = lane; s < S; s += 64) { const float2 v = pp[s]; b += v.x; g += v.y; }
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) { b += __shfl_xor(b, off, 64); g += __shfl_xor(g, off, 64); }
  if (lane == 0) { dbeta[ch] = b; dgamma[ch] = g; }
}

// du = scale*(dz - dbeta/P - xhat*dgamma/P).  ACC: added into the fp32 slab G (BN1, concat
// backward); else written as bf16 over dact (BN2: gradient of b_l).
template <bool ACC>
__global__ __launch_bounds__(256) void k_bn_bwd_apply(
    const u16* __restrict__ x, int64_t x_ld, const u16* dact, int64_t d_ld, u16* du_bf, int64_t du_ld,
    float* __restrict__ G, int64_t g_ld, int64_t P, int c, int ppb, int lsh, float inv_p,
    const float* __restrict__ gamma, const float* __restrict__ beta, const float* __restrict__ mean,
    const float* __restrict__ istd, const float* __restrict__ dgamma, const float* __restrict__ dbeta) {
  // same thread map as k_bn_bwd_partial: a thread keeps its eight channels' coefficients in
  // registers and walks pixels, four in flight
  const int L = 1 << lsh, rows = 256 >> lsh;
  const int cvl = threadIdx.x & (L - 1), pr = threadIdx.x >> lsh;
  const int ch0 = (blockIdx.x * L + cvl) * 8;
  if (ch0 >= c) return;
  const int64_t p0 = (int64_t)blockIdx.y * ppb, p1 = min(P, p0 + ppb);
  float sc[8], sf[8], mu[8], is[8], db[8], dg[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    mu[e] = mean[ch0 + e]; is[e] = istd[ch0 + e];
    bn_fold(gamma[ch0 + e], beta[ch0 + e], mu[e], is[e], sc[e], sf[e]);
    db[e] = dbeta[ch0 + e] * inv_p;
    dg[e] = dgamma[ch0 + e] * inv_p;
  }
  const u16* xp = x + ch0;
  const u16* dp = dact + ch0;
  for (int64_t pb = p0 + pr; pb < p1; pb += 4 * rows) {
    V8 xv[4], dv[4];
    float4 ga[4], gb[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {  // rows past the split are clamped here and skipped below
      const int64_t p = min(pb + u * rows, p1 - 1);
      xv[u].q = *reinterpret_cast<const uint4*>(xp + p * x_ld);
      dv[u].q = *reinterpret_cast<const uint4*>(dp + p * d_ld);
      if (ACC) {
        const float* gp = G + p * g_ld + ch0;
        ga[u] = *reinterpret_cast<const float4*>(gp);
        gb[u] = *reinterpret_cast<const float4*>(gp + 4);
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int64_t p = pb + u * rows;
      if (p < p1) {
        float r[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float xf = bf2f(xv[u].h[e]);
          const float dz = __fmaf_rn(xf, sc[e], sf[e]) > 0.f ? bf2f(dv[u].h[e]) : 0.f;
          r[e] = sc[e] * (dz - db[e] - (xf - mu[e]) * is[e] * dg[e]);
        }
        if (ACC) {
          float* gp = G + p * g_ld + ch0;
          float4 a = ga[u], b = gb[u];
          a.x += r[0]; a.y += r[1]; a.z += r[2]; a.w += r[3]; b.x += r[4]; b.y += r[5]; b.z += r[6]; b.w += r[7];
          *reinterpret_cast<float4*>(gp) = a;
          *reinterpret_cast<float4*>(gp + 4) = b;
        } else {
          V8 ov;
#pragma unroll
          for (int e = 0; e < 8; ++e) ov.h[e] = f2bf(r[e]);
          *reinterpret_cast<uint4*>(du_bf + p * du_ld + ch0) = ov.q;
        }
      }
    }
  }
}

inline unsigned grid1d(int64_t items, int per, unsigned cap) {
  int64_t g = (items + per - 1) / per;
  if (g < 1) g = 1;
  if (g > (int64_t)cap) g = cap;
  return (unsigned)g;
}

}  // namespace

// ============================================================================ launchers

hipError_t copy_rows(const void* src, int64_t sld, void* dst, int64_t dld, int64_t P, int c, hipStream_t st) {
  hipLaunchKernelGGL(k_copy_rows, dim3(grid1d(P * (c / 8), 512, 16384)), dim3(256), 0, st, (const u16*)src, sld,
                     (u16*)dst, dld, P, c / 8);
  return hipGetLastError();
}

hipError_t bn_relu_rows(const void* x, int64_t ld, const float2* fold, void* out, int64_t old, void* copy, int64_t cld,
                        int64_t P, int c, hipStream_t st) {
  hipLaunchKernelGGL(k_bn_relu_rows, dim3(grid1d(P * (c / 8), 512, 16384)), dim3(256), 0, st, (const u16*)x, ld, fold,
                     (u16*)out, old, (u16*)copy, cld, P, c / 8);
  return hipGetLastError();
}

hipError_t bf16_to_f32(const void* src, float* dst, int64_t count, hipStream_t st) {
  hipLaunchKernelGGL(k_bf16_to_f32, dim3(grid1d(count / 8, 512, 16384)), dim3(256), 0, st, (const u16*)src, dst,
                     count / 8);
  return hipGetLastError();
}

hipError_t f32_rows_to_bf16(const float* src, int64_t sld, void* dst, int64_t P, int c, hipStream_t st) {
  hipLaunchKernelGGL(k_f32_rows_to_bf16, dim3(grid1d(P * (c / 8), 512, 16384)), dim3(256), 0, st, src, sld,
                     (u16*)dst, P, c / 8);
  return hipGetLastError();
}

int stats_splits(int64_t P, int c) {
  const int groups = (c / 8 + 31) / 32;
  int s = 1024 / groups;
  if (s > 256) s = 256;
  const int64_t cap = (P + 63) / 64;
  if (s > cap) s = (int)cap;
  return s < 1 ? 1 : s;
}
size_t stats_partial_floats(int64_t P, int c) { return (size_t)c * stats_splits(P, c) * 3; }

hipError_t stats_partial(const void* x, int64_t ld, int64_t P, int c, float* part, int* T, hipStream_t st) {
  const int S = stats_splits(P, c);
  const int ppb = (int)((P + S - 1) / S);
  const int gs = (int)((P + ppb - 1) / ppb);
  *T = gs;
  hipLaunchKernelGGL(k_stats_partial, dim3((unsigned)((c / 8 + 31) / 32), (unsigned)gs), dim3(256), 0, st,
                     (const u16*)x, ld, P, c, ppb, part);
  return hipGetLastError();
}

size_t packed_layer_elems(int c, int k, int B) {
  const size_t B16 = (B + 15) & ~15, k16 = (k + 15) & ~15, B32 = (B + 31) & ~31, k32 = (k + 31) & ~31;
  const size_t c16 = (c + 15) & ~15, c32 = (c + 31) & ~31;
  return B16 * c32 + c16 * B32 + 9 * k16 * B32 + 9 * B16 * k32;
}

hipError_t pack_block_weights(const float* params, void* packed, int c0, int k, int B, int m, hipStream_t st) {
  const size_t most = packed_layer_elems(c0 + (m - 1) * k, k, B);
  unsigned gx = (unsigned)((most + 255) / 256);
  if (gx > 256) gx = 256;
  hipLaunchKernelGGL(k_pack_block_weights, dim3(gx, (unsigned)m), dim3(256), 0, st, params, (u16*)packed, c0, k, B);
  return hipGetLastError();
}

size_t packed_weight_elems(int cout, int cin, int taps) {
  return (size_t)taps * ((cout + 15) & ~15) * ((cin + 31) & ~31);
}

hipError_t pack_weights(WeightView wv, int cout, int cin, int taps, void* packed, hipStream_t st) {
  const size_t total = packed_weight_elems(cout, cin, taps);
  unsigned grid = (unsigned)((total + 255) / 256);
  if (grid > 4096) grid = 4096;
  hipLaunchKernelGGL(k_pack_weights, dim3(grid), dim3(256), 0, st, wv.w, wv.sm, wv.sc, wv.flip, cout, cin, taps,
                     (u16*)packed);
  return hipGetLastError();
}

size_t conv_stats_partial_floats(int n, int cout, int h, int w) {
  return (size_t)cout * n * ((h * w + 63) / 64) * 3;
}

// taps 1 or 9; in_f32: input is the fp32 gradient slab.  fold: BN+ReLU prologue (or null).
// spart: epilogue statistics (or null), *sT = partials per channel.
hipError_t conv(const void* in, int64_t in_ld, bool in_f32, const void* Wp, void* out, int64_t out_ld, int n,
                int cin, int cout, int h, int w, int taps, const float2* fold, float* spart, int* sT,
                hipStream_t st) {
  const int hw = h * w, M16 = (cout + 15) & ~15, K32 = (cin + 31) & ~31, mtiles = M16 / 16;
  const int64_t P = (int64_t)n * hw;
  // 1x1: flat 64-pixel tiles over all images; 3x3: tiles of one image
  const int64_t ptiles = taps == 9 ? (int64_t)((hw + 63) / 64) * n : (P + 63) / 64;
  int mt = (mtiles + 3) / 4;
  if (mt > 3) mt = 3;
  // few pixel tiles: split the output channels over more workgroups (each repeats the staging,
  // on compute units that would otherwise idle) so that a chunk costs each of them less
  while (mt > 1 && ptiles * ((mtiles + 4 * mt - 1) / (4 * mt)) < 256) --mt;
  const int gy = (mtiles + 4 * mt - 1) / (4 * mt);
  dim3 grid(taps == 9 ? (unsigned)((hw + 63) / 64) : (unsigned)ptiles, (unsigned)gy, taps == 9 ? (unsigned)n : 1u);
  const int T = (int)ptiles;
  if (sT) *sT = T;
  const int halo = taps == 9 ? w + 1 : 0;
  const size_t lds = (size_t)2 * (64 + 2 * halo) * 72 * sizeof(u16) + (fold ? (size_t)cin * 8 : 0);
  if (lds > 64 * 1024 || (taps == 9 && (64 + 2 * halo) * 8 > 8 * 256)) return hipErrorInvalidValue;
  if ((fold != nullptr) != (spart != nullptr) && fold) return hipErrorInvalidValue;
  // eight chunks or more, and about one workgroup per compute unit (with several, their phases
  // already cover one another's latencies and the ring's extra loads only cost).  (Chunks of 128
  // channels instead of 64 in this form -- half the barriers, 171-218 registers -- were slower:
  // 13.9 -> 14.3 ms per step of the DenseNet-161-shaped blocks.)
  const bool ring = taps == 1 && cin >= 512 && ptiles * gy <= 320;
#define DNB_K(TAPS, MT, TIN, PRO, STATS, RING)                                                                  \
  hipLaunchKernelGGL((k_conv<TAPS, MT, TIN, PRO, STATS, RING>), grid, dim3(256), lds, st, (const TIN*)in, in_ld, \
                     (const u16*)Wp, M16, K32, (u16*)out, out_ld, cin, cout, h, w, P, fold, spart, T)
#define DNB_K2(TAPS, MT, RING)                                                        \
  do {                                                                                \
    if (in_f32) DNB_K(TAPS, MT, float, false, false, RING);                           \
    else if (fold) DNB_K(TAPS, MT, u16, true, true, RING);                            \
    else if (spart) DNB_K(TAPS, MT, u16, false, true, RING);                          \
    else DNB_K(TAPS, MT, u16, false, false, RING);                                    \
  } while (0)
#define DNB_K3(TAPS, RING)                                                            \
  do {                                                                                \
    if (mt == 3) DNB_K2(TAPS, 3, RING); else if (mt == 2) DNB_K2(TAPS, 2, RING); else DNB_K2(TAPS, 1, RING); \
  } while (0)
  if (taps == 9) DNB_K3(9, false);
  else if (ring) DNB_K3(1, true);
  else DNB_K3(1, false);
#undef DNB_K3
#undef DNB_K2
#undef DNB_K
  return hipGetLastError();
}

// Workgroups of the row-tiled weight-gradient kernels (k_wgrad3, k_wgrad1).  Each ends with a
// partial of 147 / 196 KB that the sum kernel reads again, and both run beside the data-gradient
// chain on a helper stream, so a part of the CUs serves better than all of them.  Per step of
// the DenseNet-161-shaped blocks, with three helper streams: targets of 256 / 128 / 64 / 32
// workgroups gave 15.06 / 14.71 / 14.56 / 15.50 ms (the same order in each block taken alone,
// 56x56 to 7x7); with the one helper stream now used: 64 / 96 / 128 / 192 / 256 gave 14.83 /
// 13.87 / 13.90 / 14.19 / 14.40 ms.
constexpr int WG_TARGET = 96;

static int wgrad_tiles(int n, int h, int w, int taps) {
  const Wg3Geom q = wg3_geom(h, w);
  return (taps == 9 && q.ok) ? n * q.tpi : n * ((h * w + 63) / 64);
}
int wgrad_splits(int n, int cin, int cout, int h, int w, int taps) {
  const int tiles = wgrad_tiles(n, h, w, taps);
  const int gy = (cin + 63) / 64, gz = (cout + 63) / 64;
  // k_wgrad3: about WG_TARGET workgroups in all, evenly loaded
  int s = ((taps == 9 && wg3_geom(h, w).ok) ? WG_TARGET : 1024) / (gy * gz);
  if (s < 1) s = 1;
  if (s > tiles) s = tiles;
  if (s > 128) s = 128;
  const int tps = (tiles + s - 1) / s;
  return (tiles + tps - 1) / tps;
}
// k_wgrad1: 32-pixel tiles of the flattened pixel axis, about WG_TARGET workgroups in all
static int wgrad1_splits(int64_t P, int cin, int cout) {
  const int64_t tiles = (P + 31) / 32;
  const int gy = (cin + WG1_CG - 1) / WG1_CG, gz = (cout + WG1_MG - 1) / WG1_MG;
  int64_t s = WG_TARGET / (gy * gz);
  if (s < 1) s = 1;
  if (s > tiles) s = tiles;
  if (s > 128) s = 128;
  const int64_t tps = (tiles + s - 1) / s;
  return (int)((tiles + tps - 1) / tps);
}
size_t wgrad_partial_floats(int n, int cin, int cout, int h, int w, int taps) {
  const size_t S = (size_t)wgrad_splits(n, cin, cout, h, w, taps);
  if (taps == 9 && wg3_geom(h, w).ok) return S * ((cin + 63) / 64) * ((cout + 63) / 64) * WG3_BLOCK;
  size_t f = S * cin * cout * taps;
  if (taps == 1) {  // either 1x1 kernel may run, depending on the gradient operand's type
    const size_t f1 = (size_t)wgrad1_splits((int64_t)n * h * w, cin, cout) * ((cin + WG1_CG - 1) / WG1_CG) *
                      ((cout + WG1_MG - 1) / WG1_MG) * WG1_BLOCK;
    if (f1 > f) f = f1;
  }
  return f;
}

// g_f32: the gradient operand is the fp32 slab (3x3), else bf16 (1x1).  The caller adds the
// partials (launch_sum_partials) -- *splits says how many.
hipError_t wgrad(const void* a, int64_t a_ld, const void* g, int64_t g_ld, bool g_f32, float* part, float* dw, int n,
                 int cin, int cout, int h, int w, int taps, const float2* fold, hipStream_t st) {
  if (taps == 1 && !g_f32) {
    const int64_t P = (int64_t)n * h * w, tiles = (P + 31) / 32;
    const int S = wgrad1_splits(P, cin, cout);
    const int tps = (int)((tiles + S - 1) / S);
    dim3 grid((unsigned)S, (unsigned)((cin + WG1_CG - 1) / WG1_CG), (unsigned)((cout + WG1_MG - 1) / WG1_MG));
    if (fold)
      hipLaunchKernelGGL((k_wgrad1<true>), grid, dim3(512), 0, st, (const u16*)a, a_ld, (const u16*)g, g_ld, part,
                         cin, cout, P, tps, fold);
    else
      hipLaunchKernelGGL((k_wgrad1<false>), grid, dim3(512), 0, st, (const u16*)a, a_ld, (const u16*)g, g_ld, part,
                         cin, cout, P, tps, fold);
    const int64_t per_split = (int64_t)grid.y * grid.z * WG1_BLOCK;
    hipLaunchKernelGGL(k_sum_wgrad1, dim3((unsigned)(per_split / 256)), dim3(256), 0, st, part, S, (int)grid.y,
                       (int)grid.z, cin, cout, dw);
    return hipGetLastError();
  }
  const Wg3Geom q3 = wg3_geom(h, w);
  const bool three = taps == 9 && q3.ok;
  const int tpi = three ? q3.tpi : (h * w + 63) / 64, tiles = n * tpi;
  const int S = wgrad_splits(n, cin, cout, h, w, taps);
  const int tps = (tiles + S - 1) / S;
  dim3 grid((unsigned)S, (unsigned)((cin + 63) / 64), (unsigned)((cout + 63) / 64));
  if (three) {
#define DNB_W3(TG, PRO)                                                                                \
  hipLaunchKernelGGL((k_wgrad3<TG, PRO>), grid, dim3(512), 0, st, (const u16*)a, a_ld, (const TG*)g, \
                     g_ld, part, cin, cout, n, h, w, q3.R, q3.FR, tpi, tps, fold)
    if (g_f32) { if (fold) DNB_W3(float, true); else DNB_W3(float, false); }
    else       { if (fold) DNB_W3(u16, true); else DNB_W3(u16, false); }
#undef DNB_W3
    const int64_t per_split = (int64_t)grid.y * grid.z * WG3_BLOCK;
    hipLaunchKernelGGL(k_sum_wgrad3, dim3((unsigned)(per_split / 256)), dim3(256), 0, st, part, S,
                       (int)grid.y, (int)grid.z, cin, cout, dw);
    return hipGetLastError();
  }
#define DNB_W(TAPS, TG, PRO)                                                                              \
  hipLaunchKernelGGL((k_wgrad<TAPS, TG, PRO>), grid, dim3(256), 0, st, (const u16*)a, a_ld, (const TG*)g, \
                     g_ld, part, cin, cout, n, h, w, tpi, tps, fold)
  if (taps == 9) {
    if (g_f32) { if (fold) DNB_W(9, float, true); else DNB_W(9, float, false); }
    else       { if (fold) DNB_W(9, u16, true); else DNB_W(9, u16, false); }
  } else {
    if (g_f32) { if (fold) DNB_W(1, float, true); else DNB_W(1, float, false); }
    else       { if (fold) DNB_W(1, u16, true); else DNB_W(1, u16, false); }
  }
#undef DNB_W
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_sum_partials(part, S, (int64_t)cin * cout * taps, dw, st);
}

// channel vectors side by side in a workgroup of the BN backward kernels: 4, 8, 16 or 32
// (the count among 8, 16, 32 that leaves the fewest lanes without a vector; 4 for tiny c)
static int bn_bwd_lsh(int c) {
  const int cv = c / 8;
  if (cv <= 4) return 2;
  int best = 5, waste = ((cv + 31) / 32) * 32 - cv;
  for (int lsh = 4; lsh >= 3; --lsh) {
    const int L = 1 << lsh, w = ((cv + L - 1) / L) * L - cv;
    if (w < waste) { waste = w; best = lsh; }
  }
  return best;
}
int bn_bwd_splits(int64_t P, int c) {
  const int lsh = bn_bwd_lsh(c), L = 1 << lsh, rows = 256 >> lsh;
  const int groups = (c / 8 + L - 1) / L;
  int s = 1024 / groups;
  if (s > 256) s = 256;
  const int64_t cap = (P + 8 * rows - 1) / (8 * rows);  // at least two batches of four pixels per thread
  if (s > cap) s = (int)cap;
  return s < 1 ? 1 : s;
}
size_t bn_bwd_partial_floats(int64_t P, int c) { return (size_t)c * bn_bwd_splits(P, c) * 2; }

// BN+ReLU backward, reduction pass: dgamma / dbeta over (P, c).
hipError_t bn_relu_bwd_reduce(const void* x, int64_t x_ld, const void* dact, int64_t d_ld, int64_t P, int c,
                              const float* gamma, const float* beta, const float* mean, const float* istd,
                              float* dgamma, float* dbeta, float* part, hipStream_t st) {
  const int S = bn_bwd_splits(P, c), lsh = bn_bwd_lsh(c), L = 1 << lsh;
  const int ppb = (int)((P + S - 1) / S);
  const int gs = (int)((P + ppb - 1) / ppb);
  const dim3 grid((unsigned)((c / 8 + L - 1) / L), (unsigned)gs);
  hipLaunchKernelGGL(k_bn_bwd_partial, grid, dim3(256), 0, st, (const u16*)x, x_ld, (const u16*)dact, d_ld, P, c, ppb,
                     lsh, gamma, beta, mean, istd, part);
  hipLaunchKernelGGL(k_bn_bwd_finalize, dim3((unsigned)((c + 3) / 4)), dim3(256), 0, st, part, c, gs, dgamma, dbeta);
  return hipGetLastError();
}

// BN+ReLU backward, element-wise pass over (P, c) with dgamma / dbeta given.  G != null: du is
// accumulated into the fp32 slab (row stride g_ld); else du is written as bf16 to du_bf (may
// alias dact).  A channel sub-range of a wider BN is this call with every pointer moved to the
// range's first channel (a multiple of 8) and `c` its length; `P` is the BN's pixel count.
hipError_t bn_relu_bwd_apply(const void* x, int64_t x_ld, const void* dact, int64_t d_ld, void* du_bf, int64_t du_ld,
                             float* G, int64_t g_ld, int64_t P, int c, const float* gamma, const float* beta,
                             const float* mean, const float* istd, const float* dgamma, const float* dbeta,
                             hipStream_t st) {
  if (c <= 0) return hipSuccess;
  const int S = bn_bwd_splits(P, c), lsh = bn_bwd_lsh(c), L = 1 << lsh;
  const int ppb = (int)((P + S - 1) / S);
  const float inv_p = 1.0f / (float)P;
  // the element-wise pass wants more, shorter workgroups than the reduction
  const int ppa = (int)min((int64_t)ppb, (int64_t)(256 >> lsh) * 16);
  const dim3 grida((unsigned)((c / 8 + L - 1) / L), (unsigned)((P + ppa - 1) / ppa));
  if (G)
    hipLaunchKernelGGL((k_bn_bwd_apply<true>), grida, dim3(256), 0, st, (const u16*)x, x_ld, (const u16*)dact, d_ld,
                       (u16*)nullptr, (int64_t)0, G, g_ld, P, c, ppa, lsh, inv_p, gamma, beta, mean, istd, dgamma, dbeta);
  else
    hipLaunchKernelGGL((k_bn_bwd_apply<false>), grida, dim3(256), 0, st, (const u16*)x, x_ld, (const u16*)dact, d_ld,
                       (u16*)du_bf, du_ld, (float*)nullptr, (int64_t)0, P, c, ppa, lsh, inv_p, gamma, beta, mean, istd,
                       dgamma, dbeta);
  return hipGetLastError();
}

// Both passes over the same (P, c).
hipError_t bn_relu_bwd(const void* x, int64_t x_ld, const void* dact, int64_t d_ld, void* du_bf, int64_t du_ld,
                       float* G, int64_t g_ld, int64_t P, int c, const float* gamma, const float* beta,
                       const float* mean, const float* istd, float* dgamma, float* dbeta, float* part,
                       hipStream_t st) {
  hipError_t e = bn_relu_bwd_reduce(x, x_ld, dact, d_ld, P, c, gamma, beta, mean, istd, dgamma, dbeta, part, st);
  if (e != hipSuccess) return e;
  return bn_relu_bwd_apply(x, x_ld, dact, d_ld, du_bf, du_ld, G, g_ld, P, c, gamma, beta, mean, istd, dgamma, dbeta, st);
}

}  // namespace nhwc
}  // namespace dnb
