// Fast fp32 NCHW convolution kernels for the shapes DenseNet blocks actually have
// (pixel counts and strides that are multiples of 4, 16-byte aligned slabs).  Anything else
// runs on the generic kernels in dnb_conv_f32.hip; both compute the same sums.
//
// Common idea: the 16x16x4 fp32 MFMA puts channels on M and pixels on N (forward, data
// gradient) or channels on both M and N and pixels on K (weight gradient).  A lane never
// loads single floats from HBM: it loads 4 consecutive pixels (16 bytes) and uses them for
// four MFMAs -- four N-tiles whose columns interleave (tile t holds pixels 4j+t), or four
// K-steps.  The order of the K index inside a sum is free, so lane group g takes channels
// {g, 4+g, 8+g, 12+g} of a 16-channel chunk and a channel tail that is a multiple of 4
// costs no padding.
//
// Measurements that shaped (or failed to improve) these kernels, on the first dense block's
// shapes of DenseNet-BC-100 at batch 64 (P = 65536, B = 48, k = 12), compile-time ablation builds:
//   * forward 3x3, one tile per workgroup (v3): 28 us = ~4.4 empty launch + 3.8 staging + 4 loads
//     + 8 MFMA + 1.8 statistics + 1 K-split reduction + ...: the parts add up because all
//     workgroups of a launch are in the same phase at the same time.  The persistent kernel (v4)
//     overlaps them inside a workgroup: 19.5 us; with everything but the skeleton removed 9.4 us.
//   * 3x3 weight gradient: 27 us = 6.4 MFMA + 6.6 scattered 4-byte partial stores + 4 wave
//     reduction + ~10 rest; accumulator-order stores brought it to 22.5 us.  A two-region tree
//     reduction ((0+2)+(1+3)) was slower than the chain (29 us); staging the tile progressively
//     and prefetching the gradient operand changed nothing (neither is on the critical path).
//     Splitting the tiles instead of the pixels over the waves removed the reduction: 17.6 us.
//   * 1x1: a 3-deep register prefetch ring over the K chunks did not change the 22 us of the
//     forward kernel; 5 us remain with loads and MFMAs removed.
//   * 1x1 weight gradient: operands two steps ahead in static register stages: 17.5 -> 15.5 us on
//     average; 96 instead of 64 input channels per workgroup (fewer re-reads of the gradient
//     operand, 236 registers) changed nothing.
//   * BN-backward sums computed in the data-gradient convs' epilogues (to drop the separate
//     reduction launch) made those convs 6-15 us slower, more than the launch they saved.
constexpr int kV4Workgroups = 512;  // workgroups of the persistent 3x3 kernel (two per CU)
static_assert(kV4Workgroups % 8 == 0, "tiles are dealt to workgroups per XCD (8 of them)");

#include "dnb_internal.h"
#include <hip/hip_ext.h>

#include <type_traits>

#include "dnb_stats.h"

namespace dnb {

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ f32x4 mfma16(float a, float b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ float4 ldg4(const float* p) { return *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ float4 zero4() { return make_float4(0.f, 0.f, 0.f, 0.f); }
__device__ __forceinline__ float elem(const float4& v, int e) {
  return e == 0 ? v.x : (e == 1 ? v.y : (e == 2 ? v.z : v.w));
}

// ------------------------------------------------------------------------------- packed weights
//
// The fast forward / data-gradient kernels read their A operand straight from global memory
// (it is small and stays in L2), 16 bytes per lane, so the weights are first re-laid as
// [tap][Mpad][Kpad], zero padded to multiples of 16, with the K index permuted inside each
// 16-chunk: position 16*chunk + 4*g + ks holds channel 16*chunk + 4*ks + g.

__device__ __forceinline__ int unperm16(int pos) { return (pos & ~15) + 4 * (pos & 3) + ((pos >> 2) & 3); }

__global__ __launch_bounds__(256) void k_pack_weights(const float* __restrict__ w, int64_t sm, int64_t sc,
                                                      int flip, int cout, int cin, int taps,
                                                      float* __restrict__ outp) {
  const int M16 = (cout + 15) & ~15, K16 = (cin + 15) & ~15;
  const int64_t total = (int64_t)taps * M16 * K16;
  for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * 256) {
    const int pos = (int)(idx % K16);
    const int64_t rem = idx / K16;
    const int m = (int)(rem % M16), t = (int)(rem / M16);
    const int c = unperm16(pos);
    outp[idx] = (m < cout && c < cin) ? w[(int64_t)m * sm + (int64_t)c * sc + (flip ? taps - 1 - t : t)] : 0.f;
  }
}

// All layers of a dense block in one launch (grid.y = layer).  Per layer, in order:
// 1x1 forward [B16][C16], 1x1 data gradient [C16][B16], 3x3 forward [9][k16][B16],
// 3x3 data gradient [9][B16][k16] (transposed and flipped).
__global__ __launch_bounds__(256) void k_pack_block_weights(const float* __restrict__ params,
                                                            float* __restrict__ packed, int c0, int k,
                                                            int B) {
  const int l = blockIdx.y + 1;
  const int B16 = (B + 15) & ~15, k16 = (k + 15) & ~15;
  int64_t poff = 0, koff = 0;
  for (int i = 1; i < l; ++i) {
    const int c = c0 + (i - 1) * k, c16 = (c + 15) & ~15;
    poff += 2 * (int64_t)c + (int64_t)B * c + 2 * B + 9 * (int64_t)k * B;
    koff += 2 * (int64_t)B16 * c16 + 18 * (int64_t)k16 * B16;
  }
  const int C = c0 + (l - 1) * k, C16 = (C + 15) & ~15;
  const float* W1 = params + poff + 2 * C;
  const float* W3 = W1 + (int64_t)B * C + 2 * B;
  float* A = packed + koff;
  const int64_t n1 = (int64_t)B16 * C16, n3 = 9 * (int64_t)k16 * B16, total = 2 * n1 + 2 * n3;
  for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * 256) {
    float v = 0.f;
    if (idx < n1) {
      const int m = (int)(idx / C16), c = unperm16((int)(idx % C16));
      if (m < B && c < C) v = W1[(int64_t)m * C + c];
    } else if (idx < 2 * n1) {
      const int64_t e = idx - n1;
      const int cc = (int)(e / B16), o = unperm16((int)(e % B16));
      if (cc < C && o < B) v = W1[(int64_t)o * C + cc];
    } else if (idx < 2 * n1 + n3) {
      const int64_t e = idx - 2 * n1;
      const int t = (int)(e / (k16 * B16)), rem = (int)(e % (k16 * B16));
      const int mm = rem / B16, c = unperm16(rem % B16);
      if (mm < k && c < B) v = W3[((int64_t)mm * B + c) * 9 + t];
    } else {
      const int64_t e = idx - 2 * n1 - n3;
      const int t = (int)(e / (B16 * k16)), rem = (int)(e % (B16 * k16));
      const int cc = rem / k16, o = unperm16(rem % k16);
      if (cc < B && o < k) v = W3[((int64_t)o * B + cc) * 9 + (8 - t)];
    }
    A[idx] = v;
  }
}

// Sums the accumulators of the K-split waves of a workgroup (fixed order 0,1,2,...).  M-tile a
// is owned by wave a % nw: every other wave writes its copy of the tile to LDS, the owner adds
// the copies (its own stays in registers, inserted at its place in the order) and keeps the
// result.  red: [MT*NT][nw-1 slots][64 lanes][4].
template <int MT, int NT>
__device__ __forceinline__ void ksplit_reduce(f32x4 (&acc)[MT][NT], float* red, int wave, int lane, int nw) {
  __syncthreads();  // (wave = index inside the K group, nw = waves per K group, red = the group's buffer)
  if (nw == 1) return;
#pragma unroll
  for (int a = 0; a < MT; ++a) {
    const int owner = a % nw;
    if (wave != owner) {
      const int slot = (wave - owner - 1 + nw) % nw;
#pragma unroll
      for (int t = 0; t < NT; ++t)
        *reinterpret_cast<float4*>(&red[((((a * NT + t) * (nw - 1)) + slot) * 64 + lane) * 4]) =
            make_float4(acc[a][t][0], acc[a][t][1], acc[a][t][2], acc[a][t][3]);
    }
  }
  __syncthreads();
#pragma unroll
  for (int a = 0; a < MT; ++a) {
    const int owner = a % nw;
    if (wave == owner) {
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        f32x4 s = (f32x4){0.f, 0.f, 0.f, 0.f};
        for (int w = 0; w < nw; ++w) {
          if (w == owner) {
            s[0] += acc[a][t][0]; s[1] += acc[a][t][1]; s[2] += acc[a][t][2]; s[3] += acc[a][t][3];
          } else {
            const int slot = (w - owner - 1 + nw) % nw;
            const float4 v = *reinterpret_cast<const float4*>(
                &red[((((a * NT + t) * (nw - 1)) + slot) * 64 + lane) * 4]);
            s[0] += v.x; s[1] += v.y; s[2] += v.z; s[3] += v.w;
          }
        }
        acc[a][t] = s;
      }
    }
  }
}

// ------------------------------------------------------------------------------- 1x1, fwd/dgrad
//
// out[m][q] = sum_c W(m,c) in[c][q].  No LDS in the main loop: each lane streams its pixels of
// channel 16*chunk+4*ks+g straight from HBM into the B operand and its packed weights from L2
// into the A operand, one chunk ahead.  The workgroup is one pixel tile (16*PPL pixels):
//   KSPLIT  : its waves take alternate 16-channel chunks (many loads in flight for a long K,
//             e.g. the forward 1x1 over the whole concatenation) and are summed through LDS;
//   !KSPLIT : its waves take different M-tiles of the same pixels (short K, many output
//             channels: the data gradient of the 1x1).
// Epilogue statistics.  A wave that owns an output tile (16 channels x 16*NT pixels, lane (j,g)
// holding channels 4g+r and pixels NT*j+t) reduces each channel over the tile's valid pixels to
// (count, mean, M2) -- two passes in registers, 16-lane butterflies -- and stores it as partial
// `tile_id` of that channel: part[(m*T + tile_id)*3 ..].  The BN that consumes the conv output
// merges the T partials, so the output is never re-read for its statistics.
template <int NT>
__device__ __forceinline__ void tile_stats(const f32x4 (&acc)[NT], bool pix_ok, float cnt, int mfirst,
                                           int cout, float* __restrict__ part, int T, int tile_id) {
  const int lane = threadIdx.x & 63, j = lane & 15, g = lane >> 4;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    float s = 0.f;
#pragma unroll
    for (int t = 0; t < NT; ++t) s += pix_ok ? acc[t][r] : 0.f;
#pragma unroll
    for (int off = 1; off < 16; off <<= 1) s += __shfl_xor(s, off, 64);
    const float mu = s / cnt;
    float m2 = 0.f;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const float dlt = acc[t][r] - mu;
      m2 += pix_ok ? dlt * dlt : 0.f;
    }
#pragma unroll
    for (int off = 1; off < 16; off <<= 1) m2 += __shfl_xor(m2, off, 64);
    const int m = mfirst + 4 * g + r;
    if (j == 0 && m < cout) {
      float* p = part + ((int64_t)m * T + tile_id) * 3;
      p[0] = cnt; p[1] = mu; p[2] = m2;
    }
  }
}

// PRO  : BN + ReLU of the input is applied on the fly: v = max(0, fma(x, fold[ch].x, fold[ch].y))
//        (the fused schedule's "BN-apply+ReLU feeding straight into the conv operand").
// STATS: the epilogue writes the output's per-tile BN statistics (see tile_stats).
template <int MT, int PPL, bool KSPLIT, bool PRO, bool STATS>
__global__ __launch_bounds__(256) void k_conv1x1_v3(
    const float* __restrict__ in, int64_t in_stride, const float* __restrict__ Wp, int Kpad,
    float* __restrict__ out, int64_t out_stride, int cin, int cout, int HW,
    const float2* __restrict__ fold, float* __restrict__ spart, int sT, int wk) {
  extern __shared__ float red[];
  // KSPLIT: the workgroup's waves form wp pixel groups of wk waves; a group shares one pixel tile
  // and splits K.  !KSPLIT: all waves share the pixel tile and split M (wk = 1).
  const int tid = threadIdx.x, lane = tid & 63, wave_all = tid >> 6, nw_all = blockDim.x >> 6;
  const int wave = KSPLIT ? wave_all % wk : wave_all, nw = KSPLIT ? wk : nw_all;
  const int wpid = KSPLIT ? wave_all / wk : 0, wp = KSPLIT ? nw_all / wk : 1;
  const int j = lane & 15, g = lane >> 4;
  const int tile = blockIdx.x * wp + wpid;
  const int q = tile * (16 * PPL) + PPL * j;
  const int img = blockIdx.z;
  const bool pix_ok = q < HW;
  const float* inb = in + (int64_t)img * in_stride + q;
  const int mbase = KSPLIT ? blockIdx.y * (MT * 16) : (blockIdx.y * nw + wave) * (MT * 16);
  const int M16 = (cout + 15) & ~15;
  const int nchunks = Kpad >> 4;
  const int cstart = KSPLIT ? wave : 0, cstep = KSPLIT ? nw : 1;
  const float* wrow = Wp + (int64_t)(mbase + j) * Kpad + 4 * g;
  const bool m_ok = mbase < M16;  // this wave's first tile exists in the packed rows

  f32x4 acc[MT][PPL];
#pragma unroll
  for (int a = 0; a < MT; ++a)
#pragma unroll
    for (int t = 0; t < PPL; ++t) acc[a][t] = (f32x4){0.f, 0.f, 0.f, 0.f};

  // Ring of D chunks in registers: chunk i+D is requested right after chunk i has been fed to
  // the MFMAs, so a wave keeps D-1..D chunks (activations + weights) in flight and a single wave
  // per SIMD can cover the HBM latency.  The loop body is branch free on purpose: every load is
  // unconditional with a clamped address (out-of-range channels read the last real channel and
  // meet zero weights; out-of-range pixels read pixel 0 and are never stored; ring slots past
  // the wave's last chunk get their weights zeroed), so the compiler's wait counters stay exact
  // and loads overlap the MFMAs.
  constexpr int D = 3;
  float buf[D][4][PPL];
  float4 wbuf[D][MT];
  float2 fbuf[D][4];  // PRO: folded BN of the slot's four channels, applied when the slot is used
  float keep[D];      // 0 for ring slots past the wave's last chunk
  const float* inq = in + (int64_t)img * in_stride + (pix_ok ? q : 0);
  const int nmy = (m_ok && cstart < nchunks) ? (nchunks - cstart + cstep - 1) / cstep : 0;  // chunks of this wave
  // nothing in here may consume a loaded value: the loads must stay in flight
  auto load_chunk = [&](int i, float(&v)[4][PPL], float4(&w4)[MT], float2(&f)[4], float& kp) {
    const bool valid = i < nmy;
    kp = valid ? 1.f : 0.f;
    const int ch0 = (cstart + (valid ? i : 0) * cstep) * 16;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int ch = min(ch0 + 4 * ks + g, cin - 1);
      if (PPL == 4) {
        const float4 t = ldg4(inq + (int64_t)ch * HW);
        v[ks][0] = t.x; v[ks][1 % PPL] = t.y; v[ks][2 % PPL] = t.z; v[ks][3 % PPL] = t.w;
      } else {
        v[ks][0] = inq[(int64_t)ch * HW];
      }
      if (PRO) f[ks] = fold[ch];
    }
#pragma unroll
    for (int a = 0; a < MT; ++a) {
      // M-tiles past the padded output-channel count read tile 0's rows; they are never stored
      const int row = (mbase + a * 16 < M16) ? mbase + a * 16 + j : j;
      w4[a] = ldg4(Wp + (int64_t)row * Kpad + 4 * g + ch0);
    }
  };

  if (nmy > 0) {  // uniform per wave
#pragma unroll
    for (int d = 0; d < D; ++d) load_chunk(d, buf[d], wbuf[d], fbuf[d], keep[d]);
    for (int base = 0; base < nmy; base += D) {
#pragma unroll
      for (int d = 0; d < D; ++d) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          float bv[PPL];
#pragma unroll
          for (int t = 0; t < PPL; ++t)
            bv[t] = PRO ? fmaxf(__fmaf_rn(buf[d][ks][t], fbuf[d][ks].x, fbuf[d][ks].y), 0.f) : buf[d][ks][t];
#pragma unroll
          for (int a = 0; a < MT; ++a) {
            const float wa = elem(wbuf[d][a], ks) * keep[d];
#pragma unroll
            for (int t = 0; t < PPL; ++t) {
              acc[a][t] = mfma16(wa, bv[t], acc[a][t]);
            }
          }
        }
        // keep the refill of this slot here, D chunks ahead of its use (the scheduler would
        // otherwise sink the loads to just before they are consumed)
        __builtin_amdgcn_sched_barrier(0);
        load_chunk(base + d + D, buf[d], wbuf[d], fbuf[d], keep[d]);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }

  if (KSPLIT) ksplit_reduce<MT, PPL>(acc, red + (size_t)wpid * MT * PPL * (nw - 1) * 256, wave, lane, nw);

  const int tiles_per_img = (HW + 16 * PPL - 1) / (16 * PPL);
  const int tile_px = min(16 * PPL, HW - tile * (16 * PPL));
#pragma unroll
  for (int a = 0; a < MT; ++a) {
    if (KSPLIT && a % nw != wave) continue;  // after the reduction M-tile a lives in wave a % nw
    if (mbase + a * 16 >= M16) continue;
    if (STATS)
      if (tile_px > 0)
        tile_stats<PPL>(acc[a], pix_ok, (float)tile_px, mbase + a * 16, cout, spart, sT,
                        img * tiles_per_img + tile);
    if (pix_ok) {
      float* ob = out + (int64_t)img * out_stride + q;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int m = mbase + a * 16 + 4 * g + r;
        if (m < cout) {
          if (PPL == 4)
            *reinterpret_cast<float4*>(ob + (int64_t)m * HW) =
                make_float4(acc[a][0][r], acc[a][1 % PPL][r], acc[a][2 % PPL][r], acc[a][3 % PPL][r]);
          else
            ob[(int64_t)m * HW] = acc[a][0][r];
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------- 3x3, fwd/dgrad
//
// The workgroup owns 64 consecutive pixels of one image.  ALL input channels of that pixel
// range plus one image row of halo on both sides are staged in LDS once, with flat pixel
// indexing (origin 4 pixels before the halo so every row of taps starts 16-byte aligned).
// For tap row di a lane reads its 4 pixels and the two neighbours once; the three taps dj
// are register selections of those 6 values.  Image top/bottom come out of the zero fill
// of flat indices outside [0, HW); left/right edges only ever touch the two neighbour reads
// (W is a multiple of 4), which are masked.  Waves split K (forward: 9*B long K, k outputs)
// or M (data gradient: k*9 short K, B outputs) as in the 1x1 kernel; packed weights come
// from L2, 16 bytes per lane per (tap, chunk).
template <int MT, bool KSPLIT, bool PRO, bool STATS>
__global__ __launch_bounds__(256) void k_conv3x3_v3(
    const float* __restrict__ in, int64_t in_stride, const float* __restrict__ Wp, int Mpad,
    int Kpad, float* __restrict__ out, int64_t out_stride, int cin, int cout, int H, int W, int CS,
    const float2* __restrict__ fold, float* __restrict__ spart, int sT) {
  extern __shared__ float lds[];
  const int HW = H * W;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nthr = blockDim.x, nw = nthr >> 6;
  const int j = lane & 15, g = lane >> 4;
  const int q0 = blockIdx.x * 64, img = blockIdx.z;
  const int origin = q0 - W - 4;
  const int seg4 = (64 + 2 * W + 8) >> 2;
  const int pw = 4 * j, q = q0 + pw;
  const int wc = q % W;
  const bool maskL = wc == 0, maskR = wc + 3 == W - 1;
  const float* inb = in + (int64_t)img * in_stride;
  const int mbase = KSPLIT ? blockIdx.y * (MT * 16) : (blockIdx.y * nw + wave) * (MT * 16);
  const int nchunks = Kpad >> 4;
  const int cstart = KSPLIT ? wave : 0, cstep = KSPLIT ? nw : 1;

  // Staging: U independent 16-byte loads per thread are issued back to back (clamped addresses,
  // no branches, so they are all in flight together), then transformed and stored.
  const int rows = (cin + 3) & ~3;  // staged channel rows (tail rows zero)
  const int total = rows * seg4;
  constexpr int U = 8;
  for (int base = 0; base < total; base += nthr * U) {
    float4 v[U];
    float2 f[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int idx = base + u * nthr + tid;
      const int row = min(idx / seg4, cin - 1);
      const int qq = origin + 4 * (idx % seg4);
      v[u] = ldg4(inb + (int64_t)row * HW + min(max(qq, 0), HW - 4));
      if (PRO) f[u] = fold[row];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int idx = base + u * nthr + tid;
      const int row = idx / seg4, c4 = idx - row * seg4;
      const int qq = origin + 4 * c4;
      const bool ok = row < cin && qq >= 0 && qq < HW;
      float4 x = v[u];
      if (PRO) {  // BN + ReLU on the way in; the zero padding stays zero
        x.x = fmaxf(__fmaf_rn(x.x, f[u].x, f[u].y), 0.f); x.y = fmaxf(__fmaf_rn(x.y, f[u].x, f[u].y), 0.f);
        x.z = fmaxf(__fmaf_rn(x.z, f[u].x, f[u].y), 0.f); x.w = fmaxf(__fmaf_rn(x.w, f[u].x, f[u].y), 0.f);
      }
      if (!ok) x = zero4();
      if (idx < total) *reinterpret_cast<float4*>(&lds[row * CS + 4 * c4]) = x;
    }
  }
  __syncthreads();

  f32x4 acc[MT][4];
#pragma unroll
  for (int a = 0; a < MT; ++a)
#pragma unroll
    for (int t = 0; t < 4; ++t) acc[a][t] = (f32x4){0.f, 0.f, 0.f, 0.f};

  if (mbase < Mpad) {
    for (int ci = cstart; ci < nchunks; ci += cstep) {
      const int c0 = ci * 16;
      const int nks = min(4, (cin - c0 + 3) >> 2);
      float4 w4[9][MT];
#pragma unroll
      for (int t = 0; t < 9; ++t)
#pragma unroll
        for (int a = 0; a < MT; ++a)
          w4[t][a] = (mbase + a * 16 < Mpad)
                         ? ldg4(Wp + ((int64_t)t * Mpad + mbase + a * 16 + j) * Kpad + c0 + 4 * g)
                         : zero4();
#pragma unroll
      for (int di = -1; di <= 1; ++di) {
        const int base = pw + 4 + W + di * W;
        float4 V[4];
        float eL[4], eR[4];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          if (ks < nks) {
            const float* rowp = &lds[(c0 + 4 * ks + g) * CS + base];
            V[ks] = *reinterpret_cast<const float4*>(rowp);
            eL[ks] = maskL ? 0.f : rowp[-1];
            eR[ks] = maskR ? 0.f : rowp[4];
          } else {
            V[ks] = zero4(); eL[ks] = 0.f; eR[ks] = 0.f;
          }
        }
#pragma unroll
        for (int dj = -1; dj <= 1; ++dj) {
          const int t = (di + 1) * 3 + (dj + 1);
#pragma unroll
          for (int ks = 0; ks < 4; ++ks) {
            if (ks < nks) {
              const float b0 = dj < 0 ? eL[ks] : (dj == 0 ? V[ks].x : V[ks].y);
              const float b1 = dj < 0 ? V[ks].x : (dj == 0 ? V[ks].y : V[ks].z);
              const float b2 = dj < 0 ? V[ks].y : (dj == 0 ? V[ks].z : V[ks].w);
              const float b3 = dj < 0 ? V[ks].z : (dj == 0 ? V[ks].w : eR[ks]);
#pragma unroll
              for (int a = 0; a < MT; ++a) {
                const float wa = elem(w4[t][a], ks);
                acc[a][0] = mfma16(wa, b0, acc[a][0]);
                acc[a][1] = mfma16(wa, b1, acc[a][1]);
                acc[a][2] = mfma16(wa, b2, acc[a][2]);
                acc[a][3] = mfma16(wa, b3, acc[a][3]);
              }
            }
          }
        }
      }
    }
  }

  if (KSPLIT) ksplit_reduce<MT, 4>(acc, lds, wave, lane, nw);  // reuses the tile's LDS (barrier inside)

  const int tile_px = min(64, HW - q0);
#pragma unroll
  for (int a = 0; a < MT; ++a) {
    if (KSPLIT && a % nw != wave) continue;
    if (mbase + a * 16 >= Mpad) continue;
    if (STATS)
      tile_stats<4>(acc[a], q < HW, (float)tile_px, mbase + a * 16, cout, spart, sT,
                    img * gridDim.x + blockIdx.x);
    if (q < HW) {
      float* ob = out + (int64_t)img * out_stride + q;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int m = mbase + a * 16 + 4 * g + r;
        if (m < cout)
          *reinterpret_cast<float4*>(ob + (int64_t)m * HW) =
              make_float4(acc[a][0][r], acc[a][1][r], acc[a][2][r], acc[a][3][r]);
      }
    }
  }
}

// ------------------------------------------------------------------------------- 3x3, persistent
//
// Second 3x3 kernel, for image widths 8, 16, 32 with a multiple of 64 pixels per image and shapes
// where all packed weights of a wave fit its registers (MT M-tiles x NCH 16-channel chunks x 9
// taps: the forward 3x3 with k <= 16 outputs from B <= 48 inputs, and its data gradient).
// Differences from k_conv3x3_v3:
//   * a workgroup walks over several 64-pixel tiles (whole image rows); the next tile's rows are
//     requested from HBM before the current tile's MFMAs are issued and stored to the other LDS
//     buffer after them, so load latency, BN+ReLU staging and matrix work overlap inside one
//     workgroup (one barrier per tile);
//   * the four waves split the tile's pixels (16 each) instead of K or M: all four SIMDs work, no
//     cross-wave reduction, and the weights are read from L2 once per workgroup, not per tile;
//   * the image width is a template parameter and every staged image row keeps a 4-float zero gap
//     in front of it, so a tap is one LDS read at a compile-time offset from a single per-lane
//     base -- no edge masks and no address arithmetic between the MFMAs;
//   * two interleaved accumulators per M-tile break the MFMA dependence chain.
// LDS is addressed through lds[] with integer offsets only (generic pointers to LDS must not be
// formed here: loads through them become flat instructions).
// Workgroup b takes tiles of its own contiguous range (consecutive workgroups sit on different
// XCDs: each XCD's workgroups share halo rows through that XCD's L2).
template <int MT, int NCH, int W, bool PRO, bool STATS>
__global__ __launch_bounds__(256) void k_conv3x3_v4(
    const float* __restrict__ in, int64_t in_stride, const float* __restrict__ Wp, int Mpad,
    int Kpad, float* __restrict__ out, int64_t out_stride, int cin, int cout, int H,
    const float2* __restrict__ fold, float* __restrict__ spart, int sT, int tiles_per_img,
    int total_tiles) {
  extern __shared__ float lds[];
  constexpr int ROWS = NCH * 16;             // staged channel planes
  constexpr int RW = W + 4, TR = 64 / W;     // LDS pitch of an image row; image rows per tile
  constexpr int NR = TR + 2, W4 = W / 4;     // staged image rows (one of halo above and below)
  constexpr int CS = 144;                    // plane pitch (>= NR*RW; 144 % 32 == 16: the four planes
                                             // of a B-operand read fall on disjoint banks)
  static_assert(NR * RW <= CS, "plane pitch");
  constexpr int PER_PLANE = NR * W4, TOTAL = ROWS * PER_PLANE, U = (TOTAL + 255) / 256;
  const int HW = H * W;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j = lane & 15, g = lane >> 4;
  // two tile buffers, then [2][4 waves][MT*16][3].  Each buffer ends with 4 zero floats: the right
  // neighbour of the last staged row of the last plane (for the other planes it is the next
  // plane's leading gap).
  constexpr int BUF = ROWS * CS + 4, SST0 = 2 * BUF;

  // tiles of this workgroup: XCD x = b % 8 owns tiles [x*tpx, (x+1)*tpx), its workgroups stride it
  const int G = gridDim.x, tpx = (total_tiles + 7) >> 3, wgx = G >> 3;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int t_lo = xcd * tpx, t_hi = min(total_tiles, t_lo + tpx);
  int tile = t_lo + slot;
  if (tile >= t_hi) return;  // uniform for the workgroup

  // staging slots of this thread: the same (plane, image row, 4-pixel column) in every tile
  int sch[U], sry[U], sgo[U], slo[U];  // channel, staged row, offset in the image row, LDS offset
  float2 sfold[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int idx = min(u * 256 + tid, TOTAL - 1);
    sch[u] = idx / PER_PLANE;
    const int rem = idx - sch[u] * PER_PLANE;
    sry[u] = rem / W4;
    sgo[u] = 4 * (rem - sry[u] * W4);
    slo[u] = sch[u] * CS + sry[u] * RW + 4 + sgo[u];
    sfold[u] = (PRO && sch[u] < cin) ? fold[sch[u]] : make_float2(1.f, 0.f);
  }
  auto request = [&](int tl, float4(&v)[U]) {
    const int img = tl / tiles_per_img, y0 = (tl - img * tiles_per_img) * TR;
    const float* inb = in + (int64_t)img * in_stride;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int y = min(max(y0 - 1 + sry[u], 0), H - 1);
      v[u] = ldg4(inb + (int64_t)min(sch[u], cin - 1) * HW + y * W + sgo[u]);
    }
  };
  auto deposit = [&](int tl, const float4(&v)[U], int boff) {
    const int img = tl / tiles_per_img, y0 = (tl - img * tiles_per_img) * TR;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int y = y0 - 1 + sry[u];
      float4 x = v[u];
      if (PRO) {
        x.x = fmaxf(__fmaf_rn(x.x, sfold[u].x, sfold[u].y), 0.f); x.y = fmaxf(__fmaf_rn(x.y, sfold[u].x, sfold[u].y), 0.f);
        x.z = fmaxf(__fmaf_rn(x.z, sfold[u].x, sfold[u].y), 0.f); x.w = fmaxf(__fmaf_rn(x.w, sfold[u].x, sfold[u].y), 0.f);
      }
      if (!(sch[u] < cin && y >= 0 && y < H)) x = zero4();  // channel tail, rows above / below the image
      if (u * 256 + tid < TOTAL) *reinterpret_cast<float4*>(&lds[boff + slo[u]]) = x;
    }
  };

  // the first tile's rows are requested first (longest latency); the weights and the zero fill
  // are issued while they are in flight
  float4 v0[U];
  request(tile, v0);
  // packed weights of every tap, chunk and M-tile: 16 bytes per lane each, kept in registers
  float4 w4[9][NCH][MT];
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int ci = 0; ci < NCH; ++ci)
#pragma unroll
      for (int a = 0; a < MT; ++a)
        w4[t][ci][a] = (a * 16 < Mpad && ci * 16 < Kpad)
                           ? ldg4(Wp + ((int64_t)t * Mpad + a * 16 + j) * Kpad + ci * 16 + 4 * g)
                           : zero4();

  // the gaps between staged rows (and the pitch padding) stay zero for the whole kernel
  for (int i = tid; i < 2 * BUF / 4; i += 256) *reinterpret_cast<float4*>(&lds[4 * i]) = zero4();

  __syncthreads();  // zero fill done before the first rows land
  deposit(tile, v0, 0);
  __syncthreads();

  // this lane's pixel inside the tile and its LDS base: plane g, staged row 1 + p / W, column 4 + p % W
  const int p = 16 * wave + j;
  const int lane_base = g * CS + (p / W + 1) * RW + 4 + (p % W);

  for (int it = 0; tile < t_hi; ++it, tile += wgx) {
    const int cur = it & 1;
    const int boff = cur * BUF;
    const int nxt = tile + wgx;
    const bool more = nxt < t_hi;
    float4 vn[U];
    if (more) request(nxt, vn);

    f32x4 acc[MT][2];
#pragma unroll
    for (int a = 0; a < MT; ++a) { acc[a][0] = (f32x4){0.f, 0.f, 0.f, 0.f}; acc[a][1] = (f32x4){0.f, 0.f, 0.f, 0.f}; }
#pragma unroll
    for (int ci = 0; ci < NCH; ++ci) {
#pragma unroll
      for (int di = -1; di <= 1; ++di) {
#pragma unroll
        for (int dj = -1; dj <= 1; ++dj) {
          const int t = (di + 1) * 3 + (dj + 1);
#pragma unroll
          for (int ks = 0; ks < 4; ++ks) {
            const float b = lds[boff + lane_base + (ci * 16 + 4 * ks) * CS + di * RW + dj];
#pragma unroll
            for (int a = 0; a < MT; ++a) {
              acc[a][ks & 1] = mfma16(elem(w4[t][ci][a], ks), b, acc[a][ks & 1]);
            }
          }
        }
      }
    }

    // epilogue of this wave's 16 pixels (all inside the image: HW is a multiple of 64)
    const int img = tile / tiles_per_img, q = (tile - img * tiles_per_img) * 64 + p;
#pragma unroll
    for (int a = 0; a < MT; ++a) {
      if (a * 16 >= Mpad) continue;
      float v[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) v[r] = acc[a][0][r] + acc[a][1][r];
      if (STATS) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          float s = v[r];
#pragma unroll
          for (int off = 1; off < 16; off <<= 1) s += __shfl_xor(s, off, 64);
          const float mu = s * (1.0f / 16.0f);
          const float dlt = v[r] - mu;
          float m2 = dlt * dlt;
#pragma unroll
          for (int off = 1; off < 16; off <<= 1) m2 += __shfl_xor(m2, off, 64);
          if (j == 0) {
            float* ps = &lds[SST0 + (((cur * 4 + wave) * (MT * 16)) + a * 16 + 4 * g + r) * 3];
            ps[0] = 16.f; ps[1] = mu; ps[2] = m2;
          }
        }
      }
      float* ob = out + (int64_t)img * out_stride + q;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int m = a * 16 + 4 * g + r;
        if (m < cout) ob[(int64_t)m * HW] = v[r];
      }
    }

    if (more) deposit(nxt, vn, (cur ^ 1) * BUF);
    __syncthreads();
    if (STATS && wave == 0 && lane < MT * 16 && lane < cout) {
      const float* ps = &lds[SST0 + ((cur * 4) * (MT * 16) + lane) * 3];
      Stat3 r{ps[0], ps[1], ps[2]};
#pragma unroll
      for (int w = 1; w < 4; ++w) {
        const float* pw = ps + w * (MT * 16) * 3;
        r = stat_combine(r, Stat3{pw[0], pw[1], pw[2]});
      }
      float* o = spart + ((int64_t)lane * sT + tile) * 3;
      o[0] = r.c; o[1] = r.m; o[2] = r.m2;
    }
  }
}

// A pending sum of partials carried out by extra workgroups of a weight-gradient launch (the
// workgroups with blockIdx.x >= gx_main): kind 1 is k_sum_partials' job, kind 2 k_sum_wgrad3x3's,
// with the same grouping and order of additions, so the sums have the same bits either way.
struct SumRole {
  int kind, wgs;  // kind 0: none; wgs: workgroups the sum needs
  const float* part;
  float* out;
  int splits, G, per;
  long long count;  // elements of one partial
  int gy, gz, mtw, ctw, cin, cout;
};

__device__ __forceinline__ void sum_role(const SumRole& sr, int wg) {
  extern __shared__ float sh[];  // the launch's dynamic LDS (every weight-gradient launch has >= 1 KB)
  const int epb = 256 / sr.G;
  const int le = threadIdx.x % epb, grp = threadIdx.x / epb;
  const long long f = (long long)wg * epb + le;
  float s = 0.f;
  if (f < sr.count) {
    int i = grp * sr.per;
    const int end = min(sr.splits, i + sr.per);
    for (; i + 8 <= end; i += 8) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = sr.part[(long long)(i + u) * sr.count + f];
#pragma unroll
      for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (; i < end; ++i) s += sr.part[(long long)i * sr.count + f];
  }
  sh[threadIdx.x] = s;
  __syncthreads();
  if (grp == 0 && f < sr.count) {
    float t = sh[le];
    for (int g = 1; g < sr.G; ++g) t += sh[g * epb + le];
    if (sr.kind == 1) {
      sr.out[f] = t;
    } else {
      const int NT = sr.mtw * sr.ctw * 9;
      const int rr = (int)(f & 3), lane = (int)((f >> 2) & 63);
      const long long tl = f >> 8;
      const int tile = (int)(tl % NT), blk = (int)(tl / NT);
      const int yb = blk % sr.gy, z = blk / sr.gy;
      const int tap = tile % 9, y = (tile / 9) % sr.ctw, x = tile / (9 * sr.ctw);
      const int m = z * (sr.mtw * 16) + x * 16 + 4 * (lane >> 4) + rr;
      const int c = yb * (sr.ctw * 16) + y * 16 + (lane & 15);
      if (m < sr.cout && c < sr.cin) sr.out[((long long)m * sr.cin + c) * 9 + tap] = t;
    }
  }
}

// Adds the accumulators of the four waves of a workgroup, a0 + (a1 + (a2 + a3)) element by
// element: every wave writes its NT tiles to its own LDS region (4 * NT * 256 floats in all),
// then wave w adds up the tiles t with t % 4 == w, which it alone holds afterwards.
template <int NT>
__device__ __forceinline__ void reduce_waves_split(f32x4 (&acc)[NT], float* buf, int wave, int lane) {
#pragma unroll
  for (int t = 0; t < NT; ++t)
    *reinterpret_cast<float4*>(&buf[((wave * NT + t) * 64 + lane) * 4]) =
        make_float4(acc[t][0], acc[t][1], acc[t][2], acc[t][3]);
  __syncthreads();
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    if ((t & 3) != wave) continue;
    float4 s = *reinterpret_cast<const float4*>(&buf[((3 * NT + t) * 64 + lane) * 4]);
#pragma unroll
    for (int w = 2; w >= 0; --w) {
      const float4 v = *reinterpret_cast<const float4*>(&buf[((w * NT + t) * 64 + lane) * 4]);
      s.x = v.x + s.x; s.y = v.y + s.y; s.z = v.z + s.z; s.w = v.w + s.w;
    }
    acc[t] = (f32x4){s.x, s.y, s.z, s.w};
  }
}

// ------------------------------------------------------------------------------- 1x1 wgrad
//
// dW[m][c] = sum_{n,q} g[n][m][q] a[n][c][q].  A "step" is 16 pixels: lane (r, kk) loads pixels
// 4kk..4kk+3 of row r of both operands (16 bytes each) and issues 4 K-steps.  The four waves of
// a workgroup take alternate steps (together 256 contiguous bytes per row), keep all MTW x CTW
// tiles in registers, and are summed in LDS at the end (each wave a quarter of the tiles, which
// it then stores); the workgroup writes one partial.
struct Wg1Args {
  const float* a; int64_t a_stride; const float* g; int64_t g_stride; float* part;
  int cin, cout, HW, spi, total_steps, steps_per_wg;
  const float2* fold;
};

// the work of workgroup (bx, by, bz) of the 1x1 weight gradient's grid
template <int MTW, int CTW, bool PRO, int NST>
__device__ __forceinline__ void wgrad1x1_body(const Wg1Args& A, int bx, int by, int bz) {
  extern __shared__ float lds[];
  const float* __restrict__ a = A.a;
  const float* __restrict__ gout = A.g;
  float* __restrict__ part = A.part;
  const float2* __restrict__ fold = A.fold;
  const int64_t a_stride = A.a_stride, g_stride = A.g_stride;
  const int cin = A.cin, cout = A.cout, HW = A.HW, spi = A.spi, total_steps = A.total_steps, steps_per_wg = A.steps_per_wg;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 15, kk = lane >> 4;
  const int c0 = by * (CTW * 16), m0 = bz * (MTW * 16);
  const int s_begin = bx * steps_per_wg, s_end = min(total_steps, s_begin + steps_per_wg);

  f32x4 acc[MTW * CTW];
#pragma unroll
  for (int t = 0; t < MTW * CTW; ++t) acc[t] = (f32x4){0.f, 0.f, 0.f, 0.f};

  float2 fl[CTW];  // PRO: BN+ReLU of the activation operand, one channel per lane and c-tile
#pragma unroll
  for (int y = 0; y < CTW; ++y) {
    const int c = c0 + y * 16 + r;
    fl[y] = (PRO && c < cin) ? fold[c] : make_float2(1.f, 0.f);
  }

  // Operands are requested NST steps ahead into NST register stages (loop unrolled by NST so the
  // stages are indexed statically).  Every load is unconditional at an address clamped into
  // the tensors, so a step waits for its own operands only; what a clamped load stands in for
  // (a step past the range, pixels past the image) is zeroed when the stage is consumed, and
  // rows past cout / cin are computed on repeated data and never stored.
  const float* grow[MTW];
  const float* arow[CTW];
#pragma unroll
  for (int x = 0; x < MTW; ++x) grow[x] = gout + (int64_t)min(m0 + x * 16 + r, cout - 1) * HW;
#pragma unroll
  for (int y = 0; y < CTW; ++y) arow[y] = a + (int64_t)min(c0 + y * 16 + r, cin - 1) * HW;
  auto request = [&](int s, float4(&A)[MTW], float4(&Bv)[CTW]) {
    const int sc = min(s, total_steps - 1);
    const int img = sc / spi, q = min((sc - img * spi) * 16 + 4 * kk, HW - 4);  // HW % 4 == 0
#pragma unroll
    for (int x = 0; x < MTW; ++x) A[x] = ldg4(grow[x] + (int64_t)img * g_stride + q);
#pragma unroll
    for (int y = 0; y < CTW; ++y) Bv[y] = ldg4(arow[y] + (int64_t)img * a_stride + q);
  };
  auto step = [&](int s, float4(&A)[MTW], float4(&Bv)[CTW]) {
    const int img = s / spi, q = (s - img * spi) * 16 + 4 * kk;
    const bool ok = s < s_end && q < HW;
    float4 Au[MTW], Bu[CTW];
#pragma unroll
    for (int x = 0; x < MTW; ++x) Au[x] = ok ? A[x] : zero4();
#pragma unroll
    for (int y = 0; y < CTW; ++y) {
      Bu[y] = Bv[y];
      if (PRO) {
        Bu[y].x = fmaxf(__fmaf_rn(Bu[y].x, fl[y].x, fl[y].y), 0.f);
        Bu[y].y = fmaxf(__fmaf_rn(Bu[y].y, fl[y].x, fl[y].y), 0.f);
        Bu[y].z = fmaxf(__fmaf_rn(Bu[y].z, fl[y].x, fl[y].y), 0.f);
        Bu[y].w = fmaxf(__fmaf_rn(Bu[y].w, fl[y].x, fl[y].y), 0.f);
      }
    }
    request(s + 4 * NST, A, Bv);  // this stage's next use
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
      for (int x = 0; x < MTW; ++x)
#pragma unroll
        for (int y = 0; y < CTW; ++y) acc[x * CTW + y] = mfma16(elem(Au[x], e), elem(Bu[y], e), acc[x * CTW + y]);
  };
  {
    float4 As[NST][MTW], Bs[NST][CTW];
    const int s0 = s_begin + wave;
#pragma unroll
    for (int i = 0; i < NST; ++i) request(s0 + 4 * i, As[i], Bs[i]);
    for (int s = s0; s < s_end; s += 4 * NST) {
#pragma unroll
      for (int i = 0; i < NST; ++i)
        if (i == 0 || s + 4 * i < s_end) step(s + 4 * i, As[i], Bs[i]);
    }
  }

  reduce_waves_split<MTW * CTW>(acc, lds, wave, lane);
  float* pb = part + (int64_t)bx * cout * cin;
#pragma unroll
  for (int x = 0; x < MTW; ++x)
#pragma unroll
    for (int y = 0; y < CTW; ++y) {
      if (((x * CTW + y) & 3) != wave) continue;  // the wave that holds this tile's sum stores it
      const int c = c0 + y * 16 + r;
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        const int m = m0 + x * 16 + 4 * kk + rr;
        if (m < cout && c < cin) pb[(int64_t)m * cin + c] = acc[x * CTW + y][rr];
      }
    }
}

template <int MTW, int CTW, bool PRO>
__global__ __launch_bounds__(256) void k_wgrad1x1_fast(Wg1Args A, SumRole sr, int gx_main) {
  if ((int)blockIdx.x >= gx_main) {  // extra workgroups: a pending sum of another partial buffer
    const int wg = (((int)blockIdx.x - gx_main) * gridDim.y + blockIdx.y) * gridDim.z + blockIdx.z;
    if (wg < sr.wgs) sum_role(sr, wg);
    return;
  }
  wgrad1x1_body<MTW, CTW, PRO, 2>(A, blockIdx.x, blockIdx.y, blockIdx.z);
}

// ------------------------------------------------------------------------------- 3x3 wgrad
//
// dW[m][c][t] = sum_{n,q} g[n][m][q] a[n][c][q+shift(t)].  The workgroup stages CTW*16 channels
// of a pixel range (plus halo, as in the forward kernel) in LDS; the MTW x CTW x 9 accumulator
// tiles are split over the four waves and every wave takes all 16-pixel steps of the range.
// g comes straight from HBM (16 bytes per lane and step).
struct Wg3Args {
  const float* a; int64_t a_stride; const float* g; int64_t g_stride; float* part;
  int cin, cout, H, W, tiles_per_img, nms, PA;
  const float2* fold;
};

// the work of workgroup (bx, by, bz) of the 3x3 weight gradient's grid (gy x gz channel groups)
template <int MTW, int CTW, bool PRO>
__device__ __forceinline__ void wgrad3x3_body(const Wg3Args& A3, int bx, int by, int bz, int gy, int gz) {
  extern __shared__ float lds[];
  const float* __restrict__ a = A3.a;
  const float* __restrict__ gout = A3.g;
  float* __restrict__ part = A3.part;
  const float2* __restrict__ fold = A3.fold;
  const int64_t a_stride = A3.a_stride, g_stride = A3.g_stride;
  const int cin = A3.cin, cout = A3.cout, H = A3.H, W = A3.W, tiles_per_img = A3.tiles_per_img, nms = A3.nms, PA = A3.PA;
  const int HW = H * W;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 15, kk = lane >> 4;
  constexpr int CB = CTW * 16, NT = MTW * CTW * 9;
  const int TPIX = 4 * nms * 16;
  const int img = bx / tiles_per_img, q0 = (bx - img * tiles_per_img) * TPIX;
  const int c0 = by * CB, m0 = bz * (MTW * 16);
  const int origin = q0 - W - 4;
  const int seg4 = (TPIX + 2 * W + 8) >> 2;
  const float* ab = a + (int64_t)img * a_stride;
  const float* gb = gout + (int64_t)img * g_stride;

  // The tile is staged progressively: first the columns the first 64-pixel step needs (its pixels
  // plus the halo on both sides), then 64 more columns per step, loaded into registers before the
  // MFMAs of the current step are issued and written to LDS after them, so the HBM latency of
  // step ms+1's activations is covered by step ms's matrix work.
  auto bnrelu = [&](float4 v, float2 f) {
    v.x = fmaxf(__fmaf_rn(v.x, f.x, f.y), 0.f); v.y = fmaxf(__fmaf_rn(v.y, f.x, f.y), 0.f);
    v.z = fmaxf(__fmaf_rn(v.z, f.x, f.y), 0.f); v.w = fmaxf(__fmaf_rn(v.w, f.x, f.y), 0.f);
    return v;
  };
  // per-thread constants: thread (row group, float4 column) -> CTW rows, in every chunk
  const int prow = tid >> 4, pc4 = tid & 15;
  float2 pf[CTW];
#pragma unroll
  for (int u = 0; u < CTW; ++u) {
    pf[u] = make_float2(1.f, 0.f);
    if (PRO) pf[u] = fold[min(c0 + u * 16 + prow, cin - 1)];
  }
  const int seg0_4 = (64 + 2 * W + 8) >> 2;  // float4 columns of the first chunk
  if (seg0_4 <= 48) {
    // all of the first chunk's loads at once, unconditional at clamped addresses (conditional
    // loads are waited for one by one); what lies outside the image or the tensor is zeroed
    // when it is written to LDS
    // (threads past the chunk's last column repeat that column: same load, same store)
    float4 v0[CTW][3];
#pragma unroll
    for (int u = 0; u < CTW; ++u) {
      const float* src = ab + (int64_t)min(c0 + u * 16 + prow, cin - 1) * HW;
#pragma unroll
      for (int i = 0; i < 3; ++i)
        v0[u][i] = ldg4(src + min(max(origin + 4 * min(pc4 + 16 * i, seg0_4 - 1), 0), HW - 4));
    }
#pragma unroll
    for (int u = 0; u < CTW; ++u) {
      const int row = u * 16 + prow, ch = c0 + row;
#pragma unroll
      for (int i = 0; i < 3; ++i) {
        const int c4 = min(pc4 + 16 * i, seg0_4 - 1), qq = origin + 4 * c4;
        float4 v = v0[u][i];
        if (PRO) v = bnrelu(v, pf[u]);
        if (!(ch < cin && qq >= 0 && qq < HW)) v = zero4();
        *reinterpret_cast<float4*>(&lds[row * PA + 4 * c4]) = v;
      }
    }
  } else {
    for (int row = tid >> 4; row < CB; row += 16) {
      const int ch = c0 + row;
      const float* src = ab + (int64_t)ch * HW;
      float2 f = make_float2(1.f, 0.f);
      if (PRO && ch < cin) f = fold[ch];
      for (int c4 = tid & 15; c4 < seg0_4; c4 += 16) {
        const int qq = origin + 4 * c4;
        const bool ok = ch < cin && qq >= 0 && qq < HW;
        float4 v = ok ? ldg4(src + qq) : zero4();
        if (PRO && ok) v = bnrelu(v, f);
        *reinterpret_cast<float4*>(&lds[row * PA + 4 * c4]) = v;
      }
    }
  }
  __syncthreads();

  // The four waves split the NT accumulator tiles (contiguous ranges of (m-tile, c-tile, tap)), not
  // the pixels: every wave walks all 16-pixel steps of the tile and there is nothing to add
  // across waves at the end.  A tile's three horizontal taps share one LDS row read (16 bytes
  // plus the two edge elements).  The code of a wave's range is instantiated per wave so that
  // every tile index is static.
  constexpr int TPW = (NT + 3) / 4;
  f32x4 acc[TPW];
#pragma unroll
  for (int t = 0; t < TPW; ++t) acc[t] = (f32x4){0.f, 0.f, 0.f, 0.f};

  // gradient operand of the four steps of a pass (every wave loads all of them), one pass ahead;
  // loaded unconditionally at clamped addresses: pixels past the image are zeroed when the step
  // consumes them, rows past cout are never stored
  const float* grow[MTW];
#pragma unroll
  for (int x = 0; x < MTW; ++x) grow[x] = gb + (int64_t)min(m0 + x * 16 + r, cout - 1) * HW;
  float4 An[4][MTW];
#pragma unroll
  for (int sub = 0; sub < 4; ++sub)
#pragma unroll
    for (int x = 0; x < MTW; ++x) An[sub][x] = ldg4(grow[x] + min(q0 + sub * 16 + 4 * kk, HW - 4));

  for (int ms = 0; ms < nms; ++ms) {
    // request the next chunk: columns [64(ms+1) + 2W + 8, +64) of the tile
    float4 nxt[CTW];
    const bool more = ms + 1 < nms;
    const int ncol = 64 * (ms + 1) + 2 * W + 8 + 4 * pc4;  // column of this thread's float4
    const int nq = origin + ncol;
#pragma unroll
    for (int u = 0; u < CTW; ++u) {
      const int ch = min(c0 + u * 16 + prow, cin - 1);
      nxt[u] = ldg4(ab + (int64_t)ch * HW + min(max(nq, 0), HW - 4));
    }
    float4 A[4][MTW];
#pragma unroll
    for (int sub = 0; sub < 4; ++sub) {
      const bool in = q0 + (ms * 4 + sub) * 16 + 4 * kk < HW;
#pragma unroll
      for (int x = 0; x < MTW; ++x) A[sub][x] = in ? An[sub][x] : zero4();
    }
#pragma unroll
    for (int sub = 0; sub < 4; ++sub)
#pragma unroll
      for (int x = 0; x < MTW; ++x)
        An[sub][x] = ldg4(grow[x] + min(q0 + ((ms + 1) * 4 + sub) * 16 + 4 * kk, HW - 4));

    auto steps = [&](auto wv) {
      constexpr int WV = decltype(wv)::value;
      constexpr int T0 = WV * TPW, T1 = (T0 + TPW < NT) ? T0 + TPW : NT;
#pragma unroll
      for (int sub = 0; sub < 4; ++sub) {
        const int pw = (ms * 4 + sub) * 16 + 4 * kk, wc = (q0 + pw) % W;
        const bool maskL = wc == 0, maskR = wc + 3 == W - 1;
        float4 V = zero4();
        float eL = 0.f, eR = 0.f;
#pragma unroll
        for (int T = T0; T < T1; ++T) {
          const int x = T / (CTW * 9), y = (T / 9) % CTW, t = T % 9, di = t / 3 - 1, dj = t % 3 - 1;
          if (T == T0 || t % 3 == 0) {  // first tap of this row in the wave's range
            const int o = (y * 16 + r) * PA + pw + 4 + W + di * W;
            V = *reinterpret_cast<const float4*>(&lds[o]);
            eL = maskL ? 0.f : lds[o - 1];
            eR = maskR ? 0.f : lds[o + 4];
          }
          const float b0 = dj < 0 ? eL : (dj == 0 ? V.x : V.y);
          const float b1 = dj < 0 ? V.x : (dj == 0 ? V.y : V.z);
          const float b2 = dj < 0 ? V.y : (dj == 0 ? V.z : V.w);
          const float b3 = dj < 0 ? V.z : (dj == 0 ? V.w : eR);
          f32x4& d = acc[T - T0];
          d = mfma16(A[sub][x].x, b0, d);
          d = mfma16(A[sub][x].y, b1, d);
          d = mfma16(A[sub][x].z, b2, d);
          d = mfma16(A[sub][x].w, b3, d);
        }
      }
    };
    switch (wave) {
      case 0: steps(std::integral_constant<int, 0>{}); break;
      case 1: steps(std::integral_constant<int, 1>{}); break;
      case 2: steps(std::integral_constant<int, 2>{}); break;
      default: steps(std::integral_constant<int, 3>{}); break;
    }
    if (more) {
#pragma unroll
      for (int u = 0; u < CTW; ++u) {
        const int ch = c0 + u * 16 + prow;
        const bool okc = ch < cin && nq >= 0 && nq < HW;
        float4 v = nxt[u];
        if (PRO) v = bnrelu(v, pf[u]);
        if (!okc) v = zero4();
        *reinterpret_cast<float4*>(&lds[(u * 16 + prow) * PA + ncol]) = v;
      }
      __syncthreads();
    }
  }

  // the partial is stored in accumulator order (tile, lane, 4 rows): 16-byte stores, contiguous
  // across the wave; k_sum_wgrad3x3 adds the partials and puts the sums in OIHW order
  float* pb = part + (((int64_t)bx * gz + bz) * gy + by) * (NT * 256);
#pragma unroll
  for (int t = 0; t < TPW; ++t) {
    const int T = wave * TPW + t;
    if (T < NT)
      *reinterpret_cast<float4*>(&pb[(T * 64 + lane) * 4]) = make_float4(acc[t][0], acc[t][1], acc[t][2], acc[t][3]);
  }
}

template <int MTW, int CTW, bool PRO>
__global__ __launch_bounds__(256) void k_wgrad3x3_fast(Wg3Args A, SumRole sr, int gx_main) {
  if ((int)blockIdx.x >= gx_main) {  // extra workgroups: a pending sum of another partial buffer
    const int wg = (((int)blockIdx.x - gx_main) * gridDim.y + blockIdx.y) * gridDim.z + blockIdx.z;
    if (wg < sr.wgs) sum_role(sr, wg);
    return;
  }
  wgrad3x3_body<MTW, CTW, PRO>(A, blockIdx.x, blockIdx.y, blockIdx.z, gridDim.y, gridDim.z);
}

// One launch for the two weight gradients of a layer (they are independent of each other and of
// everything that follows them): a 1-D grid whose first n1 workgroups are the 1x1's (few and long,
// so they start first: 41.9 -> 38.4 us per launch on the first dense block of DenseNet-BC-100
// against the 3x3's first), the next n3 the 3x3's, then the BN backward reduction carried along
// (before the 3x3's it measured slower, after the sums the same; spread evenly among the weight
// gradients' workgroups, so that traffic and matrix work share every CU for the whole launch,
// 36.7 -> 44.1 us: a streaming workgroup takes the place of a second matrix one, and one wave per
// SIMD does not cover the operand latency), then the two pending sums.
// Three waves per SIMD asked of the register allocator: left alone it spends accumulation registers
// freely (139 + 52 on the k = 24 shapes) and two waves per SIMD do not cover the operand latency of
// the 1x1 role; 140 registers hold the same code without spilling.
template <int M1, int C1, int M3, int C3, bool PRO>
__global__ __launch_bounds__(256, 3) void k_wgrad_pair(Wg1Args A1, int gx1, int gy1, int gz1, int n1, Wg3Args A3, int gy3, int gz3,
                                                    int n3, SumRole s1, SumRole s3, BnBwdPartialArgs bn, int nbn) {
  int id = blockIdx.x;
  if (id < n1) {
    // Workgroups go to the 8 XCDs in turn (id % 8), each with an L2 of its own.  All the (c, m)
    // tile columns of one pixel range read the same gradient rows, and the m groups of a c column
    // the same feature rows: pixel range bx is given to XCD bx % 8 whole, so that these rows come
    // from HBM once and from that XCD's L2 afterwards (measured HBM bytes per launch 190 -> 176 MB
    // on DenseNet-BC-100's first block, 776 -> 562 MB on DenseNet-BC-250's).  n1 counts
    // ceil(gx1 / 8) ranges per XCD; the ids past the last range have no work.
    const int xcd = id & 7, slot = id >> 3, cols = gy1 * gz1;
    const int col = slot % cols, bx = (slot / cols) * 8 + xcd;
    if (bx >= gx1) return;
    // three operand stages beside the narrow 3x3 tiles of k = 12 nets (37.8 -> 37.5 us per launch on
    // the first dense block of DenseNet-BC-100), two beside the wide ones (157 against 162 us on
    // DenseNet-BC-250's, where the third stage's registers come out of the same two waves per SIMD)
    wgrad1x1_body<M1, C1, PRO, (M3 == 1 ? 3 : 2)>(A1, bx, col / gz1, col % gz1);
    return;
  }
  id -= n1;
  if (id < n3) {
    const int bz = id % gz3, by = (id / gz3) % gy3, bx = id / (gz3 * gy3);
    wgrad3x3_body<M3, C3, PRO>(A3, bx, by, bz, gy3, gz3);
    return;
  }
  id -= n3;
  if (id < nbn) {  // a BN+ReLU backward reduction of the main chain carried along
    bn_bwd_partial_body4(bn, id / bn.splits, id % bn.splits);
    return;
  }
  id -= nbn;
  if (id < s1.wgs) { sum_role(s1, id); return; }
  id -= s1.wgs;
  if (id < s3.wgs) sum_role(s3, id);
}

// Sum of the 3x3 weight-gradient partials.  A partial is gz*gy blocks of mtw*ctw*9 accumulator
// tiles in lane order (see k_wgrad3x3_fast); element f of a partial belongs to output
// (m, c, t) computed below.  256 threads = G groups x 256/G elements: group g adds partials
// [g*per, (g+1)*per) of its elements in order, the groups are added in order through LDS.
__global__ __launch_bounds__(256) void k_sum_wgrad3x3(const float* __restrict__ part, int splits, int gy, int gz,
                                                      int mtw, int ctw, int cin, int cout,
                                                      float* __restrict__ out, int G, int per) {
  __shared__ float sh[256];
  const int NT = mtw * ctw * 9;
  const int64_t F = (int64_t)gz * gy * NT * 256;
  const int epb = 256 / G;
  const int le = threadIdx.x % epb, grp = threadIdx.x / epb;
  const int64_t f = (int64_t)blockIdx.x * epb + le;
  float s = 0.f;
  if (f < F) {
    int i = grp * per;
    const int end = min(splits, i + per);
    for (; i + 8 <= end; i += 8) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = part[(int64_t)(i + u) * F + f];
#pragma unroll
      for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (; i < end; ++i) s += part[(int64_t)i * F + f];
  }
  sh[threadIdx.x] = s;
  __syncthreads();
  if (grp == 0 && f < F) {
    float t = sh[le];
    for (int g = 1; g < G; ++g) t += sh[g * epb + le];
    const int rr = (int)(f & 3), lane = (int)((f >> 2) & 63);
    const int64_t tl = f >> 8;
    const int tile = (int)(tl % NT), blk = (int)(tl / NT);
    const int yb = blk % gy, z = blk / gy;
    const int tap = tile % 9, y = (tile / 9) % ctw, x = tile / (9 * ctw);
    const int m = z * (mtw * 16) + x * 16 + 4 * (lane >> 4) + rr;
    const int c = yb * (ctw * 16) + y * 16 + (lane & 15);
    if (m < cout && c < cin) out[((int64_t)m * cin + c) * 9 + tap] = t;
  }
}

// fold[ch] = (gamma*istd, beta - mean*gamma*istd) for nch channels.  Channels in
// [fresh_lo, fresh_hi) only have partial statistics ([T][3] each): they are merged here and
// their mean / inverse std stored for the backward pass.  One workgroup per channel, 256 threads
// like the BN kernels' own merge, so both give the same bits from the same partials.
__global__ __launch_bounds__(256) void k_bn_fold(const float* __restrict__ gamma, const float* __restrict__ beta,
                                                float* mean, float* istd, const float* __restrict__ part,
                                                int T, int fresh_lo, int fresh_hi, float eps,
                                                float2* __restrict__ fold) {
  __shared__ float sh[12];
  const int ch = blockIdx.x;
  // requested before the merge: behind its barriers they would cost a second memory round trip
  const float ga = gamma[ch], be = beta[ch];
  float mu, is;
  if (ch >= fresh_lo && ch < fresh_hi) {
    const Stat3 r = stat_merge_block(part + (int64_t)(ch - fresh_lo) * T * 3, T, sh);
    mu = r.m;
    is = bn_istd(r.m2, r.c, eps);
    if (threadIdx.x == 0) { mean[ch] = mu; istd[ch] = is; }
  } else {
    mu = mean[ch];
    is = istd[ch];
  }
  if (threadIdx.x == 0) {
    float sc, sf;
    bn_fold(ga, be, mu, is, sc, sf);
    fold[ch] = make_float2(sc, sf);
  }
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int pad4mod32(int v) {  // smallest pitch >= v with pitch % 32 == 4
  int p = (v + 31) / 32 * 32 + 4;
  if (p - 32 >= v) p -= 32;
  return p;
}

}  // namespace

// ============================================================================ dispatch

bool conv_fast_ok(const float* in, int64_t in_stride, const float* out, int64_t out_stride, int h,
                  int w, int taps) {
  const int hw = h * w;
  if (hw % 4 || in_stride % 4 || out_stride % 4 || !aligned16(in) || !aligned16(out)) return false;
  if (taps == 9 && (w % 4 || w < 4)) return false;
  return true;
}

size_t packed_weight_floats(int cout, int cin, int taps) {
  return (size_t)taps * ((cout + 15) & ~15) * ((cin + 15) & ~15);
}

hipError_t launch_pack_weights(WeightView wv, int cout, int cin, int taps, float* packed, hipStream_t st) {
  const size_t total = packed_weight_floats(cout, cin, taps);
  unsigned grid = (unsigned)((total + 255) / 256);
  if (grid > 4096) grid = 4096;
  hipLaunchKernelGGL(k_pack_weights, dim3(grid), dim3(256), 0, st, wv.w, wv.sm, wv.sc, wv.flip, cout, cin,
                     taps, packed);
  return hipGetLastError();
}

size_t packed_layer_floats(int c, int k, int B) {
  const size_t B16 = (B + 15) & ~15, k16 = (k + 15) & ~15, c16 = (c + 15) & ~15;
  return 2 * B16 * c16 + 18 * k16 * B16;
}

hipError_t launch_pack_block_weights(const float* params, float* packed, int c0, int k, int B, int m,
                                     hipStream_t st) {
  const size_t most = packed_layer_floats(c0 + (m - 1) * k, k, B);
  unsigned gx = (unsigned)((most + 255) / 256);
  if (gx > 256) gx = 256;
  hipLaunchKernelGGL(k_pack_block_weights, dim3(gx, (unsigned)m), dim3(256), 0, st, params, packed, c0, k, B);
  return hipGetLastError();
}

hipError_t launch_bn_fold(const float* gamma, const float* beta, float* mean, float* istd,
                          const float* part, int T, int fresh_lo, int fresh_hi, float eps, int nch,
                          float2* fold, hipStream_t st) {
  if (nch <= 0) return hipSuccess;
  hipLaunchKernelGGL(k_bn_fold, dim3((unsigned)nch), dim3(256), 0, st, gamma, beta, mean, istd, part, T,
                     fresh_lo, fresh_hi, eps, fold);
  return hipGetLastError();
}

size_t conv_stats_partial_floats(int n, int cout, int h, int w) {
  return (size_t)cout * n * ((h * w + 15) / 16) * 3;
}

// Returns false (nothing launched) if the fast path does not cover this shape.
// fold != null: BN+ReLU prologue.  spart != null: epilogue statistics, *sT = partials per channel.
bool launch_conv_fast(const float* in, int64_t in_stride, const float* packed, float* out,
                      int64_t out_stride, int n, int cin, int cout, int h, int w, int taps,
                      const float2* fold, float* spart, int* sT, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
  const int hw = h * w, mtiles = (cout + 15) / 16, M16 = mtiles * 16;
  const int K16 = (cin + 15) & ~15, nchunks = K16 / 16;
  const int mode = fold ? 2 : (spart ? 1 : 0);  // 0 plain, 1 statistics, 2 prologue + statistics
  if (fold && !spart) return false;
  if (taps == 1) {
    const bool ksplit = nchunks >= 4;
    int nw, mt, gy;
    if (ksplit) {
      nw = 4; mt = mtiles >= 3 ? 3 : mtiles; gy = (mtiles + mt - 1) / mt;
    } else {
      nw = mtiles >= 4 ? 4 : mtiles;
      mt = (mtiles + nw - 1) / nw; if (mt > 3) mt = 3;
      gy = (mtiles + nw * mt - 1) / (nw * mt);
    }
    // 64-pixel tiles (a lane loads 16 bytes per channel row, and the weights are read once per 64
    // pixels instead of once per 16) as long as they give one workgroup per CU.  With two per CU or
    // more, two waves share a tile's K range and two tiles share the workgroup (longer contiguous
    // runs per channel row measured faster than a four-way K-split); between one and two per CU
    // (K-split shapes), one tile per workgroup and a four-way K-split: the 16x16 block of
    // DenseNet-BC-100 at batch 64 went from 18.9 to ~13 us per launch against 16-pixel tiles.
    // Smaller launches take 16-pixel tiles with a four-way K-split for more loads in flight.
    const int64_t tiles64 = (int64_t)((hw + 63) / 64) * gy * n;
    const bool one_tile = ksplit && tiles64 >= 256 && tiles64 < 512;
    const int ppl = (tiles64 >= 512 || one_tile) ? 4 : 1;
    const int tiles = (hw + 16 * ppl - 1) / (16 * ppl);
    // (with at most 16 chunks a wave takes a tile's whole K range, four tiles per workgroup and no
    // reduction: 0.9 % off the DenseNet-BC-100 step; with the long K ranges of k = 24 nets it was
    // slightly slower than the two-way split)
    const int wk = ksplit ? ((ppl == 4 && !one_tile) ? (nchunks <= 16 ? 1 : 2) : nw) : 1;
    const int wp = ksplit ? nw / wk : 1;
    dim3 grid((unsigned)((tiles + wp - 1) / wp), (unsigned)gy, (unsigned)n);
    const size_t lds = ksplit ? (size_t)wp * (wk - 1) * mt * ppl * 256 * sizeof(float) : 0;
    const int T = tiles * n;
    if (sT) *sT = T;
#define DNB_L(MT, PPL, KS, PRO, STATS)                                                                \
  hipExtLaunchKernelGGL((k_conv1x1_v3<MT, PPL, KS, PRO, STATS>), grid, dim3(64 * nw), lds, st, ev0,   \
                        ev1, 0, in, in_stride, packed, K16, out, out_stride, cin, cout, hw, fold,     \
                        spart, T, wk)
#define DNB_L3(MT, PPL, KS)                                                         \
  do {                                                                              \
    if (mode == 2) DNB_L(MT, PPL, KS, true, true);                                   \
    else if (mode == 1) DNB_L(MT, PPL, KS, false, true);                             \
    else DNB_L(MT, PPL, KS, false, false);                                           \
  } while (0)
#define DNB_L2(MT)                                                                   \
  do {                                                                               \
    if (ksplit) { if (ppl == 4) DNB_L3(MT, 4, true); else DNB_L3(MT, 1, true); }      \
    else        { if (ppl == 4) DNB_L3(MT, 4, false); else DNB_L3(MT, 1, false); }    \
  } while (0)
    switch (mt) { case 3: DNB_L2(3); break; case 2: DNB_L2(2); break; default: DNB_L2(1); break; }
#undef DNB_L2
#undef DNB_L3
#undef DNB_L
    return true;
  }
  const bool fwd13 = mtiles == 1 && nchunks == 3, dg31 = mtiles == 3 && nchunks == 1 && mode == 0;
  if ((fwd13 || dg31) && (w == 8 || w == 16 || w == 32) && hw % 64 == 0) {
    // persistent kernel: weights in registers, pixel-split waves, double-buffered tiles
    const int tpi = hw / 64, total_tiles = tpi * n;
    int G = total_tiles < kV4Workgroups ? (total_tiles + 7) / 8 * 8 : kV4Workgroups;
    const size_t lds = ((size_t)2 * (nchunks * 16 * 144 + 4) + 2 * 4 * mtiles * 16 * 3) * sizeof(float);
    if (sT) *sT = total_tiles;
#define DNB_L4(MT, NCH, WW, PRO, STATS)                                                                  \
  hipExtLaunchKernelGGL((k_conv3x3_v4<MT, NCH, WW, PRO, STATS>), dim3(G), dim3(256), lds, st, ev0, ev1,  \
                        0, in, in_stride, packed, M16, K16, out, out_stride, cin, cout, h, fold, spart,  \
                        total_tiles, tpi, total_tiles)
#define DNB_L4W(WW)                                                                  \
  do {                                                                               \
    if (dg31) DNB_L4(3, 1, WW, false, false);                                         \
    else if (mode == 2) DNB_L4(1, 3, WW, true, true);                                 \
    else if (mode == 1) DNB_L4(1, 3, WW, false, true);                                \
    else DNB_L4(1, 3, WW, false, false);                                              \
  } while (0)
    if (w == 32) DNB_L4W(32); else if (w == 16) DNB_L4W(16); else DNB_L4W(8);
#undef DNB_L4W
#undef DNB_L4
    return true;
  }
  const bool ksplit = nchunks >= 3;
  int nw, mt, gy;
  if (ksplit) {
    mt = mtiles >= 2 ? 2 : 1; gy = (mtiles + mt - 1) / mt;
    nw = (nchunks % 4 == 0) ? 4 : (nchunks % 3 == 0 ? 3 : 4);
  } else {
    nw = mtiles >= 4 ? 4 : mtiles;
    mt = mtiles > 4 ? 2 : 1;
    gy = (mtiles + nw * mt - 1) / (nw * mt);
  }
  const int CS = pad4mod32(64 + 2 * w + 8);
  const size_t tile = (size_t)((cin + 3) & ~3) * CS, red = ksplit ? (size_t)(nw - 1) * mt * 4 * 256 : 0;
  const size_t lds = (tile > red ? tile : red) * sizeof(float);
  if (lds > 64 * 1024) return false;
  dim3 grid((unsigned)((hw + 63) / 64), (unsigned)gy, (unsigned)n);
  const int T = (int)grid.x * n;
  if (sT) *sT = T;
#define DNB_L(MT, KS, PRO, STATS)                                                                      \
  hipExtLaunchKernelGGL((k_conv3x3_v3<MT, KS, PRO, STATS>), grid, dim3(64 * nw), lds, st, ev0, ev1, 0, \
                        in, in_stride, packed, M16, K16, out, out_stride, cin, cout, h, w, CS, fold,   \
                        spart, T)
#define DNB_L3(MT, KS)                                                              \
  do {                                                                              \
    if (mode == 2) DNB_L(MT, KS, true, true);                                        \
    else if (mode == 1) DNB_L(MT, KS, false, true);                                  \
    else DNB_L(MT, KS, false, false);                                                \
  } while (0)
  if (ksplit) { if (mt == 2) DNB_L3(2, true); else DNB_L3(1, true); }
  else        { if (mt == 2) DNB_L3(2, false); else DNB_L3(1, false); }
#undef DNB_L3
#undef DNB_L
  return true;
}

// ---- weight gradient plans (shared by the scratch-size query and the launcher)

struct WgFastPlan {
  bool ok;
  int mtw, ctw, gy, gz, gx;
  int spi, total_steps, steps_per_wg;  // 1x1
  int tiles_per_img, nms, PA;          // 3x3
  size_t lds;
};

static WgFastPlan plan_wgrad_fast(int n, int cin, int cout, int h, int w, int taps) {
  WgFastPlan p{};
  const int hw = h * w, mtiles = (cout + 15) / 16, ctiles = (cin + 15) / 16;
  p.ok = hw % 4 == 0 && (taps == 1 || (w % 4 == 0 && w >= 4));
  if (!p.ok) return p;
  if (taps == 1) {
    p.mtw = mtiles >= 3 ? 3 : mtiles;
    p.ctw = ctiles >= 4 ? 4 : ctiles;
    p.gy = (ctiles + p.ctw - 1) / p.ctw;
    p.gz = (mtiles + p.mtw - 1) / p.mtw;
    p.spi = (hw + 15) / 16;
    p.total_steps = n * p.spi;
    // About 128 workgroups in all, 1..16 (or 64) steps per wave.  A workgroup ends with a cross-wave sum
    // and a partial of mtw*ctw tiles to store, and every partial is read again by the sum that
    // follows, so few long workgroups beat many short ones even when they leave CUs to the other
    // roles of the launch: a target of 512 workgroups (1..8 steps) took 3.3 % more time per
    // DenseNet-BC-100 step than 128; 96 and 192 were within 0.5 % of 128.
    // With many (m, c) tile columns (wide layers, k = 24 nets) the columns alone fill the chip and the
    // pixel ranges can be longer still: a cap of 64 steps there took 1.2 % off the DenseNet-BC-250 step.
    int spw = (int)(((int64_t)p.total_steps * p.gy * p.gz + 4 * 128 - 1) / (4 * 128));
    const int cap = p.gy * p.gz > 8 ? 64 : 16;
    if (spw < 1) spw = 1;
    if (spw > cap) spw = cap;
    p.steps_per_wg = 4 * spw;
    p.gx = (p.total_steps + p.steps_per_wg - 1) / p.steps_per_wg;
    p.lds = (size_t)4 * p.mtw * p.ctw * 256 * sizeof(float);
  } else {
    p.mtw = mtiles >= 2 ? 2 : 1;
    p.ctw = p.mtw == 2 ? (ctiles >= 2 ? 2 : 1) : (ctiles >= 3 ? 3 : ctiles);
    p.gy = (ctiles + p.ctw - 1) / p.ctw;
    p.gz = (mtiles + p.mtw - 1) / p.mtw;
    // 64, 128 or 256 pixels per workgroup: the largest that fits LDS and still gives >= 128
    // workgroups (each ends with a 27 KB partial; 256 and 64 as the bound measured 0.3-0.5 % slower
    // per DenseNet-BC-100 step)
    p.nms = 1;
    for (int nms = 4; nms >= 2; nms >>= 1) {
      const int tpix = 64 * nms;
      if (tpix / 2 >= hw) continue;
      if ((size_t)p.ctw * 16 * pad4mod32(tpix + 2 * w + 8) * sizeof(float) > 64 * 1024) continue;
      if ((int64_t)((hw + tpix - 1) / tpix) * n * p.gy * p.gz >= 128) { p.nms = nms; break; }
    }
    const int tpix = 64 * p.nms;
    p.tiles_per_img = (hw + tpix - 1) / tpix;
    p.gx = n * p.tiles_per_img;
    p.PA = pad4mod32(tpix + 2 * w + 8);
    size_t tile = (size_t)p.ctw * 16 * p.PA, red = (size_t)p.mtw * p.ctw * 9 * 256;
    p.lds = (tile > red ? tile : red) * sizeof(float);
    if (p.lds > 64 * 1024) p.ok = false;
  }
  return p;
}

size_t conv_wgrad_fast_partial_floats(int n, int cin, int cout, int h, int w, int taps) {
  const WgFastPlan p = plan_wgrad_fast(n, cin, cout, h, w, taps);
  if (!p.ok) return 0;
  if (taps == 9) return (size_t)p.gx * p.gy * p.gz * p.mtw * p.ctw * 9 * 256;  // accumulator-order partials
  return (size_t)p.gx * cin * cout;
}

// Grouping of a sum of `splits` partials (the same rule the stand-alone sum kernels use).
static void sum_grouping(int kind, int splits, int* G, int* per) {
  int g = 1;
  if (kind == 2) { while (g < 16 && splits / (g * 2) >= 4) g *= 2; }   // at least 4 partials per group
  else           { while (g < 16 && splits / g > 16) g <<= 1; }         // about 16 splits per thread
  *G = g;
  *per = (splits + g - 1) / g;
}

hipError_t launch_sum_wgrad3x3(const PendingSum& p, hipStream_t st) {
  int G, per;
  sum_grouping(2, p.splits, &G, &per);
  const int epb = 256 / G;
  hipLaunchKernelGGL(k_sum_wgrad3x3, dim3((unsigned)((p.count + epb - 1) / epb)), dim3(256), 0, st, p.part, p.splits,
                     p.gy, p.gz, p.mtw, p.ctw, p.cin, p.cout, p.out, G, per);
  return hipGetLastError();
}

// Returns false if the fast path does not apply; otherwise launches the kernel, describes the sum
// of its partials in *own (left to the caller) and has *absorb carried out by extra workgroups.
bool launch_wgrad_fast(const float* in, int64_t in_stride, const float* g, int64_t g_stride,
                       float* partials, float* dw, int n, int cin, int cout, int h, int w, int taps,
                       const float2* fold, PendingSum* own, PendingSum* absorb, hipStream_t st, hipEvent_t ev0,
                       hipEvent_t ev1) {
  if (in_stride % 4 || g_stride % 4 || !aligned16(in) || !aligned16(g)) return false;
  const WgFastPlan p = plan_wgrad_fast(n, cin, cout, h, w, taps);
  if (!p.ok) return false;
  SumRole sr{};
  unsigned sx = 0;
  if (absorb && absorb->kind != 0) {
    sr.kind = absorb->kind;
    sr.part = absorb->part; sr.out = absorb->out; sr.splits = absorb->splits; sr.count = absorb->count;
    sr.gy = absorb->gy; sr.gz = absorb->gz; sr.mtw = absorb->mtw; sr.ctw = absorb->ctw;
    sr.cin = absorb->cin; sr.cout = absorb->cout;
    sum_grouping(sr.kind, sr.splits, &sr.G, &sr.per);
    const int epb = 256 / sr.G;
    sr.wgs = (int)((sr.count + epb - 1) / epb);
    sx = (unsigned)((sr.wgs + p.gy * p.gz - 1) / (p.gy * p.gz));
    absorb->kind = 0;
  }
  dim3 grid((unsigned)p.gx + sx, (unsigned)p.gy, (unsigned)p.gz);
  const int hw = h * w;
  if (taps == 1) {
    const Wg1Args A{in, in_stride, g, g_stride, partials, cin, cout, hw, p.spi, p.total_steps, p.steps_per_wg, fold};
#define DNB_L(M, C)                                                                                                  \
  do {                                                                                                               \
    if (fold) hipExtLaunchKernelGGL((k_wgrad1x1_fast<M, C, true>), grid, dim3(256), p.lds, st, ev0, ev1, 0, A, sr, p.gx); \
    else hipExtLaunchKernelGGL((k_wgrad1x1_fast<M, C, false>), grid, dim3(256), p.lds, st, ev0, ev1, 0, A, sr, p.gx);  \
  } while (0)
    const int key = p.mtw * 10 + p.ctw;
    switch (key) {
      case 34: DNB_L(3, 4); break; case 33: DNB_L(3, 3); break; case 32: DNB_L(3, 2); break; case 31: DNB_L(3, 1); break;
      case 24: DNB_L(2, 4); break; case 23: DNB_L(2, 3); break; case 22: DNB_L(2, 2); break; case 21: DNB_L(2, 1); break;
      case 14: DNB_L(1, 4); break; case 13: DNB_L(1, 3); break; case 12: DNB_L(1, 2); break; default: DNB_L(1, 1); break;
    }
#undef DNB_L
    own->kind = 1;
    own->part = partials; own->out = dw; own->splits = p.gx; own->count = (int64_t)cin * cout;
  } else {
    const Wg3Args A{in, in_stride, g, g_stride, partials, cin, cout, h, w, p.tiles_per_img, p.nms, p.PA, fold};
#define DNB_L(M, C)                                                                                                  \
  do {                                                                                                               \
    if (fold) hipExtLaunchKernelGGL((k_wgrad3x3_fast<M, C, true>), grid, dim3(256), p.lds, st, ev0, ev1, 0, A, sr, p.gx); \
    else hipExtLaunchKernelGGL((k_wgrad3x3_fast<M, C, false>), grid, dim3(256), p.lds, st, ev0, ev1, 0, A, sr, p.gx);  \
  } while (0)
    const int key = p.mtw * 10 + p.ctw;
    switch (key) {
      case 22: DNB_L(2, 2); break; case 21: DNB_L(2, 1); break;
      case 13: DNB_L(1, 3); break; case 12: DNB_L(1, 2); break; default: DNB_L(1, 1); break;
    }
#undef DNB_L
    // the 3x3 partials are in accumulator order: their sum also reorders them
    own->kind = 2;
    own->part = partials; own->out = dw; own->splits = p.gx;
    own->count = (int64_t)p.gz * p.gy * p.mtw * p.ctw * 9 * 256;
    own->gy = p.gy; own->gz = p.gz; own->mtw = p.mtw; own->ctw = p.ctw; own->cin = cin; own->cout = cout;
  }
  return true;
}

static SumRole make_sum_role(PendingSum* absorb) {
  SumRole sr{};
  if (absorb && absorb->kind != 0) {
    sr.kind = absorb->kind;
    sr.part = absorb->part; sr.out = absorb->out; sr.splits = absorb->splits; sr.count = absorb->count;
    sr.gy = absorb->gy; sr.gz = absorb->gz; sr.mtw = absorb->mtw; sr.ctw = absorb->ctw;
    sr.cin = absorb->cin; sr.cout = absorb->cout;
    sum_grouping(sr.kind, sr.splits, &sr.G, &sr.per);
    const int epb = 256 / sr.G;
    sr.wgs = (int)((sr.count + epb - 1) / epb);
    absorb->kind = 0;
  }
  return sr;
}

// Both weight gradients of a bottleneck layer in one launch: the 3x3 (in3: the bottleneck
// activations, cin3 = B channels; g3: the gradient of x_l, cout3 = k) and the 1x1 (in1: the
// concatenated features, cin1 = C_l; g1: the gradient of b_l, cout1 = B = cin3), same image
// size, both with or both without the BN+ReLU prologue.  Returns false (nothing launched,
// nothing absorbed) when the pair is not one of the instantiated combinations.
bool launch_wgrad_pair_fast(const float* in1, int64_t in1_stride, const float* g1, int64_t g1_stride, float* part1,
                            float* dw1, int cin1, const float2* fold1, const float* in3, int64_t in3_stride,
                            const float* g3, int64_t g3_stride, float* part3, float* dw3, int cout3,
                            const float2* fold3, int n, int B, int h, int w, PendingSum* own1, PendingSum* own3,
                            PendingSum* absorb1, PendingSum* absorb3, const BnBwdPartialArgs* bn, hipStream_t st,
                            hipEvent_t ev0, hipEvent_t ev1) {
  if ((fold1 != nullptr) != (fold3 != nullptr)) return false;
  if (in1_stride % 4 || g1_stride % 4 || in3_stride % 4 || g3_stride % 4 || !aligned16(in1) || !aligned16(g1) ||
      !aligned16(in3) || !aligned16(g3))
    return false;
  const WgFastPlan p1 = plan_wgrad_fast(n, cin1, B, h, w, 1), p3 = plan_wgrad_fast(n, B, cout3, h, w, 9);
  if (!p1.ok || !p3.ok || p1.mtw != 3) return false;
  const int key3 = p3.mtw * 10 + p3.ctw;
  if (key3 != 13 && key3 != 22) return false;
  const SumRole s1 = make_sum_role(absorb1), s3 = make_sum_role(absorb3);
  const int hw = h * w;
  const Wg1Args A1{in1, in1_stride, g1, g1_stride, part1, cin1, B, hw, p1.spi, p1.total_steps, p1.steps_per_wg, fold1};
  const Wg3Args A3{in3, in3_stride, g3, g3_stride, part3, B, cout3, h, w, p3.tiles_per_img, p3.nms, p3.PA, fold3};
  const int n1 = (p1.gx + 7) / 8 * 8 * p1.gy * p1.gz, n3 = p3.gx * p3.gy * p3.gz;  // 1x1: whole pixel ranges per XCD
  const BnBwdPartialArgs bna = bn ? *bn : BnBwdPartialArgs{};
  const int nbn = bn ? bn->c * bn->splits : 0;
  const dim3 grid((unsigned)(n1 + n3 + nbn + s1.wgs + s3.wgs));
  const size_t lds = p1.lds > p3.lds ? p1.lds : p3.lds;
#define DNB_P(C1, M3, C3)                                                                                             \
  do {                                                                                                                \
    if (fold1) hipExtLaunchKernelGGL((k_wgrad_pair<3, C1, M3, C3, true>), grid, dim3(256), lds, st, ev0, ev1, 0, A1,  \
                                     p1.gx, p1.gy, p1.gz, n1, A3, p3.gy, p3.gz, n3, s1, s3, bna, nbn);                       \
    else hipExtLaunchKernelGGL((k_wgrad_pair<3, C1, M3, C3, false>), grid, dim3(256), lds, st, ev0, ev1, 0, A1, p1.gx, p1.gy, \
                               p1.gz, n1, A3, p3.gy, p3.gz, n3, s1, s3, bna, nbn);                                    \
  } while (0)
#define DNB_P1(M3, C3)                                                                          \
  switch (p1.ctw) {                                                                             \
    case 4: DNB_P(4, M3, C3); break; case 3: DNB_P(3, M3, C3); break; case 2: DNB_P(2, M3, C3); break; \
    default: DNB_P(1, M3, C3); break;                                                           \
  }
  if (key3 == 13) { DNB_P1(1, 3) } else { DNB_P1(2, 2) }
#undef DNB_P1
#undef DNB_P
  own1->kind = 1;
  own1->part = part1; own1->out = dw1; own1->splits = p1.gx; own1->count = (int64_t)cin1 * B;
  own3->kind = 2;
  own3->part = part3; own3->out = dw3; own3->splits = p3.gx;
  own3->count = (int64_t)p3.gz * p3.gy * p3.mtw * p3.ctw * 9 * 256;
  own3->gy = p3.gy; own3->gz = p3.gz; own3->mtw = p3.mtw; own3->ctw = p3.ctw; own3->cin = B; own3->cout = cout3;
  return true;
}

}  // namespace dnb
