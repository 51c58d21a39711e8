// fp32 convolutions of the dense block as MFMA implicit GEMMs on gfx950 (NCHW).
//
// Forward and data gradient share one kernel: out[m][q] = sum_{c,t} W(m,c,t) * in[c][q+shift(t)].
// The 16x16x4 fp32 MFMA is used with output channels on its M axis (k = 12 pads to 16 only)
// and 16 consecutive pixels on its N axis, so activation reads and output writes run along the
// contiguous pixel axis of NCHW.  Activations are staged through LDS once per channel chunk
// with a one-row halo and the nine taps are shifted reads of that tile; the weights of the
// chunk sit beside them.
//
// The weight gradient is a GEMM over pixels, dW[m][c][t] = sum_q g[m][q] * in[c][q+shift(t)],
// split over pixel ranges across workgroups; partial results go to scratch and a second kernel
// adds them in a fixed order (no float atomics: results are reproducible run to run).
#include "dnb_internal.h"
#include "dnb_stats.h"

namespace dnb {

// fast paths (dnb_conv_f32_fast.hip)
bool conv_fast_ok(const float* in, int64_t in_stride, const float* out, int64_t out_stride, int h,
                  int w, int taps);
bool launch_conv_fast(const float* in, int64_t in_stride, const float* packed, float* out,
                      int64_t out_stride, int n, int cin, int cout, int h, int w, int taps,
                      const float2* fold, float* spart, int* sT, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1);
size_t conv_wgrad_fast_partial_floats(int n, int cin, int cout, int h, int w, int taps);
// Launches the fast weight-gradient kernel if it applies (returns false otherwise).  *own
// describes the sum of its partials, which is left to the caller; *absorb (may be null or of kind
// 0) is carried out by extra workgroups of the same launch and cleared.
bool launch_wgrad_fast(const float* in, int64_t in_stride, const float* g, int64_t g_stride,
                       float* partials, float* dw, int n, int cin, int cout, int h, int w, int taps,
                       const float2* fold, PendingSum* own, PendingSum* absorb, hipStream_t st, hipEvent_t ev0,
                       hipEvent_t ev1);
hipError_t launch_sum_wgrad3x3(const PendingSum& p, hipStream_t st);
bool launch_wgrad_pair_fast(const float* in1, int64_t in1_stride, const float* g1, int64_t g1_stride, float* part1,
                            float* dw1, int cin1, const float2* fold1, const float* in3, int64_t in3_stride,
                            const float* g3, int64_t g3_stride, float* part3, float* dw3, int cout3,
                            const float2* fold3, int n, int B, int h, int w, PendingSum* own1, PendingSum* own3,
                            PendingSum* absorb1, PendingSum* absorb3, const BnBwdPartialArgs* bn, hipStream_t st,
                            hipEvent_t ev0, hipEvent_t ev1);

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int KC = 16;  // input channels staged per step (4 MFMA k-steps)

// D(16x16) += A(16x4) * B(4x16).  Lane l supplies A[l%16][l/16] and B[l/16][l%16] and holds
// D[4*(l/16)+r][l%16] in register r.
__device__ __forceinline__ f32x4 mfma16(float a, float b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// smallest stride >= v that is 16 mod 32: four 16-lane groups reading four rows hit
// disjoint LDS banks
inline int pad16mod32(int v) {
  int r = (v + 31) / 32 * 32 + 16;
  if (r - 32 >= v) r -= 32;
  return r;
}
// smallest stride >= v that is 4 mod 64: sixteen rows x four consecutive columns are
// conflict free
inline int pad4mod64(int v) {
  int r = (v + 63) / 64 * 64 + 4;
  if (r - 64 >= v) r -= 64;
  return r;
}

template <int TAPS, int MT, int NT>
__global__ __launch_bounds__(256) void k_conv_igemm(
    const float* __restrict__ in, int64_t in_stride, const float* __restrict__ wgt, int64_t w_sm,
    int64_t w_sc, int flip, float* __restrict__ out, int64_t out_stride, int cin, int cout, int H,
    int W, int wm, int CS, int MS) {
  extern __shared__ float lds[];
  const int HW = H * W;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wn = 4 / wm;
  const int wave_m = wave % wm, wave_n = wave / wm;
  constexpr int TPW = NT * 16;  // pixels per wave
  constexpr int MW = MT * 16;   // output channels per wave
  const int TP = wn * TPW, MB = wm * MW;
  const int halo = (TAPS == 9) ? (W + 1) : 0;
  const int seg = TP + 2 * halo;
  float* al = lds;            // [KC][CS]   activations, flat pixel index with halo
  float* wl = lds + KC * CS;  // [TAPS][KC][MS] weights, output channel fastest
  const int q0 = blockIdx.x * TP, m0 = blockIdx.y * MB, img = blockIdx.z;
  const float* inb = in + (int64_t)img * in_stride;
  const int i16 = lane & 15, g = lane >> 4;

  f32x4 acc[MT][NT];
#pragma unroll
  for (int a = 0; a < MT; ++a)
#pragma unroll
    for (int b = 0; b < NT; ++b) acc[a][b] = (f32x4){0.f, 0.f, 0.f, 0.f};

  int pl[NT];
  bool lok[NT], rok[NT];
#pragma unroll
  for (int b = 0; b < NT; ++b) {
    pl[b] = wave_n * TPW + b * 16 + i16;
    const int wc = (q0 + pl[b]) % W;
    lok[b] = wc != 0;
    rok[b] = wc != W - 1;
  }

  for (int c0 = 0; c0 < cin; c0 += KC) {
    __syncthreads();
    for (int idx = tid; idx < KC * seg; idx += 256) {
      const int kc = idx / seg, s = idx - kc * seg;
      const int q = q0 - halo + s, c = c0 + kc;
      float v = 0.f;
      if (c < cin && q >= 0 && q < HW) v = inb[(int64_t)c * HW + q];
      al[kc * CS + s] = v;
    }
    for (int idx = tid; idx < TAPS * KC * MB; idx += 256) {
      // output channel fastest: conflict-free LDS writes (global reads are small and cached)
      const int t = idx / (KC * MB), rem = idx - t * (KC * MB);
      const int kc = rem / MB, mrow = rem - kc * MB;
      const int m = m0 + mrow, c = c0 + kc;
      float v = 0.f;
      if (m < cout && c < cin) v = wgt[(int64_t)m * w_sm + (int64_t)c * w_sc + (flip ? TAPS - 1 - t : t)];
      wl[(t * KC + kc) * MS + mrow] = v;
    }
    __syncthreads();
#pragma unroll
    for (int t = 0; t < TAPS; ++t) {
      const int di = (TAPS == 9) ? t / 3 - 1 : 0, dj = (TAPS == 9) ? t % 3 - 1 : 0;
      const int shift = halo + di * W + dj;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const int kc = ks * 4 + g;
        float a[MT], b[NT];
#pragma unroll
        for (int x = 0; x < MT; ++x) a[x] = wl[(t * KC + kc) * MS + wave_m * MW + x * 16 + i16];
#pragma unroll
        for (int x = 0; x < NT; ++x) {
          float v = al[kc * CS + pl[x] + shift];
          if (dj < 0 && !lok[x]) v = 0.f;
          if (dj > 0 && !rok[x]) v = 0.f;
          b[x] = v;
        }
#pragma unroll
        for (int x = 0; x < MT; ++x)
#pragma unroll
          for (int y = 0; y < NT; ++y) acc[x][y] = mfma16(a[x], b[y], acc[x][y]);
      }
    }
  }

  float* ob = out + (int64_t)img * out_stride;
#pragma unroll
  for (int x = 0; x < MT; ++x)
#pragma unroll
    for (int y = 0; y < NT; ++y) {
      const int q = q0 + pl[y];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int m = m0 + wave_m * MW + x * 16 + 4 * g + r;
        if (m < cout && q < HW) ob[(int64_t)m * HW + q] = acc[x][y][r];
      }
    }
}

// ---------------------------------------------------------------------------- weight gradient

constexpr int TPIX = 64;  // pixels staged per step of the reduction

// grid (splits, ceil(ctiles/CTW), ceil(mtiles/MTW)).  The workgroup owns the MTW*CTW*TAPS
// 16x16 output tiles of its (m, c) range; tile t goes to wave t%4, slot t/4 (at most TW slots).
template <int TAPS, int TW>
__global__ __launch_bounds__(256) void k_conv_wgrad(
    const float* __restrict__ in, int64_t in_stride, const float* __restrict__ gout,
    int64_t g_stride, float* __restrict__ part, int cin, int cout, int H, int W, int cpi /*chunks per image*/,
    int total_chunks, int cps /*chunks per split*/, int MTW, int CTW, int PA, int PG) {
  extern __shared__ float lds[];
  const int HW = H * W;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int i16 = lane & 15, kk = lane >> 4;
  const int MB = MTW * 16, CB = CTW * 16;
  const int halo = (TAPS == 9) ? (W + 1) : 0;
  const int seg = TPIX + 2 * halo;
  float* al = lds;            // [CB][PA]
  float* gl = lds + CB * PA;  // [MB][PG]
  const int split = blockIdx.x, c0 = blockIdx.y * CB, m0 = blockIdx.z * MB;
  const int ntiles = MTW * CTW * TAPS;

  f32x4 acc[TW];
  int t_mt[TW], t_ct[TW], t_tap[TW];
#pragma unroll
  for (int j = 0; j < TW; ++j) {
    acc[j] = (f32x4){0.f, 0.f, 0.f, 0.f};
    const int t = wave + 4 * j;
    const int tt = t < ntiles ? t : 0;
    t_tap[j] = tt % TAPS;
    t_ct[j] = (tt / TAPS) % CTW;
    t_mt[j] = tt / (TAPS * CTW);
  }

  const int ch_begin = split * cps, ch_end = min(total_chunks, ch_begin + cps);
  for (int chunk = ch_begin; chunk < ch_end; ++chunk) {
    const int img = chunk / cpi, q0 = (chunk - img * cpi) * TPIX;
    const float* inb = in + (int64_t)img * in_stride;
    const float* gb = gout + (int64_t)img * g_stride;
    __syncthreads();
    for (int idx = tid; idx < CB * seg; idx += 256) {
      const int row = idx / seg, s = idx - row * seg;
      const int q = q0 - halo + s, c = c0 + row;
      float v = 0.f;
      if (c < cin && q >= 0 && q < HW) v = inb[(int64_t)c * HW + q];
      al[row * PA + s] = v;
    }
    for (int idx = tid; idx < MB * TPIX; idx += 256) {
      const int row = idx / TPIX, s = idx - row * TPIX;
      const int q = q0 + s, m = m0 + row;
      float v = 0.f;
      if (m < cout && q < HW) v = gb[(int64_t)m * HW + q];
      gl[row * PG + s] = v;
    }
    __syncthreads();
#pragma unroll 4
    for (int s = 0; s < TPIX / 4; ++s) {
      const int p = 4 * s + kk;
      const int wc = (q0 + p) % W;
      const bool lok = wc != 0, rok = wc != W - 1;
#pragma unroll
      for (int j = 0; j < TW; ++j) {
        if (wave + 4 * j < ntiles) {
          const int di = (TAPS == 9) ? t_tap[j] / 3 - 1 : 0, dj = (TAPS == 9) ? t_tap[j] % 3 - 1 : 0;
          const float a = gl[(t_mt[j] * 16 + i16) * PG + p];
          float b = al[(t_ct[j] * 16 + i16) * PA + halo + p + di * W + dj];
          if (dj < 0 && !lok) b = 0.f;
          if (dj > 0 && !rok) b = 0.f;
          acc[j] = mfma16(a, b, acc[j]);
        }
      }
    }
  }

  float* pb = part + (int64_t)split * cout * cin * TAPS;
#pragma unroll
  for (int j = 0; j < TW; ++j) {
    if (wave + 4 * j < ntiles) {
      const int c = c0 + t_ct[j] * 16 + i16;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int m = m0 + t_mt[j] * 16 + 4 * kk + r;
        if (m < cout && c < cin) pb[((int64_t)m * cin + c) * TAPS + t_tap[j]] = acc[j][r];
      }
    }
  }
}

// out[e] = sum over splits of part[split][e], in a fixed order.  Block = (EPB elements) x
// (G groups); group g adds splits [g*per, (g+1)*per) with eight independent loads in flight,
// then the G group sums are added in order 0..G-1 through LDS.
__global__ __launch_bounds__(256) void k_sum_partials(const float* __restrict__ part, int splits,
                                                      int64_t count, float* __restrict__ out, int G,
                                                      int per) {
  __shared__ float sh[256];
  const int epb = 256 / G;
  const int le = threadIdx.x % epb, grp = threadIdx.x / epb;
  const int64_t e = (int64_t)blockIdx.x * epb + le;
  float s = 0.f;
  if (e < count) {
    int i = grp * per;
    const int end = min(splits, i + per);
    for (; i + 8 <= end; i += 8) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = part[(int64_t)(i + u) * count + e];
#pragma unroll
      for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (; i < end; ++i) s += part[(int64_t)i * count + e];
  }
  if (G == 1) {
    if (e < count) out[e] = s;
    return;
  }
  sh[threadIdx.x] = s;
  __syncthreads();
  if (grp == 0 && e < count) {
    float t = sh[le];
    for (int g = 1; g < G; ++g) t += sh[g * epb + le];
    out[e] = t;
  }
}

}  // namespace

hipError_t launch_sum_partials(const float* partials, int splits, int64_t count, float* out, hipStream_t st) {
  int G = 1;
  while (G < 16 && splits / G > 16) G <<= 1;  // about 16 splits per thread, at least 16 elements per row
  const int per = (splits + G - 1) / G, epb = 256 / G;
  hipLaunchKernelGGL(k_sum_partials, dim3((unsigned)((count + epb - 1) / epb)), dim3(256), 0, st, partials,
                     splits, count, out, G, per);
  return hipGetLastError();
}

namespace {

struct IgemmPlan {
  int mt, nt, wm;
  dim3 grid;
  int CS, MS;
  size_t lds;
};

IgemmPlan plan_igemm(int n, int cout, int h, int w, int taps) {
  IgemmPlan p;
  const int hw = h * w, mtiles = (cout + 15) / 16;
  // 3x3: keep the staged weights of a chunk (taps*KC*MB floats) small -> one wave column
  p.wm = taps == 9 ? 1 : (mtiles >= 12 ? 4 : (mtiles >= 6 ? 2 : 1));
  const int per_wave = (mtiles + p.wm - 1) / p.wm;
  p.mt = per_wave >= 4 ? 4 : per_wave;  // tiles per wave, at most 4 (grid.y covers the rest)
  if (p.mt == 4 && per_wave % 4 != 0 && per_wave % 3 == 0) p.mt = 3;
  const int wn = 4 / p.wm;
  const int mb = p.wm * p.mt * 16;
  const int gy = (cout + mb - 1) / mb;
  p.nt = 1;
  for (int nt = 4; nt >= 2; nt >>= 1) {
    const int tp = wn * nt * 16;
    if (tp / 2 >= hw) continue;  // tile would be mostly outside the image
    const int64_t wgs = (int64_t)((hw + tp - 1) / tp) * gy * n;
    if (wgs >= 512) { p.nt = nt; break; }  // keep at least two workgroups per compute unit
  }
  const int tp = wn * p.nt * 16;
  const int halo = taps == 9 ? w + 1 : 0;
  p.CS = pad16mod32(tp + 2 * halo);
  p.MS = pad16mod32(mb);
  p.lds = (size_t)(KC * p.CS + taps * KC * p.MS) * sizeof(float);
  p.grid = dim3((unsigned)((hw + tp - 1) / tp), (unsigned)gy, (unsigned)n);
  return p;
}

template <int TAPS, int MT>
hipError_t launch_igemm_nt(const IgemmPlan& p, const float* in, int64_t in_stride, WeightView wv,
                           float* out, int64_t out_stride, int cin, int cout, int h, int w,
                           hipStream_t st) {
#define DNB_IGEMM(NT)                                                                              \
  hipLaunchKernelGGL((k_conv_igemm<TAPS, MT, NT>), p.grid, dim3(256), p.lds, st, in, in_stride,    \
                     wv.w, wv.sm, wv.sc, wv.flip, out, out_stride, cin, cout, h, w, p.wm, p.CS, p.MS)
  switch (p.nt) {
    case 4: DNB_IGEMM(4); break;
    case 2: DNB_IGEMM(2); break;
    default: DNB_IGEMM(1); break;
  }
#undef DNB_IGEMM
  return hipGetLastError();
}

template <int TAPS>
hipError_t launch_igemm_mt(const IgemmPlan& p, const float* in, int64_t in_stride, WeightView wv,
                           float* out, int64_t out_stride, int cin, int cout, int h, int w,
                           hipStream_t st) {
  switch (p.mt) {
    case 4: return launch_igemm_nt<TAPS, 4>(p, in, in_stride, wv, out, out_stride, cin, cout, h, w, st);
    case 3: return launch_igemm_nt<TAPS, 3>(p, in, in_stride, wv, out, out_stride, cin, cout, h, w, st);
    case 2: return launch_igemm_nt<TAPS, 2>(p, in, in_stride, wv, out, out_stride, cin, cout, h, w, st);
    default: return launch_igemm_nt<TAPS, 1>(p, in, in_stride, wv, out, out_stride, cin, cout, h, w, st);
  }
}

struct WgradPlan {
  int mtw, ctw, tw;
  int cpi, total, cps, splits;
  int PA, PG;
  dim3 grid;
  size_t lds;
};

WgradPlan plan_wgrad(int n, int cin, int cout, int h, int w, int taps) {
  WgradPlan p;
  const int hw = h * w, mtiles = (cout + 15) / 16, ctiles = (cin + 15) / 16;
  if (taps == 9) {
    p.mtw = 1; p.ctw = ctiles < 3 ? ctiles : 3; p.tw = 7;   // up to 27 tiles over 4 waves
  } else {
    p.mtw = mtiles < 3 ? mtiles : 3; p.ctw = ctiles < 4 ? ctiles : 4; p.tw = 3;  // up to 12 tiles
  }
  const int gy = (ctiles + p.ctw - 1) / p.ctw, gz = (mtiles + p.mtw - 1) / p.mtw;
  p.cpi = (hw + TPIX - 1) / TPIX;
  p.total = n * p.cpi;
  int splits = 1024 / (gy * gz);
  if (splits < 1) splits = 1;
  if (splits > p.total) splits = p.total;
  if (splits > 64) splits = 64;
  p.cps = (p.total + splits - 1) / splits;
  p.splits = (p.total + p.cps - 1) / p.cps;
  const int halo = taps == 9 ? w + 1 : 0;
  p.PA = pad4mod64(TPIX + 2 * halo);
  p.PG = pad4mod64(TPIX);
  p.lds = (size_t)(p.ctw * 16 * p.PA + p.mtw * 16 * p.PG) * sizeof(float);
  p.grid = dim3((unsigned)p.splits, (unsigned)gy, (unsigned)gz);
  return p;
}

}  // namespace

hipError_t launch_conv_igemm(const float* in, int64_t in_stride, WeightView wv, const float* packed,
                             float* out, int64_t out_stride, int n, int cin, int cout, int h, int w,
                             int taps, ConvExtras* ex, hipStream_t st) {
  if (n <= 0 || cout <= 0 || h <= 0 || w <= 0) return hipSuccess;
  if (ex) ex->used_fast = false;
  if (packed && conv_fast_ok(in, in_stride, out, out_stride, h, w, taps) &&
      launch_conv_fast(in, in_stride, packed, out, out_stride, n, cin, cout, h, w, taps,
                       ex ? ex->fold : nullptr, ex ? ex->stats_part : nullptr,
                       ex ? &ex->stats_T : nullptr, st, ex ? ex->ev_start : nullptr,
                       ex ? ex->ev_stop : nullptr)) {
    if (ex) ex->used_fast = true;
    return hipGetLastError();
  }
  if (ex && ex->fold) return hipErrorInvalidValue;  // the generic kernels have no BN prologue
  const IgemmPlan p = plan_igemm(n, cout, h, w, taps);
  if (p.lds > 64 * 1024) return hipErrorInvalidValue;
  if (taps == 9) return launch_igemm_mt<9>(p, in, in_stride, wv, out, out_stride, cin, cout, h, w, st);
  return launch_igemm_mt<1>(p, in, in_stride, wv, out, out_stride, cin, cout, h, w, st);
}

bool conv_generic_fits(int n, int cin, int cout, int h, int w, int taps) {
  return plan_igemm(n, cout, h, w, taps).lds <= 64 * 1024 && plan_igemm(n, cin, h, w, taps).lds <= 64 * 1024 &&
         plan_wgrad(n, cin, cout, h, w, taps).lds <= 64 * 1024;
}

int conv_wgrad_splits(int n, int cin, int cout, int h, int w, int taps) {
  return plan_wgrad(n, cin, cout, h, w, taps).splits;
}

size_t conv_wgrad_partial_floats(int n, int cin, int cout, int h, int w, int taps) {
  const size_t a = (size_t)conv_wgrad_splits(n, cin, cout, h, w, taps) * cin * cout * taps;
  const size_t b = conv_wgrad_fast_partial_floats(n, cin, cout, h, w, taps);
  return a > b ? a : b;
}

hipError_t launch_pending_sum(PendingSum* p, hipStream_t st) {
  hipError_t e = hipSuccess;
  if (p->kind == 1) e = launch_sum_partials(p->part, p->splits, p->count, p->out, st);
  else if (p->kind == 2) e = launch_sum_wgrad3x3(*p, st);
  p->kind = 0;
  return e;
}

hipError_t launch_conv_wgrad(const float* in, int64_t in_stride, const float* g, int64_t g_stride,
                             float* dw, int n, int cin, int cout, int h, int w, int taps,
                             float* partials, const float2* fold, hipStream_t st, hipEvent_t ev0,
                             hipEvent_t ev1, bool* used_fast, PendingSum* absorb, PendingSum* defer) {
  if (defer) defer->kind = 0;
  if (cin <= 0 || cout <= 0) return absorb ? launch_pending_sum(absorb, st) : hipSuccess;
  if (used_fast) *used_fast = true;
  PendingSum own;
  if (launch_wgrad_fast(in, in_stride, g, g_stride, partials, dw, n, cin, cout, h, w, taps, fold, &own, absorb, st,
                        ev0, ev1)) {
    if (defer) { *defer = own; return hipGetLastError(); }
    return launch_pending_sum(&own, st);
  }
  if (used_fast) *used_fast = false;
  if (absorb) {
    const hipError_t e = launch_pending_sum(absorb, st);
    if (e != hipSuccess) return e;
  }
  if (fold) return hipErrorInvalidValue;  // the generic kernel has no BN prologue
  const WgradPlan p = plan_wgrad(n, cin, cout, h, w, taps);
  if (p.lds > 64 * 1024) return hipErrorInvalidValue;
  if (taps == 9)
    hipLaunchKernelGGL((k_conv_wgrad<9, 7>), p.grid, dim3(256), p.lds, st, in, in_stride, g, g_stride,
                       partials, cin, cout, h, w, p.cpi, p.total, p.cps, p.mtw, p.ctw, p.PA, p.PG);
  else
    hipLaunchKernelGGL((k_conv_wgrad<1, 3>), p.grid, dim3(256), p.lds, st, in, in_stride, g, g_stride,
                       partials, cin, cout, h, w, p.cpi, p.total, p.cps, p.mtw, p.ctw, p.PA, p.PG);
  return launch_sum_partials(partials, p.splits, (int64_t)cin * cout * taps, dw, st);
}

hipError_t launch_conv_wgrad_pair(const float* in1, int64_t in1_stride, const float* g1, int64_t g1_stride,
                                  float* dw1, int cin1, float* part1, const float2* fold1, const float* in3,
                                  int64_t in3_stride, const float* g3, int64_t g3_stride, float* dw3, int cout3,
                                  float* part3, const float2* fold3, int n, int B, int h, int w, hipStream_t st,
                                  PendingSum* pend1, PendingSum* pend3, const BnBwdPartialArgs* bn, bool* bn_done,
                                  hipEvent_t ev0, hipEvent_t ev1, bool* paired) {
  PendingSum own1, own3;
  if (paired) *paired = false;
  if (bn_done) *bn_done = false;
  if (cin1 > 0 && B > 0 && cout3 > 0 &&
      launch_wgrad_pair_fast(in1, in1_stride, g1, g1_stride, part1, dw1, cin1, fold1, in3, in3_stride, g3, g3_stride,
                             part3, dw3, cout3, fold3, n, B, h, w, &own1, &own3, pend1, pend3, bn, st, ev0, ev1)) {
    *pend1 = own1;
    *pend3 = own3;
    if (bn_done) *bn_done = bn != nullptr;
    if (paired) *paired = true;
    return hipGetLastError();
  }
  hipError_t e = launch_conv_wgrad(in3, in3_stride, g3, g3_stride, dw3, n, B, cout3, h, w, 9, part3, fold3, st, nullptr,
                                   nullptr, nullptr, pend3, &own3);
  if (e != hipSuccess) return e;
  *pend3 = own3;
  e = launch_conv_wgrad(in1, in1_stride, g1, g1_stride, dw1, n, cin1, B, h, w, 1, part1, fold1, st, nullptr, nullptr,
                        nullptr, pend1, &own1);
  *pend1 = own1;
  return e;
}

}  // namespace dnb
