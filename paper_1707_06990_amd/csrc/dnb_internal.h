// Internal declarations shared by the host orchestration and the kernel files of
// the dense-block library (fp32 NCHW path).  Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dnb {

// ---- element-wise and reduction kernels (HBM-bound) -------------------------------------

// dst[i][0:len] = src[i][0:len] for i < n; strides in elements.
hipError_t launch_copy_slab(const float* src, int64_t src_stride, float* dst, int64_t dst_stride,
                            int n, int64_t len, hipStream_t st);

// Per-channel batch statistics of x (n, c, hw; image stride `stride`): mean and
// 1/sqrt(biased var + eps).  The reduction is split over image ranges: launch_bn_stats_partial
// writes (count, mean, M2) per (channel, split) -- bn_stats_partial_floats(n, c, hw) floats --
// and the first kernel that needs the statistics merges them (StatsSrc below), so the forward
// chain has no separate finalisation launch.  launch_bn_stats = partials + a finalise kernel.
size_t bn_stats_partial_floats(int n, int c, int hw);
hipError_t launch_bn_stats_partial(const float* x, int64_t stride, int n, int c, int hw,
                                   float* partials, int* splits, hipStream_t st);
hipError_t launch_bn_stats(const float* x, int64_t stride, int n, int c, int hw, float eps,
                           float* mean, float* istd, float* partials, hipStream_t st);

// Where a kernel finds BN statistics: finalised arrays indexed by channel, except channels in
// [fresh_lo, fresh_hi), whose partials (index ch - fresh_lo) it merges itself and stores back.
struct StatsSrc {
  float* mean;
  float* istd;
  const float* part;
  int splits, fresh_lo, fresh_hi;
  float eps;
};

// out = max(0, fma(x, gamma*istd, beta - mean*gamma*istd)); if copy_out != nullptr the raw x
// is also written there (concatenation and BN+ReLU of the same data in one pass).
hipError_t launch_bn_relu(const float* x, int64_t x_stride, float* out, int64_t out_stride,
                          float* copy_out, int64_t copy_stride, int n, int c, int hw,
                          const float* gamma, const float* beta, StatsSrc s, hipStream_t st);

// BN+ReLU backward.  Pass 1 reduces dbeta = sum dz, dgamma = sum dz*xhat with
// dz = dact * [fma(x,scale,shift) > 0]; pass 2 writes
// du = gamma*istd*(dz - dbeta/P - xhat*dgamma/P), overwriting or accumulating.
// `partials` needs bn_bwd_partial_floats(n, c, hw) floats.
size_t bn_bwd_partial_floats(int n, int c, int hw);
// Describes the reduction pass (passes & 1) of launch_bn_relu_bwd for another launch to carry
// (launch_conv_wgrad_pair); false when the 16-byte form does not apply to these operands.
struct BnBwdPartialArgs;
bool bn_bwd_partial_plan(const float* x, int64_t x_stride, const float* dact, int64_t dact_stride, int n, int c,
                         int hw, const float* gamma, const float* beta, const float* mean, const float* istd,
                         float* partials, BnBwdPartialArgs* out);
hipError_t launch_bn_relu_bwd(const float* x, int64_t x_stride, const float* dact,
                              int64_t dact_stride, float* du, int64_t du_stride, bool accumulate,
                              int n, int c, int hw, const float* gamma, const float* beta,
                              const float* mean, const float* istd, float* dgamma, float* dbeta,
                              float* partials, hipStream_t st, int passes = 3 /*1 reduce | 2 apply*/,
                              hipEvent_t ev_start = nullptr, hipEvent_t ev_stop = nullptr);

// out[(img*c + ch)*hw + q] = 1 if fma(u[img*stride + ch*hw + q], scale, shift) > 0 else 0, with
// (scale, shift) = bn_fold(gamma, beta, mean, istd): the ReLU decision exactly as every kernel takes it.
hipError_t launch_relu_decisions(const float* u, int64_t stride, int n, int c, int hw, const float* gamma,
                                 const float* beta, const float* mean, const float* istd, unsigned char* out,
                                 hipStream_t st);

// the same for a bf16 tensor of P rows of c channels (pixel stride ld): out[p*c + ch]
hipError_t launch_relu_decisions_rows(const void* u, int64_t ld, int64_t P, int c, const float* gamma, const float* beta,
                                      const float* mean, const float* istd, unsigned char* out, hipStream_t st);

// ---- the classifier head of the network steps (fp32): linear + mean softmax cross-entropy, and its backward
hipError_t launch_head_forward(const float* pooled, const float* wl, const float* bl, const int32_t* labels, float* logits,
                               float* dlogits, float* terms, float* loss, int n, int c, int classes, hipStream_t st);
hipError_t launch_head_backward(const float* dlogits, const float* pooled, const float* wl, float* dpooled, float* dwl,
                                float* dbl, int n, int c, int classes, hipStream_t st);

// ---- convolutions (MFMA implicit GEMM, fp32) -----------------------------------------------

// Weight addressing for the implicit-GEMM kernel: element (m = output channel, c = input
// channel, t = tap) lives at w[m*sm + c*sc + (flip ? taps-1-t : t)].
struct WeightView {
  const float* w;
  int64_t sm, sc;
  int flip;
};

// Packed weights for the fast kernels: [taps][cout16][cin16], zero padded to multiples of 16,
// K index permuted inside each 16-chunk (see dnb_conv_f32_fast.hip).
size_t packed_weight_floats(int cout, int cin, int taps);
hipError_t launch_pack_weights(WeightView wv, int cout, int cin, int taps, float* packed, hipStream_t st);
// All layers of a block in one launch.  Layer l (input width c) occupies packed_layer_floats
// floats: 1x1 forward [B16][c16], 1x1 dgrad [c16][B16], 3x3 forward [9][k16][B16],
// 3x3 dgrad [9][B16][k16], in that order.
size_t packed_layer_floats(int c, int k, int B);
hipError_t launch_pack_block_weights(const float* params, float* packed, int c0, int k, int B, int m,
                                     hipStream_t st);

// out[n][m][q] = sum_{c,t} W(m,c,t) * in[n][c][q + shift(t)], zero outside the image.
// taps = 1 or 9.  Used for forward (W = OIHW as is) and data gradient (transposed, flipped).
// `packed` (may be null) is the same weight view packed by launch_pack_weights; with it, shapes
// whose pixel counts and strides are multiples of 4 take the fast kernels.
// Optional extras of the fast kernels:
//   fold        BN+ReLU prologue: the input is max(0, fma(x, fold[c].x, fold[c].y)) (fast path only)
//   stats_part  epilogue statistics of the output: [cout][stats_T][3] partials (count, mean, M2),
//               conv_stats_partial_floats floats; stats_T is set by the launcher
//   used_fast   set by the launcher; false = generic kernel ran, no statistics were written
//   ev_start / ev_stop  optional events stamped at the fast kernel's own start and end
struct ConvExtras {
  const float2* fold;
  float* stats_part;
  int stats_T;
  bool used_fast;
  hipEvent_t ev_start = nullptr, ev_stop = nullptr;
};
size_t conv_stats_partial_floats(int n, int cout, int h, int w);
hipError_t launch_conv_igemm(const float* in, int64_t in_stride, WeightView wv, const float* packed,
                             float* out, int64_t out_stride, int n, int cin, int cout, int h, int w,
                             int taps, ConvExtras* ex, hipStream_t st);
// whether the any-shape kernels (forward, data gradient, weight gradient) have LDS for this shape: they
// are the fallback wherever an operand is not 16-byte friendly, so a plan must not count on the fast ones
bool conv_generic_fits(int n, int cin, int cout, int h, int w, int taps);
bool conv_fast_ok(const float* in, int64_t in_stride, const float* out, int64_t out_stride, int h,
                  int w, int taps);

// fold[ch] = BN's affine map folded to (scale, shift) for nch channels; channels in
// [fresh_lo, fresh_hi) are first finalised from their [T][3] partial statistics.
hipError_t launch_bn_fold(const float* gamma, const float* beta, float* mean, float* istd,
                          const float* part, int T, int fresh_lo, int fresh_hi, float eps, int nch,
                          float2* fold, hipStream_t st);

// dW[m][c][t] = sum_{n,q} g[n][m][q] * in[n][c][q + shift(t)]  (OIHW result).
int conv_wgrad_splits(int n, int cin, int cout, int h, int w, int taps);
size_t conv_wgrad_partial_floats(int n, int cin, int cout, int h, int w, int taps);
// partial floats of the fast (16-byte-vector) weight-gradient kernel for this shape, 0 if its tile plan does not fit
size_t conv_wgrad_fast_partial_floats(int n, int cin, int cout, int h, int w, int taps);
// A sum of weight-gradient partials that a launch has left for later.  In a chain of weight
// gradients on one stream the next weight-gradient launch carries it out with extra workgroups
// (the partials are complete when that launch starts), which saves a launch per layer; what is
// left at the end of the chain is summed by launch_pending_sum.
struct PendingSum {
  int kind = 0;  // 0 nothing pending; 1 out[e] = sum_s part[s][e]; 2 the 3x3 fast kernel's accumulator-order partials
  const float* part = nullptr;
  float* out = nullptr;
  int splits = 0;
  int64_t count = 0;                                      // elements of one partial
  int gy = 0, gz = 0, mtw = 0, ctw = 0, cin = 0, cout = 0;  // kind 2: how a partial maps to OIHW
};
hipError_t launch_pending_sum(PendingSum* p, hipStream_t st);  // no-op for kind 0; clears *p
// fold != null applies the BN+ReLU prologue to `in` (fast path only).
// absorb: a pending sum (of another partial buffer) to carry out in this launch, or before it
// when the fast path does not apply; cleared.  defer: if given, this call's own sum is not
// launched when it can be deferred and is described there instead (kind 0 if it was launched).
hipError_t launch_conv_wgrad(const float* in, int64_t in_stride, const float* g, int64_t g_stride,
                             float* dw, int n, int cin, int cout, int h, int w, int taps,
                             float* partials, const float2* fold, hipStream_t st, hipEvent_t ev_start = nullptr,
                             hipEvent_t ev_stop = nullptr /*stamped around the fast kernel (not the sum)*/,
                             bool* used_fast = nullptr, PendingSum* absorb = nullptr, PendingSum* defer = nullptr);

// Both weight gradients of a bottleneck layer on one stream: the 1x1 (in1: C_l channels, g1: the
// gradient of b_l, B channels) and the 3x3 (in3: B channels, g3: the gradient of x_l, k
// channels).  One launch when the fast pair applies, else two launch_conv_wgrad calls.  *pend1 /
// *pend3: in, the previous layer's pending sums (carried out here); out, this layer's.
hipError_t launch_conv_wgrad_pair(const float* in1, int64_t in1_stride, const float* g1, int64_t g1_stride,
                                  float* dw1, int cin1, float* part1, const float2* fold1, const float* in3,
                                  int64_t in3_stride, const float* g3, int64_t g3_stride, float* dw3, int cout3,
                                  float* part3, const float2* fold3, int n, int B, int h, int w, hipStream_t st,
                                  PendingSum* pend1, PendingSum* pend3, const BnBwdPartialArgs* bn = nullptr,
                                  bool* bn_done = nullptr, hipEvent_t ev_start = nullptr, hipEvent_t ev_stop = nullptr,
                                  bool* paired = nullptr);
// (bn: a BN backward reduction to carry in the same launch, *bn_done says whether it was;
//  ev_start / ev_stop are stamped around the shared launch, *paired says whether there was one)

// out[e] = sum over splits of partials[split][e] (fixed order).
hipError_t launch_sum_partials(const float* partials, int splits, int64_t count, float* out, hipStream_t st);

// ---- bf16 / NHWC path (dnb_nhwc_bf16.hip): feature maps bf16 with channels contiguous, row
// strides ("ld") in elements; parameters, statistics, gradient slab and partials fp32.
namespace nhwc {
hipError_t copy_rows(const void* src, int64_t sld, void* dst, int64_t dld, int64_t P, int c, hipStream_t st);
// out = bf16(max(0, fma(x, fold.x, fold.y))) per channel; copy (may be null) = x  (storage 2 / storage 1)
hipError_t bn_relu_rows(const void* x, int64_t ld, const float2* fold, void* out, int64_t old, void* copy, int64_t cld,
                        int64_t P, int c, hipStream_t st);
hipError_t bf16_to_f32(const void* src, float* dst, int64_t count, hipStream_t st);
hipError_t f32_rows_to_bf16(const float* src, int64_t sld, void* dst, int64_t P, int c, hipStream_t st);
size_t stats_partial_floats(int64_t P, int c);
hipError_t stats_partial(const void* x, int64_t ld, int64_t P, int c, float* part, int* T, hipStream_t st);
// per layer, in order: 1x1 forward [B16][c32], 1x1 dgrad [c16][B32], 3x3 forward [9][k16][B32],
// 3x3 dgrad [9][B16][k32]  (bf16 elements; 16 / 32 = rounded up to that multiple)
size_t packed_layer_elems(int c, int k, int B);
hipError_t pack_block_weights(const float* params, void* packed, int c0, int k, int B, int m, hipStream_t st);
size_t packed_weight_elems(int cout, int cin, int taps);
hipError_t pack_weights(WeightView wv, int cout, int cin, int taps, void* packed, hipStream_t st);
size_t conv_stats_partial_floats(int n, int cout, int h, int w);
hipError_t conv(const void* in, int64_t in_ld, bool in_f32, const void* Wp, void* out, int64_t out_ld, int n,
                int cin, int cout, int h, int w, int taps, const float2* fold, float* spart, int* sT,
                hipStream_t st);
size_t wgrad_partial_floats(int n, int cin, int cout, int h, int w, int taps);
// writes per-split partials to `part` and their sum to dw ([cout][cin][taps])
hipError_t wgrad(const void* a, int64_t a_ld, const void* g, int64_t g_ld, bool g_f32, float* part, float* dw, int n,
                 int cin, int cout, int h, int w, int taps, const float2* fold, hipStream_t st);
size_t bn_bwd_partial_floats(int64_t P, int c);
hipError_t bn_relu_bwd(const void* x, int64_t x_ld, const void* dact, int64_t d_ld, void* du_bf, int64_t du_ld,
                       float* G, int64_t g_ld, int64_t P, int c, const float* gamma, const float* beta,
                       const float* mean, const float* istd, float* dgamma, float* dbeta, float* part,
                       hipStream_t st);
// its two passes on their own (the element-wise pass also over a channel sub-range)
hipError_t bn_relu_bwd_reduce(const void* x, int64_t x_ld, const void* dact, int64_t d_ld, int64_t P, int c,
                              const float* gamma, const float* beta, const float* mean, const float* istd,
                              float* dgamma, float* dbeta, float* part, hipStream_t st);
hipError_t bn_relu_bwd_apply(const void* x, int64_t x_ld, const void* dact, int64_t d_ld, void* du_bf, int64_t du_ld,
                             float* G, int64_t g_ld, int64_t P, int c, const float* gamma, const float* beta,
                             const float* mean, const float* istd, const float* dgamma, const float* dbeta,
                             hipStream_t st);
}  // namespace nhwc

}  // namespace dnb
