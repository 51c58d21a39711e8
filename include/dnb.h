/*
 * dnb.h -- C ABI of the memory-efficient DenseNet dense block for AMD MI355X (gfx950).
 *
 * One dense block (paper, Section 2): x_l = H_l([x_0, x_1, ..., x_{l-1}]) for
 * l = 1..m, with H_l the pre-activation composite BN -> ReLU -> 1x1 conv (to B
 * "bottleneck" channels) -> BN -> ReLU -> 3x3 conv (to k "growth" channels),
 * run forward and backward through the Shared Memory Storage scheme of
 * Section 4: the concatenated input of a layer goes to shared storage 1, its
 * BN+ReLU output to shared storage 2 (the bottleneck's second BN+ReLU output to
 * a third shared buffer); every layer overwrites them and the backward pass
 * re-populates them by recomputation before ordinary back-propagation, so the
 * only feature maps that persist are convolution outputs and feature-map memory
 * is linear in m (Section 4, last paragraph; Section 5).
 *
 * Conventions
 *   - Every pointer named x0, params, y, dy, dx0, dparams, workspace is a DEVICE
 *     pointer owned by the caller (e.g. torch.empty(...).data_ptr()), at least
 *     16-byte aligned (params and dparams: 4-byte).  The library never allocates or
 *     frees device memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = default stream).  Calls
 *     enqueue kernels on it and return without synchronising.  Calls that share
 *     a workspace must be ordered on one stream: the shared buffers are
 *     overwritten layer by layer.
 *   - Every function returning int returns DNB_OK (0) or a negative DNB_E_* code;
 *     nothing throws or aborts.  Only argument and launch errors are reported
 *     synchronously.
 *   - Tensors are dense, row-major, in the layout named by the descriptor:
 *     NCHW (n, c, h, w) or NHWC (n, h, w, c).
 *   - Built combinations: DNB_F32 + DNB_NCHW and DNB_BF16 + DNB_NHWC, each with every schedule
 *     (bf16: c0, growth, bottleneck multiples of 8); bottleneck = 0 with DNB_F32 and the shared
 *     and store-all schedules.  Others return DNB_E_UNSUPPORTED from dnb_block_create.
 *   - DNB_BF16: x0, y, dy, dx0 are bfloat16 (2 bytes per element).  params and dparams
 *     stay fp32 in the same pack layout (conv weights are rounded to bf16 when the
 *     forward packs them; parameter gradients are fp32 sums); BN statistics and all
 *     accumulation are fp32; the internal gradient slab is fp32.
 */
#ifndef DNB_H_
#define DNB_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dnb_block dnb_block; /* opaque, host side only */

enum { DNB_OK = 0, DNB_E_BADDESC = -1, DNB_E_NULL = -2, DNB_E_ALIGN = -3, DNB_E_LAUNCH = -4,
       DNB_E_UNSUPPORTED = -5, DNB_E_RANGE = -6, DNB_E_NOMEM = -7 };

enum { DNB_F32 = 0, DNB_BF16 = 1 };  /* storage type of feature maps; accumulation and BN statistics are fp32 */
enum { DNB_NCHW = 0, DNB_NHWC = 1 };
/* Section 5 compares exactly these two ways of running the same arithmetic. */
enum { DNB_SCHED_SHARED = 0,     /* Section 4: shared storage + recomputation (linear memory)   */
       DNB_SCHED_STORE_ALL = 1,  /* Section 3: every concat / BN output kept (quadratic memory) */
       /* Section 4 taken one step further: the concatenated and normalised features are
        * recomputed inside the convolutions' operand loads, in forward and backward, so the
        * shared storage is never materialised at all (same numbers, linear memory with a
        * smaller constant).  Needs w % 4 == 0 and B*(2w+72)*4 bytes <= 64 KB of LDS,
        * else dnb_block_create returns DNB_E_UNSUPPORTED. */
       DNB_SCHED_FUSED = 2 };
/* Parameter tensors of one layer, in pack order. */
enum { DNB_P_G1 = 0, DNB_P_B1 = 1, DNB_P_W1 = 2, DNB_P_G2 = 3, DNB_P_B2 = 4, DNB_P_W3 = 5 };

typedef struct {
  int32_t n, c0, h, w;  /* block input x0 is (n, c0, h, w)                            */
  int32_t layers;       /* m >= 1                                                     */
  int32_t growth;       /* k >= 1, channels added per layer                           */
  int32_t bottleneck;   /* B >= 1, width of the 1x1 conv output (4k in DenseNet-BC);  *
                         * 0 = no bottleneck: BN -> ReLU -> 3x3 on the concatenation  *
                         * (fp32 NCHW, shared and store-all schedules)                */
  int32_t dtype;        /* DNB_F32 | DNB_BF16                                         */
  int32_t layout;       /* DNB_NCHW | DNB_NHWC                                        */
  int32_t schedule;     /* DNB_SCHED_*                                                */
  float eps;            /* BN epsilon (inside the square root)                        */
} dnb_block_desc;

/* Byte accounting of one block.  With P = n*h*w pixels, s = bytes per element,
 * C_l = c0 + (l-1)k, C_m the widest layer input and C_out = c0 + m*k:
 *   shared schedule   : stored = (m*B + m*k) P s        shared = (2 C_m + B) P s
 *   fused schedule    : stored = (m*B + m*k) P s        shared = 0
 *   store-all schedule: stored = (2 sum_l C_l + m(2B + k)) P s   shared = 0
 *   both              : grad   = (C_out + C_m + B) P s
 *   peak = stored + shared + grad.
 * `stored` counts the m*k channels x_1..x_m although they live inside the
 * caller's output y (they are conv feature maps the method keeps; Section 4). */
typedef struct {
  uint64_t stored_fwd_bytes;  /* conv outputs kept from forward to backward                     */
  uint64_t shared_fwd_bytes;  /* shared storage 1, 2 and 3                                      */
  uint64_t grad_bytes;        /* gradient slab G (C_out) + the two shared gradient scratch maps */
  uint64_t peak_bytes;        /* sum of the three lines above: the feature-map memory           */
  uint64_t stats_bytes;       /* cached fp32 per-channel BN mean and 1/sqrt(var+eps)            */
  uint64_t scratch_bytes;     /* reduction partials (not feature maps)                          */
  uint64_t workspace_bytes;   /* what the caller must allocate: everything above that lives in
                                 the workspace, plus alignment padding                          */
} dnb_block_memory;

/* A dense block as Section 4 sets it up: one object owns the plan of the block-wide shared
 * storages (storage 1 for the concatenated features, storage 2 for their BN+ReLU output, the
 * third one for the bottleneck's BN+ReLU output, the shared gradient storage) and of the
 * convolution outputs that persist, for the layer shapes of Section 2 (m layers, growth k,
 * optional bottleneck B).  dnb_block_create validates the descriptor and builds that plan
 * (buffer offsets inside the caller's workspace, launch shapes) in host memory only; shapes
 * whose LDS tiles or launch plans are not built fail here (DNB_E_UNSUPPORTED), not at launch.
 * *out is set on success.  dnb_block_destroy frees the host object (and the helper streams a
 * concurrent backward created); the workspace stays the caller's. */
int dnb_block_create(const dnb_block_desc* desc, dnb_block** out);
void dnb_block_destroy(dnb_block* b);

/* Feature-map bytes the block needs at its peak (formula above; Section 4/5:
 * linear in m for DNB_SCHED_SHARED, quadratic for DNB_SCHED_STORE_ALL). */
size_t dnb_block_peak_bytes(const dnb_block* b);
/* Size of the single device workspace the caller passes to forward/backward: the feature maps
 * of dnb_block_peak_bytes that do not live in y, plus cached BN statistics (Section 4: only the
 * apply is recomputed) and reduction scratch. */
size_t dnb_block_workspace_bytes(const dnb_block* b);
/* The terms of the byte formula above one by one (Section 5 compares exactly these: what is
 * stored against what is shared). */
int dnb_block_memory_breakdown(const dnb_block* b, dnb_block_memory* out);

/* Parameter pack (the parameters of the composite function H_l, Section 2: BN scale and bias,
 * the 1x1 bottleneck weights, second BN, the 3x3 weights): fp32 for both storage types, per
 * layer l = 1..m in order
 *   g1[C_l] b1[C_l] W1[B][C_l] g2[B] b2[B] W3[k][B][3][3]
 * (OIHW).  `dparams` has the identical layout.  Offsets and counts are in elements;
 * dnb_block_param_bytes = 4 * dnb_block_param_count is what the caller allocates for each. */
size_t dnb_block_param_count(const dnb_block* b);
size_t dnb_block_param_bytes(const dnb_block* b);
int dnb_block_param_offset(const dnb_block* b, int layer /*1-based*/, int which /*DNB_P_* */,
                           size_t* offset, size_t* count);

/* Forward (Section 4, "Putting these pieces together"): for l = 1..m concat ->
 * storage 1, BN+ReLU -> storage 2, 1x1 conv -> b_l (kept), BN+ReLU -> storage 3,
 * 3x3 conv -> x_l, written straight into y.
 *   x0      in   (n, c0, h, w)
 *   params  in   parameter pack
 *   y       out  (n, c0 + m*k, h, w) = [x0, x_1, ..., x_m], oldest first
 *   workspace    >= dnb_block_workspace_bytes; must stay untouched, together with
 *                y, until the matching backward has run. */
int dnb_block_forward(dnb_block* b, const void* x0, const void* params, void* y, void* workspace,
                      void* stream);

/* Backward (Section 4): for l = m..1 re-populate the shared storage by
 * recomputing concat and BN+ReLU from the kept conv outputs and cached
 * statistics, then back-propagate through 3x3 conv, BN+ReLU, 1x1 conv, BN+ReLU
 * and the concatenation (slice-accumulate into the gradient slab).
 *   y       in   the forward's output (holds x0 and every x_l)
 *   dy      in   gradient w.r.t. y, same shape
 *   dx0     out  gradient w.r.t. x0 (overwritten)
 *   dparams out  gradient pack, fp32, same layout as params (overwritten) */
int dnb_block_backward(dnb_block* b, const void* params, const void* y, const void* dy, void* dx0,
                       void* dparams, void* workspace, void* stream);

/* The ReLU decisions of the block (Section 3: the non-linearity is applied in place, so only its
 * sign decisions are ever needed again) exactly as its kernels take them, for checking results
 * against an evaluation in another precision: one byte (1: pre-activation > 0) per element.
 *   d1  first BN of every layer: the layers' (n, C_l, h, w) arrays [NHWC: (n, h, w, C_l)] one after
 *       the other, l = 1..m; dnb_block_relu_decision_bytes(b, 1) bytes
 *   d2  second BN: m arrays of (n, B, h, w) [NHWC: (n, h, w, B)]; ..._bytes(b, 2); unused (may be
 *       NULL) without a bottleneck
 * Call after dnb_block_forward on the same y and workspace (it reads the cached statistics and
 * the kept b_l), on the same stream.  d1, d2 are device pointers owned by the caller. */
size_t dnb_block_relu_decision_bytes(const dnb_block* b, int which);
int dnb_block_relu_decisions(dnb_block* b, const void* params, const void* y, const void* workspace, void* d1,
                             void* d2, void* stream);

/* Section 4's "regular back-propagation" after re-population leaves the order of independent
 * kernels open: the backward pass can run its two weight-gradient chains on helper streams owned by the block
 * (created at the first such backward call, joined to `stream` before the call's last kernel),
 * so that they overlap the data-gradient chain.  enable = 0 puts everything on `stream` in
 * program order; results are bit-identical either way.  Default: disabled for fp32 (measured
 * slower on one MI355X), enabled for bf16. */
int dnb_block_set_concurrency(dnb_block* b, int enable);

const char* dnb_status_string(int status);

/* ---- single operations of the path (fp32 NCHW), exported for tests and
 * micro-benchmarks.  A "slab" is an (n, c, hw) tensor whose image stride
 * (elements between consecutive n) is given explicitly, so channel ranges of a
 * wider tensor can be addressed in place. */

/* Section 2 "Contiguous concatenation": dst[i][0:len] = src[i][0:len], i < n. */
int dnb_op_copy_slab(const void* src, int64_t src_stride, void* dst, int64_t dst_stride, int64_t n,
                     int64_t len, void* stream);
/* Scratch (device bytes) the two BN reductions below need for an (n, c, hw) slab. */
size_t dnb_op_bn_scratch_bytes(int64_t n, int64_t c, int64_t hw);
/* BN batch statistics per channel: mean and 1/sqrt(biased var + eps). */
int dnb_op_bn_stats(const void* x, int64_t stride, int64_t n, int64_t c, int64_t hw, float eps,
                    void* mean, void* istd, void* scratch, void* stream);
/* dnb_op_bn_stats for callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): same kernels and results, but the
 * split-reduction partials live in a 256 KiB device array inside the library instead of a
 * caller's scratch buffer.  The call allocates and frees nothing.  DNB_E_RANGE if the shape needs
 * more than 256 KiB of partials (12 bytes per channel and image split: every shape up to 1024
 * channels fits, and up to 21845 channels with one split).
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different
 * streams) race and must be ordered by the caller.  The array's device address is looked up on
 * the first call on each device (not while that call's stream is being captured). */
int dnb_op_bn_stats_static(const void* x, int64_t stride, int64_t n, int64_t c, int64_t hw, float eps,
                           void* mean, void* istd, void* stream);
/* out = max(0, gamma*(x-mean)*istd + beta) (BN apply with in-place ReLU, Section 3). */
int dnb_op_bn_relu(const void* x, int64_t x_stride, void* out, int64_t out_stride, int64_t n,
                   int64_t c, int64_t hw, const void* gamma, const void* beta, const void* mean,
                   const void* istd, void* stream);
/* Reverse of dnb_op_bn_relu.  dact = gradient w.r.t. the post-ReLU output.
 * dgamma/dbeta are overwritten; du is overwritten (accumulate = 0) or added to. */
int dnb_op_bn_relu_backward(const void* x, int64_t x_stride, const void* dact, int64_t dact_stride,
                            void* du, int64_t du_stride, int accumulate, int64_t n, int64_t c,
                            int64_t hw, const void* gamma, const void* beta, const void* mean,
                            const void* istd, void* dgamma, void* dbeta, void* scratch,
                            void* stream);
/* Second pass of dnb_op_bn_relu_backward alone (the per-element apply), reusing the partial
 * sums a previous full call left in `scratch` for the same shape: lets a benchmark time the
 * apply kernel by itself.  ev_start / ev_stop (hipEvent_t as void*, may be NULL) are stamped
 * at the kernel's own start and end on `stream`. */
int dnb_op_bn_relu_backward_apply(const void* x, int64_t x_stride, const void* dact, int64_t dact_stride,
                                  void* du, int64_t du_stride, int accumulate, int64_t n, int64_t c,
                                  int64_t hw, const void* gamma, const void* beta, const void* mean,
                                  const void* istd, void* dgamma, void* dbeta, const void* scratch,
                                  void* ev_start, void* ev_stop, void* stream);
/* Convolutions: ks = 1 or 3, stride 1, zero padding (ks-1)/2, no bias,
 * cross-correlation; weights OIHW (cout, cin, ks, ks).  `scratch` holds the re-laid
 * weights (forward, dgrad: dnb_op_conv_scratch_bytes) or the split reduction partials of
 * the weight gradient (dnb_op_conv_wgrad_scratch_bytes). */
size_t dnb_op_conv_scratch_bytes(int64_t cin, int64_t cout, int ks); /* packed weights */
int dnb_op_conv_forward(const void* x, int64_t x_stride, const void* wgt, void* out,
                        int64_t out_stride, int64_t n, int64_t cin, int64_t cout, int64_t h,
                        int64_t w, int ks, void* scratch, void* stream);
/* The fused schedule's forward convolution as one operation (the "BN-apply+ReLU feeding straight
 * into the conv operand" step plus the statistics its consumer needs):
 *   out = conv(max(0, x * scale_c + shift_c)),  (scale_c, shift_c) = fold[c] (cin float pairs),
 * and stats[(m*T + j)*3 ..] = (count, mean, sum of squared deviations) of output channel m over
 * pixel tile j, *tiles = T (host int).  `stats` needs dnb_op_conv_stats_bytes bytes.  Only for
 * shapes the 16-byte-vector kernels cover (pixel rows and strides multiples of 4; for ks = 3 the
 * staged tile must fit LDS), else DNB_E_UNSUPPORTED.  prepacked != 0: `scratch` already holds
 * the weights packed by an earlier call for the same wgt.  ev_start / ev_stop as above. */
size_t dnb_op_conv_stats_bytes(int64_t n, int64_t cout, int64_t h, int64_t w);
int dnb_op_conv_bnrelu_forward(const void* x, int64_t x_stride, const void* wgt, const void* fold, void* out,
                               int64_t out_stride, void* stats, int* tiles, int64_t n, int64_t cin, int64_t cout,
                               int64_t h, int64_t w, int ks, void* scratch, int prepacked, void* ev_start,
                               void* ev_stop, void* stream);
/* The fused schedule's weight gradient as one operation: dwgt = wgrad(max(0, x*scale_c + shift_c), dout),
 * the BN+ReLU of the activation operand recomputed in the operand load (fold as above).
 * scratch: dnb_op_conv_wgrad_scratch_bytes.  ev_start / ev_stop are stamped around the gradient
 * kernel itself (the small kernel that adds its partial sums follows it).  Same shape limits as
 * dnb_op_conv_bnrelu_forward, else DNB_E_UNSUPPORTED. */
int dnb_op_conv_bnrelu_wgrad(const void* x, int64_t x_stride, const void* fold, const void* dout,
                             int64_t dout_stride, void* dwgt, int64_t n, int64_t cin, int64_t cout, int64_t h,
                             int64_t w, int ks, void* scratch, void* ev_start, void* ev_stop, void* stream);
/* Both weight gradients of a bottleneck layer in the fused schedule, as the one launch the
 * backward pass issues for them when it runs on one stream (Section 4's recomputation folded
 * into the operand loads):
 *   dW1 (B, cin)       = 1x1 weight gradient of max(0, x1[:, :cin]*s1 + t1) and db
 *   dW3 (k, B, 3, 3)   = 3x3 weight gradient of max(0, b*s2 + t2) and g
 * x1: (n, >= cin, h, w) with image stride x1_stride; db, b: (n, B, h, w) contiguous; g: (n, k,
 * h, w) with image stride g_stride; fold1 (cin pairs), fold2 (B pairs) as above.  If bn_dact is
 * not null the launch also carries the reduction pass of the layer's first BN backward over
 * x1[:, :cin] and bn_dact (n, cin, h, w) (bn_gamma, bn_beta, bn_mean, bn_istd: cin floats each;
 * its partial sums stay in scratch, at byte offset dnb_op_layer_wgrads_bn_partials_offset, where
 * dnb_op_bn_relu_backward_apply finds them when given scratch + that offset).  The two small kernels that add the weight gradients'
 * partial sums follow the launch; ev_start / ev_stop are stamped around the launch itself.
 * scratch: dnb_op_layer_wgrads_scratch_bytes.  DNB_E_UNSUPPORTED unless B >= 48, the image is
 * 16-byte friendly (h*w % 4 == 0, w % 4 == 0) and (B, k) is a combination the paired kernel
 * is built for ((48, <=16) or (>=32 with two 16-channel tiles each way)). */
size_t dnb_op_layer_wgrads_scratch_bytes(int64_t n, int64_t cin, int64_t bottleneck, int64_t growth, int64_t h,
                                         int64_t w);
size_t dnb_op_layer_wgrads_bn_partials_offset(int64_t n, int64_t cin, int64_t bottleneck, int64_t growth, int64_t h,
                                              int64_t w);
int dnb_op_layer_wgrads(const void* x1, int64_t x1_stride, const void* fold1, const void* db, void* dw1, int64_t cin,
                        const void* b, const void* fold2, const void* g, int64_t g_stride, void* dw3, int64_t n,
                        int64_t bottleneck, int64_t growth, int64_t h, int64_t w, const void* bn_dact,
                        const void* bn_gamma, const void* bn_beta, const void* bn_mean, const void* bn_istd,
                        void* scratch, void* ev_start, void* ev_stop, void* stream);
int dnb_op_conv_dgrad(const void* dout, int64_t dout_stride, const void* wgt, void* din,
                      int64_t din_stride, int64_t n, int64_t cin, int64_t cout, int64_t h, int64_t w,
                      int ks, void* scratch, void* stream);
size_t dnb_op_conv_wgrad_scratch_bytes(int64_t n, int64_t cin, int64_t cout, int64_t h, int64_t w,
                                       int ks);
int dnb_op_conv_wgrad(const void* x, int64_t x_stride, const void* dout, int64_t dout_stride,
                      void* dwgt, int64_t n, int64_t cin, int64_t cout, int64_t h, int64_t w, int ks,
                      void* scratch, void* stream);

/* ---- single operations of the bf16 / NHWC path.  Feature maps are bf16 with channels
 * contiguous; "ld" is the pixel stride in elements, so channel ranges of a wider tensor are
 * addressed in place; channel counts are multiples of 8.  Weights and weight gradients are fp32
 * OIHW.  `scratch`: dnb_op_nhwc_scratch_bytes(n, cin, cout, h, w, ks) device bytes.  Feature-map
 * pointers and `scratch` are 16-byte aligned (else DNB_E_ALIGN); an "ld" is at least the channel
 * count and a multiple of 8 (of 4 for an fp32 tensor), else DNB_E_RANGE. */
size_t dnb_op_nhwc_scratch_bytes(int64_t n, int64_t cin, int64_t cout, int64_t h, int64_t w, int ks);
int dnb_op_nhwc_conv_forward(const void* x, int64_t x_ld, const void* wgt, void* out, int64_t out_ld, int64_t n,
                             int64_t cin, int64_t cout, int64_t h, int64_t w, int ks, void* scratch, void* stream);
/* dout is bf16, or fp32 if dout_is_f32 (the block keeps its gradient slab in fp32). */
int dnb_op_nhwc_conv_dgrad(const void* dout, int64_t dout_ld, int dout_is_f32, const void* wgt, void* din,
                           int64_t din_ld, int64_t n, int64_t cin, int64_t cout, int64_t h, int64_t w, int ks,
                           void* scratch, void* stream);
int dnb_op_nhwc_conv_wgrad(const void* x, int64_t x_ld, const void* dout, int64_t dout_ld, int dout_is_f32, void* dwgt,
                           int64_t n, int64_t cin, int64_t cout, int64_t h, int64_t w, int ks, void* scratch,
                           void* stream);
/* BN+ReLU backward over (pixels, c): du is written as bf16 to du_bf16 (may alias dact), or, if
 * du_accum_f32 != NULL, added into that fp32 tensor instead. */
int dnb_op_nhwc_bn_relu_backward(const void* x, int64_t x_ld, const void* dact, int64_t dact_ld, void* du_bf16,
                                 int64_t du_ld, void* du_accum_f32, int64_t acc_ld, int64_t pixels, int64_t c,
                                 const void* gamma, const void* beta, const void* mean, const void* istd,
                                 void* dgamma, void* dbeta, void* scratch, void* stream);

/* ------------------------------------------------------------------------------------------
 * Whole training step of a CIFAR-shaped DenseNet-BC (fp32, NCHW): the dense blocks above joined
 * by the network's glue (paper Section 2, "DenseNet Architecture": dense blocks connected by
 * transition layers; Section 5 measures such networks).
 *   stem      3x3 conv, pad 1, 3 -> 2k channels, no bias
 *   3 x       dense block of (depth-4)/6 bottleneck layers (B = 4k), run under `schedule`
 *   between   transition: BN -> ReLU -> 1x1 conv (C -> C/2) -> 2x2 average pool, stride 2
 *   tail      BN -> ReLU -> global average pool -> linear (+bias) to `classes`
 *   loss      mean over the batch of the softmax cross-entropy
 * BN uses batch statistics as in the blocks.  Parameter pack (fp32; gradients same layout):
 *   stem W[2k][3][3][3] | block0 | trans0: g[C] b[C] W[C/2][C] | block1 | trans1 | block2 |
 *   tail: g[C] b[C] Wl[classes][C] bl[classes]
 * (query the offsets).  x is (n, 3, image, image) fp32, labels n int32 in [0, classes): device
 * pointers (a sample whose label is out of range adds nothing to the loss or the gradients).
 * loss (1 float) and logits (n*classes floats, may be NULL) are device pointers too.
 * dnb_net_backward needs the preceding dnb_net_forward on the same workspace and overwrites
 * dparams.  Errors and ownership as for the block calls. */
typedef struct dnb_net dnb_net;
typedef struct {
  int32_t n, image;   /* batch; input height = width, a multiple of 4 */
  int32_t depth;      /* L = 6*layers_per_block + 4 */
  int32_t growth;     /* k */
  int32_t classes;
  int32_t schedule;   /* DNB_SCHED_* of the dense blocks */
  float eps;
} dnb_net_desc;
/* parts of the network pack for dnb_net_param_offset */
enum { DNB_NP_STEM = 0, DNB_NP_BLOCK0 = 1, DNB_NP_BLOCK1 = 2, DNB_NP_BLOCK2 = 3,
       DNB_NP_TRANS0_G = 4, DNB_NP_TRANS0_B = 5, DNB_NP_TRANS0_W = 6,
       DNB_NP_TRANS1_G = 7, DNB_NP_TRANS1_B = 8, DNB_NP_TRANS1_W = 9,
       DNB_NP_TAIL_G = 10, DNB_NP_TAIL_B = 11, DNB_NP_TAIL_WL = 12, DNB_NP_TAIL_BL = 13 };

int dnb_net_create(const dnb_net_desc* desc, dnb_net** out);
void dnb_net_destroy(dnb_net* net);
size_t dnb_net_param_count(const dnb_net* net);      /* floats in params / dparams */
int dnb_net_param_offset(const dnb_net* net, int part /*DNB_NP_* */, size_t* offset, size_t* count);
size_t dnb_net_workspace_bytes(const dnb_net* net);  /* bytes the caller allocates */
/* feature-map bytes of the whole step: the blocks' exact accounting plus the glue's feature maps */
size_t dnb_net_peak_bytes(const dnb_net* net);
/* The i-th piece carved from the workspace (i = 0, 1, ... until DNB_E_RANGE): its name ("feat",
 * "y", "block_ws", "tz", "mean", "istd", "pack": one per block `index`; "tconv", "gy", "dtz",
 * "dconv", "dfeat", "part", "pooled", "dpooled", "logits", "dlogits", "terms": shared by all
 * blocks), byte offset and size.  Host only; lets a caller or a test check the plan. */
int dnb_net_workspace_piece(const dnb_net* net, int i, const char** name, int* index, size_t* offset, size_t* bytes);
/* Every ReLU decision of the step as the kernels take it (see dnb_block_relu_decisions), one byte
 * each: for block b = 0, 1, 2 the block's d1, its d2, then the decisions of the BN+ReLU that
 * follows the block (transition b or the tail), (n, C_out_b, h_b, w_b).  Call after
 * dnb_net_forward on the same workspace and stream; `out` is a device pointer. */
size_t dnb_net_relu_decision_bytes(const dnb_net* net);
int dnb_net_relu_decisions(dnb_net* net, const void* params, const void* workspace, void* out, void* stream);
int dnb_net_set_concurrency(dnb_net* net, int enable); /* helper streams in the blocks' backward */
int dnb_net_forward(dnb_net* net, const void* x, const int32_t* labels, const void* params, float* loss,
                    float* logits, void* workspace, void* stream);
int dnb_net_backward(dnb_net* net, const void* x, const void* params, void* dparams, void* workspace,
                     void* stream);

/* The classifier head both network steps end in (paper Section 2, "DenseNet Architecture": after the
 * last dense block the features are pooled globally and classified; trained with the softmax loss), as
 * single operations.  All tensors fp32, row-major, device pointers.
 * forward:  logits (n, classes) = pooled (n, c) . wl (classes, c)^T + bl (classes);
 *           loss = mean over the batch of -log softmax(logits)[label]; dlogits (n, classes) = its
 *           gradient; a sample whose label is outside [0, classes) adds nothing to either.
 *           terms: n floats of scratch.
 * backward: dpooled (n, c) = dlogits . wl; dwl (classes, c) = dlogits^T . pooled; dbl = column sums of dlogits.
 * DNB_E_RANGE beyond n = 4096, classes = 65536, c = 2^20. */
int dnb_op_head_forward(const void* pooled, const void* wl, const void* bl, const int32_t* labels, void* logits,
                        void* dlogits, void* terms, float* loss, int64_t n, int64_t c, int64_t classes, void* stream);
int dnb_op_head_backward(const void* dlogits, const void* pooled, const void* wl, void* dpooled, void* dwl, void* dbl,
                         int64_t n, int64_t c, int64_t classes, void* stream);

/* ------------------------------------------------------------------------------------------
 * Whole training step of an ImageNet-shaped DenseNet-BC (bf16 feature maps, NHWC; fp32 accumulation,
 * statistics, parameters and parameter gradients): four dense blocks joined by the network's glue
 * (paper Section 2, "DenseNet Architecture"; the ImageNet models of Section 5 have four blocks).
 *   stem      7x7 conv, stride 2, pad 3, 3 -> 2k channels, no bias; BN -> ReLU;
 *             3x3 max pool, stride 2, pad 1 (ties: first position in window scan order)
 *   4 x       dense block of layers[b] bottleneck layers (B = 4k), run under `schedule`
 *   between   transition: BN -> ReLU -> 1x1 conv (C -> C/2) -> 2x2 average pool, stride 2
 *   tail      BN -> ReLU -> global average pool -> linear (+bias) to `classes`
 *   loss      mean over the batch of the softmax cross-entropy
 * Parameter pack (fp32; gradients same layout; query the offsets):
 *   stem W[2k][3][7][7] g[2k] b[2k] | block 0 | trans 0: g[C] b[C] W[C/2][C] | block 1 | trans 1 |
 *   block 2 | trans 2 | block 3 | tail: g[C] b[C] Wl[classes][C] bl[classes]
 * x is (n, image, image, 3) bf16 (2-byte aligned), labels n int32: device pointers.  image is a
 * multiple of 32; 2k is 16, 32, 64 or 96 (else DNB_E_UNSUPPORTED).  Errors, ownership and the
 * forward-then-backward contract as for dnb_net_*. */
typedef struct dnb_inet dnb_inet;
typedef struct {
  int32_t n, image;     /* batch; input height = width */
  int32_t growth;       /* k */
  int32_t layers[4];    /* bottleneck layers of the four dense blocks */
  int32_t classes;
  int32_t schedule;     /* DNB_SCHED_* of the dense blocks */
  float eps;
} dnb_inet_desc;
/* parts of the pack for dnb_inet_param_offset: DNB_IP_BLOCK0 + 4*b + {0: block b, 1: g, 2: b of the
 * BN that follows it, 3: W of transition b, or Wl of the tail for b = 3} */
enum { DNB_IP_STEM_W = 0, DNB_IP_STEM_G = 1, DNB_IP_STEM_B = 2, DNB_IP_BLOCK0 = 3, DNB_IP_TAIL_BL = 19 };

int dnb_inet_create(const dnb_inet_desc* desc, dnb_inet** out);
void dnb_inet_destroy(dnb_inet* net);
size_t dnb_inet_param_count(const dnb_inet* net);
int dnb_inet_param_offset(const dnb_inet* net, int part, size_t* offset, size_t* count);
size_t dnb_inet_workspace_bytes(const dnb_inet* net);
size_t dnb_inet_peak_bytes(const dnb_inet* net);   /* feature-map bytes: the blocks' exact accounting plus the glue's */
int dnb_inet_set_concurrency(dnb_inet* net, int enable);
int dnb_inet_forward(dnb_inet* net, const void* x, const int32_t* labels, const void* params, float* loss,
                     float* logits, void* workspace, void* stream);
int dnb_inet_backward(dnb_inet* net, const void* x, const void* params, void* dparams, void* workspace,
                      void* stream);
/* The integers the step decides in floating point, as its kernels take them (for checking results
 * against an evaluation in another precision): every ReLU decision, one byte each -- the stem's BN
 * (n, image/2, image/2, 2k), then per block its d1, its d2 (see dnb_block_relu_decisions) and the
 * decisions of the BN that follows it (n, h_b, w_b, C_out_b) -- and the max pool's positions 3*i + j
 * inside each window, (n, image/4, image/4, 2k).  Call after dnb_inet_forward, same workspace and
 * stream; relu and pool are device pointers. */
size_t dnb_inet_relu_decision_bytes(const dnb_inet* net);
size_t dnb_inet_pool_position_bytes(const dnb_inet* net);
int dnb_inet_decisions(dnb_inet* net, const void* params, const void* workspace, void* relu, void* pool, void* stream);

/* The glue kernels of the ImageNet-shaped step as single operations (paper Section 2, "DenseNet
 * Architecture": a convolution and pooling before the first dense block; the ImageNet models of
 * Section 5).  Tensors NHWC bf16 unless stated, device pointers; h, w even, c a multiple of 8.
 * stem_conv7:  out (n, image/2, image/2, channels) = 7x7 stride-2 pad-3 cross-correlation of
 *              x (n, image, image, 3) with w (channels, 3, 7, 7) fp32 rounded to bf16, fp32 accumulation.
 * stem_wgrad7: dw (channels, 3, 7, 7) fp32 = its weight gradient for g (n, image/2, image/2, channels).
 *              scratch: dnb_op_stem_scratch_bytes for either; channels 16, 32, 64 or 96, image a multiple
 *              of 32 (else DNB_E_UNSUPPORTED / DNB_E_BADDESC).
 * maxpool3s2_bnrelu: out (n, h/2, w/2, c) = 3x3 stride-2 pad-1 max pool of max(0, s*scale + shift),
 *              fold = c (scale, shift) pairs fp32; pos (n, h/2, w/2, c) bytes = 3*i + j of the maximum
 *              inside its window, the first in row-by-row scan order among equals, padding excluded.
 * maxpool3s2_backward: din (n, h, w, c) = adjoint of the pooling: every window's gradient goes to the
 *              position recorded in pos; an input position adds its windows' gradients in fp32. */
size_t dnb_op_stem_scratch_bytes(int64_t n, int64_t image, int64_t channels);
int dnb_op_stem_conv7(const void* x, const void* w, void* out, int64_t n, int64_t image, int64_t channels, void* scratch,
                      void* stream);
int dnb_op_stem_wgrad7(const void* x, const void* g, void* dw, int64_t n, int64_t image, int64_t channels, void* scratch,
                       void* stream);
int dnb_op_maxpool3s2_bnrelu(const void* s, const void* fold, void* out, void* pos, int64_t n, int64_t h, int64_t w,
                             int64_t c, void* stream);
int dnb_op_maxpool3s2_backward(const void* dout, const void* pos, void* din, int64_t n, int64_t h, int64_t w, int64_t c,
                               void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DNB_H_ */
