/*
 * cg_conv.h -- C ABI of the channel-gated convolution layer for AMD MI355X (gfx950).
 *
 * One layer of "Channel Gating Neural Networks" at inference time (paper Sec. 3.1,
 * Eq. 1, and the merged normalise-and-compare gate of Sec. 3.2):
 *
 *     x = [x_p, x_r]   split along input channels, x_p = channels [0, c_base)
 *     P = W_p * x_p                     base path, always evaluated
 *     d = (P >= E + Delta*sqrt(Var+eps))  one binary decision per output activation
 *                                         (Heaviside step: a tie fires)
 *     S = P + d * (W_r * x_r)           conditional path only where d = 1
 *     y = f_d(S)                        per-channel scale/shift chosen by d (the two
 *                                       batch norms of Sec. 4 folded for inference),
 *                                       optional residual add, optional ReLU
 *
 * "*" is cross-correlation with symmetric zero padding and floor output size:
 *     Ho = (H + 2*pad - kh) / stride + 1,   Wo likewise.
 *
 * Layouts.  Activations are NHWC: x[n][h][w][c] with `x_pixel_stride` elements
 * between pixels (>= c_in); y, residual: [n][ho][wo][c_out], dense.  Weights are
 * [c_out][kh][kw][c] with c = c_base (w_base) or c_in - c_base (w_cond).
 *
 * Memory.  The library allocates no device memory.  Every device buffer (x, y,
 * residual, bitmap, counts, workspace, `packed`, the weights) belongs to the caller
 * and is passed as a raw device pointer; `hip_stream` is the caller's hipStream_t
 * (NULL = the default stream).  Host arrays named in the descriptor are read during
 * cg_conv_create only.  The handle is host memory owned by the library.
 *
 * Every entry point returns a status and never throws or aborts.  All argument
 * checks happen before the first HIP call, so they behave the same on a host with
 * no GPU.  cg_last_error() gives the text of the calling thread's last failure.
 */
#ifndef CG_CONV_H
#define CG_CONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct cg_conv cg_conv; /* opaque */

enum { CG_OK = 0, CG_EINVAL = 1, CG_EUNSUPPORTED = 2, CG_ENOMEM = 3, CG_EHIP = 4 };
enum { CG_F32 = 0, CG_BF16 = 1, CG_I8 = 2, CG_I32 = 3 };
enum { CG_EPI_RELU = 1u, CG_EPI_AFFINE = 2u, CG_EPI_RESIDUAL = 4u };
/* Kernel family.  AUTO picks the row-tiled pixel-compacting matrix-core kernel (3x3 layers whose
 * channel groups are whole 32-byte runs) when the shape allows, else the large-tile matrix-core
 * kernel (3x3 and 1x1 layers, fully connected layers as 1x1 layers on a 1x1 image, channel groups of
 * whole 16-byte runs), else the plain one-thread-per-activation kernel.  All of them compute the
 * same layer. */
enum {
  CG_VARIANT_AUTO = 0,
  CG_VARIANT_NAIVE = 1,
  CG_VARIANT_MFMA_ROWS = 4,
  CG_VARIANT_TILE = 5
};

typedef struct cg_conv_desc {
  uint32_t struct_size;      /* = sizeof(cg_conv_desc); checked */
  int32_t n_max;             /* largest batch a forward call may pass */
  int32_t h, w, c_in, c_out; /* input height, width, channels; output channels */
  int32_t kh, kw;            /* kernel size: 3x3 or 1x1 */
  int32_t stride, pad;       /* stride >= 1, pad >= 0 */
  int32_t c_base;            /* base-path channels, C_in/G (Sec. 3.1: eta*c_l).
                                c_base == c_in: plain dense convolution, no gate */
  int32_t in_dtype;          /* x, W: CG_F32 | CG_BF16 | CG_I8 */
  int32_t out_dtype;         /* y, residual.  float inputs: CG_F32 | CG_BF16;
                                CG_I8 inputs: CG_I32 (raw sum) | CG_I8 (requantised) */
  uint32_t epilogue;         /* CG_EPI_* flags */
  int32_t variant;           /* CG_VARIANT_* */
  int32_t groups;            /* 0 or 1: every output channel takes channels [0, c_base) of x as its base
                                path.  G > 1: channel grouping (Sec. 3.3): input and output channels are
                                cut into G equal consecutive groups (c_base * G == c_in, G divides c_out);
                                output group i takes input group i as x_p and the other input groups, in
                                increasing channel order, as x_r.  The weight layouts stay as below: per
                                output channel, w_base holds its c_base base-path weights and w_cond the
                                weights of its c_in - c_base conditional channels in that order. */
  int64_t x_pixel_stride;    /* elements between pixels of x; 0 means c_in */

  const void* w_base;        /* DEVICE [c_out][kh][kw][c_base] */
  const void* w_cond;        /* DEVICE [c_out][kh][kw][c_in-c_base]; NULL iff dense */

  /* Gate, float inputs (HOST, [c_out]): fires iff P >= mean + delta*sqrt(var+eps).
   * delta = -inf always fires, +inf never fires.  delta_hi (nullable) adds the upper
   * threshold of the two-sided gate for saturating activations (Sec. 3.2):
   * fires iff also P <= mean + delta_hi*sqrt(var+eps). */
  const float* gate_mean;
  const float* gate_var;
  const float* delta;
  const float* delta_hi;
  float gate_eps;
  int32_t shuffle;           /* 0 | 1, needs groups > 1: store y channel-shuffled (Sec. 3.3, the optional
                                shuffle between grouped layers): channel j of output group i is written to
                                position j*G + i of its pixel, and the residual is read from that position.
                                bitmap, counts and every per-channel table keep the natural channel order. */
  /* Gate, CG_I8 inputs (HOST, [c_out]): fires iff the int32 base sum >= thr. */
  const int32_t* gate_thr_i32;

  /* Epilogue, float (HOST, [c_out], each nullable = 1 / 0): y = scale_d*S + shift_d. */
  const float* scale0;
  const float* shift0;
  const float* scale1;
  const float* shift1;
  /* Epilogue, CG_I8 -> CG_I8 (HOST, [c_out], nullable = 1 / 1 / 0):
   *   t = S*mult_d + (bias << shift) + residual*res_mult;
   *   y = clamp((t + (1 << (shift-1))) >> shift, RELU ? 0 : -128, 127)   (arithmetic shift)
   * CG_I8 -> CG_I32: y = S + residual*res_mult, ReLU if asked. */
  const int32_t* rq_mult0;
  const int32_t* rq_mult1;
  const int32_t* rq_bias;
  int32_t rq_shift;          /* 0..31 */
  int32_t rq_res_mult;

  /* Channel-wise gate (Sec. 3.2, the weight-access extension): with tau_c > 0 an output channel of
   * an image keeps its conditional path only if at least tau_c * Ho * Wo of its activations fired
   * (equality keeps it); otherwise every activation of that channel and image takes the d = 0
   * branch.  y, bitmap and counts then describe the decisions after this gate.  0 = off.
   * Costs a second pass over the base path (the sums must be complete before any conditional work). */
  float tau_c;
  int32_t tile_hint;         /* 0: the library picks the tile shape.  Otherwise a tuning hint for CG_VARIANT_TILE:
                                bits 0-3 = 32-pixel fragments per wavefront (4, 2 or 1), bits 4-7 = wavefronts
                                across the output channels (1 or 2), bits 8-11 = 16-byte channel chunks per K
                                stage of a 3x3 layer (4, 2 or 1); a zero field is picked by the library.  A
                                hint the shape cannot take makes create fail with CG_EUNSUPPORTED. */

  void* packed;              /* DEVICE, >= cg_conv_packed_bytes(desc), 256-byte aligned, caller-owned;
                                must outlive the handle; holds repacked weights and per-channel tables */
  size_t packed_bytes;
} cg_conv_desc;

/* Bytes the caller must provide in desc->packed; 0 if the descriptor is invalid
 * (cg_last_error says why). */
size_t cg_conv_packed_bytes(const cg_conv_desc* desc);

/* Validates the descriptor, folds the gate statistics into one threshold per output
 * channel (Sec. 3.2), and enqueues on `hip_stream` the copies/kernels that fill
 * desc->packed from w_base / w_cond and the host tables.  Work that uses the handle
 * must be ordered after that stream's work.  On failure *out is NULL. */
int cg_conv_create(cg_conv** out, const cg_conv_desc* desc, void* hip_stream);

/* Device scratch a forward call of batch n needs (may be 0). */
size_t cg_conv_workspace_bytes(const cg_conv* h, int32_t n);

/*
 * Enqueues one forward pass of the layer (Eq. 1) for a batch of n <= n_max images on
 * `hip_stream` and returns without waiting.  All pointers are DEVICE pointers.
 *   x         [n][h][w] pixels of x_pixel_stride elements, in_dtype
 *   residual  [n][ho][wo][c_out]; out_dtype for float inputs, int8 for CG_I8 inputs;
 *             required iff CG_EPI_RESIDUAL
 *   y         [n][ho][wo][c_out] out_dtype
 *   bitmap    nullable.  Decisions, one bit per output activation: row m = (n*Ho+ho)*Wo+wo has
 *             ceil(c_out/32) words; bit (co & 31) of word (co >> 5) is d[m][co]; unused bits 0.
 *             A dense layer (c_base == c_in) writes zeros.
 *   counts    nullable, 8-byte aligned.  2 + n*c_out words, fully overwritten: words 0,1 = number of fired gates
 *             (low, high half of a 64-bit count); word 2 + img*c_out + co = fired gates of that
 *             image and output channel (the sum the channel-wise gate of Sec. 3.2 thresholds).
 *   workspace >= cg_conv_workspace_bytes(h, n) bytes, 256-byte aligned; may be NULL if that is 0.
 * Calls on one handle may overlap only if they use distinct y / bitmap / counts / workspace.
 * Errors: CG_EINVAL (NULL where not allowed, n out of range, workspace too small),
 * CG_EHIP (a launch failed).
 */
int cg_conv_forward(cg_conv* h, int32_t n, const void* x, const void* residual, void* y,
                    uint32_t* bitmap, uint32_t* counts, void* workspace, size_t workspace_bytes,
                    void* hip_stream);

/*
 * cg_conv_forward for callers that cannot allocate device memory or pass a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and results
 * as cg_conv_forward without `workspace`: the scratch the call needs (the batch's decision bitmap when
 * counts are asked for without a bitmap; with the channel-wise gate also the first pass's bitmap, counts
 * and channel mask) lives in a fixed 16 MiB array inside the library, one copy per GPU, held until the
 * process ends.  The call allocates nothing (no hipMalloc / hipFree, no allocating library routine) and
 * relies on no previous contents of the array.  A call that needs more scratch than the array holds
 * (cg_conv_workspace_bytes(h, n) > 16 MiB) fails with CG_EUNSUPPORTED and enqueues nothing.  Every call
 * on one GPU shares that GPU's array: calls that may overlap on one GPU (different streams, different
 * threads) race on it and must be serialised by the caller; calls on one stream are ordered.
 */
int cg_conv_forward_noalloc(cg_conv* h, int32_t n, const void* x, const void* residual, void* y,
                            uint32_t* bitmap, uint32_t* counts, void* hip_stream);

/* Frees the host handle; touches no device memory.  NULL is a no-op. */
void cg_conv_destroy(cg_conv* h);

/* Output geometry of a handle: writes Ho, Wo; returns the kernel family in use (CG_VARIANT_*),
 * or -1 for a NULL handle. */
int cg_conv_info(const cg_conv* h, int32_t* ho, int32_t* wo);

/* Text of the calling thread's most recent error; never NULL. */
const char* cg_last_error(void);

/*
 * The dense pieces of a ResNet around the gated layers (the paper's experiments, Sec. 5, run
 * ResNet-18): none of them is gated.  bf16 activations and weights (NHWC / [c_out][k][k][c_in]),
 * fp32 accumulation, all pointers DEVICE, nothing allocated, work only enqueued on hip_stream.
 * Each returns CG_OK or an error code with text in cg_last_error(); arguments are checked before
 * any HIP call.
 */

/* Convolution on few input channels (the 7x7 stride-2 input layer): c_in in [1,4], c_out a multiple of
 * 64, k odd <= 7, stride 1|2, zero padding pad < k.  y[n][ho][wo][c_out] = relu?(scale*conv + shift);
 * scale / shift: [c_out] floats, nullable (= 1 / 0).  y, scale, shift 16-byte aligned. */
int cg_small_cin_conv(const void* x, const void* w, const float* scale, const float* shift, void* y, int32_t n,
                      int32_t h, int32_t wd, int32_t c_in, int32_t c_out, int32_t k, int32_t stride, int32_t pad,
                      int32_t relu, void* hip_stream);

/* The ImageNet input layer and the max pooling behind it in one kernel: 7x7 stride-2 convolution of
 * x[n][h][w][3] with w[c_out][7][7][3] (zero padding pad), scale/shift/ReLU as above, then 3x3 stride-2
 * max pooling with padding 1; only the pooled tensor y[n][(ho-1)/2+1][(wo-1)/2+1][c_out] is written
 * (ho, wo = the convolution's output size).  Equal to cg_small_cin_conv followed by cg_maxpool3x3s2. */
int cg_conv7x7s2_maxpool(const void* x, const void* w, const float* scale, const float* shift, void* y, int32_t n,
                         int32_t h, int32_t wd, int32_t c_out, int32_t pad, int32_t relu, void* hip_stream);

/* 1x1 convolution with stride (the ResNet shortcut), no padding: x[n][h][w][c_in], w[c_out][c_in] ->
 * y[n][(h-1)/stride+1][(w-1)/stride+1][c_out] = relu?(scale*conv + shift).  c_in a multiple of 16, at most
 * 512; c_out a multiple of 64; scale / shift nullable; x, w, y, scale, shift 16-byte aligned. */
int cg_pointwise_conv(const void* x, const void* w, const float* scale, const float* shift, void* y, int32_t n,
                      int32_t h, int32_t wd, int32_t c_in, int32_t c_out, int32_t stride, int32_t relu,
                      void* hip_stream);

/* 3x3 max pooling, stride 2, padding 1 (the maximum runs over the taps inside the image):
 * x[n][h][w][c] -> y[n][(h-1)/2+1][(w-1)/2+1][c]; c a multiple of 8; x, y 16-byte aligned. */
int cg_maxpool3x3s2(const void* x, void* y, int32_t n, int32_t h, int32_t wd, int32_t c, void* hip_stream);

/* Global average pooling over the hw positions of x[n][hw][c], then the fully connected layer:
 * logits[n][classes] (fp32) = wfc[classes][c] * mean + bias (bias nullable). */
int cg_avgpool_fc(const void* x, const void* wfc, const float* bias, float* logits, int32_t n, int32_t hw, int32_t c,
                  int32_t classes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* CG_CONV_H */
