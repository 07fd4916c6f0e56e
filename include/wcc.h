/*
 * wcc.h -- C ABI of libwcc: the forward path of the Wavelet Compressed
 * Convolution (WCC) layer,  WCC(K, x) = H^T T^T K_1x1 T H x  (Eq. WCC), on one
 * AMD MI355X (gfx950).
 *
 * The five stage calls are the five panels of the workflow figure (A: Haar
 * transform, B: joint shrinkage, C: 1x1 convolution on the compressed vectors,
 * D: zero filling, E: inverse Haar transform) and the steps of the explicit
 * algorithm in the appendix "Explicit WCC algorithm"; wcc_forward runs them all.
 *
 * Conventions common to every call
 * --------------------------------
 * Pointers.   Unless marked [host], every pointer is a DEVICE pointer owned by
 *             the caller, 16-byte aligned, valid until the work enqueued by the
 *             call has finished on `stream`.  The library never allocates or
 *             frees tensors and keeps no pointer after the call's stream work.
 * Workspace.  Scratch memory is one caller-owned device buffer attached with
 *             wcc_set_workspace(); its size for a given layer comes from
 *             wcc_workspace_bytes().  Calls on one context share it: two calls
 *             that overlap in time on the same context race.
 * Streams.    `stream` is a hipStream_t passed as void* (NULL = the null
 *             stream).  Calls only enqueue work: no host synchronisation and no
 *             device-to-host copy happens inside any call.
 * Errors.     Arguments are checked before anything is enqueued; a failed check
 *             returns a status and enqueues nothing.  No call aborts, throws or
 *             prints.  A HIP launch failure returns WCC_ERR_HIP.
 * Numbers.    Activations are fp32.  NaN/Inf inputs give unspecified results
 *             (never undefined behaviour on the host).
 *
 * Layouts (all row-major, last index contiguous); N = H*W, n_l = (H>>l)*(W>>l)
 * ---------------------------------------------------------------------------
 *   x     [B, C_in,  H, W]  fp32   input feature map   (bf16 if act_dtype = WCC_BF16,
 *   y     [B, C_out, H, W]  fp32   output feature map   fused calls only)
 *   coef  [B, C,     N]     fp32   wavelet vector of every channel.  Position q
 *                                  ("linear index") follows the concatenation of
 *                                  Eq. (wavelet_transform) for d = levels:
 *                                  [ y1^d | y2^d | y3^d | y4^d | y2^(d-1) | y3^(d-1)
 *                                    | y4^(d-1) | ... | y2^1 | y3^1 | y4^1 ],
 *                                  band j (1..3 -> y2..y4) of level l at offset
 *                                  j*n_l, each band row-major (H>>l) x (W>>l).
 *   norm  [B, N]            fp32   norm over channels of coef at each position (desc.norm)
 *   idx   [B, k]            int32  kept positions of each sample, strictly ascending
 *   xc    [B, C_in,  k]     fp32 (act_quant_bits = 0) or int8 codes (= 8)
 *   yc    [B, C_out, k]     fp32
 *   w     [C_out, C_in]     fp32 | bf16 | int8 codes (w_dtype)
 *   w_scale [C_out]         fp32   per-output-channel scale of int8 / int4 weight codes
 *   WCC_I4 weights          uint8  [C_out, C_in/2]: two signed 4-bit codes (two's complement,
 *                                  -7..7) a byte, channel 2i in the low nibble, 2i+1 in the
 *                                  high one; C_in must be even.  The codes are widened to int8
 *                                  by a small kernel into the workspace and then take the int8
 *                                  path (the paper's tables use 4-bit weights with 8-bit
 *                                  activations).
 */
#ifndef WCC_H
#define WCC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct wcc_ctx wcc_ctx; /* opaque; holds the workspace pointer and device facts */

typedef enum {
  WCC_OK = 0,
  WCC_ERR_NULL = 1,        /* a required pointer is NULL                                  */
  WCC_ERR_SHAPE = 2,       /* a dimension is < 1, too large, or H/W not divisible by 2^levels */
  WCC_ERR_DTYPE = 3,       /* unknown w_dtype or act_quant_bits not in {0, 8}             */
  WCC_ERR_KEEP = 4,        /* keep ratio does not give 1 <= k <= H*W                      */
  WCC_ERR_WORKSPACE = 5,   /* no workspace attached, or it is too small / misaligned      */
  WCC_ERR_UNSUPPORTED = 6, /* valid request this build has no kernel for                  */
  WCC_ERR_HIP = 7,         /* the HIP runtime reported an error                           */
  WCC_ERR_ALIGN = 8        /* a tensor pointer is not 16-byte aligned                     */
} wcc_status;

typedef enum { WCC_F32 = 0, WCC_BF16 = 1, WCC_I8 = 2, WCC_I4 = 3 } wcc_dtype;

/* Which norm over the channels ranks the positions (Alg. 1 names none): the sum of absolute
 * values, or the sum of squares -- the Euclidean norm without its square root, which orders
 * the positions the same way. */
typedef enum { WCC_NORM_L1 = 0, WCC_NORM_L2 = 1 } wcc_norm;

/* One WCC layer: the inputs of the explicit algorithm (feature-map shape,
 * kernel shape, wavelet level d, kept fraction gamma) plus storage types. */
typedef struct {
  int32_t B, C_in, C_out, H, W; /* B, C_in, C_out <= 65535; H*W <= 2^30 - 16                 */
  int32_t levels;             /* d >= 1; H and W must be divisible by 2^d (no padding)      */
  int64_t keep_num, keep_den; /* gamma = keep_num/keep_den, the fraction KEPT;
                                 k = ceil(keep_num*H*W/keep_den) in integer arithmetic      */
  int32_t w_dtype;            /* wcc_dtype of w                                             */
  int32_t act_quant_bits;     /* 0: kept coefficients stay fp32; 8: signed 8-bit codes      */
  int32_t act_dtype;          /* storage type of x and y: WCC_F32 (0, the default) or
                                 WCC_BF16.  bf16 feature maps are read exactly and written
                                 rounded to nearest even; all arithmetic stays fp32.  Only the
                                 fused calls (wcc_forward, wcc_forward_fixed,
                                 wcc_block_forward) take bf16; the stage calls return
                                 WCC_ERR_UNSUPPORTED for it                                   */
  int32_t norm;               /* wcc_norm: WCC_NORM_L1 (0, the default) or WCC_NORM_L2.  With
                                 WCC_NORM_L2 every norm tensor holds sum_c coef^2 (partial sums
                                 combined in a fixed order) and feature maps must be fp32     */
} wcc_desc;

/* Stages whose device time wcc_forward can record (wcc_set_profiling). */
enum {
  WCC_T_HAAR_FWD = 0,  /* first transform pass (channel norms), one kernel            */
  WCC_T_NORM_SELECT,   /* norm reduction + radix select + index emission               */
  WCC_T_GATHER,        /* second transform pass: kept coefficients + max|c|, one kernel */
  WCC_T_POINTWISE,     /* quantise + contraction + dequantise, one kernel              */
  WCC_T_SCATTER_IHAAR, /* scatter + inverse Haar, one kernel                           */
  WCC_T_EVENT_PAIR,    /* an empty bracket: what two event records cost by themselves  */
  WCC_T_DEPTHWISE,     /* wcc_block_forward only: the depthwise 3x3 kernel             */
  WCC_T_COUNT
};

/* ---- context --------------------------------------------------------------------------- */

/* Creates a context for HIP device `device` (makes no device allocation).  */
wcc_status wcc_create(wcc_ctx **out /*[host]*/, int device);
wcc_status wcc_destroy(wcc_ctx *ctx);

/* Bytes of workspace that any call below needs for this layer (a multiple of 256). */
wcc_status wcc_workspace_bytes(const wcc_desc *desc /*[host]*/, size_t *bytes /*[host]*/);

/* Attaches a caller-owned device buffer (256-byte aligned) as the workspace.  The
 * context only remembers the pointer; the caller frees it after the last call. */
wcc_status wcc_set_workspace(wcc_ctx *ctx, void *dev_ptr, size_t bytes);

/* k = ceil(gamma*H*W) of Alg. 1, or -1 if the descriptor is invalid.  Pure host function. */
int64_t wcc_k(const wcc_desc *desc /*[host]*/);

const char *wcc_status_string(wcc_status s);

/* When enabled, wcc_forward brackets each stage with HIP events on `stream`.
 * wcc_stage_times() waits for the last profiled wcc_forward and writes the
 * WCC_T_COUNT stage durations in milliseconds to ms [host]. */
wcc_status wcc_set_profiling(wcc_ctx *ctx, int enabled);
wcc_status wcc_stage_times(wcc_ctx *ctx, float *ms /*[host], WCC_T_COUNT floats*/);

/* ---- A: multi-level Haar transform (Eq. HaarKernel, Eq. wavelet_transform) -------------
 * coef[b,c,:] = HWT_d(x[b,c,:,:]) for the C_in channels of desc; one level maps each 2x2
 * block [[a,b],[c,d]] to y1=(a+b+c+d)/2, y2=(a-b+c-d)/2, y3=(a+b-c-d)/2, y4=(a-b-c+d)/2 and
 * recurses on y1.  If norm != NULL it also receives norm[b,q] = sum_c |coef[b,c,q]| (the
 * per-position norm over channels that Alg. 1 ranks by, read as L1), or sum_c coef[b,c,q]^2
 * with desc.norm = WCC_NORM_L2; channel partial sums are combined in a fixed order, so the
 * result does not vary from run to run.
 * x is not modified.  Needs the workspace when norm != NULL. */
wcc_status wcc_haar_fwd(wcc_ctx *ctx, const wcc_desc *desc, const float *x, float *coef,
                        float *norm /*nullable*/, void *stream);

/* ---- B: joint shrinkage, index set I (Alg. 1; Eq. T applied jointly to all channels) ----
 * Per sample b: the k positions with the largest norm, ties broken toward the lower
 * position q; idx[b,:] ascending.  Exactly one of coef / norm may be NULL: with norm given
 * it is used as is; otherwise it is computed from coef ([B,C_in,N]) into the workspace.
 * Norms are compared as fp32 numbers (they are >= 0). */
wcc_status wcc_joint_topk(wcc_ctx *ctx, const wcc_desc *desc, const float *coef /*nullable*/,
                          const float *norm /*nullable*/, int32_t *idx, void *stream);

/* ---- B': extract the kept entries of every channel, then quantise them -------------------
 * xc[b,c,j] = coef[b,c,idx[b,j]].  With act_quant_bits = 8 the kept coefficients go through
 * the signed scheme of Eq. (quantweights) with b = 8:  u = c/alpha, clip to [-1,1],
 * code = round_half_even(127*u), all in fp32, stored as int8; the value stood for is
 * alpha*code/127.  alpha = alpha_in if alpha_in > 0, else the largest |kept coefficient| of
 * the whole call (alpha = 0 gives all-zero codes).  alpha_dev (1 float, device) receives
 * alpha when act_quant_bits = 8 (required then; ignored and may be NULL otherwise).  idx
 * values outside [0, N) are clamped into the plane.  Needs the workspace when
 * act_quant_bits = 8. */
wcc_status wcc_gather_quant(wcc_ctx *ctx, const wcc_desc *desc, const float *coef,
                            const int32_t *idx, float alpha_in, void *xc, float *alpha_dev,
                            void *stream);

/* ---- C: the 1x1 convolution on the compressed signal,  y_i = sum_j k_ij x_j --------------
 * yc[b,o,j] = s_x * s_w[o] * sum_c w[o,c] * xc[b,c,j]  with s_x = alpha/127 for int8 codes
 * (alpha read from alpha_dev on the device) and 1 for fp32 xc; s_w = w_scale for int8
 * weights (required then), else 1.  Arithmetic: bf16 or int8 weights with int8 codes run on
 * the matrix cores (bf16 x bf16 -> fp32, int8 x int8 -> int32); every other combination
 * is computed with fp32 FMAs on the weights widened to fp32. */
wcc_status wcc_pointwise(wcc_ctx *ctx, const wcc_desc *desc, const void *w,
                         const float *w_scale /*nullable unless w_dtype = I8*/, const void *xc,
                         const float *alpha_dev /*nullable unless act_quant_bits = 8*/,
                         float *yc, void *stream);

/* ---- D+E: zero filling and inverse transform (T^T, then iHWT with levels reversed) -------
 * z = 0, z[b,o,idx[b,j]] = yc[b,o,j];  y[b,o,:,:] = iHWT_d(z[b,o,:]), one level mapping
 * (y1,y2,y3,y4) back to a=(y1+y2+y3+y4)/2, b=(y1-y2+y3-y4)/2, c=(y1+y2-y3-y4)/2,
 * d=(y1-y2-y3+y4)/2.  z is never materialised.  idx must be strictly ascending per sample
 * with values in [0, N).  Needs the workspace. */
wcc_status wcc_scatter_ihaar(wcc_ctx *ctx, const wcc_desc *desc, const float *yc,
                             const int32_t *idx, float *y, void *stream);

/* ---- the whole layer (Alg. 1 with the quantiser between shrinkage and convolution) ------
 * y = H^T T^T K T H x.  Intermediates live in the workspace.  Results are those of the five
 * calls above run in sequence.  idx_out ([B,k]) and alpha_out_dev (1 float) are optional. */
wcc_status wcc_forward(wcc_ctx *ctx, const wcc_desc *desc, const void *x, const void *w,
                       const float *w_scale /*nullable unless I8*/, float alpha_in, void *y,
                       int32_t *idx_out /*nullable*/, float *alpha_out_dev /*nullable*/,
                       void *stream);

/* ---- wcc_forward for callers that cannot allocate -------------------------------------------
 * For code that may not call hipMalloc and has no workspace to hand over: work recorded under
 * HIP graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments,
 * same kernels and same results as wcc_forward, but the intermediates live in a fixed array of
 * WCC_STATIC_SCRATCH_BYTES inside the library's device image (every GPU the library is loaded
 * on holds that much until the process ends) instead of the context's workspace, which is not
 * touched and need not be attached.  The call allocates and frees nothing, on the host or on
 * the device.  A layer whose wcc_workspace_bytes() exceeds WCC_STATIC_SCRATCH_BYTES returns
 * WCC_ERR_WORKSPACE and enqueues nothing.  The device that is current must be the one the
 * context was created for (else WCC_ERR_UNSUPPORTED).  All calls on one GPU share the one
 * array, whatever their context or stream: calls that overlap in time on one GPU race; every
 * buffer that must start from a known value is cleared by the call's own first kernel, so calls
 * in sequence need no clean-up in between.  Stage profiling (wcc_set_profiling) does not
 * apply. */
#define WCC_STATIC_SCRATCH_BYTES (64u << 20)
wcc_status wcc_forward_static(wcc_ctx *ctx, const wcc_desc *desc, const void *x, const void *w,
                              const float *w_scale /*nullable unless I8*/, float alpha_in, void *y,
                              int32_t *idx_out /*nullable*/, float *alpha_out_dev /*nullable*/,
                              void *stream);

/* ---- variant: the layer with an index list that does not depend on the input ------------
 * The footnote of the section "Joint hard shrinkage" mentions keeping the upper-left part of
 * the wavelet transform for any image.  idx [B,k] (strictly ascending per sample, values in
 * [0,N)) is used as the index set I of every channel; idx = NULL means the first k positions of
 * the wavelet vector (the coarsest bands first, in the order of `coef` above).  Everything after
 * the selection is as in wcc_forward (alpha = largest kept |coefficient| unless alpha_in > 0);
 * the norm pass and the selection are not run. */
wcc_status wcc_forward_fixed(wcc_ctx *ctx, const wcc_desc *desc, const void *x, const void *w,
                             const float *w_scale /*nullable unless I8*/, float alpha_in,
                             const int32_t *idx /*nullable*/, void *y,
                             float *alpha_out_dev /*nullable*/, void *stream);

/* ==== next row: the inverted residual block the paper timed (appendix "Inference times",
 * Eq. (inverted)):  y = x + K3_1x1( K_dw( K1_1x1 x ) ), both 1x1 convolutions as WCC layers
 * with the same levels / keep ratio / quantiser, K_dw a depthwise 3x3 convolution; the
 * non-linearities are left out, as in the paper's timings. ================================= */

typedef struct {
  int32_t B, C, expansion;   /* x, y [B, C, H, W]; the middle tensors have C * expansion channels */
  int32_t H, W, levels;
  int64_t keep_num, keep_den;
  int32_t w_dtype;           /* of both 1x1 kernels: w1 [C*expansion, C], w3 [C, C*expansion] */
  int32_t act_quant_bits;
  int32_t act_dtype;         /* storage type of x, y and the middle tensor (see wcc_desc);
                                WCC_BF16 needs W % 4 == 0 and t2_out = NULL                  */
  int32_t norm;              /* wcc_norm of both layers (see wcc_desc)                       */
} wcc_block_desc;

/* Workspace for wcc_block_forward: the two middle tensors plus the larger of the two layers'
 * own workspaces.  Pure host function. */
wcc_status wcc_block_workspace_bytes(const wcc_block_desc *desc, size_t *bytes);

/* 1 if wcc_block_forward, called without middle outputs (t1_out = t2_out = NULL), chains the
 * two layers of this block in the compressed domain -- the appendix "Inference times", paragraph
 * on memory bandwidth and traffic: transform, depthwise convolution and gather / scatter applied
 * per channel and in parts, the full result kept only in compressed form -- so that the expanded
 * feature maps are never formed; 0 if it forms them; -1 for an invalid descriptor.  Chained:
 * W % 4 == 0, W <= 256, levels <= 3 and at most a third of the coefficients kept.  Pure host
 * function. */
int32_t wcc_block_is_chained(const wcc_block_desc *desc);

/* K_dw: y[b,c,r,q] = sum_{i,j=0..2} w[c,i,j] * x[b,c,r+i-1,q+j-1], zero outside the plane
 * (cross-correlation, stride 1, zero padding 1, no bias; the paper names the operator only).
 * x, y [B,C,H,W] fp32 device, w [C,3,3] fp32 device; x and y must not overlap. */
wcc_status wcc_depthwise3x3(wcc_ctx *ctx, int32_t B, int32_t C, int32_t H, int32_t W,
                            const float *x, const float *w, float *y, void *stream);

/* The block.  w1_scale / w3_scale as in wcc_forward (int8 weights only); alpha of each layer is
 * the largest kept |coefficient| of that layer.  t1_out / t2_out (nullable, [B, C*expansion,
 * H, W]) receive K1's output and K_dw's output, idx1_out / idx3_out (nullable, [B,k]) the two
 * index sets: they exist for tests.  Asking for a middle output makes the call form both middle
 * tensors; without, it chains the layers where wcc_block_is_chained() says so (the second
 * layer then sees the same fp32 numbers, summed into its channel norms in another grouping, so
 * its index set may differ from the other route's where two norms are within rounding of each
 * other; with bf16 maps the chained middle tensor is not rounded to bf16).  Needs a workspace of
 * wcc_block_workspace_bytes. */
wcc_status wcc_block_forward(wcc_ctx *ctx, const wcc_block_desc *desc, const void *x,
                             const void *w1, const float *w1_scale, const float *w_dw,
                             const void *w3, const float *w3_scale, void *y,
                             void *t1_out, float *t2_out, int32_t *idx1_out, int32_t *idx3_out,
                             void *stream);

/* Which of the block's two layers (0: expand, 1: project) the stage events bracket while
 * profiling is on (default 1). */
wcc_status wcc_set_block_profile_layer(wcc_ctx *ctx, int layer);

#ifdef __cplusplus
}
#endif
#endif /* WCC_H */
