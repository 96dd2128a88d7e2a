/*
 * astl.h -- C ABI of one whole Agile Swin Transformer Layer (ASTL) for AMD MI355X (gfx950):
 * the GSWA layer of gswa.h with the LayerNorms, the MLP and the two skip connections around it
 * (Sec. "Agile Swin Transformer Block", Eq. 4-5).
 *
 * Per token (a row of C channels of the feature map x [B, H, W, C]):
 *   x1 = GSWA(LN_1(x)) + x                                      Eq. 4
 *   y  = MLP(LN_2(x1)) + x1                                     Eq. 5
 *   LN(u)   = (u - mean u) / sqrt(var u + eps) * gamma + beta   mean and (biased) variance over
 *                                                               the C channels of the token
 *   MLP(u)  = GELU(u Wfc1^T + bfc1) Wfc2^T + bfc2               two fully connected layers,
 *                                                               `hidden` features in between
 *   GELU(t) = t * (1 + erf(t / sqrt 2)) / 2
 * The paper fixes the two equations, the two layers and the GELU; the hidden width and eps are
 * descriptor fields here, and GELU is taken in its Gaussian-CDF (erf) form.
 *
 * The conventions of gswa.h hold: `desc`, `params` and `grads` are HOST pointers to structs
 * whose members are DEVICE pointers the caller owns; nothing is allocated, freed or
 * synchronised; all work is enqueued on `hip_stream`; tensors are C-contiguous and 16-byte
 * aligned, `ws` 256-byte aligned; arithmetic accumulates in fp32; gradients of parameters are
 * always fp32; the return value is a gswa_status and a failed call has enqueued nothing.
 */
#ifndef ASTL_H
#define ASTL_H

#include "gswa.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct astl_desc {
    gswa_desc attn;  /* the attention layer inside Eq. 4: map, heads, groups, window, shift, dtype,
                        flags, dqk, exactly as for gswa_forward                                */
    int32_t hidden;  /* width of the MLP's hidden layer (Eq. 5), > 0                           */
    float eps;       /* added to the variance in both LayerNorms, >= 0                         */
} astl_desc;

/* Parameters, element type desc->attn.dtype. */
typedef struct astl_params {
    const void *ln1_w, *ln1_b;                    /* gamma, beta of LN_1   [C]                   */
    const void *w_qkv, *b_qkv, *w_proj, *b_proj;  /* attention layer, layouts of gswa.h          */
    const void *bias_table;
    const void *ln2_w, *ln2_b;                    /* gamma, beta of LN_2   [C]                   */
    const void *w_fc1, *b_fc1;                    /* [hidden, C] (out, in), [hidden]             */
    const void *w_fc2, *b_fc2;                    /* [C, hidden] (out, in), [C]                  */
} astl_params;

/* Gradients of the parameters: same shapes, ALWAYS fp32, overwritten (added into with
 * GSWA_ACCUM_WGRAD in desc->attn.flags). */
typedef struct astl_grads {
    float *ln1_w, *ln1_b;
    float *w_qkv, *b_qkv, *w_proj, *b_proj;
    float *bias_table;
    float *ln2_w, *ln2_b;
    float *w_fc1, *b_fc1;
    float *w_fc2, *b_fc2;
} astl_grads;

/*
 * Sizes, in bytes, of the caller-provided device buffers (all multiples of 256; any output
 * pointer may be NULL).
 *   *saved_bytes   what astl_forward leaves for astl_backward: x1 [B*H*W, C] in the layer's
 *                  element type, the attention layer's own saved state and, where the MLP runs
 *                  on the fused kernels (bf16, C <= 64, hidden <= 128), its weights repacked for
 *                  the matrix cores (65 KB).  LayerNorm outputs, the hidden layer and its
 *                  pre-activation are never kept: backward recomputes them from x and x1.
 *   *fwd_ws_bytes  scratch of astl_forward (normalised input, attention output, the attention
 *                  layer's scratch, and one [B*H*W, hidden] buffer where the MLP is not fused);
 *                  for inference (saved == NULL) the scratch must hold *fwd_ws_bytes +
 *                  *saved_bytes.
 *   *bwd_ws_bytes  scratch of astl_backward.
 */
int astl_query_bytes(const astl_desc *desc, size_t *saved_bytes, size_t *fwd_ws_bytes,
                     size_t *bwd_ws_bytes);

/*
 * y = ASTL(x)  (Eq. 4 then Eq. 5).  saved = NULL for inference.  x and y must not overlap.
 * Errors: GSWA_EINVAL for a null pointer, a misaligned buffer, hidden <= 0, eps < 0 or an
 * invalid attention descriptor; GSWA_EUNSUPPORTED where gswa_forward would return it, or
 * C > 256.
 */
int astl_forward(const astl_desc *desc, const void *x, const astl_params *params, void *y,
                 void *saved, void *ws, void *hip_stream);

/*
 * Gradients of a scalar loss through the layer, given dy = dLoss/dy and `saved` as written by
 * astl_forward on the same desc, x and params.  dx [B,H,W,C] in the layer's element type,
 * overwritten; it may not overlap x, dy or saved.  The parameter gradients are reduced with
 * fp32 atomics on part of the path, so their last bits can differ between runs.
 */
int astl_backward(const astl_desc *desc, const void *x, const void *dy, const astl_params *params,
                  const void *saved, void *dx, const astl_grads *grads, void *ws, void *hip_stream);

/*
 * A stack of n_layers such layers applied one after the other (Sec. "Agile Swin Transformer
 * Block": the deep feature extractor is a sequence of these layers, window attention and
 * shifted-window attention alternating): layer l has shift 0 when l is even and `shift` when l
 * is odd, every layer has its own parameters, and the output of layer l is the input of layer
 * l + 1.  `params` and `grads` are HOST arrays of n_layers structs.
 *
 * checkpoint_every = 0 keeps every layer's input and saved state for the backward pass.
 * checkpoint_every = k > 0 keeps only the inputs of layers k, 2k, ... (the block boundaries);
 * astl_stack_backward then runs the forward of one block of k layers again, into its scratch,
 * before taking that block's gradients: saved memory falls from n_layers to about
 * n_layers / k + k layer states, for one more forward pass.  The result is the same either way.
 */
typedef struct astl_stack_desc {
    astl_desc layer;          /* shape of every layer; layer.attn.shift is ignored               */
    int32_t n_layers;         /* > 0                                                             */
    int32_t shift;            /* shift of the odd layers, 0 <= shift < window                     */
    int32_t checkpoint_every; /* 0, or the number of layers per recomputed block                  */
} astl_stack_desc;

/* Sizes as for astl_query_bytes; *saved_bytes covers all layers.  For inference (saved == NULL)
 * astl_stack_forward needs *fwd_ws_bytes only. */
int astl_stack_query_bytes(const astl_stack_desc *desc, size_t *saved_bytes, size_t *fwd_ws_bytes,
                           size_t *bwd_ws_bytes);

/* y = layer_{n-1}( ... layer_0(x)).  saved = NULL for inference.  x and y must not overlap. */
int astl_stack_forward(const astl_stack_desc *desc, const void *x, const astl_params *params, void *y,
                       void *saved, void *ws, void *hip_stream);

/*
 * Inference of a stack on a map of any height with scratch that does not grow with the map (Sec. "Agile
 * Swin Transformer Block"; large inputs at test time).  Every step of Eq. 4-5 acts within one window, so
 * the map goes through each layer in bands of `band_windows` rows of windows of that layer's (shifted)
 * window grid, one image at a time.  A band of a shifted layer that does not reach the map's last window
 * row is a contiguous run of image rows and needs only the column part of the shift mask; the band that
 * ends the map also takes the map's first `shift` rows.  The result is the one astl_stack_forward gives
 * for inference, bit for bit.
 *
 * x [B,H,W,C] is read only; y [B,H,W,C] receives layer 0's output and is then updated in place by the
 * later layers; x and y must not overlap.  ws: *ws_bytes of astl_stack_tiled_query_bytes, 256-byte
 * aligned: two bands of activations and one layer's scratch for a band ((band_windows + 1) * window
 * rows of one image).  band_windows >= the map's window rows means one band per image.  desc->
 * checkpoint_every is ignored.  Errors as for astl_stack_forward; band_windows <= 0 is GSWA_EINVAL.
 * Work per shifted layer grows by one row of windows per band (computed and dropped).
 */
int astl_stack_tiled_query_bytes(const astl_stack_desc *desc, int32_t band_windows, size_t *ws_bytes);
int astl_stack_forward_tiled(const astl_stack_desc *desc, const void *x, const astl_params *params, void *y,
                             int32_t band_windows, void *ws, void *hip_stream);

/* Gradients through the whole stack: dx, and grads[l] for the parameters of layer l. */
int astl_stack_backward(const astl_stack_desc *desc, const void *x, const void *dy,
                        const astl_params *params, const void *saved, void *dx, const astl_grads *grads,
                        void *ws, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* ASTL_H */
