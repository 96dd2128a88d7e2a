/*
 * gswa.h -- C ABI of the Group Shifted Window Attention (GSWA) layer for AMD MI355X (gfx950).
 *
 * One call computes one GW-MSA / GSW-MSA layer of AgileIR (Sec. "Group Shifted Window
 * Attention"): the feature map is cyclically shifted and cut into M x M windows (Sec. "Patch
 * Embedding"), its channels are split into G head groups, every group runs multi-head
 * attention inside each window on its own channel slice with its own Q/K/V projection
 * (Eq. 6), the input of group g > 0 is its slice plus the output of group g-1 (Eq. 8), and
 * the concatenated group outputs go through one output projection (Eq. 7) and back to their
 * places in the map.  Scores carry the learnable relative position bias (Sec. "Learnable
 * Relative Shifted Bias") and, when shift > 0, the additive -100 mask between tokens that
 * the cyclic shift brought together from opposite borders.
 *
 * In symbols, for image b, window (wi, wj) of the shifted frame and tokens n = r*M + c:
 *   (i, j) = (wi*M + r, wj*M + c);  src(n) = ((i + shift) mod H, (j + shift) mod W)
 *   F_g = x[b, src, g*Cg:(g+1)*Cg] (+ O_{g-1} if g > 0);  [q|k|v] = F_g Wqkv_g^T + bqkv_g
 *   S = q_h k_h^T / sqrt(d) + table[idx(n,m), head] + mask;  O_g = concat_h softmax(S) v_h
 *   y[b, src, :] = concat_g(O_g) Wproj^T + bproj
 *   idx(n,m) = (r_n - r_m + M-1)*(2M-1) + (c_n - c_m + M-1)
 * with Cg = C/groups, d = C/heads, heads/groups heads per group.
 *
 * Narrow queries and keys (Sec. "Parameter Allocation": the channels of Q and K need not match
 * those of V): with desc->dqk = e > 0 every head has e channels of q and of k while v and the
 * head's output keep d channels; the scores are then scaled by 1/sqrt(e).  dqk = 0 is the plain
 * layer (e = d).  Any window size up to 64 is accepted, including the 12 x 12 windows of
 * Sec. "Experimental Settings".
 *
 * Conventions for every entry point
 *   - `desc` is a HOST pointer.  Every other pointer is a DEVICE pointer into memory the
 *     caller owns (hipMalloc or a torch tensor); the library never allocates, frees or
 *     synchronises.  All work is enqueued on `hip_stream` (a hipStream_t; NULL = default
 *     stream).  Buffers must stay valid until that work has run.
 *     Every tensor pointer must be 16-byte aligned, `ws` 256-byte aligned (GSWA_EINVAL otherwise).
 *   - Layouts are C-contiguous with the last index fastest.
 *       x, y, dy, dx   [B, H, W, C]                         element type desc->dtype
 *       w_qkv          [groups, Rg, Cg]  (out, in)          desc->dtype
 *                      Rg = 2*hg*e + Cg out rows: q block (row hl*e + c), k block (hg*e + hl*e + c),
 *                      v block (2*hg*e + hl*d + c), hl = head in group; 3*Cg rows when dqk == 0
 *       b_qkv          [groups, Rg]                         desc->dtype
 *       w_proj         [C, C] (out, in); in column = (g*hg + hl)*d + e;  b_proj [C]
 *       bias_table     [(2*window-1)^2, heads]              desc->dtype
 *       dw_qkv, db_qkv, dw_proj, db_proj, dbias_table: shaped like their parameter, ALWAYS fp32
 *     With groups == 1 these are the usual window-attention shapes [3C,C], [C,C], [(2M-1)^2,h].
 *   - Arithmetic accumulates in fp32 for both element types.
 *   - Return value: GSWA_OK (0) or a negative gswa_status.  Arguments are validated before
 *     anything is enqueued, so a failed call has not touched any output.  Nothing throws or
 *     aborts across this boundary.
 */
#ifndef GSWA_H
#define GSWA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    GSWA_OK = 0,
    GSWA_EINVAL = -1,       /* null pointer, non-positive size, divisibility or shift range violated */
    GSWA_EUNSUPPORTED = -2, /* valid layer, but no kernel of this library covers it (e.g. LDS need)  */
    GSWA_EHIP = -3,         /* a HIP runtime call failed; gswa_last_hip_error() has its text         */
    GSWA_ETOOBIG = -4       /* gswa_backward_static: the layer's scratch exceeds the built-in buffer  */
} gswa_status;

enum { GSWA_F32 = 0, GSWA_BF16 = 1 };

enum {
    GSWA_NO_CASCADE = 1u << 0, /* drop Eq. 8: every group sees only its own channel slice          */
    GSWA_ACCUM_WGRAD = 1u << 1, /* backward adds into the five parameter gradients (no zero fill)  */
    GSWA_FORCE_STAGED = 1u << 2, /* use the one-kernel-per-step path even where a fused kernel exists */
    GSWA_DETERMINISTIC = 1u << 3 /* parameter gradients bit-identical from run to run on every path: the
                                    one-kernel-per-step path then sums them in a fixed order (every split
                                    of the token range and every window adds into a copy of its own, one
                                    launch adds the copies) instead of with fp32 atomics; costs scratch
                                    (64 copies + one bias-table gradient per window) and some time.  The
                                    fused path always sums in a fixed order                               */
};

typedef struct gswa_desc {
    int32_t B, H, W, C;    /* feature map [B, H, W, C]                                        */
    int32_t heads, groups; /* C % heads == 0, heads % groups == 0                              */
    int32_t window, shift; /* H % window == 0, W % window == 0, 0 <= shift < window            */
    int32_t dtype;         /* GSWA_F32 or GSWA_BF16: x, y, dy, dx, weights, biases, bias table */
    uint32_t flags;        /* OR of GSWA_NO_CASCADE, GSWA_ACCUM_WGRAD, GSWA_FORCE_STAGED,
                              GSWA_DETERMINISTIC                                               */
    int32_t dqk;           /* channels of q and of k per head; 0 = C / heads (the plain layer) */
} gswa_desc;

/*
 * Sizes, in bytes, of the caller-provided device buffers (Sec. "Group Shifted Window
 * Attention": the head-group loop is what bounds them).
 *   *saved_bytes   state forward leaves for backward: the concatenated group outputs
 *                  [B*H*W, C] in desc->dtype and, on the fused path, the parameters repacked
 *                  for the matrix cores (tens of KB, independent of B, H, W).  Scores and
 *                  probabilities are never kept; backward recomputes them.
 *   *fwd_ws_bytes  scratch of gswa_forward when `saved` is given (staged path: one group's
 *                  q|k|v; fused path: nothing is used).  For inference (saved == NULL) the
 *                  scratch must hold *fwd_ws_bytes + *saved_bytes: what would have been saved is
 *                  then kept there for the duration of the call.
 *   *bwd_ws_bytes  scratch of gswa_backward.  Staged path: one group's q|k|v and its gradient, plus
 *                  16 fp32 copies of the five parameter gradients (workgroups spread their atomic
 *                  adds over the copies; one launch sums them at the end) and, for bf16 layers with
 *                  64- or 144-token windows, one bias-table gradient per window.
 *                  Fused path: one partial parameter-gradient vector per workgroup of ONE head-group
 *                  launch (each launch is followed by the fixed-order sum of its partials, and the next
 *                  reuses the buffer), so this size does not grow with the group count.  Layers of
 *                  180 channels with two or three groups and 8x8 windows additionally pass ONE
 *                  group's intermediate gradients (d(q|k|v), the group's input and its gradient, as
 *                  matrix-core operand fragments) from the attention kernel to the kernel that forms
 *                  dx and the weight gradients: about 7.6 Cg bytes per token, falling with the group
 *                  count.
 * Which path serves a layer, and every size, depends only on desc (shape, dtype, flags), not on the
 * device.
 * Any output pointer may be NULL.  All sizes are multiples of 256.
 */
int gswa_query_bytes(const gswa_desc *desc, size_t *saved_bytes, size_t *fwd_ws_bytes,
                     size_t *bwd_ws_bytes);

/*
 * Which organisation of kernels serves the layer (a function of desc alone, like the sizes): for callers
 * that want to know before they commit to a shape, since the organisations differ several-fold in speed.
 *   *forward_path, *backward_path  receive one of the values below; either pointer may be NULL.
 * Returns GSWA_OK, or the error gswa_query_bytes would return for desc.
 */
enum {
    GSWA_PATH_STAGED = 0,     /* one kernel per step of Eq. 6-8 and head group (every shape, both types) */
    GSWA_PATH_FUSED = 1,      /* the whole pass in one kernel, or one per head chunk (bf16, 8x8 or 16x16
                                 windows, six heads, C = 60 or 180; backward: 8x8 windows only)          */
    GSWA_PATH_WINDOW_FWD = 2  /* forward in one launch per layer, one workgroup per window (bf16 layers
                                 with narrow q/k or 12x12 windows); their backward is GSWA_PATH_STAGED   */
};
int gswa_query_path(const gswa_desc *desc, int *forward_path, int *backward_path);

/*
 * y = GSWA(x)  (Eq. 6-8 with shift, partition, bias and mask as above).
 *   saved  NULL for inference; otherwise receives what gswa_backward needs and must be left
 *          untouched until that call has run.
 *   ws     scratch, 256-byte aligned, sized by gswa_query_bytes; contents undefined afterwards.
 *          May be NULL when the size the call needs is 0 (training forward on the fused path).
 * y, saved and ws must each be disjoint, as byte ranges of the sizes above, from every other
 * buffer of the call (GSWA_EINVAL otherwise).
 */
int gswa_forward(const gswa_desc *desc, const void *x, const void *w_qkv, const void *b_qkv,
                 const void *w_proj, const void *b_proj, const void *bias_table, void *y,
                 void *saved, void *ws, void *hip_stream);

/*
 * Gradients of a scalar loss through the layer, given dy = dLoss/dy and the `saved` buffer
 * written by gswa_forward on the same desc, x and parameters.
 *   dx                    [B,H,W,C] in desc->dtype, overwritten.
 *   dw_qkv ... dbias_table fp32, overwritten, or added into with GSWA_ACCUM_WGRAD.
 *                         The fused path sums per-workgroup partials in a fixed order (same
 *                         bits every run); the staged path reduces with fp32 atomics, so its
 *                         last bits can differ between runs unless GSWA_DETERMINISTIC is set.
 * dx, the five gradients and ws must each be disjoint, as byte ranges, from every other buffer of
 * the call (GSWA_EINVAL otherwise); ws may be NULL only if *bwd_ws_bytes is 0.
 */
int gswa_backward(const gswa_desc *desc, const void *x, const void *dy, const void *w_qkv,
                  const void *b_qkv, const void *w_proj, const void *b_proj,
                  const void *bias_table, const void *saved, void *dx, void *dw_qkv,
                  void *db_qkv, void *dw_proj, void *db_proj, void *dbias_table, void *ws,
                  void *hip_stream);

/*
 * gswa_backward for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, results and validation as gswa_backward, without `ws`: the scratch is a buffer of
 * GSWA_STATIC_SCRATCH_BYTES that lives inside the library, one per GPU, held until the process
 * ends.  The call allocates and frees nothing (its only runtime queries are hipGetDevice and,
 * on the first call per device, the address lookup of that buffer).
 *   - A layer whose *bwd_ws_bytes (gswa_query_bytes) exceeds GSWA_STATIC_SCRATCH_BYTES is
 *     rejected with GSWA_ETOOBIG before anything is enqueued.
 *   - All calls on one GPU share that GPU's buffer: two calls whose work overlaps in time on the
 *     same GPU (different streams, or different host threads) race.  Serialise them on one stream.
 *   - The buffer keeps the previous call's contents; the kernels clear what they accumulate into.
 */
#define GSWA_STATIC_SCRATCH_BYTES (96u * 1024u * 1024u)
int gswa_backward_static(const gswa_desc *desc, const void *x, const void *dy, const void *w_qkv,
                         const void *b_qkv, const void *w_proj, const void *b_proj,
                         const void *bias_table, const void *saved, void *dx, void *dw_qkv,
                         void *db_qkv, void *dw_proj, void *db_proj, void *dbias_table,
                         void *hip_stream);

/* Static text for a gswa_status value. */
const char *gswa_strerror(int status);

/* Text of the HIP error behind the calling thread's most recent GSWA_EHIP ("" if none). */
const char *gswa_last_hip_error(void);

/* Library version: major*10000 + minor*100 + patch. */
int gswa_version(void);

/*
 * Measurement aid, off by default; not part of the layer's arithmetic.  While enabled, every
 * kernel the library enqueues is bracketed by two HIP events recorded on that kernel's stream
 * (the events are created by the first gswa_profile_enable(1); at most 8192 launches are kept
 * between two collects, later ones are counted in *dropped).  gswa_profile_collect waits for
 * the recorded events, writes per-kernel totals into the HOST arrays total_ms[] and launches[]
 * (gswa_profile_kernel_count() entries each, either may be NULL) and clears the record.
 * Kernel ids are 0 .. count-1; gswa_profile_kernel_name(id) is static text.
 */
int gswa_profile_enable(int on);
int gswa_profile_kernel_count(void);
const char *gswa_profile_kernel_name(int id);
int gswa_profile_collect(double *total_ms, long long *launches, long long *dropped);

#ifdef __cplusplus
}
#endif
#endif /* GSWA_H */
