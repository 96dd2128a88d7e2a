// Fused kernels of the MLP half of a layer (Sec. "Agile Swin Transformer Block", Eq. 5, with the
// skip connection of Eq. 4 folded into its prologue) for narrow bf16 layers on the matrix cores.
#pragma once
#include "common.h"

namespace gswa {

// C <= 64 (multiple of 4) and hidden <= 128: all weights of the MLP fit in LDS as MFMA fragments.
bool astl_mlp_supported(int C, int hidden);

// Bytes of the weights repacked for the matrix cores (written by the forward, read by both passes).
size_t astl_mlp_pack_bytes();

// x1 = x + a (stored);  y = MLP(LN_2(x1)) + x1.  rows tokens of C channels.  `pack` receives the
// repacked weights (astl_mlp_pack_bytes() bytes, 16-byte aligned).
hipError_t launch_astl_mlp_fwd(long rows, int C, int hidden, float eps, const bf16_t *x, const bf16_t *a,
                               const bf16_t *ln_w, const bf16_t *ln_b, const bf16_t *w_fc1, const bf16_t *b_fc1,
                               const bf16_t *w_fc2, const bf16_t *b_fc2, bf16_t *x1, bf16_t *y, void *pack,
                               hipStream_t s);

// The backward kernel also needs one unused channel and one unused hidden feature in its padded
// tiles (C not a multiple of 32, hidden not a multiple of 64): the bias sums ride there.
bool astl_mlp_bwd_supported(int C, int hidden);

// Scratch bytes of the backward (one pair of partial weight-gradient matrices per workgroup).
size_t astl_mlp_bwd_ws_bytes(long rows, int C, int hidden);

// dx1 = dy + adjoint of MLP(LN_2(.)) at x1.  The six parameter gradients (both fully connected
// layers, gamma and beta of LN_2) are written to their final places, or added there when
// `accumulate` is set.  `zero` (may be null) is an fp32 array of nzero entries the first kernel
// clears on the way, for a later launch of the caller's.  `pack` is what the forward call of the
// same layer wrote; `ws` holds astl_mlp_bwd_ws_bytes().
hipError_t launch_astl_mlp_bwd(long rows, int C, int hidden, float eps, const bf16_t *x1, const bf16_t *dy,
                               const bf16_t *ln_w, const bf16_t *ln_b, const bf16_t *w_fc1, const bf16_t *b_fc1,
                               const bf16_t *w_fc2, bf16_t *dx1, float *dw_fc1, float *db_fc1, float *dw_fc2,
                               float *db_fc2, float *dln_w, float *dln_b, int accumulate, float *zero, long nzero,
                               const void *pack, void *ws, hipStream_t s);

} // namespace gswa
