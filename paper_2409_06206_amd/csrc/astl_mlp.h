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
// repacked weights (astl_mlp_pack_bytes() bytes, 16-byte aligned).  With next_ln_out non-null the
// kernel also writes LN(y) with the given gamma and beta there: the first step of a layer that
// follows (Eq. 4), of y as stored, at the same eps.
hipError_t launch_astl_mlp_fwd(long rows, int C, int hidden, float eps, const bf16_t *x, const bf16_t *a,
                               const bf16_t *ln_w, const bf16_t *ln_b, const bf16_t *w_fc1, const bf16_t *b_fc1,
                               const bf16_t *w_fc2, const bf16_t *b_fc2, bf16_t *x1, bf16_t *y, void *pack,
                               const bf16_t *next_ln_w, const bf16_t *next_ln_b, bf16_t *next_ln_out, hipStream_t s);

// The same forward for wide layers (64 < C <= 192, hidden <= 384): the weights are streamed through LDS in
// units of 96 hidden features.  Arguments as above (astl_mlp_wide_pack_bytes() bytes at `pack`); x1 may be
// null where nobody reads it afterwards (inference).  With bwd_pack non-null (astl_mlp_wide_bwd_pack_bytes()
// bytes) the same pack launch also writes the weights in the backward kernel's order.
bool astl_mlp_wide_supported(int C, int hidden);
size_t astl_mlp_wide_pack_bytes();
hipError_t launch_astl_mlp_wide_fwd(long rows, int C, int hidden, float eps, const bf16_t *x, const bf16_t *a,
                                    const bf16_t *ln_w, const bf16_t *ln_b, const bf16_t *w_fc1, const bf16_t *b_fc1,
                                    const bf16_t *w_fc2, const bf16_t *b_fc2, bf16_t *x1, bf16_t *y, void *pack,
                                    void *bwd_pack, const bf16_t *next_ln_w, const bf16_t *next_ln_b,
                                    bf16_t *next_ln_out, hipStream_t s);

// Backward of the same layers between the two LayerNorm adjoints, one launch: from x1 and dy it writes
// LN_2(x1) (xn), the hidden layer h and dpre = (dy W2) o GELU'(pre) for the weight gradients, and
// dn = dpre W1 for LayerNorm's adjoint (dn may be null if dx1 is not).  With dx1 non-null the kernel goes on
// through that adjoint and the skip of Eq. 5: dx1 = dy + LN_2's adjoint of dn at x1, and LN_2's d gamma, d beta
// are added into copy (workgroup mod reps) of `reps` copies rep_stride floats apart at dln_w / dln_b (fp32
// atomics, one per channel and workgroup), or with reps == 0 written as one vector [d gamma | d beta] per
// workgroup at dln_w (astl_mlp_wide_bwd_blocks(rows) vectors of 2 C floats; no atomics).  `pack` is what the forward call wrote at its bwd_pack.
size_t astl_mlp_wide_bwd_pack_bytes();
hipError_t launch_astl_mlp_wide_bwd(long rows, int C, int hidden, float eps, const bf16_t *x1, const bf16_t *dy,
                                    const bf16_t *ln_w, const bf16_t *ln_b, const bf16_t *w_fc1, const bf16_t *b_fc1,
                                    const bf16_t *w_fc2, bf16_t *xn, bf16_t *h, bf16_t *dpre, bf16_t *dn, bf16_t *dx1,
                                    float *dln_w, float *dln_b, long rep_stride, int reps, const void *pack,
                                    hipStream_t s);

// LayerNorm of bf16 rows (Eq. 4-5) for 64 < C <= 192, C a multiple of 4: out = LN(u + add) with gamma, beta; `add`
// may be null; with it, the rounded sum goes to sum_out (may be null) and is what gets normalised.
struct LnRowsArgs {
    const bf16_t *u, *add, *gamma, *beta;
    bf16_t *sum_out, *out;
    long rows;
    int C;
    float eps;
};
bool ln_rows_supported(int C);
hipError_t launch_ln_rows_fwd(const LnRowsArgs &a, hipStream_t s);
// The adjoint for the same rows: du = LN's adjoint of dout at u (+ res, may be null).  The gamma / beta sums leave as
// one vector [d gamma: C | d beta: C] per workgroup at `part` (ln_rows_bwd_blocks(rows) of them), to be summed by
// the caller in a fixed order: no atomics.
struct LnRowsBwdArgs {
    const bf16_t *u, *dout, *res, *gamma;
    bf16_t *du;
    float *part;
    long rows;
    int C;
    float eps;
};
int ln_rows_bwd_blocks(long rows);
hipError_t launch_ln_rows_bwd(const LnRowsBwdArgs &a, hipStream_t s);
// workgroups of launch_astl_mlp_wide_bwd for `rows` rows (= partial vectors it writes with reps == 0)
int astl_mlp_wide_bwd_blocks(long rows);

// The backward kernel covers the same shapes.
bool astl_mlp_bwd_supported(int C, int hidden);

// Scratch bytes of the backward (one pair of partial weight-gradient matrices per workgroup).
size_t astl_mlp_bwd_ws_bytes(long rows, int C, int hidden);

// Sums the workgroups' partial results and writes (or adds to) the six parameter gradients:
//   d Wfc1[f][c] = M1[f][c], d Wfc2[c][f] = M2[f][c]; d gamma, d beta of LN_2 and the two bias
//   gradients from the vectors behind the matrices.
// 32 entries per block, the workgroups in 8 slices with eight loads in flight per thread.
struct MlpReduceArgs {
    const float *part;
    int nparts, rows, cols; // a workgroup's partial results: [2][rows][cols], [2][cols] (LN_2), [rows], [cols] (biases)
    int C, Hd;
    int accumulate;
    float *dw1, *db1, *dw2, *db2, *dln_w, *dln_b;
};

inline unsigned astl_mlp_reduce_blocks(const MlpReduceArgs &r)
{
    return (unsigned)((2L * r.rows * r.cols + 3L * r.cols + r.rows + 31) / 32);
}

// work of block `block` of astl_mlp_reduce_blocks() blocks of 256 threads
__device__ __forceinline__ void astl_mlp_reduce_block(const MlpReduceArgs &a, int block)
{
    __shared__ float red[8][33];
    const int col = threadIdx.x & 31, slice = threadIdx.x >> 5;
    const long mats = (long)2 * a.rows * a.cols, per = mats + 3 * a.cols + a.rows;
    const long i = (long)block * 32 + col;
    float acc = 0.f;
    if (i < per) {
        float a8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        int w = slice;
        for (; w + 56 < a.nparts; w += 64) {
#pragma unroll
            for (int u = 0; u < 8; ++u) a8[u] += a.part[(long)(w + 8 * u) * per + i];
        }
        for (; w < a.nparts; w += 8) a8[0] += a.part[(long)w * per + i];
        acc = ((a8[0] + a8[1]) + (a8[2] + a8[3])) + ((a8[4] + a8[5]) + (a8[6] + a8[7]));
    }
    red[slice][col] = acc;
    __syncthreads();
    if (slice == 0 && i < per) {
        float sum = 0.f;
#pragma unroll
        for (int k8 = 0; k8 < 8; ++k8) sum += red[k8][col];
        float *dst = nullptr;
        if (i < mats) {
            const int which = (int)(i / ((long)a.rows * a.cols));
            const int rem = (int)(i % ((long)a.rows * a.cols));
            const int f = rem / a.cols, c = rem % a.cols;
            if (f < a.Hd && c < a.C) dst = which == 0 ? a.dw1 + (long)f * a.C + c : a.dw2 + (long)c * a.Hd + f;
        } else {
            const int j = (int)(i - mats);
            if (j < 2 * a.cols) {
                const int c = j % a.cols;
                if (c < a.C) dst = (j < a.cols ? a.dln_w : a.dln_b) + c;
            } else if (j < 2 * a.cols + a.rows) {
                if (j - 2 * a.cols < a.Hd) dst = a.db1 + (j - 2 * a.cols);
            } else if (j - 2 * a.cols - a.rows < a.C) {
                dst = a.db2 + (j - 2 * a.cols - a.rows);
            }
        }
        if (dst) *dst = a.accumulate ? *dst + sum : sum;
    }
}

// dx1 = dy + adjoint of MLP(LN_2(.)) at x1.  The six parameter gradients (both fully connected
// layers, gamma and beta of LN_2) are written to their final places, or added there when
// `accumulate` is set.  `zero` (may be null) is an fp32 array of nzero entries the first kernel
// clears on the way, for a later launch of the caller's.  `pack` is what the forward call of the
// same layer wrote; `ws` holds astl_mlp_bwd_ws_bytes().  `pending` (may be null): see MlpPending.  With `deferred` non-null the final sum over the
// workgroups' partial results is not launched: its arguments are returned there and the caller runs
// astl_mlp_reduce_block for astl_mlp_reduce_blocks() blocks of 256 threads in a launch of its own.
// Sums the call before left for this one (a sequence of layers, backward): `reps` copies, `stride` floats apart,
// of [w: n | b: n] at `src`; the kernel adds them up into w and b before it clears `zero` (often the same array).
struct MlpPending {
    const float *src;
    float *w, *b;
    int n, reps, accumulate;
    long stride;
};

hipError_t launch_astl_mlp_bwd(long rows, int C, int hidden, float eps, const bf16_t *x1, const bf16_t *dy,
                               const bf16_t *ln_w, const bf16_t *ln_b, const bf16_t *w_fc1, const bf16_t *b_fc1,
                               const bf16_t *w_fc2, bf16_t *dx1, float *dw_fc1, float *db_fc1, float *dw_fc2,
                               float *db_fc2, float *dln_w, float *dln_b, int accumulate, float *zero, long nzero,
                               const void *pack, void *ws, MlpReduceArgs *deferred, const MlpPending *pending,
                               hipStream_t s);

} // namespace gswa
