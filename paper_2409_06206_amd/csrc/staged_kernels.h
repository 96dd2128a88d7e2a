// Launchers of the staged (one kernel per step) GSWA path.  This path covers every valid
// layer shape in fp32 arithmetic on plain vector ALUs; the fused MFMA kernels take over the
// shapes they are built for.
#pragma once
#include "common.h"
#include "profile.h"

namespace gswa {

// out[t, n] = sum_k (a1[t,k] + a2[t,k]) * w(n,k) + bias[n] + add[t,n]
// w(n,k) = w[n*w_sn + k*w_sk]; a2, bias, add may be null.  Strides in elements.
struct LinearArgs {
    const void *a1; long lda1;
    const void *a2; long lda2;
    const void *w; long w_sn, w_sk;
    const void *bias;
    const void *add; long ldadd;
    void *out; long ldout;
    long rows; int N, K;
    int prof_id; // KernelId this launch is accounted under
    // Activation folded into the store (only where linear_act_supported() says so; 0 = none):
    //   kActGelu:     v' = the result rounded to the element type; out = GELU(v'), pre_out (may be null) = v'
    //   kActGeluGrad: out = v' * GELU'(aux[t, n])
    // i.e. a pass over the stored result folded into the store (GELU through `gauss` below).
    int act;
    void *pre_out;           // [rows, N], pitch ldout
    const void *aux; long ldaux;
    // LayerNorm folded into the operand read (only where linear_ln_supported() says so; ln_gamma null = none):
    // u = a1 + a2 rounded to the element type goes to sum_out (may be null), LN(u) = (u - mean) rstd gamma + beta
    // rounded to the element type is what the map multiplies, and goes to ln_out (may be null).  Both outputs
    // are [rows, K] of pitch lda1.
    const void *ln_gamma, *ln_beta;
    float ln_eps;
    void *sum_out, *ln_out;
    // optional (may be null): device memory free for the duration of the call; maps whose weight matrix does not
    // fit LDS (up to 576 output columns with K > 384 or more than 192 columns: a wide one-group q|k|v projection
    // and its input gradient) then run on the kernel that streams the repacked weights through LDS
    void *scratch; size_t scratch_bytes;
};
constexpr int kActGelu = 1, kActGeluGrad = 2;
// true when launch_linear<bf16_t> runs this call on the kernel that implements `act`
bool linear_act_supported(const LinearArgs &a);
// true when launch_linear<bf16_t> runs this call on the kernel that implements the LayerNorm of the operand
bool linear_ln_supported(const LinearArgs &a);

// Gaussian CDF Phi(t) and density phi(t): erf by the rational-times-exponential approximation
// 7.1.26 of Abramowitz & Stegun (absolute error below 1.5e-7); exp(-t^2/2) serves both.
__device__ __forceinline__ void gauss(float t, float &Phi, float &phi)
{
    // exp(-t^2/2) as a power of two; with x = |t|/sqrt(2) the formula's 1/(1 + 0.3275911 x) is
    // 1/(1 + 0.2316419 |t|), and its five coefficients are halved here: w = (1 - erf x)/2
    const float e = __builtin_amdgcn_exp2f(t * t * -0.72134752044448170f);
    const float k = __builtin_amdgcn_rcpf(fmaf(fabsf(t), 0.23164190f, 1.f));
    const float poly = ((((0.5307027145f * k - 0.7265760135f) * k + 0.7107068705f) * k - 0.142248368f) * k + 0.127414796f) * k;
    const float w = poly * e;
    Phi = t >= 0.f ? 1.f - w : w;
    phi = 0.39894228040143268f * e;
}

// GELU in its Gaussian-CDF form and its derivative Phi(t) + t phi(t)
__device__ __forceinline__ float gelu_f(float t) { return 0.5f * t * (1.f + erff(t * 0.70710678118654752f)); }
__device__ __forceinline__ float gelu_df(float t)
{
    return 0.5f * (1.f + erff(t * 0.70710678118654752f)) + t * 0.39894228040143268f * __expf(-0.5f * t * t);
}

// Atomic adds of many workgroups to one address serialise (tens of ns each), so the staged
// backward accumulates every parameter gradient in kGradReplicas copies (a workgroup adds into
// copy `its index mod kGradReplicas`), summed at the end by one launch.
constexpr int kGradReplicas = 16;
// Reproducible mode: the token range of a weight gradient is cut into at most this many splits and
// every split owns a copy, so each entry of a copy is one addition onto zero.
constexpr int kDetReplicas = 64;

// dw[n,k] += sum_t dout[t,n] * (a1[t,k] + a2[t,k]);  db[n] += sum_t dout[t,n]   (fp32 atomics).
// dw, db point into copy 0; copy r lies rep_stride floats further (reps copies; 1 = a single array).
struct WgradArgs {
    const void *dout; long lddout;
    const void *a1; long lda1;
    const void *a2; long lda2;
    float *dw; float *db;
    long rep_stride; int reps;
    long rows; int N, K;
    int prof_id;
    int exclusive; // nonzero: at most `reps` splits of the token range, so that every copy receives exactly
                   // one addition per entry (onto zero) and the sum over the copies has a fixed order
    void *scratch; size_t scratch_bytes; // optional (may be null): device memory free for the duration of the call;
                                         // wide layers then take the streaming kernel, which needs no atomics
    // Where the caller knows that the streaming kernel will run (wgrad_pair_streams), dw / db may be the final
    // gradient arrays instead of a zeroed copy: `direct` nonzero, and the sum then writes (accumulate 0) or adds.
    int direct, accumulate;
};

template <typename T> hipError_t launch_linear(const LinearArgs &a, hipStream_t s);
// Two maps that do not depend on each other, in one launch where the kernels allow it; `zero`
// (may be null) is an fp32 array of nzero entries to be cleared by the same launch.
template <typename T>
hipError_t launch_linear_pair(const LinearArgs &a, const LinearArgs &b, float *zero, size_t nzero, hipStream_t s);
template <typename T> hipError_t launch_wgrad(const WgradArgs &a, hipStream_t s);
// The tail of a group's backward: the weight-gradient reduction `a`, optionally a second independent
// one (`b`, may be null) and the linear map `lin` (dF of the group), which all read the same
// d(q|k|v): one launch where the kernels allow it.
// two weight gradients over the same rows and scratch: one launch and one sum where the streaming kernel takes both
template <typename T> hipError_t launch_wgrad_pair(const WgradArgs &a, const WgradArgs &b, hipStream_t s);
// true when launch_wgrad_pair<bf16_t> runs both on the streaming kernel (no copies, no atomics)
bool wgrad_pair_streams(const WgradArgs &a, const WgradArgs &b);
template <typename T>
hipError_t launch_wgrad_group(const WgradArgs &a, const WgradArgs *b, const LinearArgs &lin, hipStream_t s);

// Attention core of head group `grp` (Eq. 6 right-hand side): reads q|k|v [T, Rg] through the
// shift/partition map, writes O into columns of attn_out [T, C] at the tokens' own positions.
template <typename T>
hipError_t launch_attn_fwd(const Geom &g, int grp, const T *qkv, const T *table, T *attn_out,
                           hipStream_t s);

// Adjoint of the attention core for group `grp`.  On entry the v part of dqkv [T, Rg] holds
// dO of the group; on exit dqkv holds dq|dk|dv.  dtable (fp32) is added into: copy
// `window mod reps` of `reps` copies that lie rep_stride floats apart.  reps == 0: one copy per
// window (rep_stride apart), written with plain stores (no zero fill needed, no atomics).
template <typename T>
hipError_t launch_attn_bwd(const Geom &g, int grp, const T *qkv, T *dqkv, const T *table,
                           float *dtable, long rep_stride, int reps, hipStream_t s);

// The same two steps on the matrix cores, for bf16 layers whose windows are 64 or 144 tokens and
// whose heads are at most 32 channels wide (attn_core_mfma_supported); same buffers, same contract.
bool attn_core_mfma_supported(const Geom &g);
hipError_t launch_attn_core_fwd(const Geom &g, int grp, const bf16_t *qkv, const bf16_t *table,
                                bf16_t *attn_out, hipStream_t s);
// Its bias-table gradient is not added anywhere: every (window, head) writes its own copy,
// tpart[window][entry][head] (fp32, nW * (2M-1)^2 * heads entries, no zero fill needed), which
// launch_reduce_replicas sums.
hipError_t launch_attn_core_bwd(const Geom &g, int grp, const bf16_t *qkv, bf16_t *dqkv, const bf16_t *table,
                                float *tpart, hipStream_t s);

// The whole forward of a narrow bf16 layer with 64- or 144-token windows in one launch (one
// workgroup per window, all groups, output projection included); attn_out may be null (inference).
bool window_fwd_supported(const Geom &g);
hipError_t launch_window_fwd(const Geom &g, const bf16_t *x, const bf16_t *w_qkv, const bf16_t *b_qkv,
                             const bf16_t *w_proj, const bf16_t *b_proj, const bf16_t *table, bf16_t *y,
                             bf16_t *attn_out, hipStream_t s);

// LDS bytes the two attention kernels need for this geometry, or 0 if no strip height fits.
size_t attn_fwd_lds_bytes(const Geom &g, int *strip_rows);
size_t attn_bwd_lds_bytes(const Geom &g, int *strip_rows);

// Zero fill of up to eight fp32 arrays in one launch.
struct ZeroList {
    float *p[8];
    size_t n[8];
    int count;
};
hipError_t launch_fill_zero(const ZeroList &z, hipStream_t s);

// out_k[i] (+)= sum_r rep[r * stride + off_k + i] for up to eight output arrays laid out one after
// the other (at offsets off_k) inside every copy.
struct ReplicaSum {
    const float *rep;
    long stride;
    int reps;
    float *out[8];
    long off[8], n[8];
    int count;
    int accumulate;
    // optional: per-window copies of one more output (the bias-table gradient), summed on top of
    // its `reps` copies at offset t_off: t_out[i] (+)= sum_w tpart[w * t_n + i] + copies
    const float *tpart;
    float *t_out;
    long t_off, t_n;
    int t_windows;
};
hipError_t launch_reduce_replicas(const ReplicaSum &r, hipStream_t s);

} // namespace gswa
