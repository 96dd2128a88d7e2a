// One whole Agile Swin Transformer Layer (Sec. "Agile Swin Transformer Block", Eq. 4-5) around
// the GSWA layer: LayerNorm, skip connections and the two-layer MLP, plus the C ABI of astl.h.
// This file holds the per-token kernels (LayerNorm and its adjoint, GELU and its derivative) and
// the order in which the steps are enqueued; the matrix products are the library's linear-map
// and weight-gradient kernels.
#include "../../include/astl.h"
#include "common.h"
#include "staged_kernels.h"
#include "astl_mlp.h"
#include "fused.h"

namespace gswa {

namespace {

constexpr int kLnThreads = 256;
constexpr int kLnMaxBlocks = 1024;

// A token's row of C channels is held by 16 lanes: lane l of the 16 owns channels
// V * (16 p + l) + i, p < P, i < V (V = 4 where C is a multiple of 4: one 8- or 16-byte access).
template <typename T, int V> struct Vec;
template <> struct Vec<float, 4> { float4 v; };
template <> struct Vec<float, 1> { float v; };
template <> struct Vec<bf16_t, 4> { uint2 v; };
template <> struct Vec<bf16_t, 1> { uint16_t v; };

__device__ __forceinline__ void unpack(const Vec<float, 4> &r, float *f) { f[0] = r.v.x; f[1] = r.v.y; f[2] = r.v.z; f[3] = r.v.w; }
__device__ __forceinline__ void unpack(const Vec<float, 1> &r, float *f) { f[0] = r.v; }
__device__ __forceinline__ void unpack(const Vec<bf16_t, 4> &r, float *f)
{
    f[0] = __uint_as_float(r.v.x << 16); f[1] = __uint_as_float(r.v.x & 0xffff0000u);
    f[2] = __uint_as_float(r.v.y << 16); f[3] = __uint_as_float(r.v.y & 0xffff0000u);
}
__device__ __forceinline__ void unpack(const Vec<bf16_t, 1> &r, float *f) { f[0] = __uint_as_float((uint32_t)r.v << 16); }
__device__ __forceinline__ void pack(Vec<float, 4> &r, const float *f) { r.v = make_float4(f[0], f[1], f[2], f[3]); }
__device__ __forceinline__ void pack(Vec<float, 1> &r, const float *f) { r.v = f[0]; }
__device__ __forceinline__ void pack(Vec<bf16_t, 4> &r, const float *f)
{
    r.v.x = (uint32_t)f32_to_bf16_bits(f[0]) | (uint32_t)f32_to_bf16_bits(f[1]) << 16;
    r.v.y = (uint32_t)f32_to_bf16_bits(f[2]) | (uint32_t)f32_to_bf16_bits(f[3]) << 16;
}
__device__ __forceinline__ void pack(Vec<bf16_t, 1> &r, const float *f) { r.v = f32_to_bf16_bits(f[0]); }

// value the storage type keeps for f
template <typename T> __device__ __forceinline__ float stored(float f)
{
    if constexpr (sizeof(T) == 2) return __uint_as_float((uint32_t)f32_to_bf16_bits(f) << 16);
    return f;
}

template <typename T, int V, int P>
__device__ __forceinline__ void load_row(const T *row, int C, int l16, float (&f)[P * V])
{
#pragma unroll
    for (int p = 0; p < P; ++p) {
        const int c = V * (16 * p + l16);
        if (c < C) {
            unpack(*reinterpret_cast<const Vec<T, V> *>(row + c), &f[p * V]);
        } else {
#pragma unroll
            for (int i = 0; i < V; ++i) f[p * V + i] = 0.f;
        }
    }
}

template <typename T, int V, int P>
__device__ __forceinline__ void store_row(T *row, int C, int l16, const float (&f)[P * V])
{
#pragma unroll
    for (int p = 0; p < P; ++p) {
        const int c = V * (16 * p + l16);
        if (c < C) pack(*reinterpret_cast<Vec<T, V> *>(row + c), &f[p * V]);
    }
}

// sum over the 16 lanes that share a token
__device__ __forceinline__ float sum16(float v)
{
    v += __shfl_xor(v, 1);
    v += __shfl_xor(v, 2);
    v += __shfl_xor(v, 4);
    v += __shfl_xor(v, 8);
    return v;
}

// mean and 1/sqrt(var + eps) of a token held by 16 lanes (channels beyond C are zero in f)
template <int V, int P>
__device__ __forceinline__ void row_stats(const float (&f)[P * V], int C, int l16, float eps, float &mean, float &rstd)
{
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < P * V; ++k) s += f[k];
    mean = sum16(s) / (float)C;
    float q = 0.f;
#pragma unroll
    for (int p = 0; p < P; ++p)
#pragma unroll
        for (int i = 0; i < V; ++i) {
            const float dlt = f[p * V + i] - mean;
            q += (V * (16 * p + l16) + i < C) ? dlt * dlt : 0.f;
        }
    rstd = rsqrtf(sum16(q) / (float)C + eps);
}

struct LnArgs {
    const void *u;      // [rows, C] input of the LayerNorm ...
    const void *add;    // ... plus this (may be null): Eq. 4's skip, u + add is what gets normalised
    const void *gamma, *beta;
    void *sum_out;      // u + add in the storage type (may be null)
    void *out;          // LN(u + add)
    long rows;
    int C;
    float eps;
};

// LayerNorm of every token (Eq. 4-5).  With `add` the normalised value is the stored (rounded)
// sum, which is also what the backward pass will read back.
template <typename T, int V, int P>
__device__ __forceinline__ void ln_fwd_block(const LnArgs &a, unsigned block, unsigned nblocks)
{
    const int l16 = threadIdx.x & 15;
    const long stride = (long)nblocks * (kLnThreads / 16);
    const T *u = static_cast<const T *>(a.u), *add = static_cast<const T *>(a.add);
    float g[P * V], b[P * V];
    load_row<T, V, P>(static_cast<const T *>(a.gamma), a.C, l16, g);
    load_row<T, V, P>(static_cast<const T *>(a.beta), a.C, l16, b);
    for (long t = (long)block * (kLnThreads / 16) + (threadIdx.x >> 4); t < a.rows; t += stride) {
        float f[P * V];
        load_row<T, V, P>(u + t * a.C, a.C, l16, f);
        if (add) {
            float f2[P * V];
            load_row<T, V, P>(add + t * a.C, a.C, l16, f2);
#pragma unroll
            for (int k = 0; k < P * V; ++k) f[k] = stored<T>(f[k] + f2[k]);
            if (a.sum_out) store_row<T, V, P>(static_cast<T *>(a.sum_out) + t * a.C, a.C, l16, f);
        }
        float mean, rstd;
        row_stats<V, P>(f, a.C, l16, a.eps, mean, rstd);
#pragma unroll
        for (int k = 0; k < P * V; ++k) f[k] = (f[k] - mean) * rstd * g[k] + b[k];
        store_row<T, V, P>(static_cast<T *>(a.out) + t * a.C, a.C, l16, f);
    }
}

template <typename T, int V, int P>
__global__ __launch_bounds__(kLnThreads) void ln_fwd_kernel(LnArgs a)
{
    ln_fwd_block<T, V, P>(a, blockIdx.x, gridDim.x);
}

// The same LayerNorm with, in the first `red_blocks` workgroups of the launch, the final sum of the
// fused MLP backward's partial results: two short pieces of work that do not depend on each other.
template <typename T, int V, int P>
__global__ __launch_bounds__(kLnThreads) void ln_fwd_reduce_kernel(LnArgs a, MlpReduceArgs r, unsigned red_blocks)
{
    if (blockIdx.x < red_blocks) {
        astl_mlp_reduce_block(r, (int)blockIdx.x);
        return;
    }
    ln_fwd_block<T, V, P>(a, blockIdx.x - red_blocks, gridDim.x - red_blocks);
}

struct LnBwdArgs {
    const void *u;      // [rows, C] input the LayerNorm saw
    const void *dout;   // gradient with respect to the LayerNorm's output
    const void *res;    // gradient arriving over the skip connection, added to du (may be null)
    const void *gamma;
    void *du;           // [rows, C]
    float *dgamma, *dbeta; // copy 0 of `reps` copies rep_stride floats apart, added into
    long rep_stride;
    int reps;
    long rows;
    int C;
    float eps;
};

// Adjoint of LayerNorm: with xh = (u - mean) rstd and g = dout * gamma,
//   du = rstd (g - mean(g) - xh mean(g xh)) (+ res);  dgamma = sum_t dout xh;  dbeta = sum_t dout.
template <typename T, int V, int P>
__global__ __launch_bounds__(kLnThreads) void ln_bwd_kernel(LnBwdArgs a)
{
    __shared__ float red[kLnThreads / 64][2][16 * P * V];
    const int l16 = threadIdx.x & 15, wave = threadIdx.x >> 6;
    const long stride = (long)gridDim.x * (kLnThreads / 16);
    const T *u = static_cast<const T *>(a.u), *dout = static_cast<const T *>(a.dout);
    const T *res = static_cast<const T *>(a.res);
    float g[P * V], ag[P * V], ab[P * V];
    load_row<T, V, P>(static_cast<const T *>(a.gamma), a.C, l16, g);
#pragma unroll
    for (int k = 0; k < P * V; ++k) ag[k] = ab[k] = 0.f;
    for (long t = (long)blockIdx.x * (kLnThreads / 16) + (threadIdx.x >> 4); t < a.rows; t += stride) {
        float f[P * V], d[P * V];
        load_row<T, V, P>(u + t * a.C, a.C, l16, f);
        load_row<T, V, P>(dout + t * a.C, a.C, l16, d);
        float mean, rstd;
        row_stats<V, P>(f, a.C, l16, a.eps, mean, rstd);
        float s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int p = 0; p < P; ++p)
#pragma unroll
            for (int i = 0; i < V; ++i) {
                const int k = p * V + i;
                const bool in = V * (16 * p + l16) + i < a.C;
                f[k] = in ? (f[k] - mean) * rstd : 0.f; // xh
                ag[k] += d[k] * f[k];
                ab[k] += d[k];
                d[k] *= g[k];
                s1 += d[k];
                s2 += d[k] * f[k];
            }
        s1 = sum16(s1) / (float)a.C;
        s2 = sum16(s2) / (float)a.C;
#pragma unroll
        for (int k = 0; k < P * V; ++k) d[k] = rstd * (d[k] - s1 - f[k] * s2);
        if (res) {
            float r[P * V];
            load_row<T, V, P>(res + t * a.C, a.C, l16, r);
#pragma unroll
            for (int k = 0; k < P * V; ++k) d[k] += r[k];
        }
        store_row<T, V, P>(static_cast<T *>(a.du) + t * a.C, a.C, l16, d);
    }
    // the four tokens of a wave, then the waves of the workgroup, then one add per channel
#pragma unroll
    for (int k = 0; k < P * V; ++k) {
        ag[k] += __shfl_xor(ag[k], 16); ag[k] += __shfl_xor(ag[k], 32);
        ab[k] += __shfl_xor(ab[k], 16); ab[k] += __shfl_xor(ab[k], 32);
    }
    if ((threadIdx.x & 63) < 16) {
#pragma unroll
        for (int k = 0; k < P * V; ++k) {
            red[wave][0][k * 16 + l16] = ag[k];
            red[wave][1][k * 16 + l16] = ab[k];
        }
    }
    __syncthreads();
    const int rep = (int)(blockIdx.x % (unsigned)a.reps);
    for (int e = threadIdx.x; e < 2 * 16 * P * V; e += kLnThreads) {
        const int which = e / (16 * P * V), r = e % (16 * P * V);
        const int k = r / 16, l = r % 16, p = k / V, i = k % V;
        const int c = V * (16 * p + l) + i;
        if (c >= a.C) continue;
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < kLnThreads / 64; ++w) s += red[w][which][r];
        atomicAdd((which ? a.dbeta : a.dgamma) + (long)rep * a.rep_stride + c, s);
    }
}

unsigned ln_blocks(long rows, int max_blocks)
{
    long b = (rows + kLnThreads / 16 - 1) / (kLnThreads / 16);
    return (unsigned)(b > max_blocks ? max_blocks : (b < 1 ? 1 : b));
}

template <typename T, int V> hipError_t launch_ln_fwd_v(const LnArgs &a, const MlpReduceArgs *r, hipStream_t s)
{
    const int P = (a.C + 16 * V - 1) / (16 * V);
    const dim3 block(kLnThreads);
    if (r) {   // with the MLP's final sum in front
        const unsigned rb = astl_mlp_reduce_blocks(*r);
        const dim3 grid(rb + ln_blocks(a.rows, 4 * kLnMaxBlocks));
        KernelTimer kt(K_LN_FWD_REDUCE, s);
        if constexpr (V == 4) {
            switch (P) {
            case 1: hipLaunchKernelGGL((ln_fwd_reduce_kernel<T, 4, 1>), grid, block, 0, s, a, *r, rb); break;
            case 2: hipLaunchKernelGGL((ln_fwd_reduce_kernel<T, 4, 2>), grid, block, 0, s, a, *r, rb); break;
            case 3: hipLaunchKernelGGL((ln_fwd_reduce_kernel<T, 4, 3>), grid, block, 0, s, a, *r, rb); break;
            default: hipLaunchKernelGGL((ln_fwd_reduce_kernel<T, 4, 4>), grid, block, 0, s, a, *r, rb); break;
            }
        } else {
            if (P <= 4) hipLaunchKernelGGL((ln_fwd_reduce_kernel<T, 1, 4>), grid, block, 0, s, a, *r, rb);
            else hipLaunchKernelGGL((ln_fwd_reduce_kernel<T, 1, 16>), grid, block, 0, s, a, *r, rb);
        }
        return hipGetLastError();
    }
    KernelTimer kt(K_LN_FWD, s);
    const dim3 grid(ln_blocks(a.rows, 4 * kLnMaxBlocks));
    if constexpr (V == 4) {
        switch (P) {
        case 1: hipLaunchKernelGGL((ln_fwd_kernel<T, 4, 1>), grid, block, 0, s, a); break;
        case 2: hipLaunchKernelGGL((ln_fwd_kernel<T, 4, 2>), grid, block, 0, s, a); break;
        case 3: hipLaunchKernelGGL((ln_fwd_kernel<T, 4, 3>), grid, block, 0, s, a); break;
        default: hipLaunchKernelGGL((ln_fwd_kernel<T, 4, 4>), grid, block, 0, s, a); break;
        }
    } else {
        if (P <= 4) hipLaunchKernelGGL((ln_fwd_kernel<T, 1, 4>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((ln_fwd_kernel<T, 1, 16>), grid, block, 0, s, a);
    }
    return hipGetLastError();
}

template <typename T> hipError_t launch_ln_fwd(const LnArgs &a, hipStream_t s, const MlpReduceArgs *r = nullptr)
{
    if constexpr (sizeof(T) == 2) {
        // bf16 rows of 65 to 192 channels: the kernel with four lanes per row and whole tiles of loads in flight
        // (whatever the number of rows: a band of a map must get the arithmetic the whole map gets)
        if (!r && ln_rows_supported(a.C)) {
            LnRowsArgs n{};
            n.u = static_cast<const bf16_t *>(a.u); n.add = static_cast<const bf16_t *>(a.add);
            n.gamma = static_cast<const bf16_t *>(a.gamma); n.beta = static_cast<const bf16_t *>(a.beta);
            n.sum_out = static_cast<bf16_t *>(a.sum_out); n.out = static_cast<bf16_t *>(a.out);
            n.rows = a.rows; n.C = a.C; n.eps = a.eps;
            KernelTimer kt(K_LN_FWD, s);
            return launch_ln_rows_fwd(n, s);
        }
    }
    return (a.C % 4 == 0) ? launch_ln_fwd_v<T, 4>(a, r, s) : launch_ln_fwd_v<T, 1>(a, r, s);
}

template <typename T, int V> hipError_t launch_ln_bwd_v(const LnBwdArgs &a, hipStream_t s)
{
    const int P = (a.C + 16 * V - 1) / (16 * V);
    KernelTimer kt(K_LN_BWD, s);
    const dim3 grid(ln_blocks(a.rows, 2 * kLnMaxBlocks)), block(kLnThreads);
    if constexpr (V == 4) {
        switch (P) {
        case 1: hipLaunchKernelGGL((ln_bwd_kernel<T, 4, 1>), grid, block, 0, s, a); break;
        case 2: hipLaunchKernelGGL((ln_bwd_kernel<T, 4, 2>), grid, block, 0, s, a); break;
        case 3: hipLaunchKernelGGL((ln_bwd_kernel<T, 4, 3>), grid, block, 0, s, a); break;
        default: hipLaunchKernelGGL((ln_bwd_kernel<T, 4, 4>), grid, block, 0, s, a); break;
        }
    } else {
        if (P <= 4) hipLaunchKernelGGL((ln_bwd_kernel<T, 1, 4>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((ln_bwd_kernel<T, 1, 16>), grid, block, 0, s, a);
    }
    return hipGetLastError();
}

template <typename T> hipError_t launch_ln_bwd(const LnBwdArgs &a, hipStream_t s)
{
    return (a.C % 4 == 0) ? launch_ln_bwd_v<T, 4>(a, s) : launch_ln_bwd_v<T, 1>(a, s);
}

// (GELU and its derivative: staged_kernels.h)
// h = GELU(pre);  with dh: dh <- dh * GELU'(pre) in place (h not written)
template <typename T>
__global__ __launch_bounds__(256) void gelu_kernel(const T *pre, T *h, T *dh, long n)
{
    for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (long)gridDim.x * blockDim.x) {
        const float t = to_f32(pre[i]);
        if (dh) from_f32(dh[i], to_f32(dh[i]) * gelu_df(t));
        else from_f32(h[i], gelu_f(t));
    }
}

template <typename T> hipError_t launch_gelu(const T *pre, T *h, T *dh, long n, hipStream_t s)
{
    long blocks = (n + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    KernelTimer kt(dh ? K_GELU_BWD : K_GELU_FWD, s);
    hipLaunchKernelGGL(gelu_kernel<T>, dim3((unsigned)blocks), dim3(256), 0, s, pre, h, dh, n);
    return hipGetLastError();
}

size_t align256(size_t b) { return (b + 255) & ~size_t(255); }
template <typename... P> bool aligned16(P... p) { return (((reinterpret_cast<uintptr_t>(p)) | ...) & 15) == 0; }

// Byte offsets of everything the two calls carve out of `saved` and `ws`.
struct Plan {
    long T;
    int C, Hd;
    size_t e;
    size_t act, hid;              // bytes of a [T, C] and of a [T, hidden] tensor (256-aligned)
    size_t at_saved, at_fws, at_bws; // the attention layer's own needs
    size_t saved, fwd_ws, bwd_ws;
    size_t params;                // fp32 entries of one copy of this file's parameter gradients
    size_t reps;                  // bytes of the kGradReplicas copies
    size_t pack;                  // bytes of the MLP's repacked weights at the end of `saved` (fused MLP)
    bool fused_mlp, fused_mlp_bwd;
    bool wide_mlp;                // forward of the MLP half by the streaming kernel for wide layers
};

int make_plan(const astl_desc *d, Plan *p)
{
    if (!d) return GSWA_EINVAL;
    int rc = gswa_query_bytes(&d->attn, &p->at_saved, &p->at_fws, &p->at_bws);
    if (rc != GSWA_OK) return rc;
    if (d->hidden <= 0 || !(d->eps >= 0.f)) return GSWA_EINVAL;
    if (d->attn.C > 256 || d->hidden > (1 << 20)) return GSWA_EUNSUPPORTED;
    p->T = (long)d->attn.B * d->attn.H * d->attn.W;
    p->C = d->attn.C; p->Hd = d->hidden;
    p->e = d->attn.dtype == GSWA_F32 ? 4 : 2;
    if (p->T * (long)p->Hd >= (1L << 40)) return GSWA_EUNSUPPORTED;
    p->act = align256((size_t)p->T * p->C * p->e);
    p->hid = align256((size_t)p->T * p->Hd * p->e);
    p->fused_mlp = d->attn.dtype == GSWA_BF16 && !(d->attn.flags & GSWA_FORCE_STAGED) &&
                   astl_mlp_supported(p->C, p->Hd);
    p->fused_mlp_bwd = p->fused_mlp && astl_mlp_bwd_supported(p->C, p->Hd);
    p->wide_mlp = !p->fused_mlp && d->attn.dtype == GSWA_BF16 && !(d->attn.flags & GSWA_FORCE_STAGED) &&
                  astl_mlp_wide_supported(p->C, p->Hd);
    // (with the fused MLP backward only LN_1's two vectors go through the gradient copies)
    p->params = p->fused_mlp_bwd ? 2 * (size_t)p->C : 2 * (size_t)p->C * p->Hd + p->Hd + 5 * (size_t)p->C;
    p->reps = align256(kGradReplicas * p->params * sizeof(float));
    // (wide layers: the forward kernel's order of the MLP weights, then the backward kernel's)
    p->pack = p->fused_mlp ? astl_mlp_pack_bytes()
              : p->wide_mlp ? astl_mlp_wide_pack_bytes() + astl_mlp_wide_bwd_pack_bytes() : 0;
    p->saved = p->act + p->at_saved + p->pack;
    // forward: xn | a | max(attention scratch (+ its saved state at inference), pre | h)
    const size_t hid_f = p->fused_mlp || p->wide_mlp ? 0 : 2 * p->hid;
    p->fwd_ws = 2 * p->act + (p->at_fws > hid_f ? p->at_fws : hid_f);
    // backward: xn | dn | dx1 | max(pre | h | dh, attention scratch) | copies of the gradients
    const size_t hid_b = p->fused_mlp_bwd ? astl_mlp_bwd_ws_bytes(p->T, p->C, p->Hd) : 3 * p->hid;
    p->bwd_ws = 3 * p->act + (p->at_bws > hid_b ? p->at_bws : hid_b) + p->reps;
    return GSWA_OK;
}

#define ASTL_HIP(expr)                                         \
    do {                                                       \
        hipError_t e_ = (expr);                                \
        if (e_ != hipSuccess) return report_hip_error(e_);     \
    } while (0)
#define ASTL_RC(expr)                  \
    do {                               \
        int rc_ = (expr);              \
        if (rc_ != GSWA_OK) return rc_; \
    } while (0)

// What a sequence of layers hands from one forward call to the next: all layers of a sequence
// use the same scratch, whose first slot holds LN_1(x) of the running layer.
struct LayerLink {
    bool have_ln1;             // in: the slot already holds LN_1(x) of this layer
    const astl_params *next;   // in: the layer that follows (null: none)
    bool emitted;              // out: the slot now holds LN_1 of the next layer's input
};

template <typename T>
int forward_t(const astl_desc *d, const Plan &pl, const T *x, const astl_params *p, T *y, char *saved,
              char *ws, hipStream_t st, LayerLink *link)
{
    const long rows = pl.T;
    const int C = pl.C, Hd = pl.Hd;
    T *xn = reinterpret_cast<T *>(ws);
    T *a = reinterpret_cast<T *>(ws + pl.act);
    // at inference x1 takes a third slot of the scratch and the attention layer keeps what it
    // would have saved behind its own scratch; the caller sized ws as fwd_ws + saved for this
    T *x1 = reinterpret_cast<T *>(saved ? saved : ws + 2 * pl.act);
    char *rest = ws + (saved ? 2 : 3) * pl.act;
    void *at_saved = saved ? static_cast<void *>(saved + pl.act) : nullptr;
    // (the repacked MLP weights close the saved state, wherever that lives)
    void *pack = (saved ? saved + pl.saved : ws + pl.fwd_ws + pl.saved) - pl.pack;

    // Eq. 4: x1 = GSWA(LN_1(x)) + x
    if (!(link && link->have_ln1)) {
        LnArgs l1{};
        l1.u = x; l1.gamma = p->ln1_w; l1.beta = p->ln1_b; l1.out = xn; l1.rows = rows; l1.C = C; l1.eps = d->eps;
        ASTL_HIP(launch_ln_fwd<T>(l1, st));
    }
    if (link) link->emitted = false;
    ASTL_RC(gswa_forward(&d->attn, xn, p->w_qkv, p->b_qkv, p->w_proj, p->b_proj, p->bias_table, a, at_saved,
                         rest, st));
    if (pl.fused_mlp) {
        // Eq. 4's skip and the whole of Eq. 5 in one launch; in a sequence of layers also LN_1 of
        // the layer that follows (the slot's present content is no longer needed by then)
        const astl_params *nx = link ? link->next : nullptr;
        ASTL_HIP(launch_astl_mlp_fwd(rows, C, Hd, d->eps, (const bf16_t *)x, (const bf16_t *)a,
                                     (const bf16_t *)p->ln2_w, (const bf16_t *)p->ln2_b,
                                     (const bf16_t *)p->w_fc1, (const bf16_t *)p->b_fc1,
                                     (const bf16_t *)p->w_fc2, (const bf16_t *)p->b_fc2,
                                     (bf16_t *)x1, (bf16_t *)y, pack, nx ? (const bf16_t *)nx->ln1_w : nullptr,
                                     nx ? (const bf16_t *)nx->ln1_b : nullptr, nx ? (bf16_t *)xn : nullptr, st));
        if (link && nx) link->emitted = true;
        return GSWA_OK;
    }
    if (pl.wide_mlp) {
        // the same for wide layers, the weights streamed through LDS; x1 is stored only where the backward
        // pass will read it
        const astl_params *nx = link ? link->next : nullptr;
        ASTL_HIP(launch_astl_mlp_wide_fwd(rows, C, Hd, d->eps, (const bf16_t *)x, (const bf16_t *)a,
                                          (const bf16_t *)p->ln2_w, (const bf16_t *)p->ln2_b,
                                          (const bf16_t *)p->w_fc1, (const bf16_t *)p->b_fc1,
                                          (const bf16_t *)p->w_fc2, (const bf16_t *)p->b_fc2,
                                          saved ? (bf16_t *)x1 : nullptr, (bf16_t *)y, pack,
                                          saved ? static_cast<char *>(pack) + astl_mlp_wide_pack_bytes() : nullptr,
                                          nx ? (const bf16_t *)nx->ln1_w : nullptr,
                                          nx ? (const bf16_t *)nx->ln1_b : nullptr, nx ? (bf16_t *)xn : nullptr, st));
        if (link && nx) link->emitted = true;
        return GSWA_OK;
    }
    // Eq. 5: y = MLP(LN_2(x1)) + x1
    T *pre = reinterpret_cast<T *>(rest), *h = reinterpret_cast<T *>(rest + pl.hid);
    LinearArgs f1{};
    f1.a1 = xn; f1.lda1 = C; f1.w = p->w_fc1; f1.w_sn = C; f1.w_sk = 1; f1.bias = p->b_fc1;
    f1.out = pre; f1.ldout = Hd; f1.rows = rows; f1.N = Hd; f1.K = C; f1.prof_id = K_FC1_LINEAR;
    // Eq. 4's skip and LN_2 in the operand read of the first map where its kernel has them: x1 is
    // written from there and LN_2(x1) never leaves the registers
    LinearArgs f1n = f1;
    f1n.a1 = x; f1n.a2 = a; f1n.lda2 = C; f1n.sum_out = x1;
    f1n.ln_gamma = p->ln2_w; f1n.ln_beta = p->ln2_b; f1n.ln_eps = d->eps;
    if (sizeof(T) == 2 && linear_ln_supported(f1n)) {
        f1 = f1n;
    } else {
        LnArgs l2{};
        l2.u = x; l2.add = a; l2.gamma = p->ln2_w; l2.beta = p->ln2_b; l2.sum_out = x1; l2.out = xn;
        l2.rows = rows; l2.C = C; l2.eps = d->eps;
        ASTL_HIP(launch_ln_fwd<T>(l2, st));
    }
    if (sizeof(T) == 2 && linear_act_supported(f1)) {
        // the hidden layer straight from the product (the pre-activation is never read in this pass)
        f1.act = kActGelu; f1.out = h;
        ASTL_HIP(launch_linear<T>(f1, st));
    } else {
        ASTL_HIP(launch_linear<T>(f1, st));
        ASTL_HIP(launch_gelu<T>(pre, h, nullptr, rows * Hd, st));
    }
    LinearArgs f2{};
    f2.a1 = h; f2.lda1 = Hd; f2.w = p->w_fc2; f2.w_sn = Hd; f2.w_sk = 1; f2.bias = p->b_fc2;
    f2.add = x1; f2.ldadd = C;
    f2.out = y; f2.ldout = C; f2.rows = rows; f2.N = C; f2.K = Hd; f2.prof_id = K_FC2_LINEAR;
    ASTL_HIP(launch_linear<T>(f2, st));
    return GSWA_OK;
}

// What a sequence of layers hands from one backward call to the next (the layer BEFORE it in the network):
// the sum of the copies of LayerNorm-1's gradients is the last, tiny launch of a layer; where the next call
// starts with the fused MLP backward, that kernel's first workgroup takes the sum over on its way.
struct BackLink {
    MlpPending pending; // in: sums the previous call left (w == null: none);  out: sums this call leaves
    bool may_defer;     // in: another call of the same sequence follows and will take this call's sums
};

template <typename T>
int backward_t(const astl_desc *d, const Plan &pl, const T *x, const T *dy, const astl_params *p,
               const char *saved, T *dx, const astl_grads *g, char *ws, hipStream_t st, BackLink *link)
{
    const long rows = pl.T;
    const int C = pl.C, Hd = pl.Hd;
    const T *x1 = reinterpret_cast<const T *>(saved);
    const void *at_saved = saved + pl.act;
    T *xn = reinterpret_cast<T *>(ws);
    T *dn = reinterpret_cast<T *>(ws + pl.act);
    T *dx1 = reinterpret_cast<T *>(ws + 2 * pl.act);
    char *rest = ws + 3 * pl.act;
    float *rep = reinterpret_cast<float *>(ws + pl.bwd_ws - pl.reps);
    // one copy of the gradients: dw_fc1 | db_fc1 | dw_fc2 | db_fc2 | dln1_w | dln1_b | dln2_w | dln2_b;
    // with the fused MLP backward, which writes its six gradients itself: dln1_w | dln1_b only
    const bool own = pl.fused_mlp_bwd;
    // Wide layers whose four MLP weight gradients come from the streaming kernel (its own partial arrays and a
    // fixed-order sum straight into the gradients): no gradient copies, no atomics anywhere in this file's part
    // (Then the copies' memory is free too: the kernel's scratch runs from behind h | dpre to the end of the
    // workspace, less the LayerNorms' partial vectors, which close it.)
    bool mlp_direct = false;
    const int nparts2 = pl.wide_mlp ? astl_mlp_wide_bwd_blocks(rows) : 0;
    const int nparts1 = pl.wide_mlp ? ln_rows_bwd_blocks(rows) : 0;
    const size_t ln_bytes = align256((size_t)(nparts1 + nparts2) * 2 * C * sizeof(float));
    char *wg_scratch = ws + 3 * pl.act + 2 * pl.hid;
    size_t wg_scratch_bytes = pl.hid;
    if (pl.wide_mlp && ln_bytes <= pl.reps) {
        const size_t all = (size_t)((ws + pl.bwd_ws) - wg_scratch) - ln_bytes;
        WgradArgs t2{}, t1{};
        t2.dout = dy; t2.lddout = C; t2.a1 = ws; t2.lda1 = Hd; t2.rows = rows; t2.N = C; t2.K = Hd; t2.reps = 1;
        t1.dout = ws; t1.lddout = Hd; t1.a1 = ws; t1.lda1 = C; t1.rows = rows; t1.N = Hd; t1.K = C; t1.reps = 1;
        t2.scratch = t1.scratch = wg_scratch; t2.scratch_bytes = t1.scratch_bytes = all;
        mlp_direct = wgrad_pair_streams(t2, t1);
        if (mlp_direct) wg_scratch_bytes = all;
    }
    const long P = (long)pl.params;
    const long o_w1 = 0, o_b1 = o_w1 + (long)Hd * C, o_w2 = o_b1 + Hd, o_b2 = o_w2 + (long)C * Hd;
    const long o_g1 = own ? 0 : o_b2 + C, o_be1 = o_g1 + C, o_g2 = o_be1 + C, o_be2 = o_g2 + C;
    const int accumulate = (d->attn.flags & GSWA_ACCUM_WGRAD) ? 1 : 0;

    MlpPending pend{};
    if (link) {
        pend = link->pending;
        link->pending = MlpPending{};
    }
    if (pend.w && !own) { // (no kernel of this call takes the pending sums over: a launch of their own)
        ReplicaSum ps{};
        ps.rep = const_cast<float *>(pend.src); ps.stride = pend.stride; ps.reps = pend.reps;
        ps.out[0] = pend.w; ps.off[0] = 0; ps.n[0] = pend.n;
        ps.out[1] = pend.b; ps.off[1] = pend.n; ps.n[1] = pend.n;
        ps.count = 2;
        ps.accumulate = pend.accumulate;
        ASTL_HIP(launch_reduce_replicas(ps, st));
    }
    // (mlp_direct: nothing is added into copies at all.  The two LayerNorms' gamma / beta sums leave their kernels
    // as one vector per workgroup, in the copies' memory, and one launch sums both sets in a fixed order.)
    float *lnpart2 = reinterpret_cast<float *>(ws + pl.bwd_ws - ln_bytes);
    float *lnpart1 = lnpart2 + (size_t)nparts2 * 2 * C;
    if (!own && !mlp_direct) {
        ZeroList z{};
        z.p[0] = rep; z.n[0] = (size_t)kGradReplicas * P; z.count = 1;
        ASTL_HIP(launch_fill_zero(z, st));
    }

    // Eq. 5 backwards
    MlpReduceArgs mlp_sum{};
    if (pl.fused_mlp_bwd) {
        ASTL_HIP(launch_astl_mlp_bwd(rows, C, Hd, d->eps, (const bf16_t *)x1, (const bf16_t *)dy,
                                     (const bf16_t *)p->ln2_w, (const bf16_t *)p->ln2_b,
                                     (const bf16_t *)p->w_fc1, (const bf16_t *)p->b_fc1,
                                     (const bf16_t *)p->w_fc2, (bf16_t *)dx1, g->w_fc1, g->b_fc1, g->w_fc2,
                                     g->b_fc2, g->ln2_w, g->ln2_b, accumulate, rep, (long)kGradReplicas * P,
                                     saved + pl.saved - pl.pack, rest, &mlp_sum, pend.w ? &pend : nullptr, st));
    } else if (pl.wide_mlp) {
        // one launch from x1 and dy to dx1 (through LN_2's adjoint and the skip of Eq. 5; its gamma / beta sums
        // go into the gradient copies); LN_2(x1), h and dpre are written for the weight gradients
        T *h = reinterpret_cast<T *>(rest), *dpre = reinterpret_cast<T *>(rest + pl.hid);
        ASTL_HIP(launch_astl_mlp_wide_bwd(rows, C, Hd, d->eps, (const bf16_t *)x1, (const bf16_t *)dy,
                                          (const bf16_t *)p->ln2_w, (const bf16_t *)p->ln2_b,
                                          (const bf16_t *)p->w_fc1, (const bf16_t *)p->b_fc1,
                                          (const bf16_t *)p->w_fc2, (bf16_t *)xn, (bf16_t *)h, (bf16_t *)dpre,
                                          nullptr, (bf16_t *)dx1, mlp_direct ? lnpart2 : rep + o_g2,
                                          mlp_direct ? nullptr : rep + o_be2, P, mlp_direct ? 0 : kGradReplicas,
                                          saved + pl.saved - pl.pack + astl_mlp_wide_pack_bytes(), st));
        // d Wfc2 = dy^T h,  d Wfc1 = dpre^T LN_2(x1)
        WgradArgs w2{};
        w2.dout = dy; w2.lddout = C; w2.a1 = h; w2.lda1 = Hd;
        w2.dw = rep + o_w2; w2.db = rep + o_b2; w2.rep_stride = P; w2.reps = kGradReplicas;
        w2.rows = rows; w2.N = C; w2.K = Hd; w2.prof_id = K_FC_WGRAD;
        w2.scratch = wg_scratch; w2.scratch_bytes = wg_scratch_bytes;
        WgradArgs w1{};
        w1.dout = dpre; w1.lddout = Hd; w1.a1 = xn; w1.lda1 = C;
        w1.dw = rep + o_w1; w1.db = rep + o_b1; w1.rep_stride = P; w1.reps = kGradReplicas;
        w1.rows = rows; w1.N = Hd; w1.K = C; w1.prof_id = K_FC_WGRAD;
        w1.scratch = wg_scratch; w1.scratch_bytes = wg_scratch_bytes;
        if (mlp_direct) { // (no copies: the kernel's sum writes, or adds to, the gradients themselves)
            w2.dw = g->w_fc2; w2.db = g->b_fc2; w1.dw = g->w_fc1; w1.db = g->b_fc1;
            w2.direct = w1.direct = 1; w2.accumulate = w1.accumulate = accumulate;
        }
        ASTL_HIP(launch_wgrad_pair<T>(w2, w1, st));
    } else {
        T *pre = reinterpret_cast<T *>(rest), *h = reinterpret_cast<T *>(rest + pl.hid);
        T *dh = reinterpret_cast<T *>(rest + 2 * pl.hid);
        // recompute LN_2(x1), the pre-activation and the hidden layer
        LinearArgs f1{};
        f1.a1 = xn; f1.lda1 = C; f1.w = p->w_fc1; f1.w_sn = C; f1.w_sk = 1; f1.bias = p->b_fc1;
        f1.out = pre; f1.ldout = Hd; f1.rows = rows; f1.N = Hd; f1.K = C; f1.prof_id = K_FC1_LINEAR;
        // (LN_2 in the operand read of the first map where its kernel has it; the weight gradient below
        // still wants LN_2(x1) in memory)
        LinearArgs f1n = f1;
        f1n.a1 = x1; f1n.ln_out = xn; f1n.ln_gamma = p->ln2_w; f1n.ln_beta = p->ln2_b; f1n.ln_eps = d->eps;
        if (sizeof(T) == 2 && linear_ln_supported(f1n)) {
            f1 = f1n;
        } else {
            LnArgs l2{};
            l2.u = x1; l2.gamma = p->ln2_w; l2.beta = p->ln2_b; l2.out = xn; l2.rows = rows; l2.C = C; l2.eps = d->eps;
            ASTL_HIP(launch_ln_fwd<T>(l2, st));
        }
        if (sizeof(T) == 2 && linear_act_supported(f1)) {
            f1.act = kActGelu; f1.out = h; f1.pre_out = pre;
            ASTL_HIP(launch_linear<T>(f1, st));
        } else {
            ASTL_HIP(launch_linear<T>(f1, st));
            ASTL_HIP(launch_gelu<T>(pre, h, nullptr, rows * Hd, st));
        }
        // dh = dy Wfc2 (through the GELU in the same launch where the kernel can);  d Wfc2 = dy^T h
        LinearArgs b2{};
        b2.a1 = dy; b2.lda1 = C; b2.w = p->w_fc2; b2.w_sn = 1; b2.w_sk = Hd;
        b2.out = dh; b2.ldout = Hd; b2.rows = rows; b2.N = Hd; b2.K = C; b2.prof_id = K_FC_DLINEAR;
        const bool gelu_in_b2 = sizeof(T) == 2 && linear_act_supported(b2);
        if (gelu_in_b2) { b2.act = kActGeluGrad; b2.aux = pre; b2.ldaux = Hd; }
        ASTL_HIP(launch_linear<T>(b2, st));
        WgradArgs w2{};
        w2.dout = dy; w2.lddout = C; w2.a1 = h; w2.lda1 = Hd;
        w2.dw = rep + o_w2; w2.db = rep + o_b2; w2.rep_stride = P; w2.reps = kGradReplicas;
        w2.rows = rows; w2.N = C; w2.K = Hd; w2.prof_id = K_FC_WGRAD;
        // (dn and dx1 are not written before the last weight gradient is done: their slots serve as scratch)
        w2.scratch = ws + pl.act; w2.scratch_bytes = 2 * pl.act;
        ASTL_HIP(launch_wgrad<T>(w2, st));
        // through the GELU, then d Wfc1 = dpre^T LN_2(x1) and d LN_2(x1) = dpre Wfc1
        if (!gelu_in_b2) ASTL_HIP(launch_gelu<T>(pre, nullptr, dh, rows * Hd, st));
        WgradArgs w1{};
        w1.dout = dh; w1.lddout = Hd; w1.a1 = xn; w1.lda1 = C;
        w1.dw = rep + o_w1; w1.db = rep + o_b1; w1.rep_stride = P; w1.reps = kGradReplicas;
        w1.rows = rows; w1.N = Hd; w1.K = C; w1.prof_id = K_FC_WGRAD;
        w1.scratch = ws + pl.act; w1.scratch_bytes = 2 * pl.act;
        ASTL_HIP(launch_wgrad<T>(w1, st));
        LinearArgs b1{};
        b1.a1 = dh; b1.lda1 = Hd; b1.w = p->w_fc1; b1.w_sn = 1; b1.w_sk = C;
        b1.out = dn; b1.ldout = C; b1.rows = rows; b1.N = C; b1.K = Hd; b1.prof_id = K_FC_DLINEAR;
        ASTL_HIP(launch_linear<T>(b1, st));
        // through LN_2, plus the skip of Eq. 5: dx1
        LnBwdArgs n2{};
        n2.u = x1; n2.dout = dn; n2.res = dy; n2.gamma = p->ln2_w; n2.du = dx1;
        n2.dgamma = rep + o_g2; n2.dbeta = rep + o_be2; n2.rep_stride = P; n2.reps = kGradReplicas;
        n2.rows = rows; n2.C = C; n2.eps = d->eps;
        ASTL_HIP(launch_ln_bwd<T>(n2, st));
    }

    // Eq. 4 backwards: the attention layer on LN_1(x) (recomputed), then LN_1 and the skip
    LnArgs l1{};
    l1.u = x; l1.gamma = p->ln1_w; l1.beta = p->ln1_b; l1.out = xn; l1.rows = rows; l1.C = C; l1.eps = d->eps;
    // (the fused MLP backward's final sum rides in the same launch)
    ASTL_HIP(launch_ln_fwd<T>(l1, st, pl.fused_mlp_bwd ? &mlp_sum : nullptr));
    ASTL_RC(gswa_backward(&d->attn, xn, dx1, p->w_qkv, p->b_qkv, p->w_proj, p->b_proj, p->bias_table, at_saved,
                          dn, g->w_qkv, g->b_qkv, g->w_proj, g->b_proj, g->bias_table, rest, st));
    if (mlp_direct) {
        LnRowsBwdArgs n1{};
        n1.u = (const bf16_t *)x; n1.dout = (const bf16_t *)dn; n1.res = (const bf16_t *)dx1;
        n1.gamma = (const bf16_t *)p->ln1_w; n1.du = (bf16_t *)dx; n1.part = lnpart1;
        n1.rows = rows; n1.C = C; n1.eps = d->eps;
        {
            KernelTimer kt(K_LN_BWD, st);
            ASTL_HIP(launch_ln_rows_bwd(n1, st));
        }
        ReduceJob j1{}, j2{};
        j1.part = lnpart1; j1.nparts = nparts1; j1.n = 2 * C; j1.accumulate = accumulate;
        j1.out.ptr[0] = g->ln1_w; j1.out.begin[0] = 0; j1.out.ptr[1] = g->ln1_b; j1.out.begin[1] = C;
        j1.out.begin[2] = 2 * C; j1.out.nseg = 2;
        j2 = j1;
        j2.part = lnpart2; j2.nparts = nparts2; j2.out.ptr[0] = g->ln2_w; j2.out.ptr[1] = g->ln2_b;
        ASTL_HIP(launch_reduce_pair(j1, j2, st));
        return GSWA_OK;
    }
    LnBwdArgs n1{};
    n1.u = x; n1.dout = dn; n1.res = dx1; n1.gamma = p->ln1_w; n1.du = dx;
    n1.dgamma = rep + o_g1; n1.dbeta = rep + o_be1; n1.rep_stride = P; n1.reps = kGradReplicas;
    n1.rows = rows; n1.C = C; n1.eps = d->eps;
    ASTL_HIP(launch_ln_bwd<T>(n1, st));

    if (own && link && link->may_defer) {
        // LayerNorm-1's gradient copies stay where they are: the next call of the sequence sums them
        link->pending.src = rep + o_g1; link->pending.w = g->ln1_w; link->pending.b = g->ln1_b;
        link->pending.n = C; link->pending.reps = kGradReplicas; link->pending.stride = P;
        link->pending.accumulate = accumulate;
        return GSWA_OK;
    }
    ReplicaSum rs{};
    rs.rep = rep; rs.stride = P; rs.reps = kGradReplicas;
    if (own) {
        rs.out[0] = g->ln1_w; rs.off[0] = o_g1; rs.n[0] = C;
        rs.out[1] = g->ln1_b; rs.off[1] = o_be1; rs.n[1] = C;
        rs.count = 2;
    } else {
        rs.out[0] = g->w_fc1; rs.off[0] = o_w1; rs.n[0] = (long)Hd * C;
        rs.out[1] = g->b_fc1; rs.off[1] = o_b1; rs.n[1] = Hd;
        rs.out[2] = g->w_fc2; rs.off[2] = o_w2; rs.n[2] = (long)C * Hd;
        rs.out[3] = g->b_fc2; rs.off[3] = o_b2; rs.n[3] = C;
        rs.out[4] = g->ln1_w; rs.off[4] = o_g1; rs.n[4] = C;
        rs.out[5] = g->ln1_b; rs.off[5] = o_be1; rs.n[5] = C;
        rs.out[6] = g->ln2_w; rs.off[6] = o_g2; rs.n[6] = C;
        rs.out[7] = g->ln2_b; rs.off[7] = o_be2; rs.n[7] = C;
        rs.count = 8;
    }
    rs.accumulate = accumulate;
    ASTL_HIP(launch_reduce_replicas(rs, st));
    return GSWA_OK;
}

bool params_ok(const astl_params *p)
{
    return p->ln1_w && p->ln1_b && p->w_qkv && p->b_qkv && p->w_proj && p->b_proj && p->bias_table && p->ln2_w &&
           p->ln2_b && p->w_fc1 && p->b_fc1 && p->w_fc2 && p->b_fc2 &&
           aligned16(p->ln1_w, p->ln1_b, p->w_qkv, p->b_qkv, p->w_proj, p->b_proj, p->bias_table, p->ln2_w, p->ln2_b,
                     p->w_fc1, p->b_fc1, p->w_fc2, p->b_fc2);
}

bool grads_ok(const astl_grads *g)
{
    return g->ln1_w && g->ln1_b && g->w_qkv && g->b_qkv && g->w_proj && g->b_proj && g->bias_table && g->ln2_w &&
           g->ln2_b && g->w_fc1 && g->b_fc1 && g->w_fc2 && g->b_fc2 &&
           aligned16(g->ln1_w, g->ln1_b, g->w_qkv, g->b_qkv, g->w_proj, g->b_proj, g->bias_table, g->ln2_w, g->ln2_b,
                     g->w_fc1, g->b_fc1, g->w_fc2, g->b_fc2);
}

int forward_checked(const astl_desc *desc, const void *x, const astl_params *p, void *y, void *saved, void *ws,
                    void *hip_stream, LayerLink *link);
int backward_checked(const astl_desc *desc, const void *x, const void *dy, const astl_params *p, const void *saved,
                     void *dx, const astl_grads *g, void *ws, void *hip_stream, BackLink *link);

} // namespace

} // namespace gswa

using namespace gswa;

extern "C" {

int astl_query_bytes(const astl_desc *desc, size_t *saved_bytes, size_t *fwd_ws_bytes, size_t *bwd_ws_bytes)
{
    Plan pl;
    int rc = make_plan(desc, &pl);
    if (rc != GSWA_OK) return rc;
    if (saved_bytes) *saved_bytes = pl.saved;
    if (fwd_ws_bytes) *fwd_ws_bytes = pl.fwd_ws;
    if (bwd_ws_bytes) *bwd_ws_bytes = pl.bwd_ws;
    return GSWA_OK;
}

int astl_forward(const astl_desc *desc, const void *x, const astl_params *p, void *y, void *saved, void *ws,
                 void *hip_stream)
{
    return forward_checked(desc, x, p, y, saved, ws, hip_stream, nullptr);
}

} // extern "C"

namespace gswa {
namespace {

// astl_forward with the hand-over between the layers of a sequence (link may be null)
int forward_checked(const astl_desc *desc, const void *x, const astl_params *p, void *y, void *saved, void *ws,
                    void *hip_stream, LayerLink *link)
{
    Plan pl;
    int rc = make_plan(desc, &pl);
    if (rc != GSWA_OK) return rc;
    if (!x || !p || !y || !ws || !params_ok(p)) return GSWA_EINVAL;
    if (x == y || (reinterpret_cast<uintptr_t>(ws) & 255) || !aligned16(x, y, saved)) return GSWA_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (desc->attn.dtype == GSWA_F32)
        return forward_t<float>(desc, pl, (const float *)x, p, (float *)y, (char *)saved, (char *)ws, st, link);
    return forward_t<bf16_t>(desc, pl, (const bf16_t *)x, p, (bf16_t *)y, (char *)saved, (char *)ws, st, link);
}

} // namespace
} // namespace gswa

extern "C" {

int astl_backward(const astl_desc *desc, const void *x, const void *dy, const astl_params *p, const void *saved,
                  void *dx, const astl_grads *g, void *ws, void *hip_stream)
{
    return backward_checked(desc, x, dy, p, saved, dx, g, ws, hip_stream, nullptr);
}

} // extern "C"

namespace gswa {
namespace {

int backward_checked(const astl_desc *desc, const void *x, const void *dy, const astl_params *p, const void *saved,
                     void *dx, const astl_grads *g, void *ws, void *hip_stream, BackLink *link)
{
    Plan pl;
    int rc = make_plan(desc, &pl);
    if (rc != GSWA_OK) return rc;
    if (!x || !dy || !p || !saved || !dx || !g || !ws || !params_ok(p) || !grads_ok(g)) return GSWA_EINVAL;
    if (dx == x || dx == dy || dx == saved || (reinterpret_cast<uintptr_t>(ws) & 255)) return GSWA_EINVAL;
    if (!aligned16(x, dy, saved, dx)) return GSWA_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (desc->attn.dtype == GSWA_F32)
        return backward_t<float>(desc, pl, (const float *)x, (const float *)dy, p, (const char *)saved, (float *)dx,
                                 g, (char *)ws, st, link);
    return backward_t<bf16_t>(desc, pl, (const bf16_t *)x, (const bf16_t *)dy, p, (const char *)saved, (bf16_t *)dx,
                              g, (char *)ws, st, link);
}

} // namespace
} // namespace gswa

namespace {

// Sizes of a stack (Sec. "Agile Swin Transformer Block"): S, F, Bw are the largest saved / scratch
// needs over the two kinds of layer (unshifted, shifted), A one [T, C] activation.
struct StackPlan {
    astl_desc even, odd;
    size_t S, F, Bw, A;
    int L, k, nblocks;
    size_t saved, fwd_ws, bwd_ws;
};

int make_stack_plan(const astl_stack_desc *d, StackPlan *sp)
{
    if (!d) return GSWA_EINVAL;
    if (d->n_layers <= 0 || d->checkpoint_every < 0) return GSWA_EINVAL;
    if (d->shift < 0 || d->shift >= d->layer.attn.window) return GSWA_EINVAL;
    sp->even = d->layer; sp->even.attn.shift = 0;
    sp->odd = d->layer; sp->odd.attn.shift = d->shift;
    Plan pe, po;
    int rc = make_plan(&sp->even, &pe);
    if (rc != GSWA_OK) return rc;
    rc = make_plan(&sp->odd, &po);
    if (rc != GSWA_OK) return rc;
    sp->S = pe.saved > po.saved ? pe.saved : po.saved;
    sp->F = pe.fwd_ws > po.fwd_ws ? pe.fwd_ws : po.fwd_ws;
    sp->Bw = pe.bwd_ws > po.bwd_ws ? pe.bwd_ws : po.bwd_ws;
    sp->A = pe.act;
    sp->L = d->n_layers;
    sp->k = d->checkpoint_every > d->n_layers ? d->n_layers : d->checkpoint_every;
    // forward scratch: two activations (inference and recomputed blocks chain through them) and
    // one layer's scratch in its inference form
    sp->fwd_ws = 2 * sp->A + sp->F + sp->S;
    if (sp->k == 0) {
        sp->nblocks = 1;
        sp->saved = (size_t)sp->L * (sp->S + sp->A);
        sp->bwd_ws = 2 * sp->A + sp->Bw;
    } else {
        sp->nblocks = (sp->L + sp->k - 1) / sp->k;
        sp->saved = (size_t)(sp->nblocks > 1 ? sp->nblocks - 1 : 1) * sp->A;
        const size_t lw = sp->F > sp->Bw ? sp->F : sp->Bw;
        sp->bwd_ws = (size_t)sp->k * (sp->S + sp->A) + 2 * sp->A + lw;
    }
    return GSWA_OK;
}

} // namespace

extern "C" {

int astl_stack_query_bytes(const astl_stack_desc *desc, size_t *saved_bytes, size_t *fwd_ws_bytes,
                           size_t *bwd_ws_bytes)
{
    StackPlan sp;
    int rc = make_stack_plan(desc, &sp);
    if (rc != GSWA_OK) return rc;
    if (saved_bytes) *saved_bytes = sp.saved;
    if (fwd_ws_bytes) *fwd_ws_bytes = sp.fwd_ws;
    if (bwd_ws_bytes) *bwd_ws_bytes = sp.bwd_ws;
    return GSWA_OK;
}

int astl_stack_forward(const astl_stack_desc *desc, const void *x, const astl_params *params, void *y,
                       void *saved, void *ws, void *hip_stream)
{
    StackPlan sp;
    int rc = make_stack_plan(desc, &sp);
    if (rc != GSWA_OK) return rc;
    if (!x || !params || !y || !ws || x == y) return GSWA_EINVAL;
    if ((reinterpret_cast<uintptr_t>(ws) & 255) || !aligned16(x, y, saved)) return GSWA_EINVAL;
    for (int l = 0; l < sp.L; ++l)
        if (!params_ok(params + l)) return GSWA_EINVAL;
    char *w = static_cast<char *>(ws), *sv = static_cast<char *>(saved);
    char *abuf[2] = {w, w + sp.A};
    char *layer_ws = w + 2 * sp.A;
    const void *in = x;
    LayerLink link{};
    for (int l = 0; l < sp.L; ++l) {
        const astl_desc *ld = (l & 1) ? &sp.odd : &sp.even;
        void *out, *lsaved = nullptr;
        if (l == sp.L - 1) out = y;
        else if (sv && sp.k == 0) out = sv + (size_t)l * (sp.S + sp.A) + sp.S;       // kept with the layer's state
        else if (sv && (l + 1) % sp.k == 0) out = sv + (size_t)((l + 1) / sp.k - 1) * sp.A; // input of the next block
        else out = abuf[l & 1];
        if (sv && sp.k == 0) lsaved = sv + (size_t)l * (sp.S + sp.A);
        // LN_1 of the next layer comes out of this layer's last kernel where that kernel is the fused one
        link.have_ln1 = link.emitted;
        link.next = l + 1 < sp.L ? params + l + 1 : nullptr;
        rc = forward_checked(ld, in, params + l, out, lsaved, layer_ws, hip_stream, &link);
        if (rc != GSWA_OK) return rc;
        in = out;
    }
    return GSWA_OK;
}

} // extern "C"

namespace {

// Inference of a stack band by band (Sec. "Agile Swin Transformer Block"; every step of Eq. 4-5 stays
// inside a window, so a band of window rows of the shifted frame goes through a whole layer on its own).
struct TiledPlan {
    StackPlan sp;
    int nb;          // window rows per band
    int M, nwi;
    size_t band_act; // bytes of the largest band, [rows, W, C] (256-aligned)
    size_t layer_ws; // scratch of one layer call on the largest band (inference form)
    size_t ws;
};

int make_tiled_plan(const astl_stack_desc *d, int band_windows, TiledPlan *tp)
{
    int rc = make_stack_plan(d, &tp->sp);
    if (rc != GSWA_OK) return rc;
    if (band_windows <= 0) return GSWA_EINVAL;
    tp->M = d->layer.attn.window;
    tp->nwi = d->layer.attn.H / tp->M;
    tp->nb = band_windows < tp->nwi ? band_windows : tp->nwi;
    // window rows of the sub-problems that occur: whole bands (unshifted layers), whole bands plus the
    // row of windows that is computed and dropped (shifted layers), and the band that ends the map
    const int rem = tp->nwi % tp->nb;
    const int kinds[3] = {tp->nb, tp->nb < tp->nwi ? tp->nb + 1 : tp->nb, rem ? rem : tp->nb};
    tp->band_act = tp->layer_ws = 0;
    for (int k = 0; k < 3; ++k)
        for (int odd = 0; odd < 2; ++odd) {
            astl_desc sd = odd ? tp->sp.odd : tp->sp.even;
            sd.attn.B = 1;
            sd.attn.H = kinds[k] * tp->M;
            Plan pl;
            rc = make_plan(&sd, &pl);
            if (rc != GSWA_OK) return rc;
            if (pl.act > tp->band_act) tp->band_act = pl.act;
            if (pl.fwd_ws + pl.saved > tp->layer_ws) tp->layer_ws = pl.fwd_ws + pl.saved;
        }
    tp->ws = 2 * tp->band_act + tp->layer_ws;
    return GSWA_OK;
}

} // namespace

extern "C" {

int astl_stack_tiled_query_bytes(const astl_stack_desc *desc, int32_t band_windows, size_t *ws_bytes)
{
    TiledPlan tp;
    int rc = make_tiled_plan(desc, band_windows, &tp);
    if (rc != GSWA_OK) return rc;
    if (ws_bytes) *ws_bytes = tp.ws;
    return GSWA_OK;
}

int astl_stack_forward_tiled(const astl_stack_desc *desc, const void *x, const astl_params *params, void *y,
                             int32_t band_windows, void *ws, void *hip_stream)
{
    TiledPlan tp;
    int rc = make_tiled_plan(desc, band_windows, &tp);
    if (rc != GSWA_OK) return rc;
    if (!x || !params || !y || !ws || x == y) return GSWA_EINVAL;
    if ((reinterpret_cast<uintptr_t>(ws) & 255) || !aligned16(x, y)) return GSWA_EINVAL;
    for (int l = 0; l < tp.sp.L; ++l)
        if (!params_ok(params + l)) return GSWA_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const gswa_desc &at = desc->layer.attn;
    const int M = tp.M, nwi = tp.nwi, nb = tp.nb, H = at.H;
    const size_t row = (size_t)at.W * at.C * (at.dtype == GSWA_F32 ? 4 : 2); // bytes of one image row
    const size_t img = (size_t)H * row;
    char *xb = static_cast<char *>(ws), *yb = xb + tp.band_act, *layer_ws = yb + tp.band_act;
    auto copy_rows = [&](char *dst, const char *src, int rows) -> hipError_t {
        return rows > 0 ? hipMemcpyAsync(dst, src, (size_t)rows * row, hipMemcpyDeviceToDevice, st) : hipSuccess;
    };
    // Layer 0 reads x and writes y; every later layer works on y in place: a band's result goes to yb first
    // and over the band's own rows afterwards, which no later band of the layer reads (see below).
    const char *cur = static_cast<const char *>(x);
    char *out = static_cast<char *>(y);
    for (int l = 0; l < tp.sp.L; ++l) {
        const astl_desc *ld = (l & 1) ? &tp.sp.odd : &tp.sp.even;
        const int s = ld->attn.shift;
        for (int b = 0; b < at.B; ++b) {
            const char *ib = cur + (size_t)b * img;
            char *ob = out + (size_t)b * img;
            for (int a = 0; a < nwi; a += nb) {
                const int e = a + nb < nwi ? a + nb : nwi; // window rows [a, e) of the shifted frame
                astl_desc sd = *ld;
                sd.attn.B = 1;
                const char *src;
                if (s == 0 || e < nwi) {
                    // Image rows [aM + s, eM + s), contiguous.  As a problem of its own with the same shift,
                    // starting at image row aM: its window rows 0 .. e-a-1 are exactly these windows (no
                    // row of theirs is beyond the last M - s rows, so only the column mask applies, as in
                    // the map); one more row of windows, which wraps within the band, is computed on
                    // whatever lies there and dropped.
                    const int wr = e - a + (s ? 1 : 0);
                    sd.attn.H = wr * M;
                    src = ib + (size_t)a * M * row;
                    if (!aligned16(src)) {
                        ASTL_HIP(copy_rows(xb, src, wr * M));
                        src = xb;
                    }
                    ASTL_RC(forward_checked(&sd, src, params + l, yb, nullptr, layer_ws, hip_stream, nullptr));
                    ASTL_HIP(copy_rows(ob + ((size_t)a * M + s) * row, yb + (size_t)s * row, (e - a) * M));
                } else {
                    // The band that ends the map wraps to the map's first s rows: [rows 0 .. s | rows
                    // aM + s .. H) is an ordinary shifted problem (its last window row is the map's).
                    const int rows = (e - a) * M;
                    sd.attn.H = rows;
                    ASTL_HIP(copy_rows(xb, ib, s));
                    ASTL_HIP(copy_rows(xb + (size_t)s * row, ib + ((size_t)a * M + s) * row, rows - s));
                    ASTL_RC(forward_checked(&sd, xb, params + l, yb, nullptr, layer_ws, hip_stream, nullptr));
                    ASTL_HIP(copy_rows(ob, yb, s));
                    ASTL_HIP(copy_rows(ob + ((size_t)a * M + s) * row, yb + (size_t)s * row, rows - s));
                }
            }
        }
        cur = out;
    }
    return GSWA_OK;
}

int astl_stack_backward(const astl_stack_desc *desc, const void *x, const void *dy, const astl_params *params,
                        const void *saved, void *dx, const astl_grads *grads, void *ws, void *hip_stream)
{
    StackPlan sp;
    int rc = make_stack_plan(desc, &sp);
    if (rc != GSWA_OK) return rc;
    if (!x || !dy || !params || !saved || !dx || !grads || !ws) return GSWA_EINVAL;
    if (dx == x || dx == dy || dx == saved) return GSWA_EINVAL;
    if ((reinterpret_cast<uintptr_t>(ws) & 255) || !aligned16(x, dy, saved, dx)) return GSWA_EINVAL;
    for (int l = 0; l < sp.L; ++l)
        if (!params_ok(params + l) || !grads_ok(grads + l)) return GSWA_EINVAL;
    char *w = static_cast<char *>(ws);
    const char *sv = static_cast<const char *>(saved);
    const size_t slot = sp.S + sp.A;
    // gradient of layer l's input goes to gbuf[l & 1] (to dx for layer 0)
    auto grad_in = [&](int l, char *const *gbuf) -> const void * { return l == sp.L - 1 ? dy : gbuf[(l + 1) & 1]; };
    auto grad_out = [&](int l, char *const *gbuf) -> void * { return l == 0 ? dx : gbuf[l & 1]; };
    if (sp.k == 0) {
        char *gbuf[2] = {w, w + sp.A};
        char *layer_ws = w + 2 * sp.A;
        BackLink link{};
        for (int l = sp.L - 1; l >= 0; --l) {
            const astl_desc *ld = (l & 1) ? &sp.odd : &sp.even;
            const void *xin = l == 0 ? x : sv + (size_t)(l - 1) * slot + sp.S;
            link.may_defer = l > 0; // (layer l - 1 runs next on the same scratch, before anything else touches it)
            rc = backward_checked(ld, xin, grad_in(l, gbuf), params + l, sv + (size_t)l * slot, grad_out(l, gbuf),
                                  grads + l, layer_ws, hip_stream, &link);
            if (rc != GSWA_OK) return rc;
        }
        return GSWA_OK;
    }
    // checkpointed: per block, forward again into the scratch, then backward through the block
    char *region = w;                                  // k slots of [layer state | layer output]
    char *gbuf[2] = {w + (size_t)sp.k * slot, w + (size_t)sp.k * slot + sp.A};
    char *layer_ws = w + (size_t)sp.k * slot + 2 * sp.A;
    for (int b = sp.nblocks - 1; b >= 0; --b) {
        const int l0 = b * sp.k, l1 = (l0 + sp.k < sp.L) ? l0 + sp.k : sp.L;
        const void *block_in = b == 0 ? x : sv + (size_t)(b - 1) * sp.A;
        const void *in = block_in;
        LayerLink link{};
        for (int l = l0; l < l1; ++l) {
            const astl_desc *ld = (l & 1) ? &sp.odd : &sp.even;
            char *st = region + (size_t)(l - l0) * slot;
            link.have_ln1 = link.emitted;
            link.next = l + 1 < l1 ? params + l + 1 : nullptr;
            rc = forward_checked(ld, in, params + l, st + sp.S, st, layer_ws, hip_stream, &link);
            if (rc != GSWA_OK) return rc;
            in = st + sp.S;
        }
        BackLink blink{};
        for (int l = l1 - 1; l >= l0; --l) {
            const astl_desc *ld = (l & 1) ? &sp.odd : &sp.even;
            const void *xin = l == l0 ? block_in : region + (size_t)(l - l0 - 1) * slot + sp.S;
            blink.may_defer = l > l0; // (not across blocks: the forward pass of the next block uses the scratch)
            rc = backward_checked(ld, xin, grad_in(l, gbuf), params + l, region + (size_t)(l - l0) * slot,
                                  grad_out(l, gbuf), grads + l, layer_ws, hip_stream, &blink);
            if (rc != GSWA_OK) return rc;
        }
    }
    return GSWA_OK;
}

} // extern "C"
