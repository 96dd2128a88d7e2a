// Staged GSWA kernels: projection GEMMs, weight-gradient GEMMs and the per-(window, head)
// attention core, all in fp32 arithmetic on the vector ALUs with LDS tiles.  They read and
// write token-major buffers in the tokens' own (unshifted) order; the cyclic shift and the
// window partition exist only as the index map window_token().
#include "staged_kernels.h"
#include "fused.h"
#include "mfma.h"
#include <cmath>

namespace gswa {

static constexpr int kThreads = 256;
static constexpr size_t kLdsMax = 160 * 1024;

// ---------------------------------------------------------------------------------------
// out = (a1 + a2) * w^T-ish + bias + add      64 x 64 output tile, 4 x 4 per thread
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(kThreads) void linear_kernel(LinearArgs p)
{
    constexpr int TM = 64, TN = 64, TK = 16;
    __shared__ float As[TK][TM + 1];
    __shared__ float Ws[TK][TN + 1];
    const T *a1 = static_cast<const T *>(p.a1);
    const T *a2 = static_cast<const T *>(p.a2);
    const T *w = static_cast<const T *>(p.w);
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const long row0 = (long)blockIdx.x * TM;
    const int n0 = blockIdx.y * TN;
    const bool k_contig = (p.w_sk == 1);

    float acc[4][4] = {};
    for (int k0 = 0; k0 < p.K; k0 += TK) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int e = tid + i * kThreads;
            const int r = e >> 4, kk = e & 15;
            const long row = row0 + r;
            float v = 0.f;
            if (row < p.rows && k0 + kk < p.K) {
                v = to_f32(a1[row * p.lda1 + k0 + kk]);
                if (a2) v += to_f32(a2[row * p.lda2 + k0 + kk]);
            }
            As[kk][r] = v;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int e = tid + i * kThreads;
            const int nn = k_contig ? (e >> 4) : (e & 63);
            const int kk = k_contig ? (e & 15) : (e >> 6);
            float v = 0.f;
            if (n0 + nn < p.N && k0 + kk < p.K) v = to_f32(w[(long)(n0 + nn) * p.w_sn + (long)(k0 + kk) * p.w_sk]);
            Ws[kk][nn] = v;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < TK; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Ws[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }

    const T *bias = static_cast<const T *>(p.bias);
    const T *add = static_cast<const T *>(p.add);
    T *out = static_cast<T *>(p.out);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const long row = row0 + ty * 4 + i;
        if (row >= p.rows) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n >= p.N) continue;
            float v = acc[i][j];
            if (bias) v += to_f32(bias[n]);
            if (add) v += to_f32(add[row * p.ldadd + n]);
            from_f32(out[row * p.ldout + n], v);
        }
    }
}

// ---------------------------------------------------------------------------------------
// The same linear map on the matrix cores (bf16, even K and row strides): a workgroup takes up to
// NTC 16-column tiles of the output (blockIdx.y) and turns their weights into B-operand fragments
// in LDS once; every wave then walks over 16-row tiles: the rows are its A operand (k-slots = 8
// consecutive input channels, read as dwords, all K steps in flight together), one 16x16x32 MFMA
// per (output tile, K step).  KSM bounds the K steps (K <= 32 * KSM).
// ---------------------------------------------------------------------------------------
// One launch can serve two independent maps: the column chunks of the second follow those of the
// first along blockIdx.y (chunks_a of them; the second map is absent when gridDim.y == chunks_a).
// Body: `wl` = LDS for NTC*KS fragments; the workgroup (nthreads threads) is number `blk` of `nblk`
// that share the rows of the column chunk starting at ncol0.
// four consecutive dwords at dword alignment (the hardware reads them in one instruction)
struct __attribute__((aligned(4))) dwords4 {
    uint32_t v[4];
};

template <int KSM, int NTC>
__device__ __forceinline__ void linear_mfma_body(const LinearArgs &p, int KS, int ncol0, uint4 *wl, int nthreads,
                                                 long blk, long nblk)
{
    const uint16_t *w = static_cast<const uint16_t *>(p.w);
    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, q = lane >> 4, wave = tid >> 6;
    const int nwaves = nthreads >> 6;
    for (int i = tid; i < NTC * KS * 64; i += nthreads) {
        const int f = i >> 6, ln = i & 63;
        const int nt = f / KS, ks = f - nt * KS;
        const int n = ncol0 + 16 * nt + (ln & 15), k0 = 32 * ks + 8 * (ln >> 4);
        if (p.w_sk == 1 && !(p.w_sn & 1)) {
            // the lane's 8 input channels are contiguous: dword reads (K is even, so is w_sn)
            const uint32_t *w32 = reinterpret_cast<const uint32_t *>(w + (long)n * p.w_sn);
            uint32_t v[4];
#pragma unroll
            for (int dw = 0; dw < 4; ++dw) v[dw] = (n < p.N && k0 + 2 * dw < p.K) ? w32[(k0 >> 1) + dw] : 0u;
            wl[i] = make_uint4(v[0], v[1], v[2], v[3]);
        } else {
            uint32_t v[8];
#pragma unroll
            for (int s8 = 0; s8 < 8; ++s8)
                v[s8] = (n < p.N && k0 + s8 < p.K) ? (uint32_t)w[(long)n * p.w_sn + (long)(k0 + s8) * p.w_sk] : 0u;
            wl[i] = make_uint4(v[0] | v[1] << 16, v[2] | v[3] << 16, v[4] | v[5] << 16, v[6] | v[7] << 16);
        }
    }
    __syncthreads();

    const uint32_t *a1 = static_cast<const uint32_t *>(p.a1);
    const uint32_t *a2 = static_cast<const uint32_t *>(p.a2);
    const uint16_t *bias = static_cast<const uint16_t *>(p.bias);
    const uint16_t *add = static_cast<const uint16_t *>(p.add);
    uint16_t *out = static_cast<uint16_t *>(p.out);
    const long ntile = (p.rows + 15) / 16;
    for (long tile = blk * nwaves + wave; tile < ntile; tile += nblk * nwaves) {
        const long row = 16 * tile + l16;
        uint4 af[KSM];
#pragma unroll
        for (int ks = 0; ks < KSM; ++ks) {
            uint32_t v[4] = {0u, 0u, 0u, 0u};
            const int k0 = 32 * ks + 8 * q;
            if (ks < KS && row < p.rows) {
                if (k0 + 8 <= p.K) { // the lane's 8 channels as one 16-byte read (dword aligned)
                    const dwords4 u = *reinterpret_cast<const dwords4 *>(a1 + ((row * p.lda1 + k0) >> 1));
#pragma unroll
                    for (int dw = 0; dw < 4; ++dw) v[dw] = u.v[dw];
                    if (a2) {
                        const dwords4 u2 = *reinterpret_cast<const dwords4 *>(a2 + ((row * p.lda2 + k0) >> 1));
#pragma unroll
                        for (int dw = 0; dw < 4; ++dw)
                            v[dw] = pack_bf16x2(bf16_lo(v[dw]) + bf16_lo(u2.v[dw]), bf16_hi(v[dw]) + bf16_hi(u2.v[dw]));
                    }
                } else {
#pragma unroll
                    for (int dw = 0; dw < 4; ++dw) {
                        const int k = k0 + 2 * dw;
                        if (k < p.K) {
                            uint32_t u = a1[(row * p.lda1 + k) >> 1];
                            if (a2) {
                                const uint32_t u2 = a2[(row * p.lda2 + k) >> 1];
                                u = pack_bf16x2(bf16_lo(u) + bf16_lo(u2), bf16_hi(u) + bf16_hi(u2));
                            }
                            v[dw] = u;
                        }
                    }
                }
            }
            af[ks] = make_uint4(v[0], v[1], v[2], v[3]);
        }
        f32x4 acc[NTC];
#pragma unroll
        for (int nt = 0; nt < NTC; ++nt) acc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KSM; ++ks)
            if (ks < KS) {
#pragma unroll
                for (int nt = 0; nt < NTC; ++nt) acc[nt] = mma32(af[ks], wl[(nt * KS + ks) * 64 + lane], acc[nt]);
            }
        // result: column l16 = output feature, rows 4q + j = rows of the tile
#pragma unroll
        for (int nt = 0; nt < NTC; ++nt) {
            const int n = ncol0 + 16 * nt + l16;
            if (n >= p.N) continue;
            const float b = bias ? __uint_as_float((uint32_t)bias[n] << 16) : 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const long r = 16 * tile + 4 * q + j;
                if (r >= p.rows) continue;
                float v = acc[nt][j] + b;
                if (add) v += __uint_as_float((uint32_t)add[r * p.ldadd + n] << 16);
                out[r * p.ldout + n] = f32_to_bf16_bits(v);
            }
        }
    }
}

// blockIdx.y beyond the chunks of both maps: zero fill of `zero` (nothing to do with the maps; it
// saves the launch a separate fill kernel would take).
template <int KSM, int NTC>
__global__ __launch_bounds__(kThreads) void linear_mfma_kernel(LinearArgs pa, LinearArgs pb, int ksa, int ksb,
                                                              int chunks_a, int chunks_all, float *zero, long nzero)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lsm[];
    if ((int)blockIdx.y >= chunks_all) {
        for (long i = (long)blockIdx.x * kThreads + threadIdx.x; i < nzero; i += (long)gridDim.x * kThreads) zero[i] = 0.f;
        return;
    }
    const bool second = (int)blockIdx.y >= chunks_a;
    linear_mfma_body<KSM, NTC>(second ? pb : pa, second ? ksb : ksa,
                               ((int)blockIdx.y - (second ? chunks_a : 0)) * (16 * NTC),
                               reinterpret_cast<uint4 *>(lsm), kThreads, blockIdx.x, gridDim.x);
}

// The same map for wide layers whose whole weight matrix fits LDS as fragments (NT * KS <= 152 KB):
// one workgroup per compute unit (1024 threads; 512 where the rows' own fragments need the
// registers) builds all of them once, and a wave reads the rows
// of its 16-row tile ONCE for all output columns (the chunked kernel above reads them once per 64
// columns and rebuilds fragments per workgroup and chunk).
template <int KSM, int NTHREADS, bool LN>
__global__ __launch_bounds__(NTHREADS) void linear_mfma_wide_kernel(LinearArgs p, int KS, int NT)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lsm[];
    uint4 *wl = reinterpret_cast<uint4 *>(lsm);
    const uint16_t *w = static_cast<const uint16_t *>(p.w);
    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, q = lane >> 4, wave = tid >> 6;
    constexpr int nthreads = NTHREADS, nwaves = NTHREADS / 64;
    for (int i = tid; i < NT * KS * 64; i += nthreads) {
        const int f = i >> 6, ln = i & 63;
        const int nt = f / KS, ks = f - nt * KS;
        const int n = 16 * nt + (ln & 15), k0 = 32 * ks + 8 * (ln >> 4);
        if (p.w_sk == 1 && !(p.w_sn & 1) && !(reinterpret_cast<uintptr_t>(w) & 3)) {
            // the lane's 8 input channels are contiguous: dword reads (K is even, so is w_sn)
            const uint32_t *w32 = reinterpret_cast<const uint32_t *>(w + (long)n * p.w_sn);
            uint32_t v[4];
#pragma unroll
            for (int dw = 0; dw < 4; ++dw) v[dw] = (n < p.N && k0 + 2 * dw < p.K) ? w32[(k0 >> 1) + dw] : 0u;
            wl[i] = make_uint4(v[0], v[1], v[2], v[3]);
        } else {
            uint32_t v[8];
#pragma unroll
            for (int s8 = 0; s8 < 8; ++s8)
                v[s8] = (n < p.N && k0 + s8 < p.K) ? (uint32_t)w[(long)n * p.w_sn + (long)(k0 + s8) * p.w_sk] : 0u;
            wl[i] = make_uint4(v[0] | v[1] << 16, v[2] | v[3] << 16, v[4] | v[5] << 16, v[6] | v[7] << 16);
        }
    }
    // the linear bias as fp32 behind the fragments
    float *bias_l = reinterpret_cast<float *>(lsm + (size_t)NT * KS * 1024);
    const uint16_t *bias = static_cast<const uint16_t *>(p.bias);
    for (int n = tid; n < 16 * NT; n += nthreads) bias_l[n] = (bias && n < p.N) ? __uint_as_float((uint32_t)bias[n] << 16) : 0.f;
    // scale and shift of the LayerNorm of the operand, as (gamma, beta) pairs per channel, zero beyond K
    float2 *ln_gb = reinterpret_cast<float2 *>(bias_l + 16 * NT);
    if (LN) {
        const uint16_t *lg = static_cast<const uint16_t *>(p.ln_gamma), *lb = static_cast<const uint16_t *>(p.ln_beta);
        for (int k = tid; k < 32 * KS; k += nthreads)
            ln_gb[k] = k < p.K ? make_float2(__uint_as_float((uint32_t)lg[k] << 16), __uint_as_float((uint32_t)lb[k] << 16))
                               : make_float2(0.f, 0.f);
    }
    __syncthreads();

    const uint32_t *a1 = static_cast<const uint32_t *>(p.a1);
    const uint32_t *a2 = static_cast<const uint32_t *>(p.a2);
    const uint16_t *add = static_cast<const uint16_t *>(p.add);
    uint16_t *out = static_cast<uint16_t *>(p.out);
    uint16_t *pre_out = static_cast<uint16_t *>(p.pre_out);
    const uint16_t *aux = static_cast<const uint16_t *>(p.aux);
    const bool out_even = !(reinterpret_cast<uintptr_t>(p.out) & 3) && !(reinterpret_cast<uintptr_t>(p.pre_out) & 3);
    // What the stores add (the skip tensor) or take the GELU's derivative of: four features of a row as two dword
    // reads where its pitch is even and its base dword-aligned.
    const bool ep_add = add != nullptr;
    const uint16_t *ep_src = ep_add ? add : (p.act == kActGeluGrad ? aux : nullptr);
    const long ep_ld = ep_add ? p.ldadd : p.ldaux;
    if (ep_src && ((ep_ld & 1) || (reinterpret_cast<uintptr_t>(ep_src) & 3))) ep_src = nullptr;
    const long ntile = (p.rows + 15) / 16;
    for (long tile = (long)blockIdx.x * nwaves + wave; tile < ntile; tile += (long)gridDim.x * nwaves) {
        const long row = 16 * tile + l16;
        uint32_t af[KSM][4];
#pragma unroll
        for (int ks = 0; ks < KSM; ++ks) {
            uint32_t (&v)[4] = af[ks];
            v[0] = v[1] = v[2] = v[3] = 0u;
            const int k0 = 32 * ks + 8 * q;
            if (ks < KS && row < p.rows) {
                if (k0 + 8 <= p.K) { // the lane's 8 channels as one 16-byte read (dword aligned)
                    const dwords4 u = *reinterpret_cast<const dwords4 *>(a1 + ((row * p.lda1 + k0) >> 1));
#pragma unroll
                    for (int dw = 0; dw < 4; ++dw) v[dw] = u.v[dw];
                    if (a2) {
                        const dwords4 u2 = *reinterpret_cast<const dwords4 *>(a2 + ((row * p.lda2 + k0) >> 1));
#pragma unroll
                        for (int dw = 0; dw < 4; ++dw)
                            v[dw] = pack_bf16x2(bf16_lo(v[dw]) + bf16_lo(u2.v[dw]), bf16_hi(v[dw]) + bf16_hi(u2.v[dw]));
                    }
                } else {
#pragma unroll
                    for (int dw = 0; dw < 4; ++dw) {
                        const int k = k0 + 2 * dw;
                        if (k < p.K) {
                            uint32_t u = a1[(row * p.lda1 + k) >> 1];
                            if (a2) {
                                const uint32_t u2 = a2[(row * p.lda2 + k) >> 1];
                                u = pack_bf16x2(bf16_lo(u) + bf16_lo(u2), bf16_hi(u) + bf16_hi(u2));
                            }
                            v[dw] = u;
                        }
                    }
                }
            }
        }
        if (LN) {
            // LayerNorm of the row just read (Eq. 4-5): the row is spread over the four lanes that share l16;
            // mean, then the sum of squared distances from it, as the separate LayerNorm kernel computes them
            float sum = 0.f;
#pragma unroll
            for (int ks = 0; ks < KSM; ++ks)
#pragma unroll
                for (int dw = 0; dw < 4; ++dw) sum += bf16_lo(af[ks][dw]) + bf16_hi(af[ks][dw]); // (zero beyond K)
            const float mean = qgroup_sum(sum) / (float)p.K;
            // (each pass unpacks the row again: the unpacked values of a whole row would take twice its registers)
#pragma unroll
            for (int ks = 0; ks < KSM; ++ks)
#pragma unroll
                for (int dw = 0; dw < 4; ++dw) asm volatile("" : "+v"(af[ks][dw]));
            float dev = 0.f;
#pragma unroll
            for (int ks = 0; ks < KSM; ++ks)
#pragma unroll
                for (int dw = 0; dw < 4; ++dw)
                    if (ks < KS && 32 * ks + 8 * q + 2 * dw < p.K) {
                        const float d0 = bf16_lo(af[ks][dw]) - mean, d1 = bf16_hi(af[ks][dw]) - mean;
                        dev += d0 * d0 + d1 * d1;
                    }
            const float rstd = rsqrtf(qgroup_sum(dev) / (float)p.K + p.ln_eps);
#pragma unroll
            for (int ks = 0; ks < KSM; ++ks)
#pragma unroll
                for (int dw = 0; dw < 4; ++dw) asm volatile("" : "+v"(af[ks][dw]));
            uint32_t *so = static_cast<uint32_t *>(p.sum_out), *lo = static_cast<uint32_t *>(p.ln_out);
#pragma unroll
            for (int ks = 0; ks < KSM; ++ks)
                if (ks < KS) {
                    const int k0 = 32 * ks + 8 * q;
                    const long at = (row * p.lda1 + k0) >> 1;
                    const bool live = row < p.rows;
                    if (so && live) {
                        if (k0 + 8 <= p.K) {
                            dwords4 u;
#pragma unroll
                            for (int dw = 0; dw < 4; ++dw) u.v[dw] = af[ks][dw];
                            *reinterpret_cast<dwords4 *>(so + at) = u;
                        } else {
#pragma unroll
                            for (int dw = 0; dw < 4; ++dw)
                                if (k0 + 2 * dw < p.K) so[at + dw] = af[ks][dw];
                        }
                    }
#pragma unroll
                    for (int dw = 0; dw < 4; ++dw) {
                        const float2 g0 = ln_gb[k0 + 2 * dw], g1 = ln_gb[k0 + 2 * dw + 1];
                        af[ks][dw] = pack_bf16x2((bf16_lo(af[ks][dw]) - mean) * rstd * g0.x + g0.y,
                                                 (bf16_hi(af[ks][dw]) - mean) * rstd * g1.x + g1.y);
                    }
                    if (lo && live) {
                        if (k0 + 8 <= p.K) {
                            dwords4 u;
#pragma unroll
                            for (int dw = 0; dw < 4; ++dw) u.v[dw] = af[ks][dw];
                            *reinterpret_cast<dwords4 *>(lo + at) = u;
                        } else {
#pragma unroll
                            for (int dw = 0; dw < 4; ++dw)
                                if (k0 + 2 * dw < p.K) lo[at + dw] = af[ks][dw];
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0); // (one slice's scale and shift in registers at a time)
                }
        }
        int opq = lane; // (opaque, so that the fragment reads are not hoisted out of the tile loop)
        asm volatile("" : "+v"(opq));
        // (output tiles per group: four, or two where 16 waves share the registers)
        constexpr int GRP = NTHREADS >= 1024 ? 2 : 4;
        for (int nt0 = 0; nt0 < NT; nt0 += GRP) {
            // What the stores of this group of tiles add or multiply by (the skip tensor, the GELU's argument): four
            // consecutive features of this lane's row per tile, fetched as two dwords each BEFORE the products, so
            // that their latency passes under the matrix-core work instead of in front of every store.
            uint32_t epv[GRP][2]; // (one of the two: a map with both takes the two-byte reads below for the second)
#pragma unroll
            for (int j = 0; j < GRP; ++j) {
                const int n0 = 16 * (nt0 + j) + 4 * q;
                epv[j][0] = epv[j][1] = 0u;
                if (ep_src && row < p.rows && nt0 + j < NT && n0 + 4 <= p.N) {
                    const uint32_t *ap = reinterpret_cast<const uint32_t *>(ep_src + row * ep_ld + n0);
                    epv[j][0] = ap[0];
                    epv[j][1] = ap[1];
                }
            }
            f32x4 acc[GRP];
#pragma unroll
            for (int j = 0; j < GRP; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KSM; ++ks)
                if (ks < KS) {
#pragma unroll
                    for (int j = 0; j < GRP; ++j)   // weights as the A operand: the transposed product
                        if (nt0 + j < NT) acc[j] = mma32(wl[((nt0 + j) * KS + ks) * 64 + opq],
                                                      make_uint4(af[ks][0], af[ks][1], af[ks][2], af[ks][3]), acc[j]);
                }
            // result: column l16 = row of the tile, rows 4q + r4 = four consecutive output features
            if (row >= p.rows) continue;
#pragma unroll
            for (int j = 0; j < GRP; ++j) {
                const int n0 = 16 * (nt0 + j) + 4 * q;
                if (nt0 + j >= NT || n0 >= p.N) continue;
                const bool whole = ep_src && n0 + 4 <= p.N;
                float v[4];
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const int n = n0 + r4;
                    v[r4] = acc[j][r4];
                    if (n < p.N) {
                        if (bias) v[r4] += bias_l[n];
                        if (add) {
                            if (whole && ep_add) v[r4] += (r4 & 1) ? bf16_hi(epv[j][r4 >> 1]) : bf16_lo(epv[j][r4 >> 1]);
                            else v[r4] += __uint_as_float((uint32_t)add[row * p.ldadd + n] << 16);
                        }
                    }
                }
                uint16_t *dst = out + row * p.ldout + n0;
                const bool pair_ok = n0 + 4 <= p.N && out_even && !((row * p.ldout + n0) & 1);
                if (p.act) {
                    // the activation of the value as a separate pass would read it back: rounded to bf16
                    float r[4];
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) r[r4] = __uint_as_float((uint32_t)f32_to_bf16_bits(v[r4]) << 16);
                    if (p.act == kActGelu) {
                        if (pre_out) {
                            uint16_t *pd = pre_out + row * p.ldout + n0;
                            if (pair_ok) {
                                reinterpret_cast<uint32_t *>(pd)[0] = pack_bf16x2(r[0], r[1]);
                                reinterpret_cast<uint32_t *>(pd)[1] = pack_bf16x2(r[2], r[3]);
                            } else {
#pragma unroll
                                for (int r4 = 0; r4 < 4; ++r4)
                                    if (n0 + r4 < p.N) pd[r4] = f32_to_bf16_bits(r[r4]);
                            }
                        }
#pragma unroll
                        for (int r4 = 0; r4 < 4; ++r4) {
                            float Phi, phi;
                            gauss(r[r4], Phi, phi);
                            v[r4] = r[r4] * Phi;
                        }
                    } else {
                        float tv[4];
                        if (whole && !ep_add) {
                            tv[0] = bf16_lo(epv[j][0]); tv[1] = bf16_hi(epv[j][0]);
                            tv[2] = bf16_lo(epv[j][1]); tv[3] = bf16_hi(epv[j][1]);
                        } else {
                            const uint16_t *ap = aux + row * p.ldaux + n0;
#pragma unroll
                            for (int r4 = 0; r4 < 4; ++r4)
                                tv[r4] = n0 + r4 < p.N ? __uint_as_float((uint32_t)ap[r4] << 16) : 0.f;
                        }
#pragma unroll
                        for (int r4 = 0; r4 < 4; ++r4) {
                            const float t = tv[r4];
                            float Phi, phi;
                            gauss(t, Phi, phi);
                            v[r4] = r[r4] * fmaf(t, phi, Phi);
                        }
                    }
                }
                if (pair_ok) {
                    uint32_t *d32 = reinterpret_cast<uint32_t *>(dst);
                    d32[0] = pack_bf16x2(v[0], v[1]);
                    d32[1] = pack_bf16x2(v[2], v[3]);
                } else {
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4)
                        if (n0 + r4 < p.N) dst[r4] = f32_to_bf16_bits(v[r4]);
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// out[t, n] = sum_k a1[t, k] w(n, k) (+ bias[n]) (+ add[t, n]) for maps whose weight matrix does not fit LDS
// (up to 576 output columns, any K): the weights, repacked by a launch of their own into matrix-core fragments
// in the order they are used, are streamed through LDS in units of four K = 32 steps (double buffered, loads
// that write LDS directly, one barrier per unit); a wave owns 16 rows, reads them 16 bytes per lane and step,
// one unit ahead, and keeps the output tiles of a block of 192 columns in registers.  With more columns the
// blocks follow one another (the rows are read once per block: from L2 after the first).  The rows of the
// fragments are ordered so that a lane's results of tiles 2p and 2p + 1 are the 8 consecutive columns
// 32 p + 8 q + 0..7 of the block: 16-byte stores.
// ---------------------------------------------------------------------------------------
struct LinStream {
    static constexpr int NT = 12, HU = 4, NWV = 16;
    static constexpr int NMAX = 3 * 16 * NT; // up to three blocks of 192 output columns, one after the other
    static constexpr int FR_UNIT = NT * HU, UNIT_BYTES = FR_UNIT * 1024;
    static constexpr int FPW = (FR_UNIT + NWV - 1) / NWV;
    static constexpr size_t LDS_BYTES = 2 * (size_t)UNIT_BYTES + NMAX * sizeof(float);
    static int units(int K) { return ((K + 31) / 32 + HU - 1) / HU; }
    static int blocks(int N) { return (N + 16 * NT - 1) / (16 * NT); }
    static size_t pack_bytes(int N, int K) { return (size_t)blocks(N) * units(K) * UNIT_BYTES + NMAX * sizeof(float); }
};

// pack: [column block][unit][step of the unit][tile] fragments, then the bias as fp32 (zero beyond N)
__global__ __launch_bounds__(256) void linear_stream_pack_kernel(LinearArgs p, int nu, int nb)
{
    using L = LinStream;
    const uint16_t *w = static_cast<const uint16_t *>(p.w);
    uint16_t *d16 = static_cast<uint16_t *>(p.scratch);
    const int total = nb * nu * L::FR_UNIT * 512;
    for (int e = blockIdx.x * 256 + threadIdx.x; e < total; e += gridDim.x * 256) {
        const int j = e & 7, l = (e >> 3) & 63, fr = e >> 9;
        const int gu = fr / L::FR_UNIT, f = fr - gu * L::FR_UNIT;
        const int blk = gu / nu, u = gu - blk * nu;
        const int hs = f / L::NT, ct = f - hs * L::NT;
        const int m = l & 15, lq = l >> 4;
        const int n = 16 * L::NT * blk + 32 * (ct >> 1) + 8 * (m >> 2) + 4 * (ct & 1) + (m & 3);
        const int k = 32 * (L::HU * u + hs) + 8 * lq + j;
        d16[e] = (n < p.N && k < p.K) ? w[(long)n * p.w_sn + (long)k * p.w_sk] : (uint16_t)0;
    }
    float *bl = reinterpret_cast<float *>(static_cast<uint8_t *>(p.scratch) + (size_t)nb * nu * L::UNIT_BYTES);
    const uint16_t *bias = static_cast<const uint16_t *>(p.bias);
    for (int n = blockIdx.x * 256 + threadIdx.x; n < L::NMAX; n += gridDim.x * 256)
        bl[n] = (bias && n < p.N) ? __uint_as_float((uint32_t)bias[n] << 16) : 0.f;
}

__global__ __launch_bounds__(64 * LinStream::NWV) void linear_stream_kernel(LinearArgs p, int nu, int nb)
{
    using L = LinStream;
    constexpr int NT = L::NT, HU = L::HU;
    typedef uint32_t u32q __attribute__((ext_vector_type(4)));
    typedef u32q u32q_a4 __attribute__((aligned(4)));
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const uint8_t *pack = static_cast<const uint8_t *>(p.scratch);
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, tok = lane & 15, q = lane >> 4;
    const uint32_t *a32 = static_cast<const uint32_t *>(p.a1);
    const int tu = nu * nb; // units of a round: every column block takes all K
    int lane_r = lane;
    auto stream_unit = [&](int gu, int slot) {
        int ln = lane_r;
        asm volatile("" : "+v"(ln));
        const uint8_t *src = pack + (size_t)gu * L::UNIT_BYTES + 16 * ln;
        uint8_t *dst = lds + (size_t)slot * L::UNIT_BYTES;
#pragma unroll 1
        for (int k = 0; k < L::FPW; ++k) {
            const int f = k * L::NWV + wv;
            if (f < L::FR_UNIT) lds_dma16(src + (size_t)f * 1024, dst + (size_t)f * 1024);
        }
    };
    // the lane's pieces of a unit's four steps: columns 32 s + 8 q + 0..7 of its row (a piece that would reach
    // beyond the row is read 8 columns before the row's end instead and put right by tidy(); K is a multiple of 4)
    auto load_unit = [&](long row, int u, u32q (&b)[HU]) {
        int qq = q;
        asm volatile("" : "+v"(qq));
#pragma unroll
        for (int hs = 0; hs < HU; ++hs) {
            int k0 = 32 * (HU * u + hs) + 8 * qq;
            if (k0 + 8 > p.K) k0 = p.K - 8;
            b[hs] = *reinterpret_cast<const u32q_a4 *>(a32 + ((row * p.lda1 + k0) >> 1));
        }
    };
    auto tidy = [&](u32q v, int k0) {
        const bool whole = k0 + 8 <= p.K, half = k0 + 4 == p.K;
        return make_uint4(whole ? v.x : half ? v.z : 0u, whole ? v.y : half ? v.w : 0u, whole ? v.z : 0u, whole ? v.w : 0u);
    };

    const long ntiles = (p.rows + 15) / 16;
    const long stride = (long)gridDim.x * L::NWV;
    const int rounds = (int)((ntiles + stride - 1) / stride);
    long tile = (long)blockIdx.x * L::NWV + wv;

    stream_unit(0, 0);
    float *bias_l = reinterpret_cast<float *>(lds + 2 * L::UNIT_BYTES);
    for (int i = tid; i < L::NMAX; i += 64 * L::NWV)
        bias_l[i] = reinterpret_cast<const float *>(pack + (size_t)tu * L::UNIT_BYTES)[i];
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();

    const uint16_t *add = static_cast<const uint16_t *>(p.add);
    uint16_t *out = static_cast<uint16_t *>(p.out);
    int slot = 0;
    for (int round = 0; round < rounds; ++round, tile += stride) {
        const bool more = round + 1 < rounds;
        const long t = tile * 16 + tok;
        const bool ok = t < p.rows;
        const long tc = ok ? t : p.rows - 1;
        uint32_t lds0 = 0;
        asm volatile("" : "+v"(lds0));
        lane_r = lane;
        asm volatile("" : "+v"(lane_r));
        f32x4 acc[NT];
        u32q b[HU], bn[HU];
        load_unit(tc, 0, b);
        int u = 0, blk = 0;
        for (int gu = 0; gu < tu; ++gu) {
            if (gu + 1 < tu) stream_unit(gu + 1, slot ^ 1);
            else if (more) stream_unit(0, slot ^ 1);
            // the pieces of the next unit: of the same rows again when the next column block begins
            const int un = u + 1 < nu ? u + 1 : 0;
            if (gu + 1 < tu) load_unit(tc, un, bn);
            if (u == 0) {
#pragma unroll
                for (int ct = 0; ct < NT; ++ct) acc[ct] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
            const uint4 *wu = reinterpret_cast<const uint4 *>(lds + lds0 + (size_t)slot * L::UNIT_BYTES);
            int qq = q;
            asm volatile("" : "+v"(qq));
#pragma unroll
            for (int hs = 0; hs < HU; ++hs) {
                const uint4 bb = tidy(b[hs], 32 * (HU * u + hs) + 8 * qq);
#pragma unroll
                for (int ct = 0; ct < NT; ++ct) acc[ct] = mma32(wu[(hs * NT + ct) * 64 + lane_r], bb, acc[ct]);
            }
            if (u == nu - 1) {
                // the block's columns: tiles 2p and 2p + 1 hold the lane's columns 32 p + 8 q + 0..3 and + 4..7
#pragma unroll
                for (int pz = 0; pz < NT / 2; ++pz) {
                    const int n0 = 16 * NT * blk + 32 * pz + 8 * qq;
                    if (!ok || n0 >= p.N) continue;
                    const f32x4 lo = acc[2 * pz], hi = acc[2 * pz + 1];
                    float v[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        v[i] += bias_l[n0 + i];
                        if (add && n0 + i < p.N) v[i] += __uint_as_float((uint32_t)add[t * p.ldadd + n0 + i] << 16);
                    }
                    uint16_t *dst = out + t * p.ldout + n0;
                    const bool even = !((t * p.ldout + n0) & 1) && !(reinterpret_cast<uintptr_t>(out) & 3);
                    if (n0 + 8 <= p.N && even) {
                        u32q o = {pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7])};
                        *reinterpret_cast<u32q_a4 *>(dst) = o;
                    } else {
#pragma unroll
                        for (int i = 0; i < 8; ++i)
                            if (n0 + i < p.N) dst[i] = f32_to_bf16_bits(v[i]);
                    }
                }
            }
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
            slot ^= 1;
#pragma unroll
            for (int hs = 0; hs < HU; ++hs) b[hs] = bn[hs];
            if (++u == nu) { u = 0; ++blk; }
        }
    }
}

// Maps the streaming kernel takes: bf16 (checked by the caller), no second addend, activation or LayerNorm, at most
// 576 output columns, dword-aligned rows, scratch for the pack - and a shape the kernel that keeps a whole weight
// matrix in LDS does not take (a reduction longer than 384, or more than 192 columns).
static bool linear_stream_ok(const LinearArgs &a)
{
    if (!a.scratch || a.a2 || a.act || a.ln_gamma) return false;
    if (a.N > LinStream::NMAX || a.N < 64 || a.K < 32 || a.K % 4 || a.rows < 4096) return false;
    if (a.K <= 384 && a.N <= 16 * LinStream::NT) return false;
    if ((a.lda1 & 1) || (reinterpret_cast<uintptr_t>(a.a1) & 3) || (reinterpret_cast<uintptr_t>(a.scratch) & 15)) return false;
    return a.scratch_bytes >= LinStream::pack_bytes(a.N, a.K);
}

static hipError_t launch_linear_stream(const LinearArgs &a, hipStream_t s)
{
    using L = LinStream;
    const int nu = L::units(a.K), nb = L::blocks(a.N);
    KernelTimer kt(a.prof_id, s);
    hipLaunchKernelGGL(linear_stream_pack_kernel, dim3(128), dim3(256), 0, s, a, nu, nb);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (hipError_t ea = allow_dynamic_lds(reinterpret_cast<const void *>(linear_stream_kernel), L::LDS_BYTES); ea != hipSuccess) return ea;
    const long tiles = (a.rows + 15) / 16;
    long blocks = (tiles + L::NWV - 1) / L::NWV;
    if (blocks > device_cu_count()) blocks = device_cu_count();
    hipLaunchKernelGGL(linear_stream_kernel, dim3((unsigned)blocks), dim3(64 * L::NWV), L::LDS_BYTES, s, a, nu, nb);
    return hipGetLastError();
}

// the wide kernel serves maps with more than 64 output columns whose fragments fit LDS
static bool linear_wide_ok(const LinearArgs &a)
{
    const int nt = (a.N + 15) / 16, ks = (a.K + 31) / 32;
    // (fragments, the fp32 bias and the LayerNorm's pairs within the 160 KB of a compute unit)
    const long lds = (long)nt * ks * 1024 + (long)nt * 64 + (long)ks * 256;
    return a.N > 64 && ks <= 12 && (long)nt * ks <= 152 && lds <= 160 * 1024 && a.rows >= 4096;
}

template <int KSM, int NTHREADS, bool LN> static hipError_t launch_linear_wide_ln(const LinearArgs &a, hipStream_t s)
{
    const int nt = (a.N + 15) / 16, ks = (a.K + 31) / 32;
    // fragments | fp32 bias | (gamma, beta) of the operand's LayerNorm
    const size_t lds = (size_t)nt * ks * 1024 + (size_t)nt * 16 * sizeof(float) + (a.ln_gamma ? (size_t)ks * 32 * sizeof(float2) : 0);
    auto kern = linear_mfma_wide_kernel<KSM, NTHREADS, LN>;
    if (hipError_t ea = allow_dynamic_lds(reinterpret_cast<const void *>(kern), lds); ea != hipSuccess) return ea;
    const long ntile = (a.rows + 15) / 16;
    long blocks = (ntile + NTHREADS / 64 - 1) / (NTHREADS / 64);
    if (blocks > device_cu_count()) blocks = device_cu_count();
    KernelTimer kt(a.prof_id, s);
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(NTHREADS), lds, s, a, ks, nt);
    return hipGetLastError();
}

template <int KSM, int NTHREADS> static hipError_t launch_linear_wide_t(const LinearArgs &a, hipStream_t s)
{
    return a.ln_gamma ? launch_linear_wide_ln<KSM, NTHREADS, true>(a, s) : launch_linear_wide_ln<KSM, NTHREADS, false>(a, s);
}

// true when the matrix-core kernel can serve the call (the dword reads need even offsets)
static bool linear_mfma_ok(const LinearArgs &a)
{
    const bool even = !(a.K & 1) && !(a.lda1 & 1) && !(reinterpret_cast<uintptr_t>(a.a1) & 3) &&
                      (!a.a2 || (!(a.lda2 & 1) && !(reinterpret_cast<uintptr_t>(a.a2) & 3)));
    const bool w_ok = a.w_sk != 1 || (a.w_sn & 1) || !(reinterpret_cast<uintptr_t>(a.w) & 3);
    return even && w_ok && a.K <= 32 * 18;
}

// `b` may be null: one map only
template <int KSM, int NTC>
static hipError_t launch_linear_mfma_t(const LinearArgs &a, const LinearArgs *b, int prof_id, float *zero,
                                       long nzero, hipStream_t s)
{
    const int nta = (a.N + 15) / 16, ksa = (a.K + 31) / 32;
    const int ntb = b ? (b->N + 15) / 16 : 0, ksb = b ? (b->K + 31) / 32 : 0;
    const unsigned chunks_a = (unsigned)((nta + NTC - 1) / NTC), chunks = chunks_a + (unsigned)((ntb + NTC - 1) / NTC);
    const size_t lds = (size_t)NTC * (ksa > ksb ? ksa : ksb) * 1024;
    auto kern = linear_mfma_kernel<KSM, NTC>;
    if (hipError_t ea = allow_dynamic_lds(reinterpret_cast<const void *>(kern), lds); ea != hipSuccess) return ea;
    const long rows = b && b->rows > a.rows ? b->rows : a.rows;
    const long ntile = (rows + 15) / 16;
    // every workgroup builds its chunk's weight fragments first: with several chunks the rows are
    // spread over fewer, longer-running workgroups
    long blocks = (ntile + 3) / 4, cap = (chunks <= 2 ? 4L : 2L) * device_cu_count() / chunks;
    if (cap < 1) cap = 1;
    if (blocks > cap) blocks = cap;
    KernelTimer kt(prof_id, s);
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks, chunks + (zero && nzero > 0 ? 1 : 0)), dim3(kThreads), lds, s, a,
                       b ? *b : a, ksa, ksb, (int)chunks_a, (int)chunks, zero, nzero);
    return hipGetLastError();
}

static hipError_t launch_linear_mfma(const LinearArgs &a, const LinearArgs *b, int prof_id, float *zero, long nzero,
                                     hipStream_t s)
{
    int nt = (a.N + 15) / 16, ks = (a.K + 31) / 32;
    if (b) {
        const int ntb = (b->N + 15) / 16, ksb = (b->K + 31) / 32;
        nt = ntb > nt ? ntb : nt;
        ks = ksb > ks ? ksb : ks;
    }
    if (ks <= 2) return nt <= 4 ? launch_linear_mfma_t<2, 4>(a, b, prof_id, zero, nzero, s)
                                : launch_linear_mfma_t<2, 8>(a, b, prof_id, zero, nzero, s);
    if (ks <= 6) return launch_linear_mfma_t<6, 4>(a, b, prof_id, zero, nzero, s);
    return launch_linear_mfma_t<18, 4>(a, b, prof_id, zero, nzero, s);
}

bool linear_act_supported(const LinearArgs &a) { return a.rows > 0 && a.N > 0 && linear_mfma_ok(a) && linear_wide_ok(a); }
// (the LayerNorm's outputs are written as dwords at the operand's own offsets)
bool linear_ln_supported(const LinearArgs &a)
{
    return linear_act_supported(a) && !(reinterpret_cast<uintptr_t>(a.sum_out) & 3) && !(reinterpret_cast<uintptr_t>(a.ln_out) & 3);
}

template <typename T> hipError_t launch_linear(const LinearArgs &a, hipStream_t s)
{
    if (a.rows <= 0 || a.N <= 0) return hipSuccess;
    if constexpr (sizeof(T) == 2) {
        if (linear_mfma_ok(a) && linear_wide_ok(a))
            return (a.K + 31) / 32 <= 6 ? launch_linear_wide_t<6, 1024>(a, s) : launch_linear_wide_t<12, 512>(a, s);
        if (a.act || a.ln_gamma) return hipErrorInvalidValue; // (callers ask linear_act_supported first)
        if (linear_stream_ok(a)) return launch_linear_stream(a, s);
        if (linear_mfma_ok(a)) return launch_linear_mfma(a, nullptr, a.prof_id, nullptr, 0, s);
    }
    if (a.act || a.ln_gamma) return hipErrorInvalidValue;
    dim3 grid((unsigned)((a.rows + 63) / 64), (unsigned)((a.N + 63) / 64));
    KernelTimer kt(a.prof_id, s);
    hipLaunchKernelGGL(linear_kernel<T>, grid, dim3(kThreads), 0, s, a);
    return hipGetLastError();
}
template hipError_t launch_linear<float>(const LinearArgs &, hipStream_t);
template hipError_t launch_linear<bf16_t>(const LinearArgs &, hipStream_t);

template <typename T>
hipError_t launch_linear_pair(const LinearArgs &a, const LinearArgs &b, float *zero, size_t nzero, hipStream_t s)
{
    if constexpr (sizeof(T) == 2) {
        if (a.rows > 0 && a.N > 0 && b.rows > 0 && b.N > 0 && linear_mfma_ok(a) && linear_mfma_ok(b)) {
            if (linear_stream_ok(a)) {
                // the first map on the streaming kernel; the second on the kernel that keeps its whole weight
                // matrix in LDS and reads every row once where that one takes it, else with the fill
                hipError_t e = launch_linear_stream(a, s);
                if (e != hipSuccess) return e;
                if (!(linear_wide_ok(b) && !b.act && !b.ln_gamma))
                    return launch_linear_mfma(b, nullptr, K_LINEAR_PAIR, zero, (long)nzero, s);
                if (zero && nzero > 0) {
                    ZeroList z{};
                    z.p[0] = zero; z.n[0] = nzero; z.count = 1;
                    if (e = launch_fill_zero(z, s); e != hipSuccess) return e;
                }
                return launch_linear<T>(b, s);
            }
            return launch_linear_mfma(a, &b, K_LINEAR_PAIR, zero, (long)nzero, s);
        }
    }
    hipError_t e = hipSuccess;
    if (zero && nzero > 0) {
        ZeroList z{};
        z.p[0] = zero; z.n[0] = nzero; z.count = 1;
        e = launch_fill_zero(z, s);
        if (e != hipSuccess) return e;
    }
    e = launch_linear<T>(a, s);
    return e != hipSuccess ? e : launch_linear<T>(b, s);
}
template hipError_t launch_linear_pair<float>(const LinearArgs &, const LinearArgs &, float *, size_t, hipStream_t);
template hipError_t launch_linear_pair<bf16_t>(const LinearArgs &, const LinearArgs &, float *, size_t, hipStream_t);

// ---------------------------------------------------------------------------------------
// dw[n,k] += sum_t dout[t,n] (a1+a2)[t,k] ; db[n] += sum_t dout[t,n]
// 64 x 64 tile of dw per block, the token range split over blockIdx.z, fp32 atomics at the end
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(kThreads) void wgrad_kernel(WgradArgs p, long rows_per_split)
{
    constexpr int TT = 16;
    __shared__ float Ds[TT][64 + 1];
    __shared__ float As[TT][64 + 1];
    const T *dout = static_cast<const T *>(p.dout);
    const T *a1 = static_cast<const T *>(p.a1);
    const T *a2 = static_cast<const T *>(p.a2);
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int n0 = blockIdx.x * 64, k0 = blockIdx.y * 64;
    const long t_begin = (long)blockIdx.z * rows_per_split;
    long t_end = t_begin + rows_per_split;
    if (t_end > p.rows) t_end = p.rows;

    float *dw = p.dw + (long)(blockIdx.z % p.reps) * p.rep_stride;
    float *db = p.db ? p.db + (long)(blockIdx.z % p.reps) * p.rep_stride : nullptr;
    float acc[4][4] = {};
    float bacc[4] = {};
    for (long t0 = t_begin; t0 < t_end; t0 += TT) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int e = tid + i * kThreads;
            const int tt = e >> 6, c = e & 63;
            const long t = t0 + tt;
            float dv = 0.f, av = 0.f;
            if (t < t_end) {
                if (n0 + c < p.N) dv = to_f32(dout[t * p.lddout + n0 + c]);
                if (k0 + c < p.K) {
                    av = to_f32(a1[t * p.lda1 + k0 + c]);
                    if (a2) av += to_f32(a2[t * p.lda2 + k0 + c]);
                }
            }
            Ds[tt][c] = dv;
            As[tt][c] = av;
        }
        __syncthreads();
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = Ds[tt][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = As[tt][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                bacc[i] += a[i];
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
            }
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int n = n0 + ty * 4 + i;
        if (n >= p.N) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int k = k0 + tx * 4 + j;
            if (k < p.K) atomicAdd(&dw[(long)n * p.K + k], acc[i][j]);
        }
        if (db && blockIdx.y == 0 && tx == 0) atomicAdd(&db[n], bacc[i]);
    }
}

// ---------------------------------------------------------------------------------------
// The same reduction on the matrix cores (bf16): dw = dout^T (a1 + a2) contracts over tokens, so
// tokens are the k-slots of both operands.  Rows that allow dword-aligned 16-byte reads are fetched
// along the features and turned by a product with a 0/1 selector (see below); otherwise a lane
// gathers 8 consecutive tokens of one column two bytes at a time.
// A workgroup of 16 waves owns a 64 x 64 tile of dw and a range of tokens: wave (nw, tq) owns
// the 16 rows n = 16*nw.. of the tile (all four 16-column tiles) and every fourth 32-token step
// starting at tq; the bias sums ride in a fifth product with a column of ones.  The four token
// quarters are summed through LDS: one atomic add per output and workgroup.
// ---------------------------------------------------------------------------------------
constexpr int kWgradThreads = 1024;
// One launch can serve two independent reductions: the splits of the second follow those of the
// first along blockIdx.z (splits_a of them; no second one when gridDim.z == splits_a).
// Workgroups beyond the splits (blockIdx.z >= splits_all) serve an independent small linear map
// (out features <= 64, K <= 64) that reads the same d(q|k|v) rows: dF of the group.
__global__ __launch_bounds__(kWgradThreads) void wgrad_mfma_kernel(WgradArgs pa, WgradArgs pb, long rps_a,
                                                                   long rps_b, int splits_a, int splits_all,
                                                                   LinearArgs lin, int lin_ks)
{
    __shared__ __attribute__((aligned(16))) float red[3][4][20][64]; // [token quarter - 1][nw][accumulator][lane]
    if ((int)blockIdx.z >= splits_all) {
        const long blk = ((long)(blockIdx.z - splits_all) * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x;
        const long nblk = (long)(gridDim.z - splits_all) * gridDim.y * gridDim.x;
        linear_mfma_body<2, 4>(lin, lin_ks, 0, reinterpret_cast<uint4 *>(&red[0][0][0][0]), kWgradThreads, blk, nblk);
        return;
    }
    const bool second = (int)blockIdx.z >= splits_a;
    const WgradArgs &p = second ? pb : pa;
    const long rows_per_split = second ? rps_b : rps_a;
    const int split = (int)blockIdx.z - (second ? splits_a : 0);
    const uint16_t *dout = static_cast<const uint16_t *>(p.dout);
    const uint16_t *a1 = static_cast<const uint16_t *>(p.a1);
    const uint16_t *a2 = static_cast<const uint16_t *>(p.a2);
    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, q = lane >> 4;
    const int wave = tid >> 6, nw = wave & 3, tq = wave >> 2;
    const int n0 = blockIdx.x * 64 + 16 * nw, k0 = blockIdx.y * 64;
    const long t_begin = (long)split * rows_per_split;
    long t_end = t_begin + rows_per_split;
    if (t_end > p.rows) t_end = p.rows;
    const int n = n0 + l16;
    const bool n_ok = n < p.N;
    const uint32_t one = 0x3f80u;
    const uint4 ones = l16 == 0 ? make_uint4(one | one << 16, one | one << 16, one | one << 16, one | one << 16)
                                : make_uint4(0u, 0u, 0u, 0u);

    f32x4 acc[4], bacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kt = 0; kt < 4; ++kt) acc[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
    // Rows whose elements can be fetched as dword-aligned 16-byte pieces take the route below:
    // a lane reads 8 consecutive FEATURES of one token (the natural, coalesced direction), and the
    // matrix cores turn the tile: with the loaded tile as the A operand (m = token, k = feature)
    // and a 0/1 selector as B, the product is the tile in result layout (column = feature, rows =
    // tokens 4q..4q+3), which packed to bf16 IS the K = 16 operand that reduces over tokens.
    const bool rows16 = !((p.lddout | p.lda1 | (a2 ? p.lda2 : 0)) & 1) && !(reinterpret_cast<uintptr_t>(dout) & 3) &&
                        !(reinterpret_cast<uintptr_t>(a1) & 3) && !(a2 && (reinterpret_cast<uintptr_t>(a2) & 3));
    if (rows16 && n0 < p.N && k0 < p.K) {
        const int nb = blockIdx.x * 64 + 32 * (nw >> 1);     // the 32-feature block of dout this wave's 16 rows lie in
        // selector for the 16-feature half `h` of a 32-feature block: 1.0 in the k-slot of feature 16h + l16
        auto selector = [&](int h) {
            const int j = 16 * h + l16 - 8 * q;
            const uint32_t one1 = (j & 1) ? 0x3f800000u : 0x00003f80u;
            const int dw = (j >= 0 && j < 8) ? (j >> 1) : -1;
            return make_uint4(dw == 0 ? one1 : 0u, dw == 1 ? one1 : 0u, dw == 2 ? one1 : 0u, dw == 3 ? one1 : 0u);
        };
        const uint4 sel0 = selector(0), sel1 = selector(1);
        const uint2 ones16 = l16 == 0 ? make_uint2(0x3f803f80u, 0x3f803f80u) : make_uint2(0u, 0u);
        // 8 features of row t starting at feature f (zero beyond `width` and beyond the rows)
        auto load8 = [&](const uint16_t *base, long ld, long t, int f, int width) {
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (t < t_end && f < width) {
                if (f + 8 <= width) {
                    const dwords4 u = *reinterpret_cast<const dwords4 *>(base + t * ld + f);
                    v = make_uint4(u.v[0], u.v[1], u.v[2], u.v[3]);
                } else {
                    uint32_t e[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) e[j] = f + j < width ? (uint32_t)base[t * ld + f + j] : 0u;
                    v = make_uint4(e[0] | e[1] << 16, e[2] | e[3] << 16, e[4] | e[5] << 16, e[6] | e[7] << 16);
                }
            }
            return v;
        };
        auto add8 = [](uint4 x, uint4 y) {
            return make_uint4(pack_bf16x2(bf16_lo(x.x) + bf16_lo(y.x), bf16_hi(x.x) + bf16_hi(y.x)),
                              pack_bf16x2(bf16_lo(x.y) + bf16_lo(y.y), bf16_hi(x.y) + bf16_hi(y.y)),
                              pack_bf16x2(bf16_lo(x.z) + bf16_lo(y.z), bf16_hi(x.z) + bf16_hi(y.z)),
                              pack_bf16x2(bf16_lo(x.w) + bf16_lo(y.w), bf16_hi(x.w) + bf16_hi(y.w)));
        };
        const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};
        auto fetch = [&](long t0, uint4 &d, uint4 (&a)[2]) {
            const long t = t0 + l16;
            d = load8(dout, p.lddout, t, nb + 8 * q, p.N);
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                a[b] = load8(a1, p.lda1, t, k0 + 32 * b + 8 * q, p.K);
                if (a2) a[b] = add8(a[b], load8(a2, p.lda2, t, k0 + 32 * b + 8 * q, p.K));
            }
        };
        long t0 = t_begin + 16 * tq;
        uint4 dcur, acur[2];
        fetch(t0, dcur, acur);
        for (; t0 < t_end; t0 += 64) {
            uint4 dnext, anext[2];
            fetch(t0 + 64, dnext, anext);      // (all zero past the split's rows)
            // turn the tiles: 16 tokens x this wave's 16 rows of dout, 16 tokens x 64 columns of a
            const uint2 dT = pack_bf16x4(mma32(dcur, (nw & 1) ? sel1 : sel0, zero4));
#pragma unroll
            for (int kt = 0; kt < 4; ++kt) {
                if (k0 + 16 * kt >= p.K) continue; // uniform
                const uint2 aT = pack_bf16x4(mma32(acur[kt >> 1], (kt & 1) ? sel1 : sel0, zero4));
                acc[kt] = mma16(dT, aT, acc[kt]);
            }
            bacc = mma16(dT, ones16, bacc);
            dcur = dnext; acur[0] = anext[0]; acur[1] = anext[1];
        }
    } else
    if (n0 < p.N && k0 < p.K)
        for (long t0 = t_begin + 32 * tq; t0 < t_end; t0 += 128) {
            uint32_t av[8], bv[4][8];
#pragma unroll
            for (int s8 = 0; s8 < 8; ++s8) {
                const long t = t0 + 8 * q + s8;
                const bool t_ok = t < t_end;
                av[s8] = (t_ok && n_ok) ? (uint32_t)dout[t * p.lddout + n] : 0u;
#pragma unroll
                for (int kt = 0; kt < 4; ++kt) {
                    const int k = k0 + 16 * kt + l16;
                    uint32_t u = 0u;
                    if (t_ok && k < p.K) {
                        u = a1[t * p.lda1 + k];
                        if (a2) u = f32_to_bf16_bits(__uint_as_float(u << 16) + __uint_as_float((uint32_t)a2[t * p.lda2 + k] << 16));
                    }
                    bv[kt][s8] = u;
                }
            }
            const uint4 af = make_uint4(av[0] | av[1] << 16, av[2] | av[3] << 16, av[4] | av[5] << 16, av[6] | av[7] << 16);
#pragma unroll
            for (int kt = 0; kt < 4; ++kt) {
                if (k0 + 16 * kt >= p.K) continue; // uniform
                const uint4 bf = make_uint4(bv[kt][0] | bv[kt][1] << 16, bv[kt][2] | bv[kt][3] << 16,
                                            bv[kt][4] | bv[kt][5] << 16, bv[kt][6] | bv[kt][7] << 16);
                acc[kt] = mma32(af, bf, acc[kt]);
            }
            bacc = mma32(af, ones, bacc);
        }
    if (tq > 0) {
#pragma unroll
        for (int kt = 0; kt < 4; ++kt)
#pragma unroll
            for (int j = 0; j < 4; ++j) red[tq - 1][nw][4 * kt + j][lane] = acc[kt][j];
#pragma unroll
        for (int j = 0; j < 4; ++j) red[tq - 1][nw][16 + j][lane] = bacc[j];
    }
    __syncthreads();
    if (tq > 0 || n0 >= p.N || k0 >= p.K) return;
#pragma unroll
    for (int r = 0; r < 3; ++r) {
#pragma unroll
        for (int kt = 0; kt < 4; ++kt)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[kt][j] += red[r][nw][4 * kt + j][lane];
#pragma unroll
        for (int j = 0; j < 4; ++j) bacc[j] += red[r][nw][16 + j][lane];
    }
    // result tiles: column l16 = k, rows 4q + j = n
    float *dw = p.dw + (long)(split % p.reps) * p.rep_stride;
    float *db = p.db ? p.db + (long)(split % p.reps) * p.rep_stride : nullptr;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int nn = n0 + 4 * q + j;
        if (nn >= p.N) continue;
#pragma unroll
        for (int kt = 0; kt < 4; ++kt) {
            const int k = k0 + 16 * kt + l16;
            if (k < p.K) atomicAdd(&dw[(long)nn * p.K + k], acc[kt][j]);
        }
        if (db && blockIdx.y == 0 && l16 == 0) atomicAdd(&db[nn], bacc[j]);
    }
}

// token rows per split (a multiple of 128) and the number of splits for one reduction
static void wgrad_splits(const WgradArgs &a, long *rps, long *splits)
{
    const long tn = (a.N + 63) / 64, tk = (a.K + 63) / 64;
    // A wave waits for the loads of one 32-token step at a time (about 1.5 us under load) and every
    // split adds N*K atomic adds (about 60 per ns for the whole chip): the split count balances
    // rows / (128 * splits) steps per wave against splits * N * K adds.
    long s_ = (long)sqrt(700.0 * (double)a.rows / ((double)a.N * a.K));
    const long max_splits = (a.rows + 127) / 128;
    if (s_ > max_splits) s_ = max_splits;
    const long resident = 2L * device_cu_count() / (tn * tk); // all workgroups on the chip at once
    if (s_ > resident && resident >= 8) s_ = resident;
    if (a.exclusive && s_ > a.reps) s_ = a.reps; // every split then adds into a copy of its own
    if (s_ < 1) s_ = 1;
    long r = (a.rows + s_ - 1) / s_;
    r = (r + 127) / 128 * 128;
    *rps = r;
    *splits = (a.rows + r - 1) / r;
}

// `b` may be null: one reduction only; `lin` may be null: no linear map riding along
static hipError_t launch_wgrad_mfma(const WgradArgs &a, const WgradArgs *b, const LinearArgs *lin, hipStream_t s)
{
    long rps_a = 0, sp_a = 0, rps_b = 128, sp_b = 0;
    wgrad_splits(a, &rps_a, &sp_a);
    unsigned tn = (a.N + 63) / 64, tk = (a.K + 63) / 64;
    if (b) {
        wgrad_splits(*b, &rps_b, &sp_b);
        const unsigned tnb = (b->N + 63) / 64, tkb = (b->K + 63) / 64;
        tn = tnb > tn ? tnb : tn;
        tk = tkb > tk ? tkb : tk;
    }
    // the linear map gets about one workgroup (16 waves, a 16-row tile each) per 64 row tiles
    long lin_z = 0;
    if (lin) {
        const long want = ((lin->rows + 15) / 16 + 63) / 64;
        lin_z = (want + tn * tk - 1) / (tn * tk);
        if (lin_z < 1) lin_z = 1;
    }
    dim3 grid(tn, tk, (unsigned)(sp_a + sp_b + lin_z));
    LinearArgs none{};
    KernelTimer kt(a.prof_id, s);
    hipLaunchKernelGGL(wgrad_mfma_kernel, grid, dim3(kWgradThreads), 0, s, a, b ? *b : a, rps_a, rps_b, (int)sp_a,
                       (int)(sp_a + sp_b), lin ? *lin : none, lin ? (lin->K + 31) / 32 : 0);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Weight gradients of wide fully connected layers (Eq. 5 at C = 180, hidden 360): the 64 x 64 tiling
// above reads every row once per tile row and tile column and pays N*K memory-side atomic adds per
// split.  Here the gradient [N][K | bias] is cut into blocks of NB x KB entries (two for these layers)
// and a workgroup of eight waves owns a whole block for a share of the rows, which it streams once, 128
// tokens per pass: both operands are moved into [channel][token] LDS rows by selector MFMAs, wave w
// accumulates the row tiles of row group w % 4 against one half of the column tiles in registers over
// all its passes.  The workgroups of a share store into one partial array [N*K | N]; the library's
// fixed-order sum adds the arrays onto copy 0 of the gradient (no atomics: run-to-run identical).
// ---------------------------------------------------------------------------------------
template <int NB, int KB> struct WgradStreamCfg {
    static constexpr int NT = (NB + 15) / 16, KT = KB / 16 + 1;     // 16-row tiles of dout^T; of [a | 1]^T (column KB: ones)
    static constexpr int KSN = (NB + 31) / 32, KSK = (KB + 31) / 32; // K=32 operand steps along a row of dout, of a
    static constexpr int NWV = 8, TOK = 16 * NWV;
    static constexpr int RW = (NT + 3) / 4, CW = (KT + 1) / 2;
    static constexpr int LW = TOK + 8;                               // pitch (bf16) of the [channel][128 tokens] rows
    static constexpr size_t LDS_BYTES = (size_t)16 * (NT + KT) * LW * 2;
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
    static_assert(NB % 2 == 0 && KB % 2 == 0, "dword-granular row reads");
};

// block (n0, k0) of the gradient: dout and a point at the block's first column; `bias`: this block also
// carries the bias sums (column KB of [a | 1])
// One of the (one or two) gradients of a launch: its operands, its shape and where its [d w | d b] lies inside a
// share's partial array.
struct WgradStreamJob {
    const bf16_t *dout; long lddout;
    const bf16_t *a; long lda;
    int N, K;
    long part_off;
};

// blockIdx.y < blocks0: a block of the first gradient, otherwise of the second (both over the same rows);
// `per` = floats of a share's partial array (both gradients).
template <int NB, int KB>
__global__ __launch_bounds__(512, 1) void wgrad_stream_kernel(long rows, WgradStreamJob j0, int blocks0, WgradStreamJob j1,
                                                              float *__restrict__ part, long per)
{
    const bool second = (int)blockIdx.y >= blocks0;
    const bf16_t *__restrict__ dout = second ? j1.dout : j0.dout;
    const bf16_t *__restrict__ a = second ? j1.a : j0.a;
    const long lddout = second ? j1.lddout : j0.lddout, lda = second ? j1.lda : j0.lda;
    const int N = second ? j1.N : j0.N, K = second ? j1.K : j0.K;
    const int by = (int)blockIdx.y - (second ? blocks0 : 0);
    using P = WgradStreamCfg<NB, KB>;
    constexpr int NT = P::NT, KT = P::KT, KSN = P::KSN, KSK = P::KSK, LW = P::LW, RW = P::RW, CW = P::CW;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    uint16_t *gbuf = reinterpret_cast<uint16_t *>(lds);  // dout^T rows [feature n][token]
    uint16_t *abuf = gbuf + 16 * NT * LW;                 // [a | 1]^T rows [channel k][token]
    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, q = lane >> 4;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int rg = wv & 3, ch = wv >> 2;
    const int nkb = K / KB;                                // blocks along K; block index = nb * nkb + kb
    const int n0 = (by / nkb) * NB, k0 = (by % nkb) * KB;
    const bool bias = k0 == 0;
    dout += n0;
    a += k0;
    const uint2 ones2 = make_uint2(0x3f803f80u, 0x3f803f80u);
    const f32x4 zero4 = f32x4{0.f, 0.f, 0.f, 0.f};

    f32x4 acc[RW][CW];
#pragma unroll
    for (int r = 0; r < RW; ++r)
#pragma unroll
        for (int c = 0; c < CW; ++c) acc[r][c] = zero4;

    const long ntile = (rows + P::TOK - 1) / P::TOK;
    for (long tile = blockIdx.x; tile < ntile; tile += gridDim.x) {
        // this lane's token of the pass as operands: features 32 ks + 8 q .. + 7 of its row (a valid row is
        // read unconditionally so that the dwords merge into wide loads; rows past the end count as zero)
        const long tok = tile * P::TOK + 16 * wv + l16;
        const bool ok = tok < rows;
        const uint32_t *grow = reinterpret_cast<const uint32_t *>(dout + (ok ? tok : 0) * lddout);
        const uint32_t *arow = reinterpret_cast<const uint32_t *>(a + (ok ? tok : 0) * lda);
        uint4 gf[KSN], af[KSK];
#pragma unroll
        for (int ks = 0; ks < KSN; ++ks) {
            uint32_t v[4];
#pragma unroll
            for (int dw = 0; dw < 4; ++dw) {
                const int c = 32 * ks + 8 * q + 2 * dw;
                v[dw] = c < NB ? grow[c >> 1] : 0u;
            }
            gf[ks] = ok ? make_uint4(v[0], v[1], v[2], v[3]) : make_uint4(0u, 0u, 0u, 0u);
        }
#pragma unroll
        for (int ks = 0; ks < KSK; ++ks) {
            uint32_t v[4];
#pragma unroll
            for (int dw = 0; dw < 4; ++dw) {
                const int c = 32 * ks + 8 * q + 2 * dw;
                v[dw] = c < KB ? arow[c >> 1] : 0u;
            }
            af[ks] = ok ? make_uint4(v[0], v[1], v[2], v[3]) : make_uint4(0u, 0u, 0u, 0u);
        }
        __syncthreads(); // the previous pass's rows are consumed
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const f32x4 tN = mma32(gf[nt >> 1], select_slot(16 * nt + l16, 32 * (nt >> 1) + 8 * q), zero4);
            *reinterpret_cast<uint2 *>(gbuf + (16 * nt + l16) * LW + 16 * wv + 4 * q) = pack_bf16x4(tN);
        }
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) {
            f32x4 tN = zero4;
            if ((kt >> 1) < KSK) tN = mma32(af[(kt >> 1) < KSK ? (kt >> 1) : 0], select_slot(16 * kt + l16, 32 * (kt >> 1) + 8 * q), zero4);
            uint2 pk = pack_bf16x4(tN);
            if (16 * kt + l16 == KB) pk = bias ? ones2 : make_uint2(0u, 0u); // (rows past the end have dout = 0)
            *reinterpret_cast<uint2 *>(abuf + (16 * kt + l16) * LW + 16 * wv + 4 * q) = pk;
        }
        __syncthreads();
#pragma unroll
        for (int kp = 0; kp < P::TOK / 32; ++kp) {
            uint4 afr[RW];
#pragma unroll
            for (int r = 0; r < RW; ++r) {
                const int nt = rg * RW + r;
                const uint16_t *ar = gbuf + (16 * (nt < NT ? nt : 0) + l16) * LW + 32 * kp + 8 * q;
                afr[r] = cat(*reinterpret_cast<const uint2 *>(ar), *reinterpret_cast<const uint2 *>(ar + 4));
            }
#pragma unroll
            for (int c = 0; c < CW; ++c) {
                const int kt = ch * CW + c;
                const uint16_t *br = abuf + (16 * (kt < KT ? kt : 0) + l16) * LW + 32 * kp + 8 * q;
                const uint4 bf = cat(*reinterpret_cast<const uint2 *>(br), *reinterpret_cast<const uint2 *>(br + 4));
#pragma unroll
                for (int r = 0; r < RW; ++r) acc[r][c] = mma32(afr[r], bf, acc[r][c]);
            }
        }
    }
    float *mine = part + (size_t)blockIdx.x * per + (second ? j1.part_off : j0.part_off); // the share's [d w | d b]
#pragma unroll
    for (int r = 0; r < RW; ++r) {
        const int nt = rg * RW + r;
        if (nt < NT) {
#pragma unroll
            for (int c = 0; c < CW; ++c) {
                const int kt = ch * CW + c;
                const int col = 16 * kt + l16;
                if (kt < KT) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int n = 16 * nt + 4 * q + j;
                        if (n < NB) {
                            if (col < KB) mine[(size_t)(n0 + n) * K + k0 + col] = acc[r][c][j];
                            else if (col == KB && bias) mine[(size_t)N * K + n0 + n] = acc[r][c][j];
                        }
                    }
                }
            }
        }
    }
}

constexpr int kWgradStreamBlock = 180; // block side of the streaming kernel's one instance

// Shares of the rows (one workgroup per share and block) for these arguments, 0 where the streaming kernel
// does not apply: N or K not whole blocks, a second addend, rows that are not dword-aligned, or a scratch
// too small for a useful share of the chip.
static int wgrad_stream_shares(const WgradArgs &a)
{
    constexpr int B = kWgradStreamBlock;
    if (!a.scratch || a.a2 || a.rows < 4096) return 0;
    if (a.N % B || a.K % B) return 0;
    if (a.lddout % 2 || a.lda1 % 2 || (reinterpret_cast<uintptr_t>(a.dout) | reinterpret_cast<uintptr_t>(a.a1)) % 4) return 0;
    if (reinterpret_cast<uintptr_t>(a.scratch) % 8) return 0;
    const size_t per = ((size_t)a.N * a.K + a.N) * 4;
    const int blocks = (a.N / B) * (a.K / B);
    long shares = (long)(a.scratch_bytes / per);
    const long passes = (a.rows + 127) / 128;
    const long want = device_cu_count() / blocks; // one workgroup per compute unit
    if (shares > want) shares = want;
    if (shares > passes) shares = passes;
    return shares >= 16 ? (int)shares : 0;
}

static WgradStreamJob stream_job(const WgradArgs &a, long part_off)
{
    WgradStreamJob j{};
    j.dout = static_cast<const bf16_t *>(a.dout); j.lddout = a.lddout;
    j.a = static_cast<const bf16_t *>(a.a1); j.lda = a.lda1;
    j.N = a.N; j.K = a.K; j.part_off = part_off;
    return j;
}

// `b` may be null: one gradient.  Two gradients share the rows, the scratch and the number of shares.
static hipError_t run_wgrad_stream(const WgradArgs &a, const WgradArgs *b, int shares, hipStream_t s)
{
    constexpr int B = kWgradStreamBlock;
    using P = WgradStreamCfg<B, B>;
    auto kern = wgrad_stream_kernel<B, B>;
    if (hipError_t ea = allow_dynamic_lds(reinterpret_cast<const void *>(kern), P::LDS_BYTES); ea != hipSuccess) return ea;
    float *part = static_cast<float *>(a.scratch);
    const int total0 = a.N * a.K + a.N, total1 = b ? b->N * b->K + b->N : 0;
    const int blocks0 = (a.N / B) * (a.K / B), blocks1 = b ? (b->N / B) * (b->K / B) : 0;
    {
        KernelTimer kt(a.prof_id, s);
        hipLaunchKernelGGL(kern, dim3(shares, blocks0 + blocks1), dim3(64 * P::NWV), P::LDS_BYTES, s, a.rows,
                           stream_job(a, 0), blocks0, b ? stream_job(*b, total0) : stream_job(a, 0), part,
                           (long)total0 + total1);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    ReduceOut out{};
    out.ptr[0] = a.dw; out.begin[0] = 0;
    out.ptr[1] = a.db; out.begin[1] = a.N * a.K;
    out.begin[2] = total0;
    out.nseg = 2;
    if (b) {
        out.ptr[2] = b->dw; out.begin[2] = total0;
        out.ptr[3] = b->db; out.begin[3] = total0 + b->N * b->K;
        out.begin[4] = total0 + total1;
        out.nseg = 4;
    }
    // onto copy 0 of the gradients, or into the gradients themselves
    return launch_reduce(part, shares, total0 + total1, out, a.direct ? a.accumulate : 1, s);
}

template <typename T> hipError_t launch_wgrad(const WgradArgs &a, hipStream_t s)
{
    if (a.rows <= 0 || a.N <= 0 || a.K <= 0) return hipSuccess;
    if (a.reps < 1) return hipErrorInvalidValue;
    if constexpr (sizeof(T) == 2) {
        if (const int shares = wgrad_stream_shares(a)) return run_wgrad_stream(a, nullptr, shares, s);
        return launch_wgrad_mfma(a, nullptr, nullptr, s);
    }
    const unsigned tn = (a.N + 63) / 64, tk = (a.K + 63) / 64;
    long splits = 2048 / (long)(tn * tk);
    const long max_splits = (a.rows + 255) / 256;
    if (splits > max_splits) splits = max_splits;
    if (a.exclusive && splits > a.reps) splits = a.reps; // every split then adds into a copy of its own
    if (splits < 1) splits = 1;
    long rps = (a.rows + splits - 1) / splits;
    rps = (rps + 15) / 16 * 16;
    splits = (a.rows + rps - 1) / rps;
    dim3 grid(tn, tk, (unsigned)splits);
    KernelTimer kt(a.prof_id, s);
    hipLaunchKernelGGL(wgrad_kernel<T>, grid, dim3(kThreads), 0, s, a, rps);
    return hipGetLastError();
}
template hipError_t launch_wgrad<float>(const WgradArgs &, hipStream_t);
template hipError_t launch_wgrad<bf16_t>(const WgradArgs &, hipStream_t);

// Two weight gradients over the same rows (and the same scratch) in one launch and one sum where the streaming
// kernel takes both; otherwise one after the other.
// shares of the rows for both gradients in one launch of the streaming kernel; 0: not both there
static int wgrad_pair_shares(const WgradArgs &a, const WgradArgs &b)
{
    if (!(a.rows == b.rows && a.scratch == b.scratch && a.scratch_bytes == b.scratch_bytes && a.reps >= 1 && b.reps >= 1 &&
          a.direct == b.direct && a.accumulate == b.accumulate && wgrad_stream_shares(a) && wgrad_stream_shares(b)))
        return 0;
    constexpr int B = kWgradStreamBlock;
    const size_t per = ((size_t)a.N * a.K + a.N + (size_t)b.N * b.K + b.N) * 4;
    const int blocks = (a.N / B) * (a.K / B) + (b.N / B) * (b.K / B);
    long shares = (long)(a.scratch_bytes / per);
    const long passes = (a.rows + 127) / 128, want = device_cu_count() / blocks;
    if (shares > want) shares = want;
    if (shares > passes) shares = passes;
    // (the second gradient's part of a share's array must start on the boundary the sum's wide loads need)
    return shares >= 16 && ((size_t)a.N * a.K + a.N) % 4 == 0 ? (int)shares : 0;
}

bool wgrad_pair_streams(const WgradArgs &a, const WgradArgs &b) { return wgrad_pair_shares(a, b) > 0; }

template <typename T> hipError_t launch_wgrad_pair(const WgradArgs &a, const WgradArgs &b, hipStream_t s)
{
    if constexpr (sizeof(T) == 2) {
        if (const int shares = wgrad_pair_shares(a, b)) return run_wgrad_stream(a, &b, shares, s);
    }
    if (a.direct || b.direct) return hipErrorInvalidValue; // (callers ask wgrad_pair_streams first)
    hipError_t e = launch_wgrad<T>(a, s);
    return e != hipSuccess ? e : launch_wgrad<T>(b, s);
}
template hipError_t launch_wgrad_pair<float>(const WgradArgs &, const WgradArgs &, hipStream_t);
template hipError_t launch_wgrad_pair<bf16_t>(const WgradArgs &, const WgradArgs &, hipStream_t);

template <typename T>
hipError_t launch_wgrad_group(const WgradArgs &a, const WgradArgs *b, const LinearArgs &lin, hipStream_t s)
{
    if constexpr (sizeof(T) == 2) {
        if (const int shares = wgrad_stream_shares(a)) {
            // wide layers: the linear map on its own, the reductions from the streaming kernel (they use the
            // same scratch one after the other)
            hipError_t e = launch_linear<T>(lin, s);
            if (e != hipSuccess) return e;
            if (b) return launch_wgrad_pair<T>(a, *b, s); // (one launch for both where the kernel takes both)
            return run_wgrad_stream(a, nullptr, shares, s);
        }
        const bool wg_ok = a.rows > 0 && a.N > 0 && a.K > 0 && a.reps >= 1 &&
                           (!b || (b->rows > 0 && b->N > 0 && b->K > 0 && b->reps >= 1));
        const bool lin_ok = lin.rows > 0 && lin.N > 0 && lin.N <= 64 && lin.K <= 64 && linear_mfma_ok(lin);
        if (wg_ok && lin_ok) return launch_wgrad_mfma(a, b, &lin, s);
        if (wg_ok) {
            hipError_t e = launch_linear<T>(lin, s);
            return e != hipSuccess ? e : launch_wgrad_mfma(a, b, nullptr, s);
        }
    }
    hipError_t e = launch_linear<T>(lin, s);
    if (e != hipSuccess) return e;
    e = launch_wgrad<T>(a, s);
    if (e != hipSuccess || !b) return e;
    return launch_wgrad<T>(*b, s);
}
template hipError_t launch_wgrad_group<float>(const WgradArgs &, const WgradArgs *, const LinearArgs &, hipStream_t);
template hipError_t launch_wgrad_group<bf16_t>(const WgradArgs &, const WgradArgs *, const LinearArgs &, hipStream_t);

// ---------------------------------------------------------------------------------------
// attention core, one block per (window, head of the group)
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// Largest strip height (rows of the score tile held at once) whose LDS need fits `budget`.
static int pick_strip(int N, size_t fixed_floats, size_t per_row_floats, size_t tail_bytes,
                      size_t budget, size_t *bytes)
{
    int cand[9] = {N, 128, 64, 32, 16, 8, 4, 2, 1};
    for (int i = 0; i < 9; ++i) {
        const int rs = cand[i];
        if (rs > N || (i > 0 && rs >= N)) continue;
        size_t fl = fixed_floats + per_row_floats * rs;
        fl = (fl + 1) & ~size_t(1);
        const size_t b = fl * sizeof(float) + tail_bytes;
        if (b <= budget) {
            *bytes = b;
            return rs;
        }
    }
    *bytes = 0;
    return 0;
}

size_t attn_fwd_lds_bytes(const Geom &g, int *strip_rows)
{
    const size_t dp = g.d | 1, ep = g.dq | 1;
    const size_t tail = (size_t)g.N * (sizeof(long) + sizeof(int));
    const size_t fixed = (size_t)g.N * (2 * ep + dp);
    size_t bytes = 0;
    int rs = pick_strip(g.N, fixed, g.N + 1, tail, 64 * 1024, &bytes);
    if (rs < 8 && rs < g.N) rs = pick_strip(g.N, fixed, g.N + 1, tail, kLdsMax, &bytes);
    if (strip_rows) *strip_rows = rs;
    return bytes;
}

size_t attn_bwd_lds_bytes(const Geom &g, int *strip_rows)
{
    const size_t dp = g.d | 1, ep = g.dq | 1;
    const size_t tbl = (size_t)(2 * g.M - 1) * (2 * g.M - 1);
    const size_t tail = (size_t)g.N * (sizeof(long) + sizeof(int));
    const size_t fixed = 2 * g.N * (dp + ep) + tbl;
    const size_t per_row = dp + ep + 2 * (g.N + 1);
    size_t bytes = 0;
    int rs = pick_strip(g.N, fixed, per_row, tail, 80 * 1024, &bytes);
    if (rs < 8 && rs < g.N) rs = pick_strip(g.N, fixed, per_row, tail, kLdsMax, &bytes);
    if (strip_rows) *strip_rows = rs;
    return bytes;
}

template <typename T>
__global__ __launch_bounds__(kThreads) void attn_fwd_kernel(Geom g, int grp, const T *__restrict__ qkv,
                                                            const T *__restrict__ table,
                                                            T *__restrict__ attn_out, int RS)
{
    extern __shared__ float smem[];
    const int N = g.N, d = g.d, dp = d | 1, dq = g.dq, ep = dq | 1, Qg = g.Qg, Rg = g.Rg, M = g.M;
    const int ldS = N + 1;
    float *q = smem;
    float *k = q + N * ep;
    float *v = k + N * ep;
    float *S = v + N * dp;
    size_t fl = (size_t)N * (2 * ep + dp) + (size_t)RS * ldS;
    fl = (fl + 1) & ~size_t(1);
    long *tok = reinterpret_cast<long *>(smem + fl);
    int *reg = reinterpret_cast<int *>(tok + N);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int w = blockIdx.x, hl = blockIdx.y, hd = grp * g.hg + hl;

    for (int n = tid; n < N; n += kThreads) {
        int r;
        tok[n] = window_token(g, w, n, r);
        reg[n] = r;
    }
    __syncthreads();
    for (int e = tid; e < N * dq; e += kThreads) {
        const int n = e / dq, c = e - n * dq;
        const long base = tok[n] * Rg + hl * dq + c;
        q[n * ep + c] = to_f32(qkv[base]);
        k[n * ep + c] = to_f32(qkv[base + Qg]);
    }
    for (int e = tid; e < N * d; e += kThreads) {
        const int n = e / d, c = e - n * d;
        v[n * dp + c] = to_f32(qkv[tok[n] * Rg + 2 * Qg + hl * d + c]);
    }
    __syncthreads();

    const float scale = 1.0f / sqrtf((float)dq);
    for (int n0 = 0; n0 < N; n0 += RS) {
        const int rows = min(RS, N - n0);
        for (int e = tid; e < rows * N; e += kThreads) {
            const int r = e / N, m = e - r * N, n = n0 + r;
            float dot = 0.f;
            for (int c = 0; c < dq; ++c) dot = fmaf(q[n * ep + c], k[m * ep + c], dot);
            const int rn = n / M, cn = n - rn * M, rm = m / M, cm = m - rm * M;
            const int idx = (rn - rm + M - 1) * (2 * M - 1) + (cn - cm + M - 1);
            float sc = dot * scale + to_f32(table[(long)idx * g.heads + hd]);
            if (reg[n] != reg[m]) sc += -100.0f;
            S[r * ldS + m] = sc;
        }
        __syncthreads();
        for (int r = wave; r < rows; r += kThreads / 64) {
            float mx = -INFINITY;
            for (int m = lane; m < N; m += 64) mx = fmaxf(mx, S[r * ldS + m]);
            mx = wave_max(mx);
            float sum = 0.f;
            for (int m = lane; m < N; m += 64) {
                const float ev = expf(S[r * ldS + m] - mx);
                S[r * ldS + m] = ev;
                sum += ev;
            }
            sum = wave_sum(sum);
            const float inv = 1.0f / sum;
            for (int m = lane; m < N; m += 64) S[r * ldS + m] *= inv;
        }
        __syncthreads();
        for (int e = tid; e < rows * d; e += kThreads) {
            const int r = e / d, c = e - r * d;
            float acc = 0.f;
            for (int m = 0; m < N; ++m) acc = fmaf(S[r * ldS + m], v[m * dp + c], acc);
            from_f32(attn_out[tok[n0 + r] * g.C + hd * d + c], acc);
        }
        __syncthreads();
    }
}

template <typename T>
hipError_t launch_attn_fwd(const Geom &g, int grp, const T *qkv, const T *table, T *attn_out,
                           hipStream_t s)
{
    int rs = 0;
    const size_t lds = attn_fwd_lds_bytes(g, &rs);
    if (rs == 0) return hipErrorInvalidValue;
    auto kern = attn_fwd_kernel<T>;
    if (hipError_t ea = allow_dynamic_lds(reinterpret_cast<const void *>(kern), lds); ea != hipSuccess) return ea;
    KernelTimer kt(K_ATTN_FWD, s);
    hipLaunchKernelGGL(kern, dim3(g.nW, g.hg), dim3(kThreads), lds, s, g, grp, qkv, table, attn_out, rs);
    return hipGetLastError();
}
template hipError_t launch_attn_fwd<float>(const Geom &, int, const float *, const float *, float *, hipStream_t);
template hipError_t launch_attn_fwd<bf16_t>(const Geom &, int, const bf16_t *, const bf16_t *, bf16_t *, hipStream_t);

template <typename T>
__global__ __launch_bounds__(kThreads) void attn_bwd_kernel(Geom g, int grp, const T *__restrict__ qkv,
                                                            T *dqkv, const T *__restrict__ table,
                                                            float *dtable, long rep_stride, int reps, int RS)
{
    extern __shared__ float smem[];
    // reps == 0: every window owns a copy of its own (rep_stride apart), written with plain stores
    const bool own_copy = reps == 0;
    dtable += (long)(own_copy ? blockIdx.x : blockIdx.x % reps) * rep_stride;
    const int N = g.N, d = g.d, dp = d | 1, dq = g.dq, ep = dq | 1, Qg = g.Qg, Rg = g.Rg, M = g.M;
    const int ldS = N + 1, ntbl = (2 * M - 1) * (2 * M - 1);
    float *k = smem;
    float *v = k + N * ep;
    float *dk = v + N * dp;
    float *dv = dk + N * ep;
    float *tbl = dv + N * dp;
    float *q = tbl + ntbl;
    float *dO = q + RS * ep;
    float *P = dO + RS * dp;
    float *dS = P + RS * ldS;
    size_t fl = (size_t)2 * N * (dp + ep) + ntbl + (size_t)RS * (dp + ep + 2 * ldS);
    fl = (fl + 1) & ~size_t(1);
    long *tok = reinterpret_cast<long *>(smem + fl);
    int *reg = reinterpret_cast<int *>(tok + N);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int w = blockIdx.x, hl = blockIdx.y, hd = grp * g.hg + hl;

    for (int n = tid; n < N; n += kThreads) {
        int r;
        tok[n] = window_token(g, w, n, r);
        reg[n] = r;
    }
    for (int e = tid; e < ntbl; e += kThreads) tbl[e] = 0.f;
    __syncthreads();
    for (int e = tid; e < N * dq; e += kThreads) {
        const int n = e / dq, c = e - n * dq;
        k[n * ep + c] = to_f32(qkv[tok[n] * Rg + Qg + hl * dq + c]);
        dk[n * ep + c] = 0.f;
    }
    for (int e = tid; e < N * d; e += kThreads) {
        const int n = e / d, c = e - n * d;
        v[n * dp + c] = to_f32(qkv[tok[n] * Rg + 2 * Qg + hl * d + c]);
        dv[n * dp + c] = 0.f;
    }
    const float scale = 1.0f / sqrtf((float)dq);

    for (int n0 = 0; n0 < N; n0 += RS) {
        const int rows = min(RS, N - n0);
        __syncthreads();
        for (int e = tid; e < rows * dq; e += kThreads) {
            const int r = e / dq, c = e - r * dq;
            q[r * ep + c] = to_f32(qkv[tok[n0 + r] * Rg + hl * dq + c]);
        }
        for (int e = tid; e < rows * d; e += kThreads) {
            const int r = e / d, c = e - r * d;
            dO[r * dp + c] = to_f32(dqkv[tok[n0 + r] * Rg + 2 * Qg + hl * d + c]);
        }
        __syncthreads();
        // scores and dP = dO v^T
        for (int e = tid; e < rows * N; e += kThreads) {
            const int r = e / N, m = e - r * N, n = n0 + r;
            float dot = 0.f, dp_ = 0.f;
            for (int c = 0; c < dq; ++c) dot = fmaf(q[r * ep + c], k[m * ep + c], dot);
            for (int c = 0; c < d; ++c) dp_ = fmaf(dO[r * dp + c], v[m * dp + c], dp_);
            const int rn = n / M, cn = n - rn * M, rm = m / M, cm = m - rm * M;
            const int idx = (rn - rm + M - 1) * (2 * M - 1) + (cn - cm + M - 1);
            float sc = dot * scale + to_f32(table[(long)idx * g.heads + hd]);
            if (reg[n] != reg[m]) sc += -100.0f;
            P[r * ldS + m] = sc;
            dS[r * ldS + m] = dp_;
        }
        __syncthreads();
        // softmax and its adjoint, one wave per row; bias-table gradient pre-reduced in LDS
        for (int r = wave; r < rows; r += kThreads / 64) {
            float mx = -INFINITY;
            for (int m = lane; m < N; m += 64) mx = fmaxf(mx, P[r * ldS + m]);
            mx = wave_max(mx);
            float sum = 0.f;
            for (int m = lane; m < N; m += 64) {
                const float ev = expf(P[r * ldS + m] - mx);
                P[r * ldS + m] = ev;
                sum += ev;
            }
            sum = wave_sum(sum);
            const float inv = 1.0f / sum;
            float dotp = 0.f;
            for (int m = lane; m < N; m += 64) {
                const float pv = P[r * ldS + m] * inv;
                P[r * ldS + m] = pv;
                dotp = fmaf(pv, dS[r * ldS + m], dotp);
            }
            dotp = wave_sum(dotp);
            for (int m = lane; m < N; m += 64) {
                dS[r * ldS + m] = P[r * ldS + m] * (dS[r * ldS + m] - dotp);
            }
        }
        __syncthreads();
        // bias-table gradient of the strip: entry (dr, dc) takes the pairs (n, m = n - (dr, dc)) whose
        // key lies inside the window; one thread per entry, rows in ascending order (a fixed order)
        for (int e = tid; e < ntbl; e += kThreads) {
            const int dr = e / (2 * M - 1) - (M - 1), dc = e % (2 * M - 1) - (M - 1);
            float acc = 0.f;
            for (int r = 0; r < rows; ++r) {
                const int n = n0 + r, rn = n / M, cn = n - rn * M;
                const int rm = rn - dr, cm = cn - dc;
                if ((unsigned)rm < (unsigned)M && (unsigned)cm < (unsigned)M) acc += dS[r * ldS + rm * M + cm];
            }
            tbl[e] += acc;
        }
        // dq rows of this strip
        for (int e = tid; e < rows * dq; e += kThreads) {
            const int r = e / dq, c = e - r * dq;
            float acc = 0.f;
            for (int m = 0; m < N; ++m) acc = fmaf(dS[r * ldS + m], k[m * ep + c], acc);
            from_f32(dqkv[tok[n0 + r] * Rg + hl * dq + c], acc * scale);
        }
        // dk, dv accumulate over strips; element (m, c) belongs to one thread
        for (int e = tid; e < N * dq; e += kThreads) {
            const int m = e / dq, c = e - m * dq;
            float ak = 0.f;
            for (int r = 0; r < rows; ++r) ak = fmaf(dS[r * ldS + m], q[r * ep + c], ak);
            dk[m * ep + c] += ak * scale;
        }
        for (int e = tid; e < N * d; e += kThreads) {
            const int m = e / d, c = e - m * d;
            float av = 0.f;
            for (int r = 0; r < rows; ++r) av = fmaf(P[r * ldS + m], dO[r * dp + c], av);
            dv[m * dp + c] += av;
        }
    }
    __syncthreads();
    for (int e = tid; e < N * dq; e += kThreads) {
        const int n = e / dq, c = e - n * dq;
        from_f32(dqkv[tok[n] * Rg + Qg + hl * dq + c], dk[n * ep + c]);
    }
    for (int e = tid; e < N * d; e += kThreads) {
        const int n = e / d, c = e - n * d;
        from_f32(dqkv[tok[n] * Rg + 2 * Qg + hl * d + c], dv[n * dp + c]);
    }
    for (int e = tid; e < ntbl; e += kThreads) {
        if (own_copy) dtable[(long)e * g.heads + hd] = tbl[e];
        else atomicAdd(&dtable[(long)e * g.heads + hd], tbl[e]);
    }
}


template <typename T>
hipError_t launch_attn_bwd(const Geom &g, int grp, const T *qkv, T *dqkv, const T *table,
                           float *dtable, long rep_stride, int reps, hipStream_t s)
{
    if (reps < 0) return hipErrorInvalidValue;
    int rs = 0;
    const size_t lds = attn_bwd_lds_bytes(g, &rs);
    if (rs == 0) return hipErrorInvalidValue;
    auto kern = attn_bwd_kernel<T>;
    if (hipError_t ea = allow_dynamic_lds(reinterpret_cast<const void *>(kern), lds); ea != hipSuccess) return ea;
    KernelTimer kt(K_ATTN_BWD, s);
    hipLaunchKernelGGL(kern, dim3(g.nW, g.hg), dim3(kThreads), lds, s, g, grp, qkv, dqkv, table, dtable, rep_stride, reps, rs);
    return hipGetLastError();
}
template hipError_t launch_attn_bwd<float>(const Geom &, int, const float *, float *, const float *, float *, long, int, hipStream_t);
template hipError_t launch_attn_bwd<bf16_t>(const Geom &, int, const bf16_t *, bf16_t *, const bf16_t *, float *, long, int, hipStream_t);

__global__ void fill_zero_kernel(ZeroList z)
{
    float *p = z.p[blockIdx.y];
    const size_t n = z.n[blockIdx.y];
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        p[i] = 0.f;
}

hipError_t launch_fill_zero(const ZeroList &z, hipStream_t s)
{
    size_t longest = 0;
    for (int i = 0; i < z.count; ++i) longest = z.n[i] > longest ? z.n[i] : longest;
    if (z.count <= 0 || longest == 0) return hipSuccess;
    unsigned blocks = (unsigned)((longest + 255) / 256);
    if (blocks > 256) blocks = 256;
    KernelTimer kt(K_FILL, s);
    hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks, z.count), dim3(256), 0, s, z);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void reduce_replicas_kernel(ReplicaSum r)
{
    if ((int)blockIdx.y == r.count) {
        // the output with per-window copies: 32 entries per block, 8 slices of the windows
        __shared__ float red[8][33];
        const int col = threadIdx.x & 31, slice = threadIdx.x >> 5;
        for (long i0 = (long)blockIdx.x * 32; i0 < r.t_n; i0 += (long)gridDim.x * 32) {
            const long i = i0 + col;
            float acc = 0.f;
            if (i < r.t_n) {
                // eight loads in flight per thread
                float a8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                int w = slice;
                for (; w + 56 < r.t_windows; w += 64) {
#pragma unroll
                    for (int u = 0; u < 8; ++u) a8[u] += r.tpart[(long)(w + 8 * u) * r.t_n + i];
                }
                for (; w < r.t_windows; w += 8) a8[0] += r.tpart[(long)w * r.t_n + i];
                acc = ((a8[0] + a8[1]) + (a8[2] + a8[3])) + ((a8[4] + a8[5]) + (a8[6] + a8[7]));
                for (int c = slice; c < r.reps; c += 8) acc += r.rep[(long)c * r.stride + r.t_off + i];
            }
            red[slice][col] = acc;
            __syncthreads();
            if (slice == 0 && i < r.t_n) {
                float sum = 0.f;
#pragma unroll
                for (int k8 = 0; k8 < 8; ++k8) sum += red[k8][col];
                r.t_out[i] = r.accumulate ? r.t_out[i] + sum : sum;
            }
            __syncthreads();
        }
        return;
    }
    const int k = blockIdx.y;
    for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < r.n[k]; i += (long)gridDim.x * blockDim.x) {
        float acc = 0.f;
        for (int c = 0; c < r.reps; ++c) acc += r.rep[(long)c * r.stride + r.off[k] + i];
        r.out[k][i] = r.accumulate ? r.out[k][i] + acc : acc;
    }
}

hipError_t launch_reduce_replicas(const ReplicaSum &r, hipStream_t s)
{
    long longest = 0;
    for (int k = 0; k < r.count; ++k) longest = r.n[k] > longest ? r.n[k] : longest;
    if (r.count <= 0 || longest == 0) return hipSuccess;
    unsigned blocks = (unsigned)((longest + 255) / 256);
    const bool with_t = r.t_out && r.t_n > 0;
    if (with_t && blocks < (unsigned)((r.t_n + 31) / 32)) blocks = (unsigned)((r.t_n + 31) / 32);
    if (blocks > 256) blocks = 256;
    KernelTimer kt(K_REDUCE, s);
    hipLaunchKernelGGL(reduce_replicas_kernel, dim3(blocks, r.count + (with_t ? 1 : 0)), dim3(256), 0, s, r);
    return hipGetLastError();
}

} // namespace gswa
