// Fused forward of the MLP half of a layer (Sec. "Agile Swin Transformer Block", Eq. 5, with the skip
// connection of Eq. 4 in the prologue) for WIDE bf16 layers: the two weight matrices together (282 KB as
// matrix-core fragments at C = 180, hidden = 360) do not fit LDS, so they are streamed through it in units
// of 96 hidden features (three steps of 32), double buffered, by loads that write LDS directly, one barrier
// per unit.
//
// A wavefront owns 16 tokens from the first load to the last store; the hidden layer never leaves its
// registers.  Lane (tok = lane & 15, q = lane >> 4) holds, of its token, the channels 32 p + 8 q + 0..7
// (p < KSC): one 16-byte access per p.  Both products are taken transposed (features x tokens), weights as
// the A operand from the fragments of the unit in LDS, activations as the B operand from registers:
//   pre^T = W1 LN_2(x1)^T  reduces over channels: k-slot j of lane q in step p is channel 32 p + 8 q + j,
//                          the order the row was loaded in;
//   y^T  += W2 h^T         reduces over the unit's 32 hidden features: h^T comes out of the first product
//                          with features 16 ft + 4 q + i of token tok in the lane, and the two tiles of
//                          the unit pack into one B operand (k-slot j = feature 16 (j >> 2) + 4 q + (j & 3));
//                          the ROWS of the W2 fragments are ordered so that a lane's results of channel
//                          tiles 2p and 2p + 1 are again the channels 32 p + 8 q + 0..7: the skip of Eq. 5
//                          adds the lane's own x1 registers and y leaves in 16-byte pieces.
// Arithmetic follows the one-kernel-per-step path value by value (x1 and LN_2(x1) rounded to bf16, the
// pre-activation rounded before the GELU), so the backward pass recomputes exactly this hidden layer.
#include "astl_mlp.h"
#include "mfma.h"
#include "staged_kernels.h"
#include "profile.h"

namespace gswa {

namespace {

constexpr int kWideThreads = 512;
constexpr int kWideWaves = kWideThreads / 64;

// s_waitcnt immediate: vector-memory counter down to 2 KSC, the other counters not waited for
// (vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8)
template <int KSC> constexpr int kWaitAllBut2Ksc = ((2 * KSC) & 15) | (((2 * KSC) >> 4) << 14) | (7 << 4) | (15 << 8);

// a lane's 16-byte piece of a row as ONE four-register value (kept whole from the load to its use: loose
// dwords carried around the round loop get copied right behind the load, which waits for it)
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef u32x4 u32x4_a4 __attribute__((aligned(4)));

struct __attribute__((aligned(4))) row16 {
    uint32_t v[4];
};

struct WideMlpArgs {
    long rows;
    int C, Hd;
    float eps;
    const bf16_t *x, *a;       // x1 = x + a
    const bf16_t *ln_w, *ln_b, *w_fc1, *b_fc1, *w_fc2, *b_fc2;
    bf16_t *x1, *y;
    const bf16_t *nxt_w, *nxt_b; // optional: gamma, beta of the LayerNorm that reads y next ...
    bf16_t *xn_out;              // ... and where its output goes (null: not wanted)
    void *pack;
    void *bwd_pack;              // optional: the backward kernel's order of the same weights, written by the same launch
};

// KSC k-steps of 32 channels, KSF steps of 32 hidden features, HU of them per stream unit.
template <int KSC, int KSF> struct WideMlp {
    static constexpr int CT = 2 * KSC, FT = 2 * KSF;
    static constexpr int HU = 3;
    static_assert(KSF % HU == 0, "whole units");
    static constexpr int FR_STEP = 2 * KSC + CT;        // W1: 2 feature tiles x KSC steps | W2: CT channel tiles x 1 step
    static constexpr int FR_UNIT = HU * FR_STEP;
    static constexpr int UNIT_BYTES = FR_UNIT * 1024;
    static constexpr int FPW = (FR_UNIT + kWideWaves - 1) / kWideWaves; // fragments a wave moves per unit
    // tables behind the fragments, in the pack and in LDS alike (floats):
    //   b1 [FT * 16] | b2 [CT * 16] | (gamma, beta) of LN_2 [32 KSC][2] | (gamma, beta) of the next LN [32 KSC][2]
    static constexpr int T_B1 = 0, T_B2 = FT * 16, T_GB = T_B2 + CT * 16, T_NGB = T_GB + 64 * KSC;
    static constexpr int T_FLOATS = T_NGB + 64 * KSC;
    static constexpr size_t P_TABLES = (size_t)(KSF / HU) * UNIT_BYTES;
    static constexpr size_t P_BYTES = P_TABLES + (size_t)T_FLOATS * 4;
    static constexpr int OFF_TABLES = 2 * UNIT_BYTES;
    static constexpr size_t LDS_BYTES = (size_t)OFF_TABLES + (size_t)T_FLOATS * 4;
    static_assert(T_FLOATS % 4 == 0, "tables are copied in 16-byte pieces");
};

__device__ __forceinline__ float bfv(const bf16_t *p, long i) { return __uint_as_float((uint32_t)p[i].bits << 16); }

// Once per forward call: the weights in the order the units are streamed in, zero outside the matrices.
template <int KSC, int KSF>
__device__ __forceinline__ void wide_fwd_pack_body(const WideMlpArgs &a, int nu)
{
    using L = WideMlp<KSC, KSF>;
    const int C = a.C, Hd = a.Hd;
    uint16_t *d16 = static_cast<uint16_t *>(a.pack);
    const int total = nu * L::FR_UNIT * 512; // (nu units: steps of hidden features beyond the matrix are zero)
    for (int e = blockIdx.x * 256 + threadIdx.x; e < total; e += gridDim.x * 256) {
        const int j = e & 7, l = (e >> 3) & 63, fr = e >> 9;
        const int u = fr / L::FR_STEP, f = fr - u * L::FR_STEP; // u: step of 32 hidden features
        const int m = l & 15, lq = l >> 4;
        float v = 0.f;
        if (f < 2 * KSC) {
            const int jt = f / KSC, s = f - jt * KSC;
            const int hid = 16 * (2 * u + jt) + m, ch = 32 * s + 8 * lq + j;
            if (hid < Hd && ch < C) v = bfv(a.w_fc1, (long)hid * C + ch);
        } else {
            const int ct = f - 2 * KSC;
            const int ch = 32 * (ct >> 1) + 8 * (m >> 2) + 4 * (ct & 1) + (m & 3);
            const int hid = 16 * (2 * u + (j >> 2)) + 4 * lq + (j & 3);
            if (hid < Hd && ch < C) v = bfv(a.w_fc2, (long)ch * Hd + hid);
        }
        d16[e] = f32_to_bf16_bits(v);
    }
    float *tb = reinterpret_cast<float *>(static_cast<uint8_t *>(a.pack) + L::P_TABLES);
    for (int i = blockIdx.x * 256 + threadIdx.x; i < L::T_FLOATS; i += gridDim.x * 256) {
        float v = 0.f;
        if (i < L::T_B2) {
            if (i < Hd) v = bfv(a.b_fc1, i);
        } else if (i < L::T_GB) {
            if (i - L::T_B2 < C) v = bfv(a.b_fc2, i - L::T_B2);
        } else if (i < L::T_NGB) {
            const int c = (i - L::T_GB) >> 1;
            if (c < C) v = bfv((i & 1) ? a.ln_b : a.ln_w, c);
        } else if (a.nxt_w) {
            const int c = (i - L::T_NGB) >> 1;
            if (c < C) v = bfv((i & 1) ? a.nxt_b : a.nxt_w, c);
        }
        tb[i] = v;
    }
}

// LayerNorm of a row held as packed bf16 in the lane pattern of this file (zero beyond C): the row is
// spread over the four lanes that share tok.  Mean first, then the squared distances from it, as the
// LayerNorm kernel of the one-kernel-per-step path computes them; result rounded to bf16, zero beyond C.
// Returns (mean, 1/sqrt(var + eps)) of the row.
template <int KSC>
__device__ __forceinline__ float2 layer_norm_rows(uint32_t (&r)[KSC][4], int C, int q, float eps, const float2 *gb)
{
    asm volatile("" : "+v"(q)); // (as in load_rows)
    float sum = 0.f;
#pragma unroll
    for (int p = 0; p < KSC; ++p)
#pragma unroll
        for (int dw = 0; dw < 4; ++dw) sum += bf16_lo(r[p][dw]) + bf16_hi(r[p][dw]);
    const float mean = qgroup_sum(sum) / (float)C;
    // (each pass unpacks the row again: the unpacked values of a whole row would take twice its registers)
#pragma unroll
    for (int p = 0; p < KSC; ++p)
#pragma unroll
        for (int dw = 0; dw < 4; ++dw) asm volatile("" : "+v"(r[p][dw]));
    float dev = 0.f;
#pragma unroll
    for (int p = 0; p < KSC; ++p)
#pragma unroll
        for (int dw = 0; dw < 4; ++dw)
            if (32 * p + 8 * q + 2 * dw < C) {
                const float d0 = bf16_lo(r[p][dw]) - mean, d1 = bf16_hi(r[p][dw]) - mean;
                dev += d0 * d0 + d1 * d1;
            }
    const float rstd = rsqrtf(qgroup_sum(dev) / (float)C + eps);
#pragma unroll
    for (int p = 0; p < KSC; ++p)
#pragma unroll
        for (int dw = 0; dw < 4; ++dw) asm volatile("" : "+v"(r[p][dw]));
#pragma unroll
    for (int p = 0; p < KSC; ++p) {
#pragma unroll
        for (int dw = 0; dw < 4; ++dw) {
            const int c = 32 * p + 8 * q + 2 * dw;
            const float4 g = *reinterpret_cast<const float4 *>(gb + c); // (gamma, beta) of c and c + 1; zero beyond C
            r[p][dw] = pack_bf16x2((bf16_lo(r[p][dw]) - mean) * rstd * g.x + g.y,
                                   (bf16_hi(r[p][dw]) - mean) * rstd * g.z + g.w);
        }
        __builtin_amdgcn_sched_barrier(0); // (one step's scale and shift in registers at a time)
    }
    return make_float2(mean, rstd);
}

// sum over the 16 lanes of a row (lanes that share q), valid in the row's last lane: a prefix sum by row shifts
// on the vector ALU's data path (lanes shifted in from outside the row read zero)
__device__ __forceinline__ float row_sum_in_last_lane(float v)
{
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x111, 0xf, 0xf, true)); // row_shr:1
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x112, 0xf, 0xf, true)); // row_shr:2
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x114, 0xf, 0xf, true)); // row_shr:4
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x118, 0xf, 0xf, true)); // row_shr:8
    return v;
}

// The lane's pieces of row t: channels 32 p + 8 q + 0..7, as one 16-byte load per step that nothing here
// computes with, so that the loads can stay in flight until their registers are used; tidy_rows() then puts
// the ragged end of the row right.  A piece that would reach beyond the row is read 8 channels before the
// row's end instead (C is a multiple of 4, so a piece is whole, the row's last 4 channels, or nothing).  Rows
// beyond the last one read the last one (their results are never stored, and a token's values stay in its
// own column of every product).
template <int KSC>
__device__ __forceinline__ void load_rows(const bf16_t *base, long t, long rows, int C, int q, u32x4 (&r)[KSC])
{
    const uint32_t *b32 = reinterpret_cast<const uint32_t *>(base);
    const long tc = t < rows ? t : rows - 1;
    asm volatile("" : "+v"(q)); // (offsets and masks are made per call: kept, they would take dozens of registers)
#pragma unroll
    for (int p = 0; p < KSC; ++p) {
        int c0 = 32 * p + 8 * q;
        if (p >= KSC - 2 && c0 + 8 > C) c0 = C - 8; // (C > 32 (KSC - 2): only the last two steps can be ragged)
        r[p] = *reinterpret_cast<const u32x4_a4 *>(b32 + ((tc * C + c0) >> 1));
    }
}

// after load_rows, once the values are wanted: zero beyond C, the row's last 4 channels moved into place
template <int KSC>
__device__ __forceinline__ void tidy_rows(int C, int q, const u32x4 (&r)[KSC], uint32_t (&o)[KSC][4])
{
    asm volatile("" : "+v"(q));
#pragma unroll
    for (int p = 0; p < KSC; ++p) {
        if (p < KSC - 2) {
            o[p][0] = r[p].x; o[p][1] = r[p].y; o[p][2] = r[p].z; o[p][3] = r[p].w;
        } else {
            const int c0 = 32 * p + 8 * q;
            const bool whole = c0 + 8 <= C, half = c0 + 4 == C;
            o[p][0] = whole ? r[p].x : half ? r[p].z : 0u;
            o[p][1] = whole ? r[p].y : half ? r[p].w : 0u;
            o[p][2] = whole ? r[p].z : 0u;
            o[p][3] = whole ? r[p].w : 0u;
        }
    }
}

template <int KSC>
__device__ __forceinline__ void store_rows(bf16_t *base, long t, bool ok, int C, int q, const uint32_t (&r)[KSC][4])
{
    uint32_t *b32 = reinterpret_cast<uint32_t *>(base);
    asm volatile("" : "+v"(q)); // (as in load_rows)
#pragma unroll
    for (int p = 0; p < KSC; ++p) {
        const int c0 = 32 * p + 8 * q;
        if (p < KSC - 2 || 32 * p + 32 <= C) { // (C > 32 (KSC - 2): only the last two steps can be ragged)
            if (ok) {
                row16 u;
#pragma unroll
                for (int dw = 0; dw < 4; ++dw) u.v[dw] = r[p][dw];
                *reinterpret_cast<row16 *>(b32 + ((t * C + c0) >> 1)) = u;
            }
        } else {
#pragma unroll
            for (int dw = 0; dw < 4; ++dw)
                if (ok && c0 + 2 * dw < C) b32[(t * C + c0 + 2 * dw) >> 1] = r[p][dw];
        }
    }
}

// one step of store_rows: the lane's piece of channels 32 p + 8 q + 0..7 of row t
template <int KSC>
__device__ __forceinline__ void store_piece(bf16_t *base, long t, bool ok, int C, int q, int p, const uint32_t (&v)[4])
{
    uint32_t *b32 = reinterpret_cast<uint32_t *>(base);
    const int c0 = 32 * p + 8 * q;
    if (p < KSC - 2 || 32 * p + 32 <= C) {
        if (ok) {
            row16 u;
#pragma unroll
            for (int dw = 0; dw < 4; ++dw) u.v[dw] = v[dw];
            *reinterpret_cast<row16 *>(b32 + ((t * C + c0) >> 1)) = u;
        }
    } else {
#pragma unroll
        for (int dw = 0; dw < 4; ++dw)
            if (ok && c0 + 2 * dw < C) b32[(t * C + c0 + 2 * dw) >> 1] = v[dw];
    }
}

template <int KSC, int KSF>
__global__ __launch_bounds__(kWideThreads) void astl_mlp_wide_fwd_kernel(WideMlpArgs a, int nu)
{
    using L = WideMlp<KSC, KSF>;
    constexpr int CT = L::CT;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const uint8_t *pack = static_cast<const uint8_t *>(a.pack);
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, tok = lane & 15, q = lane >> 4;
    const int C = a.C;
    int lane_r = lane;

    // One load instruction moves one fragment (64 lanes x 16 bytes land at the wave-uniform LDS address
    // + 16 lane); wave w moves fragments w, w + 8, ... of the unit.
    auto stream_unit = [&](int u, int slot) {
        int ln = lane_r;
        asm volatile("" : "+v"(ln)); // (the per-fragment addresses are made here, not kept over the unit loop)
        const uint8_t *src = pack + (size_t)u * L::UNIT_BYTES + 16 * ln;
        uint8_t *dst = lds + (size_t)slot * L::UNIT_BYTES;
#pragma unroll 1
        for (int k = 0; k < L::FPW; ++k) { // (not unrolled: one address in registers at a time)
            const int f = k * kWideWaves + wv;
            if (f < L::FR_UNIT) lds_dma16(src + (size_t)f * 1024, dst + (size_t)f * 1024);
        }
    };

    const long ntiles = (a.rows + 15) / 16;
    const long stride = (long)gridDim.x * kWideWaves;
    const int rounds = (int)((ntiles + stride - 1) / stride);
    long tile = (long)blockIdx.x * kWideWaves + wv;

    u32x4 rx[KSC], ra[KSC];
    load_rows<KSC>(a.x, tile * 16 + tok, a.rows, C, q, rx);
    load_rows<KSC>(a.a, tile * 16 + tok, a.rows, C, q, ra);

    stream_unit(0, 0);
    for (int i = tid; i < L::T_FLOATS / 4; i += kWideThreads)
        reinterpret_cast<uint4 *>(lds + L::OFF_TABLES)[i] = reinterpret_cast<const uint4 *>(pack + L::P_TABLES)[i];
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();

    int slot = 0; // buffer the unit about to be used lies in
    for (int round = 0; round < rounds; ++round, tile += stride) {
        const bool more = round + 1 < rounds;
        const long t = tile * 16 + tok;
        const bool ok = t < a.rows;
        uint32_t lds0 = 0;
        asm volatile("" : "+v"(lds0)); // keeps the LDS reads of a round inside the round
        lane_r = lane;
        asm volatile("" : "+v"(lane_r));
        const float *tb = reinterpret_cast<const float *>(lds + lds0 + L::OFF_TABLES);

        // Eq. 4's skip; the stored (rounded) sum is what LN_2 sees here and in the backward pass
        uint32_t x1[KSC][4];
        {
            uint32_t xv[KSC][4], av[KSC][4];
            tidy_rows<KSC>(C, q, rx, xv);
            tidy_rows<KSC>(C, q, ra, av);
#pragma unroll
            for (int p = 0; p < KSC; ++p)
#pragma unroll
                for (int dw = 0; dw < 4; ++dw)
                    x1[p][dw] = pack_bf16x2(bf16_lo(xv[p][dw]) + bf16_lo(av[p][dw]), bf16_hi(xv[p][dw]) + bf16_hi(av[p][dw]));
        }
        if (a.x1) store_rows<KSC>(a.x1, t, ok, C, q, x1);
        uint32_t bx[KSC][4];
#pragma unroll
        for (int p = 0; p < KSC; ++p)
#pragma unroll
            for (int dw = 0; dw < 4; ++dw) bx[p][dw] = x1[p][dw];
        layer_norm_rows<KSC>(bx, C, q, a.eps, reinterpret_cast<const float2 *>(tb + L::T_GB));

        f32x4 yacc[CT];
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) yacc[ct] = f32x4{0.f, 0.f, 0.f, 0.f};

        // The steps of a unit, written out one after the other (the products of one step can run under the
        // GELU of the step before).
        auto unit_steps = [&](int unit) {
            const uint4 *wu = reinterpret_cast<const uint4 *>(lds + lds0 + (size_t)slot * L::UNIT_BYTES);
#pragma unroll
            for (int hs = 0; hs < L::HU; ++hs) {
                const uint4 *ws = wu + hs * L::FR_STEP * 64;
                const int f0 = 32 * (L::HU * unit + hs); // hidden features f0 + 16 jt + 4 q + i of token tok
                f32x4 h0 = f32x4{0.f, 0.f, 0.f, 0.f}, h1 = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < KSC; ++s) {
                    const uint4 b = make_uint4(bx[s][0], bx[s][1], bx[s][2], bx[s][3]);
                    h0 = mma32(ws[s * 64 + lane_r], b, h0);
                    h1 = mma32(ws[(KSC + s) * 64 + lane_r], b, h1);
                }
                const float4 b10 = *reinterpret_cast<const float4 *>(tb + L::T_B1 + f0 + 4 * q);
                const float4 b11 = *reinterpret_cast<const float4 *>(tb + L::T_B1 + f0 + 16 + 4 * q);
                // the pre-activation as the one-kernel-per-step path stores it (rounded), then the GELU
                const uint32_t pp[4] = {pack_bf16x2(h0[0] + b10.x, h0[1] + b10.y), pack_bf16x2(h0[2] + b10.z, h0[3] + b10.w),
                                        pack_bf16x2(h1[0] + b11.x, h1[1] + b11.y), pack_bf16x2(h1[2] + b11.z, h1[3] + b11.w)};
                uint32_t hp[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float r0 = bf16_lo(pp[i]), r1 = bf16_hi(pp[i]);
                    float Phi0, Phi1, phi;
                    gauss(r0, Phi0, phi);
                    gauss(r1, Phi1, phi);
                    hp[i] = pack_bf16x2(r0 * Phi0, r1 * Phi1);
                }
                const uint4 hb = make_uint4(hp[0], hp[1], hp[2], hp[3]);
#pragma unroll
                for (int ct = 0; ct < CT; ++ct) yacc[ct] = mma32(ws[(2 * KSC + ct) * 64 + lane_r], hb, yacc[ct]);
            }
        };

        // First unit of the round (written apart from the loop over the others, so that the compiler sees that
        // the row loads below are not in flight when it runs): the second unit is sent on its way into the
        // other buffer (every wave has passed the previous barrier, i.e. finished reading that buffer), and
        // BEHIND its loads the next round's rows, which have until the end of the round.
        if (nu > 1) stream_unit(1, slot ^ 1);
        else if (more) stream_unit(0, slot ^ 1);
        if (more) {
            const long tn = t + stride * 16;
            load_rows<KSC>(a.x, tn, a.rows, C, q, rx);
            load_rows<KSC>(a.a, tn, a.rows, C, q, ra);
        }
        unit_steps(0);
        // The next unit has landed in LDS before any wave reads it.  Vector-memory operations complete in the
        // order they were issued, so "at most n outstanding" covers everything older than the n youngest: here
        // those are the row loads (each of the KSC steps of the two tensors is one load instruction), which
        // stay in flight.
        if (more) __builtin_amdgcn_s_waitcnt(kWaitAllBut2Ksc<KSC>);
        else __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        slot ^= 1;
        for (int unit = 1; unit < nu; ++unit) {
            if (unit + 1 < nu) stream_unit(unit + 1, slot ^ 1);
            else if (more) stream_unit(0, slot ^ 1); // (the first unit of the next round)
            unit_steps(unit);
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
            slot ^= 1;
        }

        // bias and the skip of Eq. 5; tiles 2p and 2p + 1 hold the lane's channels 32 p + 8 q + 0..3 and + 4..7
        uint32_t yo[KSC][4];
#pragma unroll
        for (int p = 0; p < KSC; ++p) {
            const float4 b2a = *reinterpret_cast<const float4 *>(tb + L::T_B2 + 32 * p + 8 * q);
            const float4 b2b = *reinterpret_cast<const float4 *>(tb + L::T_B2 + 32 * p + 8 * q + 4);
            const f32x4 lo = yacc[2 * p], hi = yacc[2 * p + 1];
            yo[p][0] = pack_bf16x2(lo[0] + b2a.x + bf16_lo(x1[p][0]), lo[1] + b2a.y + bf16_hi(x1[p][0]));
            yo[p][1] = pack_bf16x2(lo[2] + b2a.z + bf16_lo(x1[p][1]), lo[3] + b2a.w + bf16_hi(x1[p][1]));
            yo[p][2] = pack_bf16x2(hi[0] + b2b.x + bf16_lo(x1[p][2]), hi[1] + b2b.y + bf16_hi(x1[p][2]));
            yo[p][3] = pack_bf16x2(hi[2] + b2b.z + bf16_lo(x1[p][3]), hi[3] + b2b.w + bf16_hi(x1[p][3]));
        }
        store_rows<KSC>(a.y, t, ok, C, q, yo);
        if (a.xn_out) {
            // the LayerNorm of the layer that follows, taken of y as stored (the padding channels of the lane
            // hold b2 = 0 plus x1 = 0 plus products with zero weight rows: zero)
            layer_norm_rows<KSC>(yo, C, q, a.eps, reinterpret_cast<const float2 *>(tb + L::T_NGB));
            store_rows<KSC>(a.xn_out, t, ok, C, q, yo);
        }
    }
}

// ---------------------------------------------------------------------------------------------------------
// Backward pass, the part between the two LayerNorm adjoints: one launch recomputes LN_2(x1), the
// pre-activation and the hidden layer as the forward does and takes the gradient back to LN_2's output,
//   dh = dy W2,   dpre = dh o GELU'(pre),   dn = dpre W1,
// with the hidden-sized intermediates that nobody else reads (pre, dh) never leaving the registers.  What
// the weight gradients need is written on the way: LN_2(x1), h and dpre; dn goes to LayerNorm's adjoint.
// Same organisation as the forward kernel: 16 tokens per wave, stream units of 64 hidden features holding,
// per step of 32, the fragments of W1 (pre), of W2^T (dh; both with their rows ordered so that a lane's
// results of the step's two tiles are the 8 consecutive features 32 u + 8 q + 0..7: one 16-byte store per
// tensor, and the B operand of the third product as it stands) and of W1^T (dn, rows ordered as W2's in
// the forward).  Values are rounded where the one-kernel-per-step path stores them (pre, dh, h, dpre, dn).
// ---------------------------------------------------------------------------------------------------------
struct WideMlpBwdArgs {
    long rows;
    int C, Hd;
    float eps;
    const bf16_t *x1, *dy;
    const bf16_t *ln_w, *ln_b, *w_fc1, *b_fc1, *w_fc2;
    bf16_t *xn, *h, *dpre, *dn; // LN_2(x1) [rows, C]; h, dpre [rows, Hd]; dn [rows, C] (may be null with dx1)
    // With dx1 non-null the kernel goes on through LayerNorm's adjoint and the skip of Eq. 5:
    //   dx1 = dy + adjoint of LN_2 at x1 applied to dn;  d gamma, d beta of LN_2 are added (atomically, once per
    //   workgroup and channel) into copy (workgroup index mod reps) of `reps` copies rep_stride floats apart, or,
    //   with reps == 0, written as one vector [d gamma: C | d beta: C] per workgroup at dgamma (no atomics; the
    //   caller sums astl_mlp_wide_bwd_blocks() of them).
    bf16_t *dx1;
    float *dgamma, *dbeta;
    long rep_stride;
    int reps;
    void *pack;
};

template <int KSC, int KSF> struct WideMlpBwd {
    static constexpr int CT = 2 * KSC, FT = 2 * KSF;
    static constexpr int HU = 2;
    static_assert(KSF % HU == 0, "whole units");
    static constexpr int FR_STEP = 4 * KSC + CT; // W1: 2 tiles x KSC steps | W2^T: the same | W1^T: CT tiles x 1 step
    static constexpr int FR_UNIT = HU * FR_STEP;
    static constexpr int UNIT_BYTES = FR_UNIT * 1024;
    static constexpr int FPW = (FR_UNIT + kWideWaves - 1) / kWideWaves;
    // tables (floats): b1 [FT * 16] | (gamma, beta) of LN_2 [32 KSC][2]
    static constexpr int T_B1 = 0, T_GB = FT * 16, T_FLOATS = T_GB + 64 * KSC;
    static constexpr size_t P_TABLES = (size_t)(KSF / HU) * UNIT_BYTES;
    static constexpr size_t P_BYTES = P_TABLES + (size_t)T_FLOATS * 4;
    static constexpr int OFF_TABLES = 2 * UNIT_BYTES;
    // sums of LN_2's gamma / beta gradients over the rows a wave has seen: [wave][q][gamma | beta][8 KSC] floats
    static constexpr int OFF_GSUM = OFF_TABLES + T_FLOATS * 4;
    static constexpr int GSUM_FLOATS = kWideWaves * 4 * 2 * 8 * KSC;
    static constexpr size_t LDS_BYTES = (size_t)OFF_GSUM + (size_t)GSUM_FLOATS * 4;
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
    static_assert(T_FLOATS % 4 == 0, "tables are copied in 16-byte pieces");
};

// (runs in the forward call's pack launch: the forward keeps both orders with its saved state)
template <int KSC, int KSF>
__device__ __forceinline__ void wide_bwd_pack_body(const WideMlpBwdArgs &a, int nu)
{
    using L = WideMlpBwd<KSC, KSF>;
    const int C = a.C, Hd = a.Hd;
    uint16_t *d16 = static_cast<uint16_t *>(a.pack);
    const int total = nu * L::FR_UNIT * 512; // (nu units: steps of hidden features beyond the matrix are zero)
    for (int e = blockIdx.x * 256 + threadIdx.x; e < total; e += gridDim.x * 256) {
        const int j = e & 7, l = (e >> 3) & 63, fr = e >> 9;
        const int u = fr / L::FR_STEP, f = fr - u * L::FR_STEP; // u: step of 32 hidden features
        const int m = l & 15, lq = l >> 4;
        float v = 0.f;
        if (f < 4 * KSC) {
            const int g = f < 2 * KSC ? f : f - 2 * KSC;
            const int jt = g / KSC, s = g - jt * KSC;
            const int hid = 32 * u + 8 * (m >> 2) + 4 * jt + (m & 3), ch = 32 * s + 8 * lq + j;
            if (hid < Hd && ch < C) v = f < 2 * KSC ? bfv(a.w_fc1, (long)hid * C + ch) : bfv(a.w_fc2, (long)ch * Hd + hid);
        } else {
            const int ct = f - 4 * KSC;
            const int ch = 32 * (ct >> 1) + 8 * (m >> 2) + 4 * (ct & 1) + (m & 3);
            const int hid = 32 * u + 8 * lq + j;
            if (hid < Hd && ch < C) v = bfv(a.w_fc1, (long)hid * C + ch);
        }
        d16[e] = f32_to_bf16_bits(v);
    }
    float *tb = reinterpret_cast<float *>(static_cast<uint8_t *>(a.pack) + L::P_TABLES);
    for (int i = blockIdx.x * 256 + threadIdx.x; i < L::T_FLOATS; i += gridDim.x * 256) {
        float v = 0.f;
        if (i < L::T_GB) {
            if (i < Hd) v = bfv(a.b_fc1, i);
        } else {
            const int c = (i - L::T_GB) >> 1;
            if (c < C) v = bfv((i & 1) ? a.ln_b : a.ln_w, c);
        }
        tb[i] = v;
    }
}

// a lane's 8 consecutive hidden features f .. f + 7 of row t (Hd is a multiple of 4: a piece is whole, its
// first half, or nothing)
__device__ __forceinline__ void store_hidden(bf16_t *base, long t, bool ok, int Hd, int f, uint4 v)
{
    uint32_t *b32 = reinterpret_cast<uint32_t *>(base) + ((t * Hd + f) >> 1);
    if (ok && f + 8 <= Hd) {
        row16 u;
        u.v[0] = v.x; u.v[1] = v.y; u.v[2] = v.z; u.v[3] = v.w;
        *reinterpret_cast<row16 *>(b32) = u;
    } else if (ok && f + 4 <= Hd) {
        b32[0] = v.x;
        b32[1] = v.y;
    }
}

template <int KSC, int KSF>
__global__ __launch_bounds__(kWideThreads) void astl_mlp_wide_bwd_kernel(WideMlpBwdArgs a, int nu)
{
    using L = WideMlpBwd<KSC, KSF>;
    constexpr int CT = L::CT;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const uint8_t *pack = static_cast<const uint8_t *>(a.pack);
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, tok = lane & 15, q = lane >> 4;
    const int C = a.C, Hd = a.Hd;
    int lane_r = lane;

    auto stream_unit = [&](int u, int slot) {
        int ln = lane_r;
        asm volatile("" : "+v"(ln)); // (the per-fragment addresses are made here, not kept over the unit loop)
        const uint8_t *src = pack + (size_t)u * L::UNIT_BYTES + 16 * ln;
        uint8_t *dst = lds + (size_t)slot * L::UNIT_BYTES;
#pragma unroll 1
        for (int k = 0; k < L::FPW; ++k) { // (not unrolled: one address in registers at a time)
            const int f = k * kWideWaves + wv;
            if (f < L::FR_UNIT) lds_dma16(src + (size_t)f * 1024, dst + (size_t)f * 1024);
        }
    };

    const long ntiles = (a.rows + 15) / 16;
    const long stride = (long)gridDim.x * kWideWaves;
    const int rounds = (int)((ntiles + stride - 1) / stride);
    long tile = (long)blockIdx.x * kWideWaves + wv;

    u32x4 rx[KSC], rd[KSC];
    load_rows<KSC>(a.x1, tile * 16 + tok, a.rows, C, q, rx);
    load_rows<KSC>(a.dy, tile * 16 + tok, a.rows, C, q, rd);

    stream_unit(0, 0);
    for (int i = tid; i < L::T_FLOATS / 4; i += kWideThreads)
        reinterpret_cast<uint4 *>(lds + L::OFF_TABLES)[i] = reinterpret_cast<const uint4 *>(pack + L::P_TABLES)[i];
    for (int i = tid; i < L::GSUM_FLOATS; i += kWideThreads) reinterpret_cast<float *>(lds + L::OFF_GSUM)[i] = 0.f;
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();

    int slot = 0; // buffer the unit about to be used lies in
    for (int round = 0; round < rounds; ++round, tile += stride) {
        const bool more = round + 1 < rounds;
        const long t = tile * 16 + tok;
        const bool ok = t < a.rows;
        uint32_t lds0 = 0;
        asm volatile("" : "+v"(lds0)); // keeps the LDS reads of a round inside the round
        lane_r = lane;
        asm volatile("" : "+v"(lane_r));
        const float *tb = reinterpret_cast<const float *>(lds + lds0 + L::OFF_TABLES);

        // operands of the round: LN_2(x1) (also written out for the weight gradient of the first map) and dy
        uint32_t bx[KSC][4], bd[KSC][4];
        tidy_rows<KSC>(C, q, rx, bx);
        tidy_rows<KSC>(C, q, rd, bd);
        const float2 stats = layer_norm_rows<KSC>(bx, C, q, a.eps, reinterpret_cast<const float2 *>(tb + L::T_GB));
        store_rows<KSC>(a.xn, t, ok, C, q, bx);

        f32x4 dnacc[CT];
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) dnacc[ct] = f32x4{0.f, 0.f, 0.f, 0.f};

        auto unit_steps = [&](int unit) {
            const uint4 *wu = reinterpret_cast<const uint4 *>(lds + lds0 + (size_t)slot * L::UNIT_BYTES);
#pragma unroll
            for (int hs = 0; hs < L::HU; ++hs) {
                const uint4 *ws = wu + hs * L::FR_STEP * 64;
                const int f0 = 32 * (L::HU * unit + hs) + 8 * q; // the lane's hidden features f0 + 0..7 of token tok
                f32x4 p0 = f32x4{0.f, 0.f, 0.f, 0.f}, p1 = p0, d0 = p0, d1 = p0;
#pragma unroll
                for (int s = 0; s < KSC; ++s) {
                    const uint4 b = make_uint4(bx[s][0], bx[s][1], bx[s][2], bx[s][3]);
                    p0 = mma32(ws[s * 64 + lane_r], b, p0);
                    p1 = mma32(ws[(KSC + s) * 64 + lane_r], b, p1);
                }
                const float4 b10 = *reinterpret_cast<const float4 *>(tb + L::T_B1 + f0);
                const float4 b11 = *reinterpret_cast<const float4 *>(tb + L::T_B1 + f0 + 4);
                // pre and dh as the one-kernel-per-step path stores them (rounded)
                const uint32_t pp[4] = {pack_bf16x2(p0[0] + b10.x, p0[1] + b10.y), pack_bf16x2(p0[2] + b10.z, p0[3] + b10.w),
                                        pack_bf16x2(p1[0] + b11.x, p1[1] + b11.y), pack_bf16x2(p1[2] + b11.z, p1[3] + b11.w)};
                __builtin_amdgcn_sched_barrier(0); // (the first product's accumulators are packed before the second's are live)
#pragma unroll
                for (int s = 0; s < KSC; ++s) {
                    const uint4 b = make_uint4(bd[s][0], bd[s][1], bd[s][2], bd[s][3]);
                    d0 = mma32(ws[(2 * KSC + s) * 64 + lane_r], b, d0);
                    d1 = mma32(ws[(3 * KSC + s) * 64 + lane_r], b, d1);
                }
                const uint32_t dd[4] = {pack_bf16x2(d0[0], d0[1]), pack_bf16x2(d0[2], d0[3]),
                                        pack_bf16x2(d1[0], d1[1]), pack_bf16x2(d1[2], d1[3])};
                uint32_t hp[4], gp[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float t0 = bf16_lo(pp[i]), t1 = bf16_hi(pp[i]);
                    float Phi0, phi0, Phi1, phi1;
                    gauss(t0, Phi0, phi0);
                    gauss(t1, Phi1, phi1);
                    hp[i] = pack_bf16x2(t0 * Phi0, t1 * Phi1);
                    gp[i] = pack_bf16x2(bf16_lo(dd[i]) * fmaf(t0, phi0, Phi0), bf16_hi(dd[i]) * fmaf(t1, phi1, Phi1));
                }
                const uint4 hq = make_uint4(hp[0], hp[1], hp[2], hp[3]), gq = make_uint4(gp[0], gp[1], gp[2], gp[3]);
                store_hidden(a.h, t, ok, Hd, f0, hq);
                store_hidden(a.dpre, t, ok, Hd, f0, gq);
#pragma unroll
                for (int ct = 0; ct < CT; ++ct) dnacc[ct] = mma32(ws[(4 * KSC + ct) * 64 + lane_r], gq, dnacc[ct]);
            }
        };

        // first unit of the round: see the forward kernel (the stores of the unit's own steps are younger than
        // the row loads; leaving 2 KSC operations in flight then waits for as many of the row loads as there
        // were stores, whichever way loads and stores are ordered among each other)
        if (nu > 1) stream_unit(1, slot ^ 1);
        else if (more) stream_unit(0, slot ^ 1);
        if (more) {
            const long tn = t + stride * 16;
            load_rows<KSC>(a.x1, tn, a.rows, C, q, rx);
            load_rows<KSC>(a.dy, tn, a.rows, C, q, rd);
        }
        unit_steps(0);
        if (more) __builtin_amdgcn_s_waitcnt(kWaitAllBut2Ksc<KSC>);
        else __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        slot ^= 1;
        for (int unit = 1; unit < nu; ++unit) {
            if (unit + 1 < nu) stream_unit(unit + 1, slot ^ 1);
            else if (more) stream_unit(0, slot ^ 1); // (the first unit of the next round)
            unit_steps(unit);
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
            slot ^= 1;
        }

        // dn as stored: tiles 2p and 2p + 1 hold the lane's channels 32 p + 8 q + 0..3 and + 4..7
        uint32_t dno[KSC][4];
#pragma unroll
        for (int p = 0; p < KSC; ++p) {
            const f32x4 lo = dnacc[2 * p], hi = dnacc[2 * p + 1];
            dno[p][0] = pack_bf16x2(lo[0], lo[1]);
            dno[p][1] = pack_bf16x2(lo[2], lo[3]);
            dno[p][2] = pack_bf16x2(hi[0], hi[1]);
            dno[p][3] = pack_bf16x2(hi[2], hi[3]);
        }
        if (a.dn) store_rows<KSC>(a.dn, t, ok, C, q, dno);
        if (a.dx1) {
            // LayerNorm's adjoint at x1 (re-read: the operand registers held its normalised form) with the skip
            // of Eq. 5:  xh = (x1 - mean) rstd,  g = dn gamma,  dx1 = rstd (g - mean(g) - xh mean(g xh)) + dy;
            // d gamma += dn xh, d beta += dn over the rows (dn as stored: rounded)
            u32x4 rx1[KSC];
            load_rows<KSC>(a.x1, t, a.rows, C, q, rx1);
            uint32_t xr[KSC][4];
            tidy_rows<KSC>(C, q, rx1, xr);
            const float2 *gb = reinterpret_cast<const float2 *>(tb + L::T_GB);
            const float mean = stats.x, rstd = stats.y;
            int qq = q;
            asm volatile("" : "+v"(qq));
            float s1 = 0.f, s2 = 0.f;
#pragma unroll
            for (int p = 0; p < KSC; ++p)
#pragma unroll
                for (int dw = 0; dw < 4; ++dw) {
                    const int c = 32 * p + 8 * qq + 2 * dw;
                    const bool in = c < C;
                    const float4 g = *reinterpret_cast<const float4 *>(gb + c);
                    const float g0 = bf16_lo(dno[p][dw]) * g.x, g1 = bf16_hi(dno[p][dw]) * g.z;
                    const float h0 = in ? (bf16_lo(xr[p][dw]) - mean) * rstd : 0.f;
                    const float h1 = in ? (bf16_hi(xr[p][dw]) - mean) * rstd : 0.f;
                    s1 += g0 + g1;
                    s2 += g0 * h0 + g1 * h1;
                }
            s1 = qgroup_sum(s1) / (float)C;
            s2 = qgroup_sum(s2) / (float)C;
            float *gsum = reinterpret_cast<float *>(lds + lds0 + L::OFF_GSUM) + (wv * 4 + q) * (2 * 8 * KSC);
#pragma unroll
            for (int p = 0; p < KSC; ++p) {
                float pg[8], pb[8];
                uint32_t dxo[4];
#pragma unroll
                for (int dw = 0; dw < 4; ++dw) {
                    const int c = 32 * p + 8 * qq + 2 * dw;
                    const bool in = c < C;
                    const float4 g = *reinterpret_cast<const float4 *>(gb + c);
                    const float d0 = bf16_lo(dno[p][dw]), d1 = bf16_hi(dno[p][dw]);
                    const float h0 = in ? (bf16_lo(xr[p][dw]) - mean) * rstd : 0.f;
                    const float h1 = in ? (bf16_hi(xr[p][dw]) - mean) * rstd : 0.f;
                    dxo[dw] = pack_bf16x2(rstd * (d0 * g.x - s1 - h0 * s2) + bf16_lo(bd[p][dw]),
                                             rstd * (d1 * g.z - s1 - h1 * s2) + bf16_hi(bd[p][dw]));
                    // (rows beyond the last one repeat the last one: they must not be counted)
                    pg[2 * dw] = ok ? d0 * h0 : 0.f; pg[2 * dw + 1] = ok ? d1 * h1 : 0.f;
                    pb[2 * dw] = ok ? d0 : 0.f; pb[2 * dw + 1] = ok ? d1 : 0.f;
                }
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    pg[j] = row_sum_in_last_lane(pg[j]);
                    pb[j] = row_sum_in_last_lane(pb[j]);
                }
                // (in the padding channels dn, gamma, xh and dy are zero: dx1 is -rstd s1 there, not stored)
                store_piece<KSC>(a.dx1, t, ok, C, qq, p, dxo);
                if (tok == 15) { // the row's last lane adds the 16 rows' sums to the wave's own
                    float4 *ag = reinterpret_cast<float4 *>(gsum + 8 * p), *ab = reinterpret_cast<float4 *>(gsum + 8 * KSC + 8 * p);
                    const float4 a0 = ag[0], a1 = ag[1], b0 = ab[0], b1 = ab[1];
                    ag[0] = make_float4(a0.x + pg[0], a0.y + pg[1], a0.z + pg[2], a0.w + pg[3]);
                    ag[1] = make_float4(a1.x + pg[4], a1.y + pg[5], a1.z + pg[6], a1.w + pg[7]);
                    ab[0] = make_float4(b0.x + pb[0], b0.y + pb[1], b0.z + pb[2], b0.w + pb[3]);
                    ab[1] = make_float4(b1.x + pb[4], b1.y + pb[5], b1.z + pb[6], b1.w + pb[7]);
                }
            }
        }
    }
    if (a.dx1) {
        // the waves' sums meet: one atomic add per channel and workgroup into one of the copies
        __syncthreads();
        const float *gs = reinterpret_cast<const float *>(lds + L::OFF_GSUM);
        const long rep = a.reps > 0 ? (long)(blockIdx.x % a.reps) * a.rep_stride : 0;
        for (int i = tid; i < 2 * 32 * KSC; i += kWideThreads) {
            const int which = i / (32 * KSC), c = i - which * (32 * KSC);
            if (c >= C) continue;
            const int p = c >> 5, cq = (c >> 3) & 3, j = c & 7;
            float sum = 0.f;
#pragma unroll
            for (int w = 0; w < kWideWaves; ++w) sum += gs[(w * 4 + cq) * (2 * 8 * KSC) + which * 8 * KSC + 8 * p + j];
            if (a.reps > 0) atomicAdd((which ? a.dbeta : a.dgamma) + rep + c, sum);
            else a.dgamma[(size_t)blockIdx.x * 2 * C + which * C + c] = sum; // the workgroup's own vector [d gamma | d beta]
        }
    }
}

template <int KSC, int KSF>
__global__ __launch_bounds__(256) void astl_mlp_wide_pack_kernel(WideMlpArgs a, int nu, WideMlpBwdArgs b, int nub)
{
    wide_fwd_pack_body<KSC, KSF>(a, nu);
    if (b.pack) wide_bwd_pack_body<KSC, KSF>(b, nub);
}

template <int KSC, int KSF> hipError_t launch_wide_t(const WideMlpArgs &a, hipStream_t s)
{
    using L = WideMlp<KSC, KSF>;
    const int nu = ((a.Hd + 31) / 32 + L::HU - 1) / L::HU; // stream units
    {
        KernelTimer kt(K_MLP_PACK, s);
        WideMlpBwdArgs b{};
        b.C = a.C; b.Hd = a.Hd; b.ln_w = a.ln_w; b.ln_b = a.ln_b; b.w_fc1 = a.w_fc1; b.b_fc1 = a.b_fc1; b.w_fc2 = a.w_fc2;
        b.pack = a.bwd_pack;
        using LB = WideMlpBwd<KSC, KSF>;
        const int nub = ((a.Hd + 31) / 32 + LB::HU - 1) / LB::HU;
        hipLaunchKernelGGL((astl_mlp_wide_pack_kernel<KSC, KSF>), dim3(256), dim3(256), 0, s, a, nu, b, nub);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    auto kern = astl_mlp_wide_fwd_kernel<KSC, KSF>;
    if (hipError_t ea = allow_dynamic_lds(reinterpret_cast<const void *>(kern), L::LDS_BYTES); ea != hipSuccess) return ea;
    const long tiles = (a.rows + 15) / 16;
    long blocks = (tiles + kWideWaves - 1) / kWideWaves;
    if (blocks > device_cu_count()) blocks = device_cu_count(); // (one workgroup of eight waves per compute unit)
    KernelTimer kt(K_MLP_FWD, s);
    hipLaunchKernelGGL(kern, dim3((unsigned)(blocks < 1 ? 1 : blocks)), dim3(kWideThreads), L::LDS_BYTES, s, a, nu);
    return hipGetLastError();
}


template <int KSC, int KSF> hipError_t launch_wide_bwd_t(const WideMlpBwdArgs &a, hipStream_t s)
{
    using L = WideMlpBwd<KSC, KSF>;
    const int nu = ((a.Hd + 31) / 32 + L::HU - 1) / L::HU; // stream units
    auto kern = astl_mlp_wide_bwd_kernel<KSC, KSF>;
    if (hipError_t ea = allow_dynamic_lds(reinterpret_cast<const void *>(kern), L::LDS_BYTES); ea != hipSuccess) return ea;
    KernelTimer kt(K_MLP_BWD, s);
    hipLaunchKernelGGL(kern, dim3((unsigned)astl_mlp_wide_bwd_blocks(a.rows)), dim3(kWideThreads), L::LDS_BYTES, s, a, nu);
    return hipGetLastError();
}


// ---------------------------------------------------------------------------------------------------------
// LayerNorm of bf16 rows in the lane pattern of this file: four lanes per row, 16 rows per wave, every load a
// 16-byte piece that nothing touches until the whole tile of the NEXT iteration is on its way (2 KSC, or with
// a second input 4 KSC, loads in flight per lane: what a streaming kernel needs to reach the memory's rate).
// ---------------------------------------------------------------------------------------------------------
constexpr int kLnRowsThreads = 256;

template <int KSC>
__global__ __launch_bounds__(kLnRowsThreads) void ln_rows_fwd_kernel(LnRowsArgs a)
{
    __shared__ float2 gb[32 * KSC];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, tok = lane & 15, q = lane >> 4;
    const int C = a.C;
    for (int c = tid; c < 32 * KSC; c += kLnRowsThreads)
        gb[c] = c < C ? make_float2(bfv(a.gamma, c), bfv(a.beta, c)) : make_float2(0.f, 0.f);
    const long ntiles = (a.rows + 15) / 16;
    const long stride = (long)gridDim.x * (kLnRowsThreads / 64);
    long tile = (long)blockIdx.x * (kLnRowsThreads / 64) + wv;
    u32x4 ru[KSC], rv[KSC];
    if (tile < ntiles) {
        load_rows<KSC>(a.u, tile * 16 + tok, a.rows, C, q, ru);
        if (a.add) load_rows<KSC>(a.add, tile * 16 + tok, a.rows, C, q, rv);
    }
    __syncthreads();
    for (; tile < ntiles; tile += stride) {
        const long t = tile * 16 + tok;
        const bool ok = t < a.rows;
        uint32_t x[KSC][4];
        tidy_rows<KSC>(C, q, ru, x);
        if (a.add) {
            // the stored (rounded) sum is what gets normalised
            uint32_t v[KSC][4];
            tidy_rows<KSC>(C, q, rv, v);
#pragma unroll
            for (int p = 0; p < KSC; ++p)
#pragma unroll
                for (int dw = 0; dw < 4; ++dw)
                    x[p][dw] = pack_bf16x2(bf16_lo(x[p][dw]) + bf16_lo(v[p][dw]), bf16_hi(x[p][dw]) + bf16_hi(v[p][dw]));
        }
        if (tile + stride < ntiles) { // the next tile's rows are on their way while this one is computed
            load_rows<KSC>(a.u, t + stride * 16, a.rows, C, q, ru);
            if (a.add) load_rows<KSC>(a.add, t + stride * 16, a.rows, C, q, rv);
        }
        if (a.add && a.sum_out) store_rows<KSC>(a.sum_out, t, ok, C, q, x);
        layer_norm_rows<KSC>(x, C, q, a.eps, gb);
        store_rows<KSC>(a.out, t, ok, C, q, x);
    }
}


// LayerNorm's adjoint of the same rows, same lane pattern: with xh = (u - mean) rstd and g = dout gamma,
//   du = rstd (g - mean(g) - xh mean(g xh)) (+ res);   d gamma = sum_t dout xh;   d beta = sum_t dout.
// The sums over rows as in the MLP backward kernel above (row shifts, per-wave sums in LDS); every workgroup
// writes ONE vector [d gamma: C | d beta: C] of its own, which the caller sums in a fixed order: no atomics.
template <int KSC>
__global__ __launch_bounds__(kLnRowsThreads) void ln_rows_bwd_kernel(LnRowsBwdArgs a)
{
    constexpr int NW = kLnRowsThreads / 64;
    __shared__ float gam[32 * KSC];
    __shared__ __attribute__((aligned(16))) float gsum_all[NW * 4 * 2 * 8 * KSC];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, tok = lane & 15, q = lane >> 4;
    const int C = a.C;
    for (int c = tid; c < 32 * KSC; c += kLnRowsThreads) gam[c] = c < C ? bfv(a.gamma, c) : 0.f;
    for (int i = tid; i < NW * 4 * 2 * 8 * KSC; i += kLnRowsThreads) gsum_all[i] = 0.f;
    __syncthreads();
    float *gsum = gsum_all + (wv * 4 + q) * (2 * 8 * KSC);
    const long ntiles = (a.rows + 15) / 16;
    const long stride = (long)gridDim.x * NW;
    for (long tile = (long)blockIdx.x * NW + wv; tile < ntiles; tile += stride) {
        const long t = tile * 16 + tok;
        const bool ok = t < a.rows;
        u32x4 ru[KSC], rd[KSC], rr[KSC];
        load_rows<KSC>(a.u, t, a.rows, C, q, ru);
        load_rows<KSC>(a.dout, t, a.rows, C, q, rd);
        if (a.res) load_rows<KSC>(a.res, t, a.rows, C, q, rr);
        uint32_t xu[KSC][4], xd[KSC][4];
        tidy_rows<KSC>(C, q, ru, xu);
        tidy_rows<KSC>(C, q, rd, xd);
        int qq = q;
        asm volatile("" : "+v"(qq));
        // mean and 1 / sqrt(var + eps) as the forward kernels take them
        float sum = 0.f;
#pragma unroll
        for (int p = 0; p < KSC; ++p)
#pragma unroll
            for (int dw = 0; dw < 4; ++dw) sum += bf16_lo(xu[p][dw]) + bf16_hi(xu[p][dw]);
        const float mean = qgroup_sum(sum) / (float)C;
        float dev = 0.f, s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int p = 0; p < KSC; ++p)
#pragma unroll
            for (int dw = 0; dw < 4; ++dw)
                if (32 * p + 8 * qq + 2 * dw < C) {
                    const float d0 = bf16_lo(xu[p][dw]) - mean, d1 = bf16_hi(xu[p][dw]) - mean;
                    dev += d0 * d0 + d1 * d1;
                }
        const float rstd = rsqrtf(qgroup_sum(dev) / (float)C + a.eps);
#pragma unroll
        for (int p = 0; p < KSC; ++p)
#pragma unroll
            for (int dw = 0; dw < 4; ++dw) {
                const int c = 32 * p + 8 * qq + 2 * dw;
                const bool in = c < C;
                const float2 gm = *reinterpret_cast<const float2 *>(gam + c);
                const float g0 = bf16_lo(xd[p][dw]) * gm.x, g1 = bf16_hi(xd[p][dw]) * gm.y;
                const float h0 = in ? (bf16_lo(xu[p][dw]) - mean) * rstd : 0.f;
                const float h1 = in ? (bf16_hi(xu[p][dw]) - mean) * rstd : 0.f;
                s1 += g0 + g1;
                s2 += g0 * h0 + g1 * h1;
            }
        s1 = qgroup_sum(s1) / (float)C;
        s2 = qgroup_sum(s2) / (float)C;
        uint32_t xr[KSC][4];
        if (a.res) tidy_rows<KSC>(C, q, rr, xr);
#pragma unroll
        for (int p = 0; p < KSC; ++p) {
            float pg[8], pb[8];
            uint32_t duo[4];
#pragma unroll
            for (int dw = 0; dw < 4; ++dw) {
                const int c = 32 * p + 8 * qq + 2 * dw;
                const bool in = c < C;
                const float2 gm = *reinterpret_cast<const float2 *>(gam + c);
                const float d0 = bf16_lo(xd[p][dw]), d1 = bf16_hi(xd[p][dw]);
                const float h0 = in ? (bf16_lo(xu[p][dw]) - mean) * rstd : 0.f;
                const float h1 = in ? (bf16_hi(xu[p][dw]) - mean) * rstd : 0.f;
                float o0 = rstd * (d0 * gm.x - s1 - h0 * s2), o1 = rstd * (d1 * gm.y - s1 - h1 * s2);
                if (a.res) { o0 += bf16_lo(xr[p][dw]); o1 += bf16_hi(xr[p][dw]); }
                duo[dw] = pack_bf16x2(o0, o1);
                // (rows beyond the last one repeat the last one: they must not be counted)
                pg[2 * dw] = ok ? d0 * h0 : 0.f; pg[2 * dw + 1] = ok ? d1 * h1 : 0.f;
                pb[2 * dw] = ok ? d0 : 0.f; pb[2 * dw + 1] = ok ? d1 : 0.f;
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                pg[j] = row_sum_in_last_lane(pg[j]);
                pb[j] = row_sum_in_last_lane(pb[j]);
            }
            store_piece<KSC>(a.du, t, ok, C, qq, p, duo);
            if (tok == 15) { // the row's last lane adds the 16 rows' sums to the wave's own
                float4 *ag = reinterpret_cast<float4 *>(gsum + 8 * p), *ab = reinterpret_cast<float4 *>(gsum + 8 * KSC + 8 * p);
                const float4 a0 = ag[0], a1 = ag[1], b0 = ab[0], b1 = ab[1];
                ag[0] = make_float4(a0.x + pg[0], a0.y + pg[1], a0.z + pg[2], a0.w + pg[3]);
                ag[1] = make_float4(a1.x + pg[4], a1.y + pg[5], a1.z + pg[6], a1.w + pg[7]);
                ab[0] = make_float4(b0.x + pb[0], b0.y + pb[1], b0.z + pb[2], b0.w + pb[3]);
                ab[1] = make_float4(b1.x + pb[4], b1.y + pb[5], b1.z + pb[6], b1.w + pb[7]);
            }
        }
    }
    __syncthreads();
    for (int i = tid; i < 2 * 32 * KSC; i += kLnRowsThreads) {
        const int which = i / (32 * KSC), c = i - which * (32 * KSC);
        if (c >= C) continue;
        const int p = c >> 5, cq = (c >> 3) & 3, j = c & 7;
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) sum += gsum_all[(w * 4 + cq) * (2 * 8 * KSC) + which * 8 * KSC + 8 * p + j];
        a.part[(size_t)blockIdx.x * 2 * C + which * C + c] = sum;
    }
}

} // namespace

bool astl_mlp_wide_supported(int C, int hidden)
{
    return C > 64 && C <= 192 && C % 4 == 0 && hidden >= 32 && hidden <= 384 && hidden % 4 == 0;
}

size_t astl_mlp_wide_pack_bytes() { return (WideMlp<6, 12>::P_BYTES + 255) & ~size_t(255); }

hipError_t launch_astl_mlp_wide_fwd(long rows, int C, int hidden, float eps, const bf16_t *x, const bf16_t *a,
                                    const bf16_t *ln_w, const bf16_t *ln_b, const bf16_t *w_fc1, const bf16_t *b_fc1,
                                    const bf16_t *w_fc2, const bf16_t *b_fc2, bf16_t *x1, bf16_t *y, void *pack,
                                    void *bwd_pack, const bf16_t *next_ln_w, const bf16_t *next_ln_b,
                                    bf16_t *next_ln_out, hipStream_t s)
{
    if (!astl_mlp_wide_supported(C, hidden) || rows <= 0) return hipErrorInvalidValue;
    WideMlpArgs m{};
    m.bwd_pack = bwd_pack;
    m.rows = rows; m.C = C; m.Hd = hidden; m.eps = eps;
    m.x = x; m.a = a; m.ln_w = ln_w; m.ln_b = ln_b; m.w_fc1 = w_fc1; m.b_fc1 = b_fc1; m.w_fc2 = w_fc2; m.b_fc2 = b_fc2;
    m.x1 = x1; m.y = y; m.pack = pack;
    if (next_ln_out && next_ln_w && next_ln_b) {
        m.nxt_w = next_ln_w; m.nxt_b = next_ln_b; m.xn_out = next_ln_out;
    }
    if (C <= 128) return launch_wide_t<4, 12>(m, s);
    return launch_wide_t<6, 12>(m, s);
}

size_t astl_mlp_wide_bwd_pack_bytes() { return (WideMlpBwd<6, 12>::P_BYTES + 255) & ~size_t(255); }

hipError_t launch_astl_mlp_wide_bwd(long rows, int C, int hidden, float eps, const bf16_t *x1, const bf16_t *dy,
                                    const bf16_t *ln_w, const bf16_t *ln_b, const bf16_t *w_fc1, const bf16_t *b_fc1,
                                    const bf16_t *w_fc2, bf16_t *xn, bf16_t *h, bf16_t *dpre, bf16_t *dn, bf16_t *dx1,
                                    float *dln_w, float *dln_b, long rep_stride, int reps, const void *pack,
                                    hipStream_t s)
{
    if (!astl_mlp_wide_supported(C, hidden) || rows <= 0) return hipErrorInvalidValue;
    WideMlpBwdArgs m{};
    m.rows = rows; m.C = C; m.Hd = hidden; m.eps = eps;
    m.x1 = x1; m.dy = dy; m.ln_w = ln_w; m.ln_b = ln_b; m.w_fc1 = w_fc1; m.b_fc1 = b_fc1; m.w_fc2 = w_fc2;
    m.xn = xn; m.h = h; m.dpre = dpre; m.dn = dn; m.pack = const_cast<void *>(pack);
    if ((!dn && !dx1) || (dx1 && (!dln_w || reps < 0 || (reps > 0 && !dln_b)))) return hipErrorInvalidValue;
    m.dx1 = dx1; m.dgamma = dln_w; m.dbeta = dln_b; m.rep_stride = rep_stride; m.reps = reps;
    if (C <= 128) return launch_wide_bwd_t<4, 12>(m, s);
    return launch_wide_bwd_t<6, 12>(m, s);
}

// (narrow layers keep the 16-lanes-per-row kernel in both passes: at 60 channels this one is no faster, and the
// backward's recomputation of LN_1, which shares a launch with the fused MLP's final sum there, must round as
// the forward did)
bool ln_rows_supported(int C) { return C > 64 && C <= 192 && C % 4 == 0; }

int astl_mlp_wide_bwd_blocks(long rows)
{
    const long tiles = (rows + 15) / 16;
    long blocks = (tiles + kWideWaves - 1) / kWideWaves;
    if (blocks > device_cu_count()) blocks = device_cu_count();
    return (int)(blocks < 1 ? 1 : blocks);
}

int ln_rows_bwd_blocks(long rows)
{
    const long tiles = (rows + 15) / 16;
    long blocks = (tiles + kLnRowsThreads / 64 - 1) / (kLnRowsThreads / 64);
    const long cap = 4L * device_cu_count();
    if (blocks > cap) blocks = cap;
    return (int)(blocks < 1 ? 1 : blocks);
}

hipError_t launch_ln_rows_bwd(const LnRowsBwdArgs &a, hipStream_t s)
{
    if (!ln_rows_supported(a.C) || a.rows <= 0 || !a.part) return hipErrorInvalidValue;
    const dim3 grid((unsigned)ln_rows_bwd_blocks(a.rows)), block(kLnRowsThreads);
    if (a.C <= 128) hipLaunchKernelGGL(ln_rows_bwd_kernel<4>, grid, block, 0, s, a);
    else hipLaunchKernelGGL(ln_rows_bwd_kernel<6>, grid, block, 0, s, a);
    return hipGetLastError();
}

hipError_t launch_ln_rows_fwd(const LnRowsArgs &a, hipStream_t s)
{
    if (!ln_rows_supported(a.C) || a.rows <= 0) return hipErrorInvalidValue;
    const long tiles = (a.rows + 15) / 16;
    long blocks = (tiles + kLnRowsThreads / 64 - 1) / (kLnRowsThreads / 64);
    const long cap = 8L * device_cu_count(); // (eight workgroups of four waves per compute unit: one pass at 131072 rows)
    if (blocks > cap) blocks = cap;
    const dim3 grid((unsigned)blocks), block(kLnRowsThreads);
    if (a.C <= 128) hipLaunchKernelGGL(ln_rows_fwd_kernel<4>, grid, block, 0, s, a);
    else hipLaunchKernelGGL(ln_rows_fwd_kernel<6>, grid, block, 0, s, a);
    return hipGetLastError();
}

} // namespace gswa
