// Backward of wide GSWA layers (C = 180, six heads of 30 channels, 8x8 windows, two or three
// groups) through the attention and the QKV projection, group by group in reverse order (Eq. 8 hands
// the gradient of a group's input to the output of the group before it).  Two launches per group:
//
// wide_attn_bwd_kernel: one wavefront per window, as in the forward (wide_fwd.hip): four waves per
//   workgroup, one per SIMD, the weights streamed through LDS as equal units, double buffered, one
//   workgroup barrier per unit.  Per window: dO of the group's heads = dy Wproj (adjoint of Eq. 7) plus
//   the cascade gradient (the dx slice of the next group, already final); then per head q, k, v, the
//   scores and the softmax are recomputed exactly as the forward computes them (same operands, base-2
//   units, same mask), and dP, dS, dQ, dK, dV follow.  Nothing crosses waves: the products that reduce
//   over queries take P and dS transposed by the matrix cores (a packed tile times the identity).
//   d(q|k|v) leaves as MFMA operand fragments, 1 KB per (16 tokens, head, q|k|v), stored with whole
//   cache lines.  The bias-table gradient of a head is folded from its (query, key) form to the
//   (2M-1)^2 offsets through a private piece of LDS and kept in registers across the windows of a wave.
//
// wide_qkv_grad_kernel: one workgroup per window (one wave per 16 tokens), plain GEMM work: the
//   group's dx slice = d(q|k|v) Wqkv, and d w_qkv, d b_qkv = d(q|k|v)^T [F | 1] accumulated in
//   registers over the windows of a workgroup (F = x slice + previous group's output, Eq. 8).
//
// Notation (T-form, N-form, head-padded order): fused_bwd.hip, wide_fwd.hip.
#include "fused.h"
#include "mfma.h"
#include "wide_rows.h"

namespace gswa {

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kMaskLog2 = -100.0f * kLog2e; // the additive -100 of the shift mask, in base-2 units

template <class Cf> struct WideBwdCfg {
    static constexpr int NWAVES = 4, NTHREADS = 64 * NWAVES;
    static constexpr int NTBL = 15 * 15;
    // stream units: the Wproj^T fragments of the group's heads in two halves, then per head its QKV fragments
    static constexpr int FR_UNIT = 3 * Cf::ET * Cf::KS;
    static constexpr size_t UNIT_BYTES = (size_t)FR_UNIT * 1024;
    static constexpr int NAU = 2;
    static constexpr int NU = NAU + Cf::HG;
    static constexpr int TILES_AU = FR_UNIT / Cf::KSC;             // (head, feature tile) pairs of dO per unit
    static_assert(Cf::HG * Cf::ET * Cf::KSC == NAU * FR_UNIT && FR_UNIT % Cf::KSC == 0, "dO units");
    static constexpr int FPW = (FR_UNIT + NWAVES - 1) / NWAVES;    // fragments a wave moves per unit
    static constexpr size_t OFF_BIAS = 0;                          // fp32 b_qkv [3C] (b_proj [C] behind it)
    static constexpr size_t OFF_TBL = (size_t)16 * Cf::C;          // fp32 [HG][TBW_PITCH], base-2 units: the group's heads
    static constexpr size_t OFF_FOLD = OFF_TBL + (size_t)Cf::HG * Cf::TBW_PITCH * 4; // per wave 28 x 64 fp32
    static constexpr size_t FOLD_BYTES = (size_t)28 * 64 * 4;
    static constexpr size_t OFF_W = OFF_FOLD + NWAVES * FOLD_BYTES;
    // per wave: the dy rows of its window as they lie in memory (64 tokens x C channels, image row after
    // image row), fetched ahead by direct-to-LDS loads; a few bytes of slack behind the last row, where the
    // operand reads of the zero-padded last K step reach
    static constexpr size_t STAGE_BYTES = WindowRows<Cf::C>::BYTES;
    static constexpr size_t OFF_STAGE = OFF_W + 2 * UNIT_BYTES;
    static constexpr size_t LDS_BYTES = OFF_STAGE + NWAVES * STAGE_BYTES;
    static_assert(OFF_W % 16 == 0 && OFF_STAGE % 16 == 0 && STAGE_BYTES % 16 == 0, "16-byte pieces");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
    static_assert(Cf::ET == 2 && Cf::D + 1 <= 32 && Cf::CG % Cf::D == 0, "heads of 17..31 channels");
    static_assert(NWAVES == 4, "the table sums of four waves are added pairwise");
    // d(q|k|v) in scratch: fragment ((window * 4 + token tile) * HG + head of the group) * 3 + (q|k|v)
    static constexpr int FR_TILE = Cf::HG * 3;
    // second kernel
    static constexpr int KS = Cf::KS;                  // K=32 steps over the group's channels, natural order
    static constexpr int CT = Cf::CG / 16 + 1;         // column tiles of d w_qkv, column CG carries the bias sums
    static constexpr int CTF = Cf::CTF;                // 16-channel tiles of the dx slice
    static constexpr int FT = Cf::HG * 3 * Cf::ET;     // 16-row tiles of d(q|k|v), head width padded to 32
    static constexpr int G_WAVES = 8;                  // two windows at a time
    static constexpr int G_RW = (FT + G_WAVES - 1) / G_WAVES;
    static constexpr int G_LW = 136;                   // pitch (bf16) of the [row][128 tokens] buffers (68 dwords:
                                                       // the 16 rows of an operand read fall on distinct banks)
    static constexpr size_t G_OFF_WQX = 0;
    static constexpr size_t G_OFF_G = (size_t)Cf::HG * 3 * CTF * 1024;
    static constexpr size_t G_OFF_F = G_OFF_G + (size_t)FT * 16 * G_LW * 2;
    static constexpr size_t G_LDS_BYTES = G_OFF_F + (size_t)CT * 16 * G_LW * 2;
    static_assert(G_LDS_BYTES <= 160 * 1024, "LDS budget");
    static constexpr int L_DW = 0, L_DB = 3 * Cf::CG * Cf::CG, L_END = L_DB + 3 * Cf::CG;
    static constexpr int L_TOTAL = (L_END + 3) & ~3; // stride of the partial vectors: whole 16-byte pieces
};

// transposes a packed 16x16 tile on the matrix cores: the tile as the A operand (row l16, k-slots
// 4q..4q+3) times the identity is the tile with rows and columns exchanged, exactly
__device__ __forceinline__ uint2 transpose_tile(uint2 tile, uint2 ident)
{
    return pack_bf16x4(mma16(tile, ident, f32x4{0.f, 0.f, 0.f, 0.f}));
}

template <class Cf, int GI>
__global__ __launch_bounds__(256, 1) void wide_attn_bwd_kernel(Geom g, const bf16_t *__restrict__ x,
                                                               const bf16_t *__restrict__ dy,
                                                               const bf16_t *__restrict__ attn,
                                                               const uint8_t *__restrict__ pack,
                                                               const uint8_t *__restrict__ cgf,
                                                               uint8_t *__restrict__ dqkv, uint8_t *__restrict__ ffr,
                                                               float *__restrict__ tpart)
{
    using W = WideBwdCfg<Cf>;
    constexpr int C = Cf::C, D = Cf::D, CG = Cf::CG, HG = Cf::HG, HEADS = Cf::HEADS, G = Cf::G;
    constexpr int KS = Cf::KS, KSC = Cf::KSC, TP = Cf::TBW_PITCH, NU = W::NU, NTBL = W::NTBL;
    constexpr int M = 8;

    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, q = lane >> 4;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int s = g.shift;
    const int cn = l16 & 7, rsub = l16 >> 3;
    const int per_img = g.nwi * g.nwj;
    const uint32_t tbytes = (uint32_t)g.T * (2u * C);
    const buf_t xbuf = make_buf(x, tbytes), abuf = make_buf(attn, tbytes);
    const bool casc_in = GI > 0 && g.cascade, casc_out = GI < G - 1 && g.cascade;

    // The lane index as the address arithmetic of a round sees it: opaque, re-made every round, so that
    // the per-lane addresses of a round's loads are computed where they are used and not kept (and
    // spilled) across the whole kernel.
    int lane_r = lane;
    // ---- weight stream (see wide_fwd.hip): loads that write LDS directly, one fragment per instruction ----
    auto stream_unit = [&](int u, int slot) {
        const size_t from = u < W::NAU ? Cf::P_WPT + ((size_t)GI * HG * Cf::ET * KSC + (size_t)u * W::FR_UNIT) * 1024
                                       : Cf::P_WQN + ((size_t)GI * HG + (u - W::NAU)) * W::UNIT_BYTES;
        const uint8_t *src = pack + from + 16 * lane_r;
        uint8_t *dst = lds + W::OFF_W + (size_t)slot * W::UNIT_BYTES;
#pragma unroll
        for (int k = 0; k < W::FPW; ++k) {
            const int f = k * W::NWAVES + wv;
            if (f < W::FR_UNIT) lds_dma16(src + (size_t)f * 1024, dst + (size_t)f * 1024);
        }
    };

    const int stride = W::NWAVES * (int)gridDim.x;
    const int rounds = (g.nW + stride - 1) / stride;
    uint32_t tok[4];
    bool lastrow = false, lastcol = false;
    auto window_tokens = [&](int win, uint32_t (&tk)[4], bool edges) {
        const int b = win / per_img;
        const int wr = win - b * per_img;
        const int wi = wr / g.nwj, wj = wr - wi * g.nwj;
        if (edges) {
            lastrow = s > 0 && wi == g.nwi - 1;
            lastcol = s > 0 && wj == g.nwj - 1;
        }
        int sj = wj * M + cn + s;
        if (sj >= g.W) sj -= g.W;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            int si = wi * M + 2 * t + rsub + s;
            if (si >= g.H) si -= g.H;
            tk[t] = (uint32_t)((((b * g.H + si) * g.W) + sj) * C) * 2u;
        }
    };

    // dy rows of a window -> this wave's staging buffer, in memory order (wide_rows.h)
    uint8_t *stage = lds + W::OFF_STAGE + (size_t)wv * W::STAGE_BYTES;
    auto fetch_dy = [&](int win_) { fetch_window_rows<C>(g, dy, win_, lane_r, stage); };
    // F = x slice (+ previous group's output, Eq. 8) as operands, channels in their own order: K = 32 steps,
    // lane group q holds channels 32 ks + 8 q .. + 7 (one 16-byte piece of the row)
    uint4 xh[KS][4];
    uint4 ah[KS][4]; // the previous group's output, added when the loads have landed
    auto load_x = [&](const uint32_t (&tk)[4]) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                xh[ks][t] = bload128(xbuf, tk[t] + 2u * (GI * CG) + 64u * ks + 16u * q, 0u);
                if (casc_in) ah[ks][t] = bload128(abuf, tk[t] + 2u * ((GI > 0 ? GI - 1 : 0) * CG) + 64u * ks + 16u * q, 0u);
            }
    };
    auto add_cascade = [&]() { // and the channels past the group's width, which belong to the next slice, cleared
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                uint4 v = xh[ks][t];
                if (casc_in) {
                    const uint4 a = ah[ks][t];
                    v.x = add_bf16x2(v.x, a.x);
                    v.y = add_bf16x2(v.y, a.y);
                    v.z = add_bf16x2(v.z, a.z);
                    v.w = add_bf16x2(v.w, a.w);
                }
                const int c0 = 32 * ks + 8 * q;
                if (32 * ks + 32 > CG) {
                    v.x = c0 < CG ? v.x : 0u;
                    v.y = c0 + 2 < CG ? v.y : 0u;
                    v.z = c0 + 4 < CG ? v.z : 0u;
                    v.w = c0 + 6 < CG ? v.w : 0u;
                }
                xh[ks][t] = v;
            }
    };

    int win = wv * (int)gridDim.x + (int)blockIdx.x;
    bool active = win < g.nW;

    // set-up: dy of the first window, first unit, linear biases, the bias table of the group's heads
    if (active) fetch_dy(win);
    stream_unit(0, 0);
    for (int i = tid; i < C; i += W::NTHREADS)
        reinterpret_cast<uint4 *>(lds + W::OFF_BIAS)[i] = reinterpret_cast<const uint4 *>(pack + Cf::P_BIAS)[i];
    for (int i = tid; i < HG * TP / 4; i += W::NTHREADS)
        reinterpret_cast<uint4 *>(lds + W::OFF_TBL)[i] =
            reinterpret_cast<const uint4 *>(pack + Cf::P_TBW + (size_t)GI * HG * TP * 4)[i];
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();

    // this lane's query column (rn = 2nt + rsub, cn) against key rows 4q+j of key tile kt:
    // key (2kt + q/2, 4(q%2) + j); table entry = tb0 + 30(nt - kt) - j
    const int tb0 = (rsub - (q >> 1) + M - 1) * (2 * M - 1) + (cn - 4 * (q & 1) + M - 1);
    const bool qc_w = cn >= M - s;
    bool kc_w[4], qr_w[4], kr_w[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) kc_w[j] = (4 * (q & 1) + j) >= M - s;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        qr_w[t] = (2 * t + rsub) >= M - s;
        kr_w[t] = (2 * t + (q >> 1)) >= M - s;
    }
    const f32x4 zero4 = f32x4{0.f, 0.f, 0.f, 0.f};
    uint2 ident; // identity as a K=16 operand: index l16, k-slots 4q+j
    {
        const uint32_t one = 0x3f80u;
        const int d0 = l16 - 4 * q;
        ident.x = (d0 == 0 ? one : 0u) | (d0 == 1 ? one << 16 : 0u);
        ident.y = (d0 == 2 ? one : 0u) | (d0 == 3 ? one << 16 : 0u);
    }
    // Table-gradient fold.  A lane's sums of dS over the score tiles with the same offset nt - kt cover
    // 28 (query, key) offset pairs; they are kept in the wave's piece of LDS, [offset][lane][j], and at
    // the end of a head lane l collects table entries l, l + 64, ...: entry 15 (dr + 7) + (dc + 7)
    // receives, from the lanes with 2 (dl - 3) + rsub - q/2 = dr, the slots with cn - 4 (q%2) - j = dc.
    float *fold = reinterpret_cast<float *>(lds + W::OFF_FOLD + (size_t)wv * W::FOLD_BYTES);
    f32x4 *fold4 = reinterpret_cast<f32x4 *>(fold);
    f32x4 facc[HG][7];
#pragma unroll
    for (int hl = 0; hl < HG; ++hl)
#pragma unroll
        for (int dl = 0; dl < 7; ++dl) facc[hl][dl] = f32x4{0.f, 0.f, 0.f, 0.f};

    int par = 0; // LDS buffer of the first unit of this round
    for (int round = 0; round < rounds; ++round) {
        const bool more = round + 1 < rounds;
        if (active) {
            window_tokens(win, tok, true);
            // (the rows of a later window are on their way since the last head of the window before)
            if (round == 0) load_x(tok); // lands under the dO products
        }
        uint2 dOb[HG][2][4]; // dO^T of the group's heads, packed T-form tiles

        uint32_t lds0 = 0;
        asm volatile("" : "+v"(lds0)); // keeps the LDS reads of a round inside the round
        lane_r = lane;
        asm volatile("" : "+v"(lane_r));
        const float *bqkv = reinterpret_cast<const float *>(lds + lds0 + W::OFF_BIAS);
        const float *tbl = reinterpret_cast<const float *>(lds + lds0 + W::OFF_TBL);
        uint8_t *dq_win = dqkv + (size_t)win * 4 * W::FR_TILE * 1024 + 16 * lane_r;
        const uint8_t *cg_win = cgf + (size_t)win * 4 * HG * 1024 + 16 * lane_r;

        static_for<NU>([&](auto u_) {
            constexpr int u = decltype(u_)::value;
            const uint4 *wu = reinterpret_cast<const uint4 *>(lds + lds0 + W::OFF_W + (size_t)((u + par) & 1) * W::UNIT_BYTES);
            // next unit on its way into the other buffer: every wave has passed the previous barrier,
            // i.e. finished reading it
            if (u + 1 < NU) stream_unit(u + 1, (u + 1 + par) & 1);
            else if (more) stream_unit(0, (NU + par) & 1);

            if constexpr (u < W::NAU) {
                // ---- dO^T = Wproj^T dY^T + cascade gradient (the dx slice of the next group): rows = head
                // features, column = token ----
                if (active) {
                    uint2 cg[W::TILES_AU][4];
#pragma unroll
                    for (int i = 0; i < W::TILES_AU; ++i) {
                        const int ti = u * W::TILES_AU + i, hl = ti / 2, et = ti % 2;
#pragma unroll
                        for (int t = 0; t < 4; ++t) {
                            uint2 v = make_uint2(0u, 0u);
                            if (casc_out) // the next group's dF in the layout of this accumulator (its second kernel left it)
                                v = *reinterpret_cast<const uint2 *>(cg_win + (size_t)(t * HG + hl) * 1024 + 8 * et);
                            cg[i][t] = v;
                        }
                    }
                    // one K step of dy (read from the staging buffer as operands, channels 32 ks + 8 q ..) serves
                    // every tile of the unit
                    f32x4 acc[W::TILES_AU][4];
#pragma unroll
                    for (int i = 0; i < W::TILES_AU; ++i)
#pragma unroll
                        for (int t = 0; t < 4; ++t) acc[i][t] = zero4;
                    const uint8_t *dyrow = stage + lds0 + (size_t)(rsub * M + cn) * (2 * C) + 16 * q;
#pragma unroll
                    for (int ks = 0; ks < KSC; ++ks) {
                        uint4 dyf[4];
#pragma unroll
                        for (int t = 0; t < 4; ++t) {
                            const uint8_t *p = dyrow + (size_t)t * (2 * M * 2 * C) + 64 * ks;
                            const uint2 lo = *reinterpret_cast<const uint2 *>(p);
                            const uint2 hi = *reinterpret_cast<const uint2 *>(p + 8);
                            uint4 v = cat(lo, hi);
                            const int c0 = 32 * ks + 8 * q; // first channel of this lane's slots
                            if (32 * ks + 32 > C) {
                                v.x = c0 < C ? v.x : 0u;
                                v.y = c0 + 2 < C ? v.y : 0u;
                                v.z = c0 + 4 < C ? v.z : 0u;
                                v.w = c0 + 6 < C ? v.w : 0u;
                            }
                            dyf[t] = v;
                        }
#pragma unroll
                        for (int i = 0; i < W::TILES_AU; ++i) {
                            const uint4 wf = wu[(i * KSC + ks) * 64 + lane];
#pragma unroll
                            for (int t = 0; t < 4; ++t) acc[i][t] = mma32(wf, dyf[t], acc[i][t]);
                        }
                    }
#pragma unroll
                    for (int i = 0; i < W::TILES_AU; ++i) {
                        const int ti = u * W::TILES_AU + i, hl = ti / 2, et = ti % 2;
#pragma unroll
                        for (int t = 0; t < 4; ++t) {
                            const uint2 c = cg[i][t];
                            acc[i][t] += f32x4{bf16_lo(c.x), bf16_hi(c.x), bf16_lo(c.y), bf16_hi(c.y)};
                            dOb[hl][et][t] = pack_bf16x4(acc[i][t]);
                        }
                    }
                }
            } else {
                constexpr int hl = u - W::NAU;
                if (hl == 0) {
                    // the staging buffer is free (the dO units are done): dy of this wave's next window
                    if (more && win + stride < g.nW) fetch_dy(win + stride);
                    if (active) {
                        add_cascade();
                        // F as the second kernel's operand of the weight gradient: the same fragments
                        uint4 *fdst = reinterpret_cast<uint4 *>(ffr + (size_t)win * 4 * KS * 1024) + lane_r;
#pragma unroll
                        for (int t = 0; t < 4; ++t)
#pragma unroll
                            for (int ks = 0; ks < KS; ++ks) fdst[(t * KS + ks) * 64] = xh[ks][t];
                    }
                }
                if (active) {
                    // ---- Q^T, K^T, V^T exactly as the forward computes them (rows = head features) ----
                    uint2 Qb[2][4], Kb[2][4], Vb[2][4];
#pragma unroll
                    for (int t3 = 0; t3 < 3; ++t3) {
                        f32x4 acc[2][4];
#pragma unroll
                        for (int et = 0; et < 2; ++et) {
                            f32x4 b4;
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                const int e = 16 * et + 4 * q + j;
                                const float bv = e < D ? bqkv[GI * 3 * CG + t3 * CG + hl * D + e] : 0.f;
                                b4[j] = t3 == 0 ? bv * kLog2e : bv;
                            }
#pragma unroll
                            for (int t = 0; t < 4; ++t) acc[et][t] = b4;
                        }
#pragma unroll
                        for (int ks = 0; ks < KS; ++ks) {
                            const uint4 f0 = wu[((t3 * 2 + 0) * KS + ks) * 64 + lane];
                            const uint4 f1 = wu[((t3 * 2 + 1) * KS + ks) * 64 + lane];
#pragma unroll
                            for (int t = 0; t < 4; ++t) {
                                acc[0][t] = mma32(f0, xh[ks][t], acc[0][t]);
                                acc[1][t] = mma32(f1, xh[ks][t], acc[1][t]);
                            }
                        }
#pragma unroll
                        for (int et = 0; et < 2; ++et)
#pragma unroll
                            for (int t = 0; t < 4; ++t) {
                                const uint2 pk = pack_bf16x4(acc[et][t]);
                                if (t3 == 0) Qb[et][t] = pk;
                                else if (t3 == 1) Kb[et][t] = pk;
                                else Vb[et][t] = pk;
                            }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    if (hl == HG - 1 && more && win + stride < g.nW) {
                        // F has served its last product of this window: the x slice and the cascade input of this
                        // wave's next window go into the same registers, with the rest of the head to land
                        uint32_t tkn[4];
                        window_tokens(win + stride, tkn, false);
                        load_x(tkn);
                    }
                    // N-form (rows = tokens, column = feature) of K for dQ
                    uint2 KN[2][4];
#pragma unroll
                    for (int et = 0; et < 2; ++et)
#pragma unroll
                        for (int t = 0; t < 4; ++t) KN[et][t] = transpose_tile(Kb[et][t], ident);
                    f32x4 dkT[2][4], dvT[2][4];
#pragma unroll
                    for (int et = 0; et < 2; ++et)
#pragma unroll
                        for (int t = 0; t < 4; ++t) dkT[et][t] = dvT[et][t] = zero4;
#pragma unroll
                    for (int p2 = 0; p2 < 2; ++p2) {
                        // N-forms of Q and dO of this pair of query tiles, for dK and dV
                        uint4 qn[2], on[2];
#pragma unroll
                        for (int et = 0; et < 2; ++et) {
                            qn[et] = cat(transpose_tile(Qb[et][2 * p2], ident), transpose_tile(Qb[et][2 * p2 + 1], ident));
                            on[et] = cat(transpose_tile(dOb[hl][et][2 * p2], ident),
                                         transpose_tile(dOb[hl][et][2 * p2 + 1], ident));
                        }
                        uint2 Pq[4][2], dSq[4][2]; // P and dS with rows = queries, column = key
                        // ---- S^T, P^T, dP^T, dS^T of the pair's two query tiles (rows = keys 16kt+4q+j, column =
                        // query), every stage for both tiles: two independent chains to overlap ----
                        f32x4 st[2][4], dp[2][4];
#pragma unroll
                        for (int ni = 0; ni < 2; ++ni) {
                            const int nt = 2 * p2 + ni;
                            const uint4 qop = cat(Qb[0][nt], Qb[1][nt]);
                            const uint4 oop = cat(dOb[hl][0][nt], dOb[hl][1][nt]);
#pragma unroll
                            for (int kt = 0; kt < 4; ++kt) {
                                f32x4 bt;
#pragma unroll
                                for (int j = 0; j < 4; ++j) bt[j] = tbl[hl * TP + tb0 + 30 * (nt - kt) - j];
                                st[ni][kt] = mma32(cat(Kb[0][kt], Kb[1][kt]), qop, bt);
                                dp[ni][kt] = mma32(cat(Vb[0][kt], Vb[1][kt]), oop, zero4);
                            }
                        }
                        if (lastrow || lastcol) {
#pragma unroll
                            for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                                for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                                    for (int j = 0; j < 4; ++j)
                                        if ((lastrow && qr_w[2 * p2 + ni] != kr_w[kt]) || (lastcol && qc_w != kc_w[j]))
                                            st[ni][kt][j] += kMaskLog2;
                        }
                        float mx[2], sum[2], dlt[2];
#pragma unroll
                        for (int ni = 0; ni < 2; ++ni) {
                            float m0 = fmaxf(fmaxf(st[ni][0][0], st[ni][0][1]), fmaxf(st[ni][0][2], st[ni][0][3]));
#pragma unroll
                            for (int kt = 1; kt < 4; ++kt)
#pragma unroll
                                for (int j = 0; j < 4; j += 2) m0 = fmaxf(fmaxf(m0, st[ni][kt][j]), st[ni][kt][j + 1]);
                            mx[ni] = m0;
                        }
#pragma unroll
                        for (int ni = 0; ni < 2; ++ni) mx[ni] = qgroup_max(mx[ni]);
#pragma unroll
                        for (int ni = 0; ni < 2; ++ni) {
                            float a = 0.f, b = 0.f;
#pragma unroll
                            for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                                for (int j = 0; j < 4; ++j) {
                                    const float p = __builtin_amdgcn_exp2f(st[ni][kt][j] - mx[ni]);
                                    st[ni][kt][j] = p;
                                    a += p;
                                    b = fmaf(p, dp[ni][kt][j], b);
                                }
                            sum[ni] = a;
                            dlt[ni] = b;
                        }
#pragma unroll
                        for (int ni = 0; ni < 2; ++ni) {
                            sum[ni] = qgroup_sum(sum[ni]);
                            dlt[ni] = qgroup_sum(dlt[ni]);
                        }
                        uint2 Pb[2][4], dSb[2][4];
#pragma unroll
                        for (int ni = 0; ni < 2; ++ni) {
                            const int nt = 2 * p2 + ni;
                            const float inv = __builtin_amdgcn_rcpf(sum[ni]);
                            const float delta = dlt[ni] * inv; // sum over keys of P dP
#pragma unroll
                            for (int kt = 0; kt < 4; ++kt) {
#pragma unroll
                                for (int j = 0; j < 4; ++j) {
                                    const float p = st[ni][kt][j] * inv;
                                    st[ni][kt][j] = p;
                                    dp[ni][kt][j] = p * (dp[ni][kt][j] - delta);
                                }
                                Pb[ni][kt] = pack_bf16x4(st[ni][kt]);
                                dSb[ni][kt] = pack_bf16x4(dp[ni][kt]);
                                facc[hl][nt - kt + 3] += dp[ni][kt];
                            }
                        }
                        // dQ^T = K^T dS^T (gradient of q / sqrt(d)): rows = head features, column = query
                        f32x4 d0[2], d1[2];
#pragma unroll
                        for (int ni = 0; ni < 2; ++ni) {
                            d0[ni] = d1[ni] = zero4;
#pragma unroll
                            for (int kp = 0; kp < 2; ++kp) {
                                const uint4 sop = cat(dSb[ni][2 * kp], dSb[ni][2 * kp + 1]);
                                d0[ni] = mma32(cat(KN[0][2 * kp], KN[0][2 * kp + 1]), sop, d0[ni]);
                                d1[ni] = mma32(cat(KN[1][2 * kp], KN[1][2 * kp + 1]), sop, d1[ni]);
                            }
                        }
#pragma unroll
                        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                            for (int kt = 0; kt < 4; ++kt) {
                                Pq[kt][ni] = transpose_tile(Pb[ni][kt], ident);
                                dSq[kt][ni] = transpose_tile(dSb[ni][kt], ident);
                            }
#pragma unroll
                        for (int ni = 0; ni < 2; ++ni)
                            *reinterpret_cast<uint4 *>(dq_win + (size_t)(((2 * p2 + ni) * HG + hl) * 3 + 0) * 1024) =
                                cat(pack_bf16x4(d0[ni]), pack_bf16x4(d1[ni]));
                        __builtin_amdgcn_sched_barrier(0);
                        // dK^T += Q^T dS, dV^T += dO^T P over the 32 queries of the pair
#pragma unroll
                        for (int et = 0; et < 2; ++et)
#pragma unroll
                            for (int kt = 0; kt < 4; ++kt) {
                                dkT[et][kt] = mma32(qn[et], cat(dSq[kt][0], dSq[kt][1]), dkT[et][kt]);
                                dvT[et][kt] = mma32(on[et], cat(Pq[kt][0], Pq[kt][1]), dvT[et][kt]);
                            }
                    }
                    // dK = dS^T (q / sqrt(d)): the recomputed Q carries log2(e) / sqrt(d)
#pragma unroll
                    for (int kt = 0; kt < 4; ++kt) {
                        *reinterpret_cast<uint4 *>(dq_win + (size_t)((kt * HG + hl) * 3 + 1) * 1024) =
                            cat(pack_bf16x4(dkT[0][kt] * (1.0f / kLog2e)), pack_bf16x4(dkT[1][kt] * (1.0f / kLog2e)));
                        *reinterpret_cast<uint4 *>(dq_win + (size_t)((kt * HG + hl) * 3 + 2) * 1024) =
                            cat(pack_bf16x4(dvT[0][kt]), pack_bf16x4(dvT[1][kt]));
                    }
                }
            }
            // the next unit has landed in LDS before any wave reads it
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
        });
        par = (par + NU) & 1;
        win += stride;
        active = win < g.nW;
    }

    // this wave's partial sums of the bias-table gradient (heads of this group; every wave writes): per head the
    // 28 sums of every lane go through the wave's piece of LDS, and lane l collects entries l, l + 64, ...;
    // the four waves' sums meet in LDS (the weight stream's buffers are free) and leave as one vector
    float *tmeet = reinterpret_cast<float *>(lds + W::OFF_W);
    float *mine = tmeet + (size_t)wv * (HG * NTBL);
    static_assert((size_t)W::NWAVES * HG * NTBL * 4 <= 2 * W::UNIT_BYTES, "the waves' table sums fit the stream buffers");
#pragma unroll
    for (int hl = 0; hl < HG; ++hl) {
#pragma unroll
        for (int dl = 0; dl < 7; ++dl) fold4[dl * 64 + lane] = facc[hl][dl];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int e = lane + 64 * i;
            const int R = e / 15, dc = e - 15 * R - 7, dr = R - 7;
            float acc = 0.f;
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                // lanes (rsub, q/2) = (c, c) for even dr, (c, 1 - c) for odd dr
                const int odd = dr & 1;
                const int rs = c, qh = odd ? 1 - c : c;
                const int num = dr - rs + qh; // = 2 (dl - 3)
                const int dl = (num >> 1) + 3;
                const bool rok = e < NTBL && dl >= 0 && dl <= 6;
                const int base = dl * 256 + 128 * qh + 32 * rs + 4 * dc;
#pragma unroll
                for (int ql = 0; ql < 2; ++ql)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int kc = dc + 4 * ql + j; // the contributing lane's query column
                        const bool ok = rok && kc >= 0 && kc < M;
                        const float v = fold[ok ? base + 80 * ql + 5 * j : 0];
                        acc += ok ? v : 0.f;
                    }
            }
            if (e < NTBL) mine[hl * NTBL + e] = acc;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
    __syncthreads();
    float *out = tpart + (size_t)blockIdx.x * (HEADS * NTBL) + GI * HG * NTBL;
    for (int i = tid; i < HG * NTBL; i += W::NTHREADS)
        out[i] = (tmeet[i] + tmeet[HG * NTBL + i]) + (tmeet[2 * HG * NTBL + i] + tmeet[3 * HG * NTBL + i]);
}

// The group's dx slice and weight gradients from d(q|k|v).  A workgroup of eight waves takes two windows
// at a time: wave w = token tile w % 4 of window w / 4 (the tokens whose fragments the first kernel stored
// as that tile), so a SIMD holds two waves and the weight-gradient products run over 128 tokens.
template <class Cf, int GI>
__global__ __launch_bounds__(512, 1) void wide_qkv_grad_kernel(Geom g, const uint8_t *__restrict__ ffr,
                                                               const uint8_t *__restrict__ pack,
                                                               const uint8_t *__restrict__ dqkv,
                                                               bf16_t *__restrict__ dx, uint8_t *__restrict__ cgf,
                                                               float *__restrict__ part)
{
    using W = WideBwdCfg<Cf>;
    constexpr int C = Cf::C, D = Cf::D, CG = Cf::CG, HG = Cf::HG;
    static_assert(Cf::ET == 2, "two tiles per head");
    constexpr int KS = W::KS, CT = W::CT, CTF = W::CTF, FT = W::FT, RW = W::G_RW, LW = W::G_LW;
    constexpr int M = 8, NWV = W::G_WAVES;

    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const uint4 *wqx = reinterpret_cast<const uint4 *>(lds + W::G_OFF_WQX);
    uint16_t *gbuf = reinterpret_cast<uint16_t *>(lds + W::G_OFF_G); // d(q|k|v)^T rows [feature][token]
    uint16_t *fbuf = reinterpret_cast<uint16_t *>(lds + W::G_OFF_F); // F^T rows [channel][token], row CG = 1

    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, q = lane >> 4;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int slot = wv >> 2, tt = wv & 3; // window of the pair, token tile
    const int col0 = 64 * slot + 16 * tt;  // this wave's columns of the row buffers
    const int s = g.shift;
    const int per_img = g.nwi * g.nwj;
    const int rn = 2 * tt + (l16 >> 3), cn = l16 & 7;
    const uint32_t tbytes = (uint32_t)g.T * (2u * C);
    const buf_t dxbuf = make_buf(dx, tbytes);
    const bool casc_in = GI > 0 && g.cascade;
    const uint2 ones2 = make_uint2(0x3f803f80u, 0x3f803f80u);

    // the group's Wqkv^T fragments: (head of the group, q|k|v, channel tile)
    {
        constexpr int N16 = HG * 3 * CTF * 64;
        const uint4 *src = reinterpret_cast<const uint4 *>(pack + Cf::P_WQX + (size_t)GI * HG * 3 * CTF * 1024);
        for (int i = tid; i < N16; i += 64 * NWV) reinterpret_cast<uint4 *>(lds + W::G_OFF_WQX)[i] = src[i];
    }

    // row tiles of d w_qkv this wave owns: rt = wv, wv + 8, ...
    f32x4 acc[RW][CT];
#pragma unroll
    for (int r = 0; r < RW; ++r)
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) acc[r][ct] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int npair = (g.nW + 1) / 2;
    for (int pair = blockIdx.x; pair < npair; pair += gridDim.x) {
        const int win = 2 * pair + slot;
        const bool valid = win < g.nW;
        const int b = win / per_img;
        const int wr = win - b * per_img;
        const int wi = wr / g.nwj, wj = wr - wi * g.nwj;
        int si = wi * M + rn + s, sj = wj * M + cn + s;
        if (si >= g.H) si -= g.H;
        if (sj >= g.W) sj -= g.W;
        const uint32_t tok = (uint32_t)((((b * g.H + si) * g.W) + sj) * C) * 2u;

        uint4 dq[HG * 3];
        uint4 xf[KS];
        if (valid) {
            const uint4 *dsrc = reinterpret_cast<const uint4 *>(dqkv + ((size_t)win * 4 + tt) * W::FR_TILE * 1024) + lane;
#pragma unroll
            for (int i = 0; i < HG * 3; ++i) dq[i] = dsrc[i * 64];
            // F of these tokens as the first kernel used it (x slice + previous group's output, Eq. 8)
            const uint4 *fsrc = reinterpret_cast<const uint4 *>(ffr + ((size_t)win * 4 + tt) * KS * 1024) + lane;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) xf[ks] = fsrc[ks * 64];
        } else { // the odd window out: its columns of the row buffers are zero
#pragma unroll
            for (int i = 0; i < HG * 3; ++i) dq[i] = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) xf[ks] = make_uint4(0u, 0u, 0u, 0u);
        }
        __syncthreads(); // the previous pair's rows are consumed (first pass: the weights are in place)
        // F^T rows through a selector product; d(q|k|v)^T rows by a transposed store of the packed tiles
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
            f32x4 tN = f32x4{0.f, 0.f, 0.f, 0.f};
            if ((ct >> 1) < KS)
                tN = mma32(xf[(ct >> 1) < KS ? (ct >> 1) : 0], select_slot(16 * ct + l16, 32 * (ct >> 1) + 8 * q), tN);
            uint2 pk = pack_bf16x4(tN);
            if (16 * ct + l16 == CG) pk = valid ? ones2 : make_uint2(0u, 0u);
            *reinterpret_cast<uint2 *>(fbuf + (16 * ct + l16) * LW + col0 + 4 * q) = pk;
        }
#pragma unroll
        for (int i = 0; i < HG * 3; ++i) {
            store_tile_transposed(gbuf + ((2 * i + 0) * 16 + 4 * q) * LW + col0 + (l16 & ~1), LW,
                                  make_uint2(dq[i].x, dq[i].y), lane);
            store_tile_transposed(gbuf + ((2 * i + 1) * 16 + 4 * q) * LW + col0 + (l16 & ~1), LW,
                                  make_uint2(dq[i].z, dq[i].w), lane);
        }
        // ---- dx slice of this wave's 16 tokens: dF^T = Wqkv^T d(q|k|v)^T, rows = channels ----
        if (valid) {
            f32x4 df[CTF];
#pragma unroll
            for (int ct = 0; ct < CTF; ++ct) df[ct] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int i = 0; i < HG * 3; ++i)
#pragma unroll
                for (int ct = 0; ct < CTF; ++ct) df[ct] = mma32(wqx[(i * CTF + ct) * 64 + lane], dq[i], df[ct]);
            // tile ct = (input head hl', half et'): rows = channels hl' D + 16 et' + 4q ..
#pragma unroll
            for (int ct = 0; ct < CTF; ++ct) {
                const int cl = 16 * (ct % 2) + 4 * q;
                const uint2 v = pack_bf16x4(df[ct]);
                const uint32_t off = tok + 2u * (GI * CG + (ct / 2) * D + cl);
                if (cl + 2 < D) bstore64(dxbuf, off, 0u, v);
                else if (cl < D) bstore32(dxbuf, off, 0u, v.x);
            }
            // the same tiles as the previous group's first kernel adds them to its dO (Eq. 8)
            if (casc_in) {
                uint4 *cdst = reinterpret_cast<uint4 *>(cgf + ((size_t)win * 4 + tt) * HG * 1024) + lane;
#pragma unroll
                for (int hl = 0; hl < HG; ++hl) cdst[hl * 64] = cat(pack_bf16x4(df[2 * hl]), pack_bf16x4(df[2 * hl + 1]));
            }
        }
        __syncthreads();
        // ---- d w_qkv, d b_qkv: K = the pair's 128 tokens ----
#pragma unroll
        for (int kp = 0; kp < 4; ++kp) {
            uint4 afr[RW];
#pragma unroll
            for (int r = 0; r < RW; ++r) {
                const int rt = wv + NWV * r;
                const uint16_t *ar = gbuf + (16 * (rt < FT ? rt : 0) + l16) * LW + 32 * kp + 8 * q;
                afr[r] = cat(*reinterpret_cast<const uint2 *>(ar), *reinterpret_cast<const uint2 *>(ar + 4));
            }
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
                const uint16_t *br = fbuf + (16 * ct + l16) * LW + 32 * kp + 8 * q;
                const uint4 bf = cat(*reinterpret_cast<const uint2 *>(br), *reinterpret_cast<const uint2 *>(br + 4));
#pragma unroll
                for (int r = 0; r < RW; ++r) acc[r][ct] = mma32(afr[r], bf, acc[r][ct]);
            }
        }
    }

    // flush: rows in the order of w_qkv's rows of this group, (q|k|v, head, feature); the gradient of
    // q / sqrt(d) becomes that of q
    const float scale = 1.0f / sqrtf((float)D);
    float *mine = part + (size_t)blockIdx.x * W::L_TOTAL;
#pragma unroll
    for (int r = 0; r < RW; ++r) {
        const int rt = wv + NWV * r; // (head, q|k|v, half of the head's features)
        if (rt < FT) {
            const int i = rt >> 1, et = rt & 1, hl = i / 3, t3 = i - 3 * hl;
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
                const int c = 16 * ct + l16;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int e = 16 * et + 4 * q + j;
                    if (e < D) {
                        const int row = t3 * CG + hl * D + e;
                        const float v = t3 == 0 ? acc[r][ct][j] * scale : acc[r][ct][j];
                        if (c < CG) mine[W::L_DW + row * CG + c] = v;
                        else if (c == CG) mine[W::L_DB + row] = v;
                    }
                }
            }
        }
    }
}

int attn_grid(const Geom &g, int cus)
{
    if (cus > kSizingCus) cus = kSizingCus;
    return cus > g.nW ? g.nW : cus;
}

// scratch: [ d(q|k|v) of one group | d w_qkv partials of one group | table partials | a group's dF as the
// previous group's dO tiles | a group's input F as operand fragments ]; the projection's weight
// gradient, which runs after this pass, puts its partial vectors over the same memory
template <class Cf> struct WideBwdWs {
    using W = WideBwdCfg<Cf>;
    static size_t up(size_t v) { return (v + 255) & ~size_t(255); }
    static size_t dqkv_bytes(const Geom &g) { return up((size_t)g.nW * 4 * W::FR_TILE * 1024); }
    static size_t part_bytes(const Geom &g) { return up((size_t)attn_grid(g, kSizingCus) * W::L_TOTAL * 4); }
    static size_t tbl_bytes(const Geom &g)
    {
        return up((size_t)attn_grid(g, kSizingCus) * Cf::HEADS * W::NTBL * 4);
    }
    static size_t cg_bytes(const Geom &g) { return up((size_t)g.nW * 4 * Cf::HG * 1024); }
    static size_t f_bytes(const Geom &g) { return up((size_t)g.nW * 4 * W::KS * 1024); }
    static size_t wproj_bytes(const Geom &g) { return up((size_t)attn_grid(g, kSizingCus) * (Cf::C * Cf::C + Cf::C) * 4); }
};

template <class Cf, int GI>
hipError_t run_group(const Geom &g, int grid, const bf16_t *x, const bf16_t *dy, const bf16_t *attn, const uint8_t *pack,
                     bf16_t *dx, float *dw_qkv, float *db_qkv, int accumulate, uint8_t *dqkv, float *part, float *tpart,
                     uint8_t *cgf, uint8_t *ffr, ReduceJob *last, hipStream_t s)
{
    using W = WideBwdCfg<Cf>;
    {
        auto kern = wide_attn_bwd_kernel<Cf, GI>;
        if (hipError_t ea = allow_dynamic_lds(reinterpret_cast<const void *>(kern), W::LDS_BYTES); ea != hipSuccess) return ea;
        KernelTimer kt(K_WIDE_ATTN_BWD, s);
        hipLaunchKernelGGL(kern, dim3(grid), dim3(W::NTHREADS), W::LDS_BYTES, s, g, x, dy, attn, pack, cgf, dqkv, ffr, tpart);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    {
        auto kern = wide_qkv_grad_kernel<Cf, GI>;
        if (hipError_t ea = allow_dynamic_lds(reinterpret_cast<const void *>(kern), W::G_LDS_BYTES); ea != hipSuccess) return ea;
        KernelTimer kt(K_WIDE_WGRAD, s);
        const int pairs = (g.nW + 1) / 2;
        hipLaunchKernelGGL(kern, dim3(grid < pairs ? grid : pairs), dim3(64 * W::G_WAVES), W::G_LDS_BYTES, s, g, ffr, pack,
                           dqkv, dx, cgf, part);
    }
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    ReduceOut out{};
    out.ptr[0] = dw_qkv + (size_t)GI * 3 * Cf::CG * Cf::CG; out.begin[0] = W::L_DW;
    out.ptr[1] = db_qkv + GI * 3 * Cf::CG; out.begin[1] = W::L_DB;
    out.begin[2] = W::L_END;
    out.nseg = 2;
    const int nparts = grid < (g.nW + 1) / 2 ? grid : (g.nW + 1) / 2;
    if (GI == 0 && last) { // (the last group's sum shares a launch with the bias table's)
        last->part = part; last->nparts = nparts; last->n = W::L_TOTAL; last->out = out; last->accumulate = accumulate;
        return hipSuccess;
    }
    return launch_reduce(part, nparts, W::L_TOTAL, out, accumulate, s);
}

template <class Cf, int GI>
hipError_t run_groups(const Geom &g, int grid, const bf16_t *x, const bf16_t *dy, const bf16_t *attn,
                      const uint8_t *pack, bf16_t *dx, float *dw_qkv, float *db_qkv, int accumulate, uint8_t *dqkv,
                      float *part, float *tpart, uint8_t *cgf, uint8_t *ffr, ReduceJob *last, hipStream_t s)
{
    hipError_t e = run_group<Cf, GI>(g, grid, x, dy, attn, pack, dx, dw_qkv, db_qkv, accumulate, dqkv, part, tpart, cgf, ffr, last, s);
    if (e != hipSuccess) return e;
    if constexpr (GI > 0)
        return run_groups<Cf, GI - 1>(g, grid, x, dy, attn, pack, dx, dw_qkv, db_qkv, accumulate, dqkv, part, tpart, cgf, ffr, last, s);
    return hipSuccess;
}

template <class Cf>
hipError_t run_wide_bwd(const Geom &g, const bf16_t *x, const bf16_t *dy, const bf16_t *attn, const uint8_t *pack,
                        bf16_t *dx, float *dw_qkv, float *db_qkv, float *dtable, int accumulate, void *ws, hipStream_t s)
{
    using W = WideBwdCfg<Cf>;
    using Ws = WideBwdWs<Cf>;
    uint8_t *base = static_cast<uint8_t *>(ws);
    uint8_t *dqkv = base;
    float *part = reinterpret_cast<float *>(base + Ws::dqkv_bytes(g));
    float *tpart = reinterpret_cast<float *>(base + Ws::dqkv_bytes(g) + Ws::part_bytes(g));
    uint8_t *cgf = base + Ws::dqkv_bytes(g) + Ws::part_bytes(g) + Ws::tbl_bytes(g);
    uint8_t *ffr = cgf + Ws::cg_bytes(g);
    const int grid = attn_grid(g, device_cu_count());
    ReduceJob last{};
    hipError_t e = run_groups<Cf, Cf::G - 1>(g, grid, x, dy, attn, pack, dx, dw_qkv, db_qkv, accumulate, dqkv, part,
                                             tpart, cgf, ffr, &last, s);
    if (e != hipSuccess) return e;
    ReduceOut out{};
    out.ptr[0] = dtable; out.begin[0] = 0;
    out.begin[1] = Cf::HEADS * W::NTBL;
    out.nseg = 1;
    out.tbl_heads = Cf::HEADS; out.tbl_entries = W::NTBL; out.tbl_stride = Cf::HEADS; out.tbl_head0 = 0;
    ReduceJob tbl{};
    tbl.part = tpart; tbl.nparts = grid; tbl.n = Cf::HEADS * W::NTBL; tbl.out = out; tbl.accumulate = accumulate;
    return launch_reduce_pair(last, tbl, s);
}

#define GSWA_WIDE_BWD_SHAPES(X) X(180, 6, 2) X(180, 6, 3)

} // namespace

bool wide_bwd_supported(const Geom &g)
{
    if (!wide_fwd_supported(g)) return false; // (8x8 windows, q and k of the head's width; the forward fills the fragments)
    if (g.shift % 2 != 0) return false;        // (the runs of a window's rows are fetched in 16-byte pieces)
    // 32-bit byte offsets into d(q|k|v)
    if ((size_t)g.nW * 4 * 9 * 1024 >= (size_t(1) << 32)) return false;
#define X(C_, H_, G_) \
    if (g.C == C_ && g.heads == H_ && g.groups == G_) return true;
    GSWA_WIDE_BWD_SHAPES(X)
#undef X
    return false;
}

size_t wide_bwd_ws_bytes(const Geom &g)
{
#define X(C_, H_, G_)                                                                       \
    if (g.C == C_ && g.heads == H_ && g.groups == G_) {                                     \
        using Ws = WideBwdWs<FusedCfg<C_, H_, G_>>;                                         \
        const size_t own = Ws::dqkv_bytes(g) + Ws::part_bytes(g) + Ws::tbl_bytes(g) + Ws::cg_bytes(g) + Ws::f_bytes(g); \
        return own > Ws::wproj_bytes(g) ? own : Ws::wproj_bytes(g);                         \
    }
    GSWA_WIDE_BWD_SHAPES(X)
#undef X
    return 0;
}

hipError_t launch_wide_bwd(const Geom &g, const bf16_t *x, const bf16_t *dy, const bf16_t *attn, const void *pack,
                           bf16_t *dx, float *dw_qkv, float *db_qkv, float *dtable, int accumulate, void *ws,
                           hipStream_t s)
{
#define X(C_, H_, G_)                                                                                            \
    if (g.C == C_ && g.heads == H_ && g.groups == G_)                                                            \
        return run_wide_bwd<FusedCfg<C_, H_, G_>>(g, x, dy, attn, static_cast<const uint8_t *>(pack), dx, dw_qkv, \
                                                  db_qkv, dtable, accumulate, ws, s);
    GSWA_WIDE_BWD_SHAPES(X)
#undef X
    return hipErrorInvalidValue;
}

} // namespace gswa
