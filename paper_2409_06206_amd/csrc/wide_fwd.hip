// Forward of wide GSWA layers (C = 180, six heads of 30 channels, 8x8 windows) in one launch:
// shift + partition + per-group QKV projection (Eq. 6) with the cascade add (Eq. 8) + scores with
// relative bias and shift mask + softmax + PV + output projection (Eq. 7) + merge + reverse shift.
//
// One wavefront owns one window: its 64 tokens are four 16-token tiles, K, V and the
// probabilities never leave the wave's registers.  A workgroup is four waves, one per SIMD (a
// wave then has the SIMD's whole register file: x of all groups and all head outputs stay in
// registers).  The weights of a wide layer (108 KB of QKV fragments, 72 KB of projection
// fragments) do not fit LDS together, so they pass through it as a stream of equal units, double
// buffered, one workgroup barrier per unit: the QKV fragments of one head (one group: of its q,
// k or v), then the projection in pieces of the same size.  Every fragment read from LDS serves
// the four token tiles of the wave.
//
// Everything is kept with rows = features and column = token (T-form, see fused_bwd.hip), and a
// head of 30 channels is two 16-row tiles, i.e. exactly the 32 k-slots of one K=32 MFMA step in
// "head-padded order" (lane group q: features 4q..4q+3 and 16+4q..16+4q+3).  A packed pair of
// output tiles of a head therefore is, as it lies in registers, the operand of the next group's
// QKV projection (after the cascade add onto the x operand, rounded to bf16 like a stored
// activation) and of the output projection.
#include "fused.h"
#include "mfma.h"

namespace gswa {

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kMaskLog2 = -100.0f * kLog2e; // the additive -100 of the shift mask, in base-2 units


template <class Cf> struct WideFwdCfg {
    // one wave per SIMD: a wave then has the whole register file of its SIMD (512 registers), which
    // holds a window's x, all head outputs and the staging registers of the weight stream
    static constexpr int NWAVES = 4, NTHREADS = 64 * NWAVES;
    // The weights pass through LDS as a stream of equal units, double buffered: the QKV fragments of
    // one head, then the projection fragments in pieces of the same size (whole output tiles).
    // (one group: a head's fragments are 36 KB, so a unit is one of q, k, v of a head)
    static constexpr int UPH = Cf::G == 1 ? 3 : 1;                 // units per head
    static constexpr int FR_UNIT = 3 * Cf::ET * Cf::KSX / UPH;     // fragments (1 KB) of one unit
    static constexpr size_t UNIT_BYTES = (size_t)FR_UNIT * 1024;
    static constexpr int OT_UNIT = FR_UNIT / Cf::HEADS;            // output tiles of one projection unit
    static constexpr int NPU = Cf::OT / OT_UNIT;                   // projection units
    static constexpr int NHU = Cf::HEADS * UPH;                    // head units
    static constexpr int NU = NHU + NPU;                           // units per window
    static constexpr size_t OFF_BIAS = 0;                          // fp32 b_qkv [3C], b_proj [C]
    static constexpr size_t OFF_TBL = (size_t)16 * Cf::C;          // fp32 [HEADS][TBW_PITCH]
    static constexpr size_t OFF_W = OFF_TBL + (size_t)Cf::HEADS * Cf::TBW_PITCH * 4;
    static constexpr size_t LDS_BYTES = OFF_W + 2 * UNIT_BYTES;
    static_assert(OFF_W % 16 == 0 && LDS_BYTES <= 160 * 1024, "LDS budget");
    static_assert(FR_UNIT % Cf::HEADS == 0 && Cf::OT % OT_UNIT == 0 && NU % 2 == 0,
                  "units tile the projection");
    static_assert(Cf::ET == 2 && Cf::D + 1 <= 32 && Cf::CG % Cf::D == 0, "heads of 17..31 channels: two tiles, a spare row");
};

template <int Q0> __device__ __forceinline__ float qgroup_bcast(float v)
{
    const unsigned u = __float_as_uint(v);
    u32x2 r = __builtin_amdgcn_permlane32_swap(u, u, false, false); // {groups 0,1,0,1; groups 2,3,2,3}
    const unsigned h = r[Q0 >> 1];
    r = __builtin_amdgcn_permlane16_swap(h, h, false, false);       // {even group of each pair; odd group}
    return __uint_as_float(r[Q0 & 1]);
}

template <class Cf>
__global__ __launch_bounds__(256, 1) void wide_fwd_kernel(Geom g, const bf16_t *__restrict__ x,
                                                          const uint8_t *__restrict__ pack,
                                                          bf16_t *__restrict__ y, bf16_t *__restrict__ attn)
{
    using W = WideFwdCfg<Cf>;
    constexpr int C = Cf::C, D = Cf::D, CG = Cf::CG, HG = Cf::HG, HEADS = Cf::HEADS, G = Cf::G;
    constexpr int KSX = Cf::KSX, TP = Cf::TBW_PITCH, NU = W::NU, OT_UNIT = W::OT_UNIT;
    constexpr int M = 8, NTHREADS = W::NTHREADS;
    constexpr int FPW = (W::FR_UNIT + W::NWAVES - 1) / W::NWAVES; // fragments a wave moves per unit
    constexpr int NTB = 2; // query tiles taken through the softmax together

    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, q = lane >> 4;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int s = g.shift;
    const int cn = l16 & 7, rsub = l16 >> 3;
    const int per_img = g.nwi * g.nwj;
    const uint32_t tbytes = (uint32_t)g.T * (2u * C);
    const buf_t xbuf = make_buf(x, tbytes), ybuf = make_buf(y, tbytes), abuf = make_buf(attn, attn ? tbytes : 0u);
    // second half of a head's k-slots: features 16+4q..16+4q+3, of which only those below D exist
    const uint32_t m_hx = (16 + 4 * q < D) ? 0xffffffffu : 0u, m_hy = (16 + 4 * q + 2 < D) ? 0xffffffffu : 0u;
    const uint32_t c8 = 8u * q;

    // ---- weight stream: unit u of a window = QKV fragments of a head (or of its q, k or v alone),
    // then projection fragments of OT_UNIT output tiles.  A thread stages its 16-byte pieces of the
    // next unit in registers while the current unit is computed with, and writes them to the other
    // LDS buffer afterwards; one barrier per unit. ----
    // (the lane index as a round's address arithmetic sees it: opaque, re-made every round, so that per-lane
    // addresses are computed where they are used instead of being kept, and spilled, across the kernel)
    int lane_r = lane;
    auto unit_src = [&](int u) {
        return pack + (u < W::NHU ? Cf::P_WQW + (size_t)u * W::UNIT_BYTES
                                  : Cf::P_WPW + (size_t)(u - W::NHU) * W::UNIT_BYTES);
    };
    // Loads that write LDS directly: one instruction moves one fragment (64 lanes x 16 bytes land at
    // the wave-uniform LDS address + 16 * lane).  Wave w moves fragments w, w + 4, ... of the unit.
    auto stream_unit = [&](int u, int slot) {
        const uint8_t *src = unit_src(u) + 16 * lane_r;
        uint8_t *dst = lds + W::OFF_W + (size_t)slot * W::UNIT_BYTES;
#pragma unroll
        for (int k = 0; k < FPW; ++k) {
            const int f = k * W::NWAVES + wv;
            if (f < W::FR_UNIT) lds_dma16(src + (size_t)f * 1024, dst + (size_t)f * 1024);
        }
    };

    // ---- the window of this wave: byte offsets of its tokens (tile t, this lane's column) and its x as
    // MFMA operands (all groups, head-padded order: step ks of group gi, tile t) ----
    const int stride = W::NWAVES * (int)gridDim.x;
    const int rounds = (g.nW + stride - 1) / stride;
    uint32_t tok[4];
    bool lastrow = false, lastcol = false;
    uint4 xh[G][KSX][4];
    auto window_tokens = [&](int win) {
        const int b = win / per_img;
        const int wr = win - b * per_img;
        const int wi = wr / g.nwj, wj = wr - wi * g.nwj;
        lastrow = s > 0 && wi == g.nwi - 1;
        lastcol = s > 0 && wj == g.nwj - 1;
        int sj = wj * M + cn + s;
        if (sj >= g.W) sj -= g.W;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            int si = wi * M + 2 * t + rsub + s;
            if (si >= g.H) si -= g.H;
            tok[t] = (uint32_t)((((b * g.H + si) * g.W) + sj) * C) * 2u;
        }
    };
    auto load_x = [&]() {
#pragma unroll
        for (int gi = 0; gi < G; ++gi)
#pragma unroll
            for (int ks = 0; ks < KSX; ++ks)
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const uint32_t off = tok[t] + c8 + 2u * (gi * CG + ks * D);
                    const uint2 lo = bload64(xbuf, off, 0u);
                    uint2 hi = bload64(xbuf, off + 32u, 0u);
                    hi.x &= m_hx;
                    hi.y &= m_hy;
                    xh[gi][ks][t] = cat(lo, hi);
                }
    };
    int win = wv * (int)gridDim.x + (int)blockIdx.x;
    bool active = win < g.nW;
    if (active) {
        window_tokens(win);
        load_x();
    }

    // set-up: linear biases, bias table, first unit
    stream_unit(0, 0);
    for (int i = tid; i < C; i += NTHREADS)
        reinterpret_cast<uint4 *>(lds + W::OFF_BIAS)[i] = reinterpret_cast<const uint4 *>(pack + Cf::P_BIAS)[i];
    for (int i = tid; i < HEADS * TP / 4; i += NTHREADS)
        reinterpret_cast<uint4 *>(lds + W::OFF_TBL)[i] = reinterpret_cast<const uint4 *>(pack + Cf::P_TBW)[i];
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

    for (int round = 0; round < rounds; ++round) {
        const bool more = round + 1 < rounds;
        if (active && round > 0) {
            window_tokens(win);
            load_x();
        }
        // head outputs, packed tile pairs [head][token tile]: operand of the cascade and of the projection
        uint4 Ob[HEADS][4];
        uint2 Qb[2][4], Kb[2][4], Vb[2][4];

        uint32_t lds0 = 0;
        asm volatile("" : "+v"(lds0)); // keeps the LDS reads of a round inside the round
        lane_r = lane;
        asm volatile("" : "+v"(lane_r));
        const float *bqkv = reinterpret_cast<const float *>(lds + lds0 + W::OFF_BIAS);
        const float *bproj = bqkv + 3 * C;
        const float *tbl = reinterpret_cast<const float *>(lds + lds0 + W::OFF_TBL);

        static_for<NU>([&](auto u_) {
            constexpr int u = decltype(u_)::value;
            const uint4 *wu = reinterpret_cast<const uint4 *>(lds + lds0 + W::OFF_W + (size_t)(u & 1) * W::UNIT_BYTES);
            // next unit on its way into the other buffer (the first of the next window after the last):
            // every wave has passed the previous barrier, i.e. finished reading that buffer
            if (u + 1 < NU) stream_unit(u + 1, (u + 1) & 1);
            else if (more) stream_unit(0, 0);

            if constexpr (u < W::NHU) {
                constexpr int hd = u / W::UPH, part = u % W::UPH, gi = hd / HG, hl = hd % HG;
                constexpr int T3B = part * (3 / W::UPH), T3E = T3B + 3 / W::UPH; // of q, k, v: this unit's
                if (active) {
                    if (G > 1 && part == 0 && hl == 0 && gi > 0 && g.cascade) { // Eq. 8
#pragma unroll
                        for (int ks = 0; ks < KSX; ++ks)
#pragma unroll
                            for (int t = 0; t < 4; ++t) {
                                const uint4 p = Ob[(gi > 0 ? gi - 1 : 0) * HG + ks][t];
                                uint4 &xv = xh[gi][ks][t];
                                xv.x = add_bf16x2(xv.x, p.x);
                                xv.y = add_bf16x2(xv.y, p.y);
                                xv.z = add_bf16x2(xv.z, p.z & m_hx);
                                xv.w = add_bf16x2(xv.w, p.w & m_hy);
                            }
                    }
                    // ---- Q^T, K^T (rows = head features) and V (rows = tokens): eight independent
                    // accumulator tiles per kind, so that consecutive MFMAs never wait for each other ----
#pragma unroll
                    for (int t3 = T3B; t3 < T3E; ++t3) {
                        f32x4 acc[2][4];
#pragma unroll
                        for (int et = 0; et < 2; ++et) {
                            f32x4 b4;
                            if (t3 < 2) {
#pragma unroll
                                for (int j = 0; j < 4; ++j) {
                                    const int e = 16 * et + 4 * q + j;
                                    const float bv = e < D ? bqkv[gi * 3 * CG + t3 * CG + hl * D + e] : 0.f;
                                    b4[j] = t3 == 0 ? bv * kLog2e : bv;
                                }
                            } else {
                                // column D of V is one: row D of the PV product is the sum of the probabilities
                                const int e = 16 * et + l16;
                                const float bv = e < D ? bqkv[gi * 3 * CG + 2 * CG + hl * D + e] : (e == D ? 1.f : 0.f);
                                b4 = f32x4{bv, bv, bv, bv};
                            }
#pragma unroll
                            for (int t = 0; t < 4; ++t) acc[et][t] = b4;
                        }
#pragma unroll
                        for (int ks = 0; ks < KSX; ++ks) {
                            const uint4 f0 = wu[(((t3 - T3B) * 2 + 0) * KSX + ks) * 64 + lane];
                            const uint4 f1 = wu[(((t3 - T3B) * 2 + 1) * KSX + ks) * 64 + lane];
#pragma unroll
                            for (int t = 0; t < 4; ++t) {
                                const uint4 xv = xh[gi][ks][t];
                                acc[0][t] = t3 < 2 ? mma32(f0, xv, acc[0][t]) : mma32(xv, f0, acc[0][t]);
                                acc[1][t] = t3 < 2 ? mma32(f1, xv, acc[1][t]) : mma32(xv, f1, acc[1][t]);
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
                        __builtin_amdgcn_sched_barrier(0); // (keeps the scheduler from stretching the next stage's loads over this one)
                    }
                }
                if constexpr (part == W::UPH - 1) {
                if (active) {
                    // relative bias of score tile (kt, nt) depends on nt - kt only: seven register tiles
                    f32x4 bt[7];
#pragma unroll
                    for (int dl = 0; dl < 7; ++dl)
#pragma unroll
                        for (int j = 0; j < 4; ++j) bt[dl][j] = tbl[hd * TP + tb0 + 30 * (dl - 3) - j];

                    // S^T tiles (base-2 units): rows = keys 16kt+4q+j, column = query 16nt+l16; two query
                    // tiles are taken through every stage together (independent chains)
#pragma unroll
                    for (int n0 = 0; n0 < 4; n0 += NTB) {
                        f32x4 st[NTB][4];
#pragma unroll
                        for (int ni = 0; ni < NTB; ++ni) {
                            const uint4 qop = cat(Qb[0][n0 + ni], Qb[1][n0 + ni]);
#pragma unroll
                            for (int kt = 0; kt < 4; ++kt)
                                st[ni][kt] = mma32(cat(Kb[0][kt], Kb[1][kt]), qop, bt[n0 + ni - kt + 3]);
                        }
                        if (lastrow || lastcol) {
#pragma unroll
                            for (int ni = 0; ni < NTB; ++ni)
#pragma unroll
                                for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                                    for (int j = 0; j < 4; ++j)
                                        if ((lastrow && qr_w[n0 + ni] != kr_w[kt]) || (lastcol && qc_w != kc_w[j]))
                                            st[ni][kt][j] += kMaskLog2;
                        }
                        float mx[NTB];
#pragma unroll
                        for (int ni = 0; ni < NTB; ++ni) {
                            float m0 = fmaxf(fmaxf(st[ni][0][0], st[ni][0][1]), fmaxf(st[ni][0][2], st[ni][0][3]));
#pragma unroll
                            for (int kt = 1; kt < 4; ++kt)
#pragma unroll
                                for (int j = 0; j < 4; j += 2) m0 = fmaxf(fmaxf(m0, st[ni][kt][j]), st[ni][kt][j + 1]);
                            mx[ni] = m0;
                        }
#pragma unroll
                        for (int ni = 0; ni < NTB; ++ni) mx[ni] = qgroup_max(mx[ni]);
                        uint2 Pb[NTB][4];
#pragma unroll
                        for (int ni = 0; ni < NTB; ++ni)
#pragma unroll
                            for (int kt = 0; kt < 4; ++kt) {
#pragma unroll
                                for (int j = 0; j < 4; ++j) st[ni][kt][j] = __builtin_amdgcn_exp2f(st[ni][kt][j] - mx[ni]);
                                Pb[ni][kt] = pack_bf16x4(st[ni][kt]);
                            }
                        // O^T = V^T P^T: rows = head features (row D = sum of the probabilities)
                        f32x4 o0[NTB], o1[NTB];
#pragma unroll
                        for (int ni = 0; ni < NTB; ++ni) {
                            o0[ni] = mma32(cat(Vb[0][0], Vb[0][1]), cat(Pb[ni][0], Pb[ni][1]), zero4);
                            o1[ni] = mma32(cat(Vb[1][0], Vb[1][1]), cat(Pb[ni][0], Pb[ni][1]), zero4);
                        }
#pragma unroll
                        for (int ni = 0; ni < NTB; ++ni) {
                            o0[ni] = mma32(cat(Vb[0][2], Vb[0][3]), cat(Pb[ni][2], Pb[ni][3]), o0[ni]);
                            o1[ni] = mma32(cat(Vb[1][2], Vb[1][3]), cat(Pb[ni][2], Pb[ni][3]), o1[ni]);
                        }
#pragma unroll
                        for (int ni = 0; ni < NTB; ++ni) {
                            const float inv = __builtin_amdgcn_rcpf(qgroup_bcast<(D - 16) / 4>(o1[ni][(D - 16) % 4]));
                            o0[ni] *= inv;
                            o1[ni] *= inv;
                            Ob[hd][n0 + ni] = cat(pack_bf16x4(o0[ni]), pack_bf16x4(o1[ni]));
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    // the outputs of a group leave together when the caller keeps them for the backward
                    // pass (pieces of a row then fill whole cache lines)
                    if (attn && hl == HG - 1) {
#pragma unroll
                        for (int nt = 0; nt < 4; ++nt)
#pragma unroll
                            for (int h2 = gi * HG; h2 <= hd; ++h2) {
                                // lane group q: features 8q .. 8q+7 of the head (16 contiguous bytes)
                                const uint32_t off = tok[nt] + 16u * q + 2u * (h2 * D);
                                const uint4 o = pair_rows(make_uint2(Ob[h2][nt].x, Ob[h2][nt].y),
                                                          make_uint2(Ob[h2][nt].z, Ob[h2][nt].w));
                                if (8 * q + 8 <= D) {
                                    bstore128(abuf, off, 0u, o);
                                } else {
                                    if (8 * q + 4 <= D) bstore64(abuf, off, 0u, make_uint2(o.x, o.y));
                                    if (8 * q + 6 <= D) bstore32(abuf, off + 8u, 0u, o.z);
                                }
                            }
                    }
                }
                }
            } else {
                // ---- Y^T = Wproj A^T + b for OT_UNIT output tiles: rows = output channels, column = token ----
                constexpr int pu = u - W::NHU;
                if (active) {
                    // two output tiles at a time: their packed results are regrouped so that a lane holds 16
                    // contiguous bytes of its token's row (a tile left over at the end goes out in 8-byte pieces)
                    auto project = [&](int ot, f32x4(&acc)[4]) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const int o = 16 * ot + 4 * q + j;
                            const float bv = o < C ? bproj[o] : 0.f;
#pragma unroll
                            for (int t = 0; t < 4; ++t) acc[t][j] = bv;
                        }
#pragma unroll
                        for (int hd = 0; hd < HEADS; ++hd) {
                            const uint4 wf = wu[((ot - pu * OT_UNIT) * HEADS + hd) * 64 + lane];
#pragma unroll
                            for (int t = 0; t < 4; ++t) acc[t] = mma32(wf, Ob[hd][t], acc[t]);
                        }
                    };
#pragma unroll
                    for (int oi = 0; oi + 1 < OT_UNIT; oi += 2) {
                        const int ot = pu * OT_UNIT + oi;
                        f32x4 acc0[4], acc1[4];
                        project(ot, acc0);
                        project(ot + 1, acc1);
                        const int o0 = 16 * ot + 8 * q; // first channel of this lane's eight
#pragma unroll
                        for (int t = 0; t < 4; ++t) {
                            const uint4 v = pair_rows(pack_bf16x4(acc0[t]), pack_bf16x4(acc1[t]));
                            const uint32_t off = tok[t] + 2u * o0;
                            if (o0 + 8 <= C) bstore128(ybuf, off, 0u, v);
                            else if (o0 + 4 <= C) bstore64(ybuf, off, 0u, make_uint2(v.x, v.y));
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    if (OT_UNIT % 2 == 1) {
                        const int ot = pu * OT_UNIT + OT_UNIT - 1;
                        f32x4 acc[4];
                        project(ot, acc);
                        const int o0 = 16 * ot + 4 * q;
#pragma unroll
                        for (int t = 0; t < 4; ++t)
                            if (o0 < C) bstore64(ybuf, tok[t] + c8 + 32u * ot, 0u, pack_bf16x4(acc[t]));
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
            // the next unit has landed in LDS before any wave reads it
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
        });
        win += stride;
        active = win < g.nW;
    }
}

#define GSWA_WIDE_SHAPES(X) X(180, 6, 1) X(180, 6, 2) X(180, 6, 3)

template <class Cf>
hipError_t run_wide_fwd(const Geom &g, const bf16_t *x, const uint8_t *pack, bf16_t *y, bf16_t *attn, int training,
                        hipStream_t s)
{
    using W = WideFwdCfg<Cf>;
    auto kern = wide_fwd_kernel<Cf>;
    if (hipError_t ea = allow_dynamic_lds(reinterpret_cast<const void *>(kern), W::LDS_BYTES); ea != hipSuccess) return ea;
    // one window per wave: spread the windows over the compute units before filling a workgroup
    int grid = device_cu_count();
    if (grid > g.nW) grid = g.nW;
    KernelTimer kt(K_FUSED_FWD, s);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(W::NTHREADS), W::LDS_BYTES, s, g, x, pack, y, training ? attn : nullptr);
    return hipGetLastError();
}

} // namespace

bool wide_fwd_supported(const Geom &g)
{
    if (g.M != 8 || g.dq != g.d || (long)g.T * g.C >= (1L << 31)) return false;
#define X(C_, H_, G_) \
    if (g.C == C_ && g.heads == H_ && g.groups == G_) return true;
    GSWA_WIDE_SHAPES(X)
#undef X
    return false;
}

hipError_t launch_wide_fwd(const Geom &g, const bf16_t *x, const void *pack, bf16_t *y, bf16_t *attn, int training,
                           hipStream_t s)
{
    if (training && !attn) return hipErrorInvalidValue;
#define X(C_, H_, G_)                                 \
    if (g.C == C_ && g.heads == H_ && g.groups == G_) \
        return run_wide_fwd<FusedCfg<C_, H_, G_>>(g, x, static_cast<const uint8_t *>(pack), y, attn, training, s);
    GSWA_WIDE_SHAPES(X)
#undef X
    return hipErrorInvalidValue;
}

} // namespace gswa
