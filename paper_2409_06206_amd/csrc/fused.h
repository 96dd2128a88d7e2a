// Fused per-window GSWA kernels (bf16 storage, MFMA arithmetic).
//
// Activations stay in registers in MFMA operand / result layouts (see mfma.h).  Two ways of
// giving a window to the hardware are in use:
//   * one wavefront per window (forward of narrow layers): the wave holds all 64 tokens as four
//     16-token tiles, so nothing crosses waves and no barrier is needed after the set-up;
//   * one workgroup per window, one wavefront per 16 tokens (split forward of wide layers, every
//     fused backward): K and V of a head, and in the backward the transposed score gradients,
//     cross waves through LDS.
// The shift, the window partition and their inverses are the address computation of the
// first load and the last store (Sec. "Patch Embedding", Sec. "Group Shifted Window Attention").
#pragma once
#include "common.h"
#include "profile.h"

namespace gswa {

// Compile-time shape of a fused instantiation, and the layout of its packed parameters.
//
// The parameters are rewritten once per forward call into MFMA fragment order ("lane-major":
// fragment f, lane l at f*64 + l, so one LDS read per lane fetches an operand), zero padded
// (head width to 16*ET, group width to 32*KS).  The query rows of w_qkv and b_qkv are stored
// multiplied by 1/sqrt(d), so scores need no separate scaling.  One buffer serves both passes:
//   [ WQH | WP2 | BF | WQ | BIAS | WPT | WQT | WPK ]
// forward of narrow layers: WQH, WP2, BF, BIAS; backward: WQ .. WQT.
//   WQH  Wqkv with the group's input channels in head-padded order (k-slot 16*hl' + e' <-> channel
//        hl'*D + e'), the order in which a group's output tiles lie in registers, so that the
//        cascade input of Eq. 8 is added to the x slice operand in place; K=32 steps over head
//        pairs.  Query rows carry log2(e)/sqrt(d), so the scores come out in base-2 units.  The
//        upper half of the last step multiplies four per-token inputs (1, r, c, r*c) and fills rows
//        D .. D+3 of Q^T and K^T with the terms of the shift mask (see wave_fwd_kernel).
//   WP2  Wproj, K=32 steps over head pairs
//   BF   relative-position bias times log2(e) as bf16 score-tile operands, one per head and
//        key/query tile offset
// Wide layers (C > 64) do not fit their weights in LDS at once: their forward runs per head
// chunk (SPLIT), takes the cascade input from memory, and projects in a separate GEMM that
// uses WPK; WQH, WP2 and BF are empty for them.
template <int C_, int HEADS_, int G_> struct FusedCfg {
    static constexpr int C = C_, HEADS = HEADS_, G = G_;
    static constexpr int D = C / HEADS, CG = C / G, HG = HEADS / G;
    static constexpr int ET = (D + 15) / 16;  // 16-row tiles per head (head width padded to 16*ET)
    static constexpr int KS = (CG + 31) / 32; // K=32 steps over one group's input channels
    static constexpr int KSC = (C + 31) / 32; // K=32 steps over all channels
    static constexpr int OT = (C + 15) / 16;  // 16-row tiles of the output projection
    static constexpr bool SPLIT = C > 64;
    static constexpr int NSTEP = HG / 2 + 1;   // K=32 steps over a group's heads: head pairs, then odd head | mask inputs
    static constexpr int NDLT = 7;             // key/query tile offsets -3 .. 3 of an 8x8 window
    static constexpr int N_WQH = SPLIT ? 0 : HEADS * 3 * NSTEP;  // (hd,t,step), 1 KB each
    static constexpr int N_WP2 = SPLIT ? 0 : OT * (HEADS / 2);   // (ot,pair), 1 KB each
    static constexpr int N_BF = SPLIT ? 0 : HEADS * NDLT;        // (hd,dlt), 512 B each
    static constexpr int N_WPK = SPLIT ? OT * KSC : 0;           // Wproj, K=32 over all channels: (ot,ks)
    static constexpr int N_WQ = HEADS * 3 * ET * KS;             // Wqkv on the x slice, K=32: (hd,t,et,ks)
    static constexpr int N_WPT = HEADS * ET * KSC;               // Wproj^T, K=32: (hd,et,ks)
    static constexpr int N_WQT = HEADS * 3 * ET * HG * ET;       // Wqkv^T, K=16: (hd,t,et,hlp,etp)
    static constexpr size_t P_WQH = 0;
    static constexpr size_t P_WP2 = P_WQH + (size_t)N_WQH * 1024;
    static constexpr size_t P_BF = P_WP2 + (size_t)N_WP2 * 1024;
    static constexpr size_t P_WQ = P_BF + (size_t)N_BF * 512;
    static constexpr size_t P_BIAS = P_WQ + (size_t)N_WQ * 1024; // fp32 b_qkv [3C], b_proj [C]
    static constexpr size_t P_WPT = P_BIAS + (size_t)16 * C;
    static constexpr size_t P_WQT = P_WPT + (size_t)N_WPT * 1024;
    static constexpr size_t P_WPK = P_WQT + (size_t)N_WQT * 512;
    // Wide layers, forward with one wavefront per window (wide_fwd.hip): a head is 16*ET = 32
    // k-slots, so one K=32 step carries one head in "head-padded order": lane group q holds the
    // head's features 4q..4q+3 and 16+4q..16+4q+3 -- the rows of the two result tiles of a head
    // output, which makes a packed output tile pair the operand of the next product.
    //   WQW  Wqkv, input channels of the group in head-padded order, one K=32 step per input head:
    //        (hd, t, et, step); query rows carry log2(e)/sqrt(d)
    //   WPW  Wproj, one K=32 step per head: (ot, hd)
    //   TBW  relative-position bias times log2(e), fp32, [head][TBW_PITCH]
    static constexpr int KSX = CG / D;                            // input heads of a group = K=32 steps
    static constexpr int N_WQW = SPLIT ? HEADS * 3 * ET * KSX : 0;
    static constexpr int N_WPW = SPLIT ? OT * HEADS : 0;
    static constexpr int TBW_PITCH = 228;
    static constexpr size_t P_WQW = P_WPK + (size_t)N_WPK * 1024;
    static constexpr size_t P_WPW = P_WQW + (size_t)N_WQW * 1024;
    static constexpr size_t P_TBW = P_WPW + (size_t)N_WPW * 1024;
    // Wide layers, backward with one wavefront per window (wide_bwd.hip) additionally reads
    //   WQX  Wqkv^T for dF = d(q|k|v) Wqkv, K=32: one step = the 32 k-slots of one (head, q|k|v) in
    //        head-padded order; (hd, t, ct), ct = (input head hl', half et') of the group: row l16 ->
    //        input channel hl' D + 16 et' + l16 (so that dF comes out in the tiles dO is held in);
    //        query rows carry 1/sqrt(d) like WQ
    static constexpr int CTF = HG * ET;                           // 16-row tiles of a group's input channels, per head
    static constexpr int N_WQX = SPLIT ? HEADS * 3 * CTF : 0;
    static constexpr size_t P_WQX = P_TBW + (SPLIT ? (size_t)HEADS * TBW_PITCH * 4 : 0);
    //   WQN  Wqkv on the group's channels in their own order, K=32 (the layout of WQ), query rows times
    //        log2(e)/sqrt(d) as in WQW: the backward recomputes q, k, v from 16-byte row pieces
    static constexpr int N_WQN = SPLIT ? N_WQ : 0;
    static constexpr size_t P_WQN = P_WQX + (size_t)N_WQX * 1024;
    static constexpr size_t P_END = P_WQN + (size_t)N_WQN * 1024;
};

// True when a fused forward instantiation exists for this geometry (bf16 only).
bool fused_fwd_supported(const Geom &g);
// Bytes of the packed parameters (both passes).
size_t fused_pack_bytes(const Geom &g);

// True when the forward of this geometry runs per head chunk and therefore always needs the
// attn_out buffer (for inference the caller lends scratch).
bool fused_fwd_needs_attn(const Geom &g);

// y = GSWA(x); attn_out receives the concatenated group outputs [T, C] (may be null unless
// fused_fwd_needs_attn); `pack` receives the packed parameters (fused_pack_bytes, 256-byte aligned).
// `training`: attn_out is kept by the caller for the backward pass (otherwise it is scratch and a
// kernel may leave out what only the backward would read).
hipError_t launch_fused_fwd(const Geom &g, const bf16_t *x, const bf16_t *w_qkv, const bf16_t *b_qkv,
                            const bf16_t *w_proj, const bf16_t *b_proj, const bf16_t *table,
                            bf16_t *y, bf16_t *attn_out, void *pack, int training, hipStream_t s);

// ---------------------------------------------------------------------------------------
// Parameter packing for this kernel (layout: FusedCfg, WQW / WPW / TBW)
// ---------------------------------------------------------------------------------------
// (entry i of the (N_WQW + N_WPW + N_WQX + N_WQN) * 64 + HEADS * TBW_PITCH of the wide layout; run by the extra
// blocks of the parameter-packing launch)
template <class Cf>
__device__ __forceinline__ void wide_pack_entry(int i, const bf16_t *__restrict__ w_qkv,
                                                const bf16_t *__restrict__ w_proj,
                                                const bf16_t *__restrict__ table, uint8_t *__restrict__ pack)
{
    constexpr float kLog2e = 1.4426950408889634f;
    constexpr int C = Cf::C, D = Cf::D, CG = Cf::CG, HG = Cf::HG, HEADS = Cf::HEADS, ET = Cf::ET, KSX = Cf::KSX;
    constexpr int E_WQW = Cf::N_WQW * 64, E_WPW = Cf::N_WPW * 64, E_TBW = HEADS * Cf::TBW_PITCH, E_WQX = Cf::N_WQX * 64;
    const float qscale = kLog2e / sqrtf((float)D);
    const int l16 = i & 15, q = (i >> 4) & 3;
    // feature of a head held in k-slot s of lane group q
    auto slot_feature = [&](int s) { return s < 4 ? 4 * q + s : 16 + 4 * q + (s - 4); };
    if (i < E_WQW) {
        int f = i >> 6;
        const int ks = f % KSX; f /= KSX;
        const int et = f % ET; f /= ET;
        const int t = f % 3;
        const int hd = f / 3, gi = hd / HG, hl = hd % HG;
        const int e = 16 * et + l16;
        uint32_t v[8];
        for (int s = 0; s < 8; ++s) {
            const int fe = slot_feature(s);
            float w = 0.f;
            if (e < D && fe < D)
                w = to_f32(w_qkv[((size_t)gi * 3 * CG + t * CG + hl * D + e) * CG + ks * D + fe]) * (t == 0 ? qscale : 1.0f);
            v[s] = f32_to_bf16_bits(w);
        }
        reinterpret_cast<uint4 *>(pack + Cf::P_WQW)[i] =
            make_uint4(v[0] | v[1] << 16, v[2] | v[3] << 16, v[4] | v[5] << 16, v[6] | v[7] << 16);
        return;
    }
    i -= E_WQW;
    if (i < E_WPW) {
        const int f = i >> 6;
        const int hd = f % HEADS, ot = f / HEADS;
        const int o = 16 * ot + l16;
        uint32_t v[8];
        for (int s = 0; s < 8; ++s) {
            const int fe = slot_feature(s);
            v[s] = (o < C && fe < D) ? (uint32_t)w_proj[(size_t)o * C + hd * D + fe].bits : 0u;
        }
        reinterpret_cast<uint4 *>(pack + Cf::P_WPW)[i] =
            make_uint4(v[0] | v[1] << 16, v[2] | v[3] << 16, v[4] | v[5] << 16, v[6] | v[7] << 16);
        return;
    }
    i -= E_WPW;
    if (i < E_TBW) {
        const int hd = i / Cf::TBW_PITCH, e = i % Cf::TBW_PITCH;
        reinterpret_cast<float *>(pack + Cf::P_TBW)[i] = e < 225 ? to_f32(table[e * HEADS + hd]) * kLog2e : 0.f;
        return;
    }
    i -= E_TBW;
    if (i < E_WQX) { // Wqkv^T for the backward: row l16 -> input channel (per head of the group), k-slots -> features of (hd, t)
        int f = i >> 6;
        const int ct = f % Cf::CTF; f /= Cf::CTF;
        const int t = f % 3;
        const int hd = f / 3, gi = hd / HG, hl = hd % HG;
        const int cl = 16 * (ct % ET) + (i & 15), c = (ct / ET) * D + cl; // channel inside its head, inside the group
        const int qq = (i >> 4) & 3;
        const float sc = t == 0 ? 1.0f / sqrtf((float)D) : 1.0f;
        uint32_t v[8];
        for (int s = 0; s < 8; ++s) {
            const int fe = s < 4 ? 4 * qq + s : 16 + 4 * qq + (s - 4);
            float w = 0.f;
            if (cl < D && fe < D) w = to_f32(w_qkv[((size_t)gi * 3 * CG + t * CG + hl * D + fe) * CG + c]) * sc;
            v[s] = f32_to_bf16_bits(w);
        }
        reinterpret_cast<uint4 *>(pack + Cf::P_WQX)[i] =
            make_uint4(v[0] | v[1] << 16, v[2] | v[3] << 16, v[4] | v[5] << 16, v[6] | v[7] << 16);
        return;
    }
    i -= E_WQX;
    if (i < Cf::N_WQN * 64) { // (hd, t, et, ks): row l16 -> feature 16 et + l16, k-slots -> channels 32 ks + 8 q ..
        int f = i >> 6;
        const int ks = f % Cf::KS; f /= Cf::KS;
        const int et = f % ET; f /= ET;
        const int t = f % 3;
        const int hd = f / 3, gi = hd / HG, hl = hd % HG;
        const int e = 16 * et + (i & 15);
        const int c0 = 32 * ks + 8 * ((i >> 4) & 3);
        uint32_t v[8];
        for (int s = 0; s < 8; ++s) {
            float w = 0.f;
            if (e < D && c0 + s < CG)
                w = to_f32(w_qkv[((size_t)gi * 3 * CG + t * CG + hl * D + e) * CG + c0 + s]) * (t == 0 ? qscale : 1.0f);
            v[s] = f32_to_bf16_bits(w);
        }
        reinterpret_cast<uint4 *>(pack + Cf::P_WQN)[i] =
            make_uint4(v[0] | v[1] << 16, v[2] | v[3] << 16, v[4] | v[5] << 16, v[6] | v[7] << 16);
    }
}

// Wide layers (C = 180) with 8x8 windows: the whole forward in one launch, one wavefront per
// window, the weights streamed through LDS (wide_fwd.hip).  `attn` receives the group outputs when
// `training` (the caller keeps them for the backward pass); otherwise it is not touched.
bool wide_fwd_supported(const Geom &g);
hipError_t launch_wide_fwd(const Geom &g, const bf16_t *x, const void *pack, bf16_t *y, bf16_t *attn,
                           int training, hipStream_t s);

// Sums the per-workgroup partial vectors of one launch and scatters their segments to the gradients
// (fixed summation order).  Segment k covers entries [begin[k], begin[k+1]) of a partial vector and
// goes to ptr[k] + offset, contiguously; the last segment (if tbl_heads > 0) is the bias-table
// gradient, stored head by head in the partial vector and scattered to
// dtable[entry * tbl_stride + tbl_head0 + head].
struct ReduceOut {
    static constexpr int MAXSEG = 22;
    float *ptr[MAXSEG];
    int begin[MAXSEG + 1];
    int nseg;
    int tbl_heads, tbl_entries, tbl_stride, tbl_head0;
};
hipError_t launch_reduce(const float *part, int nparts, int n, const ReduceOut &out, int accumulate, hipStream_t s);
// two such sums in one launch (the second with short vectors, e.g. a bias-table gradient)
struct ReduceJob {
    const float *part;
    int nparts, n;
    ReduceOut out;
    int accumulate;
};
hipError_t launch_reduce_pair(const ReduceJob &a, const ReduceJob &b, hipStream_t s);

// Wide layers (C = 180, two or three groups, 8x8 windows), backward of the attention and of the QKV
// projection, group by group in reverse order (wide_bwd.hip): one launch with one wavefront per
// window recomputes the group's q, k, v and probabilities and leaves d(q|k|v) in scratch and the
// bias-table gradient as per-workgroup partial sums; a second launch turns d(q|k|v) into the
// group's dx slice (the cascade gradient of the group before, Eq. 8) and its weight gradients.
// d w_proj / d b_proj are not produced here.
bool wide_bwd_supported(const Geom &g);
size_t wide_bwd_ws_bytes(const Geom &g);
hipError_t launch_wide_bwd(const Geom &g, const bf16_t *x, const bf16_t *dy, const bf16_t *attn, const void *pack,
                           bf16_t *dx, float *dw_qkv, float *db_qkv, float *dtable, int accumulate, void *ws,
                           hipStream_t s);

bool fused_bwd_supported(const Geom &g);
// Scratch of the fused backward: per-workgroup partial parameter gradients.
size_t fused_bwd_ws_bytes(const Geom &g);

// dx and the five parameter gradients from x, dy and the saved group outputs.  The parameter
// gradients are summed over per-workgroup partials in a fixed order (run-to-run identical) and
// overwrite their outputs unless `accumulate`.
// `pack` is the buffer the forward call of the same layer filled.
hipError_t launch_fused_bwd(const Geom &g, const bf16_t *x, const bf16_t *dy, const bf16_t *attn,
                            const void *pack, const bf16_t *table, bf16_t *dx, float *dw_qkv,
                            float *db_qkv, float *dw_proj, float *db_proj, float *dtable, int accumulate,
                            void *ws, hipStream_t s);

} // namespace gswa
