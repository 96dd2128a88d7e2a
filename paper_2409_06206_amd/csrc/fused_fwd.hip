// Fused GSWA forward: shift + partition + per-group QKV projection (Eq. 6) with the cascade add
// (Eq. 8) + scores with relative bias and shift mask + softmax + PV + output projection (Eq. 7)
// + window merge + reverse shift, one kernel, one pass over x and y.
#include "fused.h"
#include "mfma.h"

namespace gswa {

namespace {

constexpr float kLog2e = 1.4426950408889634f;

// ---------------------------------------------------------------------------------------
// Parameter packing (see FusedCfg): every thread assembles the operand of one (fragment, lane).
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t bf16_scaled(bf16_t w, float sc)
{
    return sc == 1.0f ? (uint32_t)w.bits : (uint32_t)f32_to_bf16_bits(to_f32(w) * sc);
}

template <class Cf>
__global__ __launch_bounds__(256) void pack_params_kernel(const bf16_t *__restrict__ w_qkv,
                                                          const bf16_t *__restrict__ b_qkv,
                                                          const bf16_t *__restrict__ w_proj,
                                                          const bf16_t *__restrict__ b_proj,
                                                          uint8_t *__restrict__ pack)
{
    constexpr int C = Cf::C, D = Cf::D, CG = Cf::CG, HG = Cf::HG, HEADS = Cf::HEADS, ET = Cf::ET;
    constexpr int KS = Cf::KS, KSC = Cf::KSC;
    constexpr int E_WC = Cf::N_WC * 64, E_WP = Cf::N_WP * 64, E_WQ = Cf::N_WQ * 64, E_WPT = Cf::N_WPT * 64,
                  E_WQT = Cf::N_WQT * 64, E_BIAS = 4 * C;
    const float qscale = 1.0f / sqrtf((float)D);
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    int l16 = i & 15, q = (i >> 4) & 3; // lane coordinates inside the current segment

    if (i < E_WC) { // cascade input: m/n-index l16 -> out feature e; k-slots 4q+j -> prev-group channel
        int f = i >> 6;
        const int etp = f % ET; f /= ET;
        const int hlp = f % HG; f /= HG;
        const int et = f % ET; f /= ET;
        const int t = f % 3; f /= 3;
        const int hl = f % HG;
        const int gi = f / HG + 1;
        const int e = 16 * et + l16;
        uint32_t v[4];
        for (int j = 0; j < 4; ++j) {
            const int ep = 16 * etp + 4 * q + j;
            v[j] = (e < D && ep < D)
                       ? bf16_scaled(w_qkv[((size_t)gi * 3 * CG + t * CG + hl * D + e) * CG + hlp * D + ep], t == 0 ? qscale : 1.0f)
                       : 0u;
        }
        reinterpret_cast<uint2 *>(pack + Cf::P_WC)[i] = make_uint2(v[0] | v[1] << 16, v[2] | v[3] << 16);
        return;
    }
    i -= E_WC;
    if (i < E_WP) { // Wproj: l16 -> output channel o; k-slots 4q+j -> input channel (hd, e)
        int f = i >> 6;
        const int et = f % ET; f /= ET;
        const int hd = f % HEADS;
        const int ot = f / HEADS;
        const int o = 16 * ot + l16;
        uint32_t v[4];
        for (int j = 0; j < 4; ++j) {
            const int e = 16 * et + 4 * q + j;
            v[j] = (o < C && e < D) ? (uint32_t)w_proj[(size_t)o * C + hd * D + e].bits : 0u;
        }
        reinterpret_cast<uint2 *>(pack + Cf::P_WP)[i] = make_uint2(v[0] | v[1] << 16, v[2] | v[3] << 16);
        return;
    }
    i -= E_WP;
    if (i < E_WQ) { // Wqkv on the x slice: l16 -> out feature e; k-slots 8q+s -> channel 32ks+8q+s
        int f = i >> 6;
        const int ks = f % KS; f /= KS;
        const int et = f % ET; f /= ET;
        const int t = f % 3;
        const int hd = f / 3, gi = hd / HG, hl = hd % HG;
        const int e = 16 * et + l16;
        uint32_t v[8];
        for (int s = 0; s < 8; ++s) {
            const int c = 32 * ks + 8 * q + s;
            v[s] = (e < D && c < CG)
                       ? bf16_scaled(w_qkv[((size_t)gi * 3 * CG + t * CG + hl * D + e) * CG + c], t == 0 ? qscale : 1.0f)
                       : 0u;
        }
        reinterpret_cast<uint4 *>(pack + Cf::P_WQ)[i] =
            make_uint4(v[0] | v[1] << 16, v[2] | v[3] << 16, v[4] | v[5] << 16, v[6] | v[7] << 16);
        return;
    }
    i -= E_WQ;
    if (i < E_BIAS) { // fp32 biases; the q third of every group scaled like its weights
        float *bias = reinterpret_cast<float *>(pack + Cf::P_BIAS);
        if (i < 3 * C) bias[i] = to_f32(b_qkv[i]) * ((i % (3 * CG)) < CG ? qscale : 1.0f);
        else bias[i] = to_f32(b_proj[i - 3 * C]);
        return;
    }
    i -= E_BIAS; // not a multiple of 64: re-derive the lane coordinates
    l16 = i & 15;
    q = (i >> 4) & 3;
    if (i < E_WPT) { // Wproj^T: l16 -> input channel (hd, e); k-slots 8q+s -> output channel o
        int f = i >> 6;
        const int ks = f % KSC; f /= KSC;
        const int et = f % ET;
        const int hd = f / ET;
        const int e = 16 * et + l16;
        uint32_t v[8];
        for (int s = 0; s < 8; ++s) {
            const int o = 32 * ks + 8 * q + s;
            v[s] = (e < D && o < C) ? (uint32_t)w_proj[(size_t)o * C + hd * D + e].bits : 0u;
        }
        reinterpret_cast<uint4 *>(pack + Cf::P_WPT)[i] =
            make_uint4(v[0] | v[1] << 16, v[2] | v[3] << 16, v[4] | v[5] << 16, v[6] | v[7] << 16);
        return;
    }
    i -= E_WPT;
    if (i < E_WQT) { // Wqkv^T: l16 -> input channel hlp*D + 16etp + l16; k-slots 4q+j -> out feature (t,hl,e)
        int f = i >> 6;
        const int etp = f % ET; f /= ET;
        const int hlp = f % HG; f /= HG;
        const int et = f % ET; f /= ET;
        const int t = f % 3;
        const int hd = f / 3, gi = hd / HG, hl = hd % HG;
        const int cp = 16 * etp + l16;
        uint32_t v[4];
        for (int j = 0; j < 4; ++j) {
            const int e = 16 * et + 4 * q + j;
            v[j] = (cp < D && e < D)
                       ? bf16_scaled(w_qkv[((size_t)gi * 3 * CG + t * CG + hl * D + e) * CG + hlp * D + cp], t == 0 ? qscale : 1.0f)
                       : 0u;
        }
        reinterpret_cast<uint2 *>(pack + Cf::P_WQT)[i] = make_uint2(v[0] | v[1] << 16, v[2] | v[3] << 16);
        return;
    }
    i -= E_WQT;
    if (i < Cf::N_WPK * 64) { // Wproj for the projection GEMM: l16 -> output channel; k-slots 8q+s -> input channel
        const int f = i >> 6;
        const int ks = f % KSC, ot = f / KSC;
        const int o = 16 * ot + l16;
        uint32_t v[8];
        for (int s = 0; s < 8; ++s) {
            const int c = 32 * ks + 8 * q + s;
            v[s] = (o < C && c < C) ? (uint32_t)w_proj[(size_t)o * C + c].bits : 0u;
        }
        reinterpret_cast<uint4 *>(pack + Cf::P_WPK)[i] =
            make_uint4(v[0] | v[1] << 16, v[2] | v[3] << 16, v[4] | v[5] << 16, v[6] | v[7] << 16);
    }
}

// fragment ids inside the packed arrays
template <class Cf> __device__ __forceinline__ constexpr int fq(int hd, int t, int et, int ks)
{
    return ((hd * 3 + t) * Cf::ET + et) * Cf::KS + ks;
}
template <class Cf> __device__ __forceinline__ constexpr int fc(int gi, int hl, int t, int et, int hlp, int etp)
{
    return (((((gi - 1) * Cf::HG + hl) * 3 + t) * Cf::ET + et) * Cf::HG + hlp) * Cf::ET + etp;
}

template <class Cf>
__global__ __launch_bounds__(256, 3) void fused_fwd_kernel(Geom g, const bf16_t *__restrict__ x,
                                                        const uint8_t *__restrict__ pack,
                                                        const bf16_t *__restrict__ table,
                                                        bf16_t *__restrict__ y, bf16_t *__restrict__ attn)
{
    constexpr int C = Cf::C, D = Cf::D, CG = Cf::CG, HG = Cf::HG, HEADS = Cf::HEADS, G = Cf::G;
    constexpr int ET = Cf::ET, KS = Cf::KS, OT = Cf::OT, VT_LD = Cf::VT_LD;
    constexpr int M = 8, NTBL = (2 * M - 1) * (2 * M - 1);
    static_assert(CG % 2 == 0 && D % 2 == 0 && C % 4 == 0, "dword-granular loads and stores");
    static_assert((size_t)NTBL * HEADS * 2 <= Cf::K_BYTES + Cf::VT_BYTES, "table staging aliases the K buffers");

    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const uint4 *wq = reinterpret_cast<const uint4 *>(lds + Cf::OFF_WQ);
    const uint2 *wc = reinterpret_cast<const uint2 *>(lds + Cf::OFF_WC);
    const uint2 *wp = reinterpret_cast<const uint2 *>(lds + Cf::OFF_WP);
    const float *bqkv = reinterpret_cast<const float *>(lds + Cf::OFF_BIAS);
    const float *bproj = bqkv + 3 * C;
    uint2 *kbuf = reinterpret_cast<uint2 *>(lds + Cf::OFF_K);
    uint16_t *vt = reinterpret_cast<uint16_t *>(lds + Cf::OFF_VT);

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, l16 = lane & 15, q = lane >> 4;

    // ---- set-up: weights into LDS, bias table into registers in score-fragment order ----
    for (int i = tid; i < (int)(Cf::FWD_PACK_BYTES / 16); i += 256)
        reinterpret_cast<uint4 *>(lds)[i] = reinterpret_cast<const uint4 *>(pack)[i];
    uint16_t *tstage = reinterpret_cast<uint16_t *>(kbuf);
    for (int i = tid; i < NTBL * HEADS; i += 256) tstage[i] = table[i].bits;
    __syncthreads();

    // this lane's token inside the window: query column of every score tile it holds
    const int rn = 2 * wv + (l16 >> 3), cn = l16 & 7;
    uint32_t bias_frag[HEADS][8];
#pragma unroll
    for (int hd = 0; hd < HEADS; ++hd)
#pragma unroll
        for (int kt = 0; kt < 4; ++kt)
#pragma unroll
            for (int jp = 0; jp < 2; ++jp) {
                uint32_t pr = 0;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int m = 16 * kt + 4 * q + 2 * jp + h;
                    const int rm = m >> 3, cm = m & 7;
                    const int idx = (rn - rm + M - 1) * (2 * M - 1) + (cn - cm + M - 1);
                    pr |= (uint32_t)tstage[idx * HEADS + hd] << (16 * h);
                }
                bias_frag[hd][kt * 2 + jp] = pr;
            }
    // shift mask: a key is masked for this lane's query when their wrap flags differ
    const int s = g.shift;
    bool rmask[4], cmask[4];
#pragma unroll
    for (int kt = 0; kt < 4; ++kt) rmask[kt] = (rn >= M - s) != ((2 * kt + (q >> 1)) >= M - s);
#pragma unroll
    for (int j = 0; j < 4; ++j) cmask[j] = (cn >= M - s) != ((4 * (q & 1) + j) >= M - s);
    __syncthreads();

    const int per_img = g.nwi * g.nwj;

    for (int win = blockIdx.x; win < g.nW; win += gridDim.x) {
        const int b = win / per_img;
        const int wr = win - b * per_img;
        const int wi = wr / g.nwj, wj = wr - wi * g.nwj;
        int si = wi * M + rn + s, sj = wj * M + cn + s;
        if (si >= g.H) si -= g.H;
        if (sj >= g.W) sj -= g.W;
        const long tok = ((long)b * g.H + si) * g.W + sj;
        const bool lastrow = s > 0 && wi == g.nwi - 1, lastcol = s > 0 && wj == g.nwj - 1;

        // x row of this lane's token as B/A operands: k-slot 8q+s of step ks <-> channel 32ks+8q+s
        const uint32_t *xrow = reinterpret_cast<const uint32_t *>(x + tok * C);
        uint4 xf[G][KS];
#pragma unroll
        for (int gi = 0; gi < G; ++gi)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                uint32_t dwv[4];
#pragma unroll
                for (int dw = 0; dw < 4; ++dw) {
                    const int c = 32 * ks + 8 * q + 2 * dw;
                    dwv[dw] = c < CG ? xrow[(gi * CG + c) >> 1] : 0u;
                }
                xf[gi][ks] = make_uint4(dwv[0], dwv[1], dwv[2], dwv[3]);
            }

        uint2 Ob[HEADS][ET];
#pragma unroll
        for (int hd = 0; hd < HEADS; ++hd) {
            const int gi = hd / HG, hl = hd % HG;
            // ---- Q^T, K^T (rows = head features) and V (rows = tokens) of this wave's tokens ----
            f32x4 qT[ET], kT[ET], vv[ET];
#pragma unroll
            for (int et = 0; et < ET; ++et) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int e = 16 * et + 4 * q + j;
                    qT[et][j] = e < D ? bqkv[gi * 3 * CG + hl * D + e] : 0.f;
                    kT[et][j] = e < D ? bqkv[gi * 3 * CG + CG + hl * D + e] : 0.f;
                }
                const int ev = 16 * et + l16;
                const float bv = ev < D ? bqkv[gi * 3 * CG + 2 * CG + hl * D + ev] : 0.f;
                vv[et] = f32x4{bv, bv, bv, bv};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    qT[et] = mma32(wq[fq<Cf>(hd, 0, et, ks) * 64 + lane], xf[gi][ks], qT[et]);
                    kT[et] = mma32(wq[fq<Cf>(hd, 1, et, ks) * 64 + lane], xf[gi][ks], kT[et]);
                    vv[et] = mma32(xf[gi][ks], wq[fq<Cf>(hd, 2, et, ks) * 64 + lane], vv[et]);
                }
                if (gi > 0 && g.cascade) {
#pragma unroll
                    for (int hlp = 0; hlp < HG; ++hlp)
#pragma unroll
                        for (int etp = 0; etp < ET; ++etp) {
                            const uint2 prev = Ob[(gi > 0 ? gi - 1 : 0) * HG + hlp][etp];
                            qT[et] = mma16(wc[fc<Cf>(gi > 0 ? gi : 1, hl, 0, et, hlp, etp) * 64 + lane], prev, qT[et]);
                            kT[et] = mma16(wc[fc<Cf>(gi > 0 ? gi : 1, hl, 1, et, hlp, etp) * 64 + lane], prev, kT[et]);
                            vv[et] = mma16(prev, wc[fc<Cf>(gi > 0 ? gi : 1, hl, 2, et, hlp, etp) * 64 + lane], vv[et]);
                        }
                }
            }
            // ---- K and V of all 64 tokens to the other waves ----
            uint2 Qb[ET];
#pragma unroll
            for (int et = 0; et < ET; ++et) {
                Qb[et] = pack_bf16x4(qT[et]);
                kbuf[(wv * ET + et) * 64 + lane] = pack_bf16x4(kT[et]);
                *reinterpret_cast<uint2 *>(vt + (et * 16 + l16) * VT_LD + 16 * wv + 4 * q) =
                    pack_bf16x4(vv[et]);
            }
            __syncthreads();

            // ---- S^T tiles: rows = keys 16kt+4q+j, column = this lane's query ----
            f32x4 st[4];
#pragma unroll
            for (int kt = 0; kt < 4; ++kt) {
                st[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int et = 0; et < ET; ++et)
                    st[kt] = mma16(kbuf[(kt * ET + et) * 64 + lane], Qb[et], st[kt]);
            }
            float mx = -INFINITY;
#pragma unroll
            for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t pr = bias_frag[hd][kt * 2 + (j >> 1)];
                    const float bv = (j & 1) ? bf16_hi(pr) : bf16_lo(pr);
                    st[kt][j] += bv;
                }
            if (lastrow || lastcol) {
#pragma unroll
                for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if ((lastrow && rmask[kt]) || (lastcol && cmask[j])) st[kt][j] += -100.0f;
            }
#pragma unroll
            for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                for (int j = 0; j < 4; ++j) mx = fmaxf(mx, st[kt][j]);
            mx = qgroup_max(mx);
            const float mxl = mx * kLog2e;
            float sum = 0.f;
            uint2 Pb[4];
#pragma unroll
            for (int kt = 0; kt < 4; ++kt) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float p = __builtin_amdgcn_exp2f(fmaf(st[kt][j], kLog2e, -mxl));
                    st[kt][j] = p;
                    sum += p;
                }
                Pb[kt] = pack_bf16x4(st[kt]);
            }
            sum = qgroup_sum(sum);
            const float inv = 1.0f / sum;

            // ---- O^T = V^T P^T: rows = head features, column = this lane's token ----
#pragma unroll
            for (int et = 0; et < ET; ++et) {
                f32x4 oT = f32x4{0.f, 0.f, 0.f, 0.f};
                const uint16_t *vrow = vt + (et * 16 + l16) * VT_LD + 4 * q;
#pragma unroll
                for (int kp = 0; kp < 2; ++kp) {
                    const uint2 a0 = *reinterpret_cast<const uint2 *>(vrow + 32 * kp);
                    const uint2 a1 = *reinterpret_cast<const uint2 *>(vrow + 32 * kp + 16);
                    oT = mma32(make_uint4(a0.x, a0.y, a1.x, a1.y),
                               make_uint4(Pb[2 * kp].x, Pb[2 * kp].y, Pb[2 * kp + 1].x, Pb[2 * kp + 1].y), oT);
                }
                oT *= inv;
                Ob[hd][et] = pack_bf16x4(oT);
                if (attn) {
                    const int e0 = 16 * et + 4 * q;
                    uint32_t *dst = reinterpret_cast<uint32_t *>(attn + tok * C + hd * D + e0);
                    if (e0 < D) dst[0] = Ob[hd][et].x;
                    if (e0 + 2 < D) dst[1] = Ob[hd][et].y;
                }
            }
            __syncthreads(); // K and V of this head are consumed; the next head may overwrite them
        }

        // ---- Y^T = Wproj A^T + b: rows = output channels, column = this lane's token ----
#pragma unroll
        for (int ot = 0; ot < OT; ++ot) {
            f32x4 acc;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int o = 16 * ot + 4 * q + j;
                acc[j] = o < C ? bproj[o] : 0.f;
            }
#pragma unroll
            for (int hd = 0; hd < HEADS; ++hd)
#pragma unroll
                for (int et = 0; et < ET; ++et)
                    acc = mma16(wp[((ot * HEADS + hd) * ET + et) * 64 + lane], Ob[hd][et], acc);
            const int o0 = 16 * ot + 4 * q;
            if (o0 < C) *reinterpret_cast<uint2 *>(y + tok * C + o0) = pack_bf16x4(acc);
        }
    }
}

// ---------------------------------------------------------------------------------------
// Split forward for wide layers: attention of heads [HB, HE) (one group or part of one), the
// cascade input of Eq. 8 read back from the group outputs in memory, no projection.  Window side
// M is 8 or 16: a workgroup has N/16 waves, wave w owns tokens 16w..16w+15 of the window and holds
// the N keys of each of its queries as N/16 score tiles.
// ---------------------------------------------------------------------------------------
template <class Cf, int HB_, int HE_, int M_> struct AttnChunkCfg {
    static constexpr int HB = HB_, HE = HE_, NH = HE - HB, M = M_, N = M * M, NWV = N / 16, KT = N / 16;
    static constexpr int NTBL = (2 * M - 1) * (2 * M - 1);
    static constexpr int VT_LD = N + 4;
    static constexpr int N_WQ = NH * 3 * Cf::ET * Cf::KS;
    static constexpr size_t SRC_WQ = Cf::P_WQ + (size_t)HB * 3 * Cf::ET * Cf::KS * 1024;
    static constexpr size_t OFF_WQ = 0;
    static constexpr size_t OFF_BIAS = (size_t)N_WQ * 1024;
    static constexpr size_t OFF_TBLF = OFF_BIAS + (size_t)16 * Cf::C;          // fp32 [NH][NTBL]
    static constexpr size_t OFF_K = OFF_TBLF + (((size_t)NH * NTBL * 4 + 15) & ~size_t(15));
    static constexpr size_t K_BYTES = (size_t)KT * Cf::ET * 64 * 8;
    static constexpr size_t OFF_VT = OFF_K + K_BYTES;
    static constexpr size_t VT_BYTES = (size_t)16 * Cf::ET * VT_LD * 2;
    static constexpr size_t LDS_BYTES = OFF_VT + VT_BYTES;
    static_assert(HB / Cf::HG == (HE - 1) / Cf::HG, "a chunk stays inside one head group");
    static_assert(M == 8 || M == 16, "window side");
};

template <class Cf, int HB, int HE, int M>
__global__ __launch_bounds__(4 * M * M, M == 8 ? 2 : 1) void fused_attn_fwd_kernel(Geom g, const bf16_t *__restrict__ x,
                                                                                   const uint8_t *__restrict__ pack,
                                                                                   const bf16_t *__restrict__ table,
                                                                                   bf16_t *attn)
{
    using A = AttnChunkCfg<Cf, HB, HE, M>;
    constexpr int C = Cf::C, D = Cf::D, CG = Cf::CG, HG = Cf::HG, HEADS = Cf::HEADS;
    constexpr int ET = Cf::ET, KS = Cf::KS, VT_LD = A::VT_LD, NH = A::NH, KT = A::KT, NTBL = A::NTBL;
    constexpr int NTHREADS = 64 * A::NWV;
    constexpr int GI = HB / HG;              // the group of this chunk
    constexpr int ROWSTEP = (16 / M) * (2 * M - 1); // table-index step from one key tile to the next
    static_assert(CG % 2 == 0 && D % 2 == 0 && C % 4 == 0, "dword-granular loads and stores");

    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const uint4 *wq = reinterpret_cast<const uint4 *>(lds + A::OFF_WQ);
    const float *bqkv = reinterpret_cast<const float *>(lds + A::OFF_BIAS);
    float *tblf = reinterpret_cast<float *>(lds + A::OFF_TBLF);
    uint2 *kbuf = reinterpret_cast<uint2 *>(lds + A::OFF_K);
    uint16_t *vt = reinterpret_cast<uint16_t *>(lds + A::OFF_VT);

    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, q = lane >> 4;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);

    for (int i = tid; i < A::N_WQ * 64; i += NTHREADS)
        reinterpret_cast<uint4 *>(lds + A::OFF_WQ)[i] = reinterpret_cast<const uint4 *>(pack + A::SRC_WQ)[i];
    for (int i = tid; i < C; i += NTHREADS)
        reinterpret_cast<uint4 *>(lds + A::OFF_BIAS)[i] = reinterpret_cast<const uint4 *>(pack + Cf::P_BIAS)[i];
    for (int i = tid; i < NTBL * NH; i += NTHREADS) tblf[i] = to_f32(table[(i % NTBL) * HEADS + HB + i / NTBL]);

    // this lane's query inside the window; key 16kt+4q+j sits at (key_r0 + (16/M)kt, key_c0 + j)
    const int nq = 16 * wv + l16, rn = nq / M, cn = nq % M;
    const int key_r0 = (4 * q) / M, key_c0 = (4 * q) % M;
    const int idx0 = (rn - key_r0 + M - 1) * (2 * M - 1) + (cn - key_c0 + M - 1);
    const int s = g.shift;
    bool cmask[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) cmask[j] = (cn >= M - s) != ((key_c0 + j) >= M - s);
    const bool q_wrapped_row = rn >= M - s;
    __syncthreads();

    const int per_img = g.nwi * g.nwj;
    const bool casc = GI > 0 && g.cascade;

    for (int win = blockIdx.x; win < g.nW; win += gridDim.x) {
        const int b = win / per_img;
        const int wr = win - b * per_img;
        const int wi = wr / g.nwj, wj = wr - wi * g.nwj;
        int si = wi * M + rn + s, sj = wj * M + cn + s;
        if (si >= g.H) si -= g.H;
        if (sj >= g.W) sj -= g.W;
        const long tok = ((long)b * g.H + si) * g.W + sj;
        const bool lastrow = s > 0 && wi == g.nwi - 1, lastcol = s > 0 && wj == g.nwj - 1;

        const uint32_t *xrow = reinterpret_cast<const uint32_t *>(x + tok * C + GI * CG);
        const uint32_t *arow = reinterpret_cast<const uint32_t *>(attn + tok * C + (GI > 0 ? GI - 1 : 0) * CG);
        uint4 xf[KS], af[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            uint32_t xv[4], av[4];
#pragma unroll
            for (int dw = 0; dw < 4; ++dw) {
                const int c = 32 * ks + 8 * q + 2 * dw;
                xv[dw] = c < CG ? xrow[c >> 1] : 0u;
                av[dw] = (casc && c < CG) ? arow[c >> 1] : 0u;
            }
            xf[ks] = make_uint4(xv[0], xv[1], xv[2], xv[3]);
            af[ks] = make_uint4(av[0], av[1], av[2], av[3]);
        }

#pragma unroll
        for (int hx = 0; hx < NH; ++hx) {
            const int hd = HB + hx, hl = hd % HG;
            f32x4 qT[ET], kT[ET], vv[ET];
#pragma unroll
            for (int et = 0; et < ET; ++et) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int e = 16 * et + 4 * q + j;
                    qT[et][j] = e < D ? bqkv[GI * 3 * CG + hl * D + e] : 0.f;
                    kT[et][j] = e < D ? bqkv[GI * 3 * CG + CG + hl * D + e] : 0.f;
                }
                const int ev = 16 * et + l16;
                const float bv = ev < D ? bqkv[GI * 3 * CG + 2 * CG + hl * D + ev] : 0.f;
                vv[et] = f32x4{bv, bv, bv, bv};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const uint4 fq_ = wq[fq<Cf>(hx, 0, et, ks) * 64 + lane];
                    const uint4 fk_ = wq[fq<Cf>(hx, 1, et, ks) * 64 + lane];
                    const uint4 fv_ = wq[fq<Cf>(hx, 2, et, ks) * 64 + lane];
                    qT[et] = mma32(fq_, xf[ks], qT[et]);
                    kT[et] = mma32(fk_, xf[ks], kT[et]);
                    vv[et] = mma32(xf[ks], fv_, vv[et]);
                    if (casc) {
                        qT[et] = mma32(fq_, af[ks], qT[et]);
                        kT[et] = mma32(fk_, af[ks], kT[et]);
                        vv[et] = mma32(af[ks], fv_, vv[et]);
                    }
                }
            }
            uint2 Qb[ET];
#pragma unroll
            for (int et = 0; et < ET; ++et) {
                Qb[et] = pack_bf16x4(qT[et]);
                kbuf[(wv * ET + et) * 64 + lane] = pack_bf16x4(kT[et]);
                *reinterpret_cast<uint2 *>(vt + (et * 16 + l16) * VT_LD + 16 * wv + 4 * q) = pack_bf16x4(vv[et]);
            }
            __syncthreads();

            // scores: tile kt holds keys 16kt+4q+j (rows) for this lane's query (column)
            f32x4 st[KT];
            float mx = -INFINITY;
#pragma unroll
            for (int kt = 0; kt < KT; ++kt) {
#pragma unroll
                for (int j = 0; j < 4; ++j) st[kt][j] = tblf[hx * NTBL + idx0 - ROWSTEP * kt - j];
#pragma unroll
                for (int et = 0; et < ET; ++et)
                    st[kt] = mma16(kbuf[(kt * ET + et) * 64 + lane], Qb[et], st[kt]);
            }
            if (lastrow || lastcol) {
#pragma unroll
                for (int kt = 0; kt < KT; ++kt) {
                    const bool rmask = q_wrapped_row != ((key_r0 + (16 / M) * kt) >= M - s);
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if ((lastrow && rmask) || (lastcol && cmask[j])) st[kt][j] += -100.0f;
                }
            }
#pragma unroll
            for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                for (int j = 0; j < 4; ++j) mx = fmaxf(mx, st[kt][j]);
            mx = qgroup_max(mx);
            const float mxl = mx * kLog2e;
            float sum = 0.f;
            uint2 Pb[KT];
#pragma unroll
            for (int kt = 0; kt < KT; ++kt) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float p = __builtin_amdgcn_exp2f(fmaf(st[kt][j], kLog2e, -mxl));
                    st[kt][j] = p;
                    sum += p;
                }
                Pb[kt] = pack_bf16x4(st[kt]);
            }
            sum = qgroup_sum(sum);
            const float inv = 1.0f / sum;
#pragma unroll
            for (int et = 0; et < ET; ++et) {
                f32x4 oT = f32x4{0.f, 0.f, 0.f, 0.f};
                const uint16_t *vrow = vt + (et * 16 + l16) * VT_LD + 4 * q;
#pragma unroll
                for (int kp = 0; kp < KT / 2; ++kp) {
                    const uint2 a0 = *reinterpret_cast<const uint2 *>(vrow + 32 * kp);
                    const uint2 a1 = *reinterpret_cast<const uint2 *>(vrow + 32 * kp + 16);
                    oT = mma32(make_uint4(a0.x, a0.y, a1.x, a1.y),
                               make_uint4(Pb[2 * kp].x, Pb[2 * kp].y, Pb[2 * kp + 1].x, Pb[2 * kp + 1].y), oT);
                }
                oT *= inv;
                const uint2 ob = pack_bf16x4(oT);
                const int e0 = 16 * et + 4 * q;
                uint32_t *dst = reinterpret_cast<uint32_t *>(attn + tok * C + hd * D + e0);
                if (e0 < D) dst[0] = ob.x;
                if (e0 + 2 < D) dst[1] = ob.y;
            }
            __syncthreads(); // K and V of this head are consumed
        }
    }
}

// y = A Wproj^T + b over plain token rows (A holds the group outputs at the tokens' own
// positions, so no index map is needed here).  64 tokens per workgroup pass.
template <class Cf>
__global__ __launch_bounds__(256, 2) void proj_gemm_kernel(long T, const bf16_t *__restrict__ attn,
                                                           const uint8_t *__restrict__ pack,
                                                           bf16_t *__restrict__ y)
{
    constexpr int C = Cf::C, OT = Cf::OT, KSC = Cf::KSC;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const uint4 *wpk = reinterpret_cast<const uint4 *>(lds);
    const float *bproj = reinterpret_cast<const float *>(lds + (size_t)Cf::N_WPK * 1024);
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, l16 = lane & 15, q = lane >> 4;
    for (int i = tid; i < Cf::N_WPK * 64; i += 256)
        reinterpret_cast<uint4 *>(lds)[i] = reinterpret_cast<const uint4 *>(pack + Cf::P_WPK)[i];
    for (int i = tid; i < C; i += 256)
        reinterpret_cast<float *>(lds + (size_t)Cf::N_WPK * 1024)[i] =
            reinterpret_cast<const float *>(pack + Cf::P_BIAS)[3 * C + i];
    __syncthreads();

    const long ntile = (T + 63) / 64;
    for (long tile = blockIdx.x; tile < ntile; tile += gridDim.x) {
        const long tok = tile * 64 + 16 * wv + l16;
        const bool live = tok < T;
        const uint32_t *arow = reinterpret_cast<const uint32_t *>(attn + (live ? tok : 0) * C);
        uint4 af[KSC];
#pragma unroll
        for (int ks = 0; ks < KSC; ++ks) {
            uint32_t v[4];
#pragma unroll
            for (int dw = 0; dw < 4; ++dw) {
                const int c = 32 * ks + 8 * q + 2 * dw;
                v[dw] = (live && c < C) ? arow[c >> 1] : 0u;
            }
            af[ks] = make_uint4(v[0], v[1], v[2], v[3]);
        }
#pragma unroll 2
        for (int ot = 0; ot < OT; ++ot) { // kept rolled: unrolling all 72 fragment reads spills
            f32x4 acc;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int o = 16 * ot + 4 * q + j;
                acc[j] = o < C ? bproj[o] : 0.f;
            }
#pragma unroll
            for (int ks = 0; ks < KSC; ++ks) acc = mma32(wpk[(ot * KSC + ks) * 64 + lane], af[ks], acc);
            const int o0 = 16 * ot + 4 * q;
            if (live && o0 < C) *reinterpret_cast<uint2 *>(y + tok * C + o0) = pack_bf16x4(acc);
        }
    }
}

int device_cu_count()
{
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
            cus = prop.multiProcessorCount;
        if (cus <= 0) cus = 256;
    }
    return cus;
}

// Forward head chunks of the split path, in launch order (a group's cascade input must be in
// memory before its chunk runs).
template <int G> struct FwdPlan;
template <> struct FwdPlan<1> { static constexpr int N = 3; static constexpr int B[3] = {0, 2, 4}, E[3] = {2, 4, 6}; };
template <> struct FwdPlan<2> { static constexpr int N = 2; static constexpr int B[2] = {0, 3}, E[2] = {3, 6}; };
template <> struct FwdPlan<3> { static constexpr int N = 3; static constexpr int B[3] = {0, 2, 4}, E[3] = {2, 4, 6}; };

template <class Cf, int M, int I = 0>
hipError_t launch_attn_chunks(const Geom &g, const bf16_t *x, const uint8_t *pack, const bf16_t *table,
                              bf16_t *attn, hipStream_t s)
{
    using Plan = FwdPlan<Cf::G>;
    if constexpr (I < Plan::N) {
        using A = AttnChunkCfg<Cf, Plan::B[I], Plan::E[I], M>;
        static_assert(A::LDS_BYTES <= 160 * 1024, "LDS budget");
        auto kern = fused_attn_fwd_kernel<Cf, Plan::B[I], Plan::E[I], M>;
        static bool attr_done = false;
        if (!attr_done && A::LDS_BYTES > 64 * 1024) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)A::LDS_BYTES);
            if (e != hipSuccess) return e;
            attr_done = true;
        }
        int grid = ((M == 8 && A::LDS_BYTES <= 80 * 1024) ? 2 : 1) * device_cu_count();
        if (grid > g.nW) grid = g.nW;
        {
            KernelTimer kt(K_ATTN_CHUNK_FWD, s);
            hipLaunchKernelGGL(kern, dim3(grid), dim3(64 * A::NWV), A::LDS_BYTES, s, g, x, pack, table, attn);
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        return launch_attn_chunks<Cf, M, I + 1>(g, x, pack, table, attn, s);
    }
    return hipSuccess;
}

template <class Cf>
hipError_t run_fwd(const Geom &g, const bf16_t *x, const bf16_t *w_qkv, const bf16_t *b_qkv,
                   const bf16_t *w_proj, const bf16_t *b_proj, const bf16_t *table, bf16_t *y,
                   bf16_t *attn, void *ws, hipStream_t s)
{
    uint8_t *pack = static_cast<uint8_t *>(ws);
    {
        constexpr int entries = (Cf::N_WC + Cf::N_WP + Cf::N_WQ + Cf::N_WPT + Cf::N_WQT + Cf::N_WPK) * 64 + 4 * Cf::C;
        KernelTimer kt(K_PACK_FWD, s);
        hipLaunchKernelGGL(pack_params_kernel<Cf>, dim3((entries + 255) / 256), dim3(256), 0, s, w_qkv, b_qkv,
                           w_proj, b_proj, pack);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if constexpr (Cf::SPLIT) {
        if (!attn) return hipErrorInvalidValue;
        e = g.M == 16 ? launch_attn_chunks<Cf, 16>(g, x, pack, table, attn, s)
                      : launch_attn_chunks<Cf, 8>(g, x, pack, table, attn, s);
        if (e != hipSuccess) return e;
        constexpr size_t lds = (size_t)Cf::N_WPK * 1024 + 4 * Cf::C;
        auto kern = proj_gemm_kernel<Cf>;
        static bool attr_done = false;
        if (!attr_done && lds > 64 * 1024) {
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            attr_done = true;
        }
        long ntile = (g.T + 63) / 64;
        int grid = 2 * device_cu_count();
        if (grid > ntile) grid = (int)ntile;
        KernelTimer kt(K_PROJ_GEMM, s);
        hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, s, g.T, attn, pack, y);
        return hipGetLastError();
    } else {
        auto kern = fused_fwd_kernel<Cf>;
        static bool attr_done = false;
        if (!attr_done && Cf::FWD_LDS_BYTES > 64 * 1024) {
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)Cf::FWD_LDS_BYTES);
            if (e != hipSuccess) return e;
            attr_done = true;
        }
        int grid = 3 * device_cu_count();
        if (grid > g.nW) grid = g.nW;
        KernelTimer kt(K_FUSED_FWD, s);
        hipLaunchKernelGGL(kern, dim3(grid), dim3(256), Cf::FWD_LDS_BYTES, s, g, x, pack, table, y, attn);
        return hipGetLastError();
    }
}

// instantiation table
#define GSWA_FUSED_SHAPES(X) X(60, 6, 1) X(60, 6, 2) X(60, 6, 3) X(60, 6, 6) X(180, 6, 1) X(180, 6, 2) X(180, 6, 3)

} // namespace

bool fused_fwd_supported(const Geom &g)
{
    if (g.M != 8 && g.M != 16) return false;
#define X(C_, H_, G_) \
    if (g.C == C_ && g.heads == H_ && g.groups == G_) return g.M == 8 || FusedCfg<C_, H_, G_>::SPLIT;
    GSWA_FUSED_SHAPES(X)
#undef X
    return false;
}

bool fused_fwd_needs_attn(const Geom &g)
{
#define X(C_, H_, G_) \
    if (g.C == C_ && g.heads == H_ && g.groups == G_) return FusedCfg<C_, H_, G_>::SPLIT;
    GSWA_FUSED_SHAPES(X)
#undef X
    return false;
}

size_t fused_pack_bytes(const Geom &g)
{
#define X(C_, H_, G_) \
    if (g.C == C_ && g.heads == H_ && g.groups == G_) return FusedCfg<C_, H_, G_>::P_END;
    GSWA_FUSED_SHAPES(X)
#undef X
    return 0;
}

hipError_t launch_fused_fwd(const Geom &g, const bf16_t *x, const bf16_t *w_qkv, const bf16_t *b_qkv,
                            const bf16_t *w_proj, const bf16_t *b_proj, const bf16_t *table,
                            bf16_t *y, bf16_t *attn_out, void *pack, hipStream_t s)
{
#define X(C_, H_, G_)                                                  \
    if (g.C == C_ && g.heads == H_ && g.groups == G_)                  \
        return run_fwd<FusedCfg<C_, H_, G_>>(g, x, w_qkv, b_qkv, w_proj, b_proj, table, y, attn_out, pack, s);
    GSWA_FUSED_SHAPES(X)
#undef X
    return hipErrorInvalidValue;
}

} // namespace gswa
