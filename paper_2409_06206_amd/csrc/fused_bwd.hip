// Fused GSWA backward for 8x8 windows, bf16 storage: one kernel recomputes q, k, v, the scores
// and the softmax of every head from x and the saved group outputs, and produces dx, the
// gradients of q|k|v and per-workgroup partial sums of the bias-table gradient.
//
// Per window, wave w owns tokens 16w..16w+15 both as queries and as keys.  Notation for a
// matrix X[tokens x features] held as an MFMA result tile (see mfma.h):
//   T-form: rows = features 4q+j, column = token l16   (packed: B operand "k=feature,n=token"
//           or A operand "m=token,k=feature")
//   N-form: rows = tokens 4q+j,  column = feature l16  (packed: B operand "k=token,n=feature"
//           or A operand "m=feature,k=token")
// Either form of a product is obtained by swapping the operands of the MFMA.
#include "fused.h"
#include "mfma.h"

namespace gswa {

namespace {

constexpr float kLog2e = 1.4426950408889634f;

template <class Cf> struct BwdCfg {
    static constexpr int C = Cf::C, D = Cf::D, CG = Cf::CG, HG = Cf::HG, HEADS = Cf::HEADS, G = Cf::G;
    static constexpr int ET = Cf::ET, KS = Cf::KS;
    static constexpr int KSC = (C + 31) / 32; // K=32 steps over all C channels of dy
    static constexpr int NTBL = 15 * 15;
    // weight fragments (lane-major)
    static constexpr int N_WQ = Cf::N_WQ;                     // recompute, K=32: (hd,t,et,ks)
    static constexpr int N_WC = Cf::N_WC;                     // recompute on cascade input, K=16
    static constexpr int N_WPT = HEADS * ET * KSC;            // Wproj^T, K=32: (hd,et,ks)
    static constexpr int N_WQT = HEADS * 3 * ET * HG * ET;    // Wqkv^T, K=16: (hd,t,et,hlp,etp)
    static constexpr size_t OFF_WQ = 0;
    static constexpr size_t OFF_WC = OFF_WQ + (size_t)N_WQ * 1024;
    static constexpr size_t OFF_WPT = OFF_WC + (size_t)N_WC * 512;
    static constexpr size_t OFF_WQT = OFF_WPT + (size_t)N_WPT * 1024;
    static constexpr size_t OFF_BIAS = OFF_WQT + (size_t)N_WQT * 512; // fp32 b_qkv [3C]
    static constexpr size_t PACK_BYTES = OFF_BIAS + (size_t)16 * C;  // (b_proj slot unused)
    // exchange buffers
    static constexpr int LD = 68;                              // row pitch (bf16) of [feature][64 tokens] and [key][64 queries]
    static constexpr size_t SZ_FRAG = (size_t)4 * ET * 64 * 8; // packed tiles of all 4 waves
    static constexpr size_t SZ_ROWS = (size_t)16 * ET * LD * 2;
    static constexpr size_t SZ_SQ = (size_t)64 * LD * 2;
    static constexpr size_t OFF_KB = PACK_BYTES;               // K, T-form packed tiles
    static constexpr size_t OFF_VB = OFF_KB + SZ_FRAG;         // V, T-form packed tiles
    static constexpr size_t OFF_KT = OFF_VB + SZ_FRAG;         // K^T rows [e][key]
    static constexpr size_t OFF_QT = OFF_KT + SZ_ROWS;         // Q^T rows [e][query], double buffered
    static constexpr size_t OFF_DOT = OFF_QT + 2 * SZ_ROWS;    // dO^T rows [e][query], double buffered
    static constexpr size_t OFF_P = OFF_DOT + 2 * SZ_ROWS;     // P  [key][query]
    static constexpr size_t OFF_DS = OFF_P + SZ_SQ;            // dS [key][query]
    static constexpr size_t LDS_BYTES = OFF_DS + SZ_SQ;
    static constexpr int TBL_N = NTBL * HEADS;
};

template <class Cf>
__global__ __launch_bounds__(256) void pack_bwd_kernel(const bf16_t *__restrict__ w_qkv,
                                                       const bf16_t *__restrict__ b_qkv,
                                                       const bf16_t *__restrict__ w_proj,
                                                       uint8_t *__restrict__ pack)
{
    using B = BwdCfg<Cf>;
    constexpr int C = B::C, D = B::D, CG = B::CG, HG = B::HG, HEADS = B::HEADS, ET = B::ET, KS = B::KS, KSC = B::KSC;
    const int gid = blockIdx.x * blockDim.x + threadIdx.x, stride = gridDim.x * blockDim.x;
    uint16_t *wq = reinterpret_cast<uint16_t *>(pack + B::OFF_WQ);
    uint16_t *wc = reinterpret_cast<uint16_t *>(pack + B::OFF_WC);
    uint16_t *wpt = reinterpret_cast<uint16_t *>(pack + B::OFF_WPT);
    uint16_t *wqt = reinterpret_cast<uint16_t *>(pack + B::OFF_WQT);
    float *bias = reinterpret_cast<float *>(pack + B::OFF_BIAS);

    for (int i = gid; i < B::N_WQ * 64; i += stride) {
        const int lane = i & 63, l16 = lane & 15, q = lane >> 4;
        int f = i >> 6;
        const int ks = f % KS; f /= KS;
        const int et = f % ET; f /= ET;
        const int t = f % 3;
        const int hd = f / 3, gi = hd / HG, hl = hd % HG;
        const int e = 16 * et + l16;
        for (int s = 0; s < 8; ++s) {
            const int c = 32 * ks + 8 * q + s;
            uint16_t v = 0;
            if (e < D && c < CG) v = w_qkv[((size_t)gi * 3 * CG + t * CG + hl * D + e) * CG + c].bits;
            wq[(size_t)i * 8 + s] = v;
        }
    }
    for (int i = gid; i < B::N_WC * 64; i += stride) {
        const int lane = i & 63, l16 = lane & 15, q = lane >> 4;
        int f = i >> 6;
        const int etp = f % ET; f /= ET;
        const int hlp = f % HG; f /= HG;
        const int et = f % ET; f /= ET;
        const int t = f % 3; f /= 3;
        const int hl = f % HG;
        const int gi = f / HG + 1;
        const int e = 16 * et + l16;
        for (int j = 0; j < 4; ++j) {
            const int ep = 16 * etp + 4 * q + j;
            uint16_t v = 0;
            if (e < D && ep < D) v = w_qkv[((size_t)gi * 3 * CG + t * CG + hl * D + e) * CG + hlp * D + ep].bits;
            wc[(size_t)i * 4 + j] = v;
        }
    }
    // Wproj^T: m-index l16 -> input channel (hd, e), k-slots -> output channel o
    for (int i = gid; i < B::N_WPT * 64; i += stride) {
        const int lane = i & 63, l16 = lane & 15, q = lane >> 4;
        int f = i >> 6;
        const int ks = f % KSC; f /= KSC;
        const int et = f % ET;
        const int hd = f / ET;
        const int e = 16 * et + l16;
        for (int s = 0; s < 8; ++s) {
            const int o = 32 * ks + 8 * q + s;
            uint16_t v = 0;
            if (e < D && o < C) v = w_proj[(size_t)o * C + hd * D + e].bits;
            wpt[(size_t)i * 8 + s] = v;
        }
    }
    // Wqkv^T: m-index l16 -> input channel of the group, tiled like the previous group's heads
    // (c = hlp*D + 16*etp + l16); k-slots -> output feature (t, hl, e = 16*et + 4q + j)
    for (int i = gid; i < B::N_WQT * 64; i += stride) {
        const int lane = i & 63, l16 = lane & 15, q = lane >> 4;
        int f = i >> 6;
        const int etp = f % ET; f /= ET;
        const int hlp = f % HG; f /= HG;
        const int et = f % ET; f /= ET;
        const int t = f % 3;
        const int hd = f / 3, gi = hd / HG, hl = hd % HG;
        const int cp = 16 * etp + l16;
        for (int j = 0; j < 4; ++j) {
            const int e = 16 * et + 4 * q + j;
            uint16_t v = 0;
            if (cp < D && e < D) v = w_qkv[((size_t)gi * 3 * CG + t * CG + hl * D + e) * CG + hlp * D + cp].bits;
            wqt[(size_t)i * 4 + j] = v;
        }
    }
    for (int i = gid; i < 4 * C; i += stride) bias[i] = i < 3 * C ? to_f32(b_qkv[i]) : 0.f;
}

template <class Cf> __device__ __forceinline__ constexpr int fq(int hd, int t, int et, int ks)
{
    return ((hd * 3 + t) * Cf::ET + et) * Cf::KS + ks;
}
template <class Cf> __device__ __forceinline__ constexpr int fc(int gi, int hl, int t, int et, int hlp, int etp)
{
    return (((((gi - 1) * Cf::HG + hl) * 3 + t) * Cf::ET + et) * Cf::HG + hlp) * Cf::ET + etp;
}
template <class Cf> __device__ __forceinline__ constexpr int fqt(int hd, int t, int et, int hlp, int etp)
{
    return ((((hd * 3 + t) * Cf::ET + et) * Cf::HG + hlp) * Cf::ET) + etp;
}

__device__ __forceinline__ uint4 cat(uint2 a, uint2 b) { return make_uint4(a.x, a.y, b.x, b.y); }

template <class Cf>
__global__ __launch_bounds__(256) void fused_bwd_kernel(Geom g, const bf16_t *__restrict__ x,
                                                        const bf16_t *__restrict__ dy,
                                                        const bf16_t *__restrict__ attn,
                                                        const uint8_t *__restrict__ pack,
                                                        const bf16_t *__restrict__ table,
                                                        bf16_t *__restrict__ dx, bf16_t *__restrict__ dqkv,
                                                        float *__restrict__ tbl_part)
{
    using B = BwdCfg<Cf>;
    constexpr int C = B::C, D = B::D, CG = B::CG, HG = B::HG, HEADS = B::HEADS, G = B::G;
    constexpr int ET = B::ET, KS = B::KS, KSC = B::KSC, LD = B::LD, NTBL = B::NTBL;
    constexpr int M = 8;
    static_assert(CG % 2 == 0 && D % 2 == 0 && C % 4 == 0, "dword-granular loads and stores");
    static_assert((size_t)NTBL * HEADS * 4 <= 2 * B::SZ_SQ, "table staging / flush aliases P and dS");

    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const uint4 *wq = reinterpret_cast<const uint4 *>(lds + B::OFF_WQ);
    const uint2 *wc = reinterpret_cast<const uint2 *>(lds + B::OFF_WC);
    const uint4 *wpt = reinterpret_cast<const uint4 *>(lds + B::OFF_WPT);
    const uint2 *wqt = reinterpret_cast<const uint2 *>(lds + B::OFF_WQT);
    const float *bqkv = reinterpret_cast<const float *>(lds + B::OFF_BIAS);
    uint2 *kb = reinterpret_cast<uint2 *>(lds + B::OFF_KB);
    uint2 *vb = reinterpret_cast<uint2 *>(lds + B::OFF_VB);
    uint16_t *ktr = reinterpret_cast<uint16_t *>(lds + B::OFF_KT);
    uint16_t *qtr = reinterpret_cast<uint16_t *>(lds + B::OFF_QT);
    uint16_t *dotr = reinterpret_cast<uint16_t *>(lds + B::OFF_DOT);
    uint16_t *pbuf = reinterpret_cast<uint16_t *>(lds + B::OFF_P);
    uint16_t *dsbuf = reinterpret_cast<uint16_t *>(lds + B::OFF_DS);

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, l16 = lane & 15, q = lane >> 4;

    for (int i = tid; i < (int)(B::PACK_BYTES / 16); i += 256)
        reinterpret_cast<uint4 *>(lds)[i] = reinterpret_cast<const uint4 *>(pack)[i];
    uint16_t *tstage = pbuf;
    for (int i = tid; i < NTBL * HEADS; i += 256) tstage[i] = table[i].bits;
    __syncthreads();

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
                    const int idx = (rn - (m >> 3) + M - 1) * (2 * M - 1) + (cn - (m & 7) + M - 1);
                    pr |= (uint32_t)tstage[idx * HEADS + hd] << (16 * h);
                }
                bias_frag[hd][kt * 2 + jp] = pr;
            }
    const int s = g.shift;
    bool rmask[4], cmask[4];
#pragma unroll
    for (int kt = 0; kt < 4; ++kt) rmask[kt] = (rn >= M - s) != ((2 * kt + (q >> 1)) >= M - s);
#pragma unroll
    for (int j = 0; j < 4; ++j) cmask[j] = (cn >= M - s) != ((4 * (q & 1) + j) >= M - s);
    // identity as an A operand: row l16, k-slots 4q+j
    uint2 ident;
    {
        const uint32_t one = 0x3f80u;
        const int d0 = l16 - 4 * q;
        ident.x = (d0 == 0 ? one : 0u) | (d0 == 1 ? one << 16 : 0u);
        ident.y = (d0 == 2 ? one : 0u) | (d0 == 3 ? one << 16 : 0u);
    }
    __syncthreads();

    f32x4 tblacc[HEADS][4];
#pragma unroll
    for (int hd = 0; hd < HEADS; ++hd)
#pragma unroll
        for (int kt = 0; kt < 4; ++kt) tblacc[hd][kt] = f32x4{0.f, 0.f, 0.f, 0.f};

    const float scale = 1.0f / sqrtf((float)D);
    const int per_img = g.nwi * g.nwj;
    int par = 0; // parity of the double-buffered exchange rows

    for (int win = blockIdx.x; win < g.nW; win += gridDim.x) {
        const int b = win / per_img;
        const int wr = win - b * per_img;
        const int wi = wr / g.nwj, wj = wr - wi * g.nwj;
        int si = wi * M + rn + s, sj = wj * M + cn + s;
        if (si >= g.H) si -= g.H;
        if (sj >= g.W) sj -= g.W;
        const long tok = ((long)b * g.H + si) * g.W + sj;
        const bool lastrow = s > 0 && wi == g.nwi - 1, lastcol = s > 0 && wj == g.nwj - 1;

        const uint32_t *xrow = reinterpret_cast<const uint32_t *>(x + tok * C);
        const uint32_t *dyrow = reinterpret_cast<const uint32_t *>(dy + tok * C);
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
        uint4 dyf[KSC];
#pragma unroll
        for (int ks = 0; ks < KSC; ++ks) {
            uint32_t dwv[4];
#pragma unroll
            for (int dw = 0; dw < 4; ++dw) {
                const int o = 32 * ks + 8 * q + 2 * dw;
                dwv[dw] = o < C ? dyrow[o >> 1] : 0u;
            }
            dyf[ks] = make_uint4(dwv[0], dwv[1], dwv[2], dwv[3]);
        }
        // saved group outputs of the previous groups, T-form packed (the cascade input, Eq. 8)
        uint2 Ob[HEADS][ET];
        if (G > 1 && g.cascade) {
#pragma unroll
            for (int hd = 0; hd < HEADS - HG; ++hd)
#pragma unroll
                for (int et = 0; et < ET; ++et) {
                    const int e0 = 16 * et + 4 * q;
                    const uint32_t *src = reinterpret_cast<const uint32_t *>(attn + tok * C + hd * D + e0);
                    Ob[hd][et].x = e0 < D ? src[0] : 0u;
                    Ob[hd][et].y = e0 + 2 < D ? src[1] : 0u;
                }
        }
        // dO of every head from the output projection (adjoint of Eq. 7), both forms
        f32x4 dOT[HEADS][ET], dON[HEADS][ET];
#pragma unroll
        for (int hd = 0; hd < HEADS; ++hd)
#pragma unroll
            for (int et = 0; et < ET; ++et) {
                dOT[hd][et] = f32x4{0.f, 0.f, 0.f, 0.f};
                dON[hd][et] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KSC; ++ks) {
                    const uint4 wf = wpt[((hd * ET + et) * KSC + ks) * 64 + lane];
                    dOT[hd][et] = mma32(wf, dyf[ks], dOT[hd][et]);
                    dON[hd][et] = mma32(dyf[ks], wf, dON[hd][et]);
                }
            }

        f32x4 dFT[HG][ET], dFN[HG][ET];
#pragma unroll
        for (int hdr = 0; hdr < HEADS; ++hdr) {
            const int hd = HEADS - 1 - hdr; // groups in reverse order
            const int gi = hd / HG, hl = hd % HG;
            const bool casc_in = gi > 0 && g.cascade;
            if (hl == HG - 1) {
#pragma unroll
                for (int hlp = 0; hlp < HG; ++hlp)
#pragma unroll
                    for (int etp = 0; etp < ET; ++etp) {
                        dFT[hlp][etp] = f32x4{0.f, 0.f, 0.f, 0.f};
                        dFN[hlp][etp] = f32x4{0.f, 0.f, 0.f, 0.f};
                    }
            }
            // ---- recompute q, k (both forms) and v (T-form) of this wave's tokens ----
            f32x4 qT[ET], qN[ET], kT[ET], kN[ET], vT[ET];
#pragma unroll
            for (int et = 0; et < ET; ++et) {
                const int ev = 16 * et + l16;
                const float bqn = ev < D ? bqkv[gi * 3 * CG + hl * D + ev] : 0.f;
                const float bkn = ev < D ? bqkv[gi * 3 * CG + CG + hl * D + ev] : 0.f;
                qN[et] = f32x4{bqn, bqn, bqn, bqn};
                kN[et] = f32x4{bkn, bkn, bkn, bkn};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int e = 16 * et + 4 * q + j;
                    qT[et][j] = e < D ? bqkv[gi * 3 * CG + hl * D + e] : 0.f;
                    kT[et][j] = e < D ? bqkv[gi * 3 * CG + CG + hl * D + e] : 0.f;
                    vT[et][j] = e < D ? bqkv[gi * 3 * CG + 2 * CG + hl * D + e] : 0.f;
                }
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const uint4 fq_ = wq[fq<Cf>(hd, 0, et, ks) * 64 + lane];
                    const uint4 fk_ = wq[fq<Cf>(hd, 1, et, ks) * 64 + lane];
                    const uint4 fv_ = wq[fq<Cf>(hd, 2, et, ks) * 64 + lane];
                    qT[et] = mma32(fq_, xf[gi][ks], qT[et]);
                    qN[et] = mma32(xf[gi][ks], fq_, qN[et]);
                    kT[et] = mma32(fk_, xf[gi][ks], kT[et]);
                    kN[et] = mma32(xf[gi][ks], fk_, kN[et]);
                    vT[et] = mma32(fv_, xf[gi][ks], vT[et]);
                }
                if (casc_in) {
#pragma unroll
                    for (int hlp = 0; hlp < HG; ++hlp)
#pragma unroll
                        for (int etp = 0; etp < ET; ++etp) {
                            const uint2 prev = Ob[(gi > 0 ? gi - 1 : 0) * HG + hlp][etp];
                            const uint2 cq = wc[fc<Cf>(gi > 0 ? gi : 1, hl, 0, et, hlp, etp) * 64 + lane];
                            const uint2 ck = wc[fc<Cf>(gi > 0 ? gi : 1, hl, 1, et, hlp, etp) * 64 + lane];
                            const uint2 cv = wc[fc<Cf>(gi > 0 ? gi : 1, hl, 2, et, hlp, etp) * 64 + lane];
                            qT[et] = mma16(cq, prev, qT[et]);
                            qN[et] = mma16(prev, cq, qN[et]);
                            kT[et] = mma16(ck, prev, kT[et]);
                            kN[et] = mma16(prev, ck, kN[et]);
                            vT[et] = mma16(cv, prev, vT[et]);
                        }
                }
            }
            // ---- exchange: K, V tiles; K^T, Q^T, dO^T rows ----
            uint2 Qb[ET], dOb[ET];
#pragma unroll
            for (int et = 0; et < ET; ++et) {
                Qb[et] = pack_bf16x4(qT[et]);
                dOb[et] = pack_bf16x4(dOT[hd][et]);
                kb[(wv * ET + et) * 64 + lane] = pack_bf16x4(kT[et]);
                vb[(wv * ET + et) * 64 + lane] = pack_bf16x4(vT[et]);
                const int row = (16 * et + l16) * LD + 16 * wv + 4 * q;
                *reinterpret_cast<uint2 *>(ktr + row) = pack_bf16x4(kN[et]);
                *reinterpret_cast<uint2 *>(qtr + par * 16 * ET * LD + row) = pack_bf16x4(qN[et]);
                *reinterpret_cast<uint2 *>(dotr + par * 16 * ET * LD + row) = pack_bf16x4(dON[hd][et]);
            }
            __syncthreads();

            // ---- query role: S^T, P^T, dP^T, dS^T for this wave's 16 queries, all 64 keys ----
            f32x4 st[4], dp[4];
#pragma unroll
            for (int kt = 0; kt < 4; ++kt) {
                st[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
                dp[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int et = 0; et < ET; ++et) {
                    st[kt] = mma16(kb[(kt * ET + et) * 64 + lane], Qb[et], st[kt]);
                    dp[kt] = mma16(vb[(kt * ET + et) * 64 + lane], dOb[et], dp[kt]);
                }
            }
#pragma unroll
            for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t pr = bias_frag[hd][kt * 2 + (j >> 1)];
                    st[kt][j] = fmaf(st[kt][j], scale, (j & 1) ? bf16_hi(pr) : bf16_lo(pr));
                }
            if (lastrow || lastcol) {
#pragma unroll
                for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if ((lastrow && rmask[kt]) || (lastcol && cmask[j])) st[kt][j] += -100.0f;
            }
            float mx = -INFINITY;
#pragma unroll
            for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                for (int j = 0; j < 4; ++j) mx = fmaxf(mx, st[kt][j]);
            mx = qgroup_max(mx);
            const float mxl = mx * kLog2e;
            float sum = 0.f;
#pragma unroll
            for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    st[kt][j] = __builtin_amdgcn_exp2f(fmaf(st[kt][j], kLog2e, -mxl));
                    sum += st[kt][j];
                }
            sum = qgroup_sum(sum);
            const float inv = 1.0f / sum;
            float delta = 0.f;
#pragma unroll
            for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    st[kt][j] *= inv;
                    delta = fmaf(st[kt][j], dp[kt][j], delta);
                }
            delta = qgroup_sum(delta);
            uint2 Pb[4], dSb[4];
#pragma unroll
            for (int kt = 0; kt < 4; ++kt) {
#pragma unroll
                for (int j = 0; j < 4; ++j) dp[kt][j] = st[kt][j] * (dp[kt][j] - delta);
                Pb[kt] = pack_bf16x4(st[kt]);
                dSb[kt] = pack_bf16x4(dp[kt]);
                tblacc[hd][kt] = mma16(ident, dSb[kt], tblacc[hd][kt]);
            }
            // transposed copies for the key role: [key][query]
#pragma unroll
            for (int kt = 0; kt < 4; ++kt) {
                const int base = (16 * kt + 4 * q) * LD + 16 * wv + l16;
                pbuf[base] = (uint16_t)(Pb[kt].x & 0xffffu);
                pbuf[base + LD] = (uint16_t)(Pb[kt].x >> 16);
                pbuf[base + 2 * LD] = (uint16_t)(Pb[kt].y & 0xffffu);
                pbuf[base + 3 * LD] = (uint16_t)(Pb[kt].y >> 16);
                dsbuf[base] = (uint16_t)(dSb[kt].x & 0xffffu);
                dsbuf[base + LD] = (uint16_t)(dSb[kt].x >> 16);
                dsbuf[base + 2 * LD] = (uint16_t)(dSb[kt].y & 0xffffu);
                dsbuf[base + 3 * LD] = (uint16_t)(dSb[kt].y >> 16);
            }
            // dQ^T = scale * K^T dS^T  (T-form: rows = features, column = own query)
            f32x4 dqT[ET];
#pragma unroll
            for (int et = 0; et < ET; ++et) {
                dqT[et] = f32x4{0.f, 0.f, 0.f, 0.f};
                const uint16_t *krow = ktr + (16 * et + l16) * LD + 4 * q;
#pragma unroll
                for (int kp = 0; kp < 2; ++kp) {
                    const uint2 a0 = *reinterpret_cast<const uint2 *>(krow + 32 * kp);
                    const uint2 a1 = *reinterpret_cast<const uint2 *>(krow + 32 * kp + 16);
                    dqT[et] = mma32(cat(a0, a1), cat(dSb[2 * kp], dSb[2 * kp + 1]), dqT[et]);
                }
                dqT[et] *= scale;
            }
            __syncthreads();

            // ---- key role: dV^T = dO^T P, dK^T = scale * Q^T dS for this wave's 16 keys ----
            f32x4 dkT[ET], dvT[ET];
            {
                const uint16_t *prow = pbuf + (16 * wv + l16) * LD + 4 * q;
                const uint16_t *srow = dsbuf + (16 * wv + l16) * LD + 4 * q;
                uint4 pf[2], sf[2];
#pragma unroll
                for (int kp = 0; kp < 2; ++kp) {
                    pf[kp] = cat(*reinterpret_cast<const uint2 *>(prow + 32 * kp),
                                 *reinterpret_cast<const uint2 *>(prow + 32 * kp + 16));
                    sf[kp] = cat(*reinterpret_cast<const uint2 *>(srow + 32 * kp),
                                 *reinterpret_cast<const uint2 *>(srow + 32 * kp + 16));
                }
#pragma unroll
                for (int et = 0; et < ET; ++et) {
                    dkT[et] = f32x4{0.f, 0.f, 0.f, 0.f};
                    dvT[et] = f32x4{0.f, 0.f, 0.f, 0.f};
                    const uint16_t *qrow = qtr + par * 16 * ET * LD + (16 * et + l16) * LD + 4 * q;
                    const uint16_t *orow = dotr + par * 16 * ET * LD + (16 * et + l16) * LD + 4 * q;
#pragma unroll
                    for (int kp = 0; kp < 2; ++kp) {
                        const uint4 qa = cat(*reinterpret_cast<const uint2 *>(qrow + 32 * kp),
                                             *reinterpret_cast<const uint2 *>(qrow + 32 * kp + 16));
                        const uint4 oa = cat(*reinterpret_cast<const uint2 *>(orow + 32 * kp),
                                             *reinterpret_cast<const uint2 *>(orow + 32 * kp + 16));
                        dkT[et] = mma32(qa, sf[kp], dkT[et]);
                        dvT[et] = mma32(oa, pf[kp], dvT[et]);
                    }
                    dkT[et] *= scale;
                }
            }
            // ---- gradients of q|k|v: to memory, and through Wqkv^T into dF of the group ----
#pragma unroll
            for (int et = 0; et < ET; ++et) {
                const uint2 gq = pack_bf16x4(dqT[et]), gk = pack_bf16x4(dkT[et]), gv = pack_bf16x4(dvT[et]);
                const int e0 = 16 * et + 4 * q;
                uint32_t *dst = reinterpret_cast<uint32_t *>(dqkv + tok * 3 * C + gi * 3 * CG + hl * D + e0);
                if (e0 < D) {
                    dst[0] = gq.x;
                    dst[CG / 2] = gk.x;
                    dst[CG] = gv.x;
                }
                if (e0 + 2 < D) {
                    dst[1] = gq.y;
                    dst[CG / 2 + 1] = gk.y;
                    dst[CG + 1] = gv.y;
                }
#pragma unroll
                for (int hlp = 0; hlp < HG; ++hlp)
#pragma unroll
                    for (int etp = 0; etp < ET; ++etp) {
                        const uint2 w0 = wqt[fqt<Cf>(hd, 0, et, hlp, etp) * 64 + lane];
                        const uint2 w1 = wqt[fqt<Cf>(hd, 1, et, hlp, etp) * 64 + lane];
                        const uint2 w2 = wqt[fqt<Cf>(hd, 2, et, hlp, etp) * 64 + lane];
                        dFT[hlp][etp] = mma16(w0, gq, dFT[hlp][etp]);
                        dFT[hlp][etp] = mma16(w1, gk, dFT[hlp][etp]);
                        dFT[hlp][etp] = mma16(w2, gv, dFT[hlp][etp]);
                        if (casc_in) {
                            dFN[hlp][etp] = mma16(gq, w0, dFN[hlp][etp]);
                            dFN[hlp][etp] = mma16(gk, w1, dFN[hlp][etp]);
                            dFN[hlp][etp] = mma16(gv, w2, dFN[hlp][etp]);
                        }
                    }
            }
            par ^= 1;

            // ---- end of a group: dx slice, and the cascade gradient into the previous group ----
            if (hl == 0) {
#pragma unroll
                for (int hlp = 0; hlp < HG; ++hlp)
#pragma unroll
                    for (int etp = 0; etp < ET; ++etp) {
                        const uint2 v = pack_bf16x4(dFT[hlp][etp]);
                        const int c0 = 16 * etp + 4 * q;
                        uint32_t *dst = reinterpret_cast<uint32_t *>(dx + tok * C + gi * CG + hlp * D + c0);
                        if (c0 < D) dst[0] = v.x;
                        if (c0 + 2 < D) dst[1] = v.y;
                        if (casc_in) {
                            dOT[(gi > 0 ? gi - 1 : 0) * HG + hlp][etp] += dFT[hlp][etp];
                            dON[(gi > 0 ? gi - 1 : 0) * HG + hlp][etp] += dFN[hlp][etp];
                        }
                    }
            }
        }
    }

    // ---- flush the bias-table gradient: (query, key) accumulators -> table entries -> partials ----
    __syncthreads();
    float *tbl = reinterpret_cast<float *>(lds + B::OFF_P);
    for (int i = tid; i < B::TBL_N; i += 256) tbl[i] = 0.f;
    __syncthreads();
#pragma unroll
    for (int hd = 0; hd < HEADS; ++hd)
#pragma unroll
        for (int kt = 0; kt < 4; ++kt)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int m = 16 * kt + 4 * q + j;
                const int idx = (rn - (m >> 3) + M - 1) * (2 * M - 1) + (cn - (m & 7) + M - 1);
                atomicAdd(&tbl[idx * HEADS + hd], tblacc[hd][kt][j]);
            }
    __syncthreads();
    for (int i = tid; i < B::TBL_N; i += 256) tbl_part[(size_t)blockIdx.x * B::TBL_N + i] = tbl[i];
}

// out[i] (+)= sum_w part[w][i]
__global__ __launch_bounds__(256) void reduce_partials_kernel(const float *__restrict__ part, int nparts,
                                                              int n, float *__restrict__ out, int accumulate)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    float acc = 0.f;
    for (int w = 0; w < nparts; ++w) acc += part[(size_t)w * n + i];
    out[i] = accumulate ? out[i] + acc : acc;
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

int bwd_grid(const Geom &g)
{
    int grid = device_cu_count();
    return grid > g.nW ? g.nW : grid;
}

template <class Cf>
hipError_t run_bwd(const Geom &g, const bf16_t *x, const bf16_t *dy, const bf16_t *attn,
                   const bf16_t *w_qkv, const bf16_t *b_qkv, const bf16_t *w_proj, const bf16_t *table,
                   bf16_t *dx, bf16_t *dqkv, float *dtable, int accumulate, void *ws, hipStream_t s)
{
    using B = BwdCfg<Cf>;
    static_assert(B::LDS_BYTES <= 160 * 1024, "LDS budget");
    uint8_t *pack = static_cast<uint8_t *>(ws);
    float *part = reinterpret_cast<float *>(pack + ((B::PACK_BYTES + 255) & ~size_t(255)));
    {
        KernelTimer kt(K_PACK_BWD, s);
        hipLaunchKernelGGL(pack_bwd_kernel<Cf>, dim3(64), dim3(256), 0, s, w_qkv, b_qkv, w_proj, pack);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    auto kern = fused_bwd_kernel<Cf>;
    static bool attr_done = false;
    if (!attr_done && B::LDS_BYTES > 64 * 1024) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)B::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    const int grid = bwd_grid(g);
    {
        KernelTimer kt(K_FUSED_BWD, s);
        hipLaunchKernelGGL(kern, dim3(grid), dim3(256), B::LDS_BYTES, s, g, x, dy, attn, pack, table, dx, dqkv, part);
    }
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    {
        KernelTimer kt(K_REDUCE, s);
        hipLaunchKernelGGL(reduce_partials_kernel, dim3((B::TBL_N + 255) / 256), dim3(256), 0, s, part, grid,
                           B::TBL_N, dtable, accumulate);
    }
    return hipGetLastError();
}

#define GSWA_FUSED_SHAPES(X) X(60, 6, 1) X(60, 6, 2) X(60, 6, 3) X(60, 6, 6)

} // namespace

bool fused_bwd_supported(const Geom &g)
{
    if (g.M != 8) return false;
#define X(C_, H_, G_) \
    if (g.C == C_ && g.heads == H_ && g.groups == G_) return true;
    GSWA_FUSED_SHAPES(X)
#undef X
    return false;
}

size_t fused_bwd_ws_bytes(const Geom &g)
{
    size_t pack = 0;
    int tbl = 0;
#define X(C_, H_, G_)                                                    \
    if (g.C == C_ && g.heads == H_ && g.groups == G_) {                  \
        pack = BwdCfg<FusedCfg<C_, H_, G_>>::PACK_BYTES;                 \
        tbl = BwdCfg<FusedCfg<C_, H_, G_>>::TBL_N;                       \
    }
    GSWA_FUSED_SHAPES(X)
#undef X
    if (!pack) return 0;
    return ((pack + 255) & ~size_t(255)) + (((size_t)bwd_grid(g) * tbl * 4 + 255) & ~size_t(255));
}

hipError_t launch_fused_bwd(const Geom &g, const bf16_t *x, const bf16_t *dy, const bf16_t *attn,
                            const bf16_t *w_qkv, const bf16_t *b_qkv, const bf16_t *w_proj,
                            const bf16_t *table, bf16_t *dx, bf16_t *dqkv, float *dtable, int accumulate,
                            void *ws, hipStream_t s)
{
#define X(C_, H_, G_)                                                   \
    if (g.C == C_ && g.heads == H_ && g.groups == G_)                   \
        return run_bwd<FusedCfg<C_, H_, G_>>(g, x, dy, attn, w_qkv, b_qkv, w_proj, table, dx, dqkv, dtable, \
                                             accumulate, ws, s);
    GSWA_FUSED_SHAPES(X)
#undef X
    return hipErrorInvalidValue;
}

} // namespace gswa
