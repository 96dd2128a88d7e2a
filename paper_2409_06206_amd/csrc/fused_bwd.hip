// Fused GSWA backward for 8x8 windows, bf16 storage.  The backward of a layer is a sequence of
// launches of fused_bwd_kernel, one per chunk of heads in reverse order; each recomputes q, k, v,
// the scores and the softmax of its heads from x and the saved group outputs, and produces the dx
// slices of its groups and per-workgroup partial sums of the parameter gradients (accumulated in
// registers over the windows a workgroup owns).  reduce_partials_kernel adds the partials in a
// fixed order.  wproj_grad_kernel is the projection's weight gradient for wide layers.
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

template <class Cf, int HB_, int HE_, bool WPROJ_ = (HE_ == Cf::HEADS)> struct BwdCfg {
    static constexpr int C = Cf::C, D = Cf::D, CG = Cf::CG, HG = Cf::HG, HEADS = Cf::HEADS, G = Cf::G;
    static constexpr int ET = Cf::ET, KS = Cf::KS;
    static constexpr int KSC = (C + 31) / 32; // K=32 steps over all C channels of dy
    static constexpr int NTBL = 15 * 15;
    static constexpr int TBL_N = NTBL * HEADS;
    // weight-gradient tiling: 16x16 tiles, one spare column (index CG resp. C) carries the bias sums
    static constexpr int CT = CG / 16 + 1;          // column tiles of d w_qkv of one head
    static constexpr int NT = 3 * ET * CT;          // tiles of one head's d w_qkv rows
    static constexpr int KT = (NT + 3) / 4;         // tiles per wave
    static constexpr int OTP = (C + 15) / 16, CTP = C / 16 + 1;
    static constexpr int NTP = OTP * CTP, KTP = (NTP + 3) / 4;
    // heads [HB, HE) of this launch: whole groups, or part of one group.  WPROJ: this launch also
    // produces d w_proj / d b_proj (narrow layers; wide ones use a kernel of its own).
    static constexpr int HB = HB_, HE = HE_, NH = HE - HB;
    static constexpr bool WPROJ = WPROJ_;
    static constexpr int GB = HB / HG, GE = (HE - 1) / HG; // lowest and highest group of the chunk
    static_assert(NH > 0 && (GB == GE || (HB % HG == 0 && HE % HG == 0)),
                  "a chunk is whole groups or lies inside one group");
    // packed parameters of these heads, copied from the buffer forward filled: [WQ | BIAS | WPT | WQT]
    static constexpr int N_WQ = NH * 3 * ET * KS, N_WPT = NH * ET * KSC, N_WQT = NH * 3 * ET * HG * ET;
    static constexpr size_t SRC_WQ = Cf::P_WQ + (size_t)HB * 3 * ET * KS * 1024;
    static constexpr size_t SRC_WPT = Cf::P_WPT + (size_t)HB * ET * KSC * 1024;
    static constexpr size_t SRC_WQT = Cf::P_WQT + (size_t)HB * 3 * ET * HG * ET * 512;
    static constexpr size_t OFF_WQ = 0;
    static constexpr size_t OFF_BIAS = OFF_WQ + (size_t)N_WQ * 1024;
    static constexpr size_t OFF_WPT = OFF_BIAS + (size_t)16 * C;
    // two heads of a wide three-head group fit LDS only without the Wproj^T fragments: those are
    // then read from the packed buffer in memory (12 reads per wave, window and head)
    static constexpr bool WPT_LDS = !(Cf::SPLIT && NH > 1 && Cf::HG == 3);
    static constexpr size_t OFF_WQT = OFF_WPT + (WPT_LDS ? (size_t)N_WPT * 1024 : 0);
    static constexpr size_t PACK_BYTES = OFF_WQT + (size_t)N_WQT * 512;
    // LDS beyond the packed weights
    static constexpr int LD = 68; // pitch (bf16) of rows read 4 at a time
    static constexpr int LW = 68; // pitch (bf16) of rows read 8 at a time (as two 8-byte halves:
                                  // 34 dwords keeps every 16-lane phase on distinct banks)
    static constexpr size_t SZ_FRAG = (size_t)4 * ET * 64 * 8;
    static constexpr size_t SZ_ROWS = (size_t)16 * ET * LD * 2;
    static constexpr size_t SZ_SQ = (size_t)64 * LW * 2; // P / dS [key][query]; also dY^T / A^T rows
    static constexpr size_t OFF_TBLF = PACK_BYTES;             // fp32 bias table [NH][225]
    static constexpr size_t OFF_KB = OFF_TBLF + (((size_t)NH * NTBL * 4 + 15) & ~size_t(15));
    static constexpr size_t OFF_VB = OFF_KB + SZ_FRAG;
    static constexpr size_t OFF_KT = OFF_VB + SZ_FRAG;         // K^T rows [e][key]
    static constexpr size_t OFF_QT = OFF_KT + SZ_ROWS;         // Q^T rows [e][query]
    static constexpr size_t OFF_DOT = OFF_QT + SZ_ROWS;        // dO^T rows [e][query]
    static constexpr size_t OFF_P = OFF_DOT + SZ_ROWS;
    static constexpr size_t OFF_DS = OFF_P + SZ_SQ;
    static constexpr size_t OFF_DQKV = OFF_DS + SZ_SQ;         // d(q|k|v)^T rows [(t,e)][token]
    static constexpr size_t SZ_DQKV = (size_t)3 * ET * 16 * LW * 2;
    static constexpr size_t OFF_F = OFF_DQKV + SZ_DQKV;        // F^T rows [c][token] of the current group
    static constexpr size_t SZ_F = (size_t)16 * CT * LW * 2;
    static constexpr size_t LDS_BYTES = OFF_F + SZ_F;
    // Per-workgroup partial sums of THIS launch only (the scratch is reused from launch to launch: the
    // head-group loop bounds it).  Rows of d w_qkv: for every group of the chunk and each of q, k, v
    // the RG rows the chunk's heads own, ((gi - GB) * 3 + t) * RG + (hl - HL0) * D + e; then the bias
    // sums in the same order, d w_proj | d b_proj where this launch produces them, and the bias-table
    // gradient head by head.
    static constexpr bool WHOLE = HB_ % HG == 0 && HE_ % HG == 0;   // whole groups (else: part of one group)
    static constexpr int NG = GE - GB + 1;
    static constexpr int RG = WHOLE ? CG : NH * D;                  // rows per (group, q|k|v)
    static constexpr int HL0 = WHOLE ? 0 : HB_ % HG;
    static constexpr int L_DWQ = 0;
    static constexpr int L_DBQ = L_DWQ + NG * 3 * RG * CG;
    static constexpr int L_DWP = L_DBQ + NG * 3 * RG;
    static constexpr int L_DBP = L_DWP + (WPROJ ? C * C : 0);
    static constexpr int L_TBL = L_DBP + (WPROJ ? C : 0);
    static constexpr int L_END = L_TBL + NH * NTBL;
    static constexpr int L_TOTAL = (L_END + 3) & ~3; // stride of the vectors: whole 16-byte pieces (the sum reads four entries per load)
    static_assert(!WPROJ || (OTP <= 2 * KSC && SZ_SQ >= (size_t)16 * OTP * LW * 2 &&
                             SZ_SQ >= (size_t)16 * CTP * LW * 2),
                  "dY^T / A^T rows alias the P / dS squares");
};

template <class Cf> __device__ __forceinline__ constexpr int fq(int hd, int t, int et, int ks)
{
    return ((hd * 3 + t) * Cf::ET + et) * Cf::KS + ks;
}
template <class Cf> __device__ __forceinline__ constexpr int fqt(int hd, int t, int et, int hlp, int etp)
{
    return ((((hd * 3 + t) * Cf::ET + et) * Cf::HG + hlp) * Cf::ET) + etp;
}

constexpr bool ranges_overlap(int a0, int a1, int b0, int b1) { return a0 < b1 && b0 < a1; }

template <class Cf, int HB, int HE, bool WPROJ>
__global__ __launch_bounds__(256, (BwdCfg<Cf, HB, HE, WPROJ>::LDS_BYTES <= 80 * 1024 ? 2 : 1))
void fused_bwd_kernel(Geom g, const bf16_t *__restrict__ x,
                                                        const bf16_t *__restrict__ dy,
                                                        const bf16_t *__restrict__ attn,
                                                        const uint8_t *__restrict__ pack,
                                                        const bf16_t *__restrict__ table,
                                                        bf16_t *dx, float *__restrict__ part)
{
    using B = BwdCfg<Cf, HB, HE, WPROJ>;
    constexpr int NH = B::NH, GB = B::GB, GE = B::GE;
    constexpr int C = B::C, D = B::D, CG = B::CG, HG = B::HG, HEADS = B::HEADS, G = B::G;
    constexpr int ET = B::ET, KS = B::KS, KSC = B::KSC, LD = B::LD, LW = B::LW, NTBL = B::NTBL;
    constexpr int CT = B::CT, NT = B::NT, KT = B::KT, OTP = B::OTP, CTP = B::CTP, NTP = B::NTP, KTP = B::KTP;
    constexpr int M = 8;
    static_assert(CG % 2 == 0 && D % 2 == 0 && C % 4 == 0, "dword-granular loads and stores");
    // The shift mask, exactly as the forward kernel of the same layer adds it: -100 for wide layers;
    // narrow layers carry it through bf16 matrix-core operands in base-2 units, where it is
    // -144 = bf16(-100 log2 e), i.e. -99.81 here.
    constexpr float kMask = Cf::SPLIT ? -100.0f : -144.0f / kLog2e;

    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const uint4 *wq = reinterpret_cast<const uint4 *>(lds + B::OFF_WQ);
    const uint4 *wpt = B::WPT_LDS ? reinterpret_cast<const uint4 *>(lds + B::OFF_WPT)
                                  : reinterpret_cast<const uint4 *>(pack + B::SRC_WPT);
    const uint2 *wqt = reinterpret_cast<const uint2 *>(lds + B::OFF_WQT);
    const float *bqkv = reinterpret_cast<const float *>(lds + B::OFF_BIAS);
    float *tblf = reinterpret_cast<float *>(lds + B::OFF_TBLF);
    uint2 *kb = reinterpret_cast<uint2 *>(lds + B::OFF_KB);
    uint2 *vb = reinterpret_cast<uint2 *>(lds + B::OFF_VB);
    uint16_t *ktr = reinterpret_cast<uint16_t *>(lds + B::OFF_KT);
    uint16_t *qtr = reinterpret_cast<uint16_t *>(lds + B::OFF_QT);
    uint16_t *dotr = reinterpret_cast<uint16_t *>(lds + B::OFF_DOT);
    uint16_t *pbuf = reinterpret_cast<uint16_t *>(lds + B::OFF_P);
    uint16_t *dsbuf = reinterpret_cast<uint16_t *>(lds + B::OFF_DS);
    uint16_t *dybuf = pbuf, *abuf = dsbuf; // dY^T and A^T rows live where P / dS go later in the window
    uint16_t *gbuf = reinterpret_cast<uint16_t *>(lds + B::OFF_DQKV);
    uint16_t *fbuf = reinterpret_cast<uint16_t *>(lds + B::OFF_F);

    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, q = lane >> 4;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6); // wave index, held in a scalar register

    // Rows of x, of the saved group outputs and of dy of this lane's token as MFMA operands (k-slots =
    // channels).  The rows of a window are fetched while the previous window is finished (the first
    // window's during the set-up), so that their latency is off the critical path.
    const int per_img = g.nwi * g.nwj;
    const int rn = 2 * wv + (l16 >> 3), cn = l16 & 7;
    const int s = g.shift;
    // window -> (image, window row, window column): quotients through a float reciprocal with a fix-up
    // (exact for operands below 2^24), a fraction of the cost of the integer divisions
    const float r_img = 1.0f / (float)per_img, r_nwj = 1.0f / (float)g.nwj;
    auto fdiv = [](int a, int d, float rd) {
        int qt = (int)((float)a * rd);
        qt += (qt + 1) * d <= a ? 1 : 0;
        qt -= qt * d > a ? 1 : 0;
        return qt;
    };
    auto token_of = [&](int win) {
        const int b = fdiv(win, per_img, r_img);
        const int wr = win - b * per_img;
        const int wi = fdiv(wr, g.nwj, r_nwj), wj = wr - wi * g.nwj;
        int si = wi * M + rn + s, sj = wj * M + cn + s;
        if (si >= g.H) si -= g.H;
        if (sj >= g.W) sj -= g.W;
        return ((long)b * g.H + si) * g.W + sj;
    };
    uint4 xf[G][KS], af[G][KS], dyf[KSC];
    uint2 cgrad[NH][ET]; // dF of the next group (Eq. 8) for the heads whose next group an earlier launch finished
    auto load_rows = [&](int win) {
        const long tok = token_of(win);
#pragma unroll
        for (int hx = 0; hx < NH; ++hx) {
            const int hd = HB + hx, gi = hd / HG, hl = hd % HG;
            const bool in_regs = HB <= (gi + 1) * HG && HE >= (gi + 2) * HG;
#pragma unroll
            for (int et = 0; et < ET; ++et) {
                cgrad[hx][et] = make_uint2(0u, 0u);
                if (gi < G - 1 && !in_regs && g.cascade) {
                    const int e0 = 16 * et + 4 * q;
                    const uint32_t *src = reinterpret_cast<const uint32_t *>(dx + tok * C + (gi + 1) * CG + hl * D + e0);
                    if (e0 < D) cgrad[hx][et].x = src[0];
                    if (e0 + 2 < D) cgrad[hx][et].y = src[1];
                }
            }
        }
        const uint32_t *xrow = reinterpret_cast<const uint32_t *>(x + tok * C);
        const uint32_t *arow = reinterpret_cast<const uint32_t *>(attn + tok * C);
        const uint32_t *dyrow = reinterpret_cast<const uint32_t *>(dy + tok * C);
#pragma unroll
        for (int gi = 0; gi < G; ++gi)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                uint32_t xv[4], av[4];
                const bool need_x = gi >= GB && gi <= GE;
                const bool need_a = WPROJ || (gi >= GB - 1 && gi < GE);
#pragma unroll
                for (int dw = 0; dw < 4; ++dw) {
                    const int c = 32 * ks + 8 * q + 2 * dw;
                    xv[dw] = (need_x && c < CG) ? xrow[(gi * CG + c) >> 1] : 0u;
                    av[dw] = (need_a && c < CG) ? arow[(gi * CG + c) >> 1] : 0u;
                }
                xf[gi][ks] = make_uint4(xv[0], xv[1], xv[2], xv[3]);
                af[gi][ks] = make_uint4(av[0], av[1], av[2], av[3]);
            }
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
    };
    // (with many groups the row registers are too many to hold two windows' worth at once)
    constexpr bool PIPE = (2 * G * KS + KSC) * 4 <= 32;
    if (PIPE && (int)blockIdx.x < g.nW) load_rows(blockIdx.x);

    // set-up copies, unrolled so that a thread's loads are all in flight before its first store
    {
        constexpr int N_Q = (int)((B::OFF_BIAS - B::OFF_WQ) / 16), N_PT = (int)((B::OFF_WQT - B::OFF_WPT) / 16);
        constexpr int N_QT = (int)((B::PACK_BYTES - B::OFF_WQT) / 16), N_T = NTBL * NH;
        constexpr int I_Q = (N_Q + 255) / 256, I_PT = (N_PT + 255) / 256, I_QT = (N_QT + 255) / 256, I_T = (N_T + 255) / 256;
        uint4 vq[I_Q], vpt[I_PT > 0 ? I_PT : 1], vqt[I_QT], vb = make_uint4(0u, 0u, 0u, 0u);
        uint16_t vt[I_T];
#pragma unroll
        for (int k = 0; k < I_Q; ++k) { const int i = 256 * k + tid; vq[k] = reinterpret_cast<const uint4 *>(pack + B::SRC_WQ)[i < N_Q ? i : 0]; }
#pragma unroll
        for (int k = 0; k < I_PT; ++k) { const int i = 256 * k + tid; vpt[k] = reinterpret_cast<const uint4 *>(pack + B::SRC_WPT)[i < N_PT ? i : 0]; }
#pragma unroll
        for (int k = 0; k < I_QT; ++k) { const int i = 256 * k + tid; vqt[k] = reinterpret_cast<const uint4 *>(pack + B::SRC_WQT)[i < N_QT ? i : 0]; }
        if (tid < C) vb = reinterpret_cast<const uint4 *>(pack + Cf::P_BIAS)[tid];
#pragma unroll
        for (int k = 0; k < I_T; ++k) { const int i = 256 * k + tid; const int ii = i < N_T ? i : 0; vt[k] = table[(ii % NTBL) * HEADS + HB + ii / NTBL].bits; }
#pragma unroll
        for (int k = 0; k < I_Q; ++k) { const int i = 256 * k + tid; if (i < N_Q) reinterpret_cast<uint4 *>(lds + B::OFF_WQ)[i] = vq[k]; }
#pragma unroll
        for (int k = 0; k < I_PT; ++k) { const int i = 256 * k + tid; if (i < N_PT) reinterpret_cast<uint4 *>(lds + B::OFF_WPT)[i] = vpt[k]; }
#pragma unroll
        for (int k = 0; k < I_QT; ++k) { const int i = 256 * k + tid; if (i < N_QT) reinterpret_cast<uint4 *>(lds + B::OFF_WQT)[i] = vqt[k]; }
        if (tid < C) reinterpret_cast<uint4 *>(lds + B::OFF_BIAS)[tid] = vb;
#pragma unroll
        for (int k = 0; k < I_T; ++k) { const int i = 256 * k + tid; if (i < N_T) tblf[i] = __uint_as_float((uint32_t)vt[k] << 16); }
    }

    // this lane's token inside the window, and the bias-table row of its (query, key 4q) pair:
    // the entry of key 16kt+4q+j is idx0 - 30kt - j
    const int idx0 = (rn - (q >> 1) + M - 1) * (2 * M - 1) + (cn - 4 * (q & 1) + M - 1);
    bool rmask[4], cmask[4];
#pragma unroll
    for (int kt = 0; kt < 4; ++kt) rmask[kt] = (rn >= M - s) != ((2 * kt + (q >> 1)) >= M - s);
#pragma unroll
    for (int j = 0; j < 4; ++j) cmask[j] = (cn >= M - s) != ((4 * (q & 1) + j) >= M - s);
    uint2 ident; // identity as a K=16 A operand: row l16, k-slots 4q+j
    {
        const uint32_t one = 0x3f80u;
        const int d0 = l16 - 4 * q;
        ident.x = (d0 == 0 ? one : 0u) | (d0 == 1 ? one << 16 : 0u);
        ident.y = (d0 == 2 ? one : 0u) | (d0 == 3 ? one << 16 : 0u);
    }
    __syncthreads();

    f32x4 tblacc[NH][4], dwacc[NH][KT], wpacc[KTP];
#pragma unroll
    for (int hd = 0; hd < NH; ++hd) {
#pragma unroll
        for (int kt = 0; kt < 4; ++kt) tblacc[hd][kt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int k = 0; k < KT; ++k) dwacc[hd][k] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int k = 0; k < KTP; ++k) wpacc[k] = f32x4{0.f, 0.f, 0.f, 0.f};

    const uint2 ones2 = make_uint2(0x3f803f80u, 0x3f803f80u);

    for (int win = blockIdx.x; win < g.nW; win += gridDim.x) {
        // (the lane index as this window's address arithmetic sees it: opaque, so that the many per-lane LDS and
        // memory addresses below are computed where they are used instead of being kept, and spilled, across windows)
        int lane_w = threadIdx.x & 63;
        asm volatile("" : "+v"(lane_w));
        const int lane = lane_w, l16 = lane & 15, q = lane >> 4;
        if (!PIPE) load_rows(win);
        // Eq. 8: the input of a group with a cascade term is F = x slice + previous group's output,
        // rounded to bf16 exactly as the forward kernels round it (it is the operand of their QKV
        // product), so that q, k, v and the probabilities are recomputed from the same values
        if (g.cascade) {
#pragma unroll
            for (int gi = (GB > 1 ? GB : 1); gi <= GE; ++gi)
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    uint4 &f = xf[gi][ks];
                    const uint4 a = af[gi - 1][ks];
                    f.x = pack_bf16x2(bf16_lo(f.x) + bf16_lo(a.x), bf16_hi(f.x) + bf16_hi(a.x));
                    f.y = pack_bf16x2(bf16_lo(f.y) + bf16_lo(a.y), bf16_hi(f.y) + bf16_hi(a.y));
                    f.z = pack_bf16x2(bf16_lo(f.z) + bf16_lo(a.z), bf16_hi(f.z) + bf16_hi(a.z));
                    f.w = pack_bf16x2(bf16_lo(f.w) + bf16_lo(a.w), bf16_hi(f.w) + bf16_hi(a.w));
                }
        }
        const long tok = token_of(win);
        const int wr = win - fdiv(win, per_img, r_img) * per_img, wi = fdiv(wr, g.nwj, r_nwj);
        const bool lastrow = s > 0 && wi == g.nwi - 1, lastcol = s > 0 && wr - wi * g.nwj == g.nwj - 1;

        // ---- d w_proj, d b_proj: dY^T and A^T rows [channel][token] through LDS, K = 64 tokens ----
        if (WPROJ) {
#pragma unroll
        for (int ot = 0; ot < OTP; ++ot) {
            f32x4 tN = mma32(dyf[ot >> 1], select_slot(16 * ot + l16, 32 * (ot >> 1) + 8 * q),
                             f32x4{0.f, 0.f, 0.f, 0.f});
            *reinterpret_cast<uint2 *>(dybuf + (16 * ot + l16) * LW + 16 * wv + 4 * q) = pack_bf16x4(tN);
        }
#pragma unroll
        for (int ct = 0; ct < CTP; ++ct) {
            f32x4 tN = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int gi = 0; gi < G; ++gi)
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
                    if (ranges_overlap(gi * CG + 32 * ks, gi * CG + (32 * ks + 32 < CG ? 32 * ks + 32 : CG),
                                       16 * ct, 16 * ct + 16))
                        tN = mma32(af[gi][ks], select_slot(16 * ct + l16, gi * CG + 32 * ks + 8 * q), tN);
            uint2 pk = pack_bf16x4(tN);
            if (16 * ct + l16 == C) pk = ones2;
            *reinterpret_cast<uint2 *>(abuf + (16 * ct + l16) * LW + 16 * wv + 4 * q) = pk;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < KTP; ++k) {
            const int ti = 4 * k + wv;
            if (ti < NTP) {
                const int ot = ti / CTP, ct = ti - ot * CTP;
                const uint16_t *ar = dybuf + (16 * ot + l16) * LW + 8 * q;
                const uint16_t *br = abuf + (16 * ct + l16) * LW + 8 * q;
#pragma unroll
                for (int kp = 0; kp < 2; ++kp)
                    wpacc[k] = mma32(cat(*reinterpret_cast<const uint2 *>(ar + 32 * kp),
                                         *reinterpret_cast<const uint2 *>(ar + 32 * kp + 4)),
                                     cat(*reinterpret_cast<const uint2 *>(br + 32 * kp),
                                         *reinterpret_cast<const uint2 *>(br + 32 * kp + 4)), wpacc[k]);
            }
        }
        }

        f32x4 dFT[HG][ET], cascT[HG][ET];
#pragma unroll
        for (int hdr = 0; hdr < NH; ++hdr) {
            const int hd = HE - 1 - hdr; // groups in reverse order
            const int hx = hd - HB;      // index into this launch's fragments and accumulators
            const int gi = hd / HG, hl = hd % HG;
            const bool casc_out = gi < G - 1 && g.cascade; // this group's output feeds the next group
            // the heads of group gi this launch processes, top first: [g_lo, g_hi]
            const int g_hi = (HE < (gi + 1) * HG ? HE : (gi + 1) * HG) - 1;
            const int g_lo = HB > gi * HG ? HB : gi * HG;
            const bool starts_group = g_hi == (gi + 1) * HG - 1; // no earlier launch touched this group
            const bool next_in_regs = HB <= (gi + 1) * HG && HE >= (gi + 2) * HG; // group gi+1 done in this launch
            if (hd == g_hi) {
#pragma unroll
                for (int hlp = 0; hlp < HG; ++hlp)
#pragma unroll
                    for (int etp = 0; etp < ET; ++etp) dFT[hlp][etp] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
            // ---- dO^T of this head: adjoint of Eq. 7, plus the gradient arriving through Eq. 8 ----
            f32x4 dOT[ET];
#pragma unroll
            for (int et = 0; et < ET; ++et) {
                dOT[et] = f32x4{0.f, 0.f, 0.f, 0.f};
                if (casc_out) {
                    if (next_in_regs) {
                        dOT[et] = cascT[hl][et];
                    } else { // the next group was finished by earlier launches: its dF is the dx slice
                        const uint32_t lo = cgrad[hx][et].x, hi = cgrad[hx][et].y;
                        dOT[et] = f32x4{bf16_lo(lo), bf16_hi(lo), bf16_lo(hi), bf16_hi(hi)};
                    }
                }
#pragma unroll
                for (int ks = 0; ks < KSC; ++ks)
                    dOT[et] = mma32(wpt[((hx * ET + et) * KSC + ks) * 64 + lane], dyf[ks], dOT[et]);
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
                    const uint4 fq_ = wq[fq<Cf>(hx, 0, et, ks) * 64 + lane];
                    const uint4 fk_ = wq[fq<Cf>(hx, 1, et, ks) * 64 + lane];
                    const uint4 fv_ = wq[fq<Cf>(hx, 2, et, ks) * 64 + lane];
                    qT[et] = mma32(fq_, xf[gi][ks], qT[et]);
                    qN[et] = mma32(xf[gi][ks], fq_, qN[et]);
                    kT[et] = mma32(fk_, xf[gi][ks], kT[et]);
                    kN[et] = mma32(xf[gi][ks], fk_, kN[et]);
                    vT[et] = mma32(fv_, xf[gi][ks], vT[et]);
                }
            }
            // ---- exchange: K, V tiles; K^T, Q^T, dO^T rows ----
            uint2 Qb[ET], dOb[ET];
#pragma unroll
            for (int et = 0; et < ET; ++et) {
                Qb[et] = pack_bf16x4(qT[et]);
                dOb[et] = pack_bf16x4(dOT[et]);
                kb[(wv * ET + et) * 64 + lane] = pack_bf16x4(kT[et]);
                vb[(wv * ET + et) * 64 + lane] = pack_bf16x4(vT[et]);
                const int row = (16 * et + l16) * LD + 16 * wv + 4 * q;
                *reinterpret_cast<uint2 *>(ktr + row) = pack_bf16x4(kN[et]);
                *reinterpret_cast<uint2 *>(qtr + row) = pack_bf16x4(qN[et]);
                store_tile_transposed(dotr + (16 * et + 4 * q) * LD + 16 * wv + (l16 & ~1), LD, dOb[et], lane);
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
                for (int j = 0; j < 4; ++j)
                    st[kt][j] += tblf[hx * NTBL + idx0 - 30 * kt - j];
            if (lastrow || lastcol) {
#pragma unroll
                for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if ((lastrow && rmask[kt]) || (lastcol && cmask[j])) st[kt][j] += kMask;
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
                tblacc[hx][kt] = mma16(ident, dSb[kt], tblacc[hx][kt]);
            }
            // transposed copies for the key role: [key][query]
#pragma unroll
            for (int kt = 0; kt < 4; ++kt) {
                const int base = (16 * kt + 4 * q) * LD + 16 * wv + (l16 & ~1);
                store_tile_transposed(pbuf + base, LD, Pb[kt], lane);
                store_tile_transposed(dsbuf + base, LD, dSb[kt], lane);
            }
            // dQ = scale * dS K in both forms: T-form feeds dF, N-form rows feed d w_qkv
            f32x4 dqT[ET];
#pragma unroll
            for (int et = 0; et < ET; ++et) {
                dqT[et] = f32x4{0.f, 0.f, 0.f, 0.f};
                f32x4 dqN = f32x4{0.f, 0.f, 0.f, 0.f};
                const uint16_t *krow = ktr + (16 * et + l16) * LD + 4 * q;
#pragma unroll
                for (int kp = 0; kp < 2; ++kp) {
                    const uint4 kf = cat(*reinterpret_cast<const uint2 *>(krow + 32 * kp),
                                         *reinterpret_cast<const uint2 *>(krow + 32 * kp + 16));
                    const uint4 sf = cat(dSb[2 * kp], dSb[2 * kp + 1]);
                    dqT[et] = mma32(kf, sf, dqT[et]);
                    dqN = mma32(sf, kf, dqN);
                }
                *reinterpret_cast<uint2 *>(gbuf + ((0 * ET + et) * 16 + l16) * LW + 16 * wv + 4 * q) = pack_bf16x4(dqN);
            }
            __syncthreads();

            // ---- key role: dV = P^T dO, dK = scale * dS^T Q for this wave's 16 keys, both forms ----
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
                    f32x4 dkN = f32x4{0.f, 0.f, 0.f, 0.f}, dvN = f32x4{0.f, 0.f, 0.f, 0.f};
                    const uint16_t *qrow = qtr + (16 * et + l16) * LD + 4 * q;
                    const uint16_t *orow = dotr + (16 * et + l16) * LD + 4 * q;
#pragma unroll
                    for (int kp = 0; kp < 2; ++kp) {
                        const uint4 qa = cat(*reinterpret_cast<const uint2 *>(qrow + 32 * kp),
                                             *reinterpret_cast<const uint2 *>(qrow + 32 * kp + 16));
                        const uint4 oa = cat(*reinterpret_cast<const uint2 *>(orow + 32 * kp),
                                             *reinterpret_cast<const uint2 *>(orow + 32 * kp + 16));
                        dkT[et] = mma32(qa, sf[kp], dkT[et]);
                        dkN = mma32(sf[kp], qa, dkN);
                        dvT[et] = mma32(oa, pf[kp], dvT[et]);
                        dvN = mma32(pf[kp], oa, dvN);
                    }
                    *reinterpret_cast<uint2 *>(gbuf + ((1 * ET + et) * 16 + l16) * LW + 16 * wv + 4 * q) = pack_bf16x4(dkN);
                    *reinterpret_cast<uint2 *>(gbuf + ((2 * ET + et) * 16 + l16) * LW + 16 * wv + 4 * q) = pack_bf16x4(dvN);
                }
            }
            // ---- first head of a group in this launch: F^T rows [channel][token] of the group input (Eq. 8) ----
            if (hd == g_hi) {
#pragma unroll
                for (int ct = 0; ct < CT; ++ct) {
                    f32x4 tN = f32x4{0.f, 0.f, 0.f, 0.f};
                    if (2 * (ct >> 1) < 2 * KS && (ct >> 1) < KS) {
                        const uint4 sel = select_slot(16 * ct + l16, 32 * (ct >> 1) + 8 * q);
                        tN = mma32(xf[gi][(ct >> 1) < KS ? (ct >> 1) : 0], sel, tN);
                    }
                    uint2 pk = pack_bf16x4(tN);
                    if (16 * ct + l16 == CG) pk = ones2;
                    *reinterpret_cast<uint2 *>(fbuf + (16 * ct + l16) * LW + 16 * wv + 4 * q) = pk;
                }
            }
            // ---- d(q|k|v) through Wqkv^T into dF of the group ----
#pragma unroll
            for (int et = 0; et < ET; ++et) {
                const uint2 gq = pack_bf16x4(dqT[et]), gk = pack_bf16x4(dkT[et]), gv = pack_bf16x4(dvT[et]);
#pragma unroll
                for (int hlp = 0; hlp < HG; ++hlp)
#pragma unroll
                    for (int etp = 0; etp < ET; ++etp) {
                        dFT[hlp][etp] = mma16(wqt[fqt<Cf>(hx, 0, et, hlp, etp) * 64 + lane], gq, dFT[hlp][etp]);
                        dFT[hlp][etp] = mma16(wqt[fqt<Cf>(hx, 1, et, hlp, etp) * 64 + lane], gk, dFT[hlp][etp]);
                        dFT[hlp][etp] = mma16(wqt[fqt<Cf>(hx, 2, et, hlp, etp) * 64 + lane], gv, dFT[hlp][etp]);
                    }
            }
            __syncthreads();

            // ---- d w_qkv (and d b_qkv in the spare column) of this head: K = 64 tokens ----
#pragma unroll
            for (int k = 0; k < KT; ++k) {
                const int ti = 4 * k + wv;
                if (ti < NT) {
                    const int r = ti / CT, ct = ti - r * CT;
                    const uint16_t *ar = gbuf + (16 * r + l16) * LW + 8 * q;
                    const uint16_t *br = fbuf + (16 * ct + l16) * LW + 8 * q;
#pragma unroll
                    for (int kp = 0; kp < 2; ++kp)
                        dwacc[hx][k] = mma32(cat(*reinterpret_cast<const uint2 *>(ar + 32 * kp),
                                                 *reinterpret_cast<const uint2 *>(ar + 32 * kp + 4)),
                                             cat(*reinterpret_cast<const uint2 *>(br + 32 * kp),
                                                 *reinterpret_cast<const uint2 *>(br + 32 * kp + 4)), dwacc[hx][k]);
                }
            }

            // ---- end of a group: dx slice; keep dF as the cascade gradient of the previous group ----
            if (hd == g_lo) {
#pragma unroll
                for (int hlp = 0; hlp < HG; ++hlp)
#pragma unroll
                    for (int etp = 0; etp < ET; ++etp) {
                        const int c0 = 16 * etp + 4 * q;
                        uint32_t *dst = reinterpret_cast<uint32_t *>(dx + tok * C + gi * CG + hlp * D + c0);
                        if (!starts_group) { // earlier launches left the other heads' share in the slice
                            const uint32_t lo = c0 < D ? dst[0] : 0u, hi = c0 + 2 < D ? dst[1] : 0u;
                            dFT[hlp][etp] += f32x4{bf16_lo(lo), bf16_hi(lo), bf16_lo(hi), bf16_hi(hi)};
                        }
                        const uint2 v = pack_bf16x4(dFT[hlp][etp]);
                        if (c0 < D) dst[0] = v.x;
                        if (c0 + 2 < D) dst[1] = v.y;
                        cascT[hlp][etp] = dFT[hlp][etp];
                    }
            }
        }
        if (PIPE && win + (int)gridDim.x < g.nW) load_rows(win + gridDim.x);
    }

    // ---- flush: this workgroup's partial sums, in parameter order.  The packed query weights
    // carry the 1/sqrt(d) of the scores, so their gradients get it back here. ----
    const float scale = 1.0f / sqrtf((float)D);
    float *mine = part + (size_t)blockIdx.x * B::L_TOTAL;
    if (WPROJ) {
#pragma unroll
    for (int k = 0; k < KTP; ++k) {
        const int ti = 4 * k + wv;
        if (ti < NTP) {
            const int ot = ti / CTP, ct = ti - ot * CTP;
            const int c = 16 * ct + l16;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int o = 16 * ot + 4 * q + j;
                if (o < C) {
                    if (c < C) mine[B::L_DWP + o * C + c] = wpacc[k][j];
                    else if (c == C) mine[B::L_DBP + o] = wpacc[k][j];
                }
            }
        }
    }
    }
#pragma unroll
    for (int hx = 0; hx < NH; ++hx) {
        const int hd = HB + hx;
        const int gi = hd / HG, hl = hd % HG;
#pragma unroll
        for (int k = 0; k < KT; ++k) {
            const int ti = 4 * k + wv;
            if (ti < NT) {
                const int r = ti / CT, ct = ti - r * CT;
                const int t = r / ET, et = r - t * ET;
                const int c = 16 * ct + l16;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int e = 16 * et + 4 * q + j;
                    if (e < D) {
                        const int row = ((gi - GB) * 3 + t) * B::RG + (hl - B::HL0) * D + e;
                        const float v = t == 0 ? dwacc[hx][k][j] * scale : dwacc[hx][k][j];
                        if (c < CG) mine[B::L_DWQ + row * CG + c] = v;
                        else if (c == CG) mine[B::L_DBQ + row] = v;
                    }
                }
            }
        }
    }
    // bias-table gradient: (query, key) accumulators -> table entries, summed in a fixed order
    float *mat = reinterpret_cast<float *>(lds + B::OFF_P); // [64 queries][64 keys] of one head, rows 65 floats
                                                            // apart (the 16 query rows a store touches then
                                                            // fall on different banks)
    constexpr int MP = 65;
    static_assert((size_t)64 * MP * 4 <= 2 * B::SZ_SQ, "table flush aliases P and dS");
#pragma unroll
    for (int hx = 0; hx < NH; ++hx) {
        __syncthreads();
#pragma unroll
        for (int kt = 0; kt < 4; ++kt)
#pragma unroll
            for (int j = 0; j < 4; ++j) mat[(16 * wv + l16) * MP + 16 * kt + 4 * q + j] = tblacc[hx][kt][j];
        __syncthreads();
        {
            // Four threads share the offsets (dr0, dc0), (dr0 - M, dc0), (dr0, dc0 - M), (dr0 - M, dc0 - M)
            // with 0 <= dr0, dc0 < M: for every query (rn, cn) exactly one of the four has its key
            // inside the window, key = ((rn - dr0) mod M, (cn - dc0) mod M), so the four entries take
            // M*M terms together and each thread sums those of two query rows: 16 reads, all in
            // flight together, the same for every thread.
            const int grp4 = tid >> 2, part = tid & 3;
            const int dr0 = grp4 >> 3, dc0 = grp4 & 7;
            float a00 = 0.f, a01 = 0.f, a10 = 0.f, a11 = 0.f; // [row wrapped][column wrapped]
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int rn = 2 * part + i;
                const bool wr = rn < dr0;
                const int rm = (rn - dr0) & (M - 1);
                float s0 = 0.f, s1 = 0.f;
#pragma unroll
                for (int cn = 0; cn < M; ++cn) {
                    const bool wc = cn < dc0;
                    const float v = mat[(rn * M + cn) * MP + rm * M + ((cn - dc0) & (M - 1))];
                    s0 += wc ? 0.f : v;
                    s1 += wc ? v : 0.f;
                }
                a00 += wr ? 0.f : s0;
                a01 += wr ? 0.f : s1;
                a10 += wr ? s0 : 0.f;
                a11 += wr ? s1 : 0.f;
            }
            a00 += __shfl_xor(a00, 1); a01 += __shfl_xor(a01, 1); a10 += __shfl_xor(a10, 1); a11 += __shfl_xor(a11, 1);
            a00 += __shfl_xor(a00, 2); a01 += __shfl_xor(a01, 2); a10 += __shfl_xor(a10, 2); a11 += __shfl_xor(a11, 2);
            // thread `part` of the four writes entry `part`
            const int e00 = (dr0 + M - 1) * (2 * M - 1) + dc0 + M - 1;
            const float val = part == 0 ? a00 : part == 1 ? a01 : part == 2 ? a10 : a11;
            const int e = e00 - ((part & 1) ? M : 0) - ((part & 2) ? M * (2 * M - 1) : 0);
            const bool ok = !((part & 1) && dc0 == 0) && !((part & 2) && dr0 == 0);
            if (ok) mine[B::L_TBL + hx * NTBL + e] = val;
        }
    }
}

// (segment table: ReduceOut, fused.h)
// A block sums 32 * V consecutive entries over all partial vectors: thread (column group, slice) adds the
// partials slice, slice + 32, ... (V entries each, one load of 4 V bytes: with V = 2 a wave half reads 256
// contiguous bytes of a partial vector), the 32 slices meet in LDS in a fixed order.
template <int V>
__device__ __forceinline__ void reduce_partials_block(const float *__restrict__ part, int nparts, int n,
                                                      const ReduceOut &out, int accumulate, int block, float *red)
{
    constexpr int SL = 32; // slices of the partials, one per wave half: few additions per thread, all loads in flight
    constexpr int RP = 32 * V + 1; // pitch of red[SL][RP]
    typedef float vec_t __attribute__((ext_vector_type(V)));
    const int col = threadIdx.x & 31, slice = threadIdx.x >> 5;
    const int i0 = (block * 32 + col) * V;
    vec_t acc = 0.f;
    if (i0 < n) {
        vec_t a[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) a[u] = 0.f;
        int w = slice;
        for (; w + 7 * SL < nparts; w += 8 * SL) {
#pragma unroll
            for (int u = 0; u < 8; ++u) a[u] += *reinterpret_cast<const vec_t *>(part + (size_t)(w + SL * u) * n + i0);
        }
        for (; w < nparts; w += SL) a[0] += *reinterpret_cast<const vec_t *>(part + (size_t)w * n + i0);
        acc = ((a[0] + a[1]) + (a[2] + a[3])) + ((a[4] + a[5]) + (a[6] + a[7]));
    }
#pragma unroll
    for (int v = 0; v < V; ++v) red[slice * RP + col * V + v] = acc[v];
    __syncthreads();
    const int c = threadIdx.x, i = block * 32 * V + c;
    if (c < 32 * V && i < n && i < out.begin[out.nseg]) { // (entries behind the last segment pad the vectors' stride)
        float t[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            t[u] = (red[(4 * u) * RP + c] + red[(4 * u + 1) * RP + c]) + (red[(4 * u + 2) * RP + c] + red[(4 * u + 3) * RP + c]);
        const float sum = ((t[0] + t[1]) + (t[2] + t[3])) + ((t[4] + t[5]) + (t[6] + t[7]));
        int seg = 0;
        while (seg < out.nseg - 1 && i >= out.begin[seg + 1]) ++seg;
        const int k = i - out.begin[seg];
        float *dst = out.ptr[seg] + k;
        if (out.tbl_heads > 0 && seg == out.nseg - 1) {
            const int hd = k / out.tbl_entries, e = k - hd * out.tbl_entries;
            dst = out.ptr[seg] + e * out.tbl_stride + out.tbl_head0 + hd;
        }
        *dst = accumulate ? *dst + sum : sum;
    }
}

template <int V>
__global__ __launch_bounds__(1024) void reduce_partials_kernel(const float *__restrict__ part, int nparts,
                                                               int n, ReduceOut out, int accumulate)
{
    __shared__ float red[32 * (32 * V + 1)];
    reduce_partials_block<V>(part, nparts, n, out, accumulate, (int)blockIdx.x, red);
}

// Two sums in one launch: blocks [0, blocks0) take the first (V entries per load), the others the second
// (one entry per load: the short vectors of a bias-table gradient).
template <int V>
__global__ __launch_bounds__(1024) void reduce_partials_pair_kernel(ReduceJob j0, int blocks0, ReduceJob j1)
{
    __shared__ float red[32 * (32 * V + 1)];
    if ((int)blockIdx.x < blocks0)
        reduce_partials_block<V>(j0.part, j0.nparts, j0.n, j0.out, j0.accumulate, (int)blockIdx.x, red);
    else
        reduce_partials_block<1>(j1.part, j1.nparts, j1.n, j1.out, j1.accumulate, (int)blockIdx.x - blocks0, red);
}

// d w_proj, d b_proj of wide layers: dY^T [A | 1] over plain token rows, 128 tokens per pass of a workgroup
// of eight waves.  Both operands are moved into [channel][token] LDS rows by selector MFMAs; wave w owns
// the output row tiles (w % 4) * RW .. + RW - 1 and half of the column tiles; the spare column C carries the
// bias sums.  The next pass's rows are fetched under the products of the pass in hand.
template <class Cf> struct WprojGradCfg {
    static constexpr int C = Cf::C, KSC = Cf::KSC;
    static constexpr int OTP = (C + 15) / 16, CTP = C / 16 + 1;
    static constexpr int NWV = 8, TOK = 16 * NWV;
    static constexpr int RW = (OTP + 3) / 4;       // row tiles per wave (four row groups)
    static constexpr int CW = (CTP + 1) / 2;       // column tiles per wave (two column halves)
    static constexpr int LW = TOK + 8;             // pitch (bf16) of the [channel][128 tokens] rows
    static constexpr size_t LDS_BYTES = (size_t)16 * (OTP + CTP) * LW * 2;
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
};

template <class Cf>
__global__ __launch_bounds__(512, 1) void wproj_grad_kernel(long T, const bf16_t *__restrict__ dy,
                                                            const bf16_t *__restrict__ attn,
                                                            float *__restrict__ part)
{
    using P = WprojGradCfg<Cf>;
    constexpr int C = Cf::C, KSC = Cf::KSC, OTP = P::OTP, CTP = P::CTP, LW = P::LW, RW = P::RW, CW = P::CW;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    uint16_t *dybuf = reinterpret_cast<uint16_t *>(lds);
    uint16_t *abuf = dybuf + 16 * OTP * LW;
    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, q = lane >> 4;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int rg = wv & 3, ch = wv >> 2;
    const uint2 ones2 = make_uint2(0x3f803f80u, 0x3f803f80u);

    f32x4 acc[RW][CW];
#pragma unroll
    for (int r = 0; r < RW; ++r)
#pragma unroll
        for (int c = 0; c < CW; ++c) acc[r][c] = f32x4{0.f, 0.f, 0.f, 0.f};

    // this lane's token of a pass as operands: channels 32 ks + 8 q .. + 7 of dy and of the saved outputs
    auto load_rows = [&](long tile, uint4 (&dyf)[KSC], uint4 (&af)[KSC]) {
        const long tok = tile * P::TOK + 16 * wv + l16;
        const bool ok = tok < T;
        const uint32_t *dyrow = reinterpret_cast<const uint32_t *>(dy + (ok ? tok : 0) * C);
        const uint32_t *arow = reinterpret_cast<const uint32_t *>(attn + (ok ? tok : 0) * C);
#pragma unroll
        for (int ks = 0; ks < KSC; ++ks) {
            uint32_t dv[4], av[4];
#pragma unroll
            for (int dw = 0; dw < 4; ++dw) {
                const int c = 32 * ks + 8 * q + 2 * dw;
                dv[dw] = c < C ? dyrow[c >> 1] : 0u; // (unconditional loads of a valid row: they merge into 16-byte ones)
                av[dw] = c < C ? arow[c >> 1] : 0u;
            }
            dyf[ks] = ok ? make_uint4(dv[0], dv[1], dv[2], dv[3]) : make_uint4(0u, 0u, 0u, 0u);
            af[ks] = ok ? make_uint4(av[0], av[1], av[2], av[3]) : make_uint4(0u, 0u, 0u, 0u);
        }
    };

    const long ntile = (T + P::TOK - 1) / P::TOK;
    uint4 dyf[KSC], af[KSC], dyn[KSC], an[KSC];
    if ((long)blockIdx.x < ntile) load_rows(blockIdx.x, dyf, af);
    for (long tile = blockIdx.x; tile < ntile; tile += gridDim.x) {
        const bool more = tile + (long)gridDim.x < ntile;
        if (more) load_rows(tile + gridDim.x, dyn, an);
        __syncthreads(); // the previous pass's rows are consumed
#pragma unroll
        for (int ot = 0; ot < OTP; ++ot) {
            const f32x4 tN = mma32(dyf[ot >> 1], select_slot(16 * ot + l16, 32 * (ot >> 1) + 8 * q),
                                   f32x4{0.f, 0.f, 0.f, 0.f});
            *reinterpret_cast<uint2 *>(dybuf + (16 * ot + l16) * LW + 16 * wv + 4 * q) = pack_bf16x4(tN);
        }
#pragma unroll
        for (int ct = 0; ct < CTP; ++ct) {
            f32x4 tN = f32x4{0.f, 0.f, 0.f, 0.f};
            if ((ct >> 1) < KSC)
                tN = mma32(af[(ct >> 1) < KSC ? (ct >> 1) : 0], select_slot(16 * ct + l16, 32 * (ct >> 1) + 8 * q), tN);
            uint2 pk = pack_bf16x4(tN);
            if (16 * ct + l16 == C) pk = ones2; // (tokens past the end have dy = 0)
            *reinterpret_cast<uint2 *>(abuf + (16 * ct + l16) * LW + 16 * wv + 4 * q) = pk;
        }
        __syncthreads();
#pragma unroll
        for (int kp = 0; kp < P::TOK / 32; ++kp) {
            uint4 afr[RW];
#pragma unroll
            for (int r = 0; r < RW; ++r) {
                const int ot = rg * RW + r;
                const uint16_t *ar = dybuf + (16 * (ot < OTP ? ot : 0) + l16) * LW + 32 * kp + 8 * q;
                afr[r] = cat(*reinterpret_cast<const uint2 *>(ar), *reinterpret_cast<const uint2 *>(ar + 4));
            }
#pragma unroll
            for (int c = 0; c < CW; ++c) {
                const int ct = ch * CW + c;
                const uint16_t *br = abuf + (16 * (ct < CTP ? ct : 0) + l16) * LW + 32 * kp + 8 * q;
                const uint4 bf = cat(*reinterpret_cast<const uint2 *>(br), *reinterpret_cast<const uint2 *>(br + 4));
#pragma unroll
                for (int r = 0; r < RW; ++r) acc[r][c] = mma32(afr[r], bf, acc[r][c]);
            }
        }
        if (more) {
#pragma unroll
            for (int ks = 0; ks < KSC; ++ks) {
                dyf[ks] = dyn[ks];
                af[ks] = an[ks];
            }
        }
    }
    float *mine = part + (size_t)blockIdx.x * (C * C + C); // [d w_proj | d b_proj]
#pragma unroll
    for (int r = 0; r < RW; ++r) {
        const int ot = rg * RW + r;
        if (ot < OTP) {
#pragma unroll
            for (int c = 0; c < CW; ++c) {
                const int ct = ch * CW + c;
                const int col = 16 * ct + l16;
                if (ct < CTP) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int o = 16 * ot + 4 * q + j;
                        if (o < C) {
                            if (col < C) mine[o * C + col] = acc[r][c][j];
                            else if (col == C) mine[C * C + o] = acc[r][c][j];
                        }
                    }
                }
            }
        }
    }
}

// Head chunks of the backward, in launch order (last group first).  Chunks are whole groups, so
// the only thing one launch hands to the next is the cascade gradient, which is the dx slice it
// wrote.  Three heads per launch keep the accumulators small enough for two workgroups per CU;
// with one group (no boundary to cut at) a single launch takes all heads at one workgroup per CU.
// Wide layers go one head per launch (their per-head weights and row buffers fill LDS); a group
// split over launches accumulates its dF in the dx slice.
template <bool SPLIT, int G> struct ChunkPlan;
template <> struct ChunkPlan<false, 1> { static constexpr int N = 1; static constexpr int B[1] = {0}, E[1] = {6}; };
template <> struct ChunkPlan<false, 2> { static constexpr int N = 2; static constexpr int B[2] = {3, 0}, E[2] = {6, 3}; };
template <> struct ChunkPlan<false, 3> { static constexpr int N = 3; static constexpr int B[3] = {4, 2, 0}, E[3] = {6, 4, 2}; };
template <> struct ChunkPlan<false, 6> { static constexpr int N = 2; static constexpr int B[2] = {3, 0}, E[2] = {6, 3}; };
template <int G> struct ChunkPlan<true, G> {
    static constexpr int N = 6;
    static constexpr int B[6] = {5, 4, 3, 2, 1, 0}, E[6] = {6, 5, 4, 3, 2, 1};
};
// (with three groups a wide group is two heads, whose weights and buffers fit LDS together; of a
// three-head group two heads fit)
template <> struct ChunkPlan<true, 3> { static constexpr int N = 3; static constexpr int B[3] = {4, 2, 0}, E[3] = {6, 4, 2}; };
template <> struct ChunkPlan<true, 2> { static constexpr int N = 4; static constexpr int B[4] = {4, 3, 1, 0}, E[4] = {6, 4, 3, 1}; };

// Workgroups of a backward launch: narrow layers with more than one group run two per compute unit.
// `cus` = the device's compute units for a launch, kSizingCus for the scratch size (a launch never
// uses more workgroups than the size was computed for).
int bwd_grid(const Geom &g, int cus)
{
    if (cus > kSizingCus) cus = kSizingCus;
    const int grid = ((g.C <= 64 && g.groups > 1) ? 2 : 1) * cus;
    return grid > g.nW ? g.nW : grid;
}

struct GradOut {
    float *dw_qkv, *db_qkv, *dw_proj, *db_proj, *dtable;
    int accumulate;
};

} // namespace

// entries per load: two or four where every partial vector starts on such a boundary and enough workgroups
// remain to fill the chip
static int reduce_width(const float *part, int n)
{
    const uintptr_t at = reinterpret_cast<uintptr_t>(part);
    if (n % 4 == 0 && at % 16 == 0 && n >= 200 * 128) return 4;
    if (n % 2 == 0 && at % 8 == 0 && n >= 200 * 64) return 2;
    return 1;
}

hipError_t launch_reduce(const float *part, int nparts, int n, const ReduceOut &out, int accumulate, hipStream_t s)
{
    KernelTimer kt(K_REDUCE, s);
    switch (reduce_width(part, n)) {
    case 4: hipLaunchKernelGGL(reduce_partials_kernel<4>, dim3((n + 127) / 128), dim3(1024), 0, s, part, nparts, n, out, accumulate); break;
    case 2: hipLaunchKernelGGL(reduce_partials_kernel<2>, dim3((n + 63) / 64), dim3(1024), 0, s, part, nparts, n, out, accumulate); break;
    default: hipLaunchKernelGGL(reduce_partials_kernel<1>, dim3((n + 31) / 32), dim3(1024), 0, s, part, nparts, n, out, accumulate); break;
    }
    return hipGetLastError();
}

hipError_t launch_reduce_pair(const ReduceJob &a, const ReduceJob &b, hipStream_t s)
{
    KernelTimer kt(K_REDUCE, s);
    const int v = reduce_width(a.part, a.n);
    const int blocks0 = (a.n + 32 * v - 1) / (32 * v), blocks1 = (b.n + 31) / 32;
    const dim3 grid(blocks0 + blocks1);
    switch (v) {
    case 4: hipLaunchKernelGGL(reduce_partials_pair_kernel<4>, grid, dim3(1024), 0, s, a, blocks0, b); break;
    case 2: hipLaunchKernelGGL(reduce_partials_pair_kernel<2>, grid, dim3(1024), 0, s, a, blocks0, b); break;
    default: hipLaunchKernelGGL(reduce_partials_pair_kernel<1>, grid, dim3(1024), 0, s, a, blocks0, b); break;
    }
    return hipGetLastError();
}

namespace {

// One chunk of heads: the kernel, then the sum of its partials into the gradients it owns.  The
// scratch is free again afterwards, so every chunk (and the projection's weight gradient of wide
// layers) uses the same buffer: its size is the largest chunk's, not the sum.
template <class Cf, int HB, int HE, bool WPROJ>
hipError_t launch_chunk(const Geom &g, int grid, const bf16_t *x, const bf16_t *dy, const bf16_t *attn,
                        const uint8_t *pack, const bf16_t *table, bf16_t *dx, float *part, const GradOut &go,
                        hipStream_t s)
{
    using B = BwdCfg<Cf, HB, HE, WPROJ>;
    static_assert(B::LDS_BYTES <= 160 * 1024, "LDS budget");
    auto kern = fused_bwd_kernel<Cf, HB, HE, WPROJ>;
    if (hipError_t ea = allow_dynamic_lds(reinterpret_cast<const void *>(kern), B::LDS_BYTES); ea != hipSuccess) return ea;
    {
        KernelTimer kt(K_FUSED_BWD, s);
        hipLaunchKernelGGL(kern, dim3(grid), dim3(256), B::LDS_BYTES, s, g, x, dy, attn, pack, table, dx, part);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    constexpr int CG = Cf::CG, D = Cf::D;
    ReduceOut out{};
    int k = 0;
    static_assert(2 * B::NG * 3 + 3 <= ReduceOut::MAXSEG, "segment table");
    for (int gi = 0; gi < B::NG; ++gi)
        for (int t = 0; t < 3; ++t) { // d w_qkv rows of (group, q|k|v) owned by the chunk's heads
            out.ptr[k] = go.dw_qkv + (size_t)((B::GB + gi) * 3 * CG + t * CG + B::HL0 * D) * CG;
            out.begin[k++] = B::L_DWQ + (gi * 3 + t) * B::RG * CG;
        }
    for (int gi = 0; gi < B::NG; ++gi)
        for (int t = 0; t < 3; ++t) {
            out.ptr[k] = go.db_qkv + (B::GB + gi) * 3 * CG + t * CG + B::HL0 * D;
            out.begin[k++] = B::L_DBQ + (gi * 3 + t) * B::RG;
        }
    if (WPROJ) {
        out.ptr[k] = go.dw_proj; out.begin[k++] = B::L_DWP;
        out.ptr[k] = go.db_proj; out.begin[k++] = B::L_DBP;
    }
    out.ptr[k] = go.dtable; out.begin[k++] = B::L_TBL;
    out.begin[k] = B::L_END;
    out.nseg = k;
    out.tbl_heads = B::NH; out.tbl_entries = B::NTBL; out.tbl_stride = Cf::HEADS; out.tbl_head0 = HB;
    return launch_reduce(part, grid, B::L_TOTAL, out, go.accumulate, s);
}

template <class Cf, int I = 0>
hipError_t launch_chunks(const Geom &g, int grid, const bf16_t *x, const bf16_t *dy, const bf16_t *attn,
                         const uint8_t *pack, const bf16_t *table, bf16_t *dx, float *part, const GradOut &go,
                         hipStream_t s)
{
    using Plan = ChunkPlan<Cf::SPLIT, Cf::G>;
    if constexpr (I < Plan::N) {
        hipError_t e = launch_chunk<Cf, Plan::B[I], Plan::E[I], !Cf::SPLIT && Plan::E[I] == Cf::HEADS>(
            g, grid, x, dy, attn, pack, table, dx, part, go, s);
        if (e != hipSuccess) return e;
        return launch_chunks<Cf, I + 1>(g, grid, x, dy, attn, pack, table, dx, part, go, s);
    }
    return hipSuccess;
}

// floats of the largest per-workgroup partial vector over the launches of a layer
template <class Cf, int I = 0> constexpr int max_partial()
{
    using Plan = ChunkPlan<Cf::SPLIT, Cf::G>;
    if constexpr (I < Plan::N) {
        constexpr int mine = BwdCfg<Cf, Plan::B[I], Plan::E[I], !Cf::SPLIT && Plan::E[I] == Cf::HEADS>::L_TOTAL;
        constexpr int rest = max_partial<Cf, I + 1>();
        return mine > rest ? mine : rest;
    } else {
        return Cf::SPLIT ? Cf::C * Cf::C + Cf::C : 0;
    }
}

// d w_proj, d b_proj of a wide layer: the kernel, then the sum of its partials.
template <class Cf>
hipError_t run_wproj_grad(const Geom &g, int grid, const bf16_t *dy, const bf16_t *attn, float *part, float *dw_proj,
                          float *db_proj, int accumulate, hipStream_t s)
{
    using P = WprojGradCfg<Cf>;
    constexpr size_t lds = P::LDS_BYTES;
    auto kern = wproj_grad_kernel<Cf>;
    if (hipError_t ea = allow_dynamic_lds(reinterpret_cast<const void *>(kern), lds); ea != hipSuccess) return ea;
    {
        KernelTimer kt(K_WPROJ_GRAD, s);
        hipLaunchKernelGGL(kern, dim3(grid), dim3(64 * P::NWV), lds, s, g.T, dy, attn, part);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    ReduceOut out{};
    out.ptr[0] = dw_proj; out.begin[0] = 0;
    out.ptr[1] = db_proj; out.begin[1] = Cf::C * Cf::C;
    out.begin[2] = Cf::C * Cf::C + Cf::C;
    out.nseg = 2;
    return launch_reduce(part, grid, Cf::C * Cf::C + Cf::C, out, accumulate, s);
}

template <class Cf>
hipError_t run_bwd(const Geom &g, const bf16_t *x, const bf16_t *dy, const bf16_t *attn,
                   const void *pack_, const bf16_t *table, bf16_t *dx, float *dw_qkv, float *db_qkv,
                   float *dw_proj, float *db_proj, float *dtable, int accumulate, void *ws, hipStream_t s)
{
    const uint8_t *pack = static_cast<const uint8_t *>(pack_);
    float *part = static_cast<float *>(ws);
    const int grid = bwd_grid(g, device_cu_count());
    if constexpr (Cf::SPLIT) {
        if (wide_bwd_supported(g)) { // (16-byte aligned tensors: the entry points check; the projection's gradient reuses the scratch afterwards)
            hipError_t e = launch_wide_bwd(g, x, dy, attn, pack_, dx, dw_qkv, db_qkv, dtable, accumulate, ws, s);
            if (e != hipSuccess) return e;
            return run_wproj_grad<Cf>(g, grid, dy, attn, part, dw_proj, db_proj, accumulate, s);
        }
    }
    const GradOut go{dw_qkv, db_qkv, dw_proj, db_proj, dtable, accumulate};
    hipError_t e = launch_chunks<Cf>(g, grid, x, dy, attn, pack, table, dx, part, go, s);
    if (e != hipSuccess) return e;
    if constexpr (Cf::SPLIT) return run_wproj_grad<Cf>(g, grid, dy, attn, part, dw_proj, db_proj, accumulate, s);
    return hipSuccess;
}

#define GSWA_FUSED_SHAPES(X) X(60, 6, 1) X(60, 6, 2) X(60, 6, 3) X(60, 6, 6) X(180, 6, 2) X(180, 6, 3)

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
    int total = 0;
#define X(C_, H_, G_) \
    if (g.C == C_ && g.heads == H_ && g.groups == G_) total = max_partial<FusedCfg<C_, H_, G_>>();
    GSWA_FUSED_SHAPES(X)
#undef X
    const size_t chunks = ((size_t)bwd_grid(g, kSizingCus) * total * 4 + 255) & ~size_t(255);
    const size_t wide = wide_bwd_supported(g) ? wide_bwd_ws_bytes(g) : 0;
    return wide > chunks ? wide : chunks;
}

hipError_t launch_fused_bwd(const Geom &g, const bf16_t *x, const bf16_t *dy, const bf16_t *attn,
                            const void *pack, const bf16_t *table, bf16_t *dx, float *dw_qkv,
                            float *db_qkv, float *dw_proj, float *db_proj, float *dtable, int accumulate,
                            void *ws, hipStream_t s)
{
#define X(C_, H_, G_)                                                   \
    if (g.C == C_ && g.heads == H_ && g.groups == G_)                   \
        return run_bwd<FusedCfg<C_, H_, G_>>(g, x, dy, attn, pack, table, dx, dw_qkv, db_qkv, dw_proj,      \
                                             db_proj, dtable, accumulate, ws, s);
    GSWA_FUSED_SHAPES(X)
#undef X
    return hipErrorInvalidValue;
}

} // namespace gswa
