// Whole GSWA forward of one window in one workgroup, for narrow bf16 layers whose windows have 64
// or 144 tokens and whose queries/keys may be narrower than the values (Sec. "Parameter
// Allocation", Sec. "Experimental Settings"): shift + partition, and for every head group the
// q|k|v projection (Eq. 6) with the cascade add (Eq. 8), scores + bias + mask + softmax + PV per
// head, then the output projection (Eq. 7) and the reverse shift.  One wavefront owns 16 tokens
// from x to y: its group outputs never leave its registers and its own rows of LDS, only K and V
// of the current group are shared between the waves of the window.
//
// Orientation (see mfma.h): Q^T and K^T tiles come out of the projection MFMA as [feature][token],
// which packed is the B operand of the score product (k-slots = features) resp. an 8-byte store
// into the token-major K rows; V comes out as [token][feature] by swapping the operands of the
// same MFMA, which packed is an 8-byte store into the channel-major V rows.  A head's q features
// are selected by zeroing the other rows of the packed Q^T tile, so the K rows of all heads of the
// group can stay interleaved.
#include "staged_kernels.h"
#include "mfma.h"

namespace gswa {

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr int QTM = 2, VTM = 4, KSM = 2; // most 16-feature tiles of q (and k), of v; most 32-channel K steps
// pitches (bf16) of the token-major K rows and of the output rows; fixed, so that the row offsets of
// the unrolled operand reads are immediates
constexpr int LKA = 16 * QTM + 4, LOR = 32 * KSM + 8;

// Uniform shape numbers and the LDS carve, the same on host and device.
struct WinLayout {
    int QTn, VTn, KSF, OTn, KSC; // tiles of q, of v per group; K steps over Cg; output tiles and K steps of the projection
    int nfg;                     // weight fragments of one group
    int LT;                      // pitch (bf16) of the channel-major rows
    int tf;                      // floats of one head's bias table (padded)
    size_t off_koff, off_tok, off_bias, off_wf, off_ks, off_vt, off_orow, bytes;
};
__host__ __device__ inline WinLayout win_layout(const Geom &g)
{
    WinLayout L;
    L.QTn = (g.Qg + 15) / 16;
    L.VTn = (g.Cg + 15) / 16;
    L.KSF = (g.Cg + 31) / 32;
    L.OTn = (g.C + 15) / 16;
    L.KSC = (g.C + 31) / 32;
    L.nfg = (2 * L.QTn + L.VTn) * L.KSF;
    L.LT = g.N + 4;
    const int ntbl = (2 * g.M - 1) * (2 * g.M - 1);
    L.tf = (ntbl + 3) & ~3;
    size_t o = (size_t)4 * L.tf * g.heads;
    L.off_koff = o; o += (size_t)4 * g.N;
    L.off_tok = o; o += (size_t)4 * g.N;
    L.off_bias = o; o += (size_t)4 * (((size_t)g.groups * g.Rg + g.C + 3) & ~size_t(3));
    L.off_wf = o; o += (size_t)1024 * ((size_t)g.groups * L.nfg + (size_t)L.OTn * L.KSC);
    L.off_ks = o; o += (size_t)2 * g.N * LKA;
    L.off_vt = o; o += (size_t)2 * 16 * L.VTn * L.LT;
    L.off_orow = o; o += (size_t)2 * g.N * LOR;
    L.bytes = o;
    return L;
}

__device__ __forceinline__ uint2 lds8(const uint16_t *p) { return *reinterpret_cast<const uint2 *>(p); }

// eight consecutive bf16 of a row (dword reads; the row and k0 are even), zero beyond kmax
__device__ __forceinline__ uint4 row8(const uint16_t *row, int k0, int kmax)
{
    const uint32_t *r32 = reinterpret_cast<const uint32_t *>(row);
    uint32_t v[4];
#pragma unroll
    for (int dw = 0; dw < 4; ++dw) v[dw] = k0 + 2 * dw < kmax ? r32[(k0 >> 1) + dw] : 0u;
    return make_uint4(v[0], v[1], v[2], v[3]);
}

__device__ __forceinline__ uint32_t add_bf16x2(uint32_t a, uint32_t b)
{
    return pack_bf16x2(bf16_lo(a) + bf16_lo(b), bf16_hi(a) + bf16_hi(b));
}

// QTN / VTN: 16-feature tiles of q (and of k) / of v per group, compile-time so that the tile loops
// carry no guards (the register budget decides how many windows a compute unit holds).
template <int NT, int QTN, int VTN>
__global__ __launch_bounds__(64 * NT) void window_fwd_kernel(Geom g, const bf16_t *__restrict__ x,
                                                            const bf16_t *__restrict__ w_qkv,
                                                            const bf16_t *__restrict__ b_qkv,
                                                            const bf16_t *__restrict__ w_proj,
                                                            const bf16_t *__restrict__ b_proj,
                                                            const bf16_t *__restrict__ table,
                                                            bf16_t *__restrict__ y, bf16_t *__restrict__ attn_out)
{
    constexpr int N = 16 * NT, NTH = 64 * NT, LT = N + 4, KSF = (VTN + 1) / 2;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const WinLayout L = win_layout(g);
    float *tb = reinterpret_cast<float *>(lds);                       // [heads][tf], base-2 units
    int *koff = reinterpret_cast<int *>(lds + L.off_koff);
    int *tok = reinterpret_cast<int *>(lds + L.off_tok);
    float *bias = reinterpret_cast<float *>(lds + L.off_bias);        // [G*Rg | C]
    uint4 *wf = reinterpret_cast<uint4 *>(lds + L.off_wf);            // [fragment][lane]
    uint16_t *Ks = reinterpret_cast<uint16_t *>(lds + L.off_ks);      // [N][LKa]: k of the group, token-major
    uint16_t *VT = reinterpret_cast<uint16_t *>(lds + L.off_vt);      // [16*VTn][LT]: v of the group, channel-major
    uint16_t *Orow = reinterpret_cast<uint16_t *>(lds + L.off_orow);  // [N][LO]: concatenated group outputs

    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, q = lane >> 4;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int w = blockIdx.x;
    constexpr int M = NT == 4 ? 8 : 12, nt1 = 2 * M - 1, ntbl = nt1 * nt1; // N = M * M is 64 or 144
    const int C = g.C, Cg = g.Cg, Qg = g.Qg, Rg = g.Rg, d = g.d, dq = g.dq, hg = g.hg, G = g.groups;
    const uint16_t *x16 = reinterpret_cast<const uint16_t *>(x);
    const uint16_t *wq16 = reinterpret_cast<const uint16_t *>(w_qkv);
    const uint16_t *wp16 = reinterpret_cast<const uint16_t *>(w_proj);

    // ---- set-up: geometry, bias tables, linear biases, weight fragments ----
    for (int n = tid; n < N; n += NTH) {
        int reg;
        tok[n] = (int)window_token(g, w, n, reg);
        const int r = n / M, c = n - r * M;
        koff[n] = (r * nt1 + c) | (reg << 16);
    }
    for (int e = tid; e < ntbl * g.heads; e += NTH) {
        const int i = e / g.heads, hd = e - i * g.heads;
        tb[hd * L.tf + i] = to_f32(table[e]) * kLog2e;
    }
    for (int e = tid; e < G * Rg + C; e += NTH) bias[e] = e < G * Rg ? to_f32(b_qkv[e]) : to_f32(b_proj[e - G * Rg]);
    // fragment (f, lane): row/column l16 of a 16-feature tile, k-slots = 8 consecutive input channels.
    // Order inside a group: q tiles, k tiles, v tiles, each with its K steps; then the projection.
    for (int i = tid; i < (G * L.nfg + L.OTn * L.KSC) * 64; i += NTH) {
        const int f = i >> 6, ln = i & 63, r16 = ln & 15, k0q = 8 * (ln >> 4);
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (f < G * L.nfg) {
            const int gi = f / L.nfg, fl = f - gi * L.nfg;
            const int tile = fl / KSF, ks = fl - tile * KSF;
            int row; // row of the group's [q | k | v] weight block, or -1
            if (tile < QTN) row = 16 * tile + r16 < Qg ? 16 * tile + r16 : -1;
            else if (tile < 2 * QTN) row = 16 * (tile - QTN) + r16 < Qg ? Qg + 16 * (tile - QTN) + r16 : -1;
            else row = 16 * (tile - 2 * QTN) + r16 < Cg ? 2 * Qg + 16 * (tile - 2 * QTN) + r16 : -1;
            if (row >= 0) v = row8(wq16 + ((long)gi * Rg + row) * Cg, 32 * ks + k0q, Cg);
        } else {
            const int fl = f - G * L.nfg;
            const int ot = fl / L.KSC, ks = fl - ot * L.KSC;
            if (16 * ot + r16 < C) v = row8(wp16 + (long)(16 * ot + r16) * C, 32 * ks + k0q, C);
        }
        wf[i] = v;
    }
    // the channels of the output rows beyond C feed zero weights, but must not hold NaN patterns
    for (int e = tid; e < N * (LOR / 2); e += NTH) reinterpret_cast<uint32_t *>(Orow)[e] = 0u;
    __syncthreads();

    const int own = 16 * wv + l16; // this lane's token as a row / column of its wave's tiles
    const int kq = koff[own];
    const int qo = (kq & 0xffff) + (M - 1) * nt1 + (M - 1), regn = kq >> 16;
    const float sc2 = kLog2e / sqrtf((float)dq), maskv = -100.0f * kLog2e;
    const uint16_t *xrow = x16 + (long)tok[own] * C;
    uint16_t *orow = Orow + own * LOR;

    for (int gi = 0; gi < G; ++gi) {
        // ---- F_g = x slice (+ output of the previous group), this lane's token, 8 channels per K step ----
        uint4 ff[KSF];
#pragma unroll
        for (int ks = 0; ks < KSF; ++ks) {
            ff[ks] = make_uint4(0u, 0u, 0u, 0u);
            {
                ff[ks] = row8(xrow + gi * Cg, 32 * ks + 8 * q, Cg);
                if (gi > 0 && g.cascade) {
                    const uint4 pv = row8(orow + (gi - 1) * Cg, 32 * ks + 8 * q, Cg);
                    ff[ks] = make_uint4(add_bf16x2(ff[ks].x, pv.x), add_bf16x2(ff[ks].y, pv.y),
                                        add_bf16x2(ff[ks].z, pv.z), add_bf16x2(ff[ks].w, pv.w));
                }
            }
        }
        const uint4 *wg = wf + (size_t)gi * L.nfg * 64;
        const float *bg = bias + gi * Rg;
        // ---- q^T (kept), k^T (to the K rows) and v (to the V rows) of the wave's 16 tokens ----
        uint2 qT[QTN];
#pragma unroll
        for (int t = 0; t < QTN; ++t) {
            qT[t] = make_uint2(0u, 0u);
            {
                f32x4 aq = {0.f, 0.f, 0.f, 0.f}, ak = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KSF; ++ks) {
                        aq = mma32(wg[(t * KSF + ks) * 64 + lane], ff[ks], aq);
                        ak = mma32(wg[((QTN + t) * KSF + ks) * 64 + lane], ff[ks], ak);
                    }
                // rows 4q + j = features 16t + 4q + j, column l16 = token
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int f = 16 * t + 4 * q + j;
                    aq[j] += f < Qg ? bg[f] : 0.f;
                    ak[j] += f < Qg ? bg[Qg + f] : 0.f;
                }
                qT[t] = pack_bf16x4(aq);
                *reinterpret_cast<uint2 *>(&Ks[own * LKA + 16 * t + 4 * q]) = pack_bf16x4(ak);
            }
        }
#pragma unroll
        for (int t = 0; t < VTN; ++t)
            {
                f32x4 av = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KSF; ++ks) av = mma32(ff[ks], wg[((2 * QTN + t) * KSF + ks) * 64 + lane], av);
                // column l16 = feature 16t + l16, rows 4q + j = tokens 16 wv + 4q + j
                const int f = 16 * t + l16;
                const float b = f < Cg ? bg[2 * Qg + f] : 0.f;
#pragma unroll
                for (int j = 0; j < 4; ++j) av[j] += b;
                *reinterpret_cast<uint2 *>(&VT[(16 * t + l16) * LT + 16 * wv + 4 * q]) = pack_bf16x4(av);
            }
        __syncthreads();

        // ---- the heads of the group ----
        f32x4 oacc[VTN];
#pragma unroll
        for (int t = 0; t < VTN; ++t) oacc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int hl = 0; hl < hg; ++hl) {
            const int hd = gi * hg + hl;
            const float *tbh = tb + hd * L.tf;
            // the key offsets do not change from head to head, but reading them again is cheaper than
            // keeping 36 of them (and what is derived from them) in registers across the loop
            uint32_t opq = 0;
            asm volatile("" : "+v"(opq));
            const int *koffh = koff + opq;
            const int f0 = hl * dq, f1 = f0 + dq; // this head's rows of the q / k block
            // Q^T with the rows of the other heads zeroed
            uint2 qm[QTN];
#pragma unroll
            for (int t = 0; t < QTN; ++t) {
                const int fb = 16 * t + 4 * q;
                const uint32_t m0 = (fb >= f0 && fb < f1) ? 0x0000ffffu : 0u, m1 = (fb + 1 >= f0 && fb + 1 < f1) ? 0xffff0000u : 0u;
                const uint32_t m2 = (fb + 2 >= f0 && fb + 2 < f1) ? 0x0000ffffu : 0u, m3 = (fb + 3 >= f0 && fb + 3 < f1) ? 0xffff0000u : 0u;
                qm[t] = make_uint2(qT[t].x & (m0 | m1), qT[t].y & (m2 | m3));
            }
            f32x4 st[NT];
            float mx = -INFINITY;
#pragma unroll
            for (int kt = 0; kt < NT; ++kt) {
                f32x4 a = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int t = 0; t < QTN; ++t)
                    if (16 * t < f1 && 16 * t + 16 > f0) // uniform: the tile holds rows of this head
                        a = mma16(lds8(&Ks[(16 * kt + l16) * LKA + 16 * t + 4 * q]), qm[t], a);
                const int4 ko = *reinterpret_cast<const int4 *>(&koffh[16 * kt + 4 * q]);
                const int kk[4] = {ko.x, ko.y, ko.z, ko.w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    float s = fmaf(a[j], sc2, tbh[qo - (kk[j] & 0xffff)]);
                    s += (kk[j] >> 16) != regn ? maskv : 0.f;
                    a[j] = s;
                    mx = fmaxf(mx, s);
                }
                st[kt] = a;
            }
            mx = qgroup_max(mx);
            float sum = 0.f;
            uint2 pb[NT]; // unnormalised probabilities, bf16: the B operand of the PV product
#pragma unroll
            for (int kt = 0; kt < NT; ++kt) {
                f32x4 p;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    p[j] = __builtin_amdgcn_exp2f(st[kt][j] - mx);
                    sum += p[j];
                }
                pb[kt] = pack_bf16x4(p);
            }
            sum = qgroup_sum(sum);
            const float inv = 1.0f / sum;
            // O^T rows of this head: channels [hl*d, hl*d + d) of the group's v block
            const int c0 = hl * d, c1 = c0 + d;
#pragma unroll
            for (int t = 0; t < VTN; ++t)
                if (16 * t < c1 && 16 * t + 16 > c0) { // uniform
                    f32x4 o = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int kt = 0; kt < NT; ++kt) o = mma16(lds8(&VT[(16 * t + l16) * LT + 16 * kt + 4 * q]), pb[kt], o);
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int c = 16 * t + 4 * q + j;
                        oacc[t][j] = (c >= c0 && c < c1) ? o[j] * inv : oacc[t][j];
                    }
                }
        }
        // ---- group output: rows 4q + j = channels 16t + 4q + j of the group, column l16 = token ----
#pragma unroll
        for (int t = 0; t < VTN; ++t)
            {
                const int c = 16 * t + 4 * q; // Cg is even: channel pairs are inside or outside together
                const uint2 pk = pack_bf16x4(oacc[t]);
                uint32_t *o32 = reinterpret_cast<uint32_t *>(orow + gi * Cg + c);
                if (c < Cg) o32[0] = pk.x;
                if (c + 2 < Cg) o32[1] = pk.y;
                if (attn_out) {
                    uint32_t *a32 = reinterpret_cast<uint32_t *>(reinterpret_cast<uint16_t *>(attn_out) +
                                                                 (long)tok[own] * C + gi * Cg + c);
                    if (c < Cg) a32[0] = pk.x;
                    if (c + 2 < Cg) a32[1] = pk.y;
                }
            }
        __syncthreads(); // K and V rows are rewritten by the next group; the output rows are read below
    }

    // ---- output projection of the wave's 16 tokens and reverse shift ----
    const uint4 *wpf = wf + (size_t)G * L.nfg * 64;
    const float *bp = bias + G * Rg;
    uint4 af[KSM];
#pragma unroll
    for (int ks = 0; ks < KSM; ++ks) af[ks] = ks < L.KSC ? row8(orow, 32 * ks + 8 * q, 32 * L.KSC) : make_uint4(0u, 0u, 0u, 0u);
    uint16_t *yrow = reinterpret_cast<uint16_t *>(y) + (long)tok[own] * C;
    for (int ot = 0; ot < L.OTn; ++ot) {
        f32x4 a = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KSM; ++ks)
            if (ks < L.KSC) a = mma32(wpf[(ot * L.KSC + ks) * 64 + lane], af[ks], a);
        const int c = 16 * ot + 4 * q; // rows 4q + j = output channels, column l16 = token
#pragma unroll
        for (int j = 0; j < 4; ++j) a[j] += c + j < C ? bp[c + j] : 0.f;
        const uint2 pk = pack_bf16x4(a);
        uint32_t *y32 = reinterpret_cast<uint32_t *>(yrow + c);
        if (c < C) y32[0] = pk.x;
        if (c + 2 < C) y32[1] = pk.y;
    }
}

} // namespace

bool window_fwd_supported(const Geom &g)
{
    const int nt = g.N / 16;
    if (g.N % 16 || (nt != 4 && nt != 9)) return false;
    if ((g.C & 3) || (g.Cg & 1) || g.C > 32 * KSM || g.Cg > 16 * VTM || g.Qg > 16 * QTM) return false;
    if (g.d > 16 || g.dq > 16 || g.T >= (1L << 31)) return false;
    const int qtn = (g.Qg + 15) / 16, vtn = (g.Cg + 15) / 16;
    if (qtn == 2 && vtn == 1) return false; // not instantiated
    return win_layout(g).bytes <= 160 * 1024;
}

namespace {
template <int NT, int QTN, int VTN>
hipError_t launch_window_fwd_t(const Geom &g, const bf16_t *x, const bf16_t *w_qkv, const bf16_t *b_qkv,
                               const bf16_t *w_proj, const bf16_t *b_proj, const bf16_t *table, bf16_t *y,
                               bf16_t *attn_out, hipStream_t s)
{
    const size_t lds = win_layout(g).bytes;
    auto kern = window_fwd_kernel<NT, QTN, VTN>;
    if (hipError_t ea = allow_dynamic_lds(reinterpret_cast<const void *>(kern), lds); ea != hipSuccess) return ea;
    KernelTimer kt(K_WINDOW_FWD, s);
    hipLaunchKernelGGL(kern, dim3(g.nW), dim3(64 * NT), lds, s, g, x, w_qkv, b_qkv, w_proj, b_proj, table, y, attn_out);
    return hipGetLastError();
}
} // namespace

#define GSWA_WINDOW_SHAPES(X) \
    X(4, 1, 1) X(4, 1, 2) X(4, 1, 3) X(4, 1, 4) X(4, 2, 2) X(4, 2, 3) X(4, 2, 4) \
    X(9, 1, 1) X(9, 1, 2) X(9, 1, 3) X(9, 1, 4) X(9, 2, 2) X(9, 2, 3) X(9, 2, 4)

hipError_t launch_window_fwd(const Geom &g, const bf16_t *x, const bf16_t *w_qkv, const bf16_t *b_qkv,
                             const bf16_t *w_proj, const bf16_t *b_proj, const bf16_t *table, bf16_t *y,
                             bf16_t *attn_out, hipStream_t s)
{
    if (!window_fwd_supported(g)) return hipErrorInvalidValue;
    const int nt = g.N / 16, qtn = (g.Qg + 15) / 16, vtn = (g.Cg + 15) / 16;
#define X(NT_, Q_, V_) \
    if (nt == NT_ && qtn == Q_ && vtn == V_) \
        return launch_window_fwd_t<NT_, Q_, V_>(g, x, w_qkv, b_qkv, w_proj, b_proj, table, y, attn_out, s);
    GSWA_WINDOW_SHAPES(X)
#undef X
    return hipErrorInvalidValue;
}

} // namespace gswa
