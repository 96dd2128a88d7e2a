// Fused GSWA forward: shift + partition + per-group QKV projection (Eq. 6) with the cascade add
// (Eq. 8) + scores with relative bias and shift mask + softmax + PV + output projection (Eq. 7)
// + window merge + reverse shift, one kernel, one pass over x and y.
#include "fused.h"
#include "mfma.h"

namespace gswa {

namespace {

constexpr float kLog2e = 1.4426950408889634f;
// Shift mask in the base-2 units of the fused forward: -100 * log2(e) rounded to bf16, so that the
// terms of the mask product cancel exactly (-144 / log2(e) = -99.8 in natural units).
constexpr float kMaskLog2 = -144.0f;

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
                                                          const bf16_t *__restrict__ table,
                                                          uint8_t *__restrict__ pack, int wide_first)
{
    // blocks from wide_first on (if not negative): the layouts of the wide one-launch kernels, same launch
    if constexpr (Cf::SPLIT) {
        if (wide_first >= 0 && (int)blockIdx.x >= wide_first) {
            wide_pack_entry<Cf>(((int)blockIdx.x - wide_first) * 256 + (int)threadIdx.x, w_qkv, w_proj, table, pack);
            return;
        }
    }
    constexpr int C = Cf::C, D = Cf::D, CG = Cf::CG, HG = Cf::HG, HEADS = Cf::HEADS, ET = Cf::ET;
    constexpr int KS = Cf::KS, KSC = Cf::KSC;
    constexpr int E_WQH = Cf::N_WQH * 64, E_WP2 = Cf::N_WP2 * 64, E_BF = Cf::N_BF * 64, E_WQ = Cf::N_WQ * 64,
                  E_WPT = Cf::N_WPT * 64, E_WQT = Cf::N_WQT * 64, E_BIAS = 4 * C;
    const float qscale = 1.0f / sqrtf((float)D);
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    int l16 = i & 15, q = (i >> 4) & 3; // lane coordinates inside the current segment

    if (i < E_WQH) { // Wqkv, head-padded input order: l16 -> out feature e; k-slot s -> head 2*step + s/4, e' = 4q + s%4
        int f = i >> 6;
        const int st = f % Cf::NSTEP; f /= Cf::NSTEP;
        const int t = f % 3;
        const int hd = f / 3, gi = hd / HG, hl = hd % HG;
        const float sc = t == 0 ? qscale * kLog2e : 1.0f;
        uint32_t v[8];
        for (int s = 0; s < 8; ++s) {
            const int hlp = 2 * st + (s >> 2), ep = 4 * q + (s & 3);
            float w = 0.f;
            if (st < HG / 2 || s < 4) {
                if (l16 < D && hlp < HG && ep < D)
                    w = to_f32(w_qkv[((size_t)gi * 3 * CG + t * CG + hl * D + l16) * CG + hlp * D + ep]) * sc;
            } else if (q == 0 && l16 >= D && l16 < D + 4) {
                // mask inputs (1, r, c, r*c) -> rows D..D+3: the query side carries the coefficients of
                //   mask(n,m) = kMask * [ (r_n|c_n) + (1-2r_n)(1-c_n) r_m + (1-2c_n)(1-r_n) c_m - (1-2r_n)(1-2c_n) r_m c_m ],
                // the key side the inputs themselves
                const int fo = l16 - D, fi = s - 4;
                const float cq[4][4] = {{0, 1, 1, -1}, {1, -2, -1, 2}, {1, -1, -2, 2}, {-1, 2, 2, -4}};
                w = t == 0 ? kMaskLog2 * cq[fo][fi] : (t == 1 && fo == fi) ? 1.0f : 0.f;
            }
            v[s] = f32_to_bf16_bits(w);
        }
        reinterpret_cast<uint4 *>(pack + Cf::P_WQH)[i] =
            make_uint4(v[0] | v[1] << 16, v[2] | v[3] << 16, v[4] | v[5] << 16, v[6] | v[7] << 16);
        return;
    }
    i -= E_WQH;
    if (i < E_WP2) { // Wproj: l16 -> output channel o; k-slot s -> head 2*pair + s/4, e = 4q + s%4
        const int f = i >> 6;
        const int pr = f % (HEADS / 2), ot = f / (HEADS / 2);
        const int o = 16 * ot + l16;
        uint32_t v[8];
        for (int s = 0; s < 8; ++s) {
            const int hd = 2 * pr + (s >> 2), e = 4 * q + (s & 3);
            v[s] = (o < C && e < D) ? (uint32_t)w_proj[(size_t)o * C + hd * D + e].bits : 0u;
        }
        reinterpret_cast<uint4 *>(pack + Cf::P_WP2)[i] =
            make_uint4(v[0] | v[1] << 16, v[2] | v[3] << 16, v[4] | v[5] << 16, v[6] | v[7] << 16);
        return;
    }
    i -= E_WP2;
    if (i < E_BF) { // bias (base-2 units) of score tile (key tile kt, query tile nt), nt - kt = dlt - 3, as a
        // B operand: column l16 = query (2nt + l16/8, l16%8), k-slots 4q+j = key (2kt + q/2, 4(q%2) + j)
        constexpr int M = 8;
        const int f = i >> 6;
        const int dlt = f % Cf::NDLT, hd = f / Cf::NDLT;
        const int dr = 2 * (dlt - 3) + (l16 >> 3) - (q >> 1);
        uint32_t v[4];
        for (int j = 0; j < 4; ++j) {
            const int dc = (l16 & 7) - 4 * (q & 1) - j;
            v[j] = f32_to_bf16_bits(to_f32(table[((dr + M - 1) * (2 * M - 1) + (dc + M - 1)) * HEADS + hd]) * kLog2e);
        }
        reinterpret_cast<uint2 *>(pack + Cf::P_BF)[i] = make_uint2(v[0] | v[1] << 16, v[2] | v[3] << 16);
        return;
    }
    i -= E_BF;
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
// ---------------------------------------------------------------------------------------
// Forward with one wavefront per window (8x8 windows, narrow layers).  The wave holds all 64
// tokens of its window as four 16-token tiles, so K, V and the probabilities never leave its
// registers and no barrier is needed after the set-up.  The vector ALUs are the scarce unit
// (the exponentials alone take a third of their time), so everything that can be phrased as a
// matrix product runs on the MFMA pipe instead:
//   * a score tile is one K=32 MFMA [K | I] [Q^T ; B]: the upper half adds the relative bias
//     tile B (it depends on the key/query tile offset only: seven operands per head);
//   * the shift mask (-100 between tokens of different wrap regions) is a rank-4 function of
//     the two tokens, carried in the zero-padded rows D..D+3 of Q^T and K^T, which the Q/K
//     projection itself fills from four per-token inputs (1, r, c, r*c);
//   * the row maximum is subtracted by a rank-1 MFMA update of the score tiles;
//   * the softmax denominator is row D of the PV product: column D of V is one;
//   * scores are in base-2 units (log2(e) folded into the query weights and the bias).
// The cascade input of Eq. 8 is added to the x operand of the next group in registers (the
// packed output tiles of a group are the k-slots of the head-padded weight fragments), rounded
// to bf16 like a stored activation.
// ---------------------------------------------------------------------------------------
template <class Cf> struct WaveFwdCfg {
    static constexpr int NWAVES = 8, NTHREADS = 64 * NWAVES;
    // LDS: the linear biases first (their many small reads then all have immediate offsets), then
    // the packed range [0, P_WQ) as it is
    static constexpr size_t OFF_BIAS = 0;
    static constexpr size_t OFF_COPY = (size_t)16 * Cf::C;
    static constexpr size_t OFF_WQH = OFF_COPY + Cf::P_WQH, OFF_WP2 = OFF_COPY + Cf::P_WP2, OFF_BF = OFF_COPY + Cf::P_BF;
    static constexpr size_t COPY_BYTES = Cf::P_WQ;
    static constexpr int COPY_IT = (int)((COPY_BYTES / 16 + NTHREADS - 1) / NTHREADS);
    static constexpr size_t LDS_BYTES = OFF_COPY + COPY_BYTES;
};

// the value of row-group Q0 (lanes 16*Q0 .. 16*Q0+15) copied to the lanes of all four groups
template <int Q0> __device__ __forceinline__ float qgroup_broadcast(float v)
{
    const unsigned u = __float_as_uint(v);
    u32x2 r = __builtin_amdgcn_permlane32_swap(u, u, false, false); // {groups 0,1,0,1; groups 2,3,2,3}
    const unsigned h = r[Q0 >> 1];
    r = __builtin_amdgcn_permlane16_swap(h, h, false, false);       // {even group of each pair; odd group}
    return __uint_as_float(r[Q0 & 1]);
}

// elementwise sum of two packed bf16 pairs, rounded to nearest even
__device__ __forceinline__ uint32_t add_bf16x2(uint32_t a, uint32_t b)
{
    return pack_bf16x2(bf16_lo(a) + bf16_lo(b), bf16_hi(a) + bf16_hi(b));
}

__device__ __forceinline__ uint4 cat(uint2 lo, uint2 hi) { return make_uint4(lo.x, lo.y, hi.x, hi.y); }

template <class Cf>
__global__ __launch_bounds__(512, 1) void wave_fwd_kernel(Geom g, const bf16_t *__restrict__ x,
                                                          const uint8_t *__restrict__ pack,
                                                          bf16_t *__restrict__ y, bf16_t *__restrict__ attn)
{
    using W = WaveFwdCfg<Cf>;
    constexpr int C = Cf::C, D = Cf::D, CG = Cf::CG, HG = Cf::HG, HEADS = Cf::HEADS;
    constexpr int OT = Cf::OT, NSTEP = Cf::NSTEP, NDLT = Cf::NDLT;
    constexpr int M = 8, NTHREADS = W::NTHREADS;
    static_assert(Cf::ET == 1 && D + 4 <= 16, "one 16-row tile per head with four spare rows");
    static_assert(CG % 2 == 0 && D % 2 == 0 && C % 4 == 0 && HEADS % 2 == 0, "dword-granular loads and stores");

    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, q = lane >> 4;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int s = g.shift;
    const int cn = l16 & 7, rsub = l16 >> 3;
    const int per_img = g.nwi * g.nwj;
    // Global tensors as buffers (see make_buf).  This lane's four channels 4q .. 4q+3 of a 16-wide
    // head tile are one 8-byte access; the pairs at or beyond D belong to the next head (or lie
    // past the tensor): they are masked to zero when read and left out when written.
    const uint32_t tbytes = (uint32_t)g.T * (2u * C);
    const buf_t xbuf = make_buf(x, tbytes), ybuf = make_buf(y, tbytes), abuf = make_buf(attn, attn ? tbytes : 0u);
    const bool lo_ok = 4 * q < D, hi_ok = 4 * q + 2 < D;
    const uint32_t m_lo = lo_ok ? 0xffffffffu : 0u, m_hi = hi_ok ? 0xffffffffu : 0u;
    const uint32_t c8 = 8u * q;

    // x of a window in head-padded operand order: tile t, head hd: channels hd*D + 4q .. 4q+3 of
    // token 16t + l16; and the mask inputs (1, r, c, r*c) of the tokens, r / c = "past the wrap in
    // the last window row / column"
    uint32_t tok[4]; // byte offset of the token's row (2*T*C fits 32 bits, checked on the host)
    uint2 xh[HEADS][4], feat[4];
    auto load_window = [&](int win) {
        const int b = win / per_img;
        const int wr = win - b * per_img;
        const int wi = wr / g.nwj, wj = wr - wi * g.nwj;
        const bool lastrow = s > 0 && wi == g.nwi - 1, lastcol = s > 0 && wj == g.nwj - 1;
        int sj = wj * M + cn + s;
        if (sj >= g.W) sj -= g.W;
        const float c = (lastcol && cn >= M - s) ? 1.f : 0.f;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            int si = wi * M + 2 * t + rsub + s;
            if (si >= g.H) si -= g.H;
            tok[t] = (uint32_t)((((b * g.H + si) * g.W) + sj) * C) * 2u;
            const float r = (lastrow && 2 * t + rsub >= M - s) ? 1.f : 0.f;
            feat[t] = make_uint2(pack_bf16x2(1.f, r), pack_bf16x2(c, r * c));
        }
    };
    // the x slice of one group: a group is fetched while the previous one is being computed
    auto load_group = [&, xbuf](int gi) {
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int hl = 0; hl < HG; ++hl) {
                const int hd = gi * HG + hl;
                xh[hd][t] = bload64(xbuf, tok[t] + c8 + 2u * (hd * D), 0u);
                xh[hd][t].x &= m_lo;
                xh[hd][t].y &= m_hi;
            }
    };

    int win = wv * gridDim.x + blockIdx.x;
    if (win < g.nW) { // in flight during the set-up
        load_window(win);
        load_group(0);
    }

    // ---- set-up: packed weights, bias operands and linear biases into LDS (unrolled, so that the
    // loads of a thread are all in flight together); the workgroups start at different offsets
    // so that they do not all ask for the same cache lines at once ----
    {
        constexpr int N16 = (int)(W::COPY_BYTES / 16);
        const int rot = (int)((blockIdx.x * 5u) % (unsigned)W::COPY_IT);
#pragma unroll
        for (int k = 0; k < W::COPY_IT; ++k) {
            int kk = k + rot;
            if (kk >= W::COPY_IT) kk -= W::COPY_IT;
            const int i = kk * NTHREADS + tid;
            if (i < N16) reinterpret_cast<uint4 *>(lds + W::OFF_COPY)[i] = reinterpret_cast<const uint4 *>(pack)[i];
        }
        if (tid < C)
            reinterpret_cast<uint4 *>(lds + W::OFF_BIAS)[tid] = reinterpret_cast<const uint4 *>(pack + Cf::P_BIAS)[tid];
    }
    __syncthreads();

    // constant operands: identity rows (upper half of the score MFMA's A operand) and the column of
    // ones that spreads -max over a score tile
    const uint2 ident = make_uint2((4 * q == l16 ? 0x3F80u : 0u) | (4 * q + 1 == l16 ? 0x3F800000u : 0u),
                                   (4 * q + 2 == l16 ? 0x3F80u : 0u) | (4 * q + 3 == l16 ? 0x3F800000u : 0u));
    const uint2 ones0 = make_uint2(q == 0 ? 0x3F80u : 0u, 0u);
    const f32x4 zero4 = f32x4{0.f, 0.f, 0.f, 0.f};

    for (; win < g.nW; win += W::NWAVES * gridDim.x) {
        // The LDS contents do not change from window to window, but their reads must stay inside
        // this loop (hoisted out, the weights of all heads would sit in registers): the offset of
        // LDS is made opaque once per window.
        uint32_t lds0 = 0;
        asm volatile("" : "+v"(lds0));
        const uint4 *wqh = reinterpret_cast<const uint4 *>(lds + lds0 + W::OFF_WQH);
        const uint4 *wp2 = reinterpret_cast<const uint4 *>(lds + lds0 + W::OFF_WP2);
        const uint2 *bfr = reinterpret_cast<const uint2 *>(lds + lds0 + W::OFF_BF);
        const float *bqkv = reinterpret_cast<const float *>(lds + lds0 + W::OFF_BIAS);
        const float *bproj = bqkv + 3 * C;
        uint2 Ob[HEADS][4];
#pragma unroll
        for (int hd = 0; hd < HEADS; ++hd) {
            const int gi = hd / HG, hl = hd % HG;
            if (hl == 0 && gi > 0 && g.cascade) { // Eq. 8: the previous group's output joins this group's input
#pragma unroll
                for (int hlp = 0; hlp < HG; ++hlp)
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        const uint2 prev = Ob[(gi > 0 ? gi - 1 : 0) * HG + hlp][t];
                        uint2 &xv = xh[gi * HG + hlp][t];
                        xv.x = add_bf16x2(xv.x, prev.x);
                        xv.y = add_bf16x2(xv.y, prev.y);
                    }
            }
            // ---- Q^T, K^T (rows = head features, then the mask terms) and V (rows = tokens) ----
            uint4 wqf[3][NSTEP];
#pragma unroll
            for (int t3 = 0; t3 < 3; ++t3)
#pragma unroll
                for (int st = 0; st < NSTEP; ++st) wqf[t3][st] = wqh[((hd * 3 + t3) * NSTEP + st) * 64 + lane];
            f32x4 bq, bk;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int e = 4 * q + j;
                bq[j] = e < D ? bqkv[gi * 3 * CG + hl * D + e] * kLog2e : 0.f;
                bk[j] = e < D ? bqkv[gi * 3 * CG + CG + hl * D + e] : 0.f;
            }
            // column D of V is one: row D of the PV product is the sum of the probabilities
            const float bvs = l16 < D ? bqkv[gi * 3 * CG + 2 * CG + hl * D + l16] : (l16 == D ? 1.f : 0.f);
            uint2 Qb[4], Kb[4], Vb[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                f32x4 qT = bq, kT = bk, vv = f32x4{bvs, bvs, bvs, bvs};
#pragma unroll
                for (int st = 0; st < HG / 2; ++st) {
                    const uint4 xb = cat(xh[gi * HG + 2 * st][t], xh[gi * HG + 2 * st + 1][t]);
                    qT = mma32(wqf[0][st], xb, qT);
                    kT = mma32(wqf[1][st], xb, kT);
                    vv = mma32(xb, wqf[2][st], vv);
                }
                {
                    const uint2 xodd = HG % 2 ? xh[gi * HG + HG - 1][t] : make_uint2(0u, 0u);
                    const uint4 xb = cat(xodd, feat[t]);
                    qT = mma32(wqf[0][NSTEP - 1], xb, qT);
                    kT = mma32(wqf[1][NSTEP - 1], xb, kT);
                    if (HG % 2) vv = mma32(xb, wqf[2][NSTEP - 1], vv);
                }
                Qb[t] = pack_bf16x4(qT);
                Kb[t] = pack_bf16x4(kT);
                Vb[t] = pack_bf16x4(vv);
            }
            uint2 bfh[NDLT];
#pragma unroll
            for (int dlt = 0; dlt < NDLT; ++dlt) bfh[dlt] = bfr[(hd * NDLT + dlt) * 64 + lane];
            if (hl == HG - 1 && gi + 1 < Cf::G) load_group(gi + 1); // this group's x is consumed

#pragma unroll
            for (int nt = 0; nt < 4; ++nt) {
                // S^T tiles (base-2 units): rows = keys 16kt+4q+j, column = query 16nt+l16
                f32x4 st[4];
#pragma unroll
                for (int kt = 0; kt < 4; ++kt) st[kt] = mma16(ident, bfh[nt - kt + 3], zero4);
#pragma unroll
                for (int kt = 0; kt < 4; ++kt) st[kt] = mma16(Kb[kt], Qb[nt], st[kt]);
                float mx = fmaxf(fmaxf(st[0][0], st[0][1]), fmaxf(st[0][2], st[0][3]));
#pragma unroll
                for (int kt = 1; kt < 4; ++kt)
#pragma unroll
                    for (int j = 0; j < 4; j += 2) mx = fmaxf(fmaxf(mx, st[kt][j]), st[kt][j + 1]);
                mx = qgroup_max(mx);
                const uint2 negmx = make_uint2(q == 0 ? pack_bf16x2(-mx, 0.f) : 0u, 0u);
                uint2 Pb[4];
#pragma unroll
                for (int kt = 0; kt < 4; ++kt) {
                    st[kt] = mma16(ones0, negmx, st[kt]); // every row of the tile: - max (to bf16)
#pragma unroll
                    for (int j = 0; j < 4; ++j) st[kt][j] = __builtin_amdgcn_exp2f(st[kt][j]);
                    Pb[kt] = pack_bf16x4(st[kt]);
                }
                // O^T = V^T P^T: rows = head features (row D = sum of the probabilities)
                f32x4 oT = mma32(cat(Vb[0], Vb[1]), cat(Pb[0], Pb[1]), zero4);
                oT = mma32(cat(Vb[2], Vb[3]), cat(Pb[2], Pb[3]), oT);
                oT *= __builtin_amdgcn_rcpf(qgroup_broadcast<D / 4>(oT[D % 4]));
                Ob[hd][nt] = pack_bf16x4(oT);
            }
            if (attn && hl == HG - 1) { // the group's output, kept for the backward: its heads together,
                                        // so that the pieces of a row reach memory as whole cache lines
                if (hi_ok) {
#pragma unroll
                    for (int nt = 0; nt < 4; ++nt)
#pragma unroll
                        for (int h2 = gi * HG; h2 <= hd; ++h2) bstore64(abuf, tok[nt] + c8 + 2u * (h2 * D), 0u, Ob[h2][nt]);
                } else if (lo_ok) {
#pragma unroll
                    for (int nt = 0; nt < 4; ++nt)
#pragma unroll
                        for (int h2 = gi * HG; h2 <= hd; ++h2) bstore32(abuf, tok[nt] + c8 + 2u * (h2 * D), 0u, Ob[h2][nt].x);
                }
            }
        }

        // ---- Y^T = Wproj A^T + b: rows = output channels, column = token ----
#pragma unroll
        for (int ot = 0; ot < OT; ++ot) {
            uint4 wpf[HEADS / 2];
#pragma unroll
            for (int pr = 0; pr < HEADS / 2; ++pr) wpf[pr] = wp2[(ot * (HEADS / 2) + pr) * 64 + lane];
            f32x4 bp;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int o = 16 * ot + 4 * q + j;
                bp[j] = o < C ? bproj[o] : 0.f;
            }
            const int o0 = 16 * ot + 4 * q;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                f32x4 acc = bp;
#pragma unroll
                for (int pr = 0; pr < HEADS / 2; ++pr) acc = mma32(wpf[pr], cat(Ob[2 * pr][t], Ob[2 * pr + 1][t]), acc);
                if (o0 < C) bstore64(ybuf, tok[t] + c8 + 32u * ot, 0u, pack_bf16x4(acc));
            }
        }
        if (win + W::NWAVES * (int)gridDim.x < g.nW) {
            load_window(win + W::NWAVES * gridDim.x);
            load_group(0);
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
        // (the lane index as this window's address arithmetic sees it: opaque, so that per-lane LDS and memory
        // addresses are computed where they are used instead of being kept, and spilled, across windows)
        int lane_w = threadIdx.x & 63;
        asm volatile("" : "+v"(lane_w));
        const int lane = lane_w, l16 = lane & 15, q = lane >> 4;
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
        uint4 xf[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            uint32_t xv[4], av[4];
#pragma unroll
            for (int dw = 0; dw < 4; ++dw) {
                const int c = 32 * ks + 8 * q + 2 * dw;
                xv[dw] = c < CG ? xrow[c >> 1] : 0u;
                av[dw] = (casc && c < CG) ? arow[c >> 1] : 0u;
            }
            // Eq. 8: F = x slice + previous group's output, rounded to bf16 once (the operand of the products below)
            xf[ks] = casc ? make_uint4(add_bf16x2(xv[0], av[0]), add_bf16x2(xv[1], av[1]), add_bf16x2(xv[2], av[2]),
                                       add_bf16x2(xv[3], av[3]))
                          : make_uint4(xv[0], xv[1], xv[2], xv[3]);
        }

#pragma unroll 1
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
        if (hipError_t ea = allow_dynamic_lds(reinterpret_cast<const void *>(kern), A::LDS_BYTES); ea != hipSuccess) return ea;
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
                   bf16_t *attn, void *ws, int training, hipStream_t s)
{
    uint8_t *pack = static_cast<uint8_t *>(ws);
    {
        constexpr int entries =
            (Cf::N_WQH + Cf::N_WP2 + Cf::N_BF + Cf::N_WQ + Cf::N_WPT + Cf::N_WQT + Cf::N_WPK) * 64 + 4 * Cf::C;
        constexpr int wide_entries = (Cf::N_WQW + Cf::N_WPW + Cf::N_WQX + Cf::N_WQN) * 64 + Cf::HEADS * Cf::TBW_PITCH;
        const int blocks = (entries + 255) / 256;
        const bool wide = Cf::SPLIT && wide_fwd_supported(g);
        KernelTimer kt(K_PACK_FWD, s);
        hipLaunchKernelGGL(pack_params_kernel<Cf>, dim3(blocks + (wide ? (wide_entries + 255) / 256 : 0)), dim3(256), 0, s,
                           w_qkv, b_qkv, w_proj, b_proj, table, pack, wide ? blocks : -1);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if constexpr (Cf::SPLIT) {
        if (wide_fwd_supported(g)) { // 8x8 windows: the whole layer in one launch
            return launch_wide_fwd(g, x, pack, y, attn, training, s);
        }
        if (!attn) return hipErrorInvalidValue;
        e = g.M == 16 ? launch_attn_chunks<Cf, 16>(g, x, pack, table, attn, s)
                      : launch_attn_chunks<Cf, 8>(g, x, pack, table, attn, s);
        if (e != hipSuccess) return e;
        constexpr size_t lds = (size_t)Cf::N_WPK * 1024 + 4 * Cf::C;
        auto kern = proj_gemm_kernel<Cf>;
        if (hipError_t ea = allow_dynamic_lds(reinterpret_cast<const void *>(kern), lds); ea != hipSuccess) return ea;
        long ntile = (g.T + 63) / 64;
        int grid = 2 * device_cu_count();
        if (grid > ntile) grid = (int)ntile;
        KernelTimer kt(K_PROJ_GEMM, s);
        hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, s, g.T, attn, pack, y);
        return hipGetLastError();
    } else {
        using W = WaveFwdCfg<Cf>;
        static_assert(W::LDS_BYTES <= 160 * 1024, "LDS budget");
        auto kern = wave_fwd_kernel<Cf>;
        if (hipError_t ea = allow_dynamic_lds(reinterpret_cast<const void *>(kern), W::LDS_BYTES); ea != hipSuccess) return ea;
        // one window per wave: spread the windows over the compute units before filling a workgroup
        int grid = device_cu_count();
        if (grid > g.nW) grid = g.nW;
        KernelTimer kt(K_FUSED_FWD, s);
        hipLaunchKernelGGL(kern, dim3(grid), dim3(64 * W::NWAVES), W::LDS_BYTES, s, g, x, pack, y, attn);
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
    if (g.C == C_ && g.heads == H_ && g.groups == G_)                                                  \
        return FusedCfg<C_, H_, G_>::SPLIT || (g.M == 8 && (long)g.T * g.C < (1L << 31)); /* 32-bit offsets */
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
                            bf16_t *y, bf16_t *attn_out, void *pack, int training, hipStream_t s)
{
#define X(C_, H_, G_)                                                  \
    if (g.C == C_ && g.heads == H_ && g.groups == G_)                  \
        return run_fwd<FusedCfg<C_, H_, G_>>(g, x, w_qkv, b_qkv, w_proj, b_proj, table, y, attn_out, pack, training, s);
    GSWA_FUSED_SHAPES(X)
#undef X
    return hipErrorInvalidValue;
}

} // namespace gswa
