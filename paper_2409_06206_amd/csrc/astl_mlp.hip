// Fused kernels of the MLP half of a layer (Sec. "Agile Swin Transformer Block", Eq. 5, with the
// skip connection of Eq. 4 in the prologue) for narrow bf16 layers.
//
// A wavefront owns 16 tokens from the first load to the last store.  Lane (tok = lane & 15,
// q = lane >> 4) holds, of its token, the channels 16 ct + 4 q + i (ct < CT, i < 4): one 8-byte
// access per ct, and exactly the channels the C layout of a transposed product hands the lane.
// Both matrix products are taken transposed (features x tokens), weights as the A operand from
// fragments in LDS, activations as the B operand straight from registers:
//   pre^T = W1 LN(x1)^T   reduces over channels: the lane's 8 k-slots of step s are the channels
//                         16 (2s) + 4q + 0..3 and 16 (2s+1) + 4q + 0..3 (the weight fragments use
//                         the same order), so the normalised row packs into B without any exchange;
//   y^T   = W2 h^T        reduces over hidden features: h^T comes out of the first product in C
//                         layout (features 16 ft + 4q + i of token tok) and two such tiles pack
//                         into one B operand the same way.
// LayerNorm's gamma is folded into the W1 fragments and beta into the bias (b1 + W1 beta), so the
// first product takes the plain normalised row.
#include "astl_mlp.h"
#include "mfma.h"
#include "staged_kernels.h"
#include "profile.h"

namespace gswa {

namespace {

constexpr int kMlpThreads = 256;
constexpr int kMlpWaves = kMlpThreads / 64;
constexpr int kFwdThreads = 512; // the forward needs few registers: eight wavefronts share one copy of the weights
constexpr int kFwdWaves = kFwdThreads / 64;

// (Gaussian CDF and density `gauss`: staged_kernels.h)
__device__ __forceinline__ float bf(const bf16_t *p, long i) { return __uint_as_float((uint32_t)p[i].bits << 16); }

// channel (or hidden feature) a lane's k-slot j of step s stands for
__device__ __forceinline__ int slot_index(int s, int q, int j) { return 16 * (2 * s + (j >> 2)) + 4 * q + (j & 3); }

// Fragments of a weight matrix as the A operand: tile `mt` of 16 output rows, k-step `s`;
// get(m, k) returns the entry for output row m and reduction index k (zero outside the matrix).
template <typename F>
__device__ __forceinline__ void build_frags(uint4 *dst, int mtiles, int ksteps, F get)
{
    uint16_t *d16 = reinterpret_cast<uint16_t *>(dst);
    const int total = mtiles * ksteps * 512;
    for (int e = blockIdx.x * kMlpThreads + threadIdx.x; e < total; e += gridDim.x * kMlpThreads) {
        const int j = e & 7, l = (e >> 3) & 63, fr = e >> 9;
        const int s = fr % ksteps, mt = fr / ksteps;
        d16[e] = f32_to_bf16_bits(get(16 * mt + (l & 15), slot_index(s, l >> 4, j)));
    }
}

struct MlpArgs {
    long rows;
    int C, Hd;
    float eps;
    const bf16_t *x, *a;       // forward: x1 = x + a;  backward: x = x1, a = dy
    const bf16_t *ln_w, *ln_b, *w_fc1, *b_fc1, *w_fc2, *b_fc2;
    bf16_t *x1, *y;            // forward outputs;  backward: y = dx1
    const bf16_t *nxt_w, *nxt_b; // forward, optional: gamma, beta of the LayerNorm that will read y next ...
    bf16_t *xn_out;            // ... and where its output goes (null: not wanted)
    float *zero;               // backward: fp32 array the kernel clears for a later launch of the caller's
    long nzero;
    // backward, optional: pend_src holds `pend_reps` copies, `pend_stride` floats apart, of two vectors
    // [pend_n | pend_n] that the call before this one left unsummed (LayerNorm-1 gradients of the layer after
    // this one in a sequence); they are summed to pend_w / pend_b before `zero` (often the same array) is cleared
    const float *pend_src;
    float *pend_w, *pend_b;
    int pend_n, pend_reps, pend_accumulate;
    long pend_stride;
    void *pack;                // weights in fragment order, written by the pack kernel
    float *part;               // backward: one pair of partial weight-gradient matrices per workgroup
};

// Layout of the packed weights (uint4 units, then floats), shared by the three kernels:
//   w1f [FT][KSC][64]  W1 diag(gamma)  rows = features, k = channels      (both passes)
//   w2f [CT][KSF][64]  W2              rows = channels, k = features      (forward)
//   w2t [FT][KSC][64]  W2^T            rows = features, k = channels      (backward)
//   w1t [CT][KSF][64]  W1^T            rows = channels, k = features      (backward)
//   b1s [FT * 16]      b1 + W1 beta;   b2s [CT * 16]
template <int KSC, int KSF> struct PackLayout {
    static constexpr int CT = 2 * KSC, FT = 2 * KSF;
    static constexpr int frag = FT * KSC * 64; // uint4 per weight matrix (CT * KSF * 64 is the same number)
    static constexpr int w1f = 0, w2f = frag, w2t = 2 * frag, w1t = 3 * frag;
    static constexpr int floats_at = 4 * frag; // in uint4 units
    static constexpr int nfloats = (FT + CT) * 16;
    static constexpr size_t bytes = (size_t)4 * frag * 16 + (size_t)nfloats * 4;
};

// Once per forward call: the MLP's weights into MFMA fragment order (gamma and beta of LN_2 folded
// into the first layer); the backward pass reads the same pack.
template <int KSC, int KSF>
__global__ __launch_bounds__(kMlpThreads) void astl_mlp_pack_kernel(MlpArgs a)
{
    using L = PackLayout<KSC, KSF>;
    constexpr int CT = L::CT, FT = L::FT;
    uint4 *pk = static_cast<uint4 *>(a.pack);
    const int C = a.C, Hd = a.Hd;
    build_frags(pk + L::w1f, FT, KSC, [&](int f, int c) { return (f < Hd && c < C) ? bf(a.w_fc1, (long)f * C + c) * bf(a.ln_w, c) : 0.f; });
    build_frags(pk + L::w2f, CT, KSF, [&](int c, int f) { return (f < Hd && c < C) ? bf(a.w_fc2, (long)c * Hd + f) : 0.f; });
    build_frags(pk + L::w2t, FT, KSC, [&](int f, int c) { return (f < Hd && c < C) ? bf(a.w_fc2, (long)c * Hd + f) : 0.f; });
    build_frags(pk + L::w1t, CT, KSF, [&](int c, int f) { return (f < Hd && c < C) ? bf(a.w_fc1, (long)f * C + c) : 0.f; });
    float *fl = reinterpret_cast<float *>(pk + L::floats_at);
    // b1 + W1 beta: one wavefront per feature
    const int lane = threadIdx.x & 63;
    for (int f = blockIdx.x * kMlpWaves + (threadIdx.x >> 6); f < FT * 16; f += gridDim.x * kMlpWaves) {
        float s = 0.f;
        if (f < Hd)
            for (int c = lane; c < C; c += 64) s += bf(a.w_fc1, (long)f * C + c) * bf(a.ln_b, c);
#pragma unroll
        for (int m = 1; m < 64; m <<= 1) s += __shfl_xor(s, m);
        if (lane == 0) fl[f] = f < Hd ? s + bf(a.b_fc1, f) : 0.f;
    }
    for (int c = blockIdx.x * kMlpThreads + threadIdx.x; c < CT * 16; c += gridDim.x * kMlpThreads)
        fl[FT * 16 + c] = c < C ? bf(a.b_fc2, c) : 0.f;
}

// copies `n` uint4 from the pack into LDS
__device__ __forceinline__ void stage(uint4 *dst, const uint4 *src, int n)
{
    for (int e = threadIdx.x; e < n; e += blockDim.x) dst[e] = src[e];
}

template <int CT>
struct Row {
    float v[CT][4];
};

// the same row as loaded: four bf16 per channel tile
template <int CT>
struct Raw {
    uint2 v[CT];
};

// 8-byte loads of a token's channels in the lane's ownership pattern (zero beyond C or the rows)
template <int CT>
__device__ __forceinline__ void load_raw(const bf16_t *base, long t, bool ok, int C, int q, Raw<CT> &r)
{
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
        const int c = 16 * ct + 4 * q;
        r.v[ct] = make_uint2(0u, 0u);
        if (ok && c < C) r.v[ct] = *reinterpret_cast<const uint2 *>(base + t * C + c);
    }
}

template <int CT>
__device__ __forceinline__ void widen(const Raw<CT> &u, Row<CT> &r)
{
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
        r.v[ct][0] = bf16_lo(u.v[ct].x); r.v[ct][1] = bf16_hi(u.v[ct].x);
        r.v[ct][2] = bf16_lo(u.v[ct].y); r.v[ct][3] = bf16_hi(u.v[ct].y);
    }
}

template <int CT>
__device__ __forceinline__ void load_own(const bf16_t *base, long t, bool ok, int C, int q, Row<CT> &r)
{
    Raw<CT> u;
    load_raw<CT>(base, t, ok, C, q, u);
    widen<CT>(u, r);
}

template <int CT>
__device__ __forceinline__ void store_own(bf16_t *base, long t, bool ok, int C, int q, const Row<CT> &r)
{
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
        const int c = 16 * ct + 4 * q;
        if (ok && c < C)
            *reinterpret_cast<uint2 *>(base + t * C + c) =
                make_uint2(pack_bf16x2(r.v[ct][0], r.v[ct][1]), pack_bf16x2(r.v[ct][2], r.v[ct][3]));
    }
}

// normalised row (zero in the padding channels) and 1/sqrt(var + eps)
template <int CT>
__device__ __forceinline__ float normalise(const Row<CT> &u, int C, int q, float eps, Row<CT> &xh)
{
    float s = 0.f;
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
        for (int i = 0; i < 4; ++i) s += u.v[ct][i];
    const float mean = qgroup_sum(s) / (float)C;
    float v = 0.f;
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
        const bool in = 16 * ct + 4 * q < C;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            xh.v[ct][i] = in ? u.v[ct][i] - mean : 0.f;
            v += xh.v[ct][i] * xh.v[ct][i];
        }
    }
    const float rstd = rsqrtf(qgroup_sum(v) / (float)C + eps);
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
        for (int i = 0; i < 4; ++i) xh.v[ct][i] *= rstd;
    return rstd;
}

// B operand of k-step s from a row in the ownership pattern
template <int CT>
__device__ __forceinline__ uint4 b_frag(const Row<CT> &r, int s)
{
    return make_uint4(pack_bf16x2(r.v[2 * s][0], r.v[2 * s][1]), pack_bf16x2(r.v[2 * s][2], r.v[2 * s][3]),
                      pack_bf16x2(r.v[2 * s + 1][0], r.v[2 * s + 1][1]), pack_bf16x2(r.v[2 * s + 1][2], r.v[2 * s + 1][3]));
}

template <int KSC, int KSF>
__global__ __launch_bounds__(kFwdThreads) void astl_mlp_fwd_kernel(MlpArgs a)
{
    constexpr int CT = 2 * KSC, FT = 2 * KSF;
    extern __shared__ __align__(16) unsigned char smem[];
    uint4 *w1f = reinterpret_cast<uint4 *>(smem);  // [FT][KSC][64]  W1 diag(gamma)
    uint4 *w2f = w1f + FT * KSC * 64;              // [CT][KSF][64]  W2
    float *b1s = reinterpret_cast<float *>(w2f + CT * KSF * 64); // [FT * 16]  b1 + W1 beta
    float *b2s = b1s + FT * 16;                    // [CT * 16]
    const int C = a.C;
    {
        using L = PackLayout<KSC, KSF>;
        const uint4 *pk = static_cast<const uint4 *>(a.pack);
        stage(w1f, pk + L::w1f, 2 * L::frag);                        // w1f and w2f lie back to back
        stage(reinterpret_cast<uint4 *>(b1s), pk + L::floats_at, L::nfloats / 4);
    }
    __syncthreads();

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, tok = lane & 15, q = lane >> 4;
    Row<CT> ngam, nbet;
    if (a.xn_out) {
        load_own<CT>(a.nxt_w, 0, true, C, q, ngam);
        load_own<CT>(a.nxt_b, 0, true, C, q, nbet);
    }
    const long ntiles = (a.rows + 15) / 16;
    const long tstep = (long)gridDim.x * kFwdWaves;
    long tile = (long)blockIdx.x * kFwdWaves + wave;
    Raw<CT> rx, ra;
    load_raw<CT>(a.x, tile * 16 + tok, tile * 16 + tok < a.rows, C, q, rx);
    load_raw<CT>(a.a, tile * 16 + tok, tile * 16 + tok < a.rows, C, q, ra);
    for (; tile < ntiles; tile += tstep) {
        const long t = tile * 16 + tok;
        const bool ok = t < a.rows;
        // (an offset the compiler cannot see through keeps the fragment reads inside the loop
        // instead of pinning every fragment in registers for the whole kernel)
        int ln = lane;
        asm volatile("" : "+v"(ln));
        Row<CT> x1, av, xh;
        widen<CT>(rx, x1);
        widen<CT>(ra, av);
        {   // the next tile's rows are on their way while this one is computed
            const long tn = t + tstep * 16;
            load_raw<CT>(a.x, tn, tn < a.rows, C, q, rx);
            load_raw<CT>(a.a, tn, tn < a.rows, C, q, ra);
        }
        // Eq. 4's skip; the stored (rounded) sum is what LN_2 sees here and in the backward pass
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t u = pack_bf16x2(x1.v[ct][i] + av.v[ct][i], 0.f);
                x1.v[ct][i] = bf16_lo(u);
            }
        store_own<CT>(a.x1, t, ok, C, q, x1);
        normalise<CT>(x1, C, q, a.eps, xh);
        uint4 bx[KSC];
#pragma unroll
        for (int s = 0; s < KSC; ++s) bx[s] = b_frag<CT>(xh, s);
        // hidden layer, transposed: features 16 ft + 4q + i of token tok
        uint2 hp[FT];
#pragma unroll
        for (int ft = 0; ft < FT; ++ft) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < KSC; ++s) acc = mma32(w1f[(ft * KSC + s) * 64 + ln], bx[s], acc);
            const float4 b1 = *reinterpret_cast<const float4 *>(b1s + 16 * ft + (ln >> 4) * 4);
            const float pre[4] = {acc[0] + b1.x, acc[1] + b1.y, acc[2] + b1.z, acc[3] + b1.w};
            float h[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float Phi, phi;
                gauss(pre[i], Phi, phi);
                h[i] = pre[i] * Phi;
            }
            hp[ft] = make_uint2(pack_bf16x2(h[0], h[1]), pack_bf16x2(h[2], h[3]));
        }
        // second layer and the skip of Eq. 5
        Row<CT> y;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < KSF; ++s)
                acc = mma32(w2f[(ct * KSF + s) * 64 + ln],
                            make_uint4(hp[2 * s].x, hp[2 * s].y, hp[2 * s + 1].x, hp[2 * s + 1].y), acc);
            const float4 b2 = *reinterpret_cast<const float4 *>(b2s + 16 * ct + (ln >> 4) * 4);
            y.v[ct][0] = acc[0] + b2.x + x1.v[ct][0];
            y.v[ct][1] = acc[1] + b2.y + x1.v[ct][1];
            y.v[ct][2] = acc[2] + b2.z + x1.v[ct][2];
            y.v[ct][3] = acc[3] + b2.w + x1.v[ct][3];
        }
        store_own<CT>(a.y, t, ok, C, q, y);
        if (a.xn_out) {
            // the LayerNorm of the layer that follows, taken of y as stored
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)
#pragma unroll
                for (int i = 0; i < 4; ++i) y.v[ct][i] = bf16_lo(pack_bf16x2(y.v[ct][i], 0.f));
            Row<CT> yh;
            normalise<CT>(y, C, q, a.eps, yh);
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)
#pragma unroll
                for (int i = 0; i < 4; ++i) yh.v[ct][i] = yh.v[ct][i] * ngam.v[ct][i] + nbet.v[ct][i];
            store_own<CT>(a.xn_out, t, ok, C, q, yh);
        }
    }
}

// Adjoint of Eq. 5.  A workgroup of eight wavefronts takes 128 tokens per round, 16 per wave.
// Phase 1, per wave: recompute LN_2(x1), the pre-activation and the hidden layer exactly as the
// forward does, dh^T = W2^T dy^T, through the GELU, dLN^T = W1^T dpre^T, LayerNorm's adjoint and
// the skip -> dx1.  The four matrices the weight gradients need go to LDS feature-major with the
// round's tokens contiguous: h^T, dpre^T, LN_2(x1)^T and dy^T.
// Phase 2, after a barrier: the products that reduce over tokens,
//   M1[f][c] = sum_t dpre[t][f] LN_2(x1)[t][c] = d Wfc1,      M2[f][c] = sum_t h[t][f] dy[t][c] = d Wfc2^T,
// wave w owning feature tile w of both (8 accumulator tiles, kept in registers over all rounds);
// the bias gradients are the same staged rows multiplied by a tile of ones (d bfc1 = row sums of
// dpre^T, d bfc2 = row sums of dy^T).  Every workgroup stores its sums; a second kernel adds them up.
constexpr int kBwdThreads = 512;
constexpr int kBwdWaves = kBwdThreads / 64;
constexpr int kTokPitch = 272;   // bytes per staged row: 128 tokens of bf16 + 16 (conflict-free 16-byte reads)

template <int KSC, int KSF> struct BwdLds {
    static constexpr int CT = 2 * KSC, FT = 2 * KSF;
    static constexpr size_t frags = (size_t)3 * FT * KSC * 1024;
    static constexpr size_t b1 = frags;
    static constexpr size_t red = b1 + (size_t)FT * 16 * 4;
    static constexpr size_t hT = red + (size_t)kBwdWaves * 2 * CT * 16 * 4;
    static constexpr size_t dpT = hT + (size_t)FT * 16 * kTokPitch;
    static constexpr size_t xnT = dpT + (size_t)FT * 16 * kTokPitch;
    static constexpr size_t dyT = xnT + (size_t)CT * 16 * kTokPitch;
    static constexpr size_t bytes = dyT + (size_t)CT * 16 * kTokPitch;
};

// four values of rows r0 .. r0+3, column `col`, into a staged matrix
__device__ __forceinline__ void stage4(unsigned char *m, int r0, int col, uint2 packed)
{
    uint16_t *p = reinterpret_cast<uint16_t *>(m + (size_t)r0 * kTokPitch) + col;
    p[0] = (uint16_t)packed.x;
    p[kTokPitch / 2] = (uint16_t)(packed.x >> 16);
    p[2 * (kTokPitch / 2)] = (uint16_t)packed.y;
    p[3 * (kTokPitch / 2)] = (uint16_t)(packed.y >> 16);
}

template <int KSC, int KSF>
__global__ __launch_bounds__(kBwdThreads) void astl_mlp_bwd_kernel(MlpArgs a)
{
    constexpr int CT = 2 * KSC, FT = 2 * KSF;
    using S = BwdLds<KSC, KSF>;
    extern __shared__ __align__(16) unsigned char smem[];
    uint4 *w1f = reinterpret_cast<uint4 *>(smem);  // [FT][KSC][64]  W1 diag(gamma): rows = features, k = channels
    uint4 *w2t = w1f + FT * KSC * 64;              // [FT][KSC][64]  W2^T:            rows = features, k = channels
    uint4 *w1t = w2t + FT * KSC * 64;              // [CT][KSF][64]  W1^T:            rows = channels, k = features
    float *b1s = reinterpret_cast<float *>(smem + S::b1);   // [FT * 16]
    float *red = reinterpret_cast<float *>(smem + S::red);  // [kBwdWaves][2][CT * 16]
    unsigned char *hT = smem + S::hT, *dpT = smem + S::dpT, *xnT = smem + S::xnT, *dyT = smem + S::dyT;
    const int C = a.C, Hd = a.Hd;
    {
        using L = PackLayout<KSC, KSF>;
        const uint4 *pk = static_cast<const uint4 *>(a.pack);
        stage(w1f, pk + L::w1f, L::frag);
        stage(w2t, pk + L::w2t, 2 * L::frag);                        // w2t and w1t lie back to back
        stage(reinterpret_cast<uint4 *>(b1s), pk + L::floats_at, FT * 16 / 4);
    }
    if (a.pend_w) {
        // the first workgroup sums the pending copies in a fixed order, then clears the array
        if (blockIdx.x == 0) {
            for (int e = threadIdx.x; e < 2 * a.pend_n; e += kBwdThreads) {
                float sum = 0.f;
                for (int r = 0; r < a.pend_reps; ++r) sum += a.pend_src[(long)r * a.pend_stride + e];
                float *dst = e < a.pend_n ? a.pend_w + e : a.pend_b + (e - a.pend_n);
                *dst = a.pend_accumulate ? *dst + sum : sum;
            }
            __syncthreads();
            for (long i = threadIdx.x; i < a.nzero; i += kBwdThreads) a.zero[i] = 0.f;
        }
    } else {
        for (long i = (long)blockIdx.x * kBwdThreads + threadIdx.x; i < a.nzero; i += (long)gridDim.x * kBwdThreads)
            a.zero[i] = 0.f;
    }
    __syncthreads();

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, tok = lane & 15, q = lane >> 4;
    Row<CT> gam, bet, acc_g, acc_b;
    load_own<CT>(a.ln_w, 0, true, C, q, gam);
    load_own<CT>(a.ln_b, 0, true, C, q, bet);
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
        for (int i = 0; i < 4; ++i) acc_g.v[ct][i] = acc_b.v[ct][i] = 0.f;
    f32x4 m1[CT], m2[CT], sb1 = {0.f, 0.f, 0.f, 0.f}, sb2 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) m1[ct] = m2[ct] = f32x4{0.f, 0.f, 0.f, 0.f};

    const long ntiles = (a.rows + 15) / 16;
    const long rounds = (ntiles + (long)gridDim.x * kBwdWaves - 1) / ((long)gridDim.x * kBwdWaves);
    long tile = (long)blockIdx.x * rounds * kBwdWaves + wave;   // a workgroup's tiles are consecutive
    Raw<CT> rx, rd;
    load_raw<CT>(a.x, tile * 16 + tok, tile * 16 + tok < a.rows, C, q, rx);
    load_raw<CT>(a.a, tile * 16 + tok, tile * 16 + tok < a.rows, C, q, rd);
    for (long r = 0; r < rounds; ++r, tile += kBwdWaves) {
        const long t = tile * 16 + tok;
        const bool ok = t < a.rows;
        int ln = lane; // (kept opaque so that the fragment reads stay inside the loop)
        asm volatile("" : "+v"(ln));
        const int col = 16 * wave + tok;   // this token's column in the staged matrices
        Row<CT> x1, dy, xh;
        widen<CT>(rx, x1);
        widen<CT>(rd, dy);
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) stage4(dyT, 16 * ct + 4 * (ln >> 4), col, rd.v[ct]);
        {   // the next round's rows are on their way while this one is computed
            const long tn = t + kBwdWaves * 16;
            load_raw<CT>(a.x, tn, tn < a.rows, C, q, rx);
            load_raw<CT>(a.a, tn, tn < a.rows, C, q, rd);
        }
        const float rstd = normalise<CT>(x1, C, q, a.eps, xh);
        uint4 bx[KSC], bd[KSC];
#pragma unroll
        for (int s = 0; s < KSC; ++s) {
            bx[s] = b_frag<CT>(xh, s);
            bd[s] = b_frag<CT>(dy, s);
        }
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {   // LN_2(x1)
            float xn[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) xn[i] = xh.v[ct][i] * gam.v[ct][i] + bet.v[ct][i];
            stage4(xnT, 16 * ct + 4 * (ln >> 4), col, make_uint2(pack_bf16x2(xn[0], xn[1]), pack_bf16x2(xn[2], xn[3])));
        }
        uint2 dp[FT];
#pragma unroll
        for (int ft = 0; ft < FT; ++ft) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f}, dh = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < KSC; ++s) {
                acc = mma32(w1f[(ft * KSC + s) * 64 + ln], bx[s], acc);
                dh = mma32(w2t[(ft * KSC + s) * 64 + ln], bd[s], dh);
            }
            const float4 b1 = *reinterpret_cast<const float4 *>(b1s + 16 * ft + (ln >> 4) * 4);
            const float pre[4] = {acc[0] + b1.x, acc[1] + b1.y, acc[2] + b1.z, acc[3] + b1.w};
            float h[4], dpre[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float Phi, phi;
                gauss(pre[i], Phi, phi);
                h[i] = pre[i] * Phi;
                dpre[i] = dh[i] * (Phi + pre[i] * phi);
            }
            dp[ft] = make_uint2(pack_bf16x2(dpre[0], dpre[1]), pack_bf16x2(dpre[2], dpre[3]));
            stage4(hT, 16 * ft + 4 * (ln >> 4), col, make_uint2(pack_bf16x2(h[0], h[1]), pack_bf16x2(h[2], h[3])));
            stage4(dpT, 16 * ft + 4 * (ln >> 4), col, dp[ft]);
        }
        // gradient at LN_2's output, then through the LayerNorm, plus the skip of Eq. 5
        Row<CT> dxh;
        float s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
            f32x4 dn = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < KSF; ++s)
                dn = mma32(w1t[(ct * KSF + s) * 64 + ln],
                           make_uint4(dp[2 * s].x, dp[2 * s].y, dp[2 * s + 1].x, dp[2 * s + 1].y), dn);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float d = ok ? dn[i] : 0.f;
                acc_g.v[ct][i] += d * xh.v[ct][i];
                acc_b.v[ct][i] += d;
                dxh.v[ct][i] = d * gam.v[ct][i];
                s1 += dxh.v[ct][i];
                s2 += dxh.v[ct][i] * xh.v[ct][i];
            }
        }
        s1 = qgroup_sum(s1) / (float)C;
        s2 = qgroup_sum(s2) / (float)C;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                dxh.v[ct][i] = rstd * (dxh.v[ct][i] - s1 - xh.v[ct][i] * s2) + dy.v[ct][i];
        store_own<CT>(a.y, t, ok, C, q, dxh);

        __syncthreads();
        // phase 2: the round's 128 tokens in four k-steps of 32
        if (wave < FT) {
            const int m = ln & 15, kq = ln >> 4;
            const uint4 ones = make_uint4(0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u); // bf16 1.0
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const size_t koff = (size_t)(32 * ks + 8 * kq) * 2;
                const uint4 a1 = *reinterpret_cast<const uint4 *>(dpT + (size_t)(16 * wave + m) * kTokPitch + koff);
                const uint4 a2 = *reinterpret_cast<const uint4 *>(hT + (size_t)(16 * wave + m) * kTokPitch + koff);
                // bias sums: a product with ones puts the sum over tokens of every row in each column
                sb1 = mma32(a1, ones, sb1);
                if (wave < CT)
                    sb2 = mma32(*reinterpret_cast<const uint4 *>(dyT + (size_t)(16 * wave + m) * kTokPitch + koff), ones, sb2);
#pragma unroll
                for (int ct = 0; ct < CT; ++ct) {
                    const uint4 b1v = *reinterpret_cast<const uint4 *>(xnT + (size_t)(16 * ct + m) * kTokPitch + koff);
                    const uint4 b2v = *reinterpret_cast<const uint4 *>(dyT + (size_t)(16 * ct + m) * kTokPitch + koff);
                    m1[ct] = mma32(a1, b1v, m1[ct]);
                    m2[ct] = mma32(a2, b2v, m2[ct]);
                }
            }
        }
        __syncthreads();
    }

    // the workgroup's sums: part[workgroup] = [2][FT*16][CT*16] matrices, [2][CT*16] LayerNorm sums,
    // [FT*16] and [CT*16] bias sums; lane holds column m, rows 4q + i
    constexpr int kMats = 2 * FT * 16 * CT * 16;
    float *part = a.part + (size_t)blockIdx.x * (kMats + 2 * CT * 16 + FT * 16 + CT * 16);
    if (wave < FT) {
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const size_t at = (size_t)(16 * wave + 4 * q + i) * (CT * 16) + 16 * ct + tok;
                part[at] = m1[ct][i];
                part[(size_t)FT * 16 * CT * 16 + at] = m2[ct][i];
            }
        if (tok == 0) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                part[kMats + 2 * CT * 16 + 16 * wave + 4 * q + i] = sb1[i];
                if (wave < CT) part[kMats + 2 * CT * 16 + FT * 16 + 16 * wave + 4 * q + i] = sb2[i];
            }
        }
    }

    // d gamma, d beta: over the 16 tokens of the wave, then the waves of the workgroup
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float g = acc_g.v[ct][i], b = acc_b.v[ct][i];
#pragma unroll
            for (int m = 1; m < 16; m <<= 1) {
                g += __shfl_xor(g, m);
                b += __shfl_xor(b, m);
            }
            if (tok == 0) {
                red[(wave * 2 + 0) * CT * 16 + 16 * ct + 4 * q + i] = g;
                red[(wave * 2 + 1) * CT * 16 + 16 * ct + 4 * q + i] = b;
            }
        }
    __syncthreads();
    for (int e = threadIdx.x; e < 2 * CT * 16; e += kBwdThreads) {
        const int which = e / (CT * 16), c = e % (CT * 16);
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < kBwdWaves; ++w) s += red[(w * 2 + which) * CT * 16 + c];
        part[kMats + e] = c < C ? s : 0.f;
    }
    (void)Hd;
}

__global__ __launch_bounds__(256) void astl_mlp_reduce_kernel(MlpReduceArgs a) { astl_mlp_reduce_block(a, (int)blockIdx.x); }

unsigned fwd_blocks(long rows)
{
    const long tiles = (rows + 15) / 16;
    long b = (tiles + kFwdWaves - 1) / kFwdWaves;
    if (b > 512) b = 512;
    return (unsigned)(b < 1 ? 1 : b);
}

template <int KSC, int KSF> size_t fwd_lds()
{
    return (size_t)(2 * KSF * KSC + 2 * KSC * KSF) * 1024 + (size_t)(2 * KSF + 2 * KSC) * 16 * sizeof(float);
}
constexpr int kBwdMaxBlocks = 256; // one workgroup per compute unit (its LDS need allows no second one)
unsigned bwd_blocks(long rows)
{
    const long tiles = (rows + 15) / 16;
    long b = (tiles + kBwdWaves - 1) / kBwdWaves;
    if (b > kBwdMaxBlocks) b = kBwdMaxBlocks;
    return (unsigned)(b < 1 ? 1 : b);
}

template <int KSC, int KSF> hipError_t launch_fwd_t(const MlpArgs &a, hipStream_t s)
{
    {
        KernelTimer kt(K_MLP_PACK, s);
        hipLaunchKernelGGL((astl_mlp_pack_kernel<KSC, KSF>), dim3(32), dim3(kMlpThreads), 0, s, a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    auto kern = astl_mlp_fwd_kernel<KSC, KSF>;
    const size_t lds = fwd_lds<KSC, KSF>();
    if (hipError_t ea = allow_dynamic_lds(reinterpret_cast<const void *>(kern), lds); ea != hipSuccess) return ea;
    KernelTimer kt(K_MLP_FWD, s);
    hipLaunchKernelGGL(kern, dim3(fwd_blocks(a.rows)), dim3(kFwdThreads), lds, s, a);
    return hipGetLastError();
}

template <int KSC, int KSF> hipError_t launch_bwd_t(const MlpArgs &a, hipStream_t s)
{
    auto kern = astl_mlp_bwd_kernel<KSC, KSF>;
    const size_t lds = BwdLds<KSC, KSF>::bytes;
    if (hipError_t ea = allow_dynamic_lds(reinterpret_cast<const void *>(kern), lds); ea != hipSuccess) return ea;
    KernelTimer kt(K_MLP_BWD, s);
    hipLaunchKernelGGL(kern, dim3(bwd_blocks(a.rows)), dim3(kBwdThreads), lds, s, a);
    return hipGetLastError();
}

size_t align256(size_t b) { return (b + 255) & ~size_t(255); }

} // namespace

bool astl_mlp_supported(int C, int hidden)
{
    return C >= 4 && C <= 64 && C % 4 == 0 && hidden >= 4 && hidden <= 128 && hidden % 4 == 0;
}

hipError_t launch_astl_mlp_fwd(long rows, int C, int hidden, float eps, const bf16_t *x, const bf16_t *a,
                               const bf16_t *ln_w, const bf16_t *ln_b, const bf16_t *w_fc1, const bf16_t *b_fc1,
                               const bf16_t *w_fc2, const bf16_t *b_fc2, bf16_t *x1, bf16_t *y, void *pack,
                               const bf16_t *next_ln_w, const bf16_t *next_ln_b, bf16_t *next_ln_out, hipStream_t s)
{
    if (!astl_mlp_supported(C, hidden)) return hipErrorInvalidValue;
    MlpArgs m{};
    m.rows = rows; m.C = C; m.Hd = hidden; m.eps = eps;
    m.x = x; m.a = a; m.ln_w = ln_w; m.ln_b = ln_b; m.w_fc1 = w_fc1; m.b_fc1 = b_fc1; m.w_fc2 = w_fc2; m.b_fc2 = b_fc2;
    m.x1 = x1; m.y = y; m.pack = pack;
    if (next_ln_out && next_ln_w && next_ln_b) {
        m.nxt_w = next_ln_w; m.nxt_b = next_ln_b; m.xn_out = next_ln_out;
    }
    if (C <= 32) return hidden <= 64 ? launch_fwd_t<1, 2>(m, s) : launch_fwd_t<1, 4>(m, s);
    return hidden <= 64 ? launch_fwd_t<2, 2>(m, s) : launch_fwd_t<2, 4>(m, s);
}

size_t astl_mlp_pack_bytes() { return align256(PackLayout<2, 4>::bytes); }

bool astl_mlp_bwd_supported(int C, int hidden) { return astl_mlp_supported(C, hidden); }

size_t astl_mlp_bwd_ws_bytes(long rows, int C, int hidden)
{
    (void)rows;
    const size_t ct16 = C <= 32 ? 32 : 64, ft16 = hidden <= 64 ? 64 : 128;
    return align256((size_t)kBwdMaxBlocks * (2 * ft16 * ct16 + 3 * ct16 + ft16) * sizeof(float));
}

hipError_t launch_astl_mlp_bwd(long rows, int C, int hidden, float eps, const bf16_t *x1, const bf16_t *dy,
                               const bf16_t *ln_w, const bf16_t *ln_b, const bf16_t *w_fc1, const bf16_t *b_fc1,
                               const bf16_t *w_fc2, bf16_t *dx1, float *dw_fc1, float *db_fc1, float *dw_fc2,
                               float *db_fc2, float *dln_w, float *dln_b, int accumulate, float *zero, long nzero,
                               const void *pack, void *ws, MlpReduceArgs *deferred, const MlpPending *pending,
                               hipStream_t s)
{
    if (!astl_mlp_bwd_supported(C, hidden)) return hipErrorInvalidValue;
    MlpArgs m{};
    m.rows = rows; m.C = C; m.Hd = hidden; m.eps = eps;
    m.x = x1; m.a = dy; m.ln_w = ln_w; m.ln_b = ln_b; m.w_fc1 = w_fc1; m.b_fc1 = b_fc1; m.w_fc2 = w_fc2;
    m.y = dx1;
    m.zero = zero; m.nzero = zero ? nzero : 0;
    if (pending && pending->w) {
        m.pend_src = pending->src; m.pend_w = pending->w; m.pend_b = pending->b; m.pend_n = pending->n; m.pend_reps = pending->reps;
        m.pend_stride = pending->stride; m.pend_accumulate = pending->accumulate;
    }
    m.pack = const_cast<void *>(pack);
    m.part = static_cast<float *>(ws);
    hipError_t e;
    if (C <= 32) e = hidden <= 64 ? launch_bwd_t<1, 2>(m, s) : launch_bwd_t<1, 4>(m, s);
    else e = hidden <= 64 ? launch_bwd_t<2, 2>(m, s) : launch_bwd_t<2, 4>(m, s);
    if (e != hipSuccess) return e;
    MlpReduceArgs r{};
    r.part = m.part; r.nparts = (int)bwd_blocks(rows);
    r.rows = hidden <= 64 ? 64 : 128; r.cols = C <= 32 ? 32 : 64;
    r.C = C; r.Hd = hidden;
    r.accumulate = accumulate;
    r.dw1 = dw_fc1; r.db1 = db_fc1; r.dw2 = dw_fc2; r.db2 = db_fc2; r.dln_w = dln_w; r.dln_b = dln_b;
    if (deferred) {   // the caller runs the sum inside a launch of its own
        *deferred = r;
        return hipSuccess;
    }
    const unsigned blocks = astl_mlp_reduce_blocks(r);
    KernelTimer kt(K_MLP_REDUCE, s);
    hipLaunchKernelGGL(astl_mlp_reduce_kernel, dim3(blocks), dim3(256), 0, s, r);
    return hipGetLastError();
}

} // namespace gswa
