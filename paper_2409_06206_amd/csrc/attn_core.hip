// Attention core of the staged path on the matrix cores (bf16 storage): one workgroup per
// (window, head), one wavefront per 16-token tile of the window, so a window of N = 16*NT tokens
// takes NT wavefronts.  Serves the shapes the fused kernels are not built for: 12 x 12 windows
// (Sec. "Experimental Settings") and queries/keys narrower than the values (Sec. "Parameter
// Allocation").  Scores, probabilities and their gradients live in registers; q, k, v and dO of
// the (window, head) are staged once in LDS, token-major and channel-major, so that every MFMA
// operand is one 8-byte LDS read.
//
// Orientation (see mfma.h): a wave computes S^T tiles [keys x its 16 queries]; packed to bf16
// they are the B operand of the products that reduce over keys (O^T = V^T P^T, dQ^T = K^T dS^T).
// The products of the backward that reduce over queries (dV, dK) need the other orientation, so
// every wave also recomputes S for its own 16 KEYS against all queries, from the row statistics
// (log-sum-exp, delta = sum_m P dP) the query role left in LDS.  LDS float atomics are slow here
// (a wave's ds_add_f32 takes ~170 clocks), so the bias-table gradient is folded from a bf16 copy
// of dS in LDS instead.
#include "staged_kernels.h"
#include "mfma.h"

namespace gswa {

namespace {

constexpr float kLog2e = 1.4426950408889634f;

template <int NT_, int ET_, int KQ_> struct CoreCfg {
    static constexpr int NT = NT_, ET = ET_, KQ = KQ_; // token tiles; 16-channel tiles of v and of q/k
    static constexpr int N = 16 * NT, NTHREADS = 64 * NT;
    // pitches in bf16 elements; the 4 spare elements keep the 16 rows of an operand read on
    // different banks
    static constexpr int LK = 16 * KQ + 4, LV = 16 * ET + 4, LT = N + 4;
};

__host__ __device__ inline int table_floats(int M)
{
    const int n = (2 * M - 1) * (2 * M - 1);
    return (n + 3) & ~3;
}

template <class Cf> size_t fwd_lds_bytes(int M)
{
    return (size_t)4 * table_floats(M) + 8 * Cf::N + 2 * ((size_t)Cf::N * Cf::LK + 16 * Cf::ET * Cf::LT);
}
template <class Cf> constexpr size_t bwd_operand_bytes()
{
    return 2 * ((size_t)2 * Cf::N * Cf::LK + 2 * 16 * Cf::KQ * Cf::LT + 2 * Cf::N * Cf::LV + 16 * Cf::ET * Cf::LT);
}
template <class Cf> size_t bwd_lds_bytes(int M)
{
    // the operand arrays are reused at the end for the N x N matrix of dS (bf16, pitch LT)
    const size_t ops = bwd_operand_bytes<Cf>(), ds = (size_t)2 * Cf::N * Cf::LT;
    return (size_t)4 * table_floats(M) + 16 * Cf::N + (ops > ds ? ops : ds);
}

__device__ __forceinline__ uint2 lds_frag(const uint16_t *p) { return *reinterpret_cast<const uint2 *>(p); }

// Token map, key offsets and the head's bias table (in base-2 units) into LDS.
// koff[n] = (r*(2M-1) + c) | region << 16 for token n = r*M + c: the table index of a (query, key)
// pair is koff(query) - koff(key) + (M-1)*(2M-1) + (M-1).
template <int N, int NTHREADS>
__device__ __forceinline__ void stage_geometry(const Geom &g, int w, int hd, const bf16_t *table, float *tb,
                                               int *koff, int *tok, int tid)
{
    constexpr int M = N == 64 ? 8 : 12, nt1 = 2 * M - 1, ntbl = nt1 * nt1; // N = M * M is 64 or 144
    for (int n = tid; n < N; n += NTHREADS) {
        int reg;
        tok[n] = (int)window_token(g, w, n, reg);
        const int r = n / M, c = n - r * M;
        koff[n] = (r * nt1 + c) | (reg << 16);
    }
    for (int e = tid; e < ntbl; e += NTHREADS) tb[e] = to_f32(table[(long)e * g.heads + hd]) * kLog2e;
}

// ---------------------------------------------------------------------------------------
// forward: O = softmax(q k^T / sqrt(dq) + bias + mask) v for one (window, head)
// ---------------------------------------------------------------------------------------
template <int NT, int ET, int KQ>
__global__ __launch_bounds__(64 * NT) void attn_core_fwd_kernel(Geom g, int grp, const bf16_t *__restrict__ qkv,
                                                               const bf16_t *__restrict__ table,
                                                               bf16_t *__restrict__ attn_out)
{
    using Cf = CoreCfg<NT, ET, KQ>;
    constexpr int N = Cf::N, NTH = Cf::NTHREADS, LK = Cf::LK, LT = Cf::LT;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    constexpr int M = NT == 4 ? 8 : 12, nt1 = 2 * M - 1; // N = M * M is 64 or 144
    float *tb = reinterpret_cast<float *>(lds);
    int *koff = reinterpret_cast<int *>(lds + 4 * table_floats(M));
    int *tok = koff + N;
    uint16_t *Ks = reinterpret_cast<uint16_t *>(tok + N); // [N][LK]   k rows
    uint16_t *VT = Ks + N * LK;                           // [16*ET][LT] v, channel-major

    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, q = lane >> 4;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int w = blockIdx.x, hl = blockIdx.y, hd = grp * g.hg + hl;
    const int d = g.d, dq = g.dq, Rg = g.Rg, Qg = g.Qg;
    const uint16_t *qkv16 = reinterpret_cast<const uint16_t *>(qkv);

    stage_geometry<N, NTH>(g, w, hd, table, tb, koff, tok, tid);
    __syncthreads();
    // k rows and v of the window (zero beyond the head's channels); a thread's loads are all
    // issued before its first LDS store (N*16 elements per channel tile = 4 per thread)
    {
        uint16_t vk[4 * KQ], vv[4 * ET];
#pragma unroll
        for (int i = 0; i < 4 * KQ; ++i) {
            const int e = tid + i * NTH, n = e / (16 * KQ), c = e - n * (16 * KQ);
            vk[i] = c < dq ? qkv16[(long)tok[n] * Rg + Qg + hl * dq + c] : (uint16_t)0;
        }
#pragma unroll
        for (int i = 0; i < 4 * ET; ++i) {
            const int e = tid + i * NTH, n = e / (16 * ET), c = e - n * (16 * ET);
            vv[i] = c < d ? qkv16[(long)tok[n] * Rg + 2 * Qg + hl * d + c] : (uint16_t)0;
        }
#pragma unroll
        for (int i = 0; i < 4 * KQ; ++i) {
            const int e = tid + i * NTH, n = e / (16 * KQ), c = e - n * (16 * KQ);
            Ks[n * LK + c] = vk[i];
        }
#pragma unroll
        for (int i = 0; i < 4 * ET; ++i) {
            const int e = tid + i * NTH, n = e / (16 * ET), c = e - n * (16 * ET);
            VT[c * LT + n] = vv[i];
        }
    }
    // this lane's query as a B operand: column l16 = query, k-slots = channels 16ks + 4q + j
    const int nq = 16 * wv + l16;
    uint2 qf[KQ];
    {
        const long base = (long)tok[nq] * Rg + hl * dq;
#pragma unroll
        for (int ks = 0; ks < KQ; ++ks) {
            uint32_t v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int c = 16 * ks + 4 * q + j;
                v[j] = c < dq ? (uint32_t)qkv16[base + c] : 0u;
            }
            qf[ks] = make_uint2(v[0] | v[1] << 16, v[2] | v[3] << 16);
        }
    }
    const int kq = koff[nq];
    const int qo = (kq & 0xffff) + (M - 1) * nt1 + (M - 1), regn = kq >> 16;
    __syncthreads();

    const float sc2 = kLog2e / sqrtf((float)dq), maskv = -100.0f * kLog2e;
    f32x4 st[NT];
    float mx = -INFINITY;
#pragma unroll
    for (int kt = 0; kt < NT; ++kt) {
        f32x4 a = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KQ; ++ks) a = mma16(lds_frag(&Ks[(16 * kt + l16) * LK + 16 * ks + 4 * q]), qf[ks], a);
        const int4 ko = *reinterpret_cast<const int4 *>(&koff[16 * kt + 4 * q]);
        const int kk[4] = {ko.x, ko.y, ko.z, ko.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float s = fmaf(a[j], sc2, tb[qo - (kk[j] & 0xffff)]);
            s += (kk[j] >> 16) != regn ? maskv : 0.f;
            a[j] = s;
            mx = fmaxf(mx, s);
        }
        st[kt] = a;
    }
    mx = qgroup_max(mx);
    float sum = 0.f;
#pragma unroll
    for (int kt = 0; kt < NT; ++kt)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float p = __builtin_amdgcn_exp2f(st[kt][j] - mx);
            st[kt][j] = p;
            sum += p;
        }
    sum = qgroup_sum(sum);
    f32x4 o[ET];
#pragma unroll
    for (int et = 0; et < ET; ++et) o[et] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kt = 0; kt < NT; ++kt) {
        const uint2 pb = pack_bf16x4(st[kt]);
#pragma unroll
        for (int et = 0; et < ET; ++et) o[et] = mma16(lds_frag(&VT[(16 * et + l16) * LT + 16 * kt + 4 * q]), pb, o[et]);
    }
    const float inv = 1.0f / sum;
    uint16_t *out16 = reinterpret_cast<uint16_t *>(attn_out) + (long)tok[nq] * g.C + hd * d;
#pragma unroll
    for (int et = 0; et < ET; ++et)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = 16 * et + 4 * q + j;
            if (c < d) out16[c] = f32_to_bf16_bits(o[et][j] * inv);
        }
}

// ---------------------------------------------------------------------------------------
// backward: dq, dk, dv and the bias-table gradient of one (window, head).  On entry the v part of
// dqkv holds dO; the kernel replaces q|k|v parts of its own tokens and head by dq|dk|dv.
// ---------------------------------------------------------------------------------------
template <int NT, int ET, int KQ>
__global__ __launch_bounds__(64 * NT) void attn_core_bwd_kernel(Geom g, int grp, const bf16_t *__restrict__ qkv,
                                                               bf16_t *dqkv, const bf16_t *__restrict__ table,
                                                               float *__restrict__ tpart)
{
    using Cf = CoreCfg<NT, ET, KQ>;
    constexpr int N = Cf::N, NTH = Cf::NTHREADS, LK = Cf::LK, LV = Cf::LV, LT = Cf::LT;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    constexpr int M = NT == 4 ? 8 : 12, nt1 = 2 * M - 1; // N = M * M is 64 or 144
    const int tf = table_floats(M);
    float *tb = reinterpret_cast<float *>(lds);
    int *koff = reinterpret_cast<int *>(tb + tf);
    int *tok = koff + N;
    float *lse = reinterpret_cast<float *>(tok + N);       // base-2 log-sum-exp of every query row
    float *dlt = lse + N;                                  // sum_m P dP of every query row
    uint16_t *Qs = reinterpret_cast<uint16_t *>(dlt + N);  // [N][LK]
    uint16_t *Ks = Qs + N * LK;                            // [N][LK]
    uint16_t *QT = Ks + N * LK;                            // [16*KQ][LT]
    uint16_t *KT = QT + 16 * KQ * LT;                      // [16*KQ][LT]
    uint16_t *Vs = KT + 16 * KQ * LT;                      // [N][LV]
    uint16_t *Os = Vs + N * LV;                            // [N][LV]  dO rows
    uint16_t *OT = Os + N * LV;                            // [16*ET][LT]  dO, channel-major

    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, q = lane >> 4;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int w = blockIdx.x, hl = blockIdx.y, hd = grp * g.hg + hl;
    const int d = g.d, dq = g.dq, Rg = g.Rg, Qg = g.Qg;
    const uint16_t *qkv16 = reinterpret_cast<const uint16_t *>(qkv);
    uint16_t *dqkv16 = reinterpret_cast<uint16_t *>(dqkv);

    stage_geometry<N, NTH>(g, w, hd, table, tb, koff, tok, tid);
    __syncthreads();
    // q, k, v, dO of the window, token-major and channel-major (zero beyond the head's channels);
    // a thread's loads are all issued before its first LDS store
    {
        uint16_t vq[4 * KQ], vk[4 * KQ], vv[4 * ET], vo[4 * ET];
#pragma unroll
        for (int i = 0; i < 4 * KQ; ++i) {
            const int e = tid + i * NTH, n = e / (16 * KQ), c = e - n * (16 * KQ);
            const long base = (long)tok[n] * Rg + hl * dq + c;
            vq[i] = c < dq ? qkv16[base] : (uint16_t)0;
            vk[i] = c < dq ? qkv16[base + Qg] : (uint16_t)0;
        }
#pragma unroll
        for (int i = 0; i < 4 * ET; ++i) {
            const int e = tid + i * NTH, n = e / (16 * ET), c = e - n * (16 * ET);
            const long base = (long)tok[n] * Rg + 2 * Qg + hl * d + c;
            vv[i] = c < d ? qkv16[base] : (uint16_t)0;
            vo[i] = c < d ? dqkv16[base] : (uint16_t)0;
        }
#pragma unroll
        for (int i = 0; i < 4 * KQ; ++i) {
            const int e = tid + i * NTH, n = e / (16 * KQ), c = e - n * (16 * KQ);
            Qs[n * LK + c] = vq[i];
            QT[c * LT + n] = vq[i];
            Ks[n * LK + c] = vk[i];
            KT[c * LT + n] = vk[i];
        }
#pragma unroll
        for (int i = 0; i < 4 * ET; ++i) {
            const int e = tid + i * NTH, n = e / (16 * ET), c = e - n * (16 * ET);
            Vs[n * LV + c] = vv[i];
            Os[n * LV + c] = vo[i];
            OT[c * LT + n] = vo[i];
        }
    }
    __syncthreads();

    const int own = 16 * wv + l16; // this lane's query (first role) and key (second role)
    const int kown = koff[own];
    const int cst = (M - 1) * nt1 + (M - 1);
    const int off_own = kown & 0xffff, reg_own = kown >> 16;
    const float scale = 1.0f / sqrtf((float)dq);
    const float sc2 = scale * kLog2e, maskv = -100.0f * kLog2e;

    uint2 dsb[NT]; // dS^T of the wave's queries (bf16), kept for the bias-table gradient at the end

    // ---- query role: statistics of the wave's 16 queries, dQ ----
    {
        uint2 qf[KQ], of[ET];
#pragma unroll
        for (int ks = 0; ks < KQ; ++ks) qf[ks] = lds_frag(&Qs[own * LK + 16 * ks + 4 * q]);
#pragma unroll
        for (int es = 0; es < ET; ++es) of[es] = lds_frag(&Os[own * LV + 16 * es + 4 * q]);
        const int qo = off_own + cst;
        f32x4 st[NT], dpt[NT];
        float mx = -INFINITY;
#pragma unroll
        for (int kt = 0; kt < NT; ++kt) {
            f32x4 a = {0.f, 0.f, 0.f, 0.f}, b = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KQ; ++ks) a = mma16(lds_frag(&Ks[(16 * kt + l16) * LK + 16 * ks + 4 * q]), qf[ks], a);
#pragma unroll
            for (int es = 0; es < ET; ++es) b = mma16(lds_frag(&Vs[(16 * kt + l16) * LV + 16 * es + 4 * q]), of[es], b);
            const int4 ko = *reinterpret_cast<const int4 *>(&koff[16 * kt + 4 * q]);
            const int kk[4] = {ko.x, ko.y, ko.z, ko.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float s = fmaf(a[j], sc2, tb[qo - (kk[j] & 0xffff)]);
                s += (kk[j] >> 16) != reg_own ? maskv : 0.f;
                a[j] = s;
                mx = fmaxf(mx, s);
            }
            st[kt] = a;
            dpt[kt] = b;
        }
        mx = qgroup_max(mx);
        float sum = 0.f;
#pragma unroll
        for (int kt = 0; kt < NT; ++kt)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float p = __builtin_amdgcn_exp2f(st[kt][j] - mx);
                st[kt][j] = p;
                sum += p;
            }
        sum = qgroup_sum(sum);
        const float inv = 1.0f / sum;
        float dl = 0.f;
#pragma unroll
        for (int kt = 0; kt < NT; ++kt)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                st[kt][j] *= inv;
                dl = fmaf(st[kt][j], dpt[kt][j], dl);
            }
        dl = qgroup_sum(dl);
        if (q == 0) {
            lse[own] = mx + __builtin_amdgcn_logf(sum); // v_log_f32 is the base-2 logarithm
            dlt[own] = dl;
        }
        f32x4 dqt[KQ];
#pragma unroll
        for (int ks = 0; ks < KQ; ++ks) dqt[ks] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kt = 0; kt < NT; ++kt) {
            f32x4 ds;
#pragma unroll
            for (int j = 0; j < 4; ++j) ds[j] = st[kt][j] * (dpt[kt][j] - dl);
            dsb[kt] = pack_bf16x4(ds);
#pragma unroll
            for (int ks = 0; ks < KQ; ++ks)
                dqt[ks] = mma16(lds_frag(&KT[(16 * ks + l16) * LT + 16 * kt + 4 * q]), dsb[kt], dqt[ks]);
        }
        uint16_t *o16 = dqkv16 + (long)tok[own] * Rg + hl * dq;
#pragma unroll
        for (int ks = 0; ks < KQ; ++ks)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int c = 16 * ks + 4 * q + j;
                if (c < dq) o16[c] = f32_to_bf16_bits(dqt[ks][j] * scale);
            }
    }
    __syncthreads();

    // ---- key role: dK and dV of the wave's 16 keys over all queries ----
    {
        uint2 kf[KQ], vf[ET];
#pragma unroll
        for (int ks = 0; ks < KQ; ++ks) kf[ks] = lds_frag(&Ks[own * LK + 16 * ks + 4 * q]);
#pragma unroll
        for (int es = 0; es < ET; ++es) vf[es] = lds_frag(&Vs[own * LV + 16 * es + 4 * q]);
        f32x4 dvt[ET], dkt[KQ];
#pragma unroll
        for (int es = 0; es < ET; ++es) dvt[es] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KQ; ++ks) dkt[ks] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            f32x4 a = {0.f, 0.f, 0.f, 0.f}, b = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KQ; ++ks) a = mma16(lds_frag(&Qs[(16 * nt + l16) * LK + 16 * ks + 4 * q]), kf[ks], a);
#pragma unroll
            for (int es = 0; es < ET; ++es) b = mma16(lds_frag(&Os[(16 * nt + l16) * LV + 16 * es + 4 * q]), vf[es], b);
            const int4 ko = *reinterpret_cast<const int4 *>(&koff[16 * nt + 4 * q]);
            const float4 ls = *reinterpret_cast<const float4 *>(&lse[16 * nt + 4 * q]);
            const float4 dl = *reinterpret_cast<const float4 *>(&dlt[16 * nt + 4 * q]);
            const int kk[4] = {ko.x, ko.y, ko.z, ko.w};
            const float lsv[4] = {ls.x, ls.y, ls.z, ls.w}, dlv[4] = {dl.x, dl.y, dl.z, dl.w};
            f32x4 p, ds;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float s = fmaf(a[j], sc2, tb[(kk[j] & 0xffff) + cst - off_own]);
                s += (kk[j] >> 16) != reg_own ? maskv : 0.f;
                p[j] = __builtin_amdgcn_exp2f(s - lsv[j]);
                ds[j] = p[j] * (b[j] - dlv[j]);
            }
            const uint2 pb = pack_bf16x4(p), dsk = pack_bf16x4(ds);
#pragma unroll
            for (int es = 0; es < ET; ++es)
                dvt[es] = mma16(lds_frag(&OT[(16 * es + l16) * LT + 16 * nt + 4 * q]), pb, dvt[es]);
#pragma unroll
            for (int ks = 0; ks < KQ; ++ks)
                dkt[ks] = mma16(lds_frag(&QT[(16 * ks + l16) * LT + 16 * nt + 4 * q]), dsk, dkt[ks]);
        }
        uint16_t *o16 = dqkv16 + (long)tok[own] * Rg;
#pragma unroll
        for (int ks = 0; ks < KQ; ++ks)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int c = 16 * ks + 4 * q + j;
                if (c < dq) o16[Qg + hl * dq + c] = f32_to_bf16_bits(dkt[ks][j] * scale);
            }
#pragma unroll
        for (int es = 0; es < ET; ++es)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int c = 16 * es + 4 * q + j;
                if (c < d) o16[2 * Qg + hl * d + c] = f32_to_bf16_bits(dvt[es][j]);
            }
    }
    // ---- bias-table gradient of this (window, head): dS of the whole window goes to LDS as an N x N
    // matrix (over the operand arrays, which nobody reads any more) and is summed per coordinate
    // offset (dr, dc) = query - key ----
    __syncthreads();
    uint16_t *DS = Qs; // [N][LT]: row = query, column = key
#pragma unroll
    for (int kt = 0; kt < NT; ++kt) *reinterpret_cast<uint2 *>(&DS[own * LT + 16 * kt + 4 * q]) = dsb[kt];
    __syncthreads();
    // Four threads share the offsets (dr0, dc0), (dr0 - M, dc0), (dr0, dc0 - M), (dr0 - M, dc0 - M),
    // 0 <= dr0, dc0 < M: for every query (rn, cn) exactly one of them has its key inside the window,
    // key = ((rn - dr0) mod M, (cn - dc0) mod M), so the four entries together take M*M terms, and
    // each thread sums a quarter of the query rows (the workgroup has 4 * M*M threads).
    {
        const int grp4 = tid >> 2, part = tid & 3;
        const int dr0 = grp4 / M, dc0 = grp4 - dr0 * M;
        float a00 = 0.f, a01 = 0.f, a10 = 0.f, a11 = 0.f; // [row wrapped][column wrapped]
        for (int rn = part * (M / 4); rn < (part + 1) * (M / 4); ++rn) {
            const bool wr = rn < dr0;
            const int rm = rn - dr0 + (wr ? M : 0);
            const uint16_t *row = &DS[(rn * M) * LT + rm * M];
            float s0 = 0.f, s1 = 0.f;
            for (int cn = 0; cn < M; ++cn) {
                const bool wc = cn < dc0;
                const float v = __uint_as_float((uint32_t)row[cn * LT + cn - dc0 + (wc ? M : 0)] << 16);
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
        // thread `part` of the four adds entry `part`
        const int e00 = (dr0 + M - 1) * nt1 + dc0 + M - 1;
        const float val = part == 0 ? a00 : part == 1 ? a01 : part == 2 ? a10 : a11;
        const int e = e00 - ((part & 1) ? M : 0) - ((part & 2) ? M * nt1 : 0);
        const bool ok = !((part & 1) && dc0 == 0) && !((part & 2) && dr0 == 0);
        // every entry of this (window, head) is written exactly once: no atomics, no zero fill
        if (ok) tpart[((long)w * ((2 * M - 1) * (2 * M - 1)) + e) * g.heads + hd] = val;
    }
}

template <int NT, int ET, int KQ>
hipError_t launch_fwd(const Geom &g, int grp, const bf16_t *qkv, const bf16_t *table, bf16_t *attn_out,
                      hipStream_t s)
{
    using Cf = CoreCfg<NT, ET, KQ>;
    const size_t lds = fwd_lds_bytes<Cf>(g.M);
    auto kern = attn_core_fwd_kernel<NT, ET, KQ>;
    if (hipError_t ea = allow_dynamic_lds(reinterpret_cast<const void *>(kern), lds); ea != hipSuccess) return ea;
    KernelTimer kt(K_ATTN_CORE_FWD, s);
    hipLaunchKernelGGL(kern, dim3(g.nW, g.hg), dim3(Cf::NTHREADS), lds, s, g, grp, qkv, table, attn_out);
    return hipGetLastError();
}

template <int NT, int ET, int KQ>
hipError_t launch_bwd(const Geom &g, int grp, const bf16_t *qkv, bf16_t *dqkv, const bf16_t *table,
                      float *tpart, hipStream_t s)
{
    using Cf = CoreCfg<NT, ET, KQ>;
    const size_t lds = bwd_lds_bytes<Cf>(g.M);
    auto kern = attn_core_bwd_kernel<NT, ET, KQ>;
    if (hipError_t ea = allow_dynamic_lds(reinterpret_cast<const void *>(kern), lds); ea != hipSuccess) return ea;
    KernelTimer kt(K_ATTN_CORE_BWD, s);
    hipLaunchKernelGGL(kern, dim3(g.nW, g.hg), dim3(Cf::NTHREADS), lds, s, g, grp, qkv, dqkv, table, tpart);
    return hipGetLastError();
}

} // namespace

bool attn_core_mfma_supported(const Geom &g)
{
    const int nt = g.N / 16;
    return g.N % 16 == 0 && (nt == 4 || nt == 9) && g.d <= 32 && g.dq <= 32 && g.T < (1L << 31);
}

#define GSWA_CORE_SHAPES(X) X(4, 1, 1) X(4, 1, 2) X(4, 2, 1) X(4, 2, 2) X(9, 1, 1) X(9, 1, 2) X(9, 2, 1) X(9, 2, 2)

hipError_t launch_attn_core_fwd(const Geom &g, int grp, const bf16_t *qkv, const bf16_t *table,
                                bf16_t *attn_out, hipStream_t s)
{
    if (!attn_core_mfma_supported(g)) return hipErrorInvalidValue;
    const int nt = g.N / 16, et = (g.d + 15) / 16, kq = (g.dq + 15) / 16;
#define X(NT_, ET_, KQ_) \
    if (nt == NT_ && et == ET_ && kq == KQ_) return launch_fwd<NT_, ET_, KQ_>(g, grp, qkv, table, attn_out, s);
    GSWA_CORE_SHAPES(X)
#undef X
    return hipErrorInvalidValue;
}

hipError_t launch_attn_core_bwd(const Geom &g, int grp, const bf16_t *qkv, bf16_t *dqkv, const bf16_t *table,
                                float *tpart, hipStream_t s)
{
    if (!attn_core_mfma_supported(g) || !tpart) return hipErrorInvalidValue;
    const int nt = g.N / 16, et = (g.d + 15) / 16, kq = (g.dq + 15) / 16;
#define X(NT_, ET_, KQ_) \
    if (nt == NT_ && et == ET_ && kq == KQ_) return launch_bwd<NT_, ET_, KQ_>(g, grp, qkv, dqkv, table, tpart, s);
    GSWA_CORE_SHAPES(X)
#undef X
    return hipErrorInvalidValue;
}

} // namespace gswa
