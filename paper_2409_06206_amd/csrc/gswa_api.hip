// C ABI of the GSWA library: argument validation, buffer carving and the order in which the
// kernels of one layer are enqueued.  No allocation, no synchronisation.
#include "../../include/gswa.h"
#include "common.h"
#include "staged_kernels.h"
#include "fused.h"

#include <map>
#include <mutex>
#include <string>
#include <utility>
#include <type_traits>

namespace {
thread_local std::string g_hip_error;
}

hipError_t gswa::allow_dynamic_lds(const void *kernel, size_t bytes)
{
    if (bytes <= 64 * 1024) return hipSuccess;
    static std::mutex mu;
    static std::map<std::pair<const void *, int>, size_t> allowed; // (kernel, device) -> limit set so far
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lk(mu);
    size_t &cur = allowed[std::make_pair(kernel, dev)];
    if (cur >= bytes) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess) cur = bytes;
    return e;
}

int gswa::report_hip_error(hipError_t e)
{
    g_hip_error = hipGetErrorString(e);
    return GSWA_EHIP;
}

namespace {

using namespace gswa;

// Scratch of gswa_backward_static: device memory owned by the library itself, one copy per GPU
// (allocated by the runtime when the code object is loaded on that GPU, held until the process
// ends).  Host code never uses the array's name as an address: static_scratch() asks the runtime
// for the device address once per device and hands that pointer on.
constexpr size_t kStaticScratchBytes = (size_t)GSWA_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device (looked up on the first call per device).
hipError_t static_scratch(void **out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

int hip_fail(hipError_t e) { return report_hip_error(e); }

#define GSWA_HIP(expr)                                \
    do {                                              \
        hipError_t e_ = (expr);                       \
        if (e_ != hipSuccess) return hip_fail(e_);    \
    } while (0)

size_t align256(size_t b) { return (b + 255) & ~size_t(255); }

// true when every pointer is 16-byte aligned (the kernels use vector loads and stores)
template <typename... P> bool aligned16(P... p) { return (((reinterpret_cast<uintptr_t>(p)) | ...) & 15) == 0; }

// Checks the descriptor (divisibility rules of the window partition and of the head groups)
// and derives the geometry.
int make_geom(const gswa_desc *d, Geom *g)
{
    if (!d) return GSWA_EINVAL;
    if (d->B <= 0 || d->H <= 0 || d->W <= 0 || d->C <= 0) return GSWA_EINVAL;
    if (d->heads <= 0 || d->groups <= 0 || d->window <= 0) return GSWA_EINVAL;
    if (d->C % d->heads || d->heads % d->groups) return GSWA_EINVAL;
    if (d->H % d->window || d->W % d->window) return GSWA_EINVAL;
    if (d->shift < 0 || d->shift >= d->window) return GSWA_EINVAL;
    if (d->dqk < 0) return GSWA_EINVAL;
    if (d->dtype != GSWA_F32 && d->dtype != GSWA_BF16) return GSWA_EINVAL;
    if (d->flags & ~(uint32_t)(GSWA_NO_CASCADE | GSWA_ACCUM_WGRAD | GSWA_FORCE_STAGED | GSWA_DETERMINISTIC))
        return GSWA_EINVAL;
    const long T = (long)d->B * d->H * d->W;
    const long nW = T / ((long)d->window * d->window);
    if (d->window > 64 || d->dqk > 4096) return GSWA_EUNSUPPORTED;
    const int dq = d->dqk > 0 ? d->dqk : d->C / d->heads;
    if (T * (2L * d->heads * dq + d->C) >= (1L << 40) || nW > 0x7fffffffL) return GSWA_EUNSUPPORTED;
    g->B = d->B; g->H = d->H; g->W = d->W; g->C = d->C;
    g->heads = d->heads; g->groups = d->groups; g->M = d->window; g->shift = d->shift;
    g->N = d->window * d->window;
    g->Cg = d->C / d->groups;
    g->hg = d->heads / d->groups;
    g->d = d->C / d->heads;
    g->dq = dq;
    g->Qg = g->hg * dq;
    g->Rg = 2 * g->Qg + g->Cg;
    g->nwi = d->H / d->window; g->nwj = d->W / d->window;
    g->nW = (int)nW;
    g->T = T;
    g->cascade = (d->flags & GSWA_NO_CASCADE) ? 0 : 1;
    int rs_f = 0, rs_b = 0;
    attn_fwd_lds_bytes(*g, &rs_f);
    attn_bwd_lds_bytes(*g, &rs_b);
    if (rs_f == 0 || rs_b == 0) return GSWA_EUNSUPPORTED;
    return GSWA_OK;
}

size_t elem_size(const gswa_desc *d) { return d->dtype == GSWA_F32 ? 4 : 2; }

// A device buffer as a byte range, for the overlap rules of the entry points.
struct Range {
    uintptr_t lo, hi;
    Range(const void *p, size_t bytes) : lo(reinterpret_cast<uintptr_t>(p)), hi(lo + (p ? bytes : 0)) {}
};
bool overlap(const Range &a, const Range &b) { return a.lo < b.hi && b.lo < a.hi; }
// true when `out` shares a byte with any of the others
template <typename... R> bool overlaps_any(const Range &out, const R &...others) { return (overlap(out, others) || ...); }

struct Sizes {
    size_t saved, qkv, fwd_ws, bwd_ws;
    size_t act;          // bytes of the saved [T, C] activation at the start of `saved`
    size_t pack;         // bytes of the packed parameters behind it (fused path)
    size_t fused_bwd_ws; // partial sums of the fused backward
    size_t params;       // fp32 entries of all five parameter gradients (one copy of the staged backward)
    size_t reps, tpart;  // bytes of the gradient copies and of the per-window bias-table gradients
    int nreps;           // gradient copies of the staged backward
    bool fused_fwd, fused_bwd;
};

bool use_fused_fwd(const gswa_desc *d, const Geom &g)
{
    return d->dtype == GSWA_BF16 && !(d->flags & GSWA_FORCE_STAGED) && g.dq == g.d && fused_fwd_supported(g);
}

Sizes make_sizes(const gswa_desc *d, const Geom &g)
{
    Sizes s;
    const size_t e = elem_size(d);
    s.saved = align256((size_t)g.T * g.C * e);
    s.qkv = align256((size_t)g.T * g.Rg * e);
    s.fwd_ws = s.qkv;
    s.params = (size_t)g.groups * g.Rg * g.Cg + (size_t)g.groups * g.Rg + (size_t)g.C * g.C + g.C +
               (size_t)(2 * g.M - 1) * (2 * g.M - 1) * g.heads;
    // (+ one bias-table gradient per window where the attention adjoint runs on the matrix cores, and
    // everywhere in the reproducible mode)
    const bool det = (d->flags & GSWA_DETERMINISTIC) != 0;
    s.tpart = (det || (d->dtype == GSWA_BF16 && attn_core_mfma_supported(g)))
                  ? align256((size_t)g.nW * (2 * g.M - 1) * (2 * g.M - 1) * g.heads * sizeof(float)) : 0;
    s.nreps = det ? kDetReplicas : kGradReplicas;
    s.reps = align256((size_t)s.nreps * s.params * sizeof(float));
    s.bwd_ws = 2 * s.qkv + s.reps + s.tpart;
    s.fused_fwd = use_fused_fwd(d, g);
    s.fused_bwd = s.fused_fwd && fused_bwd_supported(g);
    s.fused_bwd_ws = 0;
    s.pack = 0;
    s.act = s.saved;
    if (s.fused_fwd) {
        // the packed parameters ride behind the saved activation (training) or in ws (inference)
        s.pack = align256(fused_pack_bytes(g));
        s.saved = s.act + s.pack;
        // training needs no scratch; inference keeps the pack (and, when the forward is split,
        // the group outputs) in ws, which the caller sizes as fwd_ws + saved
        s.fwd_ws = 0;
    }
    if (s.fused_bwd) {
        s.fused_bwd_ws = align256(fused_bwd_ws_bytes(g));
        s.bwd_ws = s.fused_bwd_ws;
    }
    return s;
}

template <typename T>
int forward_staged(const Geom &g, const Sizes &sz, const T *x, const T *w_qkv, const T *b_qkv,
                   const T *w_proj, const T *b_proj, const T *table, T *y, T *saved, char *ws,
                   hipStream_t st)
{
    T *qkv = reinterpret_cast<T *>(ws);
    T *attn = saved ? saved : reinterpret_cast<T *>(ws + sz.qkv);
    const int C = g.C, Cg = g.Cg, Rg = g.Rg;
    for (int grp = 0; grp < g.groups; ++grp) {
        LinearArgs la{};
        la.a1 = x + grp * Cg; la.lda1 = C;
        if (grp > 0 && g.cascade) { la.a2 = attn + (grp - 1) * Cg; la.lda2 = C; }
        la.w = w_qkv + (size_t)grp * Rg * Cg; la.w_sn = Cg; la.w_sk = 1;
        la.bias = b_qkv + (size_t)grp * Rg;
        la.out = qkv; la.ldout = Rg;
        la.rows = g.T; la.N = Rg; la.K = Cg; la.prof_id = K_QKV_LINEAR;
        GSWA_HIP(launch_linear<T>(la, st));
        if constexpr (std::is_same<T, bf16_t>::value) {
            if (attn_core_mfma_supported(g)) {
                GSWA_HIP(launch_attn_core_fwd(g, grp, qkv, table, attn, st));
                continue;
            }
        }
        GSWA_HIP(launch_attn_fwd<T>(g, grp, qkv, table, attn, st));
    }
    LinearArgs lp{};
    lp.a1 = attn; lp.lda1 = C;
    lp.w = w_proj; lp.w_sn = C; lp.w_sk = 1;
    lp.bias = b_proj;
    lp.out = y; lp.ldout = C;
    lp.rows = g.T; lp.N = C; lp.K = C; lp.prof_id = K_PROJ_LINEAR;
    GSWA_HIP(launch_linear<T>(lp, st));
    return GSWA_OK;
}

template <typename T>
int backward_staged(const Geom &g, const Sizes &sz, uint32_t flags, const T *x, const T *dy,
                    const T *w_qkv, const T *b_qkv, const T *w_proj, const T *table,
                    const T *attn, T *dx, float *dw_qkv, float *db_qkv, float *dw_proj,
                    float *db_proj, float *dtable, char *ws, hipStream_t st)
{
    T *qkv = reinterpret_cast<T *>(ws);
    T *dqkv = reinterpret_cast<T *>(ws + sz.qkv);
    const int C = g.C, Cg = g.Cg, G = g.groups, Rg = g.Rg;
    // the parameter gradients are accumulated in kGradReplicas copies behind the two q|k|v buffers
    // (layout of a copy: dw_qkv | db_qkv | dw_proj | db_proj | dtable) and summed at the end
    float *rep = reinterpret_cast<float *>(ws + 2 * sz.qkv);
    float *tpart = reinterpret_cast<float *>(ws + 2 * sz.qkv + sz.reps);
    bool table_per_window = false;
    const long P = (long)sz.params;
    const long o_wq = 0, o_bq = o_wq + (long)G * Rg * Cg, o_wp = o_bq + (long)G * Rg, o_bp = o_wp + (long)C * C;
    const long o_tb = o_bp + C;
    const long n_tb = (long)(2 * g.M - 1) * (2 * g.M - 1) * g.heads;
    // (the copies are cleared by the first launch of the loop below)
    // adjoint of Eq. 7 with respect to the projection parameters
    WgradArgs wp{};
    wp.dout = dy; wp.lddout = C;
    wp.a1 = attn; wp.lda1 = C;
    const bool det = (flags & GSWA_DETERMINISTIC) != 0;
    const int nreps = sz.nreps;
    wp.dw = rep + o_wp; wp.db = rep + o_bp; wp.rep_stride = P; wp.reps = nreps; wp.exclusive = det;
    wp.rows = g.T; wp.N = C; wp.K = C; wp.prof_id = K_PROJ_WGRAD;
    // (independent of everything else: enqueued together with the first group's weight gradient)

    for (int grp = G - 1; grp >= 0; --grp) {
        const T *wg = w_qkv + (size_t)grp * Rg * Cg;
        const bool has_prev = grp > 0 && g.cascade;
        // recompute q|k|v of the group (Eq. 6, 8)
        LinearArgs la{};
        la.a1 = x + grp * Cg; la.lda1 = C;
        if (has_prev) { la.a2 = attn + (grp - 1) * Cg; la.lda2 = C; }
        la.w = wg; la.w_sn = Cg; la.w_sk = 1;
        la.bias = b_qkv + (size_t)grp * Rg;
        la.out = qkv; la.ldout = Rg;
        la.rows = g.T; la.N = Rg; la.K = Cg; la.prof_id = K_QKV_LINEAR;
        // (the per-window table gradients are written from this group's attention adjoint on: until then, in the
        // first group processed, their memory is free)
        if (grp == G - 1 && sz.tpart) { la.scratch = tpart; la.scratch_bytes = sz.tpart; }
        // dO_g = dy Wproj[:, slice g] (+ dF_{g+1}, which is dx[:, slice g+1]) into the v part of dqkv
        LinearArgs lo{};
        lo.a1 = dy; lo.lda1 = C;
        lo.w = w_proj + grp * Cg; lo.w_sn = 1; lo.w_sk = C;
        if (grp < G - 1 && g.cascade) { lo.add = dx + (grp + 1) * Cg; lo.ldadd = C; }
        lo.out = dqkv + 2 * g.Qg; lo.ldout = Rg;
        lo.rows = g.T; lo.N = Cg; lo.K = C; lo.prof_id = K_DO_LINEAR;
        GSWA_HIP(launch_linear_pair<T>(la, lo, grp == G - 1 ? rep : nullptr, (size_t)nreps * P, st));
        bool on_matrix_cores = false;
        if constexpr (std::is_same<T, bf16_t>::value) {
            if (attn_core_mfma_supported(g)) {
                GSWA_HIP(launch_attn_core_bwd(g, grp, qkv, dqkv, table, tpart, st));
                table_per_window = true;
                on_matrix_cores = true;
            }
        }
        if (!on_matrix_cores) {
            if (det) { // one copy per window, plain stores: summed in a fixed order at the end
                GSWA_HIP(launch_attn_bwd<T>(g, grp, qkv, dqkv, table, tpart, n_tb, 0, st));
                table_per_window = true;
            } else {
                GSWA_HIP(launch_attn_bwd<T>(g, grp, qkv, dqkv, table, rep + o_tb, P, nreps, st));
            }
        }
        // dF_g = dqkv Wqkv_g  ->  dx[:, slice g]
        LinearArgs lx{};
        lx.a1 = dqkv; lx.lda1 = Rg;
        lx.w = wg; lx.w_sn = 1; lx.w_sk = Cg;
        lx.out = dx + grp * Cg; lx.ldout = C;
        lx.rows = g.T; lx.N = Cg; lx.K = Rg; lx.prof_id = K_DX_LINEAR;
        lx.scratch = qkv; lx.scratch_bytes = sz.qkv; // (q|k|v of the group has had its last read)
        WgradArgs wq{};
        wq.dout = dqkv; wq.lddout = Rg;
        wq.a1 = x + grp * Cg; wq.lda1 = C;
        if (has_prev) { wq.a2 = attn + (grp - 1) * Cg; wq.lda2 = C; }
        wq.dw = rep + o_wq + (size_t)grp * Rg * Cg;
        wq.db = rep + o_bq + (size_t)grp * Rg;
        wq.rep_stride = P; wq.reps = nreps; wq.exclusive = det;
        wq.rows = g.T; wq.N = Rg; wq.K = Cg; wq.prof_id = K_QKV_WGRAD;
        // (q|k|v of the group has served its last read: its buffer is scratch for the weight gradients)
        wq.scratch = qkv; wq.scratch_bytes = sz.qkv;
        wp.scratch = qkv; wp.scratch_bytes = sz.qkv;
        GSWA_HIP(launch_wgrad_group<T>(wq, grp == G - 1 ? &wp : nullptr, lx, st));
    }
    ReplicaSum rs{};
    rs.rep = rep; rs.stride = P; rs.reps = nreps;
    rs.out[0] = dw_qkv; rs.off[0] = o_wq; rs.n[0] = (long)G * Rg * Cg;
    rs.out[1] = db_qkv; rs.off[1] = o_bq; rs.n[1] = (long)G * Rg;
    rs.out[2] = dw_proj; rs.off[2] = o_wp; rs.n[2] = (long)C * C;
    rs.out[3] = db_proj; rs.off[3] = o_bp; rs.n[3] = C;
    if (table_per_window) {
        rs.count = 4;
        rs.tpart = tpart; rs.t_out = dtable; rs.t_off = o_tb; rs.t_n = n_tb; rs.t_windows = g.nW;
    } else {
        rs.out[4] = dtable; rs.off[4] = o_tb; rs.n[4] = n_tb;
        rs.count = 5;
    }
    rs.accumulate = (flags & GSWA_ACCUM_WGRAD) ? 1 : 0;
    GSWA_HIP(launch_reduce_replicas(rs, st));
    return GSWA_OK;
}

int backward_fused(const Geom &g, const Sizes &sz, uint32_t flags, const bf16_t *x, const bf16_t *dy,
                   const bf16_t *table, const char *saved, bf16_t *dx, float *dw_qkv, float *db_qkv,
                   float *dw_proj, float *db_proj, float *dtable, char *ws, hipStream_t st)
{
    const int accumulate = (flags & GSWA_ACCUM_WGRAD) ? 1 : 0;
    GSWA_HIP(launch_fused_bwd(g, x, dy, reinterpret_cast<const bf16_t *>(saved), saved + sz.act, table, dx,
                              dw_qkv, db_qkv, dw_proj, db_proj, dtable, accumulate, ws, st));
    return GSWA_OK;
}

} // namespace

extern "C" {

int gswa_query_bytes(const gswa_desc *desc, size_t *saved_bytes, size_t *fwd_ws_bytes,
                     size_t *bwd_ws_bytes)
{
    Geom g;
    int rc = make_geom(desc, &g);
    if (rc != GSWA_OK) return rc;
    Sizes s = make_sizes(desc, g);
    if (saved_bytes) *saved_bytes = s.saved;
    if (fwd_ws_bytes) *fwd_ws_bytes = s.fwd_ws;
    if (bwd_ws_bytes) *bwd_ws_bytes = s.bwd_ws;
    return GSWA_OK;
}

int gswa_query_path(const gswa_desc *desc, int *forward_path, int *backward_path)
{
    Geom g;
    int rc = make_geom(desc, &g);
    if (rc != GSWA_OK) return rc;
    const Sizes s = make_sizes(desc, g); // (the same decisions gswa_forward and gswa_backward take)
    int fwd = GSWA_PATH_STAGED;
    if (s.fused_fwd) fwd = GSWA_PATH_FUSED;
    else if (desc->dtype == GSWA_BF16 && !(desc->flags & GSWA_FORCE_STAGED) && window_fwd_supported(g)) fwd = GSWA_PATH_WINDOW_FWD;
    if (forward_path) *forward_path = fwd;
    if (backward_path) *backward_path = s.fused_bwd ? GSWA_PATH_FUSED : GSWA_PATH_STAGED;
    return GSWA_OK;
}

int gswa_forward(const gswa_desc *desc, const void *x, const void *w_qkv, const void *b_qkv,
                 const void *w_proj, const void *b_proj, const void *bias_table, void *y,
                 void *saved, void *ws, void *hip_stream)
{
    Geom g;
    int rc = make_geom(desc, &g);
    if (rc != GSWA_OK) return rc;
    if (!x || !w_qkv || !b_qkv || !w_proj || !b_proj || !bias_table || !y) return GSWA_EINVAL;
    if (reinterpret_cast<uintptr_t>(ws) & 255) return GSWA_EINVAL;
    if (!aligned16(x, w_qkv, b_qkv, w_proj, b_proj, bias_table, y, saved)) return GSWA_EINVAL;
    Sizes s = make_sizes(desc, g);
    {
        const size_t e = elem_size(desc), act = (size_t)g.T * g.C * e;
        const size_t ws_bytes = saved ? s.fwd_ws : s.fwd_ws + s.saved;
        if (!ws && ws_bytes > 0) return GSWA_EINVAL; // no scratch is only acceptable where none is used
        const Range rx(x, act), ry(y, act), rsv(saved, s.saved), rws(ws, ws_bytes);
        const Range rwq(w_qkv, (size_t)g.groups * g.Rg * g.Cg * e), rbq(b_qkv, (size_t)g.groups * g.Rg * e);
        const Range rwp(w_proj, (size_t)g.C * g.C * e), rbp(b_proj, (size_t)g.C * e);
        const Range rtb(bias_table, (size_t)(2 * g.M - 1) * (2 * g.M - 1) * g.heads * e);
        if (overlaps_any(ry, rx, rsv, rws, rwq, rbq, rwp, rbp, rtb)) return GSWA_EINVAL;
        if (overlaps_any(rsv, rx, rws, rwq, rbq, rwp, rbp, rtb)) return GSWA_EINVAL;
        if (overlaps_any(rws, rx, rwq, rbq, rwp, rbp, rtb)) return GSWA_EINVAL;
    }
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (desc->dtype == GSWA_F32)
        return forward_staged<float>(g, s, (const float *)x, (const float *)w_qkv, (const float *)b_qkv,
                                     (const float *)w_proj, (const float *)b_proj,
                                     (const float *)bias_table, (float *)y, (float *)saved, (char *)ws, st);
    if (s.fused_fwd) {
        void *pack = saved ? static_cast<void *>(static_cast<char *>(saved) + s.act) : ws;
        void *attn = saved;
        if (!saved && fused_fwd_needs_attn(g)) attn = static_cast<char *>(ws) + s.pack;
        hipError_t e = launch_fused_fwd(g, (const bf16_t *)x, (const bf16_t *)w_qkv, (const bf16_t *)b_qkv,
                                        (const bf16_t *)w_proj, (const bf16_t *)b_proj,
                                        (const bf16_t *)bias_table, (bf16_t *)y, (bf16_t *)attn, pack, saved ? 1 : 0, st);
        return e == hipSuccess ? GSWA_OK : hip_fail(e);
    }
    if (!(desc->flags & GSWA_FORCE_STAGED) && window_fwd_supported(g)) {
        hipError_t e = launch_window_fwd(g, (const bf16_t *)x, (const bf16_t *)w_qkv, (const bf16_t *)b_qkv,
                                         (const bf16_t *)w_proj, (const bf16_t *)b_proj,
                                         (const bf16_t *)bias_table, (bf16_t *)y, (bf16_t *)saved, st);
        return e == hipSuccess ? GSWA_OK : hip_fail(e);
    }
    return forward_staged<bf16_t>(g, s, (const bf16_t *)x, (const bf16_t *)w_qkv, (const bf16_t *)b_qkv,
                                  (const bf16_t *)w_proj, (const bf16_t *)b_proj,
                                  (const bf16_t *)bias_table, (bf16_t *)y, (bf16_t *)saved, (char *)ws, st);
}

int gswa_backward(const gswa_desc *desc, const void *x, const void *dy, const void *w_qkv,
                  const void *b_qkv, const void *w_proj, const void *b_proj,
                  const void *bias_table, const void *saved, void *dx, void *dw_qkv,
                  void *db_qkv, void *dw_proj, void *db_proj, void *dbias_table, void *ws,
                  void *hip_stream)
{
    Geom g;
    int rc = make_geom(desc, &g);
    if (rc != GSWA_OK) return rc;
    if (!x || !dy || !w_qkv || !b_qkv || !w_proj || !b_proj || !bias_table || !saved || !dx ||
        !dw_qkv || !db_qkv || !dw_proj || !db_proj || !dbias_table)
        return GSWA_EINVAL;
    if (reinterpret_cast<uintptr_t>(ws) & 255) return GSWA_EINVAL;
    if (!aligned16(x, dy, w_qkv, b_qkv, w_proj, bias_table, saved, dx, dw_qkv, db_qkv, dw_proj, db_proj,
                   dbias_table))
        return GSWA_EINVAL;
    Sizes s = make_sizes(desc, g);
    {
        const size_t e = elem_size(desc), act = (size_t)g.T * g.C * e;
        if (!ws && s.bwd_ws > 0) return GSWA_EINVAL;
        const size_t n_wq = (size_t)g.groups * g.Rg * g.Cg, n_bq = (size_t)g.groups * g.Rg;
        const size_t n_wp = (size_t)g.C * g.C, n_tb = (size_t)(2 * g.M - 1) * (2 * g.M - 1) * g.heads;
        const Range rx(x, act), rdy(dy, act), rsv(saved, s.saved), rdx(dx, act), rws(ws, s.bwd_ws);
        const Range rwq(w_qkv, n_wq * e), rbq(b_qkv, n_bq * e), rwp(w_proj, n_wp * e), rbp(b_proj, (size_t)g.C * e);
        const Range rtb(bias_table, n_tb * e);
        const Range gwq(dw_qkv, n_wq * 4), gbq(db_qkv, n_bq * 4), gwp(dw_proj, n_wp * 4), gbp(db_proj, (size_t)g.C * 4);
        const Range gtb(dbias_table, n_tb * 4);
        // every output and the scratch: disjoint from every input and from each other
        if (overlaps_any(rdx, rx, rdy, rsv, rws, rwq, rbq, rwp, rbp, rtb, gwq, gbq, gwp, gbp, gtb)) return GSWA_EINVAL;
        if (overlaps_any(rws, rx, rdy, rsv, rwq, rbq, rwp, rbp, rtb, gwq, gbq, gwp, gbp, gtb)) return GSWA_EINVAL;
        if (overlaps_any(gwq, rx, rdy, rsv, rwq, rbq, rwp, rbp, rtb, gbq, gwp, gbp, gtb)) return GSWA_EINVAL;
        if (overlaps_any(gbq, rx, rdy, rsv, rwq, rbq, rwp, rbp, rtb, gwp, gbp, gtb)) return GSWA_EINVAL;
        if (overlaps_any(gwp, rx, rdy, rsv, rwq, rbq, rwp, rbp, rtb, gbp, gtb)) return GSWA_EINVAL;
        if (overlaps_any(gbp, rx, rdy, rsv, rwq, rbq, rwp, rbp, rtb, gtb)) return GSWA_EINVAL;
        if (overlaps_any(gtb, rx, rdy, rsv, rwq, rbq, rwp, rbp, rtb)) return GSWA_EINVAL;
    }
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (desc->dtype == GSWA_F32)
        return backward_staged<float>(g, s, desc->flags, (const float *)x, (const float *)dy,
                                      (const float *)w_qkv, (const float *)b_qkv, (const float *)w_proj,
                                      (const float *)bias_table, (const float *)saved, (float *)dx,
                                      (float *)dw_qkv, (float *)db_qkv, (float *)dw_proj,
                                      (float *)db_proj, (float *)dbias_table, (char *)ws, st);
    if (s.fused_bwd)
        return backward_fused(g, s, desc->flags, (const bf16_t *)x, (const bf16_t *)dy,
                              (const bf16_t *)bias_table, (const char *)saved, (bf16_t *)dx, (float *)dw_qkv,
                              (float *)db_qkv, (float *)dw_proj, (float *)db_proj, (float *)dbias_table,
                              (char *)ws, st);
    return backward_staged<bf16_t>(g, s, desc->flags, (const bf16_t *)x, (const bf16_t *)dy,
                                   (const bf16_t *)w_qkv, (const bf16_t *)b_qkv, (const bf16_t *)w_proj,
                                   (const bf16_t *)bias_table, (const bf16_t *)saved, (bf16_t *)dx,
                                   (float *)dw_qkv, (float *)db_qkv, (float *)dw_proj,
                                   (float *)db_proj, (float *)dbias_table, (char *)ws, st);
}

int gswa_backward_static(const gswa_desc *desc, const void *x, const void *dy, const void *w_qkv,
                         const void *b_qkv, const void *w_proj, const void *b_proj,
                         const void *bias_table, const void *saved, void *dx, void *dw_qkv,
                         void *db_qkv, void *dw_proj, void *db_proj, void *dbias_table,
                         void *hip_stream)
{
    Geom g;
    int rc = make_geom(desc, &g);
    if (rc != GSWA_OK) return rc;
    const Sizes s = make_sizes(desc, g);
    if (s.bwd_ws > kStaticScratchBytes) return GSWA_ETOOBIG;
    void *ws = nullptr;
    GSWA_HIP(static_scratch(&ws));
    // every kernel of the backward treats its scratch as undefined on entry and clears what it
    // accumulates into, so the previous call's contents need no fill here
    return gswa_backward(desc, x, dy, w_qkv, b_qkv, w_proj, b_proj, bias_table, saved, dx, dw_qkv, db_qkv,
                         dw_proj, db_proj, dbias_table, ws, hip_stream);
}

const char *gswa_strerror(int status)
{
    switch (status) {
    case GSWA_OK: return "ok";
    case GSWA_EINVAL: return "invalid argument (null pointer, size, divisibility or shift range)";
    case GSWA_EUNSUPPORTED: return "layer shape not covered by any kernel of this library";
    case GSWA_EHIP: return "HIP runtime call failed";
    case GSWA_ETOOBIG: return "layer needs more scratch than the library's built-in buffer holds";
    default: return "unknown status";
    }
}

const char *gswa_last_hip_error(void) { return g_hip_error.c_str(); }

int gswa_version(void) { return 100; }

} // extern "C"
