/*
 * Group Shifted Window Attention (GSWA) -- plain CPU oracle, fp64.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct
 * statement of what one GSWA layer computes (AgileIR, Sec. "Group Shifted
 * Window Attention", Eq. 6-8, plus the window partition of "Patch Embedding"
 * and the relative bias of "Learnable Relative Shifted Bias").  Only the test
 * suite, the smoke check and the CPU-baseline leg of the benchmark may call it.
 * It shares no code with the HIP library and is never a fallback for it.
 *
 * The layer, for one image b and one M x M window (wi, wj) of the shifted
 * frame, with tokens n = r*M + c:
 *
 *   (i, j)  = (wi*M + r, wj*M + c)                 position in the shifted frame
 *   src(n)  = ((i + s) mod H, (j + s) mod W)       position of that token in x
 *   reg(n)  = 3*band(i, H) + band(j, W),
 *             band(p, L) = 0 if p < L-M, 1 if p < L-s, else 2     (used when s > 0)
 *   for g = 0 .. G-1:                                              (head groups)
 *       F_g  = x[src, g*Cg:(g+1)*Cg]  (+ O_{g-1} when g > 0 and cascade)   Eq. 8
 *       QKV  = F_g Wqkv_g^T + bqkv_g                                        Eq. 6
 *       for each head hl of the group, global head hd = g*hg + hl:
 *           S[n,m] = <q_n, k_m> / sqrt(e) + table[idx(n,m), hd]
 *                    + (s > 0 and reg(n) != reg(m) ? -100 : 0)
 *           idx(n,m) = (r_n - r_m + M-1)*(2M-1) + (c_n - c_m + M-1)
 *           P = softmax over m;   O_g[:, hl*d:(hl+1)*d] = P v
 *   A = concat_g O_g ;  y[src] = A Wproj^T + bproj                          Eq. 7
 *
 * Parameter allocation (Sec. "Parameter Allocation"): the query and key of a
 * head may be narrower (or wider) than its value.  With e = dqk channels per
 * head for q and k (dqk = 0 means e = d = C/heads, the plain layer), a group
 * projects to Rg = 2*hg*e + Cg features laid out [q: hg*e | k: hg*e | v: Cg],
 * head-major inside each block, and the scores are scaled by 1/sqrt(e).
 *
 * The paper leaves the attention core, the mask and the bias indexing to the
 * shifted-window prior art it builds on ("Akin to Swin Transformer"); the
 * forms above are the readings this oracle fixes.  Eq. 8 is read as "the input
 * of group g is its channel slice plus the output of group g-1".
 *
 * Parity pins (tests, CPU only): brute-force global attention with a block
 * mask; an independently written dense shifted-window attention for G = 1;
 * shift = 0 equivalence; closed forms for zero Q/K weights; sequential
 * composition for the cascade; central finite differences for every gradient.
 * Nothing here depends on the paper's Fig. 3 (not available), so the grouped
 * data flow is pinned against the readings above only.
 *
 * The backward pass is the hand-derived adjoint of the loops above; no
 * autograd library is involved.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int B, H, W, C;
    int heads, groups;
    int window, shift;
    int cascade; /* 1: Eq. 8 applied, 0: groups independent */
    int dqk;     /* channels of q and of k per head; 0: C / heads    */
} gswa_oracle_shape;

static int shape_ok(const gswa_oracle_shape *p)
{
    if (p->B <= 0 || p->H <= 0 || p->W <= 0 || p->C <= 0) return 0;
    if (p->heads <= 0 || p->groups <= 0 || p->window <= 0) return 0;
    if (p->C % p->heads || p->heads % p->groups) return 0;
    if (p->H % p->window || p->W % p->window) return 0;
    if (p->shift < 0 || p->shift >= p->window) return 0;
    if (p->dqk < 0) return 0;
    return 1;
}

/* channels per head of q and k */
static int qk_width(const gswa_oracle_shape *p) { return p->dqk > 0 ? p->dqk : p->C / p->heads; }

static int band(int pos, int len, int M, int s)
{
    if (pos < len - M) return 0;
    if (pos < len - s) return 1;
    return 2;
}

/* Per-window scratch: everything one window needs in forward and backward. */
typedef struct {
    int N, C, Cg, d, hg, heads;
    int e, Qg, Rg; /* q/k channels per head and per group; projected features per group */
    long *src;    /* [N]   flat token offset (b*H*W + i*W + j) into x / y   */
    int *reg;     /* [N]   mask region id                                    */
    double *F;    /* [G][N][Cg]   group inputs                               */
    double *QKV;  /* [G][N][Rg]   projected q|k|v                            */
    double *P;    /* [heads][N][N] attention probabilities                   */
    double *A;    /* [N][C]  concatenated group outputs                      */
    /* backward only */
    double *dA;   /* [N][C]                                                  */
    double *dQKV; /* [N][Rg]                                                 */
    double *dP;   /* [N][N]                                                  */
    double *dS;   /* [N][N]                                                  */
    double *dF;   /* [N][Cg]                                                 */
} window_buf;

static int window_buf_alloc(window_buf *wb, const gswa_oracle_shape *p, int backward)
{
    int M = p->window;
    int N = M * M, C = p->C, G = p->groups, Cg = C / G;
    memset(wb, 0, sizeof(*wb));
    wb->N = N; wb->C = C; wb->Cg = Cg; wb->heads = p->heads;
    wb->d = C / p->heads; wb->hg = p->heads / G;
    wb->e = qk_width(p); wb->Qg = wb->hg * wb->e; wb->Rg = 2 * wb->Qg + Cg;
    wb->src = malloc(sizeof(long) * N);
    wb->reg = malloc(sizeof(int) * N);
    wb->F = malloc(sizeof(double) * G * N * Cg);
    wb->QKV = malloc(sizeof(double) * G * N * wb->Rg);
    wb->P = malloc(sizeof(double) * (size_t)p->heads * N * N);
    wb->A = malloc(sizeof(double) * N * C);
    if (!wb->src || !wb->reg || !wb->F || !wb->QKV || !wb->P || !wb->A) return 0;
    if (backward) {
        wb->dA = malloc(sizeof(double) * N * C);
        wb->dQKV = malloc(sizeof(double) * N * wb->Rg);
        wb->dP = malloc(sizeof(double) * N * N);
        wb->dS = malloc(sizeof(double) * N * N);
        wb->dF = malloc(sizeof(double) * N * Cg);
        if (!wb->dA || !wb->dQKV || !wb->dP || !wb->dS || !wb->dF) return 0;
    }
    return 1;
}

static void window_buf_free(window_buf *wb)
{
    free(wb->src); free(wb->reg); free(wb->F); free(wb->QKV); free(wb->P); free(wb->A);
    free(wb->dA); free(wb->dQKV); free(wb->dP); free(wb->dS); free(wb->dF);
}

/* Token map and mask regions of window (b, wi, wj): shift + partition. */
static void window_geometry(const gswa_oracle_shape *p, int b, int wi, int wj, window_buf *wb)
{
    int M = p->window, s = p->shift, H = p->H, W = p->W;
    for (int r = 0; r < M; ++r)
        for (int c = 0; c < M; ++c) {
            int n = r * M + c;
            int i = wi * M + r, j = wj * M + c;
            int si = (i + s) % H, sj = (j + s) % W;
            wb->src[n] = ((long)b * H + si) * W + sj;
            wb->reg[n] = s > 0 ? 3 * band(i, H, M, s) + band(j, W, M, s) : 0;
        }
}

/* Forward of one window into wb->F, QKV, P, A (Eq. 6 and 8, attention core). */
static void window_forward(const gswa_oracle_shape *p, window_buf *wb, const double *x,
                           const double *wqkv, const double *bqkv, const double *table)
{
    int M = p->window, N = wb->N, C = wb->C, G = p->groups, Cg = wb->Cg;
    int d = wb->d, hg = wb->hg, heads = wb->heads, s = p->shift;
    int e_ = wb->e, Qg = wb->Qg, Rg = wb->Rg;
    double scale = 1.0 / sqrt((double)e_);

    for (int g = 0; g < G; ++g) {
        double *F = wb->F + (size_t)g * N * Cg;
        double *QKV = wb->QKV + (size_t)g * N * Rg;
        const double *Wg = wqkv + (size_t)g * Rg * Cg;
        const double *bg = bqkv + (size_t)g * Rg;

        for (int n = 0; n < N; ++n)
            for (int c = 0; c < Cg; ++c) {
                double v = x[wb->src[n] * C + g * Cg + c];
                if (g > 0 && p->cascade) v += wb->A[n * C + (g - 1) * Cg + c];
                F[n * Cg + c] = v;
            }

        for (int n = 0; n < N; ++n)
            for (int o = 0; o < Rg; ++o) {
                double acc = bg[o];
                for (int c = 0; c < Cg; ++c) acc += F[n * Cg + c] * Wg[o * Cg + c];
                QKV[n * Rg + o] = acc;
            }

        for (int hl = 0; hl < hg; ++hl) {
            int hd = g * hg + hl;
            double *P = wb->P + (size_t)hd * N * N;
            const double *q = QKV + hl * e_;
            const double *k = QKV + Qg + hl * e_;
            const double *v = QKV + 2 * Qg + hl * d;
            for (int n = 0; n < N; ++n) {
                int rn = n / M, cn = n % M;
                double mx = -INFINITY;
                for (int m = 0; m < N; ++m) {
                    int rm = m / M, cm = m % M;
                    double dot = 0.0;
                    for (int e = 0; e < e_; ++e) dot += q[n * Rg + e] * k[m * Rg + e];
                    int idx = (rn - rm + M - 1) * (2 * M - 1) + (cn - cm + M - 1);
                    double sc = dot * scale + table[(size_t)idx * heads + hd];
                    if (s > 0 && wb->reg[n] != wb->reg[m]) sc += -100.0;
                    P[n * N + m] = sc;
                    if (sc > mx) mx = sc;
                }
                double sum = 0.0;
                for (int m = 0; m < N; ++m) {
                    P[n * N + m] = exp(P[n * N + m] - mx);
                    sum += P[n * N + m];
                }
                for (int m = 0; m < N; ++m) P[n * N + m] /= sum;
                for (int e = 0; e < d; ++e) {
                    double acc = 0.0;
                    for (int m = 0; m < N; ++m) acc += P[n * N + m] * v[m * Rg + e];
                    wb->A[n * C + g * Cg + hl * d + e] = acc;
                }
            }
        }
    }
}

/*
 * y = GSWA(x).  All arrays fp64, C-contiguous:
 *   x, y          [B, H, W, C]
 *   wqkv          [G, Rg, Cg]  rows: q block, k block, v block; inside a block head-major
 *                 (Rg = 3*Cg for the plain layer, 2*hg*dqk + Cg otherwise)
 *   bqkv          [G, Rg]
 *   wproj         [C, C] (out, in),  bproj [C]
 *   table         [(2M-1)^2, heads]
 *   attn_out      optional [B, H, W, C]: concat of the group outputs A at each token's
 *                 position in x (before the output projection)
 *   probs         optional [nW, heads, N, N], nW ordered (b, wi, wj)
 * Returns 0, or -1 for an invalid shape, -2 for allocation failure.
 */
int gswa_oracle_forward(const gswa_oracle_shape *p, const double *x, const double *wqkv,
                        const double *bqkv, const double *wproj, const double *bproj,
                        const double *table, double *y, double *attn_out, double *probs)
{
    if (!shape_ok(p)) return -1;
    int M = p->window, N = M * M, C = p->C;
    int nwi = p->H / M, nwj = p->W / M;
    long nW = (long)p->B * nwi * nwj;
    int fail = 0;

#pragma omp parallel
    {
        window_buf wb;
        int ok = window_buf_alloc(&wb, p, 0);
        if (!ok) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(static)
        for (long w = 0; w < nW; ++w) {
            if (!ok) continue;
            int b = (int)(w / (nwi * nwj));
            int wi = (int)(w / nwj % nwi), wj = (int)(w % nwj);
            window_geometry(p, b, wi, wj, &wb);
            window_forward(p, &wb, x, wqkv, bqkv, table);
            for (int n = 0; n < N; ++n)
                for (int o = 0; o < C; ++o) {
                    double acc = bproj[o];
                    for (int c = 0; c < C; ++c) acc += wb.A[n * C + c] * wproj[o * C + c];
                    y[wb.src[n] * C + o] = acc;
                }
            if (attn_out)
                for (int n = 0; n < N; ++n)
                    for (int c = 0; c < C; ++c) attn_out[wb.src[n] * C + c] = wb.A[n * C + c];
            if (probs)
                memcpy(probs + (size_t)w * p->heads * N * N, wb.P,
                       sizeof(double) * (size_t)p->heads * N * N);
        }
        window_buf_free(&wb);
    }
    return fail ? -2 : 0;
}

/*
 * Gradients of L = sum(dy * y) with respect to every input of the layer.
 * dx [B,H,W,C]; dwqkv, dbqkv, dwproj, dbproj, dtable shaped like their
 * parameters.  All outputs are overwritten.  The forward pass is recomputed
 * per window.  Returns as gswa_oracle_forward.
 */
int gswa_oracle_backward(const gswa_oracle_shape *p, const double *x, const double *dy,
                         const double *wqkv, const double *bqkv, const double *wproj,
                         const double *bproj, const double *table, double *dx, double *dwqkv,
                         double *dbqkv, double *dwproj, double *dbproj, double *dtable)
{
    (void)bproj;
    if (!shape_ok(p)) return -1;
    int M = p->window, N = M * M, C = p->C, G = p->groups, Cg = C / G;
    int heads = p->heads, d = C / heads, hg = heads / G;
    int e_ = qk_width(p), Qg = hg * e_, Rg = 2 * Qg + Cg;
    int nwi = p->H / M, nwj = p->W / M;
    long nW = (long)p->B * nwi * nwj;
    size_t n_wqkv = (size_t)G * Rg * Cg, n_bqkv = (size_t)G * Rg;
    size_t n_wproj = (size_t)C * C, n_bproj = (size_t)C;
    size_t n_table = (size_t)(2 * M - 1) * (2 * M - 1) * heads;
    size_t n_par = n_wqkv + n_bqkv + n_wproj + n_bproj + n_table;
    double scale = 1.0 / sqrt((double)e_);
    int fail = 0;

    int nthreads = 1;
#ifdef _OPENMP
    nthreads = omp_get_max_threads();
#endif
    /* one private parameter-gradient accumulator per thread, summed in thread order */
    double *acc_all = calloc((size_t)nthreads * n_par, sizeof(double));
    if (!acc_all) return -2;

#pragma omp parallel num_threads(nthreads)
    {
        int tid = 0;
#ifdef _OPENMP
        tid = omp_get_thread_num();
#endif
        double *g_wqkv = acc_all + (size_t)tid * n_par;
        double *g_bqkv = g_wqkv + n_wqkv;
        double *g_wproj = g_bqkv + n_bqkv;
        double *g_bproj = g_wproj + n_wproj;
        double *g_table = g_bproj + n_bproj;

        window_buf wb;
        int ok = window_buf_alloc(&wb, p, 1);
        if (!ok) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(static)
        for (long w = 0; w < nW; ++w) {
            if (!ok) continue;
            int b = (int)(w / (nwi * nwj));
            int wi = (int)(w / nwj % nwi), wj = (int)(w % nwj);
            window_geometry(p, b, wi, wj, &wb);
            window_forward(p, &wb, x, wqkv, bqkv, table);

            /* adjoint of y[src] = A Wproj^T + bproj */
            for (int n = 0; n < N; ++n) {
                const double *dyn = dy + wb.src[n] * C;
                for (int c = 0; c < C; ++c) {
                    double acc = 0.0;
                    for (int o = 0; o < C; ++o) acc += dyn[o] * wproj[o * C + c];
                    wb.dA[n * C + c] = acc;
                }
                for (int o = 0; o < C; ++o) {
                    g_bproj[o] += dyn[o];
                    for (int c = 0; c < C; ++c) g_wproj[o * C + c] += dyn[o] * wb.A[n * C + c];
                }
            }

            for (int g = G - 1; g >= 0; --g) {
                const double *F = wb.F + (size_t)g * N * Cg;
                const double *QKV = wb.QKV + (size_t)g * N * Rg;
                const double *Wg = wqkv + (size_t)g * Rg * Cg;
                memset(wb.dQKV, 0, sizeof(double) * N * Rg);

                for (int hl = 0; hl < hg; ++hl) {
                    int hd = g * hg + hl;
                    const double *P = wb.P + (size_t)hd * N * N;
                    const double *q = QKV + hl * e_;
                    const double *k = QKV + Qg + hl * e_;
                    const double *v = QKV + 2 * Qg + hl * d;
                    double *dq = wb.dQKV + hl * e_;
                    double *dk = wb.dQKV + Qg + hl * e_;
                    double *dv = wb.dQKV + 2 * Qg + hl * d;
                    const double *dO = wb.dA + g * Cg + hl * d; /* row stride C */

                    /* O = P v  =>  dv = P^T dO,  dP = dO v^T */
                    for (int n = 0; n < N; ++n)
                        for (int m = 0; m < N; ++m) {
                            double acc = 0.0;
                            for (int e = 0; e < d; ++e) {
                                acc += dO[n * C + e] * v[m * Rg + e];
                                dv[m * Rg + e] += P[n * N + m] * dO[n * C + e];
                            }
                            wb.dP[n * N + m] = acc;
                        }
                    /* softmax: dS = P * (dP - sum_m P dP) */
                    for (int n = 0; n < N; ++n) {
                        double dot = 0.0;
                        for (int m = 0; m < N; ++m) dot += P[n * N + m] * wb.dP[n * N + m];
                        for (int m = 0; m < N; ++m)
                            wb.dS[n * N + m] = P[n * N + m] * (wb.dP[n * N + m] - dot);
                    }
                    /* S = scale q k^T + table[idx] + mask */
                    for (int n = 0; n < N; ++n) {
                        int rn = n / M, cn = n % M;
                        for (int m = 0; m < N; ++m) {
                            int rm = m / M, cm = m % M;
                            double ds = wb.dS[n * N + m];
                            int idx = (rn - rm + M - 1) * (2 * M - 1) + (cn - cm + M - 1);
                            g_table[(size_t)idx * heads + hd] += ds;
                            for (int e = 0; e < e_; ++e) {
                                dq[n * Rg + e] += scale * ds * k[m * Rg + e];
                                dk[m * Rg + e] += scale * ds * q[n * Rg + e];
                            }
                        }
                    }
                }

                /* QKV = F Wg^T + bg */
                for (int n = 0; n < N; ++n) {
                    for (int c = 0; c < Cg; ++c) {
                        double acc = 0.0;
                        for (int o = 0; o < Rg; ++o) acc += wb.dQKV[n * Rg + o] * Wg[o * Cg + c];
                        wb.dF[n * Cg + c] = acc;
                    }
                    for (int o = 0; o < Rg; ++o) {
                        double go = wb.dQKV[n * Rg + o];
                        g_bqkv[(size_t)g * Rg + o] += go;
                        for (int c = 0; c < Cg; ++c)
                            g_wqkv[((size_t)g * Rg + o) * Cg + c] += go * F[n * Cg + c];
                    }
                }
                /* F_g = x slice (+ O_{g-1}) */
                for (int n = 0; n < N; ++n)
                    for (int c = 0; c < Cg; ++c) {
                        dx[wb.src[n] * C + g * Cg + c] = wb.dF[n * Cg + c];
                        if (g > 0 && p->cascade) wb.dA[n * C + (g - 1) * Cg + c] += wb.dF[n * Cg + c];
                    }
            }
        }
        window_buf_free(&wb);
    }

    if (!fail) {
        double *outs[5] = {dwqkv, dbqkv, dwproj, dbproj, dtable};
        size_t lens[5] = {n_wqkv, n_bqkv, n_wproj, n_bproj, n_table};
        size_t off = 0;
        for (int k = 0; k < 5; ++k) {
            for (size_t i = 0; i < lens[k]; ++i) {
                double acc = 0.0;
                for (int t = 0; t < nthreads; ++t) acc += acc_all[(size_t)t * n_par + off + i];
                outs[k][i] = acc;
            }
            off += lens[k];
        }
    }
    free(acc_all);
    return fail ? -2 : 0;
}

/* Threads the calls above will use (1 when built without OpenMP). */
int gswa_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void gswa_oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}
