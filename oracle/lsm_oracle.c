/*
 * lsm_oracle.c -- TEST INFRASTRUCTURE, not part of the product path.
 *
 * Plain, slow, fp64 CPU evaluation of the unified linear-sequence-modeling
 * recurrence (paper Eq. 5 with the incremental update k^T v of Table 1, rows
 * BLA / Lightning Attn / RetNet / GLA / Mamba2 / RWKV6) and of the read-out
 * o_s = q_s M_s (numerator of the RNN form in Sec. 2.1.1).  One token at a
 * time, exactly as the definition is written: no chunking, no blocking, no
 * reordering.  Only tests, the smoke check and the cpu_baseline leg of the
 * benchmark may call this file.  It shares no code with the GPU library.
 *
 * Conventions (readings of the paper where it is silent):
 *   - M has d_k rows and d_v columns; a vector decay multiplies ROWS of M
 *     (diag{a_s} M_{s-1}, Table 1 GLA / RWKV6 rows).
 *   - the decay is handed over as log-decay g = log a, a_t = exp(g_t).
 *   - decay acts on M_{t-1}; the token's own k_t^T v_t enters undecayed (Eq. 5).
 *   - o_t reads M_t, i.e. it sees token t itself.
 *   - no normaliser z_s, no feature map, no 1/sqrt(d) scale.
 *
 * decay kind: 0 none (a=1), 1 one value per head g[H], 2 scalar per token
 * g[B,H,T], 3 vector per token g[B,H,T,d_k].
 *
 * Every pin of this file (quadratic form, closed forms, finite differences,
 * library special cases) lives in tests/ and runs without a GPU.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_NONE = 0, ORACLE_HEAD = 1, ORACLE_SCALAR = 2, ORACLE_VECTOR = 3 };

int lsm_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* a_t[i] for token t (0-based) of sequence (b,h): Table 1 parameter column. */
static void decay_of_token(int kind, const double *g, int H, int T, int dk,
                           int b, int h, int t, double *a)
{
    int i;
    if (kind == ORACLE_NONE) {
        for (i = 0; i < dk; ++i) a[i] = 1.0;
    } else if (kind == ORACLE_HEAD) {
        double s = exp(g[h]);
        for (i = 0; i < dk; ++i) a[i] = s;
    } else if (kind == ORACLE_SCALAR) {
        double s = exp(g[((size_t)b * H + h) * T + t]);
        for (i = 0; i < dk; ++i) a[i] = s;
    } else {
        const double *gv = g + (((size_t)b * H + h) * T + t) * dk;
        for (i = 0; i < dk; ++i) a[i] = exp(gv[i]);
    }
}

/* One step of Eq. 5:  M <- diag(a) M + k^T v. */
static void recurrence_step(double *M, int dk, int dv, const double *a,
                            const double *k, const double *v)
{
    int i, j;
    for (i = 0; i < dk; ++i) {
        double *Mi = M + (size_t)i * dv;
        for (j = 0; j < dv; ++j) Mi[j] = a[i] * Mi[j] + k[i] * v[j];
    }
}

/*
 * Forward.  q,k: [B,H,T,dk]; v,o: [B,H,T,dv]; m0, mT: [B,H,dk,dv] (m0 may be
 * NULL = zeros, mT may be NULL = not wanted).  Returns 0, or -1 on bad args.
 */
int lsm_oracle_fwd(int B, int H, int T, int dk, int dv, int kind,
                   const double *q, const double *k, const double *v,
                   const double *g, const double *m0,
                   double *o, double *mT)
{
    int bh;
    if (B < 1 || H < 1 || T < 1 || dk < 1 || dv < 1 || kind < 0 || kind > 3) return -1;
    if (!q || !k || !v || !o || (kind != ORACLE_NONE && !g)) return -1;
#pragma omp parallel for schedule(dynamic, 1)
    for (bh = 0; bh < B * H; ++bh) {
        int b = bh / H, h = bh % H, t, i, j;
        double *M = (double *)calloc((size_t)dk * dv, sizeof(double));
        double *a = (double *)malloc((size_t)dk * sizeof(double));
        if (m0) memcpy(M, m0 + (size_t)bh * dk * dv, (size_t)dk * dv * sizeof(double));
        for (t = 0; t < T; ++t) {
            const double *qt = q + ((size_t)bh * T + t) * dk;
            const double *kt = k + ((size_t)bh * T + t) * dk;
            const double *vt = v + ((size_t)bh * T + t) * dv;
            double *ot = o + ((size_t)bh * T + t) * dv;
            decay_of_token(kind, g, H, T, dk, b, h, t, a);
            recurrence_step(M, dk, dv, a, kt, vt);
            for (j = 0; j < dv; ++j) ot[j] = 0.0;
            for (i = 0; i < dk; ++i)
                for (j = 0; j < dv; ++j) ot[j] += qt[i] * M[(size_t)i * dv + j];
        }
        if (mT) memcpy(mT + (size_t)bh * dk * dv, M, (size_t)dk * dv * sizeof(double));
        free(M);
        free(a);
    }
    return 0;
}

/*
 * Backward of the scalar loss  L = sum(o * d_o) + sum(M_T * d_mT)  by the
 * token-level reverse recurrence (the paper gives no backward; this is the
 * adjoint of Eq. 5 and of o_t = q_t M_t, derived by hand):
 *
 *   D = d_mT (or 0)
 *   for t = T..1:   D  += q_t^T d_o_t                 (D = dL/dM_t)
 *                   dq_t = M_t d_o_t^T
 *                   dk_t = D v_t^T ,  dv_t = k_t D
 *                   dg_t[i] = a_t[i] * sum_j D[i,j] M_{t-1}[i,j]
 *                   D   = diag(a_t) D                 (D = dL/dM_{t-1})
 *   d_m0 = D
 *
 * M_t is needed for every t; to bound memory the forward sweep keeps M only
 * at multiples of `window` tokens and each window is re-expanded with the same
 * recurrence before it is walked in reverse (storage only, same arithmetic).
 *
 * dg has the shape of g: HEAD kind sums over i, b and t; SCALAR sums over i.
 * dg may be NULL (skipped); it must be NULL-or-ignored for kind none.
 * d_m0 may be NULL.  d_mT may be NULL (= zeros).
 */
int lsm_oracle_bwd(int B, int H, int T, int dk, int dv, int kind,
                   const double *q, const double *k, const double *v,
                   const double *g, const double *m0,
                   const double *d_o, const double *d_mT,
                   double *dq, double *dk_out, double *dv_out,
                   double *dg, double *d_m0)
{
    const int window = 64;
    int bh, b, h;
    size_t sz = (size_t)dk * dv;
    int nwin = (T + window - 1) / window;
    double *dg_head_part = NULL; /* [B*H] partial sums for the per-head kind */
    if (B < 1 || H < 1 || T < 1 || dk < 1 || dv < 1 || kind < 0 || kind > 3) return -1;
    if (!q || !k || !v || !d_o || !dq || !dk_out || !dv_out) return -1;
    if (kind != ORACLE_NONE && !g) return -1;
    if (kind == ORACLE_NONE) dg = NULL;
    if (dg && kind == ORACLE_HEAD) dg_head_part = (double *)calloc((size_t)B * H, sizeof(double));

#pragma omp parallel for schedule(dynamic, 1)
    for (bh = 0; bh < B * H; ++bh) {
        int bb = bh / H, hh = bh % H, t, i, j, w;
        double *ckpt = (double *)malloc(sz * (size_t)nwin * sizeof(double));       /* M at window starts */
        double *Mw = (double *)malloc(sz * (size_t)(window + 1) * sizeof(double)); /* M inside a window  */
        double *D = (double *)calloc(sz, sizeof(double));
        double *a = (double *)malloc((size_t)dk * sizeof(double));
        double *M = (double *)calloc(sz, sizeof(double));
        double head_acc = 0.0;
        if (m0) memcpy(M, m0 + (size_t)bh * sz, sz * sizeof(double));
        for (t = 0; t < T; ++t) {
            if (t % window == 0) memcpy(ckpt + (size_t)(t / window) * sz, M, sz * sizeof(double));
            decay_of_token(kind, g, H, T, dk, bb, hh, t, a);
            recurrence_step(M, dk, dv, a, k + ((size_t)bh * T + t) * dk, v + ((size_t)bh * T + t) * dv);
        }
        if (d_mT) memcpy(D, d_mT + (size_t)bh * sz, sz * sizeof(double));
        for (w = nwin - 1; w >= 0; --w) {
            int t0 = w * window, t1 = t0 + window < T ? t0 + window : T;
            /* Mw[n] = state after t0+n tokens, n = 0..t1-t0 */
            memcpy(Mw, ckpt + (size_t)w * sz, sz * sizeof(double));
            for (t = t0; t < t1; ++t) {
                double *nxt = Mw + (size_t)(t - t0 + 1) * sz;
                memcpy(nxt, Mw + (size_t)(t - t0) * sz, sz * sizeof(double));
                decay_of_token(kind, g, H, T, dk, bb, hh, t, a);
                recurrence_step(nxt, dk, dv, a, k + ((size_t)bh * T + t) * dk, v + ((size_t)bh * T + t) * dv);
            }
            for (t = t1 - 1; t >= t0; --t) {
                const double *qt = q + ((size_t)bh * T + t) * dk;
                const double *kt = k + ((size_t)bh * T + t) * dk;
                const double *vt = v + ((size_t)bh * T + t) * dv;
                const double *dot = d_o + ((size_t)bh * T + t) * dv;
                const double *Mt = Mw + (size_t)(t - t0 + 1) * sz;   /* M_t     */
                const double *Mp = Mw + (size_t)(t - t0) * sz;       /* M_{t-1} */
                double *dqt = dq + ((size_t)bh * T + t) * dk;
                double *dkt = dk_out + ((size_t)bh * T + t) * dk;
                double *dvt = dv_out + ((size_t)bh * T + t) * dv;
                double dg_scalar = 0.0;
                decay_of_token(kind, g, H, T, dk, bb, hh, t, a);
                for (i = 0; i < dk; ++i)
                    for (j = 0; j < dv; ++j) D[(size_t)i * dv + j] += qt[i] * dot[j];
                for (j = 0; j < dv; ++j) dvt[j] = 0.0;
                for (i = 0; i < dk; ++i) {
                    double sq = 0.0, sk = 0.0, sg = 0.0;
                    for (j = 0; j < dv; ++j) {
                        sq += Mt[(size_t)i * dv + j] * dot[j];
                        sk += D[(size_t)i * dv + j] * vt[j];
                        sg += D[(size_t)i * dv + j] * Mp[(size_t)i * dv + j];
                        dvt[j] += kt[i] * D[(size_t)i * dv + j];
                    }
                    dqt[i] = sq;
                    dkt[i] = sk;
                    sg *= a[i];
                    if (dg && kind == ORACLE_VECTOR) dg[((size_t)bh * T + t) * dk + i] = sg;
                    dg_scalar += sg;
                }
                if (dg && kind == ORACLE_SCALAR) dg[(size_t)bh * T + t] = dg_scalar;
                head_acc += dg_scalar;
                for (i = 0; i < dk; ++i)
                    for (j = 0; j < dv; ++j) D[(size_t)i * dv + j] *= a[i];
            }
        }
        if (d_m0) memcpy(d_m0 + (size_t)bh * sz, D, sz * sizeof(double));
        if (dg_head_part) dg_head_part[bh] = head_acc;
        free(ckpt); free(Mw); free(D); free(a); free(M);
    }
    if (dg_head_part) {
        for (h = 0; h < H; ++h) {
            double s = 0.0;
            for (b = 0; b < B; ++b) s += dg_head_part[(size_t)b * H + h];
            dg[h] = s;
        }
        free(dg_head_part);
    }
    return 0;
}
