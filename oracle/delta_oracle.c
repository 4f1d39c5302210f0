/*
 * delta_oracle.c -- TEST INFRASTRUCTURE, not part of the product path.
 *
 * Plain, slow, fp64 CPU evaluation of the two delta-rule rows of the paper's
 * Table 1 under the unified recurrence of Eq. 5, one token at a time, exactly
 * as the rows are written:
 *
 *   DeltaNet        M_s = (I - a_s k_s^T k_s) M_{s-1} + b_s k_s^T v_s
 *   Gated DeltaNet  M_s = a_s (I - k_s^T k_s) M_{s-1} + b_s k_s^T v_s
 *
 * and of the read-out o_s = q_s M_s (Sec. 2.1.1, as for the other rows).  Both
 * rows are instances of
 *
 *   M_s = alpha_s (I - beta_s k_s^T k_s) M_{s-1} + b_s k_s^T v_s
 *
 * (DeltaNet: alpha = 1, beta = the row's a_s; Gated DeltaNet: alpha = the row's
 * a_s, beta = 1), which is what this file evaluates; alpha is handed over as
 * log alpha <= 0.  A NULL log_alpha / beta / b means the constant 1.
 *
 * The reverse pass is the adjoint of that token loop for
 *   L = <o, d_o> + <M_T, d_mT> ,
 * taken token by token backward in time; it needs M_{s-1} at every token, which
 * it gets by keeping a copy of the state every BLOCK tokens in the forward sweep
 * and replaying one block at a time.
 *
 * Conventions: M has d_k rows and d_v columns; k_s, q_s, v_s are row vectors; no
 * normaliser, no feature map, no scale.  Only tests, the smoke check and the
 * cpu_baseline leg of the benchmark may call this file.  It shares no code with
 * the GPU library.  Its pins (reduction to the diagonal-decay oracle at beta = 0,
 * the stored-value property of a unit key, the triangular-solve form of a block
 * of tokens, the gradient-step reading of the update, finite differences) live
 * in tests/ and run without a GPU.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { BLOCK = 64 };

/* one token of the recurrence, in place: M <- alpha (M - beta k^T (k M)) + b k^T v */
static void delta_token(double *M, int dk, int dv, const double *k, const double *v,
                        double alpha, double beta, double bw, double *w)
{
    int i, j;
    for (j = 0; j < dv; ++j) w[j] = 0.0;
    for (i = 0; i < dk; ++i)
        for (j = 0; j < dv; ++j) w[j] += k[i] * M[(size_t)i * dv + j];   /* w = k M_{s-1} */
    for (i = 0; i < dk; ++i)
        for (j = 0; j < dv; ++j)
            M[(size_t)i * dv + j] = alpha * (M[(size_t)i * dv + j] - beta * k[i] * w[j]) + bw * k[i] * v[j];
}

static double param_at(const double *p, size_t idx, int is_log)
{
    if (!p) return 1.0;
    return is_log ? exp(p[idx]) : p[idx];
}

int delta_oracle_fwd(int B, int H, int T, int dk, int dv,
                     const double *q, const double *k, const double *v,
                     const double *log_alpha, const double *beta, const double *bw,
                     const double *m0, double *o, double *mT)
{
    int bh;
    if (B <= 0 || H <= 0 || T < 0 || dk <= 0 || dv <= 0 || !q || !k || !v || !o) return -1;
#pragma omp parallel for schedule(dynamic)
    for (bh = 0; bh < B * H; ++bh) {
        double *M = (double *)malloc(sizeof(double) * dk * dv);
        double *w = (double *)malloc(sizeof(double) * dv);
        int t, i, j;
        if (m0) memcpy(M, m0 + (size_t)bh * dk * dv, sizeof(double) * dk * dv);
        else memset(M, 0, sizeof(double) * dk * dv);
        for (t = 0; t < T; ++t) {
            const size_t tok = (size_t)bh * T + t;
            const double *qt = q + tok * dk, *kt = k + tok * dk, *vt = v + tok * dv;
            double *ot = o + tok * dv;
            delta_token(M, dk, dv, kt, vt, param_at(log_alpha, tok, 1), param_at(beta, tok, 0), param_at(bw, tok, 0), w);
            for (j = 0; j < dv; ++j) ot[j] = 0.0;
            for (i = 0; i < dk; ++i)
                for (j = 0; j < dv; ++j) ot[j] += qt[i] * M[(size_t)i * dv + j];   /* o_s = q_s M_s */
        }
        if (mT) memcpy(mT + (size_t)bh * dk * dv, M, sizeof(double) * dk * dv);
        free(M);
        free(w);
    }
    return 0;
}

/*
 * Adjoint.  Outputs dq, dk [B,H,T,dk], dv [B,H,T,dv], d_m0 [B,H,dk,dv] always;
 * d_log_alpha, d_beta, d_bw [B,H,T] where the matching input was given (pass NULL
 * otherwise).  d_mT NULL = zeros.
 */
int delta_oracle_bwd(int B, int H, int T, int dk, int dv,
                     const double *q, const double *k, const double *v,
                     const double *log_alpha, const double *beta, const double *bw,
                     const double *m0, const double *d_o, const double *d_mT,
                     double *dq, double *dkk, double *dvv,
                     double *d_log_alpha, double *d_beta, double *d_bw, double *d_m0)
{
    int bh;
    const size_t sz = (size_t)dk * dv;
    if (B <= 0 || H <= 0 || T < 0 || dk <= 0 || dv <= 0 || !q || !k || !v || !d_o || !dq || !dkk || !dvv || !d_m0)
        return -1;
    if ((log_alpha && !d_log_alpha) || (beta && !d_beta) || (bw && !d_bw)) return -1;
#pragma omp parallel for schedule(dynamic)
    for (bh = 0; bh < B * H; ++bh) {
        const int nblk = (T + BLOCK - 1) / BLOCK;
        double *keep = (double *)malloc(sizeof(double) * sz * (nblk + 1));  /* state before each block */
        double *blk = (double *)malloc(sizeof(double) * sz * (BLOCK + 1));  /* states inside one block */
        double *dM = (double *)malloc(sizeof(double) * sz);
        double *w = (double *)malloc(sizeof(double) * dv), *z = (double *)malloc(sizeof(double) * dv);
        int t, i, j, c;
        /* forward sweep: keep[c] = M before token c BLOCK */
        if (m0) memcpy(keep, m0 + (size_t)bh * sz, sizeof(double) * sz);
        else memset(keep, 0, sizeof(double) * sz);
        for (c = 0; c < nblk; ++c) {
            memcpy(keep + (size_t)(c + 1) * sz, keep + (size_t)c * sz, sizeof(double) * sz);
            for (t = c * BLOCK; t < T && t < (c + 1) * BLOCK; ++t) {
                const size_t tok = (size_t)bh * T + t;
                delta_token(keep + (size_t)(c + 1) * sz, dk, dv, k + tok * dk, v + tok * dv, param_at(log_alpha, tok, 1),
                            param_at(beta, tok, 0), param_at(bw, tok, 0), w);
            }
        }
        if (d_mT) memcpy(dM, d_mT + (size_t)bh * sz, sizeof(double) * sz);
        else memset(dM, 0, sizeof(double) * sz);
        for (c = nblk - 1; c >= 0; --c) {
            const int t0 = c * BLOCK, t1 = (c + 1) * BLOCK < T ? (c + 1) * BLOCK : T;
            /* blk[r] = M before token t0 + r; blk[t1 - t0] = M after the block's last token */
            memcpy(blk, keep + (size_t)c * sz, sizeof(double) * sz);
            for (t = t0; t < t1; ++t) {
                const size_t tok = (size_t)bh * T + t;
                double *next = blk + (size_t)(t - t0 + 1) * sz;
                memcpy(next, blk + (size_t)(t - t0) * sz, sizeof(double) * sz);
                delta_token(next, dk, dv, k + tok * dk, v + tok * dv, param_at(log_alpha, tok, 1), param_at(beta, tok, 0),
                            param_at(bw, tok, 0), w);
            }
            for (t = t1 - 1; t >= t0; --t) {
                const size_t tok = (size_t)bh * T + t;
                const double *qt = q + tok * dk, *kt = k + tok * dk, *vt = v + tok * dv, *dot = d_o + tok * dv;
                const double *Mp = blk + (size_t)(t - t0) * sz, *Mt = blk + (size_t)(t - t0 + 1) * sz;
                const double al = param_at(log_alpha, tok, 1), be = param_at(beta, tok, 0), b_ = param_at(bw, tok, 0);
                double zw = 0.0, zv = 0.0, dMMp = 0.0;
                /* o_s = q_s M_s */
                for (i = 0; i < dk; ++i) {
                    double s = 0.0;
                    for (j = 0; j < dv; ++j) {
                        s += Mt[(size_t)i * dv + j] * dot[j];
                        dM[(size_t)i * dv + j] += qt[i] * dot[j];
                    }
                    dq[tok * dk + i] = s;
                }
                /* M_s = alpha (M_{s-1} - beta k^T w) + b k^T v,  w = k M_{s-1};  z = k dM_s */
                for (j = 0; j < dv; ++j) { w[j] = 0.0; z[j] = 0.0; }
                for (i = 0; i < dk; ++i)
                    for (j = 0; j < dv; ++j) {
                        w[j] += kt[i] * Mp[(size_t)i * dv + j];
                        z[j] += kt[i] * dM[(size_t)i * dv + j];
                        dMMp += dM[(size_t)i * dv + j] * Mp[(size_t)i * dv + j];
                    }
                for (j = 0; j < dv; ++j) { zw += z[j] * w[j]; zv += z[j] * vt[j]; }
                if (d_bw) d_bw[tok] = zv;
                if (d_beta) d_beta[tok] = -al * zw;
                if (d_log_alpha) d_log_alpha[tok] = al * (dMMp - be * zw);   /* d alpha / d log alpha = alpha */
                for (j = 0; j < dv; ++j) dvv[tok * dv + j] = b_ * z[j];
                for (i = 0; i < dk; ++i) {
                    double s = 0.0;
                    for (j = 0; j < dv; ++j)
                        s += b_ * dM[(size_t)i * dv + j] * vt[j]
                             - al * be * (dM[(size_t)i * dv + j] * w[j] + Mp[(size_t)i * dv + j] * z[j]);
                    dkk[tok * dk + i] = s;
                }
                /* dM_{s-1} = alpha (dM_s - beta k^T z) */
                for (i = 0; i < dk; ++i)
                    for (j = 0; j < dv; ++j)
                        dM[(size_t)i * dv + j] = al * (dM[(size_t)i * dv + j] - be * kt[i] * z[j]);
            }
        }
        memcpy(d_m0 + (size_t)bh * sz, dM, sizeof(double) * sz);
        free(keep); free(blk); free(dM); free(w); free(z);
    }
    return 0;
}
