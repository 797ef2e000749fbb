/*
 * CPU oracle for the gradients of the Softmax Linear Attention (SLA) forward pass, plain C, fp64.
 *
 * TEST INFRASTRUCTURE ONLY: the GPU library never calls it and shares no code with it.
 *
 * The objective is L = sum(out * d_out) + sum(final_state * d_final_state); the forward is the token-by-token
 * recurrence of Eq. 5-6 with the updates of Sec. 5.1 (as in sla_oracle.c).  The gradients are taken the plain
 * way, by walking the recurrence backwards one token at a time and undoing each assignment:
 *
 *   read-out y_t = q_t S_t, out_t = G^Q_t y_t:
 *       dG^Q_t = d_out_t . y_t      dy = G^Q_t d_out_t      dq_t = dy S_t^T      dS += q_t^T dy
 *   RetNet / GLA step S_t = diag(alpha_t) S_{t-1} + (G^K_t k_t)^T v_t:
 *       dk_t = G^K_t dS v_t^T       dv_t = G^K_t k_t dS     dG^K_t = k_t . (dS v_t^T)
 *       dalpha_t = rowsum(dS * S_{t-1})      dlog_decay_t = alpha_t dalpha_t      dS = diag(alpha_t) dS
 *   gated delta rule step Sb = a_t S_{t-1}, u = beta_t (G^K_t v_t - k_t Sb), S_t = Sb + k_t^T u:
 *       du = k_t dS                 dk_t = dS u^T           dbeta_t = du . (G^K_t v_t - k_t Sb)
 *       dG^K_t = beta_t du . v_t    dv_t = beta_t G^K_t du  w = beta_t du
 *       dk_t -= w Sb^T              dSb = dS - k_t^T w      dlog_decay_t = sum(dSb * Sb)      dS = a_t dSb
 *   gates (Eq. 4):  dlogits = G * (dG - sum_h G dG)
 *
 * It is a second implementation of oracle/sla_backward.py (which is pinned by finite differences and autograd);
 * tests/test_oracle_backward_pins.py pins this file against that one.  States are kept at every 64th token and
 * recomputed in between, so memory stays bounded at full workload sizes.  Parallel over (batch, head).
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum { B_RETNET = 0, B_GLA = 1, B_GDN = 2 };
#define CKPT 64

static void softmax_row(const float *x, int n, double *g)
{
    double m = -INFINITY, s = 0.0;
    for (int i = 0; i < n; ++i)
        if ((double)x[i] > m) m = (double)x[i];
    for (int i = 0; i < n; ++i) {
        g[i] = exp((double)x[i] - m);
        s += g[i];
    }
    for (int i = 0; i < n; ++i) g[i] /= s;
}

/* One forward step of the recurrence on S [dk x dv] (in place). */
static void step(int variant, int dk, int dv, double *S, const float *k, const float *v, double gk, const float *ld_vec,
                 double ld_scalar, double beta, double *tmp /* dv */)
{
    if (variant == B_GDN) {
        const double a = exp(ld_scalar);
        for (int i = 0; i < dk * dv; ++i) S[i] *= a;
        for (int n = 0; n < dv; ++n) {
            double ks = 0.0;
            for (int d = 0; d < dk; ++d) ks += (double)k[d] * S[d * dv + n];
            tmp[n] = beta * (gk * (double)v[n] - ks);
        }
        for (int d = 0; d < dk; ++d)
            for (int n = 0; n < dv; ++n) S[d * dv + n] += (double)k[d] * tmp[n];
        return;
    }
    for (int d = 0; d < dk; ++d) {
        const double a = variant == B_GLA ? exp((double)ld_vec[d]) : exp(ld_scalar);
        const double kd = gk * (double)k[d];
        for (int n = 0; n < dv; ++n) S[d * dv + n] = a * S[d * dv + n] + kd * (double)v[n];
    }
}

/*
 * Layouts as in sla_oracle.c: q, k [B,T,H,dk]; v, d_out [B,T,H,dv]; logits, beta, GDN decay [B,T,H]; RetNet decay [H];
 * GLA decay [B,T,H,dk]; states [B,H,dk,dv].  Outputs (fp64): dq, dk [B,T,H,dk]; dv [B,T,H,dv]; dq_logits,
 * dk_logits (may be NULL with k_logits) [B,T,H]; dlog_decay (RetNet [H], GLA [B,T,H,dk], GDN [B,T,H]);
 * dbeta [B,T,H] (GDN, else NULL); d_initial_state [B,H,dk,dv] (may be NULL).  Returns 0, or -1 on bad arguments,
 * -2 when memory runs out.
 */
int sla_oracle_backward(int variant, int B, int T, int H, int dk, int dv, const float *q, const float *k, const float *v,
                        const float *q_logits, const float *k_logits, const float *log_decay, const float *beta,
                        const float *initial_state, const float *d_out, const float *d_final_state, double *dq,
                        double *dkk, double *dvv, double *dq_logits, double *dk_logits, double *dlog_decay, double *dbeta,
                        double *d_initial_state, int nthreads)
{
    if (variant < 0 || variant > 2 || B < 0 || T < 0 || H < 1 || dk < 1 || dv < 1) return -1;
    if (!q || !k || !v || !q_logits || !log_decay || !d_out || !dq || !dkk || !dvv || !dq_logits || !dlog_decay) return -1;
    if (variant == B_GDN && (!beta || !dbeta)) return -1;
    if ((k_logits != NULL) != (dk_logits != NULL)) return -1;
    const size_t rows = (size_t)B * T, sz = (size_t)dk * dv;
    int failed = 0;
    /* gates and raw gate gradients of every token and head */
    double *gq = (double *)malloc((rows * H ? rows * H : 1) * sizeof(double));
    double *gk = (double *)malloc((rows * H ? rows * H : 1) * sizeof(double));
    double *dgq = (double *)calloc(rows * H ? rows * H : 1, sizeof(double));
    double *dgk = (double *)calloc(rows * H ? rows * H : 1, sizeof(double));
    double *dld_bh = (double *)calloc((size_t)B * H ? (size_t)B * H : 1, sizeof(double)); /* RetNet: per (b, h) */
    if (!gq || !gk || !dgq || !dgk || !dld_bh) {
        free(gq); free(gk); free(dgq); free(dgk); free(dld_bh);
        return -2;
    }
    for (size_t r = 0; r < rows; ++r) {
        softmax_row(q_logits + r * H, H, gq + r * H);
        if (k_logits)
            softmax_row(k_logits + r * H, H, gk + r * H);
        else
            for (int h = 0; h < H; ++h) gk[r * H + h] = 1.0;
    }
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#else
    (void)nthreads;
#endif
    const int nck = (T + CKPT - 1) / CKPT;
#pragma omp parallel for schedule(dynamic, 1)
    for (int bh = 0; bh < B * H; ++bh) {
        const int b = bh / H, h = bh % H;
        double *kept = (double *)malloc(((size_t)(nck ? nck : 1)) * sz * sizeof(double)); /* state entering token c * CKPT */
        double *seg = (double *)malloc((size_t)(CKPT + 1) * sz * sizeof(double));          /* states inside a segment */
        double *dS = (double *)malloc(sz * sizeof(double));
        double *tmp = (double *)malloc((size_t)(4 * dv + 2 * dk) * sizeof(double));
        if (!kept || !seg || !dS || !tmp) {
#pragma omp atomic write
            failed = 1;
            free(kept); free(seg); free(dS); free(tmp);
            continue;
        }
        double *y = tmp, *dy = tmp + dv, *du = tmp + 2 * dv, *u = tmp + 3 * dv, *dSv = tmp + 4 * dv;
        double *S = seg; /* running state of the forward sweep lives in seg[0] */
        for (size_t i = 0; i < sz; ++i) S[i] = initial_state ? (double)initial_state[(size_t)bh * sz + i] : 0.0;
        const double ld_head = variant == B_RETNET ? (double)log_decay[h] : 0.0;
#define TOK(t) ((((size_t)b * T + (t)) * H) + h)
        for (int t = 0; t < T; ++t) {
            if (t % CKPT == 0) memcpy(kept + (size_t)(t / CKPT) * sz, S, sz * sizeof(double));
            const size_t r = TOK(t);
            step(variant, dk, dv, S, k + r * dk, v + r * dv, gk[r], variant == B_GLA ? log_decay + r * dk : NULL,
                 variant == B_GDN ? (double)log_decay[r] : ld_head, variant == B_GDN ? (double)beta[r] : 0.0, u);
        }
        for (size_t i = 0; i < sz; ++i) dS[i] = d_final_state ? (double)d_final_state[(size_t)bh * sz + i] : 0.0;
        for (int c = nck - 1; c >= 0; --c) {
            const int t0 = c * CKPT, t1 = t0 + CKPT < T ? t0 + CKPT : T;
            memcpy(seg, kept + (size_t)c * sz, sz * sizeof(double)); /* seg[i] = state entering token t0 + i */
            for (int t = t0; t < t1; ++t) {
                double *nxt = seg + (size_t)(t - t0 + 1) * sz;
                memcpy(nxt, seg + (size_t)(t - t0) * sz, sz * sizeof(double));
                const size_t r = TOK(t);
                step(variant, dk, dv, nxt, k + r * dk, v + r * dv, gk[r], variant == B_GLA ? log_decay + r * dk : NULL,
                     variant == B_GDN ? (double)log_decay[r] : ld_head, variant == B_GDN ? (double)beta[r] : 0.0, u);
            }
            for (int t = t1 - 1; t >= t0; --t) {
                const size_t r = TOK(t);
                const double *Sp = seg + (size_t)(t - t0) * sz, *St = seg + (size_t)(t - t0 + 1) * sz;
                const float *qt = q + r * dk, *kt = k + r * dk, *vt = v + r * dv, *dot = d_out + r * dv;
                /* read-out */
                double g = 0.0;
                for (int n = 0; n < dv; ++n) {
                    double acc = 0.0;
                    for (int d = 0; d < dk; ++d) acc += (double)qt[d] * St[d * dv + n];
                    y[n] = acc;
                    g += (double)dot[n] * acc;
                    dy[n] = gq[r] * (double)dot[n];
                }
                dgq[r] = g;
                for (int d = 0; d < dk; ++d) {
                    double acc = 0.0;
                    for (int n = 0; n < dv; ++n) {
                        acc += dy[n] * St[d * dv + n];
                        dS[d * dv + n] += (double)qt[d] * dy[n];
                    }
                    dq[r * dk + d] = acc;
                }
                if (variant == B_GDN) {
                    const double a = exp((double)log_decay[r]), bt = (double)beta[r];
                    double db = 0.0, dg = 0.0, dl = 0.0;
                    for (int n = 0; n < dv; ++n) {
                        double ks = 0.0, kd = 0.0;
                        for (int d = 0; d < dk; ++d) {
                            ks += (double)kt[d] * (a * Sp[d * dv + n]);
                            kd += (double)kt[d] * dS[d * dv + n];
                        }
                        const double resid = gk[r] * (double)vt[n] - ks;
                        u[n] = bt * resid;
                        du[n] = kd;
                        db += kd * resid;
                        dg += kd * (double)vt[n];
                        dvv[r * dv + n] = bt * gk[r] * kd;
                    }
                    dbeta[r] = db;
                    dgk[r] = bt * dg;
                    for (int d = 0; d < dk; ++d) {
                        double acc = 0.0;
                        for (int n = 0; n < dv; ++n) {
                            const double w = bt * du[n], Sb = a * Sp[d * dv + n];
                            acc += dS[d * dv + n] * u[n] - w * Sb;
                            const double dSb = dS[d * dv + n] - (double)kt[d] * w;
                            dl += dSb * Sb;
                            dS[d * dv + n] = a * dSb;
                        }
                        dkk[r * dk + d] = acc;
                    }
                    dlog_decay[r] = dl;
                    continue;
                }
                double dg = 0.0;
                for (int d = 0; d < dk; ++d) {
                    double acc = 0.0;
                    for (int n = 0; n < dv; ++n) acc += dS[d * dv + n] * (double)vt[n];
                    dSv[d] = acc;
                    dkk[r * dk + d] = gk[r] * acc;
                    dg += (double)kt[d] * acc;
                }
                dgk[r] = dg;
                for (int n = 0; n < dv; ++n) {
                    double acc = 0.0;
                    for (int d = 0; d < dk; ++d) acc += (double)kt[d] * dS[d * dv + n];
                    dvv[r * dv + n] = gk[r] * acc;
                }
                for (int d = 0; d < dk; ++d) {
                    const double a = variant == B_GLA ? exp((double)log_decay[r * dk + d]) : exp(ld_head);
                    double dalpha = 0.0;
                    for (int n = 0; n < dv; ++n) {
                        dalpha += dS[d * dv + n] * Sp[d * dv + n];
                        dS[d * dv + n] *= a;
                    }
                    if (variant == B_GLA)
                        dlog_decay[r * dk + d] = a * dalpha;
                    else
                        dld_bh[bh] += a * dalpha;
                }
            }
        }
#undef TOK
        if (d_initial_state) memcpy(d_initial_state + (size_t)bh * sz, dS, sz * sizeof(double));
        free(kept); free(seg); free(dS); free(tmp);
    }
    if (variant == B_RETNET)
        for (int h = 0; h < H; ++h) {
            double acc = 0.0;
            for (int b = 0; b < B; ++b) acc += dld_bh[b * H + h];
            dlog_decay[h] = acc;
        }
    /* through the head softmax */
    for (size_t r = 0; r < rows; ++r) {
        double sq = 0.0, sk = 0.0;
        for (int h = 0; h < H; ++h) {
            sq += gq[r * H + h] * dgq[r * H + h];
            sk += gk[r * H + h] * dgk[r * H + h];
        }
        for (int h = 0; h < H; ++h) {
            dq_logits[r * H + h] = gq[r * H + h] * (dgq[r * H + h] - sq);
            if (dk_logits) dk_logits[r * H + h] = gk[r * H + h] * (dgk[r * H + h] - sk);
        }
    }
    free(gq); free(gk); free(dgq); free(dgk); free(dld_bh);
    return failed ? -2 : 0;
}
