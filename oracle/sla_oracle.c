/*
 * CPU oracle for the Softmax Linear Attention (SLA) forward pass.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against; the GPU library never calls it and shares no
 * code with it.  Only tests, the smoke check and the benchmark's cpu_baseline
 * leg may load it.
 *
 * What it computes (token by token, fp64 arithmetic, no chunking, no fusion):
 *
 *   gates      G^Q[t,:] = softmax over heads of q_logits[t,:]            (Eq. 4)
 *              G^K[t,:] = softmax over heads of k_logits[t,:] (or 1 if absent)
 *   RetNet     S_t = gamma_h S_{t-1} + (G^K k_t)^T v_t                   (Sec. 5.1, Softmax-RetNet)
 *   GLA        S_t = diag(alpha_t) S_{t-1} + (G^K k_t)^T v_t             (Sec. 5.1, Softmax-GLA)
 *   GDN        Sb  = a_t S_{t-1};  u = beta_t (G^K v_t - k_t Sb);
 *              S_t = Sb + k_t^T u                                        (Sec. 5.1, Softmax-GatedDeltaNet;
 *                                                                         a_t = 1 gives the printed equations)
 *   read-out   y_t = (G^Q q_t) S_t      (the state *after* token t)     (Eq. 5-6)
 *
 * S is [dk x dv] per (batch, head) in the paper's row-vector convention
 * (y = q S).  Decays are passed as logarithms: gamma_h = exp(log_decay[h]),
 * alpha_{t,h,d} = exp(log_decay[b,t,h,d]), a_{t,h} = exp(log_decay[b,t,h]).
 * Inputs are float32 arrays (the exact values the GPU sees, widened here to
 * fp64); outputs are fp64.
 *
 * Parity pins (tests/test_oracle_*.py): agreement with the quadratic masked
 * form of Appendix A on small inputs, with an independently written numpy
 * recurrence, gate invariants, closed forms for constant inputs, the
 * associative-recall property of the delta rule, and state chaining.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_RETNET = 0, ORACLE_GLA = 1, ORACLE_GDN = 2 };

/* softmax over n entries of x (stride 1), max-subtracted, into g. */
static void softmax_heads(const float *x, int n, double *g)
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

/* Number of threads the parallel loop over (batch, head) will use. */
int sla_oracle_threads(int requested)
{
#ifdef _OPENMP
    int avail = omp_get_max_threads();
    if (requested > 0 && requested < avail) return requested;
    return avail;
#else
    (void)requested;
    return 1;
#endif
}

/*
 * Returns 0 on success, -1 on a bad argument, -2 if memory runs out.
 *   q,k [B,T,H,dk]  v [B,T,H,dv]  q_logits,k_logits [B,T,H] (k_logits may be NULL)
 *   log_decay: RetNet [H] | GLA [B,T,H,dk] | GDN [B,T,H]
 *   beta: GDN [B,T,H], else NULL       initial_state: [B,H,dk,dv] or NULL
 *   out [B,T,H,dv]   final_state [B,H,dk,dv] (may be NULL)
 */
int sla_oracle_forward(int variant, int B, int T, int H, int dk, int dv,
                       const float *q, const float *k, const float *v,
                       const float *q_logits, const float *k_logits,
                       const float *log_decay, const float *beta,
                       const float *initial_state,
                       double *out, double *final_state, int nthreads)
{
    if (variant < 0 || variant > 2 || B < 0 || T < 0 || H < 1 || dk < 1 || dv < 1) return -1;
    if (!q || !k || !v || !q_logits || !log_decay || !out) return -1;
    if (variant == ORACLE_GDN && !beta) return -1;
    if ((size_t)B * T == 0) {
        if (final_state && B > 0) {
            size_t n = (size_t)B * H * dk * dv;
            for (size_t i = 0; i < n; ++i) final_state[i] = initial_state ? (double)initial_state[i] : 0.0;
        }
        return 0;
    }

    /* Gates for every (b,t,h): the only step that couples heads. */
    size_t ngate = (size_t)B * T * H;
    double *gq = (double *)malloc(ngate * sizeof(double));
    double *gk = (double *)malloc(ngate * sizeof(double));
    if (!gq || !gk) { free(gq); free(gk); return -2; }
    for (size_t bt = 0; bt < (size_t)B * T; ++bt) {
        softmax_heads(q_logits + bt * H, H, gq + bt * H);
        if (k_logits) softmax_heads(k_logits + bt * H, H, gk + bt * H);
        else for (int h = 0; h < H; ++h) gk[bt * H + h] = 1.0;
    }

    int fail = 0;
    int nt = sla_oracle_threads(nthreads);
    (void)nt;
#pragma omp parallel for num_threads(nt) schedule(dynamic, 1)
    for (int bh = 0; bh < B * H; ++bh) {
        int b = bh / H, h = bh % H;
        double *S = (double *)malloc((size_t)dk * dv * sizeof(double));
        double *u = (double *)malloc((size_t)dv * sizeof(double));
        if (!S || !u) {
#pragma omp atomic write
            fail = 1;
            free(S); free(u);
            continue;
        }
        for (int i = 0; i < dk * dv; ++i)
            S[i] = initial_state ? (double)initial_state[(size_t)bh * dk * dv + i] : 0.0;

        for (int t = 0; t < T; ++t) {
            size_t tok = ((size_t)b * T + t) * H + h;      /* index into [B,T,H] */
            const float *qt = q + tok * dk;
            const float *kt = k + tok * dk;
            const float *vt = v + tok * dv;
            double gQ = gq[tok], gK = gk[tok];

            if (variant == ORACLE_RETNET) {
                double gamma = exp((double)log_decay[h]);
                for (int d = 0; d < dk; ++d) {
                    double kd = gK * (double)kt[d];
                    for (int n = 0; n < dv; ++n)
                        S[d * dv + n] = gamma * S[d * dv + n] + kd * (double)vt[n];
                }
            } else if (variant == ORACLE_GLA) {
                const float *ld = log_decay + tok * dk;
                for (int d = 0; d < dk; ++d) {
                    double alpha = exp((double)ld[d]);
                    double kd = gK * (double)kt[d];
                    for (int n = 0; n < dv; ++n)
                        S[d * dv + n] = alpha * S[d * dv + n] + kd * (double)vt[n];
                }
            } else { /* gated delta rule */
                double a = exp((double)log_decay[tok]);
                double bt = (double)beta[tok];
                for (int i = 0; i < dk * dv; ++i) S[i] *= a;               /* Sb = a S_{t-1} */
                for (int n = 0; n < dv; ++n) u[n] = 0.0;
                for (int d = 0; d < dk; ++d)                               /* u <- k_t Sb */
                    for (int n = 0; n < dv; ++n) u[n] += (double)kt[d] * S[d * dv + n];
                for (int n = 0; n < dv; ++n)
                    u[n] = bt * (gK * (double)vt[n] - u[n]);               /* the rewritten value */
                for (int d = 0; d < dk; ++d)
                    for (int n = 0; n < dv; ++n)
                        S[d * dv + n] += (double)kt[d] * u[n];
            }

            double *ot = out + tok * dv;
            for (int n = 0; n < dv; ++n) ot[n] = 0.0;
            for (int d = 0; d < dk; ++d)                                   /* y <- q_t S_t */
                for (int n = 0; n < dv; ++n) ot[n] += (double)qt[d] * S[d * dv + n];
            for (int n = 0; n < dv; ++n) ot[n] *= gQ;
        }
        if (final_state)
            memcpy(final_state + (size_t)bh * dk * dv, S, (size_t)dk * dv * sizeof(double));
        free(S); free(u);
    }
    free(gq); free(gk);
    return fail ? -2 : 0;
}
