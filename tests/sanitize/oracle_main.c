/* Driver for the sanitizer build of oracle/sla_oracle.c (tests/test_sanitizers.py compiles both with
 * -fsanitize=address,undefined and runs this program): every variant on small seeded inputs, with and without
 * write-gate logits and an initial state, ragged and empty lengths.  Any out-of-bounds access, use of uninitialised
 * stack memory that the sanitizers can see, signed overflow or misaligned access aborts the run. */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

int sla_oracle_forward(int variant, int B, int T, int H, int dk, int dv, const float *q, const float *k, const float *v,
                       const float *q_logits, const float *k_logits, const float *log_decay, const float *beta,
                       const float *initial_state, double *out, double *final_state, int nthreads);

static unsigned long long state = 88172645463325252ULL;
static float rnd(void)
{ /* xorshift64: uniform in (-1, 1) */
    state ^= state << 13;
    state ^= state >> 7;
    state ^= state << 17;
    return (float)((double)(state >> 11) / 9007199254740992.0 * 2.0 - 1.0);
}
static float *fill(size_t n, float scale, float shift)
{
    float *p = (float *)malloc((n ? n : 1) * sizeof(float));
    for (size_t i = 0; i < n; ++i) p[i] = rnd() * scale + shift;
    return p;
}

static int run(int variant, int B, int T, int H, int dk, int dv, int with_kl, int with_s0)
{
    const size_t n = (size_t)B * T * H;
    float *q = fill(n * dk, 0.3f, 0.f), *k = fill(n * dk, 0.3f, 0.f), *v = fill(n * dv, 1.f, 0.f);
    float *ql = fill(n, 1.f, 0.f), *kl = with_kl ? fill(n, 1.f, 0.f) : NULL;
    const size_t nld = variant == 0 ? (size_t)H : (variant == 1 ? n * dk : n);
    float *ld = fill(nld, 0.05f, -0.06f), *beta = variant == 2 ? fill(n, 0.5f, 0.5f) : NULL;
    float *s0 = with_s0 ? fill((size_t)B * H * dk * dv, 0.5f, 0.f) : NULL;
    double *out = (double *)malloc((n * dv ? n * dv : 1) * sizeof(double));
    double *fin = (double *)malloc((size_t)B * H * dk * dv * sizeof(double));
    const int rc = sla_oracle_forward(variant, B, T, H, dk, dv, q, k, v, ql, kl, ld, beta, s0, out, fin, 2);
    int bad = rc != 0;
    for (size_t i = 0; i < n * dv; ++i) bad |= !isfinite(out[i]);
    for (size_t i = 0; i < (size_t)B * H * dk * dv; ++i) bad |= !isfinite(fin[i]);
    free(q); free(k); free(v); free(ql); free(kl); free(ld); free(beta); free(s0); free(out); free(fin);
    return bad;
}

int main(void)
{
    int bad = 0;
    for (int variant = 0; variant < 3; ++variant) {
        bad |= run(variant, 2, 37, 3, 8, 5, 1, 1);
        bad |= run(variant, 1, 1, 1, 4, 4, 0, 0);
        bad |= run(variant, 3, 0, 2, 4, 4, 1, 1); /* T = 0: the state passes through */
        bad |= run(variant, 1, 64, 7, 16, 16, 0, 1);
    }
    printf(bad ? "FAILED\n" : "oracle sanitizer run ok\n");
    return bad;
}
