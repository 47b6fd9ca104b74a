/* Drives every entry point of the CPU oracle on small inputs, edge cases included (T = 0, V = 1, chosen ids out
 * of range, all-masked batches, a denominator of 0), so that a build with -fsanitize=address,undefined can
 * report out-of-bounds accesses, misaligned or overflowing arithmetic and leaks.  Prints "ok" on completion. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct { int64_t n_tokens, n_clipped, n_bad_index, n_negative_staleness; double iw_min, iw_max; } oracle_stats;
void a3po_oracle_token_logprobs(const void *, int, int64_t, int64_t, int64_t, const int32_t *, double *, double *, void *);
void a3po_oracle_alpha(const int32_t *, int32_t, int64_t, double *);
void a3po_oracle_proximal_interp(const double *, const double *, const int32_t *, int32_t, int64_t, double *, double *);
int a3po_oracle_grpo_advantages(const double *, int64_t, int32_t, double, const int32_t *, int64_t, double *, double *);
void a3po_oracle_decoupled_clip(const double *, const double *, const double *, const double *, const uint8_t *, double,
                                double, int64_t, double *, double *, double *, double *, uint8_t *, double *, oracle_stats *);
void a3po_oracle_surrogate(const double *, const double *, const int32_t *, int32_t, const double *, const uint8_t *, double,
                           double, int64_t, double *, double *, double *, double *, double *, uint8_t *, double *, oracle_stats *);
void a3po_oracle_dlogits_rows(const void *, int, int64_t, int64_t, const int32_t *, const double *, const double *,
                              const int64_t *, int64_t, double *);
void a3po_oracle_loss_fwd_bwd(const void *, int, int64_t, int64_t, int64_t, const int32_t *, const double *, const int32_t *,
                              int32_t, const double *, const uint8_t *, double, double, double *, double *, double *,
                              double *, uint8_t *, uint8_t *, double *, double *, oracle_stats *);
void a3po_oracle_lmhead_logits(const uint16_t *, const uint16_t *, int64_t, int64_t, const int64_t *, int64_t, double *);
void a3po_oracle_lmhead_backward(const double *, const uint16_t *, const uint16_t *, int64_t, int64_t, int64_t, double *, double *);
void a3po_oracle_entropy(const void *, int, int64_t, int64_t, int64_t, double *);

static uint32_t rng = 12345u;
static double unif(void) { rng = rng * 1664525u + 1013904223u; return (rng >> 8) / 16777216.0; }

static void whole_path(int dt, int64_t T, int64_t V, int64_t ld, int all_masked)
{
    const size_t esz = dt == 0 ? 4 : 2;
    void *z = malloc((size_t)(T * ld + 1) * esz);
    for (int64_t i = 0; i < T * ld; ++i) {
        float f = (float)(unif() * 8 - 4);
        if (dt == 0) ((float *)z)[i] = f;
        else { uint32_t u; memcpy(&u, &f, 4); ((uint16_t *)z)[i] = (uint16_t)(u >> 16); }
    }
    int32_t *y = malloc((size_t)(T + 1) * 4), *ver = malloc((size_t)(T + 1) * 4);
    double *lb = malloc((size_t)(T + 1) * 8), *A = malloc((size_t)(T + 1) * 8);
    uint8_t *m = malloc((size_t)T + 1), *eff = malloc((size_t)T + 1), *cl = malloc((size_t)T + 1);
    double *logp = malloc((size_t)(T + 1) * 8), *lse = malloc((size_t)(T + 1) * 8), *lp = malloc((size_t)(T + 1) * 8);
    double *g = malloc((size_t)(T + 1) * 8), *dz = malloc((size_t)(T * V + 1) * 8), *H = malloc((size_t)(T + 1) * 8);
    for (int64_t t = 0; t < T; ++t) {
        y[t] = (int32_t)(unif() * (double)(V + 2)) - 1;   /* -1 and V occur: out of range on both sides */
        ver[t] = 10 - (int32_t)(unif() * 6) + (t % 7 == 0 ? 4 : 0);   /* some negative staleness */
        lb[t] = -unif() * 5;
        A[t] = unif() * 2 - 1;
        m[t] = all_masked ? 0 : (uint8_t)(unif() < 0.8);
    }
    double loss;
    oracle_stats st;
    a3po_oracle_loss_fwd_bwd(z, dt, T, V, ld, y, lb, ver, 10, A, m, 0.2, 0.0, logp, lse, lp, g, eff, cl, dz, &loss, &st);
    a3po_oracle_loss_fwd_bwd(z, dt, T, V, ld, y, lb, ver, 10, A, m, 0.2, 37.0, logp, lse, lp, g, eff, cl, NULL, &loss, NULL);
    a3po_oracle_entropy(z, dt, T, V, ld, H);
    if (!(loss == loss)) { printf("NaN loss\n"); exit(2); }
    free(z); free(y); free(ver); free(lb); free(A); free(m); free(eff); free(cl); free(logp); free(lse); free(lp); free(g);
    free(dz); free(H);
}

int main(void)
{
    whole_path(0, 0, 5, 5, 0);       /* empty batch */
    whole_path(0, 7, 1, 1, 0);       /* single-entry vocabulary */
    whole_path(0, 9, 13, 16, 0);     /* padded stride */
    whole_path(1, 9, 13, 13, 0);     /* bfloat16 bit patterns */
    whole_path(1, 6, 31, 40, 1);     /* everything masked */

    /* per-token functions on their own, NULL optional outputs */
    enum { N = 11 };
    int32_t ver[N]; double lt[N], lb[N], lp[N], al[N], A[N], iw[N], r[N], obj[N], g[N]; uint8_t m[N], cl[N];
    for (int i = 0; i < N; ++i) { ver[i] = 20 - i; lt[i] = -unif() * 3; lb[i] = -unif() * 3; A[i] = unif() - 0.5; m[i] = i & 1; }
    ver[0] = INT32_MIN; ver[1] = INT32_MAX;     /* extreme versions: 64-bit staleness */
    a3po_oracle_alpha(ver, INT32_MAX, N, al);
    a3po_oracle_proximal_interp(lb, lt, ver, 20, N, lp, NULL);
    double loss; oracle_stats st;
    a3po_oracle_decoupled_clip(lt, lb, lp, A, m, 0.2, 0.0, N, iw, r, obj, g, cl, &loss, &st);
    a3po_oracle_decoupled_clip(lt, lb, lp, A, m, 0.2, 0.0, N, NULL, NULL, NULL, NULL, NULL, NULL, NULL);
    a3po_oracle_surrogate(lt, lb, ver, 20, A, m, 0.2, 5.0, N, lp, NULL, NULL, NULL, g, NULL, &loss, &st);
    a3po_oracle_surrogate(lt, lb, ver, 20, A, m, 0.2, 0.0, 0, lp, iw, r, obj, g, cl, &loss, &st);   /* T = 0 */

    double R[8] = {1, 0, 0, 1, 1, 1, 1, 1}, as[8], at[5]; int32_t sid[5] = {0, 3, 4, 7, 7};
    if (a3po_oracle_grpo_advantages(R, 8, 4, 1e-6, sid, 5, as, at) != 0) return 3;
    if (a3po_oracle_grpo_advantages(R, 8, 3, 1e-6, NULL, 0, as, NULL) != -1) return 4;      /* 8 % 3 != 0 */
    sid[2] = 8;
    if (a3po_oracle_grpo_advantages(R, 8, 4, 1e-6, sid, 5, as, at) != -1) return 5;        /* sequence id out of range */

    /* gradient rows of a subset, LM-head products */
    float z[3 * 6]; int32_t y[3] = {0, 5, 2}; double lse[3], logp[3], gg[3] = {0.5, 0, -1}, dz[2 * 6]; int64_t rows[2] = {2, 0};
    for (int i = 0; i < 18; ++i) z[i] = (float)(unif() * 4);
    a3po_oracle_token_logprobs(z, 0, 3, 6, 6, y, logp, lse, NULL);
    a3po_oracle_dlogits_rows(z, 0, 6, 6, y, lse, gg, rows, 2, dz);
    uint16_t h[4 * 8], W[5 * 8]; double zz[2 * 5], dzz[4 * 5], dh[4 * 8], dW[5 * 8]; int64_t hr[2] = {3, 1};
    for (int i = 0; i < 32; ++i) h[i] = (uint16_t)(0x3f00 + (i & 63));
    for (int i = 0; i < 40; ++i) W[i] = (uint16_t)(0xbe00 + (i & 63));
    for (int i = 0; i < 20; ++i) dzz[i] = unif() - 0.5;
    a3po_oracle_lmhead_logits(h, W, 8, 5, hr, 2, zz);
    a3po_oracle_lmhead_backward(dzz, h, W, 4, 8, 5, dh, dW);
    a3po_oracle_lmhead_backward(dzz, h, W, 4, 8, 5, NULL, NULL);
    printf("ok\n");
    return 0;
}
