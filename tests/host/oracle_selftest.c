/* Host-only self test of the C oracle, meant to be built with -fsanitize=address,undefined: runs every
 * entry point on tiny inputs of all three storage types, including the empty problem and the argument
 * errors, and compares the forward result with a literal double loop.  Exit code 0 = clean. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_causal_conv(const void *, const void *, double *, int64_t, int64_t, int64_t, int64_t, int64_t, int, int);
int oracle_gated_conv(const void *, const void *, const void *, const void *, double *, int64_t, int64_t, int64_t,
                      int64_t, int64_t, int, int);
int oracle_gated_conv_points(const void *, const void *, const void *, const void *, const int64_t *, int64_t,
                             double *, int64_t, int64_t, int64_t, int64_t, int64_t, int, int);
int oracle_chain_points(const void *, const void *, const void *, const void *, const void *, const void *,
                        const void *, const int64_t *, int64_t, double *, int64_t, int64_t, int64_t, int64_t, int64_t,
                        int64_t, int64_t, int, int);
int oracle_gated_conv_bwd(const void *, const void *, const void *, const void *, const void *, double *, double *,
                          double *, double *, int64_t, int64_t, int64_t, int64_t, int64_t, int, int);

static double frand(unsigned *s) { *s = *s * 1664525u + 1013904223u; return ((*s >> 8) & 0xffff) / 32768.0 - 1.0; }

int main(void)
{
    enum { B = 2, L = 11, D = 6, LH = 4, DG = 3, N = B * L * D, G = D / DG };
    unsigned seed = 7;
    double *q = malloc(N * sizeof *q), *k = malloc(N * sizeof *k), *v = malloc(N * sizeof *v), *y = malloc(N * sizeof *y);
    double *h = malloc(G * LH * sizeof *h), *hf = malloc(D * 3 * sizeof *hf);
    float *qf = malloc(N * sizeof *qf);
    uint16_t *qb = malloc(N * sizeof *qb);
    for (int i = 0; i < N; ++i) { q[i] = frand(&seed); k[i] = frand(&seed); v[i] = frand(&seed); qf[i] = (float)q[i]; }
    for (int i = 0; i < N; ++i) { uint32_t bits; memcpy(&bits, &qf[i], 4); qb[i] = (uint16_t)(bits >> 16); }
    for (int i = 0; i < G * LH; ++i) h[i] = frand(&seed);
    for (int i = 0; i < D * 3; ++i) hf[i] = frand(&seed);
    int bad = 0;
    if (oracle_gated_conv(q, k, v, h, y, B, L, D, LH, DG, 0, 0)) bad++;
    for (int b = 0; b < B; ++b) for (int t = 0; t < L; ++t) for (int c = 0; c < D; ++c) {
        double z = 0;
        for (int j = 0; j < LH && j <= t; ++j) z += h[(c / DG) * LH + j] * k[(b * L + t - j) * D + c] * v[(b * L + t - j) * D + c];
        if (fabs(y[(b * L + t) * D + c] - q[(b * L + t) * D + c] * z) > 1e-12) bad++;
    }
    if (oracle_causal_conv(qf, h, y, B, L, D, LH, DG, 1, 0)) bad++;
    if (oracle_causal_conv(qb, h, y, B, L, D, LH, DG, 2, 0)) bad++;
    int64_t pts[6] = {0, 0, 0, B - 1, L - 1, D - 1};
    double out[2];
    if (oracle_gated_conv_points(q, k, v, h, pts, 2, out, B, L, D, LH, DG, 0, 0)) bad++;
    if (oracle_chain_points(q, k, v, hf, hf, hf, h, pts, 2, out, B, L, D, 3, 1, LH, DG, 0, 0)) bad++;
    double *dq = malloc(N * sizeof *dq), *dk = malloc(N * sizeof *dk), *dv = malloc(N * sizeof *dv), dh[G * LH];
    if (oracle_gated_conv_bwd(y, q, k, v, h, dq, dk, dv, dh, B, L, D, LH, DG, 0, 0)) bad++;
    /* empty problems and argument errors */
    if (oracle_gated_conv(q, k, v, h, y, 0, L, D, LH, DG, 0, 0)) bad++;
    if (oracle_gated_conv(q, k, v, h, y, B, 0, D, LH, DG, 0, 0)) bad++;
    if (oracle_gated_conv(NULL, k, v, h, y, B, L, D, LH, DG, 0, 0) != 1) bad++;
    if (oracle_gated_conv(q, k, v, h, y, B, L, D, LH, 4, 0, 0) != 2) bad++;
    if (oracle_gated_conv(q, k, v, h, y, B, L, D, 0, DG, 0, 0) != 2) bad++;
    if (oracle_gated_conv(q, k, v, h, y, B, L, D, LH, DG, 5, 0) != 3) bad++;
    pts[1] = L;
    if (oracle_gated_conv_points(q, k, v, h, pts, 2, out, B, L, D, LH, DG, 0, 0) != 2) bad++;
    free(q); free(k); free(v); free(y); free(h); free(hf); free(qf); free(qb); free(dq); free(dk); free(dv);
    printf("oracle selftest: %d problem(s)\n", bad);
    return bad != 0;
}
