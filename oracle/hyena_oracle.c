/*
 * TEST INFRASTRUCTURE -- parity oracle, not part of the product path.
 *
 * Plain fp64 CPU definition of what the Hyena-SE / Hyena-MR forward path computes:
 * a causal FIR convolution per channel (paper Sec. 3.1, Eq. 2: y_t = sum_{k<=t} h_{t-k} x_k with
 * h_k = 0 outside [0, l_h)), with one filter shared by each contiguous group of d_g channels
 * (Sec. 2.2, "Weight-sharing filter patterns"), applied to the pre-gated signal u = k (.) v and
 * post-gated by q (Sec. 2.1, Eq. 1, last line; Algorithm 1 fuses both gates around the convolution).
 * The blocked / two-stage forms of Sec. 3.1-3.2 are exact re-bracketings of this sum, so the oracle
 * is the sum itself: no blocking, no fusion, no reordering. Ascending tap index, fp64 accumulate.
 *
 * Layout: activations [B, L, D] row-major (D contiguous); filters [D/d_g, l_h] row-major, tap 0
 * multiplies the current sample. Zero left padding for every batch item on its own.
 *
 * Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may call this file.
 * It shares no code, header, table or helper with the HIP path.
 */
#include <stddef.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_F64 = 0, ORC_F32 = 1, ORC_BF16 = 2 };

/* Exact widening of one stored element to double. bf16 is the upper half of an IEEE binary32. */
static inline double orc_load(const void *p, int dt, size_t i)
{
    if (dt == ORC_F64)
        return ((const double *)p)[i];
    if (dt == ORC_F32)
        return (double)((const float *)p)[i];
    uint32_t bits = (uint32_t)((const uint16_t *)p)[i] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

static int orc_check(const void *a, const void *b, const void *c, int64_t B, int64_t L, int64_t D,
                     int64_t lh, int64_t dg, int dt, int hdt)
{
    if (!a || !b || !c)
        return 1;
    if (B < 0 || L < 0 || D < 0 || lh < 1 || dg < 1)
        return 2;
    if (D % dg != 0)
        return 2;
    if (dt < 0 || dt > 2 || hdt < 0 || hdt > 1)
        return 3;
    return 0;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Eq. 2 + grouping: y[b,t,c] = sum_{j=0}^{min(lh-1,t)} h[c/dg, j] * x[b,t-j,c].
 * This is the featurizer convolution of Eq. 1 (first three lines): no gating.
 */
int oracle_causal_conv(const void *x, const void *h, double *y, int64_t B, int64_t L, int64_t D,
                       int64_t lh, int64_t dg, int x_dtype, int h_dtype)
{
    int rc = orc_check(x, h, y, B, L, D, lh, dg, x_dtype, h_dtype);
    if (rc)
        return rc;
    int64_t rows = B * L;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        int64_t b = r / L, t = r % L;
        for (int64_t c = 0; c < D; ++c) {
            int64_t g = c / dg;
            double z = 0.0;
            for (int64_t j = 0; j < lh && j <= t; ++j) {
                size_t src = (size_t)((b * L + (t - j)) * D + c);
                z += orc_load(h, h_dtype, (size_t)(g * lh + j)) * orc_load(x, x_dtype, src);
            }
            y[(size_t)(r * D + c)] = z;
        }
    }
    return 0;
}

/*
 * Eq. 1 (last line, without the dense M) with the inner Toeplitz operator G given by Eq. 2:
 * y[b,t,c] = q[b,t,c] * sum_{j=0}^{min(lh-1,t)} h[c/dg, j] * k[b,t-j,c] * v[b,t-j,c].
 */
int oracle_gated_conv(const void *q, const void *k, const void *v, const void *h, double *y,
                      int64_t B, int64_t L, int64_t D, int64_t lh, int64_t dg, int x_dtype,
                      int h_dtype)
{
    int rc = orc_check(q, k, v, B, L, D, lh, dg, x_dtype, h_dtype);
    if (rc)
        return rc;
    if (!h || !y)
        return 1;
    int64_t rows = B * L;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        int64_t b = r / L, t = r % L;
        for (int64_t c = 0; c < D; ++c) {
            int64_t g = c / dg;
            double z = 0.0;
            for (int64_t j = 0; j < lh && j <= t; ++j) {
                size_t src = (size_t)((b * L + (t - j)) * D + c);
                double u = orc_load(k, x_dtype, src) * orc_load(v, x_dtype, src);
                z += orc_load(h, h_dtype, (size_t)(g * lh + j)) * u;
            }
            size_t dst = (size_t)(r * D + c);
            y[dst] = orc_load(q, x_dtype, dst) * z;
        }
    }
    return 0;
}

/*
 * Same sum as oracle_gated_conv, evaluated only at n listed outputs; pts holds (b,t,c) triples.
 * Lets a full-size tensor be spot-checked one output at a time.
 */
int oracle_gated_conv_points(const void *q, const void *k, const void *v, const void *h,
                             const int64_t *pts, int64_t n, double *out, int64_t B, int64_t L,
                             int64_t D, int64_t lh, int64_t dg, int x_dtype, int h_dtype)
{
    int rc = orc_check(q, k, v, B, L, D, lh, dg, x_dtype, h_dtype);
    if (rc)
        return rc;
    if (!h || !pts || !out)
        return 1;
    for (int64_t i = 0; i < n; ++i) {
        int64_t b = pts[3 * i], t = pts[3 * i + 1], c = pts[3 * i + 2];
        if (b < 0 || b >= B || t < 0 || t >= L || c < 0 || c >= D)
            return 2;
    }
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        int64_t b = pts[3 * i], t = pts[3 * i + 1], c = pts[3 * i + 2];
        int64_t g = c / dg;
        double z = 0.0;
        for (int64_t j = 0; j < lh && j <= t; ++j) {
            size_t src = (size_t)((b * L + (t - j)) * D + c);
            double u = orc_load(k, x_dtype, src) * orc_load(v, x_dtype, src);
            z += orc_load(h, h_dtype, (size_t)(g * lh + j)) * u;
        }
        out[i] = orc_load(q, x_dtype, (size_t)((b * L + t) * D + c)) * z;
    }
    return 0;
}

/* One featurized sample: x'[b,s,c] = sum_{i<=min(lf-1,s)} hf[c/dgf, i] * x[b,s-i,c]  (Eq. 1, Eq. 2). */
static double orc_featurized(const void *x, const void *hf, int64_t b, int64_t s, int64_t c,
                             int64_t L, int64_t D, int64_t lf, int64_t dgf, int x_dtype, int h_dtype)
{
    double a = 0.0;
    int64_t gf = c / dgf;
    for (int64_t i = 0; i < lf && i <= s; ++i)
        a += orc_load(hf, h_dtype, (size_t)(gf * lf + i)) *
             orc_load(x, x_dtype, (size_t)((b * L + (s - i)) * D + c));
    return a;
}

/*
 * The operator chain of Eq. 1 without the dense projections, at n listed outputs:
 * q' = h_q * q, k' = h_k * k, v' = h_v * v (featurizers, length lf, group dgf), then
 * y = q' (.) (h * (k' (.) v')) with the inner filter of length lh and group dg.
 * Every intermediate stays in fp64.
 */
int oracle_chain_points(const void *q, const void *k, const void *v, const void *hq, const void *hk,
                        const void *hv, const void *h, const int64_t *pts, int64_t n, double *out,
                        int64_t B, int64_t L, int64_t D, int64_t lf, int64_t dgf, int64_t lh,
                        int64_t dg, int x_dtype, int h_dtype)
{
    int rc = orc_check(q, k, v, B, L, D, lh, dg, x_dtype, h_dtype);
    if (rc)
        return rc;
    if (!hq || !hk || !hv || !h || !pts || !out)
        return 1;
    if (lf < 1 || dgf < 1 || D % dgf != 0)
        return 2;
    for (int64_t i = 0; i < n; ++i) {
        int64_t b = pts[3 * i], t = pts[3 * i + 1], c = pts[3 * i + 2];
        if (b < 0 || b >= B || t < 0 || t >= L || c < 0 || c >= D)
            return 2;
    }
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        int64_t b = pts[3 * i], t = pts[3 * i + 1], c = pts[3 * i + 2];
        int64_t g = c / dg;
        double z = 0.0;
        for (int64_t j = 0; j < lh && j <= t; ++j) {
            double kf = orc_featurized(k, hk, b, t - j, c, L, D, lf, dgf, x_dtype, h_dtype);
            double vf = orc_featurized(v, hv, b, t - j, c, L, D, lf, dgf, x_dtype, h_dtype);
            z += orc_load(h, h_dtype, (size_t)(g * lh + j)) * (kf * vf);
        }
        out[i] = orc_featurized(q, hq, b, t, c, L, D, lf, dgf, x_dtype, h_dtype) * z;
    }
    return 0;
}

/*
 * Backward of oracle_gated_conv: gradients of  y = q (.) (h * (k (.) v))  (Eq. 1 last line, Eq. 2) with respect
 * to q, k, v and h, given dy = dLoss/dy.  The paper describes its backward kernel only by structure (App. A.4:
 * a first pass with the forward's blocking that also accumulates partial filter gradients, a second pass that
 * reduces them); what it must compute is the chain rule of the forward definition, written out here term by
 * term in fp64:
 *     u = k*v,  z[t] = sum_j h[j] u[t-j]
 *     dq[t] = dy[t] * z[t]
 *     g[t]  = dy[t] * q[t]                               (= dLoss/dz)
 *     du[s] = sum_{j<lh, s+j<L} h[j] * g[s+j]            (the transposed, anti-causal convolution)
 *     dk[s] = du[s] * v[s],   dv[s] = du[s] * k[s]
 *     dh[g', j] = sum_b sum_{c in group g'} sum_{t>=j} g[b,t,c] * u[b,t-j,c]
 * dq, dk, dv: [B,L,D] fp64; dh: [D/dg, lh] fp64 (summed over batch, time and the channels of the group).
 */
int oracle_gated_conv_bwd(const void *dy, const void *q, const void *k, const void *v, const void *h,
                          double *dq, double *dk, double *dv, double *dh, int64_t B, int64_t L, int64_t D,
                          int64_t lh, int64_t dg, int x_dtype, int h_dtype)
{
    int rc = orc_check(q, k, v, B, L, D, lh, dg, x_dtype, h_dtype);
    if (rc)
        return rc;
    if (!dy || !h || !dq || !dk || !dv || !dh)
        return 1;
    int64_t rows = B * L;
    int64_t G = D / dg;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        int64_t b = r / L, t = r % L;
        for (int64_t c = 0; c < D; ++c) {
            int64_t g = c / dg;
            size_t at = (size_t)(r * D + c);
            /* dq: forward convolution value z[t] */
            double z = 0.0;
            for (int64_t j = 0; j < lh && j <= t; ++j) {
                size_t src = (size_t)((b * L + (t - j)) * D + c);
                z += orc_load(h, h_dtype, (size_t)(g * lh + j)) * (orc_load(k, x_dtype, src) * orc_load(v, x_dtype, src));
            }
            dq[at] = orc_load(dy, x_dtype, at) * z;
            /* du at this position: taps reach forward in time */
            double du = 0.0;
            for (int64_t j = 0; j < lh && t + j < L; ++j) {
                size_t fut = (size_t)((b * L + (t + j)) * D + c);
                du += orc_load(h, h_dtype, (size_t)(g * lh + j)) * (orc_load(dy, x_dtype, fut) * orc_load(q, x_dtype, fut));
            }
            dk[at] = du * orc_load(v, x_dtype, at);
            dv[at] = du * orc_load(k, x_dtype, at);
        }
    }
    /* filter gradient: one (group, tap) at a time, plain triple sum */
#pragma omp parallel for schedule(static) collapse(2)
    for (int64_t g = 0; g < G; ++g) {
        for (int64_t j = 0; j < lh; ++j) {
            double s = 0.0;
            for (int64_t b = 0; b < B; ++b)
                for (int64_t c = g * dg; c < (g + 1) * dg; ++c)
                    for (int64_t t = j; t < L; ++t) {
                        size_t at = (size_t)((b * L + t) * D + c);
                        size_t src = (size_t)((b * L + (t - j)) * D + c);
                        s += (orc_load(dy, x_dtype, at) * orc_load(q, x_dtype, at)) *
                             (orc_load(k, x_dtype, src) * orc_load(v, x_dtype, src));
                    }
            dh[(size_t)(g * lh + j)] = s;
        }
    }
    return 0;
}

/*
 * Backward of oracle_causal_conv, the featurizer convolutions of Eq. 1 (x' = h * x with Eq. 2, no gates): the
 * chain rule of that definition, given dy = dLoss/dx', term by term in fp64:
 *     dx[s]     = sum_{j<lh, s+j<L} h[j] * dy[s+j]            (the transposed, anti-causal convolution)
 *     dh[g', j] = sum_b sum_{c in group g'} sum_{t>=j} dy[b,t,c] * x[b,t-j,c]
 * dx: [B,L,D] fp64; dh: [D/dg, lh] fp64.
 */
int oracle_causal_conv_bwd(const void *dy, const void *x, const void *h, double *dx, double *dh, int64_t B,
                           int64_t L, int64_t D, int64_t lh, int64_t dg, int x_dtype, int h_dtype)
{
    int rc = orc_check(dy, x, h, B, L, D, lh, dg, x_dtype, h_dtype);
    if (rc)
        return rc;
    if (!dx || !dh)
        return 1;
    int64_t rows = B * L;
    int64_t G = D / dg;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        int64_t b = r / L, s = r % L;
        for (int64_t c = 0; c < D; ++c) {
            int64_t g = c / dg;
            double acc = 0.0;
            for (int64_t j = 0; j < lh && s + j < L; ++j)
                acc += orc_load(h, h_dtype, (size_t)(g * lh + j)) * orc_load(dy, x_dtype, (size_t)((b * L + (s + j)) * D + c));
            dx[(size_t)(r * D + c)] = acc;
        }
    }
#pragma omp parallel for schedule(static) collapse(2)
    for (int64_t g = 0; g < G; ++g) {
        for (int64_t j = 0; j < lh; ++j) {
            double acc = 0.0;
            for (int64_t b = 0; b < B; ++b)
                for (int64_t c = g * dg; c < (g + 1) * dg; ++c)
                    for (int64_t t = j; t < L; ++t)
                        acc += orc_load(dy, x_dtype, (size_t)((b * L + t) * D + c)) *
                               orc_load(x, x_dtype, (size_t)((b * L + (t - j)) * D + c));
            dh[(size_t)(g * lh + j)] = acc;
        }
    }
    return 0;
}

/*
 * Hyena-LI in its recurrent form (Sec. 2.1: the long implicit filter is a sum of real exponentials,
 * h_t = sum_n R_n lambda_n^(t-1), t from 1, and the operator can be evaluated as a recurrence).  Per channel c with
 * group g = c / dg and u = k (.) v:
 *     s_n[t] = lambda[g,n] * s_n[t-1] + u[t],   s_n[-1] = 0            (so s_n[t] = sum_{i<=t} lambda_n^(t-i) u[i])
 *     y[t]   = q[t] * sum_n R[g,n] * s_n[t]
 * which is the sum of the definition (oracle_gated_conv with the filter sum_n R_n lambda_n^j as long as the
 * sequence) with the order of its two sums exchanged: the same result up to fp64 rounding, at a cost linear in L.
 * It exists so that sequences too long for the quadratic definition can be compared over every output; the
 * tests pin it to the definition (small shapes in full, long sequences at sampled outputs).
 * R, lam: [D/dg, order].  One time step at a time, channels in the inner loop (they are contiguous in memory).
 */
int oracle_li_recurrent(const void *q, const void *k, const void *v, const void *R, const void *lam, double *y,
                        double *state, int64_t B, int64_t L, int64_t D, int64_t order, int64_t dg, int x_dtype,
                        int h_dtype)
{
    int rc = orc_check(q, k, v, B, L, D, order, dg, x_dtype, h_dtype);
    if (rc)
        return rc;
    if (!R || !lam || !y || !state)
        return 1;
    /* state: caller-provided scratch of B * D * order doubles, s_n of every (b, c) */
    int64_t seqs = B * D;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < seqs * order; ++i)
        state[i] = 0.0;
    enum { BLOCK = 32 }; /* channels handled by one thread at a time */
    int64_t nblk = (D + BLOCK - 1) / BLOCK;
#pragma omp parallel for schedule(static) collapse(2)
    for (int64_t b = 0; b < B; ++b) {
        for (int64_t cb = 0; cb < nblk; ++cb) {
            int64_t c_lo = cb * BLOCK, c_hi = c_lo + BLOCK < D ? c_lo + BLOCK : D;
            for (int64_t t = 0; t < L; ++t) {
                for (int64_t c = c_lo; c < c_hi; ++c) {
                    int64_t g = c / dg;
                    size_t at = (size_t)((b * L + t) * D + c);
                    double u = orc_load(k, x_dtype, at) * orc_load(v, x_dtype, at);
                    double *s = state + (size_t)((b * D + c) * order);
                    double z = 0.0;
                    for (int64_t n = 0; n < order; ++n) {
                        s[n] = orc_load(lam, h_dtype, (size_t)(g * order + n)) * s[n] + u;
                        z += orc_load(R, h_dtype, (size_t)(g * order + n)) * s[n];
                    }
                    y[at] = orc_load(q, x_dtype, at) * z;
                }
            }
        }
    }
    return 0;
}
