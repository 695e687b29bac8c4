/*
 * qn_oracle.c -- plain double-precision CPU evaluation of the server-side
 * quasi-Newton step (Arnold & Wang, Section 2, eq. (1)-(4)).
 *
 * TEST INFRASTRUCTURE ONLY: slow on purpose, no blocking, no fusion, no
 * threads; every routine is the paper's definition written out so that it can
 * be checked against the text by eye.  It shares nothing with the HIP library.
 * See qn_oracle.h for layouts and for what pins each routine.
 */
#include "qn_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

/* Exact widening of one stored element to double. */
static double elem(const void *base, int dtype, int64_t idx)
{
    if (dtype == QNO_F32)
        return (double)((const float *)base)[idx];
    if (dtype == QNO_BF16) {
        /* bfloat16 is the upper half of an IEEE binary32. */
        uint32_t bits = (uint32_t)((const uint16_t *)base)[idx] << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return (double)f;
    }
    if (dtype == QNO_F16) {
        /* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits. */
        const uint16_t h = ((const uint16_t *)base)[idx];
        const int sign = h >> 15, e = (h >> 10) & 0x1f, frac = h & 0x3ff;
        double v;
        if (e == 0)
            v = ldexp((double)frac, -24);                  /* zero and subnormals */
        else if (e == 31)
            v = frac ? NAN : INFINITY;
        else
            v = ldexp((double)(frac | 0x400), e - 25);     /* (1 + frac/1024) 2^(e-15) */
        return sign ? -v : v;
    }
    return ((const double *)base)[idx];
}

/* Section 2: g_bar = (1/m) sum_k grad J(theta_k), theta_bar likewise. */
void qno_row_means(const void *X, int dtype, int64_t n, int m, int64_t ld,
                   double *mean)
{
    for (int64_t i = 0; i < n; ++i) {
        double s = 0.0;
        for (int k = 0; k < m; ++k)
            s += elem(X, dtype, (int64_t)k * ld + i);
        mean[i] = s / (double)m;
    }
}

/* Section 2: columns of G and Theta are the worker vectors minus the mean. */
void qno_centre(const void *X, int dtype, int64_t n, int m, int64_t ld,
                const double *mean, double *Xc)
{
    for (int k = 0; k < m; ++k)
        for (int64_t i = 0; i < n; ++i)
            Xc[(int64_t)k * n + i] = elem(X, dtype, (int64_t)k * ld + i) - mean[i];
}

/* C[a,b] = sum_i G[i,a] G[i,b]. */
void qno_gram(const double *G, int64_t n, int m, double *C)
{
    for (int a = 0; a < m; ++a)
        for (int b = 0; b < m; ++b) {
            double s = 0.0;
            for (int64_t i = 0; i < n; ++i)
                s += G[(int64_t)a * n + i] * G[(int64_t)b * n + i];
            C[b * m + a] = s;
        }
}

/* w[k] = sum_i G[i,k] z[i]. */
void qno_gemv_t(const double *G, int64_t n, int m, const double *z, double *w)
{
    for (int k = 0; k < m; ++k) {
        double s = 0.0;
        for (int64_t i = 0; i < n; ++i)
            s += G[(int64_t)k * n + i] * z[i];
        w[k] = s;
    }
}

/*
 * Classical cyclic Jacobi: sweep over all pairs p < q in row order, annihilate
 * A[p,q] with a plane rotation, accumulate the rotations in V.  Stops when the
 * off-diagonal Frobenius norm is below 1e-15 of the matrix norm.
 */
int qno_jacobi_eigh(const double *C, int m, double *mu, double *V)
{
    double *A = (double *)malloc(sizeof(double) * (size_t)m * (size_t)m);
    if (!A)
        return -1;
    /* work on the symmetric part so that an input that is only symmetric up
     * to rounding is handled consistently */
    for (int a = 0; a < m; ++a)
        for (int b = 0; b < m; ++b)
            A[b * m + a] = 0.5 * (C[b * m + a] + C[a * m + b]);
    for (int a = 0; a < m; ++a)
        for (int b = 0; b < m; ++b)
            V[b * m + a] = (a == b) ? 1.0 : 0.0;

    double total = 0.0;
    for (int a = 0; a < m * m; ++a)
        total += A[a] * A[a];
    const double tol2 = 1e-30 * total;

    int sweeps = 0, converged = 0;
    for (; sweeps <= 60; ++sweeps) {
        double off = 0.0;
        for (int p = 0; p < m; ++p)
            for (int q = 0; q < m; ++q)
                if (p != q)
                    off += A[q * m + p] * A[q * m + p];
        if (off <= tol2) {
            converged = 1;
            break;
        }
        for (int p = 0; p < m - 1; ++p)
            for (int q = p + 1; q < m; ++q) {
                const double apq = A[q * m + p];
                if (apq == 0.0)
                    continue;
                const double app = A[p * m + p], aqq = A[q * m + q];
                const double zeta = (aqq - app) / (2.0 * apq);
                const double t = (zeta >= 0.0 ? 1.0 : -1.0) /
                                 (fabs(zeta) + sqrt(zeta * zeta + 1.0));
                const double cs = 1.0 / sqrt(t * t + 1.0);
                const double sn = t * cs;
                /* A <- J^T A J with J = [[cs, sn], [-sn, cs]] on (p, q) */
                for (int r = 0; r < m; ++r) { /* columns p, q */
                    const double arp = A[p * m + r], arq = A[q * m + r];
                    A[p * m + r] = cs * arp - sn * arq;
                    A[q * m + r] = sn * arp + cs * arq;
                }
                for (int r = 0; r < m; ++r) { /* rows p, q */
                    const double apr = A[r * m + p], aqr = A[r * m + q];
                    A[r * m + p] = cs * apr - sn * aqr;
                    A[r * m + q] = sn * apr + cs * aqr;
                }
                for (int r = 0; r < m; ++r) {
                    const double vrp = V[p * m + r], vrq = V[q * m + r];
                    V[p * m + r] = cs * vrp - sn * vrq;
                    V[q * m + r] = sn * vrp + cs * vrq;
                }
            }
    }

    /* sort eigenvalues descending (selection sort, carrying the columns) */
    for (int k = 0; k < m; ++k)
        mu[k] = A[k * m + k];
    for (int k = 0; k < m - 1; ++k) {
        int best = k;
        for (int l = k + 1; l < m; ++l)
            if (mu[l] > mu[best])
                best = l;
        if (best != k) {
            double t = mu[k];
            mu[k] = mu[best];
            mu[best] = t;
            for (int r = 0; r < m; ++r) {
                t = V[k * m + r];
                V[k * m + r] = V[best * m + r];
                V[best * m + r] = t;
            }
        }
    }
    free(A);
    return converged ? sweeps : -1;
}

void qno_sigma_from_mu(const double *mu, int m, double *sigma)
{
    for (int k = 0; k < m; ++k)
        sigma[k] = mu[k] > 0.0 ? sqrt(mu[k]) : 0.0;
}

/* j = number of leading sigma_k with sigma_k >= lambda * sigma_1. */
int qno_select_j(const double *sigma, int m, double lambda)
{
    if (m < 1 || !(sigma[0] > 0.0) || !isfinite(sigma[0]))
        return 0;
    int j = 0;
    while (j < m && sigma[j] >= lambda * sigma[0])
        ++j;
    return j;
}

void qno_apply_Hinv_literal(const double *Theta, const double *G, int64_t n,
                            int m, const double *sigma, const double *V, int j,
                            const double *z, double *out)
{
    double *u = (double *)malloc(sizeof(double) * (size_t)n);
    double *y = (double *)malloc(sizeof(double) * (size_t)n);
    double *zperp = (double *)malloc(sizeof(double) * (size_t)n);
    double *mapped = (double *)calloc((size_t)n, sizeof(double));
    for (int64_t i = 0; i < n; ++i)
        zperp[i] = z[i];

    for (int k = 0; k < j; ++k) {
        const double *vk = V + (size_t)k * m;
        /* u_k = G v_k / ||G v_k||_2 ,  y_k = Theta v_k */
        double nrm2 = 0.0;
        for (int64_t i = 0; i < n; ++i) {
            double gu = 0.0, ty = 0.0;
            for (int l = 0; l < m; ++l) {
                gu += G[(int64_t)l * n + i] * vk[l];
                ty += Theta[(int64_t)l * n + i] * vk[l];
            }
            u[i] = gu;
            y[i] = ty;
            nrm2 += gu * gu;
        }
        const double nrm = sqrt(nrm2);
        for (int64_t i = 0; i < n; ++i)
            u[i] /= nrm;
        /* alpha_k = z^T u_k */
        double alpha = 0.0;
        for (int64_t i = 0; i < n; ++i)
            alpha += z[i] * u[i];
        /* z_perp = z - sum alpha_k u_k ;  sum alpha_k sigma_k^-1 y_k */
        for (int64_t i = 0; i < n; ++i) {
            zperp[i] -= alpha * u[i];
            mapped[i] += alpha / sigma[k] * y[i];
        }
    }
    for (int64_t i = 0; i < n; ++i)
        out[i] = zperp[i] + mapped[i];
    free(u);
    free(y);
    free(zperp);
    free(mapped);
}

int qno_update_literal(const void *thetas, const void *grads, int dtype,
                       int64_t n, int m, int64_t ld, double tau, double lambda,
                       double *theta_new, int *j_out, double *C, double *w,
                       double *sigma, double *V)
{
    const size_t nm = (size_t)n * (size_t)m, mm = (size_t)m * (size_t)m;
    double *theta_bar = (double *)malloc(sizeof(double) * (size_t)n);
    double *g_bar = (double *)malloc(sizeof(double) * (size_t)n);
    double *Theta = (double *)malloc(sizeof(double) * nm);
    double *G = (double *)malloc(sizeof(double) * nm);
    double *Cl = (double *)malloc(sizeof(double) * mm);
    double *Vl = (double *)malloc(sizeof(double) * mm);
    double *mu = (double *)malloc(sizeof(double) * (size_t)m);
    double *sg = (double *)malloc(sizeof(double) * (size_t)m);
    double *step = (double *)malloc(sizeof(double) * (size_t)n);
    int rc = -1;
    if (theta_bar && g_bar && Theta && G && Cl && Vl && mu && sg && step) {
        qno_row_means(thetas, dtype, n, m, ld, theta_bar);
        qno_row_means(grads, dtype, n, m, ld, g_bar);
        qno_centre(thetas, dtype, n, m, ld, theta_bar, Theta);
        qno_centre(grads, dtype, n, m, ld, g_bar, G);
        qno_gram(G, n, m, Cl);
        if (qno_jacobi_eigh(Cl, m, mu, Vl) >= 0) {
            qno_sigma_from_mu(mu, m, sg);
            const int j = qno_select_j(sg, m, lambda);
            /* eq. (4) with z = g_bar, then eq. (2) */
            qno_apply_Hinv_literal(Theta, G, n, m, sg, Vl, j, g_bar, step);
            for (int64_t i = 0; i < n; ++i)
                theta_new[i] = theta_bar[i] - tau * step[i];
            *j_out = j;
            if (C)
                memcpy(C, Cl, sizeof(double) * mm);
            if (w)
                qno_gemv_t(G, n, m, g_bar, w);
            if (sigma)
                memcpy(sigma, sg, sizeof(double) * (size_t)m);
            if (V)
                memcpy(V, Vl, sizeof(double) * mm);
            rc = 0;
        }
    }
    free(theta_bar);
    free(g_bar);
    free(Theta);
    free(G);
    free(Cl);
    free(Vl);
    free(mu);
    free(sg);
    free(step);
    return rc;
}

void qno_gram_accumulate(const void *grads, int dtype, int64_t rows, int m,
                         int64_t ld, double *C_acc, double *w_acc)
{
    double *d = (double *)malloc(sizeof(double) * (size_t)m);
    for (int64_t i = 0; i < rows; ++i) {
        double gbar = 0.0;
        for (int k = 0; k < m; ++k) {
            d[k] = elem(grads, dtype, (int64_t)k * ld + i);
            gbar += d[k];
        }
        gbar /= (double)m;
        for (int k = 0; k < m; ++k)
            d[k] -= gbar;
        for (int a = 0; a < m; ++a) {
            for (int b = 0; b < m; ++b)
                C_acc[b * m + a] += d[a] * d[b];
            w_acc[a] += d[a] * gbar;
        }
    }
    free(d);
}

int qno_coefficients(const double *C, const double *w, int m, double lambda,
                     double *c, int *j_out, double *sigma, double *V,
                     double *alpha)
{
    const size_t mm = (size_t)m * (size_t)m;
    double *Vl = (double *)malloc(sizeof(double) * mm);
    double *mu = (double *)malloc(sizeof(double) * (size_t)m);
    double *sg = (double *)malloc(sizeof(double) * (size_t)m);
    int rc = -1;
    if (Vl && mu && sg && qno_jacobi_eigh(C, m, mu, Vl) >= 0) {
        qno_sigma_from_mu(mu, m, sg);
        const int j = qno_select_j(sg, m, lambda);
        for (int r = 0; r < m; ++r)
            c[r] = 0.0;
        for (int k = 0; k < m; ++k) {
            double a = 0.0;
            if (k < j) {
                /* alpha_k = g_bar^T u_k = v_k^T G^T g_bar / sigma_k */
                for (int r = 0; r < m; ++r)
                    a += Vl[k * m + r] * w[r];
                a /= sg[k];
                for (int r = 0; r < m; ++r)
                    c[r] += Vl[k * m + r] * a / sg[k];
            }
            if (alpha)
                alpha[k] = a;
        }
        *j_out = j;
        if (sigma)
            memcpy(sigma, sg, sizeof(double) * (size_t)m);
        if (V)
            memcpy(V, Vl, sizeof(double) * mm);
        rc = 0;
    }
    free(Vl);
    free(mu);
    free(sg);
    return rc;
}

void qno_apply_closed_form(const void *thetas, const void *grads, int dtype,
                           int64_t rows, int m, int64_t ld, const double *c,
                           double tau, double *theta_new)
{
    for (int64_t i = 0; i < rows; ++i) {
        double tbar = 0.0, gbar = 0.0;
        for (int k = 0; k < m; ++k) {
            tbar += elem(thetas, dtype, (int64_t)k * ld + i);
            gbar += elem(grads, dtype, (int64_t)k * ld + i);
        }
        tbar /= (double)m;
        gbar /= (double)m;
        double corr = 0.0;
        for (int k = 0; k < m; ++k) {
            const double th = elem(thetas, dtype, (int64_t)k * ld + i) - tbar;
            const double gr = elem(grads, dtype, (int64_t)k * ld + i) - gbar;
            corr += c[k] * (th - gr);
        }
        theta_new[i] = tbar - tau * (gbar + corr);
    }
}

/* ---- step size capped by 1 / sigma_max (Section 3, closing discussion) ---- */

static double cap_tau(double tau, int have, double smax, double *sigma_max)
{
    if (sigma_max)
        *sigma_max = have ? smax : 0.0;
    if (!have)
        return tau;
    return fmin(tau, 1.0 / smax);
}

double qno_tau_bounded_literal(double tau, int mode, const double *Theta,
                               const double *G, int64_t n, int m,
                               const double *sigma, const double *V, int j,
                               double *sigma_max)
{
    (void)sigma;
    if (mode == QNO_BOUND_SIGMA1) {
        /* sigma_1 = ||G v_1||_2, taken from the matrix itself */
        double s2 = 0.0;
        for (int64_t i = 0; i < n; ++i) {
            double gv = 0.0;
            for (int r = 0; r < m; ++r)
                gv += G[(int64_t)r * n + i] * V[r];
            s2 += gv * gv;
        }
        return cap_tau(tau, s2 > 0.0, sqrt(s2), sigma_max);
    }
    double smax = 0.0;
    for (int k = 0; k < j; ++k) {
        double g2 = 0.0, y2 = 0.0;
        for (int64_t i = 0; i < n; ++i) {
            double gv = 0.0, yv = 0.0;
            for (int r = 0; r < m; ++r) {
                gv += G[(int64_t)r * n + i] * V[k * m + r];
                yv += Theta[(int64_t)r * n + i] * V[k * m + r];
            }
            g2 += gv * gv;
            y2 += yv * yv;
        }
        const double q = sqrt(g2) / sqrt(y2);   /* +inf when Theta v_k = 0 */
        if (q > smax)
            smax = q;
    }
    return cap_tau(tau, j > 0, smax, sigma_max);
}

double qno_tau_bounded_from_gram(double tau, int mode, const double *Ct, int m,
                                 const double *sigma, const double *V, int j,
                                 double *sigma_max)
{
    if (mode == QNO_BOUND_SIGMA1)
        return cap_tau(tau, sigma[0] > 0.0, sigma[0], sigma_max);
    double smax = 0.0;
    for (int k = 0; k < j; ++k) {
        double y2 = 0.0;
        for (int r = 0; r < m; ++r) {
            double row = 0.0;
            for (int q = 0; q < m; ++q)
                row += Ct[q * m + r] * V[k * m + q];
            y2 += V[k * m + r] * row;
        }
        const double quot = sigma[k] / sqrt(y2 > 0.0 ? y2 : 0.0);
        if (quot > smax)
            smax = quot;
    }
    return cap_tau(tau, j > 0, smax, sigma_max);
}
