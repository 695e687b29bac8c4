/*
 * qn_oracle.h -- CPU oracle for the server-side quasi-Newton step of
 * "Accelerating SGD for Distributed Deep-Learning Using Approximated Hessian
 * Matrix" (Arnold & Wang), Section 2, eq. (1)-(4).
 *
 * TEST INFRASTRUCTURE ONLY.  This is a plain, slow, double-precision
 * evaluation of the paper's definitions.  It shares no code with the HIP
 * library and must never be called from the product path; only the tests,
 * the smoke check and the benchmark's CPU-baseline leg may load it.
 *
 * Data layout (all functions): a "worker matrix" X holds m columns of n rows;
 * element (i, k) -- row i of worker k -- lives at X[k*ld + i] with ld >= n.
 * The element type is given by qno_dtype; values are widened to double
 * exactly before any arithmetic.  Small m x m matrices are stored the same
 * way (column k at M[k*m + r]); vectors are contiguous.
 *
 * Every function is pinned by the CPU tests (tests/test_oracle_*.py):
 * closed forms (j = 0 is averaged SGD; exact quadratic lands on A^-1 b),
 * invariants of eq. (3) (secant-inverse on span{u_k}, identity on its
 * complement), engineered spectra for the cutoff rule, a library eigensolver
 * for the Jacobi routine, and literal-vs-closed-form agreement.  The capped
 * step size has no formula in the paper: its two readings are pinned against
 * library singular values and closed forms (H = h I, diagonal H).
 */
#ifndef QN_ORACLE_H
#define QN_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { QNO_F32 = 0, QNO_BF16 = 1, QNO_F64 = 2, QNO_F16 = 3 } qno_dtype;

/* Section 2, the display after eq. (1): mean over the m workers, per row.
 * mean[i] = (1/m) sum_k X[i,k].  mean has n entries. */
void qno_row_means(const void *X, int dtype, int64_t n, int m, int64_t ld,
                   double *mean);

/* Section 2: k-th column of the centred matrix is X[:,k] - mean.
 * Xc is n x m doubles with leading dimension n. */
void qno_centre(const void *X, int dtype, int64_t n, int m, int64_t ld,
                const double *mean, double *Xc);

/* C = G^T G by the plain triple loop (Section 2: V_G holds eigenvectors of
 * G^H G; real data so ^H is a transpose).  G is n x m doubles (ld = n). */
void qno_gram(const double *G, int64_t n, int m, double *C);

/* w = G^T z (the inner products that eq. (4)'s alpha_k are built from). */
void qno_gemv_t(const double *G, int64_t n, int m, const double *z, double *w);

/* Symmetric eigendecomposition of the m x m matrix C by the classical
 * sequential cyclic Jacobi method.  On return mu[0] >= mu[1] >= ... and
 * column k of V (V[k*m + r]) is the unit eigenvector of mu[k].
 * Returns the number of sweeps used, or -1 if it did not converge. */
int qno_jacobi_eigh(const double *C, int m, double *mu, double *V);

/* Section 2: sigma_k = singular values of G = sqrt of the eigenvalues of
 * G^T G (negative rounding residue clamped to zero). */
void qno_sigma_from_mu(const double *mu, int m, double *sigma);

/* Cutoff rule below eq. (3): the integer j with sigma_j >= lambda*sigma_1 and
 * sigma_{j+1} < lambda*sigma_1, sigma sorted descending.  sigma_1 = 0 (or a
 * non-finite sigma_1) gives j = 0. */
int qno_select_j(const double *sigma, int m, double lambda);

/* Eq. (3)/(4), literally: forms u_k = G v_k / ||G v_k||_2 and y_k = Theta v_k
 * explicitly for k = 1..j, alpha_k = z^T u_k, z_perp = z - sum alpha_k u_k,
 * out = z_perp + sum alpha_k sigma_k^-1 y_k.  Theta, G are the centred n x m
 * double matrices (ld = n); sigma, V from the eigendecomposition. */
void qno_apply_Hinv_literal(const double *Theta, const double *G, int64_t n,
                            int m, const double *sigma, const double *V, int j,
                            const double *z, double *out);

/* The whole step of eq. (2) evaluated literally (means, centring, Gram,
 * eigendecomposition, cutoff, explicit u_k / y_k, eq. (4), eq. (2)).
 * Needs 2*n*m doubles of scratch (allocated inside).  Optional outputs (may be
 * NULL): C (m*m), w = G^T g_bar (m), sigma (m), V (m*m).
 * Returns 0, or -1 on allocation failure / non-convergence. */
int qno_update_literal(const void *thetas, const void *grads, int dtype,
                       int64_t n, int m, int64_t ld, double tau, double lambda,
                       double *theta_new, int *j_out, double *C, double *w,
                       double *sigma, double *V);

/* ---- streaming evaluation of the same definition for large n ----
 * With c = sum_{k<=j} v_k (v_k^T w) / sigma_k^2 and w = G^T g_bar, eq. (4)
 * applied to z = g_bar equals g_bar + (Theta - G) c (substitute
 * u_k = G v_k / sigma_k and y_k = Theta v_k).  These three functions evaluate
 * that form over row chunks so that n*m doubles never have to be resident. */

/* Adds the contribution of `rows` rows (a chunk of grads starting at the
 * given pointer, same ld) to C_acc (m*m) and w_acc (m): per row, centre the m
 * gradient values about their mean g_bar_i, C += d d^T, w += d * g_bar_i. */
void qno_gram_accumulate(const void *grads, int dtype, int64_t rows, int m,
                         int64_t ld, double *C_acc, double *w_acc);

/* From C = G^T G and w = G^T g_bar: eigendecomposition, sigma, cutoff j,
 * alpha_k = v_k^T w / sigma_k, c = sum_{k<=j} v_k alpha_k / sigma_k.
 * Optional outputs sigma (m), V (m*m), alpha (m) may be NULL.
 * Returns 0, or -1 on non-convergence. */
int qno_coefficients(const double *C, const double *w, int m, double lambda,
                     double *c, int *j_out, double *sigma, double *V,
                     double *alpha);

/* theta_new_i = theta_bar_i - tau*( g_bar_i
 *                 + sum_k c_k ((theta_ki - theta_bar_i) - (g_ki - g_bar_i)) )
 * for a chunk of `rows` rows. */
void qno_apply_closed_form(const void *thetas, const void *grads, int dtype,
                           int64_t rows, int m, int64_t ld, const double *c,
                           double tau, double *theta_new);

/* ---- step size capped by 1 / sigma_max (Section 3, closing discussion) ----
 * The paper caps tau at the reciprocal of the largest singular value that the
 * method "approximates", without a formula.  Two readings are evaluated:
 *   QNO_BOUND_SIGMA1: sigma_max := sigma_1, the largest entry of Sigma_G;
 *   QNO_BOUND_SECANT: sigma_max := max_{k<=j} ||G v_k|| / ||Theta v_k||, the
 *     largest gain of the approximated Hessian along its own secant
 *     directions (eq. (3) maps u_k to y_k / sigma_k, so the forward map sends
 *     y_k = Theta v_k to sigma_k u_k = G v_k).  j = 0 leaves tau unchanged; a
 *     vanishing ||Theta v_k|| makes the estimate infinite and the cap zero.
 * Both return min(tau, 1 / sigma_max) and store sigma_max if asked. */
typedef enum { QNO_BOUND_SIGMA1 = 1, QNO_BOUND_SECANT = 2 } qno_bound;

/* Literal: forms G v_k and Theta v_k as n-vectors and takes their 2-norms
 * (Theta, G centred n x m doubles, ld = n; V from the eigendecomposition). */
double qno_tau_bounded_literal(double tau, int mode, const double *Theta,
                               const double *G, int64_t n, int m,
                               const double *sigma, const double *V, int j,
                               double *sigma_max);

/* The same from m x m quantities, for large n: ||Theta v_k||^2 =
 * v_k^T (Theta^T Theta) v_k with Ct = Theta^T Theta accumulated by
 * qno_gram_accumulate over the theta columns; ||G v_k|| = sigma_k. */
double qno_tau_bounded_from_gram(double tau, int mode, const double *Ct, int m,
                                 const double *sigma, const double *V, int j,
                                 double *sigma_max);

#ifdef __cplusplus
}
#endif
#endif /* QN_ORACLE_H */
