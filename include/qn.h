/*
 * qn.h -- C ABI of the MI355X (gfx950) server-side quasi-Newton step of
 * Arnold & Wang, "Accelerating SGD for Distributed Deep-Learning Using
 * Approximated Hessian Matrix", Section 2.
 *
 * Given m worker pairs (theta_k, grad_k) of length n the server forms
 *     theta_bar, g_bar            row means over the m workers (display after eq. (1))
 *     Theta, G                    the worker columns minus those means
 *     C = G^T G,  w = G^T g_bar   m x m Gram and m-vector
 *     sigma_k, v_k                singular values of G / eigenvectors of G^T G
 *     j                           sigma_j >= lambda*sigma_1 > sigma_{j+1}   (rule after eq. (3))
 *     c = sum_{k<=j} v_k (v_k^T w) / sigma_k^2
 *     theta_new = theta_bar - tau * ( g_bar + (Theta - G) c )
 * The last line is eq. (2) with eq. (4) applied to z = g_bar: substituting
 * u_k = G v_k / sigma_k, y_k = Theta v_k and alpha_k = g_bar^T u_k into
 * z_perp + sum_k alpha_k sigma_k^-1 y_k gives g_bar + (Theta - G) c.
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 * Pointers: every data pointer is a DEVICE pointer (HIP global memory on the
 *   current device) unless its comment says "host".  The library reads the
 *   inputs, writes the outputs, and owns nothing the caller passes in.
 * Layout: a worker matrix is m contiguous columns; worker k's vector starts at
 *   element k*ld (ld >= n; the plain entry points use ld = n).  Element type
 *   is fp32, or bfloat16 for the *_bf16 entry points; the *_ex entry points also
 *   take IEEE binary16 (QN_F16).  Accumulation is fp32 / fp64 in every case and
 *   theta_new is always fp32.  Small matrices are stored
 *   the same way: V[k*m + r] is component r of v_k.
 * Alignment: any element-aligned pointer and any n work.  Fastest when the
 *   base pointers are 16-byte aligned and ld*sizeof(elem) is a multiple of 16
 *   (true whenever n is a multiple of 4, or 8 for bfloat16, and ld = n);
 *   otherwise the Gram pass fetches element-wise and 128-bit accesses straddle
 *   cache lines: the same result, about 15 % slower at the 124M x 32 size.
 * Aliasing: theta_new must not overlap an input.
 * Streams: all work is enqueued on `stream` (a hipStream_t passed as void*;
 *   NULL is the default stream) and the call returns without synchronising.
 *   j_out is written on the device; synchronise the stream before reading it.
 * Workspace: the Gram pass and the fused steps need scratch memory (block
 *   partials, the reduced accumulators, the m x m intermediates): at most about
 *   5.6 MB on a 256-unit device, qn_workspace_bytes() gives the figure for a
 *   problem.  The *_ws entry points take it from the caller (device memory,
 *   256-byte aligned, owned by the caller, contents undefined afterwards); they
 *   allocate and free nothing, and calls with different workspaces may run
 *   concurrently on different streams.  The entry points without a workspace
 *   argument use one that the library allocates with hipMalloc on the first such
 *   call on a device and keeps until qn_shutdown(); they share it, so two of
 *   them that may overlap in time (different streams or host threads) race and
 *   must be serialised by the caller.  qn_eig, qn_apply*, qn_coef,
 *   qn_hinv_apply_ex and qn_tau_bound need no scratch memory.
 * Determinism: no floating-point atomics; the reduction tree is a function of
 *   (n, m, dtype, alignment) and the device's compute-unit count only, so
 *   results are bitwise reproducible run to run.
 * Errors: the return value is a qn_status.  Argument errors are detected on
 *   the host before anything is enqueued.  Data-dependent conditions are
 *   reported through j_out, never through the return value:
 *     j_out = 0   no direction trusted (sigma_1 = 0, m = 1, or lambda too
 *                 large): theta_new = theta_bar - tau*g_bar, averaged SGD;
 *     j_out = -1  the Gram matrix or w holds a non-finite value: c = 0 is
 *                 used (the SGD form; non-finite inputs propagate into the
 *                 rows they occupy).
 * Domain: n >= 1, 1 <= m <= QN_MAX_M, tau finite, lambda > 0 and finite.  The
 *   paper takes 0 < lambda < 1; lambda > 1 is accepted and gives j = 0.
 * Accuracy: with fp32 storage theta_new is within 1e-5 of the exact result of
 *   eq. (2)-(4) on the stored inputs in relative L2 norm (1e-3 for 16-bit
 *   storage) on well-conditioned steps.  What limits it is the Gram matrix: the
 *   streaming pass (n > 16384) forms it to about eps_C = 1e-7 of its norm
 *   (exact bf16-split products, fp32 sums over one tile, fp64 from there on;
 *   problems of up to 16384 rows take an fp64 kernel and eps_C ~ 1e-15), and the
 *   coefficient solve divides by sigma_k^2, so to first order
 *       ||d theta_new|| <= tau * eps_C * (1 + max_{k<=j} ||Theta v_k||/sigma_k)
 *                              * (sigma_1^2 ||c|| + ||w||) / sigma_j .
 *   The factor sigma_1/sigma_j is at most 1/lambda.  The bound matters when
 *   g_bar lies mostly inside span{u_1..u_j} (n of the order of m, or gradient
 *   noise far below the curvature signal): then G c cancels g_bar and theta_new
 *   can be much smaller than the terms it is made of.  The sums of the apply
 *   pass run in fp64 for fp32 storage, so they add nothing to this.
 *   Because the all-ones vector is an exact null vector of G^T G whose computed
 *   singular value is of order 1e-8*sigma_1, lambda below about 1e-6 cannot
 *   separate it and is outside the supported range.
 *   The Gram pass accumulates products of centred gradient entries in fp32 (fp64
 *   from one tile on): entries of G whose squares leave the fp32 range are outside
 *   the domain.  Below about 1e-19 in magnitude they underflow and the step
 *   degrades to j_out = 0 (averaged SGD); above about 1e19 they overflow and the
 *   step reports j_out = -1.  Scale the gradients (and tau) if they live there.
 */
#ifndef QN_H
#define QN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define QN_MAX_M 64

typedef enum {
    QN_OK = 0,
    QN_EINVAL = -1,   /* bad argument (null pointer, n < 1, m out of range, bad scalar) */
    QN_ENOMEM = -2,   /* workspace allocation failed */
    QN_ELAUNCH = -3,  /* a HIP call or kernel launch reported an error */
    QN_EARCH = -4,    /* the current device is not gfx950 */
    QN_EWORKSPACE = -5 /* workspace null, not 256-byte aligned or smaller than
                          qn_workspace_bytes() for this problem */
} qn_status;

typedef enum { QN_F32 = 0, QN_BF16 = 1, QN_F16 = 2 } qn_dtype;

typedef void *qn_stream_t; /* a hipStream_t */

/* host: static string for a status code */
const char *qn_status_string(int status);

/* Prepares the current device (architecture check, kernel attributes) and
 * allocates the library-owned workspace of the entry points that take none, now
 * instead of on first use.  Returns QN_OK, QN_ENOMEM, QN_EARCH or QN_ELAUNCH. */
int qn_init(void);

/* Frees every device's library-owned workspace.  No library work may be in flight. */
int qn_shutdown(void);

/* host: bytes of scratch memory a *_ws call on an n x m problem of this element
 * type needs on the current device (any alignment of the inputs, any ld).  A
 * pure function of its arguments and the device's compute-unit count (256 is
 * assumed when no device can be queried); never more than about 5.6 MB.
 * 0 for arguments outside the domain. */
size_t qn_workspace_bytes(int64_t n, int m, int dtype);

/* ---- the whole step: eq. (2) with the operator of eq. (3)/(4) -------------
 * thetas, grads : n x m worker matrices (device, read only)
 * tau           : step length of eq. (2)
 * lambda        : cutoff of the rule after eq. (3)
 * theta_new     : n fp32 values (device, written)
 * j_out         : one int (device, written): the selected j, or 0 / -1 as above
 * Four kernels run back to back on `stream` (Gram pass, its reduction, the
 * eigen kernel, the apply pass) with no host round trip. */
int qn_update(const float *thetas, const float *grads, int64_t n, int m,
              float tau, float lambda, float *theta_new, int *j_out,
              qn_stream_t stream);
int qn_update_bf16(const uint16_t *thetas, const uint16_t *grads, int64_t n,
                   int m, float tau, float lambda, float *theta_new,
                   int *j_out, qn_stream_t stream);

/* ---- C = G^T G and w = G^T g_bar (Section 2: the matrix whose eigenvectors
 * are V_G's columns, and the inner products behind eq. (4)'s alpha_k) --------
 * grads : n x m worker matrix (device, read only); thetas are not needed
 * C     : m*m doubles (device, written), symmetric, C 1 = 0 up to rounding
 * w     : m doubles (device, written) */
int qn_gram(const float *grads, int64_t n, int m, double *C, double *w,
            qn_stream_t stream);
int qn_gram_bf16(const uint16_t *grads, int64_t n, int m, double *C, double *w,
                 qn_stream_t stream);

/* ---- eigendecomposition of C, cutoff j, coefficients c --------------------
 * (Section 2: Sigma_G, V_G; the rule after eq. (3); alpha_k of eq. (4))
 * C, w   : as produced by qn_gram (device, read only)
 * sigma  : m doubles (device, written), descending, sqrt of the eigenvalues
 *          clamped at 0                                  -- may be NULL
 * V      : m*m doubles (device, written), V[k*m + r] = component r of v_k,
 *          ordered like sigma; signs / bases inside equal-sigma clusters are
 *          arbitrary                                     -- may be NULL
 * c      : m floats (device, written): sum_{k<=j} v_k (v_k^T w)/sigma_k^2,
 *          re-centred so that its entries sum to zero
 * j_out  : one int (device, written)
 * One workgroup; parallel cyclic Jacobi in fp64. */
int qn_eig(const double *C, const double *w, int m, float lambda,
           double *sigma, double *V, float *c, int *j_out, qn_stream_t stream);

/* ---- theta_new = theta_bar - tau*( g_bar + (Theta - G) c )  (eq. (2), (4)) -
 * c : m floats (device, read only); any values (need not sum to zero) */
int qn_apply(const float *thetas, const float *grads, int64_t n, int m,
             const float *c, float tau, float *theta_new, qn_stream_t stream);
int qn_apply_bf16(const uint16_t *thetas, const uint16_t *grads, int64_t n,
                  int m, const float *c, float tau, float *theta_new,
                  qn_stream_t stream);

/* ---- the same four with an explicit element type and leading dimension ----
 * ld >= n: worker k's vector starts at element k*ld.  This is the form a row
 * shard of a larger matrix takes (pass the shard's first row and the parent's
 * ld).  dtype is a qn_dtype. */
int qn_update_ex(const void *thetas, const void *grads, int dtype, int64_t n,
                 int m, int64_t ld, float tau, float lambda, float *theta_new,
                 int *j_out, qn_stream_t stream);
int qn_gram_ex(const void *grads, int dtype, int64_t n, int m, int64_t ld,
               double *C, double *w, qn_stream_t stream);
int qn_apply_ex(const void *thetas, const void *grads, int dtype, int64_t n,
                int m, int64_t ld, const float *c, float tau, float *theta_new,
                qn_stream_t stream);

/* ---- the same with caller-owned scratch memory --------------------------------
 * workspace : device memory, 256-byte aligned, workspace_bytes >=
 *   qn_workspace_bytes(n, m, dtype); otherwise QN_EWORKSPACE and nothing is
 *   enqueued.  The library allocates nothing in these calls.  The workspace must
 *   stay untouched until the work enqueued on `stream` has finished; the same
 *   results, bit for bit, as the entry points above. */
int qn_update_ws(const void *thetas, const void *grads, int dtype, int64_t n, int m,
                 int64_t ld, float tau, float lambda, float *theta_new, int *j_out,
                 void *workspace, size_t workspace_bytes, qn_stream_t stream);
int qn_gram_ws(const void *grads, int dtype, int64_t n, int m, int64_t ld, double *C,
               double *w, void *workspace, size_t workspace_bytes, qn_stream_t stream);

/* ---- the whole step for callers that cannot allocate -------------------------
 * For code under HIP graph capture, tight serving loops and harnesses that forbid
 * hipMalloc: qn_update_ex with its scratch memory in a static device array inside
 * the library (6 MiB, held by every device the library runs on until the process
 * ends) instead of an allocated or caller-owned workspace.  The call allocates
 * and frees nothing, also on its first use on a device (which looks up the
 * array's address and sets kernel attributes; qn_init() does the same ahead of
 * time).  Same kernels, same results bit for bit as qn_update_ex.
 * Limit: qn_workspace_bytes(n, m, dtype) must not exceed 6 MiB, else
 * QN_EWORKSPACE and nothing is enqueued (it is at most about 5.6 MB for every
 * n and m <= QN_MAX_M on a device of up to 256 compute units).
 * All calls on one device share that device's array, which keeps the last call's
 * contents; nothing in it needs clearing between calls.  Calls that may overlap
 * in time on one device (different streams or host threads) race: serialise
 * them, or use qn_update_ws. */
int qn_update_noalloc(const void *thetas, const void *grads, int dtype, int64_t n, int m,
                      int64_t ld, float tau, float lambda, float *theta_new, int *j_out,
                      qn_stream_t stream);

/* ---- the step after a single worker's Write (Section 2, opening sentence: the
 * server recomputes its step whenever one worker has written its pair, whether the
 * workers are synchronised or not) ------------------------------------------------
 * Between such steps the library keeps, in `state` (device memory of
 * qn_gram_state_bytes() bytes, 8-byte aligned, owned by the caller), the m x m
 * matrix behind eq. (3)/(4) in a form in which one worker's new gradient changes
 * one row and column.  After worker k has overwritten its column of grads (and of
 * thetas), one pass over grads with m multiply-adds per row -- instead of the
 * m (m + 1) / 2 of the full Gram pass -- brings the state up to date; the eigen
 * kernel and the apply pass then run as in qn_update.
 *   qn_gram_state_init_ws  : state from the current grads (one full Gram pass).
 *   qn_gram_state_write_ws : worker's column of grads has been overwritten since
 *                            the state was last brought up to date; updates it.
 *                            Any worker, the same one repeatedly, in any order.
 *   qn_gram_state_get      : C = G^T G and w = G^T g_bar (as qn_gram writes them)
 *                            of the matrix the state describes.
 *   qn_update_async_ws     : qn_gram_state_write_ws for `worker`, then j, c and
 *                            theta_new = theta_bar - tau (g_bar + (Theta - G) c)
 *                            for the current thetas and grads: the whole server
 *                            step after that worker's Write.
 * The state describes grads as of the last init/write; if several columns changed,
 * call qn_gram_state_write_ws once per changed worker (or init again).  n, m,
 * dtype and ld must be those of the init call.  workspace as for qn_update_ws.
 * The state's sums are fp64 over exact differences, so C from it agrees with
 * qn_gram to the latter's 1e-7. */
size_t qn_gram_state_bytes(void);
int qn_gram_state_init_ws(const void *grads, int dtype, int64_t n, int m, int64_t ld,
                          void *state, void *workspace, size_t workspace_bytes,
                          qn_stream_t stream);
int qn_gram_state_write_ws(const void *grads, int dtype, int64_t n, int m, int64_t ld,
                           int worker, void *state, void *workspace, size_t workspace_bytes,
                           qn_stream_t stream);
int qn_gram_state_get(const void *state, int m, double *C, double *w, qn_stream_t stream);
int qn_update_async_ws(const void *thetas, const void *grads, int dtype, int64_t n, int m,
                       int64_t ld, int worker, float tau, float lambda, void *state,
                       float *theta_new, int *j_out, void *workspace, size_t workspace_bytes,
                       qn_stream_t stream);

/* ---- the operator of eq. (3)/(4) on an arbitrary vector ---------------------
 *   out = Hinv z = z_perp + sum_{k<=j} alpha_k sigma_k^-1 y_k,  alpha_k = z^T u_k,
 * identity on span{u_1..u_j}^perp and the secant inverse (G v_k -> Theta v_k) on
 * the span.  Evaluated as z + (Theta - G) c_z with c_z = sum_{k<=j} v_k (v_k^T
 * G^T z) / sigma_k^2; qn_update is this operator applied to g_bar inside eq. (2).
 * z, out : n fp32 values (device); out must not overlap an input.
 * Two passes over memory: the Gram pass carries z along and yields G^T z with
 * G^T G; then the apply sweep.  j_out as for qn_update; a non-finite value in
 * z is treated like one in grads (j_out = -1, out = z). */
int qn_hinv(const float *thetas, const float *grads, const float *z, int64_t n, int m,
            float lambda, float *out, int *j_out, qn_stream_t stream);
int qn_hinv_bf16(const uint16_t *thetas, const uint16_t *grads, const float *z,
                 int64_t n, int m, float lambda, float *out, int *j_out,
                 qn_stream_t stream);
int qn_hinv_ex(const void *thetas, const void *grads, int dtype, const float *z,
               int64_t n, int m, int64_t ld, float lambda, float *out, int *j_out,
               qn_stream_t stream);
/* its pieces:
 * qn_gemv_t_ex     : w = G^T z (m doubles, device) for the centred G of grads
 *                    (one Gram pass that carries z);
 * qn_coef          : c (m floats) = sum_{k<j} v_k (v_k^T w)/sigma_k^2 from sigma, V
 *                    as written by qn_eig and j read from device memory (*j <= 0
 *                    gives c = 0); re-centred like qn_eig's c;
 * qn_hinv_apply_ex : out = z + (Theta - G) c for any c. */
int qn_gemv_t_ex(const void *grads, int dtype, const float *z, int64_t n, int m,
                 int64_t ld, double *w, qn_stream_t stream);
int qn_coef(const double *sigma, const double *V, const int *j, const double *w, int m,
            float *c, qn_stream_t stream);
int qn_hinv_apply_ex(const void *thetas, const void *grads, int dtype, const float *z,
                     int64_t n, int m, int64_t ld, const float *c, float *out,
                     qn_stream_t stream);
/* with caller-owned scratch memory (see qn_update_ws) */
int qn_hinv_ws(const void *thetas, const void *grads, int dtype, const float *z,
               int64_t n, int m, int64_t ld, float lambda, float *out, int *j_out,
               void *workspace, size_t workspace_bytes, qn_stream_t stream);
int qn_gemv_t_ws(const void *grads, int dtype, const float *z, int64_t n, int m,
                 int64_t ld, double *w, void *workspace, size_t workspace_bytes,
                 qn_stream_t stream);

/* ---- step size capped by 1 / sigma_max (Section 3, closing discussion) ------
 * The paper bounds tau above by the reciprocal of the largest singular value
 * that the method approximates and gives no formula for it.  Two estimates:
 *   QN_BOUND_SIGMA1 : sigma_1, the largest singular value of G;
 *   QN_BOUND_SECANT : max_{k<=j} ||G v_k|| / ||Theta v_k||, the largest gain of
 *                     the approximated Hessian along its secant directions
 *                     (j = 0: no estimate, tau is left alone; a vanishing
 *                     ||Theta v_k|| gives an infinite estimate and tau = 0).
 * The comparison is made in double; tau_eff = min(tau, 1 / sigma_max).
 *
 * qn_update_bounded_ex : qn_update_ex with tau replaced by tau_eff.  tau_out
 *   (device, 1 float, may be NULL) receives tau_eff.  QN_BOUND_SECANT adds one
 *   Gram pass over thetas (n*m elements read) for Theta^T Theta.
 * qn_tau_bound : the m x m piece alone.  sigma, V as written by qn_eig, j read
 *   from device memory, C_theta = Theta^T Theta (m x m doubles, e.g. the C that
 *   qn_gram_ex returns for the theta columns; unused and may be NULL for
 *   QN_BOUND_SIGMA1).  tau_out: device float; sigma_max_out: device double,
 *   may be NULL (0 when there is no estimate). */
typedef enum { QN_BOUND_SIGMA1 = 1, QN_BOUND_SECANT = 2 } qn_bound;
int qn_update_bounded_ex(const void *thetas, const void *grads, int dtype, int64_t n,
                         int m, int64_t ld, float tau, float lambda, int mode,
                         float *theta_new, int *j_out, float *tau_out,
                         qn_stream_t stream);
int qn_tau_bound(const double *sigma, const double *V, const int *j,
                 const double *C_theta, int m, float tau, int mode, float *tau_out,
                 double *sigma_max_out, qn_stream_t stream);
/* with caller-owned scratch memory (see qn_update_ws) */
int qn_update_bounded_ws(const void *thetas, const void *grads, int dtype, int64_t n,
                         int m, int64_t ld, float tau, float lambda, int mode,
                         float *theta_new, int *j_out, float *tau_out, void *workspace,
                         size_t workspace_bytes, qn_stream_t stream);

#ifdef __cplusplus
}
#endif
#endif /* QN_H */
