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
 * Workspace: the first call on a device allocates a fixed workspace (about
 *   22 MB) with hipMalloc and keeps it until qn_shutdown(); later calls
 *   allocate nothing.  Calls on the same device share it: two calls that may
 *   overlap in time (different streams or host threads) race and must be
 *   serialised by the caller.
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
    QN_EARCH = -4     /* the current device is not gfx950 */
} qn_status;

typedef enum { QN_F32 = 0, QN_BF16 = 1, QN_F16 = 2 } qn_dtype;

typedef void *qn_stream_t; /* a hipStream_t */

/* host: static string for a status code */
const char *qn_status_string(int status);

/* Allocates the current device's workspace now instead of on first use.
 * Returns QN_OK, QN_ENOMEM, QN_EARCH or QN_ELAUNCH. */
int qn_init(void);

/* Frees every device's workspace.  No library work may be in flight. */
int qn_shutdown(void);

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

/* ---- per-kernel timing (host side helper, for benchmarks) -----------------
 * Between qn_trace_begin() and qn_trace_end() every kernel the library
 * launches is bracketed by HIP events recorded on the launch stream.
 * qn_trace_end() synchronises those events and returns, per kernel id, the
 * summed duration in milliseconds and the launch count (host arrays of
 * QN_TRACE_KERNELS entries each), then disables tracing.
 * max_launches bounds the number of launches recorded (events are created in
 * qn_trace_begin, none in the timed region); further launches are not timed. */
enum {
    QN_K_GRAM = 0,     /* stage 1: streaming pass over grads, per-block partials */
    QN_K_REDUCE = 1,   /* stage 2: fixed-order fp64 sum of the partials */
    QN_K_PROJECT = 2,  /* m x m centring algebra producing C and w */
    QN_K_EIG = 3,      /* Jacobi + cutoff + coefficients */
    QN_K_APPLY = 4,    /* streaming pass over thetas and grads */
    QN_K_COEF = 5,     /* coefficients from sigma, V, j, w */
    QN_K_BOUND = 6,    /* capped step size from sigma, V, j (and Theta^T Theta) */
    QN_TRACE_KERNELS = 7
};
int qn_trace_begin(int max_launches);
int qn_trace_end(double *ms_sum /* host */, int *launches /* host */);
/* host: static name of a kernel id */
const char *qn_kernel_name(int kernel_id);

/* ---- bandwidth probes (diagnostics; not part of the method) ----------------
 * Kernels of exactly known HBM traffic.  They calibrate hardware byte counters
 * and measure the streaming ceiling that the Gram and apply passes are compared
 * with.  bytes must be a positive multiple of 16, pointers 16-byte aligned.
 * qn_probe_copy : dst[0..bytes) = src[0..bytes); reads bytes, writes bytes.
 * qn_probe_read : reads src[0..bytes) and writes qn_probe_sink_floats() floats
 *                 of no meaning to sink (the caller sizes sink with that call;
 *                 it returns -1 when no gfx950 device is current). */
int qn_probe_copy(const void *src, void *dst, int64_t bytes, qn_stream_t stream);
int qn_probe_read(const void *src, int64_t bytes, float *sink, qn_stream_t stream);
int qn_probe_sink_floats(void);

#ifdef __cplusplus
}
#endif
#endif /* QN_H */
