/*
 * qn_diag.h -- diagnostics of libqn: per-kernel event timing, bandwidth probes
 * and a Gram entry point with the kernel chosen by the caller.  Nothing here is
 * part of the method (include/qn.h is); benchmarks and tests use it.
 * Conventions (pointers, streams, status codes) are those of qn.h.
 */
#ifndef QN_DIAG_H
#define QN_DIAG_H

#include "qn.h"

#ifdef __cplusplus
extern "C" {
#endif

/* ---- per-kernel timing (host side helper, for benchmarks) -----------------
 * Between qn_trace_begin() and qn_trace_end() every kernel the library
 * launches is bracketed by HIP events recorded on the launch stream.
 * qn_trace_end() synchronises those events and returns, per kernel id, the
 * summed duration in milliseconds and the launch count (host arrays of
 * QN_TRACE_KERNELS entries each), then disables tracing.
 * max_launches bounds the number of launches recorded (events are created in
 * qn_trace_begin, none in the timed region); further launches are not timed.
 * One trace at a time per process; launches from several host threads may be
 * recorded into it concurrently. */
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

/* ---- bandwidth probes --------------------------------------------------------
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

/* ---- latency probe --------------------------------------------------------------
 * One wavefront runs `links` dependent fp64 multiply-adds (a positive multiple
 * of 8, at most 2^30) and times them inside the kernel.  out (device, 3 values):
 * out[0] = ticks of the constant 100 MHz counter, out[1] = ticks of the shader's
 * cycle counter over the same interval, out[2] = no meaning.  The chain takes a
 * fixed number of shader clocks, so out[0] follows the clock the device runs at
 * when the probe is launched -- the quantity the one-workgroup eigen kernel's
 * duration depends on. */
int qn_probe_chain(int64_t links, unsigned long long *out, qn_stream_t stream);

/* ---- qn_gram_ex with the stage-1 kernel named by the caller --------------------
 * qn_gram_ex picks its kernel from n: the fp64 vector kernel up to 16384 rows,
 * the matrix-core streaming pass above.  Both are correct at every n >= 1; this
 * entry point runs the one asked for, so that each can be compared with the
 * other and with a reference (QN_GRAM_SMALL is refused with QN_EINVAL above
 * 2^22 rows, where it would run for seconds).  z may be NULL (w = G^T g_bar) or
 * n fp32 values (w = G^T z).  Uses the library-owned workspace. */
typedef enum { QN_GRAM_AUTO = 0, QN_GRAM_STREAM = 1, QN_GRAM_SMALL = 2 } qn_gram_path;
int qn_diag_gram_ex(const void *grads, int dtype, const float *z, int64_t n, int m,
                    int64_t ld, int path, double *C, double *w, qn_stream_t stream);

#ifdef __cplusplus
}
#endif
#endif /* QN_DIAG_H */
