// Internal declarations shared by the HIP translation units of libqn.
// Not part of the public ABI (that is include/qn.h and include/qn_diag.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "qn.h"
#include "qn_diag.h"
#include "qn_launch_math.h"

namespace qn {

// ---- workspace: a view into scratch memory that somebody else owns ------------
// Carved from a caller's buffer (the *_ws entry points), from the buffer the
// library allocates once per device (the plain entry points) or from the static
// device array (qn_update_noalloc).
struct Workspace {
    double *partials;   // max_partials * gram_entries(m)
    int max_partials;   // blocks whose partial fits
    double *mraw;       // kReduceRows * gram_entries(m): reduced accumulators, raw tile layout
    double *C;          // QN_MAX_M * QN_MAX_M
    double *V;          // QN_MAX_M * QN_MAX_M
    double *Ct;         // QN_MAX_M * QN_MAX_M: Theta^T Theta for the secant bound
    double *w;          // QN_MAX_M
    double *sigma;      // QN_MAX_M
    double *wz;         // QN_MAX_M
    double *wt;         // QN_MAX_M: by-product of the Theta^T Theta pass (unused)
    float *c;           // QN_MAX_M
    float *cz;          // QN_MAX_M
    double *c64;        // QN_MAX_M: c before its rounding to fp32 (fused steps, fp32 storage)
    double *cz64;       // QN_MAX_M
    float *tau_eff;     // 1: capped step size
    int cu_count;
};

// Lays a workspace for an (n, m, dtype) problem over [base, base + bytes).
// QN_EWORKSPACE when base is null, not 256-byte aligned or bytes is below
// workspace_need(n, m, dtype, cu_count).
int carve_workspace(void *base, size_t bytes, int64_t n, int m, int dtype, int cu_count,
                    Workspace *ws);

// ---- per-device state -----------------------------------------------------------
struct Device {
    int cu_count;
    void *lib_ws;           // allocated by the plain entry points on first use, else null
    size_t lib_ws_bytes;
    void *static_scratch;   // this device's copy of the static scratch array (its device address)
};
// The current device's state; on first use checks the architecture, opts the
// kernels into their dynamic LDS sizes and looks up the address of the device's
// copy of the static scratch array.  Allocates nothing.
int get_device(Device **out);
// The library-owned workspace of the plain entry points (hipMalloc on first use).
int get_lib_workspace(int64_t n, int m, int dtype, Workspace *ws);

// ---- per-device kernel set-up (called once per device by get_device) ----------
int setup_gram_kernels();
int setup_apply_kernels();
int setup_eig_kernels();

// ---- kernel launchers (each enqueues on `stream`, returns a qn_status) ------
// Which Gram kernel a launch may use: by problem size, or forced (diagnostics).
enum GramPath { kGramAuto = 0, kGramStream = 1, kGramSmall = 2 };
// C = G^T G and, with z == nullptr, w = G^T g_bar; with z (n fp32 values) w = G^T z
int launch_gram(const void *grads, int dtype, int64_t n, int m, int64_t ld,
                Workspace *ws, const float *z, double *C, double *w, hipStream_t stream,
                int path = kGramAuto);
// The raw, pivot-shifted accumulators of a Gram pass (kReduceRows rows of
// `entries` doubles in the workspace) and what is needed to decode them.
struct RawGram {
    const double *mraw;
    int entries;
    int z_mode;     // column 0 holds d_k^T z rather than d_k^T s
    int pack;       // row blocks packed into the single column set (m <= 8)
};
// stage 1 + reduce only; launch_gram adds the projection to C and w
int launch_gram_raw(const void *grads, int dtype, int64_t n, int m, int64_t ld,
                    Workspace *ws, const float *z, RawGram *raw, hipStream_t stream,
                    int path = kGramAuto);
// raw != nullptr: C and w are formed inside the kernel from the raw accumulators;
// c64 != nullptr also receives c in double
int launch_eig(const double *C, const double *w, int m, float lambda,
               double *sigma, double *V, float *c, int *j_out,
               hipStream_t stream, const RawGram *raw = nullptr, double *c64 = nullptr);
// z == nullptr: theta_new = theta_bar - tau (g_bar + (Theta - G) c);
// z != nullptr: theta_new = z + (Theta - G) c  (tau unused);
// tau_dev != nullptr: tau is read from device memory instead of the argument;
// c64 != nullptr (fp32 storage only): the coefficients are taken from there, in
// double, instead of from c
int launch_apply(const void *thetas, const void *grads, int dtype, int64_t n,
                 int m, int64_t ld, const float *c, const float *z, float tau,
                 const float *tau_dev, float *theta_new, int cu_count, hipStream_t stream,
                 const double *c64 = nullptr);
// c = sum_{k < j} v_k (v_k^T w) / sigma_k^2, j read from device memory
int launch_coef(const double *sigma, const double *V, const int *j, const double *w,
                int m, float *c, hipStream_t stream);
// tau_out = min(tau, 1 / sigma_max) for the estimate named by mode (a qn_bound)
int launch_tau_bound(int mode, float tau, const double *sigma, const double *V,
                     const int *j, const double *Ct, int m, float *tau_out,
                     double *sigma_max_out, hipStream_t stream);

// ---- the fused steps over a given workspace (argument checks done by the caller) --
int run_update(const void *thetas, const void *grads, int dtype, int64_t n, int m,
               int64_t ld, float tau, float lambda, float *theta_new, int *j_out,
               Workspace *ws, hipStream_t stream);
int run_hinv(const void *thetas, const void *grads, int dtype, const float *z, int64_t n,
             int m, int64_t ld, float lambda, float *out, int *j_out, Workspace *ws,
             hipStream_t stream);
int run_update_bounded(const void *thetas, const void *grads, int dtype, int64_t n, int m,
                       int64_t ld, float tau, float lambda, int mode, float *theta_new,
                       int *j_out, float *tau_out, Workspace *ws, hipStream_t stream);

// argument checks shared by the entry points
inline bool bad_matrix_args(const void *a, int dtype, int64_t n, int m, int64_t ld)
{
    return a == nullptr || (dtype != QN_F32 && dtype != QN_BF16 && dtype != QN_F16) || n < 1 ||
           m < 1 || m > QN_MAX_M || ld < n;
}

// ---- tracing ------------------------------------------------------------------
// RAII bracket: records a start/stop event pair around one kernel launch when
// tracing is enabled; otherwise does nothing.
struct TraceScope {
    TraceScope(int kernel_id, hipStream_t stream);
    ~TraceScope();
    int slot;
    hipStream_t stream;
};

inline int check_launch()
{
    return hipGetLastError() == hipSuccess ? QN_OK : QN_ELAUNCH;
}

}  // namespace qn
