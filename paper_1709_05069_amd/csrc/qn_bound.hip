// Step size capped by the reciprocal of an estimate of the largest singular
// value (Section 3, closing discussion: tau_opt = 1 / sigma_max, used as an upper
// bound on tau at every update).  The paper gives no formula for the estimate;
// two readings are built:
//   QN_BOUND_SIGMA1: sigma_max := sigma_1, the largest entry of Sigma_G;
//   QN_BOUND_SECANT: sigma_max := max_{k<=j} ||G v_k|| / ||Theta v_k||, the gain
//     of the approximated Hessian along its secant directions (the inverse of
//     eq. (3) maps u_k to Theta v_k / sigma_k).  ||G v_k|| = sigma_k and
//     ||Theta v_k||^2 = v_k^T (Theta^T Theta) v_k, so it costs one more Gram pass
//     (over the theta columns) and m x m work.
// The apply pass then reads the capped tau from device memory.
#include <cmath>

#include "qn_internal.h"

namespace qn {

__global__ __launch_bounds__(64) void tau_bound_kernel(
    int mode, float tau, const double *__restrict__ sigma,
    const double *__restrict__ V, const int *__restrict__ j_ptr,
    const double *__restrict__ Ct, int m, float *__restrict__ tau_out,
    double *__restrict__ sigma_max_out)
{
    __shared__ double quot[QN_MAX_M];
    const int tid = threadIdx.x;
    int j = *j_ptr;
    j = j < 0 ? 0 : (j > m ? m : j);
    if (mode == QN_BOUND_SECANT && tid < j) {
        // y2 = v_k^T Ct v_k
        double y2 = 0.0;
        for (int r = 0; r < m; ++r) {
            double row = 0.0;
            for (int q = 0; q < m; ++q)
                row += Ct[q * m + r] * V[tid * m + q];
            y2 += V[tid * m + r] * row;
        }
        quot[tid] = sigma[tid] / sqrt(y2 > 0.0 ? y2 : 0.0);   // +inf for a vanishing ||Theta v_k||
    }
    __syncthreads();
    if (tid == 0) {
        double smax = 0.0;
        bool have = false;
        if (mode == QN_BOUND_SIGMA1) {
            smax = sigma[0];
            have = smax > 0.0;          // false for 0 and for NaN (non-finite Gram)
        } else {
            for (int k = 0; k < j; ++k)
                smax = quot[k] > smax ? quot[k] : smax;
            have = j > 0;
        }
        if (!have)
            smax = 0.0;
        // the decision is taken in double, like the cutoff
        const double t = static_cast<double>(tau);
        const double cap = have ? 1.0 / smax : t;
        *tau_out = have && cap < t ? static_cast<float>(cap) : tau;
        if (sigma_max_out)
            *sigma_max_out = smax;
    }
}

int launch_tau_bound(int mode, float tau, const double *sigma, const double *V,
                     const int *j, const double *Ct, int m, float *tau_out,
                     double *sigma_max_out, hipStream_t stream)
{
    TraceScope ts(QN_K_BOUND, stream);
    hipLaunchKernelGGL(tau_bound_kernel, dim3(1), dim3(64), 0, stream, mode, tau, sigma, V,
                       j, Ct, m, tau_out, sigma_max_out);
    return check_launch();
}

int run_update_bounded(const void *thetas, const void *grads, int dtype, int64_t n, int m,
                       int64_t ld, float tau, float lambda, int mode, float *theta_new,
                       int *j_out, float *tau_out, Workspace *ws, hipStream_t s)
{
    RawGram raw;
    int rc = launch_gram_raw(grads, dtype, n, m, ld, ws, nullptr, &raw, s);
    if (rc != QN_OK)
        return rc;
    double *c64 = dtype == QN_F32 ? ws->c64 : nullptr;
    rc = launch_eig(nullptr, nullptr, m, lambda, ws->sigma, ws->V, ws->c, j_out, s, &raw, c64);
    if (rc != QN_OK)
        return rc;
    if (mode == QN_BOUND_SECANT) {
        // Theta^T Theta by the same centred Gram pass, over the theta columns
        rc = launch_gram(thetas, dtype, n, m, ld, ws, nullptr, ws->Ct, ws->wt, s);
        if (rc != QN_OK)
            return rc;
    }
    float *tau_dev = tau_out ? tau_out : ws->tau_eff;
    rc = launch_tau_bound(mode, tau, ws->sigma, ws->V, j_out, ws->Ct, m, tau_dev, nullptr, s);
    if (rc != QN_OK)
        return rc;
    return launch_apply(thetas, grads, dtype, n, m, ld, ws->c, nullptr, tau, tau_dev,
                        theta_new, ws->cu_count, s, c64);
}

static bool bad_bounded_args(const void *thetas, const void *grads, int dtype, int64_t n,
                             int m, int64_t ld, float tau, float lambda, int mode,
                             const float *theta_new, const int *j_out)
{
    return bad_matrix_args(thetas, dtype, n, m, ld) || !grads || !theta_new || !j_out ||
           !std::isfinite(tau) || !std::isfinite(lambda) || !(lambda > 0.0f) ||
           (mode != QN_BOUND_SIGMA1 && mode != QN_BOUND_SECANT);
}

}  // namespace qn

using namespace qn;

extern "C" {

int qn_tau_bound(const double *sigma, const double *V, const int *j,
                 const double *C_theta, int m, float tau, int mode, float *tau_out,
                 double *sigma_max_out, qn_stream_t stream)
{
    if (!sigma || !V || !j || !tau_out || m < 1 || m > QN_MAX_M || !std::isfinite(tau) ||
        (mode != QN_BOUND_SIGMA1 && mode != QN_BOUND_SECANT) ||
        (mode == QN_BOUND_SECANT && !C_theta))
        return QN_EINVAL;
    Device *d = nullptr;   // architecture check
    const int rc = get_device(&d);
    if (rc != QN_OK)
        return rc;
    return launch_tau_bound(mode, tau, sigma, V, j, C_theta, m, tau_out, sigma_max_out,
                            static_cast<hipStream_t>(stream));
}

int qn_update_bounded_ex(const void *thetas, const void *grads, int dtype, int64_t n,
                         int m, int64_t ld, float tau, float lambda, int mode,
                         float *theta_new, int *j_out, float *tau_out,
                         qn_stream_t stream)
{
    if (bad_bounded_args(thetas, grads, dtype, n, m, ld, tau, lambda, mode, theta_new, j_out))
        return QN_EINVAL;
    Workspace ws;
    const int rc = get_lib_workspace(n, m, dtype, &ws);
    if (rc != QN_OK)
        return rc;
    return run_update_bounded(thetas, grads, dtype, n, m, ld, tau, lambda, mode, theta_new,
                              j_out, tau_out, &ws, static_cast<hipStream_t>(stream));
}

int qn_update_bounded_ws(const void *thetas, const void *grads, int dtype, int64_t n,
                         int m, int64_t ld, float tau, float lambda, int mode,
                         float *theta_new, int *j_out, float *tau_out, void *workspace,
                         size_t workspace_bytes, qn_stream_t stream)
{
    if (bad_bounded_args(thetas, grads, dtype, n, m, ld, tau, lambda, mode, theta_new, j_out))
        return QN_EINVAL;
    Device *d = nullptr;
    int rc = get_device(&d);
    if (rc != QN_OK)
        return rc;
    Workspace ws;
    rc = carve_workspace(workspace, workspace_bytes, n, m, dtype, d->cu_count, &ws);
    if (rc != QN_OK)
        return rc;
    return run_update_bounded(thetas, grads, dtype, n, m, ld, tau, lambda, mode, theta_new,
                              j_out, tau_out, &ws, static_cast<hipStream_t>(stream));
}

}  // extern "C"
