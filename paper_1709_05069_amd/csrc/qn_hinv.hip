// The operator of eq. (3)/(4) applied to an arbitrary vector z:
//     Hinv z = z_perp + sum_{k<=j} alpha_k sigma_k^-1 y_k,   alpha_k = z^T u_k.
// With u_k = G v_k / sigma_k and y_k = Theta v_k this is z + (Theta - G) c_z,
//     c_z = sum_{k<=j} v_k (v_k^T w_z) / sigma_k^2,   w_z = G^T z.
// w_z comes out of the Gram pass itself: the pivot lane of the matrix-core tiles
// carries z instead of the raw pivot column, so the same pass over grads gives
// G^T G and G^T z.  The eigen kernel then forms c_z exactly as it forms c from
// G^T g_bar, and the apply sweep runs in operator mode: two passes over memory.
#include <cmath>

#include "qn_internal.h"

namespace qn {

// c = sum_{k<j} v_k (v_k^T w) / sigma_k^2, re-centred; j <= 0 gives c = 0.
__global__ __launch_bounds__(64) void coef_kernel(
    const double *__restrict__ sigma, const double *__restrict__ V,
    const int *__restrict__ j_ptr, const double *__restrict__ w, int m,
    float *__restrict__ c)
{
    __shared__ double coef[QN_MAX_M], cvec[QN_MAX_M];
    const int tid = threadIdx.x;
    int j = *j_ptr;
    j = j < 0 ? 0 : (j > m ? m : j);
    if (tid < m) {
        double cf = 0.0;
        if (tid < j) {
            double dot = 0.0;
            for (int r = 0; r < m; ++r)
                dot += V[tid * m + r] * w[r];
            cf = (dot / sigma[tid]) / sigma[tid];
        }
        coef[tid] = cf;
    }
    __syncthreads();
    if (tid < m) {
        double s = 0.0;
        for (int k = 0; k < j; ++k)
            s += V[k * m + tid] * coef[k];
        cvec[tid] = s;
    }
    __syncthreads();
    if (tid < m) {
        double mean = 0.0;
        for (int r = 0; r < m; ++r)
            mean += cvec[r];
        mean /= m;
        c[tid] = static_cast<float>(cvec[tid] - mean);
    }
}

int launch_coef(const double *sigma, const double *V, const int *j, const double *w,
                int m, float *c, hipStream_t stream)
{
    TraceScope ts(QN_K_COEF, stream);
    hipLaunchKernelGGL(coef_kernel, dim3(1), dim3(64), 0, stream, sigma, V, j, w, m, c);
    return check_launch();
}

int run_hinv(const void *thetas, const void *grads, int dtype, const float *z, int64_t n,
             int m, int64_t ld, float lambda, float *out, int *j_out, Workspace *ws,
             hipStream_t s)
{
    RawGram raw;
    int rc = launch_gram_raw(grads, dtype, n, m, ld, ws, z, &raw, s);
    if (rc != QN_OK)
        return rc;
    double *c64 = dtype == QN_F32 ? ws->cz64 : nullptr;
    rc = launch_eig(nullptr, nullptr, m, lambda, nullptr, nullptr, ws->cz, j_out, s, &raw, c64);
    if (rc != QN_OK)
        return rc;
    return launch_apply(thetas, grads, dtype, n, m, ld, ws->cz, z, 0.0f, nullptr, out,
                        ws->cu_count, s, c64);
}

static bool bad_hinv_args(const void *thetas, const void *grads, int dtype, const float *z,
                          int64_t n, int m, int64_t ld, float lambda, const float *out,
                          const int *j_out)
{
    return bad_matrix_args(thetas, dtype, n, m, ld) || !grads || !z || !out || !j_out ||
           !std::isfinite(lambda) || !(lambda > 0.0f);
}

}  // namespace qn

using namespace qn;

extern "C" {

int qn_gemv_t_ex(const void *grads, int dtype, const float *z, int64_t n, int m,
                 int64_t ld, double *w, qn_stream_t stream)
{
    if (bad_matrix_args(grads, dtype, n, m, ld) || !z || !w)
        return QN_EINVAL;
    Workspace ws;
    const int rc = get_lib_workspace(n, m, dtype, &ws);
    if (rc != QN_OK)
        return rc;
    // the Gram matrix of the same pass is not asked for here
    return launch_gram(grads, dtype, n, m, ld, &ws, z, ws.Ct, w, static_cast<hipStream_t>(stream));
}

int qn_gemv_t_ws(const void *grads, int dtype, const float *z, int64_t n, int m,
                 int64_t ld, double *w, void *workspace, size_t workspace_bytes,
                 qn_stream_t stream)
{
    if (bad_matrix_args(grads, dtype, n, m, ld) || !z || !w)
        return QN_EINVAL;
    Device *d = nullptr;
    int rc = get_device(&d);
    if (rc != QN_OK)
        return rc;
    Workspace ws;
    rc = carve_workspace(workspace, workspace_bytes, n, m, dtype, d->cu_count, &ws);
    if (rc != QN_OK)
        return rc;
    return launch_gram(grads, dtype, n, m, ld, &ws, z, ws.Ct, w, static_cast<hipStream_t>(stream));
}

int qn_coef(const double *sigma, const double *V, const int *j, const double *w, int m,
            float *c, qn_stream_t stream)
{
    if (!sigma || !V || !j || !w || !c || m < 1 || m > QN_MAX_M)
        return QN_EINVAL;
    Device *d = nullptr;   // architecture check
    const int rc = get_device(&d);
    if (rc != QN_OK)
        return rc;
    return launch_coef(sigma, V, j, w, m, c, static_cast<hipStream_t>(stream));
}

int qn_hinv_apply_ex(const void *thetas, const void *grads, int dtype, const float *z,
                     int64_t n, int m, int64_t ld, const float *c, float *out,
                     qn_stream_t stream)
{
    if (bad_matrix_args(thetas, dtype, n, m, ld) || !grads || !z || !c || !out)
        return QN_EINVAL;
    Device *d = nullptr;
    const int rc = get_device(&d);
    if (rc != QN_OK)
        return rc;
    return launch_apply(thetas, grads, dtype, n, m, ld, c, z, 0.0f, nullptr, out, d->cu_count,
                        static_cast<hipStream_t>(stream));
}

int qn_hinv_ex(const void *thetas, const void *grads, int dtype, const float *z,
               int64_t n, int m, int64_t ld, float lambda, float *out, int *j_out,
               qn_stream_t stream)
{
    if (bad_hinv_args(thetas, grads, dtype, z, n, m, ld, lambda, out, j_out))
        return QN_EINVAL;
    Workspace ws;
    const int rc = get_lib_workspace(n, m, dtype, &ws);
    if (rc != QN_OK)
        return rc;
    return run_hinv(thetas, grads, dtype, z, n, m, ld, lambda, out, j_out, &ws,
                    static_cast<hipStream_t>(stream));
}

int qn_hinv_ws(const void *thetas, const void *grads, int dtype, const float *z,
               int64_t n, int m, int64_t ld, float lambda, float *out, int *j_out,
               void *workspace, size_t workspace_bytes, qn_stream_t stream)
{
    if (bad_hinv_args(thetas, grads, dtype, z, n, m, ld, lambda, out, j_out))
        return QN_EINVAL;
    Device *d = nullptr;
    int rc = get_device(&d);
    if (rc != QN_OK)
        return rc;
    Workspace ws;
    rc = carve_workspace(workspace, workspace_bytes, n, m, dtype, d->cu_count, &ws);
    if (rc != QN_OK)
        return rc;
    return run_hinv(thetas, grads, dtype, z, n, m, ld, lambda, out, j_out, &ws,
                    static_cast<hipStream_t>(stream));
}

int qn_hinv(const float *thetas, const float *grads, const float *z, int64_t n, int m,
            float lambda, float *out, int *j_out, qn_stream_t stream)
{
    return qn_hinv_ex(thetas, grads, QN_F32, z, n, m, n, lambda, out, j_out, stream);
}

int qn_hinv_bf16(const uint16_t *thetas, const uint16_t *grads, const float *z,
                 int64_t n, int m, float lambda, float *out, int *j_out,
                 qn_stream_t stream)
{
    return qn_hinv_ex(thetas, grads, QN_BF16, z, n, m, n, lambda, out, j_out, stream);
}

}  // extern "C"
