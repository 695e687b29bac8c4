// The operator of eq. (3)/(4) applied to an arbitrary vector z:
//     Hinv z = z_perp + sum_{k<=j} alpha_k sigma_k^-1 y_k,   alpha_k = z^T u_k.
// With u_k = G v_k / sigma_k and y_k = Theta v_k this is z + (Theta - G) c_z,
//     c_z = sum_{k<=j} v_k (v_k^T w_z) / sigma_k^2,   w_z = G^T z,
// so it takes one streaming pass over grads for w_z (gemv_t below), a tiny
// kernel for c_z (coef below) and the apply sweep in operator mode.
#include <cmath>

#include "qn_internal.h"

namespace qn {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));
// 128-bit global loads at element alignment (unaligned global access is enabled
// on gfx950 under HSA), so the wide path serves any element-aligned input
typedef v4f v4f_elem __attribute__((aligned(4)));
typedef v4u v4u_elem __attribute__((aligned(2)));

constexpr int kGemvThreads = 256;

template <int DT, int R>
__device__ __forceinline__ void gemv_load(const void *base, int64_t elem, float (&x)[R])
{
    if constexpr (DT == QN_F32) {
        const float *p = static_cast<const float *>(base) + elem;
        if constexpr (R == 4) {
            const v4f v = __builtin_nontemporal_load(reinterpret_cast<const v4f_elem *>(p));
            x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
        } else {
            x[0] = *p;
        }
    } else {
        const uint16_t *p = static_cast<const uint16_t *>(base) + elem;
        if constexpr (R == 8) {
            const v4u v = __builtin_nontemporal_load(reinterpret_cast<const v4u_elem *>(p));
            const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                x[2 * h + 0] = __uint_as_float(u[h] << 16);
                x[2 * h + 1] = __uint_as_float(u[h] & 0xffff0000u);
            }
        } else {
            x[0] = __uint_as_float(static_cast<uint32_t>(*p) << 16);
        }
    }
}

// acc[k] += sum over rows [row, row + R) of (grad_k - grad_0) * z   (k >= 1).
// The pivot shift keeps the products at the scale of the centred entries; the
// centring itself is finished at m-vector size: G^T z = P D^T z.
template <int DT, int R>
__device__ __forceinline__ void gemv_rows(const void *__restrict__ grads,
                                          const float *__restrict__ z, int64_t row,
                                          int m, int64_t ld, float (&acc)[QN_MAX_M])
{
    float zz[R], p[R];
    if constexpr (R == 1) {
        zz[0] = z[row];
    } else {
#pragma unroll
        for (int e = 0; e < R; e += 4) {
            const v4f v = __builtin_nontemporal_load(reinterpret_cast<const v4f_elem *>(z + row + e));
            zz[e] = v.x; zz[e + 1] = v.y; zz[e + 2] = v.z; zz[e + 3] = v.w;
        }
    }
    gemv_load<DT, R>(grads, row, p);
#pragma unroll
    for (int k = 1; k < QN_MAX_M; ++k) {
        if (k < m) {   // uniform
            float g[R];
            gemv_load<DT, R>(grads, k * ld + row, g);
            float s = 0.0f;
#pragma unroll
            for (int e = 0; e < R; ++e)
                s = fmaf(g[e] - p[e], zz[e], s);
            acc[k] += s;
        }
    }
}

template <int DT, bool VEC>
__global__ __launch_bounds__(kGemvThreads) void gemv_t_kernel(
    const void *__restrict__ grads, const float *__restrict__ z, int64_t n, int m,
    int64_t ld, double *__restrict__ partials)
{
    constexpr int R = VEC ? (DT == QN_F32 ? 4 : 8) : 1;
    float acc[QN_MAX_M];
#pragma unroll
    for (int k = 0; k < QN_MAX_M; ++k)
        acc[k] = 0.0f;

    const int64_t nvec = n / R;
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kGemvThreads;
    for (int64_t v = static_cast<int64_t>(blockIdx.x) * kGemvThreads + threadIdx.x;
         v < nvec; v += stride)
        gemv_rows<DT, R>(grads, z, v * R, m, ld, acc);
    if constexpr (R > 1) {
        const int64_t tail0 = nvec * R;
        if (blockIdx.x == 0 && tail0 + threadIdx.x < n)
            gemv_rows<DT, 1>(grads, z, tail0 + threadIdx.x, m, ld, acc);
    }

    // fixed-order reduction: butterfly inside the wavefront, then wave order
    __shared__ double red[kGemvThreads / 64][QN_MAX_M];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int k = 0; k < QN_MAX_M; ++k) {
        double v = static_cast<double>(acc[k]);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1)
            v += __shfl_xor(v, off);
        if (lane == 0)
            red[wave][k] = v;
    }
    __syncthreads();
    if (threadIdx.x < QN_MAX_M) {
        double s = 0.0;
#pragma unroll
        for (int wv = 0; wv < kGemvThreads / 64; ++wv)
            s += red[wv][threadIdx.x];
        partials[static_cast<int64_t>(blockIdx.x) * QN_MAX_M + threadIdx.x] = s;
    }
}

// Sums the block partials in block order and applies the centring projector:
// w = u - mean(u) over the m workers (u_0 = 0: the pivot column of D is zero).
constexpr int kFinishSlices = 1024 / QN_MAX_M;
__global__ __launch_bounds__(QN_MAX_M * kFinishSlices) void gemv_finish(
    const double *__restrict__ partials, int num_partials, int m,
    double *__restrict__ w)
{
    __shared__ double part[kFinishSlices][QN_MAX_M];
    __shared__ double u[QN_MAX_M];
    const int k = threadIdx.x % QN_MAX_M, slice = threadIdx.x / QN_MAX_M;
    double s = 0.0;
    for (int p = slice; p < num_partials; p += kFinishSlices)
        s += partials[static_cast<int64_t>(p) * QN_MAX_M + k];
    part[slice][k] = s;
    __syncthreads();
    if (threadIdx.x < QN_MAX_M) {
        double r = 0.0;
        for (int sl = 0; sl < kFinishSlices; ++sl)
            r += part[sl][threadIdx.x];
        u[threadIdx.x] = threadIdx.x < m ? r : 0.0;
    }
    __syncthreads();
    if (threadIdx.x < m) {
        double mean = 0.0;
        for (int x = 0; x < m; ++x)
            mean += u[x];
        mean /= m;
        w[threadIdx.x] = u[threadIdx.x] - mean;
    }
}

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

int launch_gemv_t(const void *grads, int dtype, const float *z, int64_t n, int m,
                  int64_t ld, Workspace *ws, double *w, hipStream_t stream)
{
    const bool vec = n >= (dtype == QN_F32 ? 4 : 8);   // wide loads need no more than element alignment
    const int rows_per_thread = vec ? (dtype == QN_F32 ? 4 : 8) : 1;
    const int64_t per_block = static_cast<int64_t>(kGemvThreads) * rows_per_thread;
    const int64_t want = (n + per_block - 1) / per_block;
    int64_t cap = static_cast<int64_t>(ws->cu_count) * 8;
    if (cap > kGemvMaxBlocks)
        cap = kGemvMaxBlocks;
    const int grid = static_cast<int>(want < cap ? want : cap);
    {
        TraceScope ts(QN_K_GEMV, stream);
#define QN_GEMV_LAUNCH(DTV, VECV)                                                        \
    hipLaunchKernelGGL((gemv_t_kernel<DTV, VECV>), dim3(grid), dim3(kGemvThreads), 0,   \
                       stream, grads, z, n, m, ld, ws->gemv_partials)
        if (dtype == QN_F32) {
            if (vec) QN_GEMV_LAUNCH(QN_F32, true); else QN_GEMV_LAUNCH(QN_F32, false);
        } else {
            if (vec) QN_GEMV_LAUNCH(QN_BF16, true); else QN_GEMV_LAUNCH(QN_BF16, false);
        }
#undef QN_GEMV_LAUNCH
    }
    if (check_launch() != QN_OK)
        return QN_ELAUNCH;
    {
        TraceScope ts(QN_K_GEMV, stream);
        hipLaunchKernelGGL(gemv_finish, dim3(1), dim3(QN_MAX_M * kFinishSlices), 0, stream,
                           ws->gemv_partials, grid, m, w);
    }
    return check_launch();
}

int launch_coef(const double *sigma, const double *V, const int *j, const double *w,
                int m, float *c, hipStream_t stream)
{
    TraceScope ts(QN_K_COEF, stream);
    hipLaunchKernelGGL(coef_kernel, dim3(1), dim3(64), 0, stream, sigma, V, j, w, m, c);
    return check_launch();
}

static bool bad_args(const void *a, int dtype, int64_t n, int m, int64_t ld)
{
    return a == nullptr || (dtype != QN_F32 && dtype != QN_BF16) || n < 1 || m < 1 ||
           m > QN_MAX_M || ld < n;
}

}  // namespace qn

using namespace qn;

extern "C" {

int qn_gemv_t_ex(const void *grads, int dtype, const float *z, int64_t n, int m,
                 int64_t ld, double *w, qn_stream_t stream)
{
    if (bad_args(grads, dtype, n, m, ld) || !z || !w)
        return QN_EINVAL;
    Workspace *ws = nullptr;
    const int rc = get_workspace(&ws);
    if (rc != QN_OK)
        return rc;
    return launch_gemv_t(grads, dtype, z, n, m, ld, ws, w, static_cast<hipStream_t>(stream));
}

int qn_coef(const double *sigma, const double *V, const int *j, const double *w, int m,
            float *c, qn_stream_t stream)
{
    if (!sigma || !V || !j || !w || !c || m < 1 || m > QN_MAX_M)
        return QN_EINVAL;
    Workspace *ws = nullptr;   // arch check only
    const int rc = get_workspace(&ws);
    if (rc != QN_OK)
        return rc;
    return launch_coef(sigma, V, j, w, m, c, static_cast<hipStream_t>(stream));
}

int qn_hinv_apply_ex(const void *thetas, const void *grads, int dtype, const float *z,
                     int64_t n, int m, int64_t ld, const float *c, float *out,
                     qn_stream_t stream)
{
    if (bad_args(thetas, dtype, n, m, ld) || !grads || !z || !c || !out)
        return QN_EINVAL;
    Workspace *ws = nullptr;
    const int rc = get_workspace(&ws);
    if (rc != QN_OK)
        return rc;
    return launch_apply(thetas, grads, dtype, n, m, ld, c, z, 0.0f, nullptr, out, ws->cu_count,
                        static_cast<hipStream_t>(stream));
}

int qn_hinv_ex(const void *thetas, const void *grads, int dtype, const float *z,
               int64_t n, int m, int64_t ld, float lambda, float *out, int *j_out,
               qn_stream_t stream)
{
    if (bad_args(thetas, dtype, n, m, ld) || !grads || !z || !out || !j_out ||
        !std::isfinite(lambda) || !(lambda > 0.0f))
        return QN_EINVAL;
    Workspace *ws = nullptr;
    int rc = get_workspace(&ws);
    if (rc != QN_OK)
        return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    rc = launch_gram(grads, dtype, n, m, ld, ws, ws->C, ws->w, s);
    if (rc != QN_OK)
        return rc;
    rc = launch_eig(ws->C, ws->w, m, lambda, ws->sigma, ws->V, ws->c, j_out, s);
    if (rc != QN_OK)
        return rc;
    rc = launch_gemv_t(grads, dtype, z, n, m, ld, ws, ws->wz, s);
    if (rc != QN_OK)
        return rc;
    rc = launch_coef(ws->sigma, ws->V, j_out, ws->wz, m, ws->cz, s);
    if (rc != QN_OK)
        return rc;
    return launch_apply(thetas, grads, dtype, n, m, ld, ws->cz, z, 0.0f, nullptr, out,
                        ws->cu_count, s);
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
