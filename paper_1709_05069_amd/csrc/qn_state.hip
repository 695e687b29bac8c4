// The server step after a single worker's Write (Section 2, opening: the server
// recomputes its step whenever one worker has written its pair, whether the
// workers are synchronised or not).
//
// When one worker's pair (theta_k, grad_k) changes, one column of the gradient
// matrix changes.  The m x m matrix behind eq. (3)/(4) is kept between calls in
// its pivot-shifted form
//     N[a][b] = d_a^T d_b,   t[a] = d_a^T s,   d_a = grad_a - s,   s = grad_p
// (p: the pivot worker; row and column p of N and t[p] are zero), from which
//     C = G^T G = P N P,   w = G^T g_bar = P (t + N 1 / m),   P = I - 11^T/m
// follow at m x m size exactly as in the full Gram pass (qn_gram.hip).  A Write by
// worker k != p changes d_k only, hence row and column k of N and t[k]: m + 1
// inner products of the new column with all columns.  One pass over grads with m
// multiply-adds per row replaces the m (m + 1) / 2 of the full pass: the same
// bytes, a small fraction of the arithmetic, which is what the full pass is
// short of for 16-bit storage and for m > 32.  A Write by the pivot worker itself
// first moves the pivot to another worker q at m x m size:
//     d_a' = d_a - d_q  =>  N'[a][b] = N[a][b] - N[a][q] - N[q][b] + N[q][q],
//                           t'[a]    = t[a] - t[q] + N[a][q] - N[q][q],
// so it costs the same single pass.  The eigen kernel and the apply pass then run
// as in the full step.
//
// The column pass is lane = rows like the apply pass (all m values of a row meet
// in one lane); differences, products and sums are in fp64 (the inputs are fp32
// or 16-bit, so the differences are exact), one partial per block, blocks added
// in block order: bitwise reproducible, no atomics.
#include <cmath>

#include "qn_internal.h"
#include "qn_project.h"

namespace qn {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));
typedef v4f v4f_elem __attribute__((aligned(4)));
typedef v4u v4u_elem __attribute__((aligned(2)));

// ---- the state: QN_MAX_M^2 + QN_MAX_M doubles and a two-int header -------------
constexpr size_t kStateDoubles = static_cast<size_t>(QN_MAX_M) * QN_MAX_M + QN_MAX_M;
constexpr size_t kStateBytes = (kStateDoubles * sizeof(double) + 2 * sizeof(int) + 255) / 256 * 256;
struct StateView {
    double *N;      // m x m, leading dimension m
    double *t;      // m
    int *head;      // head[0] = pivot worker, head[1] = m
};
__host__ __device__ inline StateView state_view(void *state)
{
    StateView v;
    v.N = static_cast<double *>(state);
    v.t = v.N + static_cast<size_t>(QN_MAX_M) * QN_MAX_M;
    v.head = reinterpret_cast<int *>(v.t + QN_MAX_M);
    return v;
}

constexpr int kStateThreads = 256;

// state <- the reduced raw accumulators of a full Gram pass (pivot worker 0)
__global__ __launch_bounds__(kStateThreads) void state_from_raw(
    const double *__restrict__ mraw, int entries, int m, int pack, void *state)
{
    const StateView st = state_view(state);
    for (int e = threadIdx.x; e < m * m; e += kStateThreads) {
        const int k = e / m, l = e % m;
        double q = 0.0;
        if (k >= 1 && l >= 1)
            q = raw_entry(mraw, entries, pack, k >= l ? k : l, k >= l ? l : k);
        st.N[e] = q;
    }
    for (int k = threadIdx.x; k < m; k += kStateThreads)
        st.t[k] = k >= 1 ? raw_entry(mraw, entries, pack, k, 0) : 0.0;
    if (threadIdx.x == 0) {
        st.head[0] = 0;
        st.head[1] = m;
    }
}

// If `worker` is the pivot, moves the pivot to the next worker (m x m algebra in
// LDS).  The entries that involve `worker` are left stale: the column pass that
// follows rewrites all of them.
__global__ __launch_bounds__(kStateThreads) void state_repivot(void *state, int m, int worker)
{
    const StateView st = state_view(state);
    if (st.head[0] != worker || m < 2)     // uniform
        return;
    __shared__ double Nq[QN_MAX_M];        // column q of N
    __shared__ double tq_nqq[2];
    const int q = (worker + 1) % m;
    for (int a = threadIdx.x; a < m; a += kStateThreads)
        Nq[a] = st.N[a * m + q];
    if (threadIdx.x == 0) {
        tq_nqq[0] = st.t[q];
        tq_nqq[1] = st.N[q * m + q];
    }
    __syncthreads();
    const double tq = tq_nqq[0], nqq = tq_nqq[1];
    // every entry is rewritten from its own old value and from column q, which is
    // in LDS: no read-after-write hazard between threads
    for (int e = threadIdx.x; e < m * m; e += kStateThreads) {
        const int a = e / m, b = e % m;
        st.N[e] = (a == q || b == q) ? 0.0 : st.N[e] - Nq[a] - Nq[b] + nqq;
    }
    for (int a = threadIdx.x; a < m; a += kStateThreads)
        st.t[a] = a == q ? 0.0 : st.t[a] - tq + Nq[a] - nqq;
    if (threadIdx.x == 0)
        st.head[0] = q;
}

// ---- the column pass -----------------------------------------------------------
// R rows of one column as they arrive (16 bytes, or one element) and widened to
// fp64 at the point of use, so that loads in flight cost 4 registers each.
template <int DT, int R> struct ColRaw { using type = v4u; };
template <> struct ColRaw<QN_F32, 1> { using type = float; };
template <> struct ColRaw<QN_BF16, 1> { using type = uint16_t; };
template <> struct ColRaw<QN_F16, 1> { using type = uint16_t; };

template <int DT, int R>
__device__ __forceinline__ typename ColRaw<DT, R>::type col_load(const void *base, int64_t elem)
{
    if constexpr (R == 1) {
        return static_cast<const typename ColRaw<DT, 1>::type *>(base)[elem];
    } else {
        const char *p = static_cast<const char *>(base) + elem * (DT == QN_F32 ? 4 : 2);
        if constexpr (DT == QN_F32)
            return __builtin_bit_cast(v4u, __builtin_nontemporal_load(reinterpret_cast<const v4f_elem *>(p)));
        else
            return __builtin_nontemporal_load(reinterpret_cast<const v4u_elem *>(p));
    }
}

__device__ __forceinline__ float f16_bits(uint32_t h)
{
    return static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(h)));
}

template <int DT, int R>
__device__ __forceinline__ void col_widen(const typename ColRaw<DT, R>::type &v, double (&x)[R])
{
    if constexpr (R == 1) {
        if constexpr (DT == QN_F32)
            x[0] = v;
        else if constexpr (DT == QN_BF16)
            x[0] = __uint_as_float(static_cast<uint32_t>(v) << 16);
        else
            x[0] = f16_bits(v);
    } else {
        const uint32_t u[4] = {v.x, v.y, v.z, v.w};
        if constexpr (DT == QN_F32) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                x[e] = __uint_as_float(u[e]);
        } else if constexpr (DT == QN_BF16) {
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                x[2 * h + 0] = __uint_as_float(u[h] << 16);
                x[2 * h + 1] = __uint_as_float(u[h] & 0xffff0000u);
            }
        } else {
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                x[2 * h + 0] = f16_bits(u[h] & 0xffffu);
                x[2 * h + 1] = f16_bits(u[h] >> 16);
            }
        }
    }
}

// acc[l] += sum over the R rows at `row` of x (grad_l - s), l = 0 .. MP-1 (columns
// >= m are skipped), and acc[MP] += sum of x s, where x = grad_worker - s and s is
// the pivot's value.  The pivot's own column contributes x * 0.  Columns come in
// chunks of CH whose loads are issued one chunk ahead of their use.
template <int DT, int MP, int R>
__device__ __forceinline__ void column_rows(const void *__restrict__ grads, int64_t row, int m,
                                            int64_t ld, int worker, int pivot,
                                            double (&acc)[MP + 1])
{
    using Raw = typename ColRaw<DT, R>::type;
    constexpr int CH = MP < 8 ? MP : 8;
    const Raw sr = col_load<DT, R>(grads, static_cast<int64_t>(pivot) * ld + row);
    const Raw xr = col_load<DT, R>(grads, static_cast<int64_t>(worker) * ld + row);
    Raw cur[CH] = {}, nxt[CH] = {};
#pragma unroll
    for (int u = 0; u < CH; ++u)
        if (u < m)
            cur[u] = col_load<DT, R>(grads, static_cast<int64_t>(u) * ld + row);
    double s[R], x[R];
    col_widen<DT, R>(sr, s);
    col_widen<DT, R>(xr, x);
#pragma unroll
    for (int e = 0; e < R; ++e) {
        x[e] -= s[e];
        acc[MP] = fma(x[e], s[e], acc[MP]);
    }
#pragma unroll
    for (int l0 = 0; l0 < MP; l0 += CH) {
#pragma unroll
        for (int u = 0; u < CH; ++u)
            if (l0 + CH + u < MP && l0 + CH + u < m)
                nxt[u] = col_load<DT, R>(grads, static_cast<int64_t>(l0 + CH + u) * ld + row);
#pragma unroll
        for (int u = 0; u < CH; ++u)
            if (l0 + u < m) {
                double g[R];
                col_widen<DT, R>(cur[u], g);
#pragma unroll
                for (int e = 0; e < R; ++e)
                    acc[l0 + u] = fma(x[e], g[e] - s[e], acc[l0 + u]);
            }
#pragma unroll
        for (int u = 0; u < CH; ++u)
            cur[u] = nxt[u];
    }
}

template <int DT, int MP>
__global__ __launch_bounds__(kColThreads) void gram_column_pass(
    const void *__restrict__ grads, int64_t n, int m, int64_t ld, int worker,
    const void *__restrict__ state, double *__restrict__ partials)
{
    constexpr int R = DT == QN_F32 ? 4 : 8;
    const int pivot = state_view(const_cast<void *>(state)).head[0];     // uniform
    double acc[MP + 1];
#pragma unroll
    for (int l = 0; l <= MP; ++l)
        acc[l] = 0.0;
    const int64_t nvec = n / R;
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kColThreads;
    for (int64_t v = static_cast<int64_t>(blockIdx.x) * kColThreads + threadIdx.x; v < nvec;
         v += stride)
        column_rows<DT, MP, R>(grads, v * R, m, ld, worker, pivot, acc);
    // rows past the last full vector: one each for the first threads of block 0
    const int64_t tail0 = nvec * R;
    if (blockIdx.x == 0 && tail0 + threadIdx.x < n)
        column_rows<DT, MP, 1>(grads, tail0 + threadIdx.x, m, ld, worker, pivot, acc);

    // block partial: butterfly inside each wavefront, wavefronts added in order
    __shared__ double red[kColThreads / 64][MP + 1];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int l = 0; l <= MP; ++l) {
        double v = acc[l];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1)
            v += __shfl_xor(v, off);
        if (lane == 0)
            red[wave][l] = v;
    }
    __syncthreads();
    for (int l = threadIdx.x; l <= MP; l += kColThreads) {
        double v = 0.0;
#pragma unroll
        for (int wv = 0; wv < kColThreads / 64; ++wv)
            v += red[wv][l];
        partials[static_cast<int64_t>(blockIdx.x) * (MP + 1) + l] = v;
    }
}

// Row and column `worker` of N and t[worker] from the block partials, in a fixed
// order: thread (slice, l) adds the partials slice, slice + S, ... of entry l, then
// the S slices are added in order.
__global__ __launch_bounds__(kStateThreads) void state_finalize(
    const double *__restrict__ partials, int grid, int mp, int m, int worker, void *state)
{
    const StateView st = state_view(state);
    const int pivot = st.head[0];
    const int width = mp + 1;
    const int S = kStateThreads / width;                 // >= 3 (width <= 65)
    __shared__ double part[kStateThreads];
    const int l = threadIdx.x % width, slice = threadIdx.x / width;
    if (slice < S) {
        // eight loads in flight, added in order (the order fixes the bits)
        double v = 0.0;
        int b = slice;
        for (; b + 7 * S < grid; b += 8 * S) {
            double p8[8];
#pragma unroll
            for (int i = 0; i < 8; ++i)
                p8[i] = partials[static_cast<int64_t>(b + i * S) * width + l];
#pragma unroll
            for (int i = 0; i < 8; ++i)
                v += p8[i];
        }
        for (; b < grid; b += S)
            v += partials[static_cast<int64_t>(b) * width + l];
        part[slice * width + l] = v;
    }
    __syncthreads();
    if (static_cast<int>(threadIdx.x) < width && (l == mp || l < m)) {
        double v = 0.0;
        for (int sl = 0; sl < S; ++sl)
            v += part[sl * width + l];
        if (l == mp) {
            st.t[worker] = worker == pivot ? 0.0 : v;
        } else {
            const double q = (l == pivot || worker == pivot) ? 0.0 : v;
            st.N[worker * m + l] = q;
            st.N[l * m + worker] = q;
        }
    }
}

// C = P N P and w = P (t + N 1 / m) from the state (any pivot).
__global__ __launch_bounds__(kStateThreads) void state_project(
    const void *state, int m, double *__restrict__ C, double *__restrict__ w)
{
    const StateView st = state_view(const_cast<void *>(state));
    __shared__ double rowsum[QN_MAX_M], u[QN_MAX_M];
    __shared__ double total, umean;
    const int tid = threadIdx.x;
    if (tid < m) {
        double s = 0.0;
        for (int x = 0; x < m; ++x)
            s += st.N[tid * m + x];
        rowsum[tid] = s;
        u[tid] = st.t[tid] + s / m;
    }
    __syncthreads();
    if (tid == 0) {
        double s = 0.0, su = 0.0;
        for (int x = 0; x < m; ++x) {
            s += rowsum[x];
            su += u[x];
        }
        total = s;
        umean = su / m;
    }
    __syncthreads();
    for (int e = tid; e < m * m; e += kStateThreads) {
        const int k = e / m, l = e % m;
        C[l * m + k] = st.N[e] - (rowsum[k] + rowsum[l]) / m + total / (static_cast<double>(m) * m);
    }
    if (tid < m)
        w[tid] = u[tid] - umean;
}

template <int DT>
static void launch_column_dt(int grid, const void *grads, int64_t n, int m, int64_t ld,
                             int worker, const void *state, double *partials, hipStream_t s)
{
#define QN_COL(MPV) \
    hipLaunchKernelGGL((gram_column_pass<DT, MPV>), dim3(grid), dim3(kColThreads), 0, s, grads, n, \
                       m, ld, worker, state, partials)
    switch (column_mp(m)) {
    case 4: QN_COL(4); break;
    case 8: QN_COL(8); break;
    case 16: QN_COL(16); break;
    case 32: QN_COL(32); break;
    default: QN_COL(64); break;
    }
#undef QN_COL
}

// the state after worker's Write: optional re-pivot, column pass, finalize
static int launch_state_write(const void *grads, int dtype, int64_t n, int m, int64_t ld,
                              int worker, void *state, Workspace *ws, hipStream_t s)
{
    const int mp = column_mp(m);
    const int grid = column_pass_grid(n, m, dtype, ws->cu_count, ws->max_partials);
    hipLaunchKernelGGL(state_repivot, dim3(1), dim3(kStateThreads), 0, s, state, m, worker);
    {
        TraceScope ts(QN_K_GRAM, s);
        if (dtype == QN_F32)
            launch_column_dt<QN_F32>(grid, grads, n, m, ld, worker, state, ws->partials, s);
        else if (dtype == QN_BF16)
            launch_column_dt<QN_BF16>(grid, grads, n, m, ld, worker, state, ws->partials, s);
        else
            launch_column_dt<QN_F16>(grid, grads, n, m, ld, worker, state, ws->partials, s);
    }
    {
        TraceScope ts(QN_K_REDUCE, s);
        hipLaunchKernelGGL(state_finalize, dim3(1), dim3(kStateThreads), 0, s, ws->partials, grid,
                           mp, m, worker, state);
    }
    return check_launch();
}

static bool bad_state_args(const void *grads, int dtype, int64_t n, int m, int64_t ld,
                           const void *state)
{
    return bad_matrix_args(grads, dtype, n, m, ld) || state == nullptr ||
           reinterpret_cast<uintptr_t>(state) % 8 != 0;
}

static int caller_workspace(void *workspace, size_t bytes, int64_t n, int m, int dtype,
                            Workspace *ws)
{
    Device *d = nullptr;
    const int rc = get_device(&d);
    if (rc != QN_OK)
        return rc;
    return carve_workspace(workspace, bytes, n, m, dtype, d->cu_count, ws);
}

}  // namespace qn

using namespace qn;

extern "C" {

size_t qn_gram_state_bytes(void)
{
    return kStateBytes;
}

int qn_gram_state_init_ws(const void *grads, int dtype, int64_t n, int m, int64_t ld,
                          void *state, void *workspace, size_t workspace_bytes,
                          qn_stream_t stream)
{
    if (bad_state_args(grads, dtype, n, m, ld, state))
        return QN_EINVAL;
    Workspace ws;
    int rc = caller_workspace(workspace, workspace_bytes, n, m, dtype, &ws);
    if (rc != QN_OK)
        return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    RawGram raw;
    rc = launch_gram_raw(grads, dtype, n, m, ld, &ws, nullptr, &raw, s);
    if (rc != QN_OK)
        return rc;
    hipLaunchKernelGGL(state_from_raw, dim3(1), dim3(kStateThreads), 0, s, raw.mraw, raw.entries,
                       m, raw.pack, state);
    return check_launch();
}

int qn_gram_state_write_ws(const void *grads, int dtype, int64_t n, int m, int64_t ld,
                           int worker, void *state, void *workspace, size_t workspace_bytes,
                           qn_stream_t stream)
{
    if (bad_state_args(grads, dtype, n, m, ld, state) || worker < 0 || worker >= m)
        return QN_EINVAL;
    Workspace ws;
    const int rc = caller_workspace(workspace, workspace_bytes, n, m, dtype, &ws);
    if (rc != QN_OK)
        return rc;
    return launch_state_write(grads, dtype, n, m, ld, worker, state, &ws,
                              static_cast<hipStream_t>(stream));
}

int qn_gram_state_get(const void *state, int m, double *C, double *w, qn_stream_t stream)
{
    if (!state || !C || !w || m < 1 || m > QN_MAX_M)
        return QN_EINVAL;
    Device *d = nullptr;
    const int rc = get_device(&d);
    if (rc != QN_OK)
        return rc;
    TraceScope ts(QN_K_PROJECT, static_cast<hipStream_t>(stream));
    hipLaunchKernelGGL(state_project, dim3(1), dim3(kStateThreads), 0,
                       static_cast<hipStream_t>(stream), state, m, C, w);
    return check_launch();
}

int qn_update_async_ws(const void *thetas, const void *grads, int dtype, int64_t n, int m,
                       int64_t ld, int worker, float tau, float lambda, void *state,
                       float *theta_new, int *j_out, void *workspace, size_t workspace_bytes,
                       qn_stream_t stream)
{
    if (bad_state_args(grads, dtype, n, m, ld, state) || !thetas || !theta_new || !j_out ||
        worker < 0 || worker >= m || !std::isfinite(tau) || !std::isfinite(lambda) ||
        !(lambda > 0.0f))
        return QN_EINVAL;
    Workspace ws;
    int rc = caller_workspace(workspace, workspace_bytes, n, m, dtype, &ws);
    if (rc != QN_OK)
        return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    rc = launch_state_write(grads, dtype, n, m, ld, worker, state, &ws, s);
    if (rc != QN_OK)
        return rc;
    {
        TraceScope ts(QN_K_PROJECT, s);
        hipLaunchKernelGGL(state_project, dim3(1), dim3(kStateThreads), 0, s, state, m, ws.C, ws.w);
    }
    if (check_launch() != QN_OK)
        return QN_ELAUNCH;
    double *c64 = dtype == QN_F32 ? ws.c64 : nullptr;
    rc = launch_eig(ws.C, ws.w, m, lambda, nullptr, nullptr, ws.c, j_out, s, nullptr, c64);
    if (rc != QN_OK)
        return rc;
    return launch_apply(thetas, grads, dtype, n, m, ld, ws.c, nullptr, tau, nullptr, theta_new,
                        ws.cu_count, s, c64);
}

}  // extern "C"
