// theta_new = theta_bar - tau * ( g_bar + (Theta - G) c )         (eq. (2) with
// eq. (4) applied to z = g_bar; Theta, G are the centred worker matrices of
// Section 2 and c the coefficient vector produced by the eigen step).
//
// One streaming pass: every row needs its 2m inputs once and produces one
// output, about half a flop per byte, so the kernel is bound by HBM bandwidth.
// Lane = rows (128-bit loads along each worker's contiguous column), all m
// values of a row meet in one lane, so the row means cost nothing extra.
// Every input byte is used exactly once, so the loads carry the non-temporal
// hint: measured on MI355X, a 64-stream read of this shape runs at about
// 7.0 TB/s with the hint and 6.1 TB/s without.
//
// Arithmetic per row i, with the pivots p = theta_0[i], r = grad_0[i] and the
// differences t_k = theta_k[i] - p, h_k = grad_k[i] - r (exact or correctly
// rounded; same magnitude as the centred entries, so no cancellation later):
//     theta_bar = p + St/m,  g_bar = r + Sh/m,        St = sum t_k, Sh = sum h_k
//     (Theta - G) c = sum_k c_k (t_k - h_k) - (St - Sh)/m * sum_k c_k
// which equals the centred definition for any c (the last term vanishes when
// the entries of c sum to zero, as they do when c comes from the eigen step).
// With fp32 storage the sum over k and the final combination run in fp64: when
// g_bar lies (almost) inside span{u_1..u_j} -- always for n < m -- the term G c
// cancels g_bar, and an fp32 sum would leave an error of 2^-24 |g_bar| in a
// result that can be a hundred times smaller.  The kernel is bound by HBM
// bandwidth, so the two extra fp64 operations per element are free.
//
// Operator mode (z != nullptr): the same sweep evaluates eq. (4) for an
// arbitrary vector z, out = z + (Theta - G) c_z with c_z built from G^T z, and
// tau, theta_bar and g_bar play no part.
#include "qn_internal.h"

namespace qn {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));
// 128-bit global accesses at element alignment: gfx950 under HSA runs with
// unaligned global access enabled, so one dwordx4 instruction serves any
// element-aligned address (columns of a matrix whose n is not a multiple of 4).
typedef v4f v4f_elem __attribute__((aligned(4)));
typedef v4u v4u_elem __attribute__((aligned(2)));

// worker columns whose loads are issued together (two such chunks are in flight),
// by storage type, launch shape and compiled-in worker count.  Measured on MI355X,
// chunks of 4 against 8, fp32 storage: in the staged kernel at n = 124M m = 16:
// 2.54 vs 2.63 ms, m = 32: 4.83 vs 4.88 ms, m = 8 and 64: no difference, and with
// the worker count known only at run time (m = 24, 48) chunks of 4 are 6 % slower;
// in the direct kernel (n = 8M) chunks of 4 are 2 % slower.  16-bit storage is
// indifferent.
#ifndef QN_APPLY_CHUNK_F32
#define QN_APPLY_CHUNK_F32(STAGED, MC) (((STAGED) && ((MC) == 16 || (MC) == 32)) ? 4 : 8)
#endif
#ifndef QN_APPLY_CHUNK_BF16
#define QN_APPLY_CHUNK_BF16 2
#endif
// bf16 storage: accumulate the stored values themselves instead of differences
// to the pivot (see compute_rows)
#ifndef QN_APPLY_BF16_RAW
#define QN_APPLY_BF16_RAW 1
#endif
// Type of the sum over the workers: fp64 for fp32 storage (see the header), fp32
// for the 16-bit storage types, whose own resolution is far coarser.
template <int DT> struct ApplyAcc { using type = float; };
template <> struct ApplyAcc<QN_F32> { using type = double; };
__device__ __forceinline__ float fma_acc(float a, float b, float c) { return fmaf(a, b, c); }
__device__ __forceinline__ double fma_acc(double a, float b, double c)
{
    return fma(a, static_cast<double>(b), c);
}
// c_k: from the double vector when there is one (fp32 storage, fused steps)
template <typename Acc>
__device__ __forceinline__ Acc coef_at(const float *__restrict__ c,
                                       const double *__restrict__ c64, int k)
{
    if constexpr (sizeof(Acc) == sizeof(double))
        return c64 != nullptr ? c64[k] : static_cast<double>(c[k]);
    else
        return c[k];
}
template <typename Acc>
__device__ __forceinline__ Acc coef_sum(const float *__restrict__ c,
                                        const double *__restrict__ c64, int m)
{
    Acc s = 0;
    for (int k = 0; k < m; ++k)
        s += coef_at<Acc>(c, c64, k);
    return s;
}
template <int DT, int MC, bool STAGED> struct ApplyChunk {
    static constexpr int value = DT == QN_F32 ? QN_APPLY_CHUNK_F32(STAGED, MC) : QN_APPLY_CHUNK_BF16;
};

// One load of R rows of a column kept as it arrives (16 bytes, or one element),
// and its unpacking to fp32.  The pipelined loop below carries loads across
// iterations in this form: unpacking 16-bit values at load time would make every
// iteration wait for the loads it has just issued.
template <int DT, int R> struct RawRows {
    using type = v4u;           // R == 4 fp32 values or R == 8 bf16 values
};
template <> struct RawRows<QN_F32, 1> { using type = float; };
template <> struct RawRows<QN_BF16, 1> { using type = uint16_t; };
template <> struct RawRows<QN_F16, 1> { using type = uint16_t; };

__device__ __forceinline__ float half_bits_to_float(uint32_t h)
{
    return static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(h)));
}

template <int DT, int R>
__device__ __forceinline__ typename RawRows<DT, R>::type load_raw(const void *base, int64_t elem)
{
    if constexpr (R == 1) {
        return static_cast<const typename RawRows<DT, 1>::type *>(base)[elem];
    } else {
        const char *p = static_cast<const char *>(base) + elem * (DT == QN_F32 ? 4 : 2);
        if constexpr (DT == QN_F32)
            return __builtin_bit_cast(v4u, __builtin_nontemporal_load(reinterpret_cast<const v4f_elem *>(p)));
        else
            return __builtin_nontemporal_load(reinterpret_cast<const v4u_elem *>(p));
    }
}

template <int DT, int R>
__device__ __forceinline__ void unpack_rows(const typename RawRows<DT, R>::type &v, float (&x)[R])
{
    if constexpr (R == 1) {
        if constexpr (DT == QN_F32)
            x[0] = v;
        else if constexpr (DT == QN_BF16)
            x[0] = __uint_as_float(static_cast<uint32_t>(v) << 16);
        else
            x[0] = half_bits_to_float(v);
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
                x[2 * h + 0] = half_bits_to_float(u[h] & 0xffffu);
                x[2 * h + 1] = half_bits_to_float(u[h] >> 16);
            }
        }
    }
}

template <int DT, int R>
__device__ __forceinline__ void load_vec(const void *base, int64_t elem, float (&x)[R])
{
    unpack_rows<DT, R>(load_raw<DT, R>(base, elem), x);
}

// theta_new for rows [row, row + R), from every worker column.
template <int DT, int MC, int R, bool STAGED>
__device__ __forceinline__ void compute_rows(const void *__restrict__ thetas,
                                             const void *__restrict__ grads,
                                             int64_t row, int m_rt, int64_t ld,
                                             const float *__restrict__ c,
                                             const double *__restrict__ c64,
                                             const float *__restrict__ z,
                                             typename ApplyAcc<DT>::type csum,
                                             float tau, float inv_m,
                                             float (&res)[R])
{
    constexpr int kApplyChunk = ApplyChunk<DT, MC, STAGED>::value;
    // 16-bit storage: the inputs carry 8 or 11 significant bits, so plain fp32 sums of the
    // stored values (St = sum theta_k, acc = sum c_k (theta_k - g_k), error about
    // 1e-7 of the values) are far inside the data's own resolution and save a
    // third of the arithmetic, which this path is short of (twice the elements
    // per byte).  fp32 storage keeps the pivot form.
    constexpr bool RAW = DT != QN_F32 && QN_APPLY_BF16_RAW;
    const int m = MC ? MC : m_rt;
    using Acc = typename ApplyAcc<DT>::type;   // double for fp32 storage
    float p[R], r[R], st[R], sh[R];
    Acc acc[R];
    load_vec<DT, R>(thetas, row, p);
    load_vec<DT, R>(grads, row, r);
    const float c0 = RAW ? c[0] : 0.0f;
#pragma unroll
    for (int e = 0; e < R; ++e) {
        st[e] = RAW ? p[e] : 0.0f;
        sh[e] = RAW ? r[e] : 0.0f;
        acc[e] = RAW ? c0 * (p[e] - r[e]) : 0.0f;
    }
    // Columns 1..m-1 in chunks of kApplyChunk, software-pipelined over a real
    // (not unrolled) loop: the loads of the next chunk are issued before the
    // current chunk is consumed, so 2*kApplyChunk 128-bit loads per lane stay in
    // flight while the register footprint stays bounded.
    using Raw = typename RawRows<DT, R>::type;
    Raw th[kApplyChunk] = {}, gr[kApplyChunk] = {};
#pragma unroll
    for (int u = 0; u < kApplyChunk; ++u)
        if (1 + u < m) {
            th[u] = load_raw<DT, R>(thetas, (1 + u) * ld + row);
            gr[u] = load_raw<DT, R>(grads, (1 + u) * ld + row);
        }
#pragma unroll 1
    for (int k0 = 1; k0 < m; k0 += kApplyChunk) {
        Raw thn[kApplyChunk] = {}, grn[kApplyChunk] = {};
        const int kn = k0 + kApplyChunk;
#pragma unroll
        for (int u = 0; u < kApplyChunk; ++u)
            if (kn + u < m) {
                thn[u] = load_raw<DT, R>(thetas, (kn + u) * ld + row);
                grn[u] = load_raw<DT, R>(grads, (kn + u) * ld + row);
            }
#pragma unroll
        for (int u = 0; u < kApplyChunk; ++u)
            if (k0 + u < m) {
                const Acc ck = coef_at<Acc>(c, c64, k0 + u);
                float tv[R], gv[R];
                unpack_rows<DT, R>(th[u], tv);
                unpack_rows<DT, R>(gr[u], gv);
#pragma unroll
                for (int e = 0; e < R; ++e) {
                    const float t = RAW ? tv[e] : tv[e] - p[e];
                    const float h = RAW ? gv[e] : gv[e] - r[e];
                    st[e] += t;
                    sh[e] += h;
                    acc[e] = fma_acc(ck, t - h, acc[e]);
                }
            }
#pragma unroll
        for (int u = 0; u < kApplyChunk; ++u) {
            th[u] = thn[u];
            gr[u] = grn[u];
        }
    }
    float zz[R];
    if (z != nullptr) {   // uniform
        if constexpr (R == 1) {
            zz[0] = z[row];
        } else {
#pragma unroll
            for (int e = 0; e < R; e += 4) {
                const v4f v = __builtin_nontemporal_load(reinterpret_cast<const v4f_elem *>(z + row + e));
                zz[e] = v.x; zz[e + 1] = v.y; zz[e + 2] = v.z; zz[e + 3] = v.w;
            }
        }
    }
#pragma unroll
    for (int e = 0; e < R; ++e) {
        const float mt = st[e] * inv_m, mh = sh[e] * inv_m;
        if constexpr (RAW) {    // mt, mh are theta_bar, g_bar themselves
            const float corr = acc[e] - csum * (mt - mh);
            res[e] = z != nullptr ? zz[e] + corr : mt - tau * (mh + corr);
        } else {
            // fp64 from here on: (r + mh) + corr is where g_bar meets - G c
            const double corr = acc[e] - csum * (static_cast<double>(mt) - mh);
            const double v = z != nullptr
                ? zz[e] + corr
                : (static_cast<double>(p[e]) + mt) -
                      static_cast<double>(tau) * ((static_cast<double>(r[e]) + mh) + corr);
            res[e] = static_cast<float>(v);
        }
    }
}

// Computes rows [row, row + R) and stores them straight to memory.
template <int DT, int MC, int R>
__device__ __forceinline__ void apply_rows(const void *__restrict__ thetas,
                                           const void *__restrict__ grads,
                                           int64_t row, int m_rt, int64_t ld,
                                           const float *__restrict__ c,
                                           const double *__restrict__ c64,
                                           const float *__restrict__ z,
                                           typename ApplyAcc<DT>::type csum,
                                           float tau, float inv_m,
                                           float *__restrict__ out)
{
    float res[R];
    compute_rows<DT, MC, R, false>(thetas, grads, row, m_rt, ld, c, c64, z, csum, tau, inv_m, res);
    if constexpr (R == 1) {
        out[row] = res[0];
    } else {
#pragma unroll
        for (int e = 0; e < R; e += 4) {
            v4f v = {res[e], res[e + 1], res[e + 2], res[e + 3]};
            __builtin_nontemporal_store(v, reinterpret_cast<v4f_elem *>(out + row + e));
        }
    }
}

template <int DT, int MC, bool VEC>
__global__ __launch_bounds__(kApplyThreads) void apply_kernel(
    const void *__restrict__ thetas, const void *__restrict__ grads, int64_t n,
    int m_rt, int64_t ld, const float *__restrict__ c, const double *__restrict__ c64,
    const float *__restrict__ z, float tau_host, const float *__restrict__ tau_dev,
    float *__restrict__ out)
{
    constexpr int R = VEC ? (DT == QN_F32 ? 4 : 8) : 1;
    const int m = MC ? MC : m_rt;
    const float tau = tau_dev != nullptr ? *tau_dev : tau_host;   // uniform
    using Acc = typename ApplyAcc<DT>::type;
    const Acc csum = coef_sum<Acc>(c, c64, m);
    const float inv_m = 1.0f / static_cast<float>(m);

    const int64_t nvec = n / R;
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kApplyThreads;
    for (int64_t v = static_cast<int64_t>(blockIdx.x) * kApplyThreads + threadIdx.x;
         v < nvec; v += stride)
        apply_rows<DT, MC, R>(thetas, grads, v * R, m_rt, ld, c, c64, z, csum, tau, inv_m, out);

    if constexpr (R > 1) {   // rows past the last full vector
        const int64_t tail0 = nvec * R;
        if (blockIdx.x == 0 && tail0 + threadIdx.x < n)
            apply_rows<DT, MC, 1>(thetas, grads, tail0 + threadIdx.x, m_rt, ld, c, c64, z,
                                  csum, tau, inv_m, out);
    }
}

// Large-n variant.  A thin write stream mixed into a read stream that saturates
// HBM is disproportionately expensive (measured on MI355X: the 0.5 GB of output
// at the 124M x 32 size costs 0.9 ms when every wave stores its 1 KiB as soon as
// it is computed, 0.26 ms when each CU writes 128 KiB bursts).  So one block
// per CU keeps a slab of results in LDS and writes it out in one contiguous
// burst.  Same arithmetic, same bits as apply_kernel.
// block size of the staged variant: fp32 streams best with 4 waves per CU (2 are
// too few: 7.5 vs 4.8 ms); 16-bit storage has twice the arithmetic per byte and
// takes 8 (16 waves are 0.5 ... 2 % slower at every worker count)
template <int DT> struct StagedThreads {
    static constexpr int value = staged_threads(DT);
};

template <int DT, int MC>
__global__ __launch_bounds__(StagedThreads<DT>::value) void apply_staged(
    const void *__restrict__ thetas, const void *__restrict__ grads, int64_t n,
    int m_rt, int64_t ld, const float *__restrict__ c, const double *__restrict__ c64,
    const float *__restrict__ z, float tau_host, const float *__restrict__ tau_dev,
    float *__restrict__ out, int steps)
{
    const float tau = tau_dev != nullptr ? *tau_dev : tau_host;   // uniform
    constexpr int kStagedThreads = StagedThreads<DT>::value;
    constexpr int R = DT == QN_F32 ? 4 : 8;        // rows per lane per step
    constexpr int Q = R / 4;                       // 128-bit results per lane per step
    // steps <= staged_max_steps(DT): lane-steps per thread per slab
    extern __shared__ v4f stage[];
    const int m = MC ? MC : m_rt;
    using Acc = typename ApplyAcc<DT>::type;
    const Acc csum = coef_sum<Acc>(c, c64, m);
    const float inv_m = 1.0f / static_cast<float>(m);

    const int64_t nvec = n / R;
    const int64_t slab = static_cast<int64_t>(steps) * kStagedThreads;   // lane-steps per slab
#pragma unroll 1
    for (int64_t base = static_cast<int64_t>(blockIdx.x) * slab; base < nvec;
         base += static_cast<int64_t>(gridDim.x) * slab) {
#pragma unroll 1
        for (int it = 0; it < steps; ++it) {
            const int64_t v = base + static_cast<int64_t>(it) * kStagedThreads + threadIdx.x;
            if (v < nvec) {
                float res[R];
                compute_rows<DT, MC, R, true>(thetas, grads, v * R, m_rt, ld, c, c64, z, csum, tau, inv_m, res);
#pragma unroll
                for (int h = 0; h < Q; ++h)
                    stage[(it * kStagedThreads + threadIdx.x) * Q + h] =
                        (v4f){res[4 * h], res[4 * h + 1], res[4 * h + 2], res[4 * h + 3]};
            }
        }
        __syncthreads();
        // the slab's results are contiguous in memory: rows [base*R, (base+slab)*R)
        v4f_elem *dst = reinterpret_cast<v4f_elem *>(out) + base * Q;
        const int count = static_cast<int>(staged_slab_count(nvec, base, slab) * Q);
#pragma unroll 1
        for (int i = threadIdx.x; i < count; i += kStagedThreads)
            __builtin_nontemporal_store(stage[i], dst + i);
        __syncthreads();
    }

    const int64_t tail0 = nvec * R;                // rows past the last full vector
    if (blockIdx.x == 0 && tail0 + threadIdx.x < n)
        apply_rows<DT, MC, 1>(thetas, grads, tail0 + threadIdx.x, m_rt, ld, c, c64, z, csum,
                              tau, inv_m, out);
}

template <int DT, int MC>
static void launch_mc(const ApplyPlan &plan, const void *thetas, const void *grads,
                      int64_t n, int m, int64_t ld, const float *c, const double *c64,
                      const float *z, float tau, const float *tau_dev, float *out,
                      hipStream_t stream)
{
    if (plan.shape == kApplyStaged)
        hipLaunchKernelGGL((apply_staged<DT, MC>), dim3(plan.grid), dim3(StagedThreads<DT>::value),
                           kStagedLdsBytes, stream, thetas, grads, n, m, ld, c, c64, z, tau, tau_dev,
                           out, plan.steps);
    else if (plan.shape == kApplyDirect)
        hipLaunchKernelGGL((apply_kernel<DT, MC, true>), dim3(plan.grid), dim3(kApplyThreads),
                           0, stream, thetas, grads, n, m, ld, c, c64, z, tau, tau_dev, out);
    else
        hipLaunchKernelGGL((apply_kernel<DT, MC, false>), dim3(plan.grid), dim3(kApplyThreads),
                           0, stream, thetas, grads, n, m, ld, c, c64, z, tau, tau_dev, out);
}

template <int DT>
static void launch_dt(const ApplyPlan &plan, const void *thetas, const void *grads,
                      int64_t n, int m, int64_t ld, const float *c, const double *c64,
                      const float *z, float tau, const float *tau_dev, float *out,
                      hipStream_t stream)
{
    switch (m) {
    case 4: launch_mc<DT, 4>(plan, thetas, grads, n, m, ld, c, c64, z, tau, tau_dev, out, stream); break;
    case 8: launch_mc<DT, 8>(plan, thetas, grads, n, m, ld, c, c64, z, tau, tau_dev, out, stream); break;
    case 16: launch_mc<DT, 16>(plan, thetas, grads, n, m, ld, c, c64, z, tau, tau_dev, out, stream); break;
    case 32: launch_mc<DT, 32>(plan, thetas, grads, n, m, ld, c, c64, z, tau, tau_dev, out, stream); break;
    case 64: launch_mc<DT, 64>(plan, thetas, grads, n, m, ld, c, c64, z, tau, tau_dev, out, stream); break;
    default: launch_mc<DT, 0>(plan, thetas, grads, n, m, ld, c, c64, z, tau, tau_dev, out, stream); break;
    }
}

// Per-device opt-in to 128 KiB of dynamic LDS for the staged kernels.
int setup_apply_kernels()
{
    bool ok = true;
#define QN_OPT_IN(DTV, MCV)                                                            \
    ok = ok && hipFuncSetAttribute(reinterpret_cast<const void *>(apply_staged<DTV, MCV>), \
                                   hipFuncAttributeMaxDynamicSharedMemorySize,        \
                                   kStagedLdsBytes) == hipSuccess
    QN_OPT_IN(QN_F32, 0); QN_OPT_IN(QN_F32, 4); QN_OPT_IN(QN_F32, 8);
    QN_OPT_IN(QN_F32, 16); QN_OPT_IN(QN_F32, 32); QN_OPT_IN(QN_F32, 64);
    QN_OPT_IN(QN_BF16, 0); QN_OPT_IN(QN_BF16, 4); QN_OPT_IN(QN_BF16, 8);
    QN_OPT_IN(QN_BF16, 16); QN_OPT_IN(QN_BF16, 32); QN_OPT_IN(QN_BF16, 64);
    QN_OPT_IN(QN_F16, 0); QN_OPT_IN(QN_F16, 4); QN_OPT_IN(QN_F16, 8);
    QN_OPT_IN(QN_F16, 16); QN_OPT_IN(QN_F16, 32); QN_OPT_IN(QN_F16, 64);
#undef QN_OPT_IN
    return ok ? QN_OK : QN_ELAUNCH;
}

int launch_apply(const void *thetas, const void *grads, int dtype, int64_t n,
                 int m, int64_t ld, const float *c, const float *z, float tau,
                 const float *tau_dev, float *theta_new, int cu_count, hipStream_t stream,
                 const double *c64)
{
    // launch shape, grid and slab length: a function of (n, dtype, CU count) only
    const ApplyPlan plan = apply_plan(n, dtype, cu_count);
    TraceScope ts(QN_K_APPLY, stream);
    if (dtype == QN_F32)
        launch_dt<QN_F32>(plan, thetas, grads, n, m, ld, c, c64, z, tau, tau_dev, theta_new, stream);
    else if (dtype == QN_BF16)
        launch_dt<QN_BF16>(plan, thetas, grads, n, m, ld, c, nullptr, z, tau, tau_dev, theta_new, stream);
    else
        launch_dt<QN_F16>(plan, thetas, grads, n, m, ld, c, nullptr, z, tau, tau_dev, theta_new, stream);
    return check_launch();
}

}  // namespace qn
