// C = G^T G and w = G^T g_bar for the centred gradient matrix G of Section 2
// (G's k-th column is grad_k - g_bar; V_G's columns are eigenvectors of G^T G,
// and eq. (4)'s alpha_k are built from G^T g_bar).
//
// Shifted formulation.  Centring needs all m values of a row, but the matrix
// cores want one lane per column.  So the streaming pass subtracts worker 0's
// value (the "pivot" s_i = grad_0[i]) from every other column instead of the
// row mean: D = [ s | grad_1 - s | ... | grad_{m-1} - s ].  D's entries have the
// magnitude of G's (no cancellation in fp32: the subtraction of two nearby fp32
// numbers is exact or correctly rounded), and the Gram matrix Q = D^T D holds
//     Q[k][l] = d_k^T d_l   (k, l >= 1),      Q[k][0] = d_k^T s.
// With N = Q restricted to k, l >= 1 (row/column 0 zero), t_k = Q[k][0] and the
// centring projector P = I - 11^T/m one has G = [0 | d_1 .. d_{m-1}] P and
// g_bar = s + (1/m) sum_k d_k, hence, at m x m size and in fp64,
//     C = P N P,        w = P ( t + (1/m) N 1 ).
//
// Stage 1 (gram_stage1): one streaming pass over grads on v_mfma_f32_16x16x4_f32.
//   Lane l of a wavefront owns column l%16 (and l%16 + 16 when m > 16) and the
//   row group l/16; A and B operands of the Gram product are the same register.
//   Only the lower triangle of the 2x2 tiling is computed (3 of 4 tiles).
//   MFMA accumulators run over one 128-row tile in fp32 and are then added to
//   per-lane fp64 totals; waves are combined through LDS in a fixed order and
//   each block writes one partial.  No atomics.
// Stage 2 (gram_reduce): fixed-order fp64 sum of the block partials.
// Stage 3 (gram_project): the m x m algebra above.
#include "qn_internal.h"

namespace qn {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));

constexpr int kRowsPerLane = 32;                  // per column, per tile
constexpr int kTileRows = 4 * kRowsPerLane;       // 4 row groups per wavefront

// Loads kRowsPerLane consecutive rows of one column into fp32 registers.
// VEC: 128-bit loads (caller guarantees 16-byte alignment and a full tile).
template <int DT, bool VEC>
__device__ __forceinline__ void load_rows(const void *base, int64_t elem0,
                                          int64_t rows_valid,
                                          float (&x)[kRowsPerLane])
{
    if constexpr (DT == QN_F32) {
        const float *p = static_cast<const float *>(base) + elem0;
        if constexpr (VEC) {
            const v4f *p4 = reinterpret_cast<const v4f *>(p);
#pragma unroll
            for (int i = 0; i < kRowsPerLane / 4; ++i) {
                const v4f v = p4[i];
                x[4 * i + 0] = v.x;
                x[4 * i + 1] = v.y;
                x[4 * i + 2] = v.z;
                x[4 * i + 3] = v.w;
            }
        } else {
#pragma unroll
            for (int i = 0; i < kRowsPerLane; ++i)
                x[i] = (i < rows_valid) ? p[i] : 0.0f;
        }
    } else {
        const uint16_t *p = static_cast<const uint16_t *>(base) + elem0;
        if constexpr (VEC) {
            const v4u *p4 = reinterpret_cast<const v4u *>(p);
#pragma unroll
            for (int i = 0; i < kRowsPerLane / 8; ++i) {
                const v4u v = p4[i];
                const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int h = 0; h < 4; ++h) {
                    x[8 * i + 2 * h + 0] = __uint_as_float(u[h] << 16);
                    x[8 * i + 2 * h + 1] = __uint_as_float(u[h] & 0xffff0000u);
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < kRowsPerLane; ++i)
                x[i] = (i < rows_valid)
                           ? __uint_as_float(static_cast<uint32_t>(p[i]) << 16)
                           : 0.0f;
        }
    }
}

// NT = 1: m <= 16 (one 16x16 tile); NT = 2: m <= 32 (three tiles).
template <int DT, int NT, bool VEC>
__global__ __launch_bounds__(kGramThreads) void gram_stage1(
    const void *__restrict__ grads, int64_t n, int m, int64_t ld,
    double *__restrict__ partials)
{
    constexpr int TILES = (NT == 1) ? 1 : 3;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int col = lane & 15;
    const int group = lane >> 4;
    const bool has_a = col < m;
    const bool has_b = (NT == 2) && (col + 16 < m);

    double tot[TILES][4];
#pragma unroll
    for (int t = 0; t < TILES; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r)
            tot[t][r] = 0.0;

    const int64_t num_tiles = (n + kTileRows - 1) / kTileRows;
    const int64_t wave_stride = static_cast<int64_t>(gridDim.x) * kGramWaves;
    for (int64_t tile = static_cast<int64_t>(blockIdx.x) * kGramWaves + wave;
         tile < num_tiles; tile += wave_stride) {
        const int64_t row0 = tile * kTileRows + group * kRowsPerLane;
        const bool full = (tile + 1) * kTileRows <= n;

        float a[kRowsPerLane], b[kRowsPerLane];
#pragma unroll
        for (int i = 0; i < kRowsPerLane; ++i) {
            a[i] = 0.0f;
            b[i] = 0.0f;
        }
        if (VEC && full) {
            if (has_a)
                load_rows<DT, VEC>(grads, col * ld + row0, kRowsPerLane, a);
            if (has_b)
                load_rows<DT, VEC>(grads, (col + 16) * ld + row0, kRowsPerLane, b);
        } else {
            int64_t valid = n - row0;
            valid = valid < 0 ? 0 : (valid > kRowsPerLane ? kRowsPerLane : valid);
            if (has_a && valid > 0)
                load_rows<DT, false>(grads, col * ld + row0, valid, a);
            if (has_b && valid > 0)
                load_rows<DT, false>(grads, (col + 16) * ld + row0, valid, b);
        }

        // pivot shift: lane (group*16) holds column 0 of this row group
        const int src = (lane & 48) << 2;
#pragma unroll
        for (int i = 0; i < kRowsPerLane; ++i) {
            const float s = __int_as_float(
                __builtin_amdgcn_ds_bpermute(src, __float_as_int(a[i])));
            a[i] = (col == 0) ? a[i] : (has_a ? a[i] - s : 0.0f);
            if (NT == 2)
                b[i] = has_b ? b[i] - s : 0.0f;
        }

        v4f acc[TILES];
#pragma unroll
        for (int t = 0; t < TILES; ++t)
            acc[t] = (v4f){0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int i = 0; i < kRowsPerLane; ++i) {
            acc[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[i], a[i], acc[0], 0, 0, 0);
            if constexpr (NT == 2) {
                acc[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(b[i], a[i], acc[1], 0, 0, 0);
                acc[2] = __builtin_amdgcn_mfma_f32_16x16x4f32(b[i], b[i], acc[2], 0, 0, 0);
            }
        }
#pragma unroll
        for (int t = 0; t < TILES; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                tot[t][r] += static_cast<double>(acc[t][r]);
    }

    // combine the wavefronts of the block in wave order
    __shared__ double red[kGramWaves][TILES * 4][64];
#pragma unroll
    for (int t = 0; t < TILES; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r)
            red[wave][t * 4 + r][lane] = tot[t][r];
    __syncthreads();
    constexpr int ENTRIES = TILES * kTileEntries;
    for (int e = threadIdx.x; e < ENTRIES; e += kGramThreads) {
        double s = 0.0;
#pragma unroll
        for (int wv = 0; wv < kGramWaves; ++wv)
            s += red[wv][e >> 6][e & 63];
        partials[static_cast<int64_t>(blockIdx.x) * ENTRIES + e] = s;
    }
}

// Fixed-order fp64 sum over the block partials.  Block b owns 64 entries; 16
// slices of partials are summed serially per thread, then in slice order.
constexpr int kReduceSlices = 16;
__global__ __launch_bounds__(64 * kReduceSlices) void gram_reduce(
    const double *__restrict__ partials, int num_partials, int entries,
    double *__restrict__ mraw)
{
    __shared__ double part[kReduceSlices][64];
    const int e = blockIdx.x * 64 + (threadIdx.x & 63);
    const int slice = threadIdx.x >> 6;
    double s = 0.0;
    for (int p = slice; p < num_partials; p += kReduceSlices)
        s += partials[static_cast<int64_t>(p) * entries + e];
    part[slice][threadIdx.x & 63] = s;
    __syncthreads();
    if (slice == 0) {
        double r = 0.0;
#pragma unroll
        for (int k = 0; k < kReduceSlices; ++k)
            r += part[k][threadIdx.x];
        mraw[e] = r;
    }
}

// Position of Q[k][l] (k >= l) in the raw accumulator layout: tile (k/16, l/16)
// of the lower triangle, and inside a tile element (i, j) sits in register i%4
// of lane 16*(i/4) + j.
__device__ __forceinline__ int raw_index(int k, int l)
{
    const int ti = k >> 4, tj = l >> 4;
    const int tile = ti + tj;              // (0,0)->0, (1,0)->1, (1,1)->2
    const int i = k & 15, j = l & 15;
    return (tile * 4 + (i & 3)) * 64 + (i >> 2) * 16 + j;
}

// C = P N P and w = P (t + N 1 / m) in fp64; one block of QN_MAX_M^2 threads.
__global__ __launch_bounds__(QN_MAX_M *QN_MAX_M) void gram_project(
    const double *__restrict__ mraw, int m, double *__restrict__ C,
    double *__restrict__ w)
{
    __shared__ double N[QN_MAX_M][QN_MAX_M + 1];
    __shared__ double rowsum[QN_MAX_M], u[QN_MAX_M];
    __shared__ double total, umean;
    const int k = threadIdx.x / QN_MAX_M, l = threadIdx.x % QN_MAX_M;
    double q = 0.0;
    if (k < m && l < m && k >= 1 && l >= 1)
        q = (k >= l) ? mraw[raw_index(k, l)] : mraw[raw_index(l, k)];
    N[k][l] = q;
    __syncthreads();
    if (threadIdx.x < QN_MAX_M) {
        double s = 0.0;
        for (int x = 0; x < m; ++x)
            s += N[threadIdx.x][x];
        rowsum[threadIdx.x] = s;
        const double t = (threadIdx.x >= 1 && threadIdx.x < m)
                             ? mraw[raw_index(threadIdx.x, 0)] : 0.0;
        u[threadIdx.x] = t + s / m;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double s = 0.0, su = 0.0;
        for (int x = 0; x < m; ++x) {
            s += rowsum[x];
            su += u[x];
        }
        total = s;
        umean = su / m;
    }
    __syncthreads();
    if (k < m && l < m)
        C[l * m + k] = N[k][l] - (rowsum[k] + rowsum[l]) / m + total / (static_cast<double>(m) * m);
    if (threadIdx.x < m)
        w[threadIdx.x] = u[threadIdx.x] - umean;
}

template <int DT, int NT>
static void launch_stage1(bool vec, int grid, const void *grads, int64_t n,
                          int m, int64_t ld, double *partials,
                          hipStream_t stream)
{
    if (vec)
        hipLaunchKernelGGL((gram_stage1<DT, NT, true>), dim3(grid), dim3(kGramThreads),
                           0, stream, grads, n, m, ld, partials);
    else
        hipLaunchKernelGGL((gram_stage1<DT, NT, false>), dim3(grid), dim3(kGramThreads),
                           0, stream, grads, n, m, ld, partials);
}

int launch_gram(const void *grads, int dtype, int64_t n, int m, int64_t ld,
                Workspace *ws, double *C, double *w, hipStream_t stream)
{
    const size_t esz = dtype == QN_F32 ? 4 : 2;
    const bool vec = (reinterpret_cast<uintptr_t>(grads) % 16 == 0) &&
                     ((static_cast<uint64_t>(ld) * esz) % 16 == 0);
    const int nt = m <= 16 ? 1 : 2;
    const int entries = (nt == 1 ? 1 : 3) * kTileEntries;

    // grid: a function of n only (and of the device's CU count)
    const int64_t num_tiles = (n + kTileRows - 1) / kTileRows;
    int64_t want = (num_tiles + kGramWaves - 1) / kGramWaves;
    int64_t cap = static_cast<int64_t>(ws->cu_count) * 2;
    if (cap > kGramMaxBlocks)
        cap = kGramMaxBlocks;
    const int grid = static_cast<int>(want < cap ? want : cap);

    {
        TraceScope ts(QN_K_GRAM, stream);
        if (dtype == QN_F32) {
            if (nt == 1) launch_stage1<QN_F32, 1>(vec, grid, grads, n, m, ld, ws->partials, stream);
            else launch_stage1<QN_F32, 2>(vec, grid, grads, n, m, ld, ws->partials, stream);
        } else {
            if (nt == 1) launch_stage1<QN_BF16, 1>(vec, grid, grads, n, m, ld, ws->partials, stream);
            else launch_stage1<QN_BF16, 2>(vec, grid, grads, n, m, ld, ws->partials, stream);
        }
    }
    if (check_launch() != QN_OK) return QN_ELAUNCH;
    {
        TraceScope ts(QN_K_REDUCE, stream);
        hipLaunchKernelGGL(gram_reduce, dim3(entries / 64), dim3(64 * kReduceSlices), 0,
                           stream, ws->partials, grid, entries, ws->mraw);
    }
    if (check_launch() != QN_OK) return QN_ELAUNCH;
    {
        TraceScope ts(QN_K_PROJECT, stream);
        hipLaunchKernelGGL(gram_project, dim3(1), dim3(QN_MAX_M * QN_MAX_M), 0, stream,
                           ws->mraw, m, C, w);
    }
    return check_launch();
}

}  // namespace qn
