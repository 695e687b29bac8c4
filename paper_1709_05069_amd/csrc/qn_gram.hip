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
// Stage 1: one streaming pass over grads on v_mfma_f32_16x16x4_f32.  For a Gram
//   product the A and B operands are the same register: lane l of a wavefront
//   supplies column l%16 (and l%16 + 16 when m > 16) for the row slot l/16, and
//   any assignment of rows to the four slots is valid as long as both operands
//   agree.  Only the lower triangle of the 2x2 tiling is computed (3 of 4
//   tiles).  MFMA accumulators run in fp32 over one tile and are then added to
//   per-lane fp64 totals; waves are combined through LDS in a fixed order and
//   each block writes one partial.  No atomics.
//   gram_stage1_stream: HBM -> LDS with coalesced direct-to-LDS loads carrying the
//     non-temporal hint (128-bit per lane when the columns are 16-byte aligned:
//     every wave instruction moves 1 KiB of one column; element-sized per lane
//     otherwise), two LDS stages per block, two blocks per CU; the wavefronts
//     then read their operands from LDS in the lane = column layout.
//     Measured on MI355X this load pattern sustains about 7.0 TB/s, against
//     6.4 TB/s when each lane fetches its own column straight from HBM.
//     For bf16 storage the fp32 matrix cores would be the bottleneck (twice the
//     elements per byte), so that path runs on v_mfma_f32_16x16x32_bf16: the
//     shifted fp32 value is split into two bf16 terms and the four cross
//     products are accumulated (exact for all but widely different magnitudes).
//     (Unaligned bf16 input stays on the fp32 matrix cores: 2-byte direct-to-LDS
//     loads land one value per dword.)
// Stage 2 (gram_reduce): fixed-order fp64 sum of the block partials.
// Stage 3 (gram_project): the m x m algebra above.
#include "qn_internal.h"

namespace qn {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));

#define QN_GPTR(p) ((const __attribute__((address_space(1))) void *)(p))
#define QN_LPTR(p) ((__attribute__((address_space(3))) void *)(p))

template <int NT> struct GramTiles { static constexpr int value = (NT == 1) ? 1 : 3; };

// Combines the per-lane fp64 totals of the block's wavefronts in wave order
// and writes the block's partial.  `red` must hold kGramWaves*TILES*4*64 doubles.
template <int TILES>
__device__ __forceinline__ void write_block_partial(const double (&tot)[TILES][4],
                                                    double *red, double *partials)
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
#pragma unroll
    for (int t = 0; t < TILES; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r)
            red[(wave * TILES * 4 + t * 4 + r) * 64 + lane] = tot[t][r];
    __syncthreads();
    constexpr int ENTRIES = TILES * kTileEntries;
    for (int e = threadIdx.x; e < ENTRIES; e += kGramThreads) {
        double s = 0.0;
#pragma unroll
        for (int wv = 0; wv < kGramWaves; ++wv)
            s += red[wv * ENTRIES + e];
        partials[static_cast<int64_t>(blockIdx.x) * ENTRIES + e] = s;
    }
}

// One MFMA k-step for the three lower-triangle tiles (or the single tile).
template <int NT>
__device__ __forceinline__ void gram_step(float da, float db, v4f (&acc)[GramTiles<NT>::value])
{
    acc[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(da, da, acc[0], 0, 0, 0);
    if constexpr (NT == 2) {
        acc[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(db, da, acc[1], 0, 0, 0);
        acc[2] = __builtin_amdgcn_mfma_f32_16x16x4f32(db, db, acc[2], 0, 0, 0);
    }
}

// ---------------------------------------------------------------------------
// Fast path.  Tile = kStreamRows rows of all columns; a column's rows of one tile
// are 1 KiB of contiguous memory (256 fp32 or 512 bf16 rows) and land in LDS at
// column * kColPitch (1 KiB + 16 B, which spreads the 16 columns a quarter-wave
// reads over all banks).
constexpr int kColPitch = 1040;                       // bytes per column slot
constexpr int kStageBytes = QN_MAX_M * kColPitch;     // 33 280
constexpr int kStreamLdsBytes = 2 * kStageBytes;      // two stages

// Rows per tile: a column's tile is 1 KiB in LDS.  bf16 inputs that are not
// 16-byte aligned arrive through 2-byte direct-to-LDS loads, which the hardware
// stores zero-extended, one per dword: their LDS format is 4 bytes per row.
template <int DT, bool ALIGNED> struct StreamRows {
    static constexpr int value = (DT == QN_F32 || !ALIGNED) ? 256 : 512;
};

// 16 bytes of one column from LDS as fp32 row values.  FMT 0: fp32; 1: packed
// bf16 (8 rows); 2: bf16 zero-extended to one dword per row (4 rows).
template <int FMT>
__device__ __forceinline__ void lds_rows(const char *p, float (&x)[FMT == 1 ? 8 : 4])
{
    if constexpr (FMT == 0) {
        const v4f v = *reinterpret_cast<const v4f *>(p);
        x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
    } else if constexpr (FMT == 2) {
        const v4u v = *reinterpret_cast<const v4u *>(p);
        x[0] = __uint_as_float(v.x << 16); x[1] = __uint_as_float(v.y << 16);
        x[2] = __uint_as_float(v.z << 16); x[3] = __uint_as_float(v.w << 16);
    } else {
        const v4u v = *reinterpret_cast<const v4u *>(p);
        const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            x[2 * h + 0] = __uint_as_float(u[h] << 16);
            x[2 * h + 1] = __uint_as_float(u[h] & 0xffff0000u);
        }
    }
}

typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));

// d = present ? (keep_raw ? x : x - s) : 0, split into bf16 hi + lo (see the caller).
template <int N>
__device__ __forceinline__ void split_bf16(const float (&x)[N], const float (&s)[N],
                                           bool present, bool keep_raw, v8bf &hi,
                                           v8bf &lo)
{
    static_assert(N == 8, "one K-slice is 8 rows");
    uint32_t hw[4], lw[4];
#pragma unroll
    for (int h = 0; h < 4; ++h) {
        const float d0 = present ? (keep_raw ? x[2 * h] : x[2 * h] - s[2 * h]) : 0.0f;
        const float d1 = present ? (keep_raw ? x[2 * h + 1] : x[2 * h + 1] - s[2 * h + 1]) : 0.0f;
        const uint32_t u0 = __float_as_uint(d0), u1 = __float_as_uint(d1);
        hw[h] = __builtin_amdgcn_perm(u1, u0, 0x07060302u);      // upper halves of d0, d1
        const float l0 = d0 - __uint_as_float(u0 & 0xffff0000u);
        const float l1 = d1 - __uint_as_float(u1 & 0xffff0000u);
        const v2bf lp = {static_cast<__bf16>(l0), static_cast<__bf16>(l1)};
        lw[h] = __builtin_bit_cast(uint32_t, lp);
    }
    const v4u hv = {hw[0], hw[1], hw[2], hw[3]}, lv = {lw[0], lw[1], lw[2], lw[3]};
    hi = __builtin_bit_cast(v8bf, hv);
    lo = __builtin_bit_cast(v8bf, lv);
}

// One K = 32 step of the lower-triangle tiles on the bf16 matrix cores:
// (hi + lo)(hi + lo)^T expanded into its four products.
template <int NT>
__device__ __forceinline__ void gram_step_bf16(v8bf ahi, v8bf alo, v8bf bhi, v8bf blo,
                                               v4f (&acc)[GramTiles<NT>::value])
{
#define QN_MFMA_BF16(A, B, C) C = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, B, C, 0, 0, 0)
    QN_MFMA_BF16(ahi, ahi, acc[0]);
    QN_MFMA_BF16(ahi, alo, acc[0]);
    QN_MFMA_BF16(alo, ahi, acc[0]);
    QN_MFMA_BF16(alo, alo, acc[0]);
    if constexpr (NT == 2) {
        QN_MFMA_BF16(bhi, ahi, acc[1]);
        QN_MFMA_BF16(bhi, alo, acc[1]);
        QN_MFMA_BF16(blo, ahi, acc[1]);
        QN_MFMA_BF16(blo, alo, acc[1]);
        QN_MFMA_BF16(bhi, bhi, acc[2]);
        QN_MFMA_BF16(bhi, blo, acc[2]);
        QN_MFMA_BF16(blo, bhi, acc[2]);
        QN_MFMA_BF16(blo, blo, acc[2]);
    }
#undef QN_MFMA_BF16
}

// ALIGNED: every column start is 16-byte aligned, one 128-bit load per lane moves
// a column's whole tile (1 KiB) per wave instruction.  Otherwise the same tile is
// brought in with element-sized direct-to-LDS loads (64 consecutive rows per
// wave instruction): still coalesced, any alignment, more instructions.
template <int DT, int NT, bool ALIGNED>
__global__ __launch_bounds__(kGramThreads) void gram_stage1_stream(
    const void *__restrict__ grads, int64_t n, int m, int64_t ld,
    double *__restrict__ partials)
{
    constexpr int TILES = GramTiles<NT>::value;
    constexpr int ROWS = StreamRows<DT, ALIGNED>::value; // rows per tile
    constexpr int ESZ = (DT == QN_F32) ? 4 : 2;          // element size in memory
    constexpr bool WIDE = DT == QN_BF16 && !ALIGNED;     // bf16 kept one per dword in LDS
    constexpr int LESZ = WIDE ? 4 : ESZ;                 // element size in LDS
    constexpr int FMT = DT == QN_F32 ? 0 : (WIDE ? 2 : 1);
    constexpr int RPV = 16 / LESZ;                       // rows per 16-byte LDS vector
    constexpr int COLS_PER_WAVE = QN_MAX_M / kGramWaves; // columns a wave loads
    constexpr int VEC_PER_GROUP = ROWS / kGramWaves / 4 / RPV;   // 2 either way
    extern __shared__ __attribute__((aligned(16))) char lds[];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int col = lane & 15;
    const int group = lane >> 4;
    const bool has_a = col < m;
    const bool has_b = (NT == 2) && (col + 16 < m);
    const bool is_pivot = col == 0;
    const char *base = static_cast<const char *>(grads);

    const int64_t num_tiles = (n + ROWS - 1) / ROWS;
    const int64_t mine = (num_tiles - blockIdx.x + gridDim.x - 1) / gridDim.x;

    // Brings tile number k of this block into LDS stage k % 2.
    auto fetch = [&](int64_t k) {
        const int64_t tile = blockIdx.x + k * gridDim.x;
        const int64_t row0 = tile * ROWS;
        char *stage = lds + (k & 1) * kStageBytes;
        if (row0 + ROWS <= n) {
#pragma unroll
            for (int jc = 0; jc < COLS_PER_WAVE; ++jc) {
                const int c = wave * COLS_PER_WAVE + jc;
                if (c < m) {
                    const char *g = base + (static_cast<int64_t>(c) * ld + row0) * ESZ;
                    if constexpr (ALIGNED) {
                        __builtin_amdgcn_global_load_lds(QN_GPTR(g + lane * 16),
                                                         QN_LPTR(stage + c * kColPitch),
                                                         16, 0, /*nt*/ 2);
                    } else {
#pragma unroll
                        for (int part = 0; part < ROWS / 64; ++part) {
                            const char *gp = g + (part * 64 + lane) * ESZ;
                            char *lp = stage + c * kColPitch + part * 64 * LESZ;
                            if constexpr (DT == QN_F32)
                                __builtin_amdgcn_global_load_lds(QN_GPTR(gp), QN_LPTR(lp), 4, 0, 2);
                            else
                                __builtin_amdgcn_global_load_lds(QN_GPTR(gp), QN_LPTR(lp), 2, 0, 2);
                        }
                    }
                }
            }
        } else {
            // the ragged last tile: guarded element loads, zero fill
            for (int jc = 0; jc < COLS_PER_WAVE; ++jc) {
                const int c = wave * COLS_PER_WAVE + jc;
                if (c >= m)
                    continue;
                for (int e = 0; e < RPV; ++e) {
                    const int64_t r = row0 + lane * RPV + e;
                    char *dst = stage + c * kColPitch + (lane * RPV + e) * LESZ;
                    if constexpr (DT == QN_F32) {
                        const float *src = reinterpret_cast<const float *>(base);
                        *reinterpret_cast<float *>(dst) = r < n ? src[c * ld + r] : 0.0f;
                    } else {
                        const uint16_t *src = reinterpret_cast<const uint16_t *>(base);
                        const uint16_t v = r < n ? src[c * ld + r] : static_cast<uint16_t>(0);
                        if constexpr (WIDE)
                            *reinterpret_cast<uint32_t *>(dst) = v;
                        else
                            *reinterpret_cast<uint16_t *>(dst) = v;
                    }
                }
            }
        }
    };

    double tot[TILES][4];
#pragma unroll
    for (int t = 0; t < TILES; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r)
            tot[t][r] = 0.0;

    if (mine > 0)
        fetch(0);
    for (int64_t k = 0; k < mine; ++k) {
        // tile k has landed once this wave's loads are done and every wave has
        // said so; the same barrier says everyone finished reading tile k-1,
        // whose stage the next fetch overwrites
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (k + 1 < mine)
            fetch(k + 1);

        const char *stage = lds + (k & 1) * kStageBytes;
        // this wave's rows: its share of the tile; this lane group's: a quarter of that
        const int byte0 = (wave * (ROWS / kGramWaves) + group * (ROWS / kGramWaves / 4)) * LESZ;
        v4f acc[TILES];
#pragma unroll
        for (int t = 0; t < TILES; ++t)
            acc[t] = (v4f){0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int i = 0; i < VEC_PER_GROUP; ++i) {
            float a[RPV], b[RPV], s[RPV];
            lds_rows<FMT>(stage + col * kColPitch + byte0 + 16 * i, a);
            lds_rows<FMT>(stage + byte0 + 16 * i, s);            // column 0: the pivot
            if constexpr (NT == 2)
                lds_rows<FMT>(stage + (col + 16) * kColPitch + byte0 + 16 * i, b);
            if constexpr (FMT != 1) {
#pragma unroll
                for (int e = 0; e < RPV; ++e) {
                    const float da = has_a ? (is_pivot ? a[e] : a[e] - s[e]) : 0.0f;
                    float db = 0.0f;
                    if constexpr (NT == 2)
                        db = has_b ? b[e] - s[e] : 0.0f;
                    gram_step<NT>(da, db, acc);
                }
            } else {
                // bf16 storage: the 8 rows a lane just read are one K-slice of
                // v_mfma_f32_16x16x32_bf16.  The shifted value d = x - s (exact in
                // fp32) is split as hi + lo, hi = its upper 16 bits (a bf16), lo =
                // bf16(d - hi): exact whenever d has at most 16 significant bits
                // (always, unless x and s differ by more than 2^8 in magnitude),
                // else good to 2^-16.  All four hi/lo products are accumulated.
                v8bf ahi, alo, bhi = {}, blo = {};
                split_bf16<RPV>(a, s, has_a, is_pivot, ahi, alo);
                if constexpr (NT == 2)
                    split_bf16<RPV>(b, s, has_b, false, bhi, blo);
                gram_step_bf16<NT>(ahi, alo, bhi, blo, acc);
            }
        }
#pragma unroll
        for (int t = 0; t < TILES; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                tot[t][r] += static_cast<double>(acc[t][r]);
    }
    __syncthreads();   // all reads of the stages are done: reuse them for the reduction
    write_block_partial<TILES>(tot, reinterpret_cast<double *>(lds), partials);
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
    // eight loads in flight, added in the order of p (the order fixes the bits)
    double s = 0.0;
    int p = slice;
    for (; p + 7 * kReduceSlices < num_partials; p += 8 * kReduceSlices) {
        double v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            v[u] = partials[static_cast<int64_t>(p + u * kReduceSlices) * entries + e];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            s += v[u];
    }
    for (; p < num_partials; p += kReduceSlices)
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
static int launch_stage1(bool aligned, int cu_count, const void *grads, int64_t n,
                         int m, int64_t ld, double *partials, hipStream_t stream)
{
    const int rows = aligned ? StreamRows<DT, true>::value : StreamRows<DT, false>::value;
    const int64_t num_tiles = (n + rows - 1) / rows;
    const int64_t cap = static_cast<int64_t>(cu_count) * 2;   // two 65 KB blocks per CU
    const int grid = static_cast<int>(num_tiles < cap ? num_tiles : cap);
    if (aligned)
        hipLaunchKernelGGL((gram_stage1_stream<DT, NT, true>), dim3(grid), dim3(kGramThreads),
                           kStreamLdsBytes, stream, grads, n, m, ld, partials);
    else
        hipLaunchKernelGGL((gram_stage1_stream<DT, NT, false>), dim3(grid), dim3(kGramThreads),
                           kStreamLdsBytes, stream, grads, n, m, ld, partials);
    return grid;
}

// The streaming kernels use more than the default 64 KiB of dynamic LDS; the
// opt-in is per device and is made once when the device's workspace is set up.
int setup_gram_kernels()
{
    bool ok = true;
#define QN_OPT_IN(K)                                                                   \
    ok = ok && hipFuncSetAttribute(reinterpret_cast<const void *>(K),                  \
                                   hipFuncAttributeMaxDynamicSharedMemorySize,        \
                                   kStreamLdsBytes) == hipSuccess
    QN_OPT_IN((gram_stage1_stream<QN_F32, 1, true>));
    QN_OPT_IN((gram_stage1_stream<QN_F32, 2, true>));
    QN_OPT_IN((gram_stage1_stream<QN_BF16, 1, true>));
    QN_OPT_IN((gram_stage1_stream<QN_BF16, 2, true>));
    QN_OPT_IN((gram_stage1_stream<QN_F32, 1, false>));
    QN_OPT_IN((gram_stage1_stream<QN_F32, 2, false>));
    QN_OPT_IN((gram_stage1_stream<QN_BF16, 1, false>));
    QN_OPT_IN((gram_stage1_stream<QN_BF16, 2, false>));
#undef QN_OPT_IN
    return ok ? QN_OK : QN_ELAUNCH;
}

int launch_gram(const void *grads, int dtype, int64_t n, int m, int64_t ld,
                Workspace *ws, double *C, double *w, hipStream_t stream)
{
    const size_t esz = dtype == QN_F32 ? 4 : 2;
    const bool aligned = (reinterpret_cast<uintptr_t>(grads) % 16 == 0) &&
                         ((static_cast<uint64_t>(ld) * esz) % 16 == 0);
    const int nt = m <= 16 ? 1 : 2;
    const int entries = (nt == 1 ? 1 : 3) * kTileEntries;

    // the grid is a function of (n, dtype, alignment) and the device's CU count
    // only, so the summation tree is reproducible
    int grid;
    {
        TraceScope ts(QN_K_GRAM, stream);
        if (dtype == QN_F32)
            grid = nt == 1 ? launch_stage1<QN_F32, 1>(aligned, ws->cu_count, grads, n, m, ld, ws->partials, stream)
                           : launch_stage1<QN_F32, 2>(aligned, ws->cu_count, grads, n, m, ld, ws->partials, stream);
        else
            grid = nt == 1 ? launch_stage1<QN_BF16, 1>(aligned, ws->cu_count, grads, n, m, ld, ws->partials, stream)
                           : launch_stage1<QN_BF16, 2>(aligned, ws->cu_count, grads, n, m, ld, ws->partials, stream);
    }
    if (grid < 0 || grid > kGramMaxBlocks)
        return QN_ELAUNCH;
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
