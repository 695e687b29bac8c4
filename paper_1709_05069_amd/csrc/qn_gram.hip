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
// Stage 1: one streaming pass over grads on v_mfma_f32_16x16x32_bf16.  For a
//   Gram product the A and B operands are the same register: lane l of a
//   wavefront supplies column l%16 of a column set for the 8 rows of slot l/16,
//   and any assignment of rows to the four slots is valid as long as both
//   operands agree.  The m columns form NT = 1..4 sets of 16 (m <= 16, 32, 48, 64)
//   and only the lower triangle of the NT x NT tiling is computed (1, 3, 6 or 10
//   tiles).  For m <= 8 (<= 4) two (four) row blocks of the same columns share
//   the 16 column lanes of the single set.  The shifted fp32 entry is split into
//   bf16 terms whose products the matrix cores form exactly and accumulate in
//   fp32:
//     fp32 storage: d = hi + mid + lo exactly (8 + 8 + 8 significant bits, by
//       truncation); six products (all but mid lo, lo mid, lo lo, which are below
//       2^-23 of the leading one).  This is both more accurate than fp32
//       multiply-adds on v_mfma_f32_16x16x4_f32 and 2.7x cheaper in matrix-core
//       cycles, which matters for m > 32 (ten tiles);
//     bf16 storage: d = hi + lo (exact unless a value and the pivot differ by
//       more than 2^8 in magnitude), four products.
//   Accumulators run in fp32 over one tile and are then added to per-lane fp64
//   totals; waves are combined through LDS in a fixed order and each block writes
//   one partial.  No atomics.
//   HBM -> LDS goes through coalesced direct-to-LDS loads carrying the
//   non-temporal hint (128-bit per lane when the columns are 16-byte aligned:
//   every wave instruction moves 1 KiB of one column; element-sized per lane
//   otherwise, 2-byte loads landing one value per dword), two LDS stages per
//   block; the wavefronts then read their operands from LDS in the lane = column
//   layout.  Measured on MI355X this load pattern sustains about 7.0 TB/s,
//   against 6.4 TB/s when each lane fetches its own column straight from HBM.
// Stage 2 (gram_reduce): fixed-order fp64 sum of the block partials, two levels.
// Stage 3 (gram_project, or the prologue of the eigen kernel): the m x m algebra
//   above (qn_project.h).
#include "qn_internal.h"
#include "qn_project.h"

namespace qn {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));

#define QN_GPTR(p) ((const __attribute__((address_space(1))) void *)(p))
#define QN_LPTR(p) ((__attribute__((address_space(3))) void *)(p))

// NT column sets of 16: lower-triangle tiles, tile (ti, tj), ti >= tj, at index
// ti (ti + 1) / 2 + tj.
template <int NT> struct GramTiles { static constexpr int value = NT * (NT + 1) / 2; };

// ---------------------------------------------------------------------------
// A column slot is 1 KiB of one column (ROWS rows) at slot * kColPitch in LDS
// (1 KiB + 16 B, which spreads the 16 columns a quarter-wave reads over all
// banks).  16 * NT slots per stage, two stages.
// A pass that also carries a vector z (below) keeps z's rows of the tile in
// ZSLOTS further slots of each stage (fp32: 1 KiB per 256 rows).
template <int NT, int ZSLOTS> constexpr int stage_bytes() { return gram_stage_bytes(NT, ZSLOTS); }
template <int NT, int ZSLOTS> constexpr int stream_lds_bytes() { return gram_lds_bytes(NT, ZSLOTS); }

// Rows per column slot.  bf16 inputs that are not 16-byte aligned arrive through
// 2-byte direct-to-LDS loads, which the hardware stores zero-extended, one per
// dword: their LDS format is 4 bytes per row.
template <int DT, bool ALIGNED> struct StreamRows {
    static constexpr int value = gram_slot_rows(DT, ALIGNED);
};

// 16 bytes of one column from LDS as fp32 row values.  FMT 0: fp32 (4 rows);
// 1: packed bf16 (8 rows); 2: bf16 zero-extended to one dword per row (4 rows);
// 3: packed fp16 (8 rows); 4: fp16 zero-extended to one dword per row (4 rows).
constexpr bool fmt_packed(int fmt) { return fmt == 1 || fmt == 3; }

__device__ __forceinline__ float half_bits_to_float(uint32_t h)
{
    return static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(h)));
}

template <int FMT>
__device__ __forceinline__ void lds_rows(const char *p, float (&x)[fmt_packed(FMT) ? 8 : 4])
{
    const v4u v = *reinterpret_cast<const v4u *>(p);
    const uint32_t u[4] = {v.x, v.y, v.z, v.w};
    if constexpr (FMT == 0) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            x[e] = __uint_as_float(u[e]);
    } else if constexpr (FMT == 2) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            x[e] = __uint_as_float(u[e] << 16);
    } else if constexpr (FMT == 4) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            x[e] = half_bits_to_float(u[e]);
    } else if constexpr (FMT == 1) {
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

// 8 consecutive rows of one column from LDS as fp32: one 16-byte vector of packed
// bf16, or two vectors in the 4-bytes-per-row formats.
template <int FMT>
__device__ __forceinline__ void lds_rows8(const char *p, float (&x)[8])
{
    if constexpr (fmt_packed(FMT)) {
        lds_rows<FMT>(p, x);
    } else {
        float a[4], b[4];
        lds_rows<FMT>(p, a);
        lds_rows<FMT>(p + 16, b);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            x[e] = a[e];
            x[4 + e] = b[e];
        }
    }
}

// Upper halves of two fp32 words as a bf16 pair (truncation).
__device__ __forceinline__ uint32_t upper_halves(uint32_t u0, uint32_t u1)
{
    return __builtin_amdgcn_perm(u1, u0, 0x07060302u);
}

// The shifted entry d = x - s for 8 rows (s: the pivot's rows, or zeros in the
// pivot lane, which keeps its own value), split into bf16 hi + lo: hi = the
// upper 16 bits of d, lo = bf16(d - hi).  Exact whenever d has at most 16
// significant bits (always for bf16 storage, unless x and s differ by more than
// 2^8 in magnitude), else good to 2^-16.
__device__ __forceinline__ void split_bf16(const float (&x)[8], const float (&s)[8],
                                           v8bf &hi, v8bf &lo)
{
    uint32_t hw[4], lw[4];
#pragma unroll
    for (int h = 0; h < 4; ++h) {
        const float d0 = x[2 * h] - s[2 * h], d1 = x[2 * h + 1] - s[2 * h + 1];
        const uint32_t u0 = __float_as_uint(d0), u1 = __float_as_uint(d1);
        hw[h] = upper_halves(u0, u1);
        const float l0 = d0 - __uint_as_float(u0 & 0xffff0000u);
        const float l1 = d1 - __uint_as_float(u1 & 0xffff0000u);
        const v2bf lp = {static_cast<__bf16>(l0), static_cast<__bf16>(l1)};
        lw[h] = __builtin_bit_cast(uint32_t, lp);
    }
    const v4u hv = {hw[0], hw[1], hw[2], hw[3]}, lv = {lw[0], lw[1], lw[2], lw[3]};
    hi = __builtin_bit_cast(v8bf, hv);
    lo = __builtin_bit_cast(v8bf, lv);
}

// d for 8 rows of fp32 storage, split exactly into three bf16 terms by
// truncation: hi = the leading 8 significant bits of d, mid = the leading 8 of
// d - hi, lo = the rest (at most 8 bits, so its upper half is all of it).
__device__ __forceinline__ void split3_bf16(const float (&x)[8], const float (&s)[8],
                                            v8bf &hi, v8bf &mid, v8bf &lo)
{
    uint32_t hw[4], mw[4], lw[4];
#pragma unroll
    for (int h = 0; h < 4; ++h) {
        const float d0 = x[2 * h] - s[2 * h], d1 = x[2 * h + 1] - s[2 * h + 1];
        const uint32_t u0 = __float_as_uint(d0), u1 = __float_as_uint(d1);
        hw[h] = upper_halves(u0, u1);
        const float r0 = d0 - __uint_as_float(u0 & 0xffff0000u);
        const float r1 = d1 - __uint_as_float(u1 & 0xffff0000u);
        const uint32_t v0 = __float_as_uint(r0), v1 = __float_as_uint(r1);
        mw[h] = upper_halves(v0, v1);
        const float l0 = r0 - __uint_as_float(v0 & 0xffff0000u);
        const float l1 = r1 - __uint_as_float(v1 & 0xffff0000u);
        lw[h] = upper_halves(__float_as_uint(l0), __float_as_uint(l1));
    }
    const v4u hv = {hw[0], hw[1], hw[2], hw[3]}, mv = {mw[0], mw[1], mw[2], mw[3]},
              lv = {lw[0], lw[1], lw[2], lw[3]};
    hi = __builtin_bit_cast(v8bf, hv);
    mid = __builtin_bit_cast(v8bf, mv);
    lo = __builtin_bit_cast(v8bf, lv);
}

// ALIGNED: every column start is 16-byte aligned, one 128-bit load per lane moves
// a column's whole tile (1 KiB) per wave instruction.  Otherwise the same tile is
// brought in with element-sized direct-to-LDS loads (64 consecutive rows per
// wave instruction): still coalesced, any alignment, more instructions.
// HAS_Z: the pivot lane supplies z (n fp32 values) instead of the raw pivot
// column, so the pass yields Q[k][0] = d_k^T z: the inner products G^T z are
// built from (eq. (4)'s alpha_k for an arbitrary z) at no extra pass over grads.
// PACK (NT = 1 only): for m <= 8 (<= 4) the 16 column lanes hold PACK = 2 (4)
// row blocks of the same 8 (4) columns side by side, so a tile covers PACK times
// the rows; the output tile's PACK diagonal blocks are partial Gram matrices of
// the same columns (summed in gram_project), its off-diagonal blocks are unused.
template <int DT, int NT, bool ALIGNED, bool HAS_Z, int PACK>
__global__ __launch_bounds__(kGramThreads) void gram_stage1_stream(
    const void *__restrict__ grads, int64_t n, int m, int64_t ld,
    double *__restrict__ partials, const float *__restrict__ z, int z_aligned)
{
    static_assert(PACK == 1 || NT == 1, "row blocks are packed only into a single column set");
    constexpr int TILES = GramTiles<NT>::value;
    constexpr int ROWS = StreamRows<DT, ALIGNED>::value; // rows per column slot
    constexpr int TROWS = ROWS * PACK;                   // rows per tile
    constexpr int MP = 16 / PACK;                        // column lanes per row block
    constexpr int ESZ = (DT == QN_F32) ? 4 : 2;          // element size in memory
    constexpr bool WIDE = DT != QN_F32 && !ALIGNED;      // 16-bit values kept one per dword in LDS
    constexpr int LESZ = WIDE ? 4 : ESZ;                 // element size in LDS
    constexpr int FMT = DT == QN_F32 ? 0 : (DT == QN_BF16 ? (WIDE ? 2 : 1) : (WIDE ? 4 : 3));
    constexpr int RPV = 16 / LESZ;                       // rows per 16-byte LDS vector
    constexpr int SLOTS_PER_WAVE = 16 * NT / kGramWaves; // column slots a wave loads
    constexpr int SLICES = ROWS / kGramWaves / 4 / 8;    // 8-row slices per lane group and tile
    constexpr int ZSLOTS = HAS_Z ? TROWS / 256 : 0;      // 1 KiB slots holding z's rows
    constexpr int STAGE = stage_bytes<NT, ZSLOTS>();
    constexpr int ZBASE = 16 * NT * kColPitch;           // z's rows inside a stage (contiguous)
    extern __shared__ __attribute__((aligned(16))) char lds[];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int col = lane & 15;
    const int group = lane >> 4;
    const int sub = col / MP;                            // this lane's row block (0 when PACK = 1)
    const bool is_pivot = col % MP == 0;
    // LDS slot of this lane's column in set t.  A lane whose column does not exist
    // (>= m) reads the pivot's slot instead: its shifted entry s - s is an exact
    // zero, so no per-element select is needed.
    const int pivot_slot = sub * MP;
    int my_slot[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
        my_slot[t] = (col % MP + 16 * t < m) ? col + 16 * t : pivot_slot;
    const char *base = static_cast<const char *>(grads);

    const int64_t num_tiles = (n + TROWS - 1) / TROWS;
    const int64_t mine = block_tiles(num_tiles, blockIdx.x, gridDim.x);

    // Brings tile number k of this block into LDS stage k % 2.
    auto fetch = [&](int64_t k) {
        const int64_t tile = blockIdx.x + k * gridDim.x;
        const int64_t row0 = tile * TROWS;
        char *stage = lds + (k & 1) * STAGE;
        // slot `slot` holds column slot % MP, rows [row0 + (slot / MP) * ROWS, + ROWS)
        if (row0 + TROWS <= n) {
#pragma unroll
            for (int jc = 0; jc < SLOTS_PER_WAVE; ++jc) {
                const int slot = wave * SLOTS_PER_WAVE + jc;
                const int c = PACK == 1 ? slot : slot % MP;
                if (c < m) {
                    const char *g = base + (static_cast<int64_t>(c) * ld + row0 +
                                            (PACK == 1 ? 0 : (slot / MP) * ROWS)) * ESZ;
                    if constexpr (ALIGNED) {
                        __builtin_amdgcn_global_load_lds(QN_GPTR(g + lane * 16),
                                                         QN_LPTR(stage + slot * kColPitch),
                                                         16, 0, /*nt*/ 2);
                    } else {
#pragma unroll
                        for (int part = 0; part < ROWS / 64; ++part) {
                            const char *gp = g + (part * 64 + lane) * ESZ;
                            char *lp = stage + slot * kColPitch + part * 64 * LESZ;
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
            for (int jc = 0; jc < SLOTS_PER_WAVE; ++jc) {
                const int slot = wave * SLOTS_PER_WAVE + jc;
                const int c = PACK == 1 ? slot : slot % MP;
                if (c >= m)
                    continue;
                for (int e = 0; e < RPV; ++e) {
                    const int64_t r = row0 + (PACK == 1 ? 0 : (slot / MP) * ROWS) + lane * RPV + e;
                    char *dst = stage + slot * kColPitch + (lane * RPV + e) * LESZ;
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
        if constexpr (HAS_Z) {
            // the last wave also brings in z's rows of the tile (fp32, contiguous)
            if (wave == kGramWaves - 1) {
                char *zl = stage + ZBASE;
                if (row0 + TROWS <= n) {
                    if (z_aligned) {
#pragma unroll
                        for (int part = 0; part < TROWS / 256; ++part)
                            __builtin_amdgcn_global_load_lds(
                                QN_GPTR(z + row0 + part * 256 + lane * 4),
                                QN_LPTR(zl + part * 1024), 16, 0, 2);
                    } else {
#pragma unroll
                        for (int part = 0; part < TROWS / 64; ++part)
                            __builtin_amdgcn_global_load_lds(
                                QN_GPTR(z + row0 + part * 64 + lane),
                                QN_LPTR(zl + part * 256), 4, 0, 2);
                    }
                } else {
                    for (int part = 0; part < TROWS / 64; ++part) {
                        const int64_t r = row0 + part * 64 + lane;
                        reinterpret_cast<float *>(zl)[part * 64 + lane] = r < n ? z[r] : 0.0f;
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

        const char *stage = lds + (k & 1) * STAGE;
        // this wave's rows: its share of the tile; this lane group's: a quarter of that
        const int byte0 = (wave * (ROWS / kGramWaves) + group * (ROWS / kGramWaves / 4)) * LESZ;
        v4f acc[TILES];
#pragma unroll
        for (int t = 0; t < TILES; ++t)
            acc[t] = (v4f){0.0f, 0.0f, 0.0f, 0.0f};
        {
            // The 8 rows a lane holds per column are one K-slice of
            // v_mfma_f32_16x16x32_bf16.  The shifted fp32 value is split into bf16
            // terms and the cross products that matter are accumulated in fp32.
#pragma unroll
            for (int sl = 0; sl < SLICES; ++sl) {
                const char *at = stage + byte0 + sl * 8 * LESZ;
                float x[NT][8], s[8];
                lds_rows8<FMT>(at + pivot_slot * kColPitch, s);  // the pivot: column 0 of this row block
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    lds_rows8<FMT>(at + my_slot[t] * kColPitch, x[t]);
                [[maybe_unused]] v8bf zlo = {};                  // z's third term (bf16 storage)
                if constexpr (HAS_Z) {
                    // the same 8 rows of z; only the pivot lane uses them
                    float zr[8];
                    lds_rows8<0>(stage + ZBASE + (sub * ROWS + byte0 / LESZ + sl * 8) * 4, zr);
                    if (is_pivot) {
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            x[0][e] = zr[e];
                    }
                }
                // column 0 itself is not shifted: in set 0 the pivot lane keeps its
                // own value (or z) by subtracting zeros
                float s0[8];
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    s0[e] = is_pivot ? 0.0f : s[e];
                if constexpr (DT != QN_BF16) {
                    // d = hi + mid + lo exactly (8 + 8 + 8 bits); the six products
                    // down to 2^-16 of the leading one are kept, the dropped ones
                    // (mid lo, lo mid, lo lo) are below 2^-23 of it
                    v8bf hi[NT], mid[NT], lo[NT];
#pragma unroll
                    for (int t = 0; t < NT; ++t)
                        split3_bf16(x[t], t == 0 ? s0 : s, hi[t], mid[t], lo[t]);
#pragma unroll
                    for (int ti = 0; ti < NT; ++ti)
#pragma unroll
                        for (int tj = 0; tj <= ti; ++tj) {
                            v4f &a = acc[tile_index(ti, tj)];
                            a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hi[ti], lo[tj], a, 0, 0, 0);
                            a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(lo[ti], hi[tj], a, 0, 0, 0);
                            a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(mid[ti], mid[tj], a, 0, 0, 0);
                            a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hi[ti], mid[tj], a, 0, 0, 0);
                            a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(mid[ti], hi[tj], a, 0, 0, 0);
                            a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hi[ti], hi[tj], a, 0, 0, 0);
                        }
                } else {
                    // bf16 storage: d = hi + lo, all four products
                    v8bf hi[NT], lo[NT];
#pragma unroll
                    for (int t = 0; t < NT; ++t)
                        split_bf16(x[t], t == 0 ? s0 : s, hi[t], lo[t]);
                    if constexpr (HAS_Z) {
                        // z is an arbitrary fp32 vector: its lane gets the exact
                        // three-term split, the third term through one more product
                        // per tile of column set 0
                        v8bf zh, zm, zl3;
                        split3_bf16(x[0], s0, zh, zm, zl3);
                        if (is_pivot) {
                            hi[0] = zh;
                            lo[0] = zm;
                            zlo = zl3;
                        }
#pragma unroll
                        for (int ti = 0; ti < NT; ++ti)
                            acc[tile_index(ti, 0)] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                hi[ti], zlo, acc[tile_index(ti, 0)], 0, 0, 0);
                    }
#pragma unroll
                    for (int ti = 0; ti < NT; ++ti)
#pragma unroll
                        for (int tj = 0; tj <= ti; ++tj) {
                            v4f &a = acc[tile_index(ti, tj)];
                            a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(lo[ti], lo[tj], a, 0, 0, 0);
                            a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hi[ti], lo[tj], a, 0, 0, 0);
                            a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(lo[ti], hi[tj], a, 0, 0, 0);
                            a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hi[ti], hi[tj], a, 0, 0, 0);
                        }
                }
            }
        }
#pragma unroll
        for (int t = 0; t < TILES; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                tot[t][r] += static_cast<double>(acc[t][r]);
    }
    __syncthreads();   // all reads of the stages are done: reuse them for the reduction

    // Combine the wavefronts of the block in wave order, one tile at a time
    // (256 entries of 8 waves = 16 KiB of the stage memory).
    double *red = reinterpret_cast<double *>(lds);
    constexpr int ENTRIES = TILES * kTileEntries;
#pragma unroll 1
    for (int t = 0; t < TILES; ++t) {
        // tot[t] with a loop-variant t would live in scratch: select statically
        double mine4[4];
#pragma unroll
        for (int tt = 0; tt < TILES; ++tt)
            if (tt == t) {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    mine4[r] = tot[tt][r];
            }
#pragma unroll
        for (int r = 0; r < 4; ++r)
            red[(wave * 4 + r) * 64 + lane] = mine4[r];
        __syncthreads();
        if (threadIdx.x < kTileEntries) {
            double sum = 0.0;
#pragma unroll
            for (int wv = 0; wv < kGramWaves; ++wv)
                sum += red[wv * kTileEntries + threadIdx.x];
            partials[static_cast<int64_t>(blockIdx.x) * ENTRIES + t * kTileEntries + threadIdx.x] = sum;
        }
        __syncthreads();
    }
}

// Fixed-order fp64 sum over the block partials in two levels.  Block (b, r) owns
// 64 entries and the partials p = r*16 + slice (mod 16 * kReduceRows): each of its
// 16 thread slices sums its partials serially, the slices are added in order,
// and row r of mraw receives the result; gram_project adds the rows in order.
constexpr int kReduceSlices = 16;
__global__ __launch_bounds__(64 * kReduceSlices) void gram_reduce(
    const double *__restrict__ partials, int num_partials, int entries,
    double *__restrict__ mraw)
{
    __shared__ double part[kReduceSlices][64];
    constexpr int STRIDE = kReduceSlices * kReduceRows;
    const int e = blockIdx.x * 64 + (threadIdx.x & 63);
    const int slice = threadIdx.x >> 6;
    // up to eight loads in flight, added in the order of p (the order fixes the bits)
    double s = 0.0;
    int p = blockIdx.y * kReduceSlices + slice;
    for (; p + 7 * STRIDE < num_partials; p += 8 * STRIDE) {
        double v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            v[u] = partials[static_cast<int64_t>(p + u * STRIDE) * entries + e];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            s += v[u];
    }
    for (; p < num_partials; p += STRIDE)
        s += partials[static_cast<int64_t>(p) * entries + e];
    part[slice][threadIdx.x & 63] = s;
    __syncthreads();
    if (slice == 0) {
        double r = 0.0;
#pragma unroll
        for (int k = 0; k < kReduceSlices; ++k)
            r += part[k][threadIdx.x];
        mraw[static_cast<int64_t>(blockIdx.y) * entries + e] = r;
    }
}

// C = P N P and w = P (t + N 1 / m) in fp64; one block (the algebra is in
// qn_project.h).  z_mode: column 0 of the raw matrix holds d_k^T z instead of
// d_k^T s, and w = G^T z = P t.
constexpr int kProjectThreads = 1024;
__global__ __launch_bounds__(kProjectThreads) void gram_project(
    const double *__restrict__ mraw, int entries, int m, int z_mode, int pack,
    double *__restrict__ C, double *__restrict__ w)
{
    __shared__ double N[QN_MAX_M * (QN_MAX_M + 1)];
    __shared__ double red[kMaxEntries];
    __shared__ ProjectScratch sc;
    project_raw<kProjectThreads>(
        mraw, entries, m, z_mode, pack, N, QN_MAX_M + 1, red, sc,
        [&](int k, int l, double v) { C[l * m + k] = v; },
        [&](int k, double v) { w[k] = v; });
}

// ---------------------------------------------------------------------------
// The fp64 vector kernel for small problems (gram_is_small): the same pivot-shifted
// matrix Q = D^T D, with every difference, product and sum in fp64 (differences and
// products of fp32 or 16-bit inputs are exact there), written in the same raw
// layout so that the reduction and the m x m algebra downstream do not change.
// With few rows the fp32 tile sums of the matrix-core pass have nothing to
// average over, and a step whose g_bar lies inside span{u_k} (always for n < m)
// amplifies that error; here it is of order 1e-16 instead.
// One block per 64-row tile (grid-stride above 256 blocks); thread p of a block
// owns the pairs (k, l), k >= l, numbered p, p + 256, ...
constexpr int kSmallPairsPerThread = (QN_MAX_M * (QN_MAX_M + 1) / 2 + kSmallThreads - 1) / kSmallThreads;

template <int DT>
__device__ __forceinline__ double load_elem_f64(const void *base, int64_t elem)
{
    if constexpr (DT == QN_F32)
        return static_cast<double>(static_cast<const float *>(base)[elem]);
    else if constexpr (DT == QN_BF16)
        return static_cast<double>(__uint_as_float(
            static_cast<uint32_t>(static_cast<const uint16_t *>(base)[elem]) << 16));
    else
        return static_cast<double>(half_bits_to_float(static_cast<const uint16_t *>(base)[elem]));
}

template <int DT>
__global__ __launch_bounds__(kSmallThreads) void gram_small_f64(
    const void *__restrict__ grads, int64_t n, int m, int64_t ld,
    double *__restrict__ partials, const float *__restrict__ z, int entries)
{
    constexpr int TR = kSmallTileRows;
    __shared__ double D[QN_MAX_M][TR + 1];
    __shared__ unsigned char pk[QN_MAX_M * (QN_MAX_M + 1) / 2], pl[QN_MAX_M * (QN_MAX_M + 1) / 2];
    const int tid = threadIdx.x;
    const int pairs = m * (m + 1) / 2;
    for (int k = tid; k < m; k += kSmallThreads)      // row k of the triangle starts at k (k + 1) / 2
        for (int l = 0; l <= k; ++l) {
            pk[k * (k + 1) / 2 + l] = static_cast<unsigned char>(k);
            pl[k * (k + 1) / 2 + l] = static_cast<unsigned char>(l);
        }
    double acc[kSmallPairsPerThread];
#pragma unroll
    for (int i = 0; i < kSmallPairsPerThread; ++i)
        acc[i] = 0.0;

    const int64_t tiles = (n + TR - 1) / TR;
    for (int64_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
        const int64_t row0 = tile * TR;
        __syncthreads();          // the previous tile has been consumed (and pk, pl are written)
        for (int e = tid; e < m * TR; e += kSmallThreads) {
            const int k = e / TR, r = e % TR;
            const int64_t row = row0 + r;
            double v = 0.0;
            if (row < n) {
                const double s = load_elem_f64<DT>(grads, row);          // the pivot: worker 0
                if (k == 0)
                    v = z != nullptr ? static_cast<double>(z[row]) : s;
                else
                    v = load_elem_f64<DT>(grads, k * ld + row) - s;
            }
            D[k][r] = v;
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < kSmallPairsPerThread; ++i) {
            const int p = tid + i * kSmallThreads;
            if (p < pairs) {
                const int k = pk[p], l = pl[p];
                double s = acc[i];
                for (int r = 0; r < TR; ++r)
                    s = fma(D[k][r], D[l][r], s);
                acc[i] = s;
            }
        }
    }
    // One partial per block in the raw layout (the inverse of raw_index): entry
    // (tile, reg, lane) holds Q[16 ti + 4 (lane / 16) + reg][16 tj + lane % 16];
    // entries that no pair k >= l, k < m maps to are zero.
    __syncthreads();
    double *Q = &D[0][0];            // pairs <= 2080 doubles fit D's 4160
#pragma unroll
    for (int i = 0; i < kSmallPairsPerThread; ++i) {
        const int p = tid + i * kSmallThreads;
        if (p < pairs)
            Q[p] = acc[i];
    }
    __syncthreads();
    double *out = partials + static_cast<int64_t>(blockIdx.x) * entries;
    for (int e = tid; e < entries; e += kSmallThreads) {
        const int tile = e / kTileEntries, reg = (e / 64) & 3, lane = e & 63;
        int ti = 0;
        while (tile_index(ti + 1, 0) <= tile)
            ++ti;
        const int tj = tile - tile_index(ti, 0);
        const int k = 16 * ti + 4 * (lane >> 4) + reg, l = 16 * tj + (lane & 15);
        out[e] = (k < m && l <= k) ? Q[k * (k + 1) / 2 + l] : 0.0;
    }
}

static int launch_small(int dtype, const void *grads, int64_t n, int m, int64_t ld,
                        double *partials, int max_partials, const float *z, int entries,
                        hipStream_t stream)
{
    const int grid = gram_small_grid(n, max_partials);
    if (dtype == QN_F32)
        hipLaunchKernelGGL(gram_small_f64<QN_F32>, dim3(grid), dim3(kSmallThreads), 0, stream,
                           grads, n, m, ld, partials, z, entries);
    else if (dtype == QN_BF16)
        hipLaunchKernelGGL(gram_small_f64<QN_BF16>, dim3(grid), dim3(kSmallThreads), 0, stream,
                           grads, n, m, ld, partials, z, entries);
    else
        hipLaunchKernelGGL(gram_small_f64<QN_F16>, dim3(grid), dim3(kSmallThreads), 0, stream,
                           grads, n, m, ld, partials, z, entries);
    return grid;
}

template <int DT, int NT, bool AL, bool HAS_Z, int PACK>
constexpr int instance_lds_bytes()
{
    return stream_lds_bytes<NT, gram_z_slots_packed(DT, AL, PACK, HAS_Z)>();
}

template <int DT, int NT, bool AL, bool HAS_Z, int PACK>
static int launch_instance(int cu_count, int max_partials, const void *grads, int64_t n, int m,
                           int64_t ld, double *partials, const float *z, hipStream_t stream)
{
    constexpr int LDS = instance_lds_bytes<DT, NT, AL, HAS_Z, PACK>();
    const int grid = gram_stream_grid(n, m, DT, AL, HAS_Z, cu_count, max_partials);
    const int z_aligned = reinterpret_cast<uintptr_t>(z) % 16 == 0;
    hipLaunchKernelGGL((gram_stage1_stream<DT, NT, AL, HAS_Z, PACK>), dim3(grid),
                       dim3(kGramThreads), LDS, stream, grads, n, m, ld, partials, z, z_aligned);
    return grid;
}

template <int DT, bool AL, bool HAS_Z>
static int launch_stage1(int cu_count, int max_partials, const void *grads, int64_t n, int m,
                         int64_t ld, double *partials, const float *z, hipStream_t stream)
{
#define QN_GO(NTV, PK) \
    return launch_instance<DT, NTV, AL, HAS_Z, PK>(cu_count, max_partials, grads, n, m, ld, partials, z, stream)
    static_assert(gram_pack(4) == 4 && gram_pack(8) == 2 && gram_pack(9) == 1, "pack thresholds");
    if (m <= 4) QN_GO(1, 4);
    if (m <= 8) QN_GO(1, 2);
    if (m <= 16) QN_GO(1, 1);
    if (m <= 32) QN_GO(2, 1);
    if (m <= 48) QN_GO(3, 1);
    QN_GO(4, 1);
#undef QN_GO
}

// The streaming kernels use up to 134 KiB of dynamic LDS; the opt-in above the
// default 64 KiB is per device and is made once when the device is set up.
template <int DT, int NT, bool AL, bool HAS_Z, int PACK>
static bool opt_in_one()
{
    return hipFuncSetAttribute(
               reinterpret_cast<const void *>(gram_stage1_stream<DT, NT, AL, HAS_Z, PACK>),
               hipFuncAttributeMaxDynamicSharedMemorySize,
               instance_lds_bytes<DT, NT, AL, HAS_Z, PACK>()) == hipSuccess;
}

template <int DT, int NT, int PACK>
static bool opt_in_nt()
{
    return opt_in_one<DT, NT, true, false, PACK>() && opt_in_one<DT, NT, false, false, PACK>() &&
           opt_in_one<DT, NT, true, true, PACK>() && opt_in_one<DT, NT, false, true, PACK>();
}

template <int DT>
static bool opt_in_dt()
{
    return opt_in_nt<DT, 1, 4>() && opt_in_nt<DT, 1, 2>() && opt_in_nt<DT, 1, 1>() &&
           opt_in_nt<DT, 2, 1>() && opt_in_nt<DT, 3, 1>() && opt_in_nt<DT, 4, 1>();
}

int setup_gram_kernels()
{
    return opt_in_dt<QN_F32>() && opt_in_dt<QN_BF16>() && opt_in_dt<QN_F16>() ? QN_OK : QN_ELAUNCH;
}

int launch_gram_raw(const void *grads, int dtype, int64_t n, int m, int64_t ld,
                    Workspace *ws, const float *z, RawGram *raw, hipStream_t stream, int path)
{
    const size_t esz = dtype == QN_F32 ? 4 : 2;
    const bool aligned = (reinterpret_cast<uintptr_t>(grads) % 16 == 0) &&
                         ((static_cast<uint64_t>(ld) * esz) % 16 == 0);
    const int entries = gram_entries(m);
    const bool small = path == kGramAuto ? gram_is_small(n) : path == kGramSmall;

    // the grid is a function of (n, m, dtype, alignment) and the device's CU
    // count only, so the summation tree is reproducible
    int grid;
    {
        TraceScope ts(QN_K_GRAM, stream);
        if (small) {
            grid = launch_small(dtype, grads, n, m, ld, ws->partials, ws->max_partials, z,
                                entries, stream);
        } else {
#define QN_GO(DTV, ALV, ZV) \
    grid = launch_stage1<DTV, ALV, ZV>(ws->cu_count, ws->max_partials, grads, n, m, ld, ws->partials, z, stream)
            if (dtype == QN_F32) {
                if (aligned) { if (z) QN_GO(QN_F32, true, true); else QN_GO(QN_F32, true, false); }
                else { if (z) QN_GO(QN_F32, false, true); else QN_GO(QN_F32, false, false); }
            } else if (dtype == QN_BF16) {
                if (aligned) { if (z) QN_GO(QN_BF16, true, true); else QN_GO(QN_BF16, true, false); }
                else { if (z) QN_GO(QN_BF16, false, true); else QN_GO(QN_BF16, false, false); }
            } else {
                if (aligned) { if (z) QN_GO(QN_F16, true, true); else QN_GO(QN_F16, true, false); }
                else { if (z) QN_GO(QN_F16, false, true); else QN_GO(QN_F16, false, false); }
            }
#undef QN_GO
        }
    }
    if (check_launch() != QN_OK) return QN_ELAUNCH;
    {
        TraceScope ts(QN_K_REDUCE, stream);
        hipLaunchKernelGGL(gram_reduce, dim3(entries / 64, kReduceRows),
                           dim3(64 * kReduceSlices), 0, stream, ws->partials, grid, entries,
                           ws->mraw);
    }
    raw->mraw = ws->mraw;
    raw->entries = entries;
    raw->z_mode = z != nullptr ? 1 : 0;
    raw->pack = small ? 1 : gram_pack(m);
    return check_launch();
}

int launch_gram(const void *grads, int dtype, int64_t n, int m, int64_t ld,
                Workspace *ws, const float *z, double *C, double *w, hipStream_t stream,
                int path)
{
    RawGram raw;
    const int rc = launch_gram_raw(grads, dtype, n, m, ld, ws, z, &raw, stream, path);
    if (rc != QN_OK)
        return rc;
    TraceScope ts(QN_K_PROJECT, stream);
    hipLaunchKernelGGL(gram_project, dim3(1), dim3(kProjectThreads), 0, stream, raw.mraw,
                       raw.entries, m, raw.z_mode, raw.pack, C, w);
    return check_launch();
}

}  // namespace qn
