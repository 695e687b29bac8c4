// Host-side launch arithmetic of libqn: tile counts, grid sizes, slab lengths and
// workspace sizes as functions of (n, m, dtype, alignment, compute-unit count).
// Plain C++ with no HIP dependency, so that a host compiler (and its sanitizers)
// can check the same code the launchers run: every kernel takes its grid, its
// tile count and its step count from here and from nowhere else.
#pragma once

#include <stddef.h>
#include <stdint.h>

#include "qn.h"

// functions the kernels call too
#ifdef __HIPCC__
#define QN_HD __host__ __device__
#else
#define QN_HD
#endif

namespace qn {

// ---- Gram pass ----------------------------------------------------------------
// Fixed grid, one partial per block in the raw matrix-core accumulator layout:
// kTileEntries values per 16x16 tile, 1, 3, 6 or 10 tiles (the lower triangle of
// a 1x1 .. 4x4 tiling of column sets: m <= 16, 32, 48, 64).
#ifndef QN_GRAM_THREADS
#define QN_GRAM_THREADS 512                     // 8 wavefronts
#endif
constexpr int kGramThreads = QN_GRAM_THREADS;
constexpr int kGramWaves = kGramThreads / 64;
constexpr int kGramMaxBlocks = 1024;
constexpr int kTileEntries = 256;               // 16 x 16
constexpr int kMaxTiles = 10;                   // lower triangle of a 4x4 tiling (m <= 64)
constexpr int kMaxEntries = kTileEntries * kMaxTiles;
constexpr int kReduceRows = 8;                  // rows of the two-level partial reduction
constexpr int kColPitch = 1040;                 // LDS bytes per column slot (1 KiB + 16 B skew)
constexpr int kLdsPerCu = 163840;               // 160 KiB
constexpr int kWavesPerCu = 32;

// Problems of at most this many rows take the fp64 vector kernel instead of the
// matrix-core pass (exact products and sums; the cost is negligible there).
constexpr int64_t kGramSmallRows = 16384;
constexpr int kSmallTileRows = 64;              // rows per tile of that kernel
constexpr int kSmallThreads = 256;
constexpr int kSmallMaxBlocks = 256;

constexpr int gram_sets(int m) { return (m + 15) / 16; }                 // NT
constexpr int gram_tiles(int nt) { return nt * (nt + 1) / 2; }
constexpr int gram_entries(int m) { return gram_tiles(gram_sets(m)) * kTileEntries; }
// row blocks packed side by side into the 16 column lanes of a single column set
constexpr int gram_pack(int m) { return m <= 4 ? 4 : (m <= 8 ? 2 : 1); }
// rows per 1 KiB column slot: 16-bit values that arrive through element loads are
// kept one per dword in LDS
constexpr int gram_slot_rows(int dtype, bool aligned)
{
    return (dtype == QN_F32 || !aligned) ? 256 : 512;
}
constexpr int gram_tile_rows(int dtype, bool aligned, int m)
{
    return gram_slot_rows(dtype, aligned) * gram_pack(m);
}
// slots of a stage that hold z's rows of a tile (fp32, 256 rows per slot)
constexpr int gram_z_slots_packed(int dtype, bool aligned, int pack, bool has_z)
{
    return has_z ? gram_slot_rows(dtype, aligned) * pack / 256 : 0;
}
constexpr int gram_z_slots(int dtype, bool aligned, int m, bool has_z)
{
    return gram_z_slots_packed(dtype, aligned, gram_pack(m), has_z);
}
constexpr int gram_stage_bytes(int nt, int zslots) { return (16 * nt + zslots) * kColPitch; }
constexpr int gram_lds_bytes(int nt, int zslots) { return 2 * gram_stage_bytes(nt, zslots); }
// blocks of one kernel instance that fit a compute unit: LDS and wave slots
constexpr int gram_blocks_per_cu(int lds_bytes)
{
    return kLdsPerCu / lds_bytes < kWavesPerCu / kGramWaves ? kLdsPerCu / lds_bytes
                                                            : kWavesPerCu / kGramWaves;
}
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

inline bool gram_is_small(int64_t n) { return n <= kGramSmallRows; }

// Tiles are dealt round-robin: block b of `grid` takes tiles b, b + grid, ...;
// this is how many it gets.
QN_HD inline int64_t block_tiles(int64_t tiles, int64_t block, int64_t grid)
{
    return (tiles - block + grid - 1) / grid;
}

// Blocks of the streaming pass: one per tile up to what fits the device at once,
// never more than the partials buffer holds.
inline int gram_stream_grid(int64_t n, int m, int dtype, bool aligned, bool has_z,
                            int cu_count, int max_partials)
{
    const int nt = gram_sets(m);
    const int lds = gram_lds_bytes(nt, gram_z_slots(dtype, aligned, m, has_z));
    const int64_t tiles = ceil_div(n, gram_tile_rows(dtype, aligned, m));
    int64_t cap = static_cast<int64_t>(cu_count) * gram_blocks_per_cu(lds);
    if (cap > kGramMaxBlocks)
        cap = kGramMaxBlocks;
    if (cap > max_partials)
        cap = max_partials;
    return static_cast<int>(tiles < cap ? tiles : cap);
}

inline int gram_small_grid(int64_t n, int max_partials)
{
    int64_t g = ceil_div(n, kSmallTileRows);
    if (g > kSmallMaxBlocks)
        g = kSmallMaxBlocks;
    if (g > max_partials)
        g = max_partials;
    return static_cast<int>(g);
}

// Most blocks any Gram launch of this problem can use (whatever the alignment of
// the pointers and whether a vector z rides along): what the partials buffer of a
// workspace must hold.
inline int gram_max_partials(int64_t n, int m, int dtype, int cu_count)
{
    if (gram_is_small(n))
        return gram_small_grid(n, kSmallMaxBlocks);
    int best = 0;
    for (int al = 0; al < 2; ++al) {
        const int g = gram_stream_grid(n, m, dtype, al != 0, false, cu_count, kGramMaxBlocks);
        best = g > best ? g : best;
    }
    return best;
}

// ---- single-column Gram pass (the step after one worker's Write) ----------------
// Lane = rows; a block partial is column_mp(m) + 1 doubles in the partials buffer.
constexpr int kColThreads = 256;
constexpr int column_mp(int m)
{
    return m <= 4 ? 4 : (m <= 8 ? 8 : (m <= 16 ? 16 : (m <= 32 ? 32 : 64)));
}
// Blocks per compute unit.  A lane keeps 2 + min(8, m) (+ 8 above m = 8) 16-byte
// loads in flight and the pass streams best with 70 ... 100 KB in flight per unit;
// more is slower, not faster.  Measured at n = 124M, fp32 storage, blocks per unit
// 1 / 2 / 4: m = 32: 2.25 / 2.36 / 2.49 ms, m = 16: 1.14 / 1.20 / 1.22, m = 8: 0.61 /
// 0.60 / 0.65, m = 4: 0.81 / 0.47 / 0.34, m = 2: - / 0.23 / 0.17; 16-bit storage at
// m = 4 (n = 248M): 2 blocks 0.32, 4 blocks 0.33 ms.
constexpr int column_blocks_per_cu(int m, int dtype)
{
    return m > 8 ? 1 : ((m <= 4 && dtype == QN_F32) ? 4 : 2);
}
inline int column_pass_grid(int64_t n, int m, int dtype, int cu_count, int max_partials)
{
    const int R = dtype == QN_F32 ? 4 : 8;
    const int64_t want = ceil_div(n, static_cast<int64_t>(kColThreads) * R);
    int64_t cap = static_cast<int64_t>(cu_count) * column_blocks_per_cu(m, dtype);
    const int64_t room = static_cast<int64_t>(max_partials) * gram_entries(m) / (column_mp(m) + 1);
    if (cap > room)
        cap = room;
    return static_cast<int>(want < cap ? want : cap);
}

// ---- apply pass ---------------------------------------------------------------
constexpr int kApplyThreads = 256;
#ifndef QN_STAGED_THREADS_F32
#define QN_STAGED_THREADS_F32 256
#endif
#ifndef QN_STAGED_THREADS_BF16
#define QN_STAGED_THREADS_BF16 512
#endif
#ifndef QN_STAGED_BLOCKS_PER_CU
#define QN_STAGED_BLOCKS_PER_CU 1
#endif
#ifndef QN_STAGED_LDS_KB
#define QN_STAGED_LDS_KB 128
#endif
#ifndef QN_STAGED_MIN_SLABS
#define QN_STAGED_MIN_SLABS 1
#endif
constexpr int kStagedLdsBytes = QN_STAGED_LDS_KB * 1024;
constexpr int staged_threads(int dtype)
{
    return dtype == QN_F32 ? QN_STAGED_THREADS_F32 : QN_STAGED_THREADS_BF16;
}
constexpr int apply_rows_per_lane(int dtype) { return dtype == QN_F32 ? 4 : 8; }
// lane-steps per thread that one slab of staged results (16 bytes per 4 rows) allows
constexpr int staged_max_steps(int dtype)
{
    return kStagedLdsBytes / (staged_threads(dtype) * 4 * apply_rows_per_lane(dtype));
}

enum ApplyShape { kApplyElementwise = 0, kApplyDirect = 1, kApplyStaged = 2 };
struct ApplyPlan {
    int shape;
    int grid;
    int steps;      // staged only: lane-steps per thread and slab
};

// The staged kernel: block b owns slabs b, b + grid, ... of `slab` lane-steps
// (a lane-step is R rows); the number of lane-steps of the slab at `base` that exist.
QN_HD inline int64_t staged_slab_count(int64_t nvec, int64_t base, int64_t slab)
{
    const int64_t left = nvec - base;
    return left < slab ? left : slab;
}

inline ApplyPlan apply_plan(int64_t n, int dtype, int cu_count)
{
    ApplyPlan p{};
    const int R = apply_rows_per_lane(dtype);
    // 128-bit accesses work at element alignment, so the wide path serves every
    // input; the element-wise kernel is the shape for problems smaller than one
    // vector per lane
    const bool vec = n >= R;
    const int rows_per_thread = vec ? R : 1;
    const int64_t per_block = static_cast<int64_t>(kApplyThreads) * rows_per_thread;
    const int64_t want = ceil_div(n, per_block);
    const int64_t cap = static_cast<int64_t>(cu_count) * 8;
    p.grid = static_cast<int>(want < cap ? want : cap);
    p.shape = vec ? kApplyDirect : kApplyElementwise;
    p.steps = 0;
    // large problems: one block per compute unit with LDS-staged output bursts
    // (a full slab covers 32768 rows; worth it once every unit gets at least one)
    const int64_t slab_rows = kStagedLdsBytes / 4;
    if (vec && n >= slab_rows * cu_count * QN_STAGED_MIN_SLABS) {
        p.shape = kApplyStaged;
        p.grid = cu_count * QN_STAGED_BLOCKS_PER_CU;
        // slab length: every block gets the same number of (nearly) full slabs
        const int64_t lanes = static_cast<int64_t>(p.grid) * staged_threads(dtype);
        const int64_t per_thread = ceil_div(n / R, lanes);                  // lane-steps
        const int64_t rounds = ceil_div(per_thread, staged_max_steps(dtype));
        p.steps = static_cast<int>(ceil_div(per_thread, rounds));
    }
    return p;
}

// ---- workspace ------------------------------------------------------------------
// Layout of a workspace (all offsets multiples of 256 bytes):
//   partials   gram_max_partials * gram_entries doubles   stage-1 block results
//   mraw       kReduceRows * gram_entries doubles         reduced raw accumulators
//   small      the m x m and m-sized intermediates of the fused entry points
constexpr size_t ws_align(size_t v) { return (v + 255) / 256 * 256; }
constexpr size_t kWsMatrixBytes = ws_align(sizeof(double) * QN_MAX_M * QN_MAX_M);
constexpr size_t kWsVectorBytes = ws_align(sizeof(double) * QN_MAX_M);
constexpr size_t kWsSmallBytes = 3 * kWsMatrixBytes + 9 * kWsVectorBytes;

inline size_t workspace_need(int64_t n, int m, int dtype, int cu_count)
{
    const size_t entries = static_cast<size_t>(gram_entries(m));
    const size_t parts = static_cast<size_t>(gram_max_partials(n, m, dtype, cu_count));
    return ws_align(sizeof(double) * parts * entries) +
           ws_align(sizeof(double) * kReduceRows * entries) + kWsSmallBytes;
}

}  // namespace qn
