// Host-only check of libqn's launch arithmetic (csrc/qn_launch_math.h), built
// with g++ and its address / undefined-behaviour sanitizers by tests/test_host_checks.py.
// For every m, element type, alignment, z mode, compute-unit count and a list of
// row counts up to 2^34 it verifies what the kernels rely on: grids within the
// partials buffer, every tile and every row covered exactly once, slab lengths
// within LDS, counts within 32 bits, workspace sizes consistent with the grids.
#include <cinttypes>
#include <cstdio>
#include <cstdlib>

#include "qn_launch_math.h"

using namespace qn;

static int failures = 0;
#define CHECK(cond, ...)                                   \
    do {                                                   \
        if (!(cond)) {                                     \
            std::printf("FAIL %s:%d %s : ", __FILE__, __LINE__, #cond); \
            std::printf(__VA_ARGS__);                      \
            std::printf("\n");                             \
            if (++failures > 20) std::exit(1);             \
        }                                                  \
    } while (0)

static const int64_t kRows[] = {
    1, 2, 3, 4, 7, 8, 63, 64, 65, 255, 256, 257, 511, 512, 513, 1023, 1024, 1025, 4095, 4096,
    16383, 16384, 16385, 32767, 32768, 65537, 100003, 1200000, 8388607, 8388608, 8388609,
    25600000, 124000000, 124000001, 123999998, 1000000000, 2147483647LL, 2147483648LL,
    2300000001LL, 4294967296LL, 17179869184LL};
static const int kCus[] = {1, 8, 64, 255, 256, 304, 1024};

static void check_gram(int64_t n, int m, int dtype, int cu)
{
    const int entries = gram_entries(m);
    CHECK(entries % 64 == 0 && entries > 0 && entries <= kMaxEntries, "m=%d", m);
    const int maxp = gram_max_partials(n, m, dtype, cu);
    CHECK(maxp >= 1 && maxp <= kGramMaxBlocks, "n=%" PRId64 " m=%d maxp=%d", n, m, maxp);
    const size_t need = workspace_need(n, m, dtype, cu);
    CHECK(need % 256 == 0, "need=%zu", need);
    CHECK(need >= sizeof(double) * (size_t)maxp * entries + sizeof(double) * kReduceRows * entries +
                      kWsSmallBytes, "need=%zu", need);
    CHECK(need <= sizeof(double) * (size_t)kGramMaxBlocks * kMaxEntries + (1u << 20), "need=%zu", need);
    if (gram_is_small(n)) {
        const int grid = gram_small_grid(n, maxp);
        const int64_t tiles = ceil_div(n, kSmallTileRows);
        CHECK(grid >= 1 && grid <= maxp && grid <= tiles, "small grid=%d", grid);
        int64_t covered = 0;
        for (int b = 0; b < grid; ++b)
            for (int64_t t = b; t < tiles; t += grid)
                ++covered;
        CHECK(covered == tiles, "small tiles");
    }
    // the streaming pass must be launchable at any n (diagnostics force it), within
    // the buffer laid out for the larger of the two grids
    for (int al = 0; al < 2; ++al)
        for (int z = 0; z < 2; ++z) {
            const int nt = gram_sets(m);
            const int lds = gram_lds_bytes(nt, gram_z_slots(dtype, al != 0, m, z != 0));
            CHECK(lds <= kLdsPerCu, "lds=%d", lds);
            CHECK(gram_blocks_per_cu(lds) >= 1, "lds=%d", lds);
            const int rows = gram_tile_rows(dtype, al != 0, m);
            CHECK(rows == 256 || rows == 512 || rows == 1024 || rows == 2048, "rows=%d", rows);
            const int64_t tiles = ceil_div(n, rows);
            CHECK(tiles >= 1 && tiles * rows >= n && (tiles - 1) * rows < n, "tiles");
            const int cap = gram_is_small(n) ? kGramMaxBlocks : maxp;
            const int grid = gram_stream_grid(n, m, dtype, al != 0, z != 0, cu, cap);
            CHECK(grid >= 1 && grid <= cap && grid <= tiles, "grid=%d cap=%d", grid, cap);
            if (!gram_is_small(n))
                CHECK(grid <= maxp, "n=%" PRId64 " m=%d dt=%d al=%d z=%d grid=%d maxp=%d", n, m,
                      dtype, al, z, grid, maxp);
            // every tile goes to exactly one block
            int64_t total = 0;
            const int probe[] = {0, 1, grid / 2, grid - 1};
            for (int b = 0; b < grid; ++b) {
                const int64_t mine = block_tiles(tiles, b, grid);
                CHECK(mine >= 1, "block %d has no tile", b);
                total += mine;
            }
            CHECK(total == tiles, "total=%" PRId64 " tiles=%" PRId64, total, tiles);
            for (int b : probe)
                if (b >= 0 && b < grid) {
                    const int64_t mine = block_tiles(tiles, b, grid);
                    const int64_t last = b + (mine - 1) * grid;
                    CHECK(last < tiles && last + grid >= tiles, "last tile of block %d", b);
                }
        }
}

// The single-column pass after a Write: its grid fits the device and its block
// partials (column_mp(m) + 1 doubles each) fit the partials buffer of the workspace.
static void check_column(int64_t n, int m, int dtype, int cu)
{
    const int maxp = gram_max_partials(n, m, dtype, cu);
    const int grid = column_pass_grid(n, m, dtype, cu, maxp);
    const int bpc = column_blocks_per_cu(m, dtype);
    CHECK(bpc >= 1 && bpc <= 8, "blocks per unit %d", bpc);
    CHECK(grid >= 1 && grid <= (int64_t)cu * bpc, "n=%" PRId64 " m=%d grid=%d", n, m, grid);
    CHECK((int64_t)grid * (column_mp(m) + 1) <= (int64_t)maxp * gram_entries(m),
          "n=%" PRId64 " m=%d dt=%d cu=%d grid=%d maxp=%d", n, m, dtype, cu, grid, maxp);
    const int R = dtype == QN_F32 ? 4 : 8;
    CHECK(grid <= ceil_div(n, (int64_t)kColThreads * R), "more blocks than row groups");
    CHECK(column_mp(m) >= m && column_mp(m) <= QN_MAX_M, "mp");
}

static void check_apply(int64_t n, int dtype, int cu)
{
    const ApplyPlan p = apply_plan(n, dtype, cu);
    const int R = apply_rows_per_lane(dtype);
    CHECK(p.grid >= 1, "grid=%d", p.grid);
    if (n < R)
        CHECK(p.shape == kApplyElementwise, "shape");
    if (p.shape == kApplyStaged) {
        CHECK(p.grid == cu * QN_STAGED_BLOCKS_PER_CU, "grid");
        CHECK(p.steps >= 1 && p.steps <= staged_max_steps(dtype), "steps=%d", p.steps);
        const int threads = staged_threads(dtype);
        CHECK((int64_t)p.steps * threads * R * 4 <= kStagedLdsBytes, "slab exceeds LDS");
        const int64_t nvec = n / R, slab = (int64_t)p.steps * threads;
        // the kernel's loop: block b takes the slabs at b*slab, (b + grid)*slab, ...
        int64_t covered = 0, rounds_max = 0;
        for (int b = 0; b < p.grid; ++b) {
            int64_t rounds = 0;
            for (int64_t base = (int64_t)b * slab; base < nvec; base += (int64_t)p.grid * slab) {
                const int64_t cnt = staged_slab_count(nvec, base, slab);
                CHECK(cnt >= 1 && cnt <= slab && cnt * (R / 4) < (1LL << 31), "count");
                covered += cnt;
                ++rounds;
            }
            rounds_max = rounds > rounds_max ? rounds : rounds_max;
        }
        CHECK(covered == nvec, "covered=%" PRId64 " nvec=%" PRId64, covered, nvec);
        // balanced: no block works more than one slab longer than the average
        CHECK(rounds_max * slab * p.grid < nvec + 2 * slab * p.grid, "imbalance");
    } else {
        const int64_t per_block = (int64_t)kApplyThreads * (p.shape == kApplyDirect ? R : 1);
        CHECK(p.grid <= ceil_div(n, per_block) && p.grid <= (int64_t)cu * 8, "grid=%d", p.grid);
    }
}

int main()
{
    for (int64_t n : kRows)
        for (int cu : kCus) {
            for (int dt = QN_F32; dt <= QN_F16; ++dt) {
                check_apply(n, dt, cu);
                for (int m = 1; m <= QN_MAX_M; ++m) {
                    check_gram(n, m, dt, cu);
                    check_column(n, m, dt, cu);
                }
            }
        }
    // the reduction's grid: entries / 64 blocks by kReduceRows rows
    for (int m = 1; m <= QN_MAX_M; ++m)
        CHECK(gram_entries(m) / 64 * 64 == gram_entries(m), "m=%d", m);
    // the static scratch array of qn_update_noalloc (6 MiB) holds every problem on a
    // device of up to 256 units, and the check that refuses larger needs can fire
    size_t worst256 = 0, worst1024 = 0;
    for (int m = 1; m <= QN_MAX_M; ++m)
        for (int dt = QN_F32; dt <= QN_F16; ++dt) {
            const size_t a = workspace_need((int64_t)1 << 40, m, dt, 256);
            const size_t b = workspace_need((int64_t)1 << 40, m, dt, 1024);
            worst256 = a > worst256 ? a : worst256;
            worst1024 = b > worst1024 ? b : worst1024;
        }
    CHECK(worst256 <= 6u * 1024 * 1024, "worst256=%zu", worst256);
    CHECK(worst1024 > 6u * 1024 * 1024, "worst1024=%zu", worst1024);
    if (failures) {
        std::printf("%d failure(s)\n", failures);
        return 1;
    }
    std::printf("launch arithmetic ok (worst workspace on 256 units: %zu bytes)\n", worst256);
    return 0;
}
