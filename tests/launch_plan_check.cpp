// CPU check of the launch arithmetic in psgd_internal.h (built and run by tests/test_library_host.py).
// Every column group must be owned by exactly one (sweep, workgroup) range, ranges must start on a
// 256-byte boundary, every workgroup must make the same number of sweeps, and no grid may exceed the
// partials buffer, whatever the device reports.
#include <cstdio>
#include <cstdlib>
#include <initializer_list>
#include <vector>

#include "psgd_internal.h"

using namespace psgd::plan;

static int failures = 0;
#define CHECK(cond, ...)                       \
    do {                                       \
        if (!(cond)) {                         \
            std::printf("FAIL: " __VA_ARGS__); \
            std::printf("\n");                 \
            ++failures;                        \
        }                                      \
    } while (0)

static void check_cover(int64_t ncg, int grid, int threads) {
    const SweepPlan p = sweep_plan(ncg, grid, threads);
    CHECK(p.chunk >= 1 && p.chunk <= threads, "ncg=%lld grid=%d: chunk %lld", (long long)ncg, grid, (long long)p.chunk);
    CHECK(p.count < 4 || p.chunk % kChunkAlign == 0, "ncg=%lld grid=%d: chunk %lld unaligned", (long long)ncg, grid,
          (long long)p.chunk);
    // ranges are consecutive in (sw * grid + b): they tile [0, count * grid * chunk), which must reach ncg,
    // and the range before the last sweep must not already have reached it (no sweep without work at all)
    const int64_t covered = p.count * grid * p.chunk;
    CHECK(covered >= ncg, "ncg=%lld grid=%d T=%d: only %lld covered", (long long)ncg, grid, threads, (long long)covered);
    CHECK(p.count == 0 || (p.count - 1) * grid * p.chunk < ncg, "ncg=%lld grid=%d T=%d: an empty sweep", (long long)ncg,
          grid, threads);
    // walk the ranges the way the kernel does and count owners of a few thousand probe groups
    const int64_t probes[] = {0, 1, p.chunk - 1, p.chunk, p.chunk + 1, ncg / 2, ncg - p.chunk, ncg - 2, ncg - 1};
    for (int64_t g : probes) {
        if (g < 0 || g >= ncg) continue;
        int owners = 0;
        const int64_t slot = g / p.chunk;           // the only range that can hold it
        for (int64_t s = slot > 0 ? slot - 1 : 0; s <= slot + 1; ++s) {
            const int64_t sw = s / grid, b = s % grid;
            if (sw >= p.count) continue;
            const int64_t base = (sw * grid + b) * p.chunk;
            if (base >= ncg) continue;
            const int64_t end = base + p.chunk < ncg ? base + p.chunk : ncg;
            if (g >= base && g < end && g - base < threads) ++owners;
        }
        CHECK(owners == 1, "ncg=%lld grid=%d T=%d: group %lld has %d owners", (long long)ncg, grid, threads,
              (long long)g, owners);
    }
}

int main() {
    // the five workloads' rows in 128-bit column groups, the grids an MI355X gives them, and odd neighbours
    const int64_t rows[] = {250000, 8000000, 6400000, 2000000, 25000000, 1, 15, 16, 17, 767, 768, 769, 196608, 196609,
                            786431, 786432, 786433, 123456789, (1ll << 31) + 257, (1ll << 33) + 5};
    const int grids[] = {1, 2, 7, 255, 256, 304, 1024, 4096};
    const int threads[] = {256, 768};
    for (int64_t ncg : rows)
        for (int g : grids)
            for (int t : threads) check_cover(ncg, g, t);
    // the die-contiguous mapping permutes the ranges of a sweep among the workgroups: a bijection, and the
    // workgroups of one die (b, b + 8, ...) take neighbouring ranges
    for (int grid : {1, 7, 8, 16, 255, 256, 304, 1024}) {
        std::vector<int> seen(grid, 0);
        for (int b = 0; b < grid; ++b) {
            const int64_t s = die_contiguous_slot(b, grid, 8);
            CHECK(s >= 0 && s < grid, "grid %d: slot %lld of workgroup %d", grid, (long long)s, b);
            if (s >= 0 && s < grid) ++seen[s];
        }
        for (int i = 0; i < grid; ++i) CHECK(seen[i] == 1, "grid %d: range %d taken %d times", grid, i, seen[i]);
        if (grid % 8 == 0 && grid >= 16)
            CHECK(die_contiguous_slot(8, grid, 8) == die_contiguous_slot(0, grid, 8) + 1, "grid %d: die neighbours", grid);
        else if (grid % 8 != 0)
            CHECK(die_contiguous_slot(grid - 1, grid, 8) == grid - 1, "grid %d: identity expected", grid);
    }
    // workload 5 on 256 compute units: 128 sweeps of 768-group chunks, the last range 64 groups long
    const SweepPlan w5 = sweep_plan(25000000, 256, 768);
    CHECK(w5.count == 128 && w5.chunk == 768, "workload 5 plan %lld x %lld", (long long)w5.count, (long long)w5.chunk);
    // workload 4: 10.2 sweeps' worth of groups take 11 sweeps of 720-group chunks (not 11 of 768)
    const SweepPlan w4 = sweep_plan(2000000, 256, 768);
    CHECK(w4.count == 11 && w4.chunk == 720, "workload 4 plan %lld x %lld", (long long)w4.count, (long long)w4.chunk);

    // grids never exceed the partials buffer, however many compute units a device reports
    for (int cus : {1, 64, 256, 304, 512, 513, 1024, 100000})
        for (int per_cu : {1, 4, 8}) {
            for (int64_t items : {(int64_t)0, (int64_t)1, (int64_t)255, (int64_t)256, (int64_t)1 << 20, (int64_t)1 << 40}) {
                const int g = persistent_grid(cus, items, per_cu, 256);
                CHECK(g >= 1 && g <= kMaxGrid, "persistent_grid(%d, %lld, %d) = %d", cus, (long long)items, per_cu, g);
                CHECK((int64_t)g <= (int64_t)cus * per_cu || g == 1, "persistent_grid above residency");
                const int dg = deg_grid(items, cus, per_cu);
                CHECK(dg >= 1 && dg <= kMaxGrid, "deg_grid(%lld, %d, %d) = %d", (long long)items, cus, per_cu, dg);
                CHECK(items < 1 || dg <= items, "deg_grid above the tile count");
            }
        }
    CHECK(persistent_grid(256, 25000000, 1, 768) == 256, "workload 5 grid");
    CHECK(persistent_grid(256, 1000, 4, 256) == 4, "short rows take one workgroup per 256 items");
    CHECK(deg_grid(1 << 30, 1024, 8) == kMaxGrid, "deg_grid clamp");
    // LDS plan of the tiled path: the widest power-of-two lane count whose slot table, two tile buffers and merge
    // slots fit the cap; workload shapes get full 1 KB row segments (wider for few learners), and nothing ever
    // exceeds the cap
    const size_t large = 160 * 1024 - 1024, small_cap = 40 * 1024 - 256;
    for (int n : {1, 2, 8, 16, 64, 65, 128, 300, 512})
        for (int deg : {1, 3, 5, 8, 13, 32}) {
            if ((long)n * deg > 4096) continue;
            for (int vec : {1, 4})
                for (int threads : {256, 512})
                    for (bool cd : {false, true})
                        for (size_t cap : {small_cap, large}) {
                            const int rpb = threads > 256 ? 8 : 4;
                            const TilePlan p = tile_plan(n, deg, vec, threads, cd, cap, 0, rpb);
                            if (p.lpr == 0) {
                                CHECK(cap == small_cap, "n=%d deg=%d vec=%d does not fit the large cap", n, deg, vec);
                                continue;
                            }
                            CHECK(p.lpr >= 1 && p.lpr <= threads && (p.lpr & (p.lpr - 1)) == 0, "lpr %d", p.lpr);
                            const int nrg = threads / p.lpr;
                            CHECK(p.lpr <= 64 || (n + nrg - 1) / nrg <= rpb, "n=%d: %d lanes per row leave %d rows per lane", n,
                                  p.lpr, (n + nrg - 1) / nrg);
                            CHECK(p.total <= cap, "n=%d deg=%d: %zu bytes over the cap %zu", n, deg, p.total, cap);
                            CHECK(p.tab_bytes >= (size_t)n * deg * 8 && p.tab_bytes % 16 == 0, "slot table size");
                            CHECK(p.tile_bytes >= (size_t)n * p.lpr * vec * 4 && p.tile_bytes % 16 == 0, "tile size");
                            const size_t slots = p.lpr <= 64 ? threads / 64 : nrg;
                            CHECK(p.comb_bytes == (cd ? slots * p.lpr * vec * 8 : 0), "merge slots");
                            CHECK(p.total == p.tab_bytes + 2 * p.tile_bytes + p.comb_bytes && !p.comb_in_tile, "total");
                        }
        }
    CHECK(tile_plan(128, 3, 4, 512, true, large, 0, 8).lpr == 32, "n = 128: 512-byte row segments");
    CHECK(tile_plan(70, 3, 4, 512, true, large, 0, 8).lpr == 64, "n = 70, several batches per tile: 1 KB row segments");
    CHECK(tile_plan(75, 3, 4, 512, true, large, 0, 8).lpr == 32, "n = 75 with the distance: 512-byte row segments");
    // one-batch form of the 1024-lane workgroup: whole-wavefront rows, at most 4 rows per lane, the merge slots
    // (48 KB at 16 B per lane) inside the consumed tile buffer when they do not fit beside the two tiles
    for (int n : {1, 2, 3, 5, 8, 9, 16, 20, 32, 48, 64, 65, 70, 128, 200, 256, 257, 512})
        for (int deg : {1, 3, 5, 13, 32})
            for (int vec : {1, 4})
                for (int threads : {512, 1024})
                    for (bool cd : {false, true}) {
                        if ((long)n * deg > 4096) continue;
                        const int rpb = threads == 1024 ? 4 : 8;
                        const TilePlan p = tile_plan(n, deg, vec, threads, cd, large, 0, rpb, true);
                        if (p.lpr == 0) {
                            CHECK(n > 256 || (long)n * deg * 8 > 24 * 1024, "n=%d deg=%d vec=%d cd=%d has no one-batch plan", n, deg, vec, (int)cd);
                            continue;
                        }
                        const int nrg = threads / p.lpr;
                        CHECK(p.lpr >= 16 && (p.lpr & (p.lpr - 1)) == 0 && (n + nrg - 1) / nrg <= rpb, "one-batch shape: lpr %d", p.lpr);
                        CHECK(nrg <= 64, "n=%d: %d row groups, the lanes of a column would not fit a wavefront", n, nrg);
                        CHECK(p.comb_bytes == (cd ? (size_t)nrg * p.lpr * vec * 12 : 0), "one-batch merge slots");
                        CHECK(p.total == p.tab_bytes + 2 * p.tile_bytes + (p.comb_in_tile ? 0 : p.comb_bytes) && p.total <= large,
                              "one-batch total");
                        CHECK(!p.comb_in_tile || (cd && p.comb_bytes <= p.tile_bytes), "merge slots inside a tile buffer must fit it");
                    }
    {
        const TilePlan p = tile_plan(64, 13, 4, 1024, true, large, 0, 4, true);
        CHECK(p.lpr == 64 && p.comb_in_tile, "n = 64, 13 slots, distance: 1 KB row segments, merge slots in the tile");
        CHECK(tile_plan(64, 3, 4, 1024, false, large, 0, 4, true).lpr == 64, "n = 64 without the distance");
        CHECK(tile_plan(64, 13, 4, 512, true, large, 0, 8, true).lpr == 64 && !tile_plan(64, 13, 4, 512, true, large, 0, 8, true).comb_in_tile,
              "n = 64 with the distance at 512 lanes: merge slots beside the tiles");
        CHECK(tile_plan(16, 3, 4, 1024, true, large, 0, 4, true).lpr == 256, "n = 16: 4 KB row segments, 4 rows per lane");
        CHECK(tile_plan(8, 3, 4, 1024, true, large, 0, 4, true).lpr == 512, "n = 8: 8 KB row segments");
        CHECK(tile_plan(128, 3, 4, 1024, false, large, 0, 4, true).lpr == 32, "n = 128: 512-byte row segments, 32 row groups of 4 rows");
        CHECK(tile_plan(128, 3, 4, 512, true, large, 0, 8, true).lpr == 32, "n = 128 with the distance: 16 row groups of 8 rows");
        CHECK(tile_plan(256, 3, 4, 1024, false, large, 0, 4, true).lpr == 16, "n = 256: 256-byte row segments");
        CHECK(tile_plan(257, 3, 4, 1024, false, large, 0, 4, true).lpr == 0, "n = 257: no one-batch plan");
        CHECK(!tile_plan(64, 3, 1, 1024, true, large, 0, 4, true).comb_in_tile, "4 B per lane: the merge slots fit beside the tiles");
    }
    if (failures) return 1;
    std::printf("launch plan ok\n");
    return 0;
}
