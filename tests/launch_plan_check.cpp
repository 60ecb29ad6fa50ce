// CPU check of the launch arithmetic in psgd_internal.h (built and run by tests/test_library_host.py).
// Every column group must be owned by exactly one (sweep, workgroup) range, ranges must start on a
// 256-byte boundary, every workgroup must make the same number of sweeps, and no grid may exceed the
// partials buffer, whatever the device reports.
#include <cstdio>
#include <cstdlib>
#include <initializer_list>

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
    if (failures) return 1;
    std::printf("launch plan ok\n");
    return 0;
}
