// Declarations shared by the library's own translation units (not part of the C boundary).
#ifndef PSGD_INTERNAL_H
#define PSGD_INTERNAL_H

#include <cstdint>

namespace psgd {

// Records a printf-style message for psgd_last_error() on this thread and returns `code`.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();

// Launch arithmetic of the persistent grids: plain host functions, kept apart from the kernels so that a CPU
// build can check them (every column group covered once, grids within the partials buffer).
namespace plan {

constexpr int kMaxGrid = 4096;    // upper bound on persistent workgroups = slots of the partials buffer
constexpr int kChunkAlign = 16;   // column groups (256 bytes): ranges that start at an odd 16 bytes cost 7 %

// Workgroups of `threads` lanes for `work_items` lane-sized items: one per item batch, at most `per_cu`
// per compute unit, never more than kMaxGrid.
inline int persistent_grid(int cus, int64_t work_items, int per_cu, int threads) {
    const int64_t need = (work_items + threads - 1) / threads;
    int64_t cap = (int64_t)cus * per_cu;
    if (cap > kMaxGrid) cap = kMaxGrid;
    const int64_t g = need < cap ? need : cap;
    return (int)(g < 1 ? 1 : g);
}

// Grid of the degree-K kernel: one workgroup per tile up to what is resident, within the same bound.
inline int deg_grid(int64_t ntiles, int cus, int per_cu) {
    int64_t cap = (int64_t)cus * per_cu;
    if (cap > kMaxGrid) cap = kMaxGrid;
    const int64_t g = ntiles < cap ? ntiles : cap;
    return (int)(g < 1 ? 1 : g);
}

// Which range of a sweep workgroup `b` of `grid` takes.  The hardware deals consecutive workgroups out to the
// chip's `xcds` accelerator dies in turn (each with its own L2), so taking range b would hand every die every
// xcds-th range of the row; with this mapping the workgroups that share a die (b, b + xcds, ...) take
// neighbouring ranges, and each L2 sees one contiguous stretch of every row in flight.  Measured on MI355X
// (8 dies) with the step's traffic pattern: 78.4 against 78.0 % of the HBM peak.  A bijection on 0..grid-1 when
// xcds divides grid, the identity otherwise.
#if defined(__HIPCC__)
#define PSGD_HOST_DEVICE __host__ __device__
#else
#define PSGD_HOST_DEVICE
#endif
PSGD_HOST_DEVICE inline int64_t die_contiguous_slot(int64_t b, int64_t grid, int xcds) {
    if (xcds <= 1 || grid % xcds != 0) return b;
    return (b % xcds) * (grid / xcds) + b / xcds;
}

// Even split of `ncg` column groups over a persistent grid: every workgroup makes `count` sweeps and takes
// `chunk` <= threads consecutive groups in each; workgroup b's range in sweep sw starts at
// (sw * grid + die_contiguous_slot(b)) * chunk.  With a fixed chunk of `threads` the last, partly filled sweep costs as much as a
// full one (11 instead of 10.2 on rows of 2 M groups with 256 workgroups of 768 lanes); the kernels are bound
// by bytes, so a sweep is as much faster as it is smaller.  The chunk stays a multiple of kChunkAlign.
struct SweepPlan {
    int64_t count, chunk;
};
inline SweepPlan sweep_plan(int64_t ncg, int grid, int threads) {
    SweepPlan s;
    const int64_t per = (int64_t)grid * threads;
    s.count = (ncg + per - 1) / per;
    if (s.count < 4) {   // a launch of one to three sweeps is bound by latency: full chunks, fewer of them
        s.chunk = threads;
        return s;
    }
    const int64_t parts = s.count * grid;
    s.chunk = (ncg + parts - 1) / parts;
    s.chunk = (s.chunk + kChunkAlign - 1) / kChunkAlign * kChunkAlign;
    return s;
}

// LDS of the tiled path (tables that are not one ring): the slot table (8 bytes per slot), TWO tile buffers of
// n rows x lpr lanes x vec floats (the next tile is staged while the current one is read), and, when the
// consensus distance is gathered in the same pass, the merge slots of the column sums: one double per column
// and per wavefront (lpr <= 64: row groups inside a wavefront merge by shuffles) or per row group (lpr > 64),
// plus a float per slot where row groups are whole wavefronts (lpr >= 64: each keeps its own pivot).
// `lpr`, the lanes that share a row, is the largest power of two <= threads for which all of it, plus `base`
// bytes the kernel keeps for itself, fits `cap`; rows wider than a wavefront (lpr > 64) are only taken while a
// lane still gets at most `rows_per_batch` rows, which is what few learners need to keep enough bytes in flight
// (n = 16: 256 lanes per row, 8 rows per lane).  lpr = 0 if not even one lane per row fits.
constexpr int kOneBatchMinLpr = 16;
struct TilePlan {
    int lpr;
    bool comb_in_tile;   // one-batch form only: the merge slots of the distance live in the tile buffer just consumed
    size_t tab_bytes, tile_bytes, comb_bytes, total;
};
// one_batch: plan for the large workgroup's one-batch form, which needs every row of a tile in one batch (at most
// rows_per_batch rows per lane) and at least 16 lanes per row (256-byte row segments at 16 B per lane; also what
// keeps the lanes that share a column in the merge of the distance inside one wavefront); it may put the merge
// slots into the buffer it has finished reading (one more barrier per tile) when they do not fit beside the two
// tiles.
inline TilePlan tile_plan(int n, int deg, int vec, int threads, bool cd, size_t cap, size_t base, int rows_per_batch,
                          bool one_batch = false) {
    TilePlan p;
    p.comb_in_tile = false;
    p.tab_bytes = (((size_t)n * deg * 8) + 15) & ~(size_t)15;
    for (p.lpr = threads; p.lpr >= (one_batch ? kOneBatchMinLpr : 1); p.lpr >>= 1) {
        const int nrg = threads / p.lpr;
        const int rows = (n + nrg - 1) / nrg;
        if ((one_batch || p.lpr > 64) && rows > rows_per_batch) continue;
        const int slots = (one_batch || p.lpr > 64) ? nrg : threads / 64;   // one per row group, or per wavefront where row groups share one
        p.tile_bytes = (((size_t)n * p.lpr * vec * 4) + 15) & ~(size_t)15;
        p.comb_bytes = cd ? (size_t)slots * p.lpr * vec * (one_batch ? 12 : 8) : 0;   // one-batch form: + a float per slot, the row group's own pivot
        p.total = base + p.tab_bytes + 2 * p.tile_bytes + p.comb_bytes;
        if (p.total <= cap) return p;
        if (one_batch && cd && p.comb_bytes <= p.tile_bytes && p.total - p.comb_bytes <= cap) {
            p.comb_in_tile = true;
            p.total -= p.comb_bytes;
            return p;
        }
    }
    p.lpr = 0;
    return p;
}

}  // namespace plan
}  // namespace psgd

#endif
