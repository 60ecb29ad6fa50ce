// libpsgd's HIP translation unit (gfx950 / CDNA4): the launchers and C entry points for the model-averaging step
//     X_out[i,:] = sum_s w[i,s] * X[nbr[i,s],:] - lr * G[i,:]            (Sec. 2, Eq. 2)
// and for the consensus distance sum_i ||x_i - xbar||^2 (Sec. 3).  The kernels live in the headers included
// below: psgd_device.h (shared building blocks), psgd_ring_walk.h (ring tables, registers only), psgd_tiled.h
// (any other table, LDS tiles), psgd_streams.h (global averaging, distance, gradient producer, reference streams,
// table builder).
//
// The step is bound by HBM traffic (about 7 flops against 10-12 bytes per element), so the
// design goal is to touch every X, G and X_out byte exactly once:
//   * the update is separable by column, so a lane owns a group of 4 adjacent columns
//     (one 128-bit access per row) and sees all n rows of it;
//   * when the table describes a single ring (every table of Sec. 3 does), the lane walks
//     the ring in position order holding three consecutive rows in registers, so each
//     neighbour read is a register move, not a memory access, and the update may run in
//     place because a row is only written after its old value is in registers;
//   * any other table goes through [n x columns] tiles in LDS (a neighbour read is an LDS read), double
//     buffered, with the next tiles travelling from HBM through registers while the current one is
//     computed; a tile is complete in LDS before its first output is stored, so this path too may
//     run in place.
// Tables live in device memory and are validated and classified (one ring or not) by the kernels.
// Workgroups are persistent, so table staging is paid once per launch.  On long rows the workgroups are
// large (768 lanes for the ring walk, 512 or 1024 for the tiled path), one per compute unit; the ring walk's
// wavefronts sweep the rows in lockstep, a barrier per batch of rows: the HBM then sees one 12 KB burst
// per row instead of twelve separate 1 KB requests, which is worth 1-3 % of the peak for kernels that
// write.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <mutex>

#include "psgd.h"
#include "psgd_internal.h"

// Partial sums of psgd_mix_step_cd_static, the entry point for callers that cannot allocate: one double
// per persistent workgroup.  Every GPU holds its own copy of this array at its own address; host code
// never uses the name as a pointer, only the address hipGetSymbolAddress returns for the current device.
static __device__ __align__(256) double scratch[PSGD_STATIC_SLOTS];

#include "psgd_device.h"
#include "psgd_tiled.h"
#include "psgd_ring_walk.h"
#include "psgd_streams.h"

namespace psgd {
namespace {

// ---------------------------------------------------------------------------------------
// Host helpers.
// ---------------------------------------------------------------------------------------
struct DeviceInfo {
    int cus = 0;
    double* partials = nullptr;        // hipMalloc'ed on first use: kMaxGrid partials + 1 result slot
    hipEvent_t partials_idle = nullptr;     // recorded on the previous user's stream when another stream takes over
    hipStream_t partials_stream = nullptr;  // the stream (not under capture) that used `partials` last
    bool partials_used = false;
    double* static_partials = nullptr;  // device address of ::scratch on this GPU (psgd_mix_step_cd_static)
};
constexpr int kMaxDevices = 64;
DeviceInfo g_dev[kMaxDevices];
std::mutex g_dev_mutex;

int hip_fail(hipError_t e, const char* what) {
    return fail(PSGD_EHIP, "%s: %s", what, hipGetErrorString(e));
}

// Looks up (and caches) the current device's compute-unit count.
int device_info(DeviceInfo** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail(PSGD_EHIP, "device index %d unsupported", dev);
    std::lock_guard<std::mutex> lock(g_dev_mutex);
    DeviceInfo& di = g_dev[dev];
    if (di.cus == 0) {
        int cus = 0;
        e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) return hip_fail(e, "hipDeviceGetAttribute");
        di.cus = cus > 0 ? cus : 1;
    }
    *out = &di;
    return PSGD_OK;
}

bool stream_is_capturing(hipStream_t s) {
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &st) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return st != hipStreamCaptureStatusNone;
}

// The per-device partials buffer of the fused-distance and consensus calls, handed to work that is about
// to be enqueued on `s`.  It is allocated on the first call on a device; allocation is not allowed while a
// stream is being captured, so a first call made under capture is refused with an explanation instead of
// invalidating the capture.  All calls on a device share the buffer.  As long as they come on one stream the
// stream orders them and nothing is done here (no runtime call at all: short launches are bound by host time).
// When a call arrives on another stream than the previous one, an event is recorded behind everything enqueued
// so far on the previous stream and the new stream is made to wait for it (on the device, not on the host), so
// two streams that both gather a distance are serialised instead of racing.  Streams under capture are left
// alone: the order of graph launches is the caller's.
int acquire_partials(DeviceInfo* di, hipStream_t s, double** out) {
    std::lock_guard<std::mutex> lock(g_dev_mutex);
    if (di->partials && di->partials_used && di->partials_stream == s) {
        *out = di->partials;
        return PSGD_OK;
    }
    const bool capturing = stream_is_capturing(s);
    if (!di->partials) {
        if (capturing)
            return fail(PSGD_EHIP, "the per-device partials buffer is allocated on first use, which stream capture "
                                   "forbids: make one fused-distance or consensus call on this device before capturing");
        hipError_t e = hipMalloc(reinterpret_cast<void**>(&di->partials), sizeof(double) * (kMaxGrid + 1));
        if (e != hipSuccess) return hip_fail(e, "hipMalloc(partials)");
        e = hipEventCreateWithFlags(&di->partials_idle, hipEventDisableTiming);
        if (e != hipSuccess) {
            (void)hipFree(di->partials);
            di->partials = nullptr;
            return hip_fail(e, "hipEventCreateWithFlags");
        }
    }
    *out = di->partials;
    if (capturing) return PSGD_OK;                // captured work: ordered by whoever launches the graphs
    if (di->partials_used && !stream_is_capturing(di->partials_stream)) {
        // another stream used the buffer last: wait for all it has been given so far.  If that stream no longer
        // exists the record fails; its work may still be running, so the whole device is waited for instead.
        hipError_t e = hipEventRecord(di->partials_idle, di->partials_stream);
        if (e == hipSuccess) e = hipStreamWaitEvent(s, di->partials_idle, 0);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            e = hipDeviceSynchronize();
            if (e != hipSuccess) return hip_fail(e, "hipDeviceSynchronize(partials)");
        }
    }
    di->partials_stream = s;
    di->partials_used = true;
    return PSGD_OK;
}

// Called after the last kernel that reads the partials has been enqueued on `s` (nothing to do: the next user
// on another stream records its own event behind this work).
int release_partials(DeviceInfo*, hipStream_t) { return PSGD_OK; }

// Device address of the static scratch array on the current GPU, looked up once per device.
int static_partials(DeviceInfo* di, double** out) {
    std::lock_guard<std::mutex> lock(g_dev_mutex);
    if (!di->static_partials) {
        double* ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
        if (!ptr) return fail(PSGD_EHIP, "hipGetSymbolAddress(scratch) returned a null address");
        di->static_partials = ptr;
    }
    *out = di->static_partials;
    return PSGD_OK;
}

inline bool aligned_to(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

inline bool overlaps(const void* a, size_t abytes, const void* b, size_t bbytes) {
    const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
    return a0 < b0 + bbytes && b0 < a0 + abytes;
}

inline int persistent_grid(const DeviceInfo& di, int64_t work_items, int per_cu, int threads = kThreads) {
    return plan::persistent_grid(di.cus, work_items, per_cu, threads);
}

using plan::deg_grid;

// True if any row of A ([n] rows of ra bytes, lda bytes apart) shares a byte with any row of B.
bool rows_overlap(const void* A, int64_t lda, size_t ra, const void* B, int64_t ldb, size_t rb, int n) {
    if (ra == 0 || rb == 0) return false;
    const size_t span_a = (size_t)(n - 1) * (size_t)lda + ra, span_b = (size_t)(n - 1) * (size_t)ldb + rb;
    if (!overlaps(A, span_a, B, span_b)) return false;
    if ((size_t)lda == ra && (size_t)ldb == rb) return true;  // both dense: the spans are the arrays
    if (lda == ldb) {
        // Equal pitches P: row i of A meets row j of B iff  D - ra < (i - j) P < D + rb  with D = B - A.
        // Take the largest k = i - j (|k| <= n - 1) below the upper bound; smaller k only move away
        // from the lower one.
        const int64_t P = lda;
        const int64_t D = (int64_t)(reinterpret_cast<uintptr_t>(B) - reinterpret_cast<uintptr_t>(A));
        const int64_t t = D + (int64_t)rb - 1;
        int64_t k = t >= 0 ? t / P : -((-t + P - 1) / P);       // floor(t / P)
        if (k > n - 1) k = n - 1;
        if (k < -(int64_t)(n - 1)) return false;
        return k * P > D - (int64_t)ra;
    }
    const uintptr_t a0 = reinterpret_cast<uintptr_t>(A), b0 = reinterpret_cast<uintptr_t>(B);
    for (int i = 0; i < n; ++i) {
        const uintptr_t ai = a0 + (uintptr_t)i * (uintptr_t)lda;
        for (int j = 0; j < n; ++j) {
            const uintptr_t bj = b0 + (uintptr_t)j * (uintptr_t)ldb;
            if (ai < bj + rb && bj < ai + ra) return true;
        }
    }
    return false;
}

// Workgroups of `fn` (256 threads, `lds_bytes` of dynamic LDS) that fit one compute unit, as the
// runtime computes it from the kernel's registers and LDS; remembered per (kernel, LDS size).
int resident_per_cu(const void* fn, size_t lds_bytes, int threads = kThreads) {
    struct Entry {
        const void* fn;
        size_t lds;
        int occ;
    };
    static std::mutex mu;
    static Entry cache[128];
    static int used = 0;
    std::lock_guard<std::mutex> lock(mu);
    for (int i = 0; i < used; ++i)
        if (cache[i].fn == fn && cache[i].lds == lds_bytes) return cache[i].occ;
    int q = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&q, fn, threads, lds_bytes) != hipSuccess || q < 1) q = 1;
    if (used < 128) cache[used++] = Entry{fn, lds_bytes, q};
    return q;
}

// True if the double at p shares a byte with any row of B.
bool scalar_overlaps(const double* p, const void* B, int64_t ldb, size_t rb, int n) {
    const uintptr_t p0 = reinterpret_cast<uintptr_t>(p), b0 = reinterpret_cast<uintptr_t>(B);
    for (int j = 0; j < n; ++j) {
        const uintptr_t bj = b0 + (uintptr_t)j * (uintptr_t)ldb;
        if (p0 < bj + rb && bj < p0 + sizeof(double)) return true;
    }
    return false;
}

// A workgroup gets 64 KB of dynamic LDS by default; a kernel that is to be launched with more is opted in.
// Once per kernel and device (the attribute belongs to the kernel's code object on that device).
int allow_lds(const void* fn, size_t lds_bytes) {
    if (lds_bytes <= 64 * 1024 - 256) return PSGD_OK;
    struct Entry {
        const void* fn;
        int device;
    };
    static std::mutex mu;
    static Entry done[128];
    static int used = 0;
    int device = 0;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    std::lock_guard<std::mutex> lock(mu);
    for (int i = 0; i < used; ++i)
        if (done[i].fn == fn && done[i].device == device) return PSGD_OK;
    // the most this library ever asks for (the kernels' few hundred bytes of static LDS come on top of it)
    e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsCapLarge);
    if (e != hipSuccess) return hip_fail(e, "hipFuncSetAttribute(MaxDynamicSharedMemorySize)");
    if (used < 128) done[used++] = Entry{fn, device};
    return PSGD_OK;
}
constexpr int kLaunchRefused = INT32_MIN;

// Launches one instantiation of the mix kernel on a persistent grid sized to what is
// actually resident: min(kGridPerCu, occupancy for this LDS size) workgroups per CU.
// Returns the grid size, minus the grid size (and launches nothing) when the fused distance would need more
// than `slots` partials, or kLaunchRefused when the runtime refuses the LDS size.
template <int VEC, typename GT, bool CD, int T, bool TILES>
int launch_mix_t(const DeviceInfo& di, size_t lds_bytes, hipStream_t s, const float* X, float* X_out, const GT* G,
                 const int32_t* nbr, const float* w, int n, int64_t d, Pitch ld, float neg_lr, int lpr,
                 double* partials, int slots) {
    const void* fn = reinterpret_cast<const void*>(mix_step_kernel<VEC, GT, CD, T, TILES>);
    if (allow_lds(fn, lds_bytes)) return kLaunchRefused;
    const int occ = resident_per_cu(fn, lds_bytes, T);
    const int want = T == kThreads ? kGridPerCu : 1;
    const int grid = persistent_grid(di, d / VEC, occ < want ? occ : want, T);
    if (CD && grid > slots) return -grid;   // one partial per workgroup must fit the caller's buffer: nothing is launched
    hipLaunchKernelGGL((mix_step_kernel<VEC, GT, CD, T, TILES>), dim3(grid), dim3(T), lds_bytes, s, X, X_out, G, nbr, w,
                       n, d, ld, neg_lr, lpr, make_sweeps(d / VEC, grid, T), partials);
    return grid;
}

// Long rows take the large lockstep workgroup: at least `sweeps` column groups per lane of one such
// workgroup per CU.
inline bool long_rows(const DeviceInfo& di, int64_t column_groups, int sweeps = 2) {
    return column_groups >= (int64_t)di.cus * kRingThreads * sweeps;
}

template <int VEC, typename GT, bool CD>
int launch_mix(const DeviceInfo& di, bool big, size_t lds_bytes, hipStream_t s, const float* X, float* X_out,
               const GT* G, const int32_t* nbr, const float* w, int n, int64_t d, Pitch ld, float neg_lr, int lpr,
               double* partials, int slots) {
    return big ? launch_mix_t<VEC, GT, CD, kRingThreads, false>(di, lds_bytes, s, X, X_out, G, nbr, w, n, d, ld, neg_lr, lpr,
                                                                partials, slots)
               : launch_mix_t<VEC, GT, CD, kThreads, true>(di, lds_bytes, s, X, X_out, G, nbr, w, n, d, ld, neg_lr, lpr,
                                                           partials, slots);
}

// Pitches are in elements of the array they belong to.
template <typename GT>
int mix_step_impl(const char* name, const float* X, int64_t ldx, float* X_out, int64_t ldo, const GT* G, int64_t ldg,
                  const int32_t* nbr, const float* w, int n, int64_t d, float lr, int delay_mode, bool want_cd,
                  double* cd_out, void* stream, int deg = 3, bool no_alloc = false) {
    clear_error();
    if (!X || !X_out || !G || !nbr || !w || (want_cd && !cd_out)) return fail(PSGD_EINVAL, "%s: null pointer", name);
    if (n < 1 || n > PSGD_MAX_N) return fail(PSGD_EINVAL, "%s: n=%d outside 1..%d", name, n, (int)PSGD_MAX_N);
    if (deg < 1 || deg > PSGD_MAX_DEG || (int64_t)n * deg > PSGD_MAX_TABLE)
        return fail(PSGD_EINVAL, "%s: deg=%d outside 1..%d or n*deg > %d", name, deg, (int)PSGD_MAX_DEG,
                    (int)PSGD_MAX_TABLE);
    if (d < 0) return fail(PSGD_EINVAL, "%s: d=%lld is negative", name, (long long)d);
    if (delay_mode != 0 && delay_mode != 1) return fail(PSGD_EINVAL, "%s: delay_mode=%d", name, delay_mode);
    if (n > 1 && (ldx < d || ldo < d || ldg < d))
        return fail(PSGD_EINVAL, "%s: a row pitch is smaller than d=%lld", name, (long long)d);
    if (n == 1) ldx = ldo = ldg = d;
    if (!aligned_to(X, 4) || !aligned_to(X_out, 4) || !aligned_to(G, sizeof(GT)) || !aligned_to(nbr, 4) ||
        !aligned_to(w, 4) || (want_cd && !aligned_to(cd_out, 8)))
        return fail(PSGD_EALIGN, "%s: pointer not aligned to its element size", name);
    const int64_t ldmax = ldx > ldo ? (ldx > ldg ? ldx : ldg) : (ldo > ldg ? ldo : ldg);
    if (ldmax > 0 && (int64_t)n > INT64_MAX / 8 / ldmax) return fail(PSGD_EINVAL, "%s: n * pitch overflows", name);
    const size_t xrow = (size_t)d * sizeof(float), grow = (size_t)d * sizeof(GT);
    const int64_t bx = ldx * (int64_t)sizeof(float), bo = ldo * (int64_t)sizeof(float), bg = ldg * (int64_t)sizeof(GT);
    if (static_cast<const void*>(X) == static_cast<const void*>(X_out) && ldx == ldo) {
        if (delay_mode == 1)
            return fail(PSGD_EALIAS, "%s: delay-by-one keeps X read-only, X_out must be another buffer", name);
    } else if (rows_overlap(X, bx, xrow, X_out, bo, xrow, n)) {
        return fail(PSGD_EALIAS, "%s: X_out partially overlaps X", name);
    }
    if (rows_overlap(G, bg, grow, X_out, bo, xrow, n)) return fail(PSGD_EALIAS, "%s: X_out overlaps G", name);
    if (want_cd && (scalar_overlaps(cd_out, X_out, bo, xrow, n) || scalar_overlaps(cd_out, X, bx, xrow, n) ||
                    scalar_overlaps(cd_out, G, bg, grow, n)))
        return fail(PSGD_EALIAS, "%s: the distance output overlaps a data buffer", name);
    hipStream_t s = static_cast<hipStream_t>(stream);
    DeviceInfo* di = nullptr;
    if (d == 0 && !want_cd) return PSGD_OK;
    if (int rc = device_info(&di)) return rc;
    // Where the per-workgroup partial sums of the distance go: the library's own buffer (allocated on first
    // use, shared by every call on the device, streams serialised), or the static array of the entry point
    // that may not allocate (no serialisation: that would need an event).
    double* partials = nullptr;
    int slots = kMaxGrid;
    if (want_cd) {
        if (no_alloc) {
            if (int rc = static_partials(di, &partials)) return rc;
            slots = PSGD_STATIC_SLOTS;
        } else if (int rc = acquire_partials(di, s, &partials)) {
            return rc;
        }
    }
    if (d == 0) {
        hipLaunchKernelGGL(consensus_final_kernel, dim3(1), dim3(kThreads), 0, s, partials, 0, cd_out);
        const hipError_t e0 = hipGetLastError();
        if (e0 != hipSuccess) return hip_fail(e0, "consensus_final_kernel");
        return no_alloc ? PSGD_OK : release_partials(di, s);
    }
    // 128-bit path needs every row start 16-byte aligned (8-byte for bf16 gradients).
    const bool vec4 = (d % 4 == 0) && (ldx % 4 == 0) && (ldo % 4 == 0) && (ldg % 4 == 0) && aligned_to(X, 16) &&
                      aligned_to(X_out, 16) && aligned_to(G, 4 * sizeof(GT));
    const int vec = vec4 ? 4 : 1;
    // Long rows take a large workgroup that is alone on its compute unit; short ones four small workgroups.
    const bool big = long_rows(*di, d / vec);
    const float neg_lr = -lr;
    const Pitch ld{ldx, ldo, ldg};
    int grid = 0;        // partial sums written so far (the fused distance sums this many)
    const size_t classify = lds_table_bytes(n) + (size_t)n * 4 * sizeof(int);   // the 3-slot kernels' table copy + ranking arrays
    if (deg == 3) {
        // The ring-walk kernel does the work when the table is one ring (every table of Sec. 3).  On short rows
        // it also carries the tiled path, so that one launch serves any table; on long rows the tiled kernel
        // follows it (below), because there each path wants its own workgroup shape and registers.
        size_t ring_lds = classify;
        int ring_lpr = 0;
        if (!big) {
            plan::TilePlan rp = plan::tile_plan(n, 3, vec, kThreads, want_cd, kLdsCapSmall, lds_table_bytes(n), TileShape<kThreads>::RB);
            if (rp.lpr == 0) rp = plan::tile_plan(n, 3, vec, kThreads, want_cd, kLdsCapLarge, lds_table_bytes(n), TileShape<kThreads>::RB);
            if (rp.lpr == 0) return fail(PSGD_EINVAL, "%s: n=%d does not fit the tiled path's LDS", name, n);
            ring_lpr = rp.lpr;
            if (rp.total > ring_lds) ring_lds = rp.total;
        }
        if (vec4 && want_cd)
            grid = launch_mix<4, GT, true>(*di, big, ring_lds, s, X, X_out, G, nbr, w, n, d, ld, neg_lr, ring_lpr, partials, slots);
        else if (vec4)
            grid = launch_mix<4, GT, false>(*di, big, ring_lds, s, X, X_out, G, nbr, w, n, d, ld, neg_lr, ring_lpr, partials, slots);
        else if (want_cd)
            grid = launch_mix<1, GT, true>(*di, big, ring_lds, s, X, X_out, G, nbr, w, n, d, ld, neg_lr, ring_lpr, partials, slots);
        else
            grid = launch_mix<1, GT, false>(*di, big, ring_lds, s, X, X_out, G, nbr, w, n, d, ld, neg_lr, ring_lpr, partials, slots);
        if (grid == kLaunchRefused) return PSGD_EHIP;   // allow_lds has recorded the reason
        if (grid < 0)
            return fail(PSGD_EINVAL, "%s: this launch needs %d partial sums, the buffer holds %d", name, -grid, slots);
        const hipError_t e1 = hipGetLastError();
        if (e1 != hipSuccess) return hip_fail(e1, name);
    }
    if (deg != 3 || big) {
        // Tiled kernel: every table with another slot count, and behind the ring walk for 3-slot tables, where
        // it does the work only if the table turns out not to be one ring (decided on the device by both).
        // Long rows: the 1024-lane one-batch form where the shape allows it (n <= 64 at 1 KB row segments), else
        // 512 lanes with several batches per tile.  Short rows: small workgroups, several per compute unit.
        const size_t base = 0;
        plan::TilePlan tp;
        tp.lpr = 0;
        bool deep = false;
        const int deep_threads = want_cd ? kTileThreads : kDeepThreads;
        if (big) {
            tp = plan::tile_plan(n, deg, vec, deep_threads, want_cd, kLdsCapLarge, base,
                                 want_cd ? TileShape<kTileThreads>::RB : TileShape<kDeepThreads>::RB, true);
            deep = tp.lpr != 0;
            if (!deep) tp = plan::tile_plan(n, deg, vec, kTileThreads, want_cd, kLdsCapLarge, base, TileShape<kTileThreads>::RB);
        } else {
            tp = plan::tile_plan(n, deg, vec, kThreads, want_cd, kLdsCapSmall, base, TileShape<kThreads>::RB);
            if (tp.lpr == 0) tp = plan::tile_plan(n, deg, vec, kThreads, want_cd, kLdsCapLarge, base, TileShape<kThreads>::RB);
        }
        if (tp.lpr == 0)
            return fail(PSGD_EINVAL, "%s: n=%d, deg=%d does not fit the tiled path's LDS", name, n, deg);
        const int lpr = tp.lpr;
        size_t lds_bytes = tp.total;
        if (deg == 3 && lds_bytes < tp.tab_bytes + classify) lds_bytes = tp.tab_bytes + classify;
        const int64_t ntiles = (d / vec + lpr - 1) / lpr;
        const int first = grid;
        int tgrid = 0;
#define PSGD_DEG_LAUNCH(VEC, CD, T, DEEP)                                                                                   \
    do {                                                                                                                \
        const void* fn = reinterpret_cast<const void*>(mix_deg_kernel<VEC, GT, CD, T, DEEP>);                           \
        if (int rc = allow_lds(fn, lds_bytes)) return rc;                                                               \
        int per_cu = resident_per_cu(fn, lds_bytes, T);                                                                 \
        if (per_cu > 2 * kGridPerCu) per_cu = 2 * kGridPerCu;                                                           \
        tgrid = deg_grid(ntiles, di->cus, per_cu);                                                                      \
        if (CD && first + tgrid > slots) {   /* one partial per workgroup: a smaller persistent grid still covers */    \
            tgrid = slots - first;           /* every tile                                                        */    \
            if (tgrid < 1) {                                                                                            \
                tgrid = -(first + 1);                                                                                   \
                break;                                                                                                  \
            }                                                                                                           \
        }                                                                                                               \
        hipLaunchKernelGGL((mix_deg_kernel<VEC, GT, CD, T, DEEP>), dim3(tgrid), dim3(T), lds_bytes, s, X, X_out, G,     \
                           nbr, w,                                                                                     \
                           deg, n, d, ld, neg_lr, lpr, deg == 3 ? 1 : 0, tp.comb_in_tile ? 1 : 0,                    \
                           CD ? partials + first : partials);             \
    } while (0)
#define PSGD_DEG_PICK(VEC, CD)                                                                                          \
    do {                                                                                                                \
        if (deep && tp.lpr >= 64) PSGD_DEG_LAUNCH(VEC, CD, (CD ? kTileThreads : kDeepThreads), 1);                      \
        else if (deep) PSGD_DEG_LAUNCH(VEC, CD, (CD ? kTileThreads : kDeepThreads), 2);                                 \
        else if (big) PSGD_DEG_LAUNCH(VEC, CD, kTileThreads, 0);                                                        \
        else PSGD_DEG_LAUNCH(VEC, CD, kThreads, 0);                                                                     \
    } while (0)
        if (vec4 && want_cd) PSGD_DEG_PICK(4, true);
        else if (vec4) PSGD_DEG_PICK(4, false);
        else if (want_cd) PSGD_DEG_PICK(1, true);
        else PSGD_DEG_PICK(1, false);
#undef PSGD_DEG_PICK
#undef PSGD_DEG_LAUNCH
        grid = tgrid < 0 ? tgrid : first + tgrid;
    }
    if (grid < 0)
        return fail(PSGD_EINVAL, "%s: this launch needs %d partial sums, the buffer holds %d", name, -grid, slots);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, name);
    if (want_cd) {
        hipLaunchKernelGGL(consensus_final_kernel, dim3(1), dim3(kThreads), 0, s, partials, grid, cd_out);
        e = hipGetLastError();
        if (e != hipSuccess) return hip_fail(e, "consensus_final_kernel");
        if (!no_alloc) return release_partials(di, s);
    }
    return PSGD_OK;
}

template <typename GT>
int mix_full_impl(const char* name, const float* X, int64_t ldx, float* X_out, int64_t ldo, const GT* G, int64_t ldg,
                  int n, int64_t d, float lr, int delay_mode, double* cd_out, void* stream) {
    clear_error();
    const bool want_cd = cd_out != nullptr;
    if (!X || !X_out || !G) return fail(PSGD_EINVAL, "%s: null pointer", name);
    if (n < 1 || n > PSGD_MAX_N) return fail(PSGD_EINVAL, "%s: n=%d outside 1..%d", name, n, (int)PSGD_MAX_N);
    if (d < 0) return fail(PSGD_EINVAL, "%s: d=%lld is negative", name, (long long)d);
    if (delay_mode != 0 && delay_mode != 1) return fail(PSGD_EINVAL, "%s: delay_mode=%d", name, delay_mode);
    if (n > 1 && (ldx < d || ldo < d || ldg < d))
        return fail(PSGD_EINVAL, "%s: a row pitch is smaller than d=%lld", name, (long long)d);
    if (n == 1) ldx = ldo = ldg = d;
    if (!aligned_to(X, 4) || !aligned_to(X_out, 4) || !aligned_to(G, sizeof(GT)) || (want_cd && !aligned_to(cd_out, 8)))
        return fail(PSGD_EALIGN, "%s: pointer not aligned to its element size", name);
    const int64_t ldmax = ldx > ldo ? (ldx > ldg ? ldx : ldg) : (ldo > ldg ? ldo : ldg);
    if (ldmax > 0 && (int64_t)n > INT64_MAX / 8 / ldmax) return fail(PSGD_EINVAL, "%s: n * pitch overflows", name);
    const size_t xrow = (size_t)d * sizeof(float), grow = (size_t)d * sizeof(GT);
    const int64_t bx = ldx * (int64_t)sizeof(float), bo = ldo * (int64_t)sizeof(float), bg = ldg * (int64_t)sizeof(GT);
    if (static_cast<const void*>(X) == static_cast<const void*>(X_out) && ldx == ldo) {
        if (delay_mode == 1)
            return fail(PSGD_EALIAS, "%s: delay-by-one keeps X read-only, X_out must be another buffer", name);
    } else if (rows_overlap(X, bx, xrow, X_out, bo, xrow, n)) {
        return fail(PSGD_EALIAS, "%s: X_out partially overlaps X", name);
    }
    if (rows_overlap(G, bg, grow, X_out, bo, xrow, n)) return fail(PSGD_EALIAS, "%s: X_out overlaps G", name);
    if (want_cd && (scalar_overlaps(cd_out, X_out, bo, xrow, n) || scalar_overlaps(cd_out, X, bx, xrow, n) ||
                    scalar_overlaps(cd_out, G, bg, grow, n)))
        return fail(PSGD_EALIAS, "%s: the distance output overlaps a data buffer", name);
    hipStream_t s = static_cast<hipStream_t>(stream);
    DeviceInfo* di = nullptr;
    if (d == 0 && !want_cd) return PSGD_OK;
    if (int rc = device_info(&di)) return rc;
    double* partials = nullptr;
    if (want_cd)
        if (int rc = acquire_partials(di, s, &partials)) return rc;
    if (d == 0) {
        hipLaunchKernelGGL(consensus_final_kernel, dim3(1), dim3(kThreads), 0, s, partials, 0, cd_out);
        const hipError_t e0 = hipGetLastError();
        if (e0 != hipSuccess) return hip_fail(e0, "consensus_final_kernel");
        return release_partials(di, s);
    }
    const bool vec4 = (d % 4 == 0) && (ldx % 4 == 0) && (ldo % 4 == 0) && (ldg % 4 == 0) && aligned_to(X, 16) &&
                      aligned_to(X_out, 16) && aligned_to(G, 4 * sizeof(GT));
    const bool big = long_rows(*di, vec4 ? d / 4 : d, 2);
    const int grid = big ? persistent_grid(*di, vec4 ? d / 4 : d, 1, kRingThreads)
                         : persistent_grid(*di, vec4 ? d / 4 : d, kGridPerCu);
    const dim3 g(grid), b(big ? kRingThreads : kThreads);
    const Pitch ld{ldx, ldo, ldg};
    const float neg_lr = -lr;
#define PSGD_LAUNCH_FULL(VEC, CD)                                                                                          \
    do {                                                                                                                   \
        if (big)                                                                                                           \
            hipLaunchKernelGGL((mix_full_kernel<VEC, GT, CD, kRingThreads>), g, b, 0, s, X, X_out, G, n, d, ld, neg_lr,     \
                               make_sweeps(d / VEC, grid, kRingThreads), partials);                                        \
        else                                                                                                               \
            hipLaunchKernelGGL((mix_full_kernel<VEC, GT, CD, kThreads>), g, b, 0, s, X, X_out, G, n, d, ld, neg_lr,         \
                               make_sweeps(d / VEC, grid, kThreads), partials);                                            \
    } while (0)
    if (vec4 && want_cd)
        PSGD_LAUNCH_FULL(4, true);
    else if (vec4)
        PSGD_LAUNCH_FULL(4, false);
    else if (want_cd)
        PSGD_LAUNCH_FULL(1, true);
    else
        PSGD_LAUNCH_FULL(1, false);
#undef PSGD_LAUNCH_FULL
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, name);
    if (want_cd) {
        hipLaunchKernelGGL(consensus_final_kernel, dim3(1), dim3(kThreads), 0, s, partials, grid, cd_out);
        e = hipGetLastError();
        if (e != hipSuccess) return hip_fail(e, "consensus_final_kernel");
        return release_partials(di, s);
    }
    return PSGD_OK;
}

int consensus_enqueue(const float* X, int64_t ldx, int n, int64_t d, double* out_dev, hipStream_t s,
                      double** result_slot) {
    DeviceInfo* di = nullptr;
    if (int rc = device_info(&di)) return rc;
    double* partials = nullptr;
    if (int rc = acquire_partials(di, s, &partials)) return rc;
    if (result_slot) *result_slot = partials + kMaxGrid;
    const bool vec4 = (d % 4 == 0) && (ldx % 4 == 0) && aligned_to(X, 16);
    int grid = 0;
    if (d > 0) {
        const int64_t ncg = vec4 ? d / 4 : d;
        if (long_rows(*di, ncg)) {
            grid = persistent_grid(*di, ncg, 1, kRingThreads);
            const Sweeps sw = make_sweeps(ncg, grid, kRingThreads);
            if (vec4)
                hipLaunchKernelGGL((consensus_sweep_kernel<4, kRingThreads>), dim3(grid), dim3(kRingThreads), 0, s, X, n, d,
                                   ldx, sw, partials);
            else
                hipLaunchKernelGGL((consensus_sweep_kernel<1, kRingThreads>), dim3(grid), dim3(kRingThreads), 0, s, X, n, d,
                                   ldx, sw, partials);
        } else {
            grid = persistent_grid(*di, ncg, 8);  // light kernel: 32 waves per CU
            if (vec4)
                hipLaunchKernelGGL(consensus_partial_kernel<4>, dim3(grid), dim3(kThreads), 0, s, X, n, d, ldx, partials);
            else
                hipLaunchKernelGGL(consensus_partial_kernel<1>, dim3(grid), dim3(kThreads), 0, s, X, n, d, ldx, partials);
        }
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return hip_fail(e, "consensus_partial_kernel");
    }
    // d = 0: nothing to reduce, the final kernel over zero partials writes 0
    hipLaunchKernelGGL(consensus_final_kernel, dim3(1), dim3(kThreads), 0, s, partials, grid,
                       out_dev ? out_dev : partials + kMaxGrid);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "consensus_final_kernel");
    return release_partials(di, s);
}

int consensus_check(const char* name, const float* X, int64_t ldx, int n, int64_t d) {
    if (!X) return fail(PSGD_EINVAL, "%s: null pointer", name);
    if (n < 1 || n > PSGD_MAX_N) return fail(PSGD_EINVAL, "%s: n=%d outside 1..%d", name, n, (int)PSGD_MAX_N);
    if (d < 0) return fail(PSGD_EINVAL, "%s: d=%lld is negative", name, (long long)d);
    if (n > 1 && ldx < d) return fail(PSGD_EINVAL, "%s: row pitch smaller than d", name);
    if (!aligned_to(X, 4)) return fail(PSGD_EALIGN, "%s: X not 4-byte aligned", name);
    if (ldx > 0 && (int64_t)n > INT64_MAX / 8 / ldx) return fail(PSGD_EINVAL, "%s: n * pitch overflows", name);
    return PSGD_OK;
}

int consensus_async_impl(const char* name, const float* X, int64_t ldx, int n, int64_t d, double* out_dev,
                         void* stream) {
    clear_error();
    if (!out_dev) return fail(PSGD_EINVAL, "%s: null output pointer", name);
    if (!aligned_to(out_dev, 8)) return fail(PSGD_EALIGN, "%s: out_dev not 8-byte aligned", name);
    if (int rc = consensus_check(name, X, ldx, n, d)) return rc;
    return consensus_enqueue(X, n == 1 ? d : ldx, n, d, out_dev, static_cast<hipStream_t>(stream), nullptr);
}

}  // namespace
}  // namespace psgd

extern "C" {

int psgd_mix_step(const float* X, float* X_out, const float* G, const int32_t* nbr, const float* w, int n, int64_t d,
                  float lr, int delay_mode, void* stream) {
    return psgd::mix_step_impl<float>("psgd_mix_step", X, d, X_out, d, G, d, nbr, w, n, d, lr, delay_mode, false,
                                      nullptr, stream);
}

int psgd_mix_step_bf16g(const float* X, float* X_out, const uint16_t* G_bf16, const int32_t* nbr, const float* w,
                        int n, int64_t d, float lr, int delay_mode, void* stream) {
    return psgd::mix_step_impl<uint16_t>("psgd_mix_step_bf16g", X, d, X_out, d, G_bf16, d, nbr, w, n, d, lr,
                                         delay_mode, false, nullptr, stream);
}

int psgd_mix_step_cd(const float* X, float* X_out, const float* G, const int32_t* nbr, const float* w, int n,
                     int64_t d, float lr, int delay_mode, double* cdist_out, void* stream) {
    return psgd::mix_step_impl<float>("psgd_mix_step_cd", X, d, X_out, d, G, d, nbr, w, n, d, lr, delay_mode, true,
                                      cdist_out, stream);
}

int psgd_mix_step_cd_bf16g(const float* X, float* X_out, const uint16_t* G_bf16, const int32_t* nbr, const float* w,
                           int n, int64_t d, float lr, int delay_mode, double* cdist_out, void* stream) {
    return psgd::mix_step_impl<uint16_t>("psgd_mix_step_cd_bf16g", X, d, X_out, d, G_bf16, d, nbr, w, n, d, lr,
                                         delay_mode, true, cdist_out, stream);
}

int psgd_mix_step_ex(const float* X, int64_t ldx, float* X_out, int64_t ldo, const void* G, int64_t ldg, int g_is_bf16,
                     const int32_t* nbr, const float* w, int n, int64_t d, float lr, int delay_mode,
                     double* cdist_out, void* stream) {
    if (g_is_bf16 != 0 && g_is_bf16 != 1) {
        psgd::clear_error();
        return psgd::fail(PSGD_EINVAL, "psgd_mix_step_ex: g_is_bf16=%d", g_is_bf16);
    }
    if (g_is_bf16)
        return psgd::mix_step_impl<uint16_t>("psgd_mix_step_ex", X, ldx, X_out, ldo, static_cast<const uint16_t*>(G),
                                             ldg, nbr, w, n, d, lr, delay_mode, cdist_out != nullptr, cdist_out,
                                             stream);
    return psgd::mix_step_impl<float>("psgd_mix_step_ex", X, ldx, X_out, ldo, static_cast<const float*>(G), ldg, nbr,
                                      w, n, d, lr, delay_mode, cdist_out != nullptr, cdist_out, stream);
}

int psgd_mix_step_cd_static(const float* X, int64_t ldx, float* X_out, int64_t ldo, const void* G, int64_t ldg,
                            int g_is_bf16, const int32_t* nbr, const float* w, int n, int64_t d, float lr,
                            int delay_mode, double* cdist_out, void* stream) {
    if (g_is_bf16 != 0 && g_is_bf16 != 1) {
        psgd::clear_error();
        return psgd::fail(PSGD_EINVAL, "psgd_mix_step_cd_static: g_is_bf16=%d", g_is_bf16);
    }
    if (g_is_bf16)
        return psgd::mix_step_impl<uint16_t>("psgd_mix_step_cd_static", X, ldx, X_out, ldo,
                                             static_cast<const uint16_t*>(G), ldg, nbr, w, n, d, lr, delay_mode, true,
                                             cdist_out, stream, 3, true);
    return psgd::mix_step_impl<float>("psgd_mix_step_cd_static", X, ldx, X_out, ldo, static_cast<const float*>(G), ldg,
                                      nbr, w, n, d, lr, delay_mode, true, cdist_out, stream, 3, true);
}

int psgd_mix_step_deg(const float* X, int64_t ldx, float* X_out, int64_t ldo, const void* G, int64_t ldg, int g_is_bf16,
                      const int32_t* nbr, const float* w, int deg, int n, int64_t d, float lr, int delay_mode,
                      double* cdist_out, void* stream) {
    if (g_is_bf16 != 0 && g_is_bf16 != 1) {
        psgd::clear_error();
        return psgd::fail(PSGD_EINVAL, "psgd_mix_step_deg: g_is_bf16=%d", g_is_bf16);
    }
    if (g_is_bf16)
        return psgd::mix_step_impl<uint16_t>("psgd_mix_step_deg", X, ldx, X_out, ldo, static_cast<const uint16_t*>(G),
                                             ldg, nbr, w, n, d, lr, delay_mode, cdist_out != nullptr, cdist_out,
                                             stream, deg);
    return psgd::mix_step_impl<float>("psgd_mix_step_deg", X, ldx, X_out, ldo, static_cast<const float*>(G), ldg, nbr,
                                      w, n, d, lr, delay_mode, cdist_out != nullptr, cdist_out, stream, deg);
}

int psgd_mix_full(const float* X, int64_t ldx, float* X_out, int64_t ldo, const void* G, int64_t ldg, int g_is_bf16,
                  int n, int64_t d, float lr, int delay_mode, double* cdist_out, void* stream) {
    if (g_is_bf16 != 0 && g_is_bf16 != 1) {
        psgd::clear_error();
        return psgd::fail(PSGD_EINVAL, "psgd_mix_full: g_is_bf16=%d", g_is_bf16);
    }
    if (g_is_bf16)
        return psgd::mix_full_impl<uint16_t>("psgd_mix_full", X, ldx, X_out, ldo, static_cast<const uint16_t*>(G), ldg,
                                             n, d, lr, delay_mode, cdist_out, stream);
    return psgd::mix_full_impl<float>("psgd_mix_full", X, ldx, X_out, ldo, static_cast<const float*>(G), ldg, n, d, lr,
                                      delay_mode, cdist_out, stream);
}

int psgd_build_mixing_device(int topology, int n, uint64_t seed, uint64_t* step_dev, uint64_t step_offset, int advance,
                             int32_t* nbr, float* w, void* stream) {
    using namespace psgd;
    clear_error();
    if (!nbr || !w) return fail(PSGD_EINVAL, "psgd_build_mixing_device: null output pointer");
    if (n < 1 || n > PSGD_MAX_N)
        return fail(PSGD_EINVAL, "psgd_build_mixing_device: n=%d outside 1..%d", n, (int)PSGD_MAX_N);
    if (topology == PSGD_TOPO_FULL)
        return fail(PSGD_EINVAL, "psgd_build_mixing_device: the uniform topology has no 3-slot table, use psgd_mix_full");
    if (topology != PSGD_TOPO_RING && topology != PSGD_TOPO_RAND_RING)
        return fail(PSGD_EINVAL, "psgd_build_mixing_device: unknown topology %d", topology);
    if (advance < 0) return fail(PSGD_EINVAL, "psgd_build_mixing_device: advance=%d is negative", advance);
    if (!aligned_to(nbr, 4) || !aligned_to(w, 4) || (step_dev && !aligned_to(step_dev, 8)))
        return fail(PSGD_EALIGN, "psgd_build_mixing_device: pointer not aligned to its element size");
    const size_t tb = (size_t)n * 3 * 4;
    if (overlaps(nbr, tb, w, tb) || (step_dev && (overlaps(step_dev, 8, nbr, tb) || overlaps(step_dev, 8, w, tb))))
        return fail(PSGD_EALIAS, "psgd_build_mixing_device: nbr, w and step_dev overlap");
    hipLaunchKernelGGL(build_mixing_kernel, dim3(1), dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                       topology == PSGD_TOPO_RAND_RING ? 1 : 0, n, seed, step_dev, step_offset, (uint64_t)advance, nbr, w);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "build_mixing_kernel");
    return PSGD_OK;
}

double psgd_consensus_dist(const float* X, int n, int64_t d) {
    using namespace psgd;
    clear_error();
    if (consensus_check("psgd_consensus_dist", X, d, n, d) != PSGD_OK) return NAN;
    if (d == 0 || n == 1) return 0.0;
    hipError_t e = hipDeviceSynchronize();
    if (e != hipSuccess) { hip_fail(e, "hipDeviceSynchronize"); return NAN; }
    double* slot = nullptr;
    if (consensus_enqueue(X, d, n, d, nullptr, nullptr, &slot) != PSGD_OK) return NAN;
    double host = NAN;
    e = hipMemcpy(&host, slot, sizeof(double), hipMemcpyDeviceToHost);
    if (e != hipSuccess) { hip_fail(e, "hipMemcpy(result)"); return NAN; }
    return host;
}

int psgd_consensus_dist_async(const float* X, int n, int64_t d, double* out_dev, void* stream) {
    return psgd::consensus_async_impl("psgd_consensus_dist_async", X, d, n, d, out_dev, stream);
}

int psgd_consensus_dist_ex(const float* X, int64_t ldx, int n, int64_t d, double* out_dev, void* stream) {
    return psgd::consensus_async_impl("psgd_consensus_dist_ex", X, ldx, n, d, out_dev, stream);
}

int psgd_synth_grad(const float* X_prev, const float* noise, float* G, int64_t count, float c, void* stream) {
    using namespace psgd;
    clear_error();
    if (!X_prev || !noise || !G) return fail(PSGD_EINVAL, "psgd_synth_grad: null pointer");
    if (count < 0) return fail(PSGD_EINVAL, "psgd_synth_grad: negative count");
    if (!aligned_to(X_prev, 4) || !aligned_to(noise, 4) || !aligned_to(G, 4))
        return fail(PSGD_EALIGN, "psgd_synth_grad: pointer not 4-byte aligned");
    const size_t bytes = (size_t)count * sizeof(float);
    if (overlaps(G, bytes, X_prev, bytes) || overlaps(G, bytes, noise, bytes))
        return fail(PSGD_EALIAS, "psgd_synth_grad: G overlaps an input");
    if (count == 0) return PSGD_OK;
    DeviceInfo* di = nullptr;
    if (int rc = device_info(&di)) return rc;
    const int vec4 = aligned_to(X_prev, 16) && aligned_to(noise, 16) && aligned_to(G, 16);
    const int grid = persistent_grid(*di, vec4 ? (count + 3) / 4 : count, 16);
    hipLaunchKernelGGL(synth_grad_kernel, dim3(grid), dim3(kThreads), 0, static_cast<hipStream_t>(stream), X_prev,
                       noise, G, count, c, vec4);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "synth_grad_kernel");
    return PSGD_OK;
}

int psgd_synth_grad_ex(const float* X_prev, int64_t ldx, const float* noise, int64_t ldn, float* G, int64_t ldg,
                       int n, int64_t d, float c, void* stream) {
    using namespace psgd;
    clear_error();
    if (!X_prev || !noise || !G) return fail(PSGD_EINVAL, "psgd_synth_grad_ex: null pointer");
    if (n < 1 || n > PSGD_MAX_N || d < 0) return fail(PSGD_EINVAL, "psgd_synth_grad_ex: n=%d d=%lld", n, (long long)d);
    if (n > 1 && (ldx < d || ldn < d || ldg < d)) return fail(PSGD_EINVAL, "psgd_synth_grad_ex: a row pitch is smaller than d");
    if (n == 1) ldx = ldn = ldg = d;
    if (!aligned_to(X_prev, 4) || !aligned_to(noise, 4) || !aligned_to(G, 4))
        return fail(PSGD_EALIGN, "psgd_synth_grad_ex: pointer not 4-byte aligned");
    const int64_t ldmax = ldx > ldn ? (ldx > ldg ? ldx : ldg) : (ldn > ldg ? ldn : ldg);
    if (ldmax > 0 && (int64_t)n > INT64_MAX / 8 / ldmax) return fail(PSGD_EINVAL, "psgd_synth_grad_ex: n * pitch overflows");
    const size_t row = (size_t)d * sizeof(float);
    if (rows_overlap(G, ldg * 4, row, X_prev, ldx * 4, row, n) || rows_overlap(G, ldg * 4, row, noise, ldn * 4, row, n))
        return fail(PSGD_EALIAS, "psgd_synth_grad_ex: G overlaps an input");
    if (d == 0) return PSGD_OK;
    DeviceInfo* di = nullptr;
    if (int rc = device_info(&di)) return rc;
    const bool vec4 = d % 4 == 0 && ldx % 4 == 0 && ldn % 4 == 0 && ldg % 4 == 0 && aligned_to(X_prev, 16) &&
                      aligned_to(noise, 16) && aligned_to(G, 16);
    const int grid = persistent_grid(*di, vec4 ? d / 4 : d, 8);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (vec4)
        hipLaunchKernelGGL(synth_grad_rows_kernel<4>, dim3(grid), dim3(kThreads), 0, s, X_prev, ldx, noise, ldn, G, ldg,
                           n, d, c);
    else
        hipLaunchKernelGGL(synth_grad_rows_kernel<1>, dim3(grid), dim3(kThreads), 0, s, X_prev, ldx, noise, ldn, G, ldg,
                           n, d, c);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "synth_grad_rows_kernel");
    return PSGD_OK;
}

int psgd_reference_stream(int kind, const float* X, int64_t ldx, float* X_out, int64_t ldo, const void* G, int64_t ldg,
                          int g_is_bf16, int n, int64_t d, float a, void* stream) {
    using namespace psgd;
    clear_error();
    if (kind != kRefRead && kind != kRefWrite && kind != kRefAxpy)
        return fail(PSGD_EINVAL, "psgd_reference_stream: kind=%d", kind);
    if (g_is_bf16 != 0 && g_is_bf16 != 1) return fail(PSGD_EINVAL, "psgd_reference_stream: g_is_bf16=%d", g_is_bf16);
    if (!X || !X_out || !G) return fail(PSGD_EINVAL, "psgd_reference_stream: null pointer");
    if (n < 1 || n > PSGD_MAX_N || d < 0) return fail(PSGD_EINVAL, "psgd_reference_stream: n=%d d=%lld", n, (long long)d);
    if (n > 1 && (ldx < d || ldo < d || ldg < d))
        return fail(PSGD_EINVAL, "psgd_reference_stream: a row pitch is smaller than d");
    if (n == 1) ldx = ldo = ldg = d;
    const size_t gsz = g_is_bf16 ? 2 : 4;
    if (d % 4 || ldx % 4 || ldo % 4 || ldg % 4 || !aligned_to(X, 16) || !aligned_to(X_out, 16) || !aligned_to(G, 4 * gsz))
        return fail(PSGD_EALIGN, "psgd_reference_stream: needs d and the pitches in multiples of 4 and 128-bit aligned rows");
    const int64_t ldmax = ldx > ldo ? (ldx > ldg ? ldx : ldg) : (ldo > ldg ? ldo : ldg);
    if (ldmax > 0 && (int64_t)n > INT64_MAX / 8 / ldmax) return fail(PSGD_EINVAL, "psgd_reference_stream: n * pitch overflows");
    const size_t xrow = (size_t)d * 4, grow = (size_t)d * gsz;
    if (kind != kRefRead && (rows_overlap(X, ldx * 4, xrow, X_out, ldo * 4, xrow, n) ||
                             rows_overlap(G, ldg * (int64_t)gsz, grow, X_out, ldo * 4, xrow, n)))
        return fail(PSGD_EALIAS, "psgd_reference_stream: X_out overlaps an input");
    if (d == 0) return PSGD_OK;
    DeviceInfo* di = nullptr;
    if (int rc = device_info(&di)) return rc;
    const bool big = long_rows(*di, d / 4);
    const int threads = big ? kRingThreads : kThreads;
    const int grid = persistent_grid(*di, d / 4, big ? 1 : kGridPerCu, threads);
    const Sweeps sw = make_sweeps(d / 4, grid, threads);
    const Pitch ld{ldx, ldo, ldg};
    hipStream_t s = static_cast<hipStream_t>(stream);
#define PSGD_REF_LAUNCH(KIND, GT, T)                                                                                    \
    hipLaunchKernelGGL((reference_stream_kernel<KIND, GT, T>), dim3(grid), dim3(T), 0, s, X, X_out,                      \
                       static_cast<const GT*>(G), n, d, ld, a, sw)
#define PSGD_REF_KIND(KIND)                                                                                             \
    do {                                                                                                                \
        if (g_is_bf16 && big) PSGD_REF_LAUNCH(KIND, uint16_t, kRingThreads);                                            \
        else if (g_is_bf16) PSGD_REF_LAUNCH(KIND, uint16_t, kThreads);                                                  \
        else if (big) PSGD_REF_LAUNCH(KIND, float, kRingThreads);                                                       \
        else PSGD_REF_LAUNCH(KIND, float, kThreads);                                                                    \
    } while (0)
    if (kind == kRefRead) PSGD_REF_KIND(kRefRead);
    else if (kind == kRefWrite) PSGD_REF_KIND(kRefWrite);
    else PSGD_REF_KIND(kRefAxpy);
#undef PSGD_REF_KIND
#undef PSGD_REF_LAUNCH
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "reference_stream_kernel");
    return PSGD_OK;
}

int psgd_device_status(int clear) {
    using namespace psgd;
    clear_error();
    hipError_t e = hipDeviceSynchronize();
    if (e != hipSuccess) return hip_fail(e, "hipDeviceSynchronize");
    int word = 0;
    e = hipMemcpyFromSymbol(&word, HIP_SYMBOL(g_status_word), sizeof(int));
    if (e != hipSuccess) return hip_fail(e, "hipMemcpyFromSymbol");
    if (clear && word) {
        const int zero = 0;
        e = hipMemcpyToSymbol(HIP_SYMBOL(g_status_word), &zero, sizeof(int));
        if (e != hipSuccess) return hip_fail(e, "hipMemcpyToSymbol");
    }
    return word;
}

}  // extern "C"
