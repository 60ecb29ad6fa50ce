// HIP kernels (gfx950 / CDNA4) and their launchers for the model-averaging step
//     X_out[i,:] = sum_s w[i,s] * X[nbr[i,s],:] - lr * G[i,:]            (Sec. 2, Eq. 2)
// and for the consensus distance sum_i ||x_i - xbar||^2 (Sec. 3).
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

namespace psgd {
namespace {

constexpr int kThreads = 256;        // 4 wavefronts of 64 lanes
constexpr int kRingThreads = 768;    // workgroup of the step kernels on long rows (12 wavefronts in lockstep, one per CU;
                                     // 1024 lanes would leave the fused distance too few registers)
constexpr int kDeepThreads = 1024;   // workgroup of the tiled path on long rows, one-batch form: 16 wavefronts, four per
                                     // SIMD, which is what keeps the slot loop's LDS round trips and arithmetic hidden
constexpr int kTileThreads = 512;    // the same for shapes the one-batch form does not take (more than 64 learners at
                                     // 16 B per lane): 8 wavefronts with up to 256 registers, several batches per tile
constexpr int kUnroll = 8;           // rows whose loads are in flight together per lane
using plan::kMaxGrid;                // upper bound on persistent workgroups (partials buffer sizing)
constexpr int kGridPerCu = 4;        // persistent workgroups per compute unit (16 waves per CU)
constexpr int kXcds = 8;             // accelerator dies of an MI355X: consecutive workgroups go to consecutive dies
// LDS a workgroup may ask for: a compute unit has 160 KB.  The large lockstep workgroup is alone on its CU
// and may take nearly all of it; the small one leaves room for four per CU unless the table needs more.
constexpr size_t kLdsCapLarge = 160 * 1024 - 1024;
constexpr size_t kLdsCapSmall = 40 * 1024 - 256;

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ int g_status_word = 0;

// ---------------------------------------------------------------------------------------
// Column-group value types: VEC = 4 (128-bit accesses) or 1 (any d, any 4-byte alignment).
// ---------------------------------------------------------------------------------------
template <int VEC> struct Cols;
template <> struct Cols<4> { typedef f32x4 T; };
template <> struct Cols<1> { typedef float T; };

__device__ __forceinline__ f32x4 splat4(float v) { return (f32x4){v, v, v, v}; }

__device__ __forceinline__ float vfma(float a, float b, float c) { return __builtin_fmaf(a, b, c); }
__device__ __forceinline__ f32x4 vfma(float a, f32x4 b, f32x4 c) {
    return __builtin_elementwise_fma(splat4(a), b, c);
}

// X, G and X_out are each touched once per step: mark the accesses non-temporal so they
// stream through the caches instead of displacing one another.
__device__ __forceinline__ float ld_x(const float* p, Cols<1>) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ f32x4 ld_x(const float* p, Cols<4>) {
    return __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
}
__device__ __forceinline__ void st_x(float* p, float v) { __builtin_nontemporal_store(v, p); }
__device__ __forceinline__ void st_x(float* p, f32x4 v) {
    __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(p));
}
__device__ __forceinline__ float ld_g(const float* p, Cols<1> c) { return ld_x(p, c); }
__device__ __forceinline__ f32x4 ld_g(const float* p, Cols<4> c) { return ld_x(p, c); }
// bfloat16 is the upper half of an fp32, so widening is a 16-bit shift and exact.
__device__ __forceinline__ float ld_g(const uint16_t* p, Cols<1>) {
    return __uint_as_float((uint32_t)__builtin_nontemporal_load(p) << 16);
}
__device__ __forceinline__ f32x4 ld_g(const uint16_t* p, Cols<4>) {
    const u32x2 b = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(p));
    return (f32x4){__uint_as_float(b.x << 16), __uint_as_float(b.x & 0xFFFF0000u),
                   __uint_as_float(b.y << 16), __uint_as_float(b.y & 0xFFFF0000u)};
}

// A gradient group as it arrives from memory, widened only where it is used: a value that is converted right
// after its load would make the wavefront wait for that load (and every earlier one) on the spot, which defeats
// loads that are issued early to travel during other work; bf16 groups also take half the registers this way.
template <typename GT, int VEC> struct RawG;
template <> struct RawG<float, 4> { typedef f32x4 T; };
template <> struct RawG<float, 1> { typedef float T; };
template <> struct RawG<uint16_t, 4> { typedef u32x2 T; };
template <> struct RawG<uint16_t, 1> { typedef uint16_t T; };
__device__ __forceinline__ f32x4 ld_g_raw(const float* p, Cols<4> c) { return ld_x(p, c); }
__device__ __forceinline__ float ld_g_raw(const float* p, Cols<1> c) { return ld_x(p, c); }
__device__ __forceinline__ u32x2 ld_g_raw(const uint16_t* p, Cols<4>) {
    return __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(p));
}
__device__ __forceinline__ uint16_t ld_g_raw(const uint16_t* p, Cols<1>) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ f32x4 widen_g(f32x4 v) { return v; }
__device__ __forceinline__ float widen_g(float v) { return v; }
__device__ __forceinline__ f32x4 widen_g(u32x2 b) {
    return (f32x4){__uint_as_float(b.x << 16), __uint_as_float(b.x & 0xFFFF0000u),
                   __uint_as_float(b.y << 16), __uint_as_float(b.y & 0xFFFF0000u)};
}
__device__ __forceinline__ float widen_g(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// Two barriers that are lighter than __syncthreads(), which also waits until every global load and store the
// wavefront has issued is complete.  That wait is exactly what the step kernels must avoid: their loads are
// issued early to travel during other work, and their stores need never be waited for.
//   lockstep_barrier: keeps the workgroup's wavefronts on the same batch of rows; no data passes between them.
//   lds_barrier: the wavefront's own LDS reads and writes are complete (its global ones may still travel), then
//   the barrier: LDS written before it by any wavefront is read after it by any other.
__device__ __forceinline__ void lockstep_barrier() { __builtin_amdgcn_s_barrier(); }
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// One output group.  The operation order is part of the boundary's contract.
template <typename V>
__device__ __forceinline__ V mix_one(float w0, float w1, float w2, V self, V left, V right,
                                     V g, float neg_lr) {
    V acc = self * w0;
    acc = vfma(w1, left, acc);
    acc = vfma(w2, right, acc);
    return vfma(neg_lr, g, acc);
}

// Row pitches in elements: row i of X starts at X + i * x, of X_out at X_out + i * o, of G at
// G + i * g.  Dense arrays have all three equal to d; larger pitches let a caller interleave
// the rows of several arrays across the whole HBM (see the note on placement in the header).
struct Pitch {
    int64_t x, o, g;
};

// One ring position, packed so the walk fetches it with a single 128-bit LDS read.
struct __attribute__((aligned(16))) RingEnt {
    int row;
    float w0, w1, w2;
};

// One slot of a table row as the tiled path keeps it in LDS: where the source row starts inside the tile
// (nbr * lanes-per-row, in column groups) and its weight.
struct __attribute__((aligned(8))) TileSlot {
    uint32_t off;
    float w;
};

// LDS carve-up of the 3-slot step kernel (dynamic, sized by the launcher):
//   RingEnt ring[n] | int nbr[3n] | float w[3n] | scratch
// scratch holds the ranking arrays while the table is classified and, for a table that is not one ring, the
// tiled path's slot table, tile buffers and merge slots (plan::tile_plan).
struct Lds {
    RingEnt* ring;
    int* nbr;
    float* w;
    char* scratch;
};
__host__ __device__ inline size_t lds_table_bytes(int n) {
    return (((size_t)n * (sizeof(RingEnt) + 3 * (sizeof(int) + sizeof(float)))) + 15) & ~(size_t)15;
}
__device__ __forceinline__ Lds carve(char* base, int n) {
    Lds l;
    l.ring = reinterpret_cast<RingEnt*>(base);
    l.nbr = reinterpret_cast<int*>(base + (size_t)n * sizeof(RingEnt));
    l.w = reinterpret_cast<float*>(l.nbr + 3 * n);
    l.scratch = base + lds_table_bytes(n);   // 16-byte aligned
    return l;
}

// Ring entries are the same for every lane; moving them to scalar registers keeps the row
// offsets and weights out of the vector register file.
__device__ __forceinline__ int ring_row(const RingEnt* e) { return __builtin_amdgcn_readfirstlane(e->row); }
__device__ __forceinline__ RingEnt ring_ent(const RingEnt* e) {
    RingEnt r;
    r.row = __builtin_amdgcn_readfirstlane(e->row);
    r.w0 = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(e->w0)));
    r.w1 = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(e->w1)));
    r.w2 = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(e->w2)));
    return r;
}

enum TableKind { kTableBad = 0, kTableRing = 1, kTableGeneral = 2 };

// Stage the table in LDS, check it, and decide whether it is a single ring.
//
// A ring here means: slot 0 of row i is i itself, and the left/right slots are mutually
// consistent (the right neighbour's left is i and vice versa), which makes "right" a
// bijection, and following it from learner 0 visits all n learners.  The last property is
// decided by parallel list ranking (pointer doubling) toward learner 0's left neighbour;
// the resulting distances are the ring positions, used to fill `ring` in walk order.
template <int T>
__device__ int stage_table(const int32_t* __restrict__ nbr, const float* __restrict__ w, int n,
                           const Lds& l) {
    const int tid = threadIdx.x;
    int ok = 1;
    for (int e = tid; e < 3 * n; e += T) {
        const int v = nbr[e];
        l.nbr[e] = v;
        l.w[e] = w[e];
        ok &= (unsigned)v < (unsigned)n;
    }
    if (!__syncthreads_and(ok)) return kTableBad;

    int ring = 1;
    for (int i = tid; i < n; i += T) {
        const int left = l.nbr[3 * i + 1], right = l.nbr[3 * i + 2];
        ring &= (l.nbr[3 * i] == i) & (l.nbr[3 * right + 1] == i) & (l.nbr[3 * left + 2] == i);
    }
    if (!__syncthreads_and(ring)) return kTableGeneral;

    int* nxt_a = reinterpret_cast<int*>(l.scratch);
    int* dst_a = nxt_a + n;
    int* nxt_b = dst_a + n;
    int* dst_b = nxt_b + n;
    const int tail = l.nbr[1];  // learner 0's left neighbour ends the list that starts at 0
    for (int i = tid; i < n; i += T) {
        nxt_a[i] = (i == tail) ? i : l.nbr[3 * i + 2];
        dst_a[i] = (i == tail) ? 0 : 1;
    }
    __syncthreads();
    for (int span = 1; span < n; span <<= 1) {
        for (int i = tid; i < n; i += T) {
            const int j = nxt_a[i];
            nxt_b[i] = nxt_a[j];
            dst_b[i] = dst_a[i] + dst_a[j];
        }
        __syncthreads();
        int* t = nxt_a; nxt_a = nxt_b; nxt_b = t;
        t = dst_a; dst_a = dst_b; dst_b = t;
    }
    int reached = 1;
    for (int i = tid; i < n; i += T) reached &= (nxt_a[i] == tail);
    if (!__syncthreads_and(reached)) return kTableGeneral;
    for (int i = tid; i < n; i += T) {
        const int pos = n - 1 - dst_a[i];
        RingEnt e;
        e.row = i;
        e.w0 = l.w[3 * i];
        e.w1 = l.w[3 * i + 1];
        e.w2 = l.w[3 * i + 2];
        l.ring[pos] = e;
    }
    __syncthreads();
    return kTableRing;
}

// ---------------------------------------------------------------------------------------
// Consensus distance.  Per column: with pivot s = X[0, j],
//   sum_i (x_i - xbar)^2 = sum_i (x_i - s)^2 - (sum_i (x_i - s))^2 / n,
// one pass, differences and sums in fp64 (the difference of two fp32 values is exact in
// fp64 unless their exponents are more than 29 apart, and because the pivot is one of the
// points the subtraction cancels at most a factor n).
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    return v;
}

// Sum over the workgroup (T threads); the per-wavefront sums are added in a fixed order.
template <int T = kThreads>
__device__ __forceinline__ double block_sum(double v, double* lds_waves) {
    v = wave_sum(v);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if (lane == 0) lds_waves[wave] = v;
    __syncthreads();
    double r = 0.0;
    if (threadIdx.x == 0) {
#pragma unroll
        for (int i = 0; i < T / 64; i += 2) r += lds_waves[i] + lds_waves[i + 1];
    }
    return r;  // valid in thread 0
}

template <int VEC>
__device__ __forceinline__ void acc_diff(double* a, double* b, typename Cols<VEC>::T x, const double* s);
template <>
__device__ __forceinline__ void acc_diff<1>(double* a, double* b, float x, const double* s) {
    const double df = (double)x - s[0];
    a[0] += df;
    b[0] = fma(df, df, b[0]);
}
template <>
__device__ __forceinline__ void acc_diff<4>(double* a, double* b, f32x4 x, const double* s) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const double df = (double)x[k] - s[k];
        a[k] += df;
        b[k] = fma(df, df, b[k]);
    }
}
__device__ __forceinline__ void pivot_of(float x, double* s) { s[0] = (double)x; }
__device__ __forceinline__ void pivot_of(f32x4 x, double* s) {
#pragma unroll
    for (int k = 0; k < 4; ++k) s[k] = (double)x[k];
}
__device__ __forceinline__ void floats_of(float x, float* f) { f[0] = x; }
__device__ __forceinline__ void floats_of(f32x4 x, float* f) {
#pragma unroll
    for (int k = 0; k < 4; ++k) f[k] = x[k];
}

// Running sums of one lane's column group; the first value it is given becomes the pivot (kept as
// the fp32 value it is).  The squares of all the group's columns share one accumulator: only their
// total is needed, and registers are what limits the size of the step kernel's workgroups.
template <int VEC>
struct ColStats {
    typename Cols<VEC>::T s;
    double a[VEC], sq;
    int have;
    __device__ __forceinline__ void reset() {
        have = 0;
        sq = 0.0;
#pragma unroll
        for (int k = 0; k < VEC; ++k) a[k] = 0.0;
    }
    __device__ __forceinline__ void add(typename Cols<VEC>::T x) {
        if (!have) {
            s = x;
            have = 1;
        } else {
            double xs[VEC], ps[VEC];
            pivot_of(x, xs);
            pivot_of(s, ps);
#pragma unroll
            for (int k = 0; k < VEC; ++k) {
                const double df = xs[k] - ps[k];
                a[k] += df;
                sq = fma(df, df, sq);
            }
        }
    }
    __device__ __forceinline__ double result(double inv_n) const {
        double t = sq;
#pragma unroll
        for (int k = 0; k < VEC; ++k) t -= a[k] * a[k] * inv_n;
        return t;
    }
};

// ---------------------------------------------------------------------------------------
// Ring walk: one lane, one column group, all n rows, registers only.
// Rows are visited in ring order p = 0..n-1.  `first` and `last` (positions 0 and n-1) stay
// in registers for the wrap-around, so every X element is loaded exactly once and, when
// X_out aliases X, always before the store that replaces it.
// ---------------------------------------------------------------------------------------
//
// The workgroup's wavefronts are kept on the same batch of rows by a barrier per batch: each row
// then receives one contiguous burst of (workgroup size) * 16 bytes, which the HBM serves a little
// faster than the same bytes arriving wavefront by wavefront.  Every lane of the workgroup therefore
// walks the ring the same number of times; a lane without a column group of its own (`act` false,
// ragged end of the row) shadows a valid group with its loads and stores nothing.
template <int VEC, typename GT, bool CD>
__device__ __forceinline__ void ring_walk(const float* xc, float* oc, const GT* __restrict__ gc,
                                          const RingEnt* ring, int n, Pitch ld, float neg_lr,
                                          ColStats<VEC>& stats, bool act) {
    typedef typename Cols<VEC>::T V;
    const Cols<VEC> tag{};
    const V first = ld_x(xc + (int64_t)ring_row(ring) * ld.x, tag);
    const V last = (n > 1) ? ld_x(xc + (int64_t)ring_row(ring + n - 1) * ld.x, tag) : first;
    V prev = last, cur = first;
    int p = 0;
    // Whole batches: positions p .. p+U-1, whose right neighbours p+1 .. p+U are all fresh
    // loads (none of them is position n-1 or the wrap to position 0).
    for (; p + kUnroll <= n - 2; p += kUnroll) {
        lockstep_barrier();
        RingEnt e[kUnroll];
        V xs[kUnroll], gs[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            e[u] = ring_ent(ring + p + u);
            xs[u] = ld_x(xc + (int64_t)ring_row(ring + p + u + 1) * ld.x, tag);
            gs[u] = ld_g(gc + (int64_t)e[u].row * ld.g, tag);
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const V out = mix_one<V>(e[u].w0, e[u].w1, e[u].w2, cur, prev, xs[u], gs[u], neg_lr);
            if (act) st_x(oc + (int64_t)e[u].row * ld.o, out);
            if (CD) stats.add(out);
            prev = cur;
            cur = xs[u];
        }
    }
    // Remainder (at most U + 1 positions), with the wrap-around served from registers.
    while (p < n) {
        RingEnt e[kUnroll];
        V xs[kUnroll], gs[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int pp = p + u;
            if (pp < n) {
                e[u] = ring_ent(ring + pp);
                gs[u] = ld_g(gc + (int64_t)e[u].row * ld.g, tag);
                if (pp + 1 <= n - 2) xs[u] = ld_x(xc + (int64_t)ring_row(ring + pp + 1) * ld.x, tag);
                else if (pp + 1 == n - 1) xs[u] = last;
                else xs[u] = first;
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            if (p + u < n) {
                const V out = mix_one<V>(e[u].w0, e[u].w1, e[u].w2, cur, prev, xs[u], gs[u], neg_lr);
                if (act) st_x(oc + (int64_t)e[u].row * ld.o, out);
                if (CD) stats.add(out);
                prev = cur;
                cur = xs[u];
            }
        }
        p += kUnroll;
    }
}

// ---------------------------------------------------------------------------------------
// Tiled path for tables that are not a single ring (any number of slots per row).
//
// The workgroup's T lanes form T / lpr row groups of lpr lanes; a tile is n rows by lpr column groups and lives
// in LDS, so a neighbour read is an LDS read and every X element crosses the HBM interface once.  Lane (rg,
// lane) produces rows rg, rg + nrg, ... of column group `lane` of the tile.  Two tile buffers alternate: while
// the rows of tile t are computed from one, the X rows of the workgroup's next tile are written into the
// other.  A barrier per tile separates "everyone has finished reading this buffer and writing the other" from
// the next tile.  A tile is complete in LDS before its first output is stored, and different tiles own
// different columns, so X_out may alias X.
//
// Two forms.  tile_path_deep (long rows, up to 256 learners): the tile's rows are one batch, every memory
// operation is unconditional, and a lane reloads each of its registers the moment its value has been used (see
// there).  tile_path (short rows; long rows with more learners): several batches per tile, the next tile's
// batch travelling while this tile's is computed, loads under conditions.
//
// Per output the slots are taken in table order, acc = w0 * x0, one fma per further slot, then the gradient
// term (for 3 slots exactly mix_one's order).  The slot loop is the latency-critical part (a table read, then
// a tile read that depends on it, per slot): SB rows advance together and two slots per trip, so SB * 2
// independent chains hide each other's LDS round trips.
//
// With CD the distance of the outputs is gathered in the same pass.  The rows of one column group are spread
// over the row groups.  tile_path: all of them measure against ONE pivot, the output of row 0, which every row
// group computes for itself (bit-identical: same tile, same table, same gradient bits); the squares then add up
// lane by lane and only the plain sums need merging per column: across the row groups that share a wavefront by
// shuffles, across wavefronts through one LDS slot each, summed in fixed order (tile_finish).  tile_path_deep:
// every row group measures against its own first output and the merge brings the sums to row group 0's pivot
// exactly (tile_finish_own).
// ---------------------------------------------------------------------------------------
// The value of the lane whose number differs in bit 0 (CTRL 0xB1: quad order 1,0,3,2) or bit 1 (0x4E: 2,3,0,1),
// moved inside the vector unit (no LDS round trip).  All four lanes of a quad must be active.
template <int CTRL>
__device__ __forceinline__ double lane_xor_quad(double v) {
    const long long bits = __double_as_longlong(v);
    const int lo = __builtin_amdgcn_update_dpp(0, (int)(bits & 0xFFFFFFFFll), CTRL, 0xF, 0xF, false);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(bits >> 32), CTRL, 0xF, 0xF, false);
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}

// The large workgroups are alone on their compute unit: 512 lanes with up to 256 registers per lane (8
// wavefronts x 8 rows cover n = 64 at once), or 1024 lanes with up to 128 (16 x 4).  The small one, which serves
// short rows (launches bound by latency, several workgroups per CU) and shares the 3-slot kernel with the ring
// walk there, stays frugal.
template <int T> struct TileShape {
    static constexpr int RB = T > 512 ? 4 : T > 256 ? 8 : 2;   // rows per lane and batch
    static constexpr int SB = T == 512 ? 3 : 2;   // rows whose slot chains advance together (two slots per trip each);
                                                 // more rows at once cost registers and ran slower (4: -1 to -6 %)
};

// Per-lane state of the tiled path that does not change from tile to tile.
template <int VEC>
struct TileCtx {
    const TileSlot* tab;
    int n, deg, lpr, lane, rg, nrg;
    int rows_each, rows_more;   // n = rows_each * nrg + rows_more: row group q has rows_each (+ 1 if q < rows_more) rows
    int tlane;   // the lane's column inside the tile (lane, or the last valid one for a lane beyond the ragged end)
    float neg_lr;
};

// Running sums of the distance for one lane and one tile.
template <int VEC>
struct TileStats {
    double piv[VEC], a[VEC], sq;
    float pivf[VEC];   // the pivot as the fp32 output it is (row groups with a pivot of their own keep it in this form)
    __device__ __forceinline__ void reset() {
        sq = 0.0;
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            piv[k] = a[k] = 0.0;
            pivf[k] = 0.0f;
        }
    }
};

// Rows rg + (b RB + u) nrg, u < RB, of the tile in `cur`: mix, subtract the gradient, store, gather.  With CD and
// `with_pivot` the list starts with one more item, row 0 of the lane's columns with its gradient g0: its output is
// the pivot the distance sums are taken against (computed, not stored; it rides along with the first rows so that
// its chain of LDS reads costs no latency of its own).
//
// CLAMP: nothing here is conditional except the arithmetic of the distance.  A lane without a row (or without a
// column group: the caller then points it at the last valid one) repeats the work of the lane that owns the
// clamped row and column and stores the same bits to the same place.  This is what lets loads that were issued
// early stay in flight: the compiler counts outstanding memory operations to wait for exactly the ones it
// needs, and a load or store that may or may not have been issued makes that count unknown, upon which it
// waits for all of them.
//
// OWNPIV (with CLAMP and CD): no extra item; the lane's first own output is its pivot, and the merge at the end
// of the tile brings the row groups' sums to one common pivot (tile_finish_own).
//
// `feed(j0)` runs in front of every group of SB rows and `refill(j0)` behind it (its gradients have been used,
// its outputs stored): the caller's places for the loads of the next tiles, so that they enter the memory
// pipeline a few at a time between the rows' arithmetic instead of in one burst.
struct NoFeed {
    __device__ __forceinline__ void operator()(int) const {}
};
template <int VEC, bool CD, int RB, int SB, bool CLAMP, bool OWNPIV, typename GR, typename FEED = NoFeed,
          typename REFILL = NoFeed>
__device__ __forceinline__ void tile_rows(const TileCtx<VEC>& c, const typename Cols<VEC>::T* cur, int b, const GR (&g)[RB],
                                          GR g0, bool with_pivot, bool active, float* out_col, int64_t ldo,
                                          TileStats<VEC>& st, const FEED& feed = FEED{}, const REFILL& refill = REFILL{}) {
    typedef typename Cols<VEC>::T V;
    constexpr int P = (CD && !OWNPIV) ? 1 : 0, ITEMS = RB + P;
#pragma unroll
    for (int j0 = 0; j0 < ITEMS; j0 += SB) {
        feed(j0);
        const TileSlot* tp[SB];
        bool ok[SB];
        int row[SB];
        V acc[SB];
#pragma unroll
        for (int i = 0; i < SB; ++i) {
            const int j = j0 + i;
            const bool piv = P && j == 0;
            row[i] = piv ? 0 : c.rg + (b * RB + (j - P)) * c.nrg;
            ok[i] = j < ITEMS && active && (piv ? with_pivot : row[i] < c.n);
            if (CLAMP) {
                if (row[i] > c.n - 1) row[i] = c.n - 1;
                tp[i] = c.tab + row[i] * c.deg;
            } else {
                tp[i] = c.tab + (ok[i] ? row[i] : 0) * c.deg;     // an idle item follows row 0 and stores nothing
            }
        }
        {
            TileSlot e[SB];
#pragma unroll
            for (int i = 0; i < SB; ++i) e[i] = tp[i][0];
#pragma unroll
            for (int i = 0; i < SB; ++i) acc[i] = cur[e[i].off + c.tlane] * e[i].w;
        }
        // two slots per trip; where four wavefronts share a SIMD they hide each other's round trips and the
        // registers are worth more than a longer unrolled trip
        auto trip = [&](int s) {
            TileSlot e0[SB], e1[SB];
            V x0[SB], x1[SB];
#pragma unroll
            for (int i = 0; i < SB; ++i) {
                e0[i] = tp[i][s];
                e1[i] = tp[i][s + 1];
            }
#pragma unroll
            for (int i = 0; i < SB; ++i) {
                x0[i] = cur[e0[i].off + c.tlane];
                x1[i] = cur[e1[i].off + c.tlane];
            }
#pragma unroll
            for (int i = 0; i < SB; ++i) {
                acc[i] = vfma(e0[i].w, x0[i], acc[i]);
                acc[i] = vfma(e1[i].w, x1[i], acc[i]);
            }
        };
        int s = 1;
        if (RB == 4 || (CLAMP && CD && sizeof(GR) > 8)) {
#pragma unroll 1
            for (; s + 1 < c.deg; s += 2) trip(s);
        } else {
            for (; s + 1 < c.deg; s += 2) trip(s);
        }
        if (s < c.deg) {
            TileSlot e[SB];
#pragma unroll
            for (int i = 0; i < SB; ++i) e[i] = tp[i][s];
#pragma unroll
            for (int i = 0; i < SB; ++i) acc[i] = vfma(e[i].w, cur[e[i].off + c.tlane], acc[i]);
        }
#pragma unroll
        for (int i = 0; i < SB; ++i) {
            const int j = j0 + i;
            if (P && j == 0) {
                if (CLAMP || ok[i]) pivot_of(vfma(c.neg_lr, widen_g(g0), acc[i]), st.piv);
            } else if (j < ITEMS) {
                if (CLAMP || ok[i]) {
                    const V out = vfma(c.neg_lr, widen_g(g[j - P < 0 ? 0 : j - P]), acc[i]);
                    st_x(out_col + (int64_t)row[i] * ldo, out);
                    if (CD && OWNPIV && j == 0) floats_of(out, st.pivf);
                    if (CD && ok[i]) {
                        double o[VEC];
                        pivot_of(out, o);      // widen
#pragma unroll
                        for (int k = 0; k < VEC; ++k) {
                            const double df = o[k] - (OWNPIV ? (double)st.pivf[k] : st.piv[k]);
                            st.a[k] += df;
                            st.sq = fma(df, df, st.sq);
                        }
                    }
                }
            }
        }
        refill(j0);
    }
}

// Merge of the column sums at the end of a tile (CD only).  Contains the tile's barrier: when it returns every
// read of the current buffer and every write of the other one is done.
template <int VEC, bool CD, int T>
__device__ __forceinline__ void tile_finish(const TileCtx<VEC>& c, double* comb, bool active, TileStats<VEC>& st,
                                            double inv_n, double& total) {
    if (CD) {
        // first across the row groups that share a wavefront (lanes lpr apart hold the same columns; the exchange
        // is symmetric, so all of them end with the same bits), then one slot per wavefront in LDS
        // (rows wider than a wavefront: a row group is whole wavefronts, one slot per row group)
        const int wl = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            if (c.lpr <= 64) {
                for (int off = c.lpr; off < 64; off <<= 1) st.a[k] += __shfl_xor(st.a[k], off, 64);
                if (wl < c.lpr) comb[(size_t)(wave * c.lpr + wl) * VEC + k] = st.a[k];
            } else {
                comb[(size_t)(c.rg * c.lpr + c.lane) * VEC + k] = st.a[k];
            }
        }
        total += st.sq;
    }
    lds_barrier();
    if (CD) {
        if (active && c.rg == 0) {
            const int slots = c.lpr <= 64 ? T / 64 : c.nrg;
#pragma unroll
            for (int k = 0; k < VEC; ++k) {
                double at = 0.0;
                for (int q = 0; q < slots; ++q) at += comb[(size_t)(q * c.lpr + c.lane) * VEC + k];
                total -= at * at * inv_n;
            }
        }
        lds_barrier();                                 // the merge slots are free again
    }
}

// The same for row groups that each measured against their own pivot p_q (their first output): with P = p_0,
// D_q = p_q - P and m_q rows in group q,
//     sum_i (o_i - P)   = sum_q (a_q + m_q D_q)
//     sum_i (o_i - P)^2 = sum_q (sq_q + 2 D_q a_q + m_q D_q^2)
// exactly; in fp64 the corrections are of the size of the sums themselves (every pivot is one of the outputs).
// If all outputs of a column are equal every D_q is 0 and the distance comes out exactly 0.  One slot per row
// group and column: a double for the sum and a float for the pivot.
template <int VEC, int T>
__device__ __forceinline__ void tile_finish_own(const TileCtx<VEC>& c, double* comb, float* combp, int live_cols,
                                                TileStats<VEC>& st, double inv_n, double& total) {
    // live_cols: the lanes of the tile that own a column group (all of them except in the ragged last tile)
    // slot of row group q, column k of lane l: (q VEC + k) lpr + l, so that the lanes of a wavefront write
    // neighbouring words (no bank conflicts); the merge below numbers the tile's columns in the same order
    const int cols = c.lpr * VEC;
    const size_t mine = (size_t)c.rg * cols + c.lane;
#pragma unroll
    for (int k = 0; k < VEC; ++k) {
        comb[mine + k * c.lpr] = st.a[k];
        combp[mine + k * c.lpr] = st.pivf[k];
    }
    total += st.sq;
    lds_barrier();
    // The tile has lpr * VEC columns and nrg partial sums per column.  Where there are more lanes than columns
    // (1 KB row segments: four times as many) `parts` adjacent lanes share a column, each takes nrg / parts of its
    // row groups and a symmetric exchange adds the shares up, the same bits in every lane of the column.  (Left
    // to one lane per column the loop over the row groups is a chain of LDS round trips on a quarter of the
    // wavefronts while the others wait at the barrier below.)
    // Nothing here branches on data: every lane reads VEC slots (clamped to slot 0 where it has fewer), all
    // reads are issued before the first is used, and a slot that does not count enters with weight 0.
    const int parts = c.nrg >= VEC ? c.nrg / VEC : 1;        // a power of two; the lanes of a column sit side by side in one wavefront
    const int each = c.nrg / parts;                          // row groups per lane: min(nrg, VEC)
    for (int idx = threadIdx.x; idx < cols * parts; idx += T) {
        const int col = idx / parts, part = idx % parts;
        const bool live = (col & (c.lpr - 1)) < live_cols;   // a column of a lane beyond the ragged end counts for nothing
        double aq[VEC], md[VEC];
        float pq[VEC];
        const float p0f = combp[col];                        // row group 0 owns row 0: its pivot is the common one
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            const bool on = k < each;                        // uniform
            const int q = on ? part * each + k : 0;
            const size_t at_q = (size_t)q * cols + col;
            aq[k] = comb[at_q];
            pq[k] = combp[at_q];
            md[k] = on ? (double)(c.rows_each + (q < c.rows_more ? 1 : 0)) : -1.0;   // rows q, q + nrg, ... below n
        }
        const double p0 = (double)p0f;
        double at = 0.0, corr = 0.0;
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            const double dq = (double)pq[k] - p0;
            const double tq = fma(md[k], dq, aq[k]);         // a row group without rows has a = 0 and weight 0: no share
            const double cq = dq * (tq + aq[k]);
            at += md[k] >= 0.0 ? tq : 0.0;
            corr += md[k] >= 0.0 ? cq : 0.0;
        }
        if (parts > 1) {
            at += lane_xor_quad<0xB1>(at);                   // lanes 1 apart
            corr += lane_xor_quad<0xB1>(corr);
        }
        if (parts > 2) {
            at += lane_xor_quad<0x4E>(at);                   // lanes 2 apart
            corr += lane_xor_quad<0x4E>(corr);
        }
        for (int off = 4; off < parts; off <<= 1) {
            at += __shfl_xor(at, off, 64);
            corr += __shfl_xor(corr, off, 64);
        }
        if (part == 0 && live) total += corr - at * at * inv_n;
    }
    lds_barrier();                                     // the merge slots are free again
}

template <int VEC, typename GT, bool CD, int T>
__device__ double tile_path(const float* X, float* Xout, const GT* __restrict__ G, const TileSlot* tab, char* tiles,
                            int n, int deg, Pitch ld, int64_t ncg, float neg_lr, int lpr, double inv_n) {
    typedef typename Cols<VEC>::T V;
    typedef typename RawG<GT, VEC>::T GR;
    const Cols<VEC> tag{};
    constexpr int RB = TileShape<T>::RB, SB = TileShape<T>::SB;
    TileCtx<VEC> c;
    c.tab = tab;
    c.n = n;
    c.deg = deg;
    c.lpr = lpr;
    c.lane = c.tlane = threadIdx.x % lpr;
    c.rg = threadIdx.x / lpr;
    c.nrg = T / lpr;
    c.rows_each = n / c.nrg;
    c.rows_more = n % c.nrg;
    c.neg_lr = neg_lr;
    const int lane = c.lane, rg = c.rg, nrg = c.nrg;
    const int nb = ((n + nrg - 1) / nrg + RB - 1) / RB;      // batches per tile: the same for every lane
    const size_t tile_bytes = (((size_t)n * lpr * sizeof(V)) + 15) & ~(size_t)15;
    V* cur = reinterpret_cast<V*>(tiles);
    V* nxt = reinterpret_cast<V*>(tiles + tile_bytes);
    double* comb = reinterpret_cast<double*>(tiles + 2 * tile_bytes);   // [T / 64][lpr][VEC], CD only
    const int64_t ntiles = (ncg + lpr - 1) / lpr;
    const int64_t step = gridDim.x;
    int64_t t = plan::die_contiguous_slot(blockIdx.x, gridDim.x, kXcds);   // the first of tiles t, t + step, ...
    if (t >= ntiles) return 0.0;                             // uniform: the whole workgroup has nothing to do
    double total = 0.0;
    TileStats<VEC> st;

    // Loads of one batch of one tile: X rows into xs, gradient rows into g (nothing beyond the last tile or the
    // ragged end of the rows).
    auto col_of = [&](int64_t tile) { return (tile * lpr + lane) * VEC; };
    auto live = [&](int64_t tile) { return tile < ntiles && tile * lpr + lane < ncg; };
    // `q` is the lane's row group: rg, or the same number held in a scalar register where it is known to be
    // uniform over the wavefront (row offsets and table addresses then cost no vector registers).
    auto load_x = [&](int q, int64_t tile, int b, V (&xs)[RB]) {
        const bool on = live(tile);
        const int64_t col = col_of(tile);
#pragma unroll
        for (int u = 0; u < RB; ++u) {
            const int r = q + (b * RB + u) * nrg;
            if (on && r < n) xs[u] = ld_x(X + (int64_t)r * ld.x + col, tag);
        }
    };
    auto load_g = [&](int q, int64_t tile, int b, GR (&g)[RB]) {
        const bool on = live(tile);
        const int64_t col = col_of(tile);
#pragma unroll
        for (int u = 0; u < RB; ++u) {
            const int r = q + (b * RB + u) * nrg;
            if (on && r < n) g[u] = ld_g_raw(G + (int64_t)r * ld.g + col, tag);
        }
    };
    auto stash = [&](int q, int64_t tile, int b, V* buf, const V (&xs)[RB]) {
        const bool on = live(tile);
#pragma unroll
        for (int u = 0; u < RB; ++u) {
            const int r = q + (b * RB + u) * nrg;
            if (on && r < n) buf[r * lpr + lane] = xs[u];
        }
    };

    // First tile: straight into `cur`.
    for (int b = 0; b < nb; ++b) {
        V xs[RB];
        load_x(rg, t, b, xs);
        stash(rg, t, b, cur, xs);
    }

    // Several batches per tile: batch b of the next tile travels while batch b of this one is computed, the
    // gradients one batch ahead.
    GR gcur[RB], g0 = {};
    load_g(rg, t, 0, gcur);
    if (CD && live(t)) g0 = ld_g_raw(G + col_of(t), tag);
    lds_barrier();
    for (;;) {
        const int64_t tn = t + step;
        const bool active = live(t);
        GR g0n = {};
        if (CD) st.reset();
        for (int b = 0; b < nb; ++b) {
            V xs[RB];
            GR gn[RB];
            load_x(rg, tn, b, xs);
            if (b + 1 < nb) {
                load_g(rg, t, b + 1, gn);
            } else {
                load_g(rg, tn, 0, gn);
                if (CD && live(tn)) g0n = ld_g_raw(G + col_of(tn), tag);
            }
            tile_rows<VEC, CD, RB, SB, false, false>(c, cur, b, gcur, g0, b == 0, active, Xout + col_of(t), ld.o, st);
            stash(rg, tn, b, nxt, xs);
#pragma unroll
            for (int u = 0; u < RB; ++u) gcur[u] = gn[u];
        }
        g0 = g0n;
        tile_finish<VEC, CD, T>(c, comb, active, st, inv_n, total);
        if (tn >= ntiles) break;
        V* sw = cur;
        cur = nxt;
        nxt = sw;
        t = tn;
    }
    return total;
}

// The tiled path of the large workgroup (1024 lanes without the distance, 512 with it; alone on its compute
// unit) for tables whose tile is ONE batch of rows: at most TileShape<T>::RB rows per lane (n = 64 with 1 KB row
// segments, fewer learners with wider ones, up to 256 learners with narrower ones).  The launcher picks the
// shape (plan::tile_plan, one-batch form).
// With `comb_in_tile` the merge slots of the distance are the tile buffer that has just been consumed.
//
// UQ: a row group is whole wavefronts (lpr >= 64), so its number is the same in every lane of a wavefront and is
// kept in a scalar register: row offsets and table addresses then cost no vector registers.  Narrower rows
// (n > 64 at 16 B per lane: two or four row groups share a wavefront) keep it per lane.
template <int VEC, typename GT, bool CD, int T, bool UQ>
__device__ double tile_path_deep(const float* X, float* Xout, const GT* __restrict__ G, const TileSlot* tab, char* tiles,
                                 int n, int deg, Pitch ld, int64_t ncg, float neg_lr, int lpr, double inv_n,
                                 bool comb_in_tile) {
    typedef typename Cols<VEC>::T V;
    typedef typename RawG<GT, VEC>::T GR;
    const Cols<VEC> tag{};
    constexpr int RB = TileShape<T>::RB, SB = TileShape<T>::SB;
    TileCtx<VEC> c;
    c.tab = tab;
    c.n = n;
    c.deg = deg;
    c.lpr = lpr;
    c.lane = c.tlane = threadIdx.x % lpr;
    c.nrg = T / lpr;
    c.rows_each = n / c.nrg;
    c.rows_more = n % c.nrg;
    c.neg_lr = neg_lr;
    const int lane = c.lane, nrg = c.nrg;
    const size_t tile_bytes = (((size_t)n * lpr * sizeof(V)) + 15) & ~(size_t)15;
    V* cur = reinterpret_cast<V*>(tiles);
    V* nxt = reinterpret_cast<V*>(tiles + tile_bytes);
    double* comb = reinterpret_cast<double*>(tiles + 2 * tile_bytes);   // [nrg][lpr][VEC] sums, then as many float pivots
    const int64_t ntiles = (ncg + lpr - 1) / lpr;
    const int64_t step = gridDim.x;
    int64_t t = plan::die_contiguous_slot(blockIdx.x, gridDim.x, kXcds);   // the first of tiles t, t + step, ...
    if (t >= ntiles) return 0.0;                             // uniform: the whole workgroup has nothing to do
    double total = 0.0;
    TileStats<VEC> st;
    // A tile is one batch of whole-wavefront rows (n <= 64 with 1 KB row segments, fewer learners with wider
    // ones).  A lane keeps ONE register per row for X and one for the gradients, each reloaded the moment
    // its value has been used, so every load has a whole tile's time to arrive:
    //   in front of a group of rows: X of tile t + step (loaded one tile ago) goes into the other LDS buffer,
    //       which nobody reads during this tile, and the same registers are loaded with tile t + 2 step;
    //   behind it: its gradients (tile t) have been used, the registers are loaded with tile t + step.
    // The loads thus enter the memory pipeline a few at a time between the arithmetic.  (Issued in one burst
    // at the start of the tile they hold the wavefront at the issue stage until the pipeline has taken them,
    // and the arithmetic starts only then: the two times add up instead of overlapping.)  Every load and
    // store here is unconditional (see tile_rows): rows, columns and tiles beyond the end are clamped to the
    // last valid one.
    const int q = UQ ? __builtin_amdgcn_readfirstlane((int)(threadIdx.x / lpr)) : (int)(threadIdx.x / lpr);
    c.rg = q;
    const int last_row = n - 1;
    auto cge_of = [&](int64_t tile) {                       // the lane's column group in `tile`, clamped
        const int64_t cg = tile * lpr + lane;
        return cg < ncg ? cg : ncg - 1;
    };
    auto row_of = [&](int u) {
        const int r = q + u * nrg;
        return r < last_row ? r : last_row;
    };
    V x[RB];
    GR g[RB];
    if (t * lpr + lane < ncg) {                              // the first tile: straight into `cur`
#pragma unroll
        for (int u = 0; u < RB; ++u) {
            const int r = q + u * nrg;
            if (r < n) cur[r * lpr + lane] = ld_x(X + (int64_t)r * ld.x + (t * lpr + lane) * VEC, tag);
        }
    }
    {
        const int64_t colx = cge_of(t + step) * VEC, colg = cge_of(t) * VEC;
#pragma unroll
        for (int u = 0; u < RB; ++u) {
            x[u] = ld_x(X + (int64_t)row_of(u) * ld.x + colx, tag);
            g[u] = ld_g_raw(G + (int64_t)row_of(u) * ld.g + colg, tag);
        }
    }
    lds_barrier();
    // One tile.  It runs once in front of the loop and then inside it: the waits for the loads of the tile before
    // are counted per place in the program, and a place that both the start and the loop reach waits for the
    // smaller count, the start's, where fewer operations have been issued since.
    auto one_tile = [&]() __attribute__((always_inline)) {
        const int64_t colx = cge_of(t + 2 * step) * VEC, colg = cge_of(t + step) * VEC;
        // where tile t + step goes in the other buffer: the lane's own slot, the last valid lane's at the ragged
        // end (the same value twice), and beyond the last tile anywhere (nobody will read it) - never a branch
        const int lane_to = (int)(cge_of(t + step) - (t + step) * lpr);
        const int lane_n = lane_to >= 0 ? lane_to : lane;
        auto feed = [&](int j0) {
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < SB; ++i) {
                const int u = j0 + i;
                if (u < RB) {
                    const int r = row_of(u);
                    nxt[r * lpr + lane_n] = x[u];
                    x[u] = ld_x(X + (int64_t)r * ld.x + colx, tag);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        };
        auto refill = [&](int j0) {
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < SB; ++i) {
                const int u = j0 + i;
                if (u < RB) g[u] = ld_g_raw(G + (int64_t)row_of(u) * ld.g + colg, tag);
            }
            __builtin_amdgcn_sched_barrier(0);
        };
        const int64_t cge = cge_of(t);
        const bool active = t * lpr + lane < ncg;
        c.tlane = (int)(cge - t * lpr);
        if (CD) st.reset();
        tile_rows<VEC, CD, RB, SB, true, true>(c, cur, 0, g, GR{}, false, active, Xout + cge * VEC, ld.o, st, feed, refill);
        if (CD) {
            const int64_t left = ncg - t * lpr;                       // column groups of this tile (uniform)
            double* sums = comb;
            if (comb_in_tile) {                                       // uniform
                lds_barrier();                                        // every row of `cur` has been read
                sums = reinterpret_cast<double*>(cur);
            }
            tile_finish_own<VEC, T>(c, sums, reinterpret_cast<float*>(sums + (size_t)nrg * lpr * VEC),
                                    (int)(left < lpr ? left : lpr), st, inv_n, total);
        } else {
            lds_barrier();
        }
        V* sw = cur;
        cur = nxt;
        nxt = sw;
        t += step;
    };
    one_tile();
    while (t < ntiles) one_tile();
    return total;
}

// CD = also reduce the consensus distance of the outputs into partials[blockIdx.x].
// The column groups are split evenly over the persistent grid (plan::sweep_plan): every workgroup makes the
// same number of sweeps, lanes beyond the chunk idle.
struct Sweeps {
    int64_t count, chunk;
    // first column group of this workgroup in sweep sw
    __device__ __forceinline__ int64_t base(int64_t sw) const {
        return (sw * gridDim.x + plan::die_contiguous_slot(blockIdx.x, gridDim.x, kXcds)) * chunk;
    }
};
// Computed by the launcher (the device would pay two 64-bit divisions per lane for it).
inline Sweeps make_sweeps(int64_t ncg, int grid, int threads) {
    const plan::SweepPlan p = plan::sweep_plan(ncg, grid, threads);
    return Sweeps{p.count, p.chunk};
}

// T = workgroup size: kRingThreads on long rows, kThreads (four workgroups per CU) where the row is too
// short to give every CU a large workgroup's worth of column groups twice over.
// TILES: the kernel also carries the tiled path for tables that are not one ring (short rows: one launch does
// whatever the table needs).  Without it (long rows) such a table is left to the tiled kernel, which the launcher
// enqueues right behind this one and which classifies the table the same way; this kernel then writes nothing.
template <int VEC, typename GT, bool CD, int T, bool TILES>
__global__ __launch_bounds__(T, 3) void mix_step_kernel(const float* X, float* Xout, const GT* __restrict__ G,
                                                     const int32_t* __restrict__ nbr, const float* __restrict__ w,
                                                     int n, int64_t d, Pitch ld, float neg_lr, int lpr,
                                                     Sweeps sweeps, double* __restrict__ partials) {
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    __shared__ double lds_waves[T / 64];
    const Lds l = carve(lds_raw, n);
    const int kind = stage_table<T>(nbr, w, n, l);
    if (kind == kTableBad) {
        if (blockIdx.x == 0 && threadIdx.x == 0) atomicOr(&g_status_word, 1);
        if (CD && threadIdx.x == 0) partials[blockIdx.x] = __builtin_nan("");
        return;
    }
    const int64_t ncg = d / VEC;  // the launcher picks VEC = 1 unless 4 divides d
    const double inv_n = 1.0 / (double)n;
    double total = 0.0;
    if (kind == kTableRing) {
        for (int64_t sw = 0; sw < sweeps.count; ++sw) {
            const int64_t base = sweeps.base(sw), cg = base + threadIdx.x;
            if (base >= ncg) break;                              // nothing left for this workgroup (uniform)
            const int64_t end = base + sweeps.chunk < ncg ? base + sweeps.chunk : ncg;   // uniform
            const bool act = cg < end;
            const int64_t col = (act ? cg : 0) * VEC;            // idle lanes shadow column group 0
            ColStats<VEC> stats;
            if (CD) stats.reset();
            ring_walk<VEC, GT, CD>(X + col, Xout + col, G + col, l.ring, n, ld, neg_lr, stats, act);
            if (CD && act) total += stats.result(inv_n);
        }
    } else if (TILES) {
        // The slot table in the tiled path's form, then the tile buffers (the ranking arrays that shared this
        // space are dead: stage_table ended with a barrier on every path that comes here).
        TileSlot* tab = reinterpret_cast<TileSlot*>(l.scratch);
        for (int e = threadIdx.x; e < 3 * n; e += T) tab[e] = TileSlot{(uint32_t)(l.nbr[e] * lpr), l.w[e]};
        __syncthreads();
        const size_t tab_bytes = (((size_t)n * 3 * sizeof(TileSlot)) + 15) & ~(size_t)15;
        total = tile_path<VEC, GT, CD, T>(X, Xout, G, tab, l.scratch + tab_bytes, n, 3, ld, ncg, neg_lr, lpr, inv_n);
    }
    if (CD) {
        const double bs = block_sum<T>(total, lds_waves);
        if (threadIdx.x == 0) partials[blockIdx.x] = bs;
    }
}

// Any table with `deg` slots per row (sparse doubly stochastic matrices beyond the ring: more neighbours, lazy
// walks, products of several mixing rounds, and 3-slot tables that are not one ring).  Always the tiled path.
// LDS: TileSlot tab[deg n] | two tile buffers | merge slots (plan::tile_plan).
//
// skip_rings (3-slot tables only): the launcher enqueues this kernel behind the ring-walk kernel because only
// the device can tell which of the two a table needs; both classify it with the same code, and the one it does
// not belong to writes nothing (and contributes 0 to the distance).
//
// DEEP: 0 = several batches per tile (tile_path); 1, 2 = the large workgroup's one-batch form (tile_path_deep)
// with whole-wavefront rows (1) or narrower ones (2); the launcher has planned lpr for it.
template <int VEC, typename GT, bool CD, int T, int DEEP>
__global__ __launch_bounds__(T) void mix_deg_kernel(const float* X, float* Xout, const GT* __restrict__ G,
                                                    const int32_t* __restrict__ nbr, const float* __restrict__ w,
                                                    int deg, int n, int64_t d, Pitch ld, float neg_lr, int lpr,
                                                    int skip_rings, int comb_in_tile, double* __restrict__ partials) {
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    __shared__ double lds_waves[T / 64];
    const size_t tab_bytes = (((size_t)n * deg * sizeof(TileSlot)) + 15) & ~(size_t)15;
    if (skip_rings) {
        // the tile area is free until the first tile is loaded: classify there
        const int kind = stage_table<T>(nbr, w, n, carve(lds_raw + tab_bytes, n));
        if (kind != kTableGeneral) {
            // one ring: the other kernel's work.  Invalid: it has raised the flag; the distance is NaN.
            if (CD && threadIdx.x == 0) partials[blockIdx.x] = kind == kTableRing ? 0.0 : __builtin_nan("");
            return;
        }
    }
    TileSlot* tab = reinterpret_cast<TileSlot*>(lds_raw);
    int ok = 1;
    for (int e = threadIdx.x; e < deg * n; e += T) {
        const int v = nbr[e];
        tab[e] = TileSlot{(uint32_t)(v * lpr), w[e]};
        ok &= (unsigned)v < (unsigned)n;
    }
    if (!__syncthreads_and(ok)) {
        if (blockIdx.x == 0 && threadIdx.x == 0) atomicOr(&g_status_word, 1);
        if (CD && threadIdx.x == 0) partials[blockIdx.x] = __builtin_nan("");
        return;
    }
    double total;
    if (DEEP)
        total = tile_path_deep<VEC, GT, CD, T, DEEP == 1>(X, Xout, G, tab, lds_raw + tab_bytes, n, deg, ld, d / VEC, neg_lr,
                                                          lpr, 1.0 / (double)n, comb_in_tile != 0);
    else
        total = tile_path<VEC, GT, CD, T>(X, Xout, G, tab, lds_raw + tab_bytes, n, deg, ld, d / VEC, neg_lr, lpr,
                                          1.0 / (double)n);
    if (CD) {
        const double bs = block_sum<T>(total, lds_waves);
        if (threadIdx.x == 0) partials[blockIdx.x] = bs;
    }
}

// ---------------------------------------------------------------------------------------
// Global averaging, T_u = (1/n) 1 1^T (Sec. 2: S-PSGD; Sec. 4, Eq. 13: D1D-PSGD's allreduce / L):
//     X_out[i,:] = mean_j X[j,:] - lr * G[i,:].
// A lane owns a column group: first sweep sums its n rows (fp64, so the mean carries one
// fp32 rounding whatever n is), second sweep reads G and writes the n outputs.  All of the
// lane's X loads precede its first store, so X_out may alias X.  Same bytes as the ring step.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ void add_to(double* s, float x) { s[0] += (double)x; }
__device__ __forceinline__ void add_to(double* s, f32x4 x) {
#pragma unroll
    for (int k = 0; k < 4; ++k) s[k] += (double)x[k];
}
__device__ __forceinline__ float mean_of(const double* s, double inv_n, Cols<1>) { return (float)(s[0] * inv_n); }
__device__ __forceinline__ f32x4 mean_of(const double* s, double inv_n, Cols<4>) {
    return (f32x4){(float)(s[0] * inv_n), (float)(s[1] * inv_n), (float)(s[2] * inv_n), (float)(s[3] * inv_n)};
}

// T = workgroup size, chosen as for the ring step: on long rows a large workgroup whose wavefronts
// sweep the rows in lockstep (a barrier per batch), so each row sees one long contiguous burst.
template <int VEC, typename GT, bool CD, int T>
__global__ __launch_bounds__(T) void mix_full_kernel(const float* X, float* Xout, const GT* __restrict__ G, int n,
                                                     int64_t d, Pitch ld, float neg_lr, Sweeps sweeps,
                                                     double* __restrict__ partials) {
    typedef typename Cols<VEC>::T V;
    const Cols<VEC> tag{};
    __shared__ double lds_waves[T / 64];
    const int64_t ncg = d / VEC;
    const double inv_n = 1.0 / (double)n;
    double total = 0.0;
    for (int64_t sw = 0; sw < sweeps.count; ++sw) {
        const int64_t base = sweeps.base(sw), cg = base + threadIdx.x;
        if (base >= ncg) break;                                  // nothing left for this workgroup (uniform)
        const int64_t end = base + sweeps.chunk < ncg ? base + sweeps.chunk : ncg;   // uniform
        const bool act = cg < end;                               // an idle lane shadows column group 0 and stores nothing
        const int64_t col = (act ? cg : 0) * VEC;
        const float* xc = X + col;
        const GT* gc = G + col;
        float* oc = Xout + col;
        double sum[VEC];
#pragma unroll
        for (int k = 0; k < VEC; ++k) sum[k] = 0.0;
        int r = 0;
        for (; r + kUnroll <= n; r += kUnroll) {
            lockstep_barrier();
            V xs[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) xs[u] = ld_x(xc + (int64_t)(r + u) * ld.x, tag);
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) add_to(sum, xs[u]);
        }
        for (; r < n; ++r) add_to(sum, ld_x(xc + (int64_t)r * ld.x, tag));
        const V mean = mean_of(sum, inv_n, tag);
        ColStats<VEC> stats;
        if (CD) stats.reset();
        r = 0;
        for (; r + kUnroll <= n; r += kUnroll) {
            lockstep_barrier();
            V gs[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) gs[u] = ld_g(gc + (int64_t)(r + u) * ld.g, tag);
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const V out = vfma(neg_lr, gs[u], mean);
                if (act) st_x(oc + (int64_t)(r + u) * ld.o, out);
                if (CD) stats.add(out);
            }
        }
        for (; r < n; ++r) {
            const V out = vfma(neg_lr, ld_g(gc + (int64_t)r * ld.g, tag), mean);
            if (act) st_x(oc + (int64_t)r * ld.o, out);
            if (CD) stats.add(out);
        }
        if (CD && act) total += stats.result(inv_n);
    }
    if (CD) {
        const double bs = block_sum<T>(total, lds_waves);
        if (threadIdx.x == 0) partials[blockIdx.x] = bs;
    }
}

// Consensus-distance kernels (the per-column arithmetic is defined above the ring walk).
template <int VEC>
__global__ __launch_bounds__(kThreads) void consensus_partial_kernel(const float* __restrict__ X, int n,
                                                                     int64_t d, int64_t ldx,
                                                                     double* __restrict__ partials) {
    typedef typename Cols<VEC>::T V;
    const Cols<VEC> tag{};
    __shared__ double lds4[4];
    const int64_t ncg = d / VEC;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    const double inv_n = 1.0 / (double)n;
    double total = 0.0;
    for (int64_t cg = (int64_t)blockIdx.x * kThreads + threadIdx.x; cg < ncg; cg += stride) {
        const float* xc = X + cg * VEC;
        double s[VEC], a[VEC], b[VEC];
        pivot_of(ld_x(xc, tag), s);
#pragma unroll
        for (int k = 0; k < VEC; ++k) a[k] = b[k] = 0.0;
        int r = 1;
        for (; r + kUnroll <= n; r += kUnroll) {
            V xs[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) xs[u] = ld_x(xc + (int64_t)(r + u) * ldx, tag);
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) acc_diff<VEC>(a, b, xs[u], s);
        }
        if (r < n) {
            V xs[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u)
                if (r + u < n) xs[u] = ld_x(xc + (int64_t)(r + u) * ldx, tag);
#pragma unroll
            for (int u = 0; u < kUnroll; ++u)
                if (r + u < n) acc_diff<VEC>(a, b, xs[u], s);
        }
#pragma unroll
        for (int k = 0; k < VEC; ++k) total += b[k] - a[k] * a[k] * inv_n;
    }
    const double bs = block_sum(total, lds4);
    if (threadIdx.x == 0) partials[blockIdx.x] = bs;
}

// The same distance for long rows, in the form of the step kernels: one large workgroup per compute unit whose
// wavefronts sweep the rows in lockstep batches, the column groups split evenly and die-contiguously over the
// persistent grid.  A lane owns one column group per sweep; a lane beyond the ragged end shadows column group 0
// and adds nothing.
template <int VEC, int T>
__global__ __launch_bounds__(T) void consensus_sweep_kernel(const float* __restrict__ X, int n, int64_t d, int64_t ldx,
                                                            Sweeps sweeps, double* __restrict__ partials) {
    typedef typename Cols<VEC>::T V;
    const Cols<VEC> tag{};
    __shared__ double lds_waves[T / 64];
    const int64_t ncg = d / VEC;
    const double inv_n = 1.0 / (double)n;
    double total = 0.0;
    for (int64_t sw = 0; sw < sweeps.count; ++sw) {
        const int64_t base = sweeps.base(sw), cg = base + threadIdx.x;
        if (base >= ncg) break;                                  // nothing left for this workgroup (uniform)
        const int64_t end = base + sweeps.chunk < ncg ? base + sweeps.chunk : ncg;   // uniform
        const bool act = cg < end;
        const float* xc = X + (act ? cg : 0) * VEC;
        double s[VEC], a[VEC], b[VEC];
        pivot_of(ld_x(xc, tag), s);
#pragma unroll
        for (int k = 0; k < VEC; ++k) a[k] = b[k] = 0.0;
        int r = 1;
        for (; r + kUnroll <= n; r += kUnroll) {
            lockstep_barrier();
            V xs[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) xs[u] = ld_x(xc + (int64_t)(r + u) * ldx, tag);
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) acc_diff<VEC>(a, b, xs[u], s);
        }
        for (; r < n; ++r) acc_diff<VEC>(a, b, ld_x(xc + (int64_t)r * ldx, tag), s);
        if (act) {
#pragma unroll
            for (int k = 0; k < VEC; ++k) total += b[k] - a[k] * a[k] * inv_n;
        }
    }
    const double bs = block_sum<T>(total, lds_waves);
    if (threadIdx.x == 0) partials[blockIdx.x] = bs;
}

// Fixed-order sum of the per-workgroup partials: lane t adds entries t, t+256, ... and the
// 256 lane sums go through the same shuffle/LDS tree, so the result does not depend on
// scheduling.
__global__ __launch_bounds__(kThreads) void consensus_final_kernel(const double* __restrict__ partials, int count,
                                                                   double* __restrict__ out) {
    __shared__ double lds4[4];
    double v = 0.0;
    for (int i = threadIdx.x; i < count; i += kThreads) v += partials[i];
    const double bs = block_sum(v, lds4);
    if (threadIdx.x == 0) out[0] = bs;
}

__global__ __launch_bounds__(kThreads) void synth_grad_kernel(const float* __restrict__ xp,
                                                              const float* __restrict__ noise, float* __restrict__ g,
                                                              int64_t count, float c, int vec4) {
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    const int64_t tid = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (vec4) {
        const int64_t groups = count / 4;
        for (int64_t i = tid; i < groups; i += stride) {
            const f32x4 x = ld_x(xp + 4 * i, Cols<4>{});
            const f32x4 z = ld_x(noise + 4 * i, Cols<4>{});
            st_x(g + 4 * i, vfma(c, x, z));
        }
        for (int64_t i = groups * 4 + tid; i < count; i += stride) g[i] = vfma(c, xp[i], noise[i]);
    } else {
        for (int64_t i = tid; i < count; i += stride) g[i] = vfma(c, xp[i], noise[i]);
    }
}

// Row-pitched form: a lane owns one column group and walks the n rows.
template <int VEC>
__global__ __launch_bounds__(kThreads) void synth_grad_rows_kernel(const float* __restrict__ xp, int64_t ldx,
                                                                   const float* __restrict__ noise, int64_t ldn,
                                                                   float* __restrict__ g, int64_t ldg, int n,
                                                                   int64_t d, float c) {
    const Cols<VEC> tag{};
    const int64_t ncg = d / VEC;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t cg = (int64_t)blockIdx.x * kThreads + threadIdx.x; cg < ncg; cg += stride) {
        const int64_t col = cg * VEC;
#pragma unroll 4
        for (int r = 0; r < n; ++r)
            st_x(g + (int64_t)r * ldg + col,
                 vfma(c, ld_x(xp + (int64_t)r * ldx + col, tag), ld_x(noise + (int64_t)r * ldn + col, tag)));
    }
}

// ---------------------------------------------------------------------------------------
// Reference streams (measurement support, not a step of the method): the memory traffic of the step with the
// mixing taken out, in the very form the step kernels give it -- a lane owns one 128-bit column group and
// walks the n rows, the workgroup's wavefronts sweep the rows in lockstep batches, the column groups are split
// evenly over a persistent grid.  KIND 0 only reads X and G, KIND 1 only writes X_out, KIND 2 is
// X_out = X + a * G (the step's 4 + 2 + 4 or 4 + 4 + 4 bytes per element, no neighbours).  The rate these
// reach is what the chip's memory system gives this access pattern; the step is measured against it.
// ---------------------------------------------------------------------------------------
enum { kRefRead = 0, kRefWrite = 1, kRefAxpy = 2 };

template <int KIND, typename GT, int T>
__global__ __launch_bounds__(T) void reference_stream_kernel(const float* X, float* Xout, const GT* __restrict__ G,
                                                             int n, int64_t d, Pitch ld, float a, Sweeps sweeps) {
    const Cols<4> tag{};
    const int64_t ncg = d / 4;
    f32x4 keep = splat4(0.0f);
    for (int64_t sw = 0; sw < sweeps.count; ++sw) {
        const int64_t base = sweeps.base(sw), cg = base + threadIdx.x;
        if (base >= ncg) break;                                  // nothing left for this workgroup (uniform)
        const int64_t end = base + sweeps.chunk < ncg ? base + sweeps.chunk : ncg;   // uniform
        const bool act = cg < end;                               // an idle lane shadows column group 0
        const int64_t col = (act ? cg : 0) * 4;
        const float* xc = X + col;
        const GT* gc = G + col;
        float* oc = Xout + col;
        int r = 0;
        for (; r + kUnroll <= n; r += kUnroll) {
            lockstep_barrier();
            f32x4 xs[kUnroll], gs[kUnroll];
            if (KIND != kRefWrite) {
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    xs[u] = ld_x(xc + (int64_t)(r + u) * ld.x, tag);
                    gs[u] = ld_g(gc + (int64_t)(r + u) * ld.g, tag);
                }
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                if (KIND == kRefRead) keep += xs[u] + gs[u];
                if (KIND == kRefWrite && act) st_x(oc + (int64_t)(r + u) * ld.o, splat4(a));
                if (KIND == kRefAxpy && act) st_x(oc + (int64_t)(r + u) * ld.o, vfma(a, gs[u], xs[u]));
            }
        }
        for (; r < n; ++r) {
            if (KIND == kRefRead) keep += ld_x(xc + (int64_t)r * ld.x, tag) + ld_g(gc + (int64_t)r * ld.g, tag);
            if (KIND == kRefWrite && act) st_x(oc + (int64_t)r * ld.o, splat4(a));
            if (KIND == kRefAxpy && act)
                st_x(oc + (int64_t)r * ld.o, vfma(a, ld_g(gc + (int64_t)r * ld.g, tag), ld_x(xc + (int64_t)r * ld.x, tag)));
        }
    }
    // The loads of the read-only stream must have an observer: a store that the data never triggers.
    if (KIND == kRefRead && __float_as_uint(keep.x + keep.y + keep.z + keep.w) == 0x7FC0BEEFu) Xout[0] = keep.x;
}

// ---------------------------------------------------------------------------------------
// Mixing table of one iteration, built on the device (Sec. 4: all learners derive the same
// ring from a shared seed, so the table is a function of (n, seed, step) only).  One
// workgroup: the SplitMix64 draws are counter-based (state of draw t = state0 + (t + 1) *
// increment), so all swap partners are computed in parallel; only the n - 1 swaps of the
// Durstenfeld shuffle are serial (one lane, in LDS).
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void build_mixing_kernel(int randomize, int n, uint64_t seed,
                                                                uint64_t* step_dev, uint64_t step_offset,
                                                                uint64_t advance, int32_t* __restrict__ nbr,
                                                                float* __restrict__ w) {
    __shared__ int sigma[PSGD_MAX_N];
    __shared__ int partner[PSGD_MAX_N];
    const int tid = threadIdx.x;
    const uint64_t base = step_dev ? *static_cast<volatile uint64_t*>(step_dev) : 0ull;
    const uint64_t step = base + step_offset;
    for (int p = tid; p < n; p += kThreads) sigma[p] = p;
    if (randomize) {
        constexpr uint64_t kWeyl = 0x9E3779B97F4A7C15ull;
        const uint64_t state0 = seed ^ ((step + 1ull) * kWeyl);
        for (int t = tid; t < n - 1; t += kThreads) {
            const int i = n - 1 - t;                      // draw t serves position i
            uint64_t z = state0 + (uint64_t)(t + 1) * kWeyl;
            z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
            z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
            z ^= z >> 31;
            partner[i] = (int)__umul64hi(z, (uint64_t)(i + 1));
        }
        __syncthreads();
        if (tid == 0) {
            for (int i = n - 1; i >= 1; --i) {
                const int j = partner[i], t = sigma[i];
                sigma[i] = sigma[j];
                sigma[j] = t;
            }
        }
    }
    __syncthreads();
    const float third = 1.0f / 3.0f;
    for (int p = tid; p < n; p += kThreads) {
        const int me = sigma[p];
        nbr[3 * me + 0] = me;
        nbr[3 * me + 1] = sigma[p == 0 ? n - 1 : p - 1];
        nbr[3 * me + 2] = sigma[p == n - 1 ? 0 : p + 1];
        w[3 * me + 0] = third;
        w[3 * me + 1] = third;
        w[3 * me + 2] = third;
    }
    if (tid == 0 && step_dev && advance) *step_dev = base + advance;
}

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
    static Entry cache[32];
    static int used = 0;
    std::lock_guard<std::mutex> lock(mu);
    for (int i = 0; i < used; ++i)
        if (cache[i].fn == fn && cache[i].lds == lds_bytes) return cache[i].occ;
    int q = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&q, fn, threads, lds_bytes) != hipSuccess || q < 1) q = 1;
    if (used < 32) cache[used++] = Entry{fn, lds_bytes, q};
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
int allow_lds(const void* fn, size_t lds_bytes) {
    if (lds_bytes <= 64 * 1024 - 256) return PSGD_OK;
    // the most this library ever asks for (the kernels' few hundred bytes of static LDS come on top of it)
    const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsCapLarge);
    if (e != hipSuccess) return hip_fail(e, "hipFuncSetAttribute(MaxDynamicSharedMemorySize)");
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
