// Device-side building blocks shared by the kernels of libpsgd (gfx950 / CDNA4): launch constants, column-group
// value types and their loads and stores, the LDS layout of the staged mixing table and its classification
// (one ring or not), workgroup sums, the running sums of the consensus distance (Sec. 3), and the even split of
// the column groups over a persistent grid.  Included by psgd_kernels.hip only (one translation unit).
#ifndef PSGD_DEVICE_H
#define PSGD_DEVICE_H

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>

#include "psgd.h"
#include "psgd_internal.h"

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

}  // namespace
}  // namespace psgd

#endif
