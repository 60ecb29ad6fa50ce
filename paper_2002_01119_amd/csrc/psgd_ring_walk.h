// The ring walk, the register-only form of the model-averaging step (Sec. 2, Eq. 2) for the ring tables of
// Sec. 3 (Eq. 3, Eq. 8), and its kernel mix_step_kernel.  Included by psgd_kernels.hip only.
#ifndef PSGD_RING_WALK_H
#define PSGD_RING_WALK_H

#include "psgd_device.h"
#include "psgd_tiled.h"

namespace psgd {
namespace {

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


// CD = also reduce the consensus distance of the outputs into partials[blockIdx.x].
// The column groups are split evenly over the persistent grid (plan::sweep_plan): every workgroup makes the
// same number of sweeps, lanes beyond the chunk idle.
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

}  // namespace
}  // namespace psgd

#endif
