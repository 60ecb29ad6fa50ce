// The LDS-tiled form of the model-averaging step (Sec. 2, Eq. 2) for mixing tables that are not one ring, and its
// kernel mix_deg_kernel.  Included by psgd_kernels.hip only.
#ifndef PSGD_TILED_H
#define PSGD_TILED_H

#include "psgd_device.h"

namespace psgd {
namespace {

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

}  // namespace
}  // namespace psgd

#endif
