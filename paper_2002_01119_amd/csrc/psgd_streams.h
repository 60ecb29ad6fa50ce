// The streaming kernels beside the step: global averaging T_u (Sec. 2; Sec. 4, Eq. 13), the consensus distance
// (Sec. 3), the synthetic delayed gradient of the delay-by-one workload (Sec. 4, Eq. 13/14), the reference streams
// used for measurement, and the device-side builder of the ring tables (Sec. 3, Eq. 3 and Eq. 8).  Included by
// psgd_kernels.hip only.
#ifndef PSGD_STREAMS_H
#define PSGD_STREAMS_H

#include "psgd_device.h"

namespace psgd {
namespace {

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

}  // namespace
}  // namespace psgd

#endif
