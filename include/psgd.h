/*
 * psgd.h - C boundary of the MI355X (gfx950) model-averaging library for decentralized
 * parallel SGD.
 *
 * One iteration of (A)D-PSGD updates all learners at once as
 *         W_{k+1} = W_k * T - alpha * g(Phi_k, xi_k)                       (Sec. 2, Eq. 2)
 * with W the d x L matrix of learner weights (one column per learner), T an L x L doubly
 * stochastic mixing matrix and g the matrix of per-learner gradients.  This library keeps
 * one learner per ROW: X = W^T is a row-major [n, d] fp32 array (n = L learners, d
 * parameters each) resident in one GPU's HBM, and the same update reads
 *         X_out[i, :] = sum_s w[i, s] * X[nbr[i, s], :]  -  lr * G[i, :].
 * Row i of the (nbr, w) table lists column i of T: the learners whose models feed
 * learner i, and with what weight.  For the ring topologies of Sec. 3 every row has three
 * slots in the order (self, left neighbour, right neighbour).
 *
 * Conventions for every call:
 *   - plain C types only; "host" / "device" is stated per pointer; the caller owns every
 *     buffer it passes and the library neither frees nor keeps it after the work that was
 *     enqueued by the call has run;
 *   - functions returning int give PSGD_OK (0) or a negative psgd_status; the text of the
 *     last failure on the calling thread is available from psgd_last_error();
 *   - nothing aborts or throws; the library uses the device that is current on the calling
 *     thread (hipSetDevice / torch.cuda.set_device);
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Calls that take
 *     a stream only enqueue work and return.
 */
#ifndef PSGD_H
#define PSGD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Mixing topologies (Sec. 3). */
enum {
    PSGD_TOPO_RING = 0,      /* fixed ring T_0: weights 1/3 on self and both cyclic neighbours (Eq. 3) */
    PSGD_TOPO_RAND_RING = 1, /* T_tau = P^T T_0 P with a fresh seeded permutation per step (Eq. 8)     */
    PSGD_TOPO_FULL = 2       /* T_u = (1/L) 1 1^T: no table, applied by psgd_mix_full                  */
};

enum { PSGD_DEG = 3 };       /* slots per table row: self, left, right */
enum { PSGD_MAX_N = 512 };   /* largest learner count the kernels stage in LDS */
enum { PSGD_MAX_DEG = 32, PSGD_MAX_TABLE = 4096 };  /* psgd_mix_step_deg: slots per row, n * deg */
enum { PSGD_STATIC_SLOTS = 2048 };  /* psgd_mix_step_cd_static: partial sums its fixed scratch array holds */

typedef enum {
    PSGD_OK = 0,
    PSGD_EINVAL = -1,  /* null pointer, n or d out of range, unknown topology / delay_mode */
    PSGD_EALIAS = -2,  /* buffers overlap in a way the requested mode cannot honour */
    PSGD_EALIGN = -3,  /* a pointer is not aligned to its element size */
    PSGD_EHIP = -4     /* a HIP runtime call failed (no device, launch error, ...) */
} psgd_status;

/*
 * psgd_build_mixing - neighbour and weight table of one iteration's mixing matrix.
 *
 * Fixed ring (Sec. 3, Eq. 3): nbr[i] = (i, i-1 mod n, i+1 mod n).  Randomized ring (Sec. 3,
 * Eq. 8; Sec. 4, RAND-PSGD: all learners draw the same permutation from a shared seed): a
 * permutation sigma of 0..n-1 puts learner sigma[p] at ring position p, and learner i at
 * position p gets nbr[i] = (i, sigma[p-1 mod n], sigma[p+1 mod n]).  All weights are
 * (float)1/3.  For n = 1 and n = 2 the slots repeat and their shares add.
 *
 * The permutation is a pure function of (n, seed, step): a SplitMix64 stream whose state
 * starts at seed XOR ((step + 1) * 0x9E3779B97F4A7C15 mod 2^64) drives a Durstenfeld shuffle
 * (i = n-1 .. 1, j = high 64 bits of draw * (i + 1), swap sigma[i], sigma[j]).
 * `seed` and `step` are ignored for PSGD_TOPO_RING.
 *
 *   nbr  host, int32 [n * 3], written        w  host, float [n * 3], written
 * Host only; touches no device.  Errors: PSGD_EINVAL (null pointer, n < 1 or
 * n > PSGD_MAX_N, unknown topology, or PSGD_TOPO_FULL, which has no 3-slot table).
 */
int psgd_build_mixing(int topology, int n, uint64_t seed, uint64_t step,
                      int32_t* nbr, float* w);

/*
 * psgd_build_mixing_device - the same table, built on the device by work enqueued on `stream`.
 * The shared-seed rule of Sec. 4 makes the ring of an iteration a function of (n, seed, step)
 * alone, so no host needs to take part: the iteration number itself may live in device memory.
 *
 *   step_dev     device, uint64 (8-byte aligned), or NULL.  The table is that of iteration
 *                step = (step_dev ? *step_dev : 0) + step_offset  (mod 2^64).
 *   advance      if step_dev is not NULL, *step_dev += advance after it has been read (0 leaves it).
 *   nbr, w       device, int32 / float [n * 3], written; layout and values bit-identical to
 *                psgd_build_mixing(topology, n, seed, step, ...).
 *
 * A captured HIP graph that holds this call with advance = 1 followed by a step call therefore
 * runs iteration k, k+1, ... on successive replays without any host work or upload.
 * Asynchronous.  Errors: as psgd_build_mixing, plus PSGD_EALIGN, PSGD_EALIAS (nbr, w and
 * step_dev overlap) and PSGD_EHIP.
 */
int psgd_build_mixing_device(int topology, int n, uint64_t seed, uint64_t* step_dev, uint64_t step_offset,
                             int advance, int32_t* nbr, float* w, void* stream);

/*
 * psgd_mix_step - fused model averaging and SGD step (Sec. 2, Eq. 2), gradients in fp32.
 *
 *   X      device, float [n * d] row-major, read
 *   X_out  device, float [n * d] row-major, written
 *   G      device, float [n * d] row-major, read
 *   nbr    device, int32 [n * 3]; w  device, float [n * 3]  (a table as built above, or any
 *          table whose entries lie in [0, n); they are read by the kernel when it runs)
 *   n      learners, 1 .. PSGD_MAX_N;   d  parameters per learner, >= 0 (0 is a no-op)
 *   lr     learning rate alpha
 *   delay_mode  0: G was computed from this X (D-PSGD, RAND-PSGD).  X_out may be the same
 *                  buffer as X (mixing in place).
 *               1: delay-by-one (Sec. 4, Eq. 14): G was computed from the previous iterate
 *                  while this X was being produced; X stays read-only for the gradient
 *                  producer that runs beside this step, so X_out must not be X.
 *          The arithmetic is the same in both modes.
 *
 * Per element, in fp32 and in this order: acc = w0 * x_self; acc = fma(w1, x_left, acc);
 * acc = fma(w2, x_right, acc); out = fma(-lr, g, acc).
 *
 * Enqueues its work on `stream` and returns without waiting.  The table lives in device memory,
 * so only the device can tell whether it is one ring (every table of Sec. 3 is) or a general
 * 3-slot table.  Short rows: one kernel that holds both paths.  Long rows (from about 1.5 M
 * columns): two kernels, the ring walk and behind it the tiled kernel, each shaped for its own
 * path; both classify the table and the one it does not belong to exits at once.
 * Errors: PSGD_EINVAL;
 * PSGD_EALIAS (X_out partially overlaps X, X_out overlaps G, or X_out == X with
 * delay_mode 1); PSGD_EALIGN (X, X_out, G not 4-byte aligned); PSGD_EHIP.  A table entry
 * outside [0, n) cannot be seen by the host: the kernel then writes nothing and raises the
 * flag that psgd_device_status() reports.
 */
int psgd_mix_step(const float* X, float* X_out, const float* G,
                  const int32_t* nbr, const float* w,
                  int n, int64_t d, float lr, int delay_mode, void* stream);

/*
 * psgd_mix_step_bf16g - the same step with gradients stored as bfloat16 bit patterns
 * (device, uint16 [n * d], 2-byte aligned).  Each gradient is widened exactly to fp32
 * (bits << 16) inside the kernel; everything else is as in psgd_mix_step.
 */
int psgd_mix_step_bf16g(const float* X, float* X_out, const uint16_t* G_bf16,
                        const int32_t* nbr, const float* w,
                        int n, int64_t d, float lr, int delay_mode, void* stream);

/*
 * psgd_mix_step_cd / psgd_mix_step_cd_bf16g - the same fused step (Sec. 2, Eq. 2) that also
 * returns the consensus distance of its own output, sum_i || x_out_i - mean(x_out) ||^2 (the
 * quantity Sec. 3 bounds), without reading X_out back: the lane that produces all n rows of
 * a column group keeps their running sums.  X_out is bit-identical to psgd_mix_step's.
 *
 *   cdist_out  device, double[1], 8-byte aligned, written by work enqueued on `stream`; it
 *              must not overlap X, X_out or G.  NaN if the table held an out-of-range entry.
 * The per-column sums are taken against the column's first output in fp64 and the
 * per-workgroup partials are combined in a fixed order (bit-reproducible; it agrees with
 * psgd_consensus_dist of X_out to rounding, about 1e-13 relative, not bit for bit).
 * Uses the same per-device buffer of partial sums as psgd_consensus_dist_async (allocated by
 * the first such call on a device, which therefore must not happen while `stream` is being
 * captured into a graph: PSGD_EHIP).  Calls on different streams of one device share it; the
 * library orders them on the device (a call that comes on another stream than the previous one
 * makes its stream wait for everything enqueued so far on that previous stream), so they
 * serialise instead of racing.  Work captured into graphs is exempt: graph launches that use
 * the buffer must be ordered by the caller.
 * All other arguments, modes and errors are those of psgd_mix_step; d = 0 writes 0.
 */
int psgd_mix_step_cd(const float* X, float* X_out, const float* G,
                     const int32_t* nbr, const float* w,
                     int n, int64_t d, float lr, int delay_mode, double* cdist_out, void* stream);
int psgd_mix_step_cd_bf16g(const float* X, float* X_out, const uint16_t* G_bf16,
                           const int32_t* nbr, const float* w,
                           int n, int64_t d, float lr, int delay_mode, double* cdist_out, void* stream);

/*
 * psgd_mix_step_ex - the general form of the four calls above: the same fused step (Sec. 2,
 * Eq. 2) on arrays whose rows are `ld*` ELEMENTS apart instead of d (row i of X starts at
 * X + i * ldx, of X_out at X_out + i * ldo, of G at G + i * ldg; each pitch >= d).
 *
 *   G          device, float or bf16 bit patterns, chosen by g_is_bf16 (0 / 1)
 *   cdist_out  device double[1] for the consensus distance of the output, or NULL for none
 * Everything else is as in psgd_mix_step.  Mixing in place needs X_out == X and ldo == ldx;
 * any other sharing of a byte between rows of X_out and rows of X or G is PSGD_EALIAS (the
 * rows of different arrays may interleave as long as they do not overlap).  The 128-bit
 * path needs d and all three pitches to be multiples of 4.
 *
 * Why pitches: (1) a column shard of a wider array is such a view; (2) placement.  On
 * MI355X this step was measured at 65-72 % of the HBM peak when each array is one dense
 * block of a few tens of GB, and at 76-78 % when the rows of every array are pitched a few
 * GB apart (other arrays' rows in between) so that the rows in flight cover most of the
 * device's address range.
 */
int psgd_mix_step_ex(const float* X, int64_t ldx, float* X_out, int64_t ldo,
                     const void* G, int64_t ldg, int g_is_bf16,
                     const int32_t* nbr, const float* w,
                     int n, int64_t d, float lr, int delay_mode, double* cdist_out, void* stream);

/*
 * psgd_mix_step_cd_static - psgd_mix_step_ex with a distance output, for callers that cannot
 * allocate device memory: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, same kernels and the same results as psgd_mix_step_ex
 * with cdist_out (which is required here); the one difference is where the per-workgroup
 * partial sums of the distance live: in a fixed array of PSGD_STATIC_SLOTS doubles (16 KB) that
 * is part of the library's device image, one copy per GPU, held until the process ends.  The
 * call makes no hipMalloc / hipFree and creates no event or stream.
 *
 * Limit: a launch uses one partial per persistent workgroup of its two kernels (the ring walk:
 * at most 4 per compute unit, 1024 on MI355X; the tiled kernel behind it takes what is left).
 * If the ring walk alone would need PSGD_STATIC_SLOTS or more the call fails with PSGD_EINVAL
 * and launches nothing.  n, d and the pitches are limited as in psgd_mix_step_ex.
 * Every call on a GPU uses that GPU's one array, which keeps the previous call's partials (each
 * launch overwrites the slots it reads, so nothing needs clearing).  Calls that overlap in time
 * on one GPU (two streams, or two graphs launched side by side) race on it: the caller orders
 * them.  It does not share the buffer of psgd_mix_step_cd / psgd_consensus_dist_async.
 */
int psgd_mix_step_cd_static(const float* X, int64_t ldx, float* X_out, int64_t ldo,
                            const void* G, int64_t ldg, int g_is_bf16,
                            const int32_t* nbr, const float* w,
                            int n, int64_t d, float lr, int delay_mode, double* cdist_out, void* stream);

/*
 * psgd_mix_step_deg - the step of Sec. 2, Eq. 2 for any sparse mixing matrix given as a table
 * with `deg` slots per row: X_out[i,:] = sum_{s<deg} w[i*deg+s] * X[nbr[i*deg+s],:] - lr*G[i,:]
 * (nbr, w: device, [n * deg]).  Covers what the 3-slot ring tables cannot: more neighbours per
 * learner, lazy walks, or the product of several mixing rounds collapsed into one matrix (the
 * remedy of the prior work the paper cites in Sec. 7).  1 <= deg <= PSGD_MAX_DEG and
 * n * deg <= PSGD_MAX_TABLE.  Per element: acc = w0 * x0; acc = fma(w_s, x_s, acc) for
 * s = 1..deg-1 in table order; out = fma(-lr, g, acc).  deg = 3 is psgd_mix_step_ex (ring
 * tables then take the register walk); other degrees always stage [n x columns] tiles in
 * LDS.  Everything else (pitches, gradient type, in-place rule, cdist_out gathered in the same
 * pass, errors) is as in psgd_mix_step_ex.
 */
int psgd_mix_step_deg(const float* X, int64_t ldx, float* X_out, int64_t ldo,
                      const void* G, int64_t ldg, int g_is_bf16,
                      const int32_t* nbr, const float* w, int deg,
                      int n, int64_t d, float lr, int delay_mode, double* cdist_out, void* stream);

/*
 * psgd_mix_full - the step with global averaging, T = T_u = (1/L) 1 1^T:
 *         X_out[i, :] = (1/n) sum_j X[j, :]  -  lr * G[i, :].
 * This is S-PSGD's mixing matrix (Sec. 2) and the one D1D-PSGD realises with an allreduce
 * divided by L (Sec. 4, Eq. 13); with delay_mode 1 and gradients taken one iterate earlier
 * (Eq. 14) it is the paper's delay-by-one update.  No table is needed.
 *
 * Arguments, pitches, gradient type, in-place rule, optional cdist_out, errors and
 * asynchrony are those of psgd_mix_step_ex.  Per element: the column sum is accumulated in
 * fp64 over rows 0..n-1, mean = (float)(sum / n), out = fma(-lr, g, mean).
 */
int psgd_mix_full(const float* X, int64_t ldx, float* X_out, int64_t ldo,
                  const void* G, int64_t ldg, int g_is_bf16,
                  int n, int64_t d, float lr, int delay_mode, double* cdist_out, void* stream);

/*
 * psgd_consensus_dist - sum_i || x_i - xbar ||^2 with xbar the mean of the n rows of X:
 * the distance from consensus whose decay Sec. 3 (Eqs. 5, 11, 12) bounds.
 *
 *   X  device, float [n * d] row-major, read.
 * Synchronous: waits for all work on the device, runs, waits again, returns the value.
 * Differences are taken against row 0 and accumulated in fp64; partial sums are combined
 * in a fixed order, so the result is bit-reproducible.  Returns NaN on error (see
 * psgd_last_error()).  d = 0 or n = 1 gives 0.
 */
double psgd_consensus_dist(const float* X, int n, int64_t d);

/*
 * psgd_consensus_dist_async - the same value written to out_dev (device, double[1],
 * 8-byte aligned) by work enqueued on `stream`.  Uses the per-device buffer of partial sums
 * described at psgd_mix_step_cd (allocated on first use, not under stream capture; calls from
 * different streams are serialised on the device).
 */
int psgd_consensus_dist_async(const float* X, int n, int64_t d, double* out_dev, void* stream);

/* psgd_consensus_dist_ex - psgd_consensus_dist_async for rows that are ldx (>= d) elements apart. */
int psgd_consensus_dist_ex(const float* X, int64_t ldx, int n, int64_t d, double* out_dev, void* stream);

/*
 * psgd_synth_grad - synthetic stand-in for back-propagation in the delay-by-one workload:
 * G[e] = fma(c, X_prev[e], noise[e]) over `count` fp32 elements (all device pointers,
 * 4-byte aligned; G must not overlap the inputs).  It plays the gradient producer that
 * Sec. 4 runs concurrently with the averaging of the current iterate.  Enqueues on `stream`.
 */
int psgd_synth_grad(const float* X_prev, const float* noise, float* G,
                    int64_t count, float c, void* stream);

/* psgd_synth_grad_ex - the same for [n, d] arrays whose rows are ld* (>= d) elements apart. */
int psgd_synth_grad_ex(const float* X_prev, int64_t ldx, const float* noise, int64_t ldn,
                       float* G, int64_t ldg, int n, int64_t d, float c, void* stream);

/*
 * psgd_reference_stream - measurement support, not a step of the method: the memory traffic of
 * the fused step with the mixing taken out, issued exactly as the step's kernel issues it (a lane
 * per 128-bit column group walking the n rows, workgroups sweeping the rows in lockstep batches,
 * the same persistent grid).  The rate it reaches on a given placement of the arrays is the
 * ceiling the step is compared with in the benchmark.
 *
 *   kind 0  read X and G, write nothing          (4 + 2 or 4 + 4 bytes per element)
 *   kind 1  write X_out[i, j] = a, read nothing   (4 bytes per element)
 *   kind 2  X_out = X + a * G                     (the step's 4 + 2 + 4 or 4 + 4 + 4 bytes)
 * Arguments as in psgd_mix_step_ex (all three arrays must be valid for every kind); d and the
 * pitches must be multiples of 4 and the rows 128-bit aligned (PSGD_EALIGN otherwise); X_out
 * must not overlap X or G for kinds 1 and 2.  Enqueues one kernel on `stream`.
 */
int psgd_reference_stream(int kind, const float* X, int64_t ldx, float* X_out, int64_t ldo,
                          const void* G, int64_t ldg, int g_is_bf16, int n, int64_t d, float a, void* stream);

/*
 * psgd_spread_alloc / psgd_spread_free - placement support, not a step of the method: device memory for the
 * rows of the replica arrays that is spread out PHYSICALLY while only the rows themselves stay resident.
 * On MI355X a kernel that writes many gigabytes runs at a rate that depends on where the written memory
 * lies physically (rows a few GB apart: 87 % of the HBM peak for stores; the same rows back to back: 68 %).
 *
 * Reserves one address range of n * pitch bytes on the current device and backs slot i, the bytes
 * [i * pitch, i * pitch + slot), with physical memory; slot_bytes and pitch_bytes are rounded up to the
 * allocation granularity, the pitch used is returned in *pitch_out and the start of the range in *base_out.
 * The physical memory of the slots is taken in turn with chunks of the size of the gaps between them, and
 * the gap chunks are given back before the call returns: while it runs the device must have n * pitch bytes
 * free, afterwards n * slot bytes are in use.  Addresses between the slots are not mapped: touching them
 * faults.  The memory is not cleared.  The caller lays out its rows inside the slots (row i of every array in
 * slot i, say) and passes base + offset with a row pitch of pitch / element size to the *_ex entry points.
 * psgd_spread_free(base) waits for the device and releases everything; at most 16 allocations live at a time.
 * Errors: PSGD_EINVAL (arguments, unknown base), PSGD_EHIP (the runtime refused; nothing stays allocated).
 */
int psgd_spread_alloc(int n, int64_t slot_bytes, int64_t pitch_bytes, void** base_out, int64_t* pitch_out);
int psgd_spread_free(void* base);

/*
 * psgd_interleaved_alloc / psgd_interleaved_free - placement support, not a step of the method: one block of
 * `bytes` bytes (rounded up to whole GiB) of device memory at consecutive addresses whose 1 GiB pieces come
 * from the three thirds of the device's physical memory in turn.  MI355X writes at the full rate only when
 * the rows being written are spread evenly over at least two of these thirds; on this block that holds for
 * plain dense [n, d] arrays wherever they start, so the entry points that take dense arrays
 * (psgd_mix_step, psgd_mix_step_cd_bf16g, ...) run at the rate of the spread rows (77 % of the HBM peak for
 * the step on 64 x 1e8 elements, against 59-76 % on ordinary allocations).
 *
 * While the call runs it holds all free device memory but 4 GiB (that is how it reaches every third) and
 * measures which third each 1 GiB piece lies in: two pieces written together by a small kernel on the null
 * stream take a quarter longer when they share a third.  The call therefore takes a few seconds (4 s with
 * 280 GiB free), synchronises with the device, and must not run under stream capture.  Being measured, the
 * placement does not depend on what the process allocated and freed before.  Where the measurement shows no such structure the
 * block is still valid memory, only not faster than any other.  The memory is not cleared.  At most 16 blocks
 * live at a time; psgd_interleaved_free(ptr) waits for the device and releases the block.
 * Errors: PSGD_EINVAL (arguments, unknown pointer), PSGD_EHIP (does not fit, or the runtime refused; nothing
 * stays allocated).
 */
int psgd_interleaved_alloc(int64_t bytes, void** ptr_out);
int psgd_interleaved_free(void* ptr);

/*
 * psgd_device_status - waits for the current device, then returns the sticky flag word that
 * kernels raise (bit 0: a mixing table held an entry outside [0, n) and the step wrote
 * nothing).  `clear` != 0 resets it.  Negative psgd_status on failure.
 */
int psgd_device_status(int clear);

/* Text of the last error on the calling thread ("" if none).  Static storage. */
const char* psgd_last_error(void);

/* Library version, for the binding's load check. */
int psgd_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PSGD_H */
