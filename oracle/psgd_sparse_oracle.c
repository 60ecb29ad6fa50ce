/*
 * Sparse form of the CPU oracle's update.  TEST INFRASTRUCTURE ONLY: called by the tests and by the
 * benchmark's CPU-baseline leg, never by the product path; shares no code with the HIP library.
 *
 * One iteration of decentralized parallel SGD in row-per-learner layout (Sec. 2, Eq. 2 with X = W^T):
 *     out[i, j] = sum_{s < deg} w[i, s] * X[nbr[i, s], j]  -  lr * G[i, j]
 * where row i of the (nbr, w) table lists column i of the mixing matrix T: the learners whose models feed
 * learner i, with their weights (for the rings of Sec. 3: self, left and right neighbour, 1/3 each).
 * It is the same result as the dense product T^T X - lr G of the Python oracle, which is what the tests pin
 * it against; it exists because a memory-bound gather-add, not a dense matrix product, is the fair CPU
 * baseline for the step.
 *
 * Arithmetic: every input is widened exactly to double (bf16 bit patterns by a 16-bit shift), products and
 * sums are taken in double in table order, nothing is blocked or reordered beyond the loop over columns
 * being shared out to threads (columns are independent).
 */
#include <stdint.h>
#include <string.h>

static double widen_bf16(uint16_t bits) {
    const uint32_t u = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* X: [n, d] float; G: [n, d] float or uint16 bf16 bit patterns; out: [n, d] double; all row-major, dense. */
void psgd_oracle_sparse_step(const float* X, const void* G, int g_is_bf16, const int32_t* nbr, const float* w,
                             int deg, int n, int64_t d, float lr, double* out, int threads) {
    const double lr64 = (double)lr;
    const float* Gf = (const float*)G;
    const uint16_t* Gh = (const uint16_t*)G;
    const int64_t block = 4096;                       /* columns handed to a thread at a time */
    const int64_t nblocks = (d + block - 1) / block;
    int64_t b;
    if (threads < 1) threads = 1;
#pragma omp parallel for schedule(static) num_threads(threads)
    for (b = 0; b < nblocks; ++b) {
        const int64_t lo = b * block, hi = lo + block < d ? lo + block : d;
        for (int i = 0; i < n; ++i) {
            double* o = out + (int64_t)i * d;
            for (int64_t j = lo; j < hi; ++j) {
                double acc = 0.0;
                for (int s = 0; s < deg; ++s)
                    acc += (double)w[i * deg + s] * (double)X[(int64_t)nbr[i * deg + s] * d + j];
                const double g = g_is_bf16 ? widen_bf16(Gh[(int64_t)i * d + j]) : (double)Gf[(int64_t)i * d + j];
                o[j] = acc - lr64 * g;
            }
        }
    }
}

/* Two-pass consensus distance sum_i ||x_i - xbar||^2 of a double [n, d] array (the quantity Sec. 3 bounds). */
double psgd_oracle_consensus(const double* X, int n, int64_t d, int threads) {
    double total = 0.0;
    int64_t j;
    if (threads < 1) threads = 1;
#pragma omp parallel for schedule(static) reduction(+ : total) num_threads(threads)
    for (j = 0; j < d; ++j) {
        double mean = 0.0, c = 0.0;
        for (int i = 0; i < n; ++i) mean += X[(int64_t)i * d + j];
        mean /= (double)n;
        for (int i = 0; i < n; ++i) {
            const double df = X[(int64_t)i * d + j] - mean;
            c += df * df;
        }
        total += c;
    }
    return total;
}
