// Host side of the library: mixing-table construction and the per-thread error text.
// No device work happens in this file.
#include "psgd.h"
#include "psgd_internal.h"

#include <cstdarg>
#include <cstdio>

namespace psgd {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

void clear_error() { g_err[0] = '\0'; }

namespace {

// SplitMix64: additive Weyl sequence followed by a 64-bit finaliser.
struct SplitMix64 {
    uint64_t s;
    uint64_t next() {
        s += 0x9E3779B97F4A7C15ull;
        uint64_t z = s;
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    }
};

// sigma[p] = learner at ring position p for iteration `step` (Sec. 4: every learner derives
// the same ring from the shared seed, so this must depend on (n, seed, step) only).
void draw_ring(int n, uint64_t seed, uint64_t step, int32_t* sigma) {
    for (int p = 0; p < n; ++p) sigma[p] = p;
    SplitMix64 rng{seed ^ ((step + 1ull) * 0x9E3779B97F4A7C15ull)};
    for (int i = n - 1; i >= 1; --i) {
        const unsigned __int128 wide = (unsigned __int128)rng.next() * (uint64_t)(i + 1);
        const int j = (int)(uint64_t)(wide >> 64);
        const int32_t t = sigma[i];
        sigma[i] = sigma[j];
        sigma[j] = t;
    }
}

}  // namespace
}  // namespace psgd

extern "C" {

int psgd_build_mixing(int topology, int n, uint64_t seed, uint64_t step, int32_t* nbr, float* w) {
    using namespace psgd;
    clear_error();
    if (!nbr || !w) return fail(PSGD_EINVAL, "psgd_build_mixing: null output pointer");
    if (n < 1 || n > PSGD_MAX_N)
        return fail(PSGD_EINVAL, "psgd_build_mixing: n=%d outside 1..%d", n, (int)PSGD_MAX_N);
    if (topology == PSGD_TOPO_FULL)
        return fail(PSGD_EINVAL, "psgd_build_mixing: the uniform topology has no 3-slot table, use psgd_mix_full");
    if (topology != PSGD_TOPO_RING && topology != PSGD_TOPO_RAND_RING)
        return fail(PSGD_EINVAL, "psgd_build_mixing: unknown topology %d", topology);

    int32_t sigma[PSGD_MAX_N];   // on the stack: nothing here can throw across the C boundary
    if (topology == PSGD_TOPO_RAND_RING) {
        draw_ring(n, seed, step, sigma);
    } else {
        for (int p = 0; p < n; ++p) sigma[p] = p;
    }
    // Walk the ring once: the learner at position p has the learners at p-1 and p+1 as its
    // left and right neighbours (Sec. 3: each learner averages with the two learners that are
    // adjacent to it after the shuffle).
    const float third = 1.0f / 3.0f;
    for (int p = 0; p < n; ++p) {
        const int32_t me = sigma[p];
        const int32_t left = sigma[p == 0 ? n - 1 : p - 1];
        const int32_t right = sigma[p == n - 1 ? 0 : p + 1];
        nbr[3 * me + 0] = me;
        nbr[3 * me + 1] = left;
        nbr[3 * me + 2] = right;
        w[3 * me + 0] = third;
        w[3 * me + 1] = third;
        w[3 * me + 2] = third;
    }
    return PSGD_OK;
}

const char* psgd_last_error(void) { return psgd::g_err; }

int psgd_version(void) { return 3; }

}  // extern "C"
