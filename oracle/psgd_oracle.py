"""CPU oracle for the decentralized-SGD model-averaging step.  TEST INFRASTRUCTURE ONLY.

This file is the slow, plain, fp64 statement of what the HIP library computes.  It is
imported only by the tests, by the smoke check and by the benchmark's CPU-baseline leg;
the product path never calls it.  It shares no code, table or constant with the HIP
sources and imports nothing from the GPU package.

Conventions.  The paper stores one learner per COLUMN: W is d x L and the update is
W_{k+1} = W_k T - alpha g (Sec. 2, Eq. 2).  This build stores one learner per ROW:
X = W^T is [n, d] with n = L, so the same update reads X_{k+1} = T^T X_k - lr G.
Every function here that applies a mixing matrix uses the transpose explicitly, so
an asymmetric doubly stochastic matrix is handled the way Eq. 2 states it.

Everything floating point is numpy float64.  Inputs that the GPU receives as fp32 or
bf16 bit patterns are widened exactly before any arithmetic.

Pins (tests/test_oracle_pins.py, all CPU):
  ring_matrix            literal entries of Eq. 3, double stochasticity, full circulant
                         spectrum (1 + 2 cos(2 pi k / L)) / 3, rho of Eq. 6
  splitmix64 / permutation   published SplitMix64 output vectors, bijection, determinism,
                         exhaustive-outcome uniformity for small n
  rand_ring_matrix       explicit P^T T_0 P product (Eq. 8) vs. the table form, spectrum
                         equal to the fixed ring's, E[T^T T] entries (Eq. 10) and the
                         expected Frobenius contraction (Eq. 11) by enumeration of all L!
                         permutations
  densify                asymmetric tables typed out entry by entry (one-slot cyclic shift, a
                         two-slot 3/4-1/4 table, repeated slots), gather-add scalar loops on
                         random asymmetric tables; planted transposed / overwriting / slot-dropping
                         mutants are caught
  mix_step               element-by-element triple loop, asymmetric shift matrix,
                         n = 1 reduces to Eq. 1, T_u gives the column mean, mean recurrence
  sparse_mix_step (C)    typed-out asymmetric example; equals mix_step(densify(table)) on random
                         asymmetric and ring tables, fp32 and bf16 gradients, any thread count
  consensus_dist         closed forms (equal rows -> 0; X[i,j] = i -> d n (n^2-1)/12),
                         contraction bound rho^2 of Eq. 5
  synth_grad / d1d_trajectory   reduce to the undelayed run when the X-dependent term is
                         zero; the replica mean obeys the two-term linear recurrence; on the
                         fixed ring every eigenmode follows the closed-form solution of
                         y_{k+1} = lambda y_k - lr c y_{k-1} (characteristic roots); with T_u
                         the consensus distance is (lr c)^(2 ceil(k/2)) C_0, a noise impulse
                         returns every second step, and the trajectory is linear in its
                         inputs; three planted mutants of the delay are caught.
"""
import numpy as np

TOPO_RING = 0
TOPO_RAND_RING = 1
TOPO_FULL = 2

_MASK64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15


# --------------------------------------------------------------------------------------
# Shared-seed permutation (Sec. 4, RAND-PSGD paragraph: every learner starts from the
# same seed so that all of them draw the same permutation in every iteration).
# The paper fixes no generator; this build's reading is SplitMix64 keyed by (seed, step)
# followed by a Durstenfeld shuffle with multiply-high index reduction.
# --------------------------------------------------------------------------------------
def splitmix64(state, count):
    """Return `count` successive SplitMix64 outputs starting from internal state `state`.

    One draw: state += 0x9E3779B97F4A7C15; z = state; z = (z ^ z>>30) * 0xBF58476D1CE4E5B9;
    z = (z ^ z>>27) * 0x94D049BB133111EB; output z ^ z>>31 (all mod 2^64).
    Python integers, so there is no overflow behaviour to get wrong.
    """
    out = []
    s = state & _MASK64
    for _ in range(count):
        s = (s + _GOLDEN) & _MASK64
        z = s
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
        out.append(z ^ (z >> 31))
    return out


def permutation(n, seed, step):
    """sigma(0..n-1): sigma[p] is the learner that sits at ring position p in iteration `step`.

    Generator state starts at seed XOR ((step + 1) * golden mod 2^64); the shuffle walks
    i = n-1 .. 1, draws r, takes j = floor(r * (i + 1) / 2^64) and swaps sigma[i], sigma[j].
    """
    state = (seed & _MASK64) ^ (((step + 1) * _GOLDEN) & _MASK64)
    draws = splitmix64(state, max(n - 1, 0))
    sigma = list(range(n))
    t = 0
    for i in range(n - 1, 0, -1):
        j = (draws[t] * (i + 1)) >> 64
        t += 1
        sigma[i], sigma[j] = sigma[j], sigma[i]
    return sigma


# --------------------------------------------------------------------------------------
# Dense mixing matrices, straight from their definitions.
# --------------------------------------------------------------------------------------
def ring_matrix(n):
    """T_0 of Sec. 3, Eq. 3: 1/3 on the diagonal and on the two cyclic off-diagonals.

    For n = 1 and n = 2 the neighbours coincide and their 1/3 shares add up, which is what
    keeps the circulant's Fourier spectrum valid for every n >= 1.
    """
    T = np.zeros((n, n), dtype=np.float64)
    for i in range(n):
        for j in (i, (i - 1) % n, (i + 1) % n):
            T[i, j] += 1.0 / 3.0
    return T


def uniform_matrix(n):
    """T_u = (1/L) 1 1^T of Sec. 2: global averaging (S-PSGD, and D1D-PSGD's allreduce / L)."""
    return np.full((n, n), 1.0 / n, dtype=np.float64)


def permutation_matrix(sigma):
    """P with P[p, sigma[p]] = 1: row p (a ring position) selects the learner sitting there."""
    n = len(sigma)
    P = np.zeros((n, n), dtype=np.float64)
    for p in range(n):
        P[p, sigma[p]] = 1.0
    return P


def rand_ring_matrix(sigma):
    """T_tau = P^T T_0 P of Sec. 3, Eq. 8, by two explicit matrix products."""
    P = permutation_matrix(sigma)
    return P.T @ ring_matrix(len(sigma)) @ P


def mixing_matrix(topology, n, seed=0, step=0):
    if topology == TOPO_RING:
        return ring_matrix(n)
    if topology == TOPO_RAND_RING:
        return rand_ring_matrix(permutation(n, seed, step))
    if topology == TOPO_FULL:
        return uniform_matrix(n)
    raise ValueError("unknown topology %r" % (topology,))


# --------------------------------------------------------------------------------------
# The sparse table the library hands to its kernel, derived here independently so that
# the two can be compared bit for bit.  Row i lists the learners whose models feed
# learner i (column i of T) in the slot order (self, left, right).
# --------------------------------------------------------------------------------------
def neighbour_table(topology, n, seed=0, step=0):
    """Return (nbr int32 [n,3], w float32 [n,3]) for the ring topologies."""
    if topology == TOPO_RING:
        sigma = list(range(n))
    elif topology == TOPO_RAND_RING:
        sigma = permutation(n, seed, step)
    else:
        raise ValueError("no 3-slot table for topology %r" % (topology,))
    pos = [0] * n
    for p in range(n):
        pos[sigma[p]] = p
    nbr = np.zeros((n, 3), dtype=np.int32)
    for i in range(n):
        nbr[i, 0] = i
        nbr[i, 1] = sigma[(pos[i] - 1) % n]
        nbr[i, 2] = sigma[(pos[i] + 1) % n]
    w = np.full((n, 3), np.float32(1.0) / np.float32(3.0), dtype=np.float32)
    return nbr, w


def densify(nbr, w):
    """Dense T (fp64) from a slot table: T[nbr[i,s], i] += w[i,s]; duplicate slots add."""
    nbr = np.asarray(nbr)
    w = np.asarray(w)
    n, deg = nbr.shape
    T = np.zeros((n, n), dtype=np.float64)
    for i in range(n):
        for s in range(deg):
            T[int(nbr[i, s]), i] += float(w[i, s])
    return T


# --------------------------------------------------------------------------------------
# Exact widening of the bit patterns the GPU sees.
# --------------------------------------------------------------------------------------
def bf16_bits_to_f64(bits_u16):
    """bfloat16 bit patterns (uint16) -> float64, exactly (bf16 is the top half of fp32)."""
    b = np.asarray(bits_u16, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(np.float64)


def _widen(a):
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return bf16_bits_to_f64(a)
    return a.astype(np.float64)


# --------------------------------------------------------------------------------------
# The update and the consensus distance.
# --------------------------------------------------------------------------------------
def mix_step(X, G, T, lr):
    """X_{k+1} = T^T X_k - lr G (Sec. 2, Eq. 2 in row-per-learner layout), float64 result.

    X: [n, d] fp32 (or fp64); G: [n, d] fp32, fp64 or bf16 bit patterns (uint16);
    T: dense [n, n]; lr: the learning rate exactly as the library receives it (a C float).
    """
    X64 = _widen(X)
    G64 = _widen(G)
    T64 = np.asarray(T, dtype=np.float64)
    lr64 = float(np.float32(lr))
    return T64.T @ X64 - lr64 * G64


def consensus_dist(X):
    """sum_i || x_i - xbar ||^2 with xbar the replica mean: two passes, float64."""
    X64 = _widen(X)
    xbar = X64.sum(axis=0) / X64.shape[0]
    D = X64 - xbar[None, :]
    return float((D * D).sum())


def spectrum(T):
    """Eigenvalues of a symmetric mixing matrix, descending."""
    T = np.asarray(T, dtype=np.float64)
    if not np.allclose(T, T.T, atol=1e-14):
        raise ValueError("spectrum() expects a symmetric matrix")
    return np.sort(np.linalg.eigvalsh(T))[::-1]


def spectral_rho(T):
    """rho = max(|lambda_2|, |lambda_L|) of Sec. 3 (the text around Eq. 5); 0 for L = 1."""
    lam = spectrum(T)
    if lam.shape[0] < 2:
        return 0.0
    return float(max(abs(lam[1]), abs(lam[-1])))


def ring_spectrum_closed_form(n):
    """Fourier transform of T_0's first row (Sec. 3): (1 + 2 cos(2 pi k / L)) / 3, k = 0..L-1."""
    k = np.arange(n, dtype=np.float64)
    return (1.0 + 2.0 * np.cos(2.0 * np.pi * k / n)) / 3.0


# --------------------------------------------------------------------------------------
# Delay-by-one data flow (Sec. 4, Eq. 14: Phi_k = W_{k-1}).
# --------------------------------------------------------------------------------------
def synth_grad(X_prev, noise, c):
    """Synthetic stand-in for back-propagation: G = c * X_prev + noise, float64.

    The delayed workload draws its gradient as a linear pull toward zero plus noise,
    evaluated at the iterate the learner held one step earlier.  `c` is taken exactly as
    the library receives it (a C float).
    """
    c64 = float(np.float32(c))
    return c64 * _widen(X_prev) + _widen(noise)


def run_steps(X0, grads, tables, lr):
    """Undelayed trajectory X_{k+1} = T_k^T X_k - lr G_k with given G_k; float64 throughout.

    Returns [X_0, X_1, ..., X_K].
    """
    Xs = [_widen(X0)]
    for G, T in zip(grads, tables):
        Xs.append(mix_step(Xs[-1], G, T, lr))
    return Xs


def d1d_trajectory(X0, noises, tables, lr, c):
    """Delayed trajectory: X_{k+1} = T_k^T X_k - lr G_k, G_k = synth_grad(X_{k-1}, noise_k).

    The first step has no earlier iterate, so X_{-1} := X_0 (the first gradient is taken at
    the initial weights).  float64 throughout; returns [X_0, X_1, ..., X_K].
    """
    Xs = [_widen(X0)]
    X_prev = Xs[0]
    for k, T in enumerate(tables):
        G = synth_grad(X_prev, noises[k], c)
        X_next = mix_step(Xs[-1], G, T, lr)
        X_prev = Xs[-1]
        Xs.append(X_next)
    return Xs


# --------------------------------------------------------------------------------------
# Sparse form of the update in plain C (psgd_sparse_oracle.c): the same result as mix_step with the
# densified table, computed as the gather-add it is.  Used as the CPU baseline of the benchmark (a dense
# matrix product is an unfairly slow way to apply three neighbours) and pinned against mix_step.
# --------------------------------------------------------------------------------------
_SPARSE_LIB = None


def build_sparse_lib(force=False):
    """Compile psgd_sparse_oracle.c with the host C compiler (gcc -O2 -fopenmp) next to its source."""
    import os
    import subprocess
    here = os.path.dirname(os.path.abspath(__file__))
    src = os.path.join(here, "psgd_sparse_oracle.c")
    lib = os.path.join(here, "libpsgd_sparse_oracle.so")
    if force or not os.path.exists(lib) or os.path.getmtime(lib) < os.path.getmtime(src):
        tmp = lib + ".%d.tmp" % os.getpid()
        subprocess.run([os.environ.get("CC", "gcc"), "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall",
                        src, "-o", tmp], check=True)
        os.replace(tmp, lib)
    return lib


def _sparse_lib():
    global _SPARSE_LIB
    if _SPARSE_LIB is None:
        import ctypes
        lib = ctypes.CDLL(build_sparse_lib())
        vp = ctypes.c_void_p
        lib.psgd_oracle_sparse_step.restype = None
        lib.psgd_oracle_sparse_step.argtypes = [vp, vp, ctypes.c_int, vp, vp, ctypes.c_int, ctypes.c_int,
                                                ctypes.c_int64, ctypes.c_float, vp, ctypes.c_int]
        lib.psgd_oracle_consensus.restype = ctypes.c_double
        lib.psgd_oracle_consensus.argtypes = [vp, ctypes.c_int, ctypes.c_int64, ctypes.c_int]
        _SPARSE_LIB = lib
    return _SPARSE_LIB


def sparse_mix_step(X, G, nbr, w, lr, threads=1):
    """out[i] = sum_s w[i,s] X[nbr[i,s]] - lr G[i] (Sec. 2, Eq. 2; table row i = column i of T), float64.

    X: [n, d] fp32; G: [n, d] fp32 or bf16 bit patterns (uint16); nbr int32 [n, deg]; w fp32 [n, deg]."""
    X = np.ascontiguousarray(X, dtype=np.float32)
    G = np.ascontiguousarray(G)
    if G.dtype not in (np.float32, np.uint16):
        raise ValueError("G must be float32 or uint16 bf16 bit patterns")
    nbr = np.ascontiguousarray(nbr, dtype=np.int32)
    w = np.ascontiguousarray(w, dtype=np.float32)
    n, d = X.shape
    if G.shape != (n, d) or nbr.shape != w.shape or nbr.shape[0] != n:
        raise ValueError("shape mismatch")
    if nbr.size and (nbr.min() < 0 or nbr.max() >= n):
        raise ValueError("table entry outside [0, n)")
    out = np.empty((n, d), dtype=np.float64)
    _sparse_lib().psgd_oracle_sparse_step(X.ctypes.data, G.ctypes.data, int(G.dtype == np.uint16), nbr.ctypes.data,
                                          w.ctypes.data, int(nbr.shape[1]), n, d, float(np.float32(lr)),
                                          out.ctypes.data, int(threads))
    return out


def sparse_consensus_dist(X64, threads=1):
    """Two-pass consensus distance of a float64 [n, d] array, in C (same definition as consensus_dist)."""
    X64 = np.ascontiguousarray(X64, dtype=np.float64)
    return float(_sparse_lib().psgd_oracle_consensus(X64.ctypes.data, X64.shape[0], X64.shape[1], int(threads)))
