"""Pins for the CPU oracle: everything here is checked against what the paper and the
mathematics fix, never against the oracle's own formulas re-typed.  CPU only."""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import psgd_oracle as orc
from paper_2002_01119_amd import inputs as inp

NS = [1, 2, 3, 4, 5, 6, 7, 8, 9, 16, 33, 64, 128]


# ------------------------------------------------------------------ fixed ring (Sec. 3, Eq. 3)
def test_ring_literal_entries_6x6():
    """The 6x6 instance of Eq. 3 typed out entry by entry."""
    t = 1.0 / 3.0
    want = np.array([
        [t, t, 0, 0, 0, t],
        [t, t, t, 0, 0, 0],
        [0, t, t, t, 0, 0],
        [0, 0, t, t, t, 0],
        [0, 0, 0, t, t, t],
        [t, 0, 0, 0, t, t],
    ])
    assert np.array_equal(orc.ring_matrix(6), want)


def test_ring_small_n_duplicates_add():
    assert np.allclose(orc.ring_matrix(1), [[1.0]], atol=1e-15)
    assert np.allclose(orc.ring_matrix(2), [[1 / 3, 2 / 3], [2 / 3, 1 / 3]], atol=1e-15)
    assert np.allclose(orc.ring_matrix(3), np.full((3, 3), 1 / 3), atol=1e-15)


@pytest.mark.parametrize("n", NS)
def test_doubly_stochastic(n):
    """Sec. 2: T is doubly stochastic; Sec. 3 says the same of every permuted ring."""
    mats = [orc.ring_matrix(n), orc.uniform_matrix(n)]
    for step in range(4):
        mats.append(orc.mixing_matrix(orc.TOPO_RAND_RING, n, seed=77, step=step))
    for T in mats:
        assert np.all(T >= 0)
        assert np.allclose(T.sum(axis=0), 1.0, atol=1e-12)
        assert np.allclose(T.sum(axis=1), 1.0, atol=1e-12)


@pytest.mark.parametrize("n", NS)
def test_ring_spectrum_closed_form(n):
    """Sec. 3: the eigenvalues are the Fourier transform of the first row."""
    lam = orc.spectrum(orc.ring_matrix(n))
    want = np.sort([(1 + 2 * math.cos(2 * math.pi * k / n)) / 3 for k in range(n)])[::-1]
    assert np.allclose(lam, want, atol=1e-12)
    assert np.allclose(np.sort(orc.ring_spectrum_closed_form(n))[::-1], want, atol=1e-15)
    # numpy's FFT of the first row is the same statement made by a library routine
    fft = np.sort(np.fft.fft(orc.ring_matrix(n)[0]).real)[::-1]
    assert np.allclose(lam, fft, atol=1e-12)


@pytest.mark.parametrize("n,printed", [(8, 0.8047378541), (16, 0.9492530217),
                                       (64, 0.9967898178), (128, 0.9991969708)])
def test_rho_formula(n, printed):
    """Sec. 3, Eq. 6: rho = 1/3 + (2/3) cos(2 pi / L), against the eigendecomposition."""
    rho = orc.spectral_rho(orc.ring_matrix(n))
    assert abs(rho - (1 / 3 + 2 / 3 * math.cos(2 * math.pi / n))) < 1e-12
    assert abs(rho - printed) < 5e-11


def test_rho_small_n():
    # Eq. 6 is exact from L = 3 on (L = 3 gives 0 because T_0 = T_u there); at L = 2 the
    # definition max(|lambda_2|, |lambda_L|) gives 1/3 while the cosine form gives -1/3.
    assert orc.spectral_rho(orc.ring_matrix(1)) == 0.0
    assert abs(orc.spectral_rho(orc.ring_matrix(2)) - 1 / 3) < 1e-12
    assert abs(orc.spectral_rho(orc.ring_matrix(3))) < 1e-12
    for n in range(3, 40):
        assert abs(orc.spectral_rho(orc.ring_matrix(n))
                   - (1 / 3 + 2 / 3 * math.cos(2 * math.pi / n))) < 1e-12


@pytest.mark.parametrize("n", [4, 8, 16])
def test_power_converges_to_uniform_at_rate_rho(n):
    """Sec. 3, Eqs. 4-5: T_0^k -> T_u and || T_0^k - T_u ||_2 <= rho^k."""
    T0, Tu = orc.ring_matrix(n), orc.uniform_matrix(n)
    rho = 1 / 3 + 2 / 3 * math.cos(2 * math.pi / n)
    P = np.eye(n)
    for k in range(1, 60):
        P = P @ T0
        nrm = np.linalg.norm(P - Tu, 2)
        assert nrm <= rho ** k + 1e-12
        assert nrm >= rho ** k - 1e-9          # symmetric T_0: the bound is attained
    assert np.linalg.norm(np.linalg.matrix_power(T0, 4000) - Tu, 2) < 1e-6


# ------------------------------------------------------------------ shared-seed permutation
def test_splitmix64_published_vectors(golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "splitmix64_vectors.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                rows.append([int(x) for x in line.split()])
    assert len(rows) >= 6
    for state, idx, want in rows:
        assert orc.splitmix64(state, idx + 1)[idx] == want


@pytest.mark.parametrize("n", NS)
def test_permutation_is_bijection_and_deterministic(n):
    seen = set()
    for seed in (0, 1, 3005, 2 ** 63 + 12345, 2 ** 64 - 1):
        for step in (0, 1, 2, 99, 2 ** 40):
            s1 = orc.permutation(n, seed, step)
            s2 = orc.permutation(n, seed, step)
            assert s1 == s2
            assert sorted(s1) == list(range(n))
            seen.add(tuple(s1))
    if n >= 8:
        assert len(seen) == 25       # distinct (seed, step) give distinct rings


def test_permutation_step_changes_ring():
    a = [tuple(orc.permutation(64, 3003, k)) for k in range(100)]
    assert len(set(a)) == 100


@pytest.mark.parametrize("n", [2, 3, 4, 5])
def test_permutation_uniform_over_all_outcomes(n):
    """Chi-square over all n! outcomes; the shuffle must reach each equally often."""
    draws = 2000 * math.factorial(n) if n < 5 else 60000
    counts = {}
    for t in range(draws):
        s = tuple(orc.permutation(n, 4242, t))
        counts[s] = counts.get(s, 0) + 1
    assert len(counts) == math.factorial(n)
    exp = draws / math.factorial(n)
    chi2 = sum((c - exp) ** 2 / exp for c in counts.values())
    dof = math.factorial(n) - 1
    # mean dof, variance 2 dof: six sigma keeps a correct generator from ever failing
    assert chi2 < dof + 6 * math.sqrt(2 * dof) + 6


def test_permutation_position_marginals_n64():
    n, draws = 64, 6400
    hist = np.zeros((n, n))
    for t in range(draws):
        s = orc.permutation(n, 9, t)
        for p, l in enumerate(s):
            hist[p, l] += 1
    exp = draws / n
    chi2 = ((hist - exp) ** 2 / exp).sum()
    dof = (n - 1) ** 2
    assert abs(chi2 - dof) < 6 * math.sqrt(2 * dof)


# ------------------------------------------------------------------ randomized ring (Eq. 8)
@pytest.mark.parametrize("n", [3, 4, 5, 8, 16, 64, 128])
def test_rand_ring_matches_index_form_and_table(n):
    sigma = orc.permutation(n, 3003, 17)
    T = orc.rand_ring_matrix(sigma)
    inv = np.argsort(sigma)
    T0 = orc.ring_matrix(n)
    # (P^T T_0 P)[i, j] = T_0[sigma^-1(i), sigma^-1(j)]
    assert np.array_equal(T, T0[np.ix_(inv, inv)])
    # the 3-slot table describes the same matrix (its weights are fl32(1/3))
    nbr, w = orc.neighbour_table(orc.TOPO_RAND_RING, n, 3003, 17)
    assert np.allclose(orc.densify(nbr, w), T, atol=4e-8)
    assert np.array_equal(orc.densify(nbr, np.full((n, 3), 1 / 3)) > 0, T > 0)
    # neighbours in the table are adjacent ring positions; slot order self, left, right
    for i in range(n):
        p = int(inv[i])
        assert nbr[i, 0] == i
        assert nbr[i, 1] == sigma[(p - 1) % n] and nbr[i, 2] == sigma[(p + 1) % n]
    # similar matrices: same spectrum as the fixed ring
    assert np.allclose(orc.spectrum(T), orc.spectrum(T0), atol=1e-12)
    assert np.allclose(T, T.T)


def test_fixed_ring_table_is_identity_permutation():
    for n in NS:
        nbr, w = orc.neighbour_table(orc.TOPO_RING, n)
        assert np.allclose(orc.densify(nbr, np.full((n, 3), 1 / 3)), orc.ring_matrix(n), atol=1e-15)
        assert w.dtype == np.float32 and np.all(w.view(np.uint32) == 0x3EAAAAAB)
        assert nbr.dtype == np.int32


@pytest.mark.parametrize("n", [4, 5, 6, 7])
def test_expected_gram_matrix_exhaustive(n):
    """Sec. 3, Eq. 10: E[T^T T] has 1/3 on the diagonal and 2/(3(L-1)) elsewhere,
    averaged over ALL L! permutations (no sampling)."""
    acc = np.zeros((n, n))
    cnt = 0
    for sigma in itertools.permutations(range(n)):
        T = orc.rand_ring_matrix(list(sigma))
        acc += T.T @ T
        cnt += 1
    acc /= cnt
    want = np.full((n, n), 2 / (3 * (n - 1)))
    np.fill_diagonal(want, 1 / 3)
    assert np.allclose(acc, want, atol=1e-13)


@pytest.mark.parametrize("n,k", [(4, 1), (4, 2), (4, 3), (5, 1), (5, 2), (6, 1)])
def test_expected_frobenius_contraction_exhaustive(n, k):
    """Sec. 3, Eq. 11: E || T_1 ... T_k - T_u ||_F^2 = (L-1) (1/3 - 2/(3(L-1)))^k."""
    mats = [orc.rand_ring_matrix(list(s)) for s in itertools.permutations(range(n))]
    Tu = orc.uniform_matrix(n)
    total, cnt = 0.0, 0
    for combo in itertools.product(range(len(mats)), repeat=k):
        P = np.eye(n)
        for c in combo:
            P = P @ mats[c]
        total += np.linalg.norm(P - Tu, "fro") ** 2
        cnt += 1
    want = (n - 1) * (1 / 3 - 2 / (3 * (n - 1))) ** k
    assert abs(total / cnt - want) < 1e-12
    assert want <= (n - 1) / 3 ** k + 1e-15


def test_expected_contraction_with_seeded_generator_n16():
    """Same expectation, Monte-Carlo with the oracle's own seeded permutations (L = 16)."""
    n, k, trials = 16, 3, 3000
    Tu = orc.uniform_matrix(n)
    vals = []
    for t in range(trials):
        P = np.eye(n)
        for j in range(k):
            P = P @ orc.mixing_matrix(orc.TOPO_RAND_RING, n, seed=5, step=t * k + j)
        vals.append(np.linalg.norm(P - Tu, "fro") ** 2)
    want = (n - 1) * ((n - 3) / (3 * (n - 1))) ** k
    se = np.std(vals) / math.sqrt(trials)
    assert abs(np.mean(vals) - want) < 5 * se


# ------------------------------------------------------------------ the update (Sec. 2, Eq. 2)
def _random_doubly_stochastic(n, rng, terms=5):
    """Convex combination of permutation matrices (Birkhoff): asymmetric in general."""
    c = rng.random(terms)
    c /= c.sum()
    T = np.zeros((n, n))
    for t in range(terms):
        T[np.arange(n), rng.permutation(n)] += c[t]
    return T


@pytest.mark.parametrize("n", [1, 2, 3, 5, 8, 16])
def test_mix_step_against_scalar_loops(n):
    """W_{k+1} = W_k T - alpha g evaluated entry by entry in the paper's column layout."""
    rng = np.random.default_rng(n)
    d = 7
    T = _random_doubly_stochastic(n, rng)
    X = rng.standard_normal((n, d)).astype(np.float32)
    G = rng.standard_normal((n, d)).astype(np.float32)
    lr = 0.3
    W, g = X.T.astype(np.float64), G.T.astype(np.float64)     # d x L, one column per learner
    a = float(np.float32(lr))
    want = np.zeros((d, n))
    for r in range(d):
        for l in range(n):
            s = 0.0
            for m in range(n):
                s += W[r, m] * T[m, l]
            want[r, l] = s - a * g[r, l]
    got = orc.mix_step(X, G, T, lr)
    assert np.allclose(got, want.T, rtol=0, atol=1e-14)


def test_mix_step_shift_matrix_orientation():
    """T[m, m+1] = 1: column l of W T is column l-1 of W, so learner l receives l-1's model."""
    n, d = 5, 3
    T = np.zeros((n, n))
    for m in range(n):
        T[m, (m + 1) % n] = 1.0
    X = np.arange(n * d, dtype=np.float32).reshape(n, d)
    out = orc.mix_step(X, np.zeros_like(X), T, 0.0)
    for l in range(n):
        assert np.array_equal(out[l], X[(l - 1) % n])


def test_n1_is_plain_sgd():
    """Sec. 2, Eq. 1: with one learner the update is w - alpha * gradient."""
    rng = np.random.default_rng(0)
    X = rng.standard_normal((1, 50)).astype(np.float32)
    G = rng.standard_normal((1, 50)).astype(np.float32)
    for topo in (orc.TOPO_RING, orc.TOPO_RAND_RING, orc.TOPO_FULL):
        out = orc.mix_step(X, G, orc.mixing_matrix(topo, 1, 1, 1), 0.25)
        assert np.array_equal(out, X.astype(np.float64) - 0.25 * G.astype(np.float64))


def test_uniform_matrix_gives_column_mean():
    """Sec. 2: S-PSGD's T_u replaces every learner's model by the average."""
    rng = np.random.default_rng(1)
    X = rng.standard_normal((9, 11)).astype(np.float32)
    out = orc.mix_step(X, np.zeros_like(X), orc.uniform_matrix(9), 0.1)
    mean = X.astype(np.float64).mean(axis=0)
    assert np.allclose(out, np.broadcast_to(mean, out.shape), atol=1e-15)


@pytest.mark.parametrize("topo", [orc.TOPO_RING, orc.TOPO_RAND_RING])
def test_consensus_state_is_fixed_point(topo):
    X = np.tile(np.linspace(-1, 1, 13, dtype=np.float32), (8, 1))
    out = orc.mix_step(X, np.ones_like(X), orc.mixing_matrix(topo, 8, 2, 3), 0.0)
    assert np.allclose(out, X, atol=1e-15)


@pytest.mark.parametrize("topo", [orc.TOPO_RING, orc.TOPO_RAND_RING, orc.TOPO_FULL])
def test_mean_recurrence(topo):
    """1^T T = 1^T, hence xbar_{k+1} = xbar_k - lr * gbar_k; lr = 0 preserves the mean."""
    rng = np.random.default_rng(2)
    n, d, lr = 16, 20, 0.05
    X = rng.standard_normal((n, d)).astype(np.float32)
    Gs = [rng.standard_normal((n, d)).astype(np.float32) for _ in range(6)]
    Ts = [orc.mixing_matrix(topo, n, 8, k) for k in range(6)]
    Xs = orc.run_steps(X, Gs, Ts, lr)
    a = float(np.float32(lr))
    for k in range(6):
        assert np.allclose(Xs[k + 1].mean(0), Xs[k].mean(0) - a * Gs[k].astype(np.float64).mean(0),
                           atol=1e-14)
    Xs0 = orc.run_steps(X, Gs, Ts, 0.0)
    assert np.allclose(Xs0[-1].mean(0), X.astype(np.float64).mean(0), atol=1e-14)


# ------------------------------------------------------------------ consensus distance
def test_consensus_closed_forms():
    assert orc.consensus_dist(np.tile(np.arange(5, dtype=np.float32), (7, 1))) == 0.0
    for n, d in [(1, 4), (2, 3), (8, 10), (64, 5), (128, 3)]:
        X = np.repeat(np.arange(n, dtype=np.float32)[:, None], d, axis=1)
        assert abs(orc.consensus_dist(X) - d * n * (n * n - 1) / 12) < 1e-9


def test_consensus_against_loops_and_shift_invariance():
    rng = np.random.default_rng(3)
    X = rng.standard_normal((6, 9)).astype(np.float32)
    want = 0.0
    for j in range(9):
        m = sum(float(X[i, j]) for i in range(6)) / 6
        for i in range(6):
            want += (float(X[i, j]) - m) ** 2
    assert abs(orc.consensus_dist(X) - want) < 1e-12
    # adding the same vector to every replica does not change the distance
    shift = rng.standard_normal(9)
    assert abs(orc.consensus_dist(X.astype(np.float64) + shift) - want) < 1e-12


@pytest.mark.parametrize("n", [4, 8, 16, 64])
@pytest.mark.parametrize("topo", [orc.TOPO_RING, orc.TOPO_RAND_RING])
def test_per_step_contraction_bound(n, topo):
    """Eq. 5 with k = 1 applies to every single (permuted) ring: at lr = 0,
    C_{k+1} <= rho^2 C_k deterministically."""
    rng = np.random.default_rng(n)
    X = rng.standard_normal((n, 40))
    rho = 1 / 3 + 2 / 3 * math.cos(2 * math.pi / n)
    C = orc.consensus_dist(X)
    for k in range(12):
        X = orc.mix_step(X, np.zeros_like(X), orc.mixing_matrix(topo, n, 11, k), 0.0)
        C2 = orc.consensus_dist(X)
        assert C2 <= rho * rho * C * (1 + 1e-9) + 1e-18   # n = 4 attains the bound
        C = C2


def test_expected_consensus_trajectory_random_ring():
    """Gaussian start, lr = 0: E C_k = d (n-1) sigma^2 ((n-3)/(3(n-1)))^k (from Eq. 11)."""
    n, d, sigma = 16, 200_000, 0.05
    X = inp.host_normal_f32((n, d), sigma, 123).astype(np.float64)
    lam = (n - 3) / (3 * (n - 1))
    C0 = orc.consensus_dist(X)
    assert abs(C0 / (d * (n - 1) * sigma ** 2) - 1) < 5e-3
    for k in range(1, 5):
        X = orc.mix_step(X, np.zeros_like(X), orc.mixing_matrix(orc.TOPO_RAND_RING, n, 77, k), 0.0)
    # a single realisation of k rings is not the expectation; average over ring draws instead
    vals = []
    X0 = inp.host_normal_f32((n, 20_000), sigma, 124).astype(np.float64)
    for trial in range(200):
        Y = X0
        for k in range(3):
            Y = orc.mix_step(Y, np.zeros_like(Y),
                             orc.mixing_matrix(orc.TOPO_RAND_RING, n, 500 + trial, k), 0.0)
        vals.append(orc.consensus_dist(Y))
    want = 20_000 * (n - 1) * sigma ** 2 * lam ** 3
    assert abs(np.mean(vals) / want - 1) < 5 * np.std(vals) / math.sqrt(200) / want + 5e-3


# ------------------------------------------------------------------ bf16 gradients
def test_bf16_widening_exact_and_path_equivalence():
    rng = np.random.default_rng(4)
    g32 = (rng.standard_normal((4, 64)) * 1e-3).astype(np.float32)
    bits = inp.f32_to_bf16_bits(g32)
    wide = orc.bf16_bits_to_f64(bits)
    # widening is exact: the fp32 with those top 16 bits and zero low bits
    back = (bits.astype(np.uint32) << 16).view(np.float32)
    assert np.array_equal(wide, back.astype(np.float64))
    assert np.all(np.abs(wide - g32) <= np.abs(g32) * 2.0 ** -8)
    X = rng.standard_normal((4, 64)).astype(np.float32)
    T = orc.ring_matrix(4)
    assert np.array_equal(orc.mix_step(X, bits, T, 0.05), orc.mix_step(X, back, T, 0.05))


def test_bf16_rounding_matches_torch_cpu():
    torch = pytest.importorskip("torch")
    a = inp.host_normal_f32((1000,), 1e-3, 5)
    a[:4] = np.array([1.0, 1.00390625, 1.01171875, -3.0e-40], dtype=np.float32)  # ties, subnormal
    want = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(inp.f32_to_bf16_bits(a), want)


# ------------------------------------------------------------------ delay-by-one (Sec. 4, Eq. 14)
def test_d1d_reduces_to_undelayed_when_pull_is_zero():
    rng = np.random.default_rng(6)
    n, d, K = 8, 12, 5
    X0 = rng.standard_normal((n, d)).astype(np.float32)
    noises = [rng.standard_normal((n, d)).astype(np.float32) for _ in range(K)]
    Ts = [orc.mixing_matrix(orc.TOPO_RAND_RING, n, 1, k) for k in range(K)]
    a = orc.d1d_trajectory(X0, noises, Ts, 0.1, 0.0)
    b = orc.run_steps(X0, noises, Ts, 0.1)
    for u, v in zip(a, b):
        assert np.array_equal(u, v)


def test_d1d_uses_previous_iterate_and_mean_recurrence():
    """G_k is evaluated at X_{k-1} (X_{-1} := X_0); the mean follows
    xbar_{k+1} = xbar_k - lr (c xbar_{k-1} + noisebar_k)."""
    rng = np.random.default_rng(7)
    n, d, K, lr, c = 8, 6, 6, 0.1, 0.5
    X0 = rng.standard_normal((n, d)).astype(np.float32)
    noises = [rng.standard_normal((n, d)).astype(np.float32) for _ in range(K)]
    Ts = [orc.mixing_matrix(orc.TOPO_RAND_RING, n, 2, k) for k in range(K)]
    Xs = orc.d1d_trajectory(X0, noises, Ts, lr, c)
    a = float(np.float32(lr))
    m_prev = Xs[0].mean(0)
    for k in range(K):
        want = Xs[k].mean(0) - a * (c * m_prev + noises[k].astype(np.float64).mean(0))
        assert np.allclose(Xs[k + 1].mean(0), want, atol=1e-14)
        m_prev = Xs[k].mean(0)
    # with zero noise and n = 1 it is the scalar recurrence x_{k+1} = x_k - lr c x_{k-1}
    x = [2.0, 2.0 - a * c * 2.0]
    for k in range(1, 5):
        x.append(x[k] - a * c * x[k - 1])
    Z = orc.d1d_trajectory(np.full((1, 1), 2.0, np.float32),
                           [np.zeros((1, 1), np.float32)] * 5, [np.eye(1)] * 5, lr, c)
    assert np.allclose([z[0, 0] for z in Z], x, atol=1e-14)


def _two_term_closed_form(lam, q, y0, k):
    """y_k of y_{k+1} = lam y_k - q y_{k-1} with y_{-1} = y_0, from the characteristic roots
    r^2 - lam r + q = 0 (textbook solution of a linear recurrence; complex roots allowed)."""
    disc = np.sqrt(complex(lam * lam - 4.0 * q))
    rp, rm = (lam + disc) / 2.0, (lam - disc) / 2.0
    # A + B = y0 ;  A / rp + B / rm = y0
    M = np.array([[1.0, 1.0], [1.0 / rp, 1.0 / rm]])
    A, B = np.linalg.solve(M, np.array([1.0, 1.0], dtype=complex))
    return ((A * rp ** k + B * rm ** k) * y0).real


def test_d1d_fixed_ring_modes_follow_characteristic_roots():
    """Noise-free delayed trajectory on the fixed ring: T_0 is symmetric, so in its eigenbasis
    every mode obeys the scalar recurrence y_{k+1} = lambda_j y_k - lr c y_{k-1} (Eq. 14 with a
    linear gradient), whose solution is a combination of powers of the two characteristic
    roots.  Independent of the oracle's step-by-step iteration."""
    rng = np.random.default_rng(11)
    n, d, K, lr, c = 8, 5, 14, 0.1, 0.7
    T = orc.ring_matrix(n)
    lam, V = np.linalg.eigh(T)
    X0 = rng.standard_normal((n, d)).astype(np.float32)
    zeros = [np.zeros((n, d), np.float32)] * K
    Xs = orc.d1d_trajectory(X0, zeros, [T] * K, lr, c)
    q = float(np.float32(lr)) * float(np.float32(c))
    Y0 = V.T @ X0.astype(np.float64)
    for k in (1, 2, 3, 7, 14):
        Yk = np.stack([_two_term_closed_form(lam[j], q, Y0[j], k) for j in range(n)])
        assert np.allclose(Xs[k], V @ Yk, atol=1e-12), k
    # an undelayed gradient (evaluated at X_k) gives y_k = (lambda - q)^k y_0 instead: the two differ
    Yk_undelayed = np.stack([(lam[j] - q) ** 7 * Y0[j] for j in range(n)])
    assert not np.allclose(Xs[7], V @ Yk_undelayed, atol=1e-6)


def test_d1d_with_global_averaging_closed_form():
    """The paper's own delay-by-one (Eq. 13, 14): T_u averages fully, so after one step every
    disagreement comes from the stale gradient alone: with G = c X_{k-1} and no noise the
    deviations obey v_{k+1} = -lr c v_{k-1}, hence C_k = (lr c)^(2 ceil(k/2)) C_0, and the mean
    obeys the two-term recurrence with lambda = 1."""
    rng = np.random.default_rng(12)
    n, d, K, lr, c = 6, 7, 9, 0.25, 0.9
    X0 = rng.standard_normal((n, d)).astype(np.float32)
    Tu = orc.uniform_matrix(n)
    Xs = orc.d1d_trajectory(X0, [np.zeros((n, d), np.float32)] * K, [Tu] * K, lr, c)
    q = float(np.float32(lr)) * float(np.float32(c))
    C0 = orc.consensus_dist(X0)
    m0 = X0.astype(np.float64).mean(0)
    for k in range(1, K + 1):
        assert np.isclose(orc.consensus_dist(Xs[k]), q ** (2 * ((k + 1) // 2)) * C0, rtol=1e-10, atol=0)
        assert np.allclose(Xs[k].mean(0), _two_term_closed_form(1.0, q, m0, k), atol=1e-12)
    # The trajectory is linear in (X_0, noise): response to noise alone, one impulse at step j.
    # X_{j+1} = -lr e; its deviations then return every second step scaled by -lr c:
    # C_{j+1+2m} = (lr c)^(2m) lr^2 C(e), and C_{j+2+2m} = 0.
    j = 2
    e = rng.standard_normal((n, d)).astype(np.float32)
    noises = [np.zeros((n, d), np.float32) for _ in range(K)]
    noises[j] = e
    Zs = orc.d1d_trajectory(np.zeros((n, d), np.float32), noises, [Tu] * K, lr, c)
    a = float(np.float32(lr))
    Ce = orc.consensus_dist(e)
    for k in range(K + 1):
        if k <= j:
            want = 0.0
        elif (k - j - 1) % 2 == 0:
            want = q ** (k - j - 1) * a * a * Ce
        else:
            want = 0.0
        assert np.isclose(orc.consensus_dist(Zs[k]), want, rtol=1e-10, atol=1e-24), k
    both = orc.d1d_trajectory(X0, noises, [Tu] * K, lr, c)
    for k in range(K + 1):
        assert np.allclose(both[k], Xs[k] + Zs[k], atol=1e-13)           # superposition


def test_d1d_planted_mistakes_are_caught():
    """Mutants of the delayed driver, planted on the CPU, against the closed form above."""
    def closed_form_violations(traj):
        n, d, K, lr, c = 6, 4, 6, 0.25, 0.9
        X0 = np.random.default_rng(13).standard_normal((n, d)).astype(np.float32)
        Tu = orc.uniform_matrix(n)
        Xs = traj(X0, [np.zeros((n, d), np.float32)] * K, [Tu] * K, lr, c)
        q = float(np.float32(lr)) * float(np.float32(c))
        C0 = orc.consensus_dist(X0)
        return sum(not np.isclose(orc.consensus_dist(Xs[k]), q ** (2 * ((k + 1) // 2)) * C0, rtol=1e-10, atol=0)
                   for k in range(1, K + 1))

    def no_delay(X0, noises, Ts, lr, c):            # gradient at the current iterate
        Xs = [X0.astype(np.float64)]
        for k, T in enumerate(Ts):
            Xs.append(orc.mix_step(Xs[-1], orc.synth_grad(Xs[-1], noises[k], c), T, lr))
        return Xs

    def two_step_delay(X0, noises, Ts, lr, c):      # gradient two iterates back
        Xs = [X0.astype(np.float64)]
        for k, T in enumerate(Ts):
            Xs.append(orc.mix_step(Xs[-1], orc.synth_grad(Xs[max(k - 2, 0)], noises[k], c), T, lr))
        return Xs

    def first_step_without_gradient(X0, noises, Ts, lr, c):   # X_{-1} := 0 instead of X_0
        Xs = [X0.astype(np.float64)]
        prev = np.zeros_like(Xs[0])
        for k, T in enumerate(Ts):
            nxt = orc.mix_step(Xs[-1], orc.synth_grad(prev, noises[k], c), T, lr)
            prev = Xs[-1]
            Xs.append(nxt)
        return Xs

    assert closed_form_violations(orc.d1d_trajectory) == 0
    for mutant in (no_delay, two_step_delay, first_step_without_gradient):
        assert closed_form_violations(mutant) > 0, mutant.__name__


# ------------------------------------------------------------------ planted mistakes
def _pins_for_mix(mix):
    """A bundle of the checks above, run against a candidate mix function.  Returns the
    number of pins it violates."""
    bad = 0
    rng = np.random.default_rng(8)
    n, d = 5, 3
    T = np.zeros((n, n))
    for m in range(n):
        T[m, (m + 1) % n] = 1.0
    X = np.arange(n * d, dtype=np.float32).reshape(n, d)
    out = mix(X, np.zeros_like(X), T, 0.0)
    bad += not all(np.array_equal(out[l], X[(l - 1) % n]) for l in range(n))
    X = rng.standard_normal((1, 9)).astype(np.float32)
    G = rng.standard_normal((1, 9)).astype(np.float32)
    bad += not np.allclose(mix(X, G, np.eye(1), 0.25), X.astype(np.float64) - 0.25 * G, atol=1e-14)
    X = rng.standard_normal((6, 9)).astype(np.float32)
    G = rng.standard_normal((6, 9)).astype(np.float32)
    out = mix(X, G, orc.ring_matrix(6), 0.5)
    bad += not np.allclose(out.mean(0), X.astype(np.float64).mean(0) - 0.5 * G.astype(np.float64).mean(0),
                           atol=1e-14)
    want0 = (X[5].astype(np.float64) + X[0] + X[1]) / 3 - 0.5 * G[0]
    bad += not np.allclose(out[0], want0, atol=1e-14)
    return bad


def test_planted_mistakes_are_caught():
    """Mutants of the update (planted on the CPU): each must trip at least one pin."""
    assert _pins_for_mix(orc.mix_step) == 0
    mutants = {
        "untransposed": lambda X, G, T, lr: T @ X.astype(np.float64) - lr * G.astype(np.float64),
        "wrong_sign": lambda X, G, T, lr: T.T @ X.astype(np.float64) + lr * G.astype(np.float64),
        "no_gradient": lambda X, G, T, lr: T.T @ X.astype(np.float64),
        "lr_on_mix": lambda X, G, T, lr: lr * (T.T @ X.astype(np.float64)) - G.astype(np.float64),
        "dropped_neighbour": lambda X, G, T, lr: np.triu(T).T @ X.astype(np.float64) - lr * G.astype(np.float64),
    }
    for name, m in mutants.items():
        assert _pins_for_mix(m) > 0, name


# ------------------------------------------------------------------ slot table -> dense matrix
def _pins_for_densify(densify):
    """Orientation pins for the table form of T (Sec. 2, Eq. 2: W T, so column i of T holds the weights
    of the models that feed learner i, and row i of the table lists exactly that column).  Every table
    here is asymmetric and typed out, so a transposed assignment cannot pass.  Returns the violations."""
    bad = 0
    # one slot, learner i takes the model of learner i - 1: the cyclic shift T[m, m+1] = 1
    n = 5
    nbr = np.array([[(i - 1) % n] for i in range(n)], dtype=np.int32)
    w = np.ones((n, 1), dtype=np.float32)
    shift = np.array([
        [0, 1, 0, 0, 0],
        [0, 0, 1, 0, 0],
        [0, 0, 0, 1, 0],
        [0, 0, 0, 0, 1],
        [1, 0, 0, 0, 0],
    ], dtype=np.float64)
    T = densify(nbr, w)
    bad += not np.array_equal(T, shift)
    X = np.arange(n * 3, dtype=np.float32).reshape(n, 3)
    out = orc.mix_step(X, np.zeros_like(X), T, 0.0)
    bad += not all(np.array_equal(out[l], X[(l - 1) % n]) for l in range(n))
    # two slots, weights 3/4 and 1/4 (exact in fp32), doubly stochastic but not symmetric:
    # learner 0 <- 3/4 x_0 + 1/4 x_2, learner 1 <- 3/4 x_1 + 1/4 x_0, learner 2 <- 3/4 x_2 + 1/4 x_1
    nbr2 = np.array([[0, 2], [1, 0], [2, 1]], dtype=np.int32)
    w2 = np.array([[0.75, 0.25]] * 3, dtype=np.float32)
    want2 = np.array([
        [0.75, 0.25, 0.00],     # row m = what learner m's model contributes to learners 0, 1, 2
        [0.00, 0.75, 0.25],
        [0.25, 0.00, 0.75],
    ])
    T2 = densify(nbr2, w2)
    bad += not np.array_equal(T2, want2)
    X2 = np.array([[1.0, 10.0], [2.0, 20.0], [4.0, 40.0]], dtype=np.float32)
    out2 = orc.mix_step(X2, np.zeros_like(X2), T2, 0.0)
    bad += not np.array_equal(out2, np.array([[1.75, 17.5], [1.75, 17.5], [3.5, 35.0]]))
    # a row whose slots repeat a learner adds the shares (the n = 2 ring: self 1/3, other 2/3)
    T3 = densify(np.array([[0, 1, 1], [1, 0, 0]], dtype=np.int32), np.full((2, 3), 0.25, dtype=np.float32))
    bad += not np.array_equal(T3, np.array([[0.25, 0.5], [0.5, 0.25]]))
    # unequal weights inside one row stay with their slot: learner 0 <- 1/2 x_1 + 1/2 x_2 only
    nbr4 = np.array([[1, 2], [0, 1], [2, 0]], dtype=np.int32)
    w4 = np.array([[0.5, 0.5], [0.5, 0.5], [0.5, 0.5]], dtype=np.float32)
    want4 = np.array([
        [0.0, 0.5, 0.5],
        [0.5, 0.5, 0.0],
        [0.5, 0.0, 0.5],
    ])
    bad += not np.array_equal(densify(nbr4, w4), want4)
    return bad


def test_densify_orientation_on_asymmetric_tables():
    assert _pins_for_densify(orc.densify) == 0


def test_densify_agrees_with_table_gather_on_random_asymmetric_tables():
    """Row i of the table is what learner i receives: the gather-add sum_s w[i,s] x[nbr[i,s]] written as
    scalar loops must equal the dense product with densify's matrix, for tables built from random
    permutations (slot s of every row comes from one permutation, so T is doubly stochastic, asymmetric)."""
    rng = np.random.default_rng(21)
    for n, deg in [(4, 2), (7, 3), (9, 5)]:
        nbr = np.stack([rng.permutation(n) for _ in range(deg)], axis=1).astype(np.int32)
        c = rng.random(deg)
        w = np.tile((c / c.sum()).astype(np.float32), (n, 1))
        T = orc.densify(nbr, w)
        assert not np.allclose(T, T.T)
        assert np.allclose(T.sum(0), T.sum(1)) and np.allclose(T.sum(0), float(w[0].astype(np.float64).sum()))
        X = rng.standard_normal((n, 4)).astype(np.float32)
        want = np.zeros((n, 4))
        for i in range(n):
            for s in range(deg):
                for j in range(4):
                    want[i, j] += float(w[i, s]) * float(X[nbr[i, s], j])
        assert np.allclose(orc.mix_step(X, np.zeros_like(X), T, 0.0), want, rtol=0, atol=1e-15)


def test_densify_planted_mistakes_are_caught():
    def transposed(nbr, w):
        return orc.densify(nbr, w).T

    def duplicates_overwrite(nbr, w):
        nbr, w = np.asarray(nbr), np.asarray(w)
        T = np.zeros((nbr.shape[0],) * 2)
        for i in range(nbr.shape[0]):
            for s in range(nbr.shape[1]):
                T[int(nbr[i, s]), i] = float(w[i, s])
        return T

    def last_slot_dropped(nbr, w):
        nbr, w = np.asarray(nbr), np.asarray(w)
        return orc.densify(nbr[:, :max(nbr.shape[1] - 1, 1)], w[:, :max(nbr.shape[1] - 1, 1)])

    for name, m in {"transposed": transposed, "duplicates_overwrite": duplicates_overwrite,
                    "last_slot_dropped": last_slot_dropped}.items():
        assert _pins_for_densify(m) > 0, name


# ------------------------------------------------------------------ sparse C form of the update
def test_sparse_step_typed_out_example():
    """Sec. 2, Eq. 2 on the asymmetric 3/4-1/4 table, by hand: learner 0 <- 3/4 x_0 + 1/4 x_2, and so on,
    minus lr times the gradient (lr = 1/2, exact in fp32)."""
    nbr = np.array([[0, 2], [1, 0], [2, 1]], dtype=np.int32)
    w = np.array([[0.75, 0.25]] * 3, dtype=np.float32)
    X = np.array([[1.0, 10.0], [2.0, 20.0], [4.0, 40.0]], dtype=np.float32)
    G = np.array([[2.0, 0.0], [0.0, 4.0], [-2.0, 8.0]], dtype=np.float32)
    want = np.array([[1.75 - 1.0, 17.5], [1.75, 17.5 - 2.0], [3.5 + 1.0, 35.0 - 4.0]])
    assert np.array_equal(orc.sparse_mix_step(X, G, nbr, w, 0.5), want)
    assert np.array_equal(orc.sparse_mix_step(X, G, nbr, w, 0.5, threads=4), want)


@pytest.mark.parametrize("n,deg,d", [(1, 3, 5), (2, 3, 9), (5, 1, 4097), (8, 3, 10000), (16, 5, 8200), (64, 3, 5000)])
@pytest.mark.parametrize("gkind", ["f32", "bf16"])
def test_sparse_step_equals_dense_oracle(n, deg, d, gkind):
    """The gather-add in C against the dense product T^T X - lr G (itself pinned above) on random asymmetric
    tables and on the ring tables, one and several threads, ragged column counts."""
    rng = np.random.default_rng(100 * n + deg)
    X = rng.standard_normal((n, d)).astype(np.float32)
    G = rng.standard_normal((n, d)).astype(np.float32)
    if gkind == "bf16":
        G = inp.f32_to_bf16_bits(G)
    if deg == 3:
        nbr, w = orc.neighbour_table(orc.TOPO_RAND_RING, n, 5, n)
    else:
        nbr = np.stack([rng.permutation(n) for _ in range(deg)], axis=1).astype(np.int32)
        c = rng.random(deg)
        w = np.tile((c / c.sum()).astype(np.float32), (n, 1))
    want = orc.mix_step(X, G, orc.densify(nbr, w), 0.3)
    for threads in (1, 3):
        got = orc.sparse_mix_step(X, G, nbr, w, 0.3, threads=threads)
        assert np.allclose(got, want, rtol=0, atol=1e-14 * max(1.0, np.abs(want).max()))
    assert abs(orc.sparse_consensus_dist(want, threads=2) - orc.consensus_dist(want)) <= 1e-12 * orc.consensus_dist(want) + 1e-300


def test_sparse_step_planted_mistake_is_caught():
    """Reading the table the other way round (learner i SENDS to nbr[i, s]) is the transposed matrix: the
    typed-out example above tells them apart."""
    nbr = np.array([[0, 2], [1, 0], [2, 1]], dtype=np.int32)
    w = np.array([[0.75, 0.25]] * 3, dtype=np.float32)
    X = np.array([[1.0, 10.0], [2.0, 20.0], [4.0, 40.0]], dtype=np.float32)
    Z = np.zeros_like(X)
    right = orc.sparse_mix_step(X, Z, nbr, w, 0.0)
    wrong = orc.mix_step(X, Z, orc.densify(nbr, w).T, 0.0)
    assert not np.array_equal(right, wrong)
    assert np.array_equal(right, np.array([[1.75, 17.5], [1.75, 17.5], [3.5, 35.0]]))


def test_golden_tables_still_match_oracle(golden_dir):
    """The frozen tables were written by the oracle; a drift in its generator shows here."""
    with open(os.path.join(golden_dir, "mixing_tables.txt")) as f:
        lines = [l for l in f if l.strip() and not l.startswith("#")]
    assert len(lines) >= 10
    for line in lines:
        head, rest = line.split(":")
        n, seed, step = (int(x) for x in head.split())
        sig_s, nbr_s = rest.split("|")
        assert orc.permutation(n, seed, step) == [int(x) for x in sig_s.split()]
        nbr, _ = orc.neighbour_table(orc.TOPO_RAND_RING, n, seed, step)
        assert [int(v) for v in nbr.reshape(-1)] == [int(x) for x in nbr_s.split()]
