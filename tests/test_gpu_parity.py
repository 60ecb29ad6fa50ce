"""GPU parity: the HIP library against the CPU oracle, element by element, on seeded inputs.

Tolerances (stated by the baseline: relative 1e-6 with fp32 accumulation).  One step does
four fp32 roundings on partial sums bounded by ||X||_inf + lr ||G||_inf, so the absolute
error per element is at most 4 * 2^-24 * that bound = 2.4e-7 of the largest magnitude.
"Relative" is therefore taken against the largest output magnitude (element-wise relative
error is unbounded where an output is near zero), plus the Frobenius-norm ratio.
"""
import numpy as np
import pytest

from oracle import psgd_oracle as orc
from paper_2002_01119_amd import inputs as inp

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

REL = 1e-6


@pytest.fixture(scope="module")
def psgd():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2002_01119_amd import psgd as m
    m.load()          # raises if the HIP library is not built: no fallback
    torch.cuda.set_device(0)
    return m


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def bits_dev(bits_u16):
    return torch.from_numpy(bits_u16.view(np.int16)).to("cuda:0")


def assert_close(got, want, rel=REL):
    got = np.asarray(got, dtype=np.float64)
    scale = max(np.abs(want).max(), 1e-30)
    err = np.abs(got - want).max()
    assert err <= rel * scale, "max abs err %.3g vs scale %.3g" % (err, scale)
    fro = np.linalg.norm(want)
    if fro > 0:
        assert np.linalg.norm(got - want) <= rel * fro


def run_step(psgd, X, G, nbr, w, lr, in_place=False, delay_mode=0):
    Xd = dev(X)
    Gd = bits_dev(G) if G.dtype == np.uint16 else dev(G)
    out = Xd if in_place else torch.full_like(Xd, float("nan"))
    psgd.mix_step(Xd, out, Gd, dev(nbr), dev(w), lr, delay_mode=delay_mode)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def _pitched_views(n, d, pitch, g_bf16):
    """X, X_out and G as interleaved row-pitched views of ONE pool: row i of X at i*pitch,
    of X_out right behind it, of G behind that (pitch in fp32 elements)."""
    pool = torch.zeros(n * pitch + 8, dtype=torch.float32, device="cuda:0")
    X = pool.as_strided((n, d), (pitch, 1), 0)
    Y = pool.as_strided((n, d), (pitch, 1), d)
    if g_bf16:
        gp = pool.view(torch.int16)
        G = gp.as_strided((n, d), (2 * pitch, 1), 4 * d)
    else:
        G = pool.as_strided((n, d), (pitch, 1), 2 * d)
    return pool, X, Y, G


SHAPES = [(1, 1), (1, 1000), (2, 5), (3, 4), (4, 7), (5, 1024), (8, 4100), (8, 70001),
          (16, 3 * 1024 * 4 + 4), (33, 2052), (64, 9 * 1024 + 8), (128, 4096 + 12), (512, 260)]


@pytest.mark.parametrize("n,d", SHAPES)
@pytest.mark.parametrize("topo", [orc.TOPO_RING, orc.TOPO_RAND_RING])
@pytest.mark.parametrize("gkind", ["f32", "bf16"])
def test_single_step_matches_oracle(psgd, n, d, topo, gkind):
    X = inp.host_normal_f32((n, d), 1.0, 100 + n)
    G = inp.host_normal_f32((n, d), 0.5, 200 + n)
    if gkind == "bf16":
        G = inp.f32_to_bf16_bits(G)
    nbr, w = psgd.build_mixing(topo, n, seed=9, step=n + d)
    want = orc.mix_step(X, G, orc.densify(nbr, w), 0.1)
    got = run_step(psgd, X, G, nbr, w, 0.1)
    assert not np.isnan(got).any()
    assert_close(got, want)
    got_ip = run_step(psgd, X, G, nbr, w, 0.1, in_place=True)
    assert np.array_equal(got_ip.view(np.uint32), got.view(np.uint32))     # same kernel, same bits
    got_d1 = run_step(psgd, X, G, nbr, w, 0.1, delay_mode=1)
    assert np.array_equal(got_d1.view(np.uint32), got.view(np.uint32))
    assert psgd.device_status() == 0


def test_exact_fp32_operation_order(psgd):
    """The header fixes the fp32 operation order; reproduce it with numpy fp32 scalars
    (fma emulated in fp64, which is exact for one fp32 product plus one addend up to the
    final rounding) and demand bit equality."""
    n, d = 8, 515
    X = inp.host_normal_f32((n, d), 1.0, 1)
    G = inp.host_normal_f32((n, d), 1.0, 2)
    nbr, w = psgd.build_mixing(psgd.TOPO_RAND_RING, n, 5, 5)
    lr = np.float32(0.05)
    got = run_step(psgd, X, G, nbr, w, float(lr))

    def fma32(a, b, c):
        return (a.astype(np.float64) * b.astype(np.float64) + c.astype(np.float64)).astype(np.float32)

    want = np.empty_like(X)
    for i in range(n):
        acc = (X[nbr[i, 0]] * w[i, 0]).astype(np.float32)
        acc = fma32(np.broadcast_to(w[i, 1], (d,)), X[nbr[i, 1]], acc)
        acc = fma32(np.broadcast_to(w[i, 2], (d,)), X[nbr[i, 2]], acc)
        want[i] = fma32(np.broadcast_to(-lr, (d,)), G[i], acc)
    # double rounding in the emulation can differ from a true fma in rare ties: allow 1 ulp
    # on a handful of elements, bit equality on the rest
    diff = np.abs(got.view(np.int32).astype(np.int64) - want.view(np.int32).astype(np.int64))
    assert diff.max() <= 1 and (diff > 0).mean() < 1e-3


def _general_table(n, rng, weights=(0.5, 0.3, 0.2)):
    """A doubly stochastic 3-slot table that is not a ring: w0 I + w1 P1 + w2 P2."""
    p1, p2 = rng.permutation(n), rng.permutation(n)
    nbr = np.stack([np.arange(n), p1, p2], axis=1).astype(np.int32)
    w = np.tile(np.asarray(weights, dtype=np.float32), (n, 1))
    return nbr, w


@pytest.mark.parametrize("n,d", [(4, 9), (6, 2048), (16, 4 * 3000), (64, 1025), (128, 8192 + 4), (300, 516)])
@pytest.mark.parametrize("gkind", ["f32", "bf16"])
def test_general_tables_use_the_tiled_path(psgd, n, d, gkind):
    rng = np.random.default_rng(n * 7 + d)
    nbr, w = _general_table(n, rng)
    T = orc.densify(nbr, w)
    assert np.allclose(T.sum(0), 1, atol=1e-6) and np.allclose(T.sum(1), 1, atol=1e-6)
    X = inp.host_normal_f32((n, d), 1.0, 300 + n)
    G = inp.host_normal_f32((n, d), 0.5, 400 + n)
    if gkind == "bf16":
        G = inp.f32_to_bf16_bits(G)
    want = orc.mix_step(X, G, T, 0.2)
    got = run_step(psgd, X, G, nbr, w, 0.2)
    assert_close(got, want)
    got_ip = run_step(psgd, X, G, nbr, w, 0.2, in_place=True)
    assert np.array_equal(got_ip.view(np.uint32), got.view(np.uint32))


def test_two_disjoint_rings_and_self_loops(psgd):
    """Locally consistent left/right pointers that do not form ONE ring must not take the
    ring walk: two rings of 4, and the all-self table (identity mixing)."""
    n, d = 8, 1030
    nbr = np.zeros((n, 3), np.int32)
    for base in (0, 4):
        for k in range(4):
            i = base + k
            nbr[i] = (i, base + (k - 1) % 4, base + (k + 1) % 4)
    w = np.full((n, 3), 1 / 3, np.float32)
    X = inp.host_normal_f32((n, d), 1.0, 31)
    G = inp.host_normal_f32((n, d), 1.0, 32)
    assert_close(run_step(psgd, X, G, nbr, w, 0.1), orc.mix_step(X, G, orc.densify(nbr, w), 0.1))
    ident = np.repeat(np.arange(n, dtype=np.int32)[:, None], 3, axis=1)
    assert_close(run_step(psgd, X, G, ident, w, 0.1), orc.mix_step(X, G, orc.densify(ident, w), 0.1))


def test_ring_with_per_row_weights(psgd):
    """The ring walk carries each row's own three weights (a lazy-walk style table)."""
    n, d = 16, 2056
    nbr, _ = psgd.build_mixing(psgd.TOPO_RAND_RING, n, 1, 2)
    rng = np.random.default_rng(5)
    w = rng.random((n, 3)).astype(np.float32)
    X = inp.host_normal_f32((n, d), 1.0, 41)
    G = inp.host_normal_f32((n, d), 1.0, 42)
    assert_close(run_step(psgd, X, G, nbr, w, 0.3), orc.mix_step(X, G, orc.densify(nbr, w), 0.3))


def test_out_of_range_table_is_flagged_and_writes_nothing(psgd):
    n, d = 8, 4096
    nbr, w = psgd.build_mixing(psgd.TOPO_RING, n)
    nbr = nbr.copy()
    nbr[3, 2] = n            # one past the end
    X = inp.host_normal_f32((n, d), 1.0, 51)
    G = inp.host_normal_f32((n, d), 1.0, 52)
    assert psgd.device_status() == 0
    out = run_step(psgd, X, G, nbr, w, 0.1)
    assert np.isnan(out).all()
    assert psgd.device_status(clear=True) == 1
    assert psgd.device_status() == 0
    nbr[3, 2] = -1
    out = run_step(psgd, X, G, nbr, w, 0.1)
    assert np.isnan(out).all() and psgd.device_status(clear=True) == 1


def test_binding_reports_alias_errors(psgd):
    X = torch.zeros(4, 64, device="cuda:0")
    G = torch.zeros(4, 64, device="cuda:0")
    nbr, w = psgd.build_mixing(psgd.TOPO_RING, 4)
    with pytest.raises(psgd.PsgdError) as e:
        psgd.mix_step(X, X, G, dev(nbr), dev(w), 0.1, delay_mode=1)
    assert e.value.code == psgd.EALIAS
    with pytest.raises(psgd.PsgdError):
        psgd.mix_step(X, G, G, dev(nbr), dev(w), 0.1)
    psgd.mix_step(X, X, G, dev(nbr), dev(w), 0.1, delay_mode=0)
    torch.cuda.synchronize()


def test_misaligned_views_take_the_scalar_path(psgd):
    """Buffers that are only 4-byte aligned (and 2-byte for bf16) must still be right."""
    n, d = 8, 1001
    X = inp.host_normal_f32((n, d), 1.0, 61)
    G = inp.host_normal_f32((n, d), 1.0, 62)
    Gb = inp.f32_to_bf16_bits(G)
    nbr, w = psgd.build_mixing(psgd.TOPO_RAND_RING, n, 4, 4)
    pad = torch.zeros(n * d + 1, device="cuda:0")
    pad[1:] = dev(X).reshape(-1)
    Xv = pad[1:].view(n, d)
    assert Xv.data_ptr() % 16 == 4
    out = torch.empty(n * d + 3, device="cuda:0")[3:].view(n, d)
    gpad = torch.zeros(n * d + 1, dtype=torch.int16, device="cuda:0")
    gpad[1:] = bits_dev(Gb).reshape(-1)
    Gv = gpad[1:].view(n, d)
    psgd.mix_step(Xv, out, Gv, dev(nbr), dev(w), 0.1)
    torch.cuda.synchronize()
    assert_close(out.cpu().numpy(), orc.mix_step(X, Gb, orc.densify(nbr, w), 0.1))


# ------------------------------------------------------------------------- consensus distance
@pytest.mark.parametrize("n,d", [(1, 10), (2, 1), (3, 5), (8, 4096), (8, 70001), (16, 12 * 1024 + 4),
                                 (64, 50_000), (128, 10_004), (17, 1023), (512, 300)])
def test_consensus_matches_oracle(psgd, n, d):
    X = inp.host_normal_f32((n, d), 0.05, 500 + n)
    want = orc.consensus_dist(X)
    got = psgd.consensus_dist(dev(X))
    assert abs(got - want) <= REL * max(want, 1e-300)
    out = torch.zeros(1, dtype=torch.float64, device="cuda:0")
    psgd.consensus_dist_async(dev(X), out)
    torch.cuda.synchronize()
    assert out.item() == got            # same kernels, fixed reduction order


def test_consensus_closed_forms_and_offsets(psgd):
    assert psgd.consensus_dist(dev(np.tile(np.arange(1000, dtype=np.float32), (7, 1)))) == 0.0
    for n, d in [(2, 3), (8, 1000), (64, 4096), (128, 1001)]:
        X = np.repeat(np.arange(n, dtype=np.float32)[:, None], d, axis=1)
        assert psgd.consensus_dist(dev(X)) == d * n * (n * n - 1) / 12
    # replicas that sit far from the origin but close to each other: a one-pass sum of
    # squares in fp32 would lose everything here
    base = inp.host_normal_f32((1, 5000), 100.0, 71)
    X = (base + inp.host_normal_f32((16, 5000), 1e-3, 72)).astype(np.float32)
    want = orc.consensus_dist(X)
    assert abs(psgd.consensus_dist(dev(X)) - want) <= REL * want
    # an outlier in the pivot row (row 0)
    X = inp.host_normal_f32((32, 3000), 1.0, 73)
    X[0] += 1000.0
    want = orc.consensus_dist(X)
    assert abs(psgd.consensus_dist(dev(X)) - want) <= REL * want


def test_consensus_is_reproducible(psgd):
    X = dev(inp.host_normal_f32((64, 300_000), 0.02, 81))
    vals = {psgd.consensus_dist(X) for _ in range(5)}
    assert len(vals) == 1


# ------------------------------------------------------------------------- fused step + distance
def run_step_cd(psgd, X, G, nbr, w, lr, in_place=False):
    Xd = dev(X)
    Gd = bits_dev(G) if G.dtype == np.uint16 else dev(G)
    out = Xd if in_place else torch.full_like(Xd, float("nan"))
    c = torch.full((1,), float("nan"), dtype=torch.float64, device="cuda:0")
    psgd.mix_step(Xd, out, Gd, dev(nbr), dev(w), lr, cdist_out=c)
    torch.cuda.synchronize()
    return out.cpu().numpy(), c.item()


@pytest.mark.parametrize("n,d", SHAPES)
@pytest.mark.parametrize("topo", [orc.TOPO_RING, orc.TOPO_RAND_RING])
@pytest.mark.parametrize("gkind", ["f32", "bf16"])
def test_fused_step_and_distance_match_oracle(psgd, n, d, topo, gkind):
    X = inp.host_normal_f32((n, d), 1.0, 600 + n)
    G = inp.host_normal_f32((n, d), 0.5, 700 + n)
    if gkind == "bf16":
        G = inp.f32_to_bf16_bits(G)
    nbr, w = psgd.build_mixing(topo, n, seed=19, step=n + d)
    want = orc.mix_step(X, G, orc.densify(nbr, w), 0.1)
    got, c = run_step_cd(psgd, X, G, nbr, w, 0.1)
    assert np.array_equal(got.view(np.uint32), run_step(psgd, X, G, nbr, w, 0.1).view(np.uint32))
    assert_close(got, want)
    # the distance is that of the fp32 array the kernel wrote
    c_ref = orc.consensus_dist(got)
    assert abs(c - c_ref) <= REL * c_ref + 1e-300
    assert abs(c - orc.consensus_dist(want)) <= 1e-5 * c_ref + 1e-300
    got_ip, c_ip = run_step_cd(psgd, X, G, nbr, w, 0.1, in_place=True)
    assert np.array_equal(got_ip.view(np.uint32), got.view(np.uint32)) and c_ip == c


@pytest.mark.parametrize("n,d", [(4, 9), (6, 2048), (16, 4 * 3000), (64, 1025), (128, 8192 + 4), (300, 516)])
@pytest.mark.parametrize("gkind", ["f32", "bf16"])
def test_fused_distance_on_general_tables(psgd, n, d, gkind):
    rng = np.random.default_rng(n * 11 + d)
    nbr, w = _general_table(n, rng)
    X = inp.host_normal_f32((n, d), 1.0, 800 + n)
    G = inp.host_normal_f32((n, d), 0.5, 900 + n)
    if gkind == "bf16":
        G = inp.f32_to_bf16_bits(G)
    got, c = run_step_cd(psgd, X, G, nbr, w, 0.2)
    assert_close(got, orc.mix_step(X, G, orc.densify(nbr, w), 0.2))
    c_ref = orc.consensus_dist(got)
    assert abs(c - c_ref) <= REL * c_ref
    got_ip, c_ip = run_step_cd(psgd, X, G, nbr, w, 0.2, in_place=True)
    assert np.array_equal(got_ip.view(np.uint32), got.view(np.uint32)) and c_ip == c


def test_fused_distance_special_cases(psgd):
    # outputs far from the origin and close together (large common gradient)
    n, d = 16, 5000
    X = np.tile(inp.host_normal_f32((1, d), 1.0, 1), (n, 1)) + inp.host_normal_f32((n, d), 1e-4, 2)
    G = np.full((n, d), 1000.0, np.float32)
    nbr, w = psgd.build_mixing(psgd.TOPO_RAND_RING, n, 1, 1)
    got, c = run_step_cd(psgd, X.astype(np.float32), G, nbr, w, 1.0)
    c_ref = orc.consensus_dist(got)
    assert abs(c - c_ref) <= REL * c_ref
    # invalid table: nothing written, distance NaN, flag raised
    bad = nbr.copy()
    bad[0, 1] = 99
    got, c = run_step_cd(psgd, X.astype(np.float32), G, bad, w, 1.0)
    assert np.isnan(got).all() and np.isnan(c) and psgd.device_status(clear=True) == 1
    # zero columns: distance 0
    bufs = [torch.zeros(16, device="cuda:0") for _ in range(3)]
    cz = torch.full((1,), 5.0, dtype=torch.float64, device="cuda:0")
    n4, w4 = psgd.build_mixing(psgd.TOPO_RING, 4)
    n4d, w4d = dev(n4), dev(w4)
    rc = psgd.load().psgd_mix_step_cd(bufs[0].data_ptr(), bufs[1].data_ptr(), bufs[2].data_ptr(), n4d.data_ptr(),
                                      w4d.data_ptr(), 4, 0, 0.1, 0, cz.data_ptr(), None)
    torch.cuda.synchronize()
    assert rc == 0 and cz.item() == 0.0


# ------------------------------------------------------------------------- degree-K tables
def _perm_sum_table(n, deg, rng):
    """Doubly stochastic table with `deg` slots: a convex combination of deg permutations."""
    c = rng.random(deg).astype(np.float32) + np.float32(0.1)
    c /= c.sum()
    nbr = np.stack([rng.permutation(n) for _ in range(deg)], axis=1).astype(np.int32)
    w = np.tile(c.astype(np.float32), (n, 1))
    return nbr, w


@pytest.mark.parametrize("n,d,deg", [(4, 9, 1), (6, 2048, 2), (16, 4 * 3000, 5), (64, 1025, 8), (128, 8192 + 4, 4),
                                     (128, 516, 32), (300, 516, 13), (8, 70001, 7)])
@pytest.mark.parametrize("gkind", ["f32", "bf16"])
def test_degree_k_tables(psgd, n, d, deg, gkind):
    rng = np.random.default_rng(n * 13 + deg)
    nbr, w = _perm_sum_table(n, deg, rng)
    T = orc.densify(nbr, w)
    assert np.allclose(T.sum(0), 1, atol=1e-5) and np.allclose(T.sum(1), 1, atol=1e-5)
    X = inp.host_normal_f32((n, d), 1.0, 1500 + n)
    G = inp.host_normal_f32((n, d), 0.5, 1600 + n)
    if gkind == "bf16":
        G = inp.f32_to_bf16_bits(G)
    want = orc.mix_step(X, G, T, 0.2)
    got, c = run_step_cd(psgd, X, G, nbr, w, 0.2)
    assert_close(got, want, rel=REL * max(1.0, deg / 4))      # deg + 1 roundings instead of 4
    c_ref = orc.consensus_dist(got)
    assert abs(c - c_ref) <= REL * c_ref
    got_ip, c_ip = run_step_cd(psgd, X, G, nbr, w, 0.2, in_place=True)
    assert np.array_equal(got_ip.view(np.uint32), got.view(np.uint32)) and c_ip == c
    assert np.array_equal(run_step(psgd, X, G, nbr, w, 0.2).view(np.uint32), got.view(np.uint32))


@pytest.mark.parametrize("n,deg", [(16, 3), (16, 5), (64, 9), (300, 4)])
def test_tiled_distance_far_from_origin(psgd, n, deg):
    """Replicas that agree to 1e-4 but sit at O(1) and move by a common 1000 per step: the tiled
    path measures against the output of row 0, so the large common shift must cancel exactly
    (a pivot taken from the inputs would leave only ~4 of the distance's digits)."""
    d = 4100
    rng = np.random.default_rng(n + deg)
    nbr, w = _general_table(n, rng) if deg == 3 else _perm_sum_table(n, deg, rng)
    X = (np.tile(inp.host_normal_f32((1, d), 1.0, 1), (n, 1)) + inp.host_normal_f32((n, d), 1e-4, 2)).astype(np.float32)
    G = np.full((n, d), 1000.0, np.float32)
    got, c = run_step_cd(psgd, X, G, nbr, w, 1.0)
    assert_close(got, orc.mix_step(X, G, orc.densify(nbr, w), 1.0), rel=REL * max(1.0, deg / 4))
    c_ref = orc.consensus_dist(got)
    assert c_ref > 0 and abs(c - c_ref) <= REL * c_ref


def test_two_ring_hops_as_one_degree5_table(psgd):
    """A ring that also averages with the second neighbours (5-point stencil, weights 1/5)."""
    n, d = 16, 3000
    nbr = np.stack([(np.arange(n) + k) % n for k in (0, -1, 1, -2, 2)], axis=1).astype(np.int32)
    w = np.full((n, 5), 0.2, np.float32)
    T = orc.densify(nbr, w)
    lam = orc.spectrum(T)
    want_lam = np.sort([(1 + 2 * np.cos(2 * np.pi * k / n) + 2 * np.cos(4 * np.pi * k / n)) / 5 for k in range(n)])[::-1]
    assert np.allclose(lam, want_lam, atol=1e-6)          # circulant: Fourier transform of the first row
    X = inp.host_normal_f32((n, d), 1.0, 3)
    G = inp.host_normal_f32((n, d), 1.0, 4)
    assert_close(run_step(psgd, X, G, nbr, w, 0.1), orc.mix_step(X, G, T, 0.1), rel=2 * REL)


def test_two_mixing_rounds_collapsed_into_one_table(psgd):
    """Two randomized-ring rounds per step (more communication rounds per iteration) equal one
    step with the 9-slot table of T_1 T_2."""
    n, d = 32, 4100
    n1, w1 = psgd.build_mixing(psgd.TOPO_RAND_RING, n, 5, 0)
    n2, w2 = psgd.build_mixing(psgd.TOPO_RAND_RING, n, 5, 1)
    nbr = np.zeros((n, 9), np.int32)
    w = np.zeros((n, 9), np.float32)
    for i in range(n):
        for a in range(3):
            j = n2[i, a]
            for b in range(3):
                nbr[i, 3 * a + b] = n1[j, b]
                w[i, 3 * a + b] = w2[i, a] * w1[j, b]
    assert np.allclose(orc.densify(nbr, w), orc.densify(n1, w1) @ orc.densify(n2, w2), atol=1e-7)
    X = inp.host_normal_f32((n, d), 1.0, 7)
    G = inp.host_normal_f32((n, d), 1.0, 8)
    two = run_step(psgd, run_step(psgd, X, np.zeros_like(G), n1, w1, 0.0), G, n2, w2, 0.1)
    one = run_step(psgd, X, G, nbr, w, 0.1)
    assert_close(one, two.astype(np.float64), rel=3 * REL)
    assert_close(one, orc.mix_step(X, G, orc.densify(nbr, w), 0.1), rel=3 * REL)


def test_product_of_random_rings_contracts_as_predicted(psgd):
    """Mixing the identity k times gives (T_1 ... T_k)^T itself.  Its distance from T_u must
    match the oracle's dense product and, averaged over seeds, Sec. 3's expectation
    (L-1) ((L-3)/(3(L-1)))^k (Eq. 11), which also bounds the spectral norm as in Eq. 12."""
    n, k, trials = 16, 3, 150
    Tu = orc.uniform_matrix(n)
    eye = np.eye(n, dtype=np.float32)
    zero = torch.zeros(n, n, device="cuda:0")
    fro2, spec = [], []
    for t in range(trials):
        Xd = dev(eye)
        P = np.eye(n)
        for j in range(k):
            nbr, w = psgd.build_mixing(psgd.TOPO_RAND_RING, n, 900 + t, j)
            psgd.mix_step(Xd, Xd, zero, dev(nbr), dev(w), 0.0)
            P = orc.densify(nbr, w).T @ P
        got = Xd.cpu().numpy().astype(np.float64)
        assert np.abs(got - P).max() <= 1e-6
        fro2.append(np.linalg.norm(got - Tu, "fro") ** 2)
        spec.append(np.linalg.norm(got - Tu, 2))
    want = (n - 1) * ((n - 3) / (3 * (n - 1))) ** k
    assert abs(np.mean(fro2) - want) < 5 * np.std(fro2) / np.sqrt(trials)
    assert np.mean(spec) <= np.sqrt(n - 1) / np.sqrt(3) ** k


def test_degree_table_out_of_range_is_flagged(psgd):
    n, d, deg = 8, 1024, 4
    rng = np.random.default_rng(1)
    nbr, w = _perm_sum_table(n, deg, rng)
    nbr[2, 3] = n
    X = inp.host_normal_f32((n, d), 1.0, 1)
    got, c = run_step_cd(psgd, X, X.copy(), nbr, w, 0.1)
    assert np.isnan(got).all() and np.isnan(c) and psgd.device_status(clear=True) == 1


# ------------------------------------------------------------------------- global averaging (T_u)
@pytest.mark.parametrize("n,d", SHAPES)
@pytest.mark.parametrize("gkind", ["f32", "bf16"])
def test_mix_full_matches_oracle(psgd, n, d, gkind):
    """S-PSGD's / D1D-PSGD's T_u: every learner gets the mean model, then its own gradient."""
    X = inp.host_normal_f32((n, d), 1.0, 1300 + n) + np.float32(2.0)
    G = inp.host_normal_f32((n, d), 0.5, 1400 + n)
    if gkind == "bf16":
        G = inp.f32_to_bf16_bits(G)
    want = orc.mix_step(X, G, orc.uniform_matrix(n), 0.1)
    Xd = dev(X)
    Gd = bits_dev(G) if gkind == "bf16" else dev(G)
    out = torch.full_like(Xd, float("nan"))
    c = torch.zeros(1, dtype=torch.float64, device="cuda:0")
    psgd.mix_full(Xd, out, Gd, 0.1, cdist_out=c)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert_close(got, want)
    c_ref = orc.consensus_dist(got)
    assert abs(c.item() - c_ref) <= REL * c_ref + 1e-300
    out2 = torch.full_like(Xd, float("nan"))
    psgd.mix_full(Xd, out2, Gd, 0.1, delay_mode=1)          # no distance, delay flag
    psgd.mix_full(Xd, Xd, Gd, 0.1)                          # in place
    torch.cuda.synchronize()
    assert np.array_equal(out2.cpu().numpy().view(np.uint32), got.view(np.uint32))
    assert np.array_equal(Xd.cpu().numpy().view(np.uint32), got.view(np.uint32))
    with pytest.raises(psgd.PsgdError):
        psgd.mix_full(Xd, Xd, Gd, 0.1, delay_mode=1)


def test_mix_full_pitched_and_consensus_after_averaging(psgd):
    n, d, pitch = 16, 2052, 7000
    Xh = inp.host_normal_f32((n, d), 1.0, 5)
    pool, X, Y, G = _pitched_views(n, d, pitch, False)
    X.copy_(dev(Xh))
    psgd.mix_full(X, Y, G, 0.5)            # G = 0: every replica becomes the mean
    torch.cuda.synchronize()
    got = Y.cpu().numpy()
    assert_close(got, orc.mix_step(Xh, np.zeros_like(Xh), orc.uniform_matrix(n), 0.5))
    assert np.array_equal(got, np.broadcast_to(got[0], got.shape))       # exact consensus
    c = torch.ones(1, dtype=torch.float64, device="cuda:0")
    psgd.consensus_dist_async(Y, c)
    torch.cuda.synchronize()
    assert c.item() == 0.0


# ------------------------------------------------------------------------- pitched rows
@pytest.mark.parametrize("n,d,pitch", [(2, 8, 32), (8, 4100, 3 * 4100 + 4), (16, 1001, 3100), (64, 2052, 7000),
                                       (128, 516, 2048), (5, 1, 3)])
@pytest.mark.parametrize("gkind", ["f32", "bf16"])
def test_pitched_interleaved_rows_match_dense(psgd, n, d, pitch, gkind):
    Xh = inp.host_normal_f32((n, d), 1.0, 1100 + n)
    Gh = inp.host_normal_f32((n, d), 0.5, 1200 + n)
    if gkind == "bf16":
        Gh = inp.f32_to_bf16_bits(Gh)
    nbr, w = psgd.build_mixing(psgd.TOPO_RAND_RING, n, 77, d)
    want = orc.mix_step(Xh, Gh, orc.densify(nbr, w), 0.1)
    dense = run_step(psgd, Xh, Gh, nbr, w, 0.1)
    pool, X, Y, G = _pitched_views(n, d, pitch, gkind == "bf16")
    X.copy_(dev(Xh))
    G.copy_(bits_dev(Gh) if gkind == "bf16" else dev(Gh))
    before = pool.clone()
    c = torch.zeros(1, dtype=torch.float64, device="cuda:0")
    psgd.mix_step(X, Y, G, dev(nbr), dev(w), 0.1, cdist_out=c)
    torch.cuda.synchronize()
    got = Y.cpu().numpy()
    assert np.array_equal(got.view(np.uint32), dense.view(np.uint32))
    assert_close(got, want)
    c_ref = orc.consensus_dist(got)
    assert abs(c.item() - c_ref) <= REL * c_ref + 1e-300
    # nothing outside the rows of X_out was touched
    after = pool.clone()
    Y.zero_()
    Yb = before.as_strided((n, d), (pitch, 1), d)
    Yb.zero_()
    after2 = pool.clone()
    assert torch.equal(after2, before)
    del after
    # pitched consensus distance and in-place
    c2 = torch.zeros(1, dtype=torch.float64, device="cuda:0")
    psgd.consensus_dist_async(X, c2)
    torch.cuda.synchronize()
    assert abs(c2.item() - orc.consensus_dist(Xh)) <= REL * orc.consensus_dist(Xh) + 1e-300
    psgd.mix_step(X, X, G, dev(nbr), dev(w), 0.1)
    torch.cuda.synchronize()
    assert np.array_equal(X.cpu().numpy().view(np.uint32), dense.view(np.uint32))


def test_pitched_general_table(psgd):
    n, d, pitch = 16, 1030, 4096
    rng = np.random.default_rng(3)
    nbr, w = _general_table(n, rng)
    Xh = inp.host_normal_f32((n, d), 1.0, 1)
    Gh = inp.host_normal_f32((n, d), 1.0, 2)
    pool, X, Y, G = _pitched_views(n, d, pitch, False)
    X.copy_(dev(Xh))
    G.copy_(dev(Gh))
    c = torch.zeros(1, dtype=torch.float64, device="cuda:0")
    psgd.mix_step(X, Y, G, dev(nbr), dev(w), 0.2, cdist_out=c)
    torch.cuda.synchronize()
    got = Y.cpu().numpy()
    assert_close(got, orc.mix_step(Xh, Gh, orc.densify(nbr, w), 0.2))
    assert abs(c.item() - orc.consensus_dist(got)) <= REL * orc.consensus_dist(got)


# ------------------------------------------------------------------------- gradient producer
def test_synth_grad_matches_oracle(psgd):
    for count in (1, 5, 4096, 100_003):
        Xp = inp.host_normal_f32((count,), 0.02, 91)
        Z = inp.host_normal_f32((count,), 1e-3, 92)
        G = torch.empty(count, device="cuda:0")
        psgd.synth_grad(dev(Xp), dev(Z), G, 0.01)
        torch.cuda.synchronize()
        want = orc.synth_grad(Xp, Z, 0.01)
        assert_close(G.cpu().numpy(), want, rel=2.0 ** -23)


def test_synth_grad_pitched_rows(psgd):
    n, d, pitch = 8, 1030, 4096
    pool = torch.zeros(n * pitch, device="cuda:0")
    Xp = pool.as_strided((n, d), (pitch, 1), 0)
    Z = pool.as_strided((n, d), (pitch, 1), d)
    G = pool.as_strided((n, d), (pitch, 1), 2 * d)
    Xh = inp.host_normal_f32((n, d), 0.02, 93)
    Zh = inp.host_normal_f32((n, d), 1e-3, 94)
    Xp.copy_(dev(Xh))
    Z.copy_(dev(Zh))
    psgd.synth_grad(Xp, Z, G, 0.01)
    torch.cuda.synchronize()
    assert_close(G.cpu().numpy(), orc.synth_grad(Xh, Zh, 0.01), rel=2.0 ** -23)
    assert np.array_equal(Xp.cpu().numpy(), Xh) and np.array_equal(Z.cpu().numpy(), Zh)


# ------------------------------------------------------------------------- short trajectories
@pytest.mark.parametrize("topo", [orc.TOPO_RING, orc.TOPO_RAND_RING])
def test_cfg1_full_trajectory_every_element(psgd, topo):
    """Workload 1 (n = 8, d = 1e6, 10 steps), every element of every step, free-running on
    both sides from the same X_0 and the same per-step gradients, plus the consensus
    distance after each step and the mean invariant."""
    wl = inp.workload(1)
    X0 = inp.host_normal_f32((wl.n, wl.d), wl.sigma_x, wl.seed_x)
    Xd, Yd = dev(X0), torch.empty(wl.n, wl.d, device="cuda:0")
    Xo = X0.astype(np.float64)
    for k in range(wl.steps):
        G = inp.host_normal_f32((wl.n, wl.d), wl.sigma_g, wl.seed_g * 1000 + k)
        nbr, w = psgd.build_mixing(topo, wl.n, wl.seed_perm, k)
        psgd.mix_step(Xd, Yd, dev(G), dev(nbr), dev(w), wl.lr)
        Xd, Yd = Yd, Xd
        Xo = orc.mix_step(Xo, G, orc.densify(nbr, w), wl.lr)
        got = Xd.cpu().numpy()
        assert_close(got, Xo)
        c_gpu, c_ref = psgd.consensus_dist(Xd), orc.consensus_dist(got)
        assert abs(c_gpu - c_ref) <= REL * c_ref
        assert abs(c_gpu - orc.consensus_dist(Xo)) <= 1e-5 * c_ref
    # expected value for a Gaussian start (fixed ring): C_10 ~ 2.596e4; random ring far lower
    if topo == orc.TOPO_RING:
        assert abs(c_gpu / 2.596e4 - 1) < 0.02


def test_mean_preserved_at_zero_lr(psgd):
    """Doubly stochastic mixing keeps the replica mean; with fl32(1/3) weights the drift is
    3 fl32(1/3) - 1 = 3e-8 per step, common to oracle and GPU."""
    n, d, steps = 16, 40_000, 20
    X0 = inp.host_normal_f32((n, d), 1.0, 7) + np.float32(3.0)
    G = torch.zeros(n, d, device="cuda:0")
    Xd = dev(X0)
    for k in range(steps):
        nbr, w = psgd.build_mixing(psgd.TOPO_RAND_RING, n, 12, k)
        psgd.mix_step(Xd, Xd, G, dev(nbr), dev(w), 0.0)
    torch.cuda.synchronize()
    m0 = X0.astype(np.float64).mean(0)
    m1 = Xd.cpu().numpy().astype(np.float64).mean(0)
    assert np.abs(m1 - m0).max() <= steps * 1e-7 * np.abs(m0).max()


# ------------------------------------------------------------------------- HIP graph capture
def test_steps_captured_in_a_hip_graph_replay_exactly(psgd):
    """The step only enqueues kernels (no allocation once the scratch exists, no memset), so a
    run of steps with pre-uploaded tables can be captured once and replayed.  Replays are
    interleaved with eager work and compared with the eager result every time."""
    n, d, steps = 16, 40_004, 4
    X0 = inp.host_normal_f32((n, d), 1.0, 21)
    Gh = inp.host_normal_f32((n, d), 0.1, 22)
    tabs = [psgd.build_mixing(psgd.TOPO_RAND_RING, n, 33, k) for k in range(steps)]
    nbr_d = [dev(t[0]) for t in tabs]
    w_d = [dev(t[1]) for t in tabs]
    G = dev(Gh)
    c_eager = torch.zeros(steps, dtype=torch.float64, device="cuda:0")
    c_graph = torch.zeros(steps, dtype=torch.float64, device="cuda:0")
    A, B = dev(X0), torch.empty(n, d, device="cuda:0")

    def run(cbuf, stream=None):
        src, dst = A, B
        for k in range(steps):
            psgd.mix_step(src, dst, G, nbr_d[k], w_d[k], 0.05, cdist_out=cbuf[k:k + 1], stream=stream)
            src, dst = dst, src
        return src

    final = run(c_eager)                       # also allocates the library's scratch before capture
    torch.cuda.synchronize()
    want = final.clone()
    s = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    A.copy_(dev(X0))
    torch.cuda.synchronize()
    with torch.cuda.graph(g, stream=s):
        out = run(c_graph, stream=torch.cuda.current_stream())
    for rep in range(3):
        A.copy_(dev(X0))
        B.fill_(float("nan"))
        c_graph.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, want), rep
        assert torch.equal(c_graph, c_eager), rep
        # eager work of the same library between replays
        assert abs(psgd.consensus_dist(out) - c_eager[-1].item()) <= 1e-9 * c_eager[-1].item()


def test_long_row_kernels_captured_in_a_hip_graph_replay_exactly(psgd):
    """The same on rows long enough for the large workgroups: the ring walk (with the tiled kernel enqueued
    behind it), a 5-slot table through the tiled kernel (more than 64 KB of LDS) and global averaging, every
    one with the fused distance, captured once after an eager pass and replayed between eager work."""
    n, d = 16, 1_600_004
    rng = np.random.default_rng(5)
    X0 = dev(inp.host_normal_f32((n, d), 1.0, 23))
    G = dev(inp.host_normal_f32((n, d), 0.1, 24))
    ring = [dev(t) for t in psgd.build_mixing(psgd.TOPO_RAND_RING, n, 34, 0)]
    deg5 = [dev(t) for t in _perm_sum_table(n, 5, rng)]
    c_eager = torch.zeros(3, dtype=torch.float64, device="cuda:0")
    c_graph = torch.zeros(3, dtype=torch.float64, device="cuda:0")
    A, B = X0.clone(), torch.empty(n, d, device="cuda:0")

    def run(cbuf, stream=None):
        psgd.mix_step(A, B, G, ring[0], ring[1], 0.05, cdist_out=cbuf[0:1], stream=stream)
        psgd.mix_step(B, A, G, deg5[0], deg5[1], 0.05, cdist_out=cbuf[1:2], stream=stream)
        psgd.mix_full(A, B, G, 0.05, cdist_out=cbuf[2:3], stream=stream)
        return B

    run(c_eager)
    torch.cuda.synchronize()
    want = B.clone()
    assert c_eager[0].item() > c_eager[1].item() > 0 and c_eager[2].item() > 0
    s = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    A.copy_(X0)
    torch.cuda.synchronize()
    with torch.cuda.graph(g, stream=s):
        out = run(c_graph, stream=torch.cuda.current_stream())
    for rep in range(3):
        A.copy_(X0)
        B.fill_(float("nan"))
        c_graph.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, want), rep
        assert torch.equal(c_graph, c_eager), rep
        assert abs(psgd.consensus_dist(out) - c_eager[-1].item()) <= 1e-9 * c_eager[-1].item()
    assert psgd.device_status() == 0


# ------------------------------------------------------------------------- tables built on the device
@pytest.mark.parametrize("n", [1, 2, 3, 5, 8, 64, 128, 257, 512])
def test_device_built_tables_bit_identical_to_oracle(psgd, n):
    nbr = torch.full((n, 3), -7, dtype=torch.int32, device="cuda:0")
    w = torch.full((n, 3), float("nan"), device="cuda:0")
    for topo in (psgd.TOPO_RING, psgd.TOPO_RAND_RING):
        for seed, step in ((0, 0), (1, 7), (3005, 19), (2 ** 63 + 5, 2 ** 40 + 3), (2 ** 64 - 1, 2 ** 64 - 1)):
            psgd.build_mixing_device(topo, n, seed, nbr, w, step_offset=step)
            onbr, ow = orc.neighbour_table(topo, n, seed, step)
            assert np.array_equal(nbr.cpu().numpy(), onbr), (topo, n, seed, step)
            assert np.array_equal(w.cpu().numpy().view(np.uint32), ow.view(np.uint32))


def test_device_step_counter_advances(psgd):
    n, seed = 33, 77
    nbr = torch.empty((n, 3), dtype=torch.int32, device="cuda:0")
    w = torch.empty((n, 3), device="cuda:0")
    step = torch.tensor([5], dtype=torch.int64, device="cuda:0")
    for k in range(4):
        psgd.build_mixing_device(psgd.TOPO_RAND_RING, n, seed, nbr, w, step_dev=step, step_offset=100, advance=2)
        assert np.array_equal(nbr.cpu().numpy(), orc.neighbour_table(orc.TOPO_RAND_RING, n, seed, 105 + 2 * k)[0])
        assert step.item() == 5 + 2 * (k + 1)
    psgd.build_mixing_device(psgd.TOPO_RAND_RING, n, seed, nbr, w, step_dev=step)      # advance = 0: read only
    assert step.item() == 13
    assert np.array_equal(nbr.cpu().numpy(), orc.neighbour_table(orc.TOPO_RAND_RING, n, seed, 13)[0])


def test_graph_of_table_build_and_step_walks_the_iterations(psgd):
    """One captured graph = {build the iteration's ring from the device-side counter, advance the
    counter, mix in place}.  Each replay must be the next iteration of the randomized-ring
    run: compared with the oracle's trajectory, with eager work between replays."""
    n, d, seed, lr, steps = 16, 12_004, 41, 0.05, 5
    X0 = inp.host_normal_f32((n, d), 1.0, 51)
    Gh = inp.host_normal_f32((n, d), 0.1, 52)
    X, G = dev(X0), dev(Gh)
    nbr = torch.empty((n, 3), dtype=torch.int32, device="cuda:0")
    w = torch.empty((n, 3), device="cuda:0")
    step = torch.zeros(1, dtype=torch.int64, device="cuda:0")
    c = torch.zeros(1, dtype=torch.float64, device="cuda:0")
    scratch = torch.empty_like(X)
    psgd.mix_step(X, scratch, G, dev(psgd.build_mixing(psgd.TOPO_RING, n)[0]),
                  dev(psgd.build_mixing(psgd.TOPO_RING, n)[1]), lr, cdist_out=c)     # library scratch exists before capture
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        cur = torch.cuda.current_stream()
        psgd.build_mixing_device(psgd.TOPO_RAND_RING, n, seed, nbr, w, step_dev=step, advance=1, stream=cur)
        psgd.mix_step(X, X, G, nbr, w, lr, cdist_out=c, stream=cur)
    X.copy_(dev(X0))
    step.zero_()
    torch.cuda.synchronize()
    Xo = X0.astype(np.float64)
    for k in range(steps):
        g.replay()
        torch.cuda.synchronize()
        T = orc.mixing_matrix(orc.TOPO_RAND_RING, n, seed, k)
        Xo = orc.mix_step(Xo, Gh, T, lr)
        got = X.cpu().numpy()
        assert_close(got, Xo, rel=REL * (k + 1))
        assert step.item() == k + 1
        assert np.array_equal(nbr.cpu().numpy(), orc.neighbour_table(orc.TOPO_RAND_RING, n, seed, k)[0])
        c_ref = orc.consensus_dist(got)
        assert abs(c.item() - c_ref) <= REL * c_ref
        assert abs(psgd.consensus_dist(X) - c_ref) <= REL * c_ref          # eager work between replays


def test_binding_checks_dtypes_and_devices(psgd):
    n, d = 4, 64
    X = torch.zeros(n, d, device="cuda:0")
    nbr, w = psgd.build_mixing(psgd.TOPO_RING, n)
    nb, wd = dev(nbr), dev(w)
    with pytest.raises(ValueError):
        psgd.mix_step(X.cpu(), X.clone(), X.clone(), nb, wd, 0.1)              # host X
    with pytest.raises(ValueError):
        psgd.mix_step(X, X.clone(), X.clone(), nb.cpu(), wd, 0.1)              # host table
    with pytest.raises(ValueError):
        psgd.mix_step(X, X.clone(), X.double(), nb, wd, 0.1)                   # fp64 gradients
    with pytest.raises(ValueError):
        psgd.mix_step(X.half(), X.clone(), X.clone(), nb, wd, 0.1)
    with pytest.raises(ValueError):
        psgd.synth_grad(X.bfloat16(), X.bfloat16(), X.bfloat16(), 0.1)          # 2-byte elements
    with pytest.raises(ValueError):
        psgd.consensus_dist(X.double())
    with pytest.raises(ValueError):
        psgd.mix_step(X, X.clone(), X.clone(), nb, wd, 0.1, cdist_out=torch.zeros(1, device="cuda:0"))   # fp32 distance
    assert psgd.device_status() == 0


@pytest.mark.parametrize("kind", ["ring", "general3", "deg5", "full"])
@pytest.mark.parametrize("n,d", [(4, 8_000_004), (4, 6_000_001), (16, 2_000_004), (16, 1_500_001)])
def test_many_sweeps_per_workgroup(psgd, kind, n, d):
    """Rows long enough that every persistent workgroup strides over many column groups /
    tiles (the small shapes finish in one), with a ragged last tile; every element is compared.
    n = 16 takes the tiled kernel's variant without per-row guards, n = 4 the guarded one."""
    lr = 0.1
    rng = np.random.default_rng(d % 1000 + len(kind))
    X = inp.host_normal_f32((n, d), 1.0, 61)
    G = inp.f32_to_bf16_bits(inp.host_normal_f32((n, d), 0.5, 62))
    Xd, Gd = dev(X), bits_dev(G)
    Yd = torch.full_like(Xd, float("nan"))
    c = torch.full((1,), float("nan"), dtype=torch.float64, device="cuda:0")
    if kind == "full":
        T = orc.uniform_matrix(n)
        psgd.mix_full(Xd, Yd, Gd, lr, cdist_out=c)
    else:
        if kind == "ring":
            nbr, w = psgd.build_mixing(psgd.TOPO_RAND_RING, n, 3, 4)
        elif kind == "general3":
            nbr, w = _general_table(n, rng)
        else:
            nbr, w = _perm_sum_table(n, 5, rng)
        T = orc.densify(nbr, w)
        psgd.mix_step(Xd, Yd, Gd, dev(nbr), dev(w), lr, cdist_out=c)
    torch.cuda.synchronize()
    got = Yd.cpu().numpy()
    assert_close(got, orc.mix_step(X, G, T, lr), rel=REL * (1.5 if kind == "deg5" else 1.0))
    c_ref = orc.consensus_dist(got)
    assert abs(c.item() - c_ref) <= REL * c_ref
    assert psgd.device_status() == 0


@pytest.mark.parametrize("gkind", ["f32", "bf16"])
def test_global_average_large_workgroups_every_element(psgd, gkind):
    """Rows long enough for the global-average kernel's large lockstep workgroups (they start at
    16 column groups per lane), ragged end included; every element and the distance compared."""
    n, d, lr = 4, 16_000_004, 0.2
    X = inp.host_normal_f32((n, d), 1.0, 81)
    G = inp.host_normal_f32((n, d), 0.5, 82)
    if gkind == "bf16":
        G = inp.f32_to_bf16_bits(G)
    Xd = dev(X)
    Gd = bits_dev(G) if gkind == "bf16" else dev(G)
    c = torch.full((1,), float("nan"), dtype=torch.float64, device="cuda:0")
    Yd = torch.full_like(Xd, float("nan"))
    psgd.mix_full(Xd, Yd, Gd, lr, cdist_out=c)
    torch.cuda.synchronize()
    got = Yd.cpu().numpy()
    assert_close(got, orc.mix_step(X, G, orc.uniform_matrix(n), lr))
    c_ref = orc.consensus_dist(got)
    assert abs(c.item() - c_ref) <= REL * c_ref
    psgd.mix_full(Xd, Xd, Gd, lr)                     # in place, no distance
    torch.cuda.synchronize()
    assert torch.equal(Xd, Yd)


def test_status_flag_is_sticky_until_cleared_and_long_rows_refuse_bad_tables(psgd):
    n, d = 4, 2_000_000                      # long rows: the large-workgroup variant of the step kernel
    nbr, w = psgd.build_mixing(psgd.TOPO_RING, n)
    bad = nbr.copy()
    bad[1, 2] = -1
    X = torch.ones(n, d, device="cuda:0")
    Y = torch.full_like(X, float("nan"))
    c = torch.zeros(1, dtype=torch.float64, device="cuda:0")
    psgd.mix_step(X, Y, X.clone(), dev(bad), dev(w), 0.1, cdist_out=c)
    torch.cuda.synchronize()
    assert torch.isnan(Y).all() and np.isnan(c.item())
    assert psgd.device_status(clear=False) == 1
    assert psgd.device_status(clear=False) == 1          # still raised
    psgd.mix_step(X, Y, X.clone(), dev(nbr), dev(w), 0.1, cdist_out=c)      # a good step does not lower it
    torch.cuda.synchronize()
    assert not torch.isnan(Y).any() and c.item() == 0.0
    assert psgd.device_status(clear=True) == 1
    assert psgd.device_status() == 0


def test_two_streams_gathering_distances_are_serialised(psgd):
    """All fused-distance and consensus calls on a device share one buffer of partial sums.  Calls enqueued
    back to back on two streams would race on it; the library makes the later stream wait for the earlier
    call's last kernel, so each distance must be the one of its own output, every time."""
    n, lr = 16, 0.1
    shapes = [(n, 1_600_004), (n, 70_001)]            # a long launch on one stream, a short one on the other
    data = []
    for i, (nn, d) in enumerate(shapes):
        X = inp.host_normal_f32((nn, d), 1.0 + i, 300 + i)
        G = inp.host_normal_f32((nn, d), 0.1, 310 + i)
        nbr, w = orc.neighbour_table(orc.TOPO_RAND_RING, nn, 5, i)
        data.append((dev(X), dev(G), dev(nbr), dev(w), X, G, nbr, w))
    outs = [torch.empty_like(t[0]) for t in data]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    rounds = 6
    cd = torch.full((rounds, 2), float("nan"), dtype=torch.float64, device="cuda:0")
    cs = torch.full((rounds, 2), float("nan"), dtype=torch.float64, device="cuda:0")
    torch.cuda.synchronize()
    for r in range(rounds):
        for i in (0, 1):
            Xd, Gd, nd, wd = data[i][:4]
            psgd.mix_step(Xd, outs[i], Gd, nd, wd, lr, stream=streams[i], cdist_out=cd[r, i:i + 1])
        for i in (1, 0):
            psgd.consensus_dist_async(outs[i], cs[r, i:i + 1], stream=streams[i])
    torch.cuda.synchronize()
    got, sep = cd.cpu().numpy(), cs.cpu().numpy()
    for i in (0, 1):
        X, G, nbr, w = data[i][4:]
        want = orc.mix_step(X, G, orc.densify(nbr, w), lr)
        assert_close(outs[i].cpu().numpy(), want)
        c_want = orc.consensus_dist(outs[i].cpu().numpy())
        for r in range(rounds):
            assert abs(got[r, i] - c_want) <= REL * c_want, (r, i, got[r, i], c_want)
            assert abs(sep[r, i] - c_want) <= REL * c_want, (r, i, sep[r, i], c_want)
    assert psgd.device_status() == 0


@pytest.mark.parametrize("n,d", [(3, 8), (8, 4100), (16, 1_600_004)])
@pytest.mark.parametrize("gkind", ["f32", "bf16"])
def test_reference_streams_do_what_they_say(psgd, n, d, gkind):
    """The benchmark's reference streams are measurement support, but their rates are only worth comparing
    with the step's if they move the bytes they claim: the write stream fills X_out, the x + a g stream
    equals the oracle's update with the identity as mixing matrix and lr = -a, the read stream changes nothing."""
    X = inp.host_normal_f32((n, d), 1.0, 500 + n)
    G = (inp.host_normal_bf16_bits if gkind == "bf16" else inp.host_normal_f32)((n, d), 0.5, 600 + n)
    Xd = dev(X)
    Gd = bits_dev(G) if gkind == "bf16" else dev(G)
    out = torch.full_like(Xd, float("nan"))
    psgd.reference_stream(psgd.REF_READ, Xd, out, Gd)
    torch.cuda.synchronize()
    assert torch.isnan(out).all() and np.array_equal(Xd.cpu().numpy(), X)
    psgd.reference_stream(psgd.REF_WRITE, Xd, out, Gd, a=0.25)
    torch.cuda.synchronize()
    assert (out == 0.25).all()
    psgd.reference_stream(psgd.REF_AXPY, Xd, out, Gd, a=0.5)
    torch.cuda.synchronize()
    want = orc.mix_step(X, G, np.eye(n), -0.5)
    assert_close(out.cpu().numpy(), want)
    with pytest.raises(psgd.PsgdError):
        psgd.reference_stream(psgd.REF_AXPY, Xd, Xd, Gd)          # output over an input


# ------------------------------------------------------------------------- tiled kernel on long rows
def _two_rings_table(n):
    """The even and the odd learners on two disjoint rings: 3 slots, locally consistent, not ONE ring."""
    idx = np.arange(n)
    nbr = np.stack([idx, (idx - 2) % n, (idx + 2) % n], axis=1).astype(np.int32)
    return nbr, np.tile(np.asarray([0.5, 0.25, 0.25], dtype=np.float32), (n, 1))


_LONG_ROW_CASES = (
    # the main shape, every table kind and both gradient types
    [(64, 1_600_004, k, g) for k in ("two_rings", "deg5", "deg13") for g in ("f32", "bf16")]
    # the other shapes: two or three (table kind, gradient type) pairs each
    + [(64, 1_572_867, "two_rings", "f32"), (64, 1_572_867, "deg13", "bf16"),
       (128, 1_600_004, "two_rings", "bf16"), (128, 1_600_004, "deg5", "f32"), (128, 1_600_004, "deg13", "bf16"),
       (33, 1_700_004, "deg5", "f32"), (33, 1_700_004, "deg13", "bf16"),
       (8, 1_800_004, "two_rings", "f32"), (8, 1_800_004, "deg5", "bf16"), (8, 1_800_004, "deg13", "f32"),
       (70, 1_600_004, "two_rings", "f32"), (70, 1_600_004, "deg13", "bf16"),
       (16, 1_900_004, "two_rings", "bf16"), (16, 1_900_004, "deg5", "f32"),
       (5, 2_000_004, "deg5", "f32"), (5, 2_000_004, "deg13", "bf16"),
       (48, 1_600_003, "two_rings", "f32"), (48, 1_600_003, "deg5", "bf16")])


@pytest.mark.parametrize("n,d,kind,gkind", _LONG_ROW_CASES)
def test_tiled_kernel_long_rows_every_element(psgd, n, d, kind, gkind):
    """Rows long enough for the large-workgroup tiled kernels: the 1024-lane one-batch form for n <= 64 (merge
    slots of the distance inside the consumed tile buffer at 16 B per lane; wider rows for n = 16, 8, 5; an odd
    row count per row group for n = 33, 48), the 512-lane form with several batches per tile for n = 70 and
    n = 128; d not a multiple of 4 takes one column per lane.  Every element and the fused distance against
    the oracle, out of place and in place, ragged last tile included."""
    rng = np.random.default_rng(n + d % 1000)
    if kind == "two_rings":
        if n % 2:
            pytest.skip("two rings need an even learner count")
        nbr, w = _two_rings_table(n)
    else:
        nbr, w = _perm_sum_table(n, 5 if kind == "deg5" else 13, rng)
    X = inp.host_normal_f32((n, d), 1.0, 700 + n)
    G = inp.host_normal_f32((n, d), 0.5, 710 + n)
    if gkind == "bf16":
        G = inp.f32_to_bf16_bits(G)
    want = orc.mix_step(X, G, orc.densify(nbr, w), 0.2)
    got, c = run_step_cd(psgd, X, G, nbr, w, 0.2)
    assert_close(got, want)
    c_ref = orc.consensus_dist(got)
    assert abs(c - c_ref) <= REL * c_ref
    got_ip, c_ip = run_step_cd(psgd, X, G, nbr, w, 0.2, in_place=True)
    assert np.array_equal(got_ip.view(np.uint32), got.view(np.uint32)) and c_ip == c
    got_plain = run_step(psgd, X, G, nbr, w, 0.2)                # the build without the distance
    assert np.array_equal(got_plain.view(np.uint32), got.view(np.uint32))
    assert psgd.device_status() == 0


@pytest.mark.parametrize("n,kind,gkind", [(200, "deg5", "bf16"), (256, "two_rings", "f32")])
def test_tiled_kernel_long_rows_many_learners(psgd, n, kind, gkind):
    """More than 128 learners on long rows: 256-byte row segments (16 lanes per row), four row groups per
    wavefront, in the one-batch form; every element and the fused distance against the oracle."""
    d = 1_580_004
    rng = np.random.default_rng(n)
    nbr, w = _two_rings_table(n) if kind == "two_rings" else _perm_sum_table(n, 5, rng)
    X = inp.host_normal_f32((n, d), 1.0, 720 + n)
    G = inp.host_normal_f32((n, d), 0.5, 730 + n)
    if gkind == "bf16":
        G = inp.f32_to_bf16_bits(G)
    want = orc.mix_step(X, G, orc.densify(nbr, w), 0.2)
    got, c = run_step_cd(psgd, X, G, nbr, w, 0.2)
    assert_close(got, want)
    c_ref = orc.consensus_dist(got)
    assert abs(c - c_ref) <= REL * c_ref
    got_plain = run_step(psgd, X, G, nbr, w, 0.2)                # the build without the distance
    assert np.array_equal(got_plain.view(np.uint32), got.view(np.uint32))
    assert psgd.device_status() == 0


@pytest.mark.parametrize("n,deg,gkind", [(64, 32, "f32"), (64, 32, "bf16"), (128, 32, "bf16")])
def test_tiled_kernel_long_rows_widest_tables(psgd, n, deg, gkind):
    """32 slots per row on long rows: the slot table takes 16 KB (32 KB for 128 learners) of LDS, so the merge
    slots of the distance no longer fit beside the two tile buffers and live in the buffer that has just been
    consumed (n = 64), or the rows get narrower (n = 128).  Every element and the distance against the oracle."""
    d = 1_580_004
    rng = np.random.default_rng(n + deg)
    nbr, w = _perm_sum_table(n, deg, rng)
    X = inp.host_normal_f32((n, d), 1.0, 740 + n)
    G = inp.host_normal_f32((n, d), 0.5, 750 + n)
    if gkind == "bf16":
        G = inp.f32_to_bf16_bits(G)
    want = orc.mix_step(X, G, orc.densify(nbr, w), 0.2)
    got, c = run_step_cd(psgd, X, G, nbr, w, 0.2)
    assert_close(got, want, rel=REL * deg / 4)                   # deg + 1 roundings instead of 4
    c_ref = orc.consensus_dist(got)
    assert abs(c - c_ref) <= REL * c_ref
    got_ip, c_ip = run_step_cd(psgd, X, G, nbr, w, 0.2, in_place=True)
    assert np.array_equal(got_ip.view(np.uint32), got.view(np.uint32)) and c_ip == c
    got_plain = run_step(psgd, X, G, nbr, w, 0.2)                # the build without the distance
    assert np.array_equal(got_plain.view(np.uint32), got.view(np.uint32))
    assert psgd.device_status() == 0


@pytest.mark.parametrize("n", [16, 64, 128])
def test_tiled_kernel_long_rows_distance_corner_cases(psgd, n):
    """The row groups of the large tiled kernel each measure against their own pivot and the merge brings
    them to a common one: replicas far from the origin and close together must still give the distance to
    1e-6, and identical outputs must give exactly 0."""
    d = 1_600_004
    nbr, w = _two_rings_table(n)
    base = inp.host_normal_f32((1, d), 100.0, 3)
    X = (np.tile(base, (n, 1)) + inp.host_normal_f32((n, d), 1e-3, 4)).astype(np.float32)
    G = np.full((n, d), 7.0, np.float32)
    got, c = run_step_cd(psgd, X, G, nbr, w, 1.0)
    assert_close(got, orc.mix_step(X, G, orc.densify(nbr, w), 1.0))
    c_ref = orc.consensus_dist(got)
    assert abs(c - c_ref) <= REL * c_ref
    Xe = np.tile(base, (n, 1)).astype(np.float32)
    got, c = run_step_cd(psgd, Xe, G, nbr, w, 0.5)
    assert np.array_equal(got, np.tile(got[0], (n, 1))) and c == 0.0
