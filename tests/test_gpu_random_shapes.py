"""Seeded sweep of random VALID shapes, tables and layouts against the oracle: every case draws
n, d, the table kind (fixed ring, random ring, general 3-slot, degree-K), the gradient type,
dense or pitched rows (aligned or not), in place or not, with or without the fused distance."""
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
    m.load()
    torch.cuda.set_device(0)
    return m


def _table(psgd, rng, n):
    kind = rng.choice(["ring", "rand", "general3", "deg"])
    if kind == "ring":
        return psgd.build_mixing(psgd.TOPO_RING, n) + (4,)
    if kind == "rand":
        return psgd.build_mixing(psgd.TOPO_RAND_RING, n, int(rng.integers(0, 2 ** 62)), int(rng.integers(0, 1000))) + (4,)
    deg = 3 if kind == "general3" else int(rng.integers(1, min(32, 4096 // n) + 1))
    c = rng.random(deg).astype(np.float32) + np.float32(0.05)
    c /= c.sum()
    nbr = np.stack([rng.permutation(n) for _ in range(deg)], axis=1).astype(np.int32)
    w = np.tile(c, (n, 1)).astype(np.float32)
    return nbr, w, deg + 1


@pytest.mark.parametrize("block", range(12))
def test_random_cases(psgd, block):
    rng = np.random.default_rng(1000 + block)
    for case in range(40):
        n = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 16, 17, 32, 33, 64, 100, 128, 200, 512]))
        d = int(rng.choice([1, 3, 4, 8, 60, 255, 256, 1000, 1028, 4096, 5001, 20_000]))
        if n * d > 3_000_000:
            d = max(1, 3_000_000 // n)
        nbr, w, roundings = _table(psgd, rng, n)
        bf16 = bool(rng.integers(0, 2))
        pitched = bool(rng.integers(0, 2))
        in_place = bool(rng.integers(0, 2))
        want_cd = bool(rng.integers(0, 2))
        lr = float(rng.choice([0.0, 0.05, 0.5]))
        X = inp.host_normal_f32((n, d), 1.0, int(rng.integers(1, 10 ** 6)))
        Gf = inp.host_normal_f32((n, d), 0.3, int(rng.integers(1, 10 ** 6)))
        G = inp.f32_to_bf16_bits(Gf) if bf16 else Gf
        Gt = torch.from_numpy(G.view(np.int16) if bf16 else G).to("cuda:0")
        if pitched:
            pad = int(rng.choice([0, 1, 4, 13, 64]))          # odd pads leave rows unaligned for 128-bit access
            px = 3 * d + pad
            pool = torch.zeros(n * px + 8, dtype=torch.float32, device="cuda:0")
            Xd = pool.as_strided((n, d), (px, 1), 0)
            Yd = Xd if in_place else pool.as_strided((n, d), (px, 1), d)
            Xd.copy_(torch.from_numpy(X))
            if bf16:
                Gd = pool.view(torch.int16).as_strided((n, d), (2 * px, 1), 4 * d)
            else:
                Gd = pool.as_strided((n, d), (px, 1), 2 * d)
            Gd.copy_(Gt)
        else:
            Xd = torch.from_numpy(X).to("cuda:0")
            Yd = Xd if in_place else torch.full_like(Xd, float("nan"))
            Gd = Gt
        c = torch.full((1,), float("nan"), dtype=torch.float64, device="cuda:0")
        psgd.mix_step(Xd, Yd, Gd, torch.from_numpy(nbr).to("cuda:0"), torch.from_numpy(w).to("cuda:0"), lr,
                      cdist_out=c if want_cd else None)
        torch.cuda.synchronize()
        got = Yd.cpu().numpy()
        want = orc.mix_step(X, G, orc.densify(nbr, w), lr)
        label = (block, case, n, d, nbr.shape[1], bf16, pitched, in_place, want_cd, lr)
        scale = max(np.abs(want).max(), 1e-30)
        tol = REL * max(1.0, roundings / 4)
        # With a handful of columns the outputs can cancel to far below the inputs (n = 3, d = 1: every row
        # is the mean of three numbers of size 2 that sum to 0.01).  The arithmetic then sets the floor: one
        # rounding per slot and one for the gradient term, each on a partial sum bounded by |X|max + lr |G|max.
        gmax = np.abs(orc.bf16_bits_to_f64(G)).max() if bf16 else np.abs(Gf).max()
        floor = roundings * 2.0 ** -24 * (np.abs(X).max() + lr * gmax)
        assert np.abs(got - want).max() <= max(tol * scale, floor), label
        assert np.linalg.norm(got - want) <= max(tol * np.linalg.norm(want), floor * np.sqrt(n * d)), label
        if want_cd:
            c_ref = orc.consensus_dist(got)
            assert abs(c.item() - c_ref) <= REL * c_ref + 1e-300, label
    assert psgd.device_status() == 0


@pytest.mark.parametrize("block", range(6))
def test_random_cases_global_average_distance_and_producer(psgd, block):
    """Same sweep for the table-free calls: global averaging, the distance kernels (dense and
    pitched) and the delayed workload's gradient producer."""
    rng = np.random.default_rng(5000 + block)
    for case in range(30):
        n = int(rng.choice([1, 2, 3, 5, 8, 16, 31, 64, 128, 300, 512]))
        d = int(rng.choice([1, 2, 4, 7, 64, 257, 1024, 3000, 10_004]))
        if n * d > 2_000_000:
            d = max(1, 2_000_000 // n)
        bf16 = bool(rng.integers(0, 2))
        in_place = bool(rng.integers(0, 2))
        pad = int(rng.choice([0, 0, 3, 4, 32]))
        px = 3 * d + pad
        lr = float(rng.choice([0.0, 0.1, 1.0]))
        offset = float(rng.choice([0.0, 100.0]))              # replicas far from the origin
        X = (inp.host_normal_f32((n, d), 1.0, int(rng.integers(1, 10 ** 6))) + np.float32(offset)).astype(np.float32)
        Gf = inp.host_normal_f32((n, d), 0.3, int(rng.integers(1, 10 ** 6)))
        G = inp.f32_to_bf16_bits(Gf) if bf16 else Gf
        pool = torch.zeros(n * px + 8, dtype=torch.float32, device="cuda:0")
        Xd = pool.as_strided((n, d), (px, 1), 0)
        Yd = Xd if in_place else pool.as_strided((n, d), (px, 1), d)
        Xd.copy_(torch.from_numpy(X))
        if bf16:
            Gd = pool.view(torch.int16).as_strided((n, d), (2 * px, 1), 4 * d)
            Gd.copy_(torch.from_numpy(G.view(np.int16)))
        else:
            Gd = pool.as_strided((n, d), (px, 1), 2 * d)
            Gd.copy_(torch.from_numpy(G))
        label = (block, case, n, d, bf16, in_place, pad, lr, offset)
        c = torch.full((2,), float("nan"), dtype=torch.float64, device="cuda:0")
        psgd.consensus_dist_async(Xd, c[0:1])
        psgd.mix_full(Xd, Yd, Gd, lr, cdist_out=c[1:2])
        torch.cuda.synchronize()
        c0 = orc.consensus_dist(X)
        assert abs(c[0].item() - c0) <= REL * c0 + 1e-300, label
        got = Yd.cpu().numpy()
        want = orc.mix_step(X, G, orc.uniform_matrix(n), lr)
        scale = max(np.abs(want).max(), 1e-30)
        assert np.abs(got - want).max() <= REL * scale, label
        c1 = orc.consensus_dist(got)
        assert abs(c[1].item() - c1) <= REL * c1 + 1e-300, label
        # producer: G' = c * Y + noise into a fresh pitched array
        noise = inp.host_normal_f32((n, d), 0.5, int(rng.integers(1, 10 ** 6)))
        pool2 = torch.zeros(n * (2 * d + pad) + 8, dtype=torch.float32, device="cuda:0")
        Nd = pool2.as_strided((n, d), (2 * d + pad, 1), 0)
        Od = pool2.as_strided((n, d), (2 * d + pad, 1), d)
        Nd.copy_(torch.from_numpy(noise))
        psgd.synth_grad(Yd, Nd, Od, 0.25)
        torch.cuda.synchronize()
        wantg = orc.synth_grad(got, noise, 0.25)
        assert np.abs(Od.cpu().numpy() - wantg).max() <= 2.0 ** -23 * max(np.abs(wantg).max(), 1e-30), label
