"""The two-stream delay-by-one schedule (Sec. 4, D1D-PSGD paragraph; Eq. 13 and 14: the averaging of step k
and the gradient computation of step k+1 run concurrently) against the oracle's delayed trajectory.

The schedule keeps three X buffers and two gradient buffers in rotation and orders two streams with events;
a missing or misplaced wait would let the producer read a half-written iterate or overwrite a gradient that
is still being consumed.  The oracle never sees the schedule: it runs X_{k+1} = T_k^T X_k - lr (c X_{k-1} +
noise_k) serially in fp64 from the same X_0, noise bits and tables.
"""
import numpy as np
import pytest

from oracle import psgd_oracle as orc
from paper_2002_01119_amd import inputs as inp

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

REL = 1e-6


@pytest.fixture(scope="module")
def mods():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2002_01119_amd import d1d, psgd
    psgd.load()
    torch.cuda.set_device(0)
    return psgd, d1d


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def _run(mods, n, d, steps, topo, overlap, producer_repeat=1, lr=0.1, c=0.3, seed=40):
    """Returns (list of X_1..X_K as numpy, distances, oracle trajectory X_0..X_K, oracle tables)."""
    psgd, d1d = mods
    X0 = inp.host_normal_f32((n, d), 1.0, seed)
    noises = [inp.host_normal_f32((n, d), 0.05, seed + 1 + k) for k in range(steps)]
    noise_dev = [dev(z) for z in noises]
    if topo == orc.TOPO_FULL:
        Ts = [orc.uniform_matrix(n)] * steps
        table = None
    else:
        tabs = [orc.neighbour_table(topo, n, 9, k) for k in range(steps)]
        Ts = [orc.densify(nb, w) for nb, w in tabs]
        tabs_dev = [(dev(nb), dev(w)) for nb, w in tabs]
        table = lambda k: tabs_dev[k]
    X = dev(X0)
    Y = torch.full_like(X, float("nan"))
    Xp = torch.full_like(X, float("nan"))
    Gs = [torch.full_like(X, float("nan")) for _ in range(2)]
    cd = torch.full((steps,), float("nan"), dtype=torch.float64, device="cuda:0")
    torch.cuda.synchronize()
    ms = torch.cuda.Stream()
    run = d1d.DelayByOne(X, Y, Xp, Gs, lambda k: noise_dev[k], table, lr, c, overlap=overlap, mix_stream=ms,
                         producer_repeat=producer_repeat)
    snaps = []
    for k in range(steps):
        out = run.step(cdist_out=cd[k:k + 1], more=k + 1 < steps)
        with torch.cuda.stream(ms):
            snaps.append(out.clone())            # on the mix stream, behind mix k: X_{k+1} as that step left it
    run.finish()
    torch.cuda.synchronize()
    assert psgd.device_status() == 0
    want = orc.d1d_trajectory(X0, noises, Ts, lr, c)
    return [s.cpu().numpy() for s in snaps], cd.cpu().numpy(), want


def _check(got, cdist, want, steps):
    # free-running trajectory: compare against the largest magnitude it has held (a doubly stochastic mix
    # never amplifies an earlier rounding error; five fp32 roundings per step, independent, so after k steps
    # about sqrt(k) * 1e-7 of that magnitude shows)
    scale = fro = 0.0
    for k in range(steps):
        scale = max(scale, np.abs(want[k + 1]).max(), np.abs(want[k]).max())
        fro = max(fro, np.linalg.norm(want[k + 1]), np.linalg.norm(want[k]))
        g = got[k].astype(np.float64)
        assert not np.isnan(g).any()
        tol = REL
        assert np.abs(g - want[k + 1]).max() <= tol * scale, "step %d" % k
        assert np.linalg.norm(g - want[k + 1]) <= tol * fro, "step %d" % k
        c_want = orc.consensus_dist(got[k])
        assert abs(cdist[k] - c_want) <= REL * c_want


@pytest.mark.parametrize("topo", [orc.TOPO_RAND_RING, orc.TOPO_FULL, orc.TOPO_RING])
@pytest.mark.parametrize("producer_repeat", [1, 6])
def test_overlapped_schedule_matches_oracle_every_element(mods, topo, producer_repeat):
    """Small case, every element of every iterate; producer_repeat = 6 makes the gradient producer several
    times slower than the mix, so it is the event waits (not luck) that keep step k+1's mix behind it."""
    n, d, steps = 8, 40_004, 12
    got, cdist, want = _run(mods, n, d, steps, topo, overlap=True, producer_repeat=producer_repeat)
    _check(got, cdist, want, steps)


def test_overlapped_equals_serial_bit_for_bit(mods):
    """The overlapped and the serial order enqueue the same kernels on the same data: identical bits."""
    n, d, steps = 16, 200_004, 8
    a, ca, want = _run(mods, n, d, steps, orc.TOPO_RAND_RING, overlap=True)
    b, cb, _ = _run(mods, n, d, steps, orc.TOPO_RAND_RING, overlap=False)
    for k in range(steps):
        assert np.array_equal(a[k].view(np.uint32), b[k].view(np.uint32)), k
    assert np.array_equal(ca, cb)
    _check(a, ca, want, steps)


def test_overlapped_schedule_long_rows_kernels_really_overlap(mods):
    """Rows long enough for the large lockstep workgroups (and for the two kernels to be resident together
    for milliseconds), 10 steps, every element against the oracle; the slower producer variant too."""
    n, d, steps = 8, 3_200_004, 10
    for rep in (1, 3):
        got, cdist, want = _run(mods, n, d, steps, orc.TOPO_RAND_RING, overlap=True, producer_repeat=rep, seed=90)
        _check(got, cdist, want, steps)


def test_workload4_overlapped_on_sampled_columns(mods):
    """Workload 4 at full size (n = 128, d = 8 M, randomized ring, G = 0.01 X_{k-1} + N(0, 1e-3^2)) in the
    benchmark's pitched layout and overlapped schedule, 40 steps, sampled columns against the oracle."""
    psgd, d1d = mods
    from paper_2002_01119_amd import placement as plc
    wl = inp.workload(4)
    n, d, steps = wl.n, wl.d, 40
    specs = [("X", torch.float32), ("Y", torch.float32), ("Xprev", torch.float32), ("noise", torch.float32),
             ("G0", torch.float32), ("G1", torch.float32)]
    total_mem = torch.cuda.mem_get_info()[1]
    views, pool, pitch = plc.pitched_layout(n, d, specs, int(0.65 * total_mem), "cuda:0", settle=False)
    X = inp.fill_normal_rows_(views["X"], wl.sigma_x, wl.seed_x)
    noise = inp.fill_normal_rows_(views["noise"], wl.sigma_g, wl.seed_g + 7)
    cols = inp.sample_columns(d, 2048, seed=wl.seed_x)
    cols_t = torch.from_numpy(cols).to("cuda:0")
    X0 = X.index_select(1, cols_t).cpu().numpy()
    Z = noise.index_select(1, cols_t).cpu().numpy()
    tabs = [psgd.build_mixing(wl.topology, n, wl.seed_perm, k) for k in range(steps)]
    for k in (0, 7, steps - 1):
        onbr, ow = orc.neighbour_table(wl.topology, n, wl.seed_perm, k)
        assert np.array_equal(tabs[k][0], onbr) and np.array_equal(tabs[k][1].view(np.uint32), ow.view(np.uint32))
    tabs_dev = [(dev(nb), dev(w)) for nb, w in tabs]
    cd = torch.zeros(steps, dtype=torch.float64, device="cuda:0")
    torch.cuda.synchronize()
    ms = torch.cuda.Stream()
    run = d1d.DelayByOne(X, views["Y"], views["Xprev"], [views["G0"], views["G1"]], noise, lambda k: tabs_dev[k],
                         wl.lr, wl.grad_pull, overlap=True, mix_stream=ms)
    snaps = {}
    for k in range(steps):
        out = run.step(cdist_out=cd[k:k + 1], more=k + 1 < steps)
        if k < 3 or k % 8 == 0 or k == steps - 1:
            with torch.cuda.stream(ms):
                snaps[k] = out.index_select(1, cols_t)
    run.finish()
    torch.cuda.synchronize()
    assert psgd.device_status() == 0
    want = orc.d1d_trajectory(X0, [Z] * steps, [orc.densify(nb, w) for nb, w in tabs], wl.lr, wl.grad_pull)
    scale = max(np.abs(w_).max() for w_ in want)
    fro = max(np.linalg.norm(w_) for w_ in want)
    for k, s in snaps.items():
        g = s.cpu().numpy().astype(np.float64)
        tol = REL
        assert np.abs(g - want[k + 1]).max() <= tol * scale, k
        assert np.linalg.norm(g - want[k + 1]) <= tol * fro, k
    # the fused distance of the last iterate against the separate kernel on the array as it now lies
    chk = torch.zeros(1, dtype=torch.float64, device="cuda:0")
    psgd.consensus_dist_async(run.X, chk)
    torch.cuda.synchronize()
    assert abs(chk.item() - cd[-1].item()) <= 1e-9 * chk.item()
    del views, pool, run, X, noise
    torch.cuda.empty_cache()
